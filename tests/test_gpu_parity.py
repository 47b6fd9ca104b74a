"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Tolerances (stated once, used everywhere):

  log-probs / lse      |gpu - ref| <= 1e-5 * |ref| + 1e-5          (fp32 accumulate; both dtypes)
  gradients, fp32      |gpu - ref| <= 1e-5 * |ref| + 1e-5 * |g_t|
  gradients, bf16      |gpu - ref| <= 2e-2 * |ref| + 2e-2 * |g_t|   (the stated bar), and
                       the sharper bound the arithmetic gives: one bf16 rounding of an fp32
                       value, |gpu - ref| <= 2^-8 * |ref| + 1e-5 * |g_t|
                       (row t of the gradient is g_t * (onehot - softmax), so |g_t| = d loss / d logp_t
                       is the row's natural scale: every entry is at most |g_t| in magnitude)
  loss                 |gpu - ref| <= 1e-5 * |ref| + 1e-5 * sum_t m_t |obj_t| / N
  integers, gathers    bit exact (chosen logit, counted tokens, bad indices, negative staleness);
                       the clip count is exact up to tokens whose ratio lies within 1e-4 (fp32
                       logits) / 1e-3 (bf16 logits) of a clip boundary, where either branch is accepted.
"""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu

TOL_LOGP = 1e-5
CUR = synth.CURRENT_VERSION


@pytest.fixture(scope="module")
def a3po():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2512_06547_amd as lib
    lib.lib()  # raises if the HIP library is missing: no fallback
    return lib


def dev_logits(z_np, ld=None):
    """numpy float32 / uint16(bf16 bits) [T, ld] -> cuda tensor view [T, V] with row stride ld."""
    t = torch.from_numpy(z_np)
    if z_np.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def host_rows(t):
    """cuda logits-like tensor -> float64 numpy"""
    return t.float().cpu().numpy().astype(np.float64)


def dz_tolerances(dtype):
    return (1e-5, 1e-5, None) if dtype == "f32" else (2e-2, 2e-2, 2.0 ** -8)


def assert_close_logp(gpu, ref, what):
    gpu = np.asarray(gpu, dtype=np.float64)
    err = np.abs(gpu - ref)
    bound = TOL_LOGP * np.abs(ref) + TOL_LOGP
    assert (err <= bound).all(), f"{what}: max err {err.max():.3e} at {err.argmax()}"


def assert_close_dz(gpu_rows, ref_rows, g_rows, dtype, what):
    rel, scale_tol, sharp = dz_tolerances(dtype)
    scale = np.abs(np.asarray(g_rows, dtype=np.float64)).reshape(-1, 1)
    err = np.abs(gpu_rows - ref_rows)
    assert (err <= rel * np.abs(ref_rows) + scale_tol * scale).all(), f"{what}: max err {err.max():.3e}"
    if sharp is not None:
        assert (err <= sharp * np.abs(ref_rows) + 1e-5 * scale + 1e-37).all(), f"{what}: beyond one bf16 rounding"


def make_case(w, T=None, ld=None, seed_shift=0):
    """Inputs of workload `w` (first T tokens), oracle results included."""
    tk = synth.token_arrays(w)
    T = w.T if T is None else T
    ld = w.V if ld is None else ld
    z = synth.logit_rows(w, 0, T, tk["chosen"], ld=ld)
    chosen = tk["chosen"][:T].copy()
    fwd = oracle.token_logprobs(z, chosen, V=w.V)
    lb = synth.behav_from_target(fwd["logp"], tk["noise"][:T])
    adv_seq = oracle.grpo_advantages(tk["rewards"], w.G)
    adv = adv_seq[tk["seq_id"][:T]].astype(np.float32)
    return dict(w=w, T=T, ld=ld, z=z, chosen=chosen, lb=lb, versions=tk["versions"][:T].copy(),
                adv=adv, mask=tk["mask"][:T].copy(), fwd=fwd, tk=tk)


def run_gpu(a3po, c, denom=0.0, inplace=False, dz_fill=None):
    z_d = dev_logits(c["z"])
    V = c["w"].V
    dl = z_d if inplace else None
    if dz_fill is not None and not inplace:
        dl = torch.full_like(z_d, dz_fill)
    out = a3po.loss_fwd_bwd(z_d, torch.from_numpy(c["chosen"]).cuda(), torch.from_numpy(c["lb"]).cuda(),
                            torch.from_numpy(c["versions"]).cuda(), CUR, torch.from_numpy(c["adv"]).cuda(),
                            torch.from_numpy(c["mask"]).cuda(), c["w"].clip_eps, denom=denom, V=V, dlogits=dl)
    torch.cuda.synchronize()
    return out


def check_against_oracle(a3po, c, out, denom=0.0, rows=None):
    w, T, V = c["w"], c["T"], c["w"].V
    ref = oracle.loss_fwd_bwd(c["z"], c["chosen"], c["lb"], c["versions"], CUR, c["adv"], c["mask"], w.clip_eps,
                              denom=denom, V=V, want_dz=False)
    st = a3po.stats_to_dict(out["stats"])
    # integers and masks: exact
    assert st["n_tokens"] == ref["stats"]["n_tokens"]
    assert st["n_bad_index"] == ref["stats"]["n_bad_index"]
    assert st["n_negative_staleness"] == ref["stats"]["n_negative_staleness"]
    logp = out["logp"].cpu().numpy()
    assert_close_logp(logp, ref["logp"], "logp")
    assert (logp[ref["eff_mask"] == 0] == 0).all()
    prox = out["logp_prox"].cpu().numpy()
    assert_close_logp(prox[ref["eff_mask"] == 1], ref["lp"][ref["eff_mask"] == 1], "logp_prox")
    # clip decisions: exact away from the boundary band
    sur = oracle.surrogate(ref["logp"], c["lb"], c["versions"], CUR, c["adv"], ref["eff_mask"], w.clip_eps, denom)
    tau = 1e-4 if w.dtype == "f32" else 1e-3
    near = ((np.abs(sur["r"] - (1 + w.clip_eps)) < tau) | (np.abs(sur["r"] - (1 - w.clip_eps)) < tau)) & \
           (ref["eff_mask"] == 1)
    assert abs(st["n_clipped"] - ref["stats"]["n_clipped"]) <= int(near.sum())
    if st["n_tokens"] > 0:
        assert abs(st["iw_min"] - ref["stats"]["iw_min"]) <= 1e-5 * ref["stats"]["iw_min"] + 1e-6
        assert abs(st["iw_max"] - ref["stats"]["iw_max"]) <= 1e-5 * ref["stats"]["iw_max"] + 1e-6
    else:
        assert st["iw_min"] == np.inf and st["iw_max"] == -np.inf
    # loss
    N = denom if denom > 0 else max(ref["stats"]["n_tokens"], 1)
    scale = (np.abs(sur["obj"]) * ref["eff_mask"]).sum() / N
    # tokens in the boundary band may legitimately take the other branch: widen by their obj spread
    slack = (np.abs(sur["obj"][near]).sum() * 2 * tau / N) if near.any() else 0.0
    loss = float(out["loss"].cpu()[0])
    assert abs(loss - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-5 * scale + slack + 1e-12, (loss, ref["loss"])
    # gradient rows
    rows = np.arange(T) if rows is None else np.asarray(rows)
    dz_gpu = host_rows(out["dlogits"][torch.from_numpy(rows).cuda()])[:, :V]
    dz_ref = oracle.dlogits_rows(c["z"], c["chosen"], ref["lse"], ref["g"], rows, V=V)
    ok_rows = ~near[rows]
    assert_close_dz(dz_gpu[ok_rows], dz_ref[ok_rows], ref["g"][rows][ok_rows], w.dtype, "dlogits")
    for i in np.nonzero(~ok_rows)[0]:   # boundary band: either branch
        g_other = 0.0 if ref["g"][rows[i]] != 0 else -(1.0 / N) * sur["iw"][rows[i]] * c["adv"][rows[i]] * sur["r"][rows[i]]
        alt = ref["g"].copy()
        alt[rows[i]] = g_other
        dz_alt = oracle.dlogits_rows(c["z"], c["chosen"], ref["lse"], alt, rows[i:i + 1], V=V)
        try:
            assert_close_dz(dz_gpu[i:i + 1], dz_ref[i:i + 1], ref["g"][rows[i:i + 1]], w.dtype, "dlogits(band)")
        except AssertionError:
            assert_close_dz(dz_gpu[i:i + 1], dz_alt, alt[rows[i:i + 1]], w.dtype, "dlogits(band, other branch)")
    # dead rows are exactly zero
    dead = (ref["g"][rows] == 0) & ok_rows
    assert not dz_gpu[dead].any()
    return ref, st, int(near.sum())


# ------------------------------------------------------------------------------------------ whole path

def test_tiny_workload_fp32_every_element(a3po):
    c = make_case(synth.WORKLOADS["tiny"])
    out = run_gpu(a3po, c)
    ref, st, excused = check_against_oracle(a3po, c, out)
    assert st["n_tokens"] == int(c["mask"].sum())
    print(f"tiny: N={st['n_tokens']} clipped={st['n_clipped']} excused={excused} loss={float(out['loss'].cpu()[0]):.6f}")


def test_heavy_clipping_fp32(a3po):
    # behaviour noise 0.3 with small staleness (alpha near 1 keeps the ratio wide): many tokens on
    # each side of the clip, so both gradient branches and the clip count are exercised
    w = synth.WORKLOADS["tiny"].scaled(noise_std=0.3, stale_max=4, S=8, L=64, G=8, len_lo=16, len_hi=64, V=8000)
    c = make_case(w)
    out = run_gpu(a3po, c)
    ref, st, excused = check_against_oracle(a3po, c, out)
    assert st["n_clipped"] > 10 and st["n_tokens"] - st["n_clipped"] > 10
    print(f"clipping: N={st['n_tokens']} clipped={st['n_clipped']} excused={excused}")


def test_bf16_full_vocabulary_rows_every_element(a3po):
    # 151,936 columns: 18 full sweeps of the 1024-thread row kernel plus a 560-lane ragged sweep
    w = synth.WORKLOADS["1p5b"].scaled(S=8, L=12, G=8, len_lo=6, len_hi=12)
    c = make_case(w)
    out = run_gpu(a3po, c)
    ref, st, excused = check_against_oracle(a3po, c, out)
    assert 0 < st["n_tokens"] < c["T"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,pad", [(1, 0), (7, 1), (8, 0), (1000, 0), (1001, 7), (4099, 5), (8192, 0), (8200, 8),
                                   (32000, 0), (32768, 64), (50257, 0), (50257, 7), (65537, 15),
                                   (100000, 0), (170000, 8), (100001, 0)])
def test_ragged_vocabularies_and_strides(a3po, dtype, V, pad):
    # covers: single partial sweep, exact sweep multiples, ragged tail vectors, padded strides
    # (padding columns hold a 1e30 sentinel and must be neither read nor written), strides
    # whose byte size is not a multiple of 16 (element-wise multi-pass kernel), and rows too long for the
    # registers (100,000 float32 / 170,000 bfloat16: registers plus LDS; 100,001: element-wise).
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=4, L=6, len_lo=3, len_hi=6, sigma=3.0,
                                       boost=6.0, boost_prob=0.5, noise_std=0.15, stale_max=6)
    c = make_case(w, ld=V + pad)
    out = run_gpu(a3po, c, dz_fill=7.0)
    check_against_oracle(a3po, c, out)
    if pad:
        assert (out["dlogits"][:, V:].float() == 7.0).all(), "padding columns were written"


@pytest.mark.parametrize("dtype,V,pad", [
    ("f32", 151936, 0),    # the full vocabulary in fp32: 19 sweeps in registers, 9 in LDS, 9.1 streamed twice
    ("f32", 114688, 0),    # exactly 28 sweeps: nothing streamed, the last LDS sweep full
    ("f32", 114690, 2),    # the ragged vector is the first one of the streamed part
    ("f32", 130001, 3),    # ragged end inside the streamed part, two batches
    ("f32", 86017, 3),     # 21 sweeps and one ragged vector, which lives in LDS
    ("f32", 500000, 0),    # 122 sweeps: 24 batches of streamed vectors
    ("bf16", 163848, 0),   # one vector more than the register-resident kernel holds
    ("bf16", 256000, 0),   # 31.25 sweeps
    ("bf16", 300005, 3),   # 36.6 sweeps, ragged end in the last streamed batch
])
def test_rows_beyond_the_registers(a3po, dtype, V, pad):
    # 16-byte aligned rows of more than 20 sweeps of 1024 vectors: kept in registers and LDS as far as they fit, the
    # rest read twice; every element against the oracle, padding untouched, and the in-place form bit-identical
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=4, L=6, len_lo=3, len_hi=6, sigma=3.0,
                                       boost=6.0, boost_prob=0.5, noise_std=0.15, stale_max=6)
    c = make_case(w, ld=V + pad)
    out = run_gpu(a3po, c, dz_fill=7.0)
    check_against_oracle(a3po, c, out)
    if pad:
        assert (out["dlogits"][:, V:].float() == 7.0).all(), "padding columns were written"
    inp = run_gpu(a3po, c, inplace=True)
    assert torch.equal(out["dlogits"][:, :V].contiguous().view(torch.uint8),
                       inp["dlogits"][:, :V].contiguous().view(torch.uint8))
    assert torch.equal(out["logp"], inp["logp"]) and torch.equal(out["loss"], inp["loss"])


@pytest.mark.parametrize("dtype,V,L", [("bf16", 8000, 2000), ("bf16", 32000, 1500), ("f32", 16000, 1500)])
def test_many_short_rows(a3po, dtype, V, L):
    # rows of at most four sweeps run as two workgroups per compute unit, all of them claiming rows from the one
    # queue: far more rows than workgroups, every element against the oracle
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=8, L=L, G=8, len_lo=L // 4, len_hi=L, sigma=3.0, boost=6.0,
                                       boost_prob=0.5, noise_std=0.15, stale_max=6)
    c = make_case(w)
    out = run_gpu(a3po, c)
    ref, st, excused = check_against_oracle(a3po, c, out)
    assert 0 < st["n_tokens"] < c["T"]


@pytest.mark.parametrize("dtype,V", [("f32", 32000), ("bf16", 151936), ("bf16", 4099), ("f32", 1001)])
def test_in_place_gradient(a3po, dtype, V):
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=4, L=8, len_lo=4, len_hi=8, noise_std=0.1)
    c = make_case(w)
    sep = run_gpu(a3po, c)
    inp = run_gpu(a3po, c, inplace=True)
    assert torch.equal(sep["dlogits"].view(torch.uint8), inp["dlogits"].view(torch.uint8))
    assert torch.equal(sep["logp"], inp["logp"]) and torch.equal(sep["loss"], inp["loss"])


def test_runs_are_bit_reproducible(a3po):
    c = make_case(synth.WORKLOADS["tiny"], T=512)
    a, b = run_gpu(a3po, c), run_gpu(a3po, c)
    for k in ("dlogits", "logp", "logp_prox", "loss", "stats"):
        assert torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)), k


def test_caller_denominator(a3po):
    c = make_case(synth.WORKLOADS["tiny"], T=300)
    out = run_gpu(a3po, c, denom=1234.0)
    check_against_oracle(a3po, c, out, denom=1234.0)


def test_all_masked_and_empty_batch(a3po):
    c = make_case(synth.WORKLOADS["tiny"], T=64)
    c["mask"][:] = 0
    out = run_gpu(a3po, c, dz_fill=3.0)
    st = a3po.stats_to_dict(out["stats"])
    assert st["n_tokens"] == 0 and float(out["loss"].cpu()[0]) == 0.0
    assert not out["dlogits"].any() and not out["logp"].any()
    assert st["iw_min"] == np.inf and st["iw_max"] == -np.inf
    # T == 0
    z = torch.empty((0, 128), dtype=torch.float32, device="cuda")
    e32 = torch.empty(0, dtype=torch.int32, device="cuda")
    ef = torch.empty(0, dtype=torch.float32, device="cuda")
    out = a3po.loss_fwd_bwd(z, e32, ef, e32, CUR, ef, torch.empty(0, dtype=torch.uint8, device="cuda"), 0.2)
    torch.cuda.synchronize()
    assert float(out["loss"].cpu()[0]) == 0.0 and a3po.stats_to_dict(out["stats"])["n_tokens"] == 0


def test_bad_indices_negative_staleness_zero_advantage(a3po):
    c = make_case(synth.WORKLOADS["tiny"], T=96)
    c["mask"][:] = 1
    c["chosen"][[3, 17]] = [-1, c["w"].V]       # invalid ids: masked and counted
    c["versions"][[5, 6, 40]] = CUR + 3           # negative staleness: alpha = 1, counted
    c["adv"][[8, 9]] = 0.0                        # zero advantage: zero gradient row
    out = run_gpu(a3po, c)
    ref, st, _ = check_against_oracle(a3po, c, out)
    assert st["n_bad_index"] == 2 and st["n_negative_staleness"] == 3 and st["n_tokens"] == 94
    assert not out["dlogits"][[3, 17, 8, 9]].any()


def test_zero_and_unit_staleness_give_identical_results(a3po):
    # Eq. 4: alpha(0) = alpha(1) = 1 -> the proximal policy is the behaviour policy (standard PPO)
    c = make_case(synth.WORKLOADS["tiny"], T=128)
    c["versions"][:] = CUR
    a = run_gpu(a3po, c)
    c["versions"][:] = CUR - 1
    b = run_gpu(a3po, c)
    for k in ("dlogits", "logp", "logp_prox", "loss"):
        assert torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)), k
    live = torch.from_numpy(c["mask"]).cuda().bool()
    assert torch.equal(a["logp_prox"][live], torch.from_numpy(c["lb"]).cuda()[live])


def test_huge_staleness_never_clips(a3po):
    c = make_case(synth.WORKLOADS["tiny"], T=128)
    c["versions"][:] = CUR - (1 << 24)
    out = run_gpu(a3po, c)
    assert a3po.stats_to_dict(out["stats"])["n_clipped"] == 0
    check_against_oracle(a3po, c, out)


# ------------------------------------------------------------------------------------------ stand-alone entry points

@pytest.mark.parametrize("dtype,V,pad", [("f32", 32000, 0), ("bf16", 151936, 0), ("bf16", 5001, 3), ("f32", 77, 0),
                                         ("bf16", 1, 0), ("f32", 262144, 0)])
def test_token_logprobs(a3po, dtype, V, pad):
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=4, L=10, len_lo=5, len_hi=10, sigma=3.0)
    tk = synth.token_arrays(w)
    z = synth.logit_rows(w, 0, w.T, tk["chosen"], ld=V + pad)
    y = tk["chosen"].copy()
    y[1], y[2] = -3, V            # invalid ids
    ref = oracle.token_logprobs(z, y, V=V)
    logp, lse, zy = a3po.token_logprobs(dev_logits(z), torch.from_numpy(y).cuda(), V=V)
    torch.cuda.synchronize()
    assert_close_logp(lse.cpu().numpy(), ref["lse"], "lse")
    assert_close_logp(logp.cpu().numpy(), ref["logp"], "logp")
    raw = zy.view(torch.int32 if dtype == "f32" else torch.int16).cpu().numpy()
    assert np.array_equal(raw.view(ref["chosen_raw"].dtype), ref["chosen_raw"]), "gather is not a bit copy"
    assert logp[1] == 0 and logp[2] == 0


def test_fused_logp_equals_standalone_logp_closely(a3po):
    c = make_case(synth.WORKLOADS["tiny"], T=256)
    out = run_gpu(a3po, c)
    logp, _, _ = a3po.token_logprobs(dev_logits(c["z"]), torch.from_numpy(c["chosen"]).cuda())
    live = torch.from_numpy(c["mask"]).cuda().bool()
    assert (out["logp"][live] - logp[live]).abs().max().item() < 2e-5


def test_proximal_interp(a3po):
    n = 10000
    r = np.random.default_rng(5)
    lt = (-np.abs(r.standard_normal(n) * 4)).astype(np.float32)
    lb = np.minimum(0, lt + r.standard_normal(n).astype(np.float32) * 0.3).astype(np.float32)
    ver = (CUR - r.integers(-2, 20, n)).astype(np.int32)
    lp, al = a3po.proximal_interp(torch.from_numpy(lb).cuda(), torch.from_numpy(lt).cuda(),
                                  torch.from_numpy(ver).cuda(), CUR)
    lp, al = lp.cpu().numpy(), al.cpu().numpy()
    ref_lp, ref_al = oracle.proximal_interp(lb, lt, ver, CUR)
    assert np.array_equal(al, ref_al.astype(np.float32))          # one correctly rounded reciprocal
    assert (np.abs(lp - ref_lp) <= 1e-5 * np.abs(ref_lp) + 1e-6).all()
    one = ref_al == 1.0
    assert np.array_equal(lp[one], lb[one])                        # Eq. 4: d in {0,1} -> exactly log pi_behav
    lo, hi = np.minimum(lb, lt), np.maximum(lb, lt)                # sandwich property on device outputs
    slack = 4 * np.spacing(np.maximum(np.abs(lb), np.abs(lt)))
    assert (lp >= lo - slack).all() and (lp <= hi + slack).all()
    # versions anywhere in int32: the staleness is an exact integer difference (up to 2^32 - 1), converted to
    # fp32 once, so alpha is the correctly rounded 1/d up to d = 2^24 and within one fp32 ulp of it beyond
    ver = r.integers(-2 ** 31, 2 ** 31, n).astype(np.int32)
    for cur in (2 ** 31 - 1, 0, -2 ** 31):
        lp, al = a3po.proximal_interp(torch.from_numpy(lb).cuda(), torch.from_numpy(lt).cuda(),
                                      torch.from_numpy(ver).cuda(), cur)
        ref_lp, ref_al = oracle.proximal_interp(lb, lt, ver, cur)
        al = al.cpu().numpy()
        d = np.int64(cur) - ver.astype(np.int64)
        small = d <= (1 << 24)
        assert np.array_equal(al[small], ref_al.astype(np.float32)[small])
        assert (np.abs(al[~small] - ref_al[~small]) <= 1.2e-7 * ref_al[~small]).all()
        assert (np.abs(lp.cpu().numpy() - ref_lp) <= 1e-5 * np.abs(ref_lp) + 1e-6).all()


def test_grpo_advantages(a3po):
    for G, S in ((4, 4), (8, 32), (8, 16)):
        r = np.random.default_rng(G + S)
        R = (r.random(S) < 0.4).astype(np.float32)
        R[:G] = 1.0                                                # a constant group -> exactly zero
        sid = np.repeat(np.arange(S, dtype=np.int32), 7)
        adv = a3po.grpo_advantages(torch.from_numpy(R).cuda(), G, torch.from_numpy(sid).cuda()).cpu().numpy()
        _, ref = oracle.grpo_advantages(R, G, seq_id=sid)
        assert np.array_equal(adv, ref.astype(np.float32))
        assert not adv[:G * 7].any()


@pytest.mark.parametrize("kind", ["uniform", "normal", "graded", "tiny_spread"])
def test_grpo_advantages_real_valued_rewards(a3po, kind):
    """Rewards that are not 0/1 (graded scores, reward-model outputs): within 1e-6 relative of the fp64 oracle.
    `tiny_spread`: a group whose rewards differ only in the last float32 bits, where the 1e-6 added to the
    standard deviation dominates the denominator."""
    r = np.random.default_rng(len(kind))
    G, S = 8, 48
    if kind == "uniform":
        R = r.random(S)
    elif kind == "normal":
        R = r.standard_normal(S) * 3.0 - 1.0
    elif kind == "graded":
        R = r.integers(0, 5, S) * 0.25
    else:
        R = 0.7 + r.integers(0, 4, S) * 2.0 ** -24
    R = R.astype(np.float32)
    R[G:2 * G] = R[G]                                              # a constant group -> exactly zero
    lens = r.integers(1, 40, S)
    sid = np.repeat(np.arange(S, dtype=np.int32), lens)
    adv = a3po.grpo_advantages(torch.from_numpy(R).cuda(), G, torch.from_numpy(sid).cuda()).cpu().numpy()
    seq_ref, ref = oracle.grpo_advantages(R, G, seq_id=sid)
    assert adv.dtype == np.float32 and adv.shape == ref.shape
    assert (np.abs(adv - ref) <= 1e-6 * np.abs(ref)).all(), np.abs(adv - ref).max()
    assert not adv[(sid >= G) & (sid < 2 * G)].any()
    for g0 in range(0, S, G):                                      # zero mean per group (over sequences)
        assert abs(seq_ref[g0:g0 + G].sum()) <= 1e-9 * np.abs(seq_ref[g0:g0 + G]).sum() + 1e-12
    assert np.abs(ref).max() > (0.05 if kind == "tiny_spread" else 0.5)


# ------------------------------------------------------------------------------------------ streams, graphs

def test_two_streams_with_their_own_workspaces(a3po):
    # the library keeps no global state: calls on different streams with separate outputs and workspaces may overlap
    c1 = make_case(synth.WORKLOADS["tiny"], T=512)
    c2 = make_case(synth.WORKLOADS["tiny"].scaled(stream=9, V=8000, S=8, L=64, G=8, len_lo=16, len_hi=64))
    ref1, ref2 = run_gpu(a3po, c1), run_gpu(a3po, c2)
    ins = []
    for c in (c1, c2):
        ins.append(dict(z=dev_logits(c["z"]), y=torch.from_numpy(c["chosen"]).cuda(), lb=torch.from_numpy(c["lb"]).cuda(),
                        ver=torch.from_numpy(c["versions"]).cuda(), adv=torch.from_numpy(c["adv"]).cuda(),
                        m=torch.from_numpy(c["mask"]).cuda(), eps=c["w"].clip_eps))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [None, None]
    for rep in range(3):
        for i, (st, d) in enumerate(zip(streams, ins)):
            with torch.cuda.stream(st):
                outs[i] = a3po.loss_fwd_bwd(d["z"], d["y"], d["lb"], d["ver"], CUR, d["adv"], d["m"], d["eps"])
    torch.cuda.synchronize()
    for o, r in zip(outs, (ref1, ref2)):
        for k in ("dlogits", "logp", "logp_prox", "loss", "stats"):
            assert torch.equal(o[k].view(torch.uint8), r[k].view(torch.uint8)), k


@pytest.mark.parametrize("V,L,T", [(32000, 256, 384),
                                   (512, 5000, 20000)])  # the per-token kernels on several workgroups
def test_graph_capture_and_replay(a3po, V, L, T):
    # nothing in the call allocates or synchronises, so it can be recorded into a HIP graph; every replay must
    # reproduce the eager result, also after the inputs changed in place between replays
    c = make_case(synth.WORKLOADS["tiny"].scaled(V=V, L=L, len_lo=L // 4, len_hi=L), T=T)
    z = dev_logits(c["z"])
    y, lb, ver = torch.from_numpy(c["chosen"]).cuda(), torch.from_numpy(c["lb"]).cuda(), torch.from_numpy(c["versions"]).cuda()
    adv, m = torch.from_numpy(c["adv"]).cuda(), torch.from_numpy(c["mask"]).cuda()
    dz = torch.empty_like(z)
    ws = torch.empty(a3po.workspace_bytes(c["T"], c["w"].V), dtype=torch.uint8, device="cuda")
    out = a3po.loss_fwd_bwd(z, y, lb, ver, CUR, adv, m, 0.2, dlogits=dz, workspace=ws, want_entropy=True)   # eager, allocates outputs
    torch.cuda.synchronize()
    eager1 = {k: out[k].clone() for k in ("dlogits", "logp", "loss", "stats", "entropy")}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        a3po.loss_fwd_bwd(z, y, lb, ver, CUR, adv, m, 0.2, dlogits=dz, workspace=ws, out=out, want_entropy=True)
    for rep in range(3):
        for k in ("dlogits", "logp", "entropy"):
            out[k].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k, v in eager1.items():
            assert torch.equal(out[k].view(torch.uint8), v.view(torch.uint8)), (rep, k)
    # new inputs in the same buffers: the replay follows them
    adv.mul_(-0.5)
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    replayed = {k: out[k].clone() for k in eager1}
    fresh = a3po.loss_fwd_bwd(z, y, lb, ver, CUR, adv, m, 0.2, want_entropy=True)
    torch.cuda.synchronize()
    for k in eager1:
        assert torch.equal(replayed[k].view(torch.uint8), fresh[k].view(torch.uint8)), k


# ------------------------------------------------------------------------------------------ large logits

@pytest.mark.parametrize("dtype,V,sigma,offset", [("f32", 4099, 300.0, 0.0), ("f32", 32000, 1e4, 0.0), ("bf16", 8192, 30.0, 1e3),
                                                  ("f32", 1000, 1.0, -1e6), ("bf16", 151936, 3000.0, 0.0), ("f32", 64, 1.0, 1e8)])
def test_large_logits(a3po, dtype, V, sigma, offset):
    """Logits far beyond the magnitudes language models produce, and large common offsets: the kernels take
    differences (z - max) before any scaling, so the plain bars hold whatever the magnitude of the logits is.
    What remains is the float32 representation of the results themselves: a log-prob of -3e4 cannot be held
    closer than its own spacing, and the importance ratio exp(log pi - log pi_behav) inherits that
    (`rep` below, four float32 spacings of the log-prob; about 1e-6 for ordinary log-probs).
    Nothing overflows; a third of the entries are -inf."""
    r = np.random.default_rng(int(V + sigma))
    T = 12
    z = (r.standard_normal((T, V)) * sigma + offset).astype(np.float32)
    z[r.random((T, V)) < 0.3] = -np.inf
    y = np.array([r.choice(np.nonzero(np.isfinite(z[t]))[0]) for t in range(T)], dtype=np.int32)
    if dtype == "bf16":
        u = z.view(np.uint32).astype(np.uint64)
        z = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
        z64 = synth.bf16_bits_to_f64(z)
    else:
        z64 = z.astype(np.float64)

    def close(gpu, ref, what):
        err = np.abs(np.asarray(gpu, dtype=np.float64) - ref)
        assert (err <= 1e-5 * np.abs(ref) + 1e-5).all(), f"{what}: max err {err.max():.3e}"

    ref = oracle.token_logprobs(z, y)
    logp, lse, _ = a3po.token_logprobs(dev_logits(z), torch.from_numpy(y).cuda())
    close(lse.cpu().numpy(), ref["lse"], "lse")
    close(logp.cpu().numpy(), ref["logp"], "logp")
    lb = np.minimum(0.0, ref["logp"] + r.standard_normal(T) * 0.2).astype(np.float32)
    ver = (CUR - r.integers(0, 6, T)).astype(np.int32)
    adv = r.standard_normal(T).astype(np.float32)
    m = np.ones(T, dtype=np.uint8)
    out = a3po.loss_fwd_bwd(dev_logits(z), torch.from_numpy(y).cuda(), torch.from_numpy(lb).cuda(),
                            torch.from_numpy(ver).cuda(), CUR, torch.from_numpy(adv).cuda(), torch.from_numpy(m).cuda(), 0.2)
    torch.cuda.synchronize()
    full = oracle.loss_fwd_bwd(z, y, lb, ver, CUR, adv, m, 0.2, want_dz=True)
    close(out["logp"].cpu().numpy(), full["logp"], "fused logp")
    sur = oracle.surrogate(full["logp"], lb, ver, CUR, adv, full["eff_mask"], 0.2)
    rep = 4 * 2.0 ** -24 * np.abs(full["logp"])                  # float32 spacing of the log-prob itself
    tau = (1e-4 if dtype == "f32" else 1e-3) + rep              # the clip ratio inherits it
    ok = (np.abs(np.log(sur["r"]) - np.log(1.2)) > tau) & (np.abs(np.log(sur["r"]) - np.log(0.8)) > tau)
    dz = host_rows(out["dlogits"])
    assert np.isfinite(dz).all() and not dz[~np.isfinite(z64)].any()
    rel = (2e-5 if dtype == "f32" else 2.0 ** -8) + rep[:, None]
    err = np.abs(dz - full["dz"])
    bound = rel * np.abs(full["dz"]) + (1e-5 + rep[:, None]) * np.abs(full["g"])[:, None]
    assert (err[ok] <= bound[ok]).all(), f"dlogits: max err {err[ok].max():.3e}"


_LIBRARY_LOADED_BEFORE_TORCH = r"""
import sys
sys.path.insert(0, sys.argv[1])
import paper_2512_06547_amd as a3po
a3po.lib()                      # before this script has imported torch itself
import numpy as np, torch
import oracle
r = np.random.default_rng(3)
z = r.standard_normal((40, 1031)).astype(np.float32)
y = r.integers(0, 1031, 40).astype(np.int32)
lp, lse, _ = a3po.token_logprobs(torch.from_numpy(z).cuda(), torch.from_numpy(y).cuda())
ref = oracle.token_logprobs(z.astype(np.float64), y)
assert (np.abs(lp.cpu().numpy() - ref["logp"]) <= 1e-5 * np.abs(ref["logp"]) + 1e-5).all()
print("ok")
"""


def test_library_may_be_loaded_before_torch_is_imported(a3po):
    """The library and PyTorch must share one copy of the HIP runtime, whichever the caller touches first: a fresh
    process loads the library, only then imports torch, and launches on torch's stream."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, "-c", _LIBRARY_LOADED_BEFORE_TORCH, root], capture_output=True, text=True,
                       timeout=240)
    assert p.returncode == 0 and p.stdout.strip().endswith("ok"), p.stdout[-2000:] + p.stderr[-4000:]
