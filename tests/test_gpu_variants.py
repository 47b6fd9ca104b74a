"""GPU parity of the extras of a3po_loss_fwd_bwd_ex and a3po_token_logprobs_entropy against the CPU
oracle: per-token policy entropy, per-token importance weights / clip decisions, and the two baseline
objectives the paper compares against (a caller-supplied proximal log-prob, and the coupled objective).

Tolerances beyond those of test_gpu_parity.py:
  entropy   H = lse - sum_j p_j z_j in fp32.  lse carries the log-prob tolerance (1e-5 (1 + |lse|)); every p_j
            carries the relative error of one hardware exp2 of an argument of magnitude <= ~45 (about 2e-6)
            plus the common factor exp(delta lse), so sum p_j z_j is off by at most ~1e-5 |sum p_j z_j|
            <= 1e-5 (|lse| + H).  Bar:  |gpu - ref| <= 1e-5 |ref| + 2e-5 (1 + |lse_ref|).
"""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")

from test_gpu_parity import (CUR, a3po, assert_close_dz, assert_close_logp, check_against_oracle, dev_logits,  # noqa: E402,F401
                             host_rows, make_case, run_gpu)

pytestmark = pytest.mark.gpu


def cu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_ex(a3po, c, denom=0.0, **kw):
    z_d = dev_logits(c["z"])
    ver = None if kw.pop("no_versions", False) else cu(c["versions"])
    out = a3po.loss_fwd_bwd(z_d, cu(c["chosen"]), cu(c["lb"]), ver, CUR, cu(c["adv"]), cu(c["mask"]),
                            c["w"].clip_eps, denom=denom, V=c["w"].V, **kw)
    torch.cuda.synchronize()
    return out


def assert_close_entropy(gpu, ref, lse_ref, what):
    err = np.abs(np.asarray(gpu, dtype=np.float64) - ref)
    bound = 1e-5 * np.abs(ref) + 2e-5 * (1 + np.abs(lse_ref))
    assert (err <= bound).all(), f"{what}: max err {err.max():.3e} (bound there {bound[err.argmax()]:.3e})"
    return float((err / bound).max())


ENTROPY_CASES = [
    ("f32", 32000, 0),      # 8 sweeps, everything in registers
    ("bf16", 151936, 0),    # 19 sweeps: two vectors parked in LDS, two loads issued late
    ("f32", 65537, 3),      # 17 sweeps with a ragged tail vector, padded stride
    ("bf16", 131072, 0),    # exactly 16 full sweeps
    ("bf16", 4099, 5),      # stride not a multiple of 16 bytes: multi-pass kernel
    ("f32", 7, 1),
    ("f32", 100000, 0),     # too long for the registers: registers plus LDS
    ("f32", 151936, 0),     # registers, LDS and a remainder that is read twice
    ("bf16", 300005, 3),    # the same in bfloat16 with a ragged end
]


@pytest.mark.parametrize("dtype,V,pad", ENTROPY_CASES)
def test_entropy_in_the_loss_pass(a3po, dtype, V, pad):
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=4, L=8, len_lo=4, len_hi=8, sigma=3.0, boost=6.0,
                                       boost_prob=0.5, noise_std=0.2, stale_max=3)
    c = make_case(w, ld=V + pad)
    c["adv"][1] = 0.0                                   # a counted row with zero gradient still has an entropy
    c["lb"][2] = c["lb"][2] - 1.0                       # ratio e: clipped if the advantage is positive
    c["adv"][2] = 0.7
    c["versions"][2] = CUR
    c["mask"][:3] = 1
    plain = run_gpu(a3po, c)
    out = run_ex(a3po, c, want_entropy=True)
    # asking for the entropy changes nothing else
    for k in ("dlogits", "logp", "logp_prox", "loss"):
        a, b = plain[k], out[k]
        if k == "dlogits":
            a, b = a[:, :V], b[:, :V]
        assert torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8)), k
    ref, st, _ = check_against_oracle(a3po, c, out)
    assert ref["clipped"][2] == 1 and ref["g"][2] == 0
    H_ref = oracle.entropy(c["z"], V=V) * ref["eff_mask"]
    worst = assert_close_entropy(out["entropy"].cpu().numpy(), H_ref, ref["lse"], "entropy")
    assert (out["entropy"].cpu().numpy()[ref["eff_mask"] == 0] == 0).all()
    n = max(1, int(ref["eff_mask"].sum()))
    assert abs(st["entropy_mean"] - H_ref.sum() / n) <= 1e-5 * H_ref.sum() / n + 2e-5 * (1 + np.abs(ref["lse"]).max())
    assert a3po.stats_to_dict(plain["stats"])["entropy_mean"] == 0.0
    print(f"entropy {dtype} V={V}: worst err/bound {worst:.3f}, mean {st['entropy_mean']:.4f}")


def test_entropy_with_minus_infinity_logits_and_peaked_rows(a3po):
    # masked vocabulary entries (-inf) contribute 0, a one-hot-like row has entropy ~ 0, a flat row log V
    V = 151936
    w = synth.WORKLOADS["1p5b"].scaled(S=2, L=3, G=2, len_lo=3, len_hi=3)
    c = make_case(w)
    z = synth.bf16_bits_to_f64(c["z"]).astype(np.float32)
    z[0, 1000:] = -np.inf
    z[1, :] = 0.0
    z[2, :] = -30.0
    z[2, 77] = 30.0
    z[3, ::2] = -np.inf
    zt = torch.from_numpy(z).to(torch.bfloat16)
    c["z"] = zt.view(torch.int16).numpy().view(np.uint16).copy()
    c["chosen"][:4] = [5, 9, 77, 1]
    fwd = oracle.token_logprobs(c["z"], c["chosen"], V=V)
    c["lb"] = synth.behav_from_target(fwd["logp"], c["tk"]["noise"][:c["T"]])
    c["mask"][:] = 1
    c["adv"][:] = 0.5
    out = run_ex(a3po, c, want_entropy=True)
    ref, _, _ = check_against_oracle(a3po, c, out)
    H_ref = oracle.entropy(c["z"], V=V)
    H = out["entropy"].cpu().numpy()
    assert np.isfinite(H).all()
    assert_close_entropy(H, H_ref, ref["lse"], "entropy(-inf rows)")
    assert abs(H_ref[1] - np.log(V)) < 1e-9 and H_ref[2] < 1e-15
    logp, lse, _, H2 = a3po.token_logprobs(dev_logits(c["z"]), cu(c["chosen"]), want_entropy=True)
    assert np.isfinite(H2.cpu().numpy()).all()
    assert_close_entropy(H2.cpu().numpy(), H_ref, ref["lse"], "entropy(-inf rows, forward kernel)")


@pytest.mark.parametrize("dtype,V,pad", [("f32", 32000, 0), ("bf16", 151936, 0), ("bf16", 5001, 3), ("f32", 77, 0),
                                         ("bf16", 1, 0)])
def test_token_logprobs_entropy(a3po, dtype, V, pad):
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=4, L=10, len_lo=5, len_hi=10, sigma=3.0)
    tk = synth.token_arrays(w)
    z = synth.logit_rows(w, 0, w.T, tk["chosen"], ld=V + pad)
    y = tk["chosen"].copy()
    ref = oracle.token_logprobs(z, y, V=V)
    H_ref = oracle.entropy(z, V=V)
    zd = dev_logits(z)
    logp, lse, zy, H = a3po.token_logprobs(zd, cu(y), V=V, want_entropy=True)
    logp0, lse0, zy0 = a3po.token_logprobs(zd, cu(y), V=V)
    torch.cuda.synchronize()
    assert_close_logp(lse.cpu().numpy(), ref["lse"], "lse")
    assert_close_logp(logp.cpu().numpy(), ref["logp"], "logp")
    assert torch.equal(zy.view(torch.uint8), zy0.view(torch.uint8))
    assert (lse - lse0).abs().max().item() <= 2e-5 and (logp - logp0).abs().max().item() <= 2e-5
    assert_close_entropy(H.cpu().numpy(), H_ref, ref["lse"], "entropy")


def check_given_prox(a3po, c, out, lp, denom=0.0):
    """Oracle comparison for a loss evaluated with a supplied proximal log-prob `lp` (float32 [T])."""
    w, T, V = c["w"], c["T"], c["w"].V
    fwd = oracle.token_logprobs(c["z"], c["chosen"], V=V)
    ok = (c["chosen"] >= 0) & (c["chosen"] < V)
    eff = ((c["mask"] != 0) & ok).astype(np.uint8)
    lt = np.where(eff == 1, fwd["logp"], 0.0)
    ref = oracle.decoupled_clip(lt, c["lb"], lp, c["adv"], eff, w.clip_eps, denom)
    st = a3po.stats_to_dict(out["stats"])
    assert st["n_tokens"] == ref["stats"]["n_tokens"] == int(eff.sum())
    assert st["n_negative_staleness"] == 0
    assert_close_logp(out["logp"].cpu().numpy(), lt, "logp")
    tau = 1e-4 if w.dtype == "f32" else 1e-3
    near = ((np.abs(ref["r"] - (1 + w.clip_eps)) < tau) | (np.abs(ref["r"] - (1 - w.clip_eps)) < tau)) & (eff == 1)
    assert abs(st["n_clipped"] - ref["stats"]["n_clipped"]) <= int(near.sum())
    N = denom if denom > 0 else max(int(eff.sum()), 1)
    scale = (np.abs(ref["obj"]) * eff).sum() / N
    slack = (np.abs(ref["obj"][near]).sum() * 2 * tau / N) if near.any() else 0.0
    loss = float(out["loss"].cpu()[0])
    assert abs(loss - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-5 * scale + slack + 1e-12, (loss, ref["loss"])
    if eff.any():
        assert abs(st["iw_min"] - ref["stats"]["iw_min"]) <= 1e-5 * ref["stats"]["iw_min"] + 1e-6
        assert abs(st["iw_max"] - ref["stats"]["iw_max"]) <= 1e-5 * ref["stats"]["iw_max"] + 1e-6
    rows = np.nonzero(~near)[0]
    dz_gpu = host_rows(out["dlogits"][torch.from_numpy(rows).cuda()])[:, :V]
    dz_ref = oracle.dlogits_rows(c["z"], c["chosen"], fwd["lse"], ref["g"], rows, V=V)
    assert_close_dz(dz_gpu, dz_ref, ref["g"][rows], w.dtype, "dlogits")
    assert not dz_gpu[ref["g"][rows] == 0].any()
    return ref, st, near


@pytest.mark.parametrize("dtype,V", [("f32", 8000), ("bf16", 151936)])
def test_given_proximal_logprob(a3po, dtype, V):
    # the "recompute" baseline: Eq. 2 with a proximal log-prob from a separate forward pass (here: target + noise)
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=8, L=16 if V < 10000 else 4, G=8, len_lo=3,
                                       len_hi=16 if V < 10000 else 4, noise_std=0.3, sigma=3.0)
    c = make_case(w)
    r = np.random.default_rng(11)
    lp = np.minimum(0.0, c["fwd"]["logp"] + r.standard_normal(c["T"]) * 0.15).astype(np.float32)
    out = run_ex(a3po, c, prox_mode=a3po.A3PO_PROX_GIVEN, logp_prox_in=cu(lp), want_iw=True, want_clipped=True,
                 no_versions=True)
    ref, st, near = check_given_prox(a3po, c, out, lp)
    live = ref["stats"]["n_tokens"]
    # the supplied proximal log-prob comes back untouched on counted tokens
    cnt = (c["mask"] != 0)
    assert np.array_equal(out["logp_prox"].cpu().numpy()[cnt], lp[cnt])
    iw = out["iw"].cpu().numpy()
    assert (np.abs(iw[cnt] - ref["iw"][cnt]) <= 1e-5 * ref["iw"][cnt]).all() and not iw[~cnt].any()
    cl = out["clipped"].cpu().numpy()
    assert np.array_equal(cl[cnt & ~near], ref["clipped"][cnt & ~near]) and not cl[~cnt].any()
    assert st["n_clipped"] == int(cl.sum())
    if V < 10000:
        assert st["n_clipped"] > 3 and live - st["n_clipped"] > 3


def test_given_prox_equal_to_interpolation_matches_the_a3po_path(a3po):
    # feeding Eq. 3's own proximal log-prob back in reproduces the interpolated objective
    c = make_case(synth.WORKLOADS["tiny"], T=200)
    a = run_gpu(a3po, c)
    b = run_ex(a3po, c, prox_mode=a3po.A3PO_PROX_GIVEN, logp_prox_in=a["logp_prox"].clone())
    assert torch.equal(a["logp"], b["logp"])
    sa, sb = a3po.stats_to_dict(a["stats"]), a3po.stats_to_dict(b["stats"])
    assert sa["n_tokens"] == sb["n_tokens"] and abs(sa["n_clipped"] - sb["n_clipped"]) <= 1
    la, lb_ = float(a["loss"].cpu()[0]), float(b["loss"].cpu()[0])
    assert abs(la - lb_) <= 1e-5 * abs(la) + 1e-6
    check_given_prox(a3po, c, b, a["logp_prox"].cpu().numpy())


@pytest.mark.parametrize("dtype,V", [("f32", 8000), ("bf16", 151936)])
def test_coupled_objective(a3po, dtype, V):
    # the "sync" baseline: proximal = behaviour policy, Eq. 1; importance weight exactly 1
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=8, L=16 if V < 10000 else 4, G=8, len_lo=3,
                                       len_hi=16 if V < 10000 else 4, noise_std=0.3, sigma=3.0)
    c = make_case(w)
    out = run_ex(a3po, c, prox_mode=a3po.A3PO_PROX_BEHAV, want_iw=True, no_versions=True)
    ref, st, _ = check_given_prox(a3po, c, out, c["lb"])
    cnt = c["mask"] != 0
    assert (out["iw"].cpu().numpy()[cnt] == 1.0).all() and st["iw_min"] == 1.0 and st["iw_max"] == 1.0
    assert np.array_equal(out["logp_prox"].cpu().numpy()[cnt], c["lb"][cnt])
    # and it is bit-identical to the interpolated path at zero staleness (Eq. 4: alpha(0) = 1)
    c["versions"][:] = CUR
    zero = run_gpu(a3po, c)
    for k in ("dlogits", "logp", "logp_prox", "loss"):
        assert torch.equal(zero[k].view(torch.uint8), out[k].view(torch.uint8)), k


def test_ex_host_validation(a3po):
    c = make_case(synth.WORKLOADS["tiny"], T=8)
    with pytest.raises(a3po.A3poError) as e:
        run_ex(a3po, c, prox_mode=a3po.A3PO_PROX_GIVEN)            # no logp_prox_in
    assert e.value.code == -1
    with pytest.raises(a3po.A3poError) as e:
        run_ex(a3po, c, prox_mode=7)
    assert e.value.code == -7
    with pytest.raises(a3po.A3poError) as e:
        run_ex(a3po, c, no_versions=True, want_iw=True)            # interpolation needs versions
    assert e.value.code == -1


# ---------------------------------------------------------------------------- batches of many tokens

@pytest.mark.parametrize("S,L", [(4, 512), (4, 4096), (5, 3277), (60, 1001), (200, 3001)])
def test_long_batches_of_short_rows(a3po, S, L):
    """The per-token kernels before and after the row pass split a long batch over several workgroups
    (one up to 16,384 tokens, one per 2048 up to 256 of them, equal shares beyond): token counts, statistics,
    per-token outputs and the loss must not depend on where the cuts fall.  Rows are short so that the oracle
    covers every token; the last case has more than 256 * 2048 tokens."""
    w = synth.WORKLOADS["tiny"].scaled(V=48, S=S, L=L, G=5 if S == 5 else 4, len_lo=max(1, L // 3), len_hi=L,
                                       noise_std=0.3, stale_max=6)
    c = make_case(w)
    T = c["T"]
    assert T == S * L
    c["chosen"][[0, T // 2, T - 1]] = [-1, w.V, w.V + 7]           # bad ids in the first, a middle and the last cut
    c["mask"][[0, T // 2, T - 1]] = 1
    c["versions"][[1, T - 2]] = CUR + 2                               # negative staleness at both ends
    c["mask"][[1, T - 2]] = 1
    out = run_ex(a3po, c, want_entropy=True, want_iw=True, want_clipped=True)
    ref, st, _ = check_against_oracle(a3po, c, out, rows=np.r_[0:8, T // 2 - 4:T // 2 + 4, T - 8:T])
    assert st["n_bad_index"] == 3 and st["n_negative_staleness"] >= 2
    sur = oracle.surrogate(ref["logp"], c["lb"], c["versions"], CUR, c["adv"], ref["eff_mask"], w.clip_eps)
    counted = ref["eff_mask"] == 1
    iw = out["iw"].cpu().numpy()
    assert (iw[~counted] == 0).all()
    assert (np.abs(iw[counted] - sur["iw"][counted]) <= 1e-5 * sur["iw"][counted] + 1e-6).all()
    clipped = out["clipped"].cpu().numpy()
    assert int(clipped.sum()) == st["n_clipped"] and not clipped[~counted].any()
    band = (np.abs(sur["r"] - 1.2) < 1e-4) | (np.abs(sur["r"] - 0.8) < 1e-4)
    assert np.array_equal(clipped[counted & ~band], (sur["clipped"][counted & ~band] != 0).astype(np.uint8))
    H_ref = oracle.entropy(c["z"], V=w.V) * ref["eff_mask"]
    n = max(1, int(counted.sum()))
    assert abs(st["entropy_mean"] - H_ref.sum() / n) <= 1e-5 * H_ref.sum() / n + 2e-5 * (1 + np.abs(ref["lse"]).max())
    # fixed summation order within and across workgroups: a second run gives the same bits
    again = run_ex(a3po, c, want_entropy=True)
    assert torch.equal(again["loss"], out["loss"])
