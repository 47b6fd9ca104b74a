"""GPU parity at the full sizes of the named workloads (32,768 and 131,072 rows of 151,936 bf16
logits), in the launch configuration the benchmark times: every token's log-prob, the loss, the
statistics, and a sample of gradient rows are compared with the CPU oracle; rows are generated
chunk by chunk (counter-based generator), so the host never holds the whole matrix.  Two of the
workloads then go through the other entry points the benchmark times on the same matrix: the forward-only
kernels with and without the entropy (every token), the fused kernel with the entropy, the step as 4 gradient
updates of micro-batches within the 10,240-token budget, and the vocabulary-sharded entry points on eight
column views (merged log-probs, loss and the sampled rows against the oracle, every gradient element against
the fused kernel's).

Tolerances are those of test_gpu_parity.py.
"""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu
CUR = synth.CURRENT_VERSION


@pytest.fixture(scope="module")
def a3po():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2512_06547_amd as lib
    lib.lib()
    return lib


def _run_full(a3po, name, n_sample, inplace, shards=0, extras=False):
    w = synth.WORKLOADS[name]
    tk = synth.token_arrays(w)
    T, V = w.T, w.V
    z_d = torch.empty((T, V), dtype=torch.bfloat16, device="cuda")
    logp_ref = np.empty(T)
    lse_ref = np.empty(T)
    H_ref = np.empty(T) if extras else None
    chunk = 4096
    for r0 in range(0, T, chunk):
        n = min(chunk, T - r0)
        rows = synth.logit_rows(w, r0, n, tk["chosen"])
        f = oracle.token_logprobs(rows, tk["chosen"][r0:r0 + n].copy())
        logp_ref[r0:r0 + n], lse_ref[r0:r0 + n] = f["logp"], f["lse"]
        if extras:
            H_ref[r0:r0 + n] = oracle.entropy(rows)
        z_d[r0:r0 + n].copy_(torch.from_numpy(rows).view(torch.bfloat16))
    lb = synth.behav_from_target(logp_ref, tk["noise"])
    adv_seq = oracle.grpo_advantages(tk["rewards"], w.G)
    adv = adv_seq[tk["seq_id"]].astype(np.float32)
    dev = lambda a: torch.from_numpy(a).cuda()

    adv_d = a3po.grpo_advantages(dev(tk["rewards"]), w.G, dev(tk["seq_id"]))
    assert np.array_equal(adv_d.cpu().numpy(), adv)
    out = a3po.loss_fwd_bwd(z_d, dev(tk["chosen"]), dev(lb), dev(tk["versions"]), CUR, adv_d, dev(tk["mask"]),
                            w.clip_eps, dlogits=z_d if inplace else None)
    torch.cuda.synchronize()

    mask = tk["mask"]
    sur = oracle.surrogate(np.where(mask == 1, logp_ref, 0.0), lb, tk["versions"], CUR, adv, mask, w.clip_eps)
    st = a3po.stats_to_dict(out["stats"])
    assert st["n_tokens"] == int(mask.sum()) == sur["stats"]["n_tokens"]
    assert st["n_bad_index"] == 0 and st["n_negative_staleness"] == 0
    logp = out["logp"].cpu().numpy().astype(np.float64)
    live = mask == 1
    err = np.abs(logp[live] - logp_ref[live])
    assert (err <= 1e-5 * np.abs(logp_ref[live]) + 1e-5).all(), err.max()
    assert not logp[~live].any()
    prox = out["logp_prox"].cpu().numpy().astype(np.float64)
    assert (np.abs(prox[live] - sur["lp"][live]) <= 1e-5 * np.abs(sur["lp"][live]) + 1e-5).all()
    tau = 1e-3
    near = ((np.abs(sur["r"] - (1 + w.clip_eps)) < tau) | (np.abs(sur["r"] - (1 - w.clip_eps)) < tau)) & live
    assert abs(st["n_clipped"] - sur["stats"]["n_clipped"]) <= int(near.sum())
    assert abs(st["iw_min"] - sur["stats"]["iw_min"]) <= 1e-5 * sur["stats"]["iw_min"] + 1e-6
    assert abs(st["iw_max"] - sur["stats"]["iw_max"]) <= 1e-5 * sur["stats"]["iw_max"] + 1e-6
    N = sur["stats"]["n_tokens"]
    scale = (np.abs(sur["obj"]) * mask).sum() / N
    slack = np.abs(sur["obj"][near]).sum() * 2 * tau / N
    loss = float(out["loss"].cpu()[0])
    assert abs(loss - sur["loss"]) <= 1e-5 * abs(sur["loss"]) + 1e-5 * scale + slack, (loss, sur["loss"])

    # gradient rows: first, last, and a seeded sample that includes masked, clipped and live rows
    r = np.random.default_rng(99)
    cand = [0, T - 1] + list(r.choice(T, n_sample, replace=False))
    clipped_rows = np.nonzero((sur["clipped"] == 1) & live & ~near)[0]
    cand += list(clipped_rows[:4]) + list(np.nonzero(~live)[0][:4])
    rows = np.array(sorted(set(int(c) for c in cand if not near[c])))
    zs = np.concatenate([synth.logit_rows(w, int(t), 1, tk["chosen"]) for t in rows])
    ref = oracle.dlogits_rows(zs, tk["chosen"][rows].copy(), lse_ref[rows], sur["g"][rows], np.arange(len(rows)))
    got = out["dlogits"][torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
    gs = np.abs(sur["g"][rows]).reshape(-1, 1)
    e = np.abs(got - ref)
    assert (e <= 2e-2 * np.abs(ref) + 2e-2 * gs).all()
    assert (e <= 2.0 ** -8 * np.abs(ref) + 1e-5 * gs + 1e-37).all(), "beyond one bf16 rounding"
    dead = sur["g"][rows] == 0
    assert not got[dead].any()
    assert dead.any() and (~dead).any()
    print(f"{name}: T={T} counted={N} clipped={st['n_clipped']} (oracle {sur['stats']['n_clipped']}, "
          f"{int(near.sum())} in the boundary band) loss={loss:.6f} oracle={sur['loss']:.6f} rows checked={len(rows)}")
    if extras:
        _check_extras(a3po, w, tk, z_d, out, logp_ref, lse_ref, H_ref, lb, adv, adv_d, near, dev)
    if shards:
        # the same matrix as `shards` column views through the vocabulary-sharded entry points: merged log-probs
        # against the oracle, the sampled gradient rows against the oracle, and EVERY gradient element against the
        # fused kernel's (two bf16 roundings of fp32 values that differ in their last bits: one bf16 ulp apart at most)
        assert not inplace and V % (8 * shards) == 0
        Vs = V // shards
        y_d, lb_d, ver_d, m_d = dev(tk["chosen"]), dev(lb), dev(tk["versions"]), dev(tk["mask"])
        parts = torch.empty((shards, T, 4), dtype=torch.float32, device="cuda")
        for p in range(shards):
            a3po.shard_partials(z_d[:, p * Vs:(p + 1) * Vs], y_d, p * Vs, out=parts[p])
        logp_s, lse_s, _ = a3po.shard_combine(parts, y_d, V)
        dz_s = torch.full_like(z_d, 3.0)
        ws = None
        for p in range(shards):
            o = a3po.shard_loss_bwd(z_d[:, p * Vs:(p + 1) * Vs], p * Vs, V, y_d, logp_s, lse_s, lb_d, ver_d, CUR, adv_d,
                                    m_d, w.clip_eps, dlogits=dz_s[:, p * Vs:(p + 1) * Vs], workspace=ws)
            ws = o["workspace"]
        torch.cuda.synchronize()
        err = np.abs(logp_s.cpu().numpy().astype(np.float64) - logp_ref)
        assert (err <= 1e-5 * np.abs(logp_ref) + 1e-5).all(), err.max()
        assert a3po.stats_to_dict(o["stats"])["n_tokens"] == N
        loss_s = float(o["loss"].cpu()[0])
        assert abs(loss_s - sur["loss"]) <= 1e-5 * abs(sur["loss"]) + 1e-5 * scale + slack, (loss_s, sur["loss"])
        got_s = dz_s[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        e = np.abs(got_s - ref)
        assert (e <= 2.0 ** -8 * np.abs(ref) + 1e-5 * gs + 1e-37).all(), "sharded gradient beyond one bf16 rounding"
        # rows whose clip decision sits in the boundary band may take different branches on the two paths
        g_abs = torch.from_numpy(np.where(near, np.inf, np.abs(sur["g"])).astype(np.float32)).cuda()
        worst = 0.0
        for r0 in range(0, T, 2048):
            a = dz_s[r0:r0 + 2048].float()
            b = out["dlogits"][r0:r0 + 2048].float()
            bound = 2.0 ** -7 * b.abs() + (1e-5 * g_abs[r0:r0 + 2048]).unsqueeze(1)
            bound = torch.nan_to_num(bound, nan=float("inf"))
            excess = ((a - b).abs() - bound).max().item()
            worst = max(worst, excess)
        assert worst <= 0.0, f"sharded and fused gradients differ by more than one bf16 ulp somewhere ({worst:.3e})"
        print(f"{name}: {shards} column views agree with the fused kernel on all {T}x{V} gradient elements")
        del dz_s, parts
    del out, z_d
    torch.cuda.empty_cache()


def _check_extras(a3po, w, tk, z_d, fused, logp_ref, lse_ref, H_ref, lb, adv, adv_d, near, dev):
    """The other entry points the benchmark times on this matrix, at the same size: the forward-only kernel with
    and without the entropy, the fused kernel with the entropy, and the step as 4 gradient updates of micro-batches
    within the 10,240-token budget (Section 4.1)."""
    T, V, mask = w.T, w.V, tk["mask"]
    y_d, lb_d, ver_d, m_d = dev(tk["chosen"]), dev(lb), dev(tk["versions"]), dev(mask)
    ent_bound = 1e-5 * np.abs(H_ref) + 2e-5 * (1 + np.abs(lse_ref))
    for want in (False, True):
        res = a3po.token_logprobs(z_d, y_d, want_chosen_logit=True, want_entropy=want)
        torch.cuda.synchronize()
        logp, lse, zy = res[:3]
        ent = res[3] if want else None
        for got, ref in ((logp, logp_ref), (lse, lse_ref)):
            e = np.abs(got.cpu().numpy().astype(np.float64) - ref)
            assert (e <= 1e-5 * np.abs(ref) + 1e-5).all(), e.max()
        assert torch.equal(zy, z_d[torch.arange(T, device="cuda"), y_d.long()]), "gather is a bit copy"
        if want:
            assert (np.abs(ent.cpu().numpy().astype(np.float64) - H_ref) <= ent_bound).all()
    o = a3po.loss_fwd_bwd(z_d, y_d, lb_d, ver_d, CUR, adv_d, m_d, w.clip_eps, want_entropy=True)
    torch.cuda.synchronize()
    for k in ("dlogits", "logp", "loss"):      # asking for the entropy changes nothing else
        assert torch.equal(o[k].view(torch.uint8), fused[k].view(torch.uint8)), k
    live = mask == 1
    ent = o["entropy"].cpu().numpy().astype(np.float64)
    assert (np.abs(ent - H_ref)[live] <= ent_bound[live]).all() and not ent[~live].any()
    mean_ref = H_ref[live].mean()
    assert abs(a3po.stats_to_dict(o["stats"])["entropy_mean"] - mean_ref) <= 1e-5 * mean_ref + 2e-5 * (1 + np.abs(lse_ref).max())
    del o

    first, owner = a3po.plan_microbatches(np.full(w.S, w.L, dtype=np.int64), 4, 10240)
    dz = torch.full_like(z_d, 3.0)
    ws = torch.empty(a3po.workspace_bytes(T, V), dtype=torch.uint8, device="cuda")
    res, seen = {}, set()     # per mini-batch: row range, device-resident token count, accumulated outputs
    for i, k in enumerate(owner.tolist()):
        a, e = int(first[i]) * w.L, int(first[i + 1]) * w.L
        if k not in seen:
            mine = [j for j in range(len(owner)) if owner[j] == k]
            r0, r1 = int(first[mine[0]]) * w.L, int(first[mine[-1] + 1]) * w.L
            res[k] = dict(rows=(r0, r1), denom=a3po.count_tokens(y_d[r0:r1], m_d[r0:r1], V), out={})
        prev = res[k]["out"]
        res[k]["out"] = a3po.loss_fwd_bwd(z_d[a:e], y_d[a:e], lb_d[a:e], ver_d[a:e], CUR, adv_d[a:e], m_d[a:e], w.clip_eps,
                                          V=V, dlogits=dz[a:e], workspace=ws, denom_dev=res[k]["denom"],
                                          accumulate=k in seen, out=dict(loss=prev.get("loss"), stats=prev.get("stats")))
        seen.add(k)
    torch.cuda.synchronize()
    assert len(res) == 4 and len(owner) >= 4    # (1p5b: one micro-batch per mini-batch; long: two, accumulated)
    assert not (dz.float() == 3.0).any()
    r = np.random.default_rng(7)
    for k, v in res.items():
        r0, r1 = v["rows"]
        sl = slice(r0, r1)
        sur = oracle.surrogate(np.where(mask[sl] == 1, logp_ref[sl], 0.0), lb[sl], tk["versions"][sl], CUR, adv[sl],
                               mask[sl], w.clip_eps)
        st = a3po.stats_to_dict(v["out"]["stats"])
        N = int(mask[sl].sum())
        assert st["n_tokens"] == N == int(float(v["denom"].cpu()[0]))
        nr = near[sl]
        assert abs(st["n_clipped"] - sur["stats"]["n_clipped"]) <= int(nr.sum())
        scale = (np.abs(sur["obj"]) * mask[sl]).sum() / N
        slack = np.abs(sur["obj"][nr]).sum() * 2e-3 / N
        loss = float(v["out"]["loss"].cpu()[0])
        assert abs(loss - sur["loss"]) <= 1e-5 * abs(sur["loss"]) + 2e-5 * scale + slack, (k, loss, sur["loss"])
        rows = np.array(sorted(int(t) for t in r.choice(r1 - r0, 8, replace=False) if not nr[t]))
        zs = np.concatenate([synth.logit_rows(w, r0 + int(t), 1, tk["chosen"]) for t in rows])
        ref = oracle.dlogits_rows(zs, tk["chosen"][r0 + rows].copy(), lse_ref[r0 + rows], sur["g"][rows], np.arange(len(rows)))
        got = dz[torch.from_numpy(r0 + rows).cuda()].float().cpu().numpy().astype(np.float64)
        gs = np.abs(sur["g"][rows]).reshape(-1, 1)
        assert (np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * gs + 1e-37).all(), k
    print(f"{w.name}: forward-only kernels, entropy, and {len(owner)} micro-batches in 4 mini-batches agree with the oracle")


def test_1p5b_shape_full_size(a3po):
    _run_full(a3po, "1p5b", 48, inplace=False, shards=8, extras=True)


def test_8b_shape_full_size_in_place(a3po):
    _run_full(a3po, "8b", 32, inplace=True)


def test_long_response_high_staleness_full_size(a3po):
    _run_full(a3po, "long", 32, inplace=False, shards=8, extras=True)
