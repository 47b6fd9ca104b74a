"""GPU parity of the mini-batch path: packed ragged sequences, a3po_plan_microbatches for the split,
a3po_count_tokens for each mini-batch's denominator (kept on the device), one a3po_loss_fwd_bwd_ex per
micro-batch with accumulate = 1 after the first and one workspace reused throughout.  The bar: for every
mini-batch, loss / statistics / gradient rows equal those of the CPU oracle evaluating that mini-batch
in one piece (the masked token mean of Eq. 2 over the mini-batch does not know how it was cut up).
"""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")

from test_gpu_parity import CUR, a3po, assert_close_dz, assert_close_logp, dev_logits, host_rows  # noqa: E402,F401
from test_gpu_variants import assert_close_entropy, cu  # noqa: E402

pytestmark = pytest.mark.gpu


def packed_case(w, n_prompt=3):
    """Packs the sequences of workload `w` back to back: each keeps n_prompt leading rows with mask 0 (a prompt)
    followed by its response rows (mask 1).  Returns per-row arrays, per-sequence lengths and the oracle forward."""
    tk = synth.token_arrays(w)
    keep = []
    seq_len = []
    for s in range(w.S):
        n = int(tk["lengths"][s])
        rows = np.arange(s * w.L, s * w.L + n)
        keep.append(rows)
        seq_len.append(n)
    rows = np.concatenate(keep)
    z = np.ascontiguousarray(np.concatenate([synth.logit_rows(w, int(r0[0]), len(r0), tk["chosen"]) for r0 in keep]))
    chosen = tk["chosen"][rows].copy()
    mask = np.ones(len(rows), dtype=np.uint8)
    off = np.concatenate([[0], np.cumsum(seq_len)])
    for s in range(w.S):
        mask[off[s]:off[s] + min(n_prompt, seq_len[s])] = 0
    fwd = oracle.token_logprobs(z, chosen, V=w.V)
    lb = synth.behav_from_target(fwd["logp"], tk["noise"][rows])
    adv_seq = oracle.grpo_advantages(tk["rewards"], w.G)
    adv = adv_seq[tk["seq_id"][rows]].astype(np.float32)
    return dict(w=w, z=z, chosen=chosen, mask=mask, lb=lb, adv=adv, versions=tk["versions"][rows].copy(),
                seq_len=np.asarray(seq_len, dtype=np.int64), off=off, T=len(rows))


@pytest.mark.parametrize("dtype,V,budget,n_mb,L", [
    ("f32", 8000, 160, 4, 64), ("bf16", 151936, 24, 2, 12), ("f32", 1001, 50, 3, 64),
    ("f32", 64, 20000, 2, 6000),    # micro-batches beyond 16,384 tokens: the per-token kernels run on several workgroups
])
def test_microbatches_add_up_to_the_minibatch(a3po, dtype, V, budget, n_mb, L):
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=16, L=L, G=4, len_lo=max(4, L // 6), len_hi=L,
                                       noise_std=0.3, sigma=3.0, stale_max=6)
    c = packed_case(w)
    first, owner = a3po.plan_microbatches(c["seq_len"], n_mb, budget)
    assert len(owner) > n_mb, "the case must actually split mini-batches into several micro-batches"
    z_d = dev_logits(c["z"])
    y, lb, ver, adv, m = cu(c["chosen"]), cu(c["lb"]), cu(c["versions"]), cu(c["adv"]), cu(c["mask"])
    dz = torch.full_like(z_d, 9.0)
    ws = torch.empty(a3po.workspace_bytes(c["T"], V), dtype=torch.uint8, device="cuda")   # one workspace for all calls
    logp = torch.zeros(c["T"], dtype=torch.float32, device="cuda")
    ent = torch.zeros(c["T"], dtype=torch.float32, device="cuda")
    results = {}
    for k in range(n_mb):
        mine = [i for i in range(len(owner)) if owner[i] == k]
        r0, r1 = int(c["off"][first[mine[0]]]), int(c["off"][first[mine[-1] + 1]])
        denom = a3po.count_tokens(y[r0:r1], m[r0:r1], V)                                # stays on the device
        out = {}
        for j, i in enumerate(mine):
            a, b = int(c["off"][first[i]]), int(c["off"][first[i + 1]])
            o = a3po.loss_fwd_bwd(z_d[a:b], y[a:b], lb[a:b], ver[a:b], CUR, adv[a:b], m[a:b], w.clip_eps, V=V,
                                  dlogits=dz[a:b], workspace=ws, denom_dev=denom, accumulate=j > 0,
                                  out=dict(loss=out.get("loss"), stats=out.get("stats"), logp=logp[a:b],
                                           entropy=ent[a:b]), want_entropy=True)
            out = o
        results[k] = (r0, r1, out, float(denom.cpu()[0]))
    torch.cuda.synchronize()

    for k, (r0, r1, out, denom) in results.items():
        sl = slice(r0, r1)
        ref = oracle.loss_fwd_bwd(c["z"][sl], c["chosen"][sl], c["lb"][sl], c["versions"][sl], CUR, c["adv"][sl],
                                  c["mask"][sl], w.clip_eps, V=V, want_dz=True)
        st = a3po.stats_to_dict(out["stats"])
        assert denom == ref["stats"]["n_tokens"] == st["n_tokens"]
        assert st["n_negative_staleness"] == 0 and st["n_bad_index"] == 0
        sur = oracle.surrogate(ref["logp"], c["lb"][sl], c["versions"][sl], CUR, c["adv"][sl], ref["eff_mask"],
                               w.clip_eps)
        tau = 1e-4 if dtype == "f32" else 1e-3
        near = ((np.abs(sur["r"] - 1.2) < tau) | (np.abs(sur["r"] - 0.8) < tau)) & (ref["eff_mask"] == 1)
        assert abs(st["n_clipped"] - ref["stats"]["n_clipped"]) <= int(near.sum())
        assert abs(st["iw_min"] - ref["stats"]["iw_min"]) <= 1e-5 * ref["stats"]["iw_min"] + 1e-6
        assert abs(st["iw_max"] - ref["stats"]["iw_max"]) <= 1e-5 * ref["stats"]["iw_max"] + 1e-6
        N = max(ref["stats"]["n_tokens"], 1)
        scale = (np.abs(sur["obj"]) * ref["eff_mask"]).sum() / N
        slack = (np.abs(sur["obj"][near]).sum() * 2 * tau / N) if near.any() else 0.0
        loss = float(out["loss"].cpu()[0])
        # one more fp32 addition per micro-batch than the single-call path
        assert abs(loss - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 2e-5 * scale + slack + 1e-12, (k, loss, ref["loss"])
        assert_close_logp(logp[sl].cpu().numpy(), ref["logp"], "logp")
        H_ref = oracle.entropy(c["z"][sl], V=V) * ref["eff_mask"]
        assert_close_entropy(ent[sl].cpu().numpy(), H_ref, ref["lse"], "entropy")
        assert abs(st["entropy_mean"] - H_ref.sum() / N) <= 2e-5 * (1 + np.abs(ref["lse"]).max())
        ok = ~near
        assert_close_dz(host_rows(dz[sl])[ok], ref["dz"][ok], ref["g"][ok], dtype, f"dlogits of mini-batch {k}")
        assert not host_rows(dz[sl])[(ref["g"] == 0) & ok].any()
    assert not (dz.float() == 9.0).any(), "every row of the packed stream was written by some micro-batch"
