"""GPU parity of a3po_histogram against the CPU oracle.

The operation itself compares stored float32 values with stored float32 edges, so on the same seeded
inputs the counts must be bit-identical to the oracle's.  The end-to-end case (importance weights from the
loss call, Section 4.2.2) compares the histogram of the GPU's fp32 weights with the histogram of the
oracle's fp64 weights: a token whose oracle weight lies within 1e-5 (relative) of an edge may sit on
either side of it, everything else must agree, and the totals must agree exactly.
"""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")

from test_gpu_parity import CUR, a3po, make_case  # noqa: E402,F401
from test_gpu_variants import cu, run_ex  # noqa: E402

pytestmark = pytest.mark.gpu


def values_with_special_cases(n, edges, seed):
    r = np.random.default_rng(seed)
    v = np.exp(r.standard_normal(n) * 0.4).astype(np.float32)
    k = min(n, 4 * len(edges))
    v[r.choice(n, k, replace=False)] = np.resize(edges, k)          # values exactly on an edge
    for i, x in enumerate([np.nan, np.inf, -np.inf, 0.0, -0.0, np.float32(edges[0]) - np.float32(1e-7)]):
        if i < n:
            v[(7 * i + 3) % n] = x
    return v


@pytest.mark.parametrize("T,nbins", [(1, 1), (255, 7), (100003, 16), (40000, 64), (6000, 1024), (300000, 3)])
def test_counts_equal_the_oracle_bit_for_bit(a3po, T, nbins):
    edges = np.geomspace(0.3, 3.0, nbins + 1).astype(np.float32)
    v = values_with_special_cases(T, edges, seed=T + nbins)
    sel = (np.random.default_rng(T).random(T) < 0.6).astype(np.uint8)
    for s in (None, sel):
        got = a3po.histogram(cu(v), cu(edges), select=None if s is None else cu(s))
        torch.cuda.synchronize()
        ref = oracle.histogram(v, edges, s)
        assert np.array_equal(got.cpu().numpy(), ref), (T, nbins, s is not None)
        assert int(got.sum()) == (T if s is None else int(s.sum()))


def test_repeated_edges_accumulation_and_empty_input(a3po):
    edges = np.array([0.5, 1.0, 1.0, 1.0, 2.0], dtype=np.float32)
    v = np.array([1.0, 0.25, 1.5, 2.0, 0.5, 1.0, np.nan], dtype=np.float32)
    got = a3po.histogram(cu(v), cu(edges))
    assert got.cpu().tolist() == oracle.histogram(v, edges).tolist() == [1, 1, 0, 0, 3, 1, 1]
    # two halves accumulated into one set of counts = the whole
    r = np.random.default_rng(5)
    w = np.exp(r.standard_normal(50001) * 0.5).astype(np.float32)
    e = np.linspace(0.0, 4.0, 41).astype(np.float32)
    out = a3po.histogram(cu(w[:20000]), cu(e))
    out = a3po.histogram(cu(w[20000:]), cu(e), accumulate=True, out=out)
    assert np.array_equal(out.cpu().numpy(), oracle.histogram(w, e))
    # T == 0: cleared when overwriting, untouched when accumulating
    keep = out.clone()
    a3po.histogram(torch.empty(0, device="cuda"), cu(e), accumulate=True, out=out)
    assert torch.equal(out, keep)
    a3po.histogram(torch.empty(0, device="cuda"), cu(e), out=out)
    assert not out.any()
    with pytest.raises(a3po.A3poError) as err:
        a3po.histogram(cu(w), torch.zeros(1026, device="cuda"))
    assert err.value.code == -2


def test_importance_weight_histograms_of_a_loss_call(a3po):
    w = synth.WORKLOADS["tiny"].scaled(V=8000, S=8, L=128, G=4, len_lo=40, len_hi=128, noise_std=0.3, stale_max=8)
    c = make_case(w)
    out = run_ex(a3po, c, want_iw=True, want_clipped=True)
    ref = oracle.loss_fwd_bwd(c["z"], c["chosen"], c["lb"], c["versions"], CUR, c["adv"], c["mask"], w.clip_eps, V=w.V)
    sur = oracle.surrogate(ref["logp"], c["lb"], c["versions"], CUR, c["adv"], ref["eff_mask"], w.clip_eps)
    edges = np.geomspace(0.5, 2.0, 25).astype(np.float32)
    mask_d = cu(c["mask"])

    def check(select_gpu, select_ref, what):
        got = a3po.histogram(out["iw"], cu(edges), select=select_gpu).cpu().numpy()
        want = oracle.histogram(sur["iw"], edges, select_ref)
        iw = sur["iw"][select_ref != 0]
        near = np.array([(np.abs(iw - e) <= 1e-5 * e).sum() for e in edges.astype(np.float64)])
        slack = np.concatenate([[near[0]], near[:-1] + near[1:], [near[-1]], [0]])
        assert (np.abs(got - want) <= slack).all(), (what, got, want)
        assert got.sum() == want.sum()
        return got

    all_counted = check(mask_d, ref["eff_mask"], "counted tokens")
    st = a3po.stats_to_dict(out["stats"])
    assert all_counted.sum() == st["n_tokens"]
    occupied = np.nonzero(all_counted)[0]
    assert occupied.size and all_counted[-1] == 0
    # the clip decisions of the GPU select the clipped tokens; their number is the statistic of Fig. 6
    clipped = a3po.histogram(out["iw"], cu(edges), select=out["clipped"])
    assert int(clipped.sum()) == st["n_clipped"]
    tau = 1e-4
    band = ((np.abs(sur["r"] - 1.2) < tau) | (np.abs(sur["r"] - 0.8) < tau)) & (ref["eff_mask"] == 1)
    if not band.any():
        check(out["clipped"], ((sur["clipped"] != 0) & (ref["eff_mask"] == 1)).astype(np.uint8), "clipped tokens")
