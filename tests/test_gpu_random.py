"""Seeded random shapes through the whole path and its variants, against the CPU oracle with the bars of
test_gpu_parity.py: vocabularies from 1 to 170,000 entries around every kernel boundary (register-resident,
registers plus LDS plus a streamed remainder, element-wise), padded strides, in-place gradients, entropy, the two
baseline objectives, and vocabulary shards cut at random columns (views of the matrix or contiguous copies).  Every case prints its
parameters first."""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")

from test_gpu_parity import CUR, a3po, assert_close_logp, check_against_oracle, dev_logits, make_case  # noqa: E402,F401
from test_gpu_shards import check_merged, check_partials, run_sharded  # noqa: E402
from test_gpu_variants import assert_close_entropy, check_given_prox, cu, run_ex  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes(a3po, seed):
    rng = np.random.default_rng(seed)
    for case in range(20):
        dtype = ["f32", "bf16"][rng.integers(2)]
        kind = rng.integers(6)
        if kind == 0:
            V = int(rng.integers(1, 64))
        elif kind == 1:
            V = int(rng.integers(64, 5000))
        elif kind == 2:
            V = int(rng.integers(5000, 40000))
        elif kind == 3:
            V = int(rng.choice([8192, 16384, 32768, 65536, 81920, 151936, 163840]))
        elif kind == 4:
            V = int(rng.integers(40000, 170000))
        else:
            V = int(rng.choice([1023, 1024, 1025, 8191, 8193, 81919, 81921, 163839, 163841]))
        pad = int(rng.choice([0, 0, 1, 3, 7, 8, 16, 24]))
        S = int(rng.choice([2, 4, 8]))
        L = int(rng.integers(2, 10)) if V > 20000 else int(rng.integers(2, 40))
        w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=S, L=L, G=2, len_lo=1, len_hi=L,
                                           sigma=float(rng.choice([1.0, 3.0, 6.0])), boost=float(rng.choice([0.0, 6.0])),
                                           boost_prob=0.5, noise_std=float(rng.choice([0.05, 0.3])),
                                           stale_max=int(rng.choice([0, 4, 16])), seed=int(rng.integers(1 << 30)))
        inplace, ent = bool(rng.integers(2)), bool(rng.integers(2))
        mode = int(rng.integers(3))
        nshard = int(rng.integers(1, 5))
        cuts = sorted(set(int(x) for x in rng.integers(1, max(V, 2), nshard - 1))) if V > 1 and nshard > 1 else []
        bounds = [0] + [x for x in cuts if 0 < x < V] + [V]
        views = bool(rng.integers(2)) and pad == 0
        print(f"seed {seed} case {case}: {dtype} V={V} pad={pad} S={S} L={L} inplace={inplace} entropy={ent} "
              f"mode={mode} bounds={bounds} views={views}", flush=True)

        c = make_case(w, ld=V + pad)
        z_d = dev_logits(c["z"])[:, :V]
        dl = z_d if inplace else torch.full((c["T"], V + pad), 7.0, dtype=z_d.dtype, device="cuda")[:, :V]
        out = a3po.loss_fwd_bwd(z_d, cu(c["chosen"]), cu(c["lb"]), cu(c["versions"]), CUR, cu(c["adv"]), cu(c["mask"]),
                                w.clip_eps, V=V, dlogits=dl, want_entropy=ent)
        torch.cuda.synchronize()
        ref, _, _ = check_against_oracle(a3po, c, out)
        if ent:
            assert_close_entropy(out["entropy"].cpu().numpy(), oracle.entropy(c["z"], V=V) * ref["eff_mask"], ref["lse"],
                                 "entropy")
        lp, lse, _ = a3po.token_logprobs(dev_logits(c["z"])[:, :V], cu(c["chosen"]), V=V)
        fwd = oracle.token_logprobs(c["z"], c["chosen"], V=V)
        assert_close_logp(lp.cpu().numpy(), fwd["logp"], "token_logprobs")
        assert_close_logp(lse.cpu().numpy(), fwd["lse"], "lse")
        if mode == 1:
            given = np.minimum(0.0, c["fwd"]["logp"] + rng.standard_normal(c["T"]) * 0.15).astype(np.float32)
            check_given_prox(a3po, c, run_ex(a3po, c, prox_mode=a3po.A3PO_PROX_GIVEN, logp_prox_in=cu(given),
                                             no_versions=True), given)
        elif mode == 2:
            check_given_prox(a3po, c, run_ex(a3po, c, prox_mode=a3po.A3PO_PROX_BEHAV, no_versions=True), c["lb"])
        res = run_sharded(a3po, c, bounds, views=views)
        check_partials(c, res, bounds)
        check_merged(a3po, c, res)
