"""a3po_loss_fwd_bwd_noalloc (the entry point for callers that cannot allocate: its workspace is an array
built into the library) against a3po_loss_fwd_bwd on the same inputs, through the C ABI.  Both run the same
kernels, so every output must agree bit for bit; the oracle pins a3po_loss_fwd_bwd itself in
test_gpu_parity.py.  Two calls in a row share the built-in array, the second with a smaller batch and another
vocabulary width, so anything the first call left behind would show."""
import ctypes

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


def _case(w, T):
    tk = synth.token_arrays(w)
    z = synth.logit_rows(w, 0, T, tk["chosen"])
    y = tk["chosen"][:T].copy()
    lt = oracle.token_logprobs(z, y, V=w.V)["logp"]           # recipe input: behaviour = target + noise
    lb = synth.behav_from_target(lt, tk["noise"][:T])
    adv = oracle.grpo_advantages(tk["rewards"], w.G)[tk["seq_id"][:T]].astype(np.float32)
    t = torch.from_numpy(z)
    dev = lambda a: torch.from_numpy(a).cuda()
    return dict(z=(t.view(torch.bfloat16) if z.dtype == np.uint16 else t).cuda(), y=dev(y), lb=dev(lb),
                ver=dev(tk["versions"][:T].copy()), adv=dev(adv), mask=dev(tk["mask"][:T].copy()), eps=w.clip_eps, T=T)


def _both(a3po, c, denom=0.0):
    ref = a3po.loss_fwd_bwd(c["z"], c["y"], c["lb"], c["ver"], CUR, c["adv"], c["mask"], c["eps"], denom=denom)
    T = c["T"]
    out = dict(dlogits=torch.full_like(c["z"], 7.0), logp=torch.full((T,), 7.0, device="cuda"),
               logp_prox=torch.full((T,), 7.0, device="cuda"), loss=torch.full((1,), 7.0, device="cuda"),
               stats=torch.full((a3po.STATS_DTYPE.itemsize,), 7, dtype=torch.uint8, device="cuda"))
    a3po.loss_fwd_bwd_noalloc(c["z"], c["y"], c["lb"], c["ver"], CUR, c["adv"], c["mask"], c["eps"], denom,
                              out["dlogits"], out["logp"], out["logp_prox"], out["loss"], out["stats"])
    torch.cuda.synchronize()
    for k in out:
        assert torch.equal(out[k].view(torch.uint8), ref[k].view(torch.uint8)), k
    return a3po.stats_to_dict(out["stats"])


def test_noalloc_matches_loss_fwd_bwd_two_calls_in_a_row(a3po):
    big = _case(synth.WORKLOADS["1p5b"].scaled(S=16, L=40, G=8, len_lo=10, len_hi=40), 640)   # 640 x 151,936 bf16
    small = _case(synth.WORKLOADS["tiny"], 300)                                               # 300 x 32,000 fp32
    st = _both(a3po, big)
    assert st["n_tokens"] > 0
    st = _both(a3po, small)                    # smaller batch, other dtype and width, same built-in array
    assert 0 < st["n_tokens"] <= 300
    _both(a3po, small, denom=123.0)            # and once more with a caller's denominator
    _both(a3po, big)


def test_noalloc_rejects_batches_beyond_its_array_and_handles_empty_ones(a3po):
    lib = a3po.lib()
    fake = ctypes.c_void_p(0x1000)
    # validation only: returns before any device pointer is used
    rc = lib.a3po_loss_fwd_bwd_noalloc(fake, 1, a3po.NOALLOC_MAX_TOKENS + 1, 64, 64, fake, fake, fake, 3, fake, fake,
                                       0.2, 0.0, fake, fake, None, fake, None, None)
    assert rc == -2 and "size" in a3po.strerror(rc)
    loss = torch.full((1,), 7.0, device="cuda")
    e = lambda dt: torch.empty(0, dtype=dt, device="cuda")
    z = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    a3po.loss_fwd_bwd_noalloc(z, e(torch.int32), e(torch.float32), e(torch.int32), CUR, e(torch.float32),
                              e(torch.uint8), 0.2, 0.0, z.clone(), e(torch.float32), None, loss, None)
    torch.cuda.synchronize()
    assert float(loss.cpu()[0]) == 0.0
