"""GPU parity of the fused LM-head log-prob (hidden states x LM-head weight on the matrix cores,
streamed into the online log-sum-exp) against the CPU oracle: z = h W^T by plain loops in fp64,
then the textbook log-softmax.  Tolerance: abs(gpu - ref) <= 1e-5 * abs(ref) + 2e-5 on lse and
log-probs (bf16 inputs are exact in both; the GPU accumulates H products in fp32 on the MFMA
units, which adds about sqrt(H) * 2^-24 * |z| to each logit)."""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def a3po():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2512_06547_amd as lib
    lib.lib()
    return lib


def bf16_bits(x):
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def close(gpu, ref, what):
    err = np.abs(np.asarray(gpu, dtype=np.float64) - ref)
    assert (err <= 1e-5 * np.abs(ref) + 2e-5).all(), f"{what}: max err {err.max():.3e}"


@pytest.mark.parametrize("T,H,V", [(1, 64, 1), (5, 64, 7), (256, 128, 256), (300, 192, 1000), (257, 64, 2049),
                                   (1100, 256, 4500), (2048, 128, 2304), (9000, 64, 300), (700, 320, 20000)])
def test_fused_lmhead_logprob_small(a3po, T, H, V):
    # spans: single partial tile, exact tile multiples, ragged token and vocabulary tiles, hidden sizes that are and
    # are not a multiple of the ring depth, more token-tile groups than XCDs (several sweeps per workgroup), more
    # vocabulary tiles than one round of an XCD's workgroups, XCDs that share a token group
    r = np.random.default_rng(T * 131 + V)
    h = bf16_bits(r.standard_normal((T, H)))
    W = bf16_bits(r.standard_normal((V, H)) * 0.3)
    y = r.integers(0, V, T).astype(np.int32)
    if T > 3:
        y[1], y[2] = -1, V
    z = oracle.lmhead_logits(h, W)
    ref = oracle.token_logprobs(z, y)
    logp, lse = a3po.fused_lmhead_logprob(torch.from_numpy(h).view(torch.bfloat16).cuda(),
                                          torch.from_numpy(W).view(torch.bfloat16).cuda(),
                                          torch.from_numpy(y).cuda())
    torch.cuda.synchronize()
    close(lse.cpu().numpy(), ref["lse"], "lse")
    close(logp.cpu().numpy(), ref["logp"], "logp")
    if T > 3:
        assert logp[1] == 0 and logp[2] == 0


def test_fused_lmhead_matches_materialised_path(a3po):
    # same inputs through a bf16-materialised logits matrix + a3po_token_logprobs: differs only by
    # the bf16 rounding of the logits the fused path never performs
    r = np.random.default_rng(3)
    T, H, V = 512, 256, 3000
    h = torch.from_numpy(bf16_bits(r.standard_normal((T, H)))).view(torch.bfloat16).cuda()
    W = torch.from_numpy(bf16_bits(r.standard_normal((V, H)) * 0.1)).view(torch.bfloat16).cuda()
    y = torch.from_numpy(r.integers(0, V, T).astype(np.int32)).cuda()
    logp, lse = a3po.fused_lmhead_logprob(h, W, y)
    z = (h.float() @ W.float().t()).bfloat16().contiguous()
    logp2, lse2, _ = a3po.token_logprobs(z, y)
    assert (lse - lse2).abs().max().item() < 2e-2 and (logp - logp2).abs().max().item() < 5e-2


def test_fused_lmhead_full_vocabulary_sampled_tokens(a3po):
    # the 8B-shape weight (151,936 x 4,096) with 2,048 tokens; the oracle checks a seeded token sample
    lw = synth.LMHEAD_WORKLOADS["lmhead8b"]
    T, H, V = 2048, lw.H, lw.tokens.V
    tk = synth.token_arrays(lw.tokens)
    h = synth.hidden_rows(lw, 0, T)
    W_d = torch.empty((V, H), dtype=torch.bfloat16, device="cuda")
    W_h = np.empty((V, H), dtype=np.uint16)
    for v0 in range(0, V, 16384):
        n = min(16384, V - v0)
        W_h[v0:v0 + n] = synth.weight_rows(lw, v0, n)
        W_d[v0:v0 + n].copy_(torch.from_numpy(W_h[v0:v0 + n]).view(torch.bfloat16))
    y = tk["chosen"][:T].copy()
    logp, lse = a3po.fused_lmhead_logprob(torch.from_numpy(h).view(torch.bfloat16).cuda(), W_d,
                                          torch.from_numpy(y).cuda())
    torch.cuda.synchronize()
    rows = np.array([0, 1, 255, 256, 1023, 2047, 777, 1500])
    z = oracle.lmhead_logits(h, W_h, rows=rows)
    ref = oracle.token_logprobs(z, y[rows].copy())
    close(lse.cpu().numpy()[rows], ref["lse"], "lse")
    close(logp.cpu().numpy()[rows], ref["logp"], "logp")


_FIRST_CALL_FROM_TWO_THREADS = r"""
import sys, threading
import numpy as np, torch
sys.path.insert(0, sys.argv[1])
import oracle, paper_2512_06547_amd as a3po

def bits(x):
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)

a3po.lib()
torch.cuda.set_device(0)
cases = []
for i, (T, H, V) in enumerate([(700, 128, 3000), (300, 192, 5000)]):   # one shape per kernel variant (ring-depth multiple or not)
    r = np.random.default_rng(i)
    h, W, y = bits(r.standard_normal((T, H))), bits(r.standard_normal((V, H)) * 0.3), r.integers(0, V, T).astype(np.int32)
    cases.append(dict(h=h, W=W, y=y, hd=torch.from_numpy(h).view(torch.bfloat16).cuda(),
                      Wd=torch.from_numpy(W).view(torch.bfloat16).cuda(), yd=torch.from_numpy(y).cuda(),
                      stream=torch.cuda.Stream()))
torch.cuda.synchronize()
gate, out = threading.Barrier(4), {}

def worker(k, c):
    with torch.cuda.stream(c["stream"]):
        gate.wait()                                 # all threads enter the library together: its first calls
        out[k] = a3po.fused_lmhead_logprob(c["hd"], c["Wd"], c["yd"])
        c["stream"].synchronize()

threads = [threading.Thread(target=worker, args=(k, cases[k % 2])) for k in range(4)]
[t.start() for t in threads]
[t.join() for t in threads]
assert len(out) == 4
for k in range(4):
    c = cases[k % 2]
    ref = oracle.token_logprobs(oracle.lmhead_logits(c["h"], c["W"]), c["y"])
    for got, want in ((out[k][0], ref["logp"]), (out[k][1], ref["lse"])):
        err = np.abs(got.cpu().numpy().astype(np.float64) - want)
        assert (err <= 1e-5 * np.abs(want) + 2e-5).all(), (k, err.max())
print("ok")
"""


def test_first_calls_from_several_host_threads_at_once(a3po):
    """The one-time set-up of the matrix-core kernels (their LDS limit) is race-free: a fresh process whose very
    first calls into the library come from four host threads at the same moment, on two streams and through both
    kernel variants, gets the oracle's log-probs from every call."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, "-c", _FIRST_CALL_FROM_TWO_THREADS, root], capture_output=True, text=True, timeout=240)
    assert p.returncode == 0 and p.stdout.strip().endswith("ok"), p.stdout[-2000:] + p.stderr[-4000:]


# ------------------------------------------------------------------------------------------ forward + backward
#
# The reference is the plain fp64 oracle with nothing rounded: z = h W^T, log-softmax, Eq. 2 - Eq. 4, the
# gradient rows dz in fp64, then dh = dz W and dW = dz^T h in fp64.  What the GPU path does differently, and
# the bound each difference gives (u = 2^-8: rounding a value to bfloat16 moves it by at most u |value|):
#   logits      fp32 accumulation of H products on the matrix cores; lse and log-probs never see a rounded
#               logit                                     ->  1e-5 |ref| + 2e-5 (the bar of the forward-only tests)
#   loss        moves with the log-probs; the objective is continuous across a clip boundary
#                                                         ->  1e-4 * sum m |obj| / N
#   dz          fp32 from fp32 logits (relative error ~1e-4 from lse, g and the hardware exp), then rounded ONCE
#               to bfloat16 because the matrix cores take bfloat16 operands
#   dh, dW      fp32 accumulation of those products (error below 2^-11 sum |dz||operand| at these lengths),
#               output rounded once to bfloat16
#     element-wise:  |gpu - ref| <= u |ref| + (u + 2^-10) sum |dz| |operand|
#     norm-wise:     ||gpu - ref||_F <= 1e-2 ||ref||_F  (printed; the stated bar for bfloat16 is 2e-2 relative)
# Clip decisions are integers decided by floating point: the inputs are drawn so that no counted token's
# log-ratio lies within 2e-3 of a clip bound (the log-probs agree to 2e-5), and the clip count must then be exact.

U = 2.0 ** -8


def _away_from_clip_bounds(lt, lb, ver, cur, adv, mask, rng, sigma):
    """Re-draws the behaviour noise of tokens whose ratio r = exp(alpha (lt - lb)) lies within 2e-3 (in the log)
    of 1 +- 0.2, until none is left.  Returns the float32 behaviour log-probs."""
    lb = lb.copy()
    for _ in range(100):
        sur = oracle.surrogate(lt, lb, ver, cur, adv, mask, 0.2)
        near = (np.abs(np.log(sur["r"]) - np.log(1.2)) < 2e-3) | (np.abs(np.log(sur["r"]) - np.log(0.8)) < 2e-3)
        if not near.any():
            return lb
        lb[near] = synth.behav_from_target(lt[near], (rng.standard_normal(int(near.sum())) * sigma).astype(np.float32))
    raise AssertionError("could not move every token away from the clip bounds")


def _check_backward(gpu, ref, ref_abs, what):
    err = np.abs(gpu - ref)
    bound = U * np.abs(ref) + (U + 2.0 ** -10) * ref_abs + 1e-30
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} elements off, worst {np.max(err / bound):.2f} x the bound"
    rel = np.linalg.norm(err) / max(np.linalg.norm(ref), 1e-300)
    assert rel <= 1e-2, f"{what}: norm-wise {rel:.3e}"
    return rel


@pytest.mark.parametrize("T,H,V,p_mask", [(300, 64, 1000, 0.8), (1, 64, 8, 1.0), (8192 + 300, 64, 512, 0.8),
                                          (467, 192, 1344, 0.8), (16384, 256, 4096, 1.0),
                                          (65536 + 700, 64, 512, 1.0)])
def test_fused_lmhead_loss_fwd_bwd(a3po, T, H, V, p_mask):
    """Whole path from hidden states against the un-rounded fp64 oracle.  The cases span one and several token
    chunks (8,192 tokens each), ragged tiles on every side, hidden sizes that are and are not a multiple of the
    ring depth; the last but one has every token counted with a non-zero advantage over two full chunks, the last
    one nine chunks, i.e. more than the 65,536 tokens one weight-gradient contraction takes, so the second
    contraction adds onto the result of the first."""
    r = np.random.default_rng(T + 7 * V)
    cur = 50
    h = bf16_bits(r.standard_normal((T, H)))
    W = bf16_bits(r.standard_normal((V, H)) * (2.0 / np.sqrt(H)))
    y = r.integers(0, V, T).astype(np.int32)
    mask = (r.random(T) < p_mask).astype(np.uint8)
    mask[0] = 1
    ver = (cur - r.integers(0, 5, T)).astype(np.int32)
    adv = r.standard_normal(T).astype(np.float32)
    adv[adv == 0] = 1.0
    z = oracle.lmhead_logits(h, W)                                   # fp64, never rounded
    lt = oracle.token_logprobs(z, y)["logp"]
    lb = synth.behav_from_target(lt, (r.standard_normal(T) * 0.15).astype(np.float32))
    lb = _away_from_clip_bounds(lt, lb, ver, cur, adv, mask, r, 0.15)
    ref = oracle.loss_fwd_bwd(z, y, lb, ver, cur, adv, mask, 0.2)
    # (the plain loops where they finish in seconds, the same products through the fp64 matrix product beyond)
    backward = oracle.lmhead_backward if T * H * V < 2e8 else oracle.lmhead_backward_matmul
    dh_ref, dw_ref = backward(ref["dz"], h, W)
    dh_abs, dw_abs = backward(np.abs(ref["dz"]), h & 0x7FFF, W & 0x7FFF)

    dev_ = lambda a: torch.from_numpy(a).cuda()
    out = a3po.fused_lmhead_loss_fwd_bwd(dev_(h).view(torch.bfloat16), dev_(W).view(torch.bfloat16), dev_(y), dev_(lb),
                                         dev_(ver), cur, dev_(adv), dev_(mask), 0.2)
    torch.cuda.synchronize()
    st = a3po.stats_to_dict(out["stats"])
    assert st["n_tokens"] == ref["stats"]["n_tokens"] == int(mask.sum())
    assert st["n_clipped"] == ref["stats"]["n_clipped"]
    logp = out["logp"].cpu().numpy().astype(np.float64)
    close(logp, ref["logp"], "logp")
    assert not logp[mask == 0].any()
    prox = out["logp_prox"].cpu().numpy().astype(np.float64)
    close(prox[mask == 1], ref["lp"][mask == 1], "logp_prox")
    N = max(1, st["n_tokens"])
    sur = oracle.surrogate(ref["logp"], lb, ver, cur, adv, ref["eff_mask"], 0.2)
    scale = (np.abs(sur["obj"]) * ref["eff_mask"]).sum() / N
    loss = float(out["loss"].cpu()[0])
    assert abs(loss - ref["loss"]) <= 1e-4 * scale + 1e-12, (loss, ref["loss"])
    assert abs(st["iw_min"] - ref["stats"]["iw_min"]) <= 1e-4 and abs(st["iw_max"] - ref["stats"]["iw_max"]) <= 1e-4
    dh = out["dhidden"].float().cpu().numpy().astype(np.float64)
    dw = out["dweight"].float().cpu().numpy().astype(np.float64)
    assert np.abs(dh_ref).max() > 0 and np.abs(dw_ref).max() > 0
    rh = _check_backward(dh, dh_ref, dh_abs, "dh")
    rw = _check_backward(dw, dw_ref, dw_abs, "dW")
    assert not dh[ref["g"] == 0].any(), "a token without gradient must leave its row of dh exactly zero"
    print(f"T={T} H={H} V={V}: |loss err| {abs(loss - ref['loss']):.2e} (scale {scale:.2e}), norm-wise dh {rh:.2e} dW {rw:.2e}, "
          f"{st['n_clipped']} clipped of {st['n_tokens']}")


def test_fused_lmhead_loss_matches_forward_only_entry_point(a3po):
    """Both entry points keep fp32 logits on chip for the log-sum-exp: their log-probs agree to rounding order."""
    r = np.random.default_rng(5)
    T, H, V = 3000, 128, 5000
    h = torch.from_numpy(bf16_bits(r.standard_normal((T, H)))).view(torch.bfloat16).cuda()
    W = torch.from_numpy(bf16_bits(r.standard_normal((V, H)) * 0.2)).view(torch.bfloat16).cuda()
    y = torch.from_numpy(r.integers(0, V, T).astype(np.int32)).cuda()
    logp_f, _ = a3po.fused_lmhead_logprob(h, W, y)
    one = torch.ones(T, device="cuda")
    out = a3po.fused_lmhead_loss_fwd_bwd(h, W, y, logp_f.clone(), torch.full((T,), 3, dtype=torch.int32, device="cuda"), 3,
                                         one, torch.ones(T, dtype=torch.uint8, device="cuda"), 0.2)
    torch.cuda.synchronize()
    assert (out["logp"] - logp_f).abs().max().item() <= 4e-6


def test_fused_lmhead_loss_fwd_bwd_empty_batch(a3po):
    """T == 0: loss 0, no counted tokens, an all-zero weight gradient (the buffer is written, not left as found)."""
    H, V = 64, 24
    W = torch.randn((V, H), device="cuda").bfloat16()
    h = torch.empty((0, H), dtype=torch.bfloat16, device="cuda")
    i32 = torch.empty(0, dtype=torch.int32, device="cuda")
    f32 = torch.empty(0, dtype=torch.float32, device="cuda")
    out = a3po.fused_lmhead_loss_fwd_bwd(h, W, i32, f32, i32, 3, f32, torch.empty(0, dtype=torch.uint8, device="cuda"), 0.2)
    torch.cuda.synchronize()
    assert float(out["loss"].cpu()[0]) == 0.0
    assert a3po.stats_to_dict(out["stats"])["n_tokens"] == 0
    assert out["dweight"].shape == (V, H) and not out["dweight"].any()
    assert out["dhidden"].numel() == 0


def _full_size_inputs():
    lw = synth.LMHEAD_WORKLOADS["lmhead8b"]
    T, H, V = lw.tokens.T, lw.H, lw.tokens.V
    assert (T, H, V) == (65536, 4096, 151936)
    tk = synth.token_arrays(lw.tokens)
    h = synth.hidden_rows(lw, 0, T)
    W = np.empty((V, H), dtype=np.uint16)
    W_d = torch.empty((V, H), dtype=torch.bfloat16, device="cuda")
    for v0 in range(0, V, 16384):
        n = min(16384, V - v0)
        W[v0:v0 + n] = synth.weight_rows(lw, v0, n)
        W_d[v0:v0 + n].copy_(torch.from_numpy(W[v0:v0 + n]).view(torch.bfloat16))
    return lw, tk, h, W, W_d


def _sampled_rows(r, T):
    rows = np.sort(np.concatenate([c * 8192 + r.choice(8192, 3, replace=False) for c in range(8)]))
    rows[0], rows[-1] = 0, T - 1
    return rows


def test_fused_lmhead_loss_fwd_bwd_full_size(a3po):
    """The benchmark's size (65,536 tokens x hidden 4,096 x vocabulary 151,936, eight chunks of 8,192 tokens), twice.

    (a) A batch the oracle can check in full: every token is counted (the denominator is the whole batch) but only
    24 tokens, three in each chunk, have a non-zero advantage.  Every other token then contributes exactly nothing,
    whatever its log-prob, and the un-rounded fp64 oracle evaluates the 24 rows completely: their log-probs, the
    loss, their rows of dh, and ALL of dW; the other 65,512 rows of dh must be exactly zero.
    (b) The workload's own batch, every counted token live.  The oracle checks what depends on one token at a time:
    log-probs and rows of dh of 24 sampled tokens (their behaviour log-probs come from the oracle; those of the
    other tokens are only there to make the work dense and come from the forward-only entry point).  The weight
    gradient, which mixes all tokens, is checked by a property: every gradient row of the logits sums to zero, so
    every column of dW sums to zero over the vocabulary up to rounding."""
    lw, tk, h, W, W_d = _full_size_inputs()
    T, H, V = lw.tokens.T, lw.H, lw.tokens.V
    cur = synth.CURRENT_VERSION
    r = np.random.default_rng(2512)
    rows = _sampled_rows(r, T)
    k = np.arange(len(rows))
    y = tk["chosen"].copy()
    ver = tk["versions"].copy()
    hs = h[rows]
    z = oracle.lmhead_logits(hs, W)                                  # fp64, never rounded
    fwd = oracle.token_logprobs(z, y[rows].copy())
    ones24 = np.ones(len(rows), dtype=np.uint8)
    dev_ = lambda a: torch.from_numpy(a).cuda()
    h_d = dev_(h).view(torch.bfloat16)
    hf, ha = synth.bf16_bits_to_f64(hs), synth.bf16_bits_to_f64(hs & 0x7FFF)

    def check_dh_rows(out, dz_rows):
        dh_ref, dh_abs = np.zeros((len(rows), H)), np.zeros((len(rows), H))
        for v0 in range(0, V, 16384):
            v1 = min(V, v0 + 16384)
            dh_ref += dz_rows[:, v0:v1] @ synth.bf16_bits_to_f64(W[v0:v1])
            dh_abs += np.abs(dz_rows[:, v0:v1]) @ synth.bf16_bits_to_f64(W[v0:v1] & 0x7FFF)
        got = out["dhidden"][dev_(rows)].float().cpu().numpy().astype(np.float64)
        assert np.abs(dh_ref).max() > 0
        return _check_backward(got, dh_ref, dh_abs, "dh (sampled rows)")

    # ---- (a) 24 live tokens, everything checked ----
    mask = np.ones(T, dtype=np.uint8)
    adv = np.zeros(T, dtype=np.float32)
    adv[rows] = r.choice([-1.0, 1.0], len(rows)) * (0.5 + r.random(len(rows)))
    lb = np.full(T, -12.0, dtype=np.float32)
    lb24 = synth.behav_from_target(fwd["logp"], (r.standard_normal(len(rows)) * 0.15).astype(np.float32))
    lb[rows] = _away_from_clip_bounds(fwd["logp"], lb24, ver[rows], cur, adv[rows], ones24, r, 0.15)
    ref = oracle.loss_fwd_bwd(z, y[rows].copy(), lb[rows], ver[rows], cur, adv[rows], ones24, 0.2, denom=float(T))
    assert (ref["g"] != 0).any()
    out = a3po.fused_lmhead_loss_fwd_bwd(h_d, W_d, dev_(y), dev_(lb), dev_(ver), cur, dev_(adv), dev_(mask), 0.2)
    torch.cuda.synchronize()
    st = a3po.stats_to_dict(out["stats"])
    assert st["n_tokens"] == T and st["n_bad_index"] == 0
    logp = out["logp"].cpu().numpy().astype(np.float64)
    close(logp[rows], ref["logp"], "logp (sampled)")
    assert np.isfinite(logp).all() and (logp <= 0).all()
    loss = float(out["loss"].cpu()[0])
    sur = oracle.surrogate(ref["logp"], lb[rows], ver[rows], cur, adv[rows], ones24, 0.2, float(T))
    assert abs(loss - ref["loss"]) <= 1e-4 * np.abs(sur["obj"]).sum() / T + 1e-12, (loss, ref["loss"])
    # (tokens without advantage are "clipped" or not according to their ratio alone; only the 24 are known here)
    others = torch.ones(T, dtype=torch.bool, device="cuda")
    others[dev_(rows)] = False
    assert not out["dhidden"][others].any(), "a token without advantage must leave its row of dh exactly zero"
    rh = check_dh_rows(out, ref["dz"])
    bad_w, num, den = 0, 0.0, 0.0
    for v0 in range(0, V, 16384):
        v1 = min(V, v0 + 16384)
        dw_ref = ref["dz"][:, v0:v1].T @ hf
        bound = U * np.abs(dw_ref) + (U + 2.0 ** -10) * (np.abs(ref["dz"][:, v0:v1]).T @ ha) + 1e-30
        dw = out["dweight"][v0:v1].float().cpu().numpy().astype(np.float64)
        bad_w += int((np.abs(dw - dw_ref) > bound).sum())
        num += ((dw - dw_ref) ** 2).sum()
        den += (dw_ref ** 2).sum()
    assert bad_w == 0, f"dW: {bad_w} elements off"
    assert np.sqrt(num / den) <= 1e-2
    print(f"lmhead8b (a): loss {loss:.6e} (oracle {ref['loss']:.6e}), norm-wise dh {rh:.2e} dW {np.sqrt(num / den):.2e}")
    del out

    # ---- (b) the workload's own batch: every counted token live ----
    mask = tk["mask"].copy()
    mask[rows] = 1
    adv_seq = oracle.grpo_advantages(tk["rewards"], lw.tokens.G)
    adv = adv_seq[tk["seq_id"]].astype(np.float32)
    adv[rows] = np.where(adv[rows] == 0, 1.0, adv[rows])
    logp_f, _ = a3po.fused_lmhead_logprob(h_d, W_d, dev_(y))
    lb_d = torch.clamp(logp_f + dev_(tk["noise"]), max=0.0)
    lb24 = synth.behav_from_target(fwd["logp"], tk["noise"][rows])
    lb24 = _away_from_clip_bounds(fwd["logp"], lb24, ver[rows], cur, adv[rows], ones24, r, 0.1)
    lb_d[dev_(rows)] = dev_(lb24)
    N = int(mask.sum())
    ref = oracle.loss_fwd_bwd(z, y[rows].copy(), lb24, ver[rows], cur, adv[rows], ones24, 0.2, denom=float(N))
    out = a3po.fused_lmhead_loss_fwd_bwd(h_d, W_d, dev_(y), lb_d.contiguous(), dev_(ver), cur, dev_(adv), dev_(mask), 0.2)
    torch.cuda.synchronize()
    st = a3po.stats_to_dict(out["stats"])
    assert st["n_tokens"] == N
    live = int((out["dhidden"] != 0).any(dim=1).sum().item())
    assert live > 0.5 * N, f"only {live} of {N} counted tokens carry a gradient"
    logp = out["logp"].cpu().numpy().astype(np.float64)
    close(logp[rows], ref["logp"], "logp (sampled, dense batch)")
    rh = check_dh_rows(out, ref["dz"])
    dw = out["dweight"].float()
    col = dw.sum(dim=0, dtype=torch.float64).abs().cpu().numpy()
    col_abs = dw.abs().sum(dim=0, dtype=torch.float64).cpu().numpy()
    # each of the V entries of a column carries at most U of itself in output rounding plus its share of the
    # operand rounding, and the roundings are independent: sqrt(V) U would be typical, 64 x that is the bar
    assert (col <= 64 * U / np.sqrt(V) * col_abs + 1e-30).all(), float((col / col_abs).max())
    assert float(dw.abs().max()) > 0
    print(f"lmhead8b (b): {live} live tokens of {N} counted, norm-wise dh (sampled) {rh:.2e}, "
          f"max |column sum| / column abs sum of dW {float((col / col_abs).max()):.2e}")


def test_fused_lmhead_loss_graph_capture_and_replay(a3po):
    """The whole path from hidden states allocates nothing, never synchronises and clears its buffers with fill
    kernels, so it can be recorded into a HIP graph: every replay reproduces the eager result bit for bit (with the
    program's own eager work and synchronisations between the replays), also after an input changed in place."""
    r = np.random.default_rng(77)
    T, H, V = 9000, 128, 1000                      # two chunks of counted tokens, ragged tiles
    h = torch.from_numpy(bf16_bits(r.standard_normal((T, H)))).view(torch.bfloat16).cuda()
    W = torch.from_numpy(bf16_bits(r.standard_normal((V, H)) * 0.2)).view(torch.bfloat16).cuda()
    y = torch.from_numpy(r.integers(0, V, T).astype(np.int32)).cuda()
    m = torch.from_numpy((r.random(T) < 0.95).astype(np.uint8)).cuda()
    ver = torch.from_numpy((50 - r.integers(0, 5, T)).astype(np.int32)).cuda()
    adv = torch.from_numpy(r.standard_normal(T).astype(np.float32)).cuda()
    lb = (a3po.fused_lmhead_logprob(h, W, y)[0] + 0.05 * torch.randn(T, device="cuda")).clamp(max=0.0)
    keys = ("dhidden", "dweight", "logp", "logp_prox", "loss", "stats")
    eager = a3po.fused_lmhead_loss_fwd_bwd(h, W, y, lb, ver, 50, adv, m, 0.2)
    torch.cuda.synchronize()
    want = {k: eager[k].clone() for k in keys}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        out = a3po.fused_lmhead_loss_fwd_bwd(h, W, y, lb, ver, 50, adv, m, 0.2, workspace=eager["workspace"])
    for rep in range(3):
        for k in keys:
            out[k].zero_()
        a3po.fused_lmhead_logprob(h, W, y)          # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in keys:
            assert torch.equal(out[k].view(torch.uint8), want[k].view(torch.uint8)), (rep, k)
    adv.mul_(-0.5)
    m[::7] = 0                                      # fewer counted tokens: the replay reads the new count on the device
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    fresh = a3po.fused_lmhead_loss_fwd_bwd(h, W, y, lb, ver, 50, adv, m, 0.2)
    torch.cuda.synchronize()
    for k in keys:
        assert torch.equal(out[k].view(torch.uint8), fresh[k].view(torch.uint8)), k
