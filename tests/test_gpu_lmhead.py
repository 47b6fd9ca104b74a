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
                                   (1100, 256, 4500), (2048, 128, 2304)])
def test_fused_lmhead_logprob_small(a3po, T, H, V):
    # spans: single partial tile, exact tile multiples, ragged token and vocabulary tiles, several
    # token tiles per XCD group and more vocabulary tiles than the stride of 8
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


# ------------------------------------------------------------------------------------------ forward + backward

def _bf16_round(x):
    """float64 array -> nearest bfloat16 (RNE) as bit patterns and as float64 values"""
    bits = bf16_bits(x)
    return bits, synth.bf16_bits_to_f64(bits)


def _bf16_ulp(x):
    """spacing of bfloat16 at |x| (8 significant bits)"""
    a = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


@pytest.mark.parametrize("T,H,V", [(300, 64, 1000), (1, 8, 8), (8192 + 300, 64, 512), (467, 224, 1344)])
def test_fused_lmhead_loss_fwd_bwd(a3po, T, H, V):
    """The oracle follows the same staging as the GPU path (logits rounded once to bfloat16, gradient
    rows rounded to bfloat16 before the two contractions), in fp64 otherwise.  What the two cannot
    share is the side of a rounding tie: the GPU rounds an fp32-accumulated logit, the oracle an fp64
    one, so a logit within the fp32 accumulation error (H u sum_k |h||W|, u = 2^-24) of a bfloat16
    rounding boundary may come out one ulp apart ("tie" below).  Error model, per element:
      log-probs  1e-5-ish, plus for a tied chosen logit its ulp, plus the shift of lse a tied logit causes
                 (p ulp): dev_t.  A clip decision is compared only when log r is further than 1e-3 + dev_t
                 from both clip bounds; rows of such tokens are left out of dh, and dW is then not compared.
      dh, dW     2^-7 |ref|                      bfloat16 rounding of the output
               + 2^-8 sum |dz| |operand|         every gradient entry may round the other way (fp32 vs fp64 value)
               + sum over tied (t, v) of |g_t| p ulp(z) |operand|      the entry of a tied logit itself
               + sum_t dev_t |dz| |operand|      every entry of a row whose lse moved."""
    r = np.random.default_rng(T + 7 * V)
    cur = 50
    h = bf16_bits(r.standard_normal((T, H)))
    W = bf16_bits(r.standard_normal((V, H)) * (2.0 / np.sqrt(H)))
    y = r.integers(0, V, T).astype(np.int32)
    mask = (r.random(T) < 0.8).astype(np.uint8)
    mask[0] = 1
    ver = (cur - r.integers(0, 5, T)).astype(np.int32)
    adv = r.standard_normal(T).astype(np.float32)
    z = oracle.lmhead_logits(h, W)
    zb, zr = _bf16_round(z)
    lt = oracle.token_logprobs(zb, y)["logp"]
    lb = synth.behav_from_target(lt, (r.standard_normal(T) * 0.15).astype(np.float32))
    ref = oracle.loss_fwd_bwd(zb, y, lb, ver, cur, adv, mask, 0.2)
    dzb, dzr = _bf16_round(ref["dz"])
    dh_ref, dw_ref = oracle.lmhead_backward(dzr, h, W)
    dh_abs, dw_abs = oracle.lmhead_backward(np.abs(dzr), h & 0x7FFF, W & 0x7FFF)

    # logits the two roundings may disagree on, and what that does to each row
    z_abs = oracle.lmhead_logits(h & 0x7FFF, W & 0x7FFF)
    ulp = _bf16_ulp(z)
    tie = np.abs(np.abs(z - zr) - 0.5 * ulp) <= H * 2.0 ** -24 * z_abs + 1e-300
    p = np.exp(zr - ref["lse"][:, None])
    dev = (tie * p * ulp).sum(axis=1) + tie[np.arange(T), y] * ulp[np.arange(T), y]     # |delta log pi| per token
    direct = tie * np.abs(ref["g"])[:, None] * p * ulp                                    # |delta dz| of the tied entries
    dh_tie, dw_tie = oracle.lmhead_backward(direct + dev[:, None] * np.abs(dzr), h & 0x7FFF, W & 0x7FFF)

    dev_ = lambda a: torch.from_numpy(a).cuda()
    out = a3po.fused_lmhead_loss_fwd_bwd(dev_(h).view(torch.bfloat16), dev_(W).view(torch.bfloat16), dev_(y), dev_(lb),
                                         dev_(ver), cur, dev_(adv), dev_(mask), 0.2)
    torch.cuda.synchronize()
    st = a3po.stats_to_dict(out["stats"])
    assert st["n_tokens"] == ref["stats"]["n_tokens"]
    logp = out["logp"].cpu().numpy().astype(np.float64)
    assert (np.abs(logp - ref["logp"]) <= (2e-5 + 1e-5 * np.abs(ref["logp"]) + dev) * (mask == 1) + 1e-30).all()
    assert np.quantile(np.abs(logp - ref["logp"]), 0.99) < 2e-5
    N = max(1, st["n_tokens"])
    loss = float(out["loss"].cpu()[0])
    sur = oracle.surrogate(ref["logp"], lb, ver, cur, adv, ref["eff_mask"], 0.2)
    near = ((np.abs(np.log(sur["r"]) - np.log(1.2)) < 1e-3 + dev) |
            (np.abs(np.log(sur["r"]) - np.log(0.8)) < 1e-3 + dev)) & (ref["eff_mask"] == 1)
    scale = (np.abs(sur["obj"]) * ref["eff_mask"]).sum() / N
    slack = (np.abs(sur["obj"]) * (dev + near * 0.5)).sum() / N       # a token's objective moves with its log-prob
    assert abs(loss - ref["loss"]) <= 1e-4 * scale + slack + 1e-6, (loss, ref["loss"])
    dh = out["dhidden"].float().cpu().numpy().astype(np.float64)
    dw = out["dweight"].float().cpu().numpy().astype(np.float64)
    bad_h = np.abs(dh - dh_ref) > 2.0 ** -7 * np.abs(dh_ref) + 2.0 ** -8 * dh_abs + dh_tie + 1e-30
    bad_w = np.abs(dw - dw_ref) > 2.0 ** -7 * np.abs(dw_ref) + 2.0 ** -8 * dw_abs + dw_tie + 1e-30
    assert not bad_h[~near].any(), f"dh: {bad_h[~near].sum()} elements off"
    if not near.any():
        assert not bad_w.any(), f"dW: {bad_w.sum()} elements off"
    assert np.abs(dh_ref).max() > 0 and np.abs(dw_ref).max() > 0
    # the model stays sharp: what the ties add (many of them at logits near zero, whose ulp is tiny) is small beside
    # the rounding terms
    assert np.median(dw_tie / (2.0 ** -8 * dw_abs + 1e-300)) < 1.0 and np.median(dh_tie / (2.0 ** -8 * dh_abs + 1e-300)) < 1.0


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


def test_fused_lmhead_loss_fwd_bwd_full_size(a3po):
    """The whole path from hidden states at the benchmark's size (65,536 tokens x hidden 4,096 x vocabulary
    151,936, eight chunks of 8,192 tokens).  The oracle cannot run the projection for every token, so the case
    is built to be checkable in full: every token is counted (the denominator is the whole batch), but only 24
    tokens, three in each chunk, have a non-zero advantage.  Every other token then contributes exactly nothing to
    the loss and to the gradients, whatever its log-prob is, and the oracle evaluates the 24 rows completely:
    their log-probs, the loss, their rows of dh, and ALL of dW; the other 65,512 rows of dh must be exactly zero.
    Error model as in test_fused_lmhead_loss_fwd_bwd."""
    lw = synth.LMHEAD_WORKLOADS["lmhead8b"]
    T, H, V = lw.tokens.T, lw.H, lw.tokens.V
    assert (T, H, V) == (65536, 4096, 151936)
    tk = synth.token_arrays(lw.tokens)
    cur = synth.CURRENT_VERSION
    h = synth.hidden_rows(lw, 0, T)
    W = np.empty((V, H), dtype=np.uint16)
    W_d = torch.empty((V, H), dtype=torch.bfloat16, device="cuda")
    for v0 in range(0, V, 16384):
        n = min(16384, V - v0)
        W[v0:v0 + n] = synth.weight_rows(lw, v0, n)
        W_d[v0:v0 + n].copy_(torch.from_numpy(W[v0:v0 + n]).view(torch.bfloat16))
    r = np.random.default_rng(2512)
    rows = np.sort(np.concatenate([c * 8192 + r.choice(8192, 3, replace=False) for c in range(8)]))
    rows[0], rows[-1] = 0, T - 1
    y = tk["chosen"].copy()
    mask = np.ones(T, dtype=np.uint8)
    ver = tk["versions"].copy()
    adv = np.zeros(T, dtype=np.float32)
    adv[rows] = r.choice([-1.0, 1.0], len(rows)) * (0.5 + r.random(len(rows)))

    # oracle on the 24 rows, with the GPU path's staging (logits and gradient entries rounded once to bfloat16)
    hs = h[rows]
    z = oracle.lmhead_logits(hs, W)
    zb, zr = _bf16_round(z)
    fwd = oracle.token_logprobs(zb, y[rows].copy())
    lb = np.full(T, -12.0, dtype=np.float32)
    lb[rows] = synth.behav_from_target(fwd["logp"], (r.standard_normal(len(rows)) * 0.15).astype(np.float32))
    ref = oracle.loss_fwd_bwd(zb, y[rows].copy(), lb[rows], ver[rows], cur, adv[rows], np.ones(len(rows), dtype=np.uint8),
                              0.2, denom=float(T))
    dzb, dzr = _bf16_round(ref["dz"])
    z_abs = oracle.lmhead_logits(hs & 0x7FFF, W & 0x7FFF)
    ulp = _bf16_ulp(z)
    tie = np.abs(np.abs(z - zr) - 0.5 * ulp) <= H * 2.0 ** -24 * z_abs + 1e-300
    p = np.exp(zr - ref["lse"][:, None])
    k = np.arange(len(rows))
    dev = (tie * p * ulp).sum(axis=1) + tie[k, y[rows]] * ulp[k, y[rows]]
    direct = tie * np.abs(ref["g"])[:, None] * p * ulp
    extra = direct + dev[:, None] * np.abs(dzr)
    sur = oracle.surrogate(ref["logp"], lb[rows], ver[rows], cur, adv[rows], np.ones(len(rows), dtype=np.uint8), 0.2,
                           float(T))
    near = (np.abs(np.log(sur["r"]) - np.log(1.2)) < 1e-3 + dev) | (np.abs(np.log(sur["r"]) - np.log(0.8)) < 1e-3 + dev)
    assert not near.all() and (ref["g"] != 0).any()

    dev_ = lambda a: torch.from_numpy(a).cuda()
    out = a3po.fused_lmhead_loss_fwd_bwd(dev_(h).view(torch.bfloat16), W_d, dev_(y), dev_(lb), dev_(ver), cur, dev_(adv),
                                         dev_(mask), 0.2)
    torch.cuda.synchronize()
    st = a3po.stats_to_dict(out["stats"])
    assert st["n_tokens"] == T and st["n_bad_index"] == 0
    logp = out["logp"].cpu().numpy().astype(np.float64)
    assert (np.abs(logp[rows] - ref["logp"]) <= 2e-5 + 1e-5 * np.abs(ref["logp"]) + dev).all()
    assert np.isfinite(logp).all() and (logp <= 0).all()
    loss = float(out["loss"].cpu()[0])
    scale = np.abs(sur["obj"]).sum() / T
    slack = (np.abs(sur["obj"]) * (dev + near * 0.5)).sum() / T
    assert abs(loss - ref["loss"]) <= 1e-4 * scale + slack + 1e-9, (loss, ref["loss"])
    assert abs(st["n_clipped"] - int(ref["stats"]["n_clipped"])) <= int(near.sum())

    dh = out["dhidden"]
    others = torch.ones(T, dtype=torch.bool, device="cuda")
    others[dev_(rows)] = False
    assert not dh[others].any(), "a token without advantage must leave its row of dh exactly zero"
    hf, ha = synth.bf16_bits_to_f64(hs), synth.bf16_bits_to_f64(hs & 0x7FFF)
    dh_ref, dh_abs, dh_tie = np.zeros((len(rows), H)), np.zeros((len(rows), H)), np.zeros((len(rows), H))
    bad_w = 0
    ok = ~near
    for v0 in range(0, V, 16384):
        v1 = min(V, v0 + 16384)
        Wf, Wa = synth.bf16_bits_to_f64(W[v0:v1]), synth.bf16_bits_to_f64(W[v0:v1] & 0x7FFF)
        dh_ref += dzr[:, v0:v1] @ Wf
        dh_abs += np.abs(dzr[:, v0:v1]) @ Wa
        dh_tie += extra[:, v0:v1] @ Wa
        if ok.all():
            dw_ref = dzr[:, v0:v1].T @ hf
            bound = 2.0 ** -7 * np.abs(dw_ref) + 2.0 ** -8 * (np.abs(dzr[:, v0:v1]).T @ ha) + extra[:, v0:v1].T @ ha + 1e-30
            dw = out["dweight"][v0:v1].float().cpu().numpy().astype(np.float64)
            bad_w += int((np.abs(dw - dw_ref) > bound).sum())
    got = dh[dev_(rows)].float().cpu().numpy().astype(np.float64)
    bad_h = np.abs(got - dh_ref) > 2.0 ** -7 * np.abs(dh_ref) + 2.0 ** -8 * dh_abs + dh_tie + 1e-30
    assert not bad_h[ok].any(), f"dh: {bad_h[ok].sum()} elements off"
    assert bad_w == 0, f"dW: {bad_w} elements off"
    assert np.abs(dh_ref).max() > 0
    # the forward-only kernel at the same size: fp32 logits on chip, so the 24 rows are compared with the
    # un-rounded fp64 products; every other token must agree with the chunked path up to its bf16 staging
    logp_f, lse_f = a3po.fused_lmhead_logprob(dev_(h).view(torch.bfloat16), W_d, dev_(y))
    torch.cuda.synchronize()
    exact = oracle.token_logprobs(z, y[rows].copy())
    close(lse_f.cpu().numpy()[rows], exact["lse"], "lse (forward only, full size)")
    close(logp_f.cpu().numpy()[rows], exact["logp"], "logp (forward only, full size)")
    assert (logp_f - out["logp"]).abs().max().item() < 5e-2
    print(f"lmhead8b full size: loss {loss:.6e} (oracle {ref['loss']:.6e}), {int(near.sum())} of {len(rows)} sampled tokens "
          f"in the clip band, dW compared on {'all' if ok.all() else 'no'} elements")
