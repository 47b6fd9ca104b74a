"""GPU parity of the vocabulary-sharded entry points (a3po_shard_partials / _combine / _loss_bwd): the
logits are split by columns in software, every shard goes through the C ABI on its own, and the merged
results must meet the same bars against the CPU oracle of the FULL matrix as the unsharded path does
(the definition of lse, log pi, entropy, loss and gradient does not know about shards).  The partials
themselves are pinned too: the maximum and the gathered logit bit for bit, (max, sum) against the
oracle's lse of the shard alone, (sum exp z) against the oracle's entropy of the shard alone.
"""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")

from test_gpu_parity import CUR, a3po, assert_close_logp, check_against_oracle, dev_logits, make_case  # noqa: E402,F401
from test_gpu_variants import assert_close_entropy, cu  # noqa: E402

pytestmark = pytest.mark.gpu


def host_f64(z_np):
    return z_np.astype(np.float64) if z_np.dtype == np.float32 else synth.bf16_bits_to_f64(z_np)


def run_sharded(a3po, c, bounds, views=True, inplace=False, **kw):
    """Forward partials per shard, merge, backward per shard.  bounds = [0, v1, ..., V]."""
    V, T = c["w"].V, c["T"]
    z_full = dev_logits(c["z"])[:, :V]
    P = len(bounds) - 1
    y = cu(c["chosen"])
    shards = []
    for p in range(P):
        sl = z_full[:, bounds[p]:bounds[p + 1]]
        shards.append(sl if views else sl.contiguous())
    parts = torch.empty((P, T, 4), dtype=torch.float32, device="cuda")
    for p in range(P):
        a3po.shard_partials(shards[p], y, bounds[p], out=parts[p])
    logp, lse, ent = a3po.shard_combine(parts, y, V, want_entropy=True)
    dz_full = torch.full_like(z_full, 5.0) if views and not inplace else None
    outs = []
    for p in range(P):
        if inplace:
            dl = shards[p]
        elif views:
            dl = dz_full[:, bounds[p]:bounds[p + 1]]
        else:
            dl = None
        outs.append(a3po.shard_loss_bwd(shards[p], bounds[p], V, y, logp, lse, cu(c["lb"]), cu(c["versions"]), CUR,
                                        cu(c["adv"]), cu(c["mask"]), c["w"].clip_eps, dlogits=dl, **kw))
    torch.cuda.synchronize()
    if inplace:
        dz = z_full if views else torch.cat(shards, dim=1)
    elif views:
        dz = dz_full
    else:
        dz = torch.cat([o["dlogits"] for o in outs], dim=1)
    return dict(parts=parts, logp=logp, lse=lse, entropy=ent, outs=outs, dlogits=dz, shards=shards)


def check_partials(c, res, bounds):
    V = c["w"].V
    z = host_f64(c["z"][:, :V])
    parts = res["parts"].cpu().numpy()
    raw = c["z"][:, :V]
    for p in range(len(bounds) - 1):
        v0, v1 = bounds[p], bounds[p + 1]
        zs = np.ascontiguousarray(raw[:, v0:v1])
        assert np.array_equal(parts[p, :, 0].astype(np.float64), z[:, v0:v1].max(axis=1)), "shard maximum"
        own = (c["chosen"] >= v0) & (c["chosen"] < v1)
        zy = np.where(own, z[np.arange(c["T"]), np.clip(c["chosen"], 0, V - 1)], 0.0)
        assert np.array_equal(parts[p, :, 2].astype(np.float64), zy), "gathered logit"
        yl = np.where(own, c["chosen"] - v0, 0).astype(np.int32)
        fwd = oracle.token_logprobs(zs, yl)
        lse_p = parts[p, :, 0].astype(np.float64) + np.log(parts[p, :, 1].astype(np.float64))
        assert_close_logp(lse_p, fwd["lse"], f"lse of shard {p}")
        H_p = lse_p - parts[p, :, 3].astype(np.float64) / parts[p, :, 1].astype(np.float64)
        assert_close_entropy(H_p, oracle.entropy(zs), fwd["lse"], f"entropy of shard {p}")


def check_merged(a3po, c, res):
    V = c["w"].V
    fwd = oracle.token_logprobs(c["z"], c["chosen"], V=V)
    assert_close_logp(res["lse"].cpu().numpy(), fwd["lse"], "merged lse")
    assert_close_logp(res["logp"].cpu().numpy(), fwd["logp"], "merged logp")
    assert_close_entropy(res["entropy"].cpu().numpy(), oracle.entropy(c["z"], V=V), fwd["lse"], "merged entropy")
    outs = res["outs"]
    for o in outs[1:]:   # every shard evaluates the same per-token terms: identical bits
        for k in ("loss", "stats", "logp_prox"):
            assert torch.equal(o[k].view(torch.uint8), outs[0][k].view(torch.uint8)), k
    live = torch.from_numpy(c["mask"]).cuda().bool() & (cu(c["chosen"]) >= 0) & (cu(c["chosen"]) < V)
    merged = dict(dlogits=res["dlogits"], logp=torch.where(live, res["logp"], torch.zeros_like(res["logp"])),
                  logp_prox=outs[0]["logp_prox"], loss=outs[0]["loss"], stats=outs[0]["stats"])
    return check_against_oracle(a3po, c, merged)


def test_eight_even_shards_of_the_full_vocabulary_bf16(a3po):
    w = synth.WORKLOADS["1p5b"].scaled(S=8, L=6, G=8, len_lo=3, len_hi=6, noise_std=0.2)
    c = make_case(w)
    bounds = [p * 18992 for p in range(9)]
    assert bounds[-1] == w.V
    res = run_sharded(a3po, c, bounds)
    check_partials(c, res, bounds)
    ref, st, excused = check_merged(a3po, c, res)
    # close to the unsharded kernel as well (not bit-equal: the reduction order differs)
    z = dev_logits(c["z"])
    full = a3po.loss_fwd_bwd(z, cu(c["chosen"]), cu(c["lb"]), cu(c["versions"]), CUR, cu(c["adv"]), cu(c["mask"]),
                             w.clip_eps)
    live = torch.from_numpy(c["mask"]).cuda().bool()
    assert (full["logp"][live] - res["logp"][live]).abs().max().item() < 2e-5
    print(f"8 shards: N={st['n_tokens']} clipped={st['n_clipped']} excused={excused}")


@pytest.mark.parametrize("bounds", [[0, 50000, 110008, 151936],     # one row / two chunks of a row / one row per burst
                                    [0, 50004, 151936]])             # a partial last vector next to a neighbour's
                                                                     # columns; the second base is only 8-byte aligned
def test_uneven_shards_bf16(a3po, bounds):
    w = synth.WORKLOADS["1p5b"].scaled(S=8, L=4, G=8, len_lo=2, len_hi=4, noise_std=0.3)
    c = make_case(w)
    c["chosen"][1] = bounds[1] - 1        # last column of the first shard
    c["chosen"][2] = bounds[1]            # first column of the second
    fwd = oracle.token_logprobs(c["z"], c["chosen"], V=w.V)
    c["lb"] = synth.behav_from_target(fwd["logp"], c["tk"]["noise"][:c["T"]])
    res = run_sharded(a3po, c, bounds)
    check_partials(c, res, bounds)
    check_merged(a3po, c, res)
    assert not (res["dlogits"].float() == 5.0).any(), "every column was written by exactly its own shard"


@pytest.mark.parametrize("dtype,V,bounds", [
    ("f32", 32000, [0, 8000, 16000, 24000, 32000]),
    ("f32", 4099, [0, 1001, 2002, 4099]),            # odd widths: element-wise path
    ("bf16", 5001, [0, 3, 4, 2500, 5001]),           # tiny shards, one of a single column
    ("bf16", 70000, [0, 70000]),                     # a single shard is the whole vocabulary
    ("f32", 70000, [0, 70000]),                      # 17,500 vectors per row: three column chunks per row
    ("bf16", 163848, [0, 163848]),                   # 20,481 vectors per row: three chunks, the last vector whole
    ("bf16", 45, [0, 21, 30, 37, 45]),               # a shard of exactly one 16-byte vector per row (8 columns)
    ("f32", 20, [0, 4, 8, 20]),                      # the same in fp32 (4 columns), next to a three-vector shard
])
def test_contiguous_shards(a3po, dtype, V, bounds):
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=4, L=8, len_lo=4, len_hi=8, sigma=3.0, boost=6.0,
                                       boost_prob=0.5, noise_std=0.2, stale_max=5)
    c = make_case(w)
    c["chosen"][2] = bounds[1]            # first column of a shard
    c["chosen"][3] = bounds[1] - 1        # last column of a shard
    fwd = oracle.token_logprobs(c["z"], c["chosen"], V=V)
    c["lb"] = synth.behav_from_target(fwd["logp"], c["tk"]["noise"][:c["T"]])
    res = run_sharded(a3po, c, bounds, views=False)
    check_partials(c, res, bounds)
    check_merged(a3po, c, res)


@pytest.mark.parametrize("dtype,V,pad,bounds", [
    # column offsets at every kind of position inside a 128-byte line, a row stride that is not a multiple of
    # 128 bytes (the position changes from row to row), a partial last vector
    ("bf16", 9003, 5, [0, 1032, 3120, 5208, 9003]),
    ("f32", 5000, 4, [0, 516, 1100, 5000]),
    # a row of several column chunks that starts one vector into a line, next to a shard of one vector
    ("bf16", 163856, 0, [0, 8, 163856]),
    # row stride a multiple of 128 bytes: the same position in every row
    ("bf16", 8192, 0, [0, 1096, 4112, 8192]),
])
def test_column_views_at_any_position_inside_a_cache_line(a3po, dtype, V, pad, bounds):
    """The backward maps a wavefront's stores onto whole 128-byte lines of the gradient, whatever the column
    offset and row stride of the view (shards of at least 128 vectors per row): every column must still be
    written exactly once by its own shard, and nothing outside the view."""
    w = synth.WORKLOADS["tiny"].scaled(V=V, dtype=dtype, S=4, L=40, len_lo=20, len_hi=40, sigma=3.0, boost=6.0,
                                       boost_prob=0.5, noise_std=0.2, stale_max=5)
    c = make_case(w, ld=V + pad)
    T = c["T"]
    c["chosen"][2] = bounds[1]
    c["chosen"][3] = bounds[1] - 1
    c["chosen"][4] = V - 1
    fwd = oracle.token_logprobs(c["z"], c["chosen"], V=V)
    c["lb"] = synth.behav_from_target(fwd["logp"], c["tk"]["noise"][:T])
    z_buf = dev_logits(c["z"])                                   # [T, V + pad]
    dz_buf = torch.full_like(z_buf, 5.0)
    y = cu(c["chosen"])
    P = len(bounds) - 1
    parts = torch.empty((P, T, 4), dtype=torch.float32, device="cuda")
    for p in range(P):
        a3po.shard_partials(z_buf[:, bounds[p]:bounds[p + 1]], y, bounds[p], out=parts[p])
    logp, lse, ent = a3po.shard_combine(parts, y, V, want_entropy=True)
    outs = [a3po.shard_loss_bwd(z_buf[:, bounds[p]:bounds[p + 1]], bounds[p], V, y, logp, lse, cu(c["lb"]),
                                cu(c["versions"]), CUR, cu(c["adv"]), cu(c["mask"]), w.clip_eps,
                                dlogits=dz_buf[:, bounds[p]:bounds[p + 1]]) for p in range(P)]
    torch.cuda.synchronize()
    assert (dz_buf[:, V:].float() == 5.0).all(), "padding columns are not the library's to write"
    assert not (dz_buf[:, :V].float() == 5.0).any()
    res = dict(parts=parts, logp=logp, lse=lse, entropy=ent, outs=outs, dlogits=dz_buf[:, :V])
    check_merged(a3po, c, res)
    # one shard alone, into a buffer of its own: the neighbours' columns stay as they were
    for p in range(P):
        alone = torch.full_like(z_buf, 7.0)
        a3po.shard_loss_bwd(z_buf[:, bounds[p]:bounds[p + 1]], bounds[p], V, y, logp, lse, cu(c["lb"]),
                            cu(c["versions"]), CUR, cu(c["adv"]), cu(c["mask"]), w.clip_eps,
                            dlogits=alone[:, bounds[p]:bounds[p + 1]])
        torch.cuda.synchronize()
        assert (alone[:, :bounds[p]].float() == 7.0).all() and (alone[:, bounds[p + 1]:].float() == 7.0).all()
        assert torch.equal(alone[:, bounds[p]:bounds[p + 1]], dz_buf[:, bounds[p]:bounds[p + 1]])


def test_in_place_and_bad_ids_and_variants(a3po):
    w = synth.WORKLOADS["tiny"].scaled(V=32000, S=4, L=16, len_lo=8, len_hi=16, noise_std=0.3)
    c = make_case(w, T=48)
    c["mask"][:] = 1
    c["chosen"][[3, 17]] = [-1, w.V]
    c["versions"][[5, 6]] = CUR + 2
    c["adv"][[8, 9]] = 0.0
    bounds = [0, 16000, 32000]
    sep = run_sharded(a3po, c, bounds)
    ref, st, _ = check_merged(a3po, c, sep)
    assert st["n_bad_index"] == 2 and st["n_negative_staleness"] == 2 and st["n_tokens"] == 46
    assert not sep["dlogits"][[3, 17, 8, 9]].any()
    inp = run_sharded(a3po, c, bounds, inplace=True)
    assert torch.equal(sep["dlogits"].view(torch.uint8), inp["dlogits"].contiguous().view(torch.uint8))
    # coupled objective through the sharded backward == unsharded coupled objective (per-token terms are shared code
    # paths only on the GPU side; the oracle comparison of that variant lives in test_gpu_variants.py)
    cpl = run_sharded(a3po, c, bounds, prox_mode=a3po.A3PO_PROX_BEHAV, want_iw=True)
    full = a3po.loss_fwd_bwd(dev_logits(c["z"]), cu(c["chosen"]), cu(c["lb"]), None, CUR, cu(c["adv"]), cu(c["mask"]),
                             w.clip_eps, prox_mode=a3po.A3PO_PROX_BEHAV)
    lf, ls = float(full["loss"].cpu()[0]), float(cpl["outs"][0]["loss"].cpu()[0])
    assert abs(lf - ls) <= 1e-5 * abs(lf) + 1e-6
    assert (cpl["outs"][0]["iw"].cpu().numpy()[[0, 1, 2]] == 1.0).all()


def test_shard_host_validation(a3po):
    z = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    y = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(a3po.A3poError) as e:
        a3po.shard_partials(z, y, -1)
    assert e.value.code == -2
    f = torch.zeros(4, dtype=torch.float32, device="cuda")
    m = torch.ones(4, dtype=torch.uint8, device="cuda")
    with pytest.raises(a3po.A3poError) as e:      # shard reaches past the vocabulary
        a3po.shard_loss_bwd(z, 10, 64, y, f, f, f, y, 1, f, m, 0.2)
    assert e.value.code == -2
    # a column view whose base is only element-aligned is legal: it takes the element-wise path
    zz = torch.randn((4, 64), dtype=torch.float32, device="cuda")
    part = a3po.shard_partials(zz[:, 1:33], y, 1)
    torch.cuda.synchronize()
    assert torch.equal(part[:, 0], zz[:, 1:33].max(dim=1).values)
