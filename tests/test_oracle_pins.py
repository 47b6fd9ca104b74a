"""Pins of the CPU oracle against facts that do not come from the oracle.

Each test fixes one part of ``oracle/a3po_oracle.c`` to something the paper or the
mathematics determines: closed forms, hand-worked values of Eq. 2 - Eq. 4 stored under
``tests/golden``, the sandwich property and the closed-form ratio of Section 3.1 /
Appendix A, the staleness limits of Section 3, brute force on tiny vocabularies,
central finite differences, and independent library routines (SciPy, PyTorch fp64).
"""
import math
import os

import numpy as np
import pytest
import scipy.special

import oracle
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


def _rows(path):
    out = []
    for line in open(os.path.join(GOLD, path)):
        line = line.split("#")[0].strip()
        if line:
            out.append(line.split())
    return out


def bf16_bits(x):
    """float -> nearest bfloat16 bit pattern (RNE), via float32 bit arithmetic."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


# ----------------------------------------------------------------------------- log-softmax + gather

def test_logsoftmax_normalises_to_one():
    z = (rng.standard_normal((5, 4097)) * 3).astype(np.float32)
    y = rng.integers(0, 4097, 5).astype(np.int32)
    o = oracle.token_logprobs(z, y)
    for t in range(5):
        s = math.fsum(np.exp(z[t].astype(np.float64) - o["lse"][t]))
        assert abs(s - 1.0) < 1e-12


def test_constant_row_is_minus_log_v():
    for V in (1, 2, 7, 1000, 32000):
        z = np.full((2, V), 3.25, dtype=np.float32)
        o = oracle.token_logprobs(z, np.array([0, V - 1], dtype=np.int32))
        assert np.allclose(o["logp"], -math.log(V), rtol=0, atol=1e-13)
        assert np.allclose(o["lse"], 3.25 + math.log(V), rtol=0, atol=1e-13)


def test_single_token_vocabulary_has_probability_one():
    z = np.array([[-17.5]], dtype=np.float32)
    o = oracle.token_logprobs(z, np.array([0], dtype=np.int32))
    assert o["logp"][0] == 0.0 and o["lse"][0] == -17.5


def test_shift_invariance():
    z = (rng.standard_normal((3, 513)) * 2).astype(np.float32)
    y = rng.integers(0, 513, 3).astype(np.int32)
    a = oracle.token_logprobs(z, y)
    b = oracle.token_logprobs((z.astype(np.float64) + 64.0).astype(np.float32), y)  # exact shift
    assert np.allclose(a["logp"], b["logp"], rtol=0, atol=1e-5)  # fp32 re-rounding of z+64 only
    z2 = np.round(z * 8) / 8  # multiples of 1/8 so that +64 is exact in fp32
    a = oracle.token_logprobs(z2.astype(np.float32), y)
    b = oracle.token_logprobs((z2 + 64).astype(np.float32), y)
    assert np.allclose(a["logp"], b["logp"], rtol=0, atol=1e-12)
    assert np.allclose(a["lse"] + 64, b["lse"], rtol=0, atol=1e-12)


def test_brute_force_tiny_vocabularies():
    for V in range(2, 9):
        z = (rng.standard_normal((4, V)) * 4).astype(np.float32)
        y = rng.integers(0, V, 4).astype(np.int32)
        o = oracle.token_logprobs(z, y)
        for t in range(4):
            naive = math.log(math.fsum(math.exp(float(v)) for v in z[t]))
            assert abs(o["lse"][t] - naive) < 1e-13 * max(1, abs(naive))
            assert abs(o["logp"][t] - (float(z[t, y[t]]) - naive)) < 1e-12


def test_large_logits_do_not_overflow():
    z = np.array([[1000.0, 999.0, -1000.0]], dtype=np.float32)
    o = oracle.token_logprobs(z, np.array([1], dtype=np.int32))
    assert abs(o["lse"][0] - (1000.0 + math.log1p(math.exp(-1.0)))) < 1e-12
    assert abs(o["logp"][0] - (-1.0 - math.log1p(math.exp(-1.0)))) < 1e-12


def test_against_scipy_and_torch_fp64_on_tiny_workload():
    torch = pytest.importorskip("torch")
    w = synth.WORKLOADS["tiny"]
    tk = synth.token_arrays(w)
    z = synth.logit_rows(w, 0, 64, tk["chosen"])
    y = tk["chosen"][:64]
    o = oracle.token_logprobs(z, y)
    lse = scipy.special.logsumexp(z.astype(np.float64), axis=1)
    assert np.allclose(o["lse"], lse, rtol=0, atol=1e-12)
    ce = torch.nn.functional.cross_entropy(torch.from_numpy(z).double(),
                                           torch.from_numpy(y.astype(np.int64)), reduction="none")
    assert np.allclose(o["logp"], -ce.numpy(), rtol=0, atol=1e-12)


def test_bf16_bit_patterns_decode_exactly():
    # 0x3F80 = 1, 0xC000 = -2, 0x4049 = 3.140625, 0x0000 = 0
    z = np.array([[0x3F80, 0xC000, 0x4049, 0x0000]], dtype=np.uint16)
    vals = [1.0, -2.0, 3.140625, 0.0]
    naive = math.log(math.fsum(math.exp(v) for v in vals))
    for k in range(4):
        o = oracle.token_logprobs(z, np.array([k], dtype=np.int32))
        assert abs(o["lse"][0] - naive) < 1e-13
        assert abs(o["logp"][0] - (vals[k] - naive)) < 1e-13
        assert o["chosen_raw"][0] == z[0, k]


def test_bf16_matches_f32_of_same_values():
    zf = (rng.standard_normal((6, 777)) * 3).astype(np.float32)
    zb = bf16_bits(zf)
    zf_rounded = (zb.astype(np.uint32) << 16).view(np.float32)
    y = rng.integers(0, 777, 6).astype(np.int32)
    a = oracle.token_logprobs(zb, y)
    b = oracle.token_logprobs(zf_rounded, y)
    assert np.array_equal(a["logp"], b["logp"]) and np.array_equal(a["lse"], b["lse"])


def test_row_stride_padding_is_ignored():
    V, ld = 301, 320
    z = np.full((3, ld), 1e30, dtype=np.float32)
    core = (rng.standard_normal((3, V))).astype(np.float32)
    z[:, :V] = core
    y = np.array([0, 150, 300], dtype=np.int32)
    a = oracle.token_logprobs(z, y, V=V)
    b = oracle.token_logprobs(core, y)
    assert np.array_equal(a["logp"], b["logp"])


def test_gather_is_a_raw_copy_and_bad_index_is_flagged():
    z = (rng.standard_normal((4, 50))).astype(np.float32)
    y = np.array([3, 49, -1, 50], dtype=np.int32)
    o = oracle.token_logprobs(z, y)
    assert o["chosen_raw"][0] == z[0, 3].view(np.uint32)
    assert o["chosen_raw"][1] == z[1, 49].view(np.uint32)
    assert o["chosen_raw"][2] == 0 and o["chosen_raw"][3] == 0
    assert o["logp"][2] == 0.0 and o["logp"][3] == 0.0
    assert np.isfinite(o["lse"]).all()


# ----------------------------------------------------------------------------- alpha (Eq. 4)

def test_alpha_matches_eq4_table():
    for d, num, den in _rows("eq4_alpha_table.txt"):
        d, num, den = int(d), int(num), int(den)
        a = oracle.alpha(np.array([100 - d], dtype=np.int32), 100)[0]
        assert a == num / den


def test_alpha_is_non_increasing_in_staleness():
    d = np.arange(0, 200)
    a = oracle.alpha((1000 - d).astype(np.int32), 1000)
    assert (np.diff(a) <= 0).all() and a[0] == 1.0 and a[1] == 1.0 and (a > 0).all()


def test_alpha_extreme_versions_do_not_overflow():
    a = oracle.alpha(np.array([-2**31, 2**31 - 1], dtype=np.int32), 2**31 - 1)
    assert a[0] == 1.0 / (2.0**32 - 1) and a[1] == 1.0


# ----------------------------------------------------------------------------- proximal interpolation (Eq. 3)

def _random_logps(n):
    lt = -np.abs(rng.standard_normal(n) * 4) - 1e-3
    lb = np.minimum(0.0, lt + rng.standard_normal(n) * 0.5)
    return lt, lb


def test_sandwich_property():
    n = 5000
    lt, lb = _random_logps(n)
    ver = (100 - rng.integers(0, 40, n)).astype(np.int32)
    lp, al = oracle.proximal_interp(lb, lt, ver, 100)
    lo, hi = np.minimum(lb, lt), np.maximum(lb, lt)
    slack = 4 * np.spacing(np.maximum(np.abs(lb), np.abs(lt)))
    assert (lp >= lo - slack).all() and (lp <= hi + slack).all()
    # strictly inside when 0 < alpha < 1 and the two policies differ visibly
    inner = (al < 1) & (np.abs(lb - lt) > 1e-6)
    assert (lp[inner] > lo[inner]).all() and (lp[inner] < hi[inner]).all()


def test_zero_and_unit_staleness_recover_behaviour_policy():
    lt, lb = _random_logps(100)
    for d in (0, 1):
        lp, al = oracle.proximal_interp(lb, lt, np.full(100, 7 - d, dtype=np.int32), 7)
        assert np.array_equal(lp, lb) and (al == 1).all()


def test_interpolation_weights_are_not_swapped():
    # d = 4: lp = lb/4 + 3 lt/4 -- closer to the target policy (Section 3)
    lp, _ = oracle.proximal_interp(np.array([-4.0]), np.array([-8.0]), np.array([6], dtype=np.int32), 10)
    assert lp[0] == -7.0


def test_huge_staleness_approaches_target_policy():
    lt, lb = _random_logps(50)
    d = 2**20
    lp, _ = oracle.proximal_interp(lb, lt, np.full(50, -d, dtype=np.int32), 0)
    assert (np.abs(lp - lt) <= 2.0**-20 * np.abs(lt - lb) * (1 + 1e-9) + 8 * np.spacing(np.abs(lt) + np.abs(lb))).all()


# ----------------------------------------------------------------------------- ratios (Section 3.1, Appendix A)

def test_ratio_identities():
    n = 2000
    lt, lb = _random_logps(n)
    ver = (50 - rng.integers(0, 20, n)).astype(np.int32)
    A = rng.standard_normal(n)
    o = oracle.surrogate(lt, lb, ver, 50, A, np.ones(n, np.uint8), 0.2)
    w = np.exp(lt - lb)
    al = oracle.alpha(ver, 50)
    assert np.allclose(o["r"] * o["iw"], w, rtol=1e-12)
    assert np.allclose(o["r"], w ** al, rtol=1e-12)
    assert np.allclose(o["iw"], w ** (1 - al), rtol=1e-12)


def test_infinite_staleness_limit_never_clips():
    n = 500
    lt, lb = _random_logps(n)
    A = rng.standard_normal(n)
    o = oracle.surrogate(lt, lb, np.full(n, -(2**30), dtype=np.int32), 0, A, np.ones(n, np.uint8), 0.2)
    assert np.abs(o["r"] - 1).max() < 1e-6
    assert o["stats"]["n_clipped"] == 0 and not o["clipped"].any()


def test_contraction_of_the_ratio_with_staleness():
    """Appendix A, contractive stability: r = w^alpha lies between 1 and w, so (r - 1)^2 <= (w - 1)^2 token by
    token (the dominating function of the proof); on a fixed batch the second moment of r - 1 and the number
    of clipped tokens do not grow with the staleness (Section 3.1), and both vanish in the limit."""
    n = 4000
    lt, lb = _random_logps(n)
    A = rng.standard_normal(n)
    w = np.exp(lt - lb)
    ones = np.ones(n, np.uint8)
    spread, clipped = [], []
    for d in (1, 2, 3, 4, 8, 16, 64, 1024, 2 ** 20):
        o = oracle.surrogate(lt, lb, np.full(n, 100 - d, dtype=np.int32), 100, A, ones, 0.2)
        r = o["r"]
        assert (np.minimum(1.0, w) * (1 - 1e-12) <= r).all() and (r <= np.maximum(1.0, w) * (1 + 1e-12)).all()
        assert ((r - 1) ** 2 <= (w - 1) ** 2 * (1 + 1e-9) + 1e-15).all()
        spread.append(((r - 1) ** 2).mean())
        clipped.append(o["stats"]["n_clipped"])
    assert spread[0] == pytest.approx(((w - 1) ** 2).mean(), rel=1e-12)      # d = 1: r = w
    assert all(a >= b for a, b in zip(spread, spread[1:])) and spread[-1] < 1e-9
    assert all(a >= b for a, b in zip(clipped, clipped[1:])) and clipped[0] > 0 and clipped[-1] == 0


# ----------------------------------------------------------------------------- loss (Eq. 2) and stats

def test_worked_tokens_of_eq2():
    for pt, pb, d, A, obj, clipped, dobj in _rows("eq2_worked_tokens.txt"):
        pt, pb, A, obj, dobj = map(float, (pt, pb, A, obj, dobj))
        d, clipped = int(d), int(clipped)
        o = oracle.surrogate([math.log(pt)], [math.log(pb)], np.array([10 - d], dtype=np.int32), 10,
                             [A], np.ones(1, np.uint8), 0.2)
        assert abs(o["obj"][0] - obj) < 1e-14
        assert o["clipped"][0] == clipped
        assert abs(o["loss"] - (-obj)) < 1e-14           # N = 1, loss = -objective
        assert abs(o["g"][0] - (-dobj)) < 1e-14          # gradient of the loss
        assert o["stats"]["n_clipped"] == clipped and o["stats"]["n_tokens"] == 1


def _coupled_ppo_objective(lt, lold, A, eps, mask):
    """Eq. 1 (standard PPO clip) written directly, for the d in {0,1} limit."""
    r = np.exp(lt - lold)
    per = np.minimum(r * A, np.clip(r, 1 - eps, 1 + eps) * A)
    return (per * mask).sum() / mask.sum()


def test_zero_staleness_equals_coupled_ppo():
    n = 3000
    lt, lb = _random_logps(n)
    A = rng.standard_normal(n)
    m = (rng.random(n) < 0.7).astype(np.uint8)
    for d in (0, 1):
        o = oracle.surrogate(lt, lb, np.full(n, 5 - d, dtype=np.int32), 5, A, m, 0.2)
        assert np.allclose(o["iw"], 1.0, rtol=0, atol=0)
        assert abs(o["loss"] + _coupled_ppo_objective(lt, lb, A, 0.2, m)) < 1e-13
    # d = 0 and d = 1 are bit-identical
    a = oracle.surrogate(lt, lb, np.full(n, 5, dtype=np.int32), 5, A, m, 0.2)
    b = oracle.surrogate(lt, lb, np.full(n, 4, dtype=np.int32), 5, A, m, 0.2)
    assert a["loss"] == b["loss"] and np.array_equal(a["g"], b["g"])


def test_on_policy_loss_is_minus_mean_advantage():
    n = 1000
    lt, _ = _random_logps(n)
    A = rng.standard_normal(n)
    m = (rng.random(n) < 0.5).astype(np.uint8)
    ver = (9 - rng.integers(0, 9, n)).astype(np.int32)
    o = oracle.surrogate(lt, lt, ver, 9, A, m, 0.2)
    assert abs(o["loss"] + (A * m).sum() / m.sum()) < 1e-13
    assert not o["clipped"].any()


def test_all_masked_and_scaling_and_denominator():
    n = 200
    lt, lb = _random_logps(n)
    A = rng.standard_normal(n)
    ver = (9 - rng.integers(0, 9, n)).astype(np.int32)
    z = oracle.surrogate(lt, lb, ver, 9, A, np.zeros(n, np.uint8), 0.2)
    assert z["loss"] == 0.0 and not z["g"].any() and z["stats"]["n_tokens"] == 0
    m = (rng.random(n) < 0.6).astype(np.uint8)
    a = oracle.surrogate(lt, lb, ver, 9, A, m, 0.2)
    b = oracle.surrogate(lt, lb, ver, 9, 3.0 * A, m, 0.2)
    assert abs(b["loss"] - 3.0 * a["loss"]) < 1e-13 and np.allclose(b["g"], 3 * a["g"], rtol=1e-13)
    c = oracle.surrogate(lt, lb, ver, 9, A, m, 0.2, denom=2.0 * m.sum())
    assert abs(c["loss"] - a["loss"] / 2) < 1e-14 and np.allclose(c["g"], a["g"] / 2, rtol=1e-13)
    # masked tokens never carry gradient
    assert not a["g"][m == 0].any()


def test_stats_against_direct_counts():
    n = 4000
    lt, lb = _random_logps(n)
    A = rng.standard_normal(n)
    m = (rng.random(n) < 0.6).astype(np.uint8)
    ver = (9 - rng.integers(-2, 9, n)).astype(np.int32)  # includes negative staleness
    o = oracle.surrogate(lt, lb, ver, 9, A, m, 0.2)
    w = np.exp(lt - lb)
    al = np.where(9 - ver >= 1, 1.0 / np.maximum(9 - ver, 1), 1.0)
    r = w ** al
    # Eq. 2: the clip bites when r > 1+eps with A > 0 or r < 1-eps with A < 0
    clipped = ((r > 1.2) & (A > 0)) | ((r < 0.8) & (A < 0))
    assert o["stats"]["n_clipped"] == int((clipped & (m == 1)).sum())
    assert np.array_equal(o["clipped"].astype(bool), clipped)
    iw = w ** (1 - al)
    assert abs(o["stats"]["iw_min"] - iw[m == 1].min()) < 1e-12
    assert abs(o["stats"]["iw_max"] - iw[m == 1].max()) < 1e-12
    assert o["stats"]["n_negative_staleness"] == int(((9 - ver < 0) & (m == 1)).sum())
    assert o["stats"]["n_tokens"] == int(m.sum())


def test_unclipped_gradient_is_independent_of_staleness():
    n = 1000
    lt, lb = _random_logps(n)
    lb = lt + np.clip(lb - lt, -0.1, 0.1)   # keep w inside the clip range for every alpha
    A = rng.standard_normal(n)
    m = np.ones(n, np.uint8)
    w = np.exp(lt - lb)
    for d in (0, 1, 2, 5, 17):
        o = oracle.surrogate(lt, lb, np.full(n, 20 - d, dtype=np.int32), 20, A, m, 0.2)
        assert not o["clipped"].any()
        assert np.allclose(o["g"], -A * w / n, rtol=1e-12)


# ----------------------------------------------------------------------------- gradient (chain rule on Eq. 2, frozen prox)

def _frozen_loss(z, y, lb, lp0, A, m, eps, denom=0.0):
    lt = oracle.token_logprobs(z, y)["logp"]
    return oracle.decoupled_clip(lt, lb, lp0, A, m, eps, denom)["loss"]


@pytest.mark.parametrize("T,V,seed", [(2, 3, 0), (4, 7, 1), (8, 17, 2), (5, 11, 3)])
def test_gradient_by_central_finite_differences(T, V, seed):
    r = np.random.default_rng(100 + seed)
    # logits that are exactly representable after +-h steps: use float64 maths through a
    # float32 container with values on a coarse grid plus h = 2^-10
    z0 = np.round(r.standard_normal((T, V)) * 2 * 64) / 64
    y = r.integers(0, V, T).astype(np.int32)
    ver = (10 - r.integers(0, 6, T)).astype(np.int32)
    A = r.standard_normal(T)
    m = np.ones(T, np.uint8)
    m[r.integers(0, T)] = 0
    lt0 = oracle.token_logprobs(z0.astype(np.float32), y)["logp"]
    lb = lt0 + r.uniform(-0.4, 0.4, T)
    full = oracle.loss_fwd_bwd(z0.astype(np.float32), y, lb, ver, 10, A, m, 0.2)
    # stay away from the kinks r = 1 +- eps
    rr = np.exp(full["logp"] - full["lp"])
    assume = (np.abs(rr - 1.2) > 2e-3).all() and (np.abs(rr - 0.8) > 2e-3).all()
    assert assume, "test inputs landed on a clip boundary; change the seed"
    h = 2.0**-10
    num = np.zeros((T, V))
    for t in range(T):
        for j in range(V):
            zp = z0.copy(); zp[t, j] += h
            zm = z0.copy(); zm[t, j] -= h
            fp = _frozen_loss(zp.astype(np.float32), y, lb, full["lp"], A, m, 0.2)
            fm = _frozen_loss(zm.astype(np.float32), y, lb, full["lp"], A, m, 0.2)
            num[t, j] = (fp - fm) / (2 * h)
    scale = np.abs(full["dz"]).max()
    assert np.abs(num - full["dz"]).max() < 5e-6 * scale + 1e-9
    # consistency of the frozen objective at z0 with the reported loss
    assert abs(_frozen_loss(z0.astype(np.float32), y, lb, full["lp"], A, m, 0.2) - full["loss"]) < 1e-14
    # both clipped and unclipped tokens should be exercised across the parametrisation
    assert np.abs(full["dz"].sum(axis=1)).max() < 1e-14


def test_gradient_rows_sum_to_zero_and_dead_rows_are_zero():
    T, V = 12, 129
    z = (rng.standard_normal((T, V)) * 3).astype(np.float32)
    y = rng.integers(0, V, T).astype(np.int32)
    lt = oracle.token_logprobs(z, y)["logp"]
    lb = lt + rng.uniform(-0.6, 0.6, T)
    A = rng.standard_normal(T)
    A[3] = 0.0
    m = np.ones(T, np.uint8)
    m[5] = 0
    ver = (10 - rng.integers(0, 4, T)).astype(np.int32)
    o = oracle.loss_fwd_bwd(z, y, lb, ver, 10, A, m, 0.2)
    assert np.abs(o["dz"].sum(axis=1)).max() < 1e-15
    assert not o["dz"][3].any() and not o["dz"][5].any()
    for t in np.nonzero(o["clipped"])[0]:
        assert not o["dz"][t].any()
    assert o["clipped"].any() and (~o["clipped"].astype(bool)).any()
    # the chosen column carries +g(1-p), every other column -g p
    t = int(np.nonzero((o["g"] != 0))[0][0])
    p = scipy.special.softmax(z[t].astype(np.float64))
    expect = -o["g"][t] * p
    expect[y[t]] += o["g"][t]
    assert np.allclose(o["dz"][t], expect, rtol=1e-12, atol=1e-18)


def test_bad_index_rows_are_masked_and_counted():
    T, V = 6, 33
    z = (rng.standard_normal((T, V))).astype(np.float32)
    y = np.array([1, 2, -5, 33, 4, 5], dtype=np.int32)
    lb = -np.ones(T)
    A = np.ones(T)
    m = np.array([1, 1, 1, 1, 0, 1], np.uint8)
    o = oracle.loss_fwd_bwd(z, y, lb, np.full(T, 3, np.int32), 3, A, m, 0.2)
    assert o["stats"]["n_bad_index"] == 2 and o["stats"]["n_tokens"] == 3
    assert list(o["eff_mask"]) == [1, 1, 0, 0, 0, 1]
    assert not o["dz"][2].any() and not o["dz"][3].any() and o["logp"][2] == 0.0


# ----------------------------------------------------------------------------- GRPO advantages

def test_grpo_binary_rewards_closed_form():
    for G in (4, 8):
        for k in range(1, G):
            R = np.array([1.0] * k + [0.0] * (G - k))
            adv = oracle.grpo_advantages(R, G, eps_adv=0.0)
            p = k / G
            assert np.allclose(adv[:k], math.sqrt((1 - p) / p), rtol=1e-13)
            assert np.allclose(adv[k:], -math.sqrt(p / (1 - p)), rtol=1e-13)
            adv6 = oracle.grpo_advantages(R, G)   # default eps_adv = 1e-6 only nudges it
            assert np.allclose(adv6, adv * np.std(R) / (np.std(R) + 1e-6), rtol=1e-12)


def test_grpo_groups_are_independent_sum_to_zero_and_constant_group_is_zero():
    R = np.concatenate([rng.random(8), np.full(8, 0.5), rng.random(8) * 10])
    adv = oracle.grpo_advantages(R, 8)
    assert np.abs(adv.reshape(3, 8).sum(axis=1)).max() < 1e-12
    assert not adv[8:16].any()
    only = oracle.grpo_advantages(R[16:], 8)
    assert np.array_equal(only, adv[16:])
    # unit population variance inside a group (up to eps_adv)
    assert abs(np.mean(adv[:8] ** 2) - 1) < 1e-4
    with pytest.raises(ValueError):
        oracle.grpo_advantages(R[:7], 8)


def test_grpo_broadcast_to_tokens():
    R = rng.random(8)
    sid = np.repeat(np.arange(8, dtype=np.int32), 5)
    adv_seq, adv_tok = oracle.grpo_advantages(R, 4, seq_id=sid)
    assert np.array_equal(adv_tok, adv_seq[sid])


# ----------------------------------------------------------------------------- LM-head projection

def test_lmhead_logits_against_numpy_matmul_and_hand_values():
    H, V, T = 24, 37, 9
    h = bf16_bits(rng.standard_normal((T, H)))
    W = bf16_bits(rng.standard_normal((V, H)) * 0.5)
    hf, Wf = synth.bf16_bits_to_f64(h), synth.bf16_bits_to_f64(W)
    z = oracle.lmhead_logits(h, W)
    assert np.allclose(z, hf @ Wf.T, rtol=1e-13, atol=1e-13)
    sub = oracle.lmhead_logits(h, W, rows=[7, 2])
    assert np.array_equal(sub, z[[7, 2]])
    # hand values: h = [1, 2, -1], W rows [1, 0, 0], [0.5, 0.5, 0.5], [-2, 1, 4]  ->  z = [1, 1, -4]
    h1 = bf16_bits(np.array([[1.0, 2.0, -1.0]]))
    W1 = bf16_bits(np.array([[1.0, 0, 0], [0.5, 0.5, 0.5], [-2.0, 1.0, 4.0]]))
    assert np.array_equal(oracle.lmhead_logits(h1, W1), np.array([[1.0, 1.0, -4.0]]))
    # an identity weight returns the hidden state as logits (operands not transposed by mistake)
    eye = bf16_bits(np.eye(H))
    assert np.array_equal(oracle.lmhead_logits(h, eye), hf)


def test_float64_logits_go_through_the_same_logsoftmax():
    z = rng.standard_normal((5, 33)) * 3
    y = rng.integers(0, 33, 5).astype(np.int32)
    o = oracle.token_logprobs(z, y)
    assert np.allclose(o["lse"], scipy.special.logsumexp(z, axis=1), rtol=0, atol=1e-13)
    assert np.allclose(o["logp"], z[np.arange(5), y] - o["lse"], rtol=0, atol=1e-13)
    assert np.array_equal(o["chosen_raw"], z[np.arange(5), y])


def test_lmhead_backward_against_numpy_and_finite_differences():
    H, V, T = 6, 11, 4
    h = bf16_bits(np.round(rng.standard_normal((T, H)) * 8) / 8)
    W = bf16_bits(np.round(rng.standard_normal((V, H)) * 8) / 8)
    hf, Wf = synth.bf16_bits_to_f64(h), synth.bf16_bits_to_f64(W)
    y = rng.integers(0, V, T).astype(np.int32)
    ver = (10 - rng.integers(0, 4, T)).astype(np.int32)
    A = rng.standard_normal(T)
    m = np.ones(T, np.uint8)
    z0 = oracle.lmhead_logits(h, W)
    lt0 = oracle.token_logprobs(z0, y)["logp"]
    lb = lt0 + rng.uniform(-0.1, 0.1, T)          # inside the clip range: every token carries gradient
    full = oracle.loss_fwd_bwd(z0, y, lb, ver, 10, A, m, 0.2)
    dh, dW = oracle.lmhead_backward(full["dz"], h, W)
    assert np.allclose(dh, full["dz"] @ Wf, rtol=1e-12, atol=1e-15)
    assert np.allclose(dW, full["dz"].T @ hf, rtol=1e-12, atol=1e-15)

    def frozen_loss(hm, Wm):
        lt = oracle.token_logprobs(hm @ Wm.T, y)["logp"]
        return oracle.decoupled_clip(lt, lb, full["lp"], A, m, 0.2)["loss"]

    eps = 2.0 ** -12
    num_dh = np.zeros_like(hf)
    for t in range(T):
        for k in range(H):
            hp, hm_ = hf.copy(), hf.copy()
            hp[t, k] += eps
            hm_[t, k] -= eps
            num_dh[t, k] = (frozen_loss(hp, Wf) - frozen_loss(hm_, Wf)) / (2 * eps)
    assert np.abs(num_dh - dh).max() < 1e-6 * np.abs(dh).max() + 1e-10
    num_dW = np.zeros_like(Wf)
    for v in range(V):
        for k in range(H):
            Wp, Wm_ = Wf.copy(), Wf.copy()
            Wp[v, k] += eps
            Wm_[v, k] -= eps
            num_dW[v, k] = (frozen_loss(hf, Wp) - frozen_loss(hf, Wm_)) / (2 * eps)
    assert np.abs(num_dW - dW).max() < 1e-6 * np.abs(dW).max() + 1e-10


def test_lmhead_backward_matmul_form_equals_the_loops():
    # the matrix-product form used for the larger GPU cases against the plain loops, on a ragged shape
    T, H, V = 37, 24, 53
    h = bf16_bits(rng.standard_normal((T, H)))
    W = bf16_bits(rng.standard_normal((V, H)))
    dz = rng.standard_normal((T, V)) * np.exp(rng.standard_normal((T, V)) * 3)
    dh, dW = oracle.lmhead_backward(dz, h, W)
    dh2, dW2 = oracle.lmhead_backward_matmul(dz, h, W)
    ah, aW = oracle.lmhead_backward(np.abs(dz), h & 0x7FFF, W & 0x7FFF)
    assert (np.abs(dh - dh2) <= 1e-13 * ah).all() and (np.abs(dW - dW2) <= 1e-13 * aW).all()
    assert dh2.shape == (T, H) and dW2.shape == (V, H)


# ----------------------------------------------------------------------------- entropy, loss variants

def test_entropy_closed_forms_and_scipy():
    import scipy.stats
    for V in (1, 2, 9, 1000):
        assert abs(oracle.entropy(np.full((1, V), -2.5, dtype=np.float32))[0] - math.log(V)) < 1e-12
    # two-point distribution with logit gap g: p = sigmoid(g); H = -p log p - (1-p) log(1-p)
    g = 1.75
    p = 1 / (1 + math.exp(-g))
    H = oracle.entropy(np.array([[g, 0.0]], dtype=np.float32))[0]
    assert abs(H - (-p * math.log(p) - (1 - p) * math.log(1 - p))) < 1e-14
    # a dominant logit: entropy -> 0, and -inf-like tails do not produce NaN
    assert oracle.entropy(np.array([[100.0, -1000.0, -1000.0]], dtype=np.float32))[0] < 1e-30
    z = (rng.standard_normal((6, 501)) * 3).astype(np.float32)
    ref = scipy.stats.entropy(scipy.special.softmax(z.astype(np.float64), axis=1), axis=1)
    assert np.allclose(oracle.entropy(z), ref, rtol=1e-12, atol=1e-13)
    zb = bf16_bits(z)
    assert np.allclose(oracle.entropy(zb), scipy.stats.entropy(scipy.special.softmax(synth.bf16_bits_to_f64(zb), axis=1), axis=1),
                       rtol=1e-12, atol=1e-13)


def test_given_prox_variant_reduces_to_the_interpolated_one_and_to_coupled_ppo():
    n = 500
    lt, lb = _random_logps(n)
    A = rng.standard_normal(n)
    m = (rng.random(n) < 0.7).astype(np.uint8)
    ver = (30 - rng.integers(0, 9, n)).astype(np.int32)
    a = oracle.surrogate(lt, lb, ver, 30, A, m, 0.2)
    b = oracle.decoupled_clip(lt, lb, a["lp"], A, m, 0.2)           # "recompute": prox supplied
    assert a["loss"] == b["loss"] and np.array_equal(a["g"], b["g"])
    c = oracle.decoupled_clip(lt, lb, lb, A, m, 0.2)                # prox = behaviour: Eq. 1 ("sync")
    assert abs(c["loss"] + _coupled_ppo_objective(lt, lb, A, 0.2, m)) < 1e-13 and (c["iw"] == 1).all()
    # an arbitrary recomputed prox: importance weight and ratio multiply back to w (Eq. 2)
    lp = lt + rng.standard_normal(n) * 0.05
    d = oracle.decoupled_clip(lt, lb, lp, A, m, 0.2)
    assert np.allclose(d["iw"] * d["r"], np.exp(lt - lb), rtol=1e-12)


# ----------------------------------------------------------------------------- histograms (Section 4.2.2 statistics)

def test_histogram_hand_example_numpy_and_invariants():
    nan = float("nan")
    # by hand: below 1.0 -> {0.5, -3}; [1, 1.5) -> {1.0, 1.0}; [1.5, 2) -> {1.7}; >= 2 -> {2.0, 5}; one NaN
    v = np.array([0.5, 1.0, 1.0, 1.7, 2.0, -3.0, nan, 5.0], dtype=np.float32)
    assert oracle.histogram(v, [1.0, 1.5, 2.0]).tolist() == [2, 2, 1, 2, 1]
    # a selection: tokens 1, 3, 4, 6 only
    sel = np.array([0, 1, 0, 1, 1, 0, 1, 0], dtype=np.uint8)
    assert oracle.histogram(v, [1.0, 1.5, 2.0], sel).tolist() == [0, 1, 1, 1, 1]
    # repeated edges make empty bins; a value equal to a repeated edge belongs to the bin after it
    assert oracle.histogram([1.0, 2.0, 2.0, 3.0], [2.0, 2.0, 2.0, 3.0]).tolist() == [1, 0, 0, 2, 1, 0]
    # an independent routine: numpy.histogram agrees on every half-open bin (its last bin is closed, so the
    # edge value itself is kept out of the data), and everything is counted exactly once
    x = (rng.standard_normal(5000) * 0.3).astype(np.float32)
    w = np.exp(x).astype(np.float32)
    edges = np.geomspace(0.25, 4.0, 33).astype(np.float32)
    w = w[w != edges[-1]]
    h = oracle.histogram(w, edges)
    ref, _ = np.histogram(w.astype(np.float64), bins=edges.astype(np.float64))
    assert np.array_equal(h[1:-2], ref)
    assert h[0] == (w < edges[0]).sum() and h[-2] == (w >= edges[-1]).sum() and h[-1] == 0
    assert h.sum() == len(w)
    sel = (rng.random(len(w)) < 0.4).astype(np.uint8)
    assert oracle.histogram(w, edges, sel).sum() == sel.sum()
    assert np.array_equal(oracle.histogram(w, edges, sel) + oracle.histogram(w, edges, 1 - sel), h)
    # importance weights of the surrogate: extrema reported by the statistics bracket the occupied bins
    lt, lb = _random_logps(400)
    m = (rng.random(400) < 0.7).astype(np.uint8)
    ver = (30 - rng.integers(0, 9, 400)).astype(np.int32)
    a = oracle.surrogate(lt, lb, ver, 30, rng.standard_normal(400), m, 0.2)
    hw = oracle.histogram(a["iw"], edges, m)
    occupied = np.nonzero(hw[1:-2])[0]
    assert hw[0] == 0 and hw[-2] == 0
    assert edges[occupied[0]] <= a["stats"]["iw_min"] < edges[occupied[0] + 1]
    assert edges[occupied[-1]] <= a["stats"]["iw_max"] < edges[occupied[-1] + 1]
    assert hw.sum() == a["stats"]["n_tokens"]


# ----------------------------------------------------------------------------- memory and arithmetic sanitizers

def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The oracle, built with -fsanitize=address,undefined, runs a driver over every entry point and the edge
    cases (empty batch, single-entry vocabulary, ids out of range, extreme versions) without a report."""
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fno-omit-frame-pointer", "-static-libasan", "-fopenmp", "-o", exe,
                           os.path.join(here, "oracle_sanitize_driver.c"),
                           os.path.join(os.path.dirname(here), "oracle", "a3po_oracle.c"), "-lm"])
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr[-2000:]
    assert res.stdout.strip().endswith("ok") and "runtime error" not in res.stderr and "ERROR" not in res.stderr
