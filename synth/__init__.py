"""Seeded synthetic inputs shaped like the A-3PO training workloads.

Only input manufacture lives here: counter-based logits (C, ``gen.c``) and the
small per-token / per-sequence arrays (NumPy Philox streams).  Nothing in this
module evaluates the method; both the CPU oracle's tests and the GPU path's
tests and benchmark draw their inputs from it so that they see identical bytes.

The workloads stand in for the paper's RL rollouts (Section 4.1: 1.5B and 8B
policies, several samples per prompt, ragged response lengths, integer policy
versions); datasets and weights are not used.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libsynth.so")

BASE_SEED = 20251206
CURRENT_VERSION = 100


def build(force: bool = False) -> str:
    """Compile gen.c into libsynth.so (gcc, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.synth_logit_rows.restype = None
        lib.synth_logit_rows.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_float,
            ctypes.c_void_p, ctypes.c_float, ctypes.c_float,
        ]
        lib.synth_row_boost_flags.restype = None
        lib.synth_row_boost_flags.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64,
            ctypes.c_uint32, ctypes.c_float,
        ]
        _lib = lib
    return _lib


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration (shapes and value distributions)."""
    name: str
    S: int            # sequences
    L: int            # tokens per sequence (padded length)
    V: int            # vocabulary
    dtype: str        # "f32" | "bf16"
    sigma: float      # logits ~ N(0, sigma^2)
    boost: float      # added at the chosen column of a boosted row
    boost_prob: float
    stale_max: int    # staleness d ~ U{0..stale_max} per sequence
    noise_std: float  # log pi_behav = min(0, log pi_theta + N(0, noise_std^2))
    reward_p: float   # Bernoulli rewards
    G: int            # GRPO group size (consecutive sequences)
    len_lo: int       # response length ~ U{len_lo..len_hi}
    len_hi: int
    clip_eps: float = 0.2
    stream: int = 0
    seed: int = BASE_SEED

    @property
    def T(self) -> int:
        return self.S * self.L

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "tiny": Workload("tiny", 4, 256, 32000, "f32", 2.0, 0.0, 0.0, 4, 0.05, 0.5, 4, 64, 256, stream=1),
    "1p5b": Workload("1p5b", 16, 2048, 151936, "bf16", 3.0, 8.0, 0.7, 8, 0.1, 0.3, 8, 256, 2048, stream=2),
    "8b": Workload("8b", 32, 4096, 151936, "bf16", 3.0, 8.0, 0.7, 8, 0.1, 0.3, 8, 256, 4096, stream=3),
    "long": Workload("long", 8, 16384, 151936, "bf16", 3.0, 8.0, 0.7, 16, 0.3, 0.2, 8, 3277, 16384, stream=4),
}


def _rng(w: Workload, sub: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[w.seed, (w.stream << 16) + sub]))


def token_arrays(w: Workload) -> dict:
    """Per-token and per-sequence inputs (everything except the logits).

    Returns chosen[T] i32, seq_id[T] i32, versions[T] i32, current_version,
    rewards[S] f32, lengths[S], mask[T] u8, noise[T] f32, reward_redraws.
    """
    T, S, L = w.T, w.S, w.L
    chosen = _rng(w, 1).integers(0, w.V, size=T, dtype=np.int64).astype(np.int32)
    stale = _rng(w, 2).integers(0, w.stale_max + 1, size=S, dtype=np.int64)
    lengths = _rng(w, 3).integers(w.len_lo, w.len_hi + 1, size=S, dtype=np.int64)
    redraws = 0
    while True:
        rewards = (_rng(w, 4 + 16 * redraws).random(S) < w.reward_p).astype(np.float32)
        groups = rewards.reshape(S // w.G, w.G)
        if (groups.max(axis=1) != groups.min(axis=1)).any():
            break
        redraws += 1
    noise = (_rng(w, 5).standard_normal(T) * w.noise_std).astype(np.float32)
    seq_id = np.repeat(np.arange(S, dtype=np.int32), L)
    pos = np.tile(np.arange(L, dtype=np.int64), S)
    mask = (pos < lengths[seq_id]).astype(np.uint8)
    versions = (CURRENT_VERSION - stale[seq_id]).astype(np.int32)
    return dict(chosen=chosen, seq_id=seq_id, versions=versions, current_version=CURRENT_VERSION,
                rewards=rewards, lengths=lengths, mask=mask, noise=noise, staleness=stale,
                reward_redraws=redraws)


def logit_rows(w: Workload, t0: int, nrows: int, chosen: np.ndarray | None, ld: int | None = None,
               out: np.ndarray | None = None) -> np.ndarray:
    """Rows t0..t0+nrows of the [T, V] logits; float32, or bfloat16 bit patterns as uint16.

    ``chosen`` is the full [T] array (indexed by absolute row) and only decides where a
    boosted row gets its bump.  ``ld`` (>= V) is the row stride in elements.
    """
    ld = w.V if ld is None else ld
    assert ld >= w.V
    np_dt = np.float32 if w.dtype == "f32" else np.uint16
    if out is None:
        out = np.empty((nrows, ld), dtype=np_dt)
    assert out.dtype == np_dt and out.shape == (nrows, ld) and out.flags.c_contiguous
    cptr = None
    if chosen is not None:
        assert chosen.dtype == np.int32 and chosen.flags.c_contiguous and chosen.shape[0] >= t0 + nrows
        cptr = chosen.ctypes.data
    _load().synth_logit_rows(out.ctypes.data, 0 if w.dtype == "f32" else 1, t0, nrows, w.V, ld,
                             w.seed, w.stream, w.sigma, cptr, w.boost, w.boost_prob)
    return out


def behav_from_target(logp_theta: np.ndarray, noise: np.ndarray) -> np.ndarray:
    """Behaviour log-probs of the recipe: target log-prob plus noise, clamped to <= 0."""
    return np.minimum(0.0, logp_theta.astype(np.float64) + noise.astype(np.float64)).astype(np.float32)


def bf16_bits_to_f64(u16: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float64 (format conversion only)."""
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


@dataclass(frozen=True)
class LmHeadWorkload:
    """Hidden states and LM-head weight in front of the loss path (the 8B-shape fused workload)."""
    name: str
    tokens: Workload          # per-token recipe (V of this workload is the vocabulary)
    H: int                    # hidden size
    h_sigma: float = 1.0      # hidden ~ N(0, h_sigma^2), bf16
    w_sigma: float = 0.02     # weight ~ N(0, w_sigma^2), bf16


LMHEAD_WORKLOADS = {
    "lmhead8b": LmHeadWorkload("lmhead8b", WORKLOADS["8b"].scaled(name="lmhead8b", S=16, L=4096, stream=5), 4096),
}


def hidden_rows(lw: LmHeadWorkload, t0: int, nrows: int) -> np.ndarray:
    """Rows t0.. of the [T, H] hidden states, bfloat16 bit patterns (uint16)."""
    w = lw.tokens.scaled(V=lw.H, dtype="bf16", sigma=lw.h_sigma, stream=lw.tokens.stream + 64, boost_prob=0.0)
    return logit_rows(w, t0, nrows, None)


def weight_rows(lw: LmHeadWorkload, v0: int, nrows: int) -> np.ndarray:
    """Rows v0.. of the [V, H] LM-head weight, bfloat16 bit patterns (uint16)."""
    w = lw.tokens.scaled(V=lw.H, dtype="bf16", sigma=lw.w_sigma, stream=lw.tokens.stream + 128, boost_prob=0.0)
    return logit_rows(w, v0, nrows, None)
