"""ctypes binding of liba3po.so: same names as the C entry points, argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their device
pointers and the current HIP stream to the C ABI, and returns torch tensors.  There is no
fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "liba3po.so")

A3PO_F32, A3PO_BF16 = 0, 1
A3PO_PROX_INTERP, A3PO_PROX_GIVEN, A3PO_PROX_BEHAV = 0, 1, 2
A3PO_WS_LOSS_FWD_BWD = 0
A3PO_WS_FUSED_LMHEAD = 1
A3PO_WS_FUSED_LMHEAD_LOSS = 2

# layout of a3po_stats (include/a3po.h)
STATS_DTYPE = np.dtype([("n_tokens", "<i8"), ("n_clipped", "<i8"), ("n_bad_index", "<i8"),
                        ("n_negative_staleness", "<i8"), ("iw_min", "<f4"), ("iw_max", "<f4"),
                        ("entropy_mean", "<f4"), ("reserved", "<f4")])

_P, _I64, _I32, _F32, _SZ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t



class LossOptions(ctypes.Structure):
    """a3po_loss_options (include/a3po.h)."""
    _fields_ = [("prox_mode", ctypes.c_int32), ("accumulate", ctypes.c_int32), ("logp_prox_in", ctypes.c_void_p),
                ("entropy_out", ctypes.c_void_p), ("iw_out", ctypes.c_void_p), ("clipped_out", ctypes.c_void_p),
                ("event_before_rows", ctypes.c_void_p), ("event_after_rows", ctypes.c_void_p),
                ("denom_dev", ctypes.c_void_p)]


_SIGNATURES = {
    "a3po_workspace_bytes": (_SZ, [ctypes.c_int, _I64, _I64, _I64]),
    "a3po_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "a3po_token_logprobs": (ctypes.c_int, [_P, ctypes.c_int, _I64, _I64, _I64, _P, _P, _P, _P, _P]),
    "a3po_proximal_interp": (ctypes.c_int, [_P, _P, _P, _I32, _I64, _P, _P, _P]),
    "a3po_grpo_advantages": (ctypes.c_int, [_P, _I64, _I32, _F32, _P, _I64, _P, _P]),
    "a3po_fused_lmhead_logprob": (ctypes.c_int, [_P, _P, _I64, _I64, _I64, _P, _P, _P, _P, _SZ, _P]),
    "a3po_fused_lmhead_loss_fwd_bwd": (ctypes.c_int, [_P, _P, _I64, _I64, _I64, _P, _P, _P, _I32, _P, _P, _F32, _F32,
                                                      _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "a3po_loss_fwd_bwd": (ctypes.c_int, [_P, ctypes.c_int, _I64, _I64, _I64, _P, _P, _P, _I32, _P, _P, _F32, _F32,
                                         _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "a3po_loss_fwd_bwd_noalloc": (ctypes.c_int, [_P, ctypes.c_int, _I64, _I64, _I64, _P, _P, _P, _I32, _P, _P, _F32,
                                                 _F32, _P, _P, _P, _P, _P, _P]),
    "a3po_loss_fwd_bwd_ex": (ctypes.c_int, [_P, ctypes.c_int, _I64, _I64, _I64, _P, _P, _P, _I32, _P, _P, _F32,
                                            _F32, _P, _P, _P, _P, _P, _P, _SZ, _P, ctypes.POINTER(LossOptions)]),
    "a3po_count_tokens": (ctypes.c_int, [_P, _P, _I64, _I64, _P, _P, _P]),
    "a3po_histogram": (ctypes.c_int, [_P, _P, _I64, _P, _I32, _I32, _P, _P]),
    "a3po_plan_microbatches": (ctypes.c_int, [_P, _I64, _I32, _I64, _P, _P, _I64, _P]),
    "a3po_shard_partials": (ctypes.c_int, [_P, ctypes.c_int, _I64, _I64, _I64, _P, _I64, _P, _P]),
    "a3po_shard_combine": (ctypes.c_int, [_P, _I32, _I64, _P, _I64, _P, _P, _P, _P]),
    "a3po_shard_loss_bwd": (ctypes.c_int, [_P, ctypes.c_int, _I64, _I64, _I64, _I64, _I64, _P, _P, _P, _P, _P, _I32,
                                           _P, _P, _F32, _F32, _P, _P, _P, _P, _P, _SZ, _P,
                                           ctypes.POINTER(LossOptions)]),
    "a3po_token_logprobs_entropy": (ctypes.c_int, [_P, ctypes.c_int, _I64, _I64, _I64, _P, _P, _P, _P, _P, _P]),
}

_lib = None


class A3poError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2512_06547_amd.build` "
                "(there is no fallback path)")
        # PyTorch first: it brings its own copy of the HIP runtime, and the library must bind to that same copy (a
        # stream or pointer created by one copy of the runtime means nothing to another); once PyTorch's is in the
        # process, the library's dependency on the runtime resolves to it
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        handle = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def strerror(code: int) -> str:
    return lib().a3po_strerror(int(code)).decode()


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise A3poError(rc, where)


def _torch():
    import torch
    return torch


def _stream() -> int:
    return _torch().cuda.current_stream().cuda_stream


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _logits_meta(logits, V):
    torch = _torch()
    assert logits.is_cuda and logits.dim() == 2 and logits.stride(1) == 1, "logits must be a row-major CUDA matrix"
    if logits.dtype == torch.float32:
        dt = A3PO_F32
    elif logits.dtype == torch.bfloat16:
        dt = A3PO_BF16
    else:
        raise TypeError("logits must be float32 or bfloat16")
    T = logits.shape[0]
    ld = logits.stride(0) if T > 1 else max(logits.stride(0), logits.shape[1])
    V = logits.shape[1] if V is None else int(V)
    return dt, T, V, ld


def _vec(t, dtype, n, name):
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous() and t.numel() == n, f"{name}: need contiguous {dtype}[{n}] on GPU"
    return t


def workspace_bytes(T: int, V: int = 0, H: int = 0, which: int = A3PO_WS_LOSS_FWD_BWD) -> int:
    return int(lib().a3po_workspace_bytes(which, T, V, H))


def token_logprobs(logits, chosen, V=None, want_lse=True, want_chosen_logit=True, want_entropy=False):
    """a3po_token_logprobs -> (logp[T] f32, lse[T] f32 | None, chosen_logit[T] logits.dtype | None);
    with want_entropy, a3po_token_logprobs_entropy -> (..., entropy[T] f32)."""
    torch = _torch()
    dt, T, V, ld = _logits_meta(logits, V)
    _vec(chosen, torch.int32, T, "chosen")
    dev = logits.device
    logp = torch.empty(T, dtype=torch.float32, device=dev)
    lse = torch.empty(T, dtype=torch.float32, device=dev) if want_lse else None
    zy = torch.empty(T, dtype=logits.dtype, device=dev) if want_chosen_logit else None
    if not want_entropy:
        _check(lib().a3po_token_logprobs(_ptr(logits), dt, T, V, ld, _ptr(chosen), _ptr(logp), _ptr(lse), _ptr(zy),
                                         _stream()), "a3po_token_logprobs")
        return logp, lse, zy
    ent = torch.empty(T, dtype=torch.float32, device=dev)
    _check(lib().a3po_token_logprobs_entropy(_ptr(logits), dt, T, V, ld, _ptr(chosen), _ptr(logp), _ptr(lse),
                                             _ptr(zy), _ptr(ent), _stream()), "a3po_token_logprobs_entropy")
    return logp, lse, zy, ent


def proximal_interp(logp_behav, logp_theta, versions, current_version: int, want_alpha=True):
    """a3po_proximal_interp -> (logp_prox[T] f32, alpha[T] f32 | None)."""
    torch = _torch()
    T = versions.numel()
    _vec(logp_behav, torch.float32, T, "logp_behav")
    _vec(logp_theta, torch.float32, T, "logp_theta")
    _vec(versions, torch.int32, T, "versions")
    lp = torch.empty(T, dtype=torch.float32, device=versions.device)
    al = torch.empty(T, dtype=torch.float32, device=versions.device) if want_alpha else None
    _check(lib().a3po_proximal_interp(_ptr(logp_behav), _ptr(logp_theta), _ptr(versions), int(current_version), T,
                                      _ptr(lp), _ptr(al), _stream()), "a3po_proximal_interp")
    return lp, al


def grpo_advantages(rewards, G: int, seq_id, eps_adv: float = 1e-6, out=None):
    """a3po_grpo_advantages -> adv[T] f32 (advantage of each token's sequence)."""
    torch = _torch()
    S, T = rewards.numel(), seq_id.numel()
    _vec(rewards, torch.float32, S, "rewards")
    _vec(seq_id, torch.int32, T, "seq_id")
    adv = torch.empty(T, dtype=torch.float32, device=seq_id.device) if out is None else out
    _check(lib().a3po_grpo_advantages(_ptr(rewards), S, int(G), float(eps_adv), _ptr(seq_id), T, _ptr(adv),
                                      _stream()), "a3po_grpo_advantages")
    return adv


def loss_fwd_bwd(logits, chosen, logp_behav, versions, current_version: int, advantages, loss_mask,
                 clip_eps: float, denom: float = 0.0, V=None, dlogits=None, workspace=None, out=None,
                 events=None, prox_mode: int = A3PO_PROX_INTERP, logp_prox_in=None, want_entropy=False,
                 want_iw=False, want_clipped=False, denom_dev=None, accumulate=False):
    """a3po_loss_fwd_bwd, or a3po_loss_fwd_bwd_ex when any extra is asked for: ``events=(start, stop)`` raw
    hipEvent_t handles, ``prox_mode`` / ``logp_prox_in`` (the given-proximal and coupled variants; ``versions``
    may then be None), ``want_entropy`` / ``want_iw`` / ``want_clipped`` per-token outputs, ``denom_dev`` (a
    1-element float32 device tensor that replaces ``denom``) and ``accumulate`` (add to the loss / stats in ``out``).

    dlogits: None -> a new tensor like logits; or a tensor with the same dtype and strides (may be
    ``logits`` itself for the in-place form).  ``out`` may carry preallocated output tensors from an earlier
    call.  Returns a dict with dlogits, logp, logp_prox, loss (1-element tensor), stats (uint8 tensor, see
    STATS_DTYPE), the workspace, and entropy / iw / clipped when asked for.
    """
    torch = _torch()
    dt, T, V, ld = _logits_meta(logits, V)
    dev = logits.device
    _vec(chosen, torch.int32, T, "chosen")
    _vec(logp_behav, torch.float32, T, "logp_behav")
    if versions is not None:
        _vec(versions, torch.int32, T, "versions")
    _vec(advantages, torch.float32, T, "advantages")
    _vec(loss_mask, torch.uint8, T, "loss_mask")
    if logp_prox_in is not None:
        _vec(logp_prox_in, torch.float32, T, "logp_prox_in")
    if dlogits is None:
        dlogits = torch.empty_strided(logits.shape, logits.stride(), dtype=logits.dtype, device=dev)
    assert dlogits.dtype == logits.dtype and dlogits.shape == logits.shape and dlogits.stride() == logits.stride()
    need = workspace_bytes(T, V)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out = {} if out is None else out

    def buf(name, dtype, n=T):
        t = out.get(name)
        return t if t is not None else torch.empty(n, dtype=dtype, device=dev)

    logp, prox = buf("logp", torch.float32), buf("logp_prox", torch.float32)
    loss, stats = buf("loss", torch.float32, 1), buf("stats", torch.uint8, STATS_DTYPE.itemsize)
    ent = buf("entropy", torch.float32) if want_entropy else None
    iw = buf("iw", torch.float32) if want_iw else None
    clipped = buf("clipped", torch.uint8) if want_clipped else None
    args = [_ptr(logits), dt, T, V, ld, _ptr(chosen), _ptr(logp_behav), _ptr(versions), int(current_version),
            _ptr(advantages), _ptr(loss_mask), float(clip_eps), float(denom), _ptr(dlogits), _ptr(logp), _ptr(prox),
            _ptr(loss), _ptr(stats), _ptr(workspace), workspace.numel(), _stream()]
    extras = (events is not None or prox_mode != A3PO_PROX_INTERP or logp_prox_in is not None or want_entropy
              or want_iw or want_clipped or denom_dev is not None or accumulate)
    if not extras:
        _check(lib().a3po_loss_fwd_bwd(*args), "a3po_loss_fwd_bwd")
    else:
        ev = events if events is not None else (None, None)
        opt = LossOptions(int(prox_mode), int(bool(accumulate)), _ptr(logp_prox_in), _ptr(ent), _ptr(iw),
                          _ptr(clipped), ev[0], ev[1], _ptr(denom_dev))
        _check(lib().a3po_loss_fwd_bwd_ex(*args, ctypes.byref(opt)), "a3po_loss_fwd_bwd_ex")
    res = dict(dlogits=dlogits, logp=logp, logp_prox=prox, loss=loss, stats=stats, workspace=workspace)
    if want_entropy:
        res["entropy"] = ent
    if want_iw:
        res["iw"] = iw
    if want_clipped:
        res["clipped"] = clipped
    return res


NOALLOC_MAX_TOKENS = 131072  # A3PO_NOALLOC_MAX_TOKENS


def loss_fwd_bwd_noalloc(logits, chosen, logp_behav, versions, current_version: int, advantages, loss_mask,
                         clip_eps: float, denom: float, dlogits, logp, logp_prox, loss, stats, V=None):
    """a3po_loss_fwd_bwd_noalloc: every output tensor is the caller's (dlogits like logits, logp / logp_prox
    float32[T], loss float32[1], stats uint8[sizeof a3po_stats]; logp_prox and stats may be None); the call
    itself allocates nothing, here or in the library."""
    torch = _torch()
    dt, T, V, ld = _logits_meta(logits, V)
    _vec(chosen, torch.int32, T, "chosen")
    _vec(logp_behav, torch.float32, T, "logp_behav")
    _vec(versions, torch.int32, T, "versions")
    _vec(advantages, torch.float32, T, "advantages")
    _vec(loss_mask, torch.uint8, T, "loss_mask")
    assert dlogits.dtype == logits.dtype and dlogits.shape == logits.shape and dlogits.stride() == logits.stride()
    _vec(logp, torch.float32, T, "logp")
    if logp_prox is not None:
        _vec(logp_prox, torch.float32, T, "logp_prox")
    _vec(loss, torch.float32, 1, "loss")
    if stats is not None:
        _vec(stats, torch.uint8, STATS_DTYPE.itemsize, "stats")
    _check(lib().a3po_loss_fwd_bwd_noalloc(_ptr(logits), dt, T, V, ld, _ptr(chosen), _ptr(logp_behav), _ptr(versions),
                                           int(current_version), _ptr(advantages), _ptr(loss_mask), float(clip_eps),
                                           float(denom), _ptr(dlogits), _ptr(logp), _ptr(logp_prox), _ptr(loss),
                                           _ptr(stats), _stream()), "a3po_loss_fwd_bwd_noalloc")


def count_tokens(chosen, loss_mask, V: int, want_count=False):
    """a3po_count_tokens -> denom (1-element f32 device tensor) [, count (1-element i64 device tensor)]."""
    torch = _torch()
    T = chosen.numel()
    _vec(chosen, torch.int32, T, "chosen")
    _vec(loss_mask, torch.uint8, T, "loss_mask")
    denom = torch.empty(1, dtype=torch.float32, device=chosen.device)
    cnt = torch.empty(1, dtype=torch.int64, device=chosen.device) if want_count else None
    _check(lib().a3po_count_tokens(_ptr(chosen), _ptr(loss_mask), T, int(V), _ptr(denom), _ptr(cnt), _stream()),
           "a3po_count_tokens")
    return (denom, cnt) if want_count else denom


def histogram(values, edges, select=None, accumulate=False, out=None):
    """a3po_histogram -> counts int64[nbins + 3] on the device (below, bins..., at-or-above, NaN)."""
    torch = _torch()
    T = values.numel()
    _vec(values, torch.float32, T, "values")
    if select is not None:
        _vec(select, torch.uint8, T, "select")
    nbins = edges.numel() - 1
    _vec(edges, torch.float32, nbins + 1, "edges")
    if out is None:
        if accumulate:
            raise ValueError("accumulate needs the counts of the earlier calls in `out`")
        out = torch.empty(max(nbins, 0) + 3, dtype=torch.int64, device=values.device)
    else:
        _vec(out, torch.int64, nbins + 3, "out")
    _check(lib().a3po_histogram(_ptr(values), _ptr(select), T, _ptr(edges), nbins, int(bool(accumulate)), _ptr(out),
                                _stream()), "a3po_histogram")
    return out


def plan_microbatches(seq_len, n_minibatches: int, max_tokens: int, capacity=None):
    """a3po_plan_microbatches on a host int64 array -> (micro_first_seq[n+1], micro_minibatch[n]) NumPy arrays."""
    seq_len = np.ascontiguousarray(np.asarray(seq_len, dtype=np.int64))
    S = seq_len.shape[0]
    cap = S + int(max(n_minibatches, 0)) if capacity is None else int(capacity)
    first = np.zeros(max(cap, 0) + 1, dtype=np.int64)
    mb = np.zeros(max(cap, 1), dtype=np.int32)
    n = ctypes.c_int64(0)
    _check(lib().a3po_plan_microbatches(seq_len.ctypes.data, S, int(n_minibatches), int(max_tokens), first.ctypes.data,
                                        mb.ctypes.data, cap, ctypes.addressof(n)), "a3po_plan_microbatches")
    return first[:n.value + 1].copy(), mb[:n.value].copy()


def shard_partials(logits_shard, chosen, v0: int, Vs=None, out=None):
    """a3po_shard_partials -> partial[T, 4] f32 (max, sum_exp, chosen_logit, sum_exp_z) of one column shard."""
    torch = _torch()
    dt, T, Vs, ld = _logits_meta(logits_shard, Vs)
    _vec(chosen, torch.int32, T, "chosen")
    part = torch.empty((T, 4), dtype=torch.float32, device=logits_shard.device) if out is None else out
    assert part.is_contiguous() and part.dtype == torch.float32 and part.numel() == 4 * T
    _check(lib().a3po_shard_partials(_ptr(logits_shard), dt, T, Vs, ld, _ptr(chosen), int(v0), _ptr(part), _stream()),
           "a3po_shard_partials")
    return part


def shard_combine(partials, chosen, V: int, want_lse=True, want_entropy=False):
    """a3po_shard_combine on partials[P, T, 4] -> (logp[T], lse[T] | None, entropy[T] | None)."""
    torch = _torch()
    assert partials.is_cuda and partials.dtype == torch.float32 and partials.is_contiguous() and partials.dim() == 3
    P, T = partials.shape[0], partials.shape[1]
    _vec(chosen, torch.int32, T, "chosen")
    dev = partials.device
    logp = torch.empty(T, dtype=torch.float32, device=dev)
    lse = torch.empty(T, dtype=torch.float32, device=dev) if want_lse else None
    ent = torch.empty(T, dtype=torch.float32, device=dev) if want_entropy else None
    _check(lib().a3po_shard_combine(_ptr(partials), P, T, _ptr(chosen), int(V), _ptr(logp), _ptr(lse), _ptr(ent),
                                    _stream()), "a3po_shard_combine")
    return logp, lse, ent


def shard_loss_bwd(logits_shard, v0: int, V: int, chosen, logp_theta, lse, logp_behav, versions, current_version: int,
                   advantages, loss_mask, clip_eps: float, denom: float = 0.0, Vs=None, dlogits=None, workspace=None,
                   prox_mode: int = A3PO_PROX_INTERP, logp_prox_in=None, want_iw=False, want_clipped=False):
    """a3po_shard_loss_bwd -> dict(dlogits (the shard's slice), logp_prox, loss, stats, workspace[, iw, clipped])."""
    torch = _torch()
    dt, T, Vs, ld = _logits_meta(logits_shard, Vs)
    dev = logits_shard.device
    _vec(chosen, torch.int32, T, "chosen")
    for name, t in (("logp_theta", logp_theta), ("lse", lse), ("logp_behav", logp_behav), ("advantages", advantages)):
        _vec(t, torch.float32, T, name)
    if versions is not None:
        _vec(versions, torch.int32, T, "versions")
    _vec(loss_mask, torch.uint8, T, "loss_mask")
    if dlogits is None:
        dlogits = torch.empty_strided(logits_shard.shape, logits_shard.stride(), dtype=logits_shard.dtype, device=dev)
    assert dlogits.dtype == logits_shard.dtype and dlogits.shape == logits_shard.shape
    assert dlogits.stride() == logits_shard.stride()
    if workspace is None:
        workspace = torch.empty(workspace_bytes(T, V), dtype=torch.uint8, device=dev)
    prox = torch.empty(T, dtype=torch.float32, device=dev)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    stats = torch.empty(STATS_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    iw = torch.empty(T, dtype=torch.float32, device=dev) if want_iw else None
    clipped = torch.empty(T, dtype=torch.uint8, device=dev) if want_clipped else None
    opt = LossOptions(int(prox_mode), 0, _ptr(logp_prox_in), None, _ptr(iw), _ptr(clipped), None, None, None)
    _check(lib().a3po_shard_loss_bwd(_ptr(logits_shard), dt, T, Vs, ld, int(v0), int(V), _ptr(chosen),
                                     _ptr(logp_theta), _ptr(lse), _ptr(logp_behav), _ptr(versions),
                                     int(current_version), _ptr(advantages), _ptr(loss_mask), float(clip_eps),
                                     float(denom), _ptr(dlogits), _ptr(prox), _ptr(loss), _ptr(stats), _ptr(workspace),
                                     workspace.numel(), _stream(), ctypes.byref(opt)), "a3po_shard_loss_bwd")
    res = dict(dlogits=dlogits, logp_prox=prox, loss=loss, stats=stats, workspace=workspace)
    if want_iw:
        res["iw"] = iw
    if want_clipped:
        res["clipped"] = clipped
    return res


def fused_lmhead_logprob(hidden, weight, chosen, want_lse=True, workspace=None):
    """a3po_fused_lmhead_logprob -> (logp[T] f32, lse[T] f32 | None); hidden [T,H], weight [V,H] bfloat16."""
    torch = _torch()
    assert hidden.is_cuda and weight.is_cuda and hidden.dtype == torch.bfloat16 and weight.dtype == torch.bfloat16
    assert hidden.is_contiguous() and weight.is_contiguous() and hidden.dim() == 2 and weight.dim() == 2
    T, H = hidden.shape
    V = weight.shape[0]
    assert weight.shape[1] == H
    _vec(chosen, torch.int32, T, "chosen")
    need = workspace_bytes(T, V, H, which=A3PO_WS_FUSED_LMHEAD)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=hidden.device)
    logp = torch.empty(T, dtype=torch.float32, device=hidden.device)
    lse = torch.empty(T, dtype=torch.float32, device=hidden.device) if want_lse else None
    _check(lib().a3po_fused_lmhead_logprob(_ptr(hidden), _ptr(weight), T, H, V, _ptr(chosen), _ptr(logp), _ptr(lse),
                                           _ptr(workspace), workspace.numel(), _stream()), "a3po_fused_lmhead_logprob")
    return logp, lse


def fused_lmhead_loss_fwd_bwd(hidden, weight, chosen, logp_behav, versions, current_version: int, advantages,
                              loss_mask, clip_eps: float, denom: float = 0.0, workspace=None):
    """a3po_fused_lmhead_loss_fwd_bwd -> dict(dhidden, dweight, logp, logp_prox, loss, stats, workspace)."""
    torch = _torch()
    assert hidden.is_cuda and weight.is_cuda and hidden.dtype == torch.bfloat16 and weight.dtype == torch.bfloat16
    assert hidden.is_contiguous() and weight.is_contiguous() and hidden.dim() == 2 and weight.dim() == 2
    T, H = hidden.shape
    V = weight.shape[0]
    assert weight.shape[1] == H
    dev = hidden.device
    _vec(chosen, torch.int32, T, "chosen")
    _vec(logp_behav, torch.float32, T, "logp_behav")
    _vec(versions, torch.int32, T, "versions")
    _vec(advantages, torch.float32, T, "advantages")
    _vec(loss_mask, torch.uint8, T, "loss_mask")
    need = workspace_bytes(T, V, H, which=A3PO_WS_FUSED_LMHEAD_LOSS)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    dh = torch.empty_like(hidden)
    dw = torch.empty_like(weight)
    logp = torch.empty(T, dtype=torch.float32, device=dev)
    prox = torch.empty(T, dtype=torch.float32, device=dev)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    stats = torch.empty(STATS_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    _check(lib().a3po_fused_lmhead_loss_fwd_bwd(
        _ptr(hidden), _ptr(weight), T, H, V, _ptr(chosen), _ptr(logp_behav), _ptr(versions), int(current_version),
        _ptr(advantages), _ptr(loss_mask), float(clip_eps), float(denom), _ptr(dh), _ptr(dw), _ptr(logp), _ptr(prox),
        _ptr(loss), _ptr(stats), _ptr(workspace), workspace.numel(), _stream()), "a3po_fused_lmhead_loss_fwd_bwd")
    return dict(dhidden=dh, dweight=dw, logp=logp, logp_prox=prox, loss=loss, stats=stats, workspace=workspace)


def stats_to_dict(stats_tensor) -> dict:
    """Copies a device a3po_stats to the host (synchronises) and decodes it."""
    rec = np.frombuffer(stats_tensor.cpu().numpy().tobytes(), dtype=STATS_DTYPE)[0]
    return {k: rec[k].item() for k in STATS_DTYPE.names}
