"""ctypes front end of the CPU oracle (``a3po_oracle.c``).

Test infrastructure only: the product package never imports this module.  All
floating-point results are float64.  Logits are float32 arrays or bfloat16 bit
patterns held in uint16 arrays; per-token float inputs are widened exactly to
float64 before the call.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "a3po_oracle.c")
_LIB = os.path.join(_HERE, "liba3po_oracle.so")

F32, BF16, F64 = 0, 1, 2


class Stats(ctypes.Structure):
    _fields_ = [("n_tokens", ctypes.c_int64), ("n_clipped", ctypes.c_int64),
                ("n_bad_index", ctypes.c_int64), ("n_negative_staleness", ctypes.c_int64),
                ("iw_min", ctypes.c_double), ("iw_max", ctypes.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-Wall", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None
_P = ctypes.c_void_p
_I64 = ctypes.c_int64
_I32 = ctypes.c_int32
_F64 = ctypes.c_double


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.a3po_oracle_threads.restype = ctypes.c_int
        lib.a3po_oracle_token_logprobs.restype = None
        lib.a3po_oracle_token_logprobs.argtypes = [_P, ctypes.c_int, _I64, _I64, _I64, _P, _P, _P, _P]
        lib.a3po_oracle_alpha.restype = None
        lib.a3po_oracle_alpha.argtypes = [_P, _I32, _I64, _P]
        lib.a3po_oracle_proximal_interp.restype = None
        lib.a3po_oracle_proximal_interp.argtypes = [_P, _P, _P, _I32, _I64, _P, _P]
        lib.a3po_oracle_grpo_advantages.restype = ctypes.c_int
        lib.a3po_oracle_grpo_advantages.argtypes = [_P, _I64, _I32, _F64, _P, _I64, _P, _P]
        lib.a3po_oracle_surrogate.restype = None
        lib.a3po_oracle_surrogate.argtypes = [_P, _P, _P, _I32, _P, _P, _F64, _F64, _I64,
                                              _P, _P, _P, _P, _P, _P, _P, _P]
        lib.a3po_oracle_decoupled_clip.restype = None
        lib.a3po_oracle_decoupled_clip.argtypes = [_P, _P, _P, _P, _P, _F64, _F64, _I64,
                                                   _P, _P, _P, _P, _P, _P, _P]
        lib.a3po_oracle_dlogits_rows.restype = None
        lib.a3po_oracle_dlogits_rows.argtypes = [_P, ctypes.c_int, _I64, _I64, _P, _P, _P, _P, _I64, _P]
        lib.a3po_oracle_loss_fwd_bwd.restype = None
        lib.a3po_oracle_loss_fwd_bwd.argtypes = [_P, ctypes.c_int, _I64, _I64, _I64, _P, _P, _P, _I32,
                                                 _P, _P, _F64, _F64, _P, _P, _P, _P, _P, _P, _P, _P, _P]
        lib.a3po_oracle_entropy.restype = None
        lib.a3po_oracle_entropy.argtypes = [_P, ctypes.c_int, _I64, _I64, _I64, _P]
        lib.a3po_oracle_lmhead_logits.restype = None
        lib.a3po_oracle_lmhead_logits.argtypes = [_P, _P, _I64, _I64, _P, _I64, _P]
        lib.a3po_oracle_lmhead_backward.restype = None
        lib.a3po_oracle_lmhead_backward.argtypes = [_P, _P, _P, _I64, _I64, _I64, _P, _P]
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().a3po_oracle_threads())


def _logits(z):
    z = np.ascontiguousarray(z)
    assert z.ndim == 2
    if z.dtype == np.float32:
        return z, F32
    if z.dtype == np.uint16:
        return z, BF16
    if z.dtype == np.float64:
        return z, F64
    raise TypeError("logits must be float32, float64 or uint16 (bfloat16 bits)")


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int32
    return a


def _u8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint8
    return a


def token_logprobs(z, y, V=None):
    """-> dict(logp[T], lse[T], chosen_raw[T] stored bits)."""
    z, dt = _logits(z)
    T, ld = z.shape
    V = ld if V is None else V
    y = _i32(y)
    logp = np.empty(T)
    lse = np.empty(T)
    raw = np.empty(T, dtype={F32: np.uint32, BF16: np.uint16, F64: np.float64}[dt])
    _load().a3po_oracle_token_logprobs(z.ctypes.data, dt, T, V, ld, y.ctypes.data,
                                       logp.ctypes.data, lse.ctypes.data, raw.ctypes.data)
    return dict(logp=logp, lse=lse, chosen_raw=raw)


def entropy(z, V=None):
    """Per-token policy entropy -sum p log p of softmax(z)."""
    z, dt = _logits(z)
    T, ld = z.shape
    V = ld if V is None else V
    out = np.empty(T)
    _load().a3po_oracle_entropy(z.ctypes.data, dt, T, V, ld, out.ctypes.data)
    return out


def alpha(versions, current_version):
    v = _i32(versions)
    out = np.empty(v.shape[0])
    _load().a3po_oracle_alpha(v.ctypes.data, int(current_version), v.shape[0], out.ctypes.data)
    return out


def proximal_interp(lb, lt, versions, current_version):
    lb, lt, v = _f64(lb), _f64(lt), _i32(versions)
    T = v.shape[0]
    lp = np.empty(T)
    al = np.empty(T)
    _load().a3po_oracle_proximal_interp(lb.ctypes.data, lt.ctypes.data, v.ctypes.data,
                                        int(current_version), T, lp.ctypes.data, al.ctypes.data)
    return lp, al


def grpo_advantages(rewards, G, seq_id=None, eps_adv=1e-6):
    R = _f64(rewards)
    S = R.shape[0]
    adv_seq = np.empty(S)
    if seq_id is None:
        rc = _load().a3po_oracle_grpo_advantages(R.ctypes.data, S, int(G), float(eps_adv), None, 0,
                                                 adv_seq.ctypes.data, None)
        if rc != 0:
            raise ValueError("bad group structure")
        return adv_seq
    sid = _i32(seq_id)
    adv_tok = np.empty(sid.shape[0])
    rc = _load().a3po_oracle_grpo_advantages(R.ctypes.data, S, int(G), float(eps_adv), sid.ctypes.data,
                                             sid.shape[0], adv_seq.ctypes.data, adv_tok.ctypes.data)
    if rc != 0:
        raise ValueError("bad group structure")
    return adv_seq, adv_tok


def surrogate(lt, lb, versions, current_version, A, mask, clip_eps, denom=0.0):
    """Eq. 2 with Eq. 3/4 per token.  -> dict(lp, iw, r, obj, g, clipped, loss, stats)."""
    lt, lb, A = _f64(lt), _f64(lb), _f64(A)
    v, m = _i32(versions), _u8(mask)
    T = v.shape[0]
    lp, iw, r, obj, g = (np.empty(T) for _ in range(5))
    cl = np.empty(T, dtype=np.uint8)
    loss = ctypes.c_double(0.0)
    st = Stats()
    _load().a3po_oracle_surrogate(lt.ctypes.data, lb.ctypes.data, v.ctypes.data, int(current_version),
                                  A.ctypes.data, m.ctypes.data, float(clip_eps), float(denom), T,
                                  lp.ctypes.data, iw.ctypes.data, r.ctypes.data, obj.ctypes.data,
                                  g.ctypes.data, cl.ctypes.data, ctypes.addressof(loss),
                                  ctypes.addressof(st))
    return dict(lp=lp, iw=iw, r=r, obj=obj, g=g, clipped=cl, loss=loss.value, stats=st.as_dict())


def decoupled_clip(lt, lb, lp, A, mask, clip_eps, denom=0.0):
    """Eq. 2 for a given proximal log-prob.  -> dict(iw, r, obj, g, clipped, loss, stats)."""
    lt, lb, lp, A = _f64(lt), _f64(lb), _f64(lp), _f64(A)
    m = _u8(mask)
    T = m.shape[0]
    iw, r, obj, g = (np.empty(T) for _ in range(4))
    cl = np.empty(T, dtype=np.uint8)
    loss = ctypes.c_double(0.0)
    st = Stats()
    _load().a3po_oracle_decoupled_clip(lt.ctypes.data, lb.ctypes.data, lp.ctypes.data, A.ctypes.data,
                                       m.ctypes.data, float(clip_eps), float(denom), T,
                                       iw.ctypes.data, r.ctypes.data, obj.ctypes.data, g.ctypes.data,
                                       cl.ctypes.data, ctypes.addressof(loss), ctypes.addressof(st))
    return dict(iw=iw, r=r, obj=obj, g=g, clipped=cl, loss=loss.value, stats=st.as_dict())


def dlogits_rows(z, y, lse, g, rows, V=None):
    """Dense float64 gradient rows [len(rows), V] for the listed absolute rows."""
    z, dt = _logits(z)
    T, ld = z.shape
    V = ld if V is None else V
    y, lse, g = _i32(y), _f64(lse), _f64(g)
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    out = np.empty((rows.shape[0], V))
    _load().a3po_oracle_dlogits_rows(z.ctypes.data, dt, V, ld, y.ctypes.data, lse.ctypes.data,
                                     g.ctypes.data, rows.ctypes.data, rows.shape[0], out.ctypes.data)
    return out


def loss_fwd_bwd(z, y, lb, versions, current_version, A, mask, clip_eps, denom=0.0, V=None,
                 want_dz=True):
    """Whole path.  -> dict(logp, lse, lp, g, eff_mask, clipped, dz (or None), loss, stats)."""
    z, dt = _logits(z)
    T, ld = z.shape
    V = ld if V is None else V
    y, v, m = _i32(y), _i32(versions), _u8(mask)
    lb, A = _f64(lb), _f64(A)
    logp, lse, lp, g = (np.empty(T) for _ in range(4))
    eff = np.empty(T, dtype=np.uint8)
    cl = np.empty(T, dtype=np.uint8)
    dz = np.empty((T, V)) if want_dz else None
    loss = ctypes.c_double(0.0)
    st = Stats()
    _load().a3po_oracle_loss_fwd_bwd(z.ctypes.data, dt, T, V, ld, y.ctypes.data, lb.ctypes.data,
                                     v.ctypes.data, int(current_version), A.ctypes.data, m.ctypes.data,
                                     float(clip_eps), float(denom), logp.ctypes.data, lse.ctypes.data,
                                     lp.ctypes.data, g.ctypes.data, eff.ctypes.data, cl.ctypes.data,
                                     dz.ctypes.data if want_dz else None, ctypes.addressof(loss),
                                     ctypes.addressof(st))
    return dict(logp=logp, lse=lse, lp=lp, g=g, eff_mask=eff, clipped=cl, dz=dz, loss=loss.value,
                stats=st.as_dict())


def _bf16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16 and a.ndim == 2
    return a


def lmhead_logits(h, W, rows=None):
    """z[rows, :] = h[rows] @ W.T in float64 from bfloat16 bit patterns (h [T,H], W [V,H], uint16)."""
    h, W = _bf16(h), _bf16(W)
    T, H = h.shape
    V = W.shape[0]
    assert W.shape[1] == H
    rows = np.arange(T, dtype=np.int64) if rows is None else np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    z = np.empty((rows.shape[0], V))
    _load().a3po_oracle_lmhead_logits(h.ctypes.data, W.ctypes.data, H, V, rows.ctypes.data, rows.shape[0],
                                      z.ctypes.data)
    return z


def lmhead_backward(dz, h, W, want_dh=True, want_dw=True):
    """dh = dz @ W, dW = dz.T @ h in float64 (dz [T,V] float64; h, W bfloat16 bit patterns)."""
    h, W = _bf16(h), _bf16(W)
    dz = _f64(dz)
    T, H = h.shape
    V = W.shape[0]
    assert dz.shape == (T, V)
    dh = np.empty((T, H)) if want_dh else None
    dW = np.empty((V, H)) if want_dw else None
    _load().a3po_oracle_lmhead_backward(dz.ctypes.data, h.ctypes.data, W.ctypes.data, T, H, V,
                                        dh.ctypes.data if want_dh else None, dW.ctypes.data if want_dw else None)
    return dh, dW


def lmhead_backward_matmul(dz, h, W):
    """The two products of ``lmhead_backward``, dh = dz @ W and dW = dz.T @ h, through NumPy's float64 matrix
    product instead of the plain loops: the same definition (bfloat16 operands widened exactly, float64 products
    and sums; only the order of the additions is the library's), for sizes at which the loops would take minutes.
    Pinned against the loops in tests/test_oracle_pins.py."""
    h, W = _bf16(h), _bf16(W)
    dz = _f64(dz)
    hf = (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    Wf = (W.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return dz @ Wf, dz.T @ hf


def plan_microbatches(seq_len, n_minibatches, max_tokens):
    """Reference plan of the mini-batch / micro-batch split (Section 4.1: 4 gradient updates per step,
    at most 10,240 tokens per pass), in plain Python.

    Mini-batch k holds sequences [k*S//n, (k+1)*S//n).  Inside a mini-batch sequences are taken in
    order; a non-empty sequence that would push the open micro-batch past ``max_tokens`` closes it and
    opens the next one (so a sequence longer than the budget sits alone).  Returns
    (micro_first_seq, micro_minibatch) as lists: micro-batch i = sequences
    micro_first_seq[i] .. micro_first_seq[i+1]-1.
    """
    S = len(seq_len)
    first, owner = [], []
    for k in range(n_minibatches):
        lo, hi = k * S // n_minibatches, (k + 1) * S // n_minibatches
        tokens = None                      # None: no micro-batch open in this mini-batch yet
        for s in range(lo, hi):
            n = int(seq_len[s])
            if tokens is None or (tokens > 0 and n > 0 and tokens + n > max_tokens):
                first.append(s)
                owner.append(k)
                tokens = 0
            tokens += n
    first.append(S)
    return first, owner


def histogram(values, edges, select=None):
    """Counts of a per-token quantity over bins with explicit edges (the distribution behind the
    importance-weight extrema and clipped-token counts of Section 4.2.2).

    ``edges`` is a non-decreasing array of nbins + 1 numbers.  Returns int64[nbins + 3]:
    [0] selected values below edges[0]; [1 + k] values with edges[k] <= v < edges[k+1];
    [nbins + 1] values >= edges[nbins]; [nbins + 2] NaNs.  ``select`` (optional) keeps token t only
    when select[t] != 0.  Values and edges are compared as given (float32 compares are exact in any
    wider type), so the counts are integers with no rounding question.
    """
    v = np.asarray(values, dtype=np.float64).ravel()
    e = np.asarray(edges, dtype=np.float64).ravel()
    if select is not None:
        v = v[np.asarray(select).ravel() != 0]
    nbins = len(e) - 1
    counts = np.zeros(nbins + 3, dtype=np.int64)
    for x in v:
        if x != x:
            counts[nbins + 2] += 1
            continue
        k = 0                              # number of edges that are <= x
        while k <= nbins and e[k] <= x:
            k += 1
        counts[k] += 1
    return counts
