#!/usr/bin/env python3
"""Benchmark of the A-3PO loss forward+backward hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 8b|1p5b|long|tiny|lmhead8b]

One step = one pass of the whole path over one synthetic batch already resident in HBM:
GRPO advantages -> mask count / token records -> fused row kernel (log-softmax + gather,
proximal interpolation, clipped surrogate, gradient rows) -> loss and statistics reduction.
Prints ONE JSON line (see the keys below).  The CPU oracle is timed beside it on a bounded
row sample as a reported baseline.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak
METRIC = "tokens/sec and HBM GB/s (% peak) for A-3PO loss fwd+bwd, vocab 151,936, 1 GPU"


class HipEvents:
    """hipEvent pairs created through the HIP runtime directly (timing of one kernel on its stream)."""

    def __init__(self, n: int):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0 and self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self):
        out = []
        for a, b in self.pairs:
            ms = ctypes.c_float()
            assert self.hip.hipEventSynchronize(b) == 0
            assert self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
            out.append(ms.value)
        return out

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def build_inputs(w, torch, a3po, synth, log):
    """Synthetic batch of workload `w`, resident on the GPU.  Behaviour log-probs follow the recipe
    (target log-prob + noise, clamped); the target log-probs used for that come from
    a3po_token_logprobs here (parity of that entry point is the test suite's business)."""
    import numpy as np
    tk = synth.token_arrays(w)
    T, V = w.T, w.V
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    z = torch.empty((T, V), dtype=tdt, device="cuda")
    chunk = max(1, min(T, (1 << 30) // (V * w.elem_bytes)))
    t0 = time.time()
    for r0 in range(0, T, chunk):
        n = min(chunk, T - r0)
        rows = synth.logit_rows(w, r0, n, tk["chosen"])
        ten = torch.from_numpy(rows)
        z[r0:r0 + n].copy_(ten if w.dtype == "f32" else ten.view(torch.bfloat16))
    log(f"generated {T}x{V} {w.dtype} logits in {time.time() - t0:.1f}s")
    dev = lambda a: torch.from_numpy(a).cuda()
    chosen = dev(tk["chosen"])
    logp, _, _ = a3po.token_logprobs(z, chosen, want_lse=False, want_chosen_logit=False)
    lb = torch.clamp(logp + dev(tk["noise"]), max=0.0).contiguous()
    return dict(z=z, chosen=chosen, lb=lb, versions=dev(tk["versions"]), mask=dev(tk["mask"]),
                rewards=dev(tk["rewards"]), seq_id=dev(tk["seq_id"]), cur=tk["current_version"], tk=tk)


def time_steps(a3po, torch, w, b, mask, steps, warmup, dz, ws, out, adv, extra):
    """W untimed + K timed steps; returns (seconds for K steps, [ms of the row kernel per step])."""
    ev = HipEvents(steps)

    def step(events=None):
        a3po.grpo_advantages(b["rewards"], w.G, b["seq_id"], out=adv)
        a3po.loss_fwd_bwd(b["z"], b["chosen"], b["lb"], b["versions"], b["cur"], adv, mask, w.clip_eps,
                          dlogits=dz, workspace=ws, out=out, events=events, **extra)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(ev.pairs[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_ms = ev.elapsed_ms()
    ev.close()
    return dt, kernel_ms


def measured_traffic(workload: str, phase: str):
    """HBM bytes per launch of the row kernel taken from rocprofv3 counters (profiles/), or None when
    there is no record for this workload or the kernel sources changed since the counters were taken."""
    import hashlib
    rec = os.path.join(ROOT, "profiles", "hbm_traffic_loss_rows_kernel.txt")
    if not os.path.exists(rec):
        return None
    h = hashlib.sha256()
    for name in ("a3po_common.h", "a3po_rows.hip"):   # the row kernel and the helpers it inlines
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_2512_06547_amd", "csrc", name), "rb").read())
    table, sha = {}, None
    for line in open(rec):
        parts = line.split("#")[0].split()
        if len(parts) == 2 and parts[0] == "sources_sha256":
            sha = parts[1]
        elif len(parts) == 3:
            table[(parts[0], parts[1])] = float(parts[2])
    if sha != h.hexdigest():
        return None
    return table.get((workload, phase))


def algorithmic_bytes(w, n_counted):
    """Bytes the method itself must move per step: every counted row read once and its gradient row
    written once, every other row zero-filled once, plus the per-token side arrays."""
    row = w.V * w.elem_bytes
    return row * (2 * n_counted + (w.T - n_counted)) + 30 * w.T


def cpu_baseline(w, synth, oracle, rows, block=2048):
    """The oracle's whole path (advantages, forward, every gradient row, fp64) on the first `rows`
    tokens of the same workload, on the host cores, in blocks of `block` rows to bound memory.
    Only the oracle calls are timed; generating the rows is not."""
    import numpy as np
    tk = synth.token_arrays(w)
    total = 0.0
    for r0 in range(0, rows, block):
        n = min(block, rows - r0)
        sl = slice(r0, r0 + n)
        z = synth.logit_rows(w, r0, n, tk["chosen"])
        y = tk["chosen"][sl].copy()
        fwd = oracle.token_logprobs(z, y)                   # recipe input (not timed)
        lb = synth.behav_from_target(fwd["logp"], tk["noise"][sl])
        t0 = time.perf_counter()
        _, adv = oracle.grpo_advantages(tk["rewards"], w.G, seq_id=tk["seq_id"][sl].copy())
        oracle.loss_fwd_bwd(z, y, lb, tk["versions"][sl].copy(), tk["current_version"], adv.astype(np.float32),
                            tk["mask"][sl].copy(), w.clip_eps, denom=float(max(1, tk["mask"][:rows].sum())),
                            want_dz=True)
        total += time.perf_counter() - t0
    return rows / total, total


def secondary_kernels(a3po, torch, w, b, adv, dz, ws, log, reps=10, shards=8):
    """Context for the other vocabulary-wide kernels on the same batch (torch events on the current stream, which
    is the stream the binding launches on): forward-only log-probs with and without entropy (read-once:
    V * b bytes per row), and the vocabulary-sharded path on `shards` column views (forward partials: V * b per
    row; backward: V * b read + V * b written per live row, V * b written per dead row)."""
    T, V = w.T, w.V
    row = V * w.elem_bytes

    def timed(f):
        for _ in range(2):
            f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    res = {}
    # the stand-alone interpolation of Eq. 3 / Eq. 4 on its own (the step the paper times, Section 4.2.1): O(T)
    lt = a3po.token_logprobs(b["z"], b["chosen"], want_lse=False, want_chosen_logit=False)[0]
    ms = timed(lambda: a3po.proximal_interp(b["lb"], lt, b["versions"], b["cur"], want_alpha=False))
    res["proximal_interp"] = {"ms": ms, "tokens_per_s": T / ms * 1e3}
    ms = timed(lambda: a3po.token_logprobs(b["z"], b["chosen"], want_chosen_logit=False))
    res["token_logprobs"] = {"ms": ms, "gbs": T * row / ms / 1e6, "frac": T * row / ms / 1e6 / HBM_PEAK_GBS}
    ms = timed(lambda: a3po.token_logprobs(b["z"], b["chosen"], want_chosen_logit=False, want_entropy=True))
    res["token_logprobs_entropy"] = {"ms": ms, "gbs": T * row / ms / 1e6, "frac": T * row / ms / 1e6 / HBM_PEAK_GBS}
    if V % (shards * 8) == 0:
        Vs = V // shards
        parts = torch.empty((shards, T, 4), dtype=torch.float32, device="cuda")
        views = [b["z"][:, p * Vs:(p + 1) * Vs] for p in range(shards)]
        dviews = [dz[:, p * Vs:(p + 1) * Vs] for p in range(shards)]

        def fwd():
            for p in range(shards):
                a3po.shard_partials(views[p], b["chosen"], p * Vs, out=parts[p])
            return a3po.shard_combine(parts, b["chosen"], V)

        ms = timed(fwd)
        res["shard_forward"] = {"shards": shards, "ms": ms, "gbs": T * row / ms / 1e6,
                                "frac": T * row / ms / 1e6 / HBM_PEAK_GBS}
        logp, lse, _ = fwd()
        ones = torch.ones_like(b["mask"])
        last = {}

        def bwd():
            for p in range(shards):
                last.update(a3po.shard_loss_bwd(views[p], p * Vs, V, b["chosen"], logp, lse, b["lb"], b["versions"],
                                                b["cur"], adv, ones, w.clip_eps, dlogits=dviews[p], workspace=ws))

        ms = timed(bwd)
        st = a3po.stats_to_dict(last["stats"])
        live = int((adv != 0).sum().item()) - st["n_clipped"]   # rows whose gradient is not identically zero
        nbytes = row * (2 * live + (T - live))
        res["shard_backward"] = {"shards": shards, "ms": ms, "gbs": nbytes / ms / 1e6,
                                 "frac": nbytes / ms / 1e6 / HBM_PEAK_GBS, "live_rows": live}
    # fp32 logits at the full vocabulary: a row (594 KiB) no longer fits the registers; 16,384 rows of the batch
    # (every (T / 16,384)-th) widened to fp32, every row counted; bytes as for the row kernel (read + write per
    # counted row)
    if w.elem_bytes == 2 and T >= 16384:
        n32 = 16384
        pick = slice(0, T, T // n32)
        z32 = b["z"][pick].float()
        dz32 = torch.empty_like(z32)
        tok32 = {k: b[k][pick].contiguous() for k in ("chosen", "lb", "versions")}
        adv32 = adv[pick].contiguous()
        ones32 = torch.ones(n32, dtype=b["mask"].dtype, device="cuda")
        ws32 = torch.empty(a3po.workspace_bytes(n32, V), dtype=torch.uint8, device="cuda")
        last32 = {}

        def f32_step():
            last32.update(a3po.loss_fwd_bwd(z32, tok32["chosen"], tok32["lb"], tok32["versions"], b["cur"], adv32,
                                            ones32, w.clip_eps, V=V, dlogits=dz32, workspace=ws32))

        ms = timed(f32_step)
        nbytes = V * 4 * 2 * n32  # every row is counted: read once (its log-prob is an output) and written once
        res["fp32_full_vocabulary"] = {"rows": n32, "ms": ms, "gbs": nbytes / ms / 1e6,
                                       "frac": nbytes / ms / 1e6 / HBM_PEAK_GBS}
        del z32, dz32
    # the same batch as 4 gradient updates of micro-batches within the paper's 10,240-token budget (Section 4.1):
    # plan on the host, one token count per mini-batch kept on the device, one loss call per micro-batch
    import numpy as np
    first, owner = a3po.plan_microbatches(np.full(w.S, w.L, dtype=np.int64), 4, 10240)
    spans = [(int(first[i]) * w.L, int(first[i + 1]) * w.L, int(owner[i])) for i in range(len(owner))]
    mb_rows = {k: (min(a for a, _, o in spans if o == k), max(b_ for _, b_, o in spans if o == k))
               for k in set(owner.tolist())}
    mb_out = {}

    def minibatched():
        seen = set()
        for a, e, k in spans:
            if k not in seen:
                r0, r1 = mb_rows[k]
                mb_out[("denom", k)] = a3po.count_tokens(b["chosen"][r0:r1], b["mask"][r0:r1], V)
            o = mb_out.get(("out", k), {})
            mb_out[("out", k)] = a3po.loss_fwd_bwd(
                b["z"][a:e], b["chosen"][a:e], b["lb"][a:e], b["versions"][a:e], b["cur"], adv[a:e], b["mask"][a:e],
                w.clip_eps, V=V, dlogits=dz[a:e], workspace=ws, denom_dev=mb_out[("denom", k)], accumulate=k in seen,
                out=dict(loss=o.get("loss"), stats=o.get("stats"), logp=o.get("logp"), logp_prox=o.get("logp_prox")))
            seen.add(k)

    ms = timed(minibatched)
    res["minibatched_step"] = {"ms": ms, "calls": len(spans), "minibatches": len(mb_rows), "token_budget": 10240,
                               "tokens_per_s": T / ms * 1e3}
    for k, v in res.items():
        log(f"{k}: {v['ms']:.4f} ms" + (f", {v['gbs']:.0f} GB/s" if "gbs" in v else f", {v['tokens_per_s'] / 1e6:.2f} M tokens/s"))
    return res


MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 peak


def bench_lmhead(args, torch, a3po, synth, log, name=None, steps=None, warmup=None, cpu_rows=None):
    """The fused LM-head workload (hidden states x LM-head weight in front of the loss path): one step =
    GRPO advantages + a3po_fused_lmhead_loss_fwd_bwd (projection, loss, gradient rows, dh, dW).  The
    forward-only entry point (a3po_fused_lmhead_logprob) is timed beside it.  Returns the JSON line as a dict."""
    import numpy as np
    name = args.workload if name is None else name
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    cpu_rows = args.cpu_rows if cpu_rows is None else cpu_rows
    lw = synth.LMHEAD_WORKLOADS[name]
    w = lw.tokens
    T, H, V = w.T, lw.H, w.V
    tk = synth.token_arrays(w)
    t0 = time.time()
    W = torch.empty((V, H), dtype=torch.bfloat16, device="cuda")
    for v0 in range(0, V, 16384):
        n = min(16384, V - v0)
        W[v0:v0 + n].copy_(torch.from_numpy(synth.weight_rows(lw, v0, n)).view(torch.bfloat16))
    h = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, T, 16384):
        n = min(16384, T - r0)
        h[r0:r0 + n].copy_(torch.from_numpy(synth.hidden_rows(lw, r0, n)).view(torch.bfloat16))
    log(f"generated hidden {T}x{H} and weight {V}x{H} in {time.time() - t0:.1f}s")
    dev = lambda a: torch.from_numpy(a).cuda()
    y = dev(tk["chosen"])
    ws_f = torch.empty(a3po.workspace_bytes(T, V, H, which=1), dtype=torch.uint8, device="cuda")
    logp, _ = a3po.fused_lmhead_logprob(h, W, y, workspace=ws_f)
    lb = torch.clamp(logp + dev(tk["noise"]), max=0.0).contiguous()
    ver, mask, rewards, seq_id = dev(tk["versions"]), dev(tk["mask"]), dev(tk["rewards"]), dev(tk["seq_id"])
    ws = torch.empty(a3po.workspace_bytes(T, V, H, which=2), dtype=torch.uint8, device="cuda")
    adv = torch.empty(T, dtype=torch.float32, device="cuda")

    def run_phase(m, label):
        """K timed steps with loss mask m.  Only counted tokens are projected, so the algorithmic flops are
        6 N V H with N the counted tokens (forward, dh, dW; the logits of a chunk are kept, not recomputed)."""
        def step():
            a3po.grpo_advantages(rewards, w.G, seq_id, out=adv)
            return a3po.fused_lmhead_loss_fwd_bwd(h, W, y, lb, ver, tk["current_version"], adv, m, w.clip_eps,
                                                  workspace=ws)
        out = step()
        for _ in range(warmup):
            out = step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            out = step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st = a3po.stats_to_dict(out["stats"])
        ms = dt / steps * 1e3
        flops = 6.0 * st["n_tokens"] * V * H
        tf = flops / (ms * 1e-3) / 1e12
        log(f"fwd+bwd, {label}: {ms:.1f} ms/step, {st['n_tokens']} counted tokens, {tf:.0f} TFLOP/s on 6 N V H, "
            f"{T / ms * 1e3 / 1e3:.0f} k tokens/s")
        return dict(dt=dt, ms=ms, st=st, flops=flops, tf=tf)

    rag = run_phase(mask, "workload's mask")
    one = run_phase(torch.ones_like(mask), "all-ones mask")
    dt, ms, st, flops, tf = rag["dt"], rag["ms"], rag["st"], rag["flops"], rag["tf"]

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a3po.fused_lmhead_logprob(h, W, y, workspace=ws_f)
    e0.record()
    nf = max(1, steps // 2)
    for _ in range(nf):
        a3po.fused_lmhead_logprob(h, W, y, workspace=ws_f)
    e1.record()
    torch.cuda.synchronize()
    fms = e0.elapsed_time(e1) / nf
    ftf = 2.0 * T * V * H / (fms * 1e-3) / 1e12
    log(f"fused forward only: {fms:.1f} ms, {ftf:.0f} TFLOP/s on 2TVH")

    cpu = None
    if cpu_rows > 0:
        import oracle
        n = 16
        hh = synth.hidden_rows(lw, 0, n)
        Wh = np.concatenate([synth.weight_rows(lw, v0, min(16384, V - v0)) for v0 in range(0, V, 16384)])
        t0 = time.perf_counter()
        z = oracle.lmhead_logits(hh, Wh)
        oracle.token_logprobs(z, tk["chosen"][:n].copy())
        secs = time.perf_counter() - t0
        cpu = {"value": n / secs, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"projection + log-softmax (forward only, fp64) of the first {n} tokens, {secs:.2f} s wall"}
        log(f"oracle forward: {n / secs:.2f} tokens/s on {oracle.threads()} threads")

    line = {
        "metric": "tokens/sec and MFMA TFLOP/s (% peak) for A-3PO loss fwd+bwd through the LM head, "
                  "hidden 4,096 x vocab 151,936, 1 GPU",
        "value": T * steps / dt, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{lw.name}: {w.S} seq x {w.L} tok = {T} tokens, hidden {H}, vocab {V}, bf16; logits "
                               f"only counted tokens are projected ({st['n_tokens']}; 6 N V H flops), their logits kept in fp32 8,192 tokens at a time",
                   "tokens": T, "hidden": H, "vocab": V, "counted_tokens": st["n_tokens"]},
        "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "flops": flops,
                     "kernel": "whole step (gemm_nt_kernel x 3 per chunk of 8,192 counted tokens + lmhead_dz_kernel)",
                     # not an achieved rate: the flops of a path that projects every token (6 T V H) over this
                     # step's time, for comparison with such paths; this one skips the tokens outside the loss
                     "dense_equivalent_tflops": 6.0 * T * V * H / (ms * 1e-3) / 1e12},
        "all_rows_counted": {"value": T * steps / one["dt"], "unit": "tokens/s", "ms_per_step": one["ms"],
                             "roofline": {"bound": "mfma", "achieved": one["tf"], "peak": MFMA_BF16_PEAK_TFLOPS,
                                          "unit": "TFLOP/s", "frac": one["tf"] / MFMA_BF16_PEAK_TFLOPS,
                                          "flops": one["flops"]}},
        "fused_forward": {"ms": fms, "roofline": {"bound": "mfma", "achieved": ftf, "peak": MFMA_BF16_PEAK_TFLOPS,
                                                  "unit": "TFLOP/s", "frac": ftf / MFMA_BF16_PEAK_TFLOPS,
                                                  "flops": 2.0 * T * V * H, "kernel": "gemm_nt_kernel (log-sum-exp epilogue)"}},
        "cpu_baseline": cpu,
    }
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="8b",
                    help="8b (default: the largest single-GPU logits workload), 1p5b, long, tiny, lmhead8b")
    ap.add_argument("--cpu-rows", type=int, default=32768, help="rows of the oracle baseline sample (0 = skip)")
    ap.add_argument("--phase", default="both", choices=["both", "ragged", "ones"],
                    help="time the workload's own mask, an all-ones mask, or both (default)")
    ap.add_argument("--entropy", action="store_true",
                    help="also compute the per-token policy entropy in the row kernel (a3po_loss_fwd_bwd_ex)")
    ap.add_argument("--no-secondary", dest="secondary", action="store_false",
                    help="skip the short timing of the forward-only and vocabulary-sharded kernels")
    ap.add_argument("--no-lmhead-leg", dest="lmhead_leg", action="store_false",
                    help="skip the short run of the LM-head workload (lmhead8b) reported under secondary_kernels")
    ap.add_argument("--quiet", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2512_06547_amd as a3po
    import synth

    log = (lambda *a: None) if args.quiet else (lambda *a: print("[bench]", *a, file=sys.stderr, flush=True))
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    a3po.lib()
    torch.cuda.set_device(0)
    if args.workload in synth.LMHEAD_WORKLOADS:
        print(json.dumps(bench_lmhead(args, torch, a3po, synth, log)), flush=True)
        return
    w = synth.WORKLOADS[args.workload]
    b = build_inputs(w, torch, a3po, synth, log)

    dz = torch.empty_like(b["z"])
    ws = torch.empty(a3po.workspace_bytes(w.T, w.V), dtype=torch.uint8, device="cuda")
    adv = torch.empty(w.T, dtype=torch.float32, device="cuda")
    out = {}
    extra = {"want_entropy": True} if args.entropy else {}
    first_mask = b["mask"] if args.phase in ("both", "ragged") else torch.ones_like(b["mask"])
    out.update(a3po.loss_fwd_bwd(b["z"], b["chosen"], b["lb"], b["versions"], b["cur"],
                                 a3po.grpo_advantages(b["rewards"], w.G, b["seq_id"], out=adv), first_mask,
                                 w.clip_eps, dlogits=dz, workspace=ws, **extra))
    torch.cuda.synchronize()
    log(f"stats: {a3po.stats_to_dict(out['stats'])} loss={float(out['loss'].cpu()[0]):.6f}")

    def phase(mask, label):
        dt_, kms_ = time_steps(a3po, torch, w, b, mask, args.steps, args.warmup, dz, ws, out, adv, extra)
        torch.cuda.synchronize()
        st_ = a3po.stats_to_dict(out["stats"])
        kavg_ = sum(kms_) / len(kms_)
        nbytes = algorithmic_bytes(w, st_["n_tokens"])
        gbs = nbytes / (kavg_ * 1e-3) / 1e9
        log(f"{label}: {dt_ / args.steps * 1e3:.3f} ms/step, row kernel {kavg_:.3f} ms, {gbs:.0f} GB/s "
            f"({st_['n_tokens']} counted tokens)")
        ks = sorted(kms_)
        return dict(dt=dt_, kavg=kavg_, kmed=ks[len(ks) // 2], kmin=ks[0], bytes=nbytes, gbs=gbs, st=st_)

    # the workload's own ragged mask is the headline; the all-ones mask is the case that cannot
    # skip anything (every row read once and written once)
    rag = phase(b["mask"], "ragged mask") if args.phase in ("both", "ragged") else None
    one = phase(torch.ones_like(b["mask"]), "all-ones mask") if args.phase in ("both", "ones") else None
    head = rag if rag is not None else one
    dt, kavg, bytes_cfg, ach, st = head["dt"], head["kavg"], head["bytes"], head["gbs"], head["st"]

    # context only: a plain device copy of the same matrix (read + write), the practical ceiling
    # of a mixed read/write stream on this machine
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        dz.copy_(b["z"])
    e0.record()
    for _ in range(10):
        dz.copy_(b["z"])
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * b["z"].numel() * w.elem_bytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    log(f"plain copy of the logits matrix: {copy_gbs:.0f} GB/s (read+write)")

    secondary = secondary_kernels(a3po, torch, w, b, adv, dz, ws, log) if args.secondary else None

    if args.secondary and args.lmhead_leg:
        # the LM-head workload on the same box in the same run: a few steps of the whole path from hidden states
        leg = bench_lmhead(args, torch, a3po, synth, log, name="lmhead8b", steps=3, warmup=1, cpu_rows=0)
        secondary["lmhead8b"] = {k: leg[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "config",
                                                      "roofline", "all_rows_counted", "fused_forward")}

    cpu = None
    if args.cpu_rows > 0:
        import oracle
        rows = min(args.cpu_rows, w.T)
        tps, secs = cpu_baseline(w, synth, oracle, rows)
        cpu = {"value": tps, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"whole path (fwd + all gradient rows, fp64) on the first {rows} rows of the same workload, "
                         f"{secs:.2f} s wall"}
        log(f"oracle: {tps:.1f} tokens/s on {oracle.threads()} threads ({secs:.2f}s for {rows} rows)")

    line = {
        "metric": METRIC,
        "value": w.T * args.steps / dt,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.S} seq x {w.L} tok = {w.T} tokens, vocab {w.V}, {w.dtype} logits, "
                               f"GRPO group {w.G}, staleness 0..{w.stale_max}, "
                               f"{'ragged mask' if rag is not None else 'all-ones mask'} "
                               f"({st['n_tokens']} counted tokens), separate gradient buffer"
                               f"{', per-token entropy' if args.entropy else ''}",
                   "tokens": w.T, "vocab": w.V, "counted_tokens": st["n_tokens"], "clipped_tokens": st["n_clipped"]},
        "roofline": {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": ach / HBM_PEAK_GBS,
                     "traffic": measured_traffic(w.name, "ragged" if rag is not None else "ones"),
                     "kernel": "loss_rows_kernel",
                     "kernel_ms": kavg, "kernel_ms_median": head["kmed"], "kernel_ms_min": head["kmin"],
                     "algorithmic_bytes": bytes_cfg},
        "all_rows_counted": None if one is None or rag is None else {
            "value": w.T * args.steps / one["dt"], "unit": "tokens/s", "ms_per_step": one["dt"] / args.steps * 1e3,
            "roofline": {"bound": "hbm", "achieved": one["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": one["gbs"] / HBM_PEAK_GBS, "traffic": measured_traffic(w.name, "ones"),
                         "kernel_ms": one["kavg"], "kernel_ms_median": one["kmed"], "kernel_ms_min": one["kmin"],
                         "algorithmic_bytes": one["bytes"]}},
        "cpu_baseline": cpu,
        "plain_copy_gbs": copy_gbs,
        "secondary_kernels": secondary,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
