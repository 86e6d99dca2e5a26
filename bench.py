#!/usr/bin/env python3
"""Benchmark of the VidKV hot path on one MI355X.

One "step" = one pass of the whole path over one batch of synthetic input
already resident in HBM: quantize keys (range pass, channel selection, coding
pass) and values (protected-token selection from scores, ternary coding pass)
through the one-call entry point, then one decode-attention step per layer
over the packed cache.

Prints ONE JSON line.  `value` is visual tokens per second through the whole
step on the long-video workload.  Riding along, all measured in this run:
  - per-kernel rooflines: algorithmic bytes / HIP-event time of that kernel
    alone (average, median and minimum over --kernel-iters launches), against
    the published HBM peak and against the library's own copy kernel
    (`ceiling`); the headline `roofline` is the hot kernel with the LOWEST
    fraction of peak;
  - hardware-counter figures (HBM traffic, VALU instruction count) only when
    the summary under profiles/ that holds them was written for exactly the
    kernel sources of this tree (a hash of the sources is kept with them),
    else null;
  - the other workloads (one layer, the 28-layer stack, the serving grid);
  - the CPU oracle on a bounded sample, with one thread and with all threads.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
SAL_HIDDEN, SAL_N_TEXT = 3584, 32   # hidden size of the 7B models, text-query tokens
# algorithmic size of the ternary code: 1.6-bit trits (5 per byte) + one fp16 scale per 32
# elements.  (The stored record spends 2 bits per trit, 0.3125 B per element.)
BYTES_V_PER_ELEM = 0.2625
# vector-ALU issue peak: one instruction per lane and cycle on 256 CUs x 4 SIMDs x 16 lanes
# at the 2.4 GHz peak clock
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def kernel_sources_hash() -> str:
    """SHA-256 over the device sources and the ABI header: what a counter summary under
    profiles/ must have been measured on to be quoted."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2503_16257_amd", "csrc")
    files = sorted(os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith((".hip", ".h")))
    files.append(os.path.join(ROOT, "include", "vidkv.h"))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def profiled_counters(workload: str) -> dict:
    """Counter figures from the summaries under profiles/ (lines `bench-data: <key> <kernel>
    <number>` and `bench-data: sources <hash>`), each file taken only if its hash matches
    this tree's kernel sources."""
    out = {"traffic": {}, "valu": {}, "stale": []}
    here = kernel_sources_hash()
    pdir = os.path.join(ROOT, "profiles")
    for fn in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not fn.startswith(workload) or not fn.endswith(".md"):
            continue
        with open(os.path.join(pdir, fn)) as fh:
            rows = re.findall(r"^bench-data:[ \t]+(\S+)[ \t]+(\S+)(?:[ \t]+(\S+))?[ \t]*$", fh.read(), re.M)
        if not rows:
            continue
        src = [r[1] for r in rows if r[0] == "sources"]
        if not src or src[0] != here:
            out["stale"].append(fn)
            continue
        for key, kern, num in rows:
            if key == "traffic_bytes":
                out["traffic"][kern] = float(num)
            elif key == "valu_instructions":
                out["valu"][kern] = float(num)
    return out


def algorithmic_bytes(w, salient_bits=16):
    """Bytes the method itself must move, per kernel, for workload w."""
    N = w.L * w.B * w.Hkv * w.T * 128                       # elements per tensor
    k_packed = (w.n_anom * 12 + (128 - w.n_anom) * 8) / 4096 * N
    v_packed = BYTES_V_PER_ELEM * N
    row_bytes = 2.0 if salient_bits != 2 else 0.375
    rows = row_bytes * N * (w.n_salient / max(w.T, 1))
    tail = 2 * 2 * w.L * w.B * w.Hkv * w.T_tail * 128
    qo = 2 * 2 * w.L * w.B * w.Hq * 128
    return {
        "k_range": 2.0 * N,
        "k_encode": 2.0 * N + k_packed,
        "v_encode": 2.0 * N + v_packed + rows + (4.0 * w.B * w.T if w.n_salient else 0.0),
        "attn_partial": k_packed + v_packed + rows + tail + qo,
        "fp16_input": 2 * 2.0 * N,
        # saliency scores (Eq. 7): visual and text hidden states once, scores out
        "saliency": 2.0 * w.B * (w.T + SAL_N_TEXT) * SAL_HIDDEN + 4.0 * w.B * w.T,
    }


def _oracle_pass(w, T, nh, budget_s):
    """One timed pass of the oracle over up to `nh` KV heads x T tokens; (heads done, s, s)."""
    import numpy as np
    from oracle import vidkv_oracle as O
    from paper_2503_16257_amd import synth
    n_s = (w.n_salient * T) // max(w.T, 1)
    sc = synth.saliency(w)[0, :T]
    rep = w.Hq // w.Hkv
    t_quant = t_attn = 0.0
    done = 0
    for h in range(nh):
        if t_quant + t_attn > budget_s:      # keep the leg bounded on a slow host
            break
        done += 1
        K = synth.key_head(w, h)[:T]
        V = synth.value_head(w, h)[:T]
        q = synth.query(w, 0)[0, h * rep:(h + 1) * rep]
        t0 = time.perf_counter()
        rec = O.quantize_keys_head(K, w.n_anom)
        sal = O.select_salient_tokens(sc, n_s)
        qv = O.ternary_quant(V, sal, float(np.float32(0.7)))
        t1 = time.perf_counter()
        Kd = O.dequantize_keys_head(rec)
        Vd = O.ternary_dequant(qv["codes"], qv["s16"], sal, qv["rows"])
        for j in range(rep):
            O.attention_single_query(q[j], Kd, Vd, 1.0 / np.sqrt(128.0))
        t2 = time.perf_counter()
        t_quant += t1 - t0
        t_attn += t2 - t1
    return done, t_quant, t_attn


def cpu_baseline(w, budget_tokens=196000, budget_heads=4, budget_s=10.0):
    """The oracle, as it stands, on a bounded sample: KV heads of layer 0, sequence 0, first
    `budget_tokens` tokens, all query heads of those KV heads - once with every numeric
    thread pool held to one thread, once with the pools as the host gives them."""
    from threadpoolctl import threadpool_info, threadpool_limits
    import numpy  # noqa: F401  (loads the BLAS whose pool is limited below)
    T = min(w.T, budget_tokens) // 32 * 32
    nh = min(w.Hkv, budget_heads)
    legs = {}
    with threadpool_limits(limits=1):
        legs["one_thread"] = (1,) + _oracle_pass(w, T, nh, budget_s)
    pool = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    legs["all_threads"] = (int(pool),) + _oracle_pass(w, T, nh, budget_s)

    def rate(leg):
        cores, done, tq, ta = leg
        return {"value": round(T * done / w.Hkv / (tq + ta), 1), "cores": cores,
                "heads_sampled": done, "quantize_s": round(tq, 2), "attention_s": round(ta, 2)}

    one, allt = rate(legs["one_thread"]), rate(legs["all_threads"])
    return {
        "value": allt["value"], "unit": "visual tokens/s", "cores": allt["cores"], "kind": "oracle",
        "sample": f"up to {nh} KV head(s) x {T} tokens of {w.name} (quantize K+V, select, 1 decode "
                  f"step over all query heads of those KV heads), {budget_s:.0f} s budget per leg",
        "one_thread": one, "all_threads": allt, "nproc": os.cpu_count(),
        "sched_affinity": len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else None,
    }


class Timer:
    """Launch times from events on torch's current stream (the stream the binding launches on)."""

    def __init__(self, torch):
        self.torch = torch

    def launches(self, fn, iters, batch=5, warm=3):
        """`iters` launches in batches of `batch` back-to-back launches, each batch between two
        events: average over all, median and minimum of the batch means, seconds per launch."""
        torch = self.torch
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        nb = max(1, iters // batch)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(nb)]
        k = warm
        for e0, e1 in ev:
            e0.record()
            for _ in range(batch):
                fn(k)
                k += 1
            e1.record()
        torch.cuda.synchronize()
        per = [e0.elapsed_time(e1) / batch * 1e-3 for e0, e1 in ev]
        return {"avg": sum(per) / len(per), "median": statistics.median(per), "min": min(per),
                "launches": nb * batch, "batch": batch}

    def mean(self, fn, iters, warm=2):
        return self.launches(fn, iters, batch=max(1, iters), warm=warm)["avg"]


class Job:
    """One workload resident on the device: rotated inputs and packed buffers, and the calls."""

    def __init__(self, vk, synth, torch, np, w, dev, side, use_fft=1, salient_bits=16,
                 from_host=False, in_budget=1.2e9, cache_budget=6e8):
        self.vk, self.torch, self.w, self.side = vk, torch, w, side
        self.p = vk.make_params(w.L, w.B, w.Hkv, w.Hq, w.T, w.n_anom, w.n_salient,
                                gamma=float(np.float32(0.7)), use_fft=use_fft,
                                salient_bits=salient_bits)
        p = self.p
        # NROT independent copies are rotated so that a step never finds its inputs in the
        # 256 MB last-level cache
        in_bytes = 2 * w.n_heads * w.T * 128
        self.NROT = max(2, min(6, int(in_budget // max(in_bytes, 1)) + 1)) if in_bytes < in_budget else 1
        if from_host:
            K0 = torch.empty((w.L, w.B, w.Hkv, w.T, 128), dtype=torch.float16, device=dev)
            V0 = torch.empty_like(K0)
            for hd in range(w.n_heads):
                K0.view(-1, w.T, 128)[hd].copy_(torch.from_numpy(synth.key_head(w, hd)))
                V0.view(-1, w.T, 128)[hd].copy_(torch.from_numpy(synth.value_head(w, hd)))
        else:
            K0, V0 = synth.device_kv(w, dev)
        self.Ks = [K0] + [K0.clone() for _ in range(self.NROT - 1)]
        self.Vs = [V0] + [V0.clone() for _ in range(self.NROT - 1)]
        self.sal = torch.from_numpy(synth.saliency(w)).to(dev) if w.n_salient else None
        pkb, pvb = vk.packed_keys_bytes(p), vk.packed_values_bytes(p)
        self.AROT = max(2, min(16, int(cache_budget // max(pkb + pvb, 1)) + 1))
        self.pks = [vk.alloc_bytes(pkb, dev) for _ in range(self.AROT)]
        self.pvs = [vk.alloc_bytes(pvb, dev) for _ in range(self.AROT)]
        self.ws = vk.alloc_bytes(max(vk.workspace_bytes(p, i) for i in range(4)), dev)
        self.qs = [torch.from_numpy(synth.query(w, l)).to(dev) for l in range(w.L)]
        self.out = torch.empty((w.B, w.Hq, 128), dtype=torch.float16, device=dev)
        self.cap = max(w.T_tail, 0)
        self.Kt = self.Vt = self.tl = None
        if self.cap:
            g = torch.Generator(device=dev); g.manual_seed(20250316 + w.cfg_id)
            self.Kt = torch.randn((w.B, w.Hkv, self.cap, 128), generator=g, device=dev).to(torch.float16)
            self.Vt = torch.randn((w.B, w.Hkv, self.cap, 128), generator=g, device=dev).to(torch.float16)
            self.tl = torch.full((w.B,), self.cap, dtype=torch.int32, device=dev)
        for i in range(self.AROT):                # fill every rotated packed buffer once
            self.q_kv(i)
        torch.cuda.synchronize()

    def q_keys(self, i, stages=None):
        self.vk.quantize_keys(self.p, self.Ks[i % self.NROT], self.pks[i % self.AROT], self.ws, stages=stages)

    def q_vals(self, i, stages=None):
        self.vk.quantize_values(self.p, self.Vs[i % self.NROT], self.pvs[i % self.AROT], self.ws,
                                saliency=self.sal, stages=stages)

    def attn(self, i, stages=None):
        for l in range(self.w.L):
            self.vk.decode_attention(self.p, l, self.qs[l], self.pks[i % self.AROT], self.pvs[i % self.AROT],
                                     self.out, self.ws, K_tail=self.Kt, V_tail=self.Vt,
                                     tail_capacity=self.cap, tail_len=self.tl, stages=stages,
                                     side=self.side)

    def q_kv(self, i):
        self.vk.quantize_kv(self.p, self.Ks[i % self.NROT], self.Vs[i % self.NROT], self.pks[i % self.AROT],
                            self.pvs[i % self.AROT], self.ws, saliency=self.sal, side=self.side)

    def step(self, i):
        self.q_kv(i)
        self.attn(i)


def other_workload(vk, synth, torch, np, tm, name, dev, side, steps):
    """Step and attention time of one of the smaller configurations."""
    w = synth.WORKLOADS[name]
    job = Job(vk, synth, torch, np, w, dev, side, in_budget=8e9, cache_budget=2e9)
    t_step = tm.mean(job.step, steps)
    t_at = tm.mean(job.attn, steps)
    t_q = tm.mean(job.q_kv, steps)
    ab = algorithmic_bytes(w)
    res = {"workload": name, "layers": w.L, "batch": w.B, "t_quant": w.T, "n_anom": w.n_anom,
           "n_salient": w.n_salient, "steps": steps,
           "ms_per_step": round(t_step * 1e3, 4),
           "visual_tokens_per_s": round(w.L * w.B * w.T / t_step, 1),
           "quantize_ms": round(t_q * 1e3, 4),
           "quantize_GBps_fp16_input": round(ab["fp16_input"] / t_q / 1e9, 1),
           "decode_attn_us_per_layer": round(t_at / w.L * 1e6, 2),
           "decode_attn_GBps": round(ab["attn_partial"] / t_at / 1e9, 1),
           "decode_attn_frac_of_hbm_peak": round(ab["attn_partial"] / t_at / 1e9 / HBM_PEAK_GBS, 4)}
    del job
    torch.cuda.empty_cache()
    return res


def serving_sweep(vk, synth, torch, np, tm, dev, side, iters):
    """Decode attention over the packed cache at every point of the batched-serving grid."""
    pts = synth.serving_sweep()
    w0 = pts[0]
    K, V = synth.device_kv(w0, dev)                      # the tensors do not depend on the grid point
    g = torch.Generator(device=dev); g.manual_seed(20250316)
    Kt = torch.randn((w0.B, w0.Hkv, w0.T_tail, 128), generator=g, device=dev).to(torch.float16)
    Vt = torch.randn((w0.B, w0.Hkv, w0.T_tail, 128), generator=g, device=dev).to(torch.float16)
    tl = torch.full((w0.B,), w0.T_tail, dtype=torch.int32, device=dev)
    q = torch.from_numpy(synth.query(w0, 0)).to(dev)
    out = torch.empty((w0.B, w0.Hq, 128), dtype=torch.float16, device=dev)
    rows = []
    for w in pts:
        p = vk.make_params(w.L, w.B, w.Hkv, w.Hq, w.T, w.n_anom, w.n_salient, gamma=float(np.float32(0.7)))
        # two sets of packed buffers (0.9 GB together): alternate calls read different ones
        pk = [vk.alloc_bytes(vk.packed_keys_bytes(p), dev) for _ in range(2)]
        pv = [vk.alloc_bytes(vk.packed_values_bytes(p), dev) for _ in range(2)]
        ws = vk.alloc_bytes(max(vk.workspace_bytes(p, i) for i in range(4)), dev)
        sal = torch.from_numpy(synth.saliency(w)).to(dev) if w.n_salient else None
        vk.quantize_kv(p, K, V, pk[0], pv[0], ws, saliency=sal, side=side)
        t_q = tm.mean(lambda i: vk.quantize_kv(p, K, V, pk[i & 1], pv[i & 1], ws, saliency=sal, side=side), 3, warm=1)

        def attn(i, stages=None):
            vk.decode_attention(p, 0, q, pk[i & 1], pv[i & 1], out, ws, K_tail=Kt, V_tail=Vt,
                                tail_capacity=w.T_tail, tail_len=tl, side=side, stages=stages)
        t_a = tm.mean(attn, iters)
        t_p = tm.mean(lambda i: attn(i, 1), iters)
        ab = algorithmic_bytes(w)
        rows.append({"n_anom": w.n_anom, "protected_ratio": round(w.n_salient / w.T, 3),
                     "decode_attn_us": round(t_a * 1e6, 1),
                     "attn_partial_and_tail_us": round(t_p * 1e6, 1),
                     "decode_attn_visual_tokens_per_s": round(w.B * w.T / t_a, 1),
                     "decode_attn_GBps": round(ab["attn_partial"] / t_a / 1e9, 1),
                     "frac_of_hbm_peak": round(ab["attn_partial"] / t_a / 1e9 / HBM_PEAK_GBS, 4),
                     "quantize_ms": round(t_q * 1e3, 3),
                     "quantize_GBps_fp16_input": round(ab["fp16_input"] / t_q / 1e9, 1)})
        del pk, pv, ws
    del K, V
    torch.cuda.empty_cache()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4_long")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the other workloads (one layer, the 28-layer stack, the serving grid)")
    ap.add_argument("--no-fft", action="store_true",
                    help="code the normal key channels with the non-FFT 1-bit quantizer (Eq. 4, n = 1) "
                         "instead of Eq. 5; not the headline configuration")
    ap.add_argument("--salient-bits", type=int, default=16, choices=[16, 2],
                    help="protected value tokens as fp16 rows (default) or at 2 bits (Alg. 2, STPQuant)")
    ap.add_argument("--kernel-iters", type=int, default=100)
    ap.add_argument("--sources-hash", action="store_true",
                    help="print the hash of the kernel sources (what a counter summary under "
                         "profiles/ records) and exit")
    ap.add_argument("--only", default=None,
                    choices=["k_range", "k_select", "k_encode", "v_select", "v_encode",
                             "attn_partial", "attn_merge", "copy", "saliency"],
                    help="profiling aid: after set-up run only this kernel --kernel-iters times "
                         "and exit without the JSON line")
    args = ap.parse_args()
    if args.sources_hash:
        print(kernel_sources_hash())
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2503_16257_amd import binding as vk
    from paper_2503_16257_amd import synth

    vk.lib()                                  # fail loudly if the library is not built
    dev = "cuda:0"
    side = vk.SideStream(dev)                 # the caller's side stream for the two calls that fork
    tm = Timer(torch)
    w = synth.WORKLOADS[args.workload]
    job = Job(vk, synth, torch, np, w, dev, side, use_fft=0 if args.no_fft else 1,
              salient_bits=args.salient_bits, from_host=True)

    # hidden states for the saliency scores (not part of the step: the scores are an input
    # of quantize_values; timed alone).  1.4 GB at the long-video shape, far beyond the LLC.
    Xv = Xt = None
    if w.n_salient and w.B * w.T * SAL_HIDDEN * 2 < 8e9:
        g = torch.Generator(device=dev); g.manual_seed(20250316)
        Xv = torch.randn((w.B, w.T, SAL_HIDDEN), generator=g, device=dev, dtype=torch.float16)
        Xt = torch.randn((w.B, SAL_N_TEXT, SAL_HIDDEN), generator=g, device=dev, dtype=torch.float16)
        sal_out = torch.empty((w.B, w.T), dtype=torch.float32, device=dev)
        sal_ws = vk.alloc_bytes(vk.saliency_workspace_bytes(w.B, SAL_HIDDEN), dev)

    def saliency_scores(i):
        vk.saliency_scores(Xv, Xt, sal_out, sal_ws)

    def copy(i):
        vk.calib_copy(job.Vs[(i + 1) % job.NROT], job.Ks[i % job.NROT])

    single = {"k_range": lambda i: job.q_keys(i, 1), "k_select": lambda i: job.q_keys(i, 2),
              "k_encode": lambda i: job.q_keys(i, 4), "v_select": lambda i: job.q_vals(i, 1),
              "v_encode": lambda i: job.q_vals(i, 2), "attn_partial": lambda i: job.attn(i, 1),
              "attn_merge": lambda i: job.attn(i, 2), "copy": copy, "saliency": saliency_scores}

    if args.only:
        t = tm.mean(single[args.only], args.kernel_iters)
        print(f"{args.only}: {t * 1e6:.2f} us per call over {args.kernel_iters} calls", file=sys.stderr)
        return

    # ---- the whole step: W warm-ups, exactly K timed steps
    for i in range(args.warmup):
        job.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        job.step(args.warmup + i)
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps

    # ---- per-kernel times, each kernel alone between events on its stream
    ab = algorithmic_bytes(w, args.salient_bits)
    it = args.kernel_iters
    names = ["k_range", "k_select", "k_encode", "v_encode", "attn_partial", "attn_merge", "copy"]
    if w.n_salient:
        names.insert(3, "v_select")
    kt = {n: tm.launches(single[n], it) for n in names}
    for n in ("attn_partial", "attn_merge"):             # one launch per layer inside a call
        kt[n] = {k: (v / w.L if k in ("avg", "median", "min") else v) for k, v in kt[n].items()}
    if Xv is not None:
        kt["saliency"] = tm.launches(saliency_scores, max(10, it // 5))
    calls = {"keys": tm.launches(job.q_keys, it), "values": tm.launches(job.q_vals, it),
             "keys_and_values_one_call": tm.launches(job.q_kv, it),
             "decode_attention": tm.launches(job.attn, it)}

    # the library's streaming copy kernel in this run: what a kernel that only moves bytes reaches
    copy_bytes = 2.0 * 2 * w.n_heads * w.T * 128
    ceiling = copy_bytes / kt["copy"]["avg"] / 1e9
    prof = profiled_counters(w.name) if (not args.no_fft and args.salient_bits == 16) else \
        {"traffic": {}, "valu": {}, "stale": []}

    def roof(name, launches_per_call=1.0):
        t = kt[name]
        a = ab[name] / launches_per_call / t["avg"] / 1e9
        tr = prof["traffic"].get(name)
        return {"kernel": name, "bound": "hbm", "achieved": round(a, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(a / HBM_PEAK_GBS, 4),
                "traffic": None if tr is None else round(tr),
                "algorithmic_bytes": round(ab[name] / launches_per_call),
                "us": round(t["avg"] * 1e6, 2), "us_median": round(t["median"] * 1e6, 2),
                "us_min": round(t["min"] * 1e6, 2), "launches": t["launches"],
                "ceiling": round(ceiling, 1), "frac_of_ceiling": round(a / ceiling, 4)}

    roofs = [roof("k_range"), roof("k_encode"), roof("v_encode"), roof("attn_partial", w.L)]
    vi = prof["valu"].get("attn_partial")
    if vi is not None:
        ach = vi * 64 / kt["attn_partial"]["avg"] / 1e12
        roofs[-1]["alu"] = {"bound": "alu", "achieved": round(ach, 2), "peak": round(VALU_PEAK_TLANEOPS, 2),
                            "unit": "T VALU lane-ops/s", "frac": round(ach / VALU_PEAK_TLANEOPS, 4),
                            "valu_instructions": round(vi)}
    headline = min(roofs, key=lambda r: r["frac"])       # the hot kernel furthest from its roofline
    if "saliency" in kt:                                  # outside the step, listed for its own roofline
        roofs.append(roof("saliency"))
    tokens = w.L * w.B * w.T
    three = ("keys", "values", "keys_and_values_one_call")
    res = {
        "metric": "visual tokens/s through quantize K + quantize V + 1 decode-attention step "
                  "(packed KV); quantize GB/s and decode-attn tokens/s alongside",
        "value": round(tokens / t_step, 1), "unit": "visual tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(t_step * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": w.name, "layers": w.L, "batch": w.B, "kv_heads": w.Hkv,
                   "q_heads": w.Hq, "t_quant": w.T, "t_tail": w.T_tail, "n_anom": w.n_anom,
                   "n_salient": w.n_salient, "input_rotation": job.NROT, "cache_rotation": job.AROT,
                   "key_normal_channels": "1-bit without FFT (Eq. 4)" if args.no_fft else "FFT 1-bit (Eq. 5)",
                   "protected_rows": "2-bit (Eq. 4)" if args.salient_bits == 2 else "fp16"},
        "quantize_GBps_fp16_input": round(ab["fp16_input"] / calls["keys_and_values_one_call"]["avg"] / 1e9, 1),
        "quantize_ms": {k: round(calls[k]["avg"] * 1e3, 4) for k in three},
        "quantize_ms_median": {k: round(calls[k]["median"] * 1e3, 4) for k in three},
        "quantize_ms_min": {k: round(calls[k]["min"] * 1e3, 4) for k in three},
        "decode_attn_visual_tokens_per_s": round(tokens / calls["decode_attention"]["avg"], 1),
        "decode_attn_ms": round(calls["decode_attention"]["avg"] * 1e3, 4),
        "decode_attn_ms_median": round(calls["decode_attention"]["median"] * 1e3, 4),
        "decode_attn_ms_min": round(calls["decode_attention"]["min"] * 1e3, 4),
        "kernel_us": {k: round(v["avg"] * 1e6, 2) for k, v in kt.items()},
        "kernel_us_median": {k: round(v["median"] * 1e6, 2) for k, v in kt.items()},
        "kernel_us_min": {k: round(v["min"] * 1e6, 2) for k, v in kt.items()},
        "kernel_timing": {"launches": it, "batch": kt["k_range"]["batch"],
                          "note": "batches of back-to-back launches of one kernel between two events on "
                                  "its stream; avg over all launches, median and min over the batch means"},
        "ceiling": {"kernel": "calib_copy", "GBps": round(ceiling, 1), "bytes": round(copy_bytes),
                    "us": round(kt["copy"]["avg"] * 1e6, 2),
                    "note": "the library's streaming copy of the key tensor, read + written bytes"},
        "roofline": dict(headline),
        "rooflines": roofs,
        "counters": {"kernel_sources": kernel_sources_hash(),
                     "quoted_from_profiles": bool(prof["traffic"] or prof["valu"]),
                     "stale_profiles_ignored": prof["stale"]},
    }
    if not args.no_others:
        # release the main workload's tensors before the GB-sized shapes
        del job, Xv, Xt, single
        torch.cuda.empty_cache()
        res["other_workloads"] = [
            other_workload(vk, synth, torch, np, tm, "c2_layer", dev, side, 20),
            other_workload(vk, synth, torch, np, tm, "c3_stack", dev, side, 5),
        ]
        res["serving_sweep"] = serving_sweep(vk, synth, torch, np, tm, dev, side, 20)
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
