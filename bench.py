#!/usr/bin/env python3
"""Benchmark of the VidKV hot path on one MI355X.

One "step" = one pass of the whole path over one batch of synthetic input
already resident in HBM: quantize keys (range pass, channel selection, coding
pass) and values (protected-token selection from scores, ternary coding pass)
through the one-call entry point, then one decode-attention step per layer
over the packed cache.

Prints ONE JSON line.  `value` is visual tokens per second through the whole
step; the per-kernel rooflines (algorithmic bytes / HIP-event time of that
kernel alone) and the CPU oracle's rate on a bounded sample ride along.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
SAL_HIDDEN, SAL_N_TEXT = 3584, 32   # hidden size of the 7B models, text-query tokens
BYTES_V_PER_ELEM = 0.2625      # 1.6-bit trits + one fp16 scale per 32 elements

# HBM bytes per launch (read + written) from hardware counters: rocprofv3 --pmc
# FETCH_SIZE and WRITE_SIZE, one counter per run, each kernel alone, scaled by
# what the same counters read for the library's copy kernel of known size
# (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000).  The runs and their commands are
# summarized in profiles/c4_long_hbm_traffic.md; a workload that was not
# counted reports null.
MEASURED_TRAFFIC_BYTES = {
    "c4_long": {"k_range": 200.75e6 + 0.78e6, "k_encode": 200.84e6 + 27.09e6,
                "v_encode": 201.59e6 + 41.40e6, "attn_partial": 68.61e6 + 1.86e6},
}


# The attention kernel is bound by vector-ALU issue, not by HBM: its second roofline is the
# number of VALU instructions it executes (rocprofv3 --pmc SQ_INSTS_VALU, per launch, MFMA
# instructions included; see profiles/c4_long_attention_valu.md) x 64 lanes against
# one instruction per lane and cycle on 256 CUs x 4 SIMDs x 16 lanes at 2.4 GHz.
MEASURED_VALU_INSTS = {"c4_long": {"attn_partial": 9.437e6}}
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def algorithmic_bytes(w):
    """Bytes the method itself must move, per kernel, for workload w."""
    N = w.L * w.B * w.Hkv * w.T * 128                       # elements per tensor
    k_packed = (w.n_anom * 12 + (128 - w.n_anom) * 8) / 4096 * N
    v_packed = BYTES_V_PER_ELEM * N
    rows = 2.0 * N * (w.n_salient / max(w.T, 1))
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


def cpu_baseline(w, budget_tokens=196000, budget_heads=4):
    """The oracle, as it stands, on a bounded sample: the first `budget_heads` KV heads of
    layer 0, sequence 0, first `budget_tokens` tokens, all query heads of those KV heads."""
    import numpy as np
    from oracle import vidkv_oracle as O
    from paper_2503_16257_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    T = min(w.T, budget_tokens) // 32 * 32
    nh = min(w.Hkv, budget_heads)
    n_s = (w.n_salient * T) // max(w.T, 1)
    sc = synth.saliency(w)[0, :T]
    rep = w.Hq // w.Hkv
    t_quant = t_attn = 0.0
    done = 0
    for h in range(nh):
        if t_quant + t_attn > 15.0:          # keep the leg bounded on a slow host
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
    # the sample is `done` of the Hkv KV heads of one layer of one sequence
    nh = done
    tok_equiv = T * nh / w.Hkv
    return {
        "value": tok_equiv / (t_quant + t_attn), "unit": "visual tokens/s", "cores": int(cores),
        "kind": "oracle",
        "sample": f"{nh} KV head(s) x {T} tokens of {w.name} (quantize K+V, select, 1 decode step); "
                  f"quantize {t_quant:.2f} s, attention {t_attn:.2f} s",
    }


def serving_sweep(vk, synth, torch, np, dev, iters):
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
        pk = vk.alloc_bytes(vk.packed_keys_bytes(p), dev)
        pv = vk.alloc_bytes(vk.packed_values_bytes(p), dev)
        ws = vk.alloc_bytes(max(vk.workspace_bytes(p, i) for i in range(4)), dev)
        sal = torch.from_numpy(synth.saliency(w)).to(dev) if w.n_salient else None
        t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
        t0.record()
        vk.quantize_kv(p, K, V, pk, pv, ws, saliency=sal)
        t1.record()
        torch.cuda.synchronize()
        t_q = t0.elapsed_time(t1) * 1e-3
        for _ in range(2):
            vk.decode_attention(p, 0, q, pk, pv, out, ws, K_tail=Kt, V_tail=Vt, tail_capacity=w.T_tail, tail_len=tl)
        t0.record()
        for _ in range(iters):
            vk.decode_attention(p, 0, q, pk, pv, out, ws, K_tail=Kt, V_tail=Vt, tail_capacity=w.T_tail, tail_len=tl)
        t1.record()
        torch.cuda.synchronize()
        t_a = t0.elapsed_time(t1) / iters * 1e-3
        ab = algorithmic_bytes(w)
        rows.append({"n_anom": w.n_anom, "protected_ratio": round(w.n_salient / w.T, 3),
                     "decode_attn_us": round(t_a * 1e6, 1),
                     "decode_attn_visual_tokens_per_s": round(w.B * w.T / t_a, 1),
                     "decode_attn_GBps": round(ab["attn_partial"] / t_a / 1e9, 1),
                     "frac_of_hbm_peak": round(ab["attn_partial"] / t_a / 1e9 / HBM_PEAK_GBS, 4),
                     "quantize_ms_first_call": round(t_q * 1e3, 3),
                     "quantize_GBps_fp16_input": round(ab["fp16_input"] / t_q / 1e9, 1)})
        del pk, pv, ws
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4_long")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-fft", action="store_true",
                    help="code the normal key channels with the non-FFT 1-bit quantizer (Eq. 4, n = 1) "
                         "instead of Eq. 5; not the headline configuration")
    ap.add_argument("--salient-bits", type=int, default=16, choices=[16, 2],
                    help="protected value tokens as fp16 rows (default) or at 2 bits (Alg. 2, STPQuant)")
    ap.add_argument("--kernel-iters", type=int, default=20)
    ap.add_argument("--serving-sweep", action="store_true",
                    help="also time decode attention at the 9 points of the batched-serving grid "
                         "(batch 64 x 25088 tokens + 256-token fp16 tail; n_anom in {8,16,32} x "
                         "protected ratio in {0, 5 %, 20 %}) and attach them as `serving_sweep`")
    ap.add_argument("--only", default=None,
                    choices=["k_range", "k_select", "k_encode", "v_select", "v_encode",
                             "attn_partial", "attn_merge", "copy", "saliency"],
                    help="profiling aid: after set-up run only this kernel --kernel-iters times "
                         "and exit without the JSON line")
    args = ap.parse_args()
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
    w = synth.WORKLOADS[args.workload]
    p = vk.make_params(w.L, w.B, w.Hkv, w.Hq, w.T, w.n_anom, w.n_salient,
                       gamma=float(np.float32(0.7)), use_fft=0 if args.no_fft else 1,
                       salient_bits=args.salient_bits)

    # ---- inputs, resident in HBM.  NROT independent copies are rotated so that
    # a step never finds its inputs in the 256 MB last-level cache.
    N = w.n_heads * w.T * 128
    in_bytes = 2 * N
    NROT = max(2, min(6, int(1.2e9 // max(in_bytes, 1)) + 1)) if in_bytes < 1.2e9 else 1
    K0 = torch.empty((w.L, w.B, w.Hkv, w.T, 128), dtype=torch.float16, device=dev)
    V0 = torch.empty_like(K0)
    for hd in range(w.n_heads):
        K0.view(-1, w.T, 128)[hd].copy_(torch.from_numpy(synth.key_head(w, hd)))
        V0.view(-1, w.T, 128)[hd].copy_(torch.from_numpy(synth.value_head(w, hd)))
    Ks = [K0] + [K0.clone() for _ in range(NROT - 1)]
    Vs = [V0] + [V0.clone() for _ in range(NROT - 1)]
    sal = torch.from_numpy(synth.saliency(w)).to(dev) if w.n_salient else None
    pkb, pvb = vk.packed_keys_bytes(p), vk.packed_values_bytes(p)
    AROT = max(2, min(16, int(6e8 // max(pkb + pvb, 1)) + 1))
    pks = [vk.alloc_bytes(pkb, dev) for _ in range(AROT)]
    pvs = [vk.alloc_bytes(pvb, dev) for _ in range(AROT)]
    ws = vk.alloc_bytes(max(vk.workspace_bytes(p, i) for i in range(4)), dev)
    qs = [torch.from_numpy(synth.query(w, l)).to(dev) for l in range(w.L)]
    out = torch.empty((w.B, w.Hq, 128), dtype=torch.float16, device=dev)
    cap = max(w.T_tail, 0)
    Kt = Vt = tl = None
    if cap:
        kt, vt = zip(*[synth.tail_heads(w, 0, b) for b in range(w.B)])
        Kt = torch.from_numpy(np.stack(kt)).to(dev)
        Vt = torch.from_numpy(np.stack(vt)).to(dev)
        tl = torch.full((w.B,), cap, dtype=torch.int32, device=dev)

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

    def q_keys(i, stages=None):
        vk.quantize_keys(p, Ks[i % NROT], pks[i % AROT], ws, stages=stages)

    def q_vals(i, stages=None):
        vk.quantize_values(p, Vs[i % NROT], pvs[i % AROT], ws, saliency=sal, stages=stages)

    def attn(i, stages=None):
        for l in range(w.L):
            vk.decode_attention(p, l, qs[l], pks[i % AROT], pvs[i % AROT], out, ws, K_tail=Kt,
                                V_tail=Vt, tail_capacity=cap, tail_len=tl, stages=stages, side=side)

    def q_kv(i):
        vk.quantize_kv(p, Ks[i % NROT], Vs[i % NROT], pks[i % AROT], pvs[i % AROT], ws, saliency=sal, side=side)

    def step(i):
        q_kv(i)
        attn(i)

    for i in range(AROT):                     # fill every rotated packed buffer once
        step(i)
    torch.cuda.synchronize()

    def timed(fn, iters, warm=2):
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fn(warm + i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e-3          # seconds per call

    if args.only:
        sel = {"k_range": lambda i: q_keys(i, 1), "k_select": lambda i: q_keys(i, 2),
               "k_encode": lambda i: q_keys(i, 4), "v_select": lambda i: q_vals(i, 1),
               "v_encode": lambda i: q_vals(i, 2), "attn_partial": lambda i: attn(i, 1),
               "attn_merge": lambda i: attn(i, 2),
               "copy": lambda i: vk.calib_copy(Vs[(i + 1) % NROT], Ks[i % NROT]),
               "saliency": saliency_scores}[args.only]
        t = timed(sel, args.kernel_iters)
        print(f"{args.only}: {t * 1e6:.2f} us per call over {args.kernel_iters} calls", file=sys.stderr)
        return

    # ---- the whole step: W warm-ups, exactly K timed steps
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps

    # ---- per-kernel times, each kernel alone between two events on its stream
    ab = algorithmic_bytes(w)
    it = args.kernel_iters
    kt = {
        "k_range": timed(lambda i: q_keys(i, 1), it),
        "k_select": timed(lambda i: q_keys(i, 2), it),
        "k_encode": timed(lambda i: q_keys(i, 4), it),
        "v_select": timed(lambda i: q_vals(i, 1), it) if w.n_salient else 0.0,
        "v_encode": timed(lambda i: q_vals(i, 2), it),
        "attn_partial": timed(lambda i: attn(i, 1), it) / w.L,
        "attn_merge": timed(lambda i: attn(i, 2), it) / w.L,
    }
    if Xv is not None:
        kt["saliency"] = timed(saliency_scores, max(2, it // 4))
    t_qk = timed(lambda i: q_keys(i), it)
    t_qv = timed(lambda i: q_vals(i), it)
    t_qkv = timed(lambda i: q_kv(i), it)
    t_at = timed(lambda i: attn(i), it)

    def roof(name, per_launch_div=1.0):
        a = ab[name] / per_launch_div / kt[name] / 1e9
        tr = MEASURED_TRAFFIC_BYTES.get(w.name, {}).get(name)
        return {"kernel": name, "bound": "hbm", "achieved": round(a, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(a / HBM_PEAK_GBS, 4),
                "traffic": None if tr is None else round(tr),
                "algorithmic_bytes": round(ab[name] / per_launch_div),
                "us": round(kt[name] * 1e6, 2)}

    roofs = [roof("k_range"), roof("k_encode"), roof("v_encode"), roof("attn_partial", w.L)]
    vi = MEASURED_VALU_INSTS.get(w.name, {}).get("attn_partial")
    if vi is not None and not args.no_fft and args.salient_bits == 16:
        ach = vi * 64 / kt["attn_partial"] / 1e12
        roofs[-1]["alu"] = {"bound": "alu", "achieved": round(ach, 2), "peak": round(VALU_PEAK_TLANEOPS, 2),
                            "unit": "T VALU lane-ops/s", "frac": round(ach / VALU_PEAK_TLANEOPS, 4),
                            "valu_instructions": round(vi)}
    dominant = max(roofs, key=lambda r: r["us"] * (w.L if r["kernel"] == "attn_partial" else 1))
    if "saliency" in kt:                       # outside the step, listed for its own roofline
        roofs.append(roof("saliency"))
    tokens = w.L * w.B * w.T
    res = {
        "metric": "visual tokens/s through quantize K + quantize V + 1 decode-attention step "
                  "(packed KV); quantize GB/s and decode-attn tokens/s alongside",
        "value": round(tokens / t_step, 1), "unit": "visual tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(t_step * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": w.name, "layers": w.L, "batch": w.B, "kv_heads": w.Hkv,
                   "q_heads": w.Hq, "t_quant": w.T, "t_tail": w.T_tail, "n_anom": w.n_anom,
                   "n_salient": w.n_salient, "input_rotation": NROT, "cache_rotation": AROT,
                   "key_normal_channels": "1-bit without FFT (Eq. 4)" if args.no_fft else "FFT 1-bit (Eq. 5)",
                   "protected_rows": "2-bit (Eq. 4)" if args.salient_bits == 2 else "fp16"},
        "quantize_GBps_fp16_input": round(ab["fp16_input"] / t_qkv / 1e9, 1),
        "quantize_ms": {"keys": round(t_qk * 1e3, 4), "values": round(t_qv * 1e3, 4),
                        "keys_and_values_one_call": round(t_qkv * 1e3, 4)},
        "decode_attn_visual_tokens_per_s": round(tokens / t_at, 1),
        "decode_attn_ms": round(t_at * 1e3, 4),
        "kernel_us": {k: round(v * 1e6, 2) for k, v in kt.items()},
        "roofline": {k: v for k, v in dominant.items() if k != "us"},
        "rooflines": roofs,
    }
    if args.serving_sweep:
        # release the main workload's tensors before the 3.3 GB of the serving shape
        del Ks, Vs, K0, V0, pks, pvs, Xv, Xt
        torch.cuda.empty_cache()
        res["serving_sweep"] = serving_sweep(vk, synth, torch, np, dev, args.kernel_iters)
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
