"""GPU parity at the full sizes of the five workloads, in the launch
configuration the benchmark times.  Whole tensors are drawn on the device; the
oracle checks sampled heads (copied back bit for bit) and sampled sequences."""
import numpy as np
import pytest
import torch

import parity as P
from paper_2503_16257_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check_heads(run, K, V, heads, scores_np):
    w = run.w
    stats = {}
    sal = {}
    for hd in heads:
        b = (hd // w.Hkv) % w.B
        if b not in sal:
            sal[b] = P.oracle_salient(w, b, None if scores_np is None else scores_np[b], None)
        Kh = K.view(-1, w.T, 128)[hd].cpu().numpy()
        Vh = V.view(-1, w.T, 128)[hd].cpu().numpy()
        P.check_keys_head(run, hd, Kh, stats)
        P.check_values_head(run, hd, Vh, sal[b], stats)
    P.check_near_budget(stats)
    return stats


@pytest.mark.parametrize("mode", ["headline", "one_bit_keys_two_bit_protected_rows"])
def test_long_video_full_size(mode):
    """1000 frames = 196000 tokens, 4 KV x 28 Q heads, n_a = 16, 9800 protected; in the
    headline configuration and with the non-FFT key code plus 2-bit protected rows, followed
    there by a flush of a 128-token residual block."""
    w = synth.WORKLOADS["c4_long"]
    print(f"[case] c4_long full {mode}", flush=True)
    alt = mode != "headline"
    K, V = synth.device_kv(w, DEV)
    scores = synth.saliency(w)
    run = P.GpuRun(w, DEV, K=K, V=V, saliency=torch.from_numpy(scores).to(DEV),
                   use_fft=0 if alt else 1, salient_bits=2 if alt else 0,
                   t_capacity=w.T + 128 if alt else 0)
    heads = list(range(w.n_heads))                           # all 4 KV heads
    _check_heads(run, K, V, heads, scores)
    print(f"[step] codec ok on {len(heads)} of {w.n_heads} heads", flush=True)
    q = synth.query(w, 0)
    out = run.attention(0, torch.from_numpy(q).to(DEV)).cpu().numpy()
    ref = P.oracle_attention(run, 0, 0, q[0])
    err = P.assert_out_close(out[0], ref, "c4_long")
    print(f"[step] attention ok on all {w.Hq} query heads, max err {err:.2e}", flush=True)
    if alt:
        import test_gpu_flush as F
        Kt = np.stack([synth.tail_heads(w, 0, b, 128)[0] for b in range(w.B)])
        Vt = np.stack([synth.tail_heads(w, 0, b, 128)[1] for b in range(w.B)])
        run.flush(0, torch.from_numpy(Kt).to(DEV), torch.from_numpy(Vt).to(DEV), 128, 128)
        run.advance(128)
        stats = {}
        for h in range(w.Hkv):
            F._check_block(run, h, w.T // 32, Kt[0, h], Vt[0, h], stats)
        P.check_near_budget(stats)
        q = synth.query(w, 0, step=1)
        out = run.attention(0, torch.from_numpy(q).to(DEV)).cpu().numpy()
        err = P.assert_out_close(out[0], P.oracle_attention(run, 0, 0, q[0]), "c4_long after flush")
        print(f"[step] flush + attention ok, max err {err:.2e}", flush=True)


def test_full_stack_16_decode_steps():
    """28 layers x batch 8 x 12544 tokens; 16 decode steps, one fp16 token appended per step."""
    w = synth.WORKLOADS["c3_stack"]
    print("[case] c3_stack full", flush=True)
    K, V = synth.device_kv(w, DEV)
    run = P.GpuRun(w, DEV, K=K, V=V)
    # one head of every layer, the sequence and KV head moving with the layer
    heads = [(l * w.B + (3 * l + 1) % w.B) * w.Hkv + (l % w.Hkv) for l in range(w.L)]
    heads[0], heads[-1] = 0, w.n_heads - 1
    _check_heads(run, K, V, heads, None)
    print(f"[step] codec ok on {len(heads)} heads, one per layer", flush=True)
    del K, V
    cap = 16
    # residual buffers of every layer: [L][B, Hkv, cap, 128]
    Kt = torch.zeros((w.L, w.B, w.Hkv, cap, 128), dtype=torch.float16, device=DEV)
    Vt = torch.zeros_like(Kt)
    tl = torch.zeros((w.B,), dtype=torch.int32, device=DEV)
    # (layer, sequence) pairs checked by the oracle: every layer, the sequence moving with it
    sample = [(l, (5 * l + 2) % w.B) for l in range(w.L)]
    sample[0], sample[-1] = (0, 0), (w.L - 1, w.B - 1)
    gen = torch.Generator(device=DEV); gen.manual_seed(77)
    for step in range(w.decode_steps):
        newk = torch.randn((w.L, w.B, w.Hkv, 128), generator=gen, device=DEV).to(torch.float16)
        newv = torch.randn((w.L, w.B, w.Hkv, 128), generator=gen, device=DEV).to(torch.float16)
        Kt[:, :, :, step] = newk
        Vt[:, :, :, step] = newv
        tl.fill_(step + 1)
        outs = {}
        for layer in range(w.L):
            q = torch.from_numpy(synth.query(w, layer, step)).to(DEV)
            o = run.attention(layer, q, Kt[layer], Vt[layer], cap, tl)
            if step in (0, w.decode_steps - 1):
                outs[layer] = (q, o)
        if step in (0, w.decode_steps - 1):
            for layer, b in sample:
                q, o = outs[layer]
                ref = P.oracle_attention(run, layer, b, q[b].cpu().numpy(),
                                         Kt[layer, b, :, :step + 1].cpu().numpy(),
                                         Vt[layer, b, :, :step + 1].cpu().numpy())
                P.assert_out_close(o[b].cpu().numpy(), ref, f"c3 step {step} layer {layer} seq {b}")
            print(f"[step] decode step {step} ok on {len(sample)} (layer, sequence) pairs", flush=True)


@pytest.mark.parametrize("w", synth.serving_sweep(), ids=lambda w: w.name)
def test_serving_sweep_full_size(w):
    """batch 64 x 25088 tokens + 256-token fp16 tail, n_a in {8,16,32} x p in {0, 5 %, 20 %}."""
    print(f"[case] {w.name} full", flush=True)
    K, V = synth.device_kv(w, DEV)
    scores = synth.saliency(w) if w.n_salient else None
    run = P.GpuRun(w, DEV, K=K, V=V,
                   saliency=None if scores is None else torch.from_numpy(scores).to(DEV))
    # 8 heads: the first and last sequence, and others with the KV head moving
    heads = [0, 1 * w.Hkv + 1, 9 * w.Hkv + 2, 22 * w.Hkv + 3, 37 * w.Hkv, 50 * w.Hkv + 1,
             (w.B - 1) * w.Hkv + 2, w.n_heads - 1]
    _check_heads(run, K, V, heads, scores)
    print(f"[step] codec ok on {len(heads)} heads", flush=True)
    del K, V
    q = synth.query(w, 0)
    gen = torch.Generator(device=DEV); gen.manual_seed(5)
    Kt = torch.randn((w.B, w.Hkv, w.T_tail, 128), generator=gen, device=DEV).to(torch.float16)
    Vt = torch.randn((w.B, w.Hkv, w.T_tail, 128), generator=gen, device=DEV).to(torch.float16)
    tl_np = np.full(w.B, w.T_tail, dtype=np.int32); tl_np[1] = 100
    out = run.attention(0, torch.from_numpy(q).to(DEV), Kt, Vt, w.T_tail,
                        torch.from_numpy(tl_np).to(DEV)).cpu().numpy()
    seqs = (0, 1, 7, 18, 29, 41, 52, w.B - 1)              # sequence 1 has the short tail
    worst = 0.0
    for b in seqs:
        ref = P.oracle_attention(run, 0, b, q[b], Kt[b, :, :tl_np[b]].cpu().numpy(),
                                 Vt[b, :, :tl_np[b]].cpu().numpy())
        worst = max(worst, P.assert_out_close(out[b], ref, f"{w.name} seq {b}"))
    print(f"[step] attention ok on {len(seqs)} sequences, max err {worst:.2e}", flush=True)
