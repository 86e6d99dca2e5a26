"""The decode path under HIP graph capture: the library allocates nothing, never synchronizes
and launches only on the caller's stream, so a whole multi-layer decode step can be captured once
and replayed.  Every replay (with new queries and residual tokens written into the same buffers
between replays) must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

import parity as P
from paper_2503_16257_amd import binding as vk
from paper_2503_16257_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_decode_step_of_all_layers_captured_and_replayed():
    w = synth.reduced(synth.WORKLOADS["c3_stack"], 8, L=4, B=2)
    print("[case] graph-decode", flush=True)
    run = P.GpuRun(w, DEV)
    cap = 16
    q = torch.zeros((w.L, w.B, w.Hq, 128), dtype=torch.float16, device=DEV)
    Kt = torch.zeros((w.L, w.B, w.Hkv, cap, 128), dtype=torch.float16, device=DEV)
    Vt = torch.zeros_like(Kt)
    tl = torch.zeros((w.B,), dtype=torch.int32, device=DEV)
    out = torch.zeros((w.L, w.B, w.Hq, 128), dtype=torch.float16, device=DEV)
    ws = [vk.alloc_bytes(vk.workspace_bytes(run.p, 2), DEV) for _ in range(w.L)]

    def step():
        for l in range(w.L):
            vk.decode_attention(run.p, l, q[l], run.pk, run.pv, out[l], ws[l], K_tail=Kt[l],
                                V_tail=Vt[l], tail_capacity=cap, tail_len=tl)

    def set_inputs(s):
        for l in range(w.L):
            q[l].copy_(torch.from_numpy(synth.query(w, l, step=s)))
            for b in range(w.B):
                k, v = synth.step_token(w, l, b, s)
                Kt[l, b, :, s].copy_(torch.from_numpy(k))
                Vt[l, b, :, s].copy_(torch.from_numpy(v))
        tl.fill_(s + 1)

    set_inputs(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                              # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for s in range(4):
        set_inputs(s)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.fill_(float("nan"))
        step()                                              # eager, same inputs
        torch.cuda.synchronize()
        assert torch.equal(got, out), f"replay {s} differs from the eager run"
        assert torch.isfinite(got.float()).all()
    # and the last replay against the oracle, one sampled (layer, sequence)
    l, b = 2, 1
    ref = P.oracle_attention(run, l, b, q[l, b].cpu().numpy(), Kt[l, b, :, :4].cpu().numpy(),
                             Vt[l, b, :, :4].cpu().numpy())
    P.assert_out_close(got[l, b].cpu().numpy(), ref, "graph replay")


def test_large_residual_block_forked_inside_the_capture():
    """A batch whose residual block is large enough to be forked onto the caller's side
    stream: the fork and join are captured with the rest and every replay equals the eager run."""
    w = synth.reduced(synth.WORKLOADS["c5_serving"], 8, B=32)
    print("[case] graph-decode forked residual block", flush=True)
    run = P.GpuRun(w, DEV)
    cap = 256
    g0 = torch.Generator(device=DEV)
    g0.manual_seed(77)
    q = torch.randn((w.B, w.Hq, 128), generator=g0, device=DEV, dtype=torch.float16)
    Kt = torch.randn((w.B, w.Hkv, cap, 128), generator=g0, device=DEV, dtype=torch.float16)
    Vt = torch.randn((w.B, w.Hkv, cap, 128), generator=g0, device=DEV, dtype=torch.float16)
    tl = torch.full((w.B,), 200, dtype=torch.int32, device=DEV)
    out = torch.zeros((w.B, w.Hq, 128), dtype=torch.float16, device=DEV)
    ws = vk.alloc_bytes(vk.workspace_bytes(run.p, 2), DEV)

    def step():
        vk.decode_attention(run.p, 0, q, run.pk, run.pv, out, ws, K_tail=Kt, V_tail=Vt,
                            tail_capacity=cap, tail_len=tl, side=P.side_stream(DEV))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                              # warm-up, outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for s in range(4):
        q.copy_(torch.randn(q.shape, generator=g0, device=DEV, dtype=torch.float16))
        tl.fill_(256 - 37 * s)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.fill_(float("nan"))
        step()
        torch.cuda.synchronize()
        assert torch.equal(got, out), f"replay {s} differs from the eager run"
        assert torch.isfinite(got.float()).all()
    b = 17
    n = int(tl[b])
    ref = P.oracle_attention(run, 0, b, q[b].cpu().numpy(), Kt[b, :, :n].cpu().numpy(),
                             Vt[b, :, :n].cpu().numpy())
    P.assert_out_close(got[b].cpu().numpy(), ref, "graph replay, forked residual block")


def test_quantizer_with_its_side_stream_captured_and_replayed():
    """vidkv_quantize_kv forks the protected-token selection onto the caller's side stream;
    captured, every replay must write the same bytes as the eager call."""
    w = synth.reduced(synth.WORKLOADS["c4_long"], 176)       # 35 MB of keys: large enough to fork
    print("[case] graph-quantize", flush=True)
    run = P.GpuRun(w, DEV)                                   # eager reference buffers run.pk, run.pv
    sal = torch.from_numpy(synth.saliency(w)).to(DEV)
    pk = vk.alloc_bytes(vk.packed_keys_bytes(run.p), DEV)
    pv = vk.alloc_bytes(vk.packed_values_bytes(run.p), DEV)
    ws = vk.alloc_bytes(vk.workspace_bytes(run.p, 3), DEV)
    pk0, pv0 = torch.zeros_like(pk), torch.zeros_like(pv)

    def step(dk, dv):
        vk.quantize_kv(run.p, run.K, run.V, dk, dv, ws, saliency=sal, side=P.side_stream(DEV))

    pk0.zero_(); pv0.zero_()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(pk0, pv0)                                      # eager
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(pk, pv)
    for s in range(3):
        pk.zero_(); pv.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(pk, pk0) and torch.equal(pv, pv0), f"replay {s} differs from the eager call"
