"""Seeded synthetic KV-cache inputs shaped like LLaVA-OV-7B / Qwen2.5-VL-7B.

This module only draws random inputs; it holds none of the codec's or the
attention's arithmetic, and it is the one module that both the CPU oracle's
tests and the GPU path's tests use.

The paper's workloads (activations of the two models on six video
benchmarks, Sec. 4.1) need trained weights and datasets; these tensors stand
in for them.  Shapes follow the models (28 layers, 4 KV heads, 28 query
heads, head_dim 128, 196 tokens per frame); value structure follows what the
paper describes for such caches: a few key channels with much larger
magnitude (Sec. 1, Sec. 3.1, Fig. kvcache-vis) and channel-dependent offsets.

Every tensor is generated one (layer, sequence, KV head) slab at a time from
its own counter-based stream, so any single head can be regenerated without
the rest.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

D = 128
G = 32
TOK_PER_FRAME = 196
BASE_SEED = 20250316

# tensor ids (part of the seed)
T_K, T_V, T_Q, T_SAL, T_TAIL, T_OUTL, T_HID, T_STEP = 0, 1, 2, 3, 4, 5, 6, 10


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration."""
    name: str
    cfg_id: int          # enters the seed
    L: int               # layers
    B: int               # sequences
    Hkv: int
    Hq: int
    frames: int
    T_tail: int          # fp16 residual tokens present at the first decode step
    n_anom: int          # 2-bit key channels per head
    n_salient: int       # protected value tokens per sequence
    dist: str            # "toy" | "model"
    decode_steps: int = 1

    @property
    def T(self) -> int:
        return self.frames * TOK_PER_FRAME

    @property
    def n_heads(self) -> int:
        return self.L * self.B * self.Hkv


def _w(name, cid, L, B, Hkv, Hq, frames, T_tail, n_a, p_num, p_den, dist, steps=1):
    T = frames * TOK_PER_FRAME
    return Workload(name, cid, L, B, Hkv, Hq, frames, T_tail, n_a,
                    (T * p_num) // p_den, dist, steps)


WORKLOADS = {
    # toy single head, 8 frames, 8 planted outlier channels, 10 % protected tokens
    "c1_toy": _w("c1_toy", 1, 1, 1, 1, 1, 8, 32, 64, 1, 10, "toy"),
    "c1_toy_na8": _w("c1_toy_na8", 1, 1, 1, 1, 1, 8, 32, 8, 1, 10, "toy"),
    # one LLaVA-OV-7B-shaped layer, 32 frames, K-1.5 / V-1.58
    "c2_layer": _w("c2_layer", 2, 1, 1, 4, 28, 32, 0, 64, 0, 1, "model"),
    # full 28-layer stack, batch 8, 64 frames, 16 decode steps
    "c3_stack": _w("c3_stack", 3, 28, 8, 4, 28, 64, 0, 64, 0, 1, "model", 16),
    # long video, one layer, 1000 frames, 1/8 anomalous channels, 5 % protected
    "c4_long": _w("c4_long", 4, 1, 1, 4, 28, 1000, 0, 16, 1, 20, "model"),
    # batched serving, batch 64, 128 frames, 256-token text tail (centre of the sweep)
    "c5_serving": _w("c5_serving", 5, 1, 64, 4, 28, 128, 256, 16, 1, 20, "model"),
}


def serving_sweep() -> list[Workload]:
    """The 3 x 3 grid of the serving configuration."""
    base = WORKLOADS["c5_serving"]
    out = []
    for n_a in (8, 16, 32):
        for num, den in ((0, 1), (1, 20), (1, 5)):
            out.append(replace(base, name=f"c5_na{n_a}_p{num}of{den}", n_anom=n_a,
                               n_salient=(base.T * num) // den))
    return out


def reduced(w: Workload, frames: int, L: int | None = None, B: int | None = None) -> Workload:
    """Same recipe at a smaller token / layer / batch count (for CPU-sized parity cases)."""
    T = frames * TOK_PER_FRAME
    n_s = (w.n_salient * T) // w.T
    return replace(w, name=f"{w.name}_f{frames}", frames=frames, n_salient=n_s,
                   L=w.L if L is None else L, B=w.B if B is None else B)


def _rng(w: Workload, tensor: int, *extra: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(
        key=np.random.SeedSequence([BASE_SEED, w.cfg_id, tensor, *extra]).generate_state(2, np.uint64)))


def _to_f16(x: np.ndarray) -> np.ndarray:
    return np.clip(x, -60000.0, 60000.0).astype(np.float16)


def outlier_channels(w: Workload, hd: int) -> np.ndarray:
    """Indices of the planted large-magnitude key channels of head hd."""
    r = _rng(w, T_OUTL, hd if w.dist == "model" else 0)
    n = 8 if w.dist == "toy" else 6        # toy: 8 of 128; model: round(0.05 * 128)
    return np.sort(r.choice(D, size=n, replace=False))


def _slab(w: Workload, tensor: int, hd: int, rows: int, key_outliers: bool) -> np.ndarray:
    r = _rng(w, tensor, hd)
    x = r.standard_normal((rows, D), dtype=np.float32)
    if w.dist == "toy":
        if key_outliers:
            x[:, outlier_channels(w, hd)] *= 15.0
    else:
        mu = _rng(w, tensor, hd, 7).standard_normal(D, dtype=np.float32) * 0.5
        x += mu
        if key_outliers:
            ch = outlier_channels(w, hd)
            x[:, ch] += (10.0 * r.standard_t(2, size=(rows, len(ch)))).astype(np.float32)
    return _to_f16(x)


def key_head(w: Workload, hd: int) -> np.ndarray:
    """K of head hd = (l*B + b)*Hkv + h : [T, 128] fp16."""
    return _slab(w, T_K, hd, w.T, True)


def value_head(w: Workload, hd: int) -> np.ndarray:
    return _slab(w, T_V, hd, w.T, False)


def tail_heads(w: Workload, l: int, b: int, rows: int | None = None):
    """fp16 residual K, V of (layer l, sequence b): two [Hkv, rows, 128] arrays."""
    rows = w.T_tail if rows is None else rows
    ks, vs = [], []
    for h in range(w.Hkv):
        hd = (l * w.B + b) * w.Hkv + h
        ks.append(_slab(w, T_TAIL, 2 * hd, rows, True))
        vs.append(_slab(w, T_TAIL, 2 * hd + 1, rows, False))
    return np.stack(ks), np.stack(vs)


def step_token(w: Workload, l: int, b: int, step: int):
    """The K, V row appended at decode step `step`: two [Hkv, 128] arrays."""
    ks, vs = [], []
    for h in range(w.Hkv):
        hd = (l * w.B + b) * w.Hkv + h
        ks.append(_slab(w, T_STEP + step, 2 * hd, 1, True)[0])
        vs.append(_slab(w, T_STEP + step, 2 * hd + 1, 1, False)[0])
    return np.stack(ks), np.stack(vs)


def query(w: Workload, l: int, step: int = 0) -> np.ndarray:
    """q of layer l at a decode step: [B, Hq, 128] fp16 ~ N(0, 1)."""
    r = _rng(w, T_Q, l, step)
    return _to_f16(r.standard_normal((w.B, w.Hq, D), dtype=np.float32))


def saliency(w: Workload) -> np.ndarray:
    """Cross-modal saliency scores per visual token: [B, T] float32 ~ U(0, 1)."""
    r = _rng(w, T_SAL)
    return r.random((w.B, w.T), dtype=np.float32)


HIDDEN_DIM = 3584        # hidden size of the 7B models the paper runs
N_TEXT = 32              # text-query tokens of a prompt


def hidden_states(w: Workload, b: int, rows: int | None = None, d: int = HIDDEN_DIM,
                  n_text: int = N_TEXT):
    """Hidden states of sequence b for the saliency scores: visual [rows, d] and
    text [n_text, d] fp16 ~ N(0, 1), the text rows sharing a common direction with
    a fifth of the visual rows so that the scores are not pure noise."""
    rows = w.T if rows is None else rows
    r = _rng(w, T_HID, b)
    Xt = r.standard_normal((n_text, d), dtype=np.float32)
    topic = r.standard_normal(d, dtype=np.float32)
    Xt += 0.5 * topic
    Xv = r.standard_normal((rows, d), dtype=np.float32)
    hit = r.random(rows) < 0.2
    Xv[hit] += 0.3 * topic
    return _to_f16(Xv), _to_f16(Xt)


def keys(w: Workload) -> np.ndarray:
    """Whole K tensor [L, B, Hkv, T, 128] fp16 (use key_head for big workloads)."""
    out = np.empty((w.n_heads, w.T, D), dtype=np.float16)
    for hd in range(w.n_heads):
        out[hd] = key_head(w, hd)
    return out.reshape(w.L, w.B, w.Hkv, w.T, D)


def values(w: Workload) -> np.ndarray:
    out = np.empty((w.n_heads, w.T, D), dtype=np.float16)
    for hd in range(w.n_heads):
        out[hd] = value_head(w, hd)
    return out.reshape(w.L, w.B, w.Hkv, w.T, D)


# ---------------------------------------------------------------------------
# On-device generation for the full-size workloads (GB-sized tensors): same
# recipe, drawn with torch's device generator so that it takes milliseconds.
# A head that the oracle should check is simply copied back to the host.
# ---------------------------------------------------------------------------
def device_kv(w: Workload, device: str = "cuda:0"):
    """K, V of a whole workload as [L, B, Hkv, T, 128] fp16 device tensors."""
    import torch
    out = []
    for tensor, is_key in ((T_K, True), (T_V, False)):
        g = torch.Generator(device=device)
        g.manual_seed(BASE_SEED + 1000 * w.cfg_id + tensor)
        x = torch.empty((w.n_heads, w.T, D), dtype=torch.float16, device=device)
        per = max(1, (1 << 27) // max(w.T * D, 1))           # heads per 128M-element chunk
        for h0 in range(0, w.n_heads, per):
            h1 = min(w.n_heads, h0 + per)
            y = torch.randn((h1 - h0, w.T, D), generator=g, device=device)
            if w.dist == "toy":
                if is_key:
                    for hd in range(h0, h1):
                        y[hd - h0][:, torch.from_numpy(outlier_channels(w, hd)).to(device)] *= 15.0
            else:
                y += 0.5 * torch.randn((h1 - h0, 1, D), generator=g, device=device)
                if is_key:
                    for hd in range(h0, h1):
                        ch = torch.from_numpy(outlier_channels(w, hd)).to(device)
                        z = torch.randn((w.T, len(ch)), generator=g, device=device)
                        e = -torch.log(torch.rand((w.T, len(ch)), generator=g, device=device)
                                       .clamp_min(1e-30))     # chi^2_2 / 2
                        y[hd - h0][:, ch] += 10.0 * z / torch.sqrt(e)     # Student-t, 2 dof
            x[h0:h1] = y.clamp_(-60000.0, 60000.0).to(torch.float16)
            del y
        out.append(x.view(w.L, w.B, w.Hkv, w.T, D))
    return out[0], out[1]
