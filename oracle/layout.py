"""Independent numpy reader / writer of the packed VidKV cache format.

TEST INFRASTRUCTURE: lets the oracle encode its own logical codes into bytes
and decode buffers produced by the GPU library.  Written from the format
description only; shares no code with the HIP kernels.

The cache record of Alg. 1 ({Q(K_q), Q(V_q)} plus metadata) is stored as two
flat byte buffers.  Notation: L layers, B sequences, H KV heads, D = 128,
G = 32, T quantized tokens (multiple of 32), n_a anomalous channels
(multiple of 8), n_n = D - n_a, n_s protected tokens per sequence.  A "head"
is one (l, b, h), numbered hd = (l*B + b)*H + h.  All multi-byte fields are
little-endian; every section starts on a 256-byte boundary.

Key buffer
  section PERM   : uint8 [LBH][128]: anomalous channels ascending, then normal
                   channels ascending.  "anomalous j" / "normal i" below index
                   into these two lists.
  section REC    : [LBH][T/32] records of 12*n_a + 8*n_n bytes:
      +0          codes2 : uint8 [32 tokens][n_a/4]; byte (t, q) holds the
                           2-bit codes of anomalous channels 4q..4q+3 at token
                           t, channel 4q+j in bits 2j, 2j+1.
      +8*n_a      s      : fp16 [n_a]   (Eq. 4 scale)
      +10*n_a     z      : fp16 [n_a]   (Eq. 4 zero point)
      +12*n_a     signs  : uint16 [n_n/8 blocks][16]; word (blk, k), bit e
                           (e < 8)  = sign bit of Re X[k]       of normal
                                      channel 8*blk + e,
                           bit 8+e  = sign bit of Im X[k] for k >= 1, of
                                      Re X[16] for k = 0.
                           A sign bit is 1 when the coefficient is >= 0.
      +12*n_a+4*n_n  scales : fp16 [n_n/8 blocks][2][8]: s_re then s_im of the
                           block's 8 channels.
Value buffer
  section REC    : [LBH][T/32] records of 1280 bytes:
      +0          trits  : uint32 [4 kb][16 r][4 mp]; word (kb, r, mp) holds 8
                           token slots of the two channels c = 16*m + r,
                           m = 2*mp + mh (mh = 0, 1).  Slot j = 0..7 is token
                           4*kb + j (j < 4) or 16 + 4*kb + (j-4) (j >= 4) of the
                           group.  The 2-bit field of (mh, j) starts at bit
                           8*mh + 16*(j & 1) + 2*(j >> 1): that bit = code != 0,
                           the next = code < 0.
      +1024       s      : fp16 [16 r][8 m]: Eq. 6 mean |V| of channel 16*m + r
  section IDX    : int32  [B][n_s]   protected token indices, ascending
  section MASK   : uint32 [B][T/32]  bit (t % 32) of word t/32 = token t protected
  section RANK   : uint32 [B][T/32]  number of protected tokens before group g
  section ROWS   : fp16   [L][B][H][n_s][128]  the protected rows verbatim; or, with 2-bit
                   protected rows, [L][B][H][ceil(n_s/32)] records of 1536 bytes:
                   uint8 [32 rows][32]  codes, channel 4 j + r of a row in bits 2r, 2r+1 of byte j
                   fp16  [128] s, fp16 [128] z   (Eq. 4 per channel over the record's rows)
  (IDX..ROWS are absent when n_s = 0.)
"""
from __future__ import annotations

import numpy as np

G = 32
D = 128
VREC = 1280
PREC = 1536


def _align(x: int, a: int = 256) -> int:
    return (x + a - 1) // a * a


def key_record_bytes(n_a: int) -> int:
    return 12 * n_a + 8 * (D - n_a)


def key_sections(L: int, B: int, H: int, T: int, n_a: int) -> dict:
    nh = L * B * H
    off_rec = _align(nh * D)
    total = off_rec + nh * (T // G) * key_record_bytes(n_a)
    return {"perm": 0, "rec": off_rec, "total": _align(total)}


def value_sections(L: int, B: int, H: int, T: int, n_s: int, sal_bits: int = 16) -> dict:
    nh = L * B * H
    ng = T // G
    off = _align(nh * ng * VREC)
    sec = {"rec": 0}
    if n_s > 0:
        sec["idx"] = off
        off = _align(off + 4 * B * n_s)
        sec["mask"] = off
        off = _align(off + 4 * B * ng)
        sec["rank"] = off
        off = _align(off + 4 * B * ng)
        sec["rows"] = off
        rows = nh * ((n_s + G - 1) // G) * PREC if sal_bits == 2 else 2 * nh * n_s * D
        off = _align(off + rows)
    sec["total"] = off
    return sec


# ------------------------------------------------------------------ keys ---
def pack_key_head(rec: dict, n_a: int) -> tuple[np.ndarray, np.ndarray]:
    """Logical record of one head -> (perm bytes [128], record bytes [T/32, recsize])."""
    n_n = D - n_a
    ng = rec["n_bits"].shape[0] if n_n else rec["a_codes"].shape[0]
    out = np.zeros((ng, key_record_bytes(n_a)), dtype=np.uint8)
    if n_a:
        codes = rec["a_codes"]                                   # [g, n_a, 32]
        by = np.zeros((ng, G, n_a // 4), dtype=np.uint8)
        for j in range(4):
            by |= (codes[:, j::4, :].transpose(0, 2, 1) << (2 * j)).astype(np.uint8)
        out[:, 0:8 * n_a] = by.reshape(ng, -1)
        out[:, 8 * n_a:10 * n_a] = rec["a_s16"].astype("<f2").view(np.uint8).reshape(ng, -1)
        out[:, 10 * n_a:12 * n_a] = rec["a_z16"].astype("<f2").view(np.uint8).reshape(ng, -1)
    if n_n:
        bits = rec["n_bits"].astype(np.uint16)                   # [g, n_n, 32 slots]
        nb = n_n // 8
        words = np.zeros((ng, nb, 16), dtype=np.uint16)
        for e in range(8):
            ch = bits[:, e::8, :]                                # [g, nb, 32]
            words |= ch[:, :, 0:16] << e                         # Re k = 0..15
            hi = np.concatenate([ch[:, :, 16:17], ch[:, :, 17:32]], axis=2)   # Nyquist, Im 1..15
            words |= hi << (8 + e)
        o = 12 * n_a
        out[:, o:o + 4 * n_n] = words.astype("<u2").view(np.uint8).reshape(ng, -1)
        meta = np.stack([rec["n_sre16"].reshape(ng, nb, 8),
                         rec["n_sim16"].reshape(ng, nb, 8)], axis=2)           # [g, nb, 2, 8]
        o += 4 * n_n
        out[:, o:o + 4 * n_n] = meta.astype("<f2").view(np.uint8).reshape(ng, -1)
    return rec["perm"].astype(np.uint8), out


def unpack_key_head(perm: np.ndarray, recs: np.ndarray, n_a: int) -> dict:
    """Inverse of pack_key_head: bytes -> logical record of one head."""
    n_n = D - n_a
    ng = recs.shape[0]
    perm = perm.astype(np.int64)
    r = {"perm": perm.astype(np.uint8), "anom": perm[:n_a], "norm": perm[n_a:]}
    by = recs[:, 0:8 * n_a].reshape(ng, G, n_a // 4) if n_a else np.zeros((ng, G, 0), np.uint8)
    codes = np.zeros((ng, n_a, G), dtype=np.uint8)
    for j in range(4):
        codes[:, j::4, :] = ((by >> (2 * j)) & 3).transpose(0, 2, 1)
    r["a_codes"] = codes
    r["a_s16"] = np.ascontiguousarray(recs[:, 8 * n_a:10 * n_a]).view("<f2").reshape(ng, n_a)
    r["a_z16"] = np.ascontiguousarray(recs[:, 10 * n_a:12 * n_a]).view("<f2").reshape(ng, n_a)
    nb = n_n // 8
    o = 12 * n_a
    words = np.ascontiguousarray(recs[:, o:o + 4 * n_n]).view("<u2").reshape(ng, nb, 16)
    bits = np.zeros((ng, n_n, 32), dtype=np.uint8)
    for e in range(8):
        lo = ((words >> e) & 1).astype(np.uint8)                 # [g, nb, 16]
        hi = ((words >> (8 + e)) & 1).astype(np.uint8)
        bits[:, e::8, 0:16] = lo
        bits[:, e::8, 16] = hi[:, :, 0]
        bits[:, e::8, 17:32] = hi[:, :, 1:16]
    r["n_bits"] = bits
    o += 4 * n_n
    meta = np.ascontiguousarray(recs[:, o:o + 4 * n_n]).view("<f2").reshape(ng, nb, 2, 8)
    r["n_sre16"] = meta[:, :, 0, :].reshape(ng, n_n)
    r["n_sim16"] = meta[:, :, 1, :].reshape(ng, n_n)
    return r


def key_head_views(buf: np.ndarray, L: int, B: int, H: int, T: int, n_a: int, hd: int):
    """Slice (perm, records) of head number hd out of a whole key buffer (uint8)."""
    sec = key_sections(L, B, H, T, n_a)
    rb = key_record_bytes(n_a)
    ng = T // G
    perm = buf[sec["perm"] + hd * D: sec["perm"] + (hd + 1) * D]
    recs = buf[sec["rec"] + hd * ng * rb: sec["rec"] + (hd + 1) * ng * rb].reshape(ng, rb)
    return perm, recs


# ---------------------------------------------------------------- values ---
def _trit_position(t: int) -> tuple[int, int]:
    """Token-in-group t -> (kb, slot j) of the trit word that holds it."""
    kb = (t % 16) // 4
    j = (t % 4) + (4 if t >= 16 else 0)
    return kb, j


def _trit_bit(m: int, j: int) -> int:
    """First bit of the 2-bit field of (tile m, slot j) inside its 32-bit word."""
    return 8 * (m & 1) + 16 * (j & 1) + 2 * (j >> 1)


def pack_value_head(codes: np.ndarray, s16: np.ndarray) -> np.ndarray:
    """codes [g, 128, 32] in {-1,0,1}, s16 [g, 128] -> record bytes [g, 1280]."""
    ng = codes.shape[0]
    words = np.zeros((ng, 4, 16, 4), dtype=np.uint32)
    cm = codes.reshape(ng, 8, 16, G)                              # [g, m, r, t], c = 16 m + r
    for t in range(G):
        kb, j = _trit_position(t)
        for m in range(8):
            nz = (cm[:, m, :, t] != 0).astype(np.uint32)
            ng_ = (cm[:, m, :, t] < 0).astype(np.uint32)
            words[:, kb, :, m >> 1] |= (nz | (ng_ << 1)) << _trit_bit(m, j)
    out = np.zeros((ng, VREC), dtype=np.uint8)
    out[:, 0:1024] = words.astype("<u4").view(np.uint8).reshape(ng, -1)
    st = s16.reshape(ng, 8, 16).transpose(0, 2, 1)                # [g, r, m]
    out[:, 1024:1280] = np.ascontiguousarray(st).astype("<f2").view(np.uint8).reshape(ng, -1)
    return out


def unpack_value_head(recs: np.ndarray):
    """Record bytes [g, 1280] -> (codes [g, 128, 32] int8, s16 [g, 128])."""
    ng = recs.shape[0]
    words = np.ascontiguousarray(recs[:, 0:1024]).view("<u4").reshape(ng, 4, 16, 4)
    codes = np.zeros((ng, 8, 16, G), dtype=np.int8)
    for t in range(G):
        kb, j = _trit_position(t)
        for m in range(8):
            f = (words[:, kb, :, m >> 1] >> _trit_bit(m, j)) & 3  # [g, r]
            codes[:, m, :, t] = np.where(f & 1, np.where(f & 2, -1, 1), 0).astype(np.int8)
    st = np.ascontiguousarray(recs[:, 1024:1280]).view("<f2").reshape(ng, 16, 8)
    s16 = np.ascontiguousarray(st.transpose(0, 2, 1)).reshape(ng, D)
    return codes.reshape(ng, D, G), s16


def value_head_records(buf: np.ndarray, L: int, B: int, H: int, T: int, hd: int) -> np.ndarray:
    ng = T // G
    return buf[hd * ng * VREC:(hd + 1) * ng * VREC].reshape(ng, VREC)


def pack_salient(buf: np.ndarray, sec: dict, b: int, B: int, T: int, idx: np.ndarray):
    """Write IDX / MASK / RANK of sequence b into a whole value buffer."""
    n_s = len(idx)
    ng = T // G
    buf[sec["idx"] + 4 * b * n_s: sec["idx"] + 4 * (b + 1) * n_s] = \
        idx.astype("<i4").view(np.uint8)
    flag = np.zeros(T, dtype=np.uint32)
    flag[idx] = 1
    fl = flag.reshape(ng, G)
    mask = (fl << np.arange(G, dtype=np.uint32)).sum(axis=1).astype("<u4")
    cnt = fl.sum(axis=1)
    rank = (np.cumsum(cnt) - cnt).astype("<u4")
    buf[sec["mask"] + 4 * b * ng: sec["mask"] + 4 * (b + 1) * ng] = mask.view(np.uint8)
    buf[sec["rank"] + 4 * b * ng: sec["rank"] + 4 * (b + 1) * ng] = rank.view(np.uint8)


def unpack_salient(buf: np.ndarray, sec: dict, b: int, T: int, n_s: int):
    """-> (idx [n_s] int32, mask [T/32] uint32, rank [T/32] uint32) of sequence b."""
    ng = T // G
    idx = np.ascontiguousarray(buf[sec["idx"] + 4 * b * n_s: sec["idx"] + 4 * (b + 1) * n_s]).view("<i4")
    mask = np.ascontiguousarray(buf[sec["mask"] + 4 * b * ng: sec["mask"] + 4 * (b + 1) * ng]).view("<u4")
    rank = np.ascontiguousarray(buf[sec["rank"] + 4 * b * ng: sec["rank"] + 4 * (b + 1) * ng]).view("<u4")
    return idx, mask, rank


def salient_rows(buf: np.ndarray, sec: dict, hd: int, n_s: int) -> np.ndarray:
    o = sec["rows"] + 2 * hd * n_s * D
    return np.ascontiguousarray(buf[o:o + 2 * n_s * D]).view("<f2").reshape(n_s, D)


def pack_protected2(codes: np.ndarray, s16: np.ndarray, z16: np.ndarray) -> np.ndarray:
    """2-bit protected rows of one head -> uint8 [npg * 1536].  codes [n_s, D] in 0..3,
    s16 / z16 [npg, D] fp16."""
    n_s = codes.shape[0]
    npg = (n_s + G - 1) // G
    out = np.zeros((npg, PREC), dtype=np.uint8)
    full = np.zeros((npg * G, D), dtype=np.uint8)
    full[:n_s] = codes
    q = full.reshape(npg, G, D // 4, 4).astype(np.uint32)
    by = (q[..., 0] | (q[..., 1] << 2) | (q[..., 2] << 4) | (q[..., 3] << 6)).astype(np.uint8)
    out[:, :1024] = by.reshape(npg, 1024)
    out[:, 1024:1280] = np.ascontiguousarray(s16.astype("<f2")).view(np.uint8).reshape(npg, 256)
    out[:, 1280:1536] = np.ascontiguousarray(z16.astype("<f2")).view(np.uint8).reshape(npg, 256)
    return out.reshape(-1)


def unpack_protected2(buf: np.ndarray, n_s: int):
    """Inverse of pack_protected2 for one head's records -> (codes [n_s, D], s16, z16 [npg, D])."""
    npg = (n_s + G - 1) // G
    r = np.ascontiguousarray(buf[:npg * PREC]).reshape(npg, PREC)
    by = r[:, :1024].reshape(npg, G, D // 4)
    codes = np.stack([(by >> (2 * k)) & 3 for k in range(4)], axis=-1).reshape(npg * G, D)[:n_s]
    s16 = np.ascontiguousarray(r[:, 1024:1280]).view("<f2").reshape(npg, D)
    z16 = np.ascontiguousarray(r[:, 1280:1536]).view("<f2").reshape(npg, D)
    return codes.astype(np.uint8), s16, z16
