"""Plain float64 implementation of the VidKV codec and decode attention.

TEST INFRASTRUCTURE: a slow, obviously-correct statement of what the GPU path
must compute.  It shares no code, table or constant with the HIP kernels and
is never used by the product path.

Conventions
-----------
* Inputs are the exact fp16 values (numpy float16 arrays); all arithmetic is
  float64 unless a line says otherwise.
* One "head" is the [T, D] slab of one (layer, sequence, KV head).  T is the
  number of quantized tokens, a multiple of the group size G = 32
  (Sec. 4.1, implementation details); D = 128.
* Codes are decided against the unrounded statistics; only the *stored*
  scale / zero-point are rounded to fp16 (round-to-nearest-even), and
  dequantization uses the stored fp16 values.
* Every quantizer also returns a boolean `near` array marking the elements
  whose decision variable lies within 1e-6 (relative to its natural scale) of
  a decision threshold; parity tests exclude and count those.

Readings of the paper taken here (each is listed with its alternative in the
design notes of the repository):
  - the FFT runs along the token axis, one 32-point transform per channel and
    group (Sec. 3.2 (2) transforms each channel's sequence over time);
  - Eq. 5's code is the sign bit, bit = [coef >= 0], and dequantizes to the
    symmetric levels +-s (the formula as printed would give {0, 2});
  - the real and imaginary parts are quantized as separate real channels
    (Alg. 3 views the spectrum as [l, 2d] reals), each with its own scale
    Mean(|.|) over the full 32-bin spectrum; only the 17 + 15 independent
    reals of the Hermitian spectrum are coded, which is 1 bit per element;
  - ternary values dequantize to s * code with s = Mean(|V|) (Alg. 2 names no
    other scale);
  - protected tokens keep their positions: they are left out of the group
    mean, coded 0 and stored verbatim in fp16, or (stp_quant_rows) at 2 bits;
  - a full residual block is coded on its own with the prefill's channel
    split (quantize_keys_block); the non-FFT 1-bit code is Eq. 4 with n = 1;
    the saliency scores of Eq. 7 are summed over the text tokens.
Every function here is pinned by tests/test_oracle_pins.py; none is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

G = 32          # group size along tokens (Sec. 4.1)
# Exclusion bands around the decision thresholds.  An element closer to its threshold than
# the band is flagged `near`: a correct float32 evaluation of the same formula may decide it
# the other way, so a comparison against such an evaluation leaves it out (and counts it).
# Each width is the worst-case rounding error of ANY float32 evaluation order, u = 2^-24:
#   Eq. 4 codes : (x - z) * (levels / (max - z)) is four rounded operations on a number of at
#                 most `levels` = 3 steps: 3 * 4u = 7.2e-7 steps.
#   Eq. 5 signs : a 32-term sum whose every term may be split in up to three exact partial
#                 products, i.e. at most 95 rounded additions of terms bounded by |x_t|:
#                 95u * sum|x| = 5.7e-6 * sum|x|.
#   Eq. 6 trits : mean |V| is a sum of at most 32 non-negative terms (31 additions), a
#                 division by the count and a product with gamma: 33u = 2.0e-6, relative.
BAND = 1e-6          # Eq. 4, in quantization steps
BAND_SIGN = 6e-6     # Eq. 5, times the group's sum |x|
BAND_TRIT = 2.5e-6   # Eq. 6, times the threshold alpha


# --------------------------------------------------------------------------
# Keys: channel selection (Sec. 3.2 (1); Alg. 3, MixQuant)
# --------------------------------------------------------------------------
def key_channel_range(K16: np.ndarray) -> np.ndarray:
    """Range metric R_c = max_t K[t,c] - min_t K[t,c] over all T tokens.

    Sec. 3.2 (1) ("Range R = max(K) - min(K)") and Alg. 3 (range <- Max - Min).
    max and min of fp16 values are exact; the difference is taken as ONE
    float32 subtraction because this number decides an integer (the channel
    set) and the GPU takes the same decision in float32.
    """
    assert K16.dtype == np.float16 and K16.ndim == 2
    mx = K16.max(axis=0).astype(np.float32)
    mn = K16.min(axis=0).astype(np.float32)
    return (mx - mn).astype(np.float32)


def key_channel_variance(K16: np.ndarray) -> np.ndarray:
    """Sec. 3.2 (1), Variance: sigma^2 = mean(x^2) - mean(x)^2 per channel over all tokens
    (population variance), float64.  K16 [T, D] fp16 -> [D]."""
    x = K16.astype(np.float64)
    return (x * x).mean(axis=0) - x.mean(axis=0) ** 2


def key_channel_outliers(K16: np.ndarray, M: float = 3.0) -> np.ndarray:
    """Sec. 3.2 (1), Outliers: N = sum_i 1(K_i > M * mean K) per channel with M = 3; the
    printed formula has no absolute values, which for signed, near-zero-mean channels would
    count half of all tokens - here |K_i| > M * mean|K|.  K16 [T, D] fp16 -> [D] float64."""
    a = np.abs(K16.astype(np.float64))
    return (a > M * a.mean(axis=0)).sum(axis=0).astype(np.float64)


def select_anomalous_channels(R: np.ndarray, n_a: int):
    """Top-n_a channels by range -> 2-bit ("D-mask"), the rest -> 1-bit ("N-mask").

    Alg. 3: D-mask <- TopK(range, k), N-mask <- ~D-mask.  Ties are broken
    towards the lower channel index.  Returns (anom, norm, perm): sorted
    channel indices of both sets and perm = concat(anom, norm).
    """
    D = R.shape[0]
    order = sorted(range(D), key=lambda c: (-float(R[c]), c))
    anom = np.array(sorted(order[:n_a]), dtype=np.int64)
    norm = np.array(sorted(order[n_a:]), dtype=np.int64)
    perm = np.concatenate([anom, norm]).astype(np.uint8)
    return anom, norm, perm


# --------------------------------------------------------------------------
# Keys: n-bit uniform group quantizer (Eq. 4), used with n = 2
# --------------------------------------------------------------------------
def gquant(x16: np.ndarray, bits: int = 2):
    """Eq. 4 per channel over groups of G tokens.

    x16: [T, C] fp16.  Returns dict with
      codes [T//G, C, G] uint8 in [0, 2^bits-1], s16, z16 [T//G, C] fp16,
      near [T//G, C, G] bool.
    z = min, s = (max - min) / (2^n - 1), code = clamp(round((x - z)/s), 0, 2^n-1)
    with round-half-to-even; a constant group (s = 0) codes 0 everywhere.
    """
    T, C = x16.shape
    assert T % G == 0
    x = x16.astype(np.float64).reshape(T // G, G, C).transpose(0, 2, 1)   # [g, c, t]
    levels = (1 << bits) - 1
    z = x.min(axis=2)
    s = (x.max(axis=2) - z) / levels
    safe = np.where(s > 0, s, 1.0)
    u = (x - z[..., None]) / safe[..., None]
    codes = np.clip(np.rint(u), 0, levels)
    near = np.abs(u - (np.floor(u) + 0.5)) < BAND
    flat = (s == 0)
    codes[flat] = 0
    near[flat] = False
    return {
        "codes": codes.astype(np.uint8),
        "s16": s.astype(np.float16),
        "z16": z.astype(np.float16),
        "near": near,
    }


def gdequant(codes: np.ndarray, s16: np.ndarray, z16: np.ndarray) -> np.ndarray:
    """Eq. 4, right half: X' = Q * s + z with the stored fp16 s, z.  -> [T, C] float64."""
    x = codes.astype(np.float64) * s16.astype(np.float64)[..., None] \
        + z16.astype(np.float64)[..., None]                       # [g, c, t]
    g, c, t = x.shape
    return x.transpose(0, 2, 1).reshape(g * t, c)


# --------------------------------------------------------------------------
# Keys: FFT-based 1-bit quantizer (Eq. 5; Alg. 3, 1BitQuant)
# --------------------------------------------------------------------------
def _dft_matrix() -> np.ndarray:
    """F[k, t] = exp(-2 pi i k t / 32): the direct (unnormalised) forward DFT."""
    k = np.arange(G).reshape(G, 1)
    t = np.arange(G).reshape(1, G)
    return np.exp(-2j * np.pi * ((k * t) % G) / G)


def fft1bit_quant(x16: np.ndarray):
    """Eq. 5 on the real view of the spectrum, per channel and group.

    x16: [T, C] fp16.  For every (group, channel): X = DFT_32(x) by direct
    summation.  32 sign bits are kept, in slot order
        slot k      (k = 0..16) : [Re X[k] >= 0]
        slot 16 + k (k = 1..15) : [Im X[k] >= 0]
    and two scales, the means of |Re X| and |Im X| over all 32 bins
    (s_fft = Mean(|FFT(X)|), taken per real-view channel as in Alg. 3).
    Returns bits [g, C, 32] uint8, sre16/sim16 [g, C] fp16, near [g, C, 32].
    """
    T, C = x16.shape
    assert T % G == 0
    x = x16.astype(np.float64).reshape(T // G, G, C)               # [g, t, c]
    F = _dft_matrix()
    X = np.einsum("kt,gtc->gck", F, x)                             # [g, c, k]
    re, im = X.real, X.imag
    coef = np.concatenate([re[..., 0:17], im[..., 1:16]], axis=2)  # 17 + 15 slots
    bits = (coef >= 0).astype(np.uint8)
    s_re = np.abs(re).mean(axis=2)
    s_im = np.abs(im).mean(axis=2)
    l1 = np.abs(x).sum(axis=1)                                     # [g, c]
    near = np.abs(coef) < BAND_SIGN * l1[..., None]
    return {
        "bits": bits,
        "sre16": s_re.astype(np.float16),
        "sim16": s_im.astype(np.float16),
        "near": near,
        "coef": coef,
    }


def fft1bit_spectrum(bits: np.ndarray, sre16: np.ndarray, sim16: np.ndarray) -> np.ndarray:
    """Dequantized full spectrum Xhat[g, c, 32] (complex) from bits and stored scales.

    Levels are +-s (Eq. 5 with z_fft = 0, read symmetrically); bins 0 and 16
    are real; bins 17..31 follow from Hermitian symmetry of a real signal.
    """
    sre = sre16.astype(np.float64)[..., None]
    sim = sim16.astype(np.float64)[..., None]
    sign = 2.0 * bits.astype(np.float64) - 1.0
    g, c, _ = bits.shape
    Xh = np.zeros((g, c, G), dtype=np.complex128)
    Xh[..., 0:17] = sre * sign[..., 0:17]
    Xh[..., 1:16] += 1j * sim * sign[..., 17:32]
    Xh[..., 17:32] = np.conj(Xh[..., 15:0:-1])
    return Xh


def fft1bit_dequant(bits: np.ndarray, sre16: np.ndarray, sim16: np.ndarray) -> np.ndarray:
    """Eq. 5, right half: x' = IDFT(Q * s) with the 1/32-normalised inverse.  -> [T, C]."""
    Xh = fft1bit_spectrum(bits, sre16, sim16)
    Finv = np.conj(_dft_matrix()) / G                              # [k, t] -> e^{+..}/32
    x = np.einsum("gck,kt->gtc", Xh, Finv)
    assert np.abs(x.imag).max(initial=0.0) < 1e-9 * (1.0 + np.abs(x.real).max(initial=0.0))
    g, t, c = x.shape
    return x.real.reshape(g * t, c)


# --------------------------------------------------------------------------
# Keys: MixQuant (Alg. 3) = selection + 2-bit anomalous + FFT 1-bit normal
# --------------------------------------------------------------------------
def quantize_keys_block(K16: np.ndarray, anom: np.ndarray, norm: np.ndarray,
                        use_fft: bool = True) -> dict:
    """The group coding of Alg. 3 for [T, D] tokens with a GIVEN channel split:
    Eq. 4 at 2 bits on the anomalous channels; on the others Eq. 5 (1BitQuant
    with the FFT), or with use_fft = False the "standard" 1-bit quantizer of
    Sec. 4.1, which is Alg. 3's GQuant(bit = 1) applied to the tokens
    themselves: Eq. 4 with n = 1 (z = min, s = max - min, code in {0, 1}).  In
    that case n_bits holds the codes by token and n_sre16 / n_sim16 hold s / z.

    This is also the residual flush of Alg. 1 (Decoding, the branch taken when
    the residual buffer holds R tokens) under this build's reading: the block
    of new tokens is coded with the split chosen at prefill and appended; both
    codes are local to a 32-token group, so earlier groups are not affected.
    """
    a = gquant(K16[:, anom], bits=2)
    if use_fft:
        n = fft1bit_quant(K16[:, norm])
    else:
        n1 = gquant(K16[:, norm], bits=1)
        n = {"bits": n1["codes"], "sre16": n1["s16"], "sim16": n1["z16"], "near": n1["near"]}
    return {
        "anom": anom, "norm": norm, "perm": np.concatenate([anom, norm]).astype(np.int64),
        "a_codes": a["codes"], "a_s16": a["s16"], "a_z16": a["z16"], "a_near": a["near"],
        "n_bits": n["bits"], "n_sre16": n["sre16"], "n_sim16": n["sim16"], "n_near": n["near"],
        "fft": use_fft,
    }


def quantize_keys_head(K16: np.ndarray, n_a: int, use_fft: bool = True, metric: int = 0):
    """Alg. 3 for one [T, D] head.  Returns the logical (unpacked) cache record.
    metric: 0 Range (the paper's choice), 1 Variance, 2 Outliers (its ablation)."""
    R = (key_channel_range, key_channel_variance, key_channel_outliers)[metric](K16)
    anom, norm, perm = select_anomalous_channels(R, n_a)
    rec = quantize_keys_block(K16, anom, norm, use_fft)
    rec["range"] = R
    rec["perm"] = perm
    return rec


def dequantize_keys_head(rec: dict) -> np.ndarray:
    """DeQuant of Alg. 1 (decoding) for one head -> K' [T, D] float64."""
    anom, norm = rec["anom"], rec["norm"]
    T = rec["a_codes"].shape[0] * G if len(anom) else rec["n_bits"].shape[0] * G
    out = np.zeros((T, len(anom) + len(norm)), dtype=np.float64)
    if len(anom):
        out[:, anom] = gdequant(rec["a_codes"], rec["a_s16"], rec["a_z16"])
    if len(norm):
        if rec.get("fft", True):
            out[:, norm] = fft1bit_dequant(rec["n_bits"], rec["n_sre16"], rec["n_sim16"])
        else:
            out[:, norm] = gdequant(rec["n_bits"], rec["n_sre16"], rec["n_sim16"])
    return out


# --------------------------------------------------------------------------
# Values: token protection and the ternary quantizer (Eq. 6, Eq. 7; Alg. 2)
# --------------------------------------------------------------------------
def saliency_scores(Xv16: np.ndarray, Xt16: np.ndarray) -> np.ndarray:
    """Eq. 7 (Sec. 3.3 (2)): I(i, j) = X_v(i) . X_t(j) for every visual token i
    and text token j of one sequence; the paper does not say how the text axis
    is reduced - here the scores of a visual token are summed over j.

    Xv16 [Tv, d], Xt16 [Nt, d] fp16.  Returns [Tv] float64.
    """
    I = Xv16.astype(np.float64) @ Xt16.astype(np.float64).T        # [Tv, Nt]
    return I.sum(axis=1)


def select_salient_tokens(scores: np.ndarray, n_s: int) -> np.ndarray:
    """Top-n_s tokens by saliency score (Sec. 3.3 (2): top n = p * l_v tokens).

    scores: [T] float32.  Ties go to the lower token index.  Returns the chosen
    indices in ascending order (int32).
    """
    T = scores.shape[0]
    order = sorted(range(T), key=lambda t: (-float(scores[t]), t))
    return np.array(sorted(order[:n_s]), dtype=np.int32)


def ternary_quant(V16: np.ndarray, salient_idx: np.ndarray, gamma: float):
    """Eq. 6 / Alg. 2 (1.58Quant) per channel over groups of G tokens.

    s = Mean(|V|) over the non-protected tokens of the group, alpha = gamma*s,
    code = +1 if v > alpha, -1 if v < -alpha, else 0.  Protected tokens are
    coded 0 and returned verbatim (fp16) in `rows`.
    Returns codes [g, D, G] int8, s16 [g, D] fp16, near [g, D, G], rows [n_s, D].
    """
    T, D = V16.shape
    assert T % G == 0
    keep = np.ones(T, dtype=bool)
    keep[salient_idx] = False
    x = V16.astype(np.float64).reshape(T // G, G, D).transpose(0, 2, 1)     # [g, c, t]
    m = keep.reshape(T // G, 1, G)
    n = m.sum(axis=2)                                                       # [g, 1]
    tot = (np.abs(x) * m).sum(axis=2)
    s = np.where(n > 0, tot / np.maximum(n, 1), 0.0)                        # [g, c]
    alpha = gamma * s
    codes = np.zeros(x.shape, dtype=np.int8)
    codes[x > alpha[..., None]] = 1
    codes[x < -alpha[..., None]] = -1
    codes[np.broadcast_to(~m, codes.shape)] = 0
    near = np.abs(np.abs(x) - alpha[..., None]) < BAND_TRIT * alpha[..., None]
    near &= np.broadcast_to(m, near.shape)
    return {
        "codes": codes,
        "s16": s.astype(np.float16),
        "near": near,
        "rows": V16[salient_idx].copy(),
    }


def stp_quant_rows(rows16: np.ndarray, bits: int = 2) -> dict:
    """Alg. 2, STPQuant, the protected branch: GQuant(X[E], d = channel, bit = 2).

    rows16 [n_s, D] fp16: the protected rows of one head gathered in token
    order.  Eq. 4 per channel over groups of G consecutive protected rows; the
    last group holds n_s mod G rows when that is not zero and takes its minimum
    and maximum over the rows it has.  Returns codes [n_s, D] uint8, s16 and z16
    [ceil(n_s / G), D] fp16, near [n_s, D] bool.
    """
    n_s, D = rows16.shape
    npg = (n_s + G - 1) // G
    levels = (1 << bits) - 1
    codes = np.zeros((n_s, D), dtype=np.uint8)
    near = np.zeros((n_s, D), dtype=bool)
    s_all = np.zeros((npg, D)); z_all = np.zeros((npg, D))
    for pg in range(npg):
        x = rows16[pg * G:(pg + 1) * G].astype(np.float64)          # [n <= G, D]
        z = x.min(axis=0)
        s = (x.max(axis=0) - z) / levels
        safe = np.where(s > 0, s, 1.0)
        u = (x - z) / safe
        c = np.clip(np.rint(u), 0, levels)
        nr = np.abs(u - (np.floor(u) + 0.5)) < BAND
        c[:, s == 0] = 0
        nr[:, s == 0] = False
        codes[pg * G:(pg + 1) * G] = c.astype(np.uint8)
        near[pg * G:(pg + 1) * G] = nr
        s_all[pg] = s; z_all[pg] = z
    return {"codes": codes, "s16": s_all.astype(np.float16), "z16": z_all.astype(np.float16), "near": near}


def stp_dequant_rows(codes: np.ndarray, s16: np.ndarray, z16: np.ndarray) -> np.ndarray:
    """Eq. 4, right half, for the protected rows: X' = Q * s + z with the group's stored
    fp16 s, z.  -> [n_s, D] float64."""
    n_s = codes.shape[0]
    pg = np.arange(n_s) // G
    return codes.astype(np.float64) * s16.astype(np.float64)[pg] + z16.astype(np.float64)[pg]


def ternary_dequant(codes: np.ndarray, s16: np.ndarray, salient_idx: np.ndarray,
                    rows16: np.ndarray) -> np.ndarray:
    """V' = s * code for coded tokens; protected tokens take the rows given (the verbatim
    fp16 rows, or the dequantized 2-bit rows of STPQuant). -> [T, D]."""
    x = codes.astype(np.float64) * s16.astype(np.float64)[..., None]        # [g, c, t]
    g, c, t = x.shape
    out = x.transpose(0, 2, 1).reshape(g * t, c)
    if len(salient_idx):
        out[salient_idx] = rows16.astype(np.float64)
    return out


# --------------------------------------------------------------------------
# Decode attention (Eq. 3; Alg. 1, Decoding)
# --------------------------------------------------------------------------
def attention_single_query(q16: np.ndarray, Kstar: np.ndarray, Vstar: np.ndarray,
                           scale: float) -> np.ndarray:
    """A = Softmax(scale * q K*^T) V* for one query head.

    q16 [D] fp16; K*, V* [T_total, D] float64 = dequantized cache rows followed
    by the fp16 residual rows (Alg. 1: concat along tokens).  Plain dense
    softmax in float64.
    """
    q = q16.astype(np.float64)
    S = scale * (Kstar @ q)
    S = S - S.max()
    P = np.exp(S)
    P = P / P.sum()
    return P @ Vstar


def decode_attention(q16: np.ndarray, Kdq: np.ndarray, Vdq: np.ndarray,
                     K_tail16: np.ndarray, V_tail16: np.ndarray, scale: float) -> np.ndarray:
    """Grouped-query decode step for one sequence and one layer.

    q16 [Hq, D]; Kdq, Vdq [Hkv, T, D] float64 (dequantized); tails [Hkv, Tr, D]
    fp16.  Query head h reads KV head h // (Hq // Hkv).  -> [Hq, D] float64.
    """
    Hq = q16.shape[0]
    Hkv = Kdq.shape[0]
    rep = Hq // Hkv
    out = np.zeros((Hq, q16.shape[1]), dtype=np.float64)
    for h in range(Hq):
        kv = h // rep
        Ks = np.concatenate([Kdq[kv], K_tail16[kv].astype(np.float64)], axis=0)
        Vs = np.concatenate([Vdq[kv], V_tail16[kv].astype(np.float64)], axis=0)
        out[h] = attention_single_query(q16[h], Ks, Vs, scale)
    return out
