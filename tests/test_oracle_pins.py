"""Pins of the CPU oracle against things it did not compute itself:
library routines, closed forms, invariants, brute force, and the numbers the
paper prints.  All CPU; no GPU code is touched here."""
import math
import os

import numpy as np
import pytest

from oracle import vidkv_oracle as O
from paper_2503_16257_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    vals = {}
    with open(os.path.join(HERE, "golden", "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split()
                vals[k] = float(v)
    return vals


def _f16(x):
    return np.asarray(x, dtype=np.float64).astype(np.float16)


# ------------------------------------------------------------ paper values --
def test_paper_constants_match_oracle_defaults():
    g = _golden()
    assert O.G == g["group_size"]
    assert 4 * 28 * 128 * 1000 * 196 * 256 == g["footnote_bytes"]


def test_nominal_bit_widths_from_code_counts():
    """Average code bits per element, counted from the oracle's own records,
    reproduce the bit-widths the paper quotes (Sec. 4.1, Sec. 4.2, Table 2)."""
    g = _golden()
    rng = np.random.default_rng(0)
    K = _f16(rng.standard_normal((64, 128)))
    for k, name in ((0.25, "key_bits_k0.25"), (0.5, "key_bits_k0.50"), (0.75, "key_bits_k0.75")):
        rec = O.quantize_keys_head(K, int(k * 128))
        nbits = 2 * rec["a_codes"].size + 1 * rec["n_bits"].size
        assert nbits / K.size == pytest.approx(g[name], abs=1e-12)
    assert math.log2(3) == pytest.approx(g["value_bits_ternary"], abs=0.006)
    assert 0.2 * 2 + 0.8 * g["value_bits_ternary"] == pytest.approx(g["value_bits_p0.2"], abs=0.005)


# -------------------------------------------------------------- DFT pins ----
def test_dft_matches_numpy_rfft():
    rng = np.random.default_rng(1)
    x = _f16(rng.standard_normal((3 * 32, 5)) * 3)
    q = O.fft1bit_quant(x)
    ref = np.fft.rfft(x.astype(np.float64).reshape(3, 32, 5), axis=1)       # [g, 17, c]
    coef = q["coef"]                                                        # [g, c, 32]
    np.testing.assert_allclose(coef[..., 0:17], ref.real.transpose(0, 2, 1), atol=1e-11)
    np.testing.assert_allclose(coef[..., 17:32], ref.imag.transpose(0, 2, 1)[..., 1:16], atol=1e-11)
    # scales are the full-spectrum means of |Re|, |Im|
    full = np.fft.fft(x.astype(np.float64).reshape(3, 32, 5), axis=1)
    np.testing.assert_array_equal(q["sre16"], np.abs(full.real).mean(axis=1).astype(np.float16))
    np.testing.assert_array_equal(q["sim16"], np.abs(full.imag).mean(axis=1).astype(np.float16))


def test_dequant_matches_numpy_irfft():
    rng = np.random.default_rng(2)
    bits = rng.integers(0, 2, size=(4, 7, 32)).astype(np.uint8)
    sre = _f16(rng.uniform(0.5, 4, size=(4, 7)))
    sim = _f16(rng.uniform(0.5, 4, size=(4, 7)))
    x = O.fft1bit_dequant(bits, sre, sim)                                   # [128, 7]
    sign = 2.0 * bits - 1.0
    half = np.zeros((4, 7, 17), dtype=np.complex128)
    half[..., :] = sre.astype(np.float64)[..., None] * sign[..., 0:17]
    half[..., 1:16] += 1j * sim.astype(np.float64)[..., None] * sign[..., 17:32]
    ref = np.fft.irfft(half, n=32, axis=2)                                  # [g, c, t]
    np.testing.assert_allclose(x, ref.transpose(0, 2, 1).reshape(128, 7), atol=1e-12)


def test_parseval_on_quantization_error():
    rng = np.random.default_rng(3)
    x = _f16(rng.standard_normal((2 * 32, 9)))
    q = O.fft1bit_quant(x)
    xr = O.fft1bit_dequant(q["bits"], q["sre16"], q["sim16"])
    X = np.fft.fft(x.astype(np.float64).reshape(2, 32, 9), axis=1).transpose(0, 2, 1)
    Xh = O.fft1bit_spectrum(q["bits"], q["sre16"], q["sim16"])
    lhs = ((x.astype(np.float64) - xr) ** 2).reshape(2, 32, 9).sum(axis=1)
    rhs = (np.abs(X - Xh) ** 2).sum(axis=2) / 32
    np.testing.assert_allclose(lhs, rhs, rtol=1e-10)


def test_fft_codec_closed_forms():
    """Impulse reconstructs exactly; a positive constant becomes an impulse;
    a negative constant gives 0.9375|a| at t=0 and -|a|/16 elsewhere.  These fix
    sign(0) -> bit 1, the 1/32 inverse normalisation and the Hermitian fill."""
    a = 1.5
    imp = np.zeros((32, 1)); imp[0, 0] = a
    q = O.fft1bit_quant(_f16(imp))
    assert q["bits"].min() == 1 and float(q["sre16"][0, 0]) == a and float(q["sim16"][0, 0]) == 0.0
    np.testing.assert_allclose(O.fft1bit_dequant(q["bits"], q["sre16"], q["sim16"]), imp, atol=1e-12)

    # an all-zero group has exactly zero coefficients: sign(0) codes as bit 1
    q = O.fft1bit_quant(np.zeros((32, 1), dtype=np.float16))
    assert q["bits"].min() == 1 and not q["near"].any()

    # a constant: only the DC bin is non-zero; in floating point the other bins
    # are ~1e-15, which is what the exclusion band is for.
    const = np.full((32, 1), a)
    q = O.fft1bit_quant(_f16(const))
    assert q["coef"][0, 0, 0] == pytest.approx(32 * a, abs=1e-12) and q["bits"][0, 0, 0] == 1
    assert np.abs(q["coef"][0, 0, 1:]).max() < 1e-12 and q["near"][0, 0, 1:].all()
    assert not q["near"][0, 0, 0]
    assert float(q["sre16"][0, 0]) == a and float(q["sim16"][0, 0]) == 0.0
    ones = np.ones((1, 1, 32), dtype=np.uint8)
    np.testing.assert_allclose(O.fft1bit_dequant(ones, q["sre16"], q["sim16"]), imp, atol=1e-12)

    q = O.fft1bit_quant(_f16(-const))
    assert q["bits"][0, 0, 0] == 0
    neg = ones.copy(); neg[0, 0, 0] = 0
    xr = O.fft1bit_dequant(neg, q["sre16"], q["sim16"])[:, 0]
    assert xr[0] == pytest.approx(0.9375 * a, abs=1e-12)
    np.testing.assert_allclose(xr[1:], -a / 16, atol=1e-12)


def test_fft_codec_single_tone_sign_and_slot_order():
    """x = cos(2 pi 3 t/32) has Re X[3] = +16, x = sin(...) has Im X[3] = -16:
    pins the forward sign convention and the slot numbering (slot 3, slot 19)."""
    t = np.arange(32)
    c = np.cos(2 * np.pi * 3 * t / 32).reshape(32, 1)
    s = np.sin(2 * np.pi * 3 * t / 32).reshape(32, 1)
    qc = O.fft1bit_quant(c.astype(np.float16))
    qs = O.fft1bit_quant(s.astype(np.float16))
    assert qc["coef"][0, 0, 3] == pytest.approx(16.0, abs=0.02)
    assert qs["coef"][0, 0, 16 + 3] == pytest.approx(-16.0, abs=0.02)
    assert qc["bits"][0, 0, 3] == 1 and qs["bits"][0, 0, 19] == 0


def test_fft_codec_white_noise_mse_closed_form():
    """For white N(0,1) groups the relative reconstruction MSE has a closed
    form.  With the scale equal to the sample mean of |Y| over the 32-bin view,
    sum_k (Y_k - s sign Y_k)^2 = sum Y^2 - (2*32 - n) s^2, n = bins that carry a
    level (32 for Re, 30 for Im whose bins 0 and 16 are identically zero), and
    E s^2 = (E s)^2 + Var s with E|Y| = sqrt(2 v/pi), Var|Y| = v (1 - 2/pi)."""
    c = math.sqrt(2 / math.pi)
    vr = 1 - 2 / math.pi
    es_re = c * (2 * math.sqrt(32) + 30 * 4) / 32
    var_re = (2 * 32 * vr + 4 * 15 * 16 * vr) / 32 ** 2
    es_im = c * (30 * 4) / 32
    var_im = (4 * 15 * 16 * vr) / 32 ** 2
    err_re = (2 * 32 + 30 * 16) - 32 * (es_re ** 2 + var_re)
    err_im = (30 * 16) - 34 * (es_im ** 2 + var_im)
    expect = (err_re + err_im) / 32 / 32
    assert expect == pytest.approx(0.345, abs=2e-3)
    rng = np.random.default_rng(4)
    x = _f16(rng.standard_normal((400 * 32, 16)))
    q = O.fft1bit_quant(x)
    xr = O.fft1bit_dequant(q["bits"], q["sre16"], q["sim16"])
    xd = x.astype(np.float64)
    rel = ((xd - xr) ** 2).sum() / (xd ** 2).sum()
    assert rel == pytest.approx(expect, abs=0.005)


def test_frequency_domain_scoring_identity():
    """sum_c q_c IDFT(Xhat_c) == IDFT(sum_c q_c Xhat_c): what lets a GPU kernel
    contract in the frequency domain and invert once per query head."""
    rng = np.random.default_rng(5)
    x = _f16(rng.standard_normal((32, 24)))
    qv = rng.standard_normal(24)
    q = O.fft1bit_quant(x)
    lhs = O.fft1bit_dequant(q["bits"], q["sre16"], q["sim16"]) @ qv
    Y = (O.fft1bit_spectrum(q["bits"], q["sre16"], q["sim16"])[0] * qv[:, None]).sum(axis=0)
    rhs = np.fft.ifft(Y)
    assert np.abs(rhs.imag).max() < 1e-12
    np.testing.assert_allclose(lhs, rhs.real, atol=1e-12)


# ---------------------------------------------------------- 2-bit pins ------
def test_gquant_exact_on_four_level_data_and_bounds():
    rng = np.random.default_rng(6)
    lv = rng.integers(0, 4, size=(64, 6))
    lv[0, :] = 0; lv[1, :] = 3; lv[32, :] = 0; lv[33, :] = 3
    x = _f16(-2.0 + 0.75 * lv)                     # levels exactly representable
    q = O.gquant(x, 2)
    np.testing.assert_array_equal(q["codes"], lv.reshape(2, 32, 6).transpose(0, 2, 1))
    assert np.all(q["s16"] == np.float16(0.75)) and np.all(q["z16"] == np.float16(-2.0))
    np.testing.assert_array_equal(O.gdequant(q["codes"], q["s16"], q["z16"]), x.astype(np.float64))

    y = _f16(rng.standard_normal((96, 11)) * 5)
    q = O.gquant(y, 2)
    assert q["codes"].max() <= 3
    yd = y.astype(np.float64)
    yr = O.gdequant(q["codes"], q["s16"], q["z16"])
    s = q["s16"].astype(np.float64)
    bound = (s / 2 + 3 * s * 2.0 ** -11 + 1e-12)[:, None, :].repeat(32, axis=1).reshape(96, 11)
    assert np.all(np.abs(yd - yr) <= bound)
    # group minimum reproduces exactly (code 0 -> z) and the maximum takes code 3
    yg = yd.reshape(3, 32, 11)
    cg = q["codes"].transpose(0, 2, 1)
    assert np.all(cg[yg == yg.min(axis=1, keepdims=True)] == 0)
    assert np.all(cg[yg == yg.max(axis=1, keepdims=True)] == 3)


def test_gquant_constant_group_and_half_even():
    x = np.full((32, 1), 0.5, dtype=np.float16)
    q = O.gquant(x, 2)
    assert q["codes"].max() == 0 and float(q["s16"][0, 0]) == 0 and float(q["z16"][0, 0]) == 0.5
    # values at exactly 0.5 and 1.5 steps: ties round to even (0 and 2) and are flagged near
    v = np.zeros((32, 1)); v[1] = 3.0; v[2] = 0.5; v[3] = 1.5; v[4] = 2.5
    q = O.gquant(_f16(v), 2)
    assert list(q["codes"][0, 0, :5]) == [0, 3, 0, 2, 2]
    assert list(q["near"][0, 0, :5]) == [False, False, True, True, True]


# --------------------------------------------------- channel selection ------
def test_channel_selection_brute_force_and_ties():
    rng = np.random.default_rng(7)
    R = rng.integers(0, 12, size=128).astype(np.float32)     # many ties
    for n_a in (0, 8, 16, 64, 128):
        anom, norm, perm = O.select_anomalous_channels(R, n_a)
        ref = np.lexsort((np.arange(128), -R))[:n_a]
        assert sorted(ref.tolist()) == anom.tolist()
        assert sorted(set(range(128)) - set(ref.tolist())) == norm.tolist()
        assert perm.tolist() == anom.tolist() + norm.tolist()


def test_planted_outlier_channels_are_selected():
    w = synth.WORKLOADS["c1_toy_na8"]
    K = synth.key_head(w, 0)
    planted = synth.outlier_channels(w, 0).tolist()
    anom, _, _ = O.select_anomalous_channels(O.key_channel_range(K), 8)
    assert anom.tolist() == planted
    anom64, _, _ = O.select_anomalous_channels(O.key_channel_range(K), 64)
    assert set(planted) <= set(anom64.tolist())
    w2 = synth.reduced(synth.WORKLOADS["c2_layer"], 8)
    for hd in range(2):
        K = synth.key_head(w2, hd)
        anom, _, _ = O.select_anomalous_channels(O.key_channel_range(K), 16)
        assert set(synth.outlier_channels(w2, hd).tolist()) <= set(anom.tolist())


def test_key_range_is_float32_difference():
    K = np.zeros((32, 128), dtype=np.float16)
    K[3, 5] = 60000.0; K[9, 5] = -0.00123
    R = O.key_channel_range(K)
    assert R.dtype == np.float32
    assert R[5] == np.float32(60000.0) - np.float32(np.float16(-0.00123))
    assert R[0] == 0


# -------------------------------------------------------- ternary pins ------
def test_ternary_statistics_closed_form():
    g = _golden()
    gamma = g["gamma"]
    rng = np.random.default_rng(8)
    V = _f16(rng.standard_normal((600 * 32, 8)))
    q = O.ternary_quant(V, np.zeros(0, dtype=np.int32), gamma)
    c = math.sqrt(2 / math.pi)
    alpha = gamma * c
    p0 = math.erf(alpha / math.sqrt(2))
    assert p0 == pytest.approx(0.4235, abs=1e-3)
    assert (q["codes"] == 0).mean() == pytest.approx(p0, abs=0.01)
    assert (q["codes"] == 1).mean() == pytest.approx((1 - p0) / 2, abs=0.01)
    phi = math.exp(-alpha ** 2 / 2) / math.sqrt(2 * math.pi)
    mse = 1 - 2 * c * (2 * phi) + c * c * (1 - p0)
    assert mse == pytest.approx(0.2775, abs=1e-3)
    Vd = V.astype(np.float64)
    Vr = O.ternary_dequant(q["codes"], q["s16"], np.zeros(0, dtype=np.int32), q["rows"])
    # the closed form is the large-group limit; with 32-token groups the sample
    # mean adapts to each group and the error sits about 1/32 lower.
    got = ((Vd - Vr) ** 2).sum() / (Vd ** 2).sum()
    assert mse - 0.02 < got < mse


def test_ternary_brute_force_with_protected_tokens():
    rng = np.random.default_rng(9)
    V = _f16(rng.standard_normal((64, 128)) * 2)
    idx = np.array([0, 5, 31, 33, 34, 63], dtype=np.int32)
    gamma = 0.7
    q = O.ternary_quant(V, idx, gamma)
    Vd = V.astype(np.float64)
    for g_ in range(2):
        for c in (0, 17, 127):
            toks = [t for t in range(32 * g_, 32 * g_ + 32) if t not in idx]
            s = sum(abs(Vd[t, c]) for t in toks) / len(toks)
            assert q["s16"][g_, c] == np.float16(s)
            for t in range(32 * g_, 32 * g_ + 32):
                code = q["codes"][g_, c, t - 32 * g_]
                if t in idx:
                    assert code == 0
                else:
                    assert code == (1 if Vd[t, c] > gamma * s else -1 if Vd[t, c] < -gamma * s else 0)
                    assert code * Vd[t, c] >= 0
    np.testing.assert_array_equal(q["rows"], V[idx])
    Vr = O.ternary_dequant(q["codes"], q["s16"], idx, q["rows"])
    np.testing.assert_array_equal(Vr[idx], Vd[idx])           # fp16 passthrough is exact
    assert set(np.unique(q["codes"]).tolist()) <= {-1, 0, 1}


def test_ternary_fully_protected_group():
    V = _f16(np.ones((32, 128)))
    q = O.ternary_quant(V, np.arange(32, dtype=np.int32), 0.7)
    assert q["codes"].max() == 0 and q["codes"].min() == 0 and float(q["s16"].max()) == 0.0


def test_token_selection_brute_force():
    rng = np.random.default_rng(10)
    sc = rng.integers(0, 50, size=500).astype(np.float32)     # ties
    for n in (0, 1, 50, 499, 500):
        got = O.select_salient_tokens(sc, n)
        ref = np.sort(np.lexsort((np.arange(500), -sc))[:n])
        np.testing.assert_array_equal(got, ref.astype(np.int32))


# ------------------------------------------------------ attention pins ------
def test_attention_matches_torch_sdpa_and_closed_forms():
    import torch
    rng = np.random.default_rng(11)
    q = _f16(rng.standard_normal(128))
    K = rng.standard_normal((77, 128)); V = rng.standard_normal((77, 128))
    scale = 1 / math.sqrt(128)
    out = O.attention_single_query(q, K, V, scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q.astype(np.float64)).reshape(1, 1, 1, 128),
        torch.from_numpy(K).reshape(1, 1, 77, 128), torch.from_numpy(V).reshape(1, 1, 77, 128),
        scale=scale).reshape(128).numpy()
    np.testing.assert_allclose(out, ref, atol=1e-12)
    # zero query -> plain mean of V; output stays inside each column's range
    np.testing.assert_allclose(O.attention_single_query(_f16(np.zeros(128)), K, V, scale),
                               V.mean(axis=0), atol=1e-12)
    assert np.all(out <= V.max(axis=0) + 1e-12) and np.all(out >= V.min(axis=0) - 1e-12)
    # two keys: softmax reduces to a logistic weight
    K2 = rng.standard_normal((2, 128)); V2 = rng.standard_normal((2, 128))
    d = scale * (K2[0] - K2[1]) @ q.astype(np.float64)
    w0 = 1 / (1 + math.exp(-d))
    np.testing.assert_allclose(O.attention_single_query(q, K2, V2, scale),
                               w0 * V2[0] + (1 - w0) * V2[1], atol=1e-12)
    # a dominant key selects its value row
    K3 = K.copy(); K3[40] = 500 * q.astype(np.float64)
    np.testing.assert_allclose(O.attention_single_query(q, K3, V, scale), V[40], atol=1e-9)


def test_decode_attention_gqa_mapping_and_tail():
    rng = np.random.default_rng(12)
    Hkv, Hq, T, Tr = 2, 6, 64, 5
    q = _f16(rng.standard_normal((Hq, 128)))
    Kd = rng.standard_normal((Hkv, T, 128)); Vd = rng.standard_normal((Hkv, T, 128))
    Kt = _f16(rng.standard_normal((Hkv, Tr, 128))); Vt = _f16(rng.standard_normal((Hkv, Tr, 128)))
    out = O.decode_attention(q, Kd, Vd, Kt, Vt, 0.1)
    for h in range(Hq):
        kv = h // 3
        Ks = np.vstack([Kd[kv], Kt[kv].astype(np.float64)])
        Vs = np.vstack([Vd[kv], Vt[kv].astype(np.float64)])
        s = 0.1 * Ks @ q[h].astype(np.float64)
        p = np.exp(s - s.max()); p /= p.sum()
        np.testing.assert_allclose(out[h], p @ Vs, atol=1e-12)
    # no quantized tokens at all: attention over the fp16 tail only
    out0 = O.decode_attention(q, Kd[:, :0], Vd[:, :0], Kt, Vt, 0.1)
    for h in range(Hq):
        kv = h // 3
        s = 0.1 * Kt[kv].astype(np.float64) @ q[h].astype(np.float64)
        p = np.exp(s - s.max()); p /= p.sum()
        np.testing.assert_allclose(out0[h], p @ Vt[kv].astype(np.float64), atol=1e-12)


def test_end_to_end_toy_quality():
    """On the toy workload the codec behaves as the paper describes: planted
    channels are well preserved by the 2-bit path, normal channels land at the
    white-noise 1-bit error, ternary values at theirs."""
    w = synth.WORKLOADS["c1_toy_na8"]
    K = synth.key_head(w, 0); V = synth.value_head(w, 0)
    rec = O.quantize_keys_head(K, 8)
    Kr = O.dequantize_keys_head(rec)
    Kd = K.astype(np.float64)
    rel_n = ((Kd[:, rec["norm"]] - Kr[:, rec["norm"]]) ** 2).sum() / (Kd[:, rec["norm"]] ** 2).sum()
    rel_a = ((Kd[:, rec["anom"]] - Kr[:, rec["anom"]]) ** 2).sum() / (Kd[:, rec["anom"]] ** 2).sum()
    assert rel_n == pytest.approx(0.345, abs=0.01)
    # 4 levels over a ~4.1 sigma range of 32 Gaussian samples: step^2/12 ~ 0.15
    assert 0.10 < rel_a < 0.20
    sal = O.select_salient_tokens(synth.saliency(w)[0], w.n_salient)
    assert len(sal) == 156
    qv = O.ternary_quant(V, sal, float(np.float32(0.7)))
    Vr = O.ternary_dequant(qv["codes"], qv["s16"], sal, qv["rows"])
    keep = np.ones(w.T, bool); keep[sal] = False
    Vd = V.astype(np.float64)
    assert ((Vd[keep] - Vr[keep]) ** 2).sum() / (Vd[keep] ** 2).sum() == pytest.approx(0.2775 - 0.01, abs=0.015)


def test_flush_reading_block_local_and_idempotent():
    """Residual flush (Alg. 1, Decoding).  The printed algorithm re-runs MixQuant
    on the dequantized cache concatenated with the residual block; this build
    codes only the block, with the prefill's channel split.  Two facts make the
    two agree: (1) both codes are local to a 32-token group, so coding a block
    alone gives what coding the whole sequence gives for those groups; (2)
    re-coding already dequantized groups with the same split reproduces their
    codes and sign bits, so leaving them untouched loses nothing - and it avoids
    the one thing re-coding would change: the imaginary scale, a mean over 32
    bins of which 2 are structurally zero, shrinks by 30/32 on every pass."""
    w = synth.WORKLOADS["c1_toy_na8"]
    K = synth.key_head(w, 0)[:512]
    full = O.quantize_keys_head(K, 8)
    blk = O.quantize_keys_block(K[384:512], full["anom"], full["norm"])      # last 4 groups alone
    for k in ("a_codes", "a_s16", "a_z16", "n_bits", "n_sre16", "n_sim16"):
        np.testing.assert_array_equal(blk[k], full[k][12:16], err_msg=k)
    # (2) re-code the dequantized cache (rounded to the fp16 it would be held in)
    Kd = O.dequantize_keys_head(full).astype(np.float16)
    again = O.quantize_keys_block(Kd, full["anom"], full["norm"])
    np.testing.assert_array_equal(again["a_codes"], full["a_codes"])
    assert (again["n_bits"] != full["n_bits"]).mean() < 2e-3       # only coefficients lost in fp16 rounding
    np.testing.assert_allclose(again["a_s16"].astype(np.float64), full["a_s16"].astype(np.float64), rtol=2e-3)
    np.testing.assert_allclose(again["n_sre16"].astype(np.float64), full["n_sre16"].astype(np.float64), rtol=5e-3)
    np.testing.assert_allclose(again["n_sim16"].astype(np.float64),
                               full["n_sim16"].astype(np.float64) * 30 / 32, rtol=5e-3)
    # values: a block without protected tokens is the plain 1.58Quant of Alg. 2
    V = synth.value_head(w, 0)[:128]
    none = np.zeros(0, dtype=np.int32)
    qv = O.ternary_quant(V, none, 0.7)
    s = np.abs(V.astype(np.float64)).reshape(4, 32, 128).mean(axis=1)          # [g, D]
    np.testing.assert_array_equal(qv["s16"], s.astype(np.float16))
    x = V.astype(np.float64).reshape(4, 32, 128).transpose(0, 2, 1)            # [g, D, G]
    want = np.where(x > 0.7 * s[:, :, None], 1, np.where(x < -0.7 * s[:, :, None], -1, 0))
    ok = ~qv["near"]
    np.testing.assert_array_equal(qv["codes"][ok], want[ok])


def test_saliency_scores_brute_force_and_linearity():
    """Eq. 7 summed over the text tokens: brute-force double loop on a tiny case,
    linearity in the text rows (the sum of per-text-token scores), and the
    equivalent matrix-vector form X_v . (sum_j X_t(j))."""
    rng = np.random.default_rng(21)
    Xv = _f16(rng.standard_normal((7, 24))); Xt = _f16(rng.standard_normal((3, 24)))
    got = O.saliency_scores(Xv, Xt)
    want = np.zeros(7)
    for i in range(7):
        for j in range(3):
            for c in range(24):
                want[i] += float(Xv[i, c]) * float(Xt[j, c])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    per_j = sum(O.saliency_scores(Xv, Xt[j:j + 1]) for j in range(3))
    np.testing.assert_allclose(got, per_j, atol=1e-12)
    np.testing.assert_allclose(got, Xv.astype(np.float64) @ Xt.astype(np.float64).sum(axis=0), atol=1e-12)
    # a visual token orthogonal to every text token scores 0; one equal to the only text token scores |x|^2
    e = np.zeros((2, 24), np.float16); e[0, 0] = 2.0; e[1, 1] = 3.0
    t = np.zeros((1, 24), np.float16); t[0, 1] = 3.0
    np.testing.assert_array_equal(O.saliency_scores(e, t), [0.0, 9.0])
    # the synthetic hidden states plant a common direction: those visual tokens rank on top
    w = synth.WORKLOADS["c1_toy"]
    Xv, Xt = synth.hidden_states(w, 0, rows=512, d=256)
    s = O.saliency_scores(Xv, Xt)
    top = np.argsort(-s)[:50]
    assert s[top].min() > np.median(s) + 3 * s.std() / 4


def test_stp_rows_two_bit_brute_force_and_bounds():
    """STPQuant's protected branch (Alg. 2): Eq. 4 at 2 bits per channel over groups of 32
    gathered rows, ragged last group.  Brute force on a tiny case, exactness on four-level
    data, the half-step error bound, and agreement with the key-side Eq. 4 coder on whole groups."""
    rng = np.random.default_rng(31)
    rows = _f16(rng.standard_normal((70, 128)) * 3)
    q = O.stp_quant_rows(rows)
    assert q["codes"].shape == (70, 128) and q["s16"].shape == (3, 128)
    for pg, c in ((0, 5), (1, 77), (2, 127)):                      # group 2 holds 6 rows
        col = [float(v) for v in rows[32 * pg:32 * (pg + 1), c]]
        lo, hi = min(col), max(col)
        s = (hi - lo) / 3
        want = [min(3, max(0, round((v - lo) / s))) for v in col]   # Python rounds half to even
        ok = ~q["near"][32 * pg:32 * (pg + 1), c]
        assert [w for w, k in zip(want, ok) if k] == [int(v) for v, k in zip(q["codes"][32 * pg:32 * (pg + 1), c], ok) if k]
        assert float(q["z16"][pg, c]) == lo and float(q["s16"][pg, c]) == float(np.float16(s))
    d = O.stp_dequant_rows(q["codes"], q["s16"], q["z16"])
    pg = np.arange(70) // 32
    step = q["s16"].astype(np.float64)[pg]
    assert np.all(np.abs(d - rows.astype(np.float64)) <= 0.5 * step * (1 + 2e-3) + 3 * step * 2 ** -11)
    # rows that take exactly four equally spaced values per channel come back exactly
    lv = _f16(np.array([-1.5, -0.5, 0.5, 1.5]))
    four = lv[rng.integers(0, 4, (64, 128))]
    four[0] = lv[0]; four[1] = lv[3]; four[32] = lv[0]; four[33] = lv[3]
    q4 = O.stp_quant_rows(four)
    np.testing.assert_array_equal(O.stp_dequant_rows(q4["codes"], q4["s16"], q4["z16"]), four.astype(np.float64))
    # whole groups: the same arithmetic as the key-side group quantizer
    g = O.gquant(rows[:64], bits=2)
    np.testing.assert_array_equal(q["codes"][:64].reshape(2, 32, 128).transpose(0, 2, 1), g["codes"])
    np.testing.assert_array_equal(q["s16"][:2], g["s16"])
    # a constant channel: s = 0, codes 0, value restored from z
    const = rows.copy(); const[:, 3] = np.float16(2.5)
    qc = O.stp_quant_rows(const)
    assert not qc["codes"][:, 3].any() and np.all(qc["s16"][:, 3] == 0)
    assert np.all(O.stp_dequant_rows(qc["codes"], qc["s16"], qc["z16"])[:, 3] == 2.5)


def test_standard_one_bit_quantizer_closed_forms():
    """Eq. 4 with n = 1 (the non-FFT 1-bit path of Sec. 4.1 / Alg. 3): every token maps to the
    group's minimum or maximum, whichever is nearer (ties to the minimum: round half to even);
    two-level data come back exactly; the error never exceeds half the range."""
    rng = np.random.default_rng(41)
    x = _f16(rng.standard_normal((64, 5)) * 2)
    q = O.gquant(x, bits=1)
    assert set(np.unique(q["codes"])) <= {0, 1}
    d = O.gdequant(q["codes"], q["s16"], q["z16"])
    xd = x.astype(np.float64)
    for g in range(2):
        blk = xd[32 * g:32 * g + 32]
        lo, hi = blk.min(axis=0), blk.max(axis=0)
        nearer_hi = (hi - blk) < (blk - lo)
        want = np.where(nearer_hi, 1, 0)
        ok = ~q["near"][g].T
        np.testing.assert_array_equal(q["codes"][g].T[ok], want[ok])
        np.testing.assert_array_equal(q["z16"][g].astype(np.float64), lo)
        assert np.all(np.abs(d[32 * g:32 * g + 32] - blk) <= 0.5 * (hi - lo) * (1 + 1e-3) + 1e-3)
    two = _f16(np.where(rng.random((32, 4)) < 0.5, -0.75, 1.25)); two[0] = -0.75; two[1] = 1.25
    q2 = O.gquant(two, bits=1)
    np.testing.assert_array_equal(O.gdequant(q2["codes"], q2["s16"], q2["z16"]), two.astype(np.float64))
    # exact midpoint -> code 0 (0.5 rounds to the even integer 0)
    mid = _f16(np.array([[0.0], [2.0], [1.0]] + [[0.0]] * 29))
    qm = O.gquant(mid, bits=1)
    assert qm["codes"][0, 0, 2] == 0 and qm["near"][0, 0, 2]
    # through the head-level entry: same channel split as the FFT mode, only the normal part changes
    w = synth.WORKLOADS["c1_toy_na8"]
    K = synth.key_head(w, 0)[:256]
    a = O.quantize_keys_head(K, 8)
    b = O.quantize_keys_head(K, 8, use_fft=False)
    np.testing.assert_array_equal(a["perm"], b["perm"])
    np.testing.assert_array_equal(a["a_codes"], b["a_codes"])
    g1 = O.gquant(K[:, b["norm"]], bits=1)
    np.testing.assert_array_equal(b["n_bits"], g1["codes"])
    Kb = O.dequantize_keys_head(b)
    np.testing.assert_array_equal(Kb[:, b["norm"]], O.gdequant(g1["codes"], g1["s16"], g1["z16"]))
    # white noise: a two-level code at the extremes of 32 samples is much worse than the FFT code
    Kd = K.astype(np.float64)
    err_fft = ((Kd - O.dequantize_keys_head(a))[:, a["norm"]] ** 2).mean()
    err_std = ((Kd - Kb)[:, b["norm"]] ** 2).mean()
    assert err_std > 3 * err_fft


def test_variance_and_outlier_metrics_closed_forms():
    """The two other channel metrics of Sec. 3.2 (1): numpy's variance and a brute-force count;
    on the synthetic keys all three metrics find the planted heavy-tailed channels."""
    rng = np.random.default_rng(51)
    K = _f16(rng.standard_normal((640, 128)) * rng.uniform(0.5, 2.0, 128) + rng.standard_normal(128))
    np.testing.assert_allclose(O.key_channel_variance(K), K.astype(np.float64).var(axis=0), rtol=1e-12)
    n = O.key_channel_outliers(K)
    for c in (0, 17, 127):
        a = [abs(float(v)) for v in K[:, c]]
        m = sum(a) / len(a)
        assert n[c] == sum(1 for v in a if v > 3 * m)
    # a constant channel has no spread by any metric; a two-valued one has a known variance
    K2 = K.copy(); K2[:, 5] = np.float16(1.5); K2[::2, 9] = np.float16(2.0); K2[1::2, 9] = np.float16(-2.0)
    assert O.key_channel_variance(K2)[5] == 0 and O.key_channel_outliers(K2)[5] == 0
    assert O.key_channel_variance(K2)[9] == 4.0 and O.key_channel_outliers(K2)[9] == 0
    w = synth.WORKLOADS["c2_layer"]
    Kh = synth.key_head(w, 1)
    planted = set(synth.outlier_channels(w, 1).tolist())
    for metric in (0, 1, 2):
        rec = O.quantize_keys_head(Kh[:2048], 16, metric=metric)
        assert planted <= set(rec["anom"].tolist()), metric
    assert not np.array_equal(O.quantize_keys_head(Kh[:2048], 64, metric=1)["perm"],
                              O.quantize_keys_head(Kh[:2048], 64, metric=2)["perm"])
