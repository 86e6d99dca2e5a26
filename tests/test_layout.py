"""Pins of the oracle's packed-format reader/writer: round trip, every bit of
a record owned by exactly one logical field, and a few positions worked out by
hand from the format description."""
import numpy as np
import pytest

from oracle import layout as LY


def _rand_key_rec(rng, ng, n_a):
    n_n = 128 - n_a
    perm = rng.permutation(128)
    anom = np.sort(perm[:n_a]); norm = np.sort(perm[n_a:])
    return {
        "perm": np.concatenate([anom, norm]).astype(np.uint8),
        "a_codes": rng.integers(0, 4, size=(ng, n_a, 32)).astype(np.uint8),
        "a_s16": rng.standard_normal((ng, n_a)).astype(np.float16),
        "a_z16": rng.standard_normal((ng, n_a)).astype(np.float16),
        "n_bits": rng.integers(0, 2, size=(ng, n_n, 32)).astype(np.uint8),
        "n_sre16": rng.standard_normal((ng, n_n)).astype(np.float16),
        "n_sim16": rng.standard_normal((ng, n_n)).astype(np.float16),
    }


@pytest.mark.parametrize("n_a", [0, 8, 16, 32, 64, 128])
def test_key_round_trip_and_size(n_a):
    rng = np.random.default_rng(n_a)
    rec = _rand_key_rec(rng, 3, n_a)
    perm, by = LY.pack_key_head(rec, n_a)
    assert by.shape == (3, 12 * n_a + 8 * (128 - n_a))
    back = LY.unpack_key_head(perm, by, n_a)
    for k in ("a_codes", "a_s16", "a_z16", "n_bits", "n_sre16", "n_sim16", "perm"):
        np.testing.assert_array_equal(back[k], rec[k])
    # nominal code bits per element: 2 * n_a + 1 * n_n over 128 channels
    code_bytes = 8 * n_a + 4 * (128 - n_a)
    assert code_bytes * 8 / (32 * 128) == pytest.approx(1 + n_a / 128)


def test_key_every_bit_is_one_field():
    n_a = 16
    rng = np.random.default_rng(1)
    rec = _rand_key_rec(rng, 1, n_a)
    perm, by = LY.pack_key_head(rec, n_a)
    base = LY.unpack_key_head(perm, by, n_a)
    seen = set()
    for byte in range(by.shape[1]):
        for bit in range(8):
            b2 = by.copy(); b2[0, byte] ^= (1 << bit)
            r2 = LY.unpack_key_head(perm, b2, n_a)
            changed = []
            for k in ("a_codes", "n_bits"):
                d = np.argwhere(r2[k] != base[k])
                changed += [(k, tuple(x)) for x in d]
            for k in ("a_s16", "a_z16", "n_sre16", "n_sim16"):
                d = np.argwhere(r2[k].view(np.uint16) != base[k].view(np.uint16))
                changed += [(k, tuple(x)) for x in d]
            assert len(changed) == 1, (byte, bit, changed)
            seen.add(changed[0])
    assert len(seen) == 16 * 32 + 112 * 32 + 2 * 16 + 2 * 112


def test_key_hand_positions():
    """Anomalous channel 6 at token 9 -> byte 9*(n_a/4) + 1, bits 4,5.
    Normal channel 21 (block 2, e = 5): Re X[3] -> word (2,3) bit 5;
    Im X[3] -> same word bit 13; Re X[16] -> word (2,0) bit 13."""
    n_a = 16
    rec = _rand_key_rec(np.random.default_rng(2), 1, n_a)
    for k in ("a_codes", "n_bits"):
        rec[k][:] = 0
    for k in ("a_s16", "a_z16", "n_sre16", "n_sim16"):
        rec[k][:] = 0
    rec["a_codes"][0, 6, 9] = 3
    rec["n_bits"][0, 21, 3] = 1
    rec["n_bits"][0, 21, 16 + 3] = 1
    rec["n_bits"][0, 21, 16] = 1
    rec["a_s16"][0, 5] = np.float16(2.0)      # 0x4000
    rec["n_sim16"][0, 21] = np.float16(-2.0)  # 0xC000
    _, by = LY.pack_key_head(rec, n_a)
    nz = {int(i): int(by[0, i]) for i in np.nonzero(by[0])[0]}
    o = 12 * n_a
    w23 = o + 2 * (2 * 16 + 3)
    w20 = o + 2 * (2 * 16 + 0)
    meta = o + 4 * 112 + 2 * ((2 * 2 + 1) * 8 + 5)
    assert nz == {
        9 * 4 + 1: 0x30,
        8 * n_a + 2 * 5 + 1: 0x40,
        w23: 1 << 5, w23 + 1: 1 << 5,
        w20 + 1: 1 << 5,
        meta + 1: 0xC0,
    }


def test_value_round_trip_bits_and_positions():
    rng = np.random.default_rng(3)
    codes = rng.integers(-1, 2, size=(2, 128, 32)).astype(np.int8)
    s16 = rng.standard_normal((2, 128)).astype(np.float16)
    by = LY.pack_value_head(codes, s16)
    assert by.shape == (2, 1280)
    c2, s2 = LY.unpack_value_head(by)
    np.testing.assert_array_equal(c2, codes)
    np.testing.assert_array_equal(s2, s16)
    # hand position: channel 35 (m=2 -> mp 1, mh 0; r=3), token 17 -> kb 0, slot 5
    # -> field at bit 8*0 + 16*1 + 2*2 = 20 (nz), 21 (neg) of word (0, 3, 1)
    z = np.zeros((1, 128, 32), dtype=np.int8); z[0, 35, 17] = -1
    b = LY.pack_value_head(z, np.zeros((1, 128), np.float16))
    word = (0 * 16 + 3) * 4 + 1
    nzb = {int(i): int(b[0, i]) for i in np.nonzero(b[0])[0]}
    assert nzb == {4 * word + 2: 0x30}
    # token 6 of channel 16 (m=1 -> mp 0, mh 1; r=0) -> kb 1, slot 2 -> bit 8 + 0 + 2 = 10, +1 only
    z[:] = 0; z[0, 16, 6] = 1
    b = LY.pack_value_head(z, np.zeros((1, 128), np.float16))
    nzb = {int(i): int(b[0, i]) for i in np.nonzero(b[0])[0]}
    assert nzb == {4 * ((1 * 16 + 0) * 4 + 0) + 1: 0x04}
    # scale of channel 35 sits at half index r*8 + m = 3*8 + 2
    sc = np.zeros((1, 128), np.float16); sc[0, 35] = np.float16(2.0)
    b = LY.pack_value_head(np.zeros((1, 128, 32), np.int8), sc)
    nzb = {int(i): int(b[0, i]) for i in np.nonzero(b[0])[0]}
    assert nzb == {1024 + 2 * 26 + 1: 0x40}
    # each 2-bit field of the trit area is one (channel, token)
    seen = set()
    base = np.zeros((1, 1280), dtype=np.uint8)
    for byte in range(1024):
        for f in range(4):
            b2 = base.copy(); b2[0, byte] = 1 << (2 * f)
            c3, _ = LY.unpack_value_head(b2)
            d = np.argwhere(c3 != 0)
            assert len(d) == 1 and c3[tuple(d[0])] == 1
            seen.add(tuple(d[0]))
    assert len(seen) == 128 * 32


def test_sections_and_salient_round_trip():
    L, B, H, T, n_s = 2, 3, 4, 256, 10
    ks = LY.key_sections(L, B, H, T, 16)
    assert ks["rec"] % 256 == 0 and ks["rec"] >= L * B * H * 128
    assert ks["total"] >= ks["rec"] + L * B * H * (T // 32) * 1088
    vs = LY.value_sections(L, B, H, T, n_s)
    assert vs["idx"] >= L * B * H * 8 * 1280
    for k in ("idx", "mask", "rank", "rows", "total"):
        assert vs[k] % 256 == 0
    assert vs["total"] >= vs["rows"] + 2 * L * B * H * n_s * 128
    assert LY.value_sections(L, B, H, T, 0) == {"rec": 0, "total": L * B * H * 8 * 1280}
    buf = np.zeros(vs["total"], dtype=np.uint8)
    idx = np.array([0, 31, 32, 33, 100, 101, 102, 200, 254, 255], dtype=np.int32)
    LY.pack_salient(buf, vs, 1, B, T, idx)
    i2, mask, rank = LY.unpack_salient(buf, vs, 1, T, n_s)
    np.testing.assert_array_equal(i2, idx)
    assert mask[0] == (1 | (1 << 31)) and mask[1] == 0b11 and mask[3] == (1 << 4 | 1 << 5 | 1 << 6)
    assert rank.tolist() == [0, 2, 4, 4, 7, 7, 7, 8]


def test_protected_rows_two_bit_records_roundtrip_and_size():
    rng = np.random.default_rng(8)
    for n_s in (1, 31, 32, 70, 96):
        npg = (n_s + 31) // 32
        codes = rng.integers(0, 4, (n_s, 128)).astype(np.uint8)
        s16 = rng.random((npg, 128)).astype(np.float16)
        z16 = rng.standard_normal((npg, 128)).astype(np.float16)
        buf = LY.pack_protected2(codes, s16, z16)
        assert buf.size == npg * LY.PREC
        c, s, z = LY.unpack_protected2(buf, n_s)
        np.testing.assert_array_equal(c, codes)
        np.testing.assert_array_equal(s.view(np.uint16), s16.view(np.uint16))
        np.testing.assert_array_equal(z.view(np.uint16), z16.view(np.uint16))
    # byte j of a row: channel 4 j + r in bits 2r, 2r + 1
    codes = np.zeros((1, 128), np.uint8); codes[0, 6] = 3; codes[0, 127] = 1
    buf = LY.pack_protected2(codes, np.zeros((1, 128), np.float16), np.zeros((1, 128), np.float16))
    assert buf[1] == 3 << 4 and buf[31] == 1 << 6 and buf[:1024].sum() == (3 << 4) + (1 << 6)
    a = LY.value_sections(1, 2, 4, 640, 70)
    b = LY.value_sections(1, 2, 4, 640, 70, 2)
    assert a["rows"] == b["rows"]
    assert b["total"] - b["rows"] == (8 * 3 * LY.PREC + 255) // 256 * 256
