"""GPU parity of the 2-bit protected rows (Alg. 2, STPQuant: the protected tokens
at 2 bits per channel, everything else ternary) and of decode attention over them."""
import dataclasses

import numpy as np
import pytest
import torch

import parity as P
from oracle import vidkv_oracle as O
from paper_2503_16257_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check(w, run, scores):
    stats = {}
    for hd in range(w.n_heads):
        b = (hd // w.Hkv) % w.B
        sal = P.oracle_salient(w, b, scores[b], None)
        P.check_values_head(run, hd, synth.value_head(w, hd), sal, stats)
    P.check_near_budget(stats)
    assert "v2bit" in stats and stats["v2bit"][1] == w.n_heads * w.n_salient * 128
    return stats


@pytest.mark.parametrize("case", ["toy_ragged_group", "long_mfma", "serving_batch", "fewer_than_a_group",
                                  "every_token_protected", "generic_attention_n_a_24"])
def test_two_bit_protected_rows_codec_and_attention(case):
    if case == "toy_ragged_group":
        w = synth.WORKLOADS["c1_toy"]                                   # 156 protected: 4 groups + 28 rows
    elif case == "long_mfma":
        w = synth.reduced(synth.WORKLOADS["c4_long"], 40)               # 7840 tokens, 392 protected
    elif case == "serving_batch":
        w = dataclasses.replace(synth.reduced(synth.WORKLOADS["c5_serving"], 8, B=3), n_salient=313)
    elif case == "fewer_than_a_group":
        w = dataclasses.replace(synth.reduced(synth.WORKLOADS["c4_long"], 8), n_salient=5)
    elif case == "every_token_protected":                               # the all-2-bit value cache
        w = dataclasses.replace(synth.reduced(synth.WORKLOADS["c4_long"], 8), n_salient=1568)
    else:
        w = dataclasses.replace(synth.reduced(synth.WORKLOADS["c4_long"], 8), n_anom=24)
    print(f"[case] stp2-{case}", flush=True)
    run = P.GpuRun(w, DEV, salient_bits=2)
    scores = synth.saliency(w)
    _check(w, run, scores)
    # keys are not affected by the mode
    P.check_keys_head(run, 0, synth.key_head(w, 0), {})
    q = synth.query(w, 0)
    cap = 32
    Kt = np.stack([synth.tail_heads(w, 0, b, cap)[0] for b in range(w.B)])
    Vt = np.stack([synth.tail_heads(w, 0, b, cap)[1] for b in range(w.B)])
    tl = torch.full((w.B,), cap, dtype=torch.int32, device=DEV)
    out = run.attention(0, torch.from_numpy(q).to(DEV), torch.from_numpy(Kt).to(DEV),
                        torch.from_numpy(Vt).to(DEV), cap, tl).cpu().numpy()
    for b in range(w.B):
        ref = P.oracle_attention(run, 0, b, q[b], Kt[b], Vt[b])
        P.assert_out_close(out[b], ref, f"{case} seq {b}")


def test_two_bit_rows_change_only_the_rows_section():
    """Same inputs with fp16 and with 2-bit protected rows: every other section of the value
    buffer holds the same bytes, and the 2-bit run's attention differs from the fp16 run's by
    less than the largest half step of the protected rows' quantizer."""
    w = synth.reduced(synth.WORKLOADS["c4_long"], 16)
    a = P.GpuRun(w, DEV)
    b = P.GpuRun(w, DEV, salient_bits=2)
    sec = P.LY.value_sections(w.L, w.B, w.Hkv, w.T, w.n_salient)
    assert torch.equal(a.pv[:sec["rows"]], b.pv[:sec["rows"]])
    assert b.pv.numel() < a.pv.numel()
    q = torch.from_numpy(synth.query(w, 0)).to(DEV)
    oa = a.attention(0, q).float()
    ob = b.attention(0, q).float()
    half_step = max(float(b.value_record(hd)["p_s16"].astype(np.float32).max()) for hd in range(w.n_heads)) / 2
    assert (oa - ob).abs().max() <= half_step * 1.01 and not torch.equal(oa, ob)


def test_flush_with_two_bit_protected_rows():
    """The residual flush leaves the protected-row records alone."""
    w = synth.reduced(synth.WORKLOADS["c4_long"], 8)
    run = P.GpuRun(w, DEV, salient_bits=2, t_capacity=w.T + 128)
    before = run.value_record(1)
    Kt = np.stack([synth.tail_heads(w, 0, b, 128)[0] for b in range(w.B)])
    Vt = np.stack([synth.tail_heads(w, 0, b, 128)[1] for b in range(w.B)])
    run.flush(0, torch.from_numpy(Kt).to(DEV), torch.from_numpy(Vt).to(DEV), 128, 128)
    run.advance(128)
    after = run.value_record(1)
    np.testing.assert_array_equal(before["p_codes"], after["p_codes"])
    np.testing.assert_array_equal(before["codes"], after["codes"][:w.T // 32])
    q = synth.query(w, 0, step=3)
    out = run.attention(0, torch.from_numpy(q).to(DEV)).cpu().numpy()
    P.assert_out_close(out[0], P.oracle_attention(run, 0, 0, q[0]), "stp2 after flush")
