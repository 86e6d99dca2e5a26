"""GPU parity of the Variance and Outliers channel metrics of Sec. 3.2 (1) (the paper's
ablation of how Alg. 3 picks the 2-bit channels): the permutation against the oracle's
float64 ranking, then the usual codec and attention checks on top of that split."""
import dataclasses

import numpy as np
import pytest
import torch

import parity as P
from paper_2503_16257_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("metric", [1, 2])
@pytest.mark.parametrize("case", ["toy", "layer", "long_ragged_chunk", "serving_batch"])
def test_channel_metric_selection_codec_and_attention(case, metric):
    if case == "toy":
        w = synth.WORKLOADS["c1_toy"]
    elif case == "layer":
        w = synth.WORKLOADS["c2_layer"]
    elif case == "long_ragged_chunk":
        w = synth.reduced(synth.WORKLOADS["c4_long"], 40)               # 7840 tokens = 15 chunks + 160
    else:
        w = dataclasses.replace(synth.reduced(synth.WORKLOADS["c5_serving"], 8, B=3), n_anom=32)
    print(f"[case] metric{metric}-{case}", flush=True)
    run = P.GpuRun(w, DEV, channel_metric=metric)
    stats = {}
    for hd in range(w.n_heads):
        P.check_keys_head(run, hd, synth.key_head(w, hd), stats)
    P.check_near_budget(stats)
    q = synth.query(w, 0)
    out = run.attention(0, torch.from_numpy(q).to(DEV)).cpu().numpy()
    for b in range(w.B):
        P.assert_out_close(out[b], P.oracle_attention(run, 0, b, q[b]), f"{case} seq {b}")


def test_metrics_pick_different_channels_than_range():
    w = synth.WORKLOADS["c2_layer"]
    perms = [P.GpuRun(w, DEV, channel_metric=m).key_record(0)["perm"] for m in (0, 1, 2)]
    assert not np.array_equal(perms[0], perms[1]) or not np.array_equal(perms[0], perms[2])
    for p in perms:
        assert sorted(p.tolist()) == list(range(128))
