"""The synthetic generators are deterministic, prefix-consistent and shaped like the configs."""
import numpy as np

import workloads


def test_shapes_and_determinism():
    w = workloads.get_workload("tiny")
    k, v = workloads.kv_pair(w, 0, 1)
    k2, v2 = workloads.kv_pair(w, 0, 1)
    assert k.dtype == np.float16 and k.shape == (256, 64)
    assert np.array_equal(k, k2) and np.array_equal(v, v2)
    kp, _ = workloads.kv_pair(w, 0, 1, 100)
    assert np.array_equal(kp, k[:100])
    kk, vv = workloads.kv_tensor(w)
    assert np.array_equal(kk[0, 1], k) and np.array_equal(vv[0, 1], v)
    assert workloads.query(w).shape == (1, 4, 64)


def test_outlier_channels_are_wide():
    w = workloads.get_workload("llama7b_4bit")
    k, v = workloads.kv_pair(w, 3, 5, 512)
    for x in (k, v):
        s = x.astype(np.float64).std(axis=0)
        assert (s > 8).sum() == 4
        assert np.abs(x.astype(np.float64)).max() <= workloads.kv_synth.CLIP


def test_mixed_lengths_and_layer_outliers():
    w = workloads.get_workload("llama13b_mixed")
    lens = workloads.seq_lens(w)
    assert lens.shape == (4,) and lens.min() >= 8192 and lens.max() <= 16384
    total = sum(workloads.kv_synth._outlier_channels(w, 0, h).size for h in range(w.kv_heads))
    assert total == 51
    k, _ = workloads.appended_pair(w, 0, 0)
    assert k.shape == (128, 128)
