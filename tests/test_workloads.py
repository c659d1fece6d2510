"""Synthetic workload generator: shapes, bucket layouts, and bit-reproducible values."""
import numpy as np
import torch

from workloads import buckets, configs, shapes, synth


def test_architecture_totals():
    for fn, n_t, n_p, n_b in ((shapes.resnet50, 161, 25557032, 4),
                              (shapes.bert_base, 199, 109482240, 13),
                              (shapes.gpt2_medium, 292, 354823168, 37)):
        ts = fn()
        lay = buckets.ddp_buckets(ts)
        assert len(ts) == n_t and lay.n_params == n_p and lay.n_buckets == n_b
        assert sum(l for _, l in lay.buckets) == n_p
        assert [o for o, _ in lay.buckets] == list(np.cumsum([0] + [l for _, l in lay.buckets])[:-1])
        assert sum(l for _, l, _ in lay.tensors) == n_p
    assert [l for _, l in buckets.ddp_buckets(shapes.resnet50()).buckets] == \
        [7564264, 6563840, 7091712, 4337216]
    bn = shapes.resnet50_bn_channels()
    assert len(bn) == 53 and sum(bn) == 26560 and min(bn) == 64 and max(bn) == 2048


def test_groupings_are_bijections():
    for cid in range(1, 6):
        cfg = configs.config(cid)
        for g in cfg.groupings + tuple(configs.reversed_slots(x) for x in cfg.groupings):
            assert len(g.worker_of_est) == cfg.n_logical
            assert len(set(zip(g.worker_of_est, g.slot_of_est))) == cfg.n_logical
            assert sorted(g.schedule()) == list(range(cfg.n_logical))
    g5 = configs.config(5).groupings
    assert [g5[1].worker_of_est.count(w) for w in range(7)] == [3, 5, 7, 9, 11, 13, 16]
    assert [g5[2].worker_of_est.count(w) for w in range(7)] == [3, 5, 7, 9, 11, 13, 16]


def _numpy_twin(lo, hi, key):
    """The generator's integer part written again with numpy uint64."""
    with np.errstate(over="ignore"):
        x = np.arange(lo, hi, dtype=np.uint64) + np.uint64(key)
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    s = sum(((z >> np.uint64(k)) & np.uint64(0xFFFF)).astype(np.int64) for k in (0, 16, 32, 48))
    return s - 131070


def test_generator_matches_numpy_twin_and_statistics():
    key = synth.stream_key(0x5EED0002, 3, 5)
    s = synth.field_sums(1000, 1000 + (1 << 18), key).numpy()
    assert np.array_equal(s, _numpy_twin(1000, 1000 + (1 << 18), key))
    assert abs(s.mean()) < 4 * synth.STD_S / np.sqrt(s.size)
    assert abs(s.std() / synth.STD_S - 1) < 0.02
    lay = buckets.single_bucket(1 << 18)
    v = synth.values(lay, 0, 1 << 18, 1, 0, 0, 1e-2, False).numpy()
    assert v.dtype == np.float32 and abs(v.std() / 1e-2 - 1) < 0.02


def test_generator_windows_and_streams():
    lay = buckets.ddp_buckets(shapes.resnet50())
    off, ln = lay.buckets[1]
    whole = synth.gradient(lay, 1, 11, 2, 3)
    assert whole.numel() == ln
    part = synth.values(lay, off + 5000, off + 9000, 11, 2, 3)
    assert torch.equal(whole[5000:9000], part)
    assert not torch.equal(whole, synth.gradient(lay, 1, 11, 2, 4))
    assert not torch.equal(whole, synth.gradient(lay, 1, 11, 1, 3))
    # per-tensor scale: the 1-D tensors (fan_in 1) are much larger than conv weights
    t_off, t_len, fan = lay.tensors[0]
    assert fan == 1 and t_len == 1000          # fc.bias comes first in reversed order


def test_values_at_matches_ranges():
    lay = buckets.ddp_buckets(shapes.resnet50())
    idx = torch.cat([torch.arange(a, b) for a, b in ((0, 50), (990, 1100), (2049000, 2049100),
                                                     (lay.n_params - 77, lay.n_params))])
    got = synth.values_at(lay, idx, 3, 1, 6)
    want = torch.cat([synth.values(lay, a, b, 3, 1, 6) for a, b in ((0, 50), (990, 1100), (2049000, 2049100),
                                                                    (lay.n_params - 77, lay.n_params))])
    assert torch.equal(got, want)
    p = synth.values_at(lay, idx, 3, 0, synth.STREAM_PARAM, 1.0, True)
    assert torch.equal(p, synth.params(lay, 3)[idx])
