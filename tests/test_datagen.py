"""Integer-exact checks of the input generators: two implementations of the recurrence, frozen
first values, exact flip counts, layout bookkeeping."""
import json
import os
import numpy as np
import pytest
from datagen import CounterRNG, make_workload, param_layout, param_count, round_to_bf16, init_theta
from datagen.rng import raw_py
from datagen.workloads import WORKLOADS

GOLD = os.path.join(os.path.dirname(__file__), "golden", "datagen_first8.json")


def test_rng_numpy_matches_pure_python():
    for seed, stream in ((0, 0), (20231006, 3), (2**40 + 17, 1000)):
        a = CounterRNG(seed).raw(stream, 64, offset=5)
        b = [raw_py(seed, stream, 5 + i) for i in range(64)]
        assert [int(x) for x in a] == b


def test_uniform_range_and_integers():
    r = CounterRNG(7)
    u = r.uniform(1, 100000)
    assert u.min() >= 0.0 and u.max() < 1.0 and abs(u.mean() - 0.5) < 5e-3
    k = r.integers(2, 100000, 7)
    assert k.min() == 0 and k.max() == 6
    z = r.normal(3, 200001)
    assert abs(z.mean()) < 1e-2 and abs(z.std() - 1.0) < 1e-2
    p = r.permutation(4, 1000)
    assert sorted(p.tolist()) == list(range(1000))


def test_frozen_first_values():
    """First 8 raw draws / indices / labels per workload, frozen after the two implementations
    of the recurrence agreed (tests/golden/make_datagen_golden.py wrote the file)."""
    gold = json.load(open(GOLD))
    for cfg in (1, 2, 3):
        wl = make_workload(cfg)
        g = gold[str(cfg)]
        assert [int(v) for v in CounterRNG(wl.seed).raw(1, 8)] == g["raw_stream1"]
        assert wl.train_batch(0)[:8].tolist() == g["train_batch0"]
        assert wl.y_train[:8].tolist() == g["y_train"]
        assert wl.y_meta[:8].tolist() == g["y_meta"]
        assert np.nonzero(wl.flipped)[0][:8].tolist() == g["flipped_idx"]


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_flip_count_exact(cfg):
    wl = make_workload(cfg)
    assert wl.flipped.sum() == int(np.floor(wl.noise * wl.n_train))
    assert np.all((wl.y_train != wl.y_train_clean) == wl.flipped)
    assert wl.y_train.min() >= 0 and wl.y_train.max() < wl.n_classes


def test_batches_partition_epoch():
    wl = make_workload(2)
    per = wl.n_train // wl.batch
    seen = np.concatenate([wl.train_batch(s) for s in range(per)])
    assert sorted(seen.tolist()) == list(range(wl.n_train))
    assert not np.array_equal(wl.train_batch(0), wl.train_batch(per))


def test_tokens():
    wl = make_workload(3, n_train=64, n_meta=8)
    assert wl.x_train.dtype == np.int32 and np.all(wl.x_train[:, 0] == 0)
    assert wl.x_train[:, 1:].min() >= 1 and wl.x_train.max() < wl.dims[5]


def test_param_counts():
    assert param_count("mlp", (32, 2)) == 66
    assert param_count("mlp", (784, 256, 256, 10)) == 269322
    for cfg, n in ((3, 5290500), (4, 108599814), (5, 353915906)):
        assert param_count("encoder", WORKLOADS[cfg]["dims"]) == n
    lay = param_layout("encoder", WORKLOADS[3]["dims"])
    offs = [o for _, _, o in lay]
    assert offs == sorted(offs) and offs[0] == 0


def test_bf16_rounding():
    x = np.array([1.0, 1.00390625, 1.001953125, 1.01171875, -0.3, 3.0e-5])
    r = round_to_bf16(x)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 and r[3] == 1.0 + 2.0**-6
    bits = r.astype(np.float32).view(np.uint32)
    assert np.all(bits & 0xFFFF == 0)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2**-8)
    th = init_theta(make_workload(3, n_train=8, n_meta=8))
    assert np.all(th.astype(np.float32).view(np.uint32) & 0xFFFF == 0)


def test_sequence_length_mix():
    from datagen import seq_lengths
    l = seq_lengths(77, 4000, 128)
    assert l.dtype == np.int32 and l.min() >= 1 and l.max() == 128
    assert 0.2 < np.mean(l == 128) < 0.35 and 40 < np.median(l) < 100       # a quarter truncated, the rest spread out
    assert np.array_equal(l, seq_lengths(77, 4000, 128)) and not np.array_equal(l, seq_lengths(78, 4000, 128))
    assert seq_lengths(3, 50, 4).min() >= 1
