"""Input generator: published SplitMix64 vectors, determinism, chunk and
offset independence, distribution moments, stored first values."""
import json
import math
import os

import numpy as np

from paper_2506_10401_amd import datagen

HERE = os.path.dirname(os.path.abspath(__file__))


def test_splitmix64_published_vectors():
    # first outputs of the reference SplitMix64 generator for seeds 0 and
    # 1234567 (Vigna's public-domain splitmix64.c; the same stream as
    # java.util.SplittableRandom's mix64 on a golden-gamma counter)
    got = [int(v) for v in datagen.splitmix64(0, 0, 4)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F, 0xF88BB8A8724C81EC]
    got = [int(v) for v in datagen.splitmix64(1234567, 0, 5)]
    assert got == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                   4593380528125082431, 16408922859458223821]


def test_counter_based_offsets_and_chunking():
    a = datagen.splitmix64(99, 0, 100)
    b = datagen.splitmix64(99, 40, 60)
    assert np.array_equal(a[40:], b)
    n = (1 << 20) * 2 + 12345  # spans several chunks with a ragged tail
    x = datagen.gen_normal(7, (n,), 0.0, 1.0)
    y = datagen.gen_normal(7, (n,), 0.0, 1.0)
    assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    head = datagen.gen_normal(7, (1000,), 0.0, 1.0)
    assert np.array_equal(x[:1000], head)
    u = datagen.gen_uniform(7, (n,), -1.0, 1.0)
    assert np.array_equal(u[:1000], datagen.gen_uniform(7, (1000,), -1.0, 1.0))


def test_moments_and_range():
    n = 1_000_000
    u = datagen.gen_uniform(11, (n,), -1.0, 1.0).astype(np.float64)
    assert u.min() >= -1.0 and u.max() <= 1.0
    assert abs(u.mean()) < 4 * (2 / math.sqrt(12)) / math.sqrt(n)
    assert abs(u.var() - 1 / 3) < 4 * math.sqrt(4 / 45) / math.sqrt(n)
    z = datagen.gen_normal(12, (n,), 1.0, 0.1).astype(np.float64)
    assert abs(z.mean() - 1.0) < 4 * 0.1 / math.sqrt(n)
    assert abs(z.var() - 0.01) < 4 * 0.01 * math.sqrt(2 / n)
    zs = (z - 1.0) / 0.1
    assert abs(np.mean(zs ** 3)) < 4 * math.sqrt(15 / n)       # skewness 0
    assert abs(np.mean(zs ** 4) - 3) < 4 * math.sqrt(96 / n)   # kurtosis 3


def test_shapes_dtypes_and_seeds_of_the_five_workloads():
    small = {1: {}, 2: dict(N=2, C=3, H=5, W=7), 3: dict(M=4, N=10), 4: dict(N=1, C=2, H=4, W=4, K=3),
             5: dict(B=2, L=5, D=8)}
    seen = set()
    for cfg in range(1, 6):
        t = datagen.make(cfg, **small[cfg])
        for name, (ti, shape, kind, p0, p1) in datagen.CONFIGS[cfg](**small[cfg]).items():
            assert t[name].shape == shape and t[name].dtype == np.float32
            assert t[name].flags["C_CONTIGUOUS"]
            seen.add(datagen.tensor_seed(cfg, ti))
    assert len(seen) == 3 + 4 + 3 + 3 + 3  # no two tensors share a stream
    full = datagen.CONFIGS[4]()
    assert full["wt"][4] == math.sqrt(2.0 / 576)
    assert datagen.make(2, variant=1, N=1, C=1, H=2, W=2)["X"][0, 0, 0, 0] != \
        datagen.make(2, variant=0, N=1, C=1, H=2, W=2)["X"][0, 0, 0, 0]


def test_stored_first_values():
    with open(os.path.join(HERE, "golden", "datagen_first8.json")) as f:
        gold = json.load(f)
    assert len(gold) == 24   # 16 tensors of the five workloads + 3 of the dropout chain + 5 of the conv block
    for key, rec in gold.items():
        gen = datagen.gen_uniform if rec["kind"] == "u" else datagen.gen_normal
        got = gen(int(rec["seed"], 16), (8,), rec["p0"], rec["p1"]).view(np.uint32)
        assert ["%08x" % int(b) for b in got] == rec["bits"], key
