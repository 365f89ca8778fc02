"""Host-side checks of the seeded input generators (no GPU, no oracle arithmetic)."""
import os

import numpy as np

import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_shape_grid_is_frozen_and_distinct():
    shapes = wl.c4_shapes()
    assert len(shapes) == 200 and len(set(shapes)) == 200
    with open(os.path.join(GOLDEN, "shape_grid_200.txt")) as f:
        stored = [tuple(int(x) for x in line.split()) for line in f if not line.startswith("#")]
    assert stored == shapes
    for s in shapes:
        assert all(v in wl.GRID_VALUES for v in s)


def test_generators_are_seeded_and_typed():
    a1, b1 = wl.c1_inputs()
    a2, b2 = wl.c1_inputs()
    assert a1.dtype == np.float16 and a1.shape == (256, 256) and b1.shape == (256, 256)
    assert np.array_equal(a1.view(np.uint16), a2.view(np.uint16))
    assert np.array_equal(b1.view(np.uint16), b2.view(np.uint16))
    assert -1.0 <= float(a1.min()) and float(a1.max()) <= 1.0
    a, b = wl.c2_inputs((1024, 1024, 1024))
    assert abs(float(a.astype(np.float64).std()) - 1 / 32) < 2e-3
    a, b = wl.c3_inputs((16, 4096, 4096))
    assert a.shape == (16, 4096) and b.shape == (4096, 4096)
    assert abs(float(b.astype(np.float64).std()) - 0.02) < 1e-3
    assert abs(float(a.astype(np.float64).std()) - 1.0) < 2e-2


def test_exact_families_stay_representable():
    for shape in [(64, 64, 128), (64, 64, 512), (32, 32, 2048), (16, 16, 8192)]:
        name, a, b = wl.exact_family_for(shape)
        ai, bi = a.astype(np.int64), b.astype(np.int64)
        assert np.array_equal(ai.astype(np.float16), a) and np.array_equal(bi.astype(np.float16), b)
        c = ai @ bi
        if name != "binary":
            assert np.abs(c).max() <= 2048
        else:
            assert (c < 2048).mean() > 0.9 and (c > 0).all()
    a, b = wl.small_int_inputs((8, 8, 128))
    assert set(np.unique(a)).issubset({-2, -1, 0, 1, 2})


def test_sample_positions_in_range_and_cover_edges():
    ii, jj = wl.sample_positions((1000, 3000, 64), 5000)
    assert ii.shape == jj.shape and ii.size >= 5000
    assert ii.min() == 0 and ii.max() == 999 and jj.min() == 0 and jj.max() == 2999
    pairs = set(zip(ii.tolist(), jj.tolist()))
    assert (0, 0) in pairs and (999, 2999) in pairs and (255, 256) in pairs


def test_padding_arithmetic_example_from_the_paper():
    # Section 5.2: M = 8192 with BM = 160 is padded to 8320 rows, about 1.6 % more
    with open(os.path.join(GOLDEN, "paper_padding_example.txt")) as f:
        row = [line.split() for line in f if not line.startswith("#")][0]
    M, BM, padded, pct = int(row[0]), int(row[1]), int(row[2]), float(row[3])
    tiles = -(-M // BM)
    assert tiles * BM == padded
    assert round(100.0 * (padded - M) / M, 1) == pct
