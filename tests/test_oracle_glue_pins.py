"""Pins of the oracle's glue operations between layers (suppl. "ReLU, Batch-Norm, and Pooling",
"Activations and Accumulation") against hand-computed cases and independent library routines.  CPU only."""
import numpy as np
import pytest
import torch


def test_requantize_hand_cases(orc):
    # step 1: rint ties to even, ReLU gate, clamps
    y = np.array([-3.0, -0.0, 0.0, 0.49, 0.5, 0.51, 1.5, 2.5, 3.5, 126.5, 127.5, 1e9, np.nan, -np.inf, np.inf],
                 np.float32)
    got = orc.requantize(y, 1.0)
    assert got.tolist() == [0, 0, 0, 0, 0, 1, 2, 2, 4, 126, 127, 127, 0, 0, 127]
    # without the gate, signed range
    got = orc.requantize(np.array([-200.0, -127.5, -126.5, -2.5, -0.5, 0.5, 2.5, 300.0], np.float32), 1.0, relu=False,
                         lo=-127, hi=127)
    assert got.tolist() == [-127, -127, -126, -2, 0, 0, 2, 127]
    # the scale is applied by ONE binary32 multiplication before rounding
    inv = np.float32(127.0 / 4.0)
    y = np.array([0.1, 1.0, 3.999, 4.0, 0.015748031], np.float32)
    expect = np.clip(np.rint(y * inv), 0, 127).astype(np.int8)        # numpy float32 product, rint = ties to even
    assert np.array_equal(orc.requantize(y, inv), expect)


def test_requantize_matches_float32_numpy_on_random_data(orc):
    rng = np.random.default_rng(1)
    y = (rng.standard_normal(20000) * 2).astype(np.float32)
    r = (rng.standard_normal(20000) * 2).astype(np.float32)
    ri = rng.integers(-128, 128, size=20000).astype(np.int8)
    inv = np.float32(127.0 / 6.0)
    step = np.float32(4.0 / 127.0)
    a = orc.requantize(y, inv, res_f32=r)
    assert np.array_equal(a, np.clip(np.rint(np.maximum(y + r, np.float32(0)) * inv), 0, 127).astype(np.int8))
    b = orc.requantize(y, inv, res_i8=ri, res_step=step)
    t = y + ri.astype(np.float32) * step
    assert np.array_equal(b, np.clip(np.rint(np.maximum(t, np.float32(0)) * inv), 0, 127).astype(np.int8))
    # the sum is rounded to binary32 before the gate and the scale: a float64 evaluation differs somewhere
    c64 = np.clip(np.rint(np.maximum(y.astype(np.float64) + r, 0) * float(inv)), 0, 127).astype(np.int8)
    assert np.mean(a != c64) < 1e-3
    with pytest.raises(orc.OracleError):
        orc.requantize(y, inv, res_f32=r, res_i8=ri)


@pytest.mark.parametrize("geom", [((3, 3), (2, 2), (1, 1), 9, 11), ((2, 2), (2, 2), (0, 0), 8, 8),
                                  ((3, 2), (1, 2), (1, 0), 5, 7), ((1, 1), (1, 1), (0, 0), 4, 4)])
def test_maxpool_matches_torch(orc, geom):
    kernel, stride, pad, h, w = geom
    rng = np.random.default_rng(2)
    x = rng.integers(-128, 128, size=(2, 3, h, w)).astype(np.int8)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float32)), kernel, stride, pad).numpy()
    assert np.array_equal(orc.maxpool_i8(x, kernel, stride, pad).astype(np.float32), ref)


def test_maxpool_padding_never_wins(orc):
    x = np.full((1, 1, 4, 4), -128, np.int8)
    assert np.all(orc.maxpool_i8(x, (3, 3), (2, 2), (1, 1)) == -128)


def test_avgpool_hand_cases_and_mean(orc):
    x = np.zeros((1, 3, 2, 2), np.int8)
    x[0, 0] = [[1, 2], [3, 4]]          # mean 2.5 -> ties to even: 2
    x[0, 1] = [[3, 4], [3, 4]]          # mean 3.5 -> 4
    x[0, 2] = [[-128, -128], [-128, -128]]
    assert orc.avgpool_requantize(x, 1.0, lo=-128, hi=127).tolist() == [[2, 4, -128]]
    assert orc.avgpool_requantize(x, 1.0).tolist() == [[2, 4, 0]]
    rng = np.random.default_rng(3)
    x = rng.integers(0, 128, size=(4, 16, 7, 7)).astype(np.int8)
    scale = np.float32(0.731)
    got = orc.avgpool_requantize(x, scale)
    inv = np.float32(1.0) / np.float32(49.0)
    expect = np.clip(np.rint((x.sum(axis=(2, 3)).astype(np.float32) * inv) * scale), 0, 127).astype(np.int8)
    assert np.array_equal(got, expect)
    assert np.max(np.abs(got - x.mean(axis=(2, 3)) * float(scale))) <= 0.5 + 1e-4


def test_budget_resample(orc):
    b = np.arange(2 * 4 * 6, dtype=np.uint8).reshape(2, 4, 6)
    assert np.array_equal(orc.budget_resample(b, 4, 6), b)
    assert np.array_equal(orc.budget_resample(b, 2, 3), b[:, ::2, ::2])
    up = orc.budget_resample(b, 8, 12)
    assert np.array_equal(up, np.repeat(np.repeat(b, 2, axis=1), 2, axis=2))
    # agreement with an independent nearest-neighbour routine for an awkward ratio
    rng = np.random.default_rng(4)
    b = rng.integers(0, 33, size=(3, 7, 7)).astype(np.uint8)
    ref = torch.nn.functional.interpolate(torch.from_numpy(b.astype(np.float32))[:, None], size=(14, 28),
                                          mode="nearest")[:, 0].numpy()
    assert np.array_equal(orc.budget_resample(b, 14, 28).astype(np.float32), ref)
    ref = b[:, (np.arange(3) * 7) // 3][:, :, (np.arange(5) * 7) // 5]
    assert np.array_equal(orc.budget_resample(b, 3, 5), ref)
