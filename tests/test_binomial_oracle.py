"""CPU pins of the binomial-filter oracle (no GPU needed)."""
from __future__ import annotations

import os

import numpy as np
import pytest

import oracle
from paper_2002_02268_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "binomial_3x3.txt")


def oracle_bf(img):
    return oracle.binomial3x3_f32(img)


def separated_reference(img):
    """The separated form (vertical 1-2-1, then horizontal 1-2-1, /16) through numpy's edge padding."""
    p = np.pad(img.astype(np.float64), 1, mode="edge")
    v = p[:-2, :] + 2.0 * p[1:-1, :] + p[2:, :]
    return (v[:, :-2] + 2.0 * v[:, 1:-1] + v[:, 2:]) / 16.0


def pin_golden(bf):
    lines = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert lines[0][0] == "image"
    H, W = int(lines[0][1]), int(lines[0][2])
    img = np.array(lines[1:1 + H], dtype=np.float32)
    want = np.array(lines[2 + H:2 + 2 * H], dtype=np.float64)
    assert img.shape == (H, W)
    assert np.array_equal(bf(img), want)


def pin_constant(bf):
    for shape in [(1, 1), (1, 7), (6, 1), (5, 9)]:
        assert np.array_equal(bf(np.full(shape, 3.25, np.float32)), np.full(shape, 3.25))


def pin_linear_interior(bf):
    """The weights are symmetric and sum to 16: a linear ramp is reproduced away from the edges."""
    y, x = np.mgrid[0:9, 0:11]
    img = (3 * x - 2 * y + 5).astype(np.float32)
    assert np.array_equal(bf(img)[1:-1, 1:-1], img[1:-1, 1:-1].astype(np.float64))


def pin_impulse(bf):
    img = np.zeros((7, 8), np.float32)
    img[3, 4] = 16.0
    want = np.zeros((7, 8))
    want[2:5, 3:6] = [[1, 2, 1], [2, 4, 2], [1, 2, 1]]
    assert np.array_equal(bf(img), want)
    # a corner impulse is seen through the repeated edge: taps that fall outside fold back onto it
    img = np.zeros((5, 6), np.float32)
    img[0, 0] = 16.0
    want = np.zeros((5, 6))
    want[0, 0], want[0, 1], want[1, 0], want[1, 1] = 9, 3, 3, 1
    assert np.array_equal(bf(img), want)


def pin_separable(bf):
    for shape, seed in [((13, 17), 1), ((1, 9), 2), ((8, 1), 3), ((40, 33), 4)]:
        img = synth.uniform(shape, 500 + seed, synth.TENSOR_A)
        assert np.max(np.abs(bf(img) - separated_reference(img))) <= 1e-15


def pin_integer_exact(bf):
    img = synth.small_ints((21, 19), 510, synth.TENSOR_A, -8, 8)
    p = np.pad(img.astype(np.int64), 1, mode="edge")
    acc = np.zeros((21, 19), np.int64)
    w = [[1, 2, 1], [2, 4, 2], [1, 2, 1]]
    for dy in range(3):
        for dx in range(3):
            acc += w[dy][dx] * p[dy:dy + 21, dx:dx + 19]
    assert np.array_equal(bf(img), acc / 16.0)


def pin_transpose(bf):
    img = synth.uniform((12, 15), 520, synth.TENSOR_A)
    assert np.allclose(bf(np.ascontiguousarray(img.T)), bf(img).T, rtol=0, atol=1e-15)


def pin_strided(bf):
    img = synth.uniform((9, 10), 530, synth.TENSOR_A)
    buf = np.full((9, 15), np.nan, np.float32)
    buf[:, :10] = img
    assert np.array_equal(bf(buf[:, :10]), bf(img))


ALL_PINS = [pin_golden, pin_constant, pin_linear_interior, pin_impulse, pin_separable, pin_integer_exact,
            pin_transpose, pin_strided]


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda p: p.__name__)
def test_binomial_oracle_pin(pin):
    pin(oracle_bf)


def _pad_then(img, mode, weights, scale):
    p = np.pad(img.astype(np.float64), 1, mode=mode)
    H, W = img.shape
    acc = np.zeros((H, W))
    for dy in range(3):
        for dx in range(3):
            acc += weights[dy][dx] * p[dy:dy + H, dx:dx + W]
    return acc * scale


W2D = [[1, 2, 1], [2, 4, 2], [1, 2, 1]]
MUTANTS = {
    "zero_padding": lambda img: _pad_then(img, "constant", W2D, 1 / 16),
    "reflect_padding": lambda img: _pad_then(img, "reflect", W2D, 1 / 16) if min(img.shape) > 1 else _pad_then(img, "constant", W2D, 1 / 16),
    "box_weights": lambda img: _pad_then(img, "edge", [[1, 1, 1], [1, 8, 1], [1, 1, 1]], 1 / 16),
    "centre_weight_2": lambda img: _pad_then(img, "edge", [[1, 2, 1], [2, 2, 2], [1, 2, 1]], 1 / 16),
    "missing_scale": lambda img: _pad_then(img, "edge", W2D, 1.0),
    "asymmetric": lambda img: _pad_then(img, "edge", [[1, 2, 1], [2, 4, 2], [2, 1, 1]], 1 / 16),
    "shifted": lambda img: np.roll(_pad_then(img, "edge", W2D, 1 / 16), 1, axis=1),
    "fp32_input_order": lambda img: _pad_then(img, "edge", W2D, 1 / 16).astype(np.float32).astype(np.float64) + 1e-7,
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_binomial_pins_have_teeth(name):
    tripped = []
    for pin in ALL_PINS:
        try:
            pin(MUTANTS[name])
        except AssertionError:
            tripped.append(pin.__name__)
    assert tripped, f"mutant {name} passes every pin"


def test_binomial_oracle_rejects_bad_strides():
    lib = oracle._load()
    img = np.zeros((4, 4), np.float32)
    out = np.zeros((4, 4))
    f = lambda ldi, ldo: lib.oracle_binomial3x3_f32(4, 4, img.ctypes.data_as(oracle._fp), ldi,  # noqa: E731
                                                     out.ctypes.data_as(oracle._dp), ldo)
    assert f(4, 4) == 0 and f(3, 4) == -1 and f(4, 3) == -1
