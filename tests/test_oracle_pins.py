"""Pins for the CPU oracle: what the mathematics fixes, independent of the oracle's code.

The paper (section 3; Figure 1's caption for the parameter tuple) prints no
formula or worked example, so the oracle is pinned by closed forms, worked
examples derived by hand, exact invariants, reductions to textbook routines
and a brute-force im2col + naive matmul written with its own index code.
None of these tests touches the GPU library.
"""
import itertools
import os

import numpy as np
import pytest

from paper_1904_04174_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
PADS = {"VALID": wl.PAD_VALID, "SAME": wl.PAD_SAME}


def _golden_lines(name):
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                yield line.split()


# ---------------------------------------------------------------- geometry

@pytest.mark.parametrize("h,win,stride,pad,expect", [
    # (out, pad_before, pad_after), worked by hand from the SAME/VALID rules
    (224, 7, 2, "SAME", (112, 2, 3)),
    (56, 3, 2, "SAME", (28, 0, 1)),
    (28, 1, 2, "SAME", (14, 0, 0)),
    (56, 3, 1, "SAME", (56, 1, 1)),
    (56, 3, 1, "VALID", (54, 0, 0)),
    (56, 3, 2, "VALID", (27, 0, 0)),
    (8, 3, 1, "SAME", (8, 1, 1)),
    (5, 2, 1, "SAME", (5, 0, 1)),      # even window: the single pad goes after
    (2, 5, 1, "SAME", (2, 2, 2)),      # window larger than the image is fine under SAME
    (7, 2, 3, "SAME", (3, 0, 1)),      # stride > window: (3-1)*3+2-7 = 1 -> pads 0/1
    (10, 3, 4, "VALID", (2, 0, 0)),
])
def test_geometry_values(oracle, h, win, stride, pad, expect):
    g = oracle.geometry(h, h, win, win, stride, stride, PADS[pad])
    assert (g[0], g[2], g[3]) == expect
    assert (g[1], g[4], g[5]) == expect


def test_geometry_rows_and_cols_are_independent(oracle):
    g = oracle.geometry(224, 56, 7, 3, 2, 1, wl.PAD_SAME)
    assert g == (112, 56, 2, 3, 1, 1)


def test_geometry_rejects(oracle):
    with pytest.raises(ValueError):
        oracle.geometry(2, 8, 3, 3, 1, 1, wl.PAD_VALID)   # window taller than image
    with pytest.raises(ValueError):
        oracle.geometry(8, 8, 3, 3, 0, 1, wl.PAD_SAME)    # zero stride
    with pytest.raises(ValueError):
        oracle.geometry(8, 8, 3, 3, 1, 1, 7)              # unknown padding mode


# ------------------------------------------------------------ golden values

def test_handworked_4x4(oracle):
    x = np.arange(16, dtype=np.float32).reshape(1, 4, 4, 1)
    f = np.arange(1, 10, dtype=np.float32).reshape(3, 3, 1, 1)
    count = 0
    for tok in _golden_lines("handworked_4x4.txt"):
        stride, pad, p, q = int(tok[0]), PADS[tok[1]], int(tok[2]), int(tok[3])
        want = np.array([float(v) for v in tok[4:]], dtype=np.float64).reshape(1, p, q, 1)
        got32 = oracle.forward_f32(x, f, stride, pad)
        got64 = oracle.forward_f64(x, f, stride, pad)
        assert got32.shape == want.shape
        assert np.array_equal(got32.astype(np.float64), want)
        assert np.array_equal(got64, want)
        count += 1
    assert count == 4


def test_allones_golden(oracle):
    count = 0
    for tok in _golden_lines("allones_counts.txt"):
        h, w, c, r, s, stride = (int(v) for v in tok[:6])
        pad, p, q = PADS[tok[6]], int(tok[7]), int(tok[8])
        want = np.array([float(v) for v in tok[9:]]).reshape(p, q)
        k = 3
        x = np.ones((2, h, w, c), np.float32)
        f = np.ones((r, s, c, k), np.float32)
        got = oracle.forward_f32(x, f, stride, pad)
        assert got.shape == (2, p, q, k)
        for n, kk in itertools.product(range(2), range(k)):
            assert np.array_equal(got[n, :, :, kk].astype(np.float64), want)
        count += 1
    assert count == 3


def _valid_tap_counts(extent, window, stride, out_extent, pad_before):
    """#taps inside the image for each output position, by counting."""
    return np.array([sum(1 for t in range(window) if 0 <= o * stride + t - pad_before < extent)
                     for o in range(out_extent)], dtype=np.float64)


@pytest.mark.parametrize("h,w,r,s,sr,sc,pad", [
    (9, 7, 3, 3, 1, 1, "SAME"), (9, 7, 3, 5, 2, 1, "SAME"), (10, 11, 7, 7, 2, 2, "SAME"),
    (6, 6, 2, 2, 1, 1, "SAME"), (9, 9, 3, 3, 2, 2, "VALID"), (3, 4, 5, 7, 1, 1, "SAME"),
    (12, 5, 1, 1, 2, 3, "SAME"), (8, 8, 4, 2, 3, 1, "SAME"),
])
def test_allones_closed_form(oracle, h, w, r, s, sr, sc, pad):
    c, k = 5, 2
    p, q, pt, _, pl, _ = oracle.geometry(h, w, r, s, sr, sc, PADS[pad])
    want = c * np.outer(_valid_tap_counts(h, r, sr, p, pt), _valid_tap_counts(w, s, sc, q, pl))
    got = oracle.forward_f32(np.ones((1, h, w, c), np.float32), np.ones((r, s, c, k), np.float32),
                             (sr, sc), PADS[pad])
    for kk in range(k):
        assert np.array_equal(got[0, :, :, kk].astype(np.float64), want)


# ---------------------------------------------------- exact structural pins

def test_identity_1x1(oracle):
    x, _ = wl.make_case((2, 7, 9, 6), (1, 1, 6, 6), "uniform", 11)
    f = np.eye(6, dtype=np.float32).reshape(1, 1, 6, 6)
    assert np.array_equal(oracle.forward_f32(x, f, 1, wl.PAD_SAME), x)
    assert np.array_equal(oracle.forward_f32(x, f, 1, wl.PAD_VALID), x)
    got = oracle.forward_f32(x, f, (2, 3), wl.PAD_SAME)
    assert np.array_equal(got, x[:, ::2, ::3, :])


def test_channel_permutation_1x1(oracle):
    # f[0,0,c,k] = 1 iff c == perm[k]: picks channel perm[k]; catches a C/K transpose.
    x, _ = wl.make_case((1, 5, 4, 4), (1, 1, 4, 4), "uniform", 12)
    perm = [2, 0, 3, 1]
    f = np.zeros((1, 1, 4, 4), np.float32)
    for k, c in enumerate(perm):
        f[0, 0, c, k] = 1.0
    assert np.array_equal(oracle.forward_f32(x, f, 1, wl.PAD_SAME), x[..., perm])


@pytest.mark.parametrize("r0,s0", [(0, 0), (0, 2), (1, 1), (2, 0), (2, 1)])
def test_delta_filter_is_a_shift(oracle, r0, s0):
    x, _ = wl.make_case((2, 6, 7, 3), (3, 3, 3, 3), "uniform", 13)
    f = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        f[r0, s0, c, c] = 1.0
    got = oracle.forward_f32(x, f, 1, wl.PAD_SAME)        # pads 1/1
    want = np.zeros_like(x)
    dy, dx = r0 - 1, s0 - 1
    for p in range(6):
        for q in range(7):
            if 0 <= p + dy < 6 and 0 <= q + dx < 7:
                want[:, p, q, :] = x[:, p + dy, q + dx, :]
    assert np.array_equal(got, want)


def test_filter_is_not_flipped(oracle):
    # A single 1 in the image: the output is the filter mirrored (correlation), not the filter.
    x = np.zeros((1, 5, 5, 1), np.float32)
    x[0, 2, 2, 0] = 1.0
    f = np.arange(1, 10, dtype=np.float32).reshape(3, 3, 1, 1)
    got = oracle.forward_f32(x, f, 1, wl.PAD_SAME)[0, 1:4, 1:4, 0]
    assert np.array_equal(got, f[::-1, ::-1, 0, 0])


def test_linearity(oracle):
    x, f = wl.make_case((2, 6, 5, 3), (3, 2, 3, 4), "uniform", 14)
    y, g = wl.make_case((2, 6, 5, 3), (3, 2, 3, 4), "normal", 15)
    x, y, f, g = (a.astype(np.float64) for a in (x, y, f, g))
    conv = lambda a, b: oracle.forward_f64(a, b, (2, 1), wl.PAD_SAME)
    # power-of-two coefficients: exact
    assert np.array_equal(conv(4.0 * x, f), 4.0 * conv(x, f))
    assert np.array_equal(conv(x, 0.5 * f), 0.5 * conv(x, f))
    lhs = conv(2.0 * x - 3.0 * y, f)
    rhs = 2.0 * conv(x, f) - 3.0 * conv(y, f)
    assert np.max(np.abs(lhs - rhs)) <= 1e-12 * (1 + np.max(np.abs(rhs)))
    lhs = conv(x, f + 0.25 * g)
    rhs = conv(x, f) + 0.25 * conv(x, g)
    assert np.max(np.abs(lhs - rhs)) <= 1e-12 * (1 + np.max(np.abs(rhs)))


@pytest.mark.parametrize("stride,dy,dx", [(1, 1, 2), (1, -2, 1), (2, 2, -2)])
def test_translation_equivariance_interior(oracle, stride, dy, dx):
    x, f = wl.make_case((1, 16, 16, 2), (3, 3, 2, 3), "uniform", 16)
    big = np.zeros((1, 24, 24, 2), np.float32)
    big[:, 4:20, 4:20, :] = x
    shifted = np.zeros_like(big)
    shifted[:, 4 + dy:20 + dy, 4 + dx:20 + dx, :] = x
    a = oracle.forward_f32(big, f, stride, wl.PAD_VALID)
    b = oracle.forward_f32(shifted, f, stride, wl.PAD_VALID)
    oy, ox = dy // stride, dx // stride
    p = a.shape[1]
    lo, hi = 2, p - 2
    assert np.array_equal(b[:, lo + oy:hi + oy, lo + ox:hi + ox, :], a[:, lo:hi, lo:hi, :])
    assert np.any(a[:, lo:hi, lo:hi, :] != 0)


def test_1x1_is_a_matmul(oracle):
    x, f = wl.make_case((3, 5, 4, 7), (1, 1, 7, 6), "uniform", 17)
    x64, f64 = x.astype(np.float64), f.astype(np.float64)
    want = np.zeros((3 * 5 * 4, 6))
    a, b = x64.reshape(-1, 7), f64.reshape(7, 6)
    for i in range(a.shape[0]):
        for j in range(6):
            acc = 0.0
            for c in range(7):
                acc += a[i, c] * b[c, j]
            want[i, j] = acc
    got = oracle.forward_f64(x64, f64, 1, wl.PAD_VALID).reshape(-1, 6)
    assert np.array_equal(got, want)


def test_full_window_valid_is_a_dot_product(oracle):
    x, f = wl.make_case((2, 4, 5, 3), (4, 5, 3, 2), "uniform", 18)
    got = oracle.forward_f64(x.astype(np.float64), f.astype(np.float64), 1, wl.PAD_VALID)
    assert got.shape == (2, 1, 1, 2)
    for n in range(2):
        for k in range(2):
            want = np.dot(x[n].astype(np.float64).ravel(), f[..., k].astype(np.float64).ravel())
            assert abs(got[n, 0, 0, k] - want) <= 1e-13 * (1 + abs(want))


# ------------------------------------------------ brute force: im2col + matmul

def _im2col_reference(x, f, sr, sc, pad):
    """Independent definition: build the [M x RSC] patch matrix explicitly
    (its own padding arithmetic, by placing the image in a zero canvas) and
    multiply by the [RSC x K] filter matrix with a naive loop nest, fp64."""
    n, h, w, c = x.shape
    r, s, _, k = f.shape
    if pad == wl.PAD_VALID:
        p, q = -(-(h - r + 1) // sr), -(-(w - s + 1) // sc)
        top = left = 0
    else:
        p, q = -(-h // sr), -(-w // sc)
        need_r = max((p - 1) * sr + r - h, 0)
        need_c = max((q - 1) * sc + s - w, 0)
        top, left = need_r // 2, need_c // 2
    canvas = np.zeros((n, top + h + r + sr, left + w + s + sc, c))
    canvas[:, top:top + h, left:left + w, :] = x
    cols = np.zeros((n * p * q, r * s * c))
    row = 0
    for b in range(n):
        for i in range(p):
            for j in range(q):
                cols[row] = canvas[b, i * sr:i * sr + r, j * sc:j * sc + s, :].ravel()
                row += 1
    fm = f.astype(np.float64).reshape(r * s * c, k)
    out = np.zeros((cols.shape[0], k))
    for i in range(cols.shape[0]):
        for j in range(k):
            acc = 0.0
            for t in range(cols.shape[1]):
                acc += cols[i, t] * fm[t, j]
            out[i, j] = acc
    return out.reshape(n, p, q, k)


_BRUTE = []
_rs = np.random.default_rng(2024)
for _i in range(28):
    _r, _s = (int(v) for v in _rs.choice([1, 2, 3, 5, 7], 2))
    _sr, _sc = (int(v) for v in _rs.choice([1, 2, 3], 2))
    _h, _w = int(_rs.integers(1, 10)), int(_rs.integers(1, 10))
    _c, _k = (int(v) for v in _rs.choice([1, 3, 4, 5], 2))
    _pad = wl.PAD_SAME if _i % 2 == 0 else wl.PAD_VALID
    if _pad == wl.PAD_VALID and (_r > _h or _s > _w):
        _h, _w = _h + _r, _w + _s
    _BRUTE.append((int(_rs.integers(1, 3)), _h, _w, _c, _k, _r, _s, _sr, _sc, _pad))


@pytest.mark.parametrize("case", _BRUTE)
def test_against_im2col_bruteforce(oracle, case):
    n, h, w, c, k, r, s, sr, sc, pad = case
    x, f = wl.make_case((n, h, w, c), (r, s, c, k), "uniform", 1000 + sum(case))
    want = _im2col_reference(x.astype(np.float64), f, sr, sc, pad)
    got64 = oracle.forward_f64(x.astype(np.float64), f.astype(np.float64), (sr, sc), pad)
    assert got64.shape == want.shape
    assert np.max(np.abs(got64 - want)) <= 1e-12 * (1 + np.max(np.abs(want)))
    got32 = oracle.forward_f32(x, f, (sr, sc), pad)
    assert np.array_equal(got32, want.astype(np.float32)) or \
        np.max(np.abs(got32 - want)) <= 2e-7 * (1 + np.max(np.abs(want)))
    idx = np.arange(want.size)
    pts = oracle.points_f32(x, f, idx, (sr, sc), pad)
    assert np.max(np.abs(pts - want.ravel())) <= 1e-12 * (1 + np.max(np.abs(want)))


def test_integer_inputs_are_exact(oracle):
    # integers in [-4,4]: every summation order gives the same exactly representable result
    x, f = wl.make_case((2, 9, 8, 16), (3, 3, 16, 8), "ints", 19)
    got = oracle.forward_f32(x, f, 1, wl.PAD_SAME)
    want = _im2col_reference(x.astype(np.float64), f, 1, 1, wl.PAD_SAME)
    assert np.array_equal(got.astype(np.float64), want)


def test_threads_do_not_change_the_result(oracle):
    x, f = wl.make_case((3, 9, 9, 5), (3, 3, 5, 7), "normal", 20)
    a = oracle.forward_f32(x, f, 1, wl.PAD_SAME, num_threads=1)
    b = oracle.forward_f32(x, f, 1, wl.PAD_SAME, num_threads=4)
    assert np.array_equal(a, b)


def test_empty_batch(oracle):
    x = np.zeros((0, 5, 5, 2), np.float32)
    f = np.ones((3, 3, 2, 4), np.float32)
    assert oracle.forward_f32(x, f, 1, wl.PAD_SAME).shape == (0, 5, 5, 4)


# --------------------------------------------------------- input generators

def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.0e38, 0.0],
                 np.float32)
    widened, bits = wl.round_to_bf16(x)
    # 1+2^-8 is a tie between 1 and 1+2^-7 -> even mantissa (1.0); 1+3*2^-8 ties up to 1+2^-6
    assert widened[0] == 1.0 and widened[1] == 1.0 and widened[2] == np.float32(1.0 + 2 ** -7)
    assert widened[3] == np.float32(1.0 + 2 ** -6)
    assert bits[0] == 0x3F80 and bits[6] == 0
    assert abs(widened[4] + 0.3) <= 0.3 * 2 ** -8
    again, _ = wl.round_to_bf16(widened)
    assert np.array_equal(again, widened)


def test_generators_are_seeded():
    layer = wl.LAYERS["T1"]
    a = wl.make_inputs(layer)
    b = wl.make_inputs(layer)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert a[0].shape == (1, 8, 8, 4) and a[1].shape == (3, 3, 4, 4)
    assert np.all(np.abs(a[0]) <= 1.0)
    ints = wl.make_inputs(layer, dist="ints")[0]
    assert np.array_equal(ints, np.round(ints)) and ints.min() >= -4 and ints.max() <= 4


# ------------------------------------------------------------------ fused bias + activation

def test_bias_act_hand_example(oracle):
    # 1x1 window, one channel, weight 2: out = max(2*x + bias, 0)
    x = np.array([-1.0, 3.0, 0.25, -0.5], np.float32).reshape(1, 2, 2, 1)
    f = np.array([2.0], np.float32).reshape(1, 1, 1, 1)
    b = np.array([-1.0], np.float32)
    got = oracle.forward_bias_act_f32(x, f, b, relu=True)
    assert got.reshape(-1).tolist() == [0.0, 5.0, 0.0, 0.0]
    got = oracle.forward_bias_act_f32(x, f, b, relu=False)
    assert got.reshape(-1).tolist() == [-3.0, 5.0, -0.5, -2.0]


def test_bias_act_reduces_to_the_plain_convolution(oracle):
    x, f = wl.make_case((2, 7, 6, 5), (3, 3, 5, 4), "uniform", 31)
    plain = oracle.forward_f32(x, f, 1, wl.PAD_SAME)
    assert np.array_equal(oracle.forward_bias_act_f32(x, f, None, False, 1, wl.PAD_SAME), plain)
    zero = np.zeros(4, np.float32)
    assert np.array_equal(oracle.forward_bias_act_f32(x, f, zero, False, 1, wl.PAD_SAME), plain)


def test_bias_act_zero_filter_broadcasts_the_bias(oracle):
    x, f = wl.make_case((1, 5, 5, 3), (3, 3, 3, 6), "uniform", 32)
    b = np.array([-2.0, -0.5, 0.0, 0.5, 1.0, 3.0], np.float32)
    got = oracle.forward_bias_act_f32(x, np.zeros_like(f), b, True, 2, wl.PAD_SAME)
    assert got.shape == (1, 3, 3, 6)
    assert np.array_equal(got, np.broadcast_to(np.maximum(b, 0), got.shape))


def test_bias_act_against_brute_force(oracle):
    rng = np.random.default_rng(33)
    x = rng.integers(-3, 4, (1, 4, 5, 2)).astype(np.float32)
    f = rng.integers(-3, 4, (2, 3, 2, 3)).astype(np.float32)
    b = rng.integers(-5, 6, 3).astype(np.float32)
    got = oracle.forward_bias_act_f32(x, f, b, True, 1, wl.PAD_VALID)
    want = np.zeros((1, 3, 3, 3))
    for p in range(3):
        for q in range(3):
            for k in range(3):
                acc = float(b[k])
                for r in range(2):
                    for s in range(3):
                        for c in range(2):
                            acc += float(x[0, p + r, q + s, c]) * float(f[r, s, c, k])
                want[0, p, q, k] = max(acc, 0.0)
    assert np.array_equal(got, want.astype(np.float32))


# ------------------------------------------------------------------ fused 2x2 max pooling

def test_pool_hand_example(oracle):
    # the worked 4x4 example above (input 0..15, filter 1..9, stride 1, SAME) gives
    # [[83,139,178,121],[198,303,348,225],[330,483,528,333],[181,253,274,163]]:
    # its 2x2 windows have the maxima 303, 348 / 483, 528
    x = np.arange(16, dtype=np.float32).reshape(1, 4, 4, 1)
    f = np.arange(1, 10, dtype=np.float32).reshape(3, 3, 1, 1)
    got = oracle.forward_bias_act_pool_f32(x, f, None, False, 1, wl.PAD_SAME)
    assert got.reshape(2, 2).tolist() == [[303.0, 348.0], [483.0, 528.0]]
    # a bias of -400 and the ReLU zero the first row of windows
    got = oracle.forward_bias_act_pool_f32(x, f, np.array([-400.0], np.float32), True, 1,
                                           wl.PAD_SAME)
    assert got.reshape(2, 2).tolist() == [[0.0, 0.0], [83.0, 128.0]]


def test_pool_drops_a_trailing_odd_row_and_column(oracle):
    y = np.arange(2 * 5 * 7 * 3, dtype=np.float64).reshape(2, 5, 7, 3)
    got = oracle.max_pool_2x2(y)
    assert got.shape == (2, 2, 3, 3)
    # values grow along every axis: the maximum of a window is its bottom-right element
    assert np.array_equal(got, y[:, 1:4:2, 1:6:2, :])
    assert oracle.max_pool_2x2(np.zeros((1, 1, 4, 2))).shape == (1, 0, 2, 2)


def test_pool_against_explicit_windows(oracle):
    rng = np.random.default_rng(41)
    x = rng.integers(-3, 4, (2, 7, 6, 3)).astype(np.float32)
    f = rng.integers(-3, 4, (3, 3, 3, 4)).astype(np.float32)
    b = rng.integers(-5, 6, 4).astype(np.float32)
    full = oracle.forward_bias_act_f32(x, f, b, True, 1, wl.PAD_SAME)      # 2 x 7 x 6 x 4
    got = oracle.forward_bias_act_pool_f32(x, f, b, True, 1, wl.PAD_SAME)  # 2 x 3 x 3 x 4
    assert got.shape == (2, 3, 3, 4)
    for n in range(2):
        for i in range(3):
            for j in range(3):
                for k in range(4):
                    window = [full[n, 2 * i + a, 2 * j + c, k] for a in (0, 1) for c in (0, 1)]
                    assert got[n, i, j, k] == max(window)


def test_pool_of_all_ones_closed_form(oracle):
    # all-ones input and filter: the unpooled output counts the taps inside the image, so every
    # 2x2 window of an 8x8 image holds an interior pixel (9 taps x 2 channels = 18) except none:
    # corners of the pooled map see the pixels (1,1) etc., which are interior as well
    x = np.ones((1, 8, 8, 2), np.float32)
    f = np.ones((3, 3, 2, 3), np.float32)
    got = oracle.forward_bias_act_pool_f32(x, f, None, False, 1, wl.PAD_SAME)
    assert got.shape == (1, 4, 4, 3) and np.all(got == 18.0)
    # 2x2 image: every output pixel sees 4 taps x 2 channels
    got = oracle.forward_bias_act_pool_f32(np.ones((1, 2, 2, 2), np.float32), f, None, False, 1,
                                           wl.PAD_SAME)
    assert got.shape == (1, 1, 1, 3) and np.all(got == 8.0)
