"""Pins of the CPU oracle against facts it did not produce itself.

The paper prints no numeric example, so the pins are: hand-worked cases (tests/golden),
closed forms and special cases that follow from the definition in Section 2.1, the two
decompositions the paper itself states (a 1x1 filter needs no second stage, Section 3 last
paragraph; a convolution is the sum of R*S per-tap channel reductions, Section 3 and Fig. 4),
an explicit im2col + matrix product (Section 2.3.1), library routines, and operation counts
(Section 3: reuse of filter rows and of interior input rows).
"""
import glob
import os

import numpy as np
import pytest

import oracle
from paper_2103_16234_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(path):
    rec = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rec[key] = [float(v) for v in vals]
    N, C, H, W, K, R, S, ph, pw = (int(v) for v in rec["dims"])
    P, Q = H + 2 * ph - R + 1, W + 2 * pw - S + 1
    x = np.array(rec["x"], dtype=np.float32).reshape(N, C, H, W)
    w = np.array(rec["w"], dtype=np.float32).reshape(K, C, R, S)
    y = np.array(rec["y"], dtype=np.float64).reshape(N, K, P, Q)
    ya = np.array(rec["yabs"], dtype=np.float64).reshape(N, K, P, Q)
    return x, w, ph, pw, y, ya


def _plain_cases():
    return [p for p in sorted(glob.glob(os.path.join(GOLDEN, "*.txt"))) if not os.path.basename(p).startswith("bias_relu")]


def test_hand_worked_epilogue_case():
    """Bias and ReLU after the convolution (Section 2.1), against values worked by hand."""
    path = os.path.join(GOLDEN, "bias_relu_c2k2_1x2.txt")
    x, w, ph, pw, y, ya = _read_golden(path)
    rec = {}
    for line in open(path):
        if line.startswith(("bias", "relu")):
            key, *vals = line.split()
            rec[key] = [float(v) for v in vals]
    got, got_abs = oracle.conv_bias_relu_ref(x, w, np.array(rec["bias"], dtype=np.float32), ph, pw, bool(rec["relu"][0]))
    np.testing.assert_array_equal(got, y)
    np.testing.assert_array_equal(got_abs, ya)


def test_epilogue_properties_and_library_routine():
    torch = pytest.importorskip("torch")
    x, w = _rand((2, 5, 6, 7), 61), _rand((4, 5, 3, 3), 62)
    b = _rand((4,), 63)
    plain, plain_abs = oracle.conv_ref(x, w, 1, 1)
    y0, a0 = oracle.conv_bias_relu_ref(x, w, None, 1, 1, False)            # no bias, no ReLU: the convolution itself
    np.testing.assert_array_equal(y0, plain)
    np.testing.assert_array_equal(a0, plain_abs)
    yb, ab = oracle.conv_bias_relu_ref(x, w, b, 1, 1, False)
    np.testing.assert_array_equal(yb, plain + b.astype(np.float64).reshape(1, 4, 1, 1))   # bias lands on its own channel
    np.testing.assert_array_equal(ab, plain_abs + np.abs(b.astype(np.float64)).reshape(1, 4, 1, 1))
    yr, _ = oracle.conv_bias_relu_ref(x, w, b, 1, 1, True)
    assert (yr >= 0).all() and (yr[yb > 0] == yb[yb > 0]).all() and (yr[yb <= 0] == 0).all()
    assert (yb < 0).any() and (yb > 0).any()                                 # the case exercises both branches
    zero, _ = oracle.conv_bias_relu_ref(x, np.zeros_like(w), b, 1, 1, True)  # closed form: ReLU(bias) everywhere
    np.testing.assert_array_equal(zero, np.broadcast_to(np.maximum(b.astype(np.float64), 0).reshape(1, 4, 1, 1), zero.shape))
    t = torch.nn.functional.relu(torch.nn.functional.conv2d(
        torch.from_numpy(x).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double(), padding=1)).numpy()
    np.testing.assert_allclose(yr, t, rtol=0, atol=1e-12)


@pytest.mark.parametrize("path", _plain_cases(), ids=os.path.basename)
def test_hand_worked_cases(path):
    x, w, ph, pw, y, ya = _read_golden(path)
    for nthreads in (1, 3):
        got, got_abs = oracle.conv_ref(x, w, ph, pw, nthreads=nthreads)
        assert got.shape == y.shape
        np.testing.assert_array_equal(got, y)
        np.testing.assert_array_equal(got_abs, ya)


def _rand(shape, seed, dist="upm1"):
    n = int(np.prod(shape))
    if dist == "upm1":
        return inputs.uniform_pm1(seed, n).reshape(shape)
    return inputs.small_ints(seed, n, -4, 4).reshape(shape)


# ---- independent re-statements of the definition, written without reference to the C loops ----

def _im2col_matmul(x, w, ph, pw):
    """Section 2.3.1: explicit patch matrix [C*R*S, P*Q] per image, times the [K, C*R*S] filter matrix."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P, Q = H + 2 * ph - R + 1, W + 2 * pw - S + 1
    xp = np.zeros((N, C, H + 2 * ph, W + 2 * pw), dtype=np.float64)
    xp[:, :, ph:ph + H, pw:pw + W] = x
    wm = w.astype(np.float64).reshape(K, C * R * S)
    y = np.empty((N, K, P, Q))
    for n in range(N):
        cols = np.empty((C * R * S, P * Q))
        row = 0
        for c in range(C):
            for r in range(R):
                for s in range(S):
                    cols[row] = xp[n, c, r:r + P, s:s + Q].reshape(-1)
                    row += 1
        y[n] = (wm @ cols).reshape(K, P, Q)
    return y


def _tap_decomposition(x, w, ph, pw):
    """Section 3 / Fig. 4: stage 1 gives one channel-reduced matrix per filter tap, stage 2 adds them."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P, Q = H + 2 * ph - R + 1, W + 2 * pw - S + 1
    xp = np.zeros((N, C, H + 2 * ph, W + 2 * pw), dtype=np.float64)
    xp[:, :, ph:ph + H, pw:pw + W] = x
    y = np.zeros((N, K, P, Q))
    for r in range(R):
        for s in range(S):
            # temp[n,k,p,q] = sum_c w[k,c,r,s] * xpad[n,c,p+r,q+s]
            y += np.einsum("kc,ncpq->nkpq", w[:, :, r, s].astype(np.float64), xp[:, :, r:r + P, s:s + Q])
    return y


SHAPES = [
    # N, C, H, W, K, R, S, ph, pw
    (1, 1, 5, 5, 1, 3, 3, 1, 1),
    (2, 3, 6, 7, 4, 3, 3, 1, 1),
    (1, 4, 5, 4, 3, 5, 5, 2, 2),
    (2, 5, 4, 6, 2, 1, 1, 0, 0),
    (1, 2, 7, 5, 3, 3, 3, 0, 0),
    (1, 3, 4, 4, 2, 2, 3, 1, 0),
    (1, 2, 3, 3, 2, 3, 3, 3, 3),   # padding wider than the filter overlap: all-padding windows
    (2, 2, 5, 6, 3, 1, 1, 1, 2),   # 1x1 filter with padding: a zero frame around the output
    (1, 3, 6, 6, 2, 4, 2, 2, 1),   # even filter sizes
]


@pytest.mark.parametrize("dims", SHAPES)
def test_matches_im2col_matmul_and_tap_sum(dims):
    N, C, H, W, K, R, S, ph, pw = dims
    x = _rand((N, C, H, W), 11)
    w = _rand((K, C, R, S), 12)
    y, ya = oracle.conv_ref(x, w, ph, pw, nthreads=2)
    scale = np.maximum(ya, 1e-30)
    assert np.max(np.abs(y - _im2col_matmul(x, w, ph, pw)) / scale) < 1e-12
    assert np.max(np.abs(y - _tap_decomposition(x, w, ph, pw)) / scale) < 1e-12
    # yabs is the same convolution applied to |x| and |w|
    assert np.max(np.abs(ya - _im2col_matmul(np.abs(x), np.abs(w), ph, pw)) / scale) < 1e-12


@pytest.mark.parametrize("dims", SHAPES)
def test_matches_torch_conv2d_double(dims):
    """Library cross-check: torch's CPU conv2d in fp64 is cross-correlation with zero padding."""
    torch = pytest.importorskip("torch")
    N, C, H, W, K, R, S, ph, pw = dims
    x = _rand((N, C, H, W), 21)
    w = _rand((K, C, R, S), 22)
    y, ya = oracle.conv_ref(x, w, ph, pw)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     stride=1, padding=(ph, pw)).numpy()
    assert np.max(np.abs(y - ref) / np.maximum(ya, 1e-30)) < 1e-12


def test_matches_scipy_correlate2d_single_channel():
    """C = K = 1: the layer is scipy's 2-D cross-correlation (not convolve2d, which flips)."""
    sig = pytest.importorskip("scipy.signal")
    x = _rand((1, 1, 9, 8), 31)
    w = _rand((1, 1, 3, 5), 32)
    y_valid, _ = oracle.conv_ref(x, w, 0, 0)
    ref = sig.correlate2d(x[0, 0].astype(np.float64), w[0, 0].astype(np.float64), mode="valid")
    np.testing.assert_allclose(y_valid[0, 0], ref, rtol=0, atol=1e-13)
    y_same, _ = oracle.conv_ref(x, w, 1, 2)
    ref = sig.correlate2d(x[0, 0].astype(np.float64), w[0, 0].astype(np.float64), mode="same", boundary="fill")
    np.testing.assert_allclose(y_same[0, 0], ref, rtol=0, atol=1e-13)
    flipped = sig.convolve2d(x[0, 0].astype(np.float64), w[0, 0].astype(np.float64), mode="valid")
    assert np.max(np.abs(y_valid[0, 0] - flipped)) > 1e-3


def test_identity_1x1_reproduces_input_exactly():
    """K = C and w = delta(k, c): every output plane is the matching input plane, bit for bit."""
    x = _rand((3, 6, 5, 7), 41)
    w = np.eye(6, dtype=np.float32).reshape(6, 6, 1, 1)
    y, ya = oracle.conv_ref(x, w, 0, 0)
    np.testing.assert_array_equal(y.astype(np.float32), x)
    np.testing.assert_array_equal(ya.astype(np.float32), np.abs(x))
    # a permutation of the channels moves the planes accordingly (k picks channel perm[k])
    perm = np.array([2, 0, 5, 1, 4, 3])
    wp = np.zeros((6, 6, 1, 1), dtype=np.float32)
    wp[np.arange(6), perm] = 1
    yp, _ = oracle.conv_ref(x, wp, 0, 0)
    np.testing.assert_array_equal(yp.astype(np.float32), x[:, perm])


def test_1x1_is_a_matrix_product_per_image():
    """Section 3, last paragraph: with a 1x1 filter the output is W[K,C] @ X[C, H*W] for each image."""
    x = _rand((2, 7, 4, 5), 51)
    w = _rand((3, 7, 1, 1), 52)
    y, ya = oracle.conv_ref(x, w, 0, 0)
    for n in range(2):
        ref = w[:, :, 0, 0].astype(np.float64) @ x[n].astype(np.float64).reshape(7, 20)
        np.testing.assert_allclose(y[n].reshape(3, 20), ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("R,S,ph,pw", [(3, 3, 1, 1), (5, 5, 2, 2), (3, 5, 0, 2), (2, 2, 1, 1)])
def test_shifted_delta_filter_translates_the_input(R, S, ph, pw):
    """A filter holding a single 1 at (r0, s0) shifts the image by (r0 - pad_h, s0 - pad_w), zero filled."""
    H, W = 6, 7
    x = _rand((1, 1, H, W), 61)
    P, Q = H + 2 * ph - R + 1, W + 2 * pw - S + 1
    for r0 in range(R):
        for s0 in range(S):
            w = np.zeros((1, 1, R, S), dtype=np.float32)
            w[0, 0, r0, s0] = 1
            y, _ = oracle.conv_ref(x, w, ph, pw)
            ref = np.zeros((P, Q))
            for p in range(P):
                for q in range(Q):
                    h, v = p + r0 - ph, q + s0 - pw
                    if 0 <= h < H and 0 <= v < W:
                        ref[p, q] = x[0, 0, h, v]
            np.testing.assert_array_equal(y[0, 0], ref)


@pytest.mark.parametrize("R,S", [(1, 1), (3, 3), (5, 5), (3, 5)])
def test_all_ones_counts_in_bounds_taps(R, S):
    """x = 1, w = 1, 'same' padding: y[p,q] = C * (rows of the window inside the image) * (columns inside)."""
    C, H, W, K = 3, 6, 8, 2
    ph, pw = (R - 1) // 2, (S - 1) // 2
    x = np.ones((1, C, H, W), dtype=np.float32)
    w = np.ones((K, C, R, S), dtype=np.float32)
    y, ya = oracle.conv_ref(x, w, ph, pw)
    assert y.shape == (1, K, H, W)                     # "same" output size (Section 2.1)
    rows = np.array([min(p + R - ph, H) - max(p - ph, 0) for p in range(H)])
    cols = np.array([min(q + S - pw, W) - max(q - pw, 0) for q in range(W)])
    ref = C * np.outer(rows, cols)
    for k in range(K):
        np.testing.assert_array_equal(y[0, k], ref)
    assert y[0, 0, 0, 0] == C * ((R + 1) // 2) * ((S + 1) // 2)   # corner
    assert y[0, 0, H // 2, W // 2] == C * R * S                      # interior
    np.testing.assert_array_equal(y, ya)


def test_output_size_without_padding():
    """Section 3: an unpadded convolution yields (H - R + 1) x (W - S + 1) outputs."""
    x = _rand((1, 2, 9, 11), 71)
    w = _rand((3, 2, 3, 5), 72)
    y, _ = oracle.conv_ref(x, w, 0, 0)
    assert y.shape == (1, 3, 7, 7)
    with pytest.raises(ValueError):
        oracle.conv_ref(x[:, :, :2], w, 0, 0)          # filter taller than the padded input: empty output


def test_linearity_in_input_and_filter():
    x1, x2 = _rand((2, 3, 5, 5), 81), _rand((2, 3, 5, 5), 82)
    w1, w2 = _rand((4, 3, 3, 3), 83), _rand((4, 3, 3, 3), 84)
    a, b = np.float32(0.5), np.float32(-2.0)            # powers of two: a*x1 + b*x2 is exact per term
    y11, ya = oracle.conv_ref(x1, w1, 1, 1)
    y21, _ = oracle.conv_ref(x2, w1, 1, 1)
    y12, _ = oracle.conv_ref(x1, w2, 1, 1)
    xs = (a * x1.astype(np.float64) + b * x2.astype(np.float64)).astype(np.float32)
    ysum, _ = oracle.conv_ref(xs, w1, 1, 1)
    # the rounding of xs to fp32 is the only inexact step; bound it by one ulp of each input term
    tol = 2.0 ** -23 * 3.0 * ya.max()
    assert np.max(np.abs(ysum - (a * y11 + b * y21))) <= tol
    ws = (a * w1.astype(np.float64) + b * w2.astype(np.float64)).astype(np.float32)
    ywsum, _ = oracle.conv_ref(x1, ws, 1, 1)
    assert np.max(np.abs(ywsum - (a * y11 + b * y12))) <= tol
    # exact case: scaling by a power of two commutes with every rounding
    y2, _ = oracle.conv_ref(2 * x1, w1, 1, 1)
    np.testing.assert_array_equal(y2, 2 * y11)
    yz, yza = oracle.conv_ref(np.zeros_like(x1), w1, 1, 1)
    assert not yz.any() and not yza.any()               # no hidden bias


def test_integer_inputs_give_exact_integers():
    x = _rand((2, 5, 6, 6), 91, "int")
    w = _rand((3, 5, 3, 3), 92, "int")
    y, ya = oracle.conv_ref(x, w, 1, 1)
    ref = _im2col_matmul(x, w, 1, 1)
    np.testing.assert_array_equal(y, ref)
    assert np.all(y == np.round(y))


def test_operation_and_touch_counts():
    """Section 3: without padding every filter element is used P*Q times per image, an interior input
    element R*S times per filter, a corner element once; in total N*K*P*Q*C*R*S multiply-adds."""
    N, C, H, W, K, R, S = 2, 3, 7, 8, 4, 3, 3
    x = _rand((N, C, H, W), 101)
    w = _rand((K, C, R, S), 102)
    y, xt, wt, macs = oracle.conv_ref_counted(x, w, 0, 0)
    P, Q = H - R + 1, W - S + 1
    assert macs == N * K * P * Q * C * R * S
    assert np.all(wt == N * P * Q)
    assert np.all(xt[:, :, R - 1:H - R + 1, S - 1:W - S + 1] == K * R * S)
    assert np.all(xt[:, :, 0, 0] == K) and np.all(xt[:, :, -1, -1] == K)
    assert xt.sum() == macs and wt.sum() == macs
    y2, _ = oracle.conv_ref(x, w, 0, 0)
    np.testing.assert_array_equal(y, y2)
    # with "same" padding the border windows lose their out-of-image taps
    _, xt, wt, macs = oracle.conv_ref_counted(x, w, 1, 1)
    rows = np.array([min(p + 2, H) - max(p - 1, 0) for p in range(H)])
    cols = np.array([min(q + 2, W) - max(q - 1, 0) for q in range(W)])
    assert macs == N * K * C * rows.sum() * cols.sum()
    # an input element (h, v) meets tap r of the output row p = h + pad - r, if that row exists
    rin = np.array([sum(0 <= h + 1 - r < H for r in range(R)) for h in range(H)])
    cin = np.array([sum(0 <= v + 1 - s < W for s in range(S)) for v in range(W)])
    assert np.all(xt == K * np.outer(rin, cin))
    assert xt[0, 0, 0, 0] == K * 4 and xt[0, 0, 3, 3] == K * R * S
    assert wt[0, 0, 1, 1] == N * H * W and wt[0, 0, 0, 0] == N * (H - 1) * (W - 1)


def test_points_equal_full_run():
    shape = inputs.ConvShape("t", 2, 5, 6, 7, 4, 3, 3, 1, 1, "u01", "he", 5, 6)
    x, w = inputs.make_inputs(shape)
    y, ya = oracle.conv_ref(x, w, 1, 1)
    rng = np.random.default_rng(0)
    coords = np.stack([rng.integers(0, d, 50) for d in y.shape], axis=1)
    yp, yap = oracle.conv_ref_points(x, w, 1, 1, coords)
    np.testing.assert_array_equal(yp, y[tuple(coords.T)])
    np.testing.assert_array_equal(yap, ya[tuple(coords.T)])
    with pytest.raises(ValueError):
        oracle.conv_ref_points(x, w, 1, 1, [[0, 0, 6, 0]])


def test_thread_count_does_not_change_results():
    shape = inputs.ConvShape("t", 3, 4, 5, 5, 5, 3, 3, 1, 1, "u01", "he", 7, 8)
    x, w = inputs.make_inputs(shape)
    y1, a1 = oracle.conv_ref(x, w, 1, 1, nthreads=1)
    for t in (2, 7, 64):
        yt, at = oracle.conv_ref(x, w, 1, 1, nthreads=t)
        np.testing.assert_array_equal(y1, yt)
        np.testing.assert_array_equal(a1, at)


def test_tolerance_rule():
    y = np.array([1.0, 2.0, 0.0])
    ya = np.array([10.0, 20.0, 0.0])
    ok, worst = oracle.within_tolerance(y + np.array([1e-4, 0, 5e-7]), y, ya)
    assert ok and worst <= 1.0
    ok, _ = oracle.within_tolerance(y + np.array([1.2e-4, 0, 0]), y, ya)
    assert not ok
    ok, _ = oracle.within_tolerance(y + np.array([0, 0, 2e-6]), y, ya)
    assert not ok
