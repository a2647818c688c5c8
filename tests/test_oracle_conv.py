"""Pins for the oracle's convolution, BN folding, pooling and FC.

Each test checks the oracle against something other than itself: literal values
worked by hand, closed forms, textbook identities, or an independent library
routine (torch CPU in float64).
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2207_01260_amd import synth


def nmax(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


X44 = np.arange(1, 17, dtype=np.float32).reshape(1, 1, 4, 4)
W33 = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 3, 3)


def test_hand_3x3_on_4x4_no_pad(orc):
    # cross-correlation, worked by hand; the flipped-kernel answer would be 192 at [0][0]
    z = orc.conv2d_f64(X44, W33, 1, 0)
    assert z.shape == (1, 1, 2, 2)
    assert z.ravel().tolist() == [348.0, 393.0, 528.0, 573.0]


def test_hand_3x3_on_4x4_pad1_corners(orc):
    z = orc.conv2d_f64(X44, W33, 1, 1)
    assert z.shape == (1, 1, 4, 4)
    # top-left: 1*5 + 2*6 + 5*8 + 6*9
    assert z[0, 0, 0, 0] == 111.0
    # bottom-right: 11*1 + 12*2 + 15*4 + 16*5
    assert z[0, 0, 3, 3] == 11 + 24 + 60 + 80
    # interior (1,1) equals the no-pad value at (0,0)
    assert z[0, 0, 1, 1] == 348.0 and z[0, 0, 2, 2] == 573.0


def test_hand_two_in_two_out(orc):
    # x: channel 0 all ones, channel 1 = column index; 2x2 kernels, no pad
    x = np.zeros((1, 2, 2, 3), np.float32)
    x[0, 0] = 1.0
    x[0, 1] = np.array([[0, 1, 2], [0, 1, 2]], np.float32)
    w = np.zeros((2, 2, 2, 2), np.float32)
    w[0, 0] = [[1, 1], [1, 1]]       # sums channel 0 -> 4
    w[0, 1] = [[0, 1], [0, 0]]       # picks x1[y][x+1]
    w[1, 0] = [[0, 0], [0, 0]]
    w[1, 1] = [[-1, 0], [0, 2]]      # -x1[y][x] + 2 x1[y+1][x+1]
    z = orc.conv2d_f64(x, w, 1, 0)
    assert z.shape == (1, 2, 1, 2)
    assert z[0, 0].ravel().tolist() == [4 + 1, 4 + 2]
    assert z[0, 1].ravel().tolist() == [-0 + 2 * 1, -1 + 2 * 2]


@pytest.mark.parametrize("c_in", [1, 5])
def test_all_ones_closed_form(orc, c_in):
    x = np.ones((2, c_in, 6, 7), np.float32)
    w = np.ones((3, c_in, 3, 3), np.float32)
    z = orc.conv2d_f64(x, w, 1, 1)
    assert np.all(z[:, :, 1:-1, 1:-1] == 9 * c_in)
    assert np.all(z[:, :, 0, 1:-1] == 6 * c_in) and np.all(z[:, :, 1:-1, -1] == 6 * c_in)
    for yy, xx in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(z[:, :, yy, xx] == 4 * c_in)


def test_impulse_reproduces_rotated_kernel(orc):
    # unit impulse at (3,4): correlation output around it is the kernel rotated 180 deg
    x = np.zeros((1, 1, 7, 9), np.float32)
    x[0, 0, 3, 4] = 1.0
    w = synth.tensor_normal((2, 1, 3, 3), 11, 1)
    z = orc.conv2d_f64(x, w, 1, 1)
    for o in range(2):
        patch = z[0, o, 2:5, 3:6]
        assert np.array_equal(patch, w[o, 0, ::-1, ::-1].astype(np.float64))
    assert np.count_nonzero(z) == 18


def test_1x1_equals_matmul(orc):
    x = synth.tensor_normal((3, 7, 5, 4), 12, 1)
    w = synth.tensor_normal((6, 7, 1, 1), 12, 2)
    z = orc.conv2d_f64(x, w, 1, 0)
    ref = np.empty_like(z)
    wm = w.reshape(6, 7).astype(np.float64)
    for b in range(3):
        xm = x[b].reshape(7, 20).astype(np.float64)
        for o in range(6):
            for p in range(20):
                acc = 0.0
                for c in range(7):
                    acc += xm[c, p] * wm[o, c]
                ref[b, o].flat[p] = acc
    assert np.array_equal(z, ref)


def test_linearity_power_of_two(orc):
    x = synth.tensor_normal((1, 3, 6, 6), 13, 1)
    w = synth.tensor_normal((4, 3, 3, 3), 13, 2)
    z1 = orc.conv2d_f64(x, w, 1, 1)
    z2 = orc.conv2d_f64(x * np.float32(4.0), w * np.float32(0.5), 1, 1)
    assert np.array_equal(z2, 2.0 * z1)


def test_stride2_is_subsampled_stride1(orc):
    x = synth.tensor_normal((2, 3, 9, 11), 14, 1)
    w = synth.tensor_normal((4, 3, 3, 3), 14, 2)
    z1 = orc.conv2d_f64(x, w, 1, 1)
    z2 = orc.conv2d_f64(x, w, 2, 1)
    assert np.array_equal(z2, z1[:, :, ::2, ::2])


@pytest.mark.parametrize("cfg", [
    # n, c_in, h, w, c_out, k, stride, pad, groups
    (2, 5, 9, 8, 7, 3, 1, 1, 1),
    (1, 3, 15, 13, 4, 7, 2, 3, 1),
    (2, 6, 8, 8, 6, 3, 2, 1, 6),      # depthwise
    (1, 4, 7, 7, 6, 1, 2, 0, 1),
    (1, 4, 6, 5, 8, 3, 1, 1, 2),      # grouped
    (1, 2, 5, 5, 3, 5, 1, 2, 1),
])
def test_against_torch_float64(orc, cfg):
    n, c_in, h, w, c_out, k, s, p, g = cfg
    x = synth.tensor_normal((n, c_in, h, w), 15, *cfg)
    wt = synth.tensor_normal((c_out, c_in // g, k, k), 16, *cfg)
    z = orc.conv2d_f64(x, wt, s, p, g)
    ref = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(wt).double(), None, s, p, 1, g)
    assert z.shape == tuple(ref.shape)
    assert nmax(z, ref.numpy()) < 1e-14


def test_point_matches_full(orc):
    cfg = (2, 6, 9, 8, 6, 3, 2, 1)
    n, c_in, h, w, c_out, k, s, p = cfg
    for g in (1, 6):
        x = synth.tensor_normal((n, c_in, h, w), 17, g)
        wt = synth.tensor_normal((c_out, c_in // g, k, k), 18, g)
        z = orc.conv2d_f64(x, wt, s, p, g)
        for (b, o, y, xo) in [(0, 0, 0, 0), (1, 5, 4, 3), (1, 2, 2, 0), (0, 3, 4, 3)]:
            assert orc.conv2d_point(x, wt, b, o, y, xo, s, p, g) == z[b, o, y, xo]


def _bn(c, tag):
    return (synth.tensor_uniform((c,), 0.5, 1.5, tag, 1), synth.tensor_normal((c,), tag, 2, std=0.1),
            synth.tensor_normal((c,), tag, 3, std=0.1), synth.tensor_uniform((c,), 0.5, 1.5, tag, 4))


def test_bn_matches_torch_batch_norm(orc):
    x = synth.tensor_normal((2, 5, 6, 6), 20, 1)
    w = synth.tensor_normal((7, 5, 3, 3), 20, 2)
    g, b, m, v = _bn(7, 21)
    y = orc.conv2d_bn_act(x, w, g, b, m, v, 1e-5, 1, 1, 1, synth.ACT_RELU)
    t = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), None, 1, 1)
    t = F.batch_norm(t, torch.from_numpy(m).double(), torch.from_numpy(v).double(),
                     torch.from_numpy(g).double(), torch.from_numpy(b).double(), False, 0.0, 1e-5)
    t = F.relu(t).float().numpy()
    assert nmax(y, t) < 1e-7


def test_fold_equals_unfold(orc):
    x = synth.tensor_normal((2, 5, 8, 8), 22, 1)
    w = synth.tensor_normal((9, 5, 3, 3), 22, 2, std=0.2)
    g, b, m, v = _bn(9, 23)
    for act in (synth.ACT_NONE, synth.ACT_RELU, synth.ACT_RELU6):
        y_un = orc.conv2d_bn_act(x, w, g, b, m, v, 1e-5, 1, 1, 1, act)
        wf, bf = orc.fold_bn(w, g, b, m, v, 1e-5)
        y_fo = orc.conv2d_bias_act(x, wf, bf, 1, 1, 1, act)
        assert nmax(y_fo, y_un) < 1e-6


def test_fold_values_by_hand(orc):
    # gamma=2, var=0.25-eps -> scale 4; mean=1, beta=3 -> b = 3 - 1*4 = -1
    w = np.array([0.5, -1.5], np.float32).reshape(1, 2, 1, 1)
    eps = 2.0 ** -10
    wf, bf = orc.fold_bn(w, [2.0], [3.0], [1.0], [np.float32(0.25 - eps)], eps)
    assert wf.ravel().tolist() == [2.0, -6.0] and bf.tolist() == [-1.0]
    # with a conv bias c: b = beta + (c - mean) * s
    _, bf2 = orc.fold_bn(w, [2.0], [3.0], [1.0], [np.float32(0.25 - eps)], eps, conv_bias=[2.0])
    assert bf2.tolist() == [7.0]


def test_identity_bn_is_plain_conv(orc):
    x = synth.tensor_normal((1, 3, 5, 5), 24, 1)
    w = synth.tensor_normal((4, 3, 3, 3), 24, 2)
    eps = 2.0 ** -12
    one, zero = np.ones(4, np.float32), np.zeros(4, np.float32)
    var = np.full(4, 1.0 - eps, np.float32)
    wf, bf = orc.fold_bn(w, one, zero, zero, var, eps)
    assert np.array_equal(wf, w) and np.all(bf == 0)
    y = orc.conv2d_bn_act(x, w, one, zero, zero, var, eps, 1, 1)
    assert np.array_equal(y, orc.conv2d_f64(x, w, 1, 1).astype(np.float32))


def test_activations_and_residual(orc):
    z = np.array([-2.0, 0.5, 7.0, 5.0]).reshape(1, 1, 2, 2)
    r = np.array([1.0, 1.0, 1.0, 2.0], np.float32).reshape(1, 1, 2, 2)
    assert orc.bias_act(z, [1.0], None, synth.ACT_NONE).ravel().tolist() == [-1.0, 1.5, 8.0, 6.0]
    assert orc.bias_act(z, [1.0], None, synth.ACT_RELU).ravel().tolist() == [0.0, 1.5, 8.0, 6.0]
    assert orc.bias_act(z, [1.0], None, synth.ACT_RELU6).ravel().tolist() == [0.0, 1.5, 6.0, 6.0]
    # residual is added before the activation
    assert orc.bias_act(z, [0.0], r, synth.ACT_RELU).ravel().tolist() == [0.0, 1.5, 8.0, 7.0]


def test_maxpool_ramp_and_torch(orc):
    x = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    assert orc.maxpool(x, 2, 2).ravel().tolist() == [5.0, 7.0, 13.0, 15.0]
    # 3x3/2 pad 1 with all-negative data: padding must never win
    xn = -1.0 - synth.tensor_uniform((2, 3, 9, 7), 0.0, 1.0, 30)
    y = orc.maxpool(xn, 3, 2, 1)
    t = F.max_pool2d(torch.from_numpy(xn), 3, 2, 1).numpy()
    assert np.array_equal(y, t) and np.all(y < 0)


def test_gavgpool(orc):
    x = np.full((2, 3, 4, 5), 2.5, np.float32)
    assert np.all(orc.gavgpool(x) == 2.5)
    x = synth.tensor_normal((2, 3, 7, 7), 31)
    ref = x.astype(np.float64).reshape(2, 3, -1).mean(axis=2)
    assert nmax(orc.gavgpool(x).reshape(2, 3), ref) < 1e-7


def test_fc_brute_force(orc):
    x = np.array([[1, 2, 3], [0, -1, 2]], np.float32)
    w = np.array([[1, 0, 0], [1, 1, 1], [0, 2, -1], [0.5, 0.5, 0.5]], np.float32)
    b = np.array([0, 1, 0, -10], np.float32)
    y = orc.fc(x, w, b)
    assert y.tolist() == [[1, 7, 1, -7], [0, 2, -4, -9.5]]
    assert orc.fc(x, w, b, synth.ACT_RELU).tolist() == [[1, 7, 1, 0], [0, 2, 0, 0]]


def test_timing_build_is_the_same_loops_in_float():
    """The build whose accumulator is float (for the benchmark's CPU timing row) runs the same
    loops: it agrees with the parity build to float rounding, and is not the parity build."""
    import oracle
    x = synth.tensor_normal((2, 24, 11, 11), 901)
    w = synth.tensor_normal((7, 24, 3, 3), 902, std=0.1)
    ref = oracle.conv2d_bias_act(x, w, None, 1, 1, 1, 0, None)
    oracle.timing_build(True)
    try:
        f32 = oracle.conv2d_bias_act(x, w, None, 1, 1, 1, 0, None)
    finally:
        oracle.timing_build(False)
    again = oracle.conv2d_bias_act(x, w, None, 1, 1, 1, 0, None)
    assert np.array_equal(ref, again)
    assert not np.array_equal(ref, f32)
    assert np.max(np.abs(ref - f32)) < 1e-5 * np.max(np.abs(ref))
