"""Pins for the oracle's 3-D convolutions (the video-classification experiment treats the depth axis like height and
width).  The loops are the definition; they are pinned against torch's float64 conv3d and its gradient routines applied
to the integer codes (exact below 2^53), the exact adjoint identity, and the two reductions to the pinned 2-D routines:
a volume of depth one is an image, and a filter of depth one treats every depth slice as an image of a larger batch."""
import numpy as np
import pytest
import torch

CASES = [
    # N Cin D  H  W Cout kD kH kW sD sH sW pD pH pW dD dH dW g
    (2, 3, 5, 6, 5, 4, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1),    # the 3x3x3 layer of C3D-style networks
    (1, 4, 7, 6, 6, 6, 3, 3, 3, 1, 2, 2, 1, 1, 1, 1, 1, 1, 1),    # spatial stride
    (1, 2, 8, 5, 5, 3, 3, 1, 1, 2, 1, 1, 1, 0, 0, 1, 1, 1, 1),    # temporal filter with temporal stride
    (2, 4, 4, 5, 4, 4, 1, 3, 3, 1, 1, 1, 0, 1, 1, 1, 1, 1, 1),    # spatial filter of a (2+1)-D block
    (1, 3, 4, 4, 4, 5, 1, 1, 1, 1, 1, 1, 0, 0, 0, 1, 1, 1, 1),    # pointwise
    (1, 2, 9, 7, 7, 2, 3, 3, 3, 2, 2, 2, 2, 2, 2, 2, 2, 2, 1),    # stride, dilation and padding on every axis
    (1, 4, 5, 5, 5, 4, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 4),    # depthwise
    (1, 4, 6, 5, 5, 8, 3, 3, 3, 2, 1, 1, 0, 1, 0, 1, 1, 1, 2),    # grouped, unequal padding
    (1, 2, 3, 4, 5, 2, 3, 3, 3, 1, 1, 1, 3, 3, 3, 1, 1, 1, 1),    # padding beyond the filter's reach
    (1, 2, 6, 6, 6, 2, 2, 2, 2, 1, 1, 1, 0, 0, 0, 1, 1, 1, 1),    # even extents
]


def _codes(rng, shape):
    return rng.integers(-127, 128, size=shape, dtype=np.int64).astype(np.int8)


@pytest.mark.parametrize("case", CASES)
def test_against_torch_and_the_adjoint_identity(ref, case):
    d = ref.Conv3dDesc(*case)
    rng = np.random.default_rng(sum(case))
    qX, qW, qG = _codes(rng, d.x_shape), _codes(rng, d.w_shape), _codes(rng, d.y_shape)
    accY, o1 = ref.conv3d_fwd_acc(d, qX, qW)
    accX, o2 = ref.conv3d_bwd_data_acc(d, qG, qW)
    accW, o3 = ref.conv3d_bwd_filter_acc(d, qX, qG)
    assert not (o1 or o2 or o3)
    tX, tW, tG = (torch.from_numpy(a.astype(np.float64)) for a in (qX, qW, qG))
    kw = dict(stride=(d.strideD, d.strideH, d.strideW), padding=(d.padD, d.padH, d.padW), dilation=(d.dilD, d.dilH, d.dilW),
              groups=d.groups)
    assert np.array_equal(accY, torch.nn.functional.conv3d(tX, tW, **kw).numpy().astype(np.int64))
    assert np.array_equal(accX, torch.nn.grad.conv3d_input(d.x_shape, tW, tG, **kw).numpy().astype(np.int64))
    assert np.array_equal(accW, torch.nn.grad.conv3d_weight(tX, d.w_shape, tG, **kw).numpy().astype(np.int64))
    lhs = int(np.sum(accY.astype(np.int64) * qG.astype(np.int64)))
    assert lhs == int(np.sum(accX.astype(np.int64) * qX.astype(np.int64)))
    assert lhs == int(np.sum(accW.astype(np.int64) * qW.astype(np.int64)))


def test_depth_one_is_the_two_dimensional_routine(ref):
    d3 = ref.Conv3dDesc(2, 4, 1, 7, 6, 6, 1, 3, 3, 1, 2, 1, 0, 1, 1, 1, 1, 1, 2)
    d2 = ref.ConvDesc(2, 4, 7, 6, 6, 3, 3, 2, 1, 1, 1, 1, 1, 2)
    rng = np.random.default_rng(4)
    qX, qW, qG = _codes(rng, d3.x_shape), _codes(rng, d3.w_shape), _codes(rng, d3.y_shape)
    assert np.array_equal(ref.conv3d_fwd_acc(d3, qX, qW)[0][:, :, 0], ref.conv_fwd_acc(d2, qX[:, :, 0], qW[:, :, 0])[0])
    assert np.array_equal(ref.conv3d_bwd_data_acc(d3, qG, qW)[0][:, :, 0], ref.conv_bwd_data_acc(d2, qG[:, :, 0], qW[:, :, 0])[0])
    assert np.array_equal(ref.conv3d_bwd_filter_acc(d3, qX, qG)[0][:, :, 0], ref.conv_bwd_filter_acc(d2, qX[:, :, 0], qG[:, :, 0])[0])


def test_a_filter_of_depth_one_sees_depth_slices_as_a_batch(ref):
    d3 = ref.Conv3dDesc(2, 3, 4, 6, 5, 4, 1, 3, 3, 1, 1, 1, 0, 1, 1)
    d2 = ref.ConvDesc(2 * 4, 3, 6, 5, 4, 3, 3, 1, 1, 1, 1)
    rng = np.random.default_rng(5)
    qX, qW, qG = _codes(rng, d3.x_shape), _codes(rng, d3.w_shape), _codes(rng, d3.y_shape)
    fold = lambda a: np.ascontiguousarray(a.transpose(0, 2, 1, 3, 4)).reshape(a.shape[0] * a.shape[2], a.shape[1], a.shape[3], a.shape[4])
    unfold = lambda a, like: a.reshape(like.shape[0], like.shape[2], like.shape[1], like.shape[3], like.shape[4]).transpose(0, 2, 1, 3, 4)
    accY = ref.conv3d_fwd_acc(d3, qX, qW)[0]
    assert np.array_equal(accY, unfold(ref.conv_fwd_acc(d2, fold(qX), qW[:, :, 0])[0], accY))
    accX = ref.conv3d_bwd_data_acc(d3, qG, qW)[0]
    assert np.array_equal(accX, unfold(ref.conv_bwd_data_acc(d2, fold(qG), qW[:, :, 0])[0], accX))
    assert np.array_equal(ref.conv3d_bwd_filter_acc(d3, qX, qG)[0][:, :, 0], ref.conv_bwd_filter_acc(d2, fold(qX), fold(qG))[0])


def test_layer_routines_pair_the_scales_like_the_two_dimensional_ones(ref):
    d = ref.Conv3dDesc(1, 3, 4, 5, 5, 4, 3, 3, 3, 1, 1, 1, 1, 1, 1)
    rng = np.random.default_rng(6)
    X = rng.standard_normal(d.x_shape).astype(np.float32)
    W = (0.1 * rng.standard_normal(d.w_shape)).astype(np.float32)
    f = ref.conv3d_fwd_int8(d, X, W)
    assert f.s_x == np.abs(X).max() and f.s_w == np.abs(W).max() and np.abs(f.qX).max() == 127
    assert np.array_equal(f.acc, ref.conv3d_fwd_acc(d, f.qX, f.qW)[0])
    assert np.array_equal(f.Y, ref.dequantize_acc(f.acc, f.s_x, f.s_w))
    Yf = torch.nn.functional.conv3d(torch.from_numpy(X), torch.from_numpy(W), padding=1).numpy()
    assert np.linalg.norm(f.Y - Yf) / np.linalg.norm(Yf) < 0.02
    G = (rng.standard_normal(d.y_shape) * (10.0 ** rng.uniform(-4, -1, (1, d.Cout, 1, 1, 1)))).astype(np.float32)
    q = ref.quantize_grad3d(G, np.zeros(d.Cout, np.float32))
    flat = ref.quantize_grad(G.reshape(1, d.Cout, -1, d.Wo), np.zeros(d.Cout, np.float32))
    assert np.array_equal(q.vq.ravel(), flat.vq.ravel()) and np.array_equal(q.s_chan, flat.s_chan)
    dW, accW, _ = ref.conv3d_bwd_filter_int8(d, f.qX, f.s_x, q.vq, q.s_chan)
    dX, accX, _ = ref.conv3d_bwd_data_int8(d, q.qg, q.s_global, f.qW, f.s_w)
    co = np.arange(accW.size) // (accW.size // d.Cout)
    assert np.array_equal(dW.ravel(), ref.dequantize_acc(accW.ravel(), f.s_x, q.s_chan[co]))
    assert np.array_equal(dX, ref.dequantize_acc(accX, f.s_w, q.s_global))
    # and the int8 gradients track the fp32 ones
    tX, tW, tG = torch.from_numpy(X).double(), torch.from_numpy(W).double(), torch.from_numpy(G).double()
    rdW = torch.nn.grad.conv3d_weight(tX, d.w_shape, tG, padding=1).numpy()
    err = np.linalg.norm((dW - rdW).reshape(d.Cout, -1), axis=1) / np.linalg.norm(rdW.reshape(d.Cout, -1), axis=1)
    assert np.median(err) < 0.1
