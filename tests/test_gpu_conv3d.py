"""3-D convolution layers through the C ABI against the oracle: the forward pass (both layouts of q(X), q(W), accumulators,
Y), Algorithm 1's quantizer on the 5-D gradient, and both gradients (raw accumulators bit for bit, de-quantized values
within 1e-5 per element).  The layers cover the exact folds onto the 2-D entry points (time-only filters, pointwise
layers, volumes of depth one) and the layers that run on the direct 3-D kernels (3 x 3 x 3 and its strided, dilated,
grouped and depthwise variants)."""
import numpy as np
import pytest
import torch

from oracle import daq_ref as ref
from paper_2102_04782_amd import binding as daq

pytestmark = pytest.mark.gpu

LAYERS = {
    # name:        N Cin D  H  W Cout kD kH kW sD sH sW pD pH pW dD dH dW g     exact fold?
    "c3d_3x3x3": ((2, 8, 6, 10, 9, 12, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1), 0),
    "spatial_s2": ((1, 6, 5, 11, 10, 8, 3, 3, 3, 1, 2, 2, 1, 1, 1, 1, 1, 1, 1), 0),
    "all_s2_dil2": ((1, 4, 9, 9, 9, 6, 3, 3, 3, 2, 2, 2, 2, 2, 2, 2, 2, 2, 1), 0),
    "r2plus1d_spatial": ((2, 8, 4, 9, 8, 16, 1, 3, 3, 1, 1, 1, 0, 1, 1, 1, 1, 1, 1), 0),
    "r2plus1d_temporal": ((2, 16, 8, 7, 6, 24, 3, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 1, 1), 1),
    "temporal_s2": ((1, 12, 9, 5, 5, 20, 3, 1, 1, 2, 1, 1, 1, 0, 0, 1, 1, 1, 1), 1),
    "pointwise": ((2, 40, 4, 6, 6, 72, 1, 1, 1, 1, 1, 1, 0, 0, 0, 1, 1, 1, 1), 1),
    "depth_one": ((2, 16, 1, 10, 9, 16, 1, 3, 3, 1, 1, 1, 0, 1, 1, 1, 1, 1, 1), 1),
    "grouped": ((1, 8, 5, 6, 6, 12, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 4), 0),
    "depthwise3d": ((1, 10, 5, 7, 7, 10, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 10), 0),
    "stem_3x7x7": ((1, 3, 8, 20, 20, 16, 3, 7, 7, 1, 2, 2, 1, 3, 3, 1, 1, 1, 1), 0),
    "ragged": ((3, 5, 4, 7, 5, 19, 2, 3, 2, 1, 1, 1, 0, 1, 0, 1, 1, 1, 1), 0),
    "grouped16": ((1, 32, 3, 6, 5, 48, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 2), 0),      # whole 16-channel records per group: dot4 forms
    "wide_rows": ((1, 20, 3, 5, 23, 33, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1), 0),     # rows that are not a multiple of four positions
    "h_strided": ((2, 6, 6, 9, 10, 10, 3, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1, 1, 1), 0),      # strides in depth and height, unit stride along w
    "big_pad": ((1, 4, 4, 5, 6, 5, 3, 3, 3, 1, 1, 1, 2, 2, 2, 1, 1, 1, 1), 0),          # padding wider than the filter's reach
}


def _near(got, want, what):
    assert np.allclose(np.asarray(got), np.asarray(want), rtol=1e-5, atol=0), f"{what}: {np.abs(np.asarray(got) - np.asarray(want)).max():g} off"


def _unpack(L, buf, shape5):
    n, c, dd, h, w = shape5
    return L.unpack(buf).reshape(n, c, dd, h, w)


@pytest.mark.parametrize("name", list(LAYERS), ids=list(LAYERS))
def test_layer_against_the_oracle(name):
    fields, folds = LAYERS[name]
    dev = torch.device("cuda:0")
    d, rd = daq.Conv3dDesc(*fields), ref.Conv3dDesc(*fields)
    kind, cx, cg = daq.conv3d_carriers(d)
    assert kind == folds
    assert (d.Do, d.Ho, d.Wo) == (rd.Do, rd.Ho, rd.Wo)
    rng = np.random.default_rng(20210204 + sum(ord(ch) * (i + 1) for i, ch in enumerate(name)))
    X = np.abs(rng.standard_normal(rd.x_shape)).astype(np.float32)
    W = (rng.standard_normal(rd.w_shape) * 0.1).astype(np.float32)
    scale = 10.0 ** rng.uniform(-4, -1, (1, rd.Cout, 1, 1, 1))
    G = np.where(np.arange(rd.Cout).reshape(1, -1, 1, 1, 1) % 2 == 0, rng.standard_normal(rd.y_shape),
                 rng.laplace(0, 1, rd.y_shape) * np.where(rng.random(rd.y_shape) < 0.01, 50, 1)) * scale
    G = G.astype(np.float32)
    st = (rng.uniform(0.5, 1.0, rd.Cout) * np.abs(G).max(axis=(0, 2, 3, 4))).astype(np.float32)

    f = daq.conv3d_fwd_int8(d, torch.from_numpy(X).to(dev), torch.from_numpy(W).to(dev), want_acc=True)
    rf = ref.conv3d_fwd_int8(rd, X, W)
    assert not rf.overflow
    assert f.s_x.item() == rf.s_x and f.s_w.item() == rf.s_w
    assert np.array_equal(_unpack(daq.layout_qx_nhwc(cx), f.qx_nhwc, rd.x_shape), rf.qX), "q(X), channels innermost"
    assert np.array_equal(_unpack(daq.layout_qx_cnhw(cx), f.qx_cnhw, rd.x_shape), rf.qX), "q(X), channel-major"
    if kind == 0:
        # q(W) three times: plain [Cout][Cin/g][taps], then [tap][Cout][Cin/g up to 16] and [tap][Cin][Cout/g up to 16],
        # each part rounded up to 256 bytes, every byte that holds no code zero
        qw = f.qw.cpu().numpy()
        taps, cig, cog = rd.kD * rd.kH * rd.kW, rd.Cin // rd.groups, rd.Cout // rd.groups
        cigp, cogp = -(-cig // 16) * 16, -(-cog // 16) * 16
        up = lambda v: -(-v // 256) * 256
        codes = rf.qW.reshape(rd.Cout, cig, taps)
        fwd = np.zeros((taps, rd.Cout, cigp), np.int8)
        fwd[:, :, :cig] = codes.transpose(2, 0, 1)
        bwd = np.zeros((taps, rd.Cin, cogp), np.int8)
        for co in range(rd.Cout):
            gq = co // cog
            bwd[:, gq * cig:(gq + 1) * cig, co % cog] = codes[co].T
        want = np.zeros(up(codes.size) + up(fwd.size) + up(bwd.size), np.int8)
        want[:codes.size] = codes.ravel()
        want[up(codes.size):up(codes.size) + fwd.size] = fwd.ravel()
        want[up(codes.size) + up(fwd.size):up(codes.size) + up(fwd.size) + bwd.size] = bwd.ravel()
        assert qw.size == want.size and np.array_equal(qw, want), "q(W): plain codes and the two channel-contraction copies"
    assert np.array_equal(f.acc.cpu().numpy(), rf.acc), "forward accumulators"
    _near(f.Y.cpu().numpy(), rf.Y, "Y")

    for mode, seed in ((daq.ROUND_NEAREST, 0), (daq.ROUND_STOCHASTIC, 11)):
        s_dev = torch.from_numpy(st.copy()).to(dev)
        q = daq.quantize_grad3d(d, torch.from_numpy(G).to(dev), s_dev, mode=mode, seed=seed)
        rq = ref.quantize_grad3d(G, st, mode=mode, seed=seed)
        assert np.array_equal(_unpack(daq.layout_vq(cg), q.vq, rd.y_shape), rq.vq), "vq codes"
        assert np.array_equal(_unpack(daq.layout_qg(cg), q.qg, rd.y_shape), rq.qg), "qg codes"
        assert np.array_equal(q.cls.cpu().numpy(), rq.cls) and np.array_equal(q.stats.cpu().numpy()[:, [0, 2, 3]], rq.stats[:, [0, 2, 3]])
        _near(q.s_chan.cpu().numpy(), rq.s_chan, "s_chan")
        _near(s_dev.cpu().numpy(), rq.s_state, "clip state")
        assert q.s_global.item() == rq.s_global

        accW = torch.full(rd.w_shape, -1, dtype=torch.int32, device=dev)
        accX = torch.full(rd.x_shape, -1, dtype=torch.int32, device=dev)
        dW = daq.conv3d_bwd_filter_int8(d, f.qx_cnhw, f.s_x, q.vq, q.s_chan, acc=accW)
        dX = daq.conv3d_bwd_data_int8(d, q.qg, q.s_global, f.qw, f.s_w, acc=accX)
        torch.cuda.synchronize()
        rdW, raccW, o1 = ref.conv3d_bwd_filter_int8(rd, rf.qX, rf.s_x, rq.vq, rq.s_chan)
        rdX, raccX, o2 = ref.conv3d_bwd_data_int8(rd, rq.qg, rq.s_global, rf.qW, rf.s_w)
        assert not (o1 or o2)
        assert np.array_equal(accW.cpu().numpy(), raccW), "filter-gradient accumulators"
        assert np.array_equal(accX.cpu().numpy(), raccX), "data-gradient accumulators"
        _near(dW.cpu().numpy(), rdW, "dW")
        _near(dX.cpu().numpy(), rdX, "dX")


def test_invalid_descriptors_are_refused():
    bad = daq.Conv3dDesc(1, 4, 3, 5, 5, 6, 3, 3, 3, 1, 1, 1, 0, 0, 0, 1, 1, 1, 4)       # Cout not a multiple of the groups
    with pytest.raises(daq.DaqError):
        daq.conv3d_carriers(bad)
    deep = daq.Conv3dDesc(1, 2, 2, 5, 5, 2, 3, 3, 3, 1, 1, 1, 0, 1, 1, 1, 1, 1, 1)      # the filter is deeper than the volume
    with pytest.raises(daq.DaqError):
        daq.conv3d_carriers(deep)
