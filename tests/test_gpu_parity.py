"""GPU-vs-oracle parity, through the C ABI.

Bars: int8 codes, classes and raw int32 accumulators bit-exact; fp32 scales, clip values,
statistics and de-quantized outputs within 1e-5 relative, element by element.
"""
import numpy as np
import pytest
import torch

from oracle import daq_ref as ref
from paper_2102_04782_amd import binding as daq
from paper_2102_04782_amd import workloads as wl

pytestmark = pytest.mark.gpu

RTOL = 1e-5


def dev():
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


def close(got, want, what):
    """Every fp32 value within 1e-5 of the oracle's, relative to that value itself (a zero must be a zero)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    bad = ~np.isclose(got, want, rtol=RTOL, atol=0)
    assert not bad.any(), f"{what}: {int(bad.sum())} values off, worst {np.abs(got - want).max():g}"


def descs(layer):
    return daq.ConvDesc.make(*layer.desc_fields()), ref.ConvDesc(*layer.desc_fields())


def t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev())


# ------------------------------------------------------------------------------------------------ quantizer

def check_quantize_grad(layer, dY, st, k=1.0, A=0.8, lam=0.3, mode=0, seed=0, check_padding=True, degenerate=False,
                        scheme=None, schedule=None, side=None):
    d, _ = descs(layer)
    st_dev = t(st.copy())
    out = daq.alloc_quantize_grad(d, dev())
    out.vq.fill_(55)      # every byte of the two copies, padding included, has to come from the call
    out.qg.fill_(55)
    if side is not None:
        torch.cuda.synchronize()   # the fills above ran on the current stream; the side stream knows nothing of them
        daq.quantize_grad_split(d, t(dY), st_dev, side, scheme or daq.SCHEME_DAQ, schedule or daq.SCHEDULE_AUTO, k, A, lam, mode,
                                seed, out=out)
    elif schedule is not None:
        daq.quantize_grad_ex(d, t(dY), st_dev, scheme or daq.SCHEME_DAQ, schedule, k, A, lam, mode, seed, out=out)
    elif scheme is None:
        daq.quantize_grad(d, t(dY), st_dev, k, A, lam, mode, seed, out=out)
    else:
        daq.quantize_grad_scheme(d, t(dY), st_dev, scheme, k, A, lam, mode, seed, out=out)
    torch.cuda.synchronize()
    r = ref.quantize_grad(dY, st, k, A, lam, mode, seed, scheme=scheme or ref.SCHEME_DAQ)
    # sigma == 0 channels are fragile by construction (any negative threshold counts everything)
    assert degenerate or r.fragile.sum() == 0, "seed yields a channel whose class flips under a 1-ulp change of sigma"
    stats = out.stats.cpu().numpy()
    assert np.array_equal(stats[:, 0], r.stats[:, 0]), "gmax must be exact"
    close(stats[:, 1], r.stats[:, 1], "mean")
    close(stats[:, 2], r.stats[:, 2], "sigma")
    assert np.array_equal(stats[:, 2], r.stats[:, 2]), "sigma differs in the last bit"
    assert np.array_equal(stats[:, 3], r.stats[:, 3]), "tail mass P"
    assert np.array_equal(out.cls.cpu().numpy(), r.cls), "classes"
    close(out.s_chan.cpu().numpy(), r.s_chan, "s_chan")
    close(st_dev.cpu().numpy(), r.s_state, "s_state")
    close(out.s_global.cpu().numpy(), [r.s_global], "s_global")
    Lv, Lg = daq.layout_vq(d), daq.layout_qg(d)
    assert np.array_equal(Lv.unpack(out.vq), r.vq), "vq codes"
    assert np.array_equal(Lg.unpack(out.qg), r.qg), "qg codes"
    if check_padding:
        assert Lv.padding_is_zero(out.vq), "vq padding bytes must be zero"
        assert Lg.padding_is_zero(out.qg), "qg bytes that hold no element must be zero"
    return out, r


def test_quantize_grad_config1_all_modes():
    layer, X, W, dY, st = wl.make_inputs(1)
    check_quantize_grad(layer, dY, st)
    check_quantize_grad(layer, dY, np.zeros_like(st))                      # no history
    check_quantize_grad(layer, dY, st, k=1.5, A=0.8)                       # negative coefficient
    check_quantize_grad(layer, dY, st, k=1.2, A=0.5)
    check_quantize_grad(layer, dY, 10 * st, k=1.5, A=0.8)                  # non-positive result guard
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=7)
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=2 ** 63 + 12345)
    check_quantize_grad(layer, dY, st, lam=0.0)                            # everything Gaussian
    check_quantize_grad(layer, dY, st, lam=1.0)                            # everything Inverted-T


ODD_LAYERS = [
    wl.Layer("odd_c", 3, 5, 9, 7, 19, 3, 3, 1, 1),            # C not a multiple of 16, HW not of 4
    wl.Layer("wide_c", 2, 8, 6, 6, 130, 1, 1, 1, 0),           # three 64-channel blocks, ragged
    wl.Layer("s2", 2, 6, 11, 10, 24, 3, 3, 2, 1),              # strided slot geometry
    wl.Layer("stem", 1, 3, 30, 30, 16, 7, 7, 2, 3),
    wl.Layer("dw", 2, 24, 13, 13, 24, 3, 3, 1, 1, 1, 24),      # depthwise: qg in CNHW
    wl.Layer("dw_s2", 2, 16, 12, 12, 16, 3, 3, 2, 1, 1, 16),
    wl.Layer("big_hw", 1, 4, 67, 67, 4, 3, 3, 1, 1),           # several pixel tiles with a ragged tail
    wl.Layer("one_px", 5, 4, 1, 1, 7, 1, 1, 1, 0),             # 1x1 images
    wl.Layer("w14", 3, 8, 14, 14, 20, 3, 3, 1, 1),             # rows of 14: two codes per store
    wl.Layer("w14_1x1", 4, 16, 14, 14, 70, 1, 1, 1, 0),        # no padding rows or columns at all
    wl.Layer("long_m", 40, 4, 56, 56, 4, 3, 3, 1, 1),          # workgroups loop over several chunks / tiles
    wl.Layer("c24_long", 6, 8, 41, 39, 24, 1, 1, 1, 0),        # two groups of 16 channels: waves pair up on pixel tiles, ragged last tile
    wl.Layer("c32", 3, 8, 17, 19, 32, 1, 1, 1, 0),             # two full groups
]


@pytest.mark.parametrize("layer", ODD_LAYERS, ids=lambda l: l.name)
def test_quantize_grad_ragged_shapes(layer):
    seed = wl.seed_for(9, ODD_LAYERS.index(layer))
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    check_quantize_grad(layer, dY, st)
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=99)


def test_quantize_grad_with_a_source_that_is_only_4_byte_aligned():
    layer = wl.Layer("misaligned", 2, 8, 12, 12, 10, 3, 3, 1, 1)
    seed = wl.seed_for(9, 77)
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    d, _ = descs(layer)
    buf = torch.zeros(dY.size + 4, dtype=torch.float32, device="cuda")
    for shift in (1, 2):
        g = buf[shift:shift + dY.size].view(dY.shape)
        g.copy_(t(dY))
        assert g.data_ptr() % 16 != 0 and g.is_contiguous()
        st_dev = t(st.copy())
        out = daq.quantize_grad(d, g, st_dev)
        torch.cuda.synchronize()
        r = ref.quantize_grad(dY, st)
        assert np.array_equal(daq.layout_vq(d).unpack(out.vq), r.vq)
        assert np.array_equal(daq.layout_qg(d).unpack(out.qg), r.qg)
        assert np.array_equal(out.cls.cpu().numpy(), r.cls)
        assert daq.layout_vq(d).padding_is_zero(out.vq)


def test_quantize_grad_degenerate_channels():
    layer = wl.Layer("deg", 2, 4, 8, 8, 6, 3, 3, 1, 1)
    rng = np.random.default_rng(3)
    dY = rng.normal(0, 1e-2, layer.y_shape).astype(np.float32)
    dY[:, 0] = 0.0                      # all-zero channel: scale 0, codes 0
    dY[:, 1] = 0.5                      # constant channel: sigma 0, P = 1
    dY[:, 2] = np.float32(1e-38)        # scale below 2^-100
    dY[:, 3, 0, 0] = 1e4                # one huge outlier
    st = np.zeros(6, np.float32)
    out, r = check_quantize_grad(layer, dY, st, degenerate=True)
    assert out.s_chan.cpu().numpy()[0] == 0.0 and out.s_chan.cpu().numpy()[2] == 0.0
    zero = np.zeros_like(dY)
    check_quantize_grad(layer, zero, st, degenerate=True)  # all-zero tensor: global scale 0


def test_state_carries_across_iterations_and_runs_are_deterministic():
    layer, X, W, dY, st = wl.make_inputs(1)
    d, _ = descs(layer)
    g = t(dY)
    s1 = t(st.copy())
    a = daq.quantize_grad(d, g, s1)
    b = daq.quantize_grad(d, g, s1)          # second iteration: state carried in place
    s2 = t(st.copy())
    a2 = daq.quantize_grad(d, g, s2)
    torch.cuda.synchronize()
    assert torch.equal(a.vq, a2.vq) and torch.equal(a.qg, a2.qg) and torch.equal(a.s_chan, a2.s_chan)
    r1 = ref.quantize_grad(dY, st)
    r2 = ref.quantize_grad(dY, r1.s_state)
    close(s1.cpu().numpy(), r2.s_state, "state after two iterations")
    assert np.array_equal(daq.layout_vq(d).unpack(b.vq), r2.vq)


# ------------------------------------------------------------------------------------------------ ablation schemes

SCHEMES = [(daq.SCHEME_DAQ, "daq"), (daq.SCHEME_GQ, "gq"), (daq.SCHEME_GVQ, "gvq"), (daq.SCHEME_MCS, "mcs")]


def test_scheme_constants_agree():
    assert (daq.SCHEME_DAQ, daq.SCHEME_GQ, daq.SCHEME_GVQ, daq.SCHEME_MCS) == \
           (ref.SCHEME_DAQ, ref.SCHEME_GQ, ref.SCHEME_GVQ, ref.SCHEME_MCS)


@pytest.mark.parametrize("scheme", [s for s, _ in SCHEMES], ids=[n for _, n in SCHEMES])
def test_quantize_grad_schemes_config1(scheme):
    layer, X, W, dY, st = wl.make_inputs(1)
    check_quantize_grad(layer, dY, st, scheme=scheme)
    check_quantize_grad(layer, dY, np.zeros_like(st), scheme=scheme)
    check_quantize_grad(layer, dY, st, k=1.5, A=0.8, scheme=scheme)
    check_quantize_grad(layer, dY, 10 * st, k=1.5, A=0.8, scheme=scheme)
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=7, scheme=scheme)
    check_quantize_grad(layer, dY, st, lam=0.0, scheme=scheme)
    check_quantize_grad(layer, dY, st, lam=1.0, scheme=scheme)          # the layer as a whole takes the clipped branch


@pytest.mark.parametrize("scheme", [s for s, _ in SCHEMES[1:]], ids=[n for _, n in SCHEMES[1:]])
@pytest.mark.parametrize("layer", ODD_LAYERS, ids=lambda l: l.name)
def test_quantize_grad_schemes_ragged_shapes(layer, scheme):
    seed = wl.seed_for(11, ODD_LAYERS.index(layer))
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    check_quantize_grad(layer, dY, st, scheme=scheme)
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=5, scheme=scheme)


@pytest.mark.parametrize("scheme", [s for s, _ in SCHEMES[1:]], ids=[n for _, n in SCHEMES[1:]])
def test_quantize_grad_schemes_degenerate_tensors(scheme):
    layer = wl.Layer("deg", 2, 4, 8, 8, 6, 3, 3, 1, 1)
    rng = np.random.default_rng(3)
    dY = rng.normal(0, 1e-2, layer.y_shape).astype(np.float32)
    dY[:, 0] = 0.0
    dY[:, 1] = 0.5
    dY[:, 2] = np.float32(1e-38)
    dY[:, 3, 0, 0] = 1e4
    st = np.zeros(6, np.float32)
    check_quantize_grad(layer, dY, st, degenerate=True, scheme=scheme)
    check_quantize_grad(layer, np.zeros_like(dY), st, degenerate=True, scheme=scheme)
    tiny = np.full_like(dY, np.float32(1e-38))                            # every scale below 2^-100
    check_quantize_grad(layer, tiny, st, degenerate=True, scheme=scheme)


def test_layerwise_clipping_takes_the_long_tailed_branch():
    # a tensor that is long-tailed as a whole: the layer-wise scheme clips below |g|max, with s_state[0] as history
    layer = wl.Layer("tail", 4, 8, 20, 20, 24, 3, 3, 1, 1)
    rng = np.random.default_rng(17)
    dY = (rng.laplace(0, 1e-3, layer.y_shape) * np.where(rng.random(layer.y_shape) < 0.01, 30, 1)).astype(np.float32)
    st = np.full(24, 99.0, np.float32)
    st[0] = 0.5 * np.abs(dY).max()
    out, r = check_quantize_grad(layer, dY, st, scheme=daq.SCHEME_MCS)
    assert r.cls[0] == ref.INVT and r.s_chan[0] < r.s_global
    assert np.isclose(r.s_chan[0], 0.9 * np.abs(dY).max(), rtol=1e-6)        # (1 - kA) * history + A * |g|max
    assert np.all(r.s_chan == r.s_chan[0]) and np.all(r.s_state == r.s_chan[0])


DW_LAYERS = [
    wl.Layer("dw_big", 6, 40, 28, 28, 40, 3, 3, 1, 1, 1, 40),
    wl.Layer("dw_s2_big", 4, 24, 30, 30, 24, 3, 3, 2, 1, 1, 24),
    wl.Layer("dw_5x5", 2, 8, 14, 14, 8, 5, 5, 1, 2, 1, 8),
]


@pytest.mark.parametrize("layer", DW_LAYERS, ids=lambda l: l.name)
def test_depthwise_data_gradient_from_the_per_channel_copy_end_to_end(layer):
    # quantizer -> data gradient, both on the GPU, against the same chain in the oracle
    d, rd = descs(layer)
    seed = wl.seed_for(12, DW_LAYERS.index(layer))
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    Wt = wl.make_W(layer, seed, kaiming=True)
    X = wl.make_X(layer, seed, post_relu=True)
    f = daq.conv_fwd_int8(d, t(X), t(Wt))
    q = daq.quantize_grad(d, t(dY), t(st.copy()))
    dX = daq.conv_bwd_data_int8_chan(d, q.vq, q.s_chan, f.qw, f.s_w)
    torch.cuda.synchronize()
    rq = ref.quantize_grad(dY, st)
    qW, s_w = ref.quantize_tensor(Wt)
    want = ref.conv_bwd_data_int8_chan(rd, rq.vq, rq.s_chan, qW, s_w)[0]
    got = dX.cpu().numpy()
    for c in range(layer.Cin):
        close(got[:, c], want[:, c], f"channel {c}")
    # and it is the better gradient on channels of small spread: the typical channel is far closer to the fp32 one
    exact = torch.nn.grad.conv2d_input(d.x_shape, torch.from_numpy(Wt).double(), torch.from_numpy(dY).double(),
                                       stride=layer.stride, padding=layer.pad, dilation=layer.dil, groups=layer.groups).numpy()
    glob = daq.conv_bwd_data_int8(d, q.qg, q.s_global, f.qw, f.s_w).cpu().numpy()
    err = lambda a: np.abs(a - exact).mean(axis=(0, 2, 3))
    assert np.median(err(got) / err(glob)) < 0.5


# ------------------------------------------------------------------------------------------------ bfloat16 gradients

def check_quantize_grad_bf16(layer, dY, st, scheme=daq.SCHEME_DAQ, misalign=0, **kw):
    """dY rounded to bfloat16 goes to daq_quantize_grad_bf16 and, widened, to the oracle: every output bit for bit."""
    d, _ = descs(layer)
    bits = ref.bf16_bits(dY).astype(np.uint16)
    buf = torch.zeros(bits.size + 8, dtype=torch.bfloat16, device=dev())
    g = buf[misalign:misalign + bits.size].view(dY.shape)
    g.copy_(torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev()).view(dY.shape))
    st_dev = t(st.copy())
    out = daq.quantize_grad_bf16(d, g, st_dev, scheme, **kw)
    torch.cuda.synchronize()
    r = ref.quantize_grad_bf16(bits, st, scheme=scheme, **kw)
    assert np.array_equal(out.stats.cpu().numpy(), r.stats), "statistics"
    assert np.array_equal(out.cls.cpu().numpy(), r.cls), "classes"
    close(out.s_chan.cpu().numpy(), r.s_chan, "s_chan")
    close(st_dev.cpu().numpy(), r.s_state, "s_state")
    close(out.s_global.cpu().numpy(), [r.s_global], "s_global")
    Lv, Lg = daq.layout_vq(d), daq.layout_qg(d)
    assert np.array_equal(Lv.unpack(out.vq), r.vq), "vq codes"
    assert np.array_equal(Lg.unpack(out.qg), r.qg), "qg codes"
    assert Lv.padding_is_zero(out.vq)
    # and the same bits as the fp32 entry point on the widened tensor
    st2 = t(st.copy())
    wide = daq.quantize_grad_scheme(d, g.float().contiguous(), st2, scheme, **kw)
    torch.cuda.synchronize()
    assert np.array_equal(Lv.unpack(wide.vq), Lv.unpack(out.vq)) and np.array_equal(Lg.unpack(wide.qg), Lg.unpack(out.qg))
    assert torch.equal(wide.s_chan, out.s_chan) and torch.equal(st2, st_dev) and torch.equal(wide.cls, out.cls)
    assert torch.equal(wide.stats, out.stats) and torch.equal(wide.s_global, out.s_global)


def test_quantize_grad_bf16_config1_all_modes():
    layer, X, W, dY, st = wl.make_inputs(1)
    check_quantize_grad_bf16(layer, dY, st)
    check_quantize_grad_bf16(layer, dY, np.zeros_like(st))
    check_quantize_grad_bf16(layer, dY, st, k=1.5, A=0.8)
    check_quantize_grad_bf16(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=7)
    check_quantize_grad_bf16(layer, dY, st, lam=0.0)
    check_quantize_grad_bf16(layer, dY, st, lam=1.0)
    for scheme, _ in SCHEMES[1:]:
        check_quantize_grad_bf16(layer, dY, st, scheme=scheme)


@pytest.mark.parametrize("layer", ODD_LAYERS, ids=lambda l: l.name)
def test_quantize_grad_bf16_ragged_shapes(layer):
    seed = wl.seed_for(14, ODD_LAYERS.index(layer))
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    check_quantize_grad_bf16(layer, dY, st)
    check_quantize_grad_bf16(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=99)
    for shift in (1, 2, 3):                       # sources that are only 2-, 4- or 6-byte aligned
        check_quantize_grad_bf16(layer, dY, st, misalign=shift)


def test_quantize_grad_bf16_degenerate_tensors():
    layer = wl.Layer("deg", 2, 4, 8, 8, 6, 3, 3, 1, 1)
    rng = np.random.default_rng(3)
    dY = rng.normal(0, 1e-2, layer.y_shape).astype(np.float32)
    dY[:, 0] = 0.0
    dY[:, 1] = 0.5
    dY[:, 2] = np.float32(1e-38)
    dY[:, 3, 0, 0] = 1e4
    st = np.zeros(6, np.float32)
    check_quantize_grad_bf16(layer, dY, st)
    check_quantize_grad_bf16(layer, np.zeros_like(dY), st)


def test_unknown_scheme_is_refused():
    layer, X, W, dY, st = wl.make_inputs(1)
    d, _ = descs(layer)
    with pytest.raises(daq.DaqError):
        daq.quantize_grad_scheme(d, t(dY), t(st.copy()), 4)


# ------------------------------------------------------------------------------------------------ convolutions

CONV_LAYERS = [
    wl.Layer("c3x3", 2, 16, 10, 9, 32, 3, 3, 1, 1),
    wl.Layer("c3x3_ragged", 3, 5, 9, 7, 19, 3, 3, 1, 1),
    wl.Layer("c1x1", 2, 48, 7, 7, 80, 1, 1, 1, 0),
    wl.Layer("c3x3_s2", 2, 16, 11, 10, 16, 3, 3, 2, 1),
    wl.Layer("c1x1_s2", 2, 32, 8, 8, 64, 1, 1, 2, 0),
    wl.Layer("stem7x7", 1, 3, 30, 30, 16, 7, 7, 2, 3),
    wl.Layer("dil2", 1, 16, 12, 12, 16, 3, 3, 1, 2, 2),
    wl.Layer("nopad", 2, 16, 9, 9, 16, 3, 3, 1, 0),
    wl.Layer("grouped", 2, 16, 8, 8, 32, 3, 3, 1, 1, 1, 4),
    wl.Layer("dw", 2, 24, 13, 13, 24, 3, 3, 1, 1, 1, 24),
    wl.Layer("dw_s2", 2, 16, 12, 12, 16, 3, 3, 2, 1, 1, 16),
    wl.Layer("c3x3_64", 4, 64, 14, 14, 64, 3, 3, 1, 1),
    wl.Layer("c3x3_7x7", 16, 128, 7, 7, 64, 3, 3, 1, 1),
    wl.Layer("c1x1_wide", 8, 256, 7, 7, 128, 1, 1, 1, 0),
    wl.Layer("c5x5", 2, 20, 12, 12, 24, 5, 5, 1, 2),              # 25 taps: waves split the taps
    wl.Layer("c3x3_s2_big", 8, 32, 28, 28, 96, 3, 3, 2, 1),       # strided, several tiles, K split across workgroups
    wl.Layer("stem_big", 4, 3, 64, 64, 64, 7, 7, 2, 3),           # 49 taps on eight waves, K split
    wl.Layer("c1x1_s2_big", 8, 64, 28, 28, 128, 1, 1, 2, 0),      # strided projection shortcut
    wl.Layer("c3x3_s2_dil2", 2, 16, 15, 14, 16, 3, 3, 2, 2, 2),   # stride and dilation together
    wl.Layer("c3x3_s2_pad0", 3, 20, 13, 12, 40, 3, 3, 2, 0),      # strided without padding; ragged channel tiles
    wl.Layer("c3x3_s2_w14", 2, 8, 14, 14, 24, 3, 3, 2, 1),        # row pitch 8: the shifted windows start on dword boundaries
    wl.Layer("c3x3_s2_w16", 2, 40, 9, 16, 8, 3, 3, 2, 1),         # row pitch 9
    wl.Layer("c1x1_pad", 2, 16, 6, 6, 16, 1, 1, 1, 1),            # padded 1x1
    wl.Layer("c1x1_thin16", 3, 40, 10, 12, 16, 1, 1, 1, 0),       # thin 1x1 (streaming data gradient): 16-byte pixel records, ragged row block
    wl.Layer("c1x1_thin24", 2, 144, 9, 7, 24, 1, 1, 1, 0),        # 32-byte records; groups of 32 pixels straddle images; ragged last group
    wl.Layer("c1x1_thin48", 1, 33, 5, 5, 48, 1, 1, 1, 0),         # 48-byte records: the last 16 contraction bytes are another pixel's
    wl.Layer("c1x1_thin64", 2, 96, 8, 8, 64, 1, 1, 1, 0),         # full 64-byte records, two multiplies per block
    wl.Layer("c1x1_thin96", 3, 70, 6, 7, 96, 1, 1, 1, 0),         # three contraction steps on the four-step form; three row blocks (a dead one in the last pair)
    wl.Layer("c1x1_thin160", 2, 200, 5, 5, 160, 1, 1, 1, 0),      # five steps on the eight-step form
    wl.Layer("c1x1_thin256", 1, 64, 12, 12, 256, 1, 1, 1, 0),     # all eight steps
    wl.Layer("dw_big", 6, 40, 28, 28, 40, 3, 3, 1, 1, 1, 40),     # depthwise, several slabs per channel
    wl.Layer("dw_s2_big", 4, 24, 30, 30, 24, 3, 3, 2, 1, 1, 24),
    wl.Layer("dw_s2_blk", 3, 20, 26, 28, 20, 3, 3, 2, 1, 1, 20),    # strided depthwise, 4 x 4 output blocks; ragged last row quad
    wl.Layer("dw_s2_blk_odd", 2, 8, 13, 16, 8, 3, 3, 2, 1, 1, 8),   # the same with an odd number of rows
    wl.Layer("dw_s2_blk_4", 1, 4, 4, 4, 4, 3, 3, 2, 1, 1, 4),       # a single block per plane
    wl.Layer("dw_blk_ragged", 2, 12, 10, 12, 12, 3, 3, 1, 1, 1, 12),  # unit stride, 4 x 4 output blocks; last row quad has two rows
    wl.Layer("dw_blk_odd", 3, 6, 5, 8, 6, 3, 3, 1, 1, 1, 6),          # ... one row
    wl.Layer("dw_blk_4", 1, 4, 4, 4, 4, 3, 3, 1, 1, 1, 4),
    wl.Layer("dw_5x5", 2, 8, 14, 14, 8, 5, 5, 1, 2, 1, 8),
    wl.Layer("dw_w7", 3, 16, 7, 7, 16, 3, 3, 1, 1, 1, 16),        # rows that are not a multiple of four outputs
    wl.Layer("dw_dil2", 2, 8, 12, 12, 8, 3, 3, 1, 2, 2, 8),
    wl.Layer("c1x1_huge", 1, 2048, 4, 4, 2048, 1, 1, 1, 0),       # enough 128 x 128 tiles for the four-wave GEMM form
    wl.Layer("c1x1_px128_7x7", 5, 96, 7, 7, 320, 1, 1, 1, 0),     # few pixels, long contraction: 128-pixel tiles of two images, ragged last group and row tile
    wl.Layer("c1x1_px128_14", 2, 288, 14, 14, 272, 1, 1, 1, 0),   # the same with a 9-row and a 5-row tile per image, in both directions
    wl.Layer("c3x3_px128", 5, 96, 7, 7, 128, 3, 3, 1, 1),          # 3 x 3 with few tiles: 128-pixel tiles of two images with their halos
    wl.Layer("c1x1_s2_ring", 64, 384, 28, 28, 128, 1, 1, 2, 0),   # strided 1 x 1 with two contraction chunks and 384 tiles: 256-pixel tiles, chunks in rings
    wl.Layer("c1x1_s2_ring_odd", 3, 64, 13, 11, 160, 1, 1, 2, 0),  # ... 128-pixel tiles, odd image width (zeros of the 2 x 2 blocks one by one)
    wl.Layer("c3x3_huge", 1, 1024, 4, 4, 1024, 3, 3, 1, 1),       # enough 64 x 64 tiles for the four-wave 3x3 form
    wl.Layer("c3x3_wide", 1, 16, 8, 130, 16, 3, 3, 1, 1),         # rows too long for the LDS window: global-fragment form
    wl.Layer("c3x3_wide_huge", 1, 768, 2, 130, 1024, 3, 3, 1, 1),  # the same with enough tiles for its LDS-staged sibling
    # filter gradients with many output tiles and fewer than eight K splits: each XCD takes a rectangle of the tile grid
    wl.Layer("c1x1_rect_1", 2, 512, 5, 5, 520, 1, 1, 1, 0),       # 9 x 8 tiles of 64 x 64 (ragged), one split, eight rectangles
    wl.Layer("c1x1_rect_2", 8, 320, 12, 12, 200, 1, 1, 1, 0),     # 4 x 5 tiles, a short flat axis: two splits, four rectangles each
    wl.Layer("c3x3_rect_1", 1, 232, 6, 6, 200, 3, 3, 1, 1),       # 7 x 8 tiles of 32 x 32 (ragged), one split
]


def run_convs_on_codes(layer, qX, qW, qG, s_x, s_w, s_g, s_c):
    """Feed the same int8 codes to the GPU convolutions (packed into the device layouts) and to the oracle."""
    d, rd = descs(layer)
    device = dev()
    s_x_d, s_w_d, s_g_d = (torch.tensor([v], dtype=torch.float32, device=device) for v in (s_x, s_w, s_g))
    s_c_d = t(s_c)
    qx_cnhw = t(daq.layout_qx_cnhw(d).pack(qX))
    qx_nhwc = t(daq.layout_qx_nhwc(d).pack(qX))
    qw = t(daq.layout_qw(d).pack(d, qW))
    vq = t(daq.layout_vq(d).pack(qG))
    qg = t(daq.layout_qg(d).pack(qG))

    accW = torch.empty(d.w_shape, dtype=torch.int32, device=device)
    accX = torch.empty(d.x_shape, dtype=torch.int32, device=device)
    dW = daq.conv_bwd_filter_int8(d, qx_cnhw, s_x_d, vq, s_c_d, acc=accW)
    dX = daq.conv_bwd_data_int8(d, qg, s_g_d, qw, s_w_d, acc=accX)
    torch.cuda.synchronize()

    rdW, raccW, o1 = ref.conv_bwd_filter_int8(rd, qX, s_x, qG, s_c)
    rdX, raccX, o2 = ref.conv_bwd_data_int8(rd, qG, s_g, qW, s_w)
    assert not (o1 or o2)
    assert np.array_equal(accW.cpu().numpy(), raccW), "dW accumulators"
    assert np.array_equal(accX.cpu().numpy(), raccX), "dX accumulators"
    close(dW.cpu().numpy(), rdW, "dW")
    close(dX.cpu().numpy(), rdX, "dX")
    # without the debug output the result is the same
    dW2 = daq.conv_bwd_filter_int8(d, qx_cnhw, s_x_d, vq, s_c_d)
    dX2 = daq.conv_bwd_data_int8(d, qg, s_g_d, qw, s_w_d)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW2) and torch.equal(dX, dX2)
    # both gradients in one call (the filter gradient's last stage may ride on the data-gradient launch)
    accW3, accX3 = torch.full_like(accW, -1), torch.full_like(accX, -1)
    dW3, dX3 = daq.conv_bwd_int8(d, qx_cnhw, s_x_d, vq, s_c_d, qg, s_g_d, qw, s_w_d, dW_acc=accW3, dX_acc=accX3)
    dW4, dX4 = daq.conv_bwd_int8(d, qx_cnhw, s_x_d, vq, s_c_d, qg, s_g_d, qw, s_w_d)
    torch.cuda.synchronize()
    assert np.array_equal(accW3.cpu().numpy(), raccW), "dW accumulators, combined call"
    assert np.array_equal(accX3.cpu().numpy(), raccX), "dX accumulators, combined call"
    close(dW3.cpu().numpy(), rdW, "dW, combined call")
    close(dX3.cpu().numpy(), rdX, "dX, combined call")
    assert torch.equal(dW3, dW) and torch.equal(dX3, dX) and torch.equal(dW4, dW) and torch.equal(dX4, dX)
    # depthwise layers: the data gradient from the per-channel copy, de-quantized per channel
    depthwise = layer.groups > 1 and layer.groups == layer.Cin == layer.Cout
    if depthwise and layer.kH <= 7 and layer.kW <= 7 and layer.stride & (layer.stride - 1) == 0:
        accX5 = torch.full_like(accX, -1)
        dX5 = daq.conv_bwd_data_int8_chan(d, vq, s_c_d, qw, s_w_d, acc=accX5)
        dX6 = daq.conv_bwd_data_int8_chan(d, vq, s_c_d, qw, s_w_d)
        torch.cuda.synchronize()
        rdX5, raccX5, o5 = ref.conv_bwd_data_int8_chan(rd, qG, s_c, qW, s_w)
        assert not o5 and np.array_equal(accX5.cpu().numpy(), raccX5), "dX accumulators, per-channel copy"
        got = dX5.cpu().numpy()
        for c in range(layer.Cin):                      # the tolerance is relative to each channel's own magnitude
            close(got[:, c], rdX5[:, c], f"dX from the per-channel copy, channel {c}")
        assert torch.equal(dX5, dX6)
    else:   # dense and grouped layers, and depthwise ones outside the channel-major kernels (documented)
        with pytest.raises(daq.DaqError) as e:
            daq.conv_bwd_data_int8_chan(d, vq, s_c_d, qw, s_w_d)
        assert e.value.code == daq.ERR_UNSUPPORTED


@pytest.mark.parametrize("layer", CONV_LAYERS, ids=lambda l: l.name)
def test_backward_convs_on_random_codes(layer):
    rng = np.random.default_rng(wl.seed_for(8, CONV_LAYERS.index(layer)))
    qX = rng.integers(-127, 128, layer.x_shape).astype(np.int8)
    qW = rng.integers(-127, 128, layer.w_shape).astype(np.int8)
    qG = rng.integers(-127, 128, layer.y_shape).astype(np.int8)
    s_c = (10.0 ** rng.uniform(-4, -1, layer.Cout)).astype(np.float32)
    run_convs_on_codes(layer, qX, qW, qG, 2.5, 0.11, 0.03, s_c)


def check_forward(layer, seed, schedule=None):
    d, rd = descs(layer)
    X, W = wl.make_X(layer, seed, post_relu=False), wl.make_W(layer, seed)
    f = daq.alloc_fwd(d, dev(), want_acc=True)
    for buf in (f.qx_nhwc, f.qx_cnhw, f.qw):
        buf.fill_(55)
    daq.conv_fwd_int8(d, t(X), t(W), out=f, schedule=schedule)
    torch.cuda.synchronize()
    r = ref.conv_fwd_int8(rd, X, W)
    assert not r.overflow
    close(f.s_x.cpu().numpy(), [r.s_x], "s_x")
    close(f.s_w.cpu().numpy(), [r.s_w], "s_w")
    assert np.array_equal(daq.layout_qx_nhwc(d).unpack(f.qx_nhwc), r.qX) and daq.layout_qx_nhwc(d).padding_is_zero(f.qx_nhwc)
    Lc = daq.layout_qx_cnhw(d)
    assert np.array_equal(Lc.unpack(f.qx_cnhw), r.qX) and Lc.padding_is_zero(f.qx_cnhw)
    Lw = daq.layout_qw(d)
    assert np.array_equal(f.qw.cpu().numpy(), Lw.pack(d, r.qW)), "packed filter (all three copies)"
    assert np.array_equal(f.acc.cpu().numpy(), r.acc)
    close(f.Y.cpu().numpy(), r.Y, "Y")


@pytest.mark.parametrize("layer", CONV_LAYERS, ids=lambda l: l.name)
def test_forward_layer(layer):
    check_forward(layer, wl.seed_for(7, CONV_LAYERS.index(layer)))


def full_layer_parity(config, index, layer=None):
    layer, X, W, dY, st = wl.make_inputs(config, index, layer)
    d, rd = descs(layer)
    device = dev()
    f = daq.conv_fwd_int8(d, t(X), t(W))
    st_dev = t(st.copy())
    q = daq.quantize_grad(d, t(dY), st_dev)
    accW = torch.empty(d.w_shape, dtype=torch.int32, device=device)
    accX = torch.empty(d.x_shape, dtype=torch.int32, device=device)
    dW = daq.conv_bwd_filter_int8(d, f.qx_cnhw, f.s_x, q.vq, q.s_chan, acc=accW)
    dX = daq.conv_bwd_data_int8(d, q.qg, q.s_global, f.qw, f.s_w, acc=accX)
    torch.cuda.synchronize()

    rf = ref.conv_fwd_int8(rd, X, W)
    rq = ref.quantize_grad(dY, st)
    assert rq.fragile.sum() == 0
    rdW, raccW, o1 = ref.conv_bwd_filter_int8(rd, rf.qX, rf.s_x, rq.vq, rq.s_chan)
    rdX, raccX, o2 = ref.conv_bwd_data_int8(rd, rq.qg, rq.s_global, rf.qW, rf.s_w)
    assert not (o1 or o2)
    assert np.array_equal(daq.layout_vq(d).unpack(q.vq), rq.vq)
    assert np.array_equal(daq.layout_qg(d).unpack(q.qg), rq.qg)
    assert np.array_equal(q.cls.cpu().numpy(), rq.cls)
    close(q.s_chan.cpu().numpy(), rq.s_chan, "s_chan")
    assert np.array_equal(accW.cpu().numpy(), raccW)
    assert np.array_equal(accX.cpu().numpy(), raccX)
    close(dW.cpu().numpy(), rdW, "dW")
    close(dX.cpu().numpy(), rdX, "dX")
    close(f.Y.cpu().numpy(), rf.Y, "Y")
    accW2, accX2 = torch.full_like(accW, -1), torch.full_like(accX, -1)
    dW2, dX2 = daq.conv_bwd_int8(d, f.qx_cnhw, f.s_x, q.vq, q.s_chan, q.qg, q.s_global, f.qw, f.s_w, dW_acc=accW2, dX_acc=accX2)
    torch.cuda.synchronize()
    assert np.array_equal(accW2.cpu().numpy(), raccW) and np.array_equal(accX2.cpu().numpy(), raccX)
    assert torch.equal(dW2, dW) and torch.equal(dX2, dX), "combined call differs from the two separate calls"


def test_config1_full_layer():
    full_layer_parity(1, 0)


def test_config2_full_layer():
    full_layer_parity(2, 0)


@pytest.mark.parametrize("index", [0, 1, 2])
def test_config3_layers(index):
    # the stage-4 layers at their full batch (N = 128); the oracle needs a few seconds per convolution
    full_layer_parity(3, index)


def test_accumulator_wraparound_matches_two_complement():
    # 1x1 layer with 140000 positions of 127*127: the true sum exceeds 2^31 and must wrap, not saturate
    layer = wl.Layer("wrap", 1, 16, 350, 400, 16, 1, 1, 1, 0)
    d, rd = descs(layer)
    qX = np.full(layer.x_shape, 127, np.int8)
    qG = np.full(layer.y_shape, 127, np.int8)
    device = dev()
    one = torch.ones(1, dtype=torch.float32, device=device)
    acc = torch.empty(d.w_shape, dtype=torch.int32, device=device)
    daq.conv_bwd_filter_int8(d, t(daq.layout_qx_cnhw(d).pack(qX)), one, t(daq.layout_vq(d).pack(qG)),
                             torch.ones(16, dtype=torch.float32, device=device), acc=acc)
    torch.cuda.synchronize()
    racc, ovf = ref.conv_bwd_filter_acc(rd, qX, qG)
    assert ovf and np.array_equal(acc.cpu().numpy(), racc)


def _random_layers(count, seed):
    """Seeded random small descriptors: every stride / dilation / padding / group / extent combination the entry
    points accept, at sizes the oracle finishes instantly."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        k = int(rng.choice([1, 2, 3, 3, 3, 5, 7]))
        s = int(rng.choice([1, 1, 2, 2, 3, 4]))
        dil = int(rng.choice([1, 1, 1, 2, 3]))
        pad = int(rng.integers(0, k * dil // 2 + 2))
        kind = rng.choice(["dense", "dense", "dense", "depthwise", "grouped"])
        if kind == "dense":
            cin, cout, g = int(rng.integers(1, 90)), int(rng.integers(1, 90)), 1
        elif kind == "depthwise":
            cin = cout = g = int(rng.integers(1, 40))
        else:
            g = int(rng.choice([2, 3, 4]))
            cin, cout = g * int(rng.integers(1, 9)), g * int(rng.integers(1, 9))
        h, w = int(rng.integers(1, 24)), int(rng.integers(1, 24))
        n = int(rng.integers(1, 5))
        if (h + 2 * pad - dil * (k - 1) - 1) < 0 or (w + 2 * pad - dil * (k - 1) - 1) < 0:
            continue
        out.append(wl.Layer(f"rnd{len(out)}", n, cin, h, w, cout, k, k, s, pad, dil, g))
    return out


RANDOM_LAYERS = _random_layers(48, 20210204)


@pytest.mark.parametrize("layer", RANDOM_LAYERS, ids=lambda l: f"{l.name}-N{l.N}c{l.Cin}>{l.Cout}h{l.Hin}w{l.Win}k{l.kH}s{l.stride}p{l.pad}d{l.dil}g{l.groups}")
def test_random_descriptors(layer):
    seed = wl.seed_for(6, RANDOM_LAYERS.index(layer))
    rng = np.random.default_rng(seed)
    qX = rng.integers(-127, 128, layer.x_shape).astype(np.int8)
    qW = rng.integers(-127, 128, layer.w_shape).astype(np.int8)
    qG = rng.integers(-127, 128, layer.y_shape).astype(np.int8)
    s_c = (10.0 ** rng.uniform(-4, -1, layer.Cout)).astype(np.float32)
    run_convs_on_codes(layer, qX, qW, qG, 1.5, 0.2, 0.07, s_c)
    dY = wl.make_dY(layer, seed)
    check_quantize_grad(layer, dY, wl.make_state(dY, seed), degenerate=True)
    check_quantize_grad(layer, dY, wl.make_state(dY, seed), mode=daq.ROUND_STOCHASTIC, seed=seed, degenerate=True)
    check_forward(layer, seed)


def _random_special_layers(count, seed):
    """Seeded random descriptors inside the domains of the specialised kernels: 1 x 1 layers at unit stride with up to 256
    output channels (streaming data gradient, every contraction-step count), strided 1 x 1 without padding (zero-filling
    epilogue), 3 x 3 depthwise at stride 1 and 2 with padding 1 and rows a multiple of four (4 x 4 output blocks), with
    ragged channel counts, image sizes and batch sizes."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        kind = rng.choice(["thin1x1", "thin1x1", "s2_1x1", "dw_s1", "dw_s2"])
        n = int(rng.integers(1, 5))
        if kind == "thin1x1":
            cout = int(rng.choice([int(rng.integers(1, 33)), int(rng.integers(33, 65)), int(rng.integers(65, 129)),
                                   int(rng.integers(129, 257))]))
            L = wl.Layer(f"sp{len(out)}", n, int(rng.integers(1, 200)), int(rng.integers(1, 15)), int(rng.integers(1, 15)), cout,
                         1, 1, 1, 0)
        elif kind == "s2_1x1":
            L = wl.Layer(f"sp{len(out)}", n, int(rng.integers(1, 150)), int(rng.integers(2, 20)), int(rng.integers(2, 20)),
                         int(rng.integers(1, 150)), 1, 1, 2, 0)
        else:
            ch = int(rng.integers(1, 48))
            L = wl.Layer(f"sp{len(out)}", n, ch, int(rng.integers(2, 23)), 4 * int(rng.integers(1, 8)), ch, 3, 3,
                         1 if kind == "dw_s1" else 2, 1, 1, ch)
        out.append(L)
    return out


SPECIAL_LAYERS = _random_special_layers(40, 20210205)


@pytest.mark.parametrize("layer", SPECIAL_LAYERS, ids=lambda l: f"{l.name}-N{l.N}c{l.Cin}>{l.Cout}h{l.Hin}w{l.Win}k{l.kH}s{l.stride}g{l.groups}")
def test_random_descriptors_of_the_specialised_kernels(layer):
    seed = wl.seed_for(13, SPECIAL_LAYERS.index(layer))
    rng = np.random.default_rng(seed)
    qX = rng.integers(-127, 128, layer.x_shape).astype(np.int8)
    qW = rng.integers(-127, 128, layer.w_shape).astype(np.int8)
    qG = rng.integers(-127, 128, layer.y_shape).astype(np.int8)
    s_c = (10.0 ** rng.uniform(-4, -1, layer.Cout)).astype(np.float32)
    run_convs_on_codes(layer, qX, qW, qG, 0.9, 0.3, 0.05, s_c)


SCHEDULES = [daq.SCHEDULE_THREE_SWEEPS, daq.SCHEDULE_EARLY_COPY, daq.SCHEDULE_CHANNEL_RESIDENT]


@pytest.mark.parametrize("schedule", SCHEDULES, ids=["three_sweeps", "early_copy", "channel_resident"])
def test_schedules_on_config1_all_modes(schedule):
    """Each schedule of the quantizer asked for explicitly (daq_quantize_grad_ex), on a size where the automatic choice
    would not take the early per-channel copy: wrong class guesses (lambda 0 and 1), both roundings, the clip-rule corners."""
    layer, X, W, dY, st = wl.make_inputs(1)
    check_quantize_grad(layer, dY, st, schedule=schedule)
    check_quantize_grad(layer, dY, np.zeros_like(st), schedule=schedule)
    check_quantize_grad(layer, dY, st, k=1.5, A=0.8, schedule=schedule)
    check_quantize_grad(layer, dY, 10 * st, k=1.5, A=0.8, schedule=schedule)
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=7, schedule=schedule)
    check_quantize_grad(layer, dY, st, lam=0.0, schedule=schedule)
    check_quantize_grad(layer, dY, st, lam=1.0, schedule=schedule)
    for scheme, _ in SCHEMES[1:]:          # the ablation variants keep their three sweeps under either request
        check_quantize_grad(layer, dY, st, scheme=scheme, schedule=schedule)


@pytest.mark.parametrize("schedule", SCHEDULES, ids=["three_sweeps", "early_copy", "channel_resident"])
@pytest.mark.parametrize("layer", ODD_LAYERS, ids=lambda l: l.name)
def test_schedules_on_ragged_shapes(layer, schedule):
    seed = wl.seed_for(15, ODD_LAYERS.index(layer))
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    check_quantize_grad(layer, dY, st, schedule=schedule)
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=99, schedule=schedule)
    check_quantize_grad(layer, dY, st, lam=1.0, schedule=schedule)
    check_quantize_grad(layer, dY, st, lam=0.0, schedule=schedule)


@pytest.mark.parametrize("schedule", SCHEDULES, ids=["three_sweeps", "early_copy", "channel_resident"])
def test_schedules_on_degenerate_channels_and_carried_state(schedule):
    layer = wl.Layer("deg", 2, 4, 8, 8, 6, 3, 3, 1, 1)
    rng = np.random.default_rng(3)
    dY = rng.normal(0, 1e-2, layer.y_shape).astype(np.float32)
    dY[:, 0] = 0.0
    dY[:, 1] = 0.5
    dY[:, 2] = np.float32(1e-38)
    dY[:, 3, 0, 0] = 1e4
    st = np.zeros(6, np.float32)
    check_quantize_grad(layer, dY, st, degenerate=True, schedule=schedule)
    check_quantize_grad(layer, np.zeros_like(dY), st, degenerate=True, schedule=schedule)
    # two iterations through the same state buffer
    layer, X, W, dY, st = wl.make_inputs(1)
    d, _ = descs(layer)
    s1 = t(st.copy())
    daq.quantize_grad_ex(d, t(dY), s1, schedule=schedule)
    b = daq.quantize_grad_ex(d, t(dY), s1, schedule=schedule)
    torch.cuda.synchronize()
    r2 = ref.quantize_grad(dY, ref.quantize_grad(dY, st).s_state)
    close(s1.cpu().numpy(), r2.s_state, "state after two iterations")
    assert np.array_equal(daq.layout_vq(d).unpack(b.vq), r2.vq)


@pytest.mark.parametrize("schedule", SCHEDULES, ids=["three_sweeps", "early_copy", "channel_resident"])
@pytest.mark.parametrize("layer", CONV_LAYERS, ids=lambda l: l.name)
def test_forward_layer_under_each_schedule(layer, schedule):
    """daq_conv_fwd_int8_ex: both layouts of q(X) from one sweep, or one sweep per layout; same bits."""
    check_forward(layer, wl.seed_for(7, CONV_LAYERS.index(layer)), schedule=schedule)


@pytest.mark.parametrize("schedule", [daq.SCHEDULE_AUTO] + SCHEDULES, ids=["auto", "three_sweeps", "early_copy", "channel_resident"])
@pytest.mark.parametrize("layer", [ODD_LAYERS[0], ODD_LAYERS[-2], CONV_LAYERS[9], CONV_LAYERS[11]], ids=lambda l: l.name)
def test_quantizer_on_two_streams(layer, schedule):
    """daq_quantize_grad_split: the launches only the filter gradient needs run on a second stream; same bits as the
    oracle under every schedule, for NHWC and channel-major (depthwise) global copies."""
    seed = wl.seed_for(21, layer.N * 1000 + layer.Cout)
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    side = torch.cuda.Stream()
    check_quantize_grad(layer, dY, st, schedule=schedule, side=side)
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=5, schedule=schedule, side=side)
    check_quantize_grad(layer, dY, st, scheme=daq.SCHEME_MCS, schedule=schedule, side=side)


def test_backward_step_on_two_streams():
    """Algorithm 1 for one layer as a training loop runs it: the quantizer split over two streams, the data gradient
    behind it on the first, the filter gradient on the second, no synchronisation in between - against the same
    three calls on one stream."""
    for cfg, schedule in ((1, daq.SCHEDULE_AUTO), (1, daq.SCHEDULE_THREE_SWEEPS), (2, daq.SCHEDULE_AUTO), (2, daq.SCHEDULE_EARLY_COPY)):
        layer, X, W, dY, st = wl.make_inputs(cfg)
        d, _ = descs(layer)
        f = daq.alloc_fwd(d, dev())
        daq.conv_fwd_int8(d, t(X), t(W), out=f)
        g = t(dY)
        s1, s2 = t(st.copy()), t(st.copy())
        a = daq.quantize_grad_ex(d, g, s1, schedule=schedule, mode=daq.ROUND_STOCHASTIC, seed=3)
        dW_a = daq.conv_bwd_filter_int8(d, f.qx_cnhw, f.s_x, a.vq, a.s_chan)
        dX_a = daq.conv_bwd_data_int8(d, a.qg, a.s_global, f.qw, f.s_w)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        for _ in range(3):   # repeated, so that a missing wait has several chances to show
            out = daq.alloc_quantize_grad(d, dev())
            dW_b = torch.full(d.w_shape, 7.0, device=dev())
            dX_b = torch.full(d.x_shape, 7.0, device=dev())
            s2.copy_(t(st.copy()))
            torch.cuda.synchronize()
            b = daq.quantize_grad_split(d, g, s2, side, schedule=schedule, mode=daq.ROUND_STOCHASTIC, seed=3, out=out)
            daq.conv_bwd_filter_int8(d, f.qx_cnhw, f.s_x, b.vq, b.s_chan, dW=dW_b, stream=side)
            daq.conv_bwd_data_int8(d, b.qg, b.s_global, f.qw, f.s_w, dX=dX_b)
            torch.cuda.synchronize()
            assert torch.equal(dW_a, dW_b) and torch.equal(dX_a, dX_b)
            assert torch.equal(a.vq, b.vq) and torch.equal(a.qg, b.qg) and torch.equal(s1, s2)
            assert torch.equal(a.s_chan, b.s_chan) and torch.equal(a.cls, b.cls) and torch.equal(a.stats, b.stats)


def check_quantize_from_stats(layer, dY, st, k=1.0, A=0.8, lam=0.3, mode=0, seed=0, schedule=daq.SCHEDULE_AUTO, side=None):
    """daq_quantize_grad_from_stats against the oracle taken step by step from the same statistics (Algorithm 1 after
    its first line), and - the statistics being the tensor's own - against the oracle's whole quantizer."""
    d, _ = descs(layer)
    M = float(layer.N * d.Ho * d.Wo)
    g64 = dY.astype(np.float64)
    mx = np.abs(dY).max(axis=(0, 2, 3)).astype(np.float32)
    s1, s2 = g64.sum(axis=(0, 2, 3)), (g64 * g64).sum(axis=(0, 2, 3))   # numpy's summation order, not the oracle's
    mu = s1 / M
    sigma = np.sqrt(np.maximum(s2 / M - mu * mu, 0.0)).astype(np.float32)
    cnt = ref.tail_count(dY, sigma)
    cls = np.array([ref.classify(int(c), M, lam) for c in cnt], np.uint8)
    s_new = np.array([ref.clip_value(int(cls[c]), float(mx[c]), float(st[c]), k, A) for c in range(layer.Cout)], np.float32)
    st_dev = t(st.copy())
    out = daq.alloc_quantize_grad(d, dev())
    out.vq.fill_(55)
    out.qg.fill_(55)
    torch.cuda.synchronize()
    daq.quantize_grad_from_stats(d, t(dY), t(mx), t(s1), t(s2), st_dev, side, daq.SCHEME_DAQ, schedule, k, A, lam, mode, seed,
                                 out=out)
    torch.cuda.synchronize()
    stats = out.stats.cpu().numpy()
    assert np.array_equal(stats[:, 0], mx) and np.array_equal(stats[:, 1], mu.astype(np.float32))
    assert np.array_equal(stats[:, 2], sigma), "sigma from the given sums"
    assert np.array_equal(stats[:, 3], (cnt.astype(np.float64) / M).astype(np.float32)), "tail mass"
    assert np.array_equal(out.cls.cpu().numpy(), cls)
    close(st_dev.cpu().numpy(), s_new, "s_state")
    r = ref.quantize_grad(dY, st, k, A, lam, mode, seed)
    assert r.fragile.sum() == 0 and np.array_equal(r.cls, cls), "seed: the two summation orders must agree on the classes"
    close(out.s_chan.cpu().numpy(), r.s_chan, "s_chan")
    close(out.s_global.cpu().numpy(), [r.s_global], "s_global")
    Lv, Lg = daq.layout_vq(d), daq.layout_qg(d)
    assert np.array_equal(Lv.unpack(out.vq), r.vq) and Lv.padding_is_zero(out.vq), "vq codes"
    assert np.array_equal(Lg.unpack(out.qg), r.qg) and Lg.padding_is_zero(out.qg), "qg codes"


@pytest.mark.parametrize("schedule", [daq.SCHEDULE_AUTO, daq.SCHEDULE_THREE_SWEEPS], ids=["one_sweep", "two_sweeps"])
@pytest.mark.parametrize("layer", [ODD_LAYERS[0], ODD_LAYERS[-2], CONV_LAYERS[9], CONV_LAYERS[11], CONV_LAYERS[2]], ids=lambda l: l.name)
def test_quantizer_with_the_producers_statistics(layer, schedule):
    seed = wl.seed_for(22, layer.N * 1000 + layer.Cout)
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    check_quantize_from_stats(layer, dY, st, schedule=schedule)
    check_quantize_from_stats(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=17, schedule=schedule, side=torch.cuda.Stream())
    check_quantize_from_stats(layer, dY, st, lam=0.0, schedule=schedule)     # wrong guesses of the one-sweep form
    check_quantize_from_stats(layer, dY, st, lam=1.0, k=1.5, schedule=schedule)


def test_producers_statistics_on_config1_and_bad_pointers():
    layer, X, W, dY, st = wl.make_inputs(1)
    check_quantize_from_stats(layer, dY, st)
    check_quantize_from_stats(layer, dY, np.zeros_like(st), mode=daq.ROUND_STOCHASTIC, seed=2 ** 40 + 1)
    d, _ = descs(layer)
    # the ablation rules (checked against the oracle elsewhere) with the same statistics handed over: same bits
    g = t(dY)
    g64 = g.double()
    mx, s1, s2 = g.abs().amax(dim=(0, 2, 3)).contiguous(), g64.sum(dim=(0, 2, 3)).contiguous(), (g64 * g64).sum(dim=(0, 2, 3)).contiguous()
    for scheme, _ in SCHEMES[1:]:
        sa, sb = t(st.copy()), t(st.copy())
        a = daq.quantize_grad_scheme(d, g, sa, scheme, mode=daq.ROUND_STOCHASTIC, seed=9)
        b = daq.quantize_grad_from_stats(d, g, mx, s1, s2, sb, None, scheme, mode=daq.ROUND_STOCHASTIC, seed=9)
        torch.cuda.synchronize()
        assert torch.equal(a.vq, b.vq) and torch.equal(a.qg, b.qg) and torch.equal(sa, sb) and torch.equal(a.s_chan, b.s_chan)
        assert torch.equal(a.cls, b.cls) and torch.equal(a.stats, b.stats) and torch.equal(a.s_global, b.s_global)
    z32, z64 = torch.zeros(layer.Cout + 1, device=dev()), torch.zeros(layer.Cout + 1, dtype=torch.float64, device=dev())
    out = daq.alloc_quantize_grad(d, dev())
    lib = daq.lib()
    import ctypes as C
    opts = daq.QuantizeOpts(daq.SCHEME_DAQ, daq.SCHEDULE_AUTO, 0, 0)
    def call(mxp, s1p, s2p):
        return lib.daq_quantize_grad_from_stats(C.byref(d), t(dY).data_ptr(), mxp, s1p, s2p, t(st.copy()).data_ptr(), 1.0, 0.8, 0.3,
                                                0, 0, C.byref(opts), out.vq.data_ptr(), out.qg.data_ptr(), out.s_chan.data_ptr(),
                                                out.s_global.data_ptr(), out.cls.data_ptr(), out.stats.data_ptr(),
                                                out.workspace.data_ptr(), out.workspace.numel(), None, None)
    assert call(None, z64.data_ptr(), z64.data_ptr()) == daq.ERR_INVALID_ARG
    assert call(z32.data_ptr(), z64.data_ptr() + 4, z64.data_ptr()) == daq.ERR_INVALID_ARG     # misaligned fp64 sums
    torch.cuda.synchronize()


def test_split_quantizer_with_a_single_stream_and_bad_options():
    """side_stream equal to stream: the plain entry point; options are checked as in daq_quantize_grad_ex."""
    layer, X, W, dY, st = wl.make_inputs(1)
    check_quantize_grad(layer, dY, st, mode=daq.ROUND_STOCHASTIC, seed=11, side=torch.cuda.current_stream())
    d, _ = descs(layer)
    with pytest.raises(daq.DaqError) as e:
        daq.quantize_grad_split(d, t(dY), t(st.copy()), torch.cuda.Stream(), schedule=9)
    assert e.value.code == daq.ERR_INVALID_ARG


def test_unknown_schedule_is_refused():
    layer, X, W, dY, st = wl.make_inputs(1)
    d, _ = descs(layer)
    with pytest.raises(daq.DaqError) as e:
        daq.quantize_grad_ex(d, t(dY), t(st.copy()), schedule=4)
    assert e.value.code == daq.ERR_INVALID_ARG
    with pytest.raises(daq.DaqError) as e:
        daq.conv_fwd_int8(d, t(X), t(W), schedule=7)
    assert e.value.code == daq.ERR_INVALID_ARG


@pytest.mark.parametrize("layer", CONV_LAYERS + RANDOM_LAYERS[:16] + SPECIAL_LAYERS[:16], ids=lambda l: l.name)
def test_gradients_with_bf16_results(layer):
    """The optional narrow outputs of both gradients, on every kernel path: the same accumulators and fp32 products,
    stored as bfloat16 (nearest even).  The fp32 products of the two sides are computed by the same operations, so the
    bit patterns must agree with the oracle's rounding of its own fp32 result."""
    d, rd = descs(layer)
    rng = np.random.default_rng(wl.seed_for(5, len(layer.name) + layer.Cin + 7 * layer.Cout))
    qX = rng.integers(-127, 128, layer.x_shape).astype(np.int8)
    qW = rng.integers(-127, 128, layer.w_shape).astype(np.int8)
    qG = rng.integers(-127, 128, layer.y_shape).astype(np.int8)
    s_g, s_w, s_x = 0.03, 0.11, 2.5
    s_c = (10.0 ** rng.uniform(-4, -1, layer.Cout)).astype(np.float32)
    s_g_d, s_w_d, s_x_d = (torch.tensor([v], dtype=torch.float32, device=dev()) for v in (s_g, s_w, s_x))
    qg, qw = t(daq.layout_qg(d).pack(qG)), t(daq.layout_qw(d).pack(d, qW))
    got = torch.full(d.x_shape, float("nan"), dtype=torch.bfloat16, device=dev())
    daq.conv_bwd_data_int8_bf16(d, qg, s_g_d, qw, s_w_d, dX=got)
    vq, qx = t(daq.layout_vq(d).pack(qG)), t(daq.layout_qx_cnhw(d).pack(qX))
    gotW = torch.full(d.w_shape, float("nan"), dtype=torch.bfloat16, device=dev())
    daq.conv_bwd_filter_int8_bf16(d, qx, s_x_d, vq, t(s_c), dW=gotW)
    torch.cuda.synchronize()
    want = ref.conv_bwd_data_int8_bf16(rd, qG, s_g, qW, s_w)
    assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16), want), "dX as bfloat16"
    wantW = ref.conv_bwd_filter_int8_bf16(rd, qX, s_x, qG, s_c)
    assert np.array_equal(gotW.view(torch.int16).cpu().numpy().view(np.uint16), wantW), "dW as bfloat16"


# ------------------------------------------------------------------------------------------------ clip-value search

@pytest.mark.parametrize("layer", [CONV_LAYERS[0], ODD_LAYERS[0], ODD_LAYERS[1], ODD_LAYERS[7], ODD_LAYERS[10],
                                   wl.Layer("cs_big", 16, 8, 28, 28, 70, 3, 3, 1, 1)], ids=lambda l: l.name)
@pytest.mark.parametrize("alpha,J", [(0.0, 64), (0.7, 16), (5.0, 1), (2.5, 37)])
def test_clip_search_against_the_oracle(layer, alpha, J):
    """daq_clip_search: the error table within 1e-9 of the oracle's sequential fp64 sums (the GPU sums in a fixed tree
    order, and its exp may differ from the host library's in the last bit), the chosen clip value exactly that of the
    chosen candidate, and the chosen candidate a minimiser of the ORACLE's table up to that tolerance (where two
    candidates tie to the last bits either is right)."""
    d, _ = descs(layer)
    seed = wl.seed_for(17, len(layer.name) + J)
    dY = wl.make_dY(layer, seed)
    dY[:, 0] = 0.0 if layer.Cout > 2 else dY[:, 0]          # an all-zero channel: every candidate is the zero scale
    assert alpha * np.abs(dY).max() < 600, "the weights must stay finite for the comparison to mean anything"
    err, best_s, best_j = daq.clip_search(d, t(dY), alpha, J)
    torch.cuda.synchronize()
    rerr, rs, rj = ref.clip_search(dY, alpha, J)
    err, best_s, best_j = err.cpu().numpy(), best_s.cpu().numpy(), best_j.cpu().numpy()
    assert np.allclose(err, rerr, rtol=1e-9, atol=0), f"error table: {np.abs(err / np.maximum(rerr, 1e-300) - 1).max():g} off"
    gm = np.abs(dY).max(axis=(0, 2, 3))
    assert np.array_equal(best_s, gm * (best_j.astype(np.float32) / np.float32(J)))
    rows = np.arange(layer.Cout)
    assert np.all(rerr[rows, best_j - 1] <= rerr.min(axis=1) * (1 + 1e-9))
    assert np.all((best_j >= 1) & (best_j <= J))
    same = best_j == rj
    assert same.mean() > 0.99 or layer.Cout < 100 and same.sum() >= layer.Cout - 1


def test_clip_search_refuses_bad_arguments():
    layer = CONV_LAYERS[0]
    d, _ = descs(layer)
    g = torch.zeros(d.y_shape, device=dev())
    for alpha, J in ((1.0, 0), (1.0, 65), (-1.0, 8), (float("nan"), 8)):
        with pytest.raises(daq.DaqError) as e:
            daq.clip_search(d, g, alpha, J)
        assert e.value.code == daq.ERR_INVALID_ARG
