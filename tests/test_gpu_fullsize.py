"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

Whole-tensor oracle runs are out of reach for ResNet-50 / MobileNetV2 layers at N = 64 / 128, so
the check is exact on SAMPLED outputs: the oracle evaluates a few thousand elements of G_X and a few
hundred of G_W one by one from the definition, and the raw int32 accumulators of the GPU must match
bit for bit.

The int8 operands reach the device layouts through the library's own quantizers.  The inputs are
fp32 tensors that hold integers in [-127, 127] with a +-127 in every channel, so every scale is
exactly 127 and every code equals its input (with k*A = 1 the Inverted-T rule returns |g|max as
well): the logical int8 tensors the oracle needs are the inputs themselves.
"""
import numpy as np
import pytest
import torch

from oracle import daq_ref as ref
from paper_2102_04782_amd import binding as daq
from paper_2102_04782_amd import workloads as wl

pytestmark = pytest.mark.gpu

def _distinct_layers():
    """One (config, index) per distinct convolution of ResNet-50 (N = 64) and MobileNetV2 (N = 128): 23 + 34 shapes,
    covering every kernel path at the sizes the network sweep of bench.py times."""
    seen, cases = set(), []
    for config in (4, 5):
        for index, layer in enumerate(wl.config_layers(config)):
            if layer.desc_fields() not in seen:
                seen.add(layer.desc_fields())
                cases.append((config, index))
    return cases


def _codes(shape, gen, device):
    """Integer-valued tensor with a 127 in every channel of axis 1 (and so in the tensor)."""
    q = torch.randint(-127, 128, shape, dtype=torch.int8, device=device, generator=gen)
    q[0, :, 0, 0] = 127
    return q


@pytest.mark.parametrize("config,index", _distinct_layers(), ids=lambda v: str(v))
def test_sampled_outputs_at_full_size(config, index):
    device = torch.device("cuda:0")
    layer = wl.config_layers(config)[index]
    d = daq.ConvDesc.make(*layer.desc_fields())
    rd = ref.ConvDesc(*layer.desc_fields())
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.seed_for(config, index))
    X, G = _codes(d.x_shape, gen, device), _codes(d.y_shape, gen, device)
    W = torch.randint(-127, 128, d.w_shape, dtype=torch.int8, device=device, generator=gen)
    W.view(-1)[0] = 127

    f = daq.conv_fwd_int8(d, X.float(), W.float())
    state = torch.zeros(d.Cout, device=device)
    q = daq.quantize_grad(d, G.float(), state, k=1.0, A=1.0)
    accW = torch.empty(d.w_shape, dtype=torch.int32, device=device)
    accX = torch.empty(d.x_shape, dtype=torch.int32, device=device)
    # the call the benchmark times: both gradients at once
    dW, dX = daq.conv_bwd_int8(d, f.qx_cnhw, f.s_x, q.vq, q.s_chan, q.qg, q.s_global, f.qw, f.s_w, dW_acc=accW, dX_acc=accX)
    # ... and the two separate entry points must give the same bits
    dW1 = daq.conv_bwd_filter_int8(d, f.qx_cnhw, f.s_x, q.vq, q.s_chan)
    dX1 = daq.conv_bwd_data_int8(d, q.qg, q.s_global, f.qw, f.s_w)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW1) and torch.equal(dX, dX1)
    if layer.groups > 1 and layer.groups == layer.Cin == layer.Cout:
        # depthwise: the data gradient from the per-channel copy (all scales are 127 here, so the same bits)
        assert torch.equal(daq.conv_bwd_data_int8_chan(d, q.vq, q.s_chan, f.qw, f.s_w), dX)
    assert f.s_x.item() == 127.0 and f.s_w.item() == 127.0 and q.s_global.item() == 127.0
    assert bool((q.s_chan == 127.0).all())

    rng = np.random.default_rng(wl.seed_for(config, index))
    Xh, Wh, Gh = X.cpu().numpy(), W.cpu().numpy(), G.cpu().numpy()
    ix = rng.choice(accX.numel(), size=min(4096, accX.numel()), replace=False)
    want = ref.conv_bwd_data_acc_at(rd, Gh, Wh, ix)
    ix_d = torch.from_numpy(ix).to(device)
    assert np.array_equal(accX.view(-1)[ix_d].cpu().numpy(), want), "G_X accumulators at sampled positions"
    # all scales are 127: the de-quantized value is the accumulator itself
    assert np.array_equal(dX.view(-1)[ix_d].cpu().numpy(), want.astype(np.float32))

    iw = rng.choice(accW.numel(), size=min(256, accW.numel()), replace=False)
    want = ref.conv_bwd_filter_acc_at(rd, Xh, Gh, iw)
    iw_d = torch.from_numpy(iw).to(device)
    assert np.array_equal(accW.view(-1)[iw_d].cpu().numpy(), want), "G_W accumulators at sampled positions"
    assert np.array_equal(dW.view(-1)[iw_d].cpu().numpy(), want.astype(np.float32))


def _logical_view(L, buf):
    """Strided view (N, C, H, W) of an int8 device buffer in one of the two layouts (unsplit CNHW only)."""
    if L.kind == daq.LAYOUT_NHWC:
        return buf[:L.N * L.H * L.W * L.c_pitch].view(L.N, L.H, L.W, L.c_pitch)[..., :L.C].permute(0, 3, 1, 2)
    assert L.phases_h == 1 and L.phases_w == 1 and L.org_h == 0 and L.org_w == 0
    body = buf.view(L.C, L.chan_pitch)[:, L.lead:L.lead + L.N * L.img_rows * L.row_pitch]
    return body.view(L.C, L.N, L.img_rows, L.row_pitch)[:, :, :L.H, :L.W].permute(1, 0, 2, 3)


def _distinct_gradient_shapes():
    """One (config, index) per distinct gradient tensor (N, Cout, Ho, Wo, and the layout family) of both networks."""
    seen, cases = set(), []
    for config in (4, 5):
        for index, layer in enumerate(wl.config_layers(config)):
            key = (layer.y_shape, layer.groups > 1, layer.kH, layer.stride, layer.pad)
            if key not in seen:
                seen.add(key)
                cases.append((config, index))
    return cases


@pytest.mark.parametrize("config,index", _distinct_gradient_shapes(), ids=lambda v: str(v))
def test_quantize_grad_at_full_size(config, index):
    device = torch.device("cuda:0")
    layer = wl.config_layers(config)[index]
    d = daq.ConvDesc.make(*layer.desc_fields())
    seed = wl.seed_for(config, index)
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    r = ref.quantize_grad(dY, st, want_fragile=True)
    assert r.fragile.sum() == 0, "seed yields a channel whose class flips under a 1-ulp change of sigma"
    st_dev = torch.from_numpy(st.copy()).to(device)
    out = daq.quantize_grad(d, torch.from_numpy(dY).to(device), st_dev)
    torch.cuda.synchronize()
    stats = out.stats.cpu().numpy()
    assert np.array_equal(stats[:, 0], r.stats[:, 0]) and np.array_equal(stats[:, 2], r.stats[:, 2])
    assert np.array_equal(stats[:, 3], r.stats[:, 3])
    assert np.array_equal(out.cls.cpu().numpy(), r.cls)
    assert np.allclose(out.s_chan.cpu().numpy(), r.s_chan, rtol=1e-5, atol=0)
    assert np.allclose(st_dev.cpu().numpy(), r.s_state, rtol=1e-5, atol=0)
    assert abs(out.s_global.item() - r.s_global) <= 1e-5 * r.s_global
    assert torch.equal(_logical_view(daq.layout_vq(d), out.vq), torch.from_numpy(r.vq).to(device)), "vq codes"
    assert torch.equal(_logical_view(daq.layout_qg(d), out.qg), torch.from_numpy(r.qg).to(device)), "qg codes"


@pytest.mark.parametrize("shape,lam", [((64, 32, 92, 92), 1.0), ((64, 32, 92, 92), 0.0), ((64, 16, 130, 130), 1.0),
                                       ((64, 16, 130, 130), 0.3)], ids=str)
def test_quantize_grad_large_tensor_with_wrong_class_guesses(shape, lam):
    """Gradients of 16 M elements and more: the counting pass writes the per-channel copy under a guessed class.
    lambda = 1 (every channel long-tailed) and lambda = 0 (every channel bell-shaped) make half of the guesses
    wrong, so the packing pass has to redo those channels; rows of 92 take the four-pixel stores, rows of 130
    the single-byte ones."""
    device = torch.device("cuda:0")
    n, c, h, w = shape
    layer = wl.Layer("big", n, 8, h, w, c, 1, 1, 1, 0)
    d = daq.ConvDesc.make(*layer.desc_fields())
    seed = wl.seed_for(9, 500 + c + w)
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    r = ref.quantize_grad(dY, st, 1.0, 0.8, lam, want_fragile=False)
    assert lam == 0.3 or len(set(r.cls.tolist())) == 1
    st_dev = torch.from_numpy(st.copy()).to(device)
    out = daq.quantize_grad(d, torch.from_numpy(dY).to(device), st_dev, lam=lam)
    torch.cuda.synchronize()
    assert np.array_equal(out.cls.cpu().numpy(), r.cls)
    assert np.allclose(out.s_chan.cpu().numpy(), r.s_chan, rtol=1e-5, atol=0)
    assert np.allclose(st_dev.cpu().numpy(), r.s_state, rtol=1e-5, atol=0)
    assert torch.equal(_logical_view(daq.layout_vq(d), out.vq), torch.from_numpy(r.vq).to(device)), "vq codes"
    assert torch.equal(_logical_view(daq.layout_qg(d), out.qg), torch.from_numpy(r.qg).to(device)), "qg codes"
    assert daq.layout_vq(d).padding_is_zero(out.vq), "vq padding bytes must be zero"


@pytest.mark.parametrize("scheme", [daq.SCHEME_GQ, daq.SCHEME_GVQ, daq.SCHEME_MCS], ids=["gq", "gvq", "mcs"])
@pytest.mark.parametrize("config", [2, 3])
def test_ablation_schemes_at_benchmark_sizes(config, scheme):
    """The three ablation variants of the quantizer on the benchmark's gradient tensors, whole-tensor against the oracle."""
    device = torch.device("cuda:0")
    layer = wl.config_layers(config)[0]
    d = daq.ConvDesc.make(*layer.desc_fields())
    seed = wl.seed_for(config, 0)
    dY = wl.make_dY(layer, seed)
    st = wl.make_state(dY, seed)
    r = ref.quantize_grad(dY, st, scheme=scheme)
    assert r.fragile.sum() == 0
    st_dev = torch.from_numpy(st.copy()).to(device)
    out = daq.quantize_grad_scheme(d, torch.from_numpy(dY).to(device), st_dev, scheme)
    torch.cuda.synchronize()
    assert np.array_equal(out.stats.cpu().numpy(), r.stats)
    assert np.array_equal(out.cls.cpu().numpy(), r.cls)
    assert np.array_equal(out.s_chan.cpu().numpy(), r.s_chan) and out.s_global.item() == r.s_global
    assert np.array_equal(st_dev.cpu().numpy(), r.s_state)
    Lv, Lg = daq.layout_vq(d), daq.layout_qg(d)
    want_v = torch.from_numpy(r.vq).to(device)
    want_g = torch.from_numpy(r.qg).to(device)
    assert torch.equal(_logical_view(Lv, out.vq), want_v), "vq codes"
    assert torch.equal(_logical_view(Lg, out.qg), want_g), "qg codes"


@pytest.mark.parametrize("config,index", [(2, 0), (4, 3), (4, 12), (5, 0), (5, 1), (5, 3)], ids=str)
def test_bf16_gradient_at_full_size(config, index):
    """daq_quantize_grad_bf16 on full-size gradients (the early per-channel copy, depthwise and strided layouts included):
    every output equals what the fp32 entry point - itself checked against the oracle above - returns for the widened tensor."""
    device = torch.device("cuda:0")
    layer = wl.config_layers(config)[index]
    d = daq.ConvDesc.make(*layer.desc_fields())
    seed = wl.seed_for(config, index)
    dY = torch.from_numpy(wl.make_dY(layer, seed)).to(device).to(torch.bfloat16)
    st = wl.make_state(dY.float().cpu().numpy(), seed)
    s1, s2 = torch.from_numpy(st.copy()).to(device), torch.from_numpy(st.copy()).to(device)
    a = daq.quantize_grad_bf16(d, dY, s1)
    b = daq.quantize_grad(d, dY.float().contiguous(), s2)
    torch.cuda.synchronize()
    Lv, Lg = daq.layout_vq(d), daq.layout_qg(d)
    assert torch.equal(_logical_view(Lv, a.vq), _logical_view(Lv, b.vq)), "vq codes"
    assert torch.equal(_logical_view(Lg, a.qg), _logical_view(Lg, b.qg)), "qg codes"
    assert torch.equal(a.stats, b.stats) and torch.equal(a.cls, b.cls) and torch.equal(a.s_chan, b.s_chan)
    assert torch.equal(s1, s2) and torch.equal(a.s_global, b.s_global)
    if config == 2:   # and against the oracle itself
        r = ref.quantize_grad(dY.float().cpu().numpy(), st)
        assert torch.equal(_logical_view(Lv, a.vq), torch.from_numpy(r.vq).to(device))
        assert torch.equal(_logical_view(Lg, a.qg), torch.from_numpy(r.qg).to(device))
        assert np.array_equal(a.cls.cpu().numpy(), r.cls) and np.array_equal(a.stats.cpu().numpy(), r.stats)
