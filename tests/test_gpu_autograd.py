"""GPU: the Linear / Conv2d layers whose update phase runs through the library (App. B: linear and im2col
convolution shapes of the update GEMM).  dW is compared with the oracle's prune + binary64 GEMM on the same g and
h; dx and db with torch's dense backward.  Holding the seed fixed reproduces the mask (App. B.1 sample reuse)."""
import numpy as np
import pytest
import torch

from gpu_util import DEV, to_host

pytestmark = pytest.mark.gpu


def bits(t):
    return to_host(t.contiguous())


@pytest.mark.parametrize("dtype,nmode,mode,precision", [(torch.bfloat16, "2:4", 0, "native"), (torch.bfloat16, "2:4", 1, "native"),
                                                        (torch.float32, "1:2", 0, "native"), (torch.float32, "2:4", 0, "native"),
                                                        (torch.float32, "2:4", 0, "bf16x3"), (torch.float32, "1:2", 0, "bf16x3")])
def test_linear_update_phase_matches_oracle(oracle, dtype, nmode, mode, precision):
    from paper_2203_10991_amd.autograd import NMConfig, NMLinear
    torch.manual_seed(0)
    B, S, I, O = 3, 37, 72, 40                      # T = 111: padded to 112 inside
    cfg = NMConfig(nm=nmode, mode=mode, seed=5, stream_id=2, precision=precision)
    layer = NMLinear(I, O, bias=True, cfg=cfg, device=DEV, dtype=dtype)
    x = torch.randn(B, S, I, device=DEV, dtype=dtype, requires_grad=True)
    gy = (torch.randn(B, S, O, device=DEV) * torch.exp(2 * torch.randn(B, S, O, device=DEV))).to(dtype)
    layer(x).backward(gy)
    # dense references for the phases the method leaves alone
    ref = torch.nn.Linear(I, O, device=DEV, dtype=dtype)
    ref.load_state_dict(layer.state_dict())
    x2 = x.detach().clone().requires_grad_(True)
    ref(x2).backward(gy)
    assert torch.equal(x.grad, x2.grad) and torch.equal(layer.bias.grad, ref.bias.grad)
    # update phase against the oracle
    g2 = torch.nn.functional.pad(gy.reshape(-1, O), (0, 0, 0, 1))
    h2 = torch.nn.functional.pad(x.detach().reshape(-1, I), (0, 0, 0, 1))
    oprune = oracle.prune_1of2 if nmode == "1:2" else (oracle.prune_2of4_approx if mode else oracle.prune_2of4)
    ov, om, _ = oprune(bits(g2), 5, 2)
    want, wabs = oracle.update_gemm(ov, om, bits(h2))
    got = layer.weight.grad.double().cpu().numpy()
    tol = 1e-5 if dtype == torch.float32 else 1e-2          # (bf16: dW itself is rounded to bf16 by the layer)
    assert (np.abs(got - want) <= tol * np.maximum(wabs, np.abs(want))).all()
    # same seed -> same gradient; next seed (after reuse_every steps) -> another mask
    w1 = layer.weight.grad.clone()
    layer.weight.grad = None
    layer(x).backward(gy)
    assert torch.equal(w1, layer.weight.grad)
    cfg.advance()
    layer.weight.grad = None
    layer(x).backward(gy)
    assert not torch.equal(w1, layer.weight.grad)


@pytest.mark.parametrize("dtype,nmode,mode", [(torch.bfloat16, "2:4", 0), (torch.bfloat16, "1:2", 0), (torch.float32, "2:4", 1)])
def test_linear_relu_fuses_the_activation_backward_with_the_prune(oracle, dtype, nmode, mode):
    """NMLinearReLU: g = gy * relu'(z) and its prune come from one library call (eq. (2)'s elementwise step as the
    producer).  dW against the oracle's producer step + prune + binary64 GEMM; dx, db against torch's dense backward of
    relu(linear(x))."""
    from paper_2203_10991_amd.autograd import NMConfig, NMLinearReLU
    torch.manual_seed(3)
    B, S, I, O = 2, 53, 48, 64                      # T = 106: padded to 112 inside
    cfg = NMConfig(nm=nmode, mode=mode, seed=11, stream_id=4)
    layer = NMLinearReLU(I, O, bias=True, cfg=cfg, device=DEV, dtype=dtype)
    x = torch.randn(B, S, I, device=DEV, dtype=dtype, requires_grad=True)
    gy = (torch.randn(B, S, O, device=DEV) * torch.exp(2 * torch.randn(B, S, O, device=DEV))).to(dtype)
    y = layer(x)
    y.backward(gy)
    ref = torch.nn.Linear(I, O, device=DEV, dtype=dtype)
    ref.load_state_dict(layer.state_dict())
    x2 = x.detach().clone().requires_grad_(True)
    y2 = torch.relu(ref(x2))
    y2.backward(gy)
    assert torch.equal(y, y2)
    assert torch.equal(x.grad, x2.grad) and torch.equal(layer.bias.grad, ref.bias.grad)
    # update phase against the oracle
    pad = (0, 0, 0, 6)
    u2 = torch.nn.functional.pad(gy.reshape(-1, O), pad)
    d2 = torch.nn.functional.pad((y.detach().reshape(-1, O) > 0).to(dtype), pad)
    h2 = torch.nn.functional.pad(x.detach().reshape(-1, I), pad)
    g2 = oracle.act_backward(bits(u2), bits(d2))
    oprune = oracle.prune_1of2 if nmode == "1:2" else (oracle.prune_2of4_approx if mode else oracle.prune_2of4)
    ov, om, _ = oprune(g2, 11, 4)
    want, wabs = oracle.update_gemm(ov, om, bits(h2))
    got = layer.weight.grad.double().cpu().numpy()
    tol = 1e-5 if dtype == torch.float32 else 1e-2          # (bf16: dW itself is rounded to bf16 by the layer)
    assert (np.abs(got - want) <= tol * np.maximum(wabs, np.abs(want))).all()


def test_conv2d_update_phase_matches_oracle(oracle):
    from paper_2203_10991_amd.autograd import NMConfig, NMConv2d
    torch.manual_seed(1)
    N, C, H, W, O, k = 4, 8, 10, 10, 16, 3              # I = C*k*k = 72, T = N*H*W = 400
    conv = NMConv2d(C, O, k, padding=1, bias=True, cfg=NMConfig(nm="2:4", seed=9, stream_id=1), device=DEV)
    x = torch.relu(torch.randn(N, C, H, W, device=DEV)).requires_grad_(True)
    gy = torch.randn(N, O, H, W, device=DEV) * torch.exp(2 * torch.randn(N, O, H, W, device=DEV))
    conv(x).backward(gy)
    ref = torch.nn.Conv2d(C, O, k, padding=1, device=DEV)
    ref.load_state_dict(conv.state_dict())
    x2 = x.detach().clone().requires_grad_(True)
    ref(x2).backward(gy)
    assert torch.allclose(x.grad, x2.grad, rtol=1e-4, atol=1e-4) and torch.allclose(conv.bias.grad, ref.bias.grad, rtol=1e-5, atol=1e-4)
    cols = torch.nn.functional.unfold(x.detach(), (k, k), padding=1).transpose(1, 2).reshape(-1, C * k * k)
    g2 = gy.reshape(N, O, -1).transpose(1, 2).reshape(-1, O)
    ov, om, _ = oracle.prune_2of4(bits(g2), 9, 1)
    want, wabs = oracle.update_gemm(ov, om, bits(cols))
    got = conv.weight.grad.reshape(O, -1).double().cpu().numpy()
    assert (np.abs(got - want) <= 1e-5 * wabs + 1e-30).all()
    # the estimate is unbiased: the mean over seeds approaches the dense weight gradient
    acc = torch.zeros_like(conv.weight)
    n = 200
    for s in range(n):
        conv.cfg.seed = 100 + s
        conv.weight.grad = None
        conv(x).backward(gy)
        acc += conv.weight.grad
    dense = ref.weight.grad
    err = (acc / n - dense).norm() / dense.norm()
    one = (conv.weight.grad - dense).norm() / dense.norm()
    print(f"conv dW: one draw off by {one:.3f}, mean of {n} draws off by {err:.3f}", flush=True)
    assert err < 3.0 * one / np.sqrt(n) + 1e-3


def test_conv2d_bf16_update_phase_without_im2col(oracle):
    """bf16, 3x3, stride 1, padding 1: the layer prunes on the zero-padded channels-last grid and multiplies row-shifted
    views of the activations; the oracle does the same from its own definitions"""
    from paper_2203_10991_amd.autograd import NMConfig, NMConv2d, padded_rows
    torch.manual_seed(2)
    N, C, H, W, O, k = 3, 16, 9, 10, 24, 3
    conv = NMConv2d(C, O, k, padding=1, bias=False, cfg=NMConfig(nm="2:4", seed=4, stream_id=3), device=DEV, dtype=torch.bfloat16)
    x = torch.relu(torch.randn(N, C, H, W, device=DEV)).to(torch.bfloat16).requires_grad_(True)
    gy = (torch.randn(N, O, H, W, device=DEV) * torch.exp(2 * torch.randn(N, O, H, W, device=DEV))).to(torch.bfloat16)
    conv(x).backward(gy)
    xr, wp = padded_rows(x.detach(), 1)
    gr, _ = padded_rows(gy, 1)
    rows = xr.shape[0]
    T = (rows + 15) // 16 * 16
    margin = wp + 1
    x_full = np.zeros((T + 2 * margin, C), dtype=np.uint16)
    x_full[margin:margin + rows] = bits(xr)
    g2 = np.zeros((T, O), dtype=np.uint16)
    g2[:rows] = bits(gr)
    ov, om, _ = oracle.prune_2of4(g2, 4, 3)
    shifts = [(ky - 1) * wp + (kx - 1) for ky in range(k) for kx in range(k)]
    want, wabs = oracle.update_gemm_shifted(ov, om, x_full, margin, shifts)
    want = want.reshape(O, k, k, C).transpose(0, 3, 1, 2)
    wabs = wabs.reshape(O, k, k, C).transpose(0, 3, 1, 2)
    got = conv.weight.grad.double().cpu().numpy()
    assert (np.abs(got - want) <= 1e-2 * np.maximum(wabs, np.abs(want)) + 1e-30).all()
    # dx is torch's dense backward
    ref = torch.nn.Conv2d(C, O, k, padding=1, bias=False, device=DEV, dtype=torch.bfloat16)
    ref.load_state_dict(conv.state_dict())
    x2 = x.detach().clone().requires_grad_(True)
    ref(x2).backward(gy)
    assert torch.allclose(x.grad.float(), x2.grad.float(), rtol=2e-2, atol=2e-2 * float(x2.grad.float().abs().max()))


def test_training_with_pruned_update_phase_tracks_dense_training():
    """A small teacher-student regression trained with SGD: with MVUE 2:4 in the update phase of every layer the loss
    follows the dense run (the weight gradients differ from the dense ones at every step but are unbiased, Sec. 3)."""
    from paper_2203_10991_amd.autograd import NMConfig, NMLinear
    torch.manual_seed(0)
    D, Hd, O, B = 64, 128, 32, 512
    teacher = torch.nn.Sequential(torch.nn.Linear(D, Hd), torch.nn.Tanh(), torch.nn.Linear(Hd, O)).to(DEV)
    for p in teacher.parameters():
        p.requires_grad_(False)

    def make(student_cls):
        torch.manual_seed(1)
        cfgs = [NMConfig(nm="2:4", seed=100, stream_id=i) for i in range(2)]
        if student_cls is NMLinear:
            net = torch.nn.Sequential(NMLinear(D, Hd, cfg=cfgs[0]), torch.nn.Tanh(), NMLinear(Hd, O, cfg=cfgs[1])).to(DEV)
        else:
            net = torch.nn.Sequential(torch.nn.Linear(D, Hd), torch.nn.Tanh(), torch.nn.Linear(Hd, O)).to(DEV)
        return net, cfgs

    def train(net, cfgs, steps=300):
        opt = torch.optim.SGD(net.parameters(), lr=0.05)
        gen = torch.Generator(device=DEV).manual_seed(7)
        losses = []
        for _ in range(steps):
            x = torch.randn(B, D, device=DEV, generator=gen)
            loss = torch.nn.functional.mse_loss(net(x), teacher(x))
            opt.zero_grad()
            loss.backward()
            opt.step()
            for c in cfgs:
                c.advance()
            losses.append(float(loss.detach()))
        return losses

    dense_net, _ = make(torch.nn.Linear)
    nm_net, cfgs = make(NMLinear)
    assert all(torch.equal(a, b) for a, b in zip(dense_net.state_dict().values(), nm_net.state_dict().values()))
    ld = train(dense_net, [])
    ln = train(nm_net, cfgs)
    first, last_d, last_n = sum(ld[:10]) / 10, sum(ld[-20:]) / 20, sum(ln[-20:]) / 20
    print(f"loss: start {first:.4f}, dense end {last_d:.4f}, MVUE 2:4 end {last_n:.4f}", flush=True)
    assert last_d < 0.5 * first                       # the task is learnable
    assert last_n < 0.5 * first and last_n < 1.5 * last_d + 1e-3


@pytest.mark.parametrize("nmode", ["2:4", "1:2"])
def test_linear_q8_update_phase_matches_oracle(oracle, nmode):
    """precision="q8": scales, the e4m3 cast of the activations, prune and GEMM all in the library; the oracle's own
    scale rule, cast and 8-bit path check them"""
    from paper_2203_10991_amd.autograd import NMConfig, NMLinear
    torch.manual_seed(3)
    T, I, O = 160, 48, 40
    layer = NMLinear(I, O, bias=False, cfg=NMConfig(nm=nmode, seed=6, stream_id=1, precision="q8"), device=DEV, dtype=torch.bfloat16)
    x = torch.randn(T, I, device=DEV).to(torch.bfloat16).requires_grad_(True)
    gy = (torch.randn(T, O, device=DEV) * torch.exp(2 * torch.randn(T, O, device=DEV))).to(torch.bfloat16)
    layer(x).backward(gy)
    sg, sh = oracle.pow2_scale(bits(gy), 57344.0 / (4.0 if nmode == "2:4" else 2.0)), oracle.pow2_scale(bits(x.detach()), 448.0)
    h8 = oracle.cast_e4m3(bits(x.detach()), sh)
    ov, om = oracle.prune_2of4_q8(bits(gy), 6, 1, 0, sg) if nmode == "2:4" else oracle.prune_1of2_q8(bits(gy), 6, 1, sg)
    want, wabs = oracle.update_gemm_q8(ov, om, h8, alpha=1.0 / (sg * sh))
    got = layer.weight.grad.double().cpu().numpy()
    assert (np.abs(got - want) <= 1e-2 * np.maximum(wabs, np.abs(want)) + 1e-30).all()      # (dW is rounded to bf16 by the layer)
    # and it estimates the dense weight gradient: relative error of one draw well below 1
    dense = gy.float().t() @ x.detach().float()
    rel = float((layer.weight.grad.float() - dense).norm() / dense.norm())
    print(f"q8 update phase: one draw off the dense gradient by {rel:.3f}", flush=True)
    assert rel < 0.8


def test_conv2d_q8_update_phase_without_im2col(oracle):
    """precision="q8" on a 3x3 'same' convolution: the layer's padded grids and scales, then the oracle's 8-bit shifted GEMM"""
    from paper_2203_10991_amd.autograd import NMConfig, NMConv2d, padded_rows
    torch.manual_seed(5)
    N, C, H, W, O, k = 2, 16, 8, 9, 24, 3
    conv = NMConv2d(C, O, k, padding=1, bias=False, cfg=NMConfig(nm="2:4", seed=8, stream_id=2, precision="q8"), device=DEV,
                    dtype=torch.bfloat16)
    x = torch.relu(torch.randn(N, C, H, W, device=DEV)).to(torch.bfloat16).requires_grad_(True)
    gy = (torch.randn(N, O, H, W, device=DEV) * torch.exp(2 * torch.randn(N, O, H, W, device=DEV))).to(torch.bfloat16)
    conv(x).backward(gy)
    xr, wp = padded_rows(x.detach(), 1)
    gr, _ = padded_rows(gy, 1)
    rows = xr.shape[0]
    T = (rows + 31) // 32 * 32
    margin = wp + 1
    x_full = torch.zeros((T + 2 * margin, C), dtype=torch.bfloat16, device=DEV)
    x_full[margin:margin + rows] = xr
    g2 = torch.zeros((T, O), dtype=torch.bfloat16, device=DEV)
    g2[:rows] = gr
    sg, sh = oracle.pow2_scale(bits(g2), 57344.0 / 4.0), oracle.pow2_scale(bits(x_full), 448.0)
    x8 = oracle.cast_e4m3(bits(x_full), sh)
    ov, om = oracle.prune_2of4_q8(bits(g2), 8, 2, 0, sg)
    shifts = [(ky - 1) * wp + (kx - 1) for ky in range(k) for kx in range(k)]
    want, wabs = oracle.update_gemm_q8_shifted(ov, om, x8, margin, shifts, alpha=1.0 / (sg * sh))
    want = want.reshape(O, k, k, C).transpose(0, 3, 1, 2)
    wabs = wabs.reshape(O, k, k, C).transpose(0, 3, 1, 2)
    got = conv.weight.grad.double().cpu().numpy()
    assert (np.abs(got - want) <= 1e-2 * np.maximum(wabs, np.abs(want)) + 1e-30).all()


def test_drop_in_layers_draw_fresh_samples_on_streams_of_their_own():
    """layers that are given no configuration: distinct random streams, and the samples move on after every backward
    pass without any call from the training loop"""
    from paper_2203_10991_amd.autograd import NMLinear
    torch.manual_seed(1)
    a, b = NMLinear(32, 16, device=DEV), NMLinear(32, 16, device=DEV)
    assert a.cfg.stream_id != b.cfg.stream_id and a.cfg.auto_advance
    b.load_state_dict(a.state_dict())
    x = torch.randn(64, 32, device=DEV)
    gy = torch.randn(64, 16, device=DEV) * torch.exp(torch.randn(64, 16, device=DEV))
    a(x).backward(gy); b(x).backward(gy)
    assert not torch.equal(a.weight.grad, b.weight.grad)              # same tensors, different streams
    first = a.weight.grad.clone()
    a.weight.grad = None
    a(x).backward(gy)
    assert a.cfg.step == 2 and not torch.equal(first, a.weight.grad)  # the second iteration drew new samples
