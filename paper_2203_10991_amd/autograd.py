"""Linear and Conv2d layers whose UPDATE phase runs through libnm_mvue.

Only the weight-gradient GEMM dW = g^T h (eq. (3)) sees the pruned gradient; the forward GEMM (eq. (1)) and the
backward GEMM that propagates g (eq. (2)) are torch's dense ones, as in the paper (Table 1: the neural-gradient
column accelerates the update phase only).  The random source is a pure function of (seed, stream_id, block),
so holding `seed` fixed for `reuse_every` iterations is the sample reuse of App. B.1 (up to 50 iterations
without loss) at no extra cost.

There is no fallback: tensors must live on the GPU and the HIP library must be built.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch
import torch.nn.functional as F

from . import api


@dataclass
class NMConfig:
    """How a layer prunes its neural gradient in the update phase."""
    nm: str = "2:4"            # "1:2" (Sec. 4.1) or "2:4"
    mode: int = 0              # 2:4 only: 0 = optimal MVUE (Sec. 4.2), 1 = approx-MVUE (Sec. 4.4)
    seed: int = 0              # base seed of the run
    stream_id: int = 0         # one per layer: independent random streams
    reuse_every: int = 1       # iterations that share one set of random samples (App. B.1)
    # "native": the tensors' own dtype; "q8": e5m2 kept values (stochastic rounding) and e4m3 activations on the 8-bit
    # sparse MFMA (Sec. 5, 8-bit rows); "bf16x3": float32 tensors, the update GEMM through three bf16 terms per value
    # on the sparse 16-bit path
    precision: str = "native"
    step: int = 0              # iteration counter; advance() once per optimizer step
    # True: the layer that owns this configuration advances `step` itself after every backward pass (the default
    # configuration a layer makes for itself: a drop-in layer then draws fresh samples every `reuse_every`
    # iterations without any call from the training loop).  False: the caller calls advance() once per iteration,
    # e.g. when several layers share one configuration object.
    auto_advance: bool = False

    def current_seed(self) -> int:
        return self.seed + self.step // max(1, self.reuse_every)

    def advance(self) -> None:
        self.step += 1


_next_stream_id = 0


def _own_config() -> NMConfig:
    """The configuration of a layer that was given none: a random stream of its own (stream ids count up over the
    layers of the process) that moves on by itself after every backward pass."""
    global _next_stream_id
    cfg = NMConfig(stream_id=_next_stream_id, auto_advance=True)
    _next_stream_id += 1
    return cfg


def _update_gemm(g2: torch.Tensor, h2: torch.Tensor, cfg: NMConfig) -> torch.Tensor:
    """dW[O x I] (binary32) = theta(g2)^T h2 for g2 [T x O], h2 [T x I]; T is padded with zero rows to a multiple of 16."""
    if not (g2.is_cuda and h2.is_cuda):
        raise RuntimeError("the N:M update phase runs on the GPU only (no CPU fallback)")
    T, O = g2.shape
    I = h2.shape[1]
    if O % 8 or I % 8:
        raise ValueError(f"out_features={O} and the reduction width {I} must be multiples of 8")
    if g2.dtype != h2.dtype or g2.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("g and h must both be float32 or both bfloat16")
    pad = (-T) % 16
    if pad:                                   # zero rows prune to zeros and add nothing to dW
        g2 = F.pad(g2, (0, 0, 0, pad))
        h2 = F.pad(h2, (0, 0, 0, pad))
    g2, h2 = g2.contiguous(), h2.contiguous()
    if cfg.precision == "q8":
        return _update_gemm_q8(g2, h2, cfg)
    if cfg.nm == "1:2":
        vals, meta, _ = api.mvue_prune_1of2(g2, seed=cfg.current_seed(), stream_id=cfg.stream_id)
    elif cfg.nm == "2:4":
        vals, meta, _ = api.mvue_prune_2of4(g2, seed=cfg.current_seed(), stream_id=cfg.stream_id, mode=cfg.mode)
    else:
        raise ValueError(f"unknown N:M pattern {cfg.nm!r}")
    if cfg.precision == "bf16x3" and g2.dtype != torch.float32:
        raise TypeError('precision="bf16x3" is a mode for float32 tensors')
    return api.nm_update_gemm(vals, meta, h2, f32_as_bf16x3=cfg.precision == "bf16x3")


def padded_rows(t_nchw: torch.Tensor, pad: int):
    """[N, C, H, W] -> the zero-padded channels-last grid flattened to rows: ([N*(H+2p)*(W+2p), C], W+2p)"""
    g = F.pad(t_nchw.permute(0, 2, 3, 1), (0, 0, pad, pad, pad, pad))
    return g.reshape(-1, g.shape[-1]), g.shape[2]


def _conv_update_shifted(gy: torch.Tensor, x: torch.Tensor, k: int, cfg: NMConfig) -> torch.Tensor:
    """Weight gradient [O, C, k, k] (binary32) of a k x k, stride-1, 'same' convolution without an im2col matrix:
    gradient and activation live on the zero-padded channels-last grid, kernel tap (ky, kx) is a row shift of the
    activation rows (nm_update_gemm_shifted).  The N:M blocks run along the rows of that padded grid."""
    if not (gy.is_cuda and x.is_cuda):
        raise RuntimeError("the N:M update phase runs on the GPU only (no CPU fallback)")
    pad = k // 2
    xr, wp = padded_rows(x, pad)
    gr, _ = padded_rows(gy, pad)
    rows, C = xr.shape
    O = gr.shape[1]
    q8 = cfg.precision == "q8"
    T = (rows + 31) // 32 * 32 if q8 else (rows + 15) // 16 * 16
    margin = pad * wp + pad
    x_full = torch.zeros((T + 2 * margin, C), dtype=x.dtype, device=x.device)
    x_full[margin:margin + rows] = xr
    g2 = torch.zeros((T, O), dtype=gy.dtype, device=gy.device)
    g2[:rows] = gr
    shifts = [(ky - pad) * wp + (kx - pad) for ky in range(k) for kx in range(k)]
    if q8:
        # scales and the e4m3 cast are the library's: the scale records stay in device memory (no host read-back)
        sg, sh = api.nm_q8_scale(g2, 57344.0 / 4.0), api.nm_q8_scale(x_full, 448.0)
        x8 = api.nm_cast_e4m3(x_full, sh)
        v8, m32 = api.mvue_prune_2of4_q8(g2, seed=cfg.current_seed(), stream_id=cfg.stream_id, mode=cfg.mode, scale=sg)
        dW = api.nm_update_gemm_q8_shifted(v8, m32, x8, margin, shifts, alpha=(sg, sh))
    else:
        vals, meta, _ = api.mvue_prune_2of4(g2, seed=cfg.current_seed(), stream_id=cfg.stream_id, mode=cfg.mode)
        dW = api.nm_update_gemm_shifted(vals, meta, x_full, margin, shifts)          # [O, (ky, kx, c)]
    return dW.reshape(O, k, k, C).permute(0, 3, 1, 2).contiguous()


def _update_gemm_q8(g2: torch.Tensor, h2: torch.Tensor, cfg: NMConfig) -> torch.Tensor:
    """The 8-bit update phase, all of it in the library: per-tensor power-of-two scales from the current maxima (a kept
    value is at most the sum of its block's magnitudes, hence the factor 4 or 2) as device-side records, the e4m3 cast
    of the activations, the prune and the GEMM.  No value returns to the host."""
    if cfg.nm not in ("2:4", "1:2"):
        raise ValueError(f"unknown N:M pattern {cfg.nm!r}")
    T, O = g2.shape
    I = h2.shape[1]
    if I % 16:
        raise ValueError(f"the 8-bit update GEMM needs a reduction width that is a multiple of 16, got {I}")
    pad = (-T) % 32
    if pad:
        g2 = F.pad(g2, (0, 0, 0, pad))
        h2 = F.pad(h2, (0, 0, 0, pad))
    g2, h2 = g2.contiguous(), h2.contiguous()
    sg = api.nm_q8_scale(g2, 57344.0 / (4.0 if cfg.nm == "2:4" else 2.0))    # (1:2: the sum of a pair's magnitudes)
    sh = api.nm_q8_scale(h2, 448.0)
    h8 = api.nm_cast_e4m3(h2, sh)
    if cfg.nm == "1:2":
        v8, m32 = api.mvue_prune_1of2_q8(g2, seed=cfg.current_seed(), stream_id=cfg.stream_id, scale=sg)
    else:
        v8, m32 = api.mvue_prune_2of4_q8(g2, seed=cfg.current_seed(), stream_id=cfg.stream_id, mode=cfg.mode, scale=sg)
    return api.nm_update_gemm_q8(v8, m32, h8, alpha=(sg, sh))


class _NMLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, cfg):
        ctx.save_for_backward(x, weight)
        ctx.cfg, ctx.has_bias = cfg, bias is not None
        return F.linear(x, weight, bias)

    @staticmethod
    def backward(ctx, gy):
        x, weight = ctx.saved_tensors
        dx = gy @ weight if ctx.needs_input_grad[0] else None                     # backward phase: dense (eq. (2))
        dW = None
        if ctx.needs_input_grad[1]:
            dW = _update_gemm(gy.reshape(-1, gy.shape[-1]), x.reshape(-1, x.shape[-1]), ctx.cfg).to(weight.dtype)
        db = gy.reshape(-1, gy.shape[-1]).sum(0) if ctx.has_bias and ctx.needs_input_grad[2] else None
        if ctx.cfg.auto_advance:
            ctx.cfg.advance()
        return dx, dW, db, None


class NMLinear(torch.nn.Linear):
    """torch.nn.Linear whose weight gradient is computed from the MVUE N:M pruned neural gradient."""

    def __init__(self, in_features: int, out_features: int, bias: bool = True, cfg: Optional[NMConfig] = None, **kw):
        super().__init__(in_features, out_features, bias=bias, **kw)
        self.cfg = cfg or _own_config()

    def forward(self, x):
        return _NMLinearFn.apply(x, self.weight, self.bias, self.cfg)


class _NMLinearReLUFn(torch.autograd.Function):
    """y = relu(x W^T + b).  In the backward pass the neural gradient of the linear part, g = gy * relu'(z) (the
    elementwise step of eq. (2)), is formed, written dense and pruned in ONE pass by the library
    (mvue_prune_*_producer): g is never read back for the prune.  dx and db use the dense g, as in the paper."""

    @staticmethod
    def forward(ctx, x, weight, bias, cfg):
        y = F.relu(F.linear(x, weight, bias))
        ctx.save_for_backward(x, weight, y)               # relu'(z) = [y > 0]
        ctx.cfg, ctx.has_bias = cfg, bias is not None
        return y

    @staticmethod
    def backward(ctx, gy):
        x, weight, y = ctx.saved_tensors
        cfg = ctx.cfg
        O = weight.shape[0]
        u2 = gy.reshape(-1, O)
        d2 = (y.reshape(-1, O) > 0).to(gy.dtype)
        h2 = x.reshape(-1, x.shape[-1])
        T = u2.shape[0]
        fused = (cfg.precision == "native" and cfg.nm in ("1:2", "2:4") and u2.is_cuda and O % 8 == 0 and h2.shape[1] % 8 == 0
                 and u2.dtype == h2.dtype and u2.dtype in (torch.float32, torch.bfloat16) and ctx.needs_input_grad[1])
        if fused:
            pad = (-T) % 16
            if pad:                                       # zero rows prune to zeros and add nothing to dW
                u2, d2, h2 = F.pad(u2, (0, 0, 0, pad)), F.pad(d2, (0, 0, 0, pad)), F.pad(h2, (0, 0, 0, pad))
            g2, vals, meta = api.mvue_prune_producer(u2.contiguous(), d2.contiguous(), nm=cfg.nm, seed=cfg.current_seed(),
                                                     stream_id=cfg.stream_id, mode=cfg.mode)
            dW = api.nm_update_gemm(vals, meta, h2.contiguous()).to(weight.dtype)
            g2 = g2[:T]
        else:                                             # 8-bit and three-term modes: separate product, then the usual path
            g2 = u2 * d2
            dW = _update_gemm(g2, h2, cfg).to(weight.dtype) if ctx.needs_input_grad[1] else None
        dx = (g2 @ weight).reshape(x.shape) if ctx.needs_input_grad[0] else None
        db = g2.sum(0) if ctx.has_bias and ctx.needs_input_grad[2] else None
        if cfg.auto_advance:
            cfg.advance()
        return dx, dW, db, None


class NMLinearReLU(torch.nn.Linear):
    """Linear followed by ReLU as one module, so that the activation's backward and the prune of the neural gradient
    are one kernel (the prune fused into the producer of g_l, eq. (2))."""

    def __init__(self, in_features: int, out_features: int, bias: bool = True, cfg: Optional[NMConfig] = None, **kw):
        super().__init__(in_features, out_features, bias=bias, **kw)
        self.cfg = cfg or _own_config()

    def forward(self, x):
        return _NMLinearReLUFn.apply(x, self.weight, self.bias, self.cfg)


class _NMConv2dFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, stride, padding, dilation, cfg):
        ctx.save_for_backward(x, weight)
        ctx.conv = (stride, padding, dilation)
        ctx.cfg, ctx.has_bias = cfg, bias is not None
        return F.conv2d(x, weight, bias, stride, padding, dilation)

    @staticmethod
    def backward(ctx, gy):
        x, weight = ctx.saved_tensors
        stride, padding, dilation = ctx.conv
        dx = None
        if ctx.needs_input_grad[0]:
            dx = torch.nn.grad.conv2d_input(x.shape, weight, gy, stride, padding, dilation)
        dW = None
        if ctx.needs_input_grad[1]:
            O, C, kh, kw = weight.shape
            same = (kh == kw and kh % 2 == 1 and tuple(stride) == (1, 1) and tuple(dilation) == (1, 1)
                    and tuple(padding) == (kh // 2, kw // 2))
            cmul = 16 if ctx.cfg.precision == "q8" else 8
            if same and x.dtype == torch.bfloat16 and ctx.cfg.nm == "2:4" and C % cmul == 0 and O % 8 == 0 and kh * kw <= 32:
                dW = _conv_update_shifted(gy, x, kh, ctx.cfg).to(weight.dtype)
            else:
                # im2col (App. B: the convolution's update GEMM reduces over batch x output positions):
                # h [N*L, C*kh*kw], g [N*L, O]
                cols = F.unfold(x, (kh, kw), dilation=dilation, padding=padding, stride=stride)      # [N, C*kh*kw, L]
                h2 = cols.transpose(1, 2).reshape(-1, C * kh * kw)
                g2 = gy.reshape(gy.shape[0], O, -1).transpose(1, 2).reshape(-1, O)
                dW = _update_gemm(g2, h2, ctx.cfg).reshape(O, C, kh, kw).to(weight.dtype)
        db = gy.sum((0, 2, 3)) if ctx.has_bias and ctx.needs_input_grad[2] else None
        if ctx.cfg.auto_advance:
            ctx.cfg.advance()
        return dx, dW, db, None, None, None, None


class NMConv2d(torch.nn.Conv2d):
    """torch.nn.Conv2d (groups = 1, zero padding) whose weight gradient comes from the pruned neural gradient.

    bf16, odd square kernel, stride 1, 'same' padding, MVUE 2:4: no im2col matrix is built (row-shifted views of the
    padded activation grid); anything else goes through an explicit im2col matrix."""

    def __init__(self, *args, cfg: Optional[NMConfig] = None, **kw):
        super().__init__(*args, **kw)
        if self.groups != 1 or self.padding_mode != "zeros" or isinstance(self.padding, str):
            raise ValueError("NMConv2d supports groups=1 with numeric zero padding")
        self.cfg = cfg or _own_config()

    def forward(self, x):
        return _NMConv2dFn.apply(x, self.weight, self.bias, self.stride, self.padding, self.dilation, self.cfg)
