"""torch.autograd glue over the C ABI: a linear map Z = X W whose forward product and
both gradients are the library's quantized matmuls (Methodology: forward and
backward pass of a layer).  Nothing is computed here; the functions marshal
tensors into hdqt_layer_fwd / hdqt_layer_bwd and hand the results to autograd.

The activation is not kept in fp32 for the backward pass: hdqt_layer_fwd leaves
X's codes along the batch dimension (what the weight gradient contracts over)
in a byte buffer one eighth the size of X at 4 bits.
"""
from dataclasses import dataclass, field
from typing import Optional

import torch

from . import binding as B


@dataclass
class LayerConfig:
    """Quantization of one layer's three matmuls.  The defaults are the benchmark
    configurations' setting: 4-bit codes, Hadamard block 64, 8-bit accumulators over
    tiles of 32, the gradient G rounded stochastically in both backward matmuls and
    everything else to nearest.  The paper's own backward setting (Methodology,
    stochastic-rounding paragraph; Fig. 2 ablation) also rounds the activation
    stochastically in the weight-gradient matmul: `stochastic_act=True`."""
    had_block: int = 64
    bits: int = 4
    acc_bits: int = 8
    s: int = 32
    seed: int = 0
    layer_id: int = 0
    clip_fwd: float = 1.0
    stochastic_grad: bool = True
    stochastic_act: bool = False     # X in dW = X^T G rounded stochastically (the paper's setting)
    need_input_grad: bool = True
    fold_in_matmul: bool = True      # convolution layers: hdqt_conv_bwd where the geometry is taken
    # when set to a dict, every matmul of the layer leaves its operands and results there
    # (X, W, Z in the forward pass; G, dX, dW in the backward pass) for inspection
    capture: Optional[dict] = field(default=None, repr=False, compare=False)

    def params(self, kind: int, step: int = 0) -> B.Params:
        tid = lambda role: 16 * self.layer_id + {"X": 0, "W": 1, "G": 2}[role] + 4 * kind
        NE = B.ROUND_NEAREST
        ST = B.ROUND_STOCHASTIC if self.stochastic_grad else NE
        b = self.bits
        if kind == B.GEMM_FWD:
            A, Bq = B.Operand(b, NE, self.clip_fwd, tid("X")), B.Operand(b, NE, self.clip_fwd, tid("W"))
        elif kind == B.GEMM_BWD_INPUT:
            A, Bq = B.Operand(b, ST, 1.0, tid("G")), B.Operand(b, NE, 1.0, tid("W"))
        else:
            SA = B.ROUND_STOCHASTIC if self.stochastic_act else NE
            A, Bq = B.Operand(b, SA, 1.0, tid("X")), B.Operand(b, ST, 1.0, tid("G"))
        # a fresh random stream every step: the seed advances with the step counter
        return B.Params(had_block=self.had_block, acc_bits=self.acc_bits, s=self.s,
                        seed=self.seed + step, A=A, B=Bq)


class HdqtMatmul(torch.autograd.Function):
    """Z = X W with X [M, K], W [K, N] on the GPU, fp32, contiguous."""

    @staticmethod
    def forward(ctx, X, W, cfg: LayerConfig, step: int):
        # (asked before .contiguous(): a copy made inside forward() does not require grad)
        ctx.want_dx = cfg.need_input_grad and X.requires_grad
        X, W = X.contiguous(), W.contiguous()
        pf = cfg.params(B.GEMM_FWD, step)
        pw = cfg.params(B.GEMM_BWD_WEIGHT, step)
        Z, saved = B.layer_fwd(X, W, pf, pw)
        ctx.save_for_backward(W, saved)
        ctx.cfg, ctx.step, ctx.K = cfg, step, X.shape[1]
        if cfg.capture is not None:
            cfg.capture.update(X=X.detach(), W=W.detach().clone(), Z=Z.detach(), step=step)
        return Z

    @staticmethod
    def backward(ctx, G):
        W, saved = ctx.saved_tensors
        cfg = ctx.cfg
        pi = cfg.params(B.GEMM_BWD_INPUT, ctx.step) if ctx.want_dx else None
        pw = cfg.params(B.GEMM_BWD_WEIGHT, ctx.step)
        G = G.contiguous()
        dX, dW = B.layer_bwd(G, W, saved, ctx.K, pi, pw)
        if cfg.capture is not None:
            cfg.capture.update(G=G.detach(), dX=dX, dW=dW)
        return dX, dW, None, None


class HdqtReluMatmul(torch.autograd.Function):
    """Z = max(pre, 0) W: the rectifier in front of a layer and the layer's matmul as one
    autograd node.  The backward pass returns the gradient of `pre`: the library writes the
    input gradient where the layer's input is positive and zero elsewhere, in the matmul's own
    epilogue (hdqt_layer_bwd_masked), instead of a pass over dX by the framework.  The layer's
    input is kept in fp32 for that (a framework's own rectifier keeps it too)."""

    @staticmethod
    def forward(ctx, pre, W, cfg: LayerConfig, step: int):
        ctx.want_dx = cfg.need_input_grad and pre.requires_grad
        X, W = torch.clamp_min(pre, 0.0).contiguous(), W.contiguous()
        pf = cfg.params(B.GEMM_FWD, step)
        pw = cfg.params(B.GEMM_BWD_WEIGHT, step)
        Z, saved = B.layer_fwd(X, W, pf, pw)
        ctx.save_for_backward(W, saved, X)
        ctx.cfg, ctx.step, ctx.K = cfg, step, X.shape[1]
        if cfg.capture is not None:
            cfg.capture.update(X=X.detach(), W=W.detach().clone(), Z=Z.detach(), step=step)
        return Z

    @staticmethod
    def backward(ctx, G):
        W, saved, X = ctx.saved_tensors
        cfg = ctx.cfg
        pi = cfg.params(B.GEMM_BWD_INPUT, ctx.step) if ctx.want_dx else None
        pw = cfg.params(B.GEMM_BWD_WEIGHT, ctx.step)
        G = G.contiguous()
        dPre, dW = B.layer_bwd(G, W, saved, ctx.K, pi, pw, mask=X if ctx.want_dx else None)
        if cfg.capture is not None:
            cfg.capture.update(G=G.detach(), dX=dPre, dW=dW)
        return dPre, dW, None, None


_FOLD_REFUSED = set()        # activation shapes hdqt_conv_bwd did not take (with the window used)


class HdqtConvMatmul(torch.autograd.Function):
    """Z = im2col(act) W for a stride-1, same-size convolution, without forming im2col(act):
    the forward call reads the activation (hdqt_conv_fwd).  The backward pass returns the
    gradient of the activation: the library's gradient of the im2col matrix, folded back by
    PyTorch."""

    @staticmethod
    def forward(ctx, act, W, cfg: LayerConfig, step: int, kh: int, kw: int):
        ctx.want_dx = cfg.need_input_grad and act.requires_grad
        act, W = act.contiguous(), W.contiguous()
        pf = cfg.params(B.GEMM_FWD, step)
        pw = cfg.params(B.GEMM_BWD_WEIGHT, step)
        Z, saved = B.conv_fwd(act, kh, kw, W, pf, pw)
        ctx.save_for_backward(W, saved)
        ctx.cfg, ctx.step, ctx.shape, ctx.window = cfg, step, tuple(act.shape), (kh, kw)
        if cfg.capture is not None:
            cfg.capture.update(act=act.detach(), W=W.detach().clone(), Z=Z.detach(), step=step)
        return Z

    @staticmethod
    def backward(ctx, G):
        W, saved = ctx.saved_tensors
        cfg = ctx.cfg
        Bn, Cin, H, Wd = ctx.shape
        kh, kw = ctx.window
        pi = cfg.params(B.GEMM_BWD_INPUT, ctx.step) if ctx.want_dx else None
        pw = cfg.params(B.GEMM_BWD_WEIGHT, ctx.step)
        G = G.contiguous()
        dAct = dXcol = None
        key = (ctx.shape, kh, kw)
        if pi is not None and cfg.fold_in_matmul and key not in _FOLD_REFUSED:
            # the input gradient folded onto the activation inside the matmul: the gradient of
            # the im2col matrix is never written
            try:
                dAct, dW = B.conv_bwd(G, W, saved, ctx.shape, kh, kw, pi, pw)
            except B.HdqtError as exc:
                if exc.code != -13:
                    raise
                _FOLD_REFUSED.add(key)
        if dAct is None:
            dXcol, dW = B.layer_bwd(G, W, saved, Cin * kh * kw, pi, pw)
            if dXcol is not None:
                cols = dXcol.reshape(Bn, H * Wd, Cin * kh * kw).transpose(1, 2)
                dAct = torch.nn.functional.fold(cols, output_size=(H, Wd), kernel_size=(kh, kw),
                                                padding=((kh - 1) // 2, (kw - 1) // 2))
        if cfg.capture is not None:
            cfg.capture.update(G=G.detach(), dX=dXcol, dAct=dAct, dW=dW)
        return dAct, dW, None, None, None, None


class Unfold(torch.autograd.Function):
    """act [B, C, H, W] -> its im2col matrix [B*Ho*Wo, C*k*k] by the library's one-launch kernel
    (the layers whose geometry the activation-source kernels do not read directly); the
    backward pass folds the matrix gradient back with PyTorch."""

    @staticmethod
    def forward(ctx, act, k: int, stride: int, pad: int):
        ctx.geo = (tuple(act.shape), k, stride, pad)
        return B.im2col(act, k, k, stride, pad, pad)

    @staticmethod
    def backward(ctx, dX):
        (Bn, Cin, H, W), k, stride, pad = ctx.geo
        cols = dX.reshape(Bn, -1, Cin * k * k).transpose(1, 2)
        return torch.nn.functional.fold(cols, output_size=(H, W), kernel_size=k, padding=pad,
                                        stride=stride), None, None, None


class HdqtLinear(torch.nn.Module):
    """y = x W + bias with the matmul and its gradients quantized; inputs of any
    leading shape are flattened to [M, K]."""

    def __init__(self, in_features: int, out_features: int, bias: bool = True,
                 cfg: Optional[LayerConfig] = None, device=None, relu_input: bool = False):
        super().__init__()
        self.cfg = cfg or LayerConfig()
        self.relu_input = relu_input      # y = max(x, 0) W + bias, the rectifier's backward pass inside the matmul
        w = torch.empty(in_features, out_features, device=device)
        torch.nn.init.kaiming_normal_(w.t(), nonlinearity="relu")     # fan-in = in_features
        self.weight = torch.nn.Parameter(w)
        self.bias = torch.nn.Parameter(torch.zeros(out_features, device=device)) if bias else None
        self.step = 0

    def forward(self, x):
        lead = x.shape[:-1]
        fn = HdqtReluMatmul if self.relu_input else HdqtMatmul
        z = fn.apply(x.reshape(-1, x.shape[-1]), self.weight, self.cfg, self.step)
        if self.training:
            self.step += 1
        if self.bias is not None:
            z = z + self.bias
        return z.reshape(*lead, -1)


class HdqtConv2d(torch.nn.Module):
    """Convolution as the paper runs it: the activation is unfolded (im2col, column index =
    channel * kh * kw + tap) and the products of the forward and the backward pass are the
    quantized matmuls above.  Stride-1, same-size layers whose geometry the library takes
    never form the unfolded matrix (hdqt_conv_fwd reads the activation, hdqt_conv_bwd folds the
    input gradient back inside the matmul); the others are unfolded by hdqt_im2col and their
    input gradient is folded back by PyTorch."""

    def __init__(self, in_channels: int, out_channels: int, kernel_size: int = 3, padding: int = 1,
                 stride: int = 1, cfg: Optional[LayerConfig] = None, device=None):
        super().__init__()
        self.k, self.pad, self.stride = kernel_size, padding, stride
        self.cfg = cfg or LayerConfig()
        fan_in = in_channels * kernel_size * kernel_size
        w = torch.empty(fan_in, out_channels, device=device)
        torch.nn.init.kaiming_normal_(w.t(), nonlinearity="relu")
        self.weight = torch.nn.Parameter(w)
        self.step = 0
        self.from_activation = True      # read the activation directly where the library takes the geometry
        self._refused = set()            # input shapes it did not take

    def forward(self, x):
        Bn, Cin, H, W = x.shape
        Ho = (H + 2 * self.pad - self.k) // self.stride + 1
        Wo = (W + 2 * self.pad - self.k) // self.stride + 1
        Z = None
        if (self.from_activation and self.stride == 1 and 2 * self.pad == self.k - 1 and self.training
                and tuple(x.shape) not in self._refused):
            try:
                Z = HdqtConvMatmul.apply(x, self.weight, self.cfg, self.step, self.k, self.k)
            except B.HdqtError as exc:
                if exc.code != -13:
                    raise
                self._refused.add(tuple(x.shape))
        if Z is None:
            X = Unfold.apply(x, self.k, self.stride, self.pad)                     # [B*Ho*Wo, C*k*k]
            Z = HdqtMatmul.apply(X, self.weight, self.cfg, self.step)
        if self.training:
            self.step += 1
        return Z.reshape(Bn, Ho * Wo, -1).transpose(1, 2).reshape(Bn, -1, Ho, Wo)
