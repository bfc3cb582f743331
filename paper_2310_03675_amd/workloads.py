"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws numbers and rearranges them (ReLU, im2col); it holds
none of the method's arithmetic, so the CPU oracle's tests and the GPU path's
tests can both take their inputs from it.  Everything is generated on the CPU
with a seeded torch.Generator in fp32, so both sides see identical bits.

The paper trains on CIFAR100 and three HAR datasets (Experiments section);
those are not available here and are not needed for the matmul path: the
tensors below stand in for them with the shapes, value distributions and
structure (ReLU sparsity, im2col repetition, zero borders, heavy-tailed
outliers) of such layers.
"""
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import torch

ROLE_SUBSEED = {"X": 1, "W": 2, "G": 3}


def _gen(seed: int, role: str, layer: int = 0) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 1000 + ROLE_SUBSEED[role] + 10 * layer)
    return g


def _normal(shape, std: float, g: torch.Generator) -> torch.Tensor:
    return torch.randn(shape, generator=g, dtype=torch.float32) * std


@dataclass
class Layer:
    """One matmul layer Z[M,N] = X[M,K] W[K,N] with its output gradient G[M,N]."""
    name: str
    X: torch.Tensor
    W: torch.Tensor
    G: torch.Tensor
    act: Optional[torch.Tensor] = None     # convolution layers: the activation X is unfolded from
    window: Optional[Tuple[int, int]] = None        # and its (kh, kw)

    @property
    def M(self) -> int:
        return self.X.shape[0]

    @property
    def K(self) -> int:
        return self.X.shape[1]

    @property
    def N(self) -> int:
        return self.W.shape[1]


def fc_layer(M: int = 64, K: int = 256, N: int = 128, seed: int = 0, g_var: float = 1e-3,
             layer: int = 0) -> Layer:
    """Single fully connected layer: X~N(0,1), W~N(0, var 1/K), G~N(0, var g_var)."""
    X = _normal((M, K), 1.0, _gen(seed, "X", layer))
    W = _normal((K, N), (1.0 / K) ** 0.5, _gen(seed, "W", layer))
    G = _normal((M, N), g_var ** 0.5, _gen(seed, "G", layer))
    return Layer(f"fc_{M}x{K}x{N}", X, W, G)


def im2col_1d(act: torch.Tensor, kernel: int, pad: int) -> torch.Tensor:
    """act [B, C, L] -> [B*L, C*kernel], column index c*kernel + tap, stride 1, zero pad."""
    B, C, L = act.shape
    cols = torch.nn.functional.unfold(act.unsqueeze(2), kernel_size=(1, kernel),
                                      padding=(0, pad))          # [B, C*kernel, L]
    return cols.transpose(1, 2).reshape(B * L, C * kernel).contiguous()


def im2col_2d(act: torch.Tensor, kernel: int, pad: int, stride: int = 1) -> torch.Tensor:
    """act [B, C, H, W] -> [B*Ho*Wo, C*kernel*kernel], column index c*k*k + tap."""
    B, C, _, _ = act.shape
    cols = torch.nn.functional.unfold(act, kernel_size=kernel, padding=pad, stride=stride)
    return cols.transpose(1, 2).reshape(-1, C * kernel * kernel).contiguous()


def har_conv_layer(batch: int = 256, seq: int = 128, cin: int = 64, cout: int = 128,
                   kernel: int = 5, seed: int = 0, layer: int = 0) -> Layer:
    """HAR-style 1-D convolution as an im2col matmul (M = batch*seq, K = cin*kernel)."""
    act = torch.relu(_normal((batch, cin, seq), 1.0, _gen(seed, "X", layer)))
    X = im2col_1d(act, kernel, kernel // 2)
    K = cin * kernel
    W = _normal((K, cout), (2.0 / K) ** 0.5, _gen(seed, "W", layer))
    G = _normal((batch * seq, cout), 1e-3 ** 0.5, _gen(seed, "G", layer))
    return Layer(f"har_conv_{batch * seq}x{K}x{cout}", X, W, G, act.unsqueeze(2).contiguous(), (1, kernel))


def resnet_conv_layer(batch: int = 256, cin: int = 128, cout: int = 128, hw: int = 16,
                      seed: int = 0, layer: int = 0, g_var: float = 1e-4) -> Layer:
    """CIFAR-ResNet-style 3x3 convolution (pad 1, stride 1) as an im2col matmul."""
    act = torch.relu(_normal((batch, cin, hw, hw), 1.0, _gen(seed, "X", layer)))
    X = im2col_2d(act, 3, 1)
    K = cin * 9
    W = _normal((K, cout), (2.0 / K) ** 0.5, _gen(seed, "W", layer))
    G = _normal((batch * hw * hw, cout), g_var ** 0.5, _gen(seed, "G", layer))
    return Layer(f"resnet_conv_{batch * hw * hw}x{K}x{cout}", X, W, G, act, (3, 3))


def outlier_matrix(rows: int, cols: int, seed: int, role: str, p: float = 0.01,
                   magnitude: float = 20.0) -> torch.Tensor:
    """N(0,1) entries; each independently with probability p replaced by +-magnitude
    (sign of the original draw)."""
    g = _gen(seed, role)
    base = torch.randn((rows, cols), generator=g, dtype=torch.float32)
    mask = torch.rand((rows, cols), generator=g) < p
    return torch.where(mask, torch.sign(base) * magnitude, base).contiguous()


def square_layer(size: int, seed: int = 0) -> Layer:
    """Square matmul with 1 % outliers at 20 sigma (stresses the quantization range)."""
    return Layer(f"square_{size}", outlier_matrix(size, size, seed, "X"),
                 outlier_matrix(size, size, seed, "W"), outlier_matrix(size, size, seed, "G"))


# (name, M at batch 128, K, N) of the 21 matmul layers of a CIFAR-width ResNet-18
def resnet18_layer_table(batch: int = 128) -> List[Tuple[str, int, int, int]]:
    t: List[Tuple[str, int, int, int]] = [("stem", batch * 1024, 27, 64)]
    t += [(f"s1.conv{i}", batch * 1024, 576, 64) for i in range(4)]
    t += [("s2.conv0", batch * 256, 576, 128)]
    t += [(f"s2.conv{i}", batch * 256, 1152, 128) for i in range(1, 4)]
    t += [("s2.proj", batch * 256, 64, 128)]
    t += [("s3.conv0", batch * 64, 1152, 256)]
    t += [(f"s3.conv{i}", batch * 64, 2304, 256) for i in range(1, 4)]
    t += [("s3.proj", batch * 64, 128, 256)]
    t += [("s4.conv0", batch * 16, 2304, 512)]
    t += [(f"s4.conv{i}", batch * 16, 4608, 512) for i in range(1, 4)]
    t += [("s4.proj", batch * 16, 256, 512)]
    t += [("fc", batch, 512, 100)]
    return t


def named_config(name: str, seed: int = 0) -> Dict[str, Layer]:
    """The benchmark configurations by name."""
    if name == "fc":
        return {"fc": fc_layer(seed=seed)}
    if name == "har":
        return {"har": har_conv_layer(seed=seed)}
    if name == "resnet_k576":
        return {"resnet_k576": resnet_conv_layer(256, 64, 64, 32, seed=seed)}
    if name == "resnet_k1152":
        return {"resnet_k1152": resnet_conv_layer(256, 128, 128, 16, seed=seed)}
    raise KeyError(name)
