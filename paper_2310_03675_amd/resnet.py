"""A CIFAR-width ResNet-18 whose 21 convolution / classifier matmuls (forward and both
gradients) are the library's quantized matmuls (Experiments: the paper trains residual
networks on CIFAR100 with every matmul of the training step quantized).  Batch
normalisation, ReLU, pooling, the residual additions and the unfolding of the
activations are PyTorch's and run in fp32; they are glue around the path, not part of it.

Layer names and order are those of workloads.resnet18_layer_table.
"""
from typing import Dict, Optional

import torch

from .autograd import HdqtConv2d, HdqtLinear, LayerConfig
from .workloads import resnet18_layer_table


class _Block(torch.nn.Module):
    def __init__(self, cin, cout, stride, convs, proj):
        super().__init__()
        self.conv_a, self.conv_b, self.proj = convs[0], convs[1], proj
        self.bn_a, self.bn_b = torch.nn.BatchNorm2d(cout), torch.nn.BatchNorm2d(cout)
        self.bn_p = torch.nn.BatchNorm2d(cout) if proj is not None else None

    def forward(self, x):
        h = torch.relu(self.bn_a(self.conv_a(x)))
        h = self.bn_b(self.conv_b(h))
        sc = x if self.proj is None else self.bn_p(self.proj(x))
        return torch.relu(h + sc)


class ResNet18(torch.nn.Module):
    """3x3 stem (3 -> 64 at 32x32), four stages of two basic blocks at widths 64 / 128 /
    256 / 512 with strides 1 / 2 / 2 / 2, a 1x1 stride-2 projection on the shortcut of the
    first block of stages 2-4, global average pooling and a 100-way classifier."""

    def __init__(self, num_classes: int = 100, base: Optional[LayerConfig] = None, device=None,
                 capture: Optional[Dict[str, dict]] = None):
        super().__init__()
        base = base or LayerConfig()
        names = [t[0] for t in resnet18_layer_table(1)]
        self.layer_names = names

        def cfg(name):
            c = LayerConfig(**{k: getattr(base, k) for k in
                               ("had_block", "bits", "acc_bits", "s", "seed", "clip_fwd", "stochastic_grad")})
            c.layer_id = names.index(name)
            c.need_input_grad = name != "stem"
            if capture is not None:
                c.capture = capture.setdefault(name, {})
            return c

        conv = lambda name, cin, cout, k, stride: HdqtConv2d(
            cin, cout, kernel_size=k, padding=k // 2, stride=stride, cfg=cfg(name), device=device)
        self.stem = conv("stem", 3, 64, 3, 1)
        self.bn0 = torch.nn.BatchNorm2d(64)
        blocks = []
        cin = 64
        for si, cout in enumerate((64, 128, 256, 512), start=1):
            stride = 1 if si == 1 else 2
            c = [conv(f"s{si}.conv{i}", cin if i == 0 else cout, cout, 3, stride if i == 0 else 1)
                 for i in range(4)]
            proj = conv(f"s{si}.proj", cin, cout, 1, stride) if si > 1 else None
            blocks += [_Block(cin, cout, stride, c[0:2], proj), _Block(cout, cout, 1, c[2:4], None)]
            cin = cout
        self.blocks = torch.nn.Sequential(*blocks)
        self.fc = HdqtLinear(512, num_classes, bias=True, cfg=cfg("fc"), device=device)
        if device is not None:
            self.to(device)

    def forward(self, x):
        h = torch.relu(self.bn0(self.stem(x)))
        h = self.blocks(h)
        return self.fc(h.mean(dim=(2, 3)))
