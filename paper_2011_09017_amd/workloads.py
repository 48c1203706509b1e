"""Seeded synthetic activation tensors shaped like the paper's CNN workloads.

The paper measures on ImageNet activations of AlexNet, VGG-16, ResNet-18 and
ResNet-50 (Section 5.1); none of that data is available, so these tensors stand
in for it: same shapes, a post-ReLU zero fraction, and a spatial smoothness set
by a box filter.  This module holds input generation only -- none of the
compressor's arithmetic -- and serves the tests, the benchmark and the smoke
check alike.

Recipe G(shape, k, p_zero, seed):
  1. g ~ N(0,1) i.i.d., fp32, from a seeded generator on the chosen device;
  2. f = k x k box filter of g per (n,c) plane, zero padded (avg_pool2d,
     stride 1, padding k//2, count_include_pad);
  3. f /= std(f) over the whole tensor;
  4. f -= Phi^-1(p_zero), so that about p_zero of the values are <= 0;
  5. x = relu(f).
The random stream differs between CPU and GPU generators; within one run both
the oracle and the HIP path read the same bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from statistics import NormalDist

import torch
import torch.nn.functional as F

BASE_SEED = 201109017


def activation(shape, k: int = 5, p_zero: float = 0.5, seed: int = BASE_SEED,
               device: str | torch.device = "cpu") -> torch.Tensor:
    """One synthetic post-ReLU activation tensor, fp32, contiguous NCHW."""
    assert len(shape) == 4 and k % 2 == 1
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(seed))
    g = torch.randn(tuple(shape), dtype=torch.float32, device=dev, generator=gen)
    f = F.avg_pool2d(g, k, stride=1, padding=k // 2, count_include_pad=True)
    del g
    f /= f.std()
    f -= NormalDist().inv_cdf(p_zero)
    return torch.relu_(f).contiguous()


@dataclass
class Workload:
    name: str
    config: int
    shapes: list
    k: int = 5
    p_zero: float = 0.5
    ebs: list = field(default_factory=lambda: [1e-2])

    def seed(self, tensor_index: int) -> int:
        return BASE_SEED + 1000 * self.config + tensor_index

    def numel(self) -> int:
        n = 0
        for s in self.shapes:
            n += s[0] * s[1] * s[2] * s[3]
        return n

    def tensor(self, i: int, device="cpu") -> torch.Tensor:
        return activation(self.shapes[i], self.k, self.p_zero, self.seed(i), device)


def _resnet18_stream(batch: int = 256):
    shapes = [(batch, 64, 112, 112)]
    for c, hw in ((64, 56), (128, 28), (256, 14), (512, 7)):
        shapes += [(batch, c, hw, hw)] * 4
    return shapes


WORKLOADS = {
    "cfg1_small": Workload("cfg1_small", 1, [(1, 64, 56, 56)]),
    "cfg2_vgg16_conv1_2": Workload("cfg2_vgg16_conv1_2", 2, [(32, 64, 224, 224)]),
    "cfg3_resnet50_bottleneck": Workload("cfg3_resnet50_bottleneck", 3, [(64, 256, 56, 56)],
                                         k=3, p_zero=0.6, ebs=[5e-3]),
    "cfg4_alexnet_conv1": Workload("cfg4_alexnet_conv1", 4, [(128, 96, 55, 55)],
                                   ebs=[1e-1, 1e-2, 1e-3]),
    "cfg5_resnet18_stream": Workload("cfg5_resnet18_stream", 5, _resnet18_stream()),
    "cfg5_resnet18_stream_sparse": Workload("cfg5_resnet18_stream_sparse", 5, _resnet18_stream(),
                                            p_zero=0.85),
}
