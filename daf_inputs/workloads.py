from dataclasses import dataclass
from typing import List, Sequence

import numpy as np
import torch

F32, F16, BF16 = 0, 1, 2
_TORCH = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}

CONFIG_NAMES = {
    1: "tiny_f32_4x64x32x32_g128_b2",
    2: "resnet50_conv_f32_64x256x56x56_g256_b2",
    3: "vit_bert_f16_32x1024x768_g128_b1248",
    4: "resnet18_step_f32_bs256_g256_b2",
    5: "llm_mlp_bf16_16x2048x11008_g64_b248",
}


def torch_dtype(dtype: int) -> torch.dtype:
    return _TORCH[dtype]


@dataclass
class Workload:
    """One activation tensor to be saved: flat contiguous values, group size, per-group
    (or uniform) bit widths and the stochastic-rounding seed."""
    name: str
    x: torch.Tensor            # CPU tensor of dtype torch_dtype(self.dtype), any shape, contiguous
    dtype: int                 # F32 / F16 / BF16
    group_size: int
    bits: np.ndarray           # uint8, 1 entry (uniform) or G entries
    seed: int

    @property
    def numel(self) -> int:
        return self.x.numel()

    @property
    def num_groups(self) -> int:
        return (self.numel + self.group_size - 1) // self.group_size


def to_numpy_bits(x: torch.Tensor) -> np.ndarray:
    """Flat numpy view of a CPU tensor: float32 as float32, 16-bit floats as uint16 patterns."""
    x = x.contiguous().reshape(-1)
    if x.dtype == torch.float32:
        return x.numpy()
    return x.view(torch.int16).numpy().view(np.uint16)


def bits_by_range_quantiles(x: torch.Tensor, group_size: int, classes: Sequence[int]) -> np.ndarray:
    """Stand-in bit-width policy: rank groups by (value range, group index) ascending and
    split the ranking into len(classes) equal parts; the lowest ranges get classes[0]."""
    flat = x.reshape(-1).float()
    n = flat.numel()
    G = (n + group_size - 1) // group_size
    pad = G * group_size - n
    if pad:
        flat = torch.cat([flat, flat[-1:].expand(pad)])
    g = flat.reshape(G, group_size)
    rng = (g.amax(dim=1) - g.amin(dim=1)).numpy()
    order = np.lexsort((np.arange(G), rng))          # primary key: range, ties by group index
    rank = np.empty(G, dtype=np.int64)
    rank[order] = np.arange(G)
    cls = (rank * len(classes)) // G
    return np.asarray(classes, dtype=np.uint8)[cls]


def _gen(seed: int) -> torch.Generator:
    return torch.Generator().manual_seed(seed)


def _relu_randn(shape, g):
    return torch.relu_(torch.randn(*shape, generator=g, dtype=torch.float32))


# Config 4: the activations a ResNet-18 training step saves, forward order (count, C, H, W).
_RESNET18_SAVED = [(1, 64, 112, 112), (4, 64, 56, 56), (4, 128, 28, 28), (4, 256, 14, 14), (4, 512, 7, 7)]


def make_config(cfg: int, batch_scale: float = 1.0) -> List[Workload]:
    """The workloads of configuration `cfg` (1..5).  `batch_scale` < 1 shrinks the leading
    (batch) dimension only, for parity cases the oracle finishes in seconds; the recipe is
    otherwise identical.  data seed = 1000 + cfg."""
    g = _gen(1000 + cfg)

    def B(b):
        return max(1, int(round(b * batch_scale)))

    name = CONFIG_NAMES[cfg]
    if cfg == 1:
        x = _relu_randn((B(4), 64, 32, 32), g)
        return [Workload(name, x, F32, 128, np.array([2], np.uint8), 0)]
    if cfg == 2:
        s = torch.exp(0.5 * torch.randn(256, generator=g))
        x = _relu_randn((B(64), 256, 56, 56), g) * s[None, :, None, None]
        return [Workload(name, x.contiguous(), F32, 256, np.array([2], np.uint8), 1)]
    if cfg == 3:
        x = torch.nn.functional.gelu(torch.randn(B(32), 1024, 768, generator=g)).to(torch.float16)
        bits = bits_by_range_quantiles(x, 128, (1, 2, 4, 8))
        return [Workload(name, x, F16, 128, bits, 2)]
    if cfg == 4:
        out, t = [], 0
        for count, c, h, w in _RESNET18_SAVED:
            for _ in range(count):
                x = _relu_randn((B(256), c, h, w), g)
                out.append(Workload(f"{name}_t{t}", x, F32, 256, np.array([2], np.uint8), 3 + 1000 * t))
                t += 1
        return out
    if cfg == 5:
        shape = (B(16), 2048, 11008)
        z = torch.randn(*shape, generator=g)
        chi2 = torch.zeros(shape)
        for _ in range(3):                                   # chi-square(3) = sum of 3 squared normals
            chi2 += torch.randn(*shape, generator=g) ** 2
        z /= torch.sqrt(chi2 / 3.0)                          # Student-t, nu = 3
        del chi2
        outliers = torch.randperm(shape[-1], generator=g)[: shape[-1] // 100]
        z[..., outliers] *= 20.0
        x = z.to(torch.bfloat16)
        del z
        bits = bits_by_range_quantiles(x, 64, (2, 4, 8))
        return [Workload(name, x, BF16, 64, bits, 4)]
    raise ValueError(f"unknown config {cfg}")
