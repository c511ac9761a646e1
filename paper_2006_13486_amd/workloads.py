"""Workload table and seeded synthetic inputs.

Holds none of the method's arithmetic: only shapes, factor sizes, seeds and
value distributions.  Tests hand the arrays made here to both the library and
the CPU oracle, so the two sides see identical bits.

The shapes are convolution layers lowered to GEMM (M = C_out, K = 9*C_in,
N = batch*H*W, batch 128) of the two networks of the paper's Table 1
(VGG19 and WRN-40-4 on CIFAR) and the 4096^3 SDMM of Tables 2-3; the values
are synthetic stand-ins (Gaussian kept weights, post-ReLU Gaussian
activations), no dataset or trained weight is involved.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple

import numpy as np

F32 = 0        # fp32 in, fp32 out
BF16 = 1       # bf16 in, fp32 accumulate, fp32 out


@dataclass(frozen=True)
class Workload:
    name: str
    rows: Tuple[int, int, int, int]      # |G_o.U|, |G_r.U|, |G_i.U|, |G_b.U|
    cols: Tuple[int, int, int, int]      # |G_o.V|, |G_r.V|, |G_i.V|, |G_b.V|
    row_deg: Tuple[int, int, int, int]   # d_l of each factor (== cols -> complete)
    N: int
    dtype: int = F32
    mask_seed: int = 1
    w_seed: int = 2
    i_seed: int = 3
    w_std: float = 0.02
    i_dist: str = "relu_normal"          # or "uniform"
    roles: Tuple[int, ...] = ()          # more than four base graphs: the factor (0..3) each belongs to

    @property
    def M(self) -> int:
        return int(np.prod(self.rows))

    @property
    def K(self) -> int:
        return int(np.prod(self.cols))

    @property
    def rowdeg(self) -> int:
        return int(np.prod(self.row_deg))

    @property
    def nnz(self) -> int:
        return self.M * self.rowdeg

    @property
    def density(self) -> float:
        return self.rowdeg / self.K

    @property
    def flops(self) -> int:
        """Algorithmic flops: two per kept weight per column of I."""
        return 2 * self.nnz * self.N

    @property
    def in_bytes(self) -> int:
        return 2 if self.dtype == BF16 else 4

    @property
    def algorithmic_bytes(self) -> int:
        """I read once, O written once (fp32), kept weights read once."""
        return self.K * self.N * self.in_bytes + self.M * self.N * 4 + self.nnz * self.in_bytes


TINY = Workload("tiny_fp32_64x64x256", (4, 2, 4, 2), (4, 2, 4, 2), (2, 2, 2, 2), 256,
                F32, 1, 2, 3, 1.0, "uniform")
VGG19_CONV5 = Workload("vgg19_conv5_fp32_512x4608x2048_d8", (16, 4, 4, 2), (16, 4, 8, 9),
                       (8, 4, 2, 9), 2048, F32, 11, 12, 13)
VGG19_CONV3_BF16 = Workload("vgg19_conv3_bf16_256x2304x8192_d4", (8, 4, 4, 2), (8, 4, 8, 9),
                            (4, 4, 4, 9), 8192, BF16, 21, 22, 23)
WRN_G1 = Workload("wrn40_4_group1_fp32_64x576x131072_d8", (8, 2, 4, 1), (8, 2, 4, 9),
                  (2, 2, 2, 9), 131072, F32, 31, 32, 33)

CONFIGS = [TINY, VGG19_CONV5, VGG19_CONV3_BF16, WRN_G1]

# (images, height, width) of the convolution each lowered configuration comes from: N = images * height * width
CONV_GEOMETRY = {VGG19_CONV5.name: (128, 4, 4), VGG19_CONV3_BF16.name: (128, 8, 8), WRN_G1.name: (128, 32, 32)}

# VGG19 on CIFAR (Table 1's network): (C_in, C_out, H) of the 16 conv layers.
VGG19_LAYERS = [(3, 64, 32), (64, 64, 32), (64, 128, 16), (128, 128, 16),
                (128, 256, 8), (256, 256, 8), (256, 256, 8), (256, 256, 8),
                (256, 512, 4), (512, 512, 4), (512, 512, 4), (512, 512, 4),
                (512, 512, 2), (512, 512, 2), (512, 512, 2), (512, 512, 2)]


def _sparse_ok(a: int, c: int, d: int) -> bool:
    if d == c:
        return True
    e = a * d // c
    q = c // d
    return d >= 2 and e >= 2 and a % q == 0


def vgg19_sweep_workload(layer: int, log2_inv_density: int, dtype: int, batch: int = 128) -> Workload:
    """Factor sizes for layer `layer` (0-based) of VGG19 at density 2^-log2_inv_density.

    The first layer (K = 27) stays dense, as the paper keeps it unsparsified.
    Cells that coincide with a fixed configuration reuse its factoring."""
    cin, cout, h = VGG19_LAYERS[layer]
    N = batch * h * h
    base = 1000 + 10 * layer
    if layer == 0:
        return Workload(f"vgg19_L{layer}_dense", (cout, 1, 1, 1), (3, 1, 1, 9), (3, 1, 1, 9), N, dtype,
                        base, base + 1, base + 2)
    for fixed in (VGG19_CONV5, VGG19_CONV3_BF16):
        if (fixed.M, fixed.K, fixed.N, fixed.dtype) == (cout, 9 * cin, N, dtype) and \
                fixed.K // fixed.rowdeg == 1 << log2_inv_density:
            return replace(fixed, name=f"vgg19_L{layer}_d{1 << log2_inv_density}_{'bf16' if dtype else 'fp32'}",
                           mask_seed=base, w_seed=base + 1, i_seed=base + 2)
    a4, c4 = (2 if cout > 64 else 1), 9
    a2 = 2 if cout == 64 else 4
    c2 = 2 if cin == 64 else 4
    a3 = 4
    c3 = 4 if cin == 64 else 8
    if log2_inv_density == 1:
        l1, l3 = 1, 0
    else:
        l1, l3 = log2_inv_density - 1, 1
    while True:
        a1 = cout // (a2 * a3 * a4)
        c1 = 9 * cin // (c2 * c3 * c4)
        d1, d3 = c1 >> l1, c3 >> l3
        if d1 >= 1 and _sparse_ok(a1, c1, d1) and _sparse_ok(a3, c3, d3):
            break
        if a2 == 1 or c2 == 1:
            d1 = max(d1, 1)
            break
        a2 //= 2
        c2 //= 2
    return Workload(f"vgg19_L{layer}_d{1 << log2_inv_density}_{'bf16' if dtype else 'fp32'}",
                    (a1, a2, a3, a4), (c1, c2, c3, c4), (d1, c2, d3, c4), N, dtype,
                    base, base + 1, base + 2)


def sdmm4096_table2(sp_o_log2: int, sp_i_log2: int, N: int = 4096) -> Workload:
    """Table 2's SDMM: sizes (32,128),(4,1),(32,32),(1,1); density of G_o and
    G_i given as 2^-sp_o_log2 and 2^-sp_i_log2."""
    return Workload(f"sdmm4096_t2_o{1 << sp_o_log2}_i{1 << sp_i_log2}", (32, 4, 32, 1), (128, 1, 32, 1),
                    (128 >> sp_o_log2, 1, 32 >> sp_i_log2, 1), N, F32, 41, 42, 43)


def sdmm4096_table3(gr: int, gb: int, log2_inv_density: int, N: int = 4096) -> Workload:
    """Table 3's SDMM: G_t = G_r x G_i x G_b fixed at (128,32), G_o 50 % sparse,
    G_r = (gr,1), G_b = (gb,1); the rest of the sparsity sits in G_i."""
    a3 = 128 // (gr * gb)
    l3 = log2_inv_density - 1
    return Workload(f"sdmm4096_t3_r{gr}_b{gb}_d{1 << log2_inv_density}", (32, gr, a3, gb), (128, 1, 32, 1),
                    (64, 1, 32 >> l3, 1), N, F32, 51, 52, 53)


# --------------------------------------------------------------------------
# seeded values
# --------------------------------------------------------------------------
def kept_weights(w: Workload) -> np.ndarray:
    """data[M][rowdeg] ~ N(0, w_std), float32, canonical (ascending-column) order."""
    g = np.random.Generator(np.random.PCG64(w.w_seed))
    return (g.standard_normal((w.M, w.rowdeg), dtype=np.float32) * np.float32(w.w_std)).astype(np.float32)


def activations(w: Workload, N: int | None = None) -> np.ndarray:
    """I[K][N] float32: U[-1,1] or max(0, N(0,1)) (post-ReLU activations)."""
    N = w.N if N is None else N
    g = np.random.Generator(np.random.PCG64(w.i_seed))
    if w.i_dist == "uniform":
        return g.uniform(-1.0, 1.0, size=(w.K, N)).astype(np.float32)
    x = g.standard_normal((w.K, N), dtype=np.float32)
    np.maximum(x, 0, out=x)
    return x


def device_activations(w: Workload, device):
    """I[K][N] float32 on `device`, max(0, N(0,1)) (U[-1,1] for "uniform") from torch's seeded generator: for
    full-size cells whose host copy would take longer to draw than the product to check.  The values differ
    from activations() (another generator); callers read back the columns they hand to the oracle."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(w.i_seed)
    if w.i_dist == "uniform":
        return torch.rand((w.K, w.N), generator=g, device=device) * 2 - 1
    return torch.randn((w.K, w.N), generator=g, device=device).clamp_(min=0)


def output_gradients(w: Workload, N: int | None = None) -> np.ndarray:
    """dO[M][N] float32 ~ N(0, 1): the gradient arriving at the layer's output in a training
    step (dense, signed), seeded from the activations' seed."""
    N = w.N if N is None else N
    g = np.random.Generator(np.random.PCG64(w.i_seed + 7919))
    return g.standard_normal((w.M, N), dtype=np.float32)


def conv_activations(w: Workload, images: int, height: int, width: int) -> np.ndarray:
    """X[channel][image][height][width] float32 ~ max(0, N(0,1)) for the fused 3x3
    convolution (channels = K / 9), seeded like `activations`."""
    g = np.random.Generator(np.random.PCG64(w.i_seed))
    x = g.standard_normal((w.K // 9, images, height, width), dtype=np.float32)
    np.maximum(x, 0, out=x)
    return x


def zero_padded(x: np.ndarray) -> np.ndarray:
    """[C][B][H][W] -> [C][B][H+2][W+2] with a zero border (the layout rbgp_conv3x3 reads)."""
    C, B, H, W = x.shape
    out = np.zeros((C, B, H + 2, W + 2), dtype=x.dtype)
    out[:, :, 1:-1, 1:-1] = x
    return out


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16) with torch's conversion."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_as_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
