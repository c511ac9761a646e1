"""GPU parity of the tile family (RBGP_KERNEL_MFMA_TILE, bf16 modes): every nonzero of G_o as a
dense block, I staged in LDS by producer waves, 32-row MFMAs; against the CPU oracle."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl
from tests import gpu_harness as gh
from tests.test_gpu_bf16_output import check_bf16_output

pytestmark = pytest.mark.gpu

TILE = rb.KERNEL_MFMA_TILE

SHAPES = [
    # rows, cols, row degrees: 32 rows per tile; stage lengths 288, 144, 72 (padded to 80), 32, 36 (padded to 64), 320
    ((8, 4, 4, 2), (8, 4, 8, 9), (4, 4, 4, 9)),
    ((4, 2, 8, 2), (8, 2, 8, 9), (4, 2, 4, 9)),
    ((6, 2, 4, 4), (6, 2, 4, 9), (3, 2, 2, 9)),
    ((8, 4, 8, 1), (16, 1, 32, 1), (4, 1, 8, 1)),
    ((2, 1, 32, 1), (2, 1, 4, 9), (2, 1, 2, 9)),
    ((3, 4, 4, 2), (3, 4, 8, 10), (3, 4, 4, 10)),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s[1])))
@pytest.mark.parametrize("N", [64, 200, 1000])
def test_shapes(shape, N):
    rows, cols, deg = shape
    w = wl.Workload("tile_" + "x".join(map(str, cols)), rows, cols, deg, N, wl.BF16, 91, 92, 93, 1.0)
    gh.check_parity(w, kernel=TILE, ld_pad=(-N) % 8, expect_kernel=TILE)


def _random_tile_shapes(count, seed):
    """Seeded random shapes with 32 rows per tile and at most 320 columns per tile that the sampler accepts."""
    g = np.random.Generator(np.random.PCG64(seed))
    shapes = []
    while len(shapes) < count:
        lo, li = int(g.integers(0, 3)), int(g.integers(0, 3))
        a_o = int(g.choice([1, 2, 3, 4, 5, 6, 8, 12])) << lo
        c_o = int(g.choice([1, 2, 3, 4, 8])) << lo
        a_r, a_b = [(1, 1), (2, 1), (1, 2), (4, 1), (2, 2), (4, 2), (2, 4), (8, 1)][int(g.integers(0, 8))]
        a_i = 32 // (a_r * a_b)
        c_i = int(g.choice([1, 2, 4])) << li
        c_r, c_b = int(g.choice([1, 2, 3, 4])), int(g.choice([1, 3, 9, 10]))
        rows, cols = (a_o, a_r, a_i, a_b), (c_o, c_r, c_i, c_b)
        deg = (c_o >> lo, c_r, c_i >> li, c_b)
        if c_r * c_i * c_b > 320:
            continue
        try:
            mask = rb.rbgp_make_mask(rows, cols, deg, 700 + len(shapes))
            rb.rbgp_mask_set_kernel(mask, TILE)
        except rb.RbgpError:
            continue
        shapes.append((rows, cols, deg, int(g.integers(1, 700))))
    return shapes


def test_random_shapes():
    for idx, (rows, cols, deg, N) in enumerate(_random_tile_shapes(24, 77)):
        w = wl.Workload(f"tile_random{idx}", rows, cols, deg, N, wl.BF16, 700 + idx, 800 + idx, 900 + idx, 1.0)
        gh.check_parity(w, kernel=TILE, ld_pad=(-N) % 8, expect_kernel=TILE)


def test_conv3_full_size_and_bf16_output():
    gh.check_parity(wl.VGG19_CONV3_BF16, kernel=TILE, expect_kernel=TILE)
    assert check_bf16_output(wl.VGG19_CONV3_BF16, N=1000, kernel=TILE) == TILE


@pytest.mark.parametrize("N,ld_pad", [(1, 7), (63, 1), (65, 7), (257, 15), (8190, 2)])
def test_ragged_columns(N, ld_pad):
    gh.check_parity(wl.VGG19_CONV3_BF16, N=N, kernel=TILE, ld_pad=ld_pad, expect_kernel=TILE)


def test_one_hot_input_returns_the_dense_weights():
    """I = identity: O must equal the dense W_s bit for bit (pins the packing and every index)."""
    w = wl.Workload("tile_one_hot", (4, 2, 8, 2), (8, 2, 8, 9), (4, 2, 4, 9), 0, wl.BF16, 94, 95, 96, 1.0)
    w = replace(w, N=w.K)
    vb = wl.to_bf16_bits(wl.kept_weights(w))
    eye = wl.to_bf16_bits(np.eye(w.K, dtype=np.float32))
    out, used = gh.library_spmm(w, vb, eye, kernel=TILE)
    assert used == TILE
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    dense = orc.scatter_values(orc.kron_mask(Bs), wl.bf16_bits_as_f32(vb))
    assert np.array_equal(out, dense.astype(np.float32))


def test_family_limits():
    import torch
    mask = gh.make_mask(wl.VGG19_CONV5)                      # fp32 calls take the default family
    rb.rbgp_mask_set_kernel(mask, TILE)
    assert rb.rbgp_mask_kernel(mask, rb.F32) == rb.KERNEL_MFMA_REG
    assert rb.rbgp_mask_kernel(mask, rb.BF16_F32ACC) == TILE
    w = wl.WRN_G1                                            # 8 rows per tile: not covered
    with pytest.raises(rb.RbgpError) as e:
        rb.rbgp_mask_set_kernel(gh.make_mask(w), TILE)
    assert e.value.code == rb.EUNSUPPORTED
    w = replace(wl.VGG19_CONV3_BF16, N=64)
    mask = gh.make_mask(w)
    rb.rbgp_mask_set_kernel(mask, TILE)
    packed = torch.zeros(rb.rbgp_packed_bytes(mask, rb.BF16), dtype=torch.uint8, device="cuda:0")
    I_d = torch.zeros((w.K, w.N + 4), dtype=torch.int16, device="cuda:0")
    O_d = torch.zeros((w.M, w.N), dtype=torch.float32, device="cuda:0")
    with pytest.raises(rb.RbgpError) as e:                   # leading dimension not a multiple of 8
        rb.rbgp_spmm(mask, rb.BF16_F32ACC, w.M, w.K, w.N, packed.data_ptr(), I_d.data_ptr(), w.N + 4, O_d.data_ptr(), w.N, 0)
    assert e.value.code == rb.ESHAPE
    with pytest.raises(rb.RbgpError) as e:                   # fused convolution: image width a multiple of 8
        rb.rbgp_conv3x3(mask, rb.BF16_F32ACC, w.M, w.K // 9, 4, 4, 4, packed.data_ptr(), I_d.data_ptr(), O_d.data_ptr(), 64, 0)
    assert e.value.code == rb.ESHAPE
    torch.cuda.synchronize()


CONV_CASES = [
    # workload (32 rows per tile, K = 9 * channels), images, height, width
    (wl.VGG19_CONV3_BF16, 128, 8, 8),                                   # 256 -> 256 channels, 8x8 pixels, batch 128
    (replace(wl.VGG19_CONV3_BF16, name="tile_conv3_ragged"), 33, 8, 8),  # 33 column tiles
    (wl.Workload("tile_conv_w16", (4, 2, 8, 2), (8, 2, 8, 9), (4, 2, 4, 9), 0, wl.BF16, 61, 62, 63, 1.0), 3, 5, 16),
    (wl.Workload("tile_conv_w32", (6, 2, 4, 4), (6, 2, 4, 9), (3, 2, 2, 9), 0, wl.BF16, 64, 65, 66, 1.0), 2, 3, 32),
    (wl.Workload("tile_conv_pad", (2, 1, 32, 1), (2, 1, 4, 9), (2, 1, 2, 9), 0, wl.BF16, 67, 68, 69, 1.0), 5, 4, 8),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: c[0].name)
def test_fused_conv3x3(case):
    """rbgp_conv3x3 on the tile family (the producers read the padded activations instead of the lowered
    matrix) = the oracle's product with the explicitly lowered input; fp32 and bf16 output."""
    w, B, H, W = case
    vals_lib, X_lib = wl.to_bf16_bits(wl.kept_weights(w)), wl.to_bf16_bits(wl.conv_activations(w, B, H, W))
    vals, X = wl.bf16_bits_as_f32(vals_lib), wl.bf16_bits_as_f32(X_lib)
    ref, den = gh.oracle_spmm(w, vals, orc.im2col_3x3(X))
    out = gh.library_conv3x3(w, vals_lib, X_lib, kernel=TILE)
    err = orc.normalised_error(out, ref, den)
    print(f"[gpu]   normalised error {err:.3e}", flush=True)
    assert err <= gh.TOL[wl.BF16], err
    out16 = gh.library_conv3x3(w, vals_lib, X_lib, kernel=TILE, out_bf16=True)
    assert np.array_equal((out16.view(np.uint32) >> 16).astype(np.uint16), orc.f32_to_bf16_bits(out))


@pytest.mark.parametrize("case", [
    (wl.VGG19_CONV3_BF16, 16, 8, 8),                                     # transposed: 32 x 288 tiles again
    (wl.Workload("tile_dx_w16", (4, 4, 4, 2), (4, 4, 8, 9), (2, 4, 8, 9), 0, wl.BF16, 71, 72, 73, 1.0), 3, 5, 16),
    (wl.Workload("tile_dx_ragged", (8, 2, 2, 4), (4, 4, 8, 9), (4, 4, 4, 9), 0, wl.BF16, 74, 75, 76, 1.0), 5, 3, 8),
], ids=lambda c: c[0].name)
def test_fused_conv3x3_input_gradient(case):
    """dX of the fused convolution = rbgp_conv3x3 of the zero-padded dO on the mask of the transposed
    convolution (32 rows per tile whenever |G_r.V| |G_i.V| = 32), run on the tile family; against the
    oracle's transposed product folded back onto the pixels."""
    from oracle import naive_c
    w, B, H, W = case
    w = replace(w, N=B * H * W)
    vl, dOl = wl.to_bf16_bits(wl.kept_weights(w)), wl.to_bf16_bits(wl.output_gradients(w))
    vals, dO = wl.bf16_bits_as_f32(vl), wl.bf16_bits_as_f32(dOl)
    got, used = gh.library_conv3x3_input_gradient(w, vl, dOl, B, H, W, kernel=TILE)
    assert used == TILE
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    mask = orc.kron_mask(Bs)
    Wd = orc.scatter_values(mask, vals)
    maskT, WT = np.ascontiguousarray(mask.T), np.ascontiguousarray(Wd.T)
    dI, dI_den = naive_c.spmm(maskT, WT, dO), naive_c.spmm_abs(maskT, WT, dO)
    ref = orc.col2im_3x3(dI, B, H, W).reshape(w.K // 9, -1)
    den = orc.col2im_3x3(dI_den, B, H, W).reshape(w.K // 9, -1)
    err = orc.normalised_error(got, ref, den)
    print(f"[gpu]   normalised error {err:.3e}", flush=True)
    assert err <= gh.TOL[wl.BF16], err
