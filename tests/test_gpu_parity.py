"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs, element by element."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu

GEN, MFMA, REG = rb.KERNEL_GENERIC, rb.KERNEL_MFMA, rb.KERNEL_MFMA_REG
FILLED = rb.KERNEL_MFMA_REG_FILLED


# ------------------------------------------------------------------ fixed configurations, full size
@pytest.mark.parametrize("w", wl.CONFIGS, ids=lambda w: w.name)
def test_config_full_size_default_launch(w):
    """The launch configuration bench.py times (library defaults)."""
    gh.check_parity(w, expect_kernel=REG)


@pytest.mark.parametrize("w", [wl.TINY, wl.VGG19_CONV5, wl.VGG19_CONV3_BF16], ids=lambda w: w.name)
def test_config_generic_kernel(w):
    gh.check_parity(w, N=min(w.N, 1024), kernel=GEN, expect_kernel=GEN)


@pytest.mark.parametrize("tune", [(1, 64, 0), (2, 128, 0), (1, 64, 2), (2, 128, 1)])
@pytest.mark.parametrize("w", [wl.VGG19_CONV5, wl.VGG19_CONV3_BF16, wl.WRN_G1], ids=lambda w: w.name)
def test_config_tile_shapes(w, tune):
    gh.check_parity(w, N=1536 if w.N > 4096 else w.N, kernel=MFMA, tune=tune)


@pytest.mark.parametrize("pairing", [0, 1, 2])
@pytest.mark.parametrize("w", [wl.TINY, wl.VGG19_CONV5, wl.VGG19_CONV3_BF16, wl.WRN_G1], ids=lambda w: w.name)
def test_config_register_family_row_pairing(w, pairing):
    """Fixed pairs of tile rows (1) and tile-by-tile pairing (2; fp32 masks with two tile rows of 8
    per MFMA group only: the conv5 shape, the others must refuse it), at a ragged N."""
    N = 1000 if w.N > 4096 else w.N
    if pairing == 2 and w is not wl.VGG19_CONV5:
        with pytest.raises(rb.RbgpError) as e:
            gh.check_parity(w, N=N, kernel=REG, tune=(0, 0, 0, pairing), expect_kernel=REG)
        assert e.value.code == rb.EUNSUPPORTED
        return
    gh.check_parity(w, N=N, kernel=REG, tune=(0, 0, 0, pairing), expect_kernel=REG)


# masks with two tile rows of 8 rows per MFMA group, for the tile-by-tile pairing of the fp32 register kernels
PAIRING_SHAPES = [
    ((4, 4, 4, 2), (4, 4, 8, 9), (2, 4, 2, 9)),     # 4 tile rows: one quad
    ((8, 2, 2, 3), (8, 2, 4, 3), (4, 2, 2, 3)),     # R = 6 (two idle rows per half), stages of 12 steps padded to 18
    ((6, 4, 2, 2), (4, 1, 4, 9), (2, 1, 2, 9)),     # 6 tile rows: a quad with two rows missing
    ((2, 8, 2, 1), (4, 2, 2, 4), (2, 2, 1, 4)),     # 2 tile rows: a quad with one L row and one H row
    ((16, 1, 2, 8), (16, 2, 4, 2), (4, 2, 2, 2)),   # 16 tile rows of degree 4 (two lifts): tiles without a partner
    ((4, 21, 2, 1), (4, 1, 2, 9), (2, 1, 1, 9)),    # |G_r.U| = 21: three tile rows of 7 per row of G_o
]


@pytest.mark.parametrize("shape", range(len(PAIRING_SHAPES)))
def test_fp32_register_family_tile_by_tile_pairing(shape):
    """The pairing kernel against the oracle (and the fixed-pair kernel on the same inputs) on small masks
    that exercise incomplete quads, idle rows, padded stages and partnerless tiles, at two ragged N with
    an odd leading dimension; the host tables pass the library's own consistency check."""
    a, c, d = PAIRING_SHAPES[shape]
    for N in (200, 129):
        w = wl.Workload(f"pairing_{shape}", a, c, d, N, wl.F32, 100 + shape, 200 + shape, 300 + shape, 1.0)
        rb.rbgp_mask_check_tables(gh.make_mask(w))
        assert rb.rbgp_mask_reg_plan(gh.make_mask(w))[7] > 0
        gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 2), ld_pad=3, expect_kernel=REG)
        gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 1), ld_pad=3, expect_kernel=REG)


@pytest.mark.parametrize("cw", [64, 128])
@pytest.mark.parametrize("split", [1, 2, 4])
@pytest.mark.parametrize("groups", [1, 2, 4])
def test_bf16_register_family_row_groups_and_stage_split(groups, split, cw):
    """bf16 register kernels: every (16-row groups per wave, waves per column tile,
    columns per wave) combination, on the conv3 shape (ragged last tile) and on shapes
    with fewer tile rows than one cluster holds, a partial 4-row block, an odd stage
    count, 12 tile rows."""
    tune = (0, cw, 0, 0, groups, split)
    gh.check_parity(wl.VGG19_CONV3_BF16, N=1000, kernel=REG, tune=tune, expect_kernel=REG)
    w = wl.Workload("bf16_small_cluster", (2, 1, 4, 3), (4, 2, 4, 9), (2, 2, 2, 9), 330, wl.BF16, 11, 12, 13, 1.0)
    gh.check_parity(w, kernel=REG, tune=tune, ld_pad=6, expect_kernel=REG)   # (ldI must be a multiple of 8)
    w = wl.Workload("bf16_rs4", (6, 2, 4, 2), (6, 1, 4, 9), (3, 1, 2, 9), 200, wl.BF16, 21, 22, 23, 1.0)
    gh.check_parity(w, kernel=REG, tune=tune, expect_kernel=REG)
    w = wl.Workload("bf16_12_tile_rows", (12, 1, 2, 3), (8, 1, 4, 9), (2, 1, 2, 9), 136, wl.BF16, 31, 32, 33, 1.0)
    gh.check_parity(w, kernel=REG, tune=tune, expect_kernel=REG)


@pytest.mark.parametrize("split", [2, 4])
def test_fp32_register_family_stage_split(split):
    """fp32 register kernels with the stage list split over 2 or 4 waves (LDS reduction)."""
    tune = (0, 0, 0, 0, 0, split)
    for w, N in [(wl.TINY, None), (wl.VGG19_CONV5, 520), (wl.WRN_G1, 1000)]:
        gh.check_parity(w, N=N, kernel=REG, tune=tune, expect_kernel=REG)
    w = wl.Workload("fp32_small_cluster", (2, 1, 4, 3), (4, 2, 4, 9), (2, 2, 2, 9), 331, wl.F32, 11, 12, 13, 1.0)
    gh.check_parity(w, kernel=REG, tune=tune, ld_pad=2, expect_kernel=REG)   # odd leading dimension
    gh.check_parity(wl.VGG19_CONV5, kernel=REG, tune=tune, expect_kernel=REG)


def test_bf16_register_family_full_size_split_shapes():
    for tune in [(0, 128, 0, 0, 4, 4), (0, 128, 0, 0, 2, 2), (0, 64, 0, 0, 4, 2), (0, 64, 0, 0, 2, 2), (0, 64, 0, 0, 1, 1)]:
        gh.check_parity(wl.VGG19_CONV3_BF16, kernel=REG, tune=tune, expect_kernel=REG)


def test_lds_family_full_size():
    for w in (wl.VGG19_CONV5, wl.VGG19_CONV3_BF16, wl.WRN_G1):
        gh.check_parity(w, kernel=MFMA, expect_kernel=MFMA)


# ------------------------------------------------------------------ ragged and degenerate sizes
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("N,ld_pad", [(1, 7), (63, 1), (64, 0), (65, 3), (200, 8), (257, 15)])
def test_ragged_columns(N, ld_pad, dtype):
    """Column counts that leave a partial tile, with a padded leading dimension
    (pad columns of O must stay untouched)."""
    epc = 8 if dtype == wl.BF16 else 4
    pad = (-N) % epc + ld_pad // epc * epc            # keeps ldI a multiple of the 16-byte chunk
    w = replace(wl.VGG19_CONV5, rows=(4, 4, 4, 2), cols=(4, 4, 8, 9), row_deg=(2, 4, 2, 9), dtype=dtype,
                name=f"ragged_{dtype}")
    for tune in [(1, 64, 0), (2, 128, 0)]:
        gh.check_parity(w, N=N, kernel=MFMA, tune=tune, ld_pad=pad)
    gh.check_parity(w, N=N, kernel=GEN, ld_pad=ld_pad)
    for pairing in (1, 2):
        gh.check_parity(w, N=N, kernel=REG, tune=(0, 0, 0, pairing if dtype == wl.F32 else 1), ld_pad=ld_pad if dtype == wl.F32 else pad,
                        expect_kernel=REG)
    if dtype == wl.BF16:                              # 128-column wave tiles, with and without a stage split
        gh.check_parity(w, N=N, kernel=REG, tune=(0, 128), ld_pad=pad, expect_kernel=REG)
        gh.check_parity(w, N=N, kernel=REG, tune=(0, 128, 0, 0, 2, 2), ld_pad=pad, expect_kernel=REG)


def test_empty_input_is_a_noop():
    import torch
    w = wl.TINY
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 1)
    O = torch.full((w.M, 4), 5.0, device="cuda:0")
    rb.rbgp_spmm(mask, w.dtype, w.M, w.K, 0, 0, 0, 0, O.data_ptr(), 0, 0)
    torch.cuda.synchronize()
    assert bool((O == 5.0).all())


def test_misaligned_input_is_rejected_by_the_mfma_family():
    import torch
    w = wl.TINY
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 1)
    rb.rbgp_mask_set_kernel(mask, MFMA)
    packed = torch.zeros(rb.rbgp_packed_bytes(mask, w.dtype), dtype=torch.uint8, device="cuda:0")
    I = torch.zeros(w.K * 70 + 8, device="cuda:0")
    O = torch.zeros(w.M * 70, device="cuda:0")
    with pytest.raises(rb.RbgpError) as ei:
        rb.rbgp_spmm(mask, w.dtype, w.M, w.K, 66, packed.data_ptr(), I.data_ptr(), 66, O.data_ptr(), 66, 0)
    assert ei.value.code == rb.ESHAPE
    with pytest.raises(rb.RbgpError) as ei:
        rb.rbgp_spmm(mask, w.dtype, w.M, w.K, 64, packed.data_ptr(), I.data_ptr() + 4, 64, O.data_ptr(), 64, 0)
    assert ei.value.code == rb.ESHAPE
    torch.cuda.synchronize()


# ------------------------------------------------------------------ exact cases
@pytest.mark.parametrize("kernel", [GEN, MFMA, REG])
@pytest.mark.parametrize("w", [wl.TINY, replace(wl.WRN_G1, N=576)], ids=lambda w: w.name)
def test_one_hot_input_returns_dense_weights_exactly(w, kernel):
    """I = identity: every output is one kept weight times 1 plus zeros, exact
    in fp32.  Pins the pack permutation and every index bit for bit."""
    vals = wl.kept_weights(w)
    I = np.eye(w.K, dtype=np.float32)
    out, _ = gh.library_spmm(w, vals, I, kernel, tag="one-hot")
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    W = orc.scatter_values(orc.kron_mask(Bs), vals)
    assert np.array_equal(out, W)


def test_one_hot_bf16_exact():
    w = replace(wl.TINY, dtype=wl.BF16, name="tiny_bf16")
    vb = wl.to_bf16_bits(wl.kept_weights(w))
    Ib = wl.to_bf16_bits(np.eye(w.K, dtype=np.float32))
    for kernel in (GEN, MFMA, REG):
        out, _ = gh.library_spmm(w, vb, Ib, kernel, tag="one-hot bf16")
        Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
        W = orc.scatter_values(orc.kron_mask(Bs), wl.bf16_bits_as_f32(vb))
        assert np.array_equal(out, W)


def test_all_complete_factors_is_a_dense_gemm():
    w = wl.Workload("dense_32x72", (2, 4, 2, 2), (1, 2, 4, 9), (1, 2, 4, 9), 300, wl.F32, 1, 2, 3)
    if gh.family_covers(w, MFMA):      # (a complete G_i counts as row repetition: 16 rows share a column set here,
        gh.check_parity(w, kernel=MFMA, ld_pad=0)   #  more than the LDS family's blocks hold)
    gh.check_parity(w, kernel=REG, expect_kernel=REG)
    gh.check_parity(w, kernel=GEN)


# ------------------------------------------------------------------ shapes across the kernel table
FUZZ = [
    # rows, cols, row_deg  (G_r, G_b complete)                     covers
    ((2, 1, 2, 1), (4, 1, 4, 1), (2, 1, 2, 1)),                    # R=1, KS=2
    ((4, 2, 8, 1), (4, 3, 8, 1), (2, 3, 4, 1)),                    # R=2, KS=4, |G_r.V|=3
    ((2, 1, 16, 4), (2, 1, 16, 2), (2, 1, 8, 2)),                  # R=4, KS=16
    ((4, 4, 16, 1), (8, 1, 32, 1), (4, 1, 8, 1)),                  # Table-2-like: R=4, KS=8, 16 groups
    ((2, 2, 32, 2), (4, 1, 64, 1), (2, 1, 32, 1)),                 # KS=32, 32 groups
    ((4, 2, 4, 4), (4, 2, 8, 9), (2, 2, 4, 9)),                    # R=8, KS=36
    ((2, 4, 4, 2), (2, 2, 16, 9), (1, 2, 8, 9)),                   # KS=72
    ((4, 1, 4, 3), (4, 2, 4, 9), (2, 2, 2, 9)),                    # R=3 (partial 4-row block)
    ((2, 3, 4, 2), (2, 2, 4, 9), (1, 2, 2, 9)),                    # R=6 (one full, one partial block)
    # the remaining (stage size, row group) pairs of the register family's kernel table
    ((2, 4, 16, 1), (2, 1, 16, 1), (2, 1, 8, 1)),                  # KC=8,  RS=4
    ((4, 2, 4, 1), (4, 1, 4, 9), (2, 1, 2, 9)),                    # KC=18, RS=2
    ((4, 2, 4, 1), (4, 2, 4, 9), (2, 2, 2, 9)),                    # KC=36, RS=2
    ((4, 1, 4, 2), (4, 2, 8, 9), (2, 2, 4, 9)),                    # KC=72, RS=2
    ((4, 2, 4, 2), (4, 1, 4, 9), (2, 1, 2, 9)),                    # KC=18, RS=4
    ((4, 2, 4, 2), (4, 2, 8, 9), (2, 2, 4, 9)),                    # KC=72, RS=4
    ((4, 4, 4, 2), (4, 1, 4, 9), (2, 1, 2, 9)),                    # KC=18, RS=8
    # stages whose length is padded to the next kernel size
    ((4, 2, 4, 2), (4, 2, 4, 3), (2, 2, 2, 3)),                    # 12 steps in KC=18
    ((2, 1, 8, 4), (2, 3, 8, 3), (1, 3, 2, 3)),                    # 18 = 3 x 2 x 3
    ((4, 2, 4, 1), (4, 1, 12, 9), (2, 1, 6, 9)),                   # 54 steps in KC=72
    ((4, 4, 4, 1), (4, 5, 4, 1), (2, 5, 1, 1)),                    # 5 steps in KC=8
    ((4, 1, 8, 3), (4, 3, 8, 3), (2, 3, 2, 3)),                    # R=3, 18 steps
    # more than 16 rows per tile row: rows of G_r move into the tile-row index
    ((2, 8, 4, 3), (2, 2, 4, 9), (1, 2, 2, 9)),                    # R=24 -> 2 x 12
    ((4, 4, 2, 9), (4, 4, 4, 2), (2, 4, 2, 2)),                    # R=36 -> 4 x 9 (a transposed 3x3 layer)
    # a complete G_i joins G_r in the kernels' view (all the sparsity in G_o)
    ((2, 2, 32, 2), (4, 1, 32, 1), (2, 1, 32, 1)),                 # 128 rows share a column set
    ((2, 4, 4, 2), (2, 2, 8, 9), (1, 2, 8, 9)),                    # R=32 -> 2 x 16, stages of 72
    ((8, 4, 4, 2), (8, 4, 8, 9), (4, 4, 8, 9)),                    # a VGG19 layer at density 1/2
    ((4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9)),                    # R=16, stages of 36
]
REG_COVERED = set(range(5, 23))               # must run on the register family


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("idx", range(len(FUZZ)))
def test_shapes_across_the_kernel_table(idx, dtype):
    rows, cols, deg = FUZZ[idx]
    w = wl.Workload(f"fuzz{idx}_{dtype}", rows, cols, deg, 328, dtype, 100 + idx, 200 + idx, 300 + idx, 1.0)
    if gh.family_covers(w, MFMA):
        gh.check_parity(w, kernel=MFMA, tune=(1, 64, 0))
        gh.check_parity(w, kernel=MFMA, tune=(2, 128, 0))
    else:
        assert idx >= 9                       # the first nine shapes are inside the LDS family's table
    gh.check_parity(w, kernel=GEN)
    if gh.family_covers(w, FILLED):           # few rows per column set and a sparse G_i: the mask with G_i filled in
        gh.check_parity(w, kernel=FILLED, expect_kernel=FILLED)
        gh.check_parity(w, kernel=FILLED, tune=(0, 0, 0, 0, 0, 2), ld_pad=8, expect_kernel=FILLED)
    covered = gh.family_covers(w, REG)
    assert covered or idx not in REG_COVERED
    if covered:
        # tile-by-tile pairing of the tile rows where the library's plan has it (fp32, two tile rows per MFMA group)
        pairing = dtype == wl.F32 and rb.rbgp_mask_reg_plan(gh.make_mask(w))[7] > 0
        for tune in [(0, 0, 0, 1), (0, 0, 0, 0, 0, 2)] + ([(0, 0, 0, 2)] if pairing else []) + \
                ([(0, 64, 0, 0, 2, 1), (0, 128, 0, 0, 1, 4)] if dtype == wl.BF16 else []):
            gh.check_parity(w, kernel=REG, tune=tune, expect_kernel=REG)


# stage lists as long as or longer than the 64 stages one wave holds: split over 2 or 4 waves of the workgroup
LONG_LISTS = [
    ((4, 2, 2, 1), (128, 1, 2, 1), (64, 1, 2, 1)),     # 64 tiles per tile row (complete G_i joins G_r): 2 waves
    ((4, 4, 1, 2), (256, 1, 1, 2), (128, 1, 1, 2)),    # G_o of 256 tile columns at 1/2, two tile rows per cluster: 3 waves
    ((4, 2, 4, 2), (64, 4, 8, 9), (32, 4, 4, 9)),      # two stages of 72 steps per tile, four tile rows per cluster
    ((8, 1, 4, 1), (64, 2, 4, 2), (16, 2, 1, 2)),      # clusters of 8 tile rows whose union fills one wave's table to the last lane
]


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("idx", range(len(LONG_LISTS)))
def test_register_family_stage_lists_beyond_one_wave(idx, dtype):
    """Clusters that walk 64..256 stages: beyond 64 the register kernels split the list over the waves of a workgroup
    whatever N is (default launch), also with the largest split asked for; the tables pass the self check."""
    rows, cols, deg = LONG_LISTS[idx]
    for N in (200, 1100):
        w = wl.Workload(f"long{idx}_{dtype}", rows, cols, deg, N, dtype, 400 + idx, 500 + idx, 600 + idx, 1.0)
        m = gh.make_mask(w)
        rb.rbgp_mask_check_tables(m)
        assert 64 <= rb.rbgp_mask_reg_plan(m)[5] <= 256
        gh.check_parity(w, kernel=REG, expect_kernel=REG, ld_pad=8)
        gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 0, 0, 4), expect_kernel=REG)
    if rb.rbgp_mask_reg_plan(m)[5] > 64:         # one wave cannot hold this list
        with pytest.raises(rb.RbgpError) as e:
            gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 0, 0, 1), expect_kernel=REG)
        assert e.value.code == rb.EUNSUPPORTED
    else:
        gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 0, 0, 1), expect_kernel=REG)


# masks with at most four rows per column set and a sparse G_i (the shapes of Table 3's slow rows, small)
FILLED_SHAPES = [
    ((4, 1, 16, 1), (8, 1, 8, 1), (4, 1, 4, 1)),       # R = 1: 16 rows per tile row after the fill, stages of 8 steps
    ((2, 2, 32, 1), (4, 1, 32, 1), (2, 1, 8, 1)),      # R = 2, G_i at 1/4: 64 rows -> four 16-row groups per tile row
    ((4, 1, 8, 4), (8, 3, 8, 2), (2, 3, 2, 2)),        # R = 4 from G_b, |G_r.V| = 3: stages of 48 steps padded to 72
    ((2, 1, 12, 1), (64, 1, 4, 1), (64, 1, 2, 1)),     # complete G_o of 64 tiles: a stage list split over two waves
    ((8, 1, 4, 3), (8, 1, 8, 1), (2, 1, 2, 1)),        # R = 3, 12 rows per tile row: a partial 16-row group
]


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("idx", range(len(FILLED_SHAPES)))
def test_register_family_on_the_mask_with_g_i_filled_in(idx, dtype):
    """RBGP_KERNEL_MFMA_REG_FILLED against the oracle of the ORIGINAL mask: the zeros stored where G_i has no
    edge must change nothing; forward and transposed products, ragged N, padded leading dimension."""
    rows, cols, deg = FILLED_SHAPES[idx]
    w = wl.Workload(f"filled{idx}_{dtype}", rows, cols, deg, 328, dtype, 700 + idx, 800 + idx, 900 + idx, 1.0)   # (bf16: ldI % 8 == 0)
    m = gh.make_mask(w)
    rb.rbgp_mask_check_tables(m)
    assert rb.rbgp_mask_reg_plan(m)[13] > 0
    gh.check_parity(w, kernel=FILLED, expect_kernel=FILLED)
    gh.check_parity(w, N=1096, kernel=FILLED, ld_pad=8, expect_kernel=FILLED)
    # transposed product: the filled family where the transposed mask has one, else whatever it runs on
    (vl, Il, dOl), f32 = gh.backward_inputs(w)
    want_dI, den, _, _ = gh.oracle_backward(w, *f32)
    mt = rb.rbgp_mask_transpose(m)
    kernel = FILLED if rb.rbgp_mask_reg_plan(mt)[13] > 0 else rb.KERNEL_AUTO
    got, used = gh.library_spmm_transposed(w, vl, dOl, kernel=kernel)
    assert kernel == rb.KERNEL_AUTO or used == FILLED
    assert orc.normalised_error(got, want_dI, den) <= gh.TOL[w.dtype]


def test_filled_family_is_what_auto_takes_for_one_row_per_column_set():
    """Table 3, G_r = G_b = (1, 1): the default launch is the filled family (both dtypes); never for the mask of a
    lowered 3x3 convolution, never where no filled mask exists."""
    w = wl.sdmm4096_table3(1, 1, 3)
    m = gh.make_mask(w)
    assert rb.rbgp_mask_kernel(m, wl.F32) == FILLED and rb.rbgp_mask_kernel(m, wl.BF16) == FILLED
    assert rb.rbgp_mask_kernel(gh.make_mask(wl.WRN_G1), wl.F32) == REG
    with pytest.raises(rb.RbgpError) as e:
        rb.rbgp_mask_set_kernel(gh.make_mask(wl.VGG19_CONV5), FILLED)
    assert e.value.code == rb.EUNSUPPORTED


# masks whose rows of G_r move into the tile-row index (more than 16 rows per column set): fp32 waves that take 2 or 4
# of the tile rows that share their tiles
ROW_GROUP_SHAPES = [
    ((2, 8, 4, 3), (2, 2, 4, 9), (1, 2, 2, 9), (2,)),        # R = 24 -> 2 x 12, stages of 36
    ((4, 4, 2, 11), (4, 4, 4, 2), (2, 4, 2, 2), (2, 4)),     # R = 44 -> 4 x 11, stages of 16 in 18
    ((2, 2, 32, 2), (4, 1, 32, 1), (2, 1, 32, 1), (2,)),     # complete G_i: 128 rows -> 8 x 16, stages of 32 (no kernel of 4 groups)
    ((2, 4, 4, 2), (2, 2, 8, 9), (1, 2, 8, 9), (2,)),        # R = 32 -> 2 x 16, stages of 72
    ((4, 8, 1, 8), (8, 2, 1, 9), (4, 2, 1, 9), (2, 4)),      # R = 64 -> 4 x 16, stages of 18
]


@pytest.mark.parametrize("idx", range(len(ROW_GROUP_SHAPES)))
def test_fp32_register_family_row_groups_per_wave(idx):
    """RBGP_TUNE_ROW_GROUPS on the fp32 register kernels (2 or 4 tile rows with the same tiles per wave), ragged N,
    padded leading dimension, alone and with a split stage list; refused where the tile rows do not come in such groups."""
    rows, cols, deg, groups = ROW_GROUP_SHAPES[idx]
    w = wl.Workload(f"rowgroups{idx}", rows, cols, deg, 333, wl.F32, 40 + idx, 50 + idx, 60 + idx, 1.0)
    for ng in groups:
        gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 0, ng), ld_pad=3, expect_kernel=REG)
        gh.check_parity(w, N=64, kernel=REG, tune=(0, 0, 0, 0, ng), expect_kernel=REG)
    gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 0, 2, 2), expect_kernel=REG)     # with a split stage list as well
    gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 0, 2, 0, 0, 2), ld_pad=1, expect_kernel=REG)   # two register sets
    gh.check_parity(w, N=200, kernel=REG, tune=(0, 0, 0, 0, groups[-1], 4), ld_pad=1, expect_kernel=REG)
    if 4 not in groups:
        with pytest.raises(rb.RbgpError) as e:
            gh.check_parity(w, kernel=REG, tune=(0, 0, 0, 0, 4), expect_kernel=REG)
        assert e.value.code == rb.EUNSUPPORTED


# more than 16 rows per column set with a composite |G_b.U|: the register family runs on the same mask factored as
# G_o (x) G_r (x) (G_i (x) J(q, 1)) (x) J(|G_b.U| / q, .), whose MFMA groups are fuller.  (rows, cols, degrees, rows per
# group before and after)
REGROUP_SHAPES = [
    ((4, 4, 2, 9), (4, 4, 4, 2), (2, 4, 2, 2), 9, 12),      # a transposed 3x3 layer: 36 rows, 4 x 9 -> 3 x 12
    ((4, 8, 2, 9), (4, 2, 2, 2), (2, 2, 1, 2), 9, 12),      # 72 rows: 8 x 9 -> 6 x 12, stages of 4 steps in 8
    ((2, 32, 1, 9), (2, 4, 2, 2), (1, 4, 2, 2), 9, 16),     # 288 rows: 32 x 9 -> 18 x 16
    ((4, 4, 4, 12), (4, 2, 4, 3), (2, 2, 2, 3), 12, 16),    # 48 rows: 4 x 12 -> 3 x 16
]


@pytest.mark.parametrize("idx", range(len(REGROUP_SHAPES)))
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_register_family_on_the_regrouped_mask(idx, dtype):
    rows, cols, deg, before, after = REGROUP_SHAPES[idx]
    N = 333 if dtype == wl.F32 else 328
    w = wl.Workload(f"regroup{idx}", rows, cols, deg, N, dtype, 250 + idx, 260 + idx, 270 + idx, 1.0)
    mask = rb.rbgp_make_mask(rows, cols, deg, w.mask_seed)
    plan = rb.rbgp_mask_reg_plan(mask)
    assert plan[14] == after                      # rows of the MFMA group in use on the regrouped mask
    rb.rbgp_mask_check_tables(mask)
    gh.check_parity(w, kernel=REG, ld_pad=3 if dtype == wl.F32 else 8, expect_kernel=REG)
    gh.check_parity(w, N=64, kernel=REG, expect_kernel=REG)
    gh.check_parity(w, N=2312, kernel=REG, tune=(0, 0, 0, 0, 0, 1), expect_kernel=REG)
    gh.check_parity(w, N=200, kernel=REG, tune=(0, 0, 0, 0, 0, 2), expect_kernel=REG)
    gh.check_parity(w, kernel=rb.KERNEL_AUTO)
    gh.check_parity(w, kernel=GEN, expect_kernel=GEN)   # the generic family runs the mask as given: same results


# a complete G_o: the register family runs on the same mask with G_o (x) G_r merged into one tile column, whose
# stages are longer (rows, cols, degrees, steps per stage before and after)
MERGED_COLUMN_SHAPES = [
    ((4, 2, 2, 4), (4, 2, 4, 2), (4, 2, 2, 2), 8, 32),          # 4 tiles of 8 steps -> one stage of 32
    ((8, 2, 2, 2), (8, 1, 4, 4), (8, 1, 2, 4), 8, 72),          # 8 tiles of 8 steps -> one stage of 64 in 72
    ((8, 1, 4, 1), (8, 2, 4, 2), (8, 2, 2, 2), 8, 72),          # one row per column set
    ((2, 4, 1, 2), (128, 1, 1, 2), (128, 1, 1, 2), 8, 72),      # 128 tiles of 2 steps in 8 -> 4 stages of 64 in 72
    ((4, 4, 8, 1), (32, 1, 8, 1), (32, 1, 2, 1), 8, 72),        # Table 2's shape with a complete G_o, small
]


@pytest.mark.parametrize("idx", range(len(MERGED_COLUMN_SHAPES)))
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_register_family_on_the_mask_with_merged_tile_columns(idx, dtype):
    rows, cols, deg, before, after = MERGED_COLUMN_SHAPES[idx]
    N = 333 if dtype == wl.F32 else 328
    w = wl.Workload(f"merged{idx}", rows, cols, deg, N, dtype, 280 + idx, 290 + idx, 295 + idx, 1.0)
    mask = rb.rbgp_make_mask(rows, cols, deg, w.mask_seed)
    plan = rb.rbgp_mask_reg_plan(mask)
    assert plan[2] == before and plan[14] > 0 and plan[15] > 0
    rb.rbgp_mask_check_tables(mask)
    gh.check_parity(w, kernel=REG, ld_pad=3 if dtype == wl.F32 else 8, expect_kernel=REG)
    gh.check_parity(w, N=64 if dtype == wl.F32 else 128, kernel=REG, expect_kernel=REG)
    gh.check_parity(w, N=2312, kernel=REG, tune=(0, 0, 0, 0, 0, 1), expect_kernel=REG)
    gh.check_parity(w, N=200, kernel=REG, tune=(0, 0, 0, 0, 0, 2), expect_kernel=REG)
    gh.check_parity(w, kernel=GEN, expect_kernel=GEN)


def test_regrouped_masks_randomised():
    """Seeded random masks with a composite |G_b.U| and up to 16 x 15 rows per column set, fp32, register family:
    the result is the oracle's whether or not the library regroups the mask; at least a third of them are regrouped."""
    g = np.random.Generator(np.random.PCG64(20))
    ran = regrouped = 0
    for it in range(60):
        a_o, c_o = int(g.choice([2, 4, 8])), int(g.choice([2, 4, 8]))
        d_o = int(g.choice([x for x in (1, 2, 4, 8) if x <= c_o]))
        a_r, c_r = int(g.choice([2, 4, 8, 16])), int(g.choice([1, 2, 4]))
        a_i, c_i = int(g.choice([1, 2, 4])), int(g.choice([1, 2, 4]))
        d_i = int(g.choice([x for x in (1, 2, 4) if x <= c_i]))
        a_b, c_b = int(g.choice([4, 6, 8, 9, 10, 12, 15])), int(g.choice([1, 2, 3]))
        rows, cols, deg = (a_o, a_r, a_i, a_b), (c_o, c_r, c_i, c_b), (d_o, c_r, d_i, c_b)
        try:
            mask = rb.rbgp_make_mask(rows, cols, deg, 300 + it)
        except rb.RbgpError:
            continue                                  # (not a shape the sampler accepts)
        plan = rb.rbgp_mask_reg_plan(mask)
        if plan[0] == 0:
            continue
        rb.rbgp_mask_check_tables(mask)
        w = wl.Workload(f"regroup_rand{it}", rows, cols, deg, int(g.choice([64, 200, 333])), wl.F32, 300 + it, 301 + it,
                        302 + it, 1.0)
        gh.check_parity(w, kernel=REG, ld_pad=int(g.choice([0, 3])), expect_kernel=REG)
        ran += 1
        regrouped += plan[14] > 0
    assert ran >= 30 and 3 * regrouped >= ran


def test_fp32_row_groups_on_the_fused_convolution_and_refusals():
    # a density-1/2 VGG19 layer shape (complete G_i joins G_r: 32 rows per column set), images 8 pixels wide: tap-grouped
    w = wl.Workload("rowgroups_conv", (4, 4, 4, 2), (4, 2, 8, 9), (2, 2, 8, 9), 0, wl.F32, 71, 72, 73, 1.0)
    X = wl.conv_activations(w, 6, 8, 8)
    want, den = gh.oracle_spmm(w, wl.kept_weights(w), orc.im2col_3x3(X))
    for ng in (1, 2):
        for sets in (1, 2):
            out = gh.library_conv3x3(w, wl.kept_weights(w), X, tune=(0, 0, 0, 0, ng, 0, 0, sets), kernel=REG)
            assert orc.normalised_error(out, want, den) <= gh.TOL[w.dtype]
    # a mask with 8 rows per column set has no such groups
    with pytest.raises(rb.RbgpError) as e:
        gh.check_parity(wl.VGG19_CONV5, N=256, kernel=REG, tune=(0, 0, 0, 0, 2), expect_kernel=REG)
    assert e.value.code == rb.EUNSUPPORTED


# stages of 8 contraction steps, every stage list of the same length (a multiple of 4): waves that take several
# column tiles one after the other.  (rows, cols, degrees, column tiles per wave to try, row groups per wave)
COLUMN_TILE_SHAPES = [
    ((8, 4, 4, 9), (8, 4, 2, 2), (4, 4, 1, 2), (2, 4, 8), 1),    # a transposed 3x3 layer: 36 rows -> 4 x 9, lists of 4
    ((8, 4, 4, 11), (8, 4, 2, 2), (4, 4, 1, 2), (2, 4), 2),      # 44 rows -> 4 x 11: two of the four tile rows per wave
    ((8, 4, 4, 9), (8, 3, 4, 2), (4, 3, 1, 2), (4,), 1),         # stages of 6 steps in 8
]


@pytest.mark.parametrize("idx", range(len(COLUMN_TILE_SHAPES)))
def test_fp32_register_family_column_tiles_per_wave(idx):
    """RBGP_TUNE_COLUMN_TILES: N of one tile, of several waves' worth with a ragged last tile and a last wave that has
    fewer tiles than the others, padded leading dimension."""
    rows, cols, deg, tiles, ng = COLUMN_TILE_SHAPES[idx]
    w = wl.Workload(f"coltiles{idx}", rows, cols, deg, 333, wl.F32, 140 + idx, 150 + idx, 160 + idx, 1.0)
    for ct in tiles:
        tune = (0, 0, 0, 0, ng, 1, ct)   # (no split of the stage lists, which small N would bring)
        gh.check_parity(w, kernel=REG, tune=tune, ld_pad=3, expect_kernel=REG)          # 6 tiles
        gh.check_parity(w, N=64, kernel=REG, tune=tune, expect_kernel=REG)              # one tile
        gh.check_parity(w, N=2309, kernel=REG, tune=tune, ld_pad=1, expect_kernel=REG)  # 37 tiles


def test_column_tiles_per_wave_refusals_and_default():
    # stage lists of different lengths (sparse G_o, two tile rows per group: no kernel of this kind), a split list,
    # stages of more than 8 steps, bf16: refused
    ragged = wl.Workload("coltiles_ragged", (16, 2, 2, 4), (16, 2, 4, 2), (8, 2, 2, 2), 256, wl.F32, 171, 172, 173, 1.0)
    long_steps = wl.Workload("coltiles_18", (8, 4, 4, 9), (8, 4, 4, 2), (4, 4, 2, 2), 256, wl.F32, 174, 175, 176, 1.0)
    ok = wl.Workload("coltiles_ok", (8, 4, 4, 9), (8, 4, 2, 2), (4, 4, 1, 2), 256, wl.F32, 177, 178, 179, 1.0)
    for w, tune in ((ragged, (0, 0, 0, 0, 0, 1, 2)), (long_steps, (0, 0, 0, 0, 0, 1, 2)), (ok, (0, 0, 0, 0, 0, 2, 2)),
                    (ok, (0, 0, 0, 0, 0, 1, 3)), (ok, (0, 0, 0, 0, 0, 1, 32)), (replace(ok, dtype=wl.BF16), (0, 0, 0, 0, 0, 1, 2))):
        with pytest.raises(rb.RbgpError) as e:
            gh.check_parity(w, kernel=REG, tune=tune, expect_kernel=REG)
        assert e.value.code == rb.EUNSUPPORTED
    # the library's own choice on the backward data product of the headline layer (64 tile rows of 9 rows, 8 stages of
    # 8 steps): whatever it takes, the result is the oracle's
    gh.check_parity(ok, N=8192, kernel=rb.KERNEL_AUTO)


# stages of 72 steps with 2, 4, 8 and 16 weight rows per tile row: the kernels with one register set (two waves per SIMD)
ONE_SET_SHAPES = [((4, 1, 4, 2), 2), ((4, 2, 4, 2), 4), ((4, 4, 4, 2), 8), ((4, 4, 4, 4), 16)]


# stages of 72, 36, 32 and 18 steps: columns and left degrees of the factors
ONE_SET_STAGES = {72: ((4, 4, 4, 9), (2, 4, 2, 9)), 36: ((4, 2, 4, 9), (2, 2, 2, 9)), 32: ((4, 4, 4, 4), (2, 4, 2, 4)),
                  18: ((4, 1, 4, 9), (2, 1, 2, 9))}


@pytest.mark.parametrize("idx", range(len(ONE_SET_SHAPES)))
@pytest.mark.parametrize("steps", sorted(ONE_SET_STAGES))
def test_fp32_register_family_one_register_set(idx, steps):
    """RBGP_TUNE_REGISTER_SETS = 1: ragged N, padded leading dimension, one column tile, a split stage list."""
    rows, rs = ONE_SET_SHAPES[idx]
    cols, deg = ONE_SET_STAGES[steps]
    w = wl.Workload(f"oneset{steps}_{idx}", rows, cols, deg, 333, wl.F32, 180 + idx, 190 + idx, 200 + idx, 1.0)
    plan = rb.rbgp_mask_reg_plan(rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed))
    assert 16 // plan[0] == rs and plan[2] == steps
    pairing = 1 if rs == 8 else 0   # (8 rows: the fixed pairs, not the tile-by-tile pairing kernel)
    for N, split, pad in ((333, 1, 3), (64, 0, 0), (2309, 1, 1), (200, 2, 0), (130, 4, 2)):
        gh.check_parity(w, N=N, kernel=REG, tune=(0, 0, 0, pairing, 0, split, 0, 1), ld_pad=pad, expect_kernel=REG)
    gh.check_parity(w, N=333, kernel=REG, tune=(0, 0, 0, pairing, 0, 0, 0, 2), expect_kernel=REG)


@pytest.mark.parametrize("idx", range(len(ONE_SET_SHAPES)))
@pytest.mark.parametrize("steps", [72, 36])
def test_bf16_register_family_one_register_set(idx, steps):
    """The bf16 kernels with one register set (128-column tiles, one or two row groups, stages of 72 and 36 steps):
    ragged N, a split stage list, the bf16-output mode; 64-column tiles have no such variant."""
    rows, rs = ONE_SET_SHAPES[idx]
    cols, deg = ((4, 4, 4, 9), (2, 4, 2, 9)) if steps == 72 else ((4, 2, 4, 9), (2, 2, 2, 9))
    w = wl.Workload(f"oneset_bf16_{steps}_{idx}", rows, cols, deg, 328, wl.BF16, 210 + idx, 220 + idx, 230 + idx, 1.0)
    assert rb.rbgp_mask_reg_plan(rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed))[2] == steps
    for N, groups, split in ((328, 1, 1), (1096, 2, 1), (136, 1, 2), (2312, 2, 4), (128, 1, 0)):
        gh.check_parity(w, N=N, kernel=REG, tune=(0, 128, 0, 0, groups, split, 0, 1), expect_kernel=REG)
    # bf16 output: the rounding of what the fp32-output mode of the same launch stores
    vl, Il, vf, If = gh.host_inputs(w, 328)
    out16, _ = gh.library_spmm(w, vl, Il, REG, (0, 128, 0, 0, 1, 1, 0, 1), out_bf16=True)
    out32, _ = gh.library_spmm(w, vl, Il, REG, (0, 128, 0, 0, 1, 1, 0, 1))
    assert np.array_equal((out16.view(np.uint32) >> 16).astype(np.uint16), orc.f32_to_bf16_bits(out32))
    with pytest.raises(rb.RbgpError) as e:
        gh.check_parity(w, N=328, kernel=REG, tune=(0, 64, 0, 0, 1, 1, 0, 1), expect_kernel=REG)
    assert e.value.code == rb.EUNSUPPORTED
    if rs == 16:   # four groups per wave: built for stages of up to 36 steps
        if steps == 36:
            gh.check_parity(w, N=1096, kernel=REG, tune=(0, 128, 0, 0, 4, 1, 0, 1), expect_kernel=REG)
        else:
            with pytest.raises(rb.RbgpError) as e:
                gh.check_parity(w, N=1096, kernel=REG, tune=(0, 128, 0, 0, 4, 1, 0, 1), expect_kernel=REG)
            assert e.value.code == rb.EUNSUPPORTED


def test_bf16_one_register_set_on_short_stages():
    """Stages of 32 and 18 steps: with two groups only where a wave has a single stage, with four groups always."""
    one_stage32 = wl.Workload("oneset_bf16_single32", (4, 4, 2, 2), (1, 4, 4, 2), (1, 4, 4, 2), 1096, wl.BF16, 241, 242, 243, 1.0)
    one_stage18 = wl.Workload("oneset_bf16_single18", (4, 2, 4, 2), (1, 2, 4, 4), (1, 2, 2, 4), 1096, wl.BF16, 244, 245, 246, 1.0)
    for w in (one_stage32, one_stage18):
        for sets in (1, 2, 0):
            gh.check_parity(w, kernel=REG, tune=(0, 128, 0, 0, 2, 1, 0, sets), expect_kernel=REG)
    gh.check_parity(one_stage32, kernel=REG, tune=(0, 128, 0, 0, 4, 1, 0, 1), expect_kernel=REG)
    several = wl.Workload("oneset_bf16_several18", (4, 4, 4, 4), (4, 1, 4, 9), (2, 1, 2, 9), 1096, wl.BF16, 247, 248, 249, 1.0)
    gh.check_parity(several, kernel=REG, tune=(0, 128, 0, 0, 4, 1, 0, 1), expect_kernel=REG)
    with pytest.raises(rb.RbgpError) as e:
        gh.check_parity(several, kernel=REG, tune=(0, 128, 0, 0, 2, 1, 0, 1), expect_kernel=REG)
    assert e.value.code == rb.EUNSUPPORTED


def test_one_register_set_on_the_headline_layer_and_refusals():
    gh.check_parity(wl.VGG19_CONV5, N=512, kernel=REG, tune=(0, 0, 0, 1, 0, 0, 0, 1), expect_kernel=REG)
    # the fused convolution on 4-pixel-wide images (no tap grouping): the same kernel reading the activations
    w = wl.VGG19_CONV5
    X = wl.conv_activations(w, 9, 4, 4)
    want, den = gh.oracle_spmm(w, wl.kept_weights(w), orc.im2col_3x3(X))
    for sets in (1, 2):
        out = gh.library_conv3x3(w, wl.kept_weights(w), X, tune=(0, 0, 0, 1, 0, 0, 0, sets), kernel=REG)
        assert orc.normalised_error(out, want, den) <= gh.TOL[w.dtype]
    short = wl.Workload("oneset_8", (8, 4, 4, 9), (8, 4, 2, 2), (4, 4, 1, 2), 256, wl.F32, 174, 175, 176, 1.0)
    for w, tune in ((short, (0, 0, 0, 0, 0, 0, 0, 1)),                       # stages of 8 steps
                    (wl.VGG19_CONV5, (0, 0, 0, 2, 0, 0, 0, 1)),              # with the tile-by-tile pairing kernel
                    (wl.VGG19_CONV5, (0, 0, 0, 1, 0, 0, 0, 3)),              # not a value of the knob
                    (replace(wl.VGG19_CONV3_BF16, N=256), (0, 64, 0, 0, 0, 0, 0, 1))):   # bf16 on 64-column tiles
        with pytest.raises(rb.RbgpError) as e:
            gh.check_parity(w, N=256, kernel=REG, tune=tune, expect_kernel=REG)
        assert e.value.code == rb.EUNSUPPORTED


def test_activations_beyond_4_gib():
    """An I of 4.6 GB (WRN shape, 2 000 037 columns, odd leading dimension): the kernels'
    32-bit offsets must only span one stage.  A sample of output columns is checked."""
    w = replace(wl.WRN_G1, N=2_000_037, name="wrn_4gib")
    vl, Il, vf, If = gh.host_inputs(w)
    cols = np.r_[0:64, 1_000_000:1_000_064, 1_999_936:2_000_037]
    ref, den = gh.oracle_spmm(w, vf, np.ascontiguousarray(If[:, cols]))
    for kernel in (rb.KERNEL_AUTO, MFMA, GEN):
        out, used = gh.library_spmm(w, vl, Il, kernel=kernel, tune=(1, 64, 0) if kernel == MFMA else None,
                                    ld_pad=3 if kernel == MFMA else 0, tag="beyond 4 GiB")
        assert used == (REG if kernel == rb.KERNEL_AUTO else kernel)
        err = orc.normalised_error(out[:, cols], ref, den)
        assert err <= gh.TOL[w.dtype], err
        assert np.all(np.isfinite(out[:, ::4099]))


# ------------------------------------------------------------------ fused 3x3 convolution
CONV_CASES = [
    # workload (K = 9 * channels), images, height, width
    (wl.Workload("conv_small", (4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9), 0, wl.F32, 61, 62, 63, 1.0), 3, 4, 8),
    (wl.Workload("conv_ragged", (4, 1, 4, 3), (4, 2, 4, 9), (2, 2, 2, 9), 0, wl.F32, 64, 65, 66, 1.0), 5, 3, 4),
    (wl.Workload("conv_wide", (4, 2, 4, 1), (4, 2, 4, 9), (2, 2, 2, 9), 0, wl.F32, 67, 68, 69, 1.0), 2, 5, 32),
    (wl.VGG19_CONV5, 128, 4, 4),          # the headline layer: 512 -> 512 channels, 4x4 pixels, batch 128
    (wl.WRN_G1, 8, 32, 32),               # WRN-40-4 group 1 at batch 8
    (wl.VGG19_CONV3_BF16, 128, 8, 8),     # bf16: 256 -> 256 channels, 8x8 pixels (128-column wave tiles)
    (replace(wl.VGG19_CONV3_BF16, name="conv3_bf16_4x4"), 33, 4, 4),     # bf16, 64-column tiles, ragged N
    (replace(wl.Workload("conv_small_bf16", (4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9), 0, wl.BF16, 71, 72, 73, 1.0)), 3, 5, 8),
    # stages padded to the next kernel size: 54 -> 72 steps, 9 -> 18 steps, 27 -> 36 steps with 16 rows per tile row
    (wl.Workload("conv_pad54", (4, 2, 4, 1), (4, 1, 12, 9), (2, 1, 6, 9), 0, wl.F32, 74, 75, 76, 1.0), 2, 4, 8),
    (wl.Workload("conv_pad9_bf16", (4, 1, 2, 1), (4, 1, 2, 9), (2, 1, 1, 9), 0, wl.BF16, 77, 78, 79, 1.0), 3, 3, 12),
    (wl.Workload("conv_pad27_r16", (4, 4, 4, 4), (4, 3, 4, 9), (2, 3, 1, 9), 0, wl.F32, 80, 81, 82, 1.0), 2, 4, 16),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: c[0].name)
def test_fused_conv3x3_equals_spmm_on_the_lowered_input(case):
    """rbgp_conv3x3 on padded activations = the oracle's product with the explicitly
    lowered input (im2col written out in the oracle)."""
    w, B, H, W = case
    vals = wl.kept_weights(w)
    X = wl.conv_activations(w, B, H, W)
    if w.dtype == wl.BF16:                # both sides consume the same bf16 bits
        vals_lib, X_lib = wl.to_bf16_bits(vals), wl.to_bf16_bits(X)
        vals, X = wl.bf16_bits_as_f32(vals_lib), wl.bf16_bits_as_f32(X_lib)
    else:
        vals_lib, X_lib = vals, X
    ref, den = gh.oracle_spmm(w, vals, orc.im2col_3x3(X))
    tunes = [None, (0, 0, 0, 0, 0, 2)] + ([(0, 64, 0, 0, 2, 1)] if w.dtype == wl.BF16 else [])
    for tune in tunes:
        out = gh.library_conv3x3(w, vals_lib, X_lib, tune=tune)
        err = orc.normalised_error(out, ref, den)
        print(f"[gpu]   normalised error {err:.3e}", flush=True)
        assert err <= gh.TOL[w.dtype], err


def test_fused_conv3x3_random_geometries():
    """Thirty seeded random (mask, images, height, width, dtype, stage split) combinations."""
    g = np.random.Generator(np.random.PCG64(77))
    shapes = [c[0] for c in CONV_CASES[:3]] + [
        wl.Workload("conv_r6", (2, 3, 4, 2), (2, 2, 4, 9), (1, 2, 2, 9), 0, wl.F32, 81, 82, 83, 1.0),
        wl.Workload("conv_kc18", (4, 2, 4, 2), (4, 1, 4, 9), (2, 1, 2, 9), 0, wl.F32, 84, 85, 86, 1.0),
        wl.Workload("conv_8x8", (8, 2, 4, 1), (8, 2, 4, 9), (2, 2, 2, 9), 0, wl.F32, 87, 88, 89, 1.0)]
    ran = 0
    for it in range(30):
        dtype = int(g.integers(0, 2))
        w = replace(shapes[it % len(shapes)], dtype=dtype, name=f"conv_random{it}")
        B, H, W = int(g.integers(1, 7)), int(g.integers(1, 8)), int(g.choice([4, 8, 12, 16, 20, 32, 64]))
        vals, X = wl.kept_weights(w), wl.conv_activations(w, B, H, W)
        if dtype == wl.BF16:
            vals_lib, X_lib = wl.to_bf16_bits(vals), wl.to_bf16_bits(X)
            vals, X = wl.bf16_bits_as_f32(vals_lib), wl.bf16_bits_as_f32(X_lib)
        else:
            vals_lib, X_lib = vals, X
        out = gh.library_conv3x3(w, vals_lib, X_lib, tune=(0, 0, 0, 0, 0, int(g.choice([0, 1, 2, 4]))))
        ref, den = gh.oracle_spmm(w, vals, orc.im2col_3x3(X))
        err = orc.normalised_error(out, ref, den)
        assert err <= gh.TOL[dtype], (w.rows, B, H, W, dtype, err)
        ran += 1
    assert ran == 30


def test_fused_conv3x3_argument_checks():
    import torch
    w, B, H, W = CONV_CASES[0]
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    buf = torch.zeros(1 << 20, dtype=torch.float32, device="cuda:0")
    args = (buf.data_ptr(), buf.data_ptr(), buf.data_ptr())
    for bad, code in [(dict(width=6), rb.ESHAPE), (dict(cin=w.K // 9 + 1), rb.ESHAPE)]:
        with pytest.raises(rb.RbgpError) as ei:
            rb.rbgp_conv3x3(mask, bad.get("dtype", rb.F32), w.M, bad.get("cin", w.K // 9), B, H, bad.get("width", W),
                            args[0], args[1], args[2], B * H * bad.get("width", W), 0)
        assert ei.value.code == code
    # a mask whose G_b does not have the nine taps
    m2 = rb.rbgp_make_mask(wl.TINY.rows, wl.TINY.cols, wl.TINY.row_deg, 1)
    with pytest.raises(rb.RbgpError):
        rb.rbgp_conv3x3(m2, rb.F32, wl.TINY.M, wl.TINY.K // 9, 1, 4, 4, args[0], args[1], args[2], 16, 0)


def test_masks_outside_rbgp4_roles_use_the_generic_kernel():
    """Sparse G_r / G_b (general four-factor RBGP): the kernels' view folds them into G_o / G_i and the MFMA
    kernels run; more than 16 rows in G_b alone leaves the register family."""
    w = wl.Workload("general_rbgp", (4, 4, 4, 2), (4, 4, 8, 4), (2, 2, 4, 2), 130, wl.F32, 5, 6, 7, 1.0)
    gh.check_parity(w, expect_kernel=REG)
    gh.check_parity(w, kernel=GEN)
    gh.check_parity(replace(w, dtype=wl.BF16), ld_pad=2, expect_kernel=REG)     # (bf16: leading dimension a multiple of 4)
    big_gb = wl.Workload("big_gb", (2, 1, 2, 32), (2, 1, 4, 3), (2, 1, 2, 3), 96, wl.F32, 8, 9, 10, 1.0)
    assert not gh.family_covers(big_gb, REG)
    gh.check_parity(big_gb)


def test_sdmm4096_paper_workload_sampled():
    """Table 2's 4096^3 SDMM at 87.5 % sparsity, (50 %, 75 %) split: full shape
    on the GPU, a sample of output columns checked against the oracle."""
    w = wl.sdmm4096_table2(1, 2)
    vl, Il, vf, If = gh.host_inputs(w)
    cols = np.r_[0:64, 2000:2064, 4032:4096]
    ref, den = gh.oracle_spmm(w, vf, np.ascontiguousarray(If[:, cols]))
    # the default launch (the register family on the mask with G_o filled in and merged with G_r), the register family on
    # the mask as given (stage lists split over the waves of a workgroup) and the LDS family
    for kernel, want in ((rb.KERNEL_AUTO, FILLED), (REG, REG), (MFMA, MFMA), (FILLED, FILLED)):
        out, used = gh.library_spmm(w, vl, Il, kernel=kernel, tag="table2")
        assert used == want
        assert orc.normalised_error(out[:, cols], ref, den) <= gh.TOL[w.dtype]


# ------------------------------------------------------------------ random masks, library defaults
def _random_shapes(count, seed):
    """Seeded random four-factor shapes (G_r, G_b complete) that the sampler accepts."""
    g = np.random.Generator(np.random.PCG64(seed))
    shapes = []
    while len(shapes) < count:
        lo, li = int(g.integers(0, 3)), int(g.integers(0, 3))            # log2 of G_o's / G_i's inverse density
        a_o = int(g.choice([1, 2, 3, 4, 6, 8, 12, 16])) << lo
        c_o = int(g.choice([1, 2, 3, 4, 8])) << lo
        a_i = int(g.choice([1, 2, 4])) << li
        c_i = int(g.choice([1, 2, 4])) << li
        a_r, c_r = int(g.choice([1, 2, 3, 4, 8])), int(g.choice([1, 2, 3, 4]))
        a_b, c_b = int(g.choice([1, 2, 3, 4, 24])), int(g.choice([1, 3, 9, 9]))
        rows, cols = (a_o, a_r, a_i, a_b), (c_o, c_r, c_i, c_b)
        deg = (c_o >> lo, c_r, c_i >> li, c_b)
        if a_o * a_r * a_i * a_b > 2048 or c_o * c_r * c_i * c_b > 4096:
            continue
        try:
            rb.rbgp_make_mask(rows, cols, deg, 900 + len(shapes))
        except rb.RbgpError:
            continue
        shapes.append((rows, cols, deg, int(g.integers(1, 700))))
    return shapes


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_random_masks_with_library_defaults(dtype):
    """Forty seeded random shapes, ragged column counts, whatever kernel and launch shape the
    library chooses for them."""
    used = set()
    for idx, (rows, cols, deg, N) in enumerate(_random_shapes(40, 2024)):
        w = wl.Workload(f"random{idx}_{dtype}", rows, cols, deg, N, dtype, 900 + idx, 1000 + idx, 1100 + idx, 1.0)
        vl, Il, vf, If = gh.host_inputs(w)
        out, kernel = gh.library_spmm(w, vl, Il, ld_pad=(-N) % 8)    # a leading dimension every family accepts
        used.add(kernel)
        ref, den = gh.oracle_spmm(w, vf, If)
        err = orc.normalised_error(out, ref, den)
        assert err <= gh.TOL[dtype], (rows, cols, deg, N, kernel, err)
    assert rb.KERNEL_MFMA_REG in used and len(used) >= 2, used


# ------------------------------------------------------------------ more than four base graphs
K_WORKLOADS = [
    wl.Workload("k6_two_sparse_in_go_taps_3x3", (2, 2, 2, 4, 2, 2), (4, 2, 2, 8, 3, 3), (2, 1, 2, 4, 3, 3), 200, wl.F32,
                91, 92, 93, 1.0, roles=(0, 0, 1, 2, 3, 3)),
    wl.Workload("k5_three_in_gi", (4, 4, 2, 2, 3), (4, 8, 2, 4, 1), (2, 4, 2, 2, 1), 136, wl.F32,
                94, 95, 96, 1.0, roles=(0, 2, 2, 2, 3)),
    wl.Workload("k3_no_gb", (4, 2, 4), (8, 2, 4), (2, 2, 2), 72, wl.F32, 97, 98, 99, 1.0, roles=(0, 1, 2)),
    wl.Workload("k5_sparse_gr", (4, 2, 2, 4, 2), (4, 4, 2, 4, 2), (2, 2, 2, 2, 2), 100, wl.F32,
                100, 101, 102, 1.0, roles=(0, 1, 1, 2, 3)),          # sparse graph given to G_r: regrouped by the library
    wl.Workload("k5_sparse_graph_joins_go", (4, 2, 2, 4, 2), (4, 4, 2, 4, 2), (2, 2, 2, 2, 2), 100, wl.F32,
                100, 101, 102, 1.0, roles=(0, 0, 1, 2, 3)),          # the same graphs, the sparse second one in G_o: MFMA
]


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("w", K_WORKLOADS, ids=lambda w: w.name)
def test_masks_of_more_than_four_base_graphs(w, dtype):
    """Section 5: a mask is configured by the number of base graphs and their types; the library
    folds them into the four factors of its kernels."""
    w = replace(w, dtype=dtype)
    err = gh.check_parity(w)
    assert gh.family_covers(w, REG)
    gh.check_parity(w, kernel=REG, expect_kernel=REG)
    gh.check_parity(w, kernel=GEN)
    # backward products of the same masks
    lib, f32 = gh.backward_inputs(w)
    dI_ref, dI_den, dW_ref, dW_den = gh.oracle_backward(w, *f32)
    dI, _ = gh.library_spmm_transposed(w, lib[0], lib[2])
    assert orc.normalised_error(dI, dI_ref, dI_den) <= gh.TOL[dtype]
    dW = gh.library_sddmm(w, lib[2], lib[1])
    assert orc.normalised_error(dW, dW_ref, dW_den) <= gh.TOL[dtype]


def test_non_finite_input_stays_in_its_column():
    """An infinity in one element of I: on the plain kernel it reaches exactly the rows of W_s that keep a
    weight in that column of the mask (the sum of Section 5 runs over kept weights only); on the MFMA
    families, whose padding multiplies zero weights by real rows of I, it may spoil other rows of the same
    column of O, and never another column."""
    w = replace(wl.VGG19_CONV5, rows=(4, 4, 4, 2), cols=(4, 4, 8, 9), row_deg=(2, 4, 2, 9), name="non_finite")
    N, k_bad, n_bad = 200, 37, 77
    vl, Il, vf, If = gh.host_inputs(w, N)
    I_bad = Il.copy()
    I_bad[k_bad, n_bad] = np.inf
    mask = gh.make_mask(w)
    touched = rb.rbgp_mask_dense(mask).reshape(w.M, w.K)[:, k_bad].astype(bool)
    assert touched.any() and not touched.all()
    for kernel in (GEN, MFMA, REG):
        clean, _ = gh.library_spmm(w, vl, Il, kernel=kernel, tag="finite")
        spoilt, _ = gh.library_spmm(w, vl, I_bad, kernel=kernel, tag="one infinity")
        others = np.ones(N, bool)
        others[n_bad] = False
        assert np.array_equal(clean[:, others].view(np.uint32), spoilt[:, others].view(np.uint32))
        assert not np.isfinite(spoilt[touched, n_bad]).any()
        if kernel == GEN:
            assert np.array_equal(clean[~touched, n_bad].view(np.uint32), spoilt[~touched, n_bad].view(np.uint32))
