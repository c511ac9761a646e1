"""Host-side checks of the C-ABI library (no GPU call): every declared symbol
is exported, and the sampler / index expansion agree with the oracle, which was
written separately from the same description."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names += re.findall(r"\b(rbgp_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = rb.load()
    declared = _declared_functions()
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(rb.SIGNATURES) == declared      # the binding covers the whole header


SHAPES = [w for w in wl.CONFIGS] + [wl.sdmm4096_table2(1, 2), wl.sdmm4096_table3(2, 2, 3),
                                    wl.vgg19_sweep_workload(5, 4, wl.F32)]


@pytest.mark.parametrize("w", SHAPES, ids=lambda w: w.name)
def test_make_mask_matches_oracle_sampler_bit_for_bit(w):
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    Bs, infos = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    sh = rb.rbgp_mask_shape(mask)
    assert (sh["M"], sh["K"], sh["rowdeg"], sh["nnz"]) == (w.M, w.K, w.rowdeg, w.nnz)
    for i in range(4):
        a, c, d, adj = rb.rbgp_mask_factor(mask, i)
        assert (a, c, d) == (w.rows[i], w.cols[i], w.row_deg[i])
        assert np.array_equal(adj, orc.adjacency_lists(Bs[i]))
        sp = rb.rbgp_mask_spectrum(mask, i)
        assert sp["status"] == infos[i]["status"] and sp["tries"] == infos[i]["tries"]
        assert sp["sigma1"] == pytest.approx(infos[i]["sigma1"], abs=1e-7)
        assert sp["sigma2"] == pytest.approx(infos[i]["sigma2"], abs=1e-7)
        assert sp["bound"] == pytest.approx(infos[i]["bound"], abs=1e-12)
        if sp["status"] == rb.SPEC_OK:
            assert sp["sigma2"] <= sp["bound"] * (1 + 1e-9)


@pytest.mark.parametrize("w", [wl.TINY, wl.WRN_G1, wl.VGG19_CONV3_BF16], ids=lambda w: w.name)
def test_columns_and_dense_match_kronecker_definition(w):
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    dense = orc.kron_mask(Bs)
    assert np.array_equal(rb.rbgp_mask_dense(mask), dense)
    assert np.array_equal(rb.rbgp_mask_columns(mask), orc.canonical_columns(dense))
    sh = rb.rbgp_mask_shape(mask)
    assert sh["coldeg"] == int(dense.sum(0)[0])


def test_equal_arguments_give_identical_masks_and_seeds_differ():
    w = wl.VGG19_CONV5
    a = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 77)
    b = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 77)
    c = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 78)
    assert np.array_equal(rb.rbgp_mask_factor(a, 0)[3], rb.rbgp_mask_factor(b, 0)[3])
    assert np.array_equal(rb.rbgp_mask_factor(a, 2)[3], rb.rbgp_mask_factor(b, 2)[3])
    assert not np.array_equal(rb.rbgp_mask_factor(a, 0)[3], rb.rbgp_mask_factor(c, 0)[3])


def test_spectral_solver_closed_forms():
    # complete factors
    m = rb.rbgp_make_mask((4, 2, 1, 1), (9, 2, 1, 1), (9, 2, 1, 1), 0)
    sp = rb.rbgp_mask_spectrum(m, 0)
    assert sp["status"] == rb.SPEC_COMPLETE and sp["sigma1"] == pytest.approx(6.0) and sp["sigma2"] == 0
    # 4x4 2-regular: either an 8-cycle (2, sqrt2) or two 4-cycles (2, 2); both meet the bound 2
    seen = set()
    for seed in range(20):
        m = rb.rbgp_make_mask((4, 1, 1, 1), (4, 1, 1, 1), (2, 1, 1, 1), seed)
        sp = rb.rbgp_mask_spectrum(m, 0)
        assert sp["sigma1"] == pytest.approx(2.0, abs=1e-9)
        assert min(abs(sp["sigma2"] - 2.0), abs(sp["sigma2"] - math.sqrt(2))) < 1e-9
        seen.add(round(sp["sigma2"], 6))
    assert len(seen) == 2
    # star forest 4x8 (degrees 2,1): sigma_2 = sigma_1 = sqrt2 > bound 1 -> DEGENERATE
    m = rb.rbgp_make_mask((4, 1, 1, 1), (8, 1, 1, 1), (2, 1, 1, 1), 3)
    sp = rb.rbgp_mask_spectrum(m, 0)
    assert sp["status"] == rb.SPEC_DEGENERATE and sp["tries"] == 1
    assert sp["sigma2"] == pytest.approx(math.sqrt(2)) and sp["bound"] == pytest.approx(1.0)


def test_error_codes():
    lib = rb.load()
    out = ctypes.c_void_p()
    good = (ctypes.c_int32 * 4)(4, 2, 4, 2)

    def mk(rows, cols, deg, tries=0, outp=ctypes.byref(out)):
        r = (ctypes.c_int32 * 4)(*rows)
        c = (ctypes.c_int32 * 4)(*cols)
        d = (ctypes.c_int32 * 4)(*deg)
        return lib.rbgp_make_mask(r, c, d, 1, tries, outp)

    assert lib.rbgp_make_mask(None, good, good, 1, 0, ctypes.byref(out)) == rb.EINVAL
    assert mk((4, 2, 4, 2), (4, 2, 4, 2), (2, 2, 2, 2), outp=None) == rb.EINVAL
    assert mk((4, 2, 4, 2), (6, 2, 4, 2), (2, 2, 2, 2)) == rb.EINVAL      # 6/2 = 3 is not 2^L
    assert mk((4, 2, 4, 2), (4, 2, 4, 2), (3, 2, 2, 2)) == rb.EINVAL      # 3 does not divide 4
    assert mk((3, 2, 4, 2), (4, 2, 4, 2), (2, 2, 2, 2)) == rb.EINVAL      # rows not divisible by 2^L
    assert mk((4, 2, 4, 0), (4, 2, 4, 2), (2, 2, 2, 2)) == rb.EINVAL
    assert mk((4, 2, 4, 2), (4, 2, 4, 2), (2, 2, 5, 2)) == rb.EINVAL      # degree above cols
    assert out.value is None
    # a 32x32 degree-4 factor is rejected on some first samples: max_tries=1 must then fail
    codes = {mk((32, 1, 1, 1), (32, 1, 1, 1), (4, 1, 1, 1), tries=1) for _ in range(1)}
    fails = 0
    for seed in range(40):
        r = (ctypes.c_int32 * 4)(32, 1, 1, 1)
        d = (ctypes.c_int32 * 4)(4, 1, 1, 1)
        o = ctypes.c_void_p()
        rc = lib.rbgp_make_mask(r, r, d, seed, 1, ctypes.byref(o))
        assert rc in (rb.OK, rb.ENOTRAMANUJAN)
        if rc == rb.OK:
            lib.rbgp_mask_free(o)
        else:
            fails += 1
            assert o.value is None
    assert fails > 0
    assert lib.rbgp_mask_shape(None, None, None, None, None, None) == rb.EINVAL
    assert lib.rbgp_packed_bytes(None, 0) == 0
    assert lib.rbgp_strerror(rb.ESHAPE).decode().startswith("shape")
    lib.rbgp_mask_free(None)


def test_spmm_argument_checks_need_no_gpu():
    w = wl.TINY
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 1)
    lib = rb.load()
    assert lib.rbgp_spmm(mask.handle, 0, w.M + 1, w.K, 8, None, None, 8, None, 8, None) == rb.ESHAPE
    assert lib.rbgp_spmm(mask.handle, 0, w.M, w.K, 8, None, None, 4, None, 8, None) == rb.ESHAPE
    assert lib.rbgp_spmm(mask.handle, 7, w.M, w.K, 8, None, None, 8, None, 8, None) == rb.EINVAL
    assert lib.rbgp_spmm(mask.handle, 0, w.M, w.K, 0, None, None, 0, None, 0, None) == rb.OK     # empty: no-op
    assert lib.rbgp_spmm(None, 0, w.M, w.K, 8, None, None, 8, None, 8, None) == rb.EINVAL


def test_kernel_selection_and_packed_size():
    w = wl.VGG19_CONV5
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 1)
    assert rb.rbgp_mask_kernel(mask, rb.F32) == rb.KERNEL_MFMA_REG
    assert rb.rbgp_mask_kernel(mask, rb.BF16_F32ACC) == rb.KERNEL_MFMA_REG
    padded = rb.rbgp_packed_bytes(mask, rb.F32)
    assert padded >= w.nnz * 4
    rb.rbgp_mask_set_kernel(mask, rb.KERNEL_GENERIC)
    assert rb.rbgp_mask_kernel(mask, rb.F32) == rb.KERNEL_GENERIC
    assert rb.rbgp_packed_bytes(mask, rb.F32) == w.nnz * 4
    assert rb.rbgp_packed_bytes(mask, rb.BF16_F32ACC) == w.nnz * 2
    # a mask whose G_r and G_b are sparse: the kernels' view moves them into G_o and G_i (same mask, same
    # canonical order), so the MFMA families still apply; the inputs stay visible as base graphs
    m2 = rb.rbgp_make_mask((4, 4, 4, 4), (4, 4, 4, 4), (2, 2, 2, 2), 1)
    assert rb.rbgp_mask_kernel(m2, rb.F32) == rb.KERNEL_MFMA_REG
    assert [rb.rbgp_mask_factor(m2, i)[:3] for i in range(4)] == [(16, 16, 4), (1, 1, 1), (16, 16, 4), (1, 1, 1)]
    assert [(g["rows"], g["cols"], g["deg"], g["role"]) for g in (rb.rbgp_mask_base(m2, i) for i in range(4))] == \
           [(4, 4, 2, 0), (4, 4, 2, 1), (4, 4, 2, 2), (4, 4, 2, 3)]
    Bs, _ = orc.sample_factors((4, 4, 4, 4), (4, 4, 4, 4), (2, 2, 2, 2), 1)
    assert np.array_equal(rb.rbgp_mask_dense(m2), orc.kron_mask(Bs))
    assert np.array_equal(rb.rbgp_mask_columns(m2).reshape(256, -1), orc.canonical_columns(orc.kron_mask(Bs)))
    # more than 16 rows in G_b alone is outside the register family; 64 tiles per tile row outside both
    m3 = rb.rbgp_make_mask((2, 1, 2, 32), (2, 1, 4, 1), (2, 1, 2, 1), 1)
    assert rb.rbgp_mask_kernel(m3, rb.F32) != rb.KERNEL_MFMA_REG
    with pytest.raises(rb.RbgpError) as ei:
        rb.rbgp_mask_set_kernel(m3, rb.KERNEL_MFMA_REG)
    assert ei.value.code == rb.EUNSUPPORTED


LAYOUT_SHAPES = [
    (wl.TINY.rows, wl.TINY.cols, wl.TINY.row_deg),
    (wl.VGG19_CONV5.rows, wl.VGG19_CONV5.cols, wl.VGG19_CONV5.row_deg),
    (wl.VGG19_CONV3_BF16.rows, wl.VGG19_CONV3_BF16.cols, wl.VGG19_CONV3_BF16.row_deg),
    (wl.WRN_G1.rows, wl.WRN_G1.cols, wl.WRN_G1.row_deg),
    ((4, 1, 4, 3), (4, 2, 4, 9), (2, 2, 2, 9)),        # R = 3: partial row block
    ((2, 3, 4, 2), (2, 2, 4, 9), (1, 2, 2, 9)),        # R = 6
    ((2, 4, 16, 1), (2, 1, 16, 1), (2, 1, 8, 1)),      # stage of 8 contraction steps
    ((4, 2, 4, 1), (4, 1, 4, 9), (2, 1, 2, 9)),        # stage of 18
    ((32, 4, 32, 1), (128, 1, 32, 1), (64, 1, 8, 1)),  # Table 2 of the paper
    ((4, 2, 4, 2), (4, 2, 4, 3), (2, 2, 2, 3)),        # stage of 12 steps, padded to 18
    ((2, 1, 8, 4), (2, 3, 8, 3), (1, 3, 2, 3)),        # stage of 18 from 3 x 2 x 3
    ((4, 2, 4, 1), (4, 1, 12, 9), (2, 1, 6, 9)),       # stage of 54, padded to 72
    ((4, 4, 4, 1), (4, 5, 4, 1), (2, 5, 1, 1)),        # stage of 5, padded to 8
    ((2, 8, 4, 3), (2, 2, 4, 9), (1, 2, 2, 9)),        # R = 24: two of G_r's rows move into the tile-row index
    ((4, 4, 2, 9), (4, 4, 4, 2), (2, 4, 2, 2)),        # R = 36 (a transposed 3x3 layer): all four of them do
]


@pytest.mark.parametrize("dtype", [rb.F32, rb.BF16_F32ACC])
@pytest.mark.parametrize("kernel", [rb.KERNEL_GENERIC, rb.KERNEL_MFMA, rb.KERNEL_MFMA_REG, rb.KERNEL_MFMA_TILE,
                                    rb.KERNEL_MFMA_REG_FILLED])
@pytest.mark.parametrize("shape", LAYOUT_SHAPES, ids=lambda s: "x".join(map(str, s[0])))
def test_pack_layout_holds_every_kept_value_exactly_once(shape, kernel, dtype):
    """Whatever the kernel family's layout, packing is a permutation of the kept values
    plus zero padding (host-side table, no GPU)."""
    rows, cols, deg = shape
    mask = rb.rbgp_make_mask(rows, cols, deg, 5)
    try:
        rb.rbgp_mask_set_kernel(mask, kernel)
    except rb.RbgpError as e:
        assert e.code == rb.EUNSUPPORTED
        pytest.skip("family does not cover this mask")
    if kernel == rb.KERNEL_MFMA_TILE and dtype == rb.F32:
        pytest.skip("the tile family has bf16 kernels only")
    nnz = rb.rbgp_mask_shape(mask)["nnz"]
    layout = rb.rbgp_pack_layout(mask, dtype)
    assert layout.size * (4 if dtype == rb.F32 else 2) == rb.rbgp_packed_bytes(mask, dtype)
    kept = layout[layout >= 0]
    assert kept.size == nnz
    assert np.array_equal(np.sort(kept), np.arange(nnz, dtype=np.int32))
    assert np.all(layout[layout < 0] == -1)
    if rb.rbgp_mask_kernel(mask, dtype) == rb.KERNEL_GENERIC:
        assert np.array_equal(layout, np.arange(nnz, dtype=np.int32))     # canonical order itself


@pytest.mark.parametrize("dtype", [rb.F32, rb.BF16_F32ACC])
@pytest.mark.parametrize("shape", [((4, 2, 8, 1), (4, 3, 8, 1), (2, 3, 4, 1)), ((2, 1, 16, 4), (2, 1, 16, 2), (2, 1, 8, 2)),
                                   ((4, 1, 8, 3), (8, 1, 8, 1), (2, 1, 2, 1))], ids=lambda s: "x".join(map(str, s[0])))
def test_filled_layout_is_the_register_layout_of_the_filled_mask(shape, dtype):
    """RBGP_KERNEL_MFMA_REG_FILLED stores the mask inside the layout of a superset of it: G_o (x) J (x) G_b (G_i filled
    in) or J(1,1) (x) J (x) G_i (x) G_b with G_o and G_r merged into one complete factor (G_o filled in), whichever the library
    estimates cheaper.  Both supersets can be made through the public call with the same seed (every factor is sampled
    from the seed, its position and its own sizes alone), so the register-family layout of one of them, carried over
    position by position through the (row, column) each kept value sits at, must be the filled layout: this mask's
    value where it keeps the position, a zero elsewhere."""
    rows, cols, deg = shape
    mask = rb.rbgp_make_mask(rows, cols, deg, 9)
    rb.rbgp_mask_set_kernel(mask, rb.KERNEL_MFMA_REG_FILLED)
    dense = rb.rbgp_mask_dense(mask).astype(bool)
    M, K = dense.shape
    index = np.full((M, K), -1, dtype=np.int64)                  # canonical index of every kept position
    index[dense] = np.arange(dense.sum())                        # (row-major over kept positions = ascending columns per row)
    candidates = [((rows[0], rows[1] * rows[2], 1, rows[3]), (cols[0], cols[1] * cols[2], 1, cols[3]),
                   (deg[0], cols[1] * cols[2], 1, cols[3])),
                  ((1, rows[0] * rows[1], rows[2], rows[3]), (1, cols[0] * cols[1], cols[2], cols[3]),
                   (1, cols[0] * cols[1], deg[2], cols[3]))]
    got, matches = rb.rbgp_pack_layout(mask, dtype), 0
    for frows, fcols, fdeg in candidates:
        full = rb.rbgp_make_mask(frows, fcols, fdeg, 9)
        rb.rbgp_mask_set_kernel(full, rb.KERNEL_MFMA_REG)
        dense_full = rb.rbgp_mask_dense(full).astype(bool)
        if np.any(dense & ~dense_full):                          # (another sample of the shared factor: not a superset)
            continue
        cols_full = rb.rbgp_mask_columns(full).reshape(M, -1)
        lay_full = rb.rbgp_pack_layout(full, dtype)
        want = np.full(lay_full.shape, -1, dtype=np.int64)
        keep = lay_full >= 0
        r, t = np.divmod(lay_full[keep].astype(np.int64), cols_full.shape[1])
        want[keep] = index[r, cols_full[r, t]]
        if want.shape == got.shape and np.array_equal(got, want):
            matches += 1
            assert rb.rbgp_packed_bytes(mask, dtype) == rb.rbgp_packed_bytes(full, dtype)
    assert matches >= 1


def test_automatic_choice_on_the_masks_of_tables_2_and_3():
    """What RBGP_KERNEL_AUTO resolves to on the paper's 4096^3 masks (host-side estimate, fitted to measurements of
    all 27 on every family): one row per column set -> a filled mask (G_i filled in, or, at 1/16, G_o filled in and
    merged with G_r); G_o complete -> the register family (on the merged tile column); a half-full G_o with a sparse
    G_i -> G_o filled in (174 against 317 us at 1/16); G_o and G_i both at 1/4 -> LDS family in fp32; never the LDS
    family in bf16."""
    k = lambda w, dt: rb.rbgp_mask_kernel(rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed), dt)
    for d in (2, 3, 4):
        assert k(wl.sdmm4096_table3(1, 1, d), rb.F32) == rb.KERNEL_MFMA_REG_FILLED
    assert k(wl.sdmm4096_table3(2, 1, 3), rb.F32) == rb.KERNEL_MFMA_REG_FILLED
    assert k(wl.sdmm4096_table3(4, 1, 2), rb.F32) == rb.KERNEL_MFMA_REG_FILLED
    assert k(wl.sdmm4096_table3(4, 1, 4), rb.F32) == rb.KERNEL_MFMA_REG_FILLED
    assert k(wl.sdmm4096_table2(0, 2), rb.F32) == rb.KERNEL_MFMA_REG
    assert k(wl.sdmm4096_table2(3, 1), rb.F32) == rb.KERNEL_MFMA_REG_FILLED
    assert k(wl.sdmm4096_table2(2, 2), rb.F32) == rb.KERNEL_MFMA
    assert k(wl.sdmm4096_table2(3, 1), rb.BF16_F32ACC) == rb.KERNEL_MFMA_REG_FILLED
    for w in [wl.sdmm4096_table3(r, b, d) for (r, b) in ((1, 1), (2, 1), (4, 1), (2, 2)) for d in (2, 3, 4)]:
        assert k(w, rb.BF16_F32ACC) != rb.KERNEL_MFMA
    for w in wl.CONFIGS:                       # the fixed configurations stay where they were
        assert k(w, w.dtype) == rb.KERNEL_MFMA_REG
    # the mask of a lowered 3x3 convolution never takes the filled family by itself (rbgp_conv3x3 reads the register layout)
    conv = rb.rbgp_make_mask((32, 1, 16, 1), (32, 1, 8, 9), (16, 1, 2, 9), 3)
    assert rb.rbgp_mask_reg_plan(conv)[13] > 0 and rb.rbgp_mask_kernel(conv, rb.F32) != rb.KERNEL_MFMA_REG_FILLED


def test_every_vgg19_sweep_mask_runs_on_the_register_family():
    """The masks of the VGG19 layer sweep, their transposes and the masks of their transposed convolutions resolve to
    the register family whatever the estimates say: rbgp_conv3x3 and the fused gradients need its layout."""
    for layer in range(1, 16):
        for d in (1, 2, 3, 4):
            w = wl.vgg19_sweep_workload(layer, d, wl.F32)
            try:
                m = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
            except rb.RbgpError as e:
                assert e.code == rb.ENOTRAMANUJAN
                continue
            for mask in (m, rb.rbgp_mask_transpose(m), rb.rbgp_mask_conv3x3_transpose(m)):
                for dt in (rb.F32, rb.BF16_F32ACC):
                    assert rb.rbgp_mask_kernel(mask, dt) == rb.KERNEL_MFMA_REG, (w.name, dt)


def test_the_two_bf16_modes_share_kernel_choice_and_layout():
    """RBGP_BF16 only changes how rbgp_spmm / rbgp_conv3x3 store O: packed buffers are interchangeable."""
    for rows, cols, deg in LAYOUT_SHAPES[:4]:
        mask = rb.rbgp_make_mask(rows, cols, deg, 5)
        for kernel in (rb.KERNEL_AUTO, rb.KERNEL_GENERIC):
            rb.rbgp_mask_set_kernel(mask, kernel)
            assert rb.rbgp_mask_kernel(mask, rb.BF16) == rb.rbgp_mask_kernel(mask, rb.BF16_F32ACC)
            assert rb.rbgp_packed_bytes(mask, rb.BF16) == rb.rbgp_packed_bytes(mask, rb.BF16_F32ACC)
            assert np.array_equal(rb.rbgp_pack_layout(mask, rb.BF16), rb.rbgp_pack_layout(mask, rb.BF16_F32ACC))
    lib = rb.load()
    assert lib.rbgp_mask_kernel(mask.handle, 3) == rb.EINVAL
    assert lib.rbgp_packed_bytes(mask.handle, 3) == 0
    w = wl.TINY
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 1)
    assert lib.rbgp_spmm(mask.handle, rb.BF16, w.M + 1, w.K, 8, None, None, 8, None, 8, None) == rb.ESHAPE
    assert lib.rbgp_spmm(mask.handle, rb.BF16, w.M, w.K, 0, None, None, 0, None, 0, None) == rb.OK


# ---------------------------------------------------------------- transposed mask (backward data product)
@pytest.mark.parametrize("shape", LAYOUT_SHAPES[:6] + LAYOUT_SHAPES[9:], ids=lambda s: "x".join(map(str, s[0])))
def test_transposed_mask_and_order_match_the_oracle(shape):
    rows, cols, deg = shape
    seed = 5
    mask = rb.rbgp_make_mask(rows, cols, deg, seed)
    mask_t = rb.rbgp_mask_transpose(mask)
    sh, sht = rb.rbgp_mask_shape(mask), rb.rbgp_mask_shape(mask_t)
    assert (sht["M"], sht["K"], sht["rowdeg"], sht["coldeg"], sht["nnz"]) == \
           (sh["K"], sh["M"], sh["coldeg"], sh["rowdeg"], sh["nnz"])
    Bs, _ = orc.sample_factors(rows, cols, deg, seed)
    dense = orc.kron_mask(Bs)
    assert np.array_equal(rb.rbgp_mask_dense(mask_t), dense.T)
    order = rb.rbgp_transpose_order(mask)
    if dense.size <= 1 << 22:          # the oracle's order is a Python double loop
        assert np.array_equal(order, orc.transpose_order(dense))
    else:                              # large masks: a bijection that moves every value to its transposed place
        assert np.array_equal(np.sort(order), np.arange(sh["nnz"]))
        cols_f = rb.rbgp_mask_columns(mask).reshape(-1)
        cols_t = rb.rbgp_mask_columns(mask_t).reshape(-1)
        s = np.arange(sh["nnz"])
        assert np.array_equal(cols_f[order], s // sht["rowdeg"])         # row of W^T = column of W
        assert np.array_equal(cols_t, order // sh["rowdeg"])             # column of W^T = row of W
    # spectrum and factor sizes of the transposed factors
    for i in range(4):
        f, ft = rb.rbgp_mask_factor(mask, i), rb.rbgp_mask_factor(mask_t, i)
        assert (ft[0], ft[1]) == (f[1], f[0])
        assert rb.rbgp_mask_spectrum(mask_t, i) == rb.rbgp_mask_spectrum(mask, i)
    # transposing twice gives the mask back
    assert np.array_equal(rb.rbgp_mask_dense(rb.rbgp_mask_transpose(mask_t)), dense)


def test_pack_transposed_needs_a_transposed_mask():
    w = wl.TINY
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 1)
    vals = np.zeros(w.M * w.rowdeg, dtype=np.float32)
    with pytest.raises(rb.RbgpError) as ei:
        rb.rbgp_pack_transposed(mask, rb.F32, vals, 256)
    assert ei.value.code == rb.EINVAL


def test_sddmm_argument_checks_need_no_gpu():
    w = wl.TINY
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 1)
    lib = rb.load()
    assert lib.rbgp_sddmm(mask.handle, 0, w.M + 1, w.K, 8, 256, 8, 256, 8, 256, None) == rb.ESHAPE
    assert lib.rbgp_sddmm(mask.handle, 0, w.M, w.K, 8, 256, 4, 256, 8, 256, None) == rb.ESHAPE     # ld_dO < N
    assert lib.rbgp_sddmm(mask.handle, 0, w.M, w.K, 8, 256, 8, 256, 8, None, None) == rb.EINVAL    # no output
    assert lib.rbgp_sddmm(mask.handle, 0, w.M, w.K, 8, 258, 8, 256, 8, 256, None) == rb.ESHAPE     # misaligned
    assert lib.rbgp_sddmm(mask.handle, 7, w.M, w.K, 8, 256, 8, 256, 8, 256, None) == rb.EINVAL
    assert lib.rbgp_sddmm(None, 0, w.M, w.K, 8, 256, 8, 256, 8, 256, None) == rb.EINVAL


# ---------------------------------------------------------------- more than four base graphs
K_MASKS = [
    # rows, cols, row_deg, roles
    ((2, 2, 2, 4, 2, 2), (4, 2, 2, 8, 3, 3), (2, 1, 2, 4, 3, 3), (0, 0, 1, 2, 3, 3)),   # two sparse graphs in G_o, 3 x 3 taps
    ((4, 2, 4), (8, 2, 4), (2, 2, 2), (0, 1, 2)),                                       # three: no G_b
    ((4, 4, 2, 2, 3), (4, 8, 2, 4, 1), (2, 4, 2, 2, 1), (0, 2, 2, 2, 3)),                # three graphs in G_i, none in G_r
    ((8,), (16,), (4,), (2,)),                                                          # a single sparse graph
]


@pytest.mark.parametrize("case", K_MASKS, ids=lambda c: "x".join(map(str, c[0])))
def test_general_k_mask_is_the_product_of_its_base_graphs(case):
    rows, cols, deg, roles = case
    seed = 11
    mask = rb.rbgp_make_mask_k(rows, cols, deg, roles, seed)
    Bs, infos = orc.sample_factors(rows, cols, deg, seed)
    dense = orc.kron_mask(Bs)
    assert np.array_equal(rb.rbgp_mask_dense(mask), dense)
    sh = rb.rbgp_mask_shape(mask)
    assert (sh["M"], sh["K"]) == dense.shape and sh["rowdeg"] == int(dense[0].sum())
    # canonical order = ascending column per row
    assert np.array_equal(rb.rbgp_mask_columns(mask).reshape(sh["M"], -1), orc.canonical_columns(dense))
    # the base graphs, one by one
    assert rb.rbgp_mask_num_base(mask) == len(rows)
    for i, (B, info) in enumerate(zip(Bs, infos)):
        g = rb.rbgp_mask_base(mask, i)
        assert (g["rows"], g["cols"], g["deg"], g["role"]) == (rows[i], cols[i], deg[i], roles[i])
        assert np.array_equal(g["adj"], orc.adjacency_lists(B))
        assert g["status"] == info["status"] and g["tries"] == info["tries"]
        assert math.isclose(g["sigma1"], info["sigma1"], rel_tol=1e-9)
        assert math.isclose(g["sigma2"], info["sigma2"], rel_tol=1e-7, abs_tol=1e-9)
    # the four factors of the kernels' view: products of the base graphs of each role
    for role in range(4):
        mine = [B for B, r in zip(Bs, roles) if r == role]
        F = orc.kron_mask(mine) if mine else np.ones((1, 1), dtype=np.uint8)
        r_, c_, d_, adj = rb.rbgp_mask_factor(mask, role)
        assert (r_, c_) == F.shape and np.array_equal(adj, orc.adjacency_lists(F))
        sp = rb.rbgp_mask_spectrum(mask, role)
        sv = np.linalg.svd(F.astype(np.float64), compute_uv=False)
        assert math.isclose(sp["sigma1"], sv[0], rel_tol=1e-9)
        assert math.isclose(sp["sigma2"], sv[1] if sv.size > 1 else 0.0, rel_tol=1e-7, abs_tol=1e-7)
        if len(mine) > 1 and not all(int(B.min()) == 1 for B in mine):
            assert sp["status"] in (rb.SPEC_PRODUCT, rb.SPEC_DEGENERATE)
    # transposing keeps the base graphs (transposed)
    mt = rb.rbgp_mask_transpose(mask)
    assert rb.rbgp_mask_num_base(mt) == len(rows)
    assert np.array_equal(rb.rbgp_mask_base(mt, 0)["adj"], orc.adjacency_lists(Bs[0].T.copy()))


def test_four_base_graphs_in_order_is_rbgp_make_mask():
    w = wl.VGG19_CONV5
    a = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, 3)
    b = rb.rbgp_make_mask_k(w.rows, w.cols, w.row_deg, (0, 1, 2, 3), 3)
    assert np.array_equal(rb.rbgp_mask_columns(a), rb.rbgp_mask_columns(b))
    for i in range(4):
        assert rb.rbgp_mask_spectrum(a, i) == rb.rbgp_mask_spectrum(b, i)


def test_general_k_argument_checks():
    with pytest.raises(rb.RbgpError) as ei:
        rb.rbgp_make_mask_k((2, 2), (2, 2), (2, 2), (1, 0), 1)          # roles must not decrease
    assert ei.value.code == rb.EINVAL
    with pytest.raises(rb.RbgpError) as ei:
        rb.rbgp_make_mask_k((2, 2), (2, 2), (2, 2), (0, 4), 1)          # role out of range
    assert ei.value.code == rb.EINVAL
    with pytest.raises(rb.RbgpError) as ei:
        rb.rbgp_make_mask_k((2,) * 17, (2,) * 17, (2,) * 17, (0,) * 17, 1)
    assert ei.value.code == rb.EINVAL


@pytest.mark.parametrize("shape", [(512, 1024, 16), (1024, 1024, 16), (768, 384, 6)], ids=lambda s: "x".join(map(str, s)))
def test_base_graphs_of_a_thousand_vertices_match_the_oracle(shape):
    """Appendix, "Generating RBG graph": graphs with thousands of vertices.  Above 192 vertices the
    library finds sigma_2 by Lanczos iteration on the complement of the constant vector instead of
    a dense eigen-solver; the oracle takes numpy's SVD.  Same samples accepted, same graph."""
    a, c, d = shape
    seed = 1
    mask = rb.rbgp_make_mask((a, 1, 1, 1), (c, 1, 1, 1), (d, 1, 1, 1), seed)
    Bs, infos = orc.sample_factors((a,), (c,), (d,), seed)
    assert np.array_equal(rb.rbgp_mask_factor(mask, 0)[3], orc.adjacency_lists(Bs[0]))
    sp = rb.rbgp_mask_spectrum(mask, 0)
    assert sp["tries"] == infos[0]["tries"] and sp["status"] == infos[0]["status"]
    assert math.isclose(sp["sigma1"], infos[0]["sigma1"], rel_tol=1e-10)
    assert math.isclose(sp["sigma2"], infos[0]["sigma2"], rel_tol=1e-9)
    assert sp["sigma2"] <= sp["bound"]


# ---------------------------------------------------------------- transposed 3x3 convolution
@pytest.mark.parametrize("shape", [((4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9)), ((4, 1, 4, 3), (4, 2, 4, 9), (2, 2, 2, 9)),
                                   ((2, 3, 4, 1), (2, 2, 4, 9), (1, 2, 2, 9))], ids=lambda s: "x".join(map(str, s[0])))
def test_conv3x3_transposed_mask_holds_the_flipped_kernel(shape):
    """W'[c][9 m + tap'] = W[m][9 c + (8 - tap')]: mask and value order of the convolution that
    computes the gradient with respect to the input."""
    rows, cols, deg = shape
    mask = rb.rbgp_make_mask(rows, cols, deg, 4)
    mx = rb.rbgp_mask_conv3x3_transpose(mask)
    sh, shx = rb.rbgp_mask_shape(mask), rb.rbgp_mask_shape(mx)
    M, K = sh["M"], sh["K"]
    assert (shx["M"], shx["K"], shx["nnz"]) == (K // 9, 9 * M, sh["nnz"])
    dense = rb.rbgp_mask_dense(mask).astype(np.int64)
    vals = np.arange(1, sh["nnz"] + 1, dtype=np.float64).reshape(M, -1)
    W = orc.scatter_values(dense, vals)                                   # distinct values: tracks every entry
    Wx = np.zeros((K // 9, 9 * M))
    for m in range(M):
        for c in range(K // 9):
            for tap in range(9):
                Wx[c, 9 * m + tap] = W[m, 9 * c + 8 - tap]
    assert np.array_equal(rb.rbgp_mask_dense(mx), (Wx != 0).astype(np.uint8))
    order = rb.rbgp_mask_original_order(mx)
    valsx = vals.reshape(-1)[order].reshape(shx["M"], -1)
    assert np.array_equal(orc.scatter_values((Wx != 0).astype(np.uint8), valsx), Wx)
    # the plain transpose reports the same table as rbgp_transpose_order
    assert np.array_equal(rb.rbgp_mask_original_order(rb.rbgp_mask_transpose(mask)), rb.rbgp_transpose_order(mask))
    with pytest.raises(rb.RbgpError):
        rb.rbgp_mask_original_order(mask)
    with pytest.raises(rb.RbgpError) as ei:
        rb.rbgp_mask_conv3x3_transpose(rb.rbgp_make_mask(wl.TINY.rows, wl.TINY.cols, wl.TINY.row_deg, 1))
    assert ei.value.code == rb.EUNSUPPORTED


# ------------------------------------------------------------------ index tables of the register family
def _all_workload_shapes():
    from tests import test_gpu_parity as tp
    shapes = [(w.rows, w.cols, w.row_deg) for w in wl.CONFIGS]
    for layer in range(len(wl.VGG19_LAYERS)):
        for d in (1, 2, 3, 4):
            w = wl.vgg19_sweep_workload(layer, d, wl.F32)
            shapes.append((w.rows, w.cols, w.row_deg))
    for o, i in [(0, 2), (1, 1), (0, 3), (1, 2), (2, 1), (0, 4), (1, 3), (2, 2), (3, 1)]:
        w = wl.sdmm4096_table2(o, i)
        shapes.append((w.rows, w.cols, w.row_deg))
    for gr, gb in [(1, 1), (2, 1), (4, 1), (1, 2), (1, 4), (2, 2)]:
        w = wl.sdmm4096_table3(gr, gb, 3)
        shapes.append((w.rows, w.cols, w.row_deg))
    shapes += list(tp.FUZZ) + list(tp.PAIRING_SHAPES)
    return sorted(set(shapes))


def test_index_tables_are_consistent_for_every_workload_shape():
    """The library's own check of the tables its register kernels read -- every (tile row, tile, stage)
    multiplied exactly once by a stage of that tile, fragment positions inside the packed buffer, rows of I
    inside the stage -- on every mask shape of the benchmarks and GPU tests, their transposes and the masks
    of their transposed convolutions."""
    count = 0
    for rows, cols, deg in _all_workload_shapes():
        try:
            mask = rb.rbgp_make_mask(rows, cols, deg, 77)
        except rb.RbgpError as e:          # (a cell whose factor cannot be sampled is recorded by the sweep, not hidden)
            assert e.code == rb.ENOTRAMANUJAN
            continue
        derived = [mask, rb.rbgp_mask_transpose(mask)]
        if cols[3] == 9 and deg[3] == 9:
            derived.append(rb.rbgp_mask_conv3x3_transpose(mask))
        for m in derived:
            rb.rbgp_mask_check_tables(m)
            info = rb.rbgp_mask_reg_plan(m)
            if info[0]:                    # the family covers the mask
                MG, NSTG, TR, ncl, longest, total = info[0], info[1], info[3], info[4], info[5], info[6]
                d_o = rb.rbgp_mask_factor(m, 0)[2]
                per_row = d_o * NSTG
                assert ncl == -(-TR // MG) and per_row <= longest <= MG * per_row
                assert -(-TR * per_row // MG) <= total <= ncl * MG * per_row
                if info[7]:                # tile-by-tile pairing: never more work than one stage per (tile row, tile)
                    assert info[0] == 2 and info[7] == -(-TR // 4)
                    assert -(-TR * per_row // 2) <= info[9] <= TR * per_row
                    assert info[10] <= info[8] <= 2 * info[10] and info[8] >= min(TR, 2) * per_row // 2
            count += 1
    assert count > 150


def test_pairing_of_the_conv5_mask_multiplies_no_zero_rows():
    """VGG19 conv5 at density 1/8: G_o is one 2-lift of the complete graph on (8, 8) vertices, so the tile
    rows u and u + 8 have complementary tiles (Appendix: the clone of an edge is the identity pair or the
    crossover pair).  Fixed pairs of tile rows walk 9 or 10 tiles for 8 each; quads of two complementary
    pairs walk 8 tiles per SIMD with all 16 rows of every MFMA group rows of the mask."""
    w = wl.VGG19_CONV5
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    _, _, d_o, adj = rb.rbgp_mask_factor(mask, 0)
    has = np.zeros((16, 16), bool)
    for u in range(16):
        has[u, adj[u]] = True
    assert all((has[u] ^ has[u + 8]).all() for u in range(8))
    info = rb.rbgp_mask_reg_plan(mask)
    assert info[:7] == [2, 1, 72, 16, 8, 10, 76]
    assert info[7:11] == [4, 8, 64, info[10]] and info[9] == 16 * d_o // 2
