"""GPU parity of the backward products (gradients of O = W_s x I for a fixed mask, Section 6)
against the CPU oracle, through the C ABI: dI = W_s^T x dO on the transposed mask, and
dW = (dO x I^T) sampled on the mask."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl
from tests import gpu_harness as gh
from tests.test_gpu_parity import FUZZ

pytestmark = pytest.mark.gpu

GEN, MFMA, REG = rb.KERNEL_GENERIC, rb.KERNEL_MFMA, rb.KERNEL_MFMA_REG


def _check_backward(w, N=None, ld_pad=0, kernels=(rb.KERNEL_AUTO,), data=True, weights=True):
    lib, f32 = gh.backward_inputs(w, N)
    dI_ref, dI_den, dW_ref, dW_den = gh.oracle_backward(w, *f32)
    for kernel in kernels:
        if data:
            dI, used = gh.library_spmm_transposed(w, lib[0], lib[2], kernel=kernel, ld_pad=ld_pad)
            err = orc.normalised_error(dI, dI_ref, dI_den)
            print(f"[gpu]   dI kernel {used} normalised error {err:.3e}", flush=True)
            assert err <= gh.TOL[w.dtype], ("dI", w.name, kernel, err)
        if weights:
            dW = gh.library_sddmm(w, lib[2], lib[1], kernel=kernel, ld_pad=ld_pad)
            err = orc.normalised_error(dW, dW_ref, dW_den)
            print(f"[gpu]   dW normalised error {err:.3e}", flush=True)
            assert err <= gh.TOL[w.dtype], ("dW", w.name, kernel, err)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("idx", range(len(FUZZ)))
def test_backward_products_across_the_kernel_table(idx, dtype):
    rows, cols, deg = FUZZ[idx]
    w = wl.Workload(f"bwd{idx}_{dtype}", rows, cols, deg, 328, dtype, 400 + idx, 500 + idx, 600 + idx, 1.0)
    _check_backward(w, kernels=(rb.KERNEL_AUTO, GEN))


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("N,ld_pad", [(1, 7), (15, 1), (16, 0), (33, 3), (200, 8), (1000, 0), (2049, 15)])
def test_backward_products_ragged_batch(N, ld_pad, dtype):
    """Batch sizes around the kernels' column steps (16 / 32 per iteration, ranges of the split),
    odd leading dimensions included (bf16 with an odd one runs on the plain kernel)."""
    w = wl.Workload(f"bwd_ragged_{dtype}", (4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9), N, dtype, 41, 42, 43, 1.0)
    _check_backward(w, ld_pad=ld_pad)


@pytest.mark.parametrize("w", [wl.TINY, wl.VGG19_CONV5, wl.VGG19_CONV3_BF16], ids=lambda w: w.name)
def test_backward_products_config_full_size(w):
    _check_backward(w)


def test_weight_gradient_wrn_full_batch():
    """131072 columns: the batch is cut into many ranges whose partial sums are added in a second kernel."""
    _check_backward(wl.WRN_G1, data=False)


def test_backward_data_product_wrn_sampled_batch():
    _check_backward(replace(wl.WRN_G1, N=4096), weights=False)


def test_weight_gradient_repeated_calls_and_growing_batch():
    """The partial-sum buffer is kept with the mask: a small batch first, then a larger one, then the
    small one again, every result checked."""
    mask_w = wl.Workload("bwd_grow", (4, 2, 4, 2), (4, 2, 8, 9), (2, 2, 4, 9), 0, wl.F32, 51, 52, 53, 1.0)
    for N in (96, 4000, 96):
        _check_backward(replace(mask_w, N=N), data=False)


def test_weight_gradient_empty_batch_stores_zeros():
    w = replace(wl.TINY, N=0)
    dW = gh.library_sddmm(w, np.zeros((w.M, 0), np.float32), np.zeros((w.K, 0), np.float32))
    assert not dW.any()


@pytest.mark.parametrize("kernel", [rb.KERNEL_AUTO, GEN])
def test_weight_gradient_one_hot_inputs_are_exact(kernel):
    """dO = ones in column n of every row, I = distinct powers of two in the same column: dW repeats
    the value of I at each kept column exactly."""
    w = replace(wl.TINY, N=40)
    dO = np.zeros((w.M, w.N), np.float32); dO[:, 17] = 1.0
    I = np.zeros((w.K, w.N), np.float32); I[:, 17] = np.ldexp(1.0, np.arange(w.K) % 24 - 12).astype(np.float32)
    I[:, 3] = 5.0                                   # a column that dO does not touch
    dW = gh.library_sddmm(w, dO, I, kernel=kernel)
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    cols = rb.rbgp_mask_columns(mask).reshape(w.M, w.rowdeg)
    assert np.array_equal(dW, I[cols, 17])


def test_masks_outside_rbgp4_roles_take_the_plain_kernels():
    w = wl.Workload("bwd_sparse_gr", (4, 4, 4, 2), (4, 4, 4, 2), (2, 2, 2, 2), 100, wl.F32, 1, 2, 3, 1.0)
    _check_backward(w)


def test_weight_gradient_bf16_odd_leading_dimension():
    w = wl.Workload("bwd_odd_ld", (4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9), 77, wl.BF16, 44, 45, 46, 1.0)
    _check_backward(w, data=False)


def test_pack_transposed_from_device_values_matches_host_values():
    """The same kept values, resident on the device in the forward mask's order, packed for both products."""
    import torch
    w = wl.Workload("bwd_devpack", (4, 2, 4, 2), (4, 2, 8, 9), (2, 2, 4, 9), 64, wl.F32, 54, 55, 56, 1.0)
    mask = gh.make_mask(w)
    mask_t = rb.rbgp_mask_transpose(mask)
    vals = wl.kept_weights(w).reshape(-1)
    stream = torch.cuda.current_stream().cuda_stream
    nbytes = rb.rbgp_packed_bytes(mask_t, w.dtype)
    a = torch.zeros(nbytes, dtype=torch.uint8, device="cuda:0")
    b = torch.zeros(nbytes, dtype=torch.uint8, device="cuda:0")
    rb.rbgp_pack_transposed(mask_t, w.dtype, vals, a.data_ptr(), stream)
    vals_d = torch.from_numpy(vals).to("cuda:0")
    rb.rbgp_pack_transposed_device(mask_t, w.dtype, vals_d.data_ptr(), b.data_ptr(), stream)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    # and it is the transposed mask's own packing of the reordered values
    c = torch.zeros(nbytes, dtype=torch.uint8, device="cuda:0")
    rb.rbgp_pack(mask_t, w.dtype, np.ascontiguousarray(vals[rb.rbgp_transpose_order(mask)]), c.data_ptr(), stream)
    torch.cuda.synchronize()
    assert torch.equal(a, c)


# ------------------------------------------------------------------ weight gradient of the fused 3x3 convolution
CONV_GRAD_CASES = [
    # workload (K = 9 * channels), images, height, width
    (wl.Workload("cgrad_small", (4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9), 0, wl.F32, 61, 62, 63, 1.0), 3, 4, 8),
    (wl.Workload("cgrad_ragged", (4, 1, 4, 3), (4, 2, 4, 9), (2, 2, 2, 9), 0, wl.F32, 64, 65, 66, 1.0), 5, 3, 4),
    (wl.Workload("cgrad_wide", (4, 2, 4, 1), (4, 2, 4, 9), (2, 2, 2, 9), 0, wl.F32, 67, 68, 69, 1.0), 2, 5, 32),
    (wl.Workload("cgrad_pad54", (4, 2, 4, 1), (4, 1, 12, 9), (2, 1, 6, 9), 0, wl.F32, 74, 75, 76, 1.0), 2, 4, 8),
    (wl.Workload("cgrad_bf16", (4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9), 0, wl.BF16, 71, 72, 73, 1.0), 3, 5, 8),
    (wl.Workload("cgrad_bf16_wide", (4, 2, 4, 1), (4, 2, 4, 9), (2, 2, 2, 9), 0, wl.BF16, 77, 78, 79, 1.0), 7, 3, 16),
    (wl.VGG19_CONV5, 128, 4, 4),                                        # the headline layer
    (replace(wl.VGG19_CONV3_BF16, name="cgrad_conv3_bf16"), 128, 8, 8),
    (replace(wl.WRN_G1, name="cgrad_wrn_batch8"), 8, 32, 32),
]


@pytest.mark.parametrize("case", CONV_GRAD_CASES, ids=lambda c: c[0].name)
def test_fused_conv3x3_weight_gradient_equals_sddmm_on_the_lowered_input(case):
    w, B, H, W = case
    w = replace(w, N=B * H * W)
    X = wl.conv_activations(w, B, H, W)
    dO = wl.output_gradients(w)
    if w.dtype == wl.BF16:
        Xl, dOl = wl.to_bf16_bits(X), wl.to_bf16_bits(dO)
        X, dO = wl.bf16_bits_as_f32(Xl), wl.bf16_bits_as_f32(dOl)
    else:
        Xl, dOl = X, dO
    got = gh.library_conv3x3_sddmm(w, dOl, Xl)
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    mask = orc.kron_mask(Bs)
    I = orc.im2col_3x3(X)
    ref, den = orc.sddmm_definition(mask, dO, I), orc.sddmm_definition(mask, np.abs(dO), np.abs(I))
    err = orc.normalised_error(got, ref, den)
    print(f"[gpu]   normalised error {err:.3e}", flush=True)
    assert err <= gh.TOL[w.dtype], err


def test_fused_conv3x3_weight_gradient_argument_checks():
    w = wl.Workload("cgrad_args", (4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9), 0, wl.F32, 1, 2, 3, 1.0)
    mask = gh.make_mask(w)
    lib = rb.load()
    C = w.K // 9
    assert lib.rbgp_conv3x3_sddmm(mask.handle, 0, w.M, C, 2, 4, 6, 256, 48, 256, 256, None) == rb.ESHAPE      # width % 4
    assert lib.rbgp_conv3x3_sddmm(mask.handle, 1, w.M, C, 2, 4, 4, 256, 32, 256, 256, None) == rb.ESHAPE      # bf16: width % 8
    assert lib.rbgp_conv3x3_sddmm(mask.handle, 0, w.M, C + 1, 2, 4, 4, 256, 32, 256, 256, None) == rb.ESHAPE
    assert lib.rbgp_conv3x3_sddmm(mask.handle, 0, w.M, C, 2, 4, 4, 256, 16, 256, 256, None) == rb.ESHAPE      # ld_dO < N
    assert lib.rbgp_conv3x3_sddmm(mask.handle, 0, w.M, C, 2, 4, 4, 256, 32, None, 256, None) == rb.EINVAL
    tiny = gh.make_mask(wl.TINY)                                                                             # |G_b.V| != 9
    assert lib.rbgp_conv3x3_sddmm(tiny.handle, 0, wl.TINY.M, wl.TINY.K // 9, 1, 1, 4, 256, 4, 256, 256, None) in (rb.ESHAPE, rb.EUNSUPPORTED)


# ------------------------------------------------------------------ gradient of the fused convolution w.r.t. its input
@pytest.mark.parametrize("case", CONV_GRAD_CASES, ids=lambda c: c[0].name)
def test_fused_conv3x3_input_gradient_is_the_transposed_convolution(case):
    w, B, H, W = case
    w = replace(w, N=B * H * W)
    vals, dO = wl.kept_weights(w), wl.output_gradients(w)
    if w.dtype == wl.BF16:
        vl, dOl = wl.to_bf16_bits(vals), wl.to_bf16_bits(dO)
        vals, dO = wl.bf16_bits_as_f32(vl), wl.bf16_bits_as_f32(dOl)
    else:
        vl, dOl = vals, dO
    got, used = gh.library_conv3x3_input_gradient(w, vl, dOl, B, H, W)
    assert used == REG
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    mask = orc.kron_mask(Bs)
    Wd = orc.scatter_values(mask, vals)
    maskT, WT = np.ascontiguousarray(mask.T), np.ascontiguousarray(Wd.T)
    from oracle import naive_c
    dI, dI_den = naive_c.spmm(maskT, WT, dO), naive_c.spmm_abs(maskT, WT, dO)
    ref = orc.col2im_3x3(dI, B, H, W).reshape(w.K // 9, -1)
    den = orc.col2im_3x3(dI_den, B, H, W).reshape(w.K // 9, -1)
    err = orc.normalised_error(got, ref, den)
    print(f"[gpu]   normalised error {err:.3e}", flush=True)
    assert err <= gh.TOL[w.dtype], err


def test_training_step_replays_from_a_hip_graph():
    """Forward, input gradient and weight gradient of a fused 3x3 layer captured into one graph after a
    warm-up call (which builds the library's tables and its partial-sum buffer): three replays on fresh
    inputs, with eager work and synchronisations in between, each compared with the eager result."""
    import torch
    w = wl.Workload("graph_layer", (4, 2, 4, 2), (4, 2, 8, 9), (2, 2, 4, 9), 0, wl.F32, 31, 32, 33, 1.0)
    B, H, W = 6, 8, 8
    N = B * H * W
    C = w.K // 9
    mask = gh.make_mask(w)
    mask_x = rb.rbgp_mask_conv3x3_transpose(mask)
    vals = wl.kept_weights(w).reshape(-1)
    dev = "cuda:0"
    packed = torch.zeros(rb.rbgp_packed_bytes(mask, w.dtype), dtype=torch.uint8, device=dev)
    packed_x = torch.zeros(rb.rbgp_packed_bytes(mask_x, w.dtype), dtype=torch.uint8, device=dev)
    st0 = torch.cuda.current_stream().cuda_stream
    rb.rbgp_pack(mask, w.dtype, vals, packed.data_ptr(), st0)
    rb.rbgp_pack_transposed(mask_x, w.dtype, vals, packed_x.data_ptr(), st0)
    X = torch.zeros(C, B, H + 2, W + 2, device=dev)
    dO = torch.zeros(w.M, B, H + 2, W + 2, device=dev)          # padded: read by the input-gradient convolution
    dO_flat = torch.zeros(w.M, N, device=dev)                   # the same values as a matrix: read by the weight gradient
    O = torch.zeros(w.M, N, device=dev)
    dX = torch.zeros(C, N, device=dev)
    dW = torch.zeros(w.M * w.rowdeg, device=dev)

    def step(stream):
        rb.rbgp_conv3x3(mask, w.dtype, w.M, C, B, H, W, packed.data_ptr(), X.data_ptr(), O.data_ptr(), N, stream)
        rb.rbgp_conv3x3(mask_x, w.dtype, C, w.M, B, H, W, packed_x.data_ptr(), dO.data_ptr(), dX.data_ptr(), N, stream)
        rb.rbgp_conv3x3_sddmm(mask, w.dtype, w.M, C, B, H, W, dO_flat.data_ptr(), N, X.data_ptr(), dW.data_ptr(), stream)

    def fresh_inputs(seed):
        g = torch.Generator(device=dev).manual_seed(seed)
        X[:, :, 1:-1, 1:-1] = torch.randn(C, B, H, W, device=dev, generator=g)
        d = torch.randn(w.M, B, H, W, device=dev, generator=g)
        dO[:, :, 1:-1, 1:-1] = d
        dO_flat.copy_(d.reshape(w.M, N))

    fresh_inputs(0)
    step(st0)                                                    # warm-up: tables, partial sums
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream().cuda_stream)
    for seed in (1, 2, 3):
        fresh_inputs(seed)
        step(torch.cuda.current_stream().cuda_stream)            # eager reference
        torch.cuda.synchronize()
        ref = [t.clone() for t in (O, dX, dW)]
        for t in (O, dX, dW):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((O, dX, dW), ref):
            assert torch.equal(got, want)                        # same kernels, same order of sums: bit-identical
