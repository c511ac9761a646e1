"""GPU parity of the bf16-output mode (RBGP_BF16): rbgp_spmm / rbgp_conv3x3 round their fp32
sums to bfloat16 when they store O.

Two checks per case.  (1) Against the oracle: every stored value lies within half a bfloat16
unit in the last place of the exact (fp64) sum, plus the fp32 accumulation error.  (2) The
rounding itself, decided on both sides from the same fp32 number: the bits equal the oracle's
round-to-nearest-even of what the same launch stores in RBGP_BF16_F32ACC mode (same kernel, same
summation order, fp32 output)."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu

GEN, MFMA, REG = rb.KERNEL_GENERIC, rb.KERNEL_MFMA, rb.KERNEL_MFMA_REG

HALF_ULP = 2.0 ** -8          # half a unit in the last place of a bfloat16, relative to the value
ACC_TOL = 4e-6                # fp32 accumulation error relative to sum |w||i| (measured: below 1e-6)


def check_bf16_output(w, N=None, kernel=rb.KERNEL_AUTO, tune=None, ld_pad=0, ref=None):
    vl, Il, vf, If = gh.host_inputs(w, N)
    out16, used = gh.library_spmm(w, vl, Il, kernel, tune, ld_pad, tag="bf16 out", out_bf16=True)
    out32, used32 = gh.library_spmm(w, vl, Il, kernel, tune, ld_pad, tag="fp32 out")
    assert used == used32
    want_bits = orc.f32_to_bf16_bits(out32)
    assert not np.any(out16.view(np.uint32) & 0xFFFF)
    got_bits = (out16.view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(got_bits, want_bits), f"{np.count_nonzero(got_bits != want_bits)} values rounded differently"
    if ref is None:
        ref = gh.oracle_spmm(w, vf, If)
    exact, den = ref
    bound = HALF_ULP * np.abs(exact) + ACC_TOL * den + 1e-38
    worst = float(np.max(np.abs(out16.astype(np.float64) - exact) / bound))
    print(f"[gpu]   worst error / bound {worst:.3f}", flush=True)
    assert worst <= 1.0
    return used


@pytest.mark.parametrize("cw", [64, 128])
@pytest.mark.parametrize("groups,split", [(1, 1), (2, 2), (4, 4), (1, 4), (4, 1)])
def test_register_family(groups, split, cw):
    """Every wave-tile width, with and without row groups and the stage split; ragged last tile."""
    tune = (0, cw, 0, 0, groups, split)
    assert check_bf16_output(wl.VGG19_CONV3_BF16, N=1000, kernel=REG, tune=tune) == REG
    w = wl.Workload("bf16_rs4", (6, 2, 4, 2), (6, 1, 4, 9), (3, 1, 2, 9), 200, wl.BF16, 21, 22, 23, 1.0)
    assert check_bf16_output(w, kernel=REG, tune=tune) == REG


@pytest.mark.parametrize("N,ld_pad", [(1, 7), (63, 1), (64, 0), (65, 3), (200, 8), (257, 15), (1002, 2), (1004, 0)])
def test_ragged_columns_and_leading_dimensions(N, ld_pad):
    """Leading dimensions of O that allow 16-byte, 8-byte or only 2-byte stores; the padding of
    O stays untouched (checked by the harness)."""
    w = replace(wl.VGG19_CONV5, rows=(4, 4, 4, 2), cols=(4, 4, 8, 9), row_deg=(2, 4, 2, 9), dtype=wl.BF16,
                name="ragged_bf16_out")
    ref = gh.oracle_spmm(w, *gh.host_inputs(w, N)[2:])
    pad4 = (-N) % 4 + ld_pad // 4 * 4           # register family: ldI a multiple of 4
    pad8 = (-N) % 8 + ld_pad // 8 * 8           # LDS family, 128-column tiles: a multiple of 8
    assert check_bf16_output(w, N=N, kernel=REG, ld_pad=pad4, ref=ref) == REG
    assert check_bf16_output(w, N=N, kernel=REG, tune=(0, 128, 0, 0, 2, 2), ld_pad=pad8, ref=ref) == REG
    for tune in [(1, 64, 0), (2, 128, 0)]:
        assert check_bf16_output(w, N=N, kernel=MFMA, tune=tune, ld_pad=pad8, ref=ref) == MFMA
    assert check_bf16_output(w, N=N, kernel=GEN, ld_pad=ld_pad, ref=ref) == GEN


def test_full_size_default_launch():
    """The VGG19 conv3 configuration at full size with the library's defaults."""
    assert check_bf16_output(wl.VGG19_CONV3_BF16) == REG


def test_lds_family_and_generic_kernel():
    assert check_bf16_output(wl.VGG19_CONV3_BF16, N=1536, kernel=MFMA) == MFMA
    assert check_bf16_output(wl.VGG19_CONV3_BF16, N=520, kernel=GEN) == GEN
    w = replace(wl.TINY, dtype=wl.BF16, name="tiny_bf16_out")
    for kernel in (REG, MFMA, GEN):
        check_bf16_output(w, kernel=kernel)


@pytest.mark.parametrize("case", [
    (wl.VGG19_CONV3_BF16, 128, 8, 8),
    (replace(wl.VGG19_CONV3_BF16, name="conv3_bf16_4x4"), 33, 4, 4),
    (wl.Workload("conv_small_bf16", (4, 2, 2, 4), (4, 2, 4, 9), (2, 2, 4, 9), 0, wl.BF16, 71, 72, 73, 1.0), 3, 5, 8),
], ids=lambda c: c[0].name)
def test_fused_conv3x3(case):
    w, B, H, W = case
    vals_lib, X_lib = wl.to_bf16_bits(wl.kept_weights(w)), wl.to_bf16_bits(wl.conv_activations(w, B, H, W))
    vals, X = wl.bf16_bits_as_f32(vals_lib), wl.bf16_bits_as_f32(X_lib)
    exact, den = gh.oracle_spmm(w, vals, orc.im2col_3x3(X))
    for tune in [None, (0, 0, 0, 0, 0, 2), (0, 64, 0, 0, 2, 1)]:
        out16 = gh.library_conv3x3(w, vals_lib, X_lib, tune=tune, out_bf16=True)
        out32 = gh.library_conv3x3(w, vals_lib, X_lib, tune=tune)
        assert np.array_equal((out16.view(np.uint32) >> 16).astype(np.uint16), orc.f32_to_bf16_bits(out32))
        bound = HALF_ULP * np.abs(exact) + ACC_TOL * den + 1e-38
        assert float(np.max(np.abs(out16.astype(np.float64) - exact) / bound)) <= 1.0


def test_transposed_product_and_weight_gradient_take_the_mode():
    """dI = W_s^T dO stored as bf16 (what the layer below consumes in a bf16 training step);
    rbgp_sddmm treats the two bf16 modes alike (dW stays fp32)."""
    import torch
    w = replace(wl.VGG19_CONV3_BF16, N=776)
    (vl, Il, dOl), _ = gh.backward_inputs(w)
    dI32, _ = gh.library_spmm_transposed(w, vl, dOl)
    mask = gh.make_mask(w)
    mask_t = rb.rbgp_mask_transpose(mask)
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(rb.rbgp_packed_bytes(mask_t, rb.BF16), dtype=torch.uint8, device="cuda:0")
    assert rb.rbgp_packed_bytes(mask_t, rb.BF16) == rb.rbgp_packed_bytes(mask_t, rb.BF16_F32ACC)
    rb.rbgp_pack_transposed(mask_t, rb.BF16, vl, packed.data_ptr(), stream)
    dO_d = torch.from_numpy(dOl.view(np.int16)).to("cuda:0")
    dI_d = torch.full((w.K, w.N), 0x7FC0, dtype=torch.int16, device="cuda:0")
    print("[gpu] transposed product, bf16 output", flush=True)
    rb.rbgp_spmm(mask_t, rb.BF16, w.K, w.M, w.N, packed.data_ptr(), dO_d.data_ptr(), w.N, dI_d.data_ptr(), w.N, stream)
    torch.cuda.synchronize()
    assert np.array_equal(dI_d.cpu().numpy().view(np.uint16), orc.f32_to_bf16_bits(dI32))

    I_d = torch.from_numpy(Il.view(np.int16)).to("cuda:0")
    dW = [torch.full((w.nnz,), float("nan"), dtype=torch.float32, device="cuda:0") for _ in range(2)]
    for dt, out in zip((rb.BF16_F32ACC, rb.BF16), dW):
        print(f"[gpu] sddmm dtype {dt}", flush=True)
        rb.rbgp_sddmm(mask, dt, w.M, w.K, w.N, dO_d.data_ptr(), w.N, I_d.data_ptr(), w.N, out.data_ptr(), stream)
    torch.cuda.synchronize()
    assert torch.equal(dW[0], dW[1])


def test_argument_checks():
    import torch
    w = replace(wl.VGG19_CONV3_BF16, N=64)
    mask = gh.make_mask(w)
    packed = torch.zeros(rb.rbgp_packed_bytes(mask, rb.BF16), dtype=torch.uint8, device="cuda:0")
    I_d = torch.zeros((w.K, w.N), dtype=torch.int16, device="cuda:0")
    O_d = torch.zeros((w.M, w.N + 8), dtype=torch.int16, device="cuda:0")
    with pytest.raises(rb.RbgpError) as e:      # O not aligned to its element
        rb.rbgp_spmm(mask, rb.BF16, w.M, w.K, w.N, packed.data_ptr(), I_d.data_ptr(), w.N, O_d.data_ptr() + 1, w.N, 0)
    assert e.value.code == rb.ESHAPE
    with pytest.raises(rb.RbgpError) as e:      # no such mode
        rb.rbgp_spmm(mask, 3, w.M, w.K, w.N, packed.data_ptr(), I_d.data_ptr(), w.N, O_d.data_ptr(), w.N, 0)
    assert e.value.code == rb.EINVAL
    torch.cuda.synchronize()


def test_two_layer_chain_in_bf16_from_a_hip_graph():
    """What the mode is for: layer 1 stores its output as bf16 and layer 2 reads it as its input, no
    conversion pass in between.  Layer 1 on the tile family, layer 2 on the register family; both
    launches captured into one graph after a warm-up call; three replays on fresh inputs, each bit-equal
    to the eager calls and, for the final output, within the bf16 tolerance of the oracle's two products
    (the oracle rounds its own intermediate to bf16 with its own converter)."""
    import torch
    N = 1000
    w1 = wl.Workload("chain_l1", (8, 4, 4, 2), (8, 4, 8, 9), (4, 4, 4, 9), N, wl.BF16, 21, 22, 23, 0.05)
    w2 = wl.Workload("chain_l2", (4, 2, 4, 2), (8, 2, 4, 4), (4, 2, 2, 4), N, wl.BF16, 24, 25, 26, 0.05)
    assert w1.M == w2.K
    m1, m2 = gh.make_mask(w1), gh.make_mask(w2)
    rb.rbgp_mask_set_kernel(m1, rb.KERNEL_MFMA_TILE)
    v1, v2 = wl.to_bf16_bits(wl.kept_weights(w1)), wl.to_bf16_bits(wl.kept_weights(w2))
    dev = "cuda:0"
    st0 = torch.cuda.current_stream().cuda_stream
    p1 = torch.zeros(rb.rbgp_packed_bytes(m1, rb.BF16), dtype=torch.uint8, device=dev)
    p2 = torch.zeros(rb.rbgp_packed_bytes(m2, rb.BF16), dtype=torch.uint8, device=dev)
    rb.rbgp_pack(m1, rb.BF16, v1, p1.data_ptr(), st0)
    rb.rbgp_pack(m2, rb.BF16, v2, p2.data_ptr(), st0)
    I1 = torch.zeros((w1.K, N), dtype=torch.int16, device=dev)
    O1 = torch.zeros((w1.M, N), dtype=torch.int16, device=dev)      # bf16 bits: output of layer 1, input of layer 2
    O2 = torch.zeros((w2.M, N), dtype=torch.float32, device=dev)

    def step(stream):
        rb.rbgp_spmm(m1, rb.BF16, w1.M, w1.K, N, p1.data_ptr(), I1.data_ptr(), N, O1.data_ptr(), N, stream)
        rb.rbgp_spmm(m2, rb.BF16_F32ACC, w2.M, w2.K, N, p2.data_ptr(), O1.data_ptr(), N, O2.data_ptr(), N, stream)

    print("[gpu] bf16 chain: warm-up", flush=True)
    step(st0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream().cuda_stream)
    Bs1, _ = orc.sample_factors(w1.rows, w1.cols, w1.row_deg, w1.mask_seed)
    Bs2, _ = orc.sample_factors(w2.rows, w2.cols, w2.row_deg, w2.mask_seed)
    mk1, mk2 = orc.kron_mask(Bs1), orc.kron_mask(Bs2)
    W1 = orc.scatter_values(mk1, wl.bf16_bits_as_f32(v1))
    W2 = orc.scatter_values(mk2, wl.bf16_bits_as_f32(v2))
    for seed in (1, 2, 3):
        print(f"[gpu] bf16 chain: replay {seed}", flush=True)
        Ib = wl.to_bf16_bits(wl.activations(replace(w1, i_seed=100 + seed)))
        I1.copy_(torch.from_numpy(Ib.view(np.int16)))
        step(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        ref1, ref2 = O1.clone(), O2.clone()
        O1.fill_(0x7FC0)
        O2.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O1, ref1) and torch.equal(O2, ref2)
        mid = orc.spmm_definition(mk1, W1, wl.bf16_bits_as_f32(Ib))
        mid_bits = orc.f32_to_bf16_bits(mid.astype(np.float32))
        got_mid = O1.cpu().numpy().view(np.uint16)
        # the two sides round sums that differ in their last bits, so a few codes differ (by more than one unit
        # where a sum cancels to nearly nothing); the bound is the one of check_bf16_output
        differ = np.count_nonzero(got_mid != mid_bits)
        den1 = orc.spmm_definition(mk1, np.abs(W1), np.abs(wl.bf16_bits_as_f32(Ib)))
        bound = HALF_ULP * np.abs(mid) + ACC_TOL * den1 + 1e-38
        assert float(np.max(np.abs(orc.bf16_bits_to_f32(got_mid).astype(np.float64) - mid) / bound)) <= 1.0
        assert differ <= mid_bits.size // 200, differ
        mid_f = orc.bf16_bits_to_f32(mid_bits)
        exact = orc.spmm_definition(mk2, W2, mid_f)
        den = orc.spmm_definition(mk2, np.abs(W2), np.abs(mid_f))
        err = orc.normalised_error(O2.cpu().numpy(), exact, den)
        print(f"[gpu]   codes that differ {differ} of {mid_bits.size}, final normalised error {err:.2e}", flush=True)
        assert err <= gh.TOL[wl.BF16]
