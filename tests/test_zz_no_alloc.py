"""rbgp_sddmm_static, the entry point that allocates nothing on the device (its tables and partial sums
live in a fixed array inside the library), against rbgp_sddmm: same results bit for bit, within the
oracle's tolerance, on two calls in a row of which the second is smaller, across a change of mask
(the array's tables are replaced), on the plain kernel and in bf16; free device memory does not move;
problems beyond the array are refused."""
import numpy as np
import pytest

from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu


def _both(w, N, kernel=rb.KERNEL_AUTO, mask_static=None):
    """dW from rbgp_sddmm and from rbgp_sddmm_static (fresh mask objects unless one is given), and the inputs."""
    import torch
    dev = torch.device("cuda:0")
    dO = wl.output_gradients(w, N)
    I = wl.activations(w, N)
    if w.dtype == wl.BF16:
        dO_lib, I_lib = wl.to_bf16_bits(dO), wl.to_bf16_bits(I)
        dO_f, I_f = wl.bf16_bits_as_f32(dO_lib), wl.bf16_bits_as_f32(I_lib)
        as_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev)
    else:
        dO_lib, I_lib, dO_f, I_f = dO, I, dO, I
        as_dev = lambda a: torch.from_numpy(a).to(dev)
    dO_d, I_d = as_dev(dO_lib), as_dev(I_lib)
    stream = torch.cuda.current_stream().cuda_stream
    outs = []
    for static in (False, True):
        mask = mask_static if (static and mask_static is not None) else gh.make_mask(w)
        if kernel != rb.KERNEL_AUTO:
            rb.rbgp_mask_set_kernel(mask, kernel)
        dW = torch.full((w.nnz + 64,), float("nan"), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        fn = rb.rbgp_sddmm_static if static else rb.rbgp_sddmm
        fn(mask, w.dtype, w.M, w.K, N, dO_d.data_ptr(), N, I_d.data_ptr(), N, dW.data_ptr(), stream)
        torch.cuda.synchronize()
        if static:
            assert torch.cuda.mem_get_info()[0] == free0, "the allocation-free call changed the free device memory"
        out = dW.cpu().numpy()
        assert np.all(np.isnan(out[w.nnz:])), "kernel wrote past the nnz values"
        outs.append(out[:w.nnz].reshape(w.M, w.rowdeg))
    return outs[0], outs[1], dO_f, I_f


def _check(w, N, kernel=rb.KERNEL_AUTO, mask_static=None):
    print(f"[gpu] sddmm static vs sddmm {w.name} N={N} kernel={kernel}", flush=True)
    ref_entry, got, dO_f, I_f = _both(w, N, kernel, mask_static)
    assert np.array_equal(ref_entry.view(np.uint32), got.view(np.uint32)), "differs from rbgp_sddmm"
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    dense = orc.kron_mask(Bs)
    ref = orc.sddmm_definition(dense, dO_f, I_f)
    den = orc.sddmm_definition(dense, np.abs(dO_f), np.abs(I_f))
    err = orc.normalised_error(got, ref, den)
    print(f"[gpu]   normalised error {err:.3e}", flush=True)
    assert err <= gh.TOL[w.dtype], err


def test_two_calls_in_a_row_second_smaller():
    """Partial sums in the array (several workgroups per unit), then a smaller call on the same mask
    object: the tables stay, the partial sums of the first call must not leak into the second."""
    w = wl.TINY
    mask = gh.make_mask(w)
    _check(w, 4096, mask_static=mask)
    _check(w, 1536, mask_static=mask)
    _check(w, 64, mask_static=mask)      # one workgroup per unit: straight into dW


def test_change_of_mask_dtype_and_kernel():
    """Another mask replaces the tables; bf16; the plain kernel (its adjacency lists go through the array)."""
    small = wl.Workload("static_rs8", (4, 4, 4, 2), (4, 4, 8, 9), (2, 4, 2, 9), 0, wl.F32, 71, 72, 73, 1.0)
    _check(small, 1000)
    _check(wl.TINY, 2048)
    _check(wl.Workload("static_bf16", (4, 2, 4, 2), (4, 2, 4, 9), (2, 2, 2, 9), 0, wl.BF16, 81, 82, 83, 1.0), 1200)
    _check(wl.TINY, 300, kernel=rb.KERNEL_GENERIC)
    _check(small, 1000)


def test_empty_batch_and_limits():
    import torch
    w = wl.TINY
    mask = gh.make_mask(w)
    dW = torch.full((w.nnz,), 5.0, dtype=torch.float32, device="cuda:0")
    rb.rbgp_sddmm_static(mask, w.dtype, w.M, w.K, 0, 0, 0, 0, 0, dW.data_ptr(), 0)
    torch.cuda.synchronize()
    assert bool((dW == 0).all())         # N == 0 stores zeros, as rbgp_sddmm does
    # adjacency lists of 512 KiB do not fit the 256 KiB of tables
    big = rb.rbgp_make_mask((4096, 1, 1, 1), (4096, 1, 1, 1), (32, 1, 1, 1), 5)
    rb.rbgp_mask_set_kernel(big, rb.KERNEL_GENERIC)
    x = torch.zeros((4096, 64), dtype=torch.float32, device="cuda:0")
    out = torch.zeros((4096 * 32,), dtype=torch.float32, device="cuda:0")
    with pytest.raises(rb.RbgpError) as e:
        rb.rbgp_sddmm_static(big, wl.F32, 4096, 4096, 64, x.data_ptr(), 64, x.data_ptr(), 64, out.data_ptr(), 0)
    assert e.value.code == rb.ETOOLARGE
    with pytest.raises(rb.RbgpError) as e:
        rb.rbgp_sddmm_static(mask, w.dtype, w.M + 1, w.K, 64, x.data_ptr(), 64, x.data_ptr(), 64, out.data_ptr(), 0)
    assert e.value.code == rb.ESHAPE
