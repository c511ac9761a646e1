"""Shared helpers of the GPU parity tests: run the library through its C ABI on
seeded inputs and compute the oracle's answer for the same bits."""
import numpy as np

from oracle import naive_c
from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl

TOL = {wl.F32: 1e-5, wl.BF16: 1e-2}     # max |err| / sum_k |W||I| per output


def host_inputs(w, N=None, vals=None, I=None):
    """(values for the library, I for the library, float32 views for the oracle)."""
    vals = wl.kept_weights(w) if vals is None else vals
    I = wl.activations(w, N) if I is None else I
    if w.dtype == wl.BF16:
        vb, Ib = wl.to_bf16_bits(vals), wl.to_bf16_bits(I)
        return vb, Ib, wl.bf16_bits_as_f32(vb), wl.bf16_bits_as_f32(Ib)
    return vals, I, vals, I


def library_spmm(w, vals_lib, I_lib, kernel=rb.KERNEL_AUTO, tune=None, ld_pad=0, tag=""):
    import torch
    dev = torch.device("cuda:0")
    N = I_lib.shape[1]
    print(f"[gpu] {w.name} N={N} kernel={kernel} tune={tune} ld_pad={ld_pad} {tag}", flush=True)
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    if kernel != rb.KERNEL_AUTO:
        rb.rbgp_mask_set_kernel(mask, kernel)
    for knob, value in enumerate(tune or ()):
        rb.rbgp_mask_tune(mask, knob, value)
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(max(rb.rbgp_packed_bytes(mask, w.dtype), 16), dtype=torch.uint8, device=dev)
    rb.rbgp_pack(mask, w.dtype, np.ascontiguousarray(vals_lib), packed.data_ptr(), stream)
    ldI = N + ld_pad
    tdt = torch.float32 if w.dtype == wl.F32 else torch.int16
    I_host = np.zeros((w.K, ldI), dtype=I_lib.dtype)
    I_host[:, :N] = I_lib
    I_d = torch.from_numpy(I_host.view(np.int16) if w.dtype == wl.BF16 else I_host).to(dev)
    assert I_d.dtype == tdt
    ldO = N + ld_pad
    O_d = torch.full((w.M, max(ldO, 1)), float("nan"), dtype=torch.float32, device=dev)
    rb.rbgp_spmm(mask, w.dtype, w.M, w.K, N, packed.data_ptr(), I_d.data_ptr(), ldI, O_d.data_ptr(), ldO, stream)
    torch.cuda.synchronize()
    out = O_d.cpu().numpy()
    if ld_pad:
        assert np.all(np.isnan(out[:, N:])), "kernel wrote outside the N columns"
    used = rb.rbgp_mask_kernel(mask, w.dtype)
    return out[:, :N], used


def library_conv3x3(w, vals, X, dtype=None, tune=None, tag=""):
    """Run rbgp_conv3x3 on X[C][B][H][W] (padded here: layout work, not arithmetic)."""
    import torch
    dev = torch.device("cuda:0")
    C, B, H, W = X.shape
    N = B * H * W
    dtype = w.dtype if dtype is None else dtype
    print(f"[gpu] conv3x3 {w.name} C={C} B={B} H={H} W={W} dtype={dtype} tune={tune} {tag}", flush=True)
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    for knob, value in enumerate(tune or ()):
        rb.rbgp_mask_tune(mask, knob, value)
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(max(rb.rbgp_packed_bytes(mask, dtype), 16), dtype=torch.uint8, device=dev)
    rb.rbgp_pack(mask, dtype, np.ascontiguousarray(vals), packed.data_ptr(), stream)
    Xp = wl.zero_padded(X)
    X_d = torch.from_numpy(Xp.view(np.int16) if Xp.dtype == np.uint16 else Xp).to(dev)
    O_d = torch.full((w.M, N), float("nan"), dtype=torch.float32, device=dev)
    rb.rbgp_conv3x3(mask, dtype, w.M, C, B, H, W, packed.data_ptr(), X_d.data_ptr(), O_d.data_ptr(), N, stream)
    torch.cuda.synchronize()
    return O_d.cpu().numpy()


def family_covers(w, kernel):
    """Whether a kernel family accepts this mask (host-side query, no GPU call)."""
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    try:
        rb.rbgp_mask_set_kernel(mask, kernel)
    except rb.RbgpError:
        return False
    return rb.rbgp_mask_kernel(mask, w.dtype) == kernel


def oracle_spmm(w, vals_f32, I_f32):
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    mask = orc.kron_mask(Bs)
    W = orc.scatter_values(mask, vals_f32)
    return naive_c.spmm(mask, W, I_f32), naive_c.spmm_abs(mask, W, I_f32)


def check_parity(w, N=None, kernel=rb.KERNEL_AUTO, tune=None, ld_pad=0, expect_kernel=None):
    vl, Il, vf, If = host_inputs(w, N)
    out, used = library_spmm(w, vl, Il, kernel, tune, ld_pad)
    if expect_kernel is not None:
        assert used == expect_kernel
    ref, den = oracle_spmm(w, vf, If)
    err = orc.normalised_error(out, ref, den)
    print(f"[gpu]   normalised error {err:.3e}", flush=True)
    assert err <= TOL[w.dtype], err
    return err
