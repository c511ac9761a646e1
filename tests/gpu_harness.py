"""Shared helpers of the GPU parity tests: run the library through its C ABI on
seeded inputs and compute the oracle's answer for the same bits."""
import numpy as np

from oracle import naive_c
from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl

TOL = {wl.F32: 1e-5, wl.BF16: 1e-2}     # max |err| / sum_k |W||I| per output


def make_mask(w):
    """The library's mask of a workload: four base graphs, or more with their roles."""
    if w.roles:
        return rb.rbgp_make_mask_k(w.rows, w.cols, w.row_deg, w.roles, w.mask_seed)
    return rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)


def host_inputs(w, N=None, vals=None, I=None):
    """(values for the library, I for the library, float32 views for the oracle)."""
    vals = wl.kept_weights(w) if vals is None else vals
    I = wl.activations(w, N) if I is None else I
    if w.dtype == wl.BF16:
        vb, Ib = wl.to_bf16_bits(vals), wl.to_bf16_bits(I)
        return vb, Ib, wl.bf16_bits_as_f32(vb), wl.bf16_bits_as_f32(Ib)
    return vals, I, vals, I


def _output(rows, ld, out_bf16):
    """Device matrix for O filled with NaN (fp32, or bf16 NaN bits for the bf16-output mode)."""
    import torch
    if out_bf16:
        return torch.full((rows, max(ld, 1)), 0x7FC0, dtype=torch.int16, device="cuda:0")
    return torch.full((rows, max(ld, 1)), float("nan"), dtype=torch.float32, device="cuda:0")


def _output_to_host(O_d, out_bf16):
    """fp32 values of O (bf16 bits widened exactly; this is a reinterpretation, not arithmetic)."""
    if out_bf16:
        return wl.bf16_bits_as_f32(O_d.cpu().numpy().view(np.uint16))
    return O_d.cpu().numpy()


def library_spmm(w, vals_lib, I_lib, kernel=rb.KERNEL_AUTO, tune=None, ld_pad=0, tag="", out_bf16=False):
    import torch
    dev = torch.device("cuda:0")
    N = I_lib.shape[1]
    print(f"[gpu] {w.name} N={N} kernel={kernel} tune={tune} ld_pad={ld_pad} {tag}", flush=True)
    mask = make_mask(w)
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
    O_d = _output(w.M, ldO, out_bf16)
    rb.rbgp_spmm(mask, rb.BF16 if out_bf16 else w.dtype, w.M, w.K, N, packed.data_ptr(), I_d.data_ptr(), ldI,
                 O_d.data_ptr(), ldO, stream)
    torch.cuda.synchronize()
    out = _output_to_host(O_d, out_bf16)
    if ld_pad:
        assert np.all(np.isnan(out[:, N:])), "kernel wrote outside the N columns"
    used = rb.rbgp_mask_kernel(mask, w.dtype)
    return out[:, :N], used


def library_conv3x3(w, vals, X, dtype=None, tune=None, tag="", out_bf16=False, kernel=rb.KERNEL_AUTO):
    """Run rbgp_conv3x3 on X[C][B][H][W] (padded here: layout work, not arithmetic)."""
    import torch
    dev = torch.device("cuda:0")
    C, B, H, W = X.shape
    N = B * H * W
    dtype = w.dtype if dtype is None else dtype
    print(f"[gpu] conv3x3 {w.name} C={C} B={B} H={H} W={W} dtype={dtype} tune={tune} kernel={kernel} {tag}", flush=True)
    mask = make_mask(w)
    if kernel != rb.KERNEL_AUTO:
        rb.rbgp_mask_set_kernel(mask, kernel)
    for knob, value in enumerate(tune or ()):
        rb.rbgp_mask_tune(mask, knob, value)
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(max(rb.rbgp_packed_bytes(mask, dtype), 16), dtype=torch.uint8, device=dev)
    rb.rbgp_pack(mask, dtype, np.ascontiguousarray(vals), packed.data_ptr(), stream)
    Xp = wl.zero_padded(X)
    X_d = torch.from_numpy(Xp.view(np.int16) if Xp.dtype == np.uint16 else Xp).to(dev)
    O_d = _output(w.M, N, out_bf16)
    rb.rbgp_conv3x3(mask, rb.BF16 if out_bf16 else dtype, w.M, C, B, H, W, packed.data_ptr(), X_d.data_ptr(),
                    O_d.data_ptr(), N, stream)
    torch.cuda.synchronize()
    return _output_to_host(O_d, out_bf16)


def _to_device(a, ld_pad):
    """Host matrix -> device tensor with `ld_pad` extra columns (NaN / bf16 NaN bits) per row."""
    import torch
    rows, N = a.shape
    if a.dtype == np.uint16:
        host = np.full((rows, N + ld_pad), 0x7FC0, dtype=np.uint16)
        host[:, :N] = a
        return torch.from_numpy(host.view(np.int16)).to("cuda:0")
    host = np.full((rows, N + ld_pad), np.nan, dtype=np.float32)
    host[:, :N] = a
    return torch.from_numpy(host).to("cuda:0")


def library_spmm_transposed(w, vals_lib, dO_lib, kernel=rb.KERNEL_AUTO, tune=None, ld_pad=0, tag=""):
    """dI = W_s^T x dO through rbgp_mask_transpose / rbgp_pack_transposed / rbgp_spmm; vals_lib are
    the kept values in the canonical order of the forward mask."""
    import torch
    N = dO_lib.shape[1]
    print(f"[gpu] transposed {w.name} N={N} kernel={kernel} tune={tune} ld_pad={ld_pad} {tag}", flush=True)
    mask = make_mask(w)
    mask_t = rb.rbgp_mask_transpose(mask)
    if kernel != rb.KERNEL_AUTO:
        rb.rbgp_mask_set_kernel(mask_t, kernel)
    for knob, value in enumerate(tune or ()):
        rb.rbgp_mask_tune(mask_t, knob, value)
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(max(rb.rbgp_packed_bytes(mask_t, w.dtype), 16), dtype=torch.uint8, device="cuda:0")
    rb.rbgp_pack_transposed(mask_t, w.dtype, np.ascontiguousarray(vals_lib), packed.data_ptr(), stream)
    dO_d = _to_device(dO_lib, ld_pad)
    if ld_pad:   # the padding columns are inside the leading dimension and may be read by the bf16 kernels
        dO_d[:, N:] = 0
    ld = N + ld_pad
    dI_d = torch.full((w.K, max(ld, 1)), float("nan"), dtype=torch.float32, device="cuda:0")
    rb.rbgp_spmm(mask_t, w.dtype, w.K, w.M, N, packed.data_ptr(), dO_d.data_ptr(), ld, dI_d.data_ptr(), ld, stream)
    torch.cuda.synchronize()
    out = dI_d.cpu().numpy()
    if ld_pad:
        assert np.all(np.isnan(out[:, N:])), "kernel wrote outside the N columns"
    return out[:, :N], rb.rbgp_mask_kernel(mask_t, w.dtype)


def library_sddmm(w, dO_lib, I_lib, kernel=rb.KERNEL_AUTO, ld_pad=0, calls=1, tag=""):
    """dW[M][rowdeg] = (dO x I^T) on the mask through rbgp_sddmm."""
    import torch
    N = I_lib.shape[1]
    print(f"[gpu] sddmm {w.name} N={N} kernel={kernel} ld_pad={ld_pad} {tag}", flush=True)
    mask = make_mask(w)
    if kernel != rb.KERNEL_AUTO:
        rb.rbgp_mask_set_kernel(mask, kernel)
    stream = torch.cuda.current_stream().cuda_stream
    dO_d, I_d = _to_device(dO_lib, ld_pad), _to_device(I_lib, ld_pad)
    dW_d = torch.full((w.M * w.rowdeg + 64,), float("nan"), dtype=torch.float32, device="cuda:0")
    for _ in range(calls):
        rb.rbgp_sddmm(mask, w.dtype, w.M, w.K, N, dO_d.data_ptr(), N + ld_pad, I_d.data_ptr(), N + ld_pad,
                      dW_d.data_ptr(), stream)
    torch.cuda.synchronize()
    out = dW_d.cpu().numpy()
    assert np.all(np.isnan(out[w.M * w.rowdeg:])), "kernel wrote past the nnz values"
    return out[:w.M * w.rowdeg].reshape(w.M, w.rowdeg)


def library_conv3x3_sddmm(w, dO_lib, X, tag=""):
    """dW through rbgp_conv3x3_sddmm on X[C][B][H][W] (padded here: layout work, not arithmetic)."""
    import torch
    C, B, H, W = X.shape
    N = B * H * W
    print(f"[gpu] conv3x3 sddmm {w.name} C={C} B={B} H={H} W={W} dtype={w.dtype} {tag}", flush=True)
    mask = make_mask(w)
    stream = torch.cuda.current_stream().cuda_stream
    Xp = wl.zero_padded(X)
    X_d = torch.from_numpy(Xp.view(np.int16) if Xp.dtype == np.uint16 else Xp).to("cuda:0")
    dO_d = _to_device(dO_lib, 0)
    dW_d = torch.full((w.M * w.rowdeg + 64,), float("nan"), dtype=torch.float32, device="cuda:0")
    rb.rbgp_conv3x3_sddmm(mask, w.dtype, w.M, C, B, H, W, dO_d.data_ptr(), N, X_d.data_ptr(), dW_d.data_ptr(), stream)
    torch.cuda.synchronize()
    out = dW_d.cpu().numpy()
    assert np.all(np.isnan(out[w.M * w.rowdeg:])), "kernel wrote past the nnz values"
    return out[:w.M * w.rowdeg].reshape(w.M, w.rowdeg)


def library_conv3x3_input_gradient(w, vals_lib, dO_lib, B, H, W, tag="", kernel=rb.KERNEL_AUTO):
    """dX[C][B*H*W] of the fused 3x3 convolution: rbgp_conv3x3 on the mask of the transposed convolution,
    reading dO[M][B][H][W] zero-padded."""
    import torch
    N = B * H * W
    print(f"[gpu] conv3x3 input gradient {w.name} B={B} H={H} W={W} dtype={w.dtype} {tag}", flush=True)
    mask = make_mask(w)
    mx = rb.rbgp_mask_conv3x3_transpose(mask)
    if kernel != rb.KERNEL_AUTO:
        rb.rbgp_mask_set_kernel(mx, kernel)
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(max(rb.rbgp_packed_bytes(mx, w.dtype), 16), dtype=torch.uint8, device="cuda:0")
    rb.rbgp_pack_transposed(mx, w.dtype, np.ascontiguousarray(vals_lib).reshape(-1), packed.data_ptr(), stream)
    dOp = wl.zero_padded(np.ascontiguousarray(dO_lib).reshape(w.M, B, H, W))
    dO_d = torch.from_numpy(dOp.view(np.int16) if dOp.dtype == np.uint16 else dOp).to("cuda:0")
    C = w.K // 9
    dX_d = torch.full((C, N), float("nan"), dtype=torch.float32, device="cuda:0")
    rb.rbgp_conv3x3(mx, w.dtype, C, w.M, B, H, W, packed.data_ptr(), dO_d.data_ptr(), dX_d.data_ptr(), N, stream)
    torch.cuda.synchronize()
    return dX_d.cpu().numpy(), rb.rbgp_mask_kernel(mx, w.dtype)


def oracle_backward(w, vals_f32, I_f32, dO_f32):
    """(dI, its denominators sum_m |W||dO|, dW, its denominators sum_n |dO||I|) from the oracle."""
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    mask = orc.kron_mask(Bs)
    W = orc.scatter_values(mask, vals_f32)
    maskT, WT = np.ascontiguousarray(mask.T), np.ascontiguousarray(W.T)
    dI, dI_den = naive_c.spmm(maskT, WT, dO_f32), naive_c.spmm_abs(maskT, WT, dO_f32)
    dW = orc.sddmm_definition(mask, dO_f32, I_f32)
    dW_den = orc.sddmm_definition(mask, np.abs(dO_f32), np.abs(I_f32))
    return dI, dI_den, dW, dW_den


def backward_inputs(w, N=None):
    """(vals, I, dO for the library; float32 views of the same bits for the oracle)."""
    vals, I, dO = wl.kept_weights(w), wl.activations(w, N), wl.output_gradients(w, N)
    if w.dtype == wl.BF16:
        b = [wl.to_bf16_bits(x) for x in (vals, I, dO)]
        return b, [wl.bf16_bits_as_f32(x) for x in b]
    return [vals, I, dO], [vals, I, dO]


def family_covers(w, kernel):
    """Whether a kernel family accepts this mask (host-side query, no GPU call)."""
    mask = make_mask(w)
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
