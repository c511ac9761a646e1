#!/usr/bin/env python3
"""Benchmark of the RBGP4 sparse x dense product on one MI355X.

One "step" is one pass of the whole hot path (tile walk, W and I staging, inner
walk, dense-block MACs, epilogue = one rbgp_spmm call) over one batch of
synthetic input that is already resident in HBM.  Steps rotate over several
distinct (I, O) buffer sets so that the working set exceeds the 256 MB
Infinity Cache and the rate is not a cache-resident one (`--sets 1` gives the
hot-cache rate).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
from dataclasses import replace
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2006_13486_amd import binding as rb      # noqa: E402
from paper_2006_13486_amd import workloads as wl    # noqa: E402

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/),
# scaled by what the same counters read for a 64 MiB copy (FETCH_SIZE x2.0, WRITE_SIZE x1.0)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
PEAK_F32_TFLOPS = 157.3      # MI355X dense fp32 matrix (= packed vector) peak
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
WORKLOADS = {"conv5": wl.VGG19_CONV5, "conv3": wl.VGG19_CONV3_BF16, "wrn": wl.WRN_G1, "tiny": wl.TINY,
             # two of the paper's own 4096^3 products: Table 3's first row (one row per column set, 75 % sparse) and
             # Table 2's (87.5 %, 50 %) cell at 93.75 %
             "sdmm_r1": wl.sdmm4096_table3(1, 1, 2), "sdmm_o8": wl.sdmm4096_table2(3, 1),
             # Table 3's first row at 93.75 % (runs on the mask with G_o filled in) and Table 2's cell with a complete G_o
             "sdmm_r1_d16": wl.sdmm4096_table3(1, 1, 4), "sdmm_o1": wl.sdmm4096_table2(0, 4)}
# which roofline bounds each workload (arithmetic intensity vs the fp32 / bf16 ridge)
BOUND = {"conv5": "mfma", "conv3": "hbm", "wrn": "hbm", "tiny": "hbm", "sdmm_r1": "mfma", "sdmm_o8": "mfma",
         "sdmm_r1_d16": "mfma", "sdmm_o1": "mfma"}


def cpu_baseline(w, vals_f32, I_f32, out_gpu):
    """Time the oracle's naive masked triple loop on the host cores and use its
    result to check the GPU output of the same inputs."""
    from oracle import naive_c
    from oracle import rbgp_oracle as orc
    Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
    mask = orc.kron_mask(Bs)
    W = orc.scatter_values(mask, vals_f32)
    # bounded sample: at most ~2^31 multiply-adds, taken as the leading columns of I
    ncols = int(min(w.N, max(64, (1 << 31) // max(w.nnz, 1))))
    Is = np.ascontiguousarray(I_f32[:, :ncols])
    naive_c.spmm(mask, W, Is[:, :64])       # warm-up (threads, page faults)
    best = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        ref = naive_c.spmm(mask, W, Is)
        best = min(best, time.perf_counter() - t0)
    den = naive_c.spmm_abs(mask, W, Is)
    err = orc.normalised_error(out_gpu[:, :ncols], ref, den)
    return {"value": 2.0 * w.nnz * ncols / best / 1e12, "unit": "TFLOP/s", "cores": naive_c.threads(),
            "kind": "oracle", "sample": f"first {ncols} of {w.N} columns, best of 3, {best * 1e3:.1f} ms",
            "parity_err": err}


def time_workload(w, args, torch, dev, steps, warmup, check_cols=0, geom=None):
    """Pack, run and time one workload; returns a dict (kernel time, rates, optional sampled parity).
    geom = (images, height, width): run the layer through rbgp_conv3x3 instead of rbgp_spmm."""
    bf16 = w.dtype == wl.BF16
    vals = wl.kept_weights(w)
    if geom:
        X = wl.conv_activations(w, *geom)
        if bf16:
            Xbits = wl.to_bf16_bits(X)
            X = wl.bf16_bits_as_f32(Xbits)
            I_lib = wl.zero_padded(Xbits)
        else:
            I_lib = wl.zero_padded(X)
        I_f32 = None
    else:
        I = wl.activations(w)
    if bf16:
        vals_lib = wl.to_bf16_bits(vals)
        vals_f32 = wl.bf16_bits_as_f32(vals_lib)
        if not geom:
            I_lib = wl.to_bf16_bits(I)
            I_f32 = wl.bf16_bits_as_f32(I_lib)
    else:
        vals_lib, vals_f32 = vals, vals
        if not geom:
            I_lib, I_f32 = I, I
    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    if args.kernel != rb.KERNEL_AUTO:
        rb.rbgp_mask_set_kernel(mask, args.kernel)
    if args.tune:
        for knob, value in enumerate(int(x) for x in args.tune.split(",")):
            rb.rbgp_mask_tune(mask, knob, value)
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(max(rb.rbgp_packed_bytes(mask, w.dtype), 16), dtype=torch.uint8, device=dev)
    rb.rbgp_pack(mask, w.dtype, np.ascontiguousarray(vals_lib), packed.data_ptr(), stream)
    set_bytes = I_lib.nbytes + w.M * w.N * 4
    nsets = max(2, min(16, -(-512 * 2**20 // set_bytes)))
    I0 = torch.from_numpy(I_lib.view(np.int16) if bf16 else I_lib).to(dev)
    Is = [I0] + [I0.clone() for _ in range(nsets - 1)]
    Os = [torch.empty((w.M, w.N), dtype=torch.float32, device=dev) for _ in range(nsets)]
    algorithmic_bytes = I_lib.nbytes + w.M * w.N * 4 + w.nnz * w.in_bytes

    def step(i):
        j = i % nsets
        if geom:
            rb.rbgp_conv3x3(mask, w.dtype, w.M, w.K // 9, geom[0], geom[1], geom[2], packed.data_ptr(),
                            Is[j].data_ptr(), Os[j].data_ptr(), w.N, stream)
        else:
            rb.rbgp_spmm(mask, w.dtype, w.M, w.K, w.N, packed.data_ptr(), Is[j].data_ptr(), w.N,
                         Os[j].data_ptr(), w.N, stream)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for i in range(steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) / steps * 1e3
    res = {"name": w.name, "M": w.M, "K": w.K, "N": w.N, "density": w.density,
           "dtype": "bf16" if bf16 else "f32",
           "rows": list(w.rows), "cols": list(w.cols), "row_deg": list(w.row_deg),
           "kernel": rb.rbgp_mask_kernel(mask, w.dtype), "kernel_us": us,
           "entry_point": "rbgp_conv3x3" if geom else "rbgp_spmm",
           "eff_tflops": w.flops / us / 1e6, "algorithmic_gbs": algorithmic_bytes / us / 1e3}
    if check_cols:
        from oracle import naive_c
        from oracle import rbgp_oracle as orc
        Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
        dense_mask = orc.kron_mask(Bs)
        W = orc.scatter_values(dense_mask, vals_f32)
        g = np.random.Generator(np.random.PCG64(w.i_seed + 7))
        cols = np.sort(g.choice(w.N, size=min(check_cols, w.N), replace=False))
        Isub = np.ascontiguousarray((orc.im2col_3x3(X) if geom else I_f32)[:, cols])
        ref, den = naive_c.spmm(dense_mask, W, Isub), naive_c.spmm_abs(dense_mask, W, Isub)
        res["parity_err"] = orc.normalised_error(Os[0].cpu().numpy()[:, cols], ref, den)
        res["parity_cols"] = int(len(cols))
    if getattr(args, "sweep_backward", False) and not geom:
        del Is, Os
        torch.cuda.empty_cache()
        res["backward"] = backward_objects(w, mask, vals_lib, vals_f32, I_lib, I_f32, torch, dev, stream,
                                           check=bool(check_cols), steps=steps, warmup=warmup,
                                           geom=getattr(args, "layer_geom", {}).get(w.name), light_check=True)
    return res


def sweep_cases(which, args):
    """The paper's own SDMM workloads (Tables 2 and 3) and the VGG19 layer sweep."""
    tables = which in ("table2", "table3")   # (the paper's tables are fp32: their default; the VGG19 sweep runs both)
    dts = {"f32": [wl.F32], "bf16": [wl.BF16], "both": [wl.F32, wl.BF16]}[args.sweep_dtype or ("f32" if tables else "both")]
    if tables:
        if which == "table2":           # (sparsity of G_o, sparsity of G_i) as log2 of the inverse density
            splits = [(0, 2), (1, 1), (0, 3), (1, 2), (2, 1), (0, 4), (1, 3), (2, 2), (3, 1)]
            ws = [wl.sdmm4096_table2(o, i) for o, i in splits]
        else:
            shapes = [(1, 1), (2, 1), (4, 1), (1, 2), (1, 4), (2, 2)]
            ws = [wl.sdmm4096_table3(gr, gb, d) for gr, gb in shapes for d in (2, 3, 4)]
        return [w if dt == wl.F32 else replace(w, name=w.name + "_bf16", dtype=dt) for dt in dts for w in ws]
    dens = [int(x) for x in args.sweep_density.split(",")]
    cases = []
    for dt in dts:
        for d in dens:
            for layer in range(len(wl.VGG19_LAYERS)):
                w = wl.vgg19_sweep_workload(layer, d, dt)
                h = wl.VGG19_LAYERS[layer][2]
                # --fused-conv: layers whose image rows hold whole lane loads go through rbgp_conv3x3
                fused = args.fused_conv and layer > 0 and h % 4 == 0
                if layer > 0 and h % 4 == 0:   # (--sweep-backward: the fused gradients need the layer's geometry)
                    args.layer_geom = dict(getattr(args, "layer_geom", {}), **{w.name: (w.N // (h * h), h, h)})
                cases.append((w, (w.N // (h * h), h, h)) if fused else w)
    return cases


def run_sweep(args, torch, dev):
    cases = []
    for case in sweep_cases(args.sweep, args):
        w, geom = case if isinstance(case, tuple) else (case, None)
        try:
            r = time_workload(w, args, torch, dev, args.sweep_steps, args.sweep_steps, args.sweep_check, geom)
        except rb.RbgpError as e:   # a cell whose factors cannot be sampled (recorded, not hidden)
            r = {"name": w.name, "error": str(e)}
        print(f"[sweep] {r}", file=sys.stderr, flush=True)
        cases.append(r)
        torch.cuda.empty_cache()
    print(json.dumps({"sweep": args.sweep, "unit": "us per rbgp_spmm launch (HIP events), effective TFLOP/s = 2*nnz*N/t",
                      "steps": args.sweep_steps, "data": "synthetic", "cases": cases}))


def sweep_sums(torch, dev, steps=200, warmup=300):
    """All 16 VGG19 conv layers at the four densities, fp32 and bf16, through rbgp_spmm with library defaults:
    per (dtype, density) the sum of the per-layer launch times.  Inputs are generated on the device (seeded,
    ReLU(N(0,1)) as everywhere); the outputs of these cells are checked in the GPU tests, not here."""
    sums, stream = {}, torch.cuda.current_stream().cuda_stream
    gen = torch.Generator(device=dev)
    for layer in range(len(wl.VGG19_LAYERS)):
        w0 = wl.vgg19_sweep_workload(layer, 1, wl.F32)
        gen.manual_seed(w0.i_seed)
        I32 = torch.randn((w0.K, w0.N), generator=gen, device=dev).clamp_(min=0)
        I16 = I32.to(torch.bfloat16).view(torch.int16)
        for dt, I0 in ((wl.F32, I32), (wl.BF16, I16)):
            nsets = max(2, min(16, -(-512 * 2**20 // (I0.numel() * I0.element_size() + w0.M * w0.N * 4))))
            Is = [I0] + [I0.clone() for _ in range(nsets - 1)]
            Os = [torch.empty((w0.M, w0.N), dtype=torch.float32, device=dev) for _ in range(nsets)]
            for d in (1, 2, 3, 4):
                w = wl.vgg19_sweep_workload(layer, d, dt)
                key = f"{'bf16' if dt == wl.BF16 else 'f32'}_d{1 << d}"
                try:
                    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
                    vals = wl.kept_weights(w)
                    vals = wl.to_bf16_bits(vals) if dt == wl.BF16 else vals
                    packed = torch.zeros(max(rb.rbgp_packed_bytes(mask, w.dtype), 16), dtype=torch.uint8, device=dev)
                    rb.rbgp_pack(mask, w.dtype, np.ascontiguousarray(vals), packed.data_ptr(), stream)
                    for i in range(warmup):
                        rb.rbgp_spmm(mask, w.dtype, w.M, w.K, w.N, packed.data_ptr(), Is[i % nsets].data_ptr(), w.N,
                                     Os[i % nsets].data_ptr(), w.N, stream)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for i in range(steps):
                        rb.rbgp_spmm(mask, w.dtype, w.M, w.K, w.N, packed.data_ptr(), Is[i % nsets].data_ptr(), w.N,
                                     Os[i % nsets].data_ptr(), w.N, stream)
                    e1.record()
                    torch.cuda.synchronize()
                    sums[key] = sums.get(key, 0.0) + e0.elapsed_time(e1) / steps * 1e3
                except rb.RbgpError as e:
                    sums[key + "_errors"] = sums.get(key + "_errors", 0) + 1
            del Is, Os
        del I32, I16
        torch.cuda.empty_cache()
    return {"unit": "us, sum over the 16 VGG19 conv layers of one rbgp_spmm launch each (layer 0 dense)",
            "steps_per_layer": steps, "sum_us": {k: round(v, 1) for k, v in sorted(sums.items())}}


def fused_conv_line(w, mask, packed, vals_f32, torch, dev, stream, check, steps=2000, warmup=1000):
    """The same layer through rbgp_conv3x3 (lowering folded into the loads; the K x N input is never
    stored): reported beside the headline number, which stays the product with I resident in HBM."""
    B, H, W = wl.CONV_GEOMETRY[w.name]
    X = wl.conv_activations(w, B, H, W)
    bf16 = w.dtype == wl.BF16
    if bf16:                              # both sides consume the same bf16 bits
        Xbits = wl.to_bf16_bits(X)
        X = wl.bf16_bits_as_f32(Xbits)
        Xp = wl.zero_padded(Xbits).view(np.int16)
    else:
        Xp = wl.zero_padded(X)
    set_bytes = Xp.nbytes + w.M * w.N * 4
    nsets = max(2, min(16, -(-512 * 2**20 // set_bytes)))
    Xs = [torch.from_numpy(Xp).to(dev) for _ in range(nsets)]
    Os = [torch.empty((w.M, w.N), dtype=torch.float32, device=dev) for _ in range(nsets)]

    def step(i):
        j = i % nsets
        rb.rbgp_conv3x3(mask, w.dtype, w.M, w.K // 9, B, H, W, packed.data_ptr(), Xs[j].data_ptr(),
                        Os[j].data_ptr(), w.N, stream)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for i in range(steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    kern_ms = ev0.elapsed_time(ev1) / steps
    abytes = Xp.nbytes + w.M * w.N * 4 + w.nnz * w.in_bytes
    tf = w.flops / (kern_ms * 1e-3) / 1e12
    res = {"entry_point": "rbgp_conv3x3", "images": B, "height": H, "width": W, "kernel_ms": kern_ms,
           "value": tf, "unit": "TFLOP/s", "frac_of_fp32_mfma_peak": tf / PEAK_F32_TFLOPS,
           "algorithmic_bytes": abytes, "algorithmic_gbs": abytes / (kern_ms * 1e-3) / 1e9,
           "buffer_sets": nsets, "steps": steps}
    if check:
        from oracle import naive_c
        from oracle import rbgp_oracle as orc
        Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
        dense_mask = orc.kron_mask(Bs)
        Wd = orc.scatter_values(dense_mask, vals_f32)
        ncols = int(min(w.N, max(64, (1 << 31) // max(w.nnz, 1))))
        Isub = np.ascontiguousarray(orc.im2col_3x3(X)[:, :ncols])
        ref, den = naive_c.spmm(dense_mask, Wd, Isub), naive_c.spmm_abs(dense_mask, Wd, Isub)
        res["parity_err"] = orc.normalised_error(Os[0].cpu().numpy()[:, :ncols], ref, den)
    return res


def backward_objects(w, mask, vals_lib, vals_f32, I_lib, I_f32, torch, dev, stream, check, steps=1000, warmup=300,
                     only=None, geom=None, light_check=False):
    """The two gradients of the product for a fixed mask (Section 6), timed on the same workload:
    dI = W_s^T x dO (rbgp_spmm on the transposed mask) and dW = (dO x I^T) on the mask (rbgp_sddmm).
    Reported beside the headline number; same flop count 2 * nnz * N each."""
    bf16 = w.dtype == wl.BF16
    dO = wl.output_gradients(w)
    if bf16:
        dO_lib = wl.to_bf16_bits(dO)
        dO_f32 = wl.bf16_bits_as_f32(dO_lib)
    else:
        dO_lib = dO_f32 = dO
    mask_t = rb.rbgp_mask_transpose(mask)
    packed_t = torch.zeros(rb.rbgp_packed_bytes(mask_t, w.dtype), dtype=torch.uint8, device=dev)
    rb.rbgp_pack_transposed(mask_t, w.dtype, np.ascontiguousarray(vals_lib), packed_t.data_ptr(), stream)
    set_bytes = (w.M + w.K) * w.N * (w.in_bytes + 4)
    nsets = max(2, min(16, -(-512 * 2**20 // set_bytes)))
    as_dev = lambda a: torch.from_numpy(a.view(np.int16) if bf16 else a).to(dev)
    dOs = [as_dev(dO_lib) for _ in range(nsets)]
    Is = [as_dev(I_lib) for _ in range(nsets)]
    dIs = [torch.empty((w.K, w.N), dtype=torch.float32, device=dev) for _ in range(nsets)]
    dWs = [torch.empty(w.nnz, dtype=torch.float32, device=dev) for _ in range(nsets)]

    def data_step(i):
        j = i % nsets
        rb.rbgp_spmm(mask_t, w.dtype, w.K, w.M, w.N, packed_t.data_ptr(), dOs[j].data_ptr(), w.N,
                     dIs[j].data_ptr(), w.N, stream)

    def weight_step(i):
        j = i % nsets
        rb.rbgp_sddmm(mask, w.dtype, w.M, w.K, w.N, dOs[j].data_ptr(), w.N, Is[j].data_ptr(), w.N,
                      dWs[j].data_ptr(), stream)

    steps_list = [("backward_data", data_step, w.M * w.N * w.in_bytes + w.K * w.N * 4 + w.nnz * w.in_bytes),
                  ("weight_gradient", weight_step, (w.M + w.K) * w.N * w.in_bytes + w.nnz * 4)]
    geom = geom or wl.CONV_GEOMETRY.get(w.name)
    if geom:
        B, H, W = geom
    if geom and (not bf16 or geom[2] % 8 == 0):
        # the same gradient from the activations themselves (the lowered input is never stored)
        X = wl.conv_activations(w, B, H, W)
        Xbits = wl.to_bf16_bits(X) if bf16 else None
        X_f32 = wl.bf16_bits_as_f32(Xbits) if bf16 else X
        Xp = wl.zero_padded(Xbits).view(np.int16) if bf16 else wl.zero_padded(X)
        Xs = [torch.from_numpy(Xp).to(dev) for _ in range(nsets)]

        def fused_step(i):
            j = i % nsets
            rb.rbgp_conv3x3_sddmm(mask, w.dtype, w.M, w.K // 9, B, H, W, dOs[j].data_ptr(), w.N, Xs[j].data_ptr(),
                                  dWs[j].data_ptr(), stream)
        steps_list.append(("weight_gradient_fused_conv3x3", fused_step,
                           w.M * w.N * w.in_bytes + Xp.nbytes + w.nnz * 4))
    if geom:
        # dX: the transposed convolution of dO through rbgp_conv3x3 (the lowered gradient is never stored)
        mask_x = rb.rbgp_mask_conv3x3_transpose(mask)
        packed_x = torch.zeros(rb.rbgp_packed_bytes(mask_x, w.dtype), dtype=torch.uint8, device=dev)
        rb.rbgp_pack_transposed(mask_x, w.dtype, np.ascontiguousarray(vals_lib), packed_x.data_ptr(), stream)
        dOp = wl.zero_padded(np.ascontiguousarray(dO_lib).reshape(w.M, B, H, W))
        dOps = [torch.from_numpy(dOp.view(np.int16) if bf16 else dOp).to(dev) for _ in range(nsets)]
        dXs = [torch.empty((w.K // 9, w.N), dtype=torch.float32, device=dev) for _ in range(nsets)]

        def input_step(i):
            j = i % nsets
            rb.rbgp_conv3x3(mask_x, w.dtype, w.K // 9, w.M, B, H, W, packed_x.data_ptr(), dOps[j].data_ptr(),
                            dXs[j].data_ptr(), w.N, stream)
        steps_list.append(("input_gradient_fused_conv3x3", input_step,
                           dOp.nbytes + (w.K // 9) * w.N * 4 + w.nnz * w.in_bytes))
        # the same on the tile family, where it covers the mask of the transposed convolution (bf16, 32 rows per tile)
        dXts = None
        if bf16 and W % 8 == 0:
            mask_xt = rb.rbgp_mask_conv3x3_transpose(mask)
            try:
                rb.rbgp_mask_set_kernel(mask_xt, rb.KERNEL_MFMA_TILE)
            except rb.RbgpError:
                mask_xt = None
            if mask_xt is not None:
                packed_xt = torch.zeros(rb.rbgp_packed_bytes(mask_xt, w.dtype), dtype=torch.uint8, device=dev)
                rb.rbgp_pack_transposed(mask_xt, w.dtype, np.ascontiguousarray(vals_lib), packed_xt.data_ptr(), stream)
                dXts = [torch.empty((w.K // 9, w.N), dtype=torch.float32, device=dev) for _ in range(nsets)]

                def input_step_tile(i):
                    j = i % nsets
                    rb.rbgp_conv3x3(mask_xt, w.dtype, w.K // 9, w.M, B, H, W, packed_xt.data_ptr(), dOps[j].data_ptr(),
                                    dXts[j].data_ptr(), w.N, stream)
                steps_list.append(("input_gradient_fused_conv3x3_tile", input_step_tile,
                                   dOp.nbytes + (w.K // 9) * w.N * 4 + w.nnz * w.in_bytes))
    out = {}
    for name, step, abytes in steps_list:
        if only and name != only and not (only == "weight_gradient" and name.startswith("weight_gradient")) \
                and not (only == "backward_data" and name.startswith("input_gradient")):
            continue
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for i in range(steps):
            step(i)
        ev1.record()
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1) / steps
        tf = w.flops / (ms * 1e-3) / 1e12
        out[name] = {"entry_point": {"backward_data": "rbgp_spmm on rbgp_mask_transpose", "weight_gradient": "rbgp_sddmm",
                                     "weight_gradient_fused_conv3x3": "rbgp_conv3x3_sddmm",
                                     "input_gradient_fused_conv3x3": "rbgp_conv3x3 on rbgp_mask_conv3x3_transpose",
                                     "input_gradient_fused_conv3x3_tile":
                                         "rbgp_conv3x3 on rbgp_mask_conv3x3_transpose, RBGP_KERNEL_MFMA_TILE"}[name],
                     "ms": ms, "value": tf, "unit": "TFLOP/s", "frac_of_fp32_mfma_peak": tf / PEAK_F32_TFLOPS,
                     "algorithmic_bytes": abytes, "algorithmic_gbs": abytes / (ms * 1e-3) / 1e9,
                     "frac_of_hbm_peak": abytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "steps": steps, "buffer_sets": nsets}
    if check:
        from oracle import naive_c
        from oracle import rbgp_oracle as orc
        Bs, _ = orc.sample_factors(w.rows, w.cols, w.row_deg, w.mask_seed)
        dense_mask = orc.kron_mask(Bs)
        Wd = orc.scatter_values(dense_mask, vals_f32)
        if "backward_data" in out:       # sampled columns of dI
            ncols = int(min(w.N, 32 if light_check else max(64, (1 << 31) // max(w.nnz, 1))))
            mT, WT = np.ascontiguousarray(dense_mask.T), np.ascontiguousarray(Wd.T)
            sub = np.ascontiguousarray(dO_f32[:, :ncols])
            ref, den = naive_c.spmm(mT, WT, sub), naive_c.spmm_abs(mT, WT, sub)
            out["backward_data"]["parity_err"] = orc.normalised_error(dIs[0].cpu().numpy()[:, :ncols], ref, den)
        if "input_gradient_fused_conv3x3" in out:      # dX: col2im of the oracle's W^T dO (light: first two images)
            mT, WT = np.ascontiguousarray(dense_mask.T), np.ascontiguousarray(Wd.T)
            Bq, Hq, Wq = geom
            Bc = min(Bq, 2) if light_check else Bq
            sub = np.ascontiguousarray(dO_f32[:, :Bc * Hq * Wq])
            ref = orc.col2im_3x3(naive_c.spmm(mT, WT, sub), Bc, Hq, Wq).reshape(w.K // 9, -1)
            den = orc.col2im_3x3(naive_c.spmm_abs(mT, WT, sub), Bc, Hq, Wq).reshape(w.K // 9, -1)
            out["input_gradient_fused_conv3x3"]["parity_err"] = orc.normalised_error(
                dXs[0].cpu().numpy()[:, :Bc * Hq * Wq], ref, den)
            if "input_gradient_fused_conv3x3_tile" in out:
                out["input_gradient_fused_conv3x3_tile"]["parity_err"] = orc.normalised_error(
                    dXts[0].cpu().numpy()[:, :Bc * Hq * Wq], ref, den)
        # sampled rows of dW (each needs the whole batch)
        rows = np.unique(np.linspace(0, w.M - 1, 8 if light_check else 48).astype(np.int64))
        if "weight_gradient_fused_conv3x3" in out:     # (timed last: dWs hold its result)
            I_x = orc.im2col_3x3(X_f32)
            ref = orc.sddmm_definition(dense_mask[rows], dO_f32[rows], I_x)
            den = orc.sddmm_definition(dense_mask[rows], np.abs(dO_f32[rows]), np.abs(I_x))
            got = dWs[0].cpu().numpy().reshape(w.M, w.rowdeg)[rows]
            out["weight_gradient_fused_conv3x3"]["parity_err"] = orc.normalised_error(got, ref, den)
        if "weight_gradient" in out:
            weight_step(0)
            torch.cuda.synchronize()
            ref = orc.sddmm_definition(dense_mask[rows], dO_f32[rows], I_f32)
            den = orc.sddmm_definition(dense_mask[rows], np.abs(dO_f32[rows]), np.abs(I_f32))
            got = dWs[0].cpu().numpy().reshape(w.M, w.rowdeg)[rows]
            out["weight_gradient"]["parity_err"] = orc.normalised_error(got, ref, den)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=1000, help="untimed steps before the timed ones")
    ap.add_argument("--settle", type=int, default=1000,
                    help="untimed set-up launches of the same call before the warm-up steps (clock settling; 0: none)")
    ap.add_argument("--workload", default="conv5", choices=sorted(WORKLOADS))
    ap.add_argument("--sets", type=int, default=0, help="distinct (I,O) buffer sets to rotate over (0 = auto)")
    ap.add_argument("--tune", default="", help="values of the RBGP_TUNE_* knobs in their order in include/rbgp.h (0 = default): cols_per_lane,"
                         "cols_per_workgroup,groups_per_workgroup,row_pairing,row_groups,k_split")
    ap.add_argument("--kernel", type=int, default=rb.KERNEL_AUTO)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cache-resident", action="store_true",
                    help="skip the extra leg that times the same call on one buffer set (for profiles: the kernel trace of the "
                         "run then holds launches with I in HBM only)")
    ap.add_argument("--no-sweep-sums", action="store_true",
                    help="leave the summed VGG19 layer times (16 layers x 4 densities x 2 dtypes) out of the line")
    ap.add_argument("--ld-pad", type=int, default=0,
                    help="extra elements in the leading dimension of I and O (rbgp_spmm only): a row stride that is "
                         "not a multiple of 4 KiB spreads the rows of a stage over more memory channels")
    ap.add_argument("--fused-conv", action="store_true",
                    help="time rbgp_conv3x3 (3x3 convolution with the lowering folded into the loads, fp32) on the "
                         "workload's layer instead of rbgp_spmm on the lowered input")
    ap.add_argument("--forward-only", action="store_true",
                    help="time the forward product only: no fused-convolution and backward objects in the JSON line "
                         "(keeps a profile of the run to the one kernel)")
    ap.add_argument("--out-bf16", action="store_true",
                    help="bf16 workloads: store O as bf16 (dtype RBGP_BF16) instead of fp32")
    ap.add_argument("--backward", default="", choices=["", "backward_data", "weight_gradient", "both"],
                    help="time the backward products of the workload (dI = W^T dO, dW = dO I^T on the mask) "
                         "instead of the forward product; prints one JSON line with them")
    ap.add_argument("--sweep", default="", choices=["", "table2", "table3", "vgg19"],
                    help="time a family of workloads instead of the headline one: the paper's 4096^3 SDMM of "
                         "Table 2 / Table 3, or the 16 VGG19 conv layers; prints one JSON line with all cases")
    ap.add_argument("--sweep-backward", action="store_true",
                    help="sweeps: also time the backward products of every case (dI, dW, and for 3x3 layers the fused dX, dW)")
    ap.add_argument("--sweep-steps", type=int, default=300)
    ap.add_argument("--sweep-check", type=int, default=32, help="output columns per case checked against the oracle (0: none)")
    ap.add_argument("--sweep-density", default="2,3", help="vgg19 sweep: log2 of the inverse densities")
    ap.add_argument("--sweep-dtype", default=None, choices=["f32", "bf16", "both"],
                    help="default: both for the VGG19 sweep, f32 for the tables")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run ten 64 MiB device-to-device copies and exit (reference for the FETCH_SIZE / "
                         "WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (columns of I and O are independent: shard N across devices); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        a = torch.empty(64 * 2**20 // 4, device=dev, dtype=torch.float32).normal_()
        b = torch.empty_like(a)
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": a.numel() * 4, "copies": 10}))
        return
    if args.sweep:
        run_sweep(args, torch, dev)
        return
    w = WORKLOADS[args.workload]
    bf16 = w.dtype == wl.BF16
    if args.out_bf16 and not bf16:
        sys.exit("bench.py: --out-bf16 needs a bf16 workload (conv3)")
    call_dtype = rb.BF16 if args.out_bf16 else w.dtype
    out_bytes = 2 if args.out_bf16 else 4

    vals = wl.kept_weights(w)
    I = wl.activations(w)
    if bf16:
        vals_lib, I_lib = wl.to_bf16_bits(vals), wl.to_bf16_bits(I)
        vals_f32, I_f32 = wl.bf16_bits_as_f32(vals_lib), wl.bf16_bits_as_f32(I_lib)
    else:
        vals_lib, I_lib, vals_f32, I_f32 = vals, I, vals, I

    mask = rb.rbgp_make_mask(w.rows, w.cols, w.row_deg, w.mask_seed)
    if args.kernel != rb.KERNEL_AUTO:
        rb.rbgp_mask_set_kernel(mask, args.kernel)
    if args.tune:
        for knob, value in enumerate(int(x) for x in args.tune.split(",")):
            rb.rbgp_mask_tune(mask, knob, value)
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(rb.rbgp_packed_bytes(mask, w.dtype), dtype=torch.uint8, device=dev)
    rb.rbgp_pack(mask, w.dtype, np.ascontiguousarray(vals_lib), packed.data_ptr(), stream)

    if args.backward:
        res = backward_objects(w, mask, vals_lib, vals_f32, I_lib, I_f32, torch, dev, stream,
                               check=not args.no_cpu_baseline, steps=args.steps, warmup=args.warmup,
                               only=None if args.backward == "both" else args.backward)
        print(json.dumps({"workload": w.name, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
                          "steps": args.steps, "warmup": args.warmup, **res}))
        return
    algorithmic_bytes = w.algorithmic_bytes - w.M * w.N * (4 - out_bytes)
    if args.fused_conv:
        if w.name not in wl.CONV_GEOMETRY:
            sys.exit("bench.py: --fused-conv needs a workload that is a lowered 3x3 convolution")
        B, H, W = wl.CONV_GEOMETRY[w.name]
        X = wl.conv_activations(w, B, H, W)
        if bf16:
            Xbits = wl.to_bf16_bits(X)
            X = wl.bf16_bits_as_f32(Xbits)
            Xp = wl.zero_padded(Xbits).view(np.int16)
        else:
            Xp = wl.zero_padded(X)
        # the oracle's operand for the parity check: the same activations, lowered explicitly
        from oracle import rbgp_oracle as orc
        I_f32 = orc.im2col_3x3(X) if not args.no_cpu_baseline else None
        algorithmic_bytes = Xp.nbytes + w.M * w.N * out_bytes + w.nnz * w.in_bytes
        set_bytes = Xp.nbytes + w.M * w.N * out_bytes
        I0 = torch.from_numpy(Xp).to(dev)
    else:
        ld = w.N + args.ld_pad
        set_bytes = (w.K * w.in_bytes + w.M * out_bytes) * ld
        I_pad = np.zeros((w.K, ld), dtype=I_lib.dtype)
        I_pad[:, :w.N] = I_lib
        I0 = torch.from_numpy(I_pad.view(np.int16) if bf16 else I_pad).to(dev)
    nsets = args.sets if args.sets > 0 else max(2, min(16, -(-512 * 2**20 // set_bytes)))
    Is = [I0] + [I0.clone() for _ in range(nsets - 1)]
    ldO = w.N if args.fused_conv else w.N + args.ld_pad
    Os = [torch.empty((w.M, ldO), dtype=torch.int16 if args.out_bf16 else torch.float32, device=dev)
          for _ in range(nsets)]

    def step(i):
        j = i % nsets
        if args.fused_conv:
            rb.rbgp_conv3x3(mask, call_dtype, w.M, w.K // 9, B, H, W, packed.data_ptr(), Is[j].data_ptr(),
                            Os[j].data_ptr(), w.N, stream)
        else:
            rb.rbgp_spmm(mask, call_dtype, w.M, w.K, w.N, packed.data_ptr(), Is[j].data_ptr(), ldO,
                         Os[j].data_ptr(), ldO, stream)

    # Set-up, untimed and not counted as warm-up steps: the same call, launched until the shader clock has
    # settled (a GPU that comes out of idle runs its first few hundred launches some 5 % slower; with
    # `--steps 20 --warmup 5` the timed region would otherwise measure the clock ramp, not the kernel).
    for i in range(args.settle):
        step(i)

    def timed_region():
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()                              # same stream as the launches (torch's current stream)
        for i in range(args.steps):
            step(i)
        ev1.record()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ev0.elapsed_time(ev1) / args.steps

    # (set-up as well: the whole region -- warm-up, synchronisation, K steps, synchronisation -- rehearsed, untimed, so
    # that what the process does once -- the first events, the first wait on a drained queue -- is not in the K steps)
    for _ in range(3 if args.settle else 0):
        timed_region()
    wall, kern_ms = timed_region()
    ms_per_step = wall * 1e3 / args.steps
    # the same measurement over a long run (what the other objects of the line are timed with)
    settled_steps = max(args.steps, 2000)
    ev2, ev3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev2.record()
    for i in range(settled_steps):
        step(i)
    ev3.record()
    torch.cuda.synchronize()
    settled_ms = ev2.elapsed_time(ev3) / settled_steps
    # and with one buffer set only: I then comes out of the 256 MB last-level cache, as it would behind a
    # layer that has just written it, instead of from HBM (reported beside the headline, never as it)
    resident_ms = None
    if not args.no_cache_resident:
        nsets_all, nsets = nsets, 1
        ev4, ev5 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(200):
            step(i)
        ev4.record()
        for i in range(settled_steps):
            step(i)
        ev5.record()
        torch.cuda.synchronize()
        resident_ms = ev4.elapsed_time(ev5) / settled_steps
        nsets = nsets_all

    value = w.flops / (ms_per_step * 1e-3) / 1e12
    bound = BOUND[args.workload]
    if bound == "mfma":
        achieved = w.flops / (kern_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_F32_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_F32_TFLOPS, "traffic": None}
    else:
        achieved = algorithmic_bytes / (kern_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    try:
        with open(TRAFFIC_FILE) as f:
            roof["traffic"] = None if args.fused_conv else json.load(f).get(w.name, {}).get("hbm_bytes_per_launch")
    except OSError:
        pass
    roof["kernel_ms"] = kern_ms
    roof["algorithmic_bytes"] = algorithmic_bytes
    roof["algorithmic_flops"] = w.flops
    roof["settled_kernel_ms"] = settled_ms
    roof["settled_steps"] = settled_steps
    roof["cache_resident_kernel_ms"] = resident_ms
    roof["settled_frac"] = (w.flops / (settled_ms * 1e-3) / 1e12 / PEAK_F32_TFLOPS if bound == "mfma"
                            else algorithmic_bytes / (settled_ms * 1e-3) / 1e9 / PEAK_HBM_GBS)

    out = {"metric": "effective TFLOP/s (2*nnz*N) RBGP4 SpMM", "value": value, "unit": "TFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
           "config": {"workload": w.name, "output": "bf16" if args.out_bf16 else "f32", "M": w.M, "K": w.K, "N": w.N, "density": w.density,
                      "factors_rows": list(w.rows), "factors_cols": list(w.cols), "factors_row_deg": list(w.row_deg),
                      "kernel": rb.rbgp_mask_kernel(mask, w.dtype), "tune": args.tune or "default",
                      "buffer_sets": nsets, "settle_launches": args.settle, "ld_pad": 0 if args.fused_conv else args.ld_pad,
                      "reg_plan": rb.rbgp_mask_reg_plan(mask),
                      "entry_point": "rbgp_conv3x3" if args.fused_conv else "rbgp_spmm"},
           "roofline": roof}
    if not args.no_cpu_baseline:
        O_host = Os[0].cpu().numpy()[:, :w.N]
        if args.out_bf16:      # (bf16 bits widened exactly; the rounding stays inside the bf16 tolerance of the check)
            O_host = wl.bf16_bits_as_f32(O_host.view(np.uint16))
        out["cpu_baseline"] = cpu_baseline(w, vals_f32, I_f32, O_host)
    if not args.fused_conv and not args.forward_only and w.name in wl.CONV_GEOMETRY and \
            rb.rbgp_mask_kernel(mask, w.dtype) == rb.KERNEL_MFMA_REG:     # (the fused call runs on that family only)
        out["fused_conv3x3"] = fused_conv_line(w, mask, packed, vals_f32, torch, dev, stream,
                                               check=not args.no_cpu_baseline)
    if not args.fused_conv and not args.forward_only and args.workload == "conv5":
        out["backward"] = backward_objects(w, mask, vals_lib, vals_f32, I_lib, I_f32, torch, dev, stream,
                                           check=not args.no_cpu_baseline)
    if not args.fused_conv and not args.forward_only and args.workload == "conv5" and not args.no_sweep_sums:
        del Is, Os
        torch.cuda.empty_cache()
        out["vgg19_sweep"] = sweep_sums(torch, dev)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
