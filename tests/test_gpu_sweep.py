"""GPU parity of the layer sweep (all VGG19 conv shapes x four densities x two dtypes) and of the
4096^3 SDMM shapes of Table 3 (Section 6, "RBGP4 runtime characteristics"), at full size with the
library's default launch: what `bench.py` times in its sweeps.  The inputs are drawn on the device
(seeded); a sample of output columns goes back to the host and is compared element by element with
the oracle's product of the same input bits (normalised error, tolerance of the dtype)."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import naive_c
from oracle import rbgp_oracle as orc
from paper_2006_13486_amd import binding as rb
from paper_2006_13486_amd import workloads as wl
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu

# the distinct (C_in, C_out, H) of the 16 layers, by the first layer that has them
DISTINCT_LAYERS = sorted({shape: i for i, shape in reversed(list(enumerate(wl.VGG19_LAYERS)))}.values())
_inputs = {}


def _device_inputs(w):
    """(fp32 matrix, bf16 bits) of the layer's input on the device, kept for the cells that share it."""
    import torch
    key = (w.K, w.N, w.i_seed)
    if key not in _inputs:
        _inputs.clear()                      # one layer's inputs at a time (up to 300 MB)
        torch.cuda.empty_cache()
        I32 = wl.device_activations(w, torch.device("cuda:0"))
        _inputs[key] = (I32, I32.to(torch.bfloat16).view(torch.int16))
    return _inputs[key]


def _check_sampled(w, ncols=48, expect_kernel=None):
    import torch
    dev = torch.device("cuda:0")
    I32, I16 = _device_inputs(w)
    I_d = I16 if w.dtype == wl.BF16 else I32
    vals = wl.kept_weights(w)
    vals_lib = wl.to_bf16_bits(vals) if w.dtype == wl.BF16 else vals
    vals_f32 = wl.bf16_bits_as_f32(vals_lib) if w.dtype == wl.BF16 else vals
    mask = gh.make_mask(w)
    rb.rbgp_mask_check_tables(mask)
    used = rb.rbgp_mask_kernel(mask, w.dtype)
    print(f"[gpu] {w.name} rows={w.rows} cols={w.cols} deg={w.row_deg} N={w.N} kernel={used} "
          f"plan={rb.rbgp_mask_reg_plan(mask)[:11]}", flush=True)
    if expect_kernel is not None:
        assert used == expect_kernel
    stream = torch.cuda.current_stream().cuda_stream
    packed = torch.zeros(max(rb.rbgp_packed_bytes(mask, w.dtype), 16), dtype=torch.uint8, device=dev)
    rb.rbgp_pack(mask, w.dtype, np.ascontiguousarray(vals_lib), packed.data_ptr(), stream)
    O = torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device=dev)
    rb.rbgp_spmm(mask, w.dtype, w.M, w.K, w.N, packed.data_ptr(), I_d.data_ptr(), w.N, O.data_ptr(), w.N, stream)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(O).any()), "an output element was not written"
    g = np.random.Generator(np.random.PCG64(w.i_seed + 7))
    cols = np.sort(g.choice(w.N, size=min(ncols, w.N), replace=False))
    cols[0], cols[-1] = 0, w.N - 1           # the two ends of the batch are always in the sample
    cols_d = torch.from_numpy(cols).to(dev)
    sub = I_d[:, cols_d].cpu().numpy()
    I_sub = wl.bf16_bits_as_f32(sub.view(np.uint16)) if w.dtype == wl.BF16 else sub
    got = O[:, cols_d].cpu().numpy()
    ref, den = gh.oracle_spmm(w, vals_f32, np.ascontiguousarray(I_sub))
    err = orc.normalised_error(got, ref, den)
    print(f"[gpu]   normalised error {err:.3e} on {len(cols)} columns", flush=True)
    assert err <= gh.TOL[w.dtype], err


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("log2_inv_density", [1, 2, 3, 4])
@pytest.mark.parametrize("layer", DISTINCT_LAYERS)
def test_vgg19_sweep_cell(layer, log2_inv_density, dtype):
    """Every distinct layer shape of the sweep at every density and dtype (layer 0 is dense whatever the
    density: it runs once per dtype)."""
    if layer == 0 and log2_inv_density != 1:
        pytest.skip("the first layer stays dense")
    _check_sampled(wl.vgg19_sweep_workload(layer, log2_inv_density, dtype))


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("gr,gb", [(1, 1), (2, 1), (4, 1), (1, 2), (1, 4), (2, 2)])
def test_sdmm4096_table3_shape(gr, gb, dtype):
    """Table 3's six (G_r, G_b) shapes at 87.5 % sparsity (G_o at 50 %), on whatever family the library takes for
    them (the mask itself or the mask with G_i filled in, stage lists split over the waves of a workgroup)."""
    _check_sampled(replace(wl.sdmm4096_table3(gr, gb, 3), dtype=dtype))


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("o,i", [(0, 3), (2, 1), (3, 1)])
def test_sdmm4096_table2_split(o, i, dtype):
    """Table 2: all the sparsity in G_i, most of it in G_o, and G_o at 1/8."""
    _check_sampled(replace(wl.sdmm4096_table2(o, i), dtype=dtype))


def test_sdmm4096_table3_first_row_at_every_density():
    """One row per column set (G_r = G_b = (1, 1)): the filled family at 75, 87.5 and 93.75 %."""
    for d in (2, 3, 4):
        _check_sampled(wl.sdmm4096_table3(1, 1, d))
