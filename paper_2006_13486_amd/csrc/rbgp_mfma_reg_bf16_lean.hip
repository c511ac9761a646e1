// Register-streaming MFMA kernel, bf16 inputs: the variants with one register set and more waves per SIMD --
// 128-column tiles; stages of 36 and 72 steps with one or two groups, the shorter stages with two or four groups
// (four: one tile row per group).  Kernel: rbgp_reg_bf16_kernel.h.
#include "rbgp_reg_bf16_kernel.h"

namespace {

#define RBGP_BL(KC, RS) {KC, RS, 1, 128, spmm_reg_bf16<KC, RS, 1, 128, true>}, {KC, RS, 2, 128, spmm_reg_bf16<KC, RS, 2, 128, true>}
#define RBGP_BL2(KC, RS) {KC, RS, 2, 128, spmm_reg_bf16<KC, RS, 2, 128, true>}
const Entry kLeanTable[] = {RBGP_BL(36, 2), RBGP_BL(72, 2), RBGP_BL(36, 4),  RBGP_BL(72, 4),
                            RBGP_BL(36, 8), RBGP_BL(72, 8), RBGP_BL(36, 16), RBGP_BL(72, 16),
                            RBGP_BL2(18, 2), RBGP_BL2(32, 2), RBGP_BL2(18, 4),  RBGP_BL2(32, 4),
                            RBGP_BL2(18, 8), RBGP_BL2(32, 8), RBGP_BL2(18, 16), RBGP_BL2(32, 16),
                            {18, 16, 4, 128, spmm_reg_bf16<18, 16, 4, 128, true>},
                            {32, 16, 4, 128, spmm_reg_bf16<32, 16, 4, 128, true>},
                            {36, 16, 4, 128, spmm_reg_bf16<36, 16, 4, 128, true>}};

}  // namespace

rbgp_reg_fn rbgp_reg_bf16_lean_kernel(int KC, int RS, int G, int CW) {
  for (const Entry &e : kLeanTable)
    if (e.KC == KC && e.RS == RS && e.G == G && e.CW == CW) return e.fn;
  return nullptr;
}
