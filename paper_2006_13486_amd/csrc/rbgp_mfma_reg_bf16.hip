// Register-streaming MFMA kernel for O = W_s x I (Section 5, "GPU Implementation"), bf16 inputs: the 64-column wave
// tiles (two register sets) and the lookup of every variant.  The kernel itself is in rbgp_reg_bf16_kernel.h.
#include "rbgp_reg_bf16_kernel.h"

namespace {

#define RBGP_B1(KC, RS, G) {KC, RS, G, 64, spmm_reg_bf16<KC, RS, G, 64>}
#define RBGP_B(KC, RS) RBGP_B1(KC, RS, 1), RBGP_B1(KC, RS, 2), RBGP_B1(KC, RS, 4)
const Entry kTable[] = {RBGP_B(8, 2),  RBGP_B(18, 2),  RBGP_B(32, 2),  RBGP_B(36, 2),  RBGP_B(72, 2),
                        RBGP_B(8, 4),  RBGP_B(18, 4),  RBGP_B(32, 4),  RBGP_B(36, 4),  RBGP_B(72, 4),
                        RBGP_B(8, 8),  RBGP_B(18, 8),  RBGP_B(32, 8),  RBGP_B(36, 8),  RBGP_B(72, 8),
                        RBGP_B(8, 16), RBGP_B(18, 16), RBGP_B(32, 16), RBGP_B(36, 16), RBGP_B(72, 16)};

}  // namespace

rbgp_reg_fn rbgp_reg_bf16_wide_kernel(int KC, int RS, int G);   // rbgp_mfma_reg_bf16_wide.hip

rbgp_reg_fn rbgp_reg_bf16_kernel(int KC, int RS, int G, int CW) {
  if (CW == 128) return rbgp_reg_bf16_wide_kernel(KC, RS, G);
  for (const Entry &e : kTable)
    if (e.KC == KC && e.RS == RS && e.G == G && e.CW == CW) return e.fn;
  return nullptr;
}
