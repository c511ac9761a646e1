// Internal definitions shared by the host part (sampler, mask object) and the
// device part (tables, pack, SpMM launchers) of the library.  Not installed.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/rbgp.h"

struct rbgp_device_state;  // defined in rbgp_device.hip

// Shape of the MFMA kernels' work decomposition for one mask (see rbgp_device.hip).
struct rbgp_mfma_plan {
  bool ok = false;
  int R = 0;    // rows sharing one column set: |G_r.U| * |G_b.U|
  int RB = 0;   // 4-row blocks per group: ceil(R / 4)
  int KS = 0;   // contraction length of one group in one stage: d_i * |G_b.V|
  int NCH = 0;  // 16-wide chunks of KS
  int SR = 0;   // rows of I staged per stage: |G_i.V| * |G_b.V|
  int64_t packed_elems = 0;
};

struct rbgp_mask {
  int32_t a[4], c[4], d[4], e[4];     // rows, cols, left degree, right degree of each factor
  std::vector<int32_t> adj[4];        // adjacency lists, a[i] x d[i], ascending
  double sigma1[4], sigma2[4], bound[4];
  int status[4], tries[4];
  int64_t M, K, rowdeg, coldeg, nnz;
  int kernel_choice;                  // RBGP_KERNEL_*
  rbgp_mfma_plan plan;
  mutable rbgp_device_state *dev;     // lazily created device tables
};

// device part
void rbgp_device_release(rbgp_device_state *dev);
// host part
void rbgp_plan_mfma(rbgp_mask *m);
// canonical index (m * rowdeg + t) of every packed element, -1 for padding
void rbgp_build_pack_perm(const rbgp_mask *m, int kernel, std::vector<int32_t> &perm);
