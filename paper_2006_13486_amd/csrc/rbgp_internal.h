// Internal definitions shared by the host part (sampler, mask object) and the
// device part (tables, pack, SpMM launchers) of the library.  Not installed.
#pragma once

#include <cstddef>
#include <cstdint>
#include <new>
#include <vector>

#include "../../include/rbgp.h"

struct rbgp_device_state;  // defined in rbgp_device.hip

// No C++ exception crosses the C boundary: an entry point that can allocate host memory returns through this.
#define RBGP_GUARDED(expr)              \
  try {                                 \
    return (expr);                      \
  } catch (const std::bad_alloc &) {    \
    return RBGP_ENOMEM;                 \
  } catch (...) {                       \
    return RBGP_EINVAL;                 \
  }

// MFMA_REG bf16 kernels: a stage of KC contraction steps = rbgp_bf16_blocks32(KC) blocks of 32 steps
// plus, if rbgp_bf16_tail16(KC), one block of 16 (a remainder above 16 takes a whole block of 32)
constexpr int rbgp_bf16_blocks32(int KC) { return KC / 32 + (KC % 32 > 16 ? 1 : 0); }
constexpr bool rbgp_bf16_tail16(int KC) { return KC % 32 != 0 && KC % 32 <= 16; }

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

// Shape of the register-streaming MFMA kernels (see rbgp_mfma_reg.hip).
struct rbgp_reg_plan {
  bool ok = false;
  int fold = 1;  // G_r being complete, G_o (x) G_r = (G_o with every row repeated `fold` times) (x)
                 //   (a complete graph on |G_r.U| / fold rows): when |G_r.U| * |G_b.U| exceeds the 16 rows
                 //   of an MFMA group, `fold` of G_r's rows move into the tile-row index
  int TR = 0;    // tile rows: |G_o.U| * fold; tile row u has the tiles of G_o's row u / fold
  int A2 = 0;    // rows of G_r inside a tile row: |G_r.U| / fold
  int R = 0, RB = 0;   // rows of a tile row that share one column set: A2 * |G_b.U|
  int KT = 0;    // contraction length of one group in one tile: |G_r.V| * d_i * |G_b.V|
  int VC = 0;    // G_r columns per stage
  int KCR = 0;   // contraction length per stage: VC * d_i * |G_b.V|
  int KC = 0;    // KCR rounded up to a stage size the kernels are built for (8, 18, 32, 36, 72); the
                 //   positions past KCR hold zero weights and read row 0 of the stage
  int NSTG = 0;  // stages per tile: |G_r.V| / VC
  int RS = 0;    // weight rows per tile row inside a 16-row MFMA group: R rounded up to 2^k
  int MG = 0;    // tile rows per MFMA group: 16 / RS
  int NO = 0;    // load slots per stage: ceil(KC / 4)
  int NQ = 0;    // 16-byte weight loads per lane, group and stage: ceil(NO / 4)
  int SRC = 0;   // rows of I spanned by one stage: VC * |G_i.V| * |G_b.V|
  int64_t packed_elems = 0;       // fp32 layout
  int64_t packed_elems_bf16 = 0;  // bf16 layout
};

// fp32 register-streaming kernels: which step of a stage's contraction list
// ((v_r % VC) * d_i + j_i) * |G_b.V| + v_b  sits at position kk of the packed fragment and of the
// row table (position kk = 4 * slot + lane group).  Identity, except for masks whose G_b is the
// nine taps of a 3x3 convolution (|G_b.V| = 9 complete) with a stage of a multiple of 12 steps:
// there the three horizontal taps (dx = -1, 0, +1) of one (channel, dy) pair occupy three
// consecutive slots of ONE lane group, so that the fused convolution can build all three from
// one load of the pixel row.  The order of the steps inside a stage does not matter to the product.
inline bool rbgp_reg_tap_grouped(const rbgp_mask *m);
inline int rbgp_reg_step(const rbgp_mask *m, int kk);

// Register-streaming family: a wave keeps its stage list in a lane-held table, one stage per lane (64 stages;
// reads past its count are turned into sentinels by the count); a cluster's list may be up to four times that
// and is then split over the waves of a workgroup (wave k takes stages k, k + S, ...).
constexpr int kRegWaveStages = 64, kRegMaxStages = 256;

// Clustering of the tile rows for the register-streaming family (host tables).
struct rbgp_reg_clusters {
  int U = 0;                      // tile rows per cluster
  int ncl = 0;
  int max_stages = 0;             // longest stage list (a wave holds at most 60 stages, one per lane; a longer list,
                                  //   up to 240, is split over 2 or 4 waves of the workgroup)
  int tstride = 64;               // entries per table row: 64, or 256 where a list exceeds 60 stages
  std::vector<int32_t> members;   // [ncl][U] tile rows, -1: none
  std::vector<int32_t> stages;    // [ncl][1+U][tstride]: base row of I per stage, then per member the
                                  //   position of its weight fragment (-1: member lacks the tile); -1 past the end
  std::vector<int32_t> counts;    // [ncl] stages per cluster
};

// Lo/hi pairing of the tile rows for the fp32 register-streaming kernels whose MFMA groups hold two
// tile rows of 8 rows (rbgp_mfma_reg_dual.hip).  Tile rows come in quads (L0, L1, H0, H1).  Wave
// (x, y) of a quad multiplies the tiles that L_x and H_y share: L_x's weights in rows 0..7 of the
// group, H_y's in rows 8..15.  A tile that finds no partner in the quad gets a stage with the other
// half zero.  Every (tile row, tile) pair is multiplied exactly once; the two waves of L_x together
// walk L_x's tiles (and run on one SIMD), the sums of a tile row are added up from its two waves.
struct rbgp_reg_dual {
  bool ok = false;
  int nq = 0;                     // quads
  int max_stages = 0;             // most stages of the two waves of an L row
  int max_wave = 0;               // longest stage list of a wave
  int64_t total_stages = 0;       // over all waves
  std::vector<int32_t> members;   // [nq][4]: L0, L1, H0, H1 (-1: none)
  std::vector<int32_t> stages;    // [nq][x][y][3][64]: per wave and stage (one per lane) the base row of I, the
                                  //   position of L_x's weight fragment among L_x's (-1: none), the position of
                                  //   H_y's among its own (-1: none); -1 past the end (sentinel stages)
  std::vector<int32_t> counts;    // [nq][x][y]: stages of the wave
};

// One sampled base graph of a mask made from more than four of them.
struct rbgp_base_graph {
  int32_t a, c, d, e, role;
  std::vector<int32_t> adj;           // a x d, ascending
  double sigma1, sigma2, bound;
  int status, tries;
};

struct rbgp_mask {
  int32_t a[4], c[4], d[4], e[4];     // rows, cols, left degree, right degree of each factor
  std::vector<int32_t> adj[4];        // adjacency lists, a[i] x d[i], ascending
  double sigma1[4], sigma2[4], bound[4];
  int status[4], tries[4];
  int64_t M, K, rowdeg, coldeg, nnz;
  uint64_t uid;                       // unique per mask object of the process (never 0)
  int kernel_choice;                  // RBGP_KERNEL_*
  std::vector<rbgp_base_graph> base;  // the sampled base graphs, in product order (four for rbgp_make_mask)
  std::vector<int32_t> from_original; // masks made by rbgp_mask_transpose: canonical index in the
                                      //   original mask of every kept value, in this mask's order
  rbgp_mfma_plan plan;
  rbgp_reg_plan reg;
  rbgp_reg_clusters reg_clusters;     // clusters of reg.MG tile rows (when reg.ok)
  rbgp_reg_dual reg_dual;             // lo/hi pairing (when reg.ok, reg.MG == 2 and at most 32 tile rows)
  mutable rbgp_device_state *dev;     // lazily created device tables
  rbgp_mask *filled = nullptr;        // RBGP_KERNEL_MFMA_REG_FILLED: the mask G_o (x) J (x) G_b with G_r and G_i
                                      //   replaced by the complete graph on their vertices (same M, K, same row and
                                      //   column numbering; a superset of this mask), or nullptr; owned
  int filled_kind = 0;                // 0: G_i filled in; 1: G_o filled in (and merged with G_r into one tile column)
  rbgp_mask *regroup = nullptr;       // RBGP_KERNEL_MFMA_REG, fp32, on a mask with more than 16 rows per column set: the SAME mask
                                      //   (same entries, same canonical order of the kept values) factored as
                                      //   G_o (x) G_r (x) (G_i (x) J(q, 1)) (x) J(|G_b.U| / q, |G_b.V|), whose rows per
                                      //   column set fill more of a 16-row MFMA group; the register family then runs on
                                      //   it (tables, plan and packed layout are its own), or nullptr; owned.  Or, where
                                      //   G_o is complete, the same mask with G_o (x) G_r merged into one tile column
                                      //   J(a_o, 1) (x) J(a_r, c_o c_r), whose stages are longer (then for bf16 as well)
  bool regroup_bf16 = false;          // the bf16 kernels run on `regroup` too
};

inline bool rbgp_reg_tap_grouped(const rbgp_mask *m) {
  return m->reg.ok && m->c[3] == 9 && m->d[3] == 9 && m->reg.KC % 12 == 0 && m->reg.KCR == m->reg.KC;
}
inline int rbgp_reg_step(const rbgp_mask *m, int kk) {
  if (!rbgp_reg_tap_grouped(m)) return kk;
  const int slot = kk / 4, g = kk % 4;
  const int pair = (slot / 3) * 4 + g;          // (channel-like index, dy) pair handled by lane group g
  const int dxi = slot % 3, dyi = pair % 3;
  return (pair / 3) * 9 + 3 * dyi + dxi;
}

enum { RBGP_NUM_KERNELS = 6 };   // one more than the largest RBGP_KERNEL_* value

// Shape of the tile kernels (rbgp_mfma_tile.hip): every nonzero of G_o is a dense TM x TK block of W_s
// (zero where the inner graphs have no edge), multiplied in 32-row blocks by 16-step MFMAs.
struct rbgp_tile_plan {
  bool ok = false;
  int TM = 0;    // rows of a tile: |G_r.U| * |G_i.U| * |G_b.U| (32)
  int TK = 0;    // columns of a tile: |G_r.V| * |G_i.V| * |G_b.V|
  int TKP = 0;   // TK rounded up to a stage length the kernels are built for (16 x 2, 4, 5, 8, 9, 16, 18, 20);
                 //   the padding holds zero weights
  int64_t packed_elems = 0;   // |G_o.U| * d_o * TKP * TM
};
inline rbgp_tile_plan rbgp_plan_tile(const rbgp_mask *m) {
  rbgp_tile_plan p;
  const int64_t tm = int64_t(m->a[1]) * m->a[2] * m->a[3], tk = int64_t(m->c[1]) * m->c[2] * m->c[3];
  if (tm != 32 || tk > 320 || m->c[0] > 256) return p;
  p.TM = int(tm); p.TK = int(tk);
  for (int nc : {20, 18, 16, 9, 8, 5, 4, 2})
    if (16 * nc >= tk) p.TKP = 16 * nc;
  p.packed_elems = int64_t(m->a[0]) * m->d[0] * p.TKP * p.TM;
  p.ok = p.packed_elems * 2 < (int64_t(1) << 30);   // (32-bit offsets into the packed weights)
  return p;
}

// device part
void rbgp_device_release(rbgp_device_state *dev);
void rbgp_set_hip_error(const char *msg);
// register-streaming family (rbgp_mfma_reg.hip); `state` is its lazily built table cache
bool rbgp_reg_covers(const rbgp_mask *m);
// geometry of a fused 3x3 convolution (stride 1, zero padding 1): N = images * height * width
struct rbgp_conv_geometry {
  int64_t images, height, width;
};
// conv == nullptr: I is the K x N matrix; else I is the zero-padded activation tensor
// [K / 9][images][height + 2][width + 2] and ldI is ignored.  out_bf16 (bf16 only): O holds bf16 bits
int rbgp_reg_launch(const rbgp_mask *m, void **state, const int *tune, bool bf16, bool out_bf16, int64_t N,
                    const void *packed, const void *I, int64_t ldI, void *O, int64_t ldO, void *stream,
                    const rbgp_conv_geometry *conv = nullptr);
void rbgp_reg_release(void *state);
// tile family (rbgp_mfma_tile.hip; bf16 inputs only); needs rbgp_plan_tile(m).ok; conv as for rbgp_reg_launch
// (image width a multiple of 8)
int rbgp_tile_launch(const rbgp_mask *m, void **state, bool out_bf16, int64_t N, const void *packed, const void *I,
                     int64_t ldI, void *O, int64_t ldO, void *stream, const rbgp_conv_geometry *conv = nullptr);
void rbgp_tile_release(void *state);
// weight-gradient kernels (rbgp_sddmm.hip); use_mfma needs rbgp_reg_covers(m)
// conv != nullptr (needs use_mfma): I is the zero-padded activation tensor of a 3x3 convolution, ldI is ignored
int rbgp_sddmm_launch(const rbgp_mask *m, void **state, const int32_t *const dev_adj[4], bool use_mfma, bool bf16,
                      int64_t N, const void *dO, int64_t ld_dO, const void *I, int64_t ldI, float *dW, void *stream,
                      const rbgp_conv_geometry *conv = nullptr);
// the same through the static scratch array of rbgp_sddmm.hip: no device allocation, tables uploaded as kernel arguments
int rbgp_sddmm_static_launch(const rbgp_mask *m, bool use_mfma, bool bf16, int64_t N, const void *dO, int64_t ld_dO,
                             const void *I, int64_t ldI, float *dW, void *stream);
void rbgp_sddmm_release(void *state);
uint64_t rbgp_next_uid();
// host part
void rbgp_plan_mfma(rbgp_mask *m);
void rbgp_plan_reg(rbgp_mask *m);
void rbgp_reg_cluster(const rbgp_mask *m, int U, rbgp_reg_clusters *out);
void rbgp_reg_plan_dual(const rbgp_mask *m, rbgp_reg_dual *out);
// builds m->filled where the register family covers it (called once, when the mask is made)
void rbgp_plan_filled(rbgp_mask *m);
// builds m->regroup where that factoring uses more rows of the MFMA group (called once, when the mask is made)
void rbgp_plan_regroup(rbgp_mask *m);
// canonical index (m * rowdeg + t) of every packed element, -1 for padding
void rbgp_build_pack_perm(const rbgp_mask *m, int kernel, bool bf16, std::vector<int32_t> &perm);
