// Shared by the register-streaming MFMA kernels (fp32 and bf16 translation units):
// kernel parameter block and small device helpers.
#ifndef RBGP_REG_COMMON_H
#define RBGP_REG_COMMON_H

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

namespace rbgp_reg {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// fp32 -> bfloat16 bits, round to nearest, ties to even: the conversion instruction of gfx950
// (v_cvt_pk_bf16_f32, two values each), which the compiler selects for these casts.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ uint32_t bf16_bits(float x) { return bf16_pair(x, 0.f) & 0xffffu; }

struct RegParams {
  const float *Wp;         // packed weights (fp32, or bf16 bits for the bf16 kernels)
  const float *I;          // activations (same)
  float *O;                // fp32, or bf16 bits when obf16 is set (ldO counts elements of that type)
  int obf16;               // bf16 kernels: round the sums to bf16 when storing O
  const int32_t *rowtab;   // [a_i][NO*4]: stage-relative I row of each contraction step (padding -> 0)
  const int32_t *stages;   // [ncl][1+MG][tstride]: per stage the base row of the stage, then per
                           //   cluster member j_o * NSTG + (stage within the tile), the position of its
                           //   weight fragment among the member's fragments; -1 past the end (sentinel
                           //   stages) and when the member does not have the tile.  Wave k of the S that split a
                           //   list holds stage k + l * S in lane l.
  int tstride;             // 64, or 256 where a list has more than 60 stages (its last entry is always a sentinel)
  const int32_t *counts;   // [ncl] stages of each cluster (<= 60 per wave: <= 60 * S)
  const int32_t *members;  // [ncl][MG] tile rows of each cluster (-1: none)
  int64_t N, ldI, ldO;
  uint32_t w_bytes;        // extent of the packed weights (buffer descriptor)
  uint32_t row_bytes;      // ldI in bytes
  uint32_t n_bytes;        // N in bytes (N rounded up to a lane's load for bf16): extent of the last row of I
  int last_row, src_rows;  // K - 1; rows of I one stage spans
  // Fused 3x3 convolution (fp32 kernels): I is not materialised; row k = 9 * channel + tap of it is
  // read from the zero-padded activations X[channel][image][H+2][W+2].  Then the "row" unit of the
  // three fields above is a channel (row_bytes = bytes of one channel of X, last_row = channels - 1,
  // src_rows = channels one stage spans, n_bytes = row_bytes) and rowtab holds byte offsets
  // (channel and tap shift) instead of rows.
  int conv;                // 1: fused convolution
  int conv_h, conv_w;      // image height and width (W a multiple of 4)
  const int32_t *colbase;  // fused convolution: byte offset, inside a channel of X, of the first pixel of every
                           //   group of columns one lane loads (4, or 8 with the wide bf16 tile); padded to whole tiles
  int a2, a3, a4, R;
  int fpm;                 // weight fragments per member: d_o * NSTG
  int rowofs[16];          // output row of weight row r of a group, relative to its (tile row, u_i) base
  int tm;                  // rows of one tile row: a_r * a_i * a_b
  int ntiles;              // column tiles: ceil(N / columns per wave)
  int lgS;                 // log2 of the waves that share a column tile (split of the stage list)
  int ncl;                 // clusters of tile rows (pairing kernel: quads)
  int ct, ct_cnt;          // fp32 kernels with stages of up to 8 steps: column tiles a wave takes one after the other (1 elsewhere)
                           //   and, when that is more than one, the stages of every cluster's list (all equal, a multiple of 4)
  // Workgroups (one-dimensional grid) are dealt round-robin to the 8 XCDs, so workgroup id & 7 is the XCD, each with
  // its own L2; within an XCD they start in the order of their ids.  A unit is a (G_i vertex, group of column
  // tiles) pair; the clusters of a unit are always neighbours on one XCD (they read the same rows of I).  order:
  //  2  column group g on XCD g & 7, all G_i vertices of a column group together: the workgroups that run at the same
  //     time read neighbouring columns on all eight XCDs (long runs of every row of I are wanted at once, which the
  //     memory likes), and G_i vertices that share rows of I share an L2.  For batches of at least 8 column groups.
  //  1  the units in (G_i vertex, column group) order, dealt to the XCDs in blocks of per_xcd items: an XCD reads one
  //     wide contiguous span of the rows of its G_i vertices.  Where every row of I belongs to one G_i vertex (right
  //     degree 1) and the batch is a few dozen column groups: on the VGG19 conv5 shape the XCDs then finish
  //     together, with order 2 every other XCD ran 1.4 us longer.
  //  0  as 1 in (column group, G_i vertex) order: small batches whose G_i vertices share rows of I.
  int per_xcd;             // items (cluster, unit) per XCD
  int ngroups;             // groups of column tiles (one group per workgroup)
  int order;
};

constexpr int kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format (gfx9 family)
constexpr int kOob = 0x40000000;        // byte offset beyond any packed weight buffer (reads return 0)

// (cluster, G_i vertex, group of column tiles) of this workgroup; false: none (the workgroup leaves)
struct WgCoord {
  int cl, u3, ntq;
};
__device__ __forceinline__ bool wg_coord(const RegParams &p, WgCoord *c) {
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  if (p.order == 2) {
    const int per_group = p.ncl * p.a3, q = slot / per_group, rem = slot - q * per_group;
    c->ntq = xcd + 8 * q;
    if (c->ntq >= p.ngroups) return false;
    c->u3 = rem / p.ncl;
    c->cl = rem - c->u3 * p.ncl;
    return true;
  }
  const int item = xcd * p.per_xcd + slot;
  if (item >= p.ncl * p.a3 * p.ngroups) return false;
  const int unit = item / p.ncl;
  c->cl = item - unit * p.ncl;
  if (p.order == 1) {
    c->u3 = unit / p.ngroups;
    c->ntq = unit - c->u3 * p.ngroups;
  } else {
    c->ntq = unit / p.a3;
    c->u3 = unit - c->ntq * p.a3;
  }
  return true;
}

__device__ __forceinline__ f32x4 load_x4(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
  return f32x4{__uint_as_float(v[0]), __uint_as_float(v[1]), __uint_as_float(v[2]), __uint_as_float(v[3])};
}

}  // namespace rbgp_reg

namespace rbgp_reg {
// Parameter block of the lo/hi pairing kernel (rbgp_mfma_reg_dual.hip): RegParams plus one table
// buffer in device memory laid out for few, wide loads (a wave reads it with 7 load instructions; 2048
// waves reading the same few KB with 25 narrow loads each is a burst of 50 000 load instructions at the
// head of every launch).  Measured alternatives for the 1.4 us between wave start and "tables there":
// tables inside the kernel arguments read by vector loads 1.6 us, by scalar loads 2.7 - 5 us (only the
// first bytes of the arguments arrive fast, 0.3 us); 16 copies of the buffer on different L2 channels
// 1.6 - 2.3 us (the one copy is fetched from memory once and then shared; it is not a hot spot).
struct DualParams {
  RegParams r;          // (rowtab / stages / counts / members are not used)
  const int32_t *tab;   // row table [a_i][4 lane groups][rt_stride] (stage-relative row of I of step 4 * o + g at [g][o]) first
  int rt_stride;        // NO rounded up to 4
  int cmax;             // stages stored per wave (>= the longest stage list)
  int o_stages;         // word offsets into tab of: stages [quad][x][y][cmax][4] (base row of I, position of L_x's
                        //   weight fragment, of H_y's, unused)
  int o_quads;          //   [quad][8]: L0, L1, H0, H1 (-1: none), then the stage counts of waves (0,0) (0,1) (1,0) (1,1)
};
}  // namespace rbgp_reg

typedef void (*rbgp_reg_fn)(rbgp_reg::RegParams);
typedef void (*rbgp_dual_fn)(rbgp_reg::DualParams);
// bf16 kernel for KC contraction steps per stage, RS weight rows per tile row, G 16-row
// groups per wave and CW (64 or 128) columns per wave; nullptr when that combination is not built.
rbgp_reg_fn rbgp_reg_bf16_kernel(int KC, int RS, int G, int CW);
// the same with one register set (two waves per SIMD); nullptr where that variant is not built
rbgp_reg_fn rbgp_reg_bf16_lean_kernel(int KC, int RS, int G, int CW);
// fp32 kernel with lo/hi pairing of the tile rows (8-row halves; tables of rbgp_reg_dual in the
// stages / counts / members fields); nullptr when KC is not built.
rbgp_dual_fn rbgp_reg_dual_kernel(int KC);

#endif
