// Gradient of the kept values of W_s for a fixed mask (Section 6: masks are predefined and stay
// fixed during training):  dW[m][t] = sum_n dO[m][n] * I[k][n]  for the t-th kept column k of
// row m -- the dense product dO x I^T sampled on the mask.
//
// MFMA kernel (RBGP4 masks covered by the register-streaming family).  The work unit is a nonzero
// tile column seen from the weights' side: for one column v_o of G_o, VC columns of G_r (a
// "stage" of the forward kernels) and one G_i vertex u_i, every tile row that has the tile (the
// co-adjacency list of v_o, e_o entries) owns a dense block of R kept rows x KCR contraction
// steps, and all these blocks together are ONE dense product: (e_o * R rows of dO) x (KCR rows
// of I)^T, contracted over the batch columns n.  Rows are grouped 16 at a time (MG = 16 / RS
// tile rows x RS rows, as in the forward kernels' MFMA groups), steps 16 at a time; a wave owns
// RB row groups x NB step groups (all of the stage) and a range of columns, so that every loaded
// row of I is used for RB * 16 rows of dO and vice versa.
// The operand layout of v_mfma_f32_16x16x4_f32 (four of them per 16-byte load, one per loaded
// column) and of v_mfma_f32_16x16x32_bf16 (one per load) is: lane l holds row l % 16 of the 16
// rows at column offset 4 (8 for bf16) * (l / 16).  Loading in that layout makes every group of
// four consecutive lanes touch four cache lines and runs at a third of the L1 rate, so the loads
// use a layout with 64 contiguous bytes per four lanes and the data passes through a wave-private
// LDS tile (one 16-byte write and one 16-byte read per lane and load) into the operand layout.
// (ds_bpermute, one per register, does the same without memory but costs 16 cycles each, which
// made the LDS crossbar the bound.)  The accumulators hold the 16 x 16 blocks of dW.  Rows that
// do not exist (list shorter than the row groups, R < RS, KCR not a multiple of 16) load some
// valid row instead and their results are dropped: an output element depends on its own two
// rows only.
// The batch is cut into ranges so that the chip is filled: the four waves of a workgroup take
// consecutive ranges and add their accumulators through LDS; several workgroups per unit write
// partial dW's and a second kernel adds those in a fixed order (reproducible sums).  (Letting
// the last workgroup of a unit add the partial sums instead needs device-scope fences, which on
// this chip write back and invalidate the L2 of the XCD: measured 2.5 times slower.)
//
// Plain kernel (any four-factor mask): one wave per kept value, lanes stride over n.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <new>
#include <vector>

#include "rbgp_internal.h"

#define RBGP_HIP(call)                                                          \
  do {                                                                          \
    hipError_t e_ = (call);                                                     \
    if (e_ != hipSuccess) {                                                     \
      char buf_[256];                                                           \
      std::snprintf(buf_, sizeof buf_, "%s: %s", #call, hipGetErrorString(e_)); \
      rbgp_set_hip_error(buf_);                                                 \
      return RBGP_EHIP;                                                         \
    }                                                                           \
  } while (0)

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef f32x4 f32x4_u __attribute__((aligned(4)));
typedef bf16x8 bf16x8_u __attribute__((aligned(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct SddmmParams {
  const void *dO, *I;
  float *out;               // [workgroups per unit][nnz] partial sums (dW itself when there is one)
  const int32_t *colrows;   // [c_o][EO]: tile rows that have tile column v_o, ascending
  const int32_t *colpos;    // [c_o][EO]: position of v_o in that tile row's adjacency list
  const int32_t *rowtab;    // [a_i][16 * NB]: stage-relative row of I of contraction step kk (padding -> 0)
  int64_t N, ld_dO, ldI, nnz;
  int64_t chunk;            // columns per range (a multiple of the columns per iteration)
  int EO, RBG;              // tile rows per tile column; groups of RB row groups per unit
  int nbt, halves;          // 16-step groups of a stage; workgroups that share them (each takes NB consecutive ones)
  int NSTG, stage_rows;     // stages per tile; rows of I between the bases of consecutive stages (VC * c_i * c_b)
  int tile_rows;            // rows of I per tile column (c_r * c_i * c_b)
  int a2, a3, a4, R, lgRS, MG, KCR, rowdeg;
  // "All of G_i" units (GI kernels): a unit is a (tile column, stage) and takes the rows of every G_i vertex
  // together -- 16-row groups run over (tile row of the list, u_i, row of R) -- against ALL rows of I the
  // stage spans, whether G_i connects them or not; the epilogue stores the kept products only.  For
  // masks with few rows per (tile column, u_i) (sparse G_o, small G_r, G_b) this fills the 16 MFMA rows
  // that would be padding, and every row of I is loaded once instead of once per adjacent u_i.
  int src_rows;             // gi: rows of I one stage spans (VC * c_i * c_b)
  const int32_t *spos;      // gi: [a_i][16 * NB]: position inside the stage's kept values of (u_i, stage row), -1: not kept
  // Fused 3x3 convolution (CONV kernels): I is not materialised; row k = 9 * channel + tap of it is read
  // from the zero-padded activations X[channel][image][H + 2][W + 2] (pointer I).
  const int32_t *colbase;   // element offset, inside a channel of X, of the first pixel of every group of
                            //   columns one lane loads (4 fp32 / 8 bf16), padded with valid offsets
  int64_t chan_elems;       // elements of one channel of X
  int64_t x_bytes;          // size of X
  int conv_w2;              // W + 2
};

template <bool BF16>
struct Operand;
template <>
struct Operand<false> {
  typedef f32x4 reg;
  static constexpr int CPL = 4;   // columns per lane and load
  static __device__ __forceinline__ reg zero() { return reg{0.f, 0.f, 0.f, 0.f}; }
  static __device__ __forceinline__ reg load(const void *base, int64_t elem) {
    return *reinterpret_cast<const f32x4_u *>(static_cast<const float *>(base) + elem);
  }
  static __device__ __forceinline__ reg load_tail(const void *base, int64_t elem, int valid) {
    const float *p = static_cast<const float *>(base) + elem;
    reg r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = e < valid ? p[e] : 0.f;
    return r;
  }
  typedef f32x4 accum;
  static __device__ __forceinline__ void mac(const reg &a, const reg &b, accum &acc) {
#pragma unroll
    for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t], acc, 0, 0, 0);
  }
  static __device__ __forceinline__ float total(const accum &acc, int i) { return acc[i]; }
};
template <>
struct Operand<true> {
  typedef bf16x8 reg;
  static constexpr int CPL = 8;
  static __device__ __forceinline__ reg zero() { return reg{0, 0, 0, 0, 0, 0, 0, 0}; }
  static __device__ __forceinline__ reg load(const void *base, int64_t elem) {
    return *reinterpret_cast<const bf16x8_u *>(static_cast<const uint16_t *>(base) + elem);
  }
  static __device__ __forceinline__ reg load_tail(const void *base, int64_t elem, int valid) {
    const uint16_t *p = static_cast<const uint16_t *>(base) + elem;
    union { reg v; uint16_t h[8]; } r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r.h[e] = e < valid ? p[e] : uint16_t(0);
    return r.v;
  }
  typedef f32x4 accum;
  static __device__ __forceinline__ void mac(const reg &a, const reg &b, accum &acc) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
  }
  static __device__ __forceinline__ float total(const accum &acc, int i) { return acc[i]; }
};

// RB: groups of 16 rows of dO per wave; NB: groups of 16 contraction steps per stage (KCR <= 16 * NB).
// grid.x = ((v_o * NSTG + stage) * a_i + u_i) * RBG + group of RB row groups; grid.y = workgroups
// along the batch.
template <int RB, int NB, bool BF16, bool CONV, bool GI>
__global__ __launch_bounds__(256) void sddmm_reg(SddmmParams p) {
  typedef Operand<BF16> Op;
  typedef typename Op::reg reg;
  constexpr int CPL = Op::CPL, CPI = 4 * CPL;   // columns per lane load / per iteration
  constexpr int NL = RB + NB;                   // loads per iteration
  __shared__ float red[4][RB * NB * 4][64];
  __shared__ u32x4 stage[4][NL][64];   // per wave: one 16 x 64-byte tile per load of an iteration
  const int lane = threadIdx.x & 63, j = lane & 15, q = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // load layout: lane l reads row l / 4 of the 16, 16-byte segment l % 4; operand layout: lane l
  // holds row l % 16, segment l / 16
  const int lr = lane >> 2, ls = lane & 3;
  // a tile in LDS: 16-byte slot 4 * row + (segment ^ ((row >> 1) & 3)); the exclusive-or spreads both
  // the writes (load layout) and the reads (operand layout) of eight consecutive lanes over all banks
  const int wslot = 4 * lr + (ls ^ ((lr >> 1) & 3)), rslot = 4 * j + (q ^ ((j >> 1) & 3));
  // Workgroups go to the eight XCDs round-robin in launch order, and each XCD has its own L2: the
  // a_i * RBG workgroups that share the rows of I of one (tile column, stage) take launch slots with
  // the same remainder modulo 8 (when the number of such groups is a multiple of 8).
  int x = blockIdx.x;
  const int per_group = (GI ? 1 : p.a3) * p.RBG * p.halves, groups = gridDim.x / per_group;
  if (groups % 8 == 0) {
    const int xcd = x % 8, slot = x / 8;
    x = ((slot / per_group) * 8 + xcd) * per_group + slot % per_group;
  }
  const int b0 = (x % p.halves) * NB; x /= p.halves;   // first 16-step group of this workgroup
  const int g = x % p.RBG; x /= p.RBG;
  int u3 = 0;
  if constexpr (!GI) { u3 = x % p.a3; x /= p.a3; }
  const int sg = x % p.NSTG, v1 = x / p.NSTG;
  const int RS = 1 << p.lgRS;
  const int32_t *crow = p.colrows + v1 * p.EO, *cpos = p.colpos + v1 * p.EO;
  const int base = v1 * p.tile_rows + sg * p.stage_rows;

  // row r16 of row group rb of this workgroup: (row of dO, or -1; its entry of the tile-row list; its u_i)
  struct RowOf { int64_t row; int entry, ui; };
  auto row_of = [&](int rb, int r16) {
    RowOf o{-1, 0, u3};
    int ri;
    if constexpr (GI) {
      const int rho = (g * RB + rb) * 16 + r16;
      ri = rho % p.R;
      o.ui = (rho / p.R) % p.a3;
      o.entry = rho / (p.R * p.a3);
    } else {
      o.entry = (g * RB + rb) * p.MG + (r16 >> p.lgRS);
      ri = r16 & (RS - 1);
    }
    if (o.entry < p.EO && ri < p.R)
      o.row = ((int64_t(crow[o.entry]) * p.a2 + ri / p.a4) * p.a3 + o.ui) * p.a4 + ri % p.a4;
    return o;
  };
  int64_t off[NL];   // element offset of this lane's 16 bytes in iteration 0: dO rows, then I rows
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int64_t row = row_of(rb, lr).row;
    off[rb] = (row < 0 ? 0 : row) * p.ld_dO + ls * CPL;
  }
#pragma unroll
  for (int b = 0; b < NB; ++b) {   // padding steps read row 0 of the stage
    const int sr = 16 * (b0 + b) + lr;
    const int k = base + (GI ? (sr < p.src_rows ? sr : 0) : (b0 + b < p.nbt ? p.rowtab[(u3 * p.nbt + b0 + b) * 16 + lr] : 0));
    if constexpr (CONV) {   // channel k / 9, tap k % 9 = 3 * (dy + 1) + (dx + 1): the shift of the tap inside the channel
      const int tap = k % 9;
      off[RB + b] = int64_t(k / 9) * p.chan_elems + (tap / 3 - 1) * p.conv_w2 + (tap % 3 - 1);
    } else {
      off[RB + b] = int64_t(k) * p.ldI + ls * CPL;
    }
  }
  // CONV: where this lane's group of columns starts inside a channel (columns are pixels in image order)
  auto pixel = [&](int64_t n) { return CONV ? int64_t(p.colbase[n / CPL + ls]) : n; };
  // CONV: the tap shifts leave the 16-byte loads of X aligned to an element only (2 bytes for bf16), so
  // they go through a buffer descriptor (any alignment, 32-bit byte offsets: X is below 2 GiB)
  constexpr int ES = BF16 ? 2 : 4;
  __amdgpu_buffer_rsrc_t xrsrc;
  if constexpr (CONV)
    xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.I), 0, int(p.x_bytes), 0x00020000);
  auto load_x = [&](int64_t elem) {
    return __builtin_bit_cast(reg, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, int(elem * ES), 0, 0));
  };
  // (`at`: pixel(n), looked up by the caller -- ahead of time inside the loop, where a lookup right before its use
  // would have to wait for every load in flight)
  auto load_all = [&](reg *r, int64_t n, int64_t at) {
#pragma unroll
    for (int i = 0; i < RB; ++i) r[i] = Op::load(p.dO, off[i] + n);
#pragma unroll
    for (int i = RB; i < NL; ++i) {
      if constexpr (CONV) r[i] = load_x(off[i] + at);
      else r[i] = Op::load(p.I, off[i] + at);
    }
  };
  // load layout -> operand layout through this wave's tiles (LDS instructions of one wave execute in order)
  auto transpose_all = [&](reg *d, const reg *r) {
#pragma unroll
    for (int i = 0; i < NL; ++i) stage[wave][i][wslot] = __builtin_bit_cast(u32x4, r[i]);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < NL; ++i) d[i] = __builtin_bit_cast(reg, stage[wave][i][rslot]);
    __builtin_amdgcn_wave_barrier();
  };
  typename Op::accum acc[RB][NB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int e = 0; e < int(sizeof(typename Op::accum) / sizeof(float)); ++e) acc[rb][b][e] = 0.f;
  auto mac_all = [&](const reg *o) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) Op::mac(o[rb], o[RB + b], acc[rb][b]);
  };

  const int64_t n_lo = (int64_t(blockIdx.y) * 4 + wave) * p.chunk;
  const int64_t n_hi = n_lo + p.chunk < p.N ? n_lo + p.chunk : p.N;   // (n_lo may lie past N: empty range)
  int64_t n = n_lo;
  const int64_t iters = n_hi > n_lo ? (n_hi - n_lo) / CPI : 0;   // whole iterations
  if (iters > 0) {
    // In flight: the global loads of iterations k + 1 .. k + D - 1 (a ring of D register sets), the
    // permutation of iteration k, the MFMAs of k - 1.  One loop body fills, runs and drains the
    // pipeline, so that the distance between a load and its use is the same on every path into
    // the loop, and it has no branch, so that the permutations and loads are issued between the
    // MFMAs: steps that have nothing to multiply (k = 0, and k > iters when the loop overshoots)
    // multiply zeros.  Past the last iteration the loads repeat the last one (in bounds).
    constexpr int D = 3;
    // iterations in ascending column order: the two 64-byte halves of a cache line are consumed by
    // consecutive iterations, while the line is still in the L1
    const int64_t n_last = n_lo + (iters - 1) * CPI;
    auto column = [&](int64_t k) {
      const int64_t c = n_lo + k * CPI;
      return c < n_last ? c : n_last;
    };
    reg raw[D][NL], cur[NL], nxt[NL];
    int64_t at_next[D];   // pixel(column(k + D)) of the step that refills set d next, requested one round earlier
#pragma unroll
    for (int d = 0; d < D; ++d) load_all(raw[d], column(d), pixel(column(d)));
#pragma unroll
    for (int d = 0; d < D; ++d) at_next[d] = pixel(column(D + d));
#pragma unroll
    for (int i = 0; i < NL; ++i) cur[i] = Op::zero();
    for (int64_t k0 = 0; k0 <= iters; k0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const int64_t k = k0 + d;
        transpose_all(nxt, raw[d]);
        const int64_t at = at_next[d];
        at_next[d] = pixel(column(k + 2 * D));
        load_all(raw[d], column(k + D), at);
        mac_all(cur);
        const bool live = k < iters;   // nxt holds iteration k
#pragma unroll
        for (int i = 0; i < RB; ++i) cur[i] = live ? nxt[i] : Op::zero();
#pragma unroll
        for (int i = RB; i < NL; ++i) cur[i] = nxt[i];
        // issue order of this step: LDS writes and reads, then the loads, spread behind the MFMAs
        constexpr int M = RB * NB * (BF16 ? 1 : 4), DS = NL * 2, VM = NL;
        constexpr int Md = M >= 4 ? (M * 3) / 4 : M, Mv = M - Md;
        constexpr int dsq = (DS + Md - 1) / Md, vmq = Mv ? (VM + Mv - 1) / Mv : VM;
#pragma unroll
        for (int mi = 0; mi < M; ++mi) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                      // MFMA
          if (mi < Md) __builtin_amdgcn_sched_group_barrier(0x080, dsq, 0);       // LDS
          else __builtin_amdgcn_sched_group_barrier(0x020, vmq, 0);               // global loads
        }
        if (Mv == 0) __builtin_amdgcn_sched_group_barrier(0x020, vmq, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    n = n_lo + iters * CPI;
  }
  if (n < n_hi) {   // ragged end of the batch: columns at and past n_hi count as zero on both sides
    const int64_t left = n_hi - (n + ls * CPL);
    const int valid = left <= 0 ? 0 : left >= CPL ? CPL : int(left);
    reg r[NL], o[NL];
#pragma unroll
    for (int i = 0; i < RB; ++i) r[i] = Op::load_tail(p.dO, off[i] + n, valid);
    const int64_t at = pixel(n);   // (CONV: N is a multiple of the group, so `valid` is all or nothing)
#pragma unroll
    for (int i = RB; i < NL; ++i) {
      if constexpr (CONV) r[i] = valid ? load_x(off[i] + at) : Op::zero();
      else r[i] = Op::load_tail(p.I, off[i] + at, valid);
    }
    transpose_all(o, r);
    mac_all(o);
  }

  // acc[rb][b][i] = dW block element (row 4 * q + i of row group rb, contraction step 16 * b + j);
  // after the exchange wave w holds the sums for i == w
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) red[wave][(rb * NB + b) * 4 + i][lane] = Op::total(acc[rb][b], i);
  __syncthreads();
  const int r16 = 4 * q + wave;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const RowOf o = row_of(rb, r16);
    if (o.row < 0) continue;
    // the stage is fragment cpos * NSTG + sg of the row: KCR consecutive kept values
    float *dst = p.out + int64_t(blockIdx.y) * p.nnz + o.row * p.rowdeg + int64_t(cpos[o.entry] * p.NSTG + sg) * p.KCR;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int e = (rb * NB + b) * 4 + wave;
      // contraction step of this lane's column: 16 * b + j, or (gi) wherever G_i puts stage row 16 * b + j for u_i
      const int st = 16 * (b0 + b) + j;
      const int kk = b0 + b >= p.nbt ? -1 : GI ? p.spos[o.ui * p.nbt * 16 + st] : (st < p.KCR ? st : -1);
      const float v = (red[0][e][lane] + red[1][e][lane]) + (red[2][e][lane] + red[3][e][lane]);
      if (kk >= 0) dst[kk] = v;
    }
  }
}

__global__ __launch_bounds__(256) void sddmm_reduce(const float *__restrict__ part, float *__restrict__ dW,
                                                    int64_t nnz, int nsplit) {
  const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= nnz) return;
  float s = 0.f;
  for (int k = 0; k < nsplit; ++k) s += part[int64_t(k) * nnz + i];   // fixed order
  dW[i] = s;
}

__global__ __launch_bounds__(256) void sddmm_zero(float *__restrict__ dW, int64_t nnz) {
  const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < nnz) dW[i] = 0.f;
}

struct GenericParams {
  const int32_t *adj[4];
  int a[4], c[4], d[4];
  int64_t N, ld_dO, ldI, nnz;
  int rowdeg;
};

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(uint16_t x) { return __uint_as_float(uint32_t(x) << 16); }

template <typename TIn>
__global__ __launch_bounds__(256) void sddmm_generic(GenericParams p, const TIn *__restrict__ dO,
                                                     const TIn *__restrict__ I, float *__restrict__ dW) {
  const int lane = threadIdx.x & 63;
  for (int64_t idx = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6); idx < p.nnz; idx += int64_t(gridDim.x) * 4) {
    const int64_t m = idx / p.rowdeg;
    int t = int(idx % p.rowdeg);
    int64_t r = m;
    const int u3 = int(r % p.a[3]); r /= p.a[3];
    const int u2 = int(r % p.a[2]); r /= p.a[2];
    const int u1 = int(r % p.a[1]); r /= p.a[1];
    const int u0 = int(r);
    const int j3 = t % p.d[3]; t /= p.d[3];
    const int j2 = t % p.d[2]; t /= p.d[2];
    const int j1 = t % p.d[1]; t /= p.d[1];
    const int j0 = t;
    int64_t k = p.adj[0][u0 * p.d[0] + j0];
    k = k * p.c[1] + p.adj[1][u1 * p.d[1] + j1];
    k = k * p.c[2] + p.adj[2][u2 * p.d[2] + j2];
    k = k * p.c[3] + p.adj[3][u3 * p.d[3] + j3];
    const TIn *a = dO + m * p.ld_dO, *b = I + k * p.ldI;
    float acc = 0.f;
    for (int64_t n = lane; n < p.N; n += 64) acc = __builtin_fmaf(to_f32(a[n]), to_f32(b[n]), acc);
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) acc += __shfl_xor(acc, sh, 64);
    if (lane == 0) dW[idx] = acc;
  }
}

struct SddmmState {
  int32_t *colrows = nullptr, *colpos = nullptr, *rowtab = nullptr, *spos = nullptr;
  int EO = 0;
  float *partial = nullptr;
  size_t partial_bytes = 0;
  int32_t *colbase[2] = {nullptr, nullptr};           // fused convolution, fp32 / bf16 groups
  int64_t conv_key[2][3] = {{0, 0, 0}, {0, 0, 0}};    // images, height, width of colbase
};

template <typename T>
int upload(const std::vector<T> &h, T **d) {
  RBGP_HIP(hipMalloc(reinterpret_cast<void **>(d), h.size() * sizeof(T) + 16));
  RBGP_HIP(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
  return RBGP_OK;
}

typedef void (*sddmm_fn)(SddmmParams);
template <int RB, bool BF16, bool CONV, bool GI>
sddmm_fn pick_nb(int NB) {
  switch (NB) {
    case 1: return sddmm_reg<RB, 1, BF16, CONV, GI>;
    case 2: return sddmm_reg<RB, 2, BF16, CONV, GI>;
    case 3: return sddmm_reg<RB, 3, BF16, CONV, GI>;
    case 4: return sddmm_reg<RB, 4, BF16, CONV, GI>;
    case 5: return sddmm_reg<RB, 5, BF16, CONV, GI>;
  }
  return nullptr;
}
template <bool CONV, bool GI>
sddmm_fn find_kernel(int RB, int NB, bool bf16) {
  switch (RB) {
    case 1: return bf16 ? pick_nb<1, true, CONV, GI>(NB) : pick_nb<1, false, CONV, GI>(NB);
    case 2: return bf16 ? pick_nb<2, true, CONV, GI>(NB) : pick_nb<2, false, CONV, GI>(NB);
  }
  return nullptr;
}

// Host tables of the MFMA kernel.
struct SddmmHostTables {
  std::vector<int32_t> colrows, colpos, rt, sp;
  int EO = 0;
};

void make_host_tables(const rbgp_mask *m, SddmmHostTables *h) {
  const rbgp_reg_plan &pl = m->reg;
  const int NB = (pl.KCR + 15) / 16;
  // co-adjacency of the tile rows: tile row u has the tiles of G_o's row u / fold
  const int c1 = m->c[0], d1 = m->d[0], EO = m->e[0] * pl.fold;
  h->colrows.assign(size_t(c1) * EO, 0);
  h->colpos.assign(size_t(c1) * EO, 0);
  std::vector<int> fill(size_t(c1), 0);
  for (int u = 0; u < pl.TR; ++u)
    for (int jj = 0; jj < d1; ++jj) {
      const int v = m->adj[0][size_t(u / pl.fold) * d1 + jj];
      h->colrows[size_t(v) * EO + fill[size_t(v)]] = u;
      h->colpos[size_t(v) * EO + fill[size_t(v)]++] = jj;
    }
  const int a3 = m->a[2], d3 = m->d[2], c3 = m->c[2], c4 = m->c[3];
  h->rt.assign(size_t(a3) * NB * 16, 0);
  for (int u3 = 0; u3 < a3; ++u3)
    for (int kk = 0; kk < pl.KCR; ++kk) {
      const int v4 = kk % c4, j3 = (kk / c4) % d3, vv = kk / (c4 * d3);
      h->rt[(size_t(u3) * NB) * 16 + kk] = (vv * c3 + m->adj[2][size_t(u3) * d3 + j3]) * c4 + v4;
    }
  // "all of G_i" units: where G_i puts every row of a stage, per u_i
  const int NBG = (pl.SRC + 15) / 16;
  h->sp.assign(size_t(a3) * NBG * 16, -1);
  for (int u3 = 0; u3 < a3; ++u3)
    for (int j3 = 0; j3 < d3; ++j3)
      for (int vv = 0; vv < pl.VC; ++vv)
        for (int v4 = 0; v4 < c4; ++v4)
          h->sp[size_t(u3) * NBG * 16 + (size_t(vv) * c3 + m->adj[2][size_t(u3) * d3 + j3]) * c4 + v4] = (vv * d3 + j3) * c4 + v4;
  h->EO = EO;
}

// The state is touched only when every table is on the device.
int build_state(const rbgp_mask *m, SddmmState *st) {
  SddmmHostTables h;
  make_host_tables(m, &h);
  int32_t *colrows = nullptr, *colpos = nullptr, *rowtab = nullptr, *spos = nullptr;
  int rc = upload(h.colrows, &colrows);
  if (!rc) rc = upload(h.colpos, &colpos);
  if (!rc) rc = upload(h.rt, &rowtab);
  if (!rc) rc = upload(h.sp, &spos);
  if (rc) {
    if (colrows) (void)hipFree(colrows);
    if (colpos) (void)hipFree(colpos);
    if (rowtab) (void)hipFree(rowtab);
    if (spos) (void)hipFree(spos);
    return rc;
  }
  st->colrows = colrows; st->colpos = colpos; st->rowtab = rowtab; st->spos = spos;
  st->EO = h.EO;
  return RBGP_OK;
}

// What a launch reads and writes besides the caller's buffers: the index tables and the partial sums,
// in memory of the mask's state (rbgp_sddmm) or in the static scratch array (rbgp_sddmm_static).
struct SddmmBuffers {
  const int32_t *adj[4] = {nullptr, nullptr, nullptr, nullptr};   // plain kernel
  const int32_t *colrows = nullptr, *colpos = nullptr, *rowtab = nullptr, *spos = nullptr;   // MFMA kernel
  int EO = 0;
  float *partial = nullptr;
  size_t partial_bytes = 0;
  SddmmState *grow = nullptr;   // may enlarge `partial` with hipMalloc (nullptr: a larger need is RBGP_ETOOLARGE)
};

// Allocation-free variant: everything above lives in this array, per GPU.
constexpr size_t kStaticTableBytes = size_t(256) << 10;
constexpr size_t kStaticPartialBytes = size_t(16) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticTableBytes + kStaticPartialBytes];
constexpr int kMaxDevices = 64;
struct StaticSlot {
  unsigned char *ptr = nullptr;   // device address of `scratch` on this GPU
  uint64_t key = 0;               // uid of the mask whose tables the array holds (0: none)
};
StaticSlot g_static[kMaxDevices];

// Tables reach the array as kernel arguments, a chunk per launch: no staging copy, nothing allocated.
struct ArgChunk {
  int32_t v[960];
};
__global__ __launch_bounds__(256) void table_write(ArgChunk c, int32_t *__restrict__ dst, int n) {
  for (int i = threadIdx.x; i < n; i += 256) dst[i] = c.v[i];
}

}  // namespace

void rbgp_sddmm_release(void *state) {
  SddmmState *st = static_cast<SddmmState *>(state);
  if (!st) return;
  if (st->colrows) (void)hipFree(st->colrows);
  if (st->colpos) (void)hipFree(st->colpos);
  if (st->rowtab) (void)hipFree(st->rowtab);
  if (st->spos) (void)hipFree(st->spos);
  if (st->partial) (void)hipFree(st->partial);
  for (int32_t *t : st->colbase)
    if (t) (void)hipFree(t);
  delete st;
}

namespace {

int launch_core(const rbgp_mask *m, SddmmBuffers &B, SddmmState *st, bool use_mfma, bool bf16, int64_t N, const void *dO,
                int64_t ld_dO, const void *I, int64_t ldI, float *dW, hipStream_t hs, const rbgp_conv_geometry *conv) {
  const int64_t nnz = m->nnz;
  if (N == 0) {
    sddmm_zero<<<dim3(unsigned((nnz + 255) / 256)), dim3(256), 0, hs>>>(dW, nnz);
    RBGP_HIP(hipGetLastError());
    return RBGP_OK;
  }
  if (!use_mfma) {
    GenericParams gp;
    for (int i = 0; i < 4; ++i) {
      gp.adj[i] = B.adj[i];
      gp.a[i] = m->a[i]; gp.c[i] = m->c[i]; gp.d[i] = m->d[i];
    }
    gp.N = N; gp.ld_dO = ld_dO; gp.ldI = ldI; gp.nnz = nnz; gp.rowdeg = int(m->rowdeg);
    const int64_t blocks = std::min<int64_t>((nnz + 3) / 4, 1 << 20);
    if (bf16)
      sddmm_generic<uint16_t><<<dim3(unsigned(blocks)), dim3(256), 0, hs>>>(
          gp, static_cast<const uint16_t *>(dO), static_cast<const uint16_t *>(I), dW);
    else
      sddmm_generic<float><<<dim3(unsigned(blocks)), dim3(256), 0, hs>>>(gp, static_cast<const float *>(dO),
                                                                        static_cast<const float *>(I), dW);
    RBGP_HIP(hipGetLastError());
    return RBGP_OK;
  }

  const rbgp_reg_plan &pl = m->reg;
  // row groups of 16 (MG tile rows) per tile column and u_i, RB of them per wave: two row groups per wave
  // halve the rows of I fetched per MFMA; four would starve the chip of waves at the layer sizes of
  // the paper (measured: slower on every VGG19 / WRN shape tried)
  int NB = (pl.KCR + 15) / 16;
  int groups = (B.EO + pl.MG - 1) / pl.MG;
  int RB = groups >= 2 ? 2 : 1;
  int RBG = (groups + RB - 1) / RB;
  // or "all of G_i" units, where they need fewer MFMAs per column of the batch
  const int gi_groups = (B.EO * m->a[2] * pl.R + 15) / 16, gi_NB = (pl.SRC + 15) / 16;
  const int gi_RB = gi_groups >= 2 ? 2 : 1, gi_RBG = (gi_groups + gi_RB - 1) / gi_RB;
  const bool gi = gi_NB <= 5 && gi_RBG * gi_RB * gi_NB < m->a[2] * RBG * RB * NB;
  if (gi) { NB = gi_NB; groups = gi_groups; RB = gi_RB; RBG = gi_RBG; }
  const int nbt = NB;
  // ranges of the batch: enough waves for a few per SIMD (1024 SIMDs), at least two iterations each
  const int cpi = bf16 ? 32 : 16;
  int64_t blocks = int64_t(m->c[0]) * pl.NSTG * (gi ? 1 : m->a[2]) * RBG;
  // Where one wave per SIMD would need five to eight column ranges per unit, i.e. two workgroups and the
  // second kernel that adds their partial sums, two workgroups that split the stage's 16-step groups
  // instead need neither (conv5 shape: 24.4 -> 22.5 us fp32, 13.7 -> 11.0 us bf16; the fused-convolution
  // variant, whose loads of X cost more, is slower that way and keeps whole stages).
  int halves = 1;
  if (!conv && NB >= 4 && blocks * 4 < 1024 && blocks * 8 >= 1024 && N >= 8 * 2 * cpi) {
    halves = 2;
    NB = (NB + 1) / 2;
    blocks *= 2;
  }
  sddmm_fn fn = conv ? (gi ? find_kernel<true, true>(RB, NB, bf16) : find_kernel<true, false>(RB, NB, bf16))
                     : (gi ? find_kernel<false, true>(RB, NB, bf16) : find_kernel<false, false>(RB, NB, bf16));
  if (!fn) return RBGP_EUNSUPPORTED;
  // one wave per SIMD (1024 SIMDs): longer ranges amortise the fill of the load pipeline and keep
  // the partial sums few; more waves per SIMD measured slower
  int64_t ranges = (1024 + blocks - 1) / blocks;                         // column ranges = waves per unit
  ranges = std::max<int64_t>(1, std::min(ranges, (N + 2 * cpi - 1) / (2 * cpi)));
  ranges = std::min<int64_t>((ranges + 3) / 4 * 4, 4096);                // four per workgroup
  const int64_t chunk = ((N + ranges - 1) / ranges + cpi - 1) / cpi * cpi;
  const int64_t nsplit = ((N + chunk - 1) / chunk + 3) / 4;              // workgroups per unit = partial sums
  if (nsplit > 1) {
    const size_t need = size_t(nsplit) * size_t(nnz) * sizeof(float);
    if (B.partial_bytes < need) {
      if (!B.grow) return RBGP_ETOOLARGE;
      SddmmState *g = B.grow;
      if (g->partial) RBGP_HIP(hipFree(g->partial));   // (waits for launches that still use it)
      g->partial = nullptr;
      g->partial_bytes = 0;
      RBGP_HIP(hipMalloc(reinterpret_cast<void **>(&g->partial), need));
      g->partial_bytes = need;
      B.partial = g->partial;
      B.partial_bytes = need;
    }
  }
  SddmmParams p;
  p.colbase = nullptr; p.chan_elems = 0; p.conv_w2 = 0; p.x_bytes = 0;
  if (conv) {
    const int64_t H = conv->height, W = conv->width, grp = bf16 ? 8 : 4;
    int64_t *key = st->conv_key[bf16];
    int32_t **cb = &st->colbase[bf16];
    if (*cb && (key[0] != conv->images || key[1] != H || key[2] != W)) {
      RBGP_HIP(hipFree(*cb));   // (waits for launches that still read the old table)
      *cb = nullptr;
    }
    if (!*cb) {
      // one entry per group of columns (pixels n .. n + grp - 1 of one image row), then enough valid
      // entries for the lanes of a last, partly empty iteration
      std::vector<int32_t> h(size_t((N + grp - 1) / grp + 8), int32_t(W + 3));
      for (int64_t n = 0; n < N; n += grp) {
        const int64_t img = n / (H * W), y = (n % (H * W)) / W, x = n % W;
        h[size_t(n / grp)] = int32_t((img * (H + 2) + y + 1) * (W + 2) + x + 1);
      }
      int rc = upload(h, cb);
      if (rc) return rc;
      key[0] = conv->images; key[1] = H; key[2] = W;
    }
    p.colbase = *cb;
    p.chan_elems = conv->images * (H + 2) * (W + 2);
    p.conv_w2 = int(W + 2);
    p.x_bytes = p.chan_elems * (m->K / 9) * (bf16 ? 2 : 4);
    if (p.x_bytes >= (int64_t(1) << 31)) return RBGP_EUNSUPPORTED;
  }
  p.dO = dO; p.I = I;
  p.out = nsplit > 1 ? B.partial : dW;
  p.colrows = B.colrows; p.colpos = B.colpos; p.rowtab = B.rowtab;
  p.N = N; p.ld_dO = ld_dO; p.ldI = ldI; p.nnz = nnz; p.chunk = chunk;
  p.src_rows = pl.SRC; p.spos = B.spos;
  p.nbt = nbt; p.halves = halves;
  p.EO = B.EO; p.RBG = RBG; p.NSTG = pl.NSTG; p.stage_rows = pl.SRC;
  p.tile_rows = m->c[1] * m->c[2] * m->c[3];
  p.a2 = pl.A2; p.a3 = m->a[2]; p.a4 = m->a[3]; p.R = pl.R;
  p.lgRS = 0;
  while ((1 << p.lgRS) < pl.RS) ++p.lgRS;
  p.MG = pl.MG; p.KCR = pl.KCR; p.rowdeg = int(m->rowdeg);
  fn<<<dim3(unsigned(blocks), unsigned(nsplit)), dim3(256), 0, hs>>>(p);
  RBGP_HIP(hipGetLastError());
  if (nsplit > 1) {
    sddmm_reduce<<<dim3(unsigned((nnz + 255) / 256)), dim3(256), 0, hs>>>(B.partial, dW, nnz, int(nsplit));
    RBGP_HIP(hipGetLastError());
  }
  return RBGP_OK;
}

}  // namespace

int rbgp_sddmm_launch(const rbgp_mask *m, void **state, const int32_t *const dev_adj[4], bool use_mfma, bool bf16,
                      int64_t N, const void *dO, int64_t ld_dO, const void *I, int64_t ldI, float *dW, void *stream,
                      const rbgp_conv_geometry *conv) {
  if (conv && !use_mfma) return RBGP_EUNSUPPORTED;
  SddmmBuffers B;
  SddmmState *st = nullptr;
  for (int i = 0; i < 4; ++i) B.adj[i] = dev_adj[i];
  if (use_mfma && N > 0) {
    st = static_cast<SddmmState *>(*state);
    if (!st) {
      st = new (std::nothrow) SddmmState();
      if (!st) return RBGP_ENOMEM;
      *state = st;
    }
    if (!st->colrows) {
      int rc = build_state(m, st);
      if (rc) return rc;
    }
    B.colrows = st->colrows; B.colpos = st->colpos; B.rowtab = st->rowtab; B.spos = st->spos;
    B.EO = st->EO;
    B.partial = st->partial; B.partial_bytes = st->partial_bytes;
    B.grow = st;
  }
  return launch_core(m, B, st, use_mfma, bf16, N, dO, ld_dO, I, ldI, dW, static_cast<hipStream_t>(stream), conv);
}

int rbgp_sddmm_static_launch(const rbgp_mask *m, bool use_mfma, bool bf16, int64_t N, const void *dO, int64_t ld_dO,
                             const void *I, int64_t ldI, float *dW, void *stream) {
  hipStream_t hs = static_cast<hipStream_t>(stream);
  int dev = -1;
  RBGP_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return RBGP_EUNSUPPORTED;
  StaticSlot &slot = g_static[dev];
  if (!slot.ptr) {   // once per GPU: the address of this GPU's copy of the array
    unsigned char *p = nullptr;
    RBGP_HIP(hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch)));
    if (!p) return RBGP_EHIP;
    slot.ptr = p;
  }
  SddmmBuffers B;
  if (N > 0) {
    // table area: the four adjacency lists (plain kernel) or the MFMA kernel's four tables, 16-byte aligned
    std::vector<int32_t> all;
    size_t off[4] = {0, 0, 0, 0};
    try {
      SddmmHostTables h;
      if (use_mfma) make_host_tables(m, &h);
      const std::vector<int32_t> *src[4] = {use_mfma ? &h.colrows : &m->adj[0], use_mfma ? &h.colpos : &m->adj[1],
                                            use_mfma ? &h.rt : &m->adj[2], use_mfma ? &h.sp : &m->adj[3]};
      for (int i = 0; i < 4; ++i) {
        off[i] = all.size();
        all.insert(all.end(), src[i]->begin(), src[i]->end());
        all.resize((all.size() + 3) / 4 * 4, 0);
      }
      B.EO = h.EO;
    } catch (const std::bad_alloc &) {
      return RBGP_ENOMEM;
    }
    if (all.size() * sizeof(int32_t) > kStaticTableBytes) return RBGP_ETOOLARGE;
    int32_t *tab = reinterpret_cast<int32_t *>(slot.ptr);
    const uint64_t key = m->uid * 2 + (use_mfma ? 1 : 0);
    if (slot.key != key) {
      slot.key = 0;
      for (size_t at = 0; at < all.size(); at += 960) {
        ArgChunk c;
        const int n = int(std::min<size_t>(960, all.size() - at));
        std::copy(all.begin() + at, all.begin() + at + n, c.v);
        table_write<<<dim3(1), dim3(256), 0, hs>>>(c, tab + at, n);
        RBGP_HIP(hipGetLastError());
      }
      slot.key = key;
    }
    if (use_mfma) {
      B.colrows = tab + off[0]; B.colpos = tab + off[1]; B.rowtab = tab + off[2]; B.spos = tab + off[3];
    } else {
      for (int i = 0; i < 4; ++i) B.adj[i] = tab + off[i];
    }
    B.partial = reinterpret_cast<float *>(slot.ptr + kStaticTableBytes);
    B.partial_bytes = kStaticPartialBytes;
  }
  return launch_core(m, B, nullptr, use_mfma, bf16, N, dO, ld_dO, I, ldI, dW, hs, nullptr);
}
