// Register-streaming MFMA kernel for O = W_s x I (Section 5, "GPU Implementation"),
// bf16 inputs with fp32 accumulation: v_mfma_f32_16x16x16_bf16.
//
// Same walk as the fp32 kernel (tile skipping through G_o's adjacency, row repetition
// over the R rows that share a column set, one G_i vertex per wave), with two changes
// that follow from bf16 on this chip being bound by the load path, not the matrix core:
//
//  * A wave owns G 16-row MFMA groups (G * 16/RS tile rows), not one.  Every row of I it
//    loads is multiplied into all of them, so I crosses the L1 path 1/G as often; a tile
//    row that lacks the tile multiplies zeros, which the bf16 matrix core has room for.
//  * The stage list of a cluster can be split over S = 1, 2 or 4 waves of the workgroup
//    (wave k takes stages k, k + S, ...), which keeps the chip full when larger clusters
//    leave fewer independent (cluster, column tile) pairs; the partial sums meet in LDS.
//
// The matrix core wants, per lane, four consecutive contraction steps of ONE column, while
// I holds consecutive columns of one row.  A lane therefore loads 8 bytes (columns 4j..4j+3)
// from each of its four rows (contraction steps 16kb + 4kg .. +3 of k-block kb, kg = lane/16)
// and transposes the 4x4 block of bf16 in registers (8 v_perm_b32), which yields the B
// operands of four MFMAs (one per column offset w), shared by all G groups.  The weights
// are packed k-major by rbgp_pack, so an A operand is an 8-byte piece of a 16-byte load.
#include <hip/hip_runtime.h>

#include "rbgp_reg_common.h"

using namespace rbgp_reg;

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ u32x2 load_x2(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
  return __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
}
__device__ __forceinline__ u32x4 load_u4(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
}
__device__ __forceinline__ s16x4 as_s16x4(unsigned lo, unsigned hi) {
  u32x2 v = {lo, hi};
  return __builtin_bit_cast(s16x4, v);
}

template <int KC, int RS, int G>
__global__ __launch_bounds__(256) void spmm_reg_bf16(RegParams p) {
  constexpr int MG = 16 / RS;            // tile rows per 16-row group
  constexpr int U = G * MG;              // tile rows per cluster
  constexpr int NKB = (KC + 15) / 16;    // k-blocks (16 contraction steps) per stage
  constexpr int NQ = (NKB + 1) / 2;      // weights of two k-blocks come as one 16-byte load
  constexpr int QB = 4 * RS * 16;        // bytes of one such load across the fragment
  constexpr int FB = NQ * QB;            // bytes of one weight fragment
  constexpr int CW = 64;
  extern __shared__ __attribute__((aligned(16))) unsigned char red[];   // [wave][G*4 units][64 lanes] x 16 B
  const int lane = threadIdx.x & 63;
  const int wid = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  const int lgS = p.lgS, S = 1 << lgS;
  const int ks = wid & (S - 1);          // this wave's share of the stage list
  // workgroup -> (XCD, cluster, G_i vertex, 4/S neighbouring column tiles); see the fp32 kernel
  const int xcd = blockIdx.x & 7, cl = blockIdx.x >> 3, u3 = blockIdx.y;
  const int nt = ((xcd + 8 * int(blockIdx.z)) << (2 - lgS)) + (wid >> lgS);
  const bool valid = nt < p.ntiles;
  if (lgS == 0 && !valid) return;        // (with S > 1 every wave reaches the barrier below)
  const int64_t n0 = int64_t(nt) * CW;
  const int kg = lane >> 4, j = lane & 15;
  const int mi = j / RS, ri = j % RS;

  int mem[U];
#pragma unroll
  for (int mm = 0; mm < U; ++mm) mem[mm] = p.members[cl * U + mm];
  const int32_t *rt = p.rowtab + u3 * (NKB * 16) + kg * 4;
  int rrow[NKB][4];
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int t = 0; t < 4; ++t) rrow[kb][t] = rt[kb * 16 + t];
  const int32_t *stg = p.stages + int64_t(cl) * (1 + U) * 64 + lane;
  const int tb = stg[0];
  int tf[U];
#pragma unroll
  for (int mm = 0; mm < U; ++mm) tf[mm] = stg[(1 + mm) * 64];
  const int cnt = p.counts[cl];
  const int cntw = cnt > ks ? (cnt - ks + S - 1) >> lgS : 0;   // stages of this wave
  const int rov = p.rowofs[lane & 15];   // lane-held copies, read back with bpermute in the epilogue
  const int memv = p.members[cl * U + (lane & (U - 1))];

  // byte offset of this lane's 8 bytes (4 bf16 columns) in each of its rows, relative to the stage base
  int off[NKB][4];
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int t = 0; t < 4; ++t) off[kb][t] = rrow[kb][t] * (int(p.ldI) * 2) + j * 8;
  const int alane = (kg * RS + ri) * 16;

  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void *>(static_cast<const void *>(p.Wp)), 0, p.w_bytes, kRsrcFlags);
  // table lane of the wave's s-th stage; lanes past the cluster's count hold sentinels
  // (base row -1 -> a descriptor of zero extent: zeros, no memory access)
  auto table_lane = [&](int s) {
    const int gs = ks + (s << lgS);
    return gs < 63 ? gs : 63;
  };
  auto b_rsrc = [&](int tl, int *sofs) {
    const int base_row = __builtin_amdgcn_readlane(tb, tl);
    *sofs = int((int64_t(base_row < 0 ? 0 : base_row) * p.ldI + n0) * 2);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(static_cast<const void *>(p.I)), 0,
                                             (base_row >= 0 && valid) ? p.i_bytes : 0u, kRsrcFlags);
  };
  // per-lane byte offset of the stage's weights for group gi; a tile row that lacks the tile
  // reads past the end of the packed buffer, which returns zeros
  auto a_addr = [&](int tl, int gi) {
    int addr = 0;
#pragma unroll
    for (int mm = 0; mm < MG; ++mm) {
      const int fi = __builtin_amdgcn_readlane(tf[gi * MG + mm], tl);
      const int u1 = mem[gi * MG + mm];
      const int sv = (fi >= 0 && u1 >= 0) ? ((u1 * p.fpm + fi) * p.a3 + u3) * FB : kOob;
      addr = mi == mm ? sv : addr;
    }
    return addr + alane;
  };
  __builtin_amdgcn_s_waitcnt(0);   // drain the table loads outside the loop (see the fp32 kernel)

  f32x4 acc[G][4];
#pragma unroll
  for (int gi = 0; gi < G; ++gi)
#pragma unroll
    for (int w = 0; w < 4; ++w) acc[gi][w] = f32x4{0.f, 0.f, 0.f, 0.f};

  // the MFMAs of one k-block: transpose the lane's 4x4 block of bf16, then per group one MFMA
  // per column offset
  auto kblock = [&](const u32x2 (&raw)[4], const u32x4 (&A)[G][NQ], int q, int half) {
    const unsigned x01l = __builtin_amdgcn_perm(raw[1][0], raw[0][0], 0x05040100u);
    const unsigned x23l = __builtin_amdgcn_perm(raw[3][0], raw[2][0], 0x05040100u);
    const unsigned x01h = __builtin_amdgcn_perm(raw[1][0], raw[0][0], 0x07060302u);
    const unsigned x23h = __builtin_amdgcn_perm(raw[3][0], raw[2][0], 0x07060302u);
    const unsigned y01l = __builtin_amdgcn_perm(raw[1][1], raw[0][1], 0x05040100u);
    const unsigned y23l = __builtin_amdgcn_perm(raw[3][1], raw[2][1], 0x05040100u);
    const unsigned y01h = __builtin_amdgcn_perm(raw[1][1], raw[0][1], 0x07060302u);
    const unsigned y23h = __builtin_amdgcn_perm(raw[3][1], raw[2][1], 0x07060302u);
    const s16x4 b0 = as_s16x4(x01l, x23l), b1 = as_s16x4(x01h, x23h);
    const s16x4 b2 = as_s16x4(y01l, y23l), b3 = as_s16x4(y01h, y23h);
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
      const s16x4 a = half ? as_s16x4(A[gi][q][2], A[gi][q][3]) : as_s16x4(A[gi][q][0], A[gi][q][1]);
      acc[gi][0] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b0, acc[gi][0], 0, 0, 0);
      acc[gi][1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b1, acc[gi][1], 0, 0, 0);
      acc[gi][2] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b2, acc[gi][2], 0, 0, 0);
      acc[gi][3] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b3, acc[gi][3], 0, 0, 0);
    }
  };

  // One stage: every k-block's rows of I and every pair of k-blocks' weights are refilled for
  // the wave's stage s + 2 right after their last use, so about two stages of loads are in
  // flight; the loop body is branch-free and its wait counts are exact.
  auto stage = [&](int s, u32x2 (&B)[NKB][4], u32x4 (&A)[G][NQ], auto reload) {
    constexpr bool RELOAD = decltype(reload)::value;
    int sofs = 0, av[G] = {};
    __amdgpu_buffer_rsrc_t rb2 = rw;
    if constexpr (RELOAD) {
      const int tl = table_lane(s + 2);
      rb2 = b_rsrc(tl, &sofs);
#pragma unroll
      for (int gi = 0; gi < G; ++gi) av[gi] = a_addr(tl, gi);
    }
    static_for<0, NKB>([&](auto kc) {
      constexpr int kb = decltype(kc)::value;
      kblock(B[kb], A, kb / 2, kb % 2);
      if constexpr (RELOAD) {
#pragma unroll
        for (int t = 0; t < 4; ++t) B[kb][t] = load_x2(rb2, off[kb][t], sofs);
        if constexpr (kb % 2 == 1 || kb == NKB - 1) {
#pragma unroll
          for (int gi = 0; gi < G; ++gi) A[gi][kb / 2] = load_u4(rw, av[gi], (kb / 2) * QB);
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the loads where they are: the wait counts depend on it
      }
    });
  };
  auto fill = [&](int s, u32x2 (&B)[NKB][4], u32x4 (&A)[G][NQ]) {
    int sofs, av[G];
    const int tl = table_lane(s);
    const __amdgpu_buffer_rsrc_t rb2 = b_rsrc(tl, &sofs);
#pragma unroll
    for (int gi = 0; gi < G; ++gi) av[gi] = a_addr(tl, gi);
    static_for<0, NKB>([&](auto kc) {
      constexpr int kb = decltype(kc)::value;
#pragma unroll
      for (int t = 0; t < 4; ++t) B[kb][t] = load_x2(rb2, off[kb][t], sofs);
      if constexpr (kb % 2 == 1 || kb == NKB - 1) {
#pragma unroll
        for (int gi = 0; gi < G; ++gi) A[gi][kb / 2] = load_u4(rw, av[gi], (kb / 2) * QB);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  u32x2 B0[NKB][4], B1[NKB][4];
  u32x4 A0[G][NQ], A1[G][NQ];
  fill(0, B0, A0);
  fill(1, B1, A1);
  {
    int s = 0;
    for (; s + 1 < cntw; s += 2) {
      stage(s, B0, A0, std::true_type{});
      stage(s + 1, B1, A1, std::true_type{});
    }
    if (s < cntw) stage(s, B0, A0, std::false_type{});
  }
  __builtin_amdgcn_s_waitcnt(0);

  // Epilogue.  Unit (gi, t) = register t of group gi's four accumulators: weight row
  // 4*(lane/16) + t of the group, lane j the columns 4j + w.
  const bool vec_ok = (p.ldO % 4 == 0) && (reinterpret_cast<uintptr_t>(p.O) % 16 == 0) && (n0 + j * 4 + 4 <= p.N);
  auto store_unit = [&](int gi, int t, f32x4 v) {
    const int i16 = 4 * kg + t, mm = i16 / RS, r = i16 % RS;
    const int u1 = __builtin_amdgcn_ds_bpermute((gi * MG + mm) * 4, memv);
    const int ro = __builtin_amdgcn_ds_bpermute(r * 4, rov);
    if (valid && u1 >= 0 && r < p.R) {
      const int64_t m = int64_t(u1) * p.tm + u3 * p.a4 + ro;
      float *o = p.O + m * p.ldO + n0 + j * 4;
      if (vec_ok) {
        *reinterpret_cast<f32x4 *>(o) = v;
      } else {
#pragma unroll
        for (int w = 0; w < 4; ++w)
          if (n0 + j * 4 + w < p.N) o[w] = v[w];
      }
    }
  };
  if (lgS == 0) {
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
      for (int t = 0; t < 4; ++t) store_unit(gi, t, f32x4{acc[gi][0][t], acc[gi][1][t], acc[gi][2][t], acc[gi][3][t]});
  } else {
    // The S waves of a column tile each own the units u with u % S == their share: a wave
    // leaves the other units in LDS and, after the barrier, adds up the ones it owns (in
    // wave order, so the result does not depend on timing) and stores them.
    f32x4 *mine = reinterpret_cast<f32x4 *>(red) + (wid * (G * 4)) * 64 + lane;
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int u = gi * 4 + t;
        if ((u & (S - 1)) != ks) mine[u * 64] = f32x4{acc[gi][0][t], acc[gi][1][t], acc[gi][2][t], acc[gi][3][t]};
      }
    __syncthreads();
    const int w0 = wid & ~(S - 1);
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int u = gi * 4 + t;
        if ((u & (S - 1)) == ks) {
          f32x4 v = {0.f, 0.f, 0.f, 0.f};
          for (int k = 0; k < S; ++k) {
            const f32x4 part = k == ks ? f32x4{acc[gi][0][t], acc[gi][1][t], acc[gi][2][t], acc[gi][3][t]}
                                       : reinterpret_cast<const f32x4 *>(red)[((w0 + k) * (G * 4) + u) * 64 + lane];
            v += part;
          }
          store_unit(gi, t, v);
        }
      }
  }
}

struct Entry {
  int KC, RS, G;
  rbgp_reg_fn fn;
};
#define RBGP_B(KC, RS) {KC, RS, 1, spmm_reg_bf16<KC, RS, 1>}, {KC, RS, 2, spmm_reg_bf16<KC, RS, 2>}, \
                       {KC, RS, 4, spmm_reg_bf16<KC, RS, 4>}
const Entry kTable[] = {RBGP_B(8, 4),  RBGP_B(18, 2), RBGP_B(36, 2), RBGP_B(72, 2), RBGP_B(18, 4),
                        RBGP_B(36, 4), RBGP_B(72, 4), RBGP_B(18, 8), RBGP_B(36, 8), RBGP_B(72, 8)};

}  // namespace

rbgp_reg_fn rbgp_reg_bf16_kernel(int KC, int RS, int G) {
  for (const Entry &e : kTable)
    if (e.KC == KC && e.RS == RS && e.G == G) return e.fn;
  return nullptr;
}
