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
// The matrix core wants, per lane, eight (four in the 16-step form) consecutive contraction
// steps of ONE column, while I holds consecutive columns of one row.  A lane therefore loads
// NC = 4 or 8 columns (8 or 16 bytes; a wave covers 16 * NC columns) from each of its eight
// rows (contraction steps 32b + 8kg .. +7 of block b, kg = lane/16) and transposes the
// 8 x NC block of bf16 in registers (4 v_perm_b32 per column), which yields the B operands
// of NC MFMAs (one per column offset w), shared by all G groups.  The 16-byte form moves twice the bytes per
// load instruction, and the load path's rate is set by instructions (measured: about 29
// bytes/clock/CU with 8-byte loads against 45-50 with 16-byte ones).  The weights are packed
// k-major by rbgp_pack, so an A operand is one 16-byte load (its first 8 bytes in the
// 16-step form).
// (This header holds the kernel template; the translation units rbgp_mfma_reg_bf16*.hip instantiate disjoint parts
// of the kernel table so that they compile side by side.)
#ifndef RBGP_REG_BF16_KERNEL_H
#define RBGP_REG_BF16_KERNEL_H

#include <hip/hip_runtime.h>

#include "rbgp_internal.h"
#include "rbgp_reg_common.h"

using namespace rbgp_reg;

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// one lane's piece of a row of I: LW dwords = 2 * LW bf16 columns
template <int LW>
struct Raw {
  unsigned d[LW];
};
template <int LW>
__device__ __forceinline__ Raw<LW> load_raw(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
  Raw<LW> x;
  if constexpr (LW == 2) {
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
    x.d[0] = v[0]; x.d[1] = v[1];
  } else {
    static_assert(LW == 4, "8 or 16 bytes per lane");
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    x.d[0] = v[0]; x.d[1] = v[1]; x.d[2] = v[2]; x.d[3] = v[3];
  }
  return x;
}
__device__ __forceinline__ u32x4 load_u4(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
}
__device__ __forceinline__ s16x4 as_s16x4(unsigned lo, unsigned hi) {
  u32x2 v = {lo, hi};
  return __builtin_bit_cast(s16x4, v);
}

// LEAN: one register set instead of two -- every block's rows of I and weights are refilled in place for the wave's
// next stage right after their last use -- so that two waves fit a SIMD where the two sets fill the register file of one.
template <int KC, int RS, int G, int CW, bool LEAN = false>
__global__ __launch_bounds__(256, LEAN ? 2 : 1) void spmm_reg_bf16(RegParams p) {
  constexpr int NC = CW / 16;            // columns per lane: 4 or 8
  constexpr int LW = NC / 2;             // dwords per lane and row
  constexpr int NH = NC / 4;             // 16-byte pieces of a lane's output row
  constexpr int MG = 16 / RS;            // tile rows per 16-row group
  constexpr int U = G * MG;              // tile rows per cluster
  // A stage's KC contraction steps are cut into NK32 blocks of 32 (v_mfma_f32_16x16x32_bf16)
  // and, when at most 16 remain, one block of 16 (v_mfma_f32_16x16x16_bf16).
  constexpr int NK32 = rbgp_bf16_blocks32(KC);
  constexpr bool TAIL = rbgp_bf16_tail16(KC);
  constexpr int NB = NK32 + (TAIL ? 1 : 0);   // blocks = 16-byte weight loads per lane and stage
  constexpr int NLD = 8 * NK32 + (TAIL ? 4 : 0);   // rows of I a lane loads per stage
  constexpr int QB = 4 * RS * 16;        // bytes of one weight load across the fragment
  constexpr int FB = NB * QB;            // bytes of one weight fragment
  extern __shared__ __attribute__((aligned(16))) unsigned char red[];   // partial sums of a split stage list
  const int lane = threadIdx.x & 63;
  const int wid = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  const int lgS = p.lgS, S = 1 << lgS;
  const int ks = wid & (S - 1);          // this wave's share of the stage list
  // workgroup -> (cluster, G_i vertex, 4/S neighbouring column tiles); see wg_coord
  WgCoord wg;
  if (!wg_coord(p, &wg)) return;         // (the whole workgroup)
  const int cl = wg.cl, u3 = wg.u3, ntq = wg.ntq;
  const int nt = (ntq << (2 - lgS)) + (wid >> lgS);
  const bool valid = nt < p.ntiles;
  if (lgS == 0 && !valid) return;        // (with S > 1 every wave reaches the barrier below)
  const int64_t n0 = int64_t(nt) * CW;
  // byte offset of the wave's first column (fused convolution: part of `off` below)
  const uint32_t n0b = p.conv ? 0u : uint32_t(nt) * uint32_t(CW * 2);
  const int kg = lane >> 4, j = lane & 15;
  const int mi = j / RS, ri = j % RS;

  int mem[U];
#pragma unroll
  for (int mm = 0; mm < U; ++mm) mem[mm] = p.members[cl * U + mm];
  // stage-relative row of I of each of the lane's loads (padding steps -> row 0)
  const int32_t *rt = p.rowtab + u3 * (32 * NK32 + (TAIL ? 16 : 0));
  int rrow[NLD];
#pragma unroll
  for (int b = 0; b < NK32; ++b)
#pragma unroll
    for (int t = 0; t < 8; ++t) rrow[8 * b + t] = rt[32 * b + 8 * kg + t];
  if constexpr (TAIL) {
#pragma unroll
    for (int t = 0; t < 4; ++t) rrow[8 * NK32 + t] = rt[32 * NK32 + 4 * kg + t];
  }
  // the wave's own stages, one per lane: stage ks + lane * S of the cluster's list
  const int TS = p.tstride;
  const int own = ks + (lane << lgS);
  const int32_t *stg = p.stages + int64_t(cl) * (1 + U) * TS + (own < TS ? own : TS - 1);
  const int tb = stg[0];
  int tf[U];
#pragma unroll
  for (int mm = 0; mm < U; ++mm) tf[mm] = stg[(1 + mm) * TS];
  const int cnt = p.counts[cl];
  const int cntw = __builtin_amdgcn_readfirstlane(cnt > ks ? (cnt - ks + S - 1) >> lgS : 0);   // stages of this wave
  const int rov = p.rowofs[lane & 15];   // lane-held copies, read back with bpermute in the epilogue
  const int memv = p.members[cl * U + (lane & (U - 1))];

  // byte offset of this lane's NC bf16 columns in each of its rows, relative to the stage base
  int off[NLD];
  if (p.conv) {
    // Fused 3x3 convolution (see the fp32 kernel): the lane's NC columns are NC pixels of one
    // image row (W % NC == 0); the table holds channel offset + tap shift in bytes.  A tap
    // shift of one pixel makes the load 2-byte aligned, which the memory path accepts.
    const int colbase = p.colbase[nt < p.ntiles ? int(n0 / NC) + j : 0];   // (host table: no integer division here)
#pragma unroll
    for (int i = 0; i < NLD; ++i) off[i] = rrow[i] + colbase;
  } else {
#pragma unroll
    for (int i = 0; i < NLD; ++i) off[i] = rrow[i] * (int(p.ldI) * 2) + j * (NC * 2);
  }
  const int alane = (kg * RS + ri) * 16;

  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void *>(static_cast<const void *>(p.Wp)), 0, p.w_bytes, kRsrcFlags);
  // table lane of the wave's s-th stage; lanes past the cluster's count hold sentinels
  // (base row -1 -> a descriptor of zero extent: zeros, no memory access)
  auto table_lane = [&](int s) { return s < 63 ? s : 63; };
  // Once per stage (= per table lane), with vector instructions: the start and extent of the
  // stage's part of I and the offset of each tile row's weights (see the fp32 kernel); the
  // loop only reads them back.  A tile row that lacks the tile reads past the end of the
  // packed buffer, which returns zeros.
  const int tbu = p.conv ? int(uint32_t(tb < 0 ? 0 : tb) / 9u) : (tb < 0 ? 0 : tb);   // first row (channel) of the stage
  const uint64_t i_first = reinterpret_cast<uint64_t>(p.I) + uint64_t(uint32_t(tbu)) * p.row_bytes + n0b;
  const int ib_lo = int(uint32_t(i_first)), ib_hi = int(uint32_t(i_first >> 32));
  const int rows_left = p.last_row - tbu < p.src_rows ? p.last_row - tbu : p.src_rows;
  const int ib_ext = (tb >= 0 && valid) ? int(uint32_t(rows_left) * p.row_bytes + (p.n_bytes - n0b)) : 0;
  int aoff[U];
#pragma unroll
  for (int mm = 0; mm < U; ++mm)
    aoff[mm] = (tf[mm] >= 0 && mem[mm] >= 0) ? ((mem[mm] * p.fpm + tf[mm]) * p.a3 + u3) * FB : kOob;
  // (`live`: the stage is one of the wave's; all 64 table lanes may hold stages, and one past the count is made a
  // sentinel here: zero extent, weights past the end of the buffer)
  auto b_rsrc = [&](int tl, bool live, int *sofs) {
    const uint64_t base = uint64_t(uint32_t(__builtin_amdgcn_readlane(ib_lo, tl))) |
                          (uint64_t(uint32_t(__builtin_amdgcn_readlane(ib_hi, tl))) << 32);
    *sofs = 0;
    const int ext = __builtin_amdgcn_readlane(ib_ext, tl);
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(base), 0, live ? ext : 0, kRsrcFlags);
  };
  auto a_addr = [&](int tl, bool live, int gi) {
    int addr = 0;
#pragma unroll
    for (int mm = 0; mm < MG; ++mm) {
      const int sv = __builtin_amdgcn_readlane(aoff[gi * MG + mm], tl);
      addr = mi == mm ? sv : addr;
    }
    return (live ? addr : kOob) + alane;
  };
  // (the kernel arguments the epilogue needs, read here with the tables: fetched after the loop, they would add
  // scalar-load latencies to the end of every wave)
  float *const out = p.O;
  const int64_t out_ld = p.ldO, out_n = p.N;
  const int out_tm = p.tm, out_a4 = p.a4, out_r = p.R, out_bf16 = p.obf16;
  __builtin_amdgcn_s_waitcnt(0);   // drain the table loads outside the loop (see the fp32 kernel)

  f32x4 acc[G][NC];
#pragma unroll
  for (int gi = 0; gi < G; ++gi)
#pragma unroll
    for (int w = 0; w < NC; ++w) acc[gi][w] = f32x4{0.f, 0.f, 0.f, 0.f};

  // The MFMAs of block b: transpose the lane's 8 x NC (4 x NC) block of bf16 (dword d of a
  // row holds columns 2d and 2d+1), then per group one MFMA per column offset.
  auto block = [&](auto bc, const Raw<LW> (&B)[NLD], const u32x4 (&A)[G][NB]) {
    constexpr int b = decltype(bc)::value;
    constexpr unsigned LO = 0x05040100u, HI = 0x07060302u;
    if constexpr (b < NK32) {
      const Raw<LW> *r = &B[8 * b];
      bf16x8 bo[NC];
#pragma unroll
      for (int d = 0; d < LW; ++d) {
        bo[2 * d] = __builtin_bit_cast(
            bf16x8, u32x4{__builtin_amdgcn_perm(r[1].d[d], r[0].d[d], LO), __builtin_amdgcn_perm(r[3].d[d], r[2].d[d], LO),
                          __builtin_amdgcn_perm(r[5].d[d], r[4].d[d], LO), __builtin_amdgcn_perm(r[7].d[d], r[6].d[d], LO)});
        bo[2 * d + 1] = __builtin_bit_cast(
            bf16x8, u32x4{__builtin_amdgcn_perm(r[1].d[d], r[0].d[d], HI), __builtin_amdgcn_perm(r[3].d[d], r[2].d[d], HI),
                          __builtin_amdgcn_perm(r[5].d[d], r[4].d[d], HI), __builtin_amdgcn_perm(r[7].d[d], r[6].d[d], HI)});
      }
#pragma unroll
      for (int gi = 0; gi < G; ++gi) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, A[gi][b]);
#pragma unroll
        for (int w = 0; w < NC; ++w) acc[gi][w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bo[w], acc[gi][w], 0, 0, 0);
      }
    } else {
      const Raw<LW> *r = &B[8 * NK32];
      s16x4 bo[NC];
#pragma unroll
      for (int d = 0; d < LW; ++d) {
        bo[2 * d] = as_s16x4(__builtin_amdgcn_perm(r[1].d[d], r[0].d[d], LO), __builtin_amdgcn_perm(r[3].d[d], r[2].d[d], LO));
        bo[2 * d + 1] = as_s16x4(__builtin_amdgcn_perm(r[1].d[d], r[0].d[d], HI), __builtin_amdgcn_perm(r[3].d[d], r[2].d[d], HI));
      }
#pragma unroll
      for (int gi = 0; gi < G; ++gi) {
        const s16x4 a = as_s16x4(A[gi][b][0], A[gi][b][1]);
#pragma unroll
        for (int w = 0; w < NC; ++w) acc[gi][w] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, bo[w], acc[gi][w], 0, 0, 0);
      }
    }
  };
  // the loads of block b: its rows of I, then its weights for every group
  auto load_block = [&](auto bc, Raw<LW> (&B)[NLD], u32x4 (&A)[G][NB], __amdgpu_buffer_rsrc_t rb2, int sofs,
                        const int (&av)[G]) {
    constexpr int b = decltype(bc)::value;
    constexpr int first = 8 * b, n = b < NK32 ? 8 : 4;
#pragma unroll
    for (int t = 0; t < n; ++t) B[first + t] = load_raw<LW>(rb2, off[first + t], sofs);
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
      // (the 16-step block uses half of its weight quad: it stays whole until here, else a register of it that
      // the compiler gave to something else would have to wait for the quad's pending load, i.e. for every load)
      asm volatile("" ::"v"(A[gi][b]));
      A[gi][b] = load_u4(rw, av[gi], b * QB);
    }
    __builtin_amdgcn_sched_barrier(0);   // keep the loads where they are: the wait counts depend on it
  };

  // One stage: every block's rows of I and weights are refilled for the wave's stage s + DIST (the number of register
  // sets) right after their last use, so about DIST stages of loads are in flight; the loop body is
  // branch-free and its wait counts are exact.
  constexpr int DIST = LEAN ? 1 : 2;
  auto stage = [&](int s, Raw<LW> (&B)[NLD], u32x4 (&A)[G][NB], auto reload) {
    constexpr bool RELOAD = decltype(reload)::value;
    int sofs = 0, av[G] = {};
    __amdgpu_buffer_rsrc_t rb2 = rw;
    if constexpr (RELOAD) {
      const int tl = table_lane(s + DIST);
      const bool live = s + DIST < cntw;
      rb2 = b_rsrc(tl, live, &sofs);
#pragma unroll
      for (int gi = 0; gi < G; ++gi) av[gi] = a_addr(tl, live, gi);
    }
    static_for<0, NB>([&](auto bc) {
      block(bc, B, A);
      if constexpr (RELOAD) load_block(bc, B, A, rb2, sofs, av);
    });
  };
  auto fill = [&](int s, Raw<LW> (&B)[NLD], u32x4 (&A)[G][NB]) {
    int sofs, av[G];
    const int tl = table_lane(s);
    const bool live = s < cntw;
    const __amdgpu_buffer_rsrc_t rb2 = b_rsrc(tl, live, &sofs);
#pragma unroll
    for (int gi = 0; gi < G; ++gi) av[gi] = a_addr(tl, live, gi);
    static_for<0, NB>([&](auto bc) { load_block(bc, B, A, rb2, sofs, av); });
  };

  if constexpr (LEAN) {
    Raw<LW> B0[NLD];
    u32x4 A0[G][NB];
    fill(0, B0, A0);
    for (int s = 0; s < cntw; ++s) stage(s, B0, A0, std::true_type{});   // (past the end: sentinels, no memory access)
  } else {
    Raw<LW> B0[NLD], B1[NLD];
    u32x4 A0[G][NB], A1[G][NB];
    fill(0, B0, A0);
    fill(1, B1, A1);   // (issued before any MFMA waits: measured faster than interleaving it with stage 0)
    int s = 0;
    for (; s + 1 < cntw; s += 2) {
      stage(s, B0, A0, std::true_type{});
      stage(s + 1, B1, A1, std::true_type{});
    }
    if (s < cntw) stage(s, B0, A0, std::false_type{});
  }
  __builtin_amdgcn_s_waitcnt(0);

  // Epilogue.  Unit (gi, t) = register t of group gi's NC accumulators: weight row
  // 4*(lane/16) + t of the group, lane j the columns NC*j + w.
  // (bf16 output: a lane's NC columns are 2 * NC bytes, stored whole when they are aligned)
  const bool obf = out_bf16 != 0;
  const bool vec_ok = (n0 + j * NC + NC <= out_n) &&
                      (obf ? (out_ld % NC == 0) && (reinterpret_cast<uintptr_t>(out) % (2 * NC) == 0)
                           : (out_ld % 4 == 0) && (reinterpret_cast<uintptr_t>(out) % 16 == 0));
  auto unit_piece = [&](int gi, int t, int h) {
    return f32x4{acc[gi][4 * h][t], acc[gi][4 * h + 1][t], acc[gi][4 * h + 2][t], acc[gi][4 * h + 3][t]};
  };
  auto store_unit = [&](int gi, int t, const f32x4 (&v)[NH]) {
    const int i16 = 4 * kg + t, mm = i16 / RS, r = i16 % RS;
    const int u1 = __builtin_amdgcn_ds_bpermute((gi * MG + mm) * 4, memv);
    const int ro = __builtin_amdgcn_ds_bpermute(r * 4, rov);
    if (valid && u1 >= 0 && r < out_r) {
      const int64_t m = int64_t(u1) * out_tm + u3 * out_a4 + ro;
      if (obf) {
        uint16_t *o = reinterpret_cast<uint16_t *>(out) + m * out_ld + n0 + j * NC;
        if (vec_ok) {
          if constexpr (NH == 2) {
            const u32x4 w = {bf16_pair(v[0][0], v[0][1]), bf16_pair(v[0][2], v[0][3]), bf16_pair(v[1][0], v[1][1]),
                             bf16_pair(v[1][2], v[1][3])};
            __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>(o));
          } else {
            const u32x2 w = {bf16_pair(v[0][0], v[0][1]), bf16_pair(v[0][2], v[0][3])};
            __builtin_nontemporal_store(w, reinterpret_cast<u32x2 *>(o));
          }
        } else {
#pragma unroll
          for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int w = 0; w < 4; ++w)
              if (n0 + j * NC + 4 * h + w < out_n) o[4 * h + w] = uint16_t(bf16_bits(v[h][w]));
        }
        return;
      }
      float *o = out + m * out_ld + n0 + j * NC;
      if (vec_ok) {
#pragma unroll
        for (int h = 0; h < NH; ++h) __builtin_nontemporal_store(v[h], reinterpret_cast<f32x4 *>(o) + h);
      } else {
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
          for (int w = 0; w < 4; ++w)
            if (n0 + j * NC + 4 * h + w < out_n) o[4 * h + w] = v[h][w];
      }
    }
  };
  if (lgS == 0) {
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        f32x4 v[NH];
#pragma unroll
        for (int h = 0; h < NH; ++h) v[h] = unit_piece(gi, t, h);
        store_unit(gi, t, v);
      }
  } else {
    // The S waves of a column tile each own the units u with u % S == their share.  A wave
    // leaves the units it does not own in LDS (its region holds them densely: unit u of
    // owner o sits at (u / S) * (S - 1) + o - (o > share)) and, after the barrier, adds up
    // the ones it owns in wave order, so the result does not depend on timing.
    constexpr int NU = G * 4;
    f32x4 *const red4 = reinterpret_cast<f32x4 *>(red);
    const int per_wave = (NU >> lgS) * (S - 1);
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int o = u & (S - 1);
      if (o != ks) {
        const int slot = wid * per_wave + (u >> lgS) * (S - 1) + o - (o > ks ? 1 : 0);
#pragma unroll
        for (int h = 0; h < NH; ++h) red4[(slot * NH + h) * 64 + lane] = unit_piece(u / 4, u % 4, h);
      }
    }
    __syncthreads();
    const int w0 = wid & ~(S - 1);
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      if ((u & (S - 1)) == ks) {
        f32x4 v[NH];
#pragma unroll
        for (int h = 0; h < NH; ++h) v[h] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < S; ++k) {
          if (k == ks) {
#pragma unroll
            for (int h = 0; h < NH; ++h) v[h] += unit_piece(u / 4, u % 4, h);
          } else {
            const int slot = (w0 + k) * per_wave + (u >> lgS) * (S - 1) + ks - (ks > k ? 1 : 0);
#pragma unroll
            for (int h = 0; h < NH; ++h) v[h] += red4[(slot * NH + h) * 64 + lane];
          }
        }
        store_unit(u / 4, u % 4, v);
      }
    }
  }
}

struct Entry {
  int KC, RS, G, CW;
  rbgp_reg_fn fn;
};

}  // namespace

#endif
