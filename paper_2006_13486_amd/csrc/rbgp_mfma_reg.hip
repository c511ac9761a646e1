// Register-streaming MFMA kernels for O = W_s x I (Section 5, "GPU
// Implementation"): the fp32 kernel, and the launcher and device tables of both
// dtypes (the bf16 kernel is in rbgp_reg_bf16_kernel.h).
//
// Work decomposition.  One wavefront owns: a cluster of U tile rows u_o, one G_i
// vertex u_i (so, per tile row, the R = |G_r.U|*|G_b.U| rows that share a column
// set: row repetition, Section 5) and 64 columns of O.  It walks the union of the
// cluster's nonzero tiles (tile skipping through G_o's adjacency, Section 5)
// stage by stage; a stage is VC columns of G_r of one tile.  The rows of I a stage
// touches are loaded straight from global memory into VGPRs and each loaded row
// is used for every tile row of the cluster that has the tile: the register-level
// reuse the paper obtains from row repetition, extended across tile rows.  No
// LDS, no barrier in the main loop: waves are independent; loads are issued one
// stage ahead (two or four in the variants with several register sets), slot by
// slot, into the registers the previous MFMAs just released, and the compiler's
// vmcnt bookkeeping provides the software pipeline.  (LDS is
// used once, after the loop, when the stage list of a cluster is split over
// several waves for small N.)
// The same kernel serves the fused 3x3 convolution: only the addresses of the
// loads differ (see `off` in the prologue).
//
// Arithmetic.  v_mfma_f32_16x16x1_4b_f32: four independent 16x16 outer products
// per instruction.  The 64 lanes form 4 groups of 16 (= the 4 blocks).  One
// 16-byte-per-lane load (a "slot") brings 4 rows of I x 64 columns: group g reads
// contraction step 4*o + g of the stage, lane j of the group columns 4j..4j+3.
// Block g multiplies its row of I by the weights of that contraction step for 16
// weight rows: 16/RS tile rows of the cluster (RS = R rounded up to a power of
// two) that share the tile, RS rows each; a tile row that lacks the tile
// contributes zeros.  The four blocks thus accumulate different contraction steps
// of the same 16 x 16 outputs in different accumulator registers, which are
// added in the epilogue.  The 4x4x1 form would multiply no structural zero, but
// one wave per SIMD cannot issue it fast enough (measured: 8-cycle instructions
// issue every 13 cycles and every other instruction costs an issue slot too); the
// 32-cycle 16x16x1 form hides the whole instruction stream behind the matrix core.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <new>
#include <type_traits>
#include <vector>

#include "rbgp_internal.h"
#include "rbgp_reg_common.h"

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

using namespace rbgp_reg;

namespace {

// KC: contraction steps per stage; RS: weight rows per tile row in the 16-row MFMA group
// (cluster size MG = 16 / RS).  The weights stream from global memory like I (they are L2 hits).
// TAPS (fused 3x3 convolution on a tap-grouped layout, image width dividing 64): slots 3p,
// 3p+1, 3p+2 of a lane group are the taps dx = -1, 0, +1 of one (channel, dy) pair, i.e. three
// windows of the same pixel row shifted by one pixel.  Only the middle one is loaded; the other
// two are put together from it and the neighbouring lane's pixel (DPP), zero at an image border.
// Stages of 8 steps make short waves (a transposed 3x3 layer: 64 MFMAs per wave) whose time is mostly
// latency; four of them per SIMD (<= 128 registers, which the compiler meets without spilling) instead
// of the three it would otherwise leave room for: the conv5 backward data product 32 -> 29 us.
// NG (one tile row per group only, RS = 16): 16-row groups per wave.  Where rows of G_r moved into the tile-row
// index, NG consecutive tile rows have the very same tiles; one wave then takes NG of them, and every loaded row
// of I feeds NG groups of MFMAs: the rows of I cross the load path of the CU 1/NG as often (a stage of 72 steps
// asks for 23 KB per 2304 MFMA cycles and wave, ~40 B/clk per CU with four waves, close to what the path
// delivers), at NG times the accumulators.  Two groups with stages of up to 32 steps (36 tap-grouped) still fit two
// waves per SIMD without spilling; the larger ones get one.
// CTILES (stages of up to 8 steps): the variant whose waves take several column tiles one after the other.
// LEAN (stages of 18 steps and more): one register set instead of two -- every slot is refilled in place for the next
// stage right after its last use -- so that more waves fit a SIMD (72 steps: two instead of one; 32 and 36 steps:
// three instead of two; 18 steps: four instead of three; two groups of 36 steps or of 72 tap-grouped ones: two
// instead of one).
template <int KC, int RS, bool TAPS = false, int NG = 1, bool CTILES = false, bool LEAN = false>
__global__ __launch_bounds__(256, (LEAN || (NG == 2 && (KC <= 32 || (KC == 36 && TAPS))) ? 2
                                   : KC <= 8 && NG == 1                                   ? (CTILES ? 2 : RS >= 4 ? 4 : 3)
                                                                                          : 1)) void spmm_reg(RegParams p) {
  static_assert(!CTILES || (KC <= 8 && !TAPS), "column tiles per wave: short stages, not the fused convolution");
  static_assert(!LEAN || (KC > 8 && !CTILES), "one register set: the long stages");
  static_assert(!TAPS || KC % 12 == 0, "tap-grouped stages are multiples of 12 steps");
  static_assert(NG == 1 || RS == 16, "several groups per wave: one tile row per group");
  constexpr int MG = 16 / RS;            // tile rows per MFMA group = cluster size
  constexpr int NO = (KC + 3) / 4;       // load slots per stage (4 contraction steps each)
  constexpr int NQ = (NO + 3) / 4;       // weight registers per stage come as NQ 16-byte loads
  constexpr int QB = 4 * RS * 16;        // bytes of one such load across the fragment
  constexpr int FB = NQ * QB;            // bytes of one weight fragment (one tile row, one G_i vertex)
  constexpr int CW = 64;                 // columns per wave
  extern __shared__ __attribute__((aligned(16))) unsigned char wlds[];
  const int lane = threadIdx.x & 63;
  const int wid = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);

  // A workgroup is one (cluster, G_i vertex) pair on four neighbouring column tiles.  Same
  // columns of I -> same XCD (one L2): workgroups are dealt round-robin to the 8 XCDs.
  // (grid x = 8 * clusters is a multiple of 8, so the XCD of a workgroup is x & 7 whatever y, z)
  // The column-tile index is the slowest grid dimension: all (cluster, G_i vertex) pairs of the
  // same columns are dispatched together, so I comes from HBM once however large N is.
  // The stage list of a cluster can be split over S = 1, 2 or 4 waves of the workgroup (wave
  // k takes stages k, k + S, ...; the partial sums meet in LDS): the workgroup then covers
  // 4 / S column tiles.  Used when N is too small to give every SIMD a wave otherwise.
  const int lgS = p.lgS, S = 1 << lgS;
  const int ks = wid & (S - 1);
  WgCoord wg;
  if (!wg_coord(p, &wg)) return;
  const int cl = wg.cl * NG, u3 = wg.u3, ntq = wg.ntq;   // (NG > 1: the first of the wave's NG tile rows; all share its tables)
  // Register sets = stages of loads in flight.  Two for the long stages; a stage of 8 steps is 8 MFMAs (256
  // cycles), and two of them ahead cover far less than a memory access takes: such kernels keep four.
  constexpr int D = LEAN ? 1 : KC <= 8 ? 4 : 2;
  // Short stages, every stage list of the same length: a wave takes `ct` neighbouring column tiles one after the
  // other as ONE list of ct * (stages per tile) stages (lane l of the stage table then serves column tile
  // l / stages-per-tile), so the tables are fetched once and the first rows of the next tile are on their way while
  // the last stages of this one are multiplied; the sums of a tile are stored when its last stage is done.
  const int ct = CTILES ? p.ct : 1;
  const int nt = ((ntq << (2 - lgS)) + (wid >> lgS)) * ct;   // (the first of them)
  const int64_t n0 = int64_t(nt) * CW;
  const int g = lane >> 4, j = lane & 15;
  const int mi = j / RS, ri = j % RS;    // as a weight lane: member of the group, row of the member

  // Everything the prologue needs is requested at once: cluster members, row table, stage
  // table (one stage per lane, read back with readlane), stage count.
  int mem[MG];
#pragma unroll
  for (int mm = 0; mm < MG; ++mm) mem[mm] = p.members[cl * MG + mm];
  const int32_t *rt = p.rowtab + u3 * (NO * 4) + g;
  int rrow[NO];
#pragma unroll
  for (int o = 0; o < NO; ++o) rrow[o] = rt[o * 4];
  // the wave's own stages, one per lane: stage ks + lane * S of the cluster's list
  const int TS = p.tstride;
  int own = ks + (lane << lgS), ctile = 0;
  if (CTILES) {
    ctile = lane / p.ct_cnt;
    own = lane - ctile * p.ct_cnt;
  }
  // byte offset of the first column (of the lane's table entry's tile) in a row of I (fused convolution: the
  // lane's own column offset inside a channel of X, see `off` below)
  const uint32_t n0b = p.conv ? 0u : uint32_t(nt + ctile) * uint32_t(CW * 4);
  const bool tile_ok = nt + ctile < p.ntiles;
  const int32_t *stg = p.stages + int64_t(cl) * (1 + MG) * TS + (own < TS ? own : TS - 1);
  const int tb = stg[0];
  int tf[MG];
#pragma unroll
  for (int mm = 0; mm < MG; ++mm) tf[mm] = stg[(1 + mm) * TS];
  const int cnt0 = p.counts[cl];
  const int tiles_here = p.ntiles - nt < ct ? p.ntiles - nt : ct;
  const int cnt = __builtin_amdgcn_readfirstlane(   // stages of this wave
      CTILES ? p.ct_cnt * (tiles_here > 0 ? tiles_here : 0) : cnt0 > ks ? (cnt0 - ks + S - 1) >> lgS : 0);
  const int rov = p.rowofs[lane & 15];   // lane-held copies, read back with bpermute in the epilogue
  const int memv = p.members[cl * MG + (lane & (MG - 1))];
  // table lane of the wave's s-th stage (all 64 lanes may hold stages: a stage past the wave's count is made a
  // sentinel where it is read back -- zero extent, weights past the end of the buffer)
  auto table_lane = [&](int s) { return s < 63 ? s : 63; };

  // byte offset of this lane's 16 bytes in every slot, relative to the stage base.  Columns
  // past N read whatever follows inside I (or zeros past its end): they are never stored.
  int off[NO];
  bool row_start = false, row_end = false;   // TAPS: the lane's four pixels touch the left / right image border
  if (p.conv) {
    // Fused 3x3 convolution: column n = (image * H + y) * W + x of the lowered input is pixel
    // (y + dy, x + dx) of the zero-padded image; the lane's four columns lie in one image row
    // (W % 4 == 0), so a tap is a constant shift of one 16-byte load.  The table entry already
    // holds channel * bytes per channel + shift of the tap.
    // (host table: no integer division here; its two low bits flag the image borders)
    const int cb = p.colbase[nt < p.ntiles ? int(n0 >> 2) + j : 0];   // (a wave past the last tile loads nothing)
    const int colbase = cb & ~3;
#pragma unroll
    for (int o = 0; o < NO; ++o) off[o] = rrow[o] + colbase;
    row_start = cb & 1;
    row_end = cb & 2;
  } else {
#pragma unroll
    for (int o = 0; o < NO; ++o) off[o] = rrow[o] * (int(p.ldI) * 4) + j * 16;   // < 2^31: checked by the host
  }
  const int alane = (g * RS + ri) * 16;
  const bool valid = nt < p.ntiles;

  const __amdgpu_buffer_rsrc_t rw =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.Wp), 0, p.w_bytes, kRsrcFlags);
  // Once per stage (= per table lane), with vector instructions: where the stage's part of I
  // starts and how far it extends, and where each member's weights are.  The loop then only
  // reads these back (readlane), which keeps the scalar work between two stages short enough
  // to hide behind the last MFMAs of a stage.
  // The descriptor of a stage starts at the stage's first row and the wave's first column, so
  // the 32-bit offsets inside it only span one stage (I itself may exceed 4 GiB).  A stage
  // touches at most p.src_rows rows: its extent fits 32 bits, and only where the stage reaches
  // the last row of I does the extent end inside it, at the last column.  A stage past the end
  // gets extent zero: its loads return zeros without a memory access.
  const int tbu = p.conv ? int(uint32_t(tb < 0 ? 0 : tb) / 9u) : (tb < 0 ? 0 : tb);   // first row (channel) of the stage
  const uint64_t i_first = reinterpret_cast<uint64_t>(p.I) + uint64_t(uint32_t(tbu)) * p.row_bytes + n0b;
  const int ib_lo = int(uint32_t(i_first)), ib_hi = int(uint32_t(i_first >> 32));
  const int rows_left = p.last_row - tbu < p.src_rows ? p.last_row - tbu : p.src_rows;
  const int ib_ext = (tb >= 0 && tile_ok) ? int(uint32_t(rows_left) * p.row_bytes + (p.n_bytes - n0b)) : 0;
  // per-lane byte offset of each member's weights: a tile row that lacks the tile reads at an
  // offset past the weight buffer (zeros)
  int aoff[MG];
#pragma unroll
  for (int mm = 0; mm < MG; ++mm)
    aoff[mm] = (tf[mm] >= 0 && mem[mm] >= 0) ? ((mem[mm] * p.fpm + tf[mm]) * p.a3 + u3) * FB : kOob;
  auto b_rsrc = [&](int s, int *sofs) {
    const int tl = table_lane(s);
    const uint64_t base = uint64_t(uint32_t(__builtin_amdgcn_readlane(ib_lo, tl))) |
                          (uint64_t(uint32_t(__builtin_amdgcn_readlane(ib_hi, tl))) << 32);
    *sofs = 0;
    const int ext = __builtin_amdgcn_readlane(ib_ext, tl);
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(base), 0, s < cnt ? ext : 0, kRsrcFlags);
  };

  f32x4 Bs[D][NO];
  f32x4 As[D][NG][NQ];
  if (!valid && lgS == 0) return;   // (with a split stage list every wave reaches the barrier below)
  // Drain every outstanding load count here: a wait for the table loads inside the loop
  // would run on every iteration and drain the prefetched stages with it.
  __builtin_amdgcn_s_waitcnt(0);

  f32x16 acc[NG][4];
#pragma unroll
  for (int k = 0; k < NG; ++k)
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[k][w][v] = 0.f;
  const int gstr = p.fpm * p.a3 * FB;   // NG > 1: from one tile row's weights to the next one's (same tile, same stage)

  // Loads are unconditional so that the wait counts are exact (sentinel stages and absent
  // tiles read zeros, see above).
  auto a_addr = [&](int s) {
    int addr = 0;
    const int tl = table_lane(s);
#pragma unroll
    for (int mm = 0; mm < MG; ++mm) {
      const int sv = __builtin_amdgcn_readlane(aoff[mm], tl);
      addr = mi == mm ? sv : addr;
    }
    return (s < cnt ? addr : kOob) + alane;
  };
  auto a_load = [&](int addr, int q) { return load_x4(rw, addr, q * QB); };

  // The four B operands of slot o (one per column offset w).  TAPS: from the pair's middle window
  // c (pixels x .. x+3): dx = -1 is {left neighbour, c0, c1, c2}, dx = +1 is {c1, c2, c3, right
  // neighbour}; the neighbours are the adjacent lanes' pixels, or zero outside the image.
  auto operand = [&](const f32x4 (&B)[NO], auto oc) {
    constexpr int o = decltype(oc)::value;
    if constexpr (!TAPS) {
      return B[o];
    } else {
      constexpr int dxi = o % 3;
      const f32x4 c = B[o - dxi + 1];
      if constexpr (dxi == 1) {
        return c;
      } else if constexpr (dxi == 0) {
        const int nb = __builtin_amdgcn_update_dpp(0, __float_as_int(c[3]), 0x111 /* row_shr:1 */, 0xf, 0xf, true);
        return f32x4{row_start ? 0.f : __int_as_float(nb), c[0], c[1], c[2]};
      } else {
        const int nb = __builtin_amdgcn_update_dpp(0, __float_as_int(c[0]), 0x101 /* row_shl:1 */, 0xf, 0xf, true);
        return f32x4{c[1], c[2], c[3], row_end ? 0.f : __int_as_float(nb)};
      }
    }
  };

  // One stage: MFMAs of stage s from (B, A); every B slot and every weight quad is
  // refilled for stage s + D right after its last use (RELOAD), so that about D stages
  // of loads are in flight at any time.  Every real stage has work (the stage list is the
  // union of the cluster's tiles), so the loop body is branch-free and its wait counts
  // are exact.
  auto stage = [&](int s, f32x4 (&B)[NO], f32x4 (&A)[NG][NQ], auto reload) {
    constexpr bool RELOAD = decltype(reload)::value;
    int sofs = 0, av = 0;
    __amdgpu_buffer_rsrc_t rb2 = rw;
    if constexpr (RELOAD) {
      rb2 = b_rsrc(s + D, &sofs);
      av = a_addr(s + D);
    }
    static_for<0, NO>([&](auto oc) {
      constexpr int o = decltype(oc)::value;
      const f32x4 b = operand(B, oc);
#pragma unroll
      for (int k = 0; k < NG; ++k) {
        const float a = A[k][o / 4][o % 4];
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[k][w] = __builtin_amdgcn_mfma_f32_16x16x1f32(a, b[w], acc[k][w], 0, 0, 0);
      }
      if constexpr (RELOAD) {
        if constexpr (!TAPS)
          B[o] = load_x4(rb2, off[o], sofs);
        else if constexpr (o % 3 == 2)
          B[o - 1] = load_x4(rb2, off[o - 1], sofs);   // the pair's middle window, after its last use
        if constexpr (o % 4 == 3 || o == NO - 1) {
          // (a last quad that is used in part stays whole until here: a register of it that the compiler gave to
          // something else would have to wait for the quad's pending load, i.e. for every load in flight)
#pragma unroll
          for (int k = 0; k < NG; ++k) {
            asm volatile("" ::"v"(A[k][o / 4]));
            A[k][o / 4] = a_load(av + k * gstr, o / 4);
          }
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the loads where they are: the wait counts depend on it
      }
    });
  };
  // loads of stage s in the same order as the refills above
  auto fill = [&](int s, f32x4 (&B)[NO], f32x4 (&A)[NG][NQ]) {
    int sofs;
    const __amdgpu_buffer_rsrc_t rb2 = b_rsrc(s, &sofs);
    const int av = a_addr(s);
    static_for<0, NO>([&](auto oc) {
      constexpr int o = decltype(oc)::value;
      if constexpr (!TAPS)
        B[o] = load_x4(rb2, off[o], sofs);
      else if constexpr (o % 3 == 2)
        B[o - 1] = load_x4(rb2, off[o - 1], sofs);
      if constexpr (o % 4 == 3 || o == NO - 1) {
#pragma unroll
        for (int k = 0; k < NG; ++k) A[k][o / 4] = a_load(av + k * gstr, o / 4);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // Stage 0 starts as soon as its own data is there: the loads of stage 1 (into the second
  // register set) and the refills for stage 2 are issued between its MFMAs.
  auto first_stage = [&](f32x4 (&B)[NO], f32x4 (&A)[NG][NQ], f32x4 (&Bn)[NO], f32x4 (&An)[NG][NQ]) {
    int sofs1, sofs2;
    const __amdgpu_buffer_rsrc_t rb1 = b_rsrc(1, &sofs1), rb2 = b_rsrc(2, &sofs2);
    const int av1 = a_addr(1), av2 = a_addr(2);
    static_for<0, NO>([&](auto oc) {
      constexpr int o = decltype(oc)::value;
      const f32x4 b = operand(B, oc);
#pragma unroll
      for (int k = 0; k < NG; ++k) {
        const float a = A[k][o / 4][o % 4];
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[k][w] = __builtin_amdgcn_mfma_f32_16x16x1f32(a, b[w], acc[k][w], 0, 0, 0);
      }
      if constexpr (!TAPS) {
        Bn[o] = load_x4(rb1, off[o], sofs1);
        B[o] = load_x4(rb2, off[o], sofs2);
      } else if constexpr (o % 3 == 2) {
        Bn[o - 1] = load_x4(rb1, off[o - 1], sofs1);
        B[o - 1] = load_x4(rb2, off[o - 1], sofs2);
      }
      if constexpr (o % 4 == 3 || o == NO - 1) {
#pragma unroll
        for (int k = 0; k < NG; ++k) {
          An[k][o / 4] = a_load(av1 + k * gstr, o / 4);
          asm volatile("" ::"v"(A[k][o / 4]));
          A[k][o / 4] = a_load(av2 + k * gstr, o / 4);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // epilogue: add the four blocks (contraction steps 0..3 mod 4).  Unit t of the sum holds
  // weight row 4*(lane/16) + t of the group, lane j the columns 4j + w (of the column tile that starts at n0c).
  auto unit = [&](int t, int k = 0) {
    f32x4 v;
#pragma unroll
    for (int w = 0; w < 4; ++w) v[w] = (acc[k][w][t] + acc[k][w][4 + t]) + (acc[k][w][8 + t] + acc[k][w][12 + t]);
    return v;
  };
  // (the kernel arguments the stores need, read once: inside the store helpers they would be fetched again per unit)
  float *const out = p.O;
  const int64_t out_ld = p.ldO, out_n = p.N;
  const int out_tm = p.tm, out_a4 = p.a4, out_r = p.R;
  const bool out_aligned = (out_ld % 4 == 0) && (reinterpret_cast<uintptr_t>(out) % 16 == 0);
  auto vec_ok_at = [&](int64_t n0c) { return out_aligned && (n0c + j * 4 + 4 <= out_n); };
  auto store_unit = [&](int t, f32x4 v, int k, int64_t n0c, bool vec_ok) {
    const int i16 = 4 * g + t, mm = i16 / RS, r = i16 % RS;
    int u1 = __builtin_amdgcn_ds_bpermute(mm * 4, memv);
    if constexpr (NG > 1) u1 = u1 >= 0 ? u1 + k : u1;   // (group k is the tile row after group k - 1's)
    const int ro = __builtin_amdgcn_ds_bpermute(r * 4, rov);
    if (valid && u1 >= 0 && r < out_r) {
      const int64_t m = int64_t(u1) * out_tm + u3 * out_a4 + ro;
      float *o = out + m * out_ld + n0c + j * 4;
      if (vec_ok) {
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(o));
      } else {
#pragma unroll
        for (int w = 0; w < 4; ++w)
          if (n0c + j * 4 + w < out_n) o[w] = v[w];
      }
    }
  };
  auto store_tile = [&](int64_t n0c) {
    const bool vec_ok = vec_ok_at(n0c);
#pragma unroll
    for (int k = 0; k < NG; ++k)
#pragma unroll
      for (int t = 0; t < 4; ++t) store_unit(t, unit(t, k), k, n0c, vec_ok);
  };

  // The register sets take turns; stages past the end read zeros (sentinel table lanes).
  if constexpr (D == 2) {
    f32x4(&B0)[NO] = Bs[0], (&B1)[NO] = Bs[1];
    f32x4(&A0)[NG][NQ] = As[0], (&A1)[NG][NQ] = As[1];
    fill(0, B0, A0);
    first_stage(B0, A0, B1, A1);
    if (cnt > 1) {   // the loop is reachable only through stage 1, which keeps its wait counts exact
      stage(1, B1, A1, std::true_type{});
      int s = 2;
      for (; s + 1 < cnt; s += 2) {
        stage(s, B0, A0, std::true_type{});
        stage(s + 1, B1, A1, std::true_type{});
      }
      if (s < cnt) stage(s, B0, A0, std::false_type{});
    }
  } else {
    // all D sets are requested up front; whole rounds of D stages refill as they go (branch-free: exact wait
    // counts); the last, partial round only consumes what is already on its way
    static_for<0, D>([&](auto kc) { fill(decltype(kc)::value, Bs[decltype(kc)::value], As[decltype(kc)::value]); });
    int s = 0;
    if constexpr (CTILES) {
      // several column tiles, one list: every tile has p.ct_cnt stages, a multiple of D, so a tile ends with a
      // round; its sums are stored while the first stages of the next tile are already in flight
      int left = p.ct_cnt;
      int64_t n0c = n0;
      for (; s + D <= cnt; s += D) {
        static_for<0, D>([&](auto kc) {
          constexpr int k = decltype(kc)::value;
          stage(s + k, Bs[k], As[k], std::true_type{});
        });
        left -= D;
        if (left == 0) {
          store_tile(n0c);
#pragma unroll
          for (int k = 0; k < NG; ++k)
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
              for (int v = 0; v < 16; ++v) acc[k][w][v] = 0.f;
          n0c += CW;
          left = p.ct_cnt;
        }
      }
      return;
    }
    for (; s + D <= cnt; s += D)
      static_for<0, D>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        stage(s + k, Bs[k], As[k], std::true_type{});
      });
    static_for<0, D>([&](auto kc) {
      constexpr int k = decltype(kc)::value;
      if (s + k < cnt) stage(s + k, Bs[k], As[k], std::false_type{});
    });
  }
  __builtin_amdgcn_s_waitcnt(0);

  if (lgS == 0) {
    store_tile(n0);
  } else {
    // The S waves of a column tile each own the units t with t % S == their share.  A wave
    // leaves the units it does not own in LDS (densely: unit t of owner o sits at
    // (t / S) * (S - 1) + o - (o > share); one such block per group and wave) and, after the barrier,
    // adds up the ones it owns in wave order, so the result does not depend on timing.
    f32x4 *const red4 = reinterpret_cast<f32x4 *>(wlds);
    const int per_wave = (4 >> lgS) * (S - 1);
    const bool vec_ok = vec_ok_at(n0);
#pragma unroll
    for (int k = 0; k < NG; ++k)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int o = t & (S - 1);
        if (o != ks)
          red4[((k * 4 + wid) * per_wave + (t >> lgS) * (S - 1) + o - (o > ks ? 1 : 0)) * 64 + lane] = unit(t, k);
      }
    __syncthreads();
    const int w0 = wid & ~(S - 1);
#pragma unroll
    for (int k = 0; k < NG; ++k)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        if ((t & (S - 1)) == ks) {
          f32x4 v = {0.f, 0.f, 0.f, 0.f};
          for (int kk = 0; kk < S; ++kk) {
            if (kk == ks)
              v += unit(t, k);
            else
              v += red4[((k * 4 + w0 + kk) * per_wave + (t >> lgS) * (S - 1) + ks - (ks > kk ? 1 : 0)) * 64 + lane];
          }
          store_unit(t, v, k, n0, vec_ok);
        }
      }
  }
}

typedef rbgp_reg_fn reg_fn;
template <int KC, int RS>
constexpr reg_fn taps_kernel() {   // the tap-grouped variant exists for stages of a multiple of 12 steps
  if constexpr (KC % 12 == 0)
    return spmm_reg<KC, RS, true>;
  else
    return nullptr;
}
template <int KC, int RS, int NG>
constexpr reg_fn taps_kernel_ng() {
  if constexpr (KC % 12 == 0)
    return spmm_reg<KC, RS, true, NG>;
  else
    return nullptr;
}
struct RegEntry {
  int KC, RS;
  reg_fn global_fn, taps_fn;
};
#define RBGP_R(KC, RS) {KC, RS, spmm_reg<KC, RS>, taps_kernel<KC, RS>()}
// several 16-row groups per wave (one tile row each): two for every stage size, four for the short stages
struct RegGroupEntry {
  int KC, NG;
  reg_fn global_fn, taps_fn;
};
#define RBGP_RG(KC, NG) {KC, NG, spmm_reg<KC, 16, false, NG>, taps_kernel_ng<KC, 16, NG>()}
const RegGroupEntry kRegGroupTable[] = {RBGP_RG(8, 2),  RBGP_RG(18, 2), RBGP_RG(32, 2), RBGP_RG(36, 2), RBGP_RG(72, 2),
                                        RBGP_RG(8, 4),  RBGP_RG(18, 4)};
const RegGroupEntry *find_reg_groups(int KC, int NG) {
  for (const RegGroupEntry &e : kRegGroupTable)
    if (e.KC == KC && e.NG == NG) return &e;
  return nullptr;
}
// one register set (stages of 18 steps and more): {KC, RS, tap-grouped, NG, kernel}
struct RegLeanEntry {
  int KC, RS;
  bool taps;
  int NG;
  reg_fn fn;
};
#define RBGP_L1(KC, RS) {KC, RS, false, 1, spmm_reg<KC, RS, false, 1, false, true>}
#define RBGP_L1T(KC, RS) {KC, RS, true, 1, spmm_reg<KC, RS, true, 1, false, true>}
#define RBGP_L4(KC) RBGP_L1(KC, 2), RBGP_L1(KC, 4), RBGP_L1(KC, 8), RBGP_L1(KC, 16)
#define RBGP_L4T(KC) RBGP_L1T(KC, 2), RBGP_L1T(KC, 4), RBGP_L1T(KC, 8), RBGP_L1T(KC, 16)
const RegLeanEntry kRegLeanTable[] = {RBGP_L4(18),  RBGP_L4(32),  RBGP_L4(36), RBGP_L4(72),
                                      RBGP_L4T(36), RBGP_L4T(72),
                                      {36, 16, false, 2, spmm_reg<36, 16, false, 2, false, true>},
                                      {36, 16, true, 2, spmm_reg<36, 16, true, 2, false, true>},
                                      {72, 16, true, 2, spmm_reg<72, 16, true, 2, false, true>}};
reg_fn find_reg_lean(int KC, int RS, bool taps, int NG) {
  for (const RegLeanEntry &e : kRegLeanTable)
    if (e.KC == KC && e.RS == RS && e.taps == taps && e.NG == NG) return e.fn;
  return nullptr;
}
// waves that take several column tiles (stages of 8 steps): {RS, NG, kernel}
struct RegTilesEntry {
  int RS, NG;
  reg_fn fn;
};
// (one tile row per group only: with several, the stage lists are of one length only where G_o is complete, and such
// masks run with G_o (x) G_r merged, rbgp_plan_regroup, on longer stages)
const RegTilesEntry kRegTilesTable[] = {{16, 1, spmm_reg<8, 16, false, 1, true>}, {16, 2, spmm_reg<8, 16, false, 2, true>}};
reg_fn find_reg_tiles(int KC, int RS, int NG) {
  if (KC != 8) return nullptr;
  for (const RegTilesEntry &e : kRegTilesTable)
    if (e.RS == RS && e.NG == NG) return e.fn;
  return nullptr;
}
const RegEntry kRegTable[] = {RBGP_R(8, 2),  RBGP_R(18, 2),  RBGP_R(32, 2),  RBGP_R(36, 2),  RBGP_R(72, 2),
                              RBGP_R(8, 4),  RBGP_R(18, 4),  RBGP_R(32, 4),  RBGP_R(36, 4),  RBGP_R(72, 4),
                              RBGP_R(8, 8),  RBGP_R(18, 8),  RBGP_R(32, 8),  RBGP_R(36, 8),  RBGP_R(72, 8),
                              RBGP_R(8, 16), RBGP_R(18, 16), RBGP_R(32, 16), RBGP_R(36, 16), RBGP_R(72, 16)};

const RegEntry *find_reg(int KC, int RS) {
  for (const RegEntry &e : kRegTable)
    if (e.KC == KC && e.RS == RS) return &e;
  return nullptr;
}

struct RegTables {  // device tables of the clustering
  int ncl = 0, tstride = 64, max_stages = 0;
  int32_t *stages = nullptr, *counts = nullptr, *members = nullptr;
};

struct RegState {
  int32_t *rowtab = nullptr;       // fp32 kernels: [a_i][NO*4]
  std::vector<int32_t> rowtab_host, rowtab_conv_host;   //   host copies, plain and fused convolution (they travel in the
                                                        //   kernel arguments of the pairing kernel)
  int32_t *rowtab_bf16 = nullptr;  // bf16 kernels: [a_i][NKB*16]
  int32_t *rowtab_conv[2] = {nullptr, nullptr};   // fused convolution, fp32 / bf16: byte offsets for the geometry below
  int32_t *colbase[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};   // [dtype][wide tile]: pixel offsets of the column groups
  int64_t conv_key[2][3] = {{0, 0, 0}, {0, 0, 0}};  // images, height, width of rowtab_conv
  RegTables tab;                   // fp32: clusters of one 16-row group
  int32_t *dual_tab[2] = {nullptr, nullptr};   // fp32 lo/hi pairing: the kernel's one table buffer, plain / fused convolution
  RegTables tab_bf16[3];           // bf16: clusters of 1, 2, 4 groups
  bool g2_shared = false;          // the clusters of two groups have (nearly) half the stages in total: their tile rows share their tiles
  int g2_stages = -1, g2_ncl = 0;  // longest stage list and number of the clusters of two groups (-2: too long,
                                   //   or their stage lists add up to more than 0.8 of those of one group)
};

template <typename T>
int upload(const std::vector<T> &h, T **d) {
  RBGP_HIP(hipMalloc(reinterpret_cast<void **>(d), h.size() * sizeof(T) + 16));
  RBGP_HIP(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
  return RBGP_OK;
}

void free_tables(RegTables *t) {
  if (t->stages) (void)hipFree(t->stages);
  if (t->counts) (void)hipFree(t->counts);
  if (t->members) (void)hipFree(t->members);
  *t = RegTables();
}

// Upload three tables; the state is touched only when all three are on the device.
int upload_tables(const rbgp_reg_clusters &cl, RegTables *t) {
  const int ncl = cl.ncl;
  const std::vector<int32_t> &stages = cl.stages, &counts = cl.counts, &members = cl.members;
  RegTables fresh;
  fresh.ncl = ncl;
  fresh.tstride = cl.tstride;
  fresh.max_stages = cl.max_stages;
  int rc = upload(stages, &fresh.stages);
  if (!rc) rc = upload(counts, &fresh.counts);
  if (!rc) rc = upload(members, &fresh.members);
  if (rc) {
    free_tables(&fresh);
    return rc;
  }
  *t = fresh;
  return RBGP_OK;
}

// Upload the clustering of the tile rows (clusters of U) and its stage tables.
int build_tables(const rbgp_mask *m, int U, RegTables *t) {
  rbgp_reg_clusters fresh;
  const rbgp_reg_clusters *cl = &m->reg_clusters;
  if (U != cl->U) {
    rbgp_reg_cluster(m, U, &fresh);
    cl = &fresh;
  }
  if (cl->max_stages > kRegMaxStages) return RBGP_EUNSUPPORTED;   // one stage per lane plus sentinels, four waves
  return upload_tables(*cl, t);
}

}  // namespace

bool rbgp_reg_covers(const rbgp_mask *m) {
  const rbgp_reg_plan &p = m->reg;
  if (!p.ok) return false;
  // every cluster's stage list must fit the per-lane table
  if (m->reg_clusters.max_stages > kRegMaxStages) return false;
  return find_reg(p.KC, p.RS) != nullptr;
}

void rbgp_reg_release(void *state) {
  RegState *st = static_cast<RegState *>(state);
  if (!st) return;
  if (st->rowtab) (void)hipFree(st->rowtab);
  if (st->rowtab_bf16) (void)hipFree(st->rowtab_bf16);
  for (int32_t *t : st->rowtab_conv)
    if (t) (void)hipFree(t);
  for (auto &pair : st->colbase)
    for (int32_t *t : pair)
      if (t) (void)hipFree(t);
  free_tables(&st->tab);
  for (int32_t *t : st->dual_tab)
    if (t) (void)hipFree(t);
  for (RegTables &t : st->tab_bf16) free_tables(&t);
  delete st;
}

int rbgp_reg_launch(const rbgp_mask *m, void **state, const int *tune, bool bf16, bool out_bf16, int64_t N,
                    const void *packed, const void *I, int64_t ldI, void *O, int64_t ldO, void *stream,
                    const rbgp_conv_geometry *conv) {
  const rbgp_reg_plan &pl = m->reg;
  if (!rbgp_reg_covers(m)) return RBGP_EUNSUPPORTED;
  if (out_bf16 && !bf16) return RBGP_EINVAL;
  // Fused 3x3 convolution: the nine taps are the columns of a complete G_b and an image row holds
  // whole lane loads (4 columns; 8 with the wide bf16 tile); "I" is then the padded activation
  // tensor and ldI is not used.
  int64_t chs = 0;   // bytes of one channel of X
  if (conv) {
    if (m->c[3] != 9 || m->d[3] != 9) return RBGP_EUNSUPPORTED;
    if (conv->images <= 0 || conv->height <= 0 || conv->width <= 0 || conv->width % 4) return RBGP_ESHAPE;
    if (N != conv->images * conv->height * conv->width) return RBGP_ESHAPE;
    if (reinterpret_cast<uintptr_t>(I) % 4) return RBGP_ESHAPE;
    chs = conv->images * (conv->height + 2) * (conv->width + 2) * (bf16 ? 2 : 4);
    if ((int64_t(pl.SRC) / 9 + 1) * chs >= (int64_t(1) << 31)) return RBGP_EUNSUPPORTED;
    ldI = N;   // (only the checks below read it)
  }
  // I and the packed weights are addressed through 32-bit buffer offsets
  const int es = bf16 ? 2 : 4;
  // bf16: a lane loads 8 bytes (4 columns; 64-column wave tile) or 16 bytes (8 columns;
  // 128-column tile) per row.  The wide tile is the default where the operands allow it and
  // enough column tiles remain to fill the chip.
  int CW = 64;
  if (bf16) {
    const bool ok64 = conv ? true : (ldI % 4 == 0) && (reinterpret_cast<uintptr_t>(I) % 8 == 0);
    const bool ok128 = conv ? conv->width % 8 == 0 : (ldI % 8 == 0) && (reinterpret_cast<uintptr_t>(I) % 16 == 0);
    const int tc = tune[RBGP_TUNE_COLS_PER_WORKGROUP];
    if (tc != 0 && tc != 64 && tc != 128) return RBGP_EUNSUPPORTED;
    if (tc)
      CW = tc;
    else if (ok128 && int64_t((pl.TR + pl.MG - 1) / pl.MG) * m->a[2] * ((N + 127) / 128) >= 512)
      CW = 128;
    if (!(CW == 128 ? ok128 : ok64)) return RBGP_ESHAPE;
  }
  const int NC = CW / 16;
  // (bf16: two columns share a dword, and a dword that crosses the end of the descriptor reads
  // as zero, so the last row's extent (n_bytes below) is rounded up to the bytes a lane loads;
  // the condition on ldI keeps that inside the K x ldI array)
  const int64_t w_bytes = (bf16 ? pl.packed_elems_bf16 : pl.packed_elems) * es;
  // 32-bit offsets address one stage of I (its rows span SRC * ldI elements; I as a whole may be
  // larger) and the packed weights
  if ((!conv && (int64_t(pl.SRC) * ldI + CW) * es >= (int64_t(1) << 31)) || w_bytes >= (int64_t(1) << 30))
    return RBGP_EUNSUPPORTED;
  RegState *st = static_cast<RegState *>(*state);
  if (!st) {
    st = new (std::nothrow) RegState();
    if (!st) return RBGP_ENOMEM;
    *state = st;
  }
  int32_t **rowtab = conv ? &st->rowtab_conv[bf16] : bf16 ? &st->rowtab_bf16 : &st->rowtab;
  int64_t *ckey = st->conv_key[bf16];
  if (conv && *rowtab && (ckey[0] != conv->images || ckey[1] != conv->height || ckey[2] != conv->width)) {
    (void)hipFree(*rowtab);   // (waits for launches that still read the old table)
    *rowtab = nullptr;
    if (!bf16 && st->dual_tab[1]) {
      (void)hipFree(st->dual_tab[1]);
      st->dual_tab[1] = nullptr;
    }
    for (int32_t *&t : st->colbase[bf16]) {
      if (t) (void)hipFree(t);
      t = nullptr;
    }
  }
  if (!*rowtab) {
    const int a3 = m->a[2], d3 = m->d[2], c3 = m->c[2], c4 = m->c[3];
    const int len = bf16 ? 32 * rbgp_bf16_blocks32(pl.KC) + (rbgp_bf16_tail16(pl.KC) ? 16 : 0) : pl.NO * 4;   // contraction steps, padded (padding -> row 0)
    std::vector<int32_t> rt(size_t(a3) * len, 0);
    for (int u3 = 0; u3 < a3; ++u3)
      for (int kk = 0; kk < pl.KCR; ++kk) {
        const int st = bf16 ? kk : rbgp_reg_step(m, kk);   // step of the contraction list at position kk
        const int v4 = st % c4, j3 = (st / c4) % d3, vv = st / (c4 * d3);
        rt[size_t(u3) * len + kk] = (vv * c3 + m->adj[2][size_t(u3) * d3 + j3]) * c4 + v4;
      }
    if (conv) {   // stage-relative row 9 * channel + tap -> byte offset of the channel plus the shift of the tap
      for (int32_t &r : rt) {
        const int tap = r % 9, dy = tap / 3 - 1, dx = tap % 3 - 1;
        r = int32_t((r / 9) * chs + (dy * (conv->width + 2) + dx) * es);
      }
      ckey[0] = conv->images; ckey[1] = conv->height; ckey[2] = conv->width;
    }
    int rc = upload(rt, rowtab);
    if (rc) return rc;
    if (!bf16) (conv ? st->rowtab_conv_host : st->rowtab_host) = rt;
  }
  const int64_t ntiles = (N + CW - 1) / CW;
  // bf16: 16-row groups per wave (G) and waves per column tile (S).  More groups mean fewer
  // passes of I through the load path at the price of multiplied zeros; on the VGG19 conv3 shape
  // the two balance out, so the default is one group unless the rule below finds two worth it.
  // The stage list is split when there are fewer (cluster, G_i vertex, column tile) triples than SIMDs.
  int G = 1, lgS = 0;
  {
    const int tg = bf16 ? tune[RBGP_TUNE_ROW_GROUPS] : 0, ts = tune[RBGP_TUNE_K_SPLIT];
    if (tg) {
      if (tg != 1 && tg != 2 && tg != 4) return RBGP_EUNSUPPORTED;   // (too long a stage list is rejected below)
      G = tg;
    } else if (bf16 && !ts && (pl.TR + pl.MG - 1) / pl.MG >= 2) {
      // Two groups per wave halve the bytes of I that cross the L1 path.  Measured on the VGG19 layers (bf16,
      // densities 1/2 and 1/4): that pays (3-22 %) where the larger clusters still give every SIMD a wave
      // without a split, or where each wave of the split keeps a dozen stages to amortise the reduction; it
      // costs 7-25 % where neither holds, and 7-15 % where G_o is so sparse that the tile rows of a larger
      // cluster share few tiles (density 1/16: the stage lists of the clusters then add up to nearly as many
      // stages as before, each multiplied into twice the rows).
      if (st->g2_stages == -1) {
        rbgp_reg_clusters c2;
        rbgp_reg_cluster(m, 2 * pl.MG, &c2);
        int64_t total1 = 0, total2 = 0;
        for (int32_t c : m->reg_clusters.counts) total1 += c;
        for (int32_t c : c2.counts) total2 += c;
        st->g2_stages = (c2.max_stages > kRegMaxStages || m->reg_clusters.U != pl.MG || 5 * total2 > 4 * total1) ? -2 : c2.max_stages;
        st->g2_ncl = c2.ncl;
        st->g2_shared = 20 * total2 <= 11 * total1;
      }
      if (st->g2_stages > 0) {
        const int64_t waves2 = int64_t(st->g2_ncl) * m->a[2] * ntiles;
        int S2 = 1;
        while (S2 < 4 && waves2 * S2 < 1024) S2 *= 2;
        // (the fused convolution issues more loads per step -- nine shifted windows per channel -- and gains
        // 15-22 % on every VGG19 layer that keeps the chip full, however short the split lists)
        // (and where the tile rows of a larger cluster have the same tiles -- rows of G_r moved into the tile-row
        // index -- the second group costs no extra stage at all: 12-17 % faster on the density-1/2 layers)
        // (with the one-register-set kernels of the 128-column tiles a split in two pays from six stages per wave on:
        // VGG19 conv3 16.97 -> 16.35 us, layers 5, 6, 9-11 at density 1/4 8-9 % faster)
        const int enough = (S2 == 2 && CW == 128) ? 6 : 12;
        if (waves2 * S2 >= 1024 && (S2 == 1 || conv || st->g2_shared || st->g2_stages / S2 >= enough)) G = 2;
        // Four tile rows with the very same tiles (at least four of G_r's rows moved into the tile-row index, as on the
        // filled masks of Tables 2-3): four groups per wave, where the chip stays full and the accumulators fit without
        // spilling (stages of up to 36 steps).  4096^3 with one row per column set: 182 / 122 / 111 us with 1 / 2 / 4 groups.
        // (stage lists of 16: 53.9 us against 51.1 with two groups -- long lists only)
        if (G == 2 && st->g2_shared && pl.MG == 1 && pl.fold % 4 == 0 && pl.KC <= 36 && st->g2_stages >= 32) {
          const int64_t waves4 = int64_t(pl.TR / 4) * m->a[2] * ntiles;
          int S4 = 1;
          while (S4 < 4 && (waves4 * S4 < 1024 || st->g2_stages > kRegWaveStages * S4)) S4 *= 2;
          if (waves4 * S4 >= 1024 && st->g2_stages <= kRegWaveStages * S4) G = 4;
        }
      }
    }
    const int64_t ncl = (pl.TR + G * pl.MG - 1) / (G * pl.MG);
    if (ts) {
      if (ts != 1 && ts != 2 && ts != 4) return RBGP_EUNSUPPORTED;
      lgS = ts == 4 ? 2 : ts == 2 ? 1 : 0;
    } else {
      while (lgS < 2 && ((ncl * m->a[2] * ntiles) << lgS) < 1024) ++lgS;
    }
  }
  const RegEntry *e = find_reg(pl.KC, pl.RS);
  if (!e) return RBGP_EUNSUPPORTED;
  // fused convolution on a tap-grouped layout whose image rows tile the 64 columns of a wave:
  // the variant that loads one of the three horizontal taps and builds the others.  Measured on
  // the VGG19 layers: 5-15 % faster for images 8 to 32 pixels wide, slower for 4-pixel-wide ones
  // (every lane is a whole image row there: nothing to share, only the extra instructions).
  const bool taps = conv && !bf16 && rbgp_reg_tap_grouped(m) && e->taps_fn && conv->width >= 8 && 64 % conv->width == 0;
  // fp32, two tile rows per MFMA group: lo/hi pairing of the tile rows (rbgp_mfma_reg_dual.hip) where its
  // busiest SIMD walks fewer stages than the longest cluster of the fixed pairs, and there are enough
  // (tile row, G_i vertex, column tile) triples to fill every SIMD without splitting stage lists.
  bool dual = false;
  {
    const int tp = tune[RBGP_TUNE_ROW_PAIRING];
    if (tp < 0 || tp > 2) return RBGP_EUNSUPPORTED;
    const bool can = !bf16 && !taps && m->reg_dual.ok && rbgp_reg_dual_kernel(pl.KC) && !tune[RBGP_TUNE_K_SPLIT];
    if (tp == 2 && !can) return RBGP_EUNSUPPORTED;
    dual = can && (tp == 2 || (tp == 0 && lgS == 0 && m->reg_dual.max_stages < m->reg_clusters.max_stages));
  }
  if (dual) lgS = 1;   // (two column tiles per workgroup, as with a stage list split in two)
  RegTables *tab = bf16 ? &st->tab_bf16[G == 4 ? 2 : G == 2 ? 1 : 0] : &st->tab;
  if (!dual && !tab->stages) {
    int rc = build_tables(m, G * pl.MG, tab);
    if (rc) return rc;
  }
  if (!dual) {
    // a stage list longer than a wave's table is split over enough waves of the workgroup
    int need = 0;
    while ((kRegWaveStages << need) < tab->max_stages) ++need;
    if (need > lgS) {
      if (tune[RBGP_TUNE_K_SPLIT]) return RBGP_EUNSUPPORTED;
      lgS = need;
    }
  }
  // fp32, rows of G_r moved into the tile-row index: NG of the `fold` tile rows that share their tiles per wave
  // (see spmm_reg), as many as still leave every SIMD a wave; tuning knob RBGP_TUNE_ROW_GROUPS overrides.
  int NGf = 1;
  const RegGroupEntry *ge = nullptr;
  bool ident = !bf16 && !dual && pl.MG == 1 && pl.fold > 1;   // (clusters of one tile row that come in tile-row order)
  for (int c = 0; c < m->reg_clusters.ncl && ident; ++c) ident = m->reg_clusters.members[size_t(c)] == c;
  if (!bf16 && !dual && pl.MG == 1 && pl.fold > 1) {
    auto fits = [&](int ng) {
      const RegGroupEntry *g = find_reg_groups(pl.KC, ng);
      return ident && pl.fold % ng == 0 && g && (!taps || g->taps_fn);
    };
    const int tg = tune[RBGP_TUNE_ROW_GROUPS];
    if (tg > 1) {
      if (!fits(tg)) return RBGP_EUNSUPPORTED;
      NGf = tg;
    } else if (tg == 0) {
      // (not for short waves: with several groups a SIMD holds one wave instead of up to four, and a wave of a few
      // hundred MFMAs is mostly latency -- the conv5 backward data product, 8 stages of 8 steps: 29.6 us with one
      // group, 39.8 / 35.3 with two / four; the density-1/2 VGG19 layers, 8-16 stages of 72 steps: 6-19 % faster with two)
      const int64_t steps = int64_t(tab->max_stages) * pl.KC;
      for (int ng : {4, 2})
        if (fits(ng) && steps >= (128 * ng << lgS) && ((int64_t(tab->ncl / ng) * m->a[2] * ntiles) << lgS) >= 1024) {
          NGf = ng;
          break;
        }
      // (the kernels of two groups with stages of up to 32 steps fit two waves per SIMD, like those of one group or
      // nearly so: there two groups pay from 64 steps on, while every SIMD still gets its two waves)
      if (NGf == 1 && fits(2) && pl.KC <= 32 && !taps && steps >= (64 << lgS) &&
          ((int64_t(tab->ncl / 2) * m->a[2] * ntiles) << lgS) >= 2048)
        NGf = 2;
    }
    if (NGf > 1) ge = find_reg_groups(pl.KC, NGf);
  } else if (!bf16 && tune[RBGP_TUNE_ROW_GROUPS] > 1) {
    return RBGP_EUNSUPPORTED;
  }
  // fp32, stages of up to 8 steps (short waves, mostly latency): column tiles per wave (see spmm_reg); tuning knob
  // RBGP_TUNE_COLUMN_TILES overrides.
  int CT = 1;
  {
    const int tc = tune[RBGP_TUNE_COLUMN_TILES];
    bool can = !bf16 && !dual && !conv && find_reg_tiles(pl.KC, pl.RS, NGf) && lgS == 0 && tab->max_stages > 0 && tab->max_stages % 4 == 0 &&
               m->reg_clusters.U == pl.MG;
    for (size_t c = 0; can && c < m->reg_clusters.counts.size(); ++c) can = m->reg_clusters.counts[c] == tab->max_stages;
    auto fits = [&](int c) { return can && (c == 2 || c == 4 || c == 8) && tab->max_stages * c <= kRegWaveStages; };
    auto waves = [&](int ng, int c) { return int64_t(tab->ncl / ng) * m->a[2] * ((ntiles + c - 1) / c); };
    if (tc > 1) {
      if (!fits(tc)) return RBGP_EUNSUPPORTED;
      CT = tc;
    } else if (tc == 0 && NGf == 2) {
      for (int c : {4, 2})
        if (fits(c) && waves(2, c) >= 2048) {
          CT = c;
          break;
        }
    } else if (tc == 0 && NGf == 1) {
      // Measured on the conv5 backward data product (64 tile rows of 9 rows, 8 stages of 8 steps, 16 384 such
      // waves), us per launch on one box: one tile per wave 31.2, four 29.6; two of the tile rows that share their
      // tiles per wave as well (each row of dO loaded half as often; two waves per SIMD) 27.8 with four tiles, 28.8
      // with two, 32.4 with eight.  The waves must still fill the SIMDs: three each with one row group, two with two.
      if (tune[RBGP_TUNE_ROW_GROUPS] == 0 && ident && pl.fold % 2 == 0 && find_reg_tiles(pl.KC, pl.RS, 2) && fits(4) &&
          waves(2, 4) >= 2048) {
        NGf = 2;
        CT = 4;
      } else {
        for (int c : {4, 2})
          if (fits(c) && waves(1, c) >= 3072) {
            CT = c;
            break;
          }
      }
    }
  }
  // One register set with more waves per SIMD instead of two sets (see spmm_reg, spmm_reg_bf16) wherever that variant
  // is built; tuning knob RBGP_TUNE_REGISTER_SETS overrides.
  bool lean = false;
  {
    const int tr = tune[RBGP_TUNE_REGISTER_SETS];
    if (tr < 0 || tr > 2) return RBGP_EUNSUPPORTED;
    // (bf16, two groups of short stages: only where a wave has a single stage -- nothing to prefetch, so the second set
    // buys nothing and the extra waves do, 27.6 -> 22.2 us on the dense first VGG19 layer; with several short stages
    // the two sets keep more bytes in flight, 18.5 against 23.6 us on layer 2 at density 1/8)
    const bool can = bf16 ? rbgp_reg_bf16_lean_kernel(pl.KC, pl.RS, G, CW) != nullptr &&
                                (pl.KC > 32 || G == 4 || tab->max_stages <= (1 << lgS))
                          : !dual && CT == 1 && find_reg_lean(pl.KC, pl.RS, taps, NGf);
    if (tr == 1 && !can) return RBGP_EUNSUPPORTED;
    // (measured on the fp32 VGG19 layers at every density, batches of 512 to 131 072 columns, split lists included:
    // stages of 72 steps 1-19 % faster than two sets in every cell, the shorter stages and the tap-grouped kernels
    // 1-2 % over the forward, fused and backward sweeps (single cells up to 12 %); bf16 on 128-column tiles: 1-13 %
    // faster in 38 of 41 cells, 2-6 % slower in three; so it is the default wherever it applies)
    lean = can && tr != 2;
  }
  const int ncl = dual ? m->reg_dual.nq : tab->ncl / NGf;
  const int fpm = m->d[0] * pl.NSTG;
  // LDS: partial sums of the split -- per wave the (S - 1) / S of its 4G units it does not own; lo/hi pairing:
  // the four units of half of the eight waves
  size_t lds = dual ? size_t(16) * 1024
                    : size_t(4) * ((4 * G) >> lgS) * ((1 << lgS) - 1) * (bf16 ? NC / 4 : 1) * 1024;
  lds *= NGf;   // (fp32 with several groups per wave: one such block per group)

  RegParams rp;
  rp.Wp = static_cast<const float *>(packed);
  rp.I = static_cast<const float *>(I);
  rp.O = static_cast<float *>(O);
  rp.obf16 = out_bf16 ? 1 : 0;
  rp.rowtab = *rowtab;
  rp.stages = dual ? nullptr : tab->stages; rp.counts = dual ? nullptr : tab->counts; rp.members = dual ? nullptr : tab->members;
  rp.tstride = tab->tstride;
  rp.N = N; rp.ldI = ldI; rp.ldO = ldO;
  rp.w_bytes = uint32_t(w_bytes);
  rp.row_bytes = uint32_t(ldI * es);
  rp.n_bytes = uint32_t((bf16 ? (N + NC - 1) / NC * NC : N) * es);
  rp.last_row = int(m->K - 1);
  rp.src_rows = pl.SRC;
  rp.colbase = nullptr;
  if (conv) {
    // pixel offset of every group of NC columns (one lane's load), padded to whole wave tiles with a
    // pixel inside X; fp32: bit 0 / bit 1 flag a group at the left / right border of its image row
    int32_t **cbt = &st->colbase[bf16][CW == 128];
    if (!*cbt) {
      const int64_t H = conv->height, W = conv->width;
      std::vector<int32_t> cb(size_t(ntiles) * (CW / NC), int32_t((W + 3) * es));
      for (int64_t n = 0; n < N; n += NC) {
        const int64_t img = n / (H * W), y = (n % (H * W)) / W, x = n % W;
        int32_t v = int32_t(((img * (H + 2) + y + 1) * (W + 2) + x + 1) * es);
        if (!bf16) v |= (x == 0 ? 1 : 0) | (x + 4 == W ? 2 : 0);
        cb[size_t(n / NC)] = v;
      }
      int rc = upload(cb, cbt);
      if (rc) return rc;
    }
    rp.colbase = *cbt;
  }
  rp.conv = conv ? 1 : 0;
  rp.conv_h = conv ? int(conv->height) : 0;
  rp.conv_w = conv ? int(conv->width) : 0;
  if (conv) {   // the unit of the stage descriptors is a channel of X
    rp.row_bytes = uint32_t(chs);
    rp.n_bytes = uint32_t(chs);
    rp.last_row = int(m->K / 9 - 1);
    rp.src_rows = pl.SRC / 9;
  }
  rp.a2 = pl.A2; rp.a3 = m->a[2]; rp.a4 = m->a[3]; rp.R = pl.R;
  rp.fpm = fpm;
  rp.tm = pl.A2 * m->a[2] * m->a[3];
  for (int r = 0; r < 16; ++r) rp.rowofs[r] = (r / m->a[3]) * m->a[2] * m->a[3] + r % m->a[3];
  rp.ntiles = int(ntiles);
  rp.lgS = lgS;
  const int64_t tiles_per_wg = (4 >> lgS) * CT;
  rp.ct = CT;
  rp.ct_cnt = tab->max_stages;
  const int64_t nquads = (ntiles + tiles_per_wg - 1) / tiles_per_wg;
  // one-dimensional grid, items dealt to the XCDs in blocks (see RegParams)
  // (measured on one box, us: conv5 18.0 / 18.2 / 18.2 with order 1 / 0 / 2; conv3 bf16 20.2 / 17.8 / 17.6; WRN 90.9 / 76.4 / 75.9)
  rp.order = (m->e[2] == 1 && nquads <= 64) ? 1 : nquads >= 8 ? 2 : 0;
  const int64_t items = int64_t(ncl) * m->a[2] * nquads;
  const int64_t per_xcd = rp.order == 2 ? int64_t(ncl) * m->a[2] * ((nquads + 7) / 8) : (items + 7) / 8;
  if (per_xcd * 8 > 0x7fffffff) return RBGP_EUNSUPPORTED;
  rp.ncl = ncl;
  rp.per_xcd = int(per_xcd);
  rp.ngroups = int(nquads);
  reg_fn fn = dual     ? nullptr
              : bf16   ? (lean ? rbgp_reg_bf16_lean_kernel(pl.KC, pl.RS, G, CW) : rbgp_reg_bf16_kernel(pl.KC, pl.RS, G, CW))
              : CT > 1 ? find_reg_tiles(pl.KC, pl.RS, NGf)
              : lean   ? find_reg_lean(pl.KC, pl.RS, taps, NGf)
              : ge   ? (taps ? ge->taps_fn : ge->global_fn)
              : taps ? e->taps_fn
                     : e->global_fn;
  if (!fn && !dual) return RBGP_EUNSUPPORTED;
  if (lds > 64 * 1024 && fn)   // (cheap host-side call; repeated because fn varies with the knobs)
    RBGP_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 int(lds)));
  if (dual) {
    DualParams dq;
    dq.r = rp;
    const rbgp_reg_dual &du = m->reg_dual;
    const int NP4 = (pl.NO + 3) / 4 * 4, n_row = m->a[2] * 4 * NP4, cmax = std::max(du.max_wave, 1);
    dq.rt_stride = NP4;
    dq.cmax = cmax;
    dq.o_stages = n_row;
    dq.o_quads = dq.o_stages + du.nq * 4 * cmax * 4;
    int32_t **dtab = &st->dual_tab[conv ? 1 : 0];
    if (!*dtab) {   // (the fused convolution's table goes with its row table when the geometry changes)
      std::vector<int32_t> h(size_t(dq.o_quads) + size_t(du.nq) * 8, 0);
      const std::vector<int32_t> &rt = conv ? st->rowtab_conv_host : st->rowtab_host;
      for (int u = 0; u < m->a[2]; ++u)
        for (int o = 0; o < pl.NO; ++o)
          for (int gg = 0; gg < 4; ++gg) h[(size_t(u) * 4 + gg) * NP4 + o] = rt[(size_t(u) * pl.NO + o) * 4 + gg];
      for (int wv = 0; wv < du.nq * 4; ++wv)
        for (int sg = 0; sg < cmax; ++sg)
          for (int k = 0; k < 3; ++k)
            h[size_t(dq.o_stages) + (size_t(wv) * cmax + sg) * 4 + k] = du.stages[(size_t(wv) * 3 + k) * 64 + sg];
      for (int q = 0; q < du.nq; ++q)
        for (int k = 0; k < 4; ++k) {
          h[size_t(dq.o_quads) + size_t(q) * 8 + k] = du.members[size_t(q) * 4 + k];
          h[size_t(dq.o_quads) + size_t(q) * 8 + 4 + k] = du.counts[size_t(q) * 4 + k];
        }
      int rc = upload(h, dtab);
      if (rc) return rc;
    }
    dq.tab = *dtab;
    rbgp_dual_fn dfn = rbgp_reg_dual_kernel(pl.KC);
    hipLaunchKernelGGL(dfn, dim3(unsigned(8 * per_xcd)), dim3(512), lds, static_cast<hipStream_t>(stream), dq);
  } else {
    hipLaunchKernelGGL(fn, dim3(unsigned(8 * per_xcd)), dim3(256), lds, static_cast<hipStream_t>(stream), rp);
  }
  RBGP_HIP(hipGetLastError());
  return RBGP_OK;
}
