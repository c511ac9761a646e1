// Register-streaming MFMA kernel for O = W_s x I (Section 5, "GPU Implementation"), fp32, for masks
// whose rows repeat in groups of 5..8 (R = |G_r.U| * |G_b.U|, Section 5 "row repetition"): the 16 rows
// of an MFMA group are two tile rows, and this kernel pairs them tile by tile.
//
// The kernel of rbgp_mfma_reg.hip gives a wave a fixed pair of tile rows and walks the union of their
// tiles; where only one of the two has a tile, half of the MFMA rows multiply zeros.  Here the tile
// rows come in quads (L0, L1, H0, H1; chosen on the host, rbgp_reg_plan_dual) and wave (x, y) of a
// quad walks the tiles that L_x and H_y SHARE (tile skipping through G_o's adjacency, Section 5):
// L_x's weights in rows 0..7 ("lo") of the group, H_y's in rows 8..15 ("hi").  With L0, L1 and H0, H1
// of complementary tile sets every stage multiplies 16 rows of the mask and the two waves of a tile
// row together walk its d_o tiles, the minimum.  The eight waves of a workgroup are the four pairs of a
// quad on two neighbouring column tiles; waves (x, 0) and (x, 1) of a column tile sit on one SIMD (waves
// k and k + 4 of a workgroup do), where their stage counts add up to L_x's tiles however the tiles
// divide between H0 and H1.  At the end the partial sums of a tile row (two waves each) meet in LDS.
// Everything else (loads of I straight into VGPRs, 16x16x1 four-block MFMA, weight fragments, stage
// descriptors, the fused 3x3 convolution's addressing) is the scheme of rbgp_mfma_reg.hip, whose
// packed layout this kernel reads unchanged; with two waves per SIMD a wave has 256 registers and
// keeps one stage of loads in flight (each slot is refilled for the next stage right after its use).
#include <hip/hip_runtime.h>

#include "rbgp_reg_common.h"

using namespace rbgp_reg;

namespace {

// KC: contraction steps per stage.  RegParams: stages / counts / members hold the tables of
// rbgp_reg_dual (per quad and wave), ncl the number of quads.
template <int KC>
__global__ __launch_bounds__(512) void spmm_reg_dual(DualParams dp) {
  const RegParams &p = dp.r;
  constexpr int RS = 8;
  constexpr int NO = (KC + 3) / 4;       // load slots per stage (4 contraction steps each)
  constexpr int NQ = (NO + 3) / 4;       // weight registers per stage come as NQ 16-byte loads
  constexpr int QB = 4 * RS * 16;        // bytes of one such load across the fragment
  constexpr int FB = NQ * QB;            // bytes of one weight fragment (one tile row, one G_i vertex)
  constexpr int CW = 64;                 // columns per wave
  extern __shared__ __attribute__((aligned(16))) unsigned char xlds[];
  const int lane = threadIdx.x & 63;
  const int wid = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  // wave k: SIMD k & 3 = (column tile of the pair, x); y = k >> 2
  const int ct = (wid >> 1) & 1, x = wid & 1, y = wid >> 2;

  // A workgroup is one (quad, G_i vertex) pair on two neighbouring column tiles, four waves each (see wg_coord
  // for how the workgroups map to the XCDs).
  WgCoord wg;
  if (!wg_coord(p, &wg)) return;   // (the whole workgroup leaves)
  const int cl = wg.cl, u3 = wg.u3;
  const int nt = (wg.ntq << 1) + ct;
  const int64_t n0 = int64_t(nt) * CW;
  const uint32_t n0b = p.conv ? 0u : uint32_t(nt) * uint32_t(CW * 4);
  const int g = lane >> 4, j = lane & 15;
  const int mi = j / RS, ri = j % RS;    // as a weight lane: lo or hi half, row of the half

  // Everything the prologue needs is requested at once, with 16-byte loads.
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  const int32_t *tab = dp.tab;
  const i32x4 *qd = reinterpret_cast<const i32x4 *>(tab + dp.o_quads) + cl * 2;
  const i32x4 quad_rows = qd[0], quad_counts = qd[1];
  const int cmax = dp.cmax;
  // (the kernel arguments the epilogue needs, read here with the tables: fetched after the loop, they would add
  // scalar-load latencies to the end of every wave)
  float *const out = p.O;
  const int64_t out_ld = p.ldO, out_n = p.N;
  const int out_tm = p.tm, out_a4 = p.a4, out_r = p.R;
  const i32x4 *stg = reinterpret_cast<const i32x4 *>(tab + dp.o_stages) + ((cl * 2 + x) * 2 + y) * cmax;
  const i32x4 entry = stg[lane < cmax ? lane : cmax - 1];
  // stage-relative row of I of contraction step 4 * o + g, for this lane's g
  int rrow[NO];
  {
    constexpr int NP = (NO + 3) / 4;
    const i32x4 *rt = reinterpret_cast<const i32x4 *>(tab) + (u3 * 4 + g) * NP;
    i32x4 piece[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) piece[k] = rt[k];
#pragma unroll
    for (int o = 0; o < NO; ++o) rrow[o] = piece[o / 4][o % 4];
  }
  const int rowL = __builtin_amdgcn_readfirstlane(x ? quad_rows[1] : quad_rows[0]);
  const int rowH = __builtin_amdgcn_readfirstlane(y ? quad_rows[3] : quad_rows[2]);
  const int cnt = __builtin_amdgcn_readfirstlane(quad_counts[x * 2 + y]);   // stages of this wave
  const int tb = lane < cnt ? entry[0] : -1, tflo = lane < cnt ? entry[1] : -1, tfhi = lane < cnt ? entry[2] : -1;
  const int rov = p.rowofs[lane & 15];   // lane-held copy, read back with bpermute in the epilogue
  auto table_lane = [&](int s) { return s < 63 ? s : 63; };   // lanes past the count hold sentinels

  // byte offset of this lane's 16 bytes in every slot, relative to the stage base
  int off[NO];
  if (p.conv) {
    const int cb = p.colbase[nt < p.ntiles ? int(n0 >> 2) + j : 0];
    const int colbase = cb & ~3;
#pragma unroll
    for (int o = 0; o < NO; ++o) off[o] = rrow[o] + colbase;
  } else {
#pragma unroll
    for (int o = 0; o < NO; ++o) off[o] = rrow[o] * (int(p.ldI) * 4) + j * 16;   // < 2^31: checked by the host
  }
  const int alane = (g * RS + ri) * 16;
  const bool valid = nt < p.ntiles;

  const __amdgpu_buffer_rsrc_t rw =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.Wp), 0, p.w_bytes, kRsrcFlags);
  // Once per stage (= per table lane), with vector instructions: where the stage's part of I starts
  // and how far it extends, and where the weights of its two halves are; the loop reads these back
  // with readlane.  (Descriptor conventions as in rbgp_mfma_reg.hip.)
  const int tbu = p.conv ? int(uint32_t(tb < 0 ? 0 : tb) / 9u) : (tb < 0 ? 0 : tb);
  const uint64_t i_first = reinterpret_cast<uint64_t>(p.I) + uint64_t(uint32_t(tbu)) * p.row_bytes + n0b;
  const int ib_lo = int(uint32_t(i_first)), ib_hi = int(uint32_t(i_first >> 32));
  const int rows_left = p.last_row - tbu < p.src_rows ? p.last_row - tbu : p.src_rows;
  const int ib_ext = (tb >= 0 && valid) ? int(uint32_t(rows_left) * p.row_bytes + (p.n_bytes - n0b)) : 0;
  const int aoff_lo = (tflo >= 0 && rowL >= 0) ? ((rowL * p.fpm + tflo) * p.a3 + u3) * FB : kOob;
  const int aoff_hi = (tfhi >= 0 && rowH >= 0) ? ((rowH * p.fpm + tfhi) * p.a3 + u3) * FB : kOob;
  auto b_rsrc = [&](int s) {
    const int tl = table_lane(s);
    const uint64_t base = uint64_t(uint32_t(__builtin_amdgcn_readlane(ib_lo, tl))) |
                          (uint64_t(uint32_t(__builtin_amdgcn_readlane(ib_hi, tl))) << 32);
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(base), 0, __builtin_amdgcn_readlane(ib_ext, tl),
                                             kRsrcFlags);
  };
  auto a_addr = [&](int s) {
    const int tl = table_lane(s);
    const int lo = __builtin_amdgcn_readlane(aoff_lo, tl), hi = __builtin_amdgcn_readlane(aoff_hi, tl);
    return (mi == 0 ? lo : hi) + alane;
  };

  // Drain the table loads here: a wait for them inside the loop would drain the prefetched stages too.
  __builtin_amdgcn_s_waitcnt(0);

  f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

  f32x4 B[NO];
  f32x4 A[NQ];
  // Loads of stage 0, the eight waves of the workgroup in step: the load path of the CU takes the
  // instructions in the order they are issued and returns their data in that order, so without the
  // barriers the waves that issue first get their whole stage before the others get their first row,
  // and half of the SIMD's waves sit idle at the start (measured: 0.4 us per launch).
  {
    const __amdgpu_buffer_rsrc_t rb = b_rsrc(0);
    const int av = a_addr(0);
    static_for<0, NO>([&](auto oc) {
      constexpr int o = decltype(oc)::value;
      B[o] = load_x4(rb, off[o], 0);
      if constexpr (o % 4 == 3 || o == NO - 1) A[o / 4] = load_x4(rw, av, (o / 4) * QB);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (o != NO - 1) __builtin_amdgcn_s_barrier();
    });
  }
  // One stage: every B slot and every weight quad is refilled for the next stage right after its
  // last use.  Loads are unconditional (sentinel stages and absent halves read zeros through the
  // descriptors) so that the wait counts are exact.
  for (int s = 0; s < cnt; ++s) {
    // the wave of the SIMD with more stages left goes first: the two advance together, and the
    // loads of each have the other's stage to arrive in
    {
      const int left = cnt - s;
      if (left >= 4) __builtin_amdgcn_s_setprio(3);
      else if (left == 3) __builtin_amdgcn_s_setprio(2);
      else if (left == 2) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
    }
    const __amdgpu_buffer_rsrc_t rb = b_rsrc(s + 1);
    const int av = a_addr(s + 1);
    static_for<0, NO>([&](auto oc) {
      constexpr int o = decltype(oc)::value;
      const float a = A[o / 4][o % 4];
      const f32x4 b = B[o];
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x1f32(a, b[c], acc[c], 0, 0, 0);
      B[o] = load_x4(rb, off[o], 0);
      if constexpr (o % 4 == 3 || o == NO - 1) {
        // (a last quad that is used in part stays whole until here: a register of it that the compiler
        // gave to something else would have to wait for the quad's pending load, i.e. for every load)
        asm volatile("" ::"v"(A[o / 4]));
        A[o / 4] = load_x4(rw, av, (o / 4) * QB);
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the loads where they are: the wait counts depend on it
    });
  }
  __builtin_amdgcn_s_waitcnt(0);

  // Epilogue.  Unit t: the four blocks (contraction steps 0..3 mod 4) added; it holds weight row
  // 4 * (lane / 16) + t of the group -- lanes 0..31 rows of L_x, lanes 32..63 rows of H_y -- and lane j
  // the columns 4j + c.  Of a column tile's four waves, (0, 0) stores L0 and H0, (1, 1) stores L1 and
  // H1; the other two leave their units in LDS: L_x = (x, 0) + (x, 1), H_y = (0, y) + (1, y).
  auto unit = [&](int t) {
    f32x4 v;
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = (acc[c][t] + acc[c][4 + t]) + (acc[c][8 + t] + acc[c][12 + t]);
    return v;
  };
  f32x4 *const x4 = reinterpret_cast<f32x4 *>(xlds);   // [column tile][x of the giver][unit][lane]
  if (x != y) {
#pragma unroll
    for (int t = 0; t < 4; ++t) x4[((ct * 2 + x) * 4 + t) * 64 + lane] = unit(t);
  }
  __syncthreads();
  if (x != y) return;
  const bool vec_ok = (out_ld % 4 == 0) && (reinterpret_cast<uintptr_t>(out) % 16 == 0) && (n0 + j * 4 + 4 <= out_n);
  const int u1 = g < 2 ? rowL : rowH;
  // wave (0, 0): lo rows from (0, 1), hi rows from (1, 0); wave (1, 1): lo rows from (1, 0), hi rows from (0, 1)
  const int giver = g < 2 ? x : 1 - x;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const f32x4 other = x4[((ct * 2 + giver) * 4 + t) * 64 + lane];
    const f32x4 mine = unit(t);
    // (wave (., 0)'s sum first for a lo row, wave (0, .)'s for a hi row, whichever wave adds them)
    const f32x4 v = mine + other;
    const int r = 4 * (g & 1) + t;
    const int ro = __builtin_amdgcn_ds_bpermute(r * 4, rov);
    if (valid && u1 >= 0 && r < out_r) {
      const int64_t m = int64_t(u1) * out_tm + u3 * out_a4 + ro;
      float *o = out + m * out_ld + n0 + j * 4;
      if (vec_ok) {
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(o));
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (n0 + j * 4 + c < out_n) o[c] = v[c];
      }
    }
  }
}

}  // namespace

rbgp_dual_fn rbgp_reg_dual_kernel(int KC) {
  switch (KC) {
    case 8: return spmm_reg_dual<8>;
    case 18: return spmm_reg_dual<18>;
    case 32: return spmm_reg_dual<32>;
    case 36: return spmm_reg_dual<36>;
    case 72: return spmm_reg_dual<72>;
  }
  return nullptr;
}
