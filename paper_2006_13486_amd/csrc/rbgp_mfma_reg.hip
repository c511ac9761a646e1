// Register-streaming MFMA kernels for O = W_s x I (Section 5, "GPU
// Implementation"), fp32.
//
// Work decomposition.  One wavefront owns: a cluster of U tile rows u_o, one G_i
// vertex u_i (so, per tile row, the R = |G_r.U|*|G_b.U| rows that share a column
// set: row repetition, Section 5) and 64 columns of O.  It walks the union of the
// cluster's nonzero tiles (tile skipping through G_o's adjacency, Section 5)
// stage by stage; a stage is VC columns of G_r of one tile.  The rows of I a stage
// touches are loaded straight from global memory into VGPRs and each loaded row
// is used for every tile row of the cluster that has the tile: the register-level
// reuse the paper obtains from row repetition, extended across tile rows.  No
// LDS, no barrier: waves are independent; loads are issued two stages ahead, slot
// by slot, into the registers the previous MFMAs just released, and the
// compiler's vmcnt bookkeeping provides the software pipeline.
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
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

struct RegParams {
  const float *Wp;
  const float *I;
  float *O;
  const int32_t *rowtab;   // [a_i][NO*4]: stage-relative I row of each contraction step (padding -> 0)
  const int32_t *stages;   // [ncl][2+U][64]: per stage (one per lane, first real stage in lane 2) the
                           //   base row of the stage, the bit mask of MFMA groups with work, then per
                           //   cluster member the index of its weight fragment block; -1 (mask 0) in
                           //   lanes 0, 1 and past the end (sentinel stages) and when the member does
                           //   not have the tile
  const int32_t *counts;   // [ncl] stages of each cluster (<= 58)
  const int32_t *members;  // [ncl][U] tile rows of each cluster (-1: none)
  int64_t N, ldI, ldO;
  uint32_t i_bytes, w_bytes;  // extents of I and of the packed weights (buffer descriptors)
  int a2, a3, a4, R;
  int items_per_tile;      // ncl * a3
  int wgs_per_tile;        // ceil(items_per_tile / waves per workgroup)
  int ntiles;              // ceil(N / 64)
};

constexpr int kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format (gfx9 family)
constexpr int kOob = 0x40000000;        // byte offset beyond any packed weight buffer (reads return 0)

__device__ __forceinline__ f32x4 load_x4(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
  return f32x4{__uint_as_float(v[0]), __uint_as_float(v[1]), __uint_as_float(v[2]), __uint_as_float(v[3])};
}

// KC: contraction steps per stage; RS: weight rows per tile row in a 16-row MFMA group;
// P: MFMA groups per wave (cluster size U = P * 16 / RS).
template <int KC, int RS, int P>
__global__ __launch_bounds__(256) void spmm_reg(RegParams p) {
  constexpr int MG = 16 / RS;            // tile rows per MFMA group
  constexpr int U = MG * P;
  constexpr int NO = (KC + 3) / 4;       // load slots per stage (4 contraction steps each)
  constexpr int NQ = (NO + 3) / 4;       // weight registers per group and stage come as NQ 16-byte loads
  constexpr int QB = 4 * RS * 16;        // bytes of one such load across the fragment
  constexpr int FB = NQ * QB;            // bytes of one weight fragment (one tile row, one G_i vertex)
  constexpr int CW = 64;                 // columns per wave
  const int lane = threadIdx.x & 63;
  const int wid = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  const int wpw = __builtin_amdgcn_readfirstlane(int(blockDim.x) >> 6);

  // same columns of I -> same XCD (one L2): workgroups are dealt round-robin to the 8 XCDs
  const int bid = blockIdx.x, xcd = bid & 7, slot = bid >> 3;
  const int nt = xcd + 8 * (slot / p.wgs_per_tile);
  const int item = (slot % p.wgs_per_tile) * wpw + wid;
  if (nt >= p.ntiles || item >= p.items_per_tile) return;
  const int cl = item / p.a3, u3 = item - cl * p.a3;
  const int64_t n0 = int64_t(nt) * CW;
  const int g = lane >> 4, j = lane & 15;
  const int mi = j / RS, ri = j % RS;    // as a weight lane: member of the group, row of the member

  // byte offset of this lane's 16 bytes in every slot, relative to the stage base.  Columns
  // past N read whatever follows inside I (or zeros past its end): they are never stored.
  int off[NO];
  {
    const int32_t *rt = p.rowtab + u3 * (NO * 4) + g;
#pragma unroll
    for (int o = 0; o < NO; ++o) off[o] = int((int64_t(rt[o * 4]) * p.ldI + j * 4) * 4);
  }
  const int alane = (g * RS + ri) * 16;

  // stage table of the cluster, one stage per lane, read back with readlane
  const int32_t *stg = p.stages + int64_t(cl) * (2 + U) * 64 + lane;
  const int tb = stg[0], ta = stg[64];
  int tf[U];
#pragma unroll
  for (int u = 0; u < U; ++u) tf[u] = stg[(2 + u) * 64];
  const int cnt = p.counts[cl];
  // Drain the table loads here: a wait for them inside the loop would run on every
  // iteration and drain the prefetched stages with it.
  __builtin_amdgcn_s_waitcnt(0);

  f32x16 acc[P][4];
#pragma unroll
  for (int pg = 0; pg < P; ++pg)
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[pg][w][v] = 0.f;

  const __amdgpu_buffer_rsrc_t rw =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.Wp), 0, p.w_bytes, kRsrcFlags);

  // Loads are unconditional so that the wait counts are exact: a stage past the end reads
  // I through a descriptor of zero extent and a tile row that lacks the tile reads its
  // weights at an offset past the buffer; both return zeros without touching memory.
  auto b_rsrc = [&](int s, int *sofs) {
    const int base_row = __builtin_amdgcn_readlane(tb, s);
    *sofs = int((int64_t(base_row < 0 ? 0 : base_row) * p.ldI + n0) * 4);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.I), 0, base_row >= 0 ? p.i_bytes : 0u,
                                             kRsrcFlags);
  };
  // per-lane byte offset of the weights of MFMA group pg at stage s
  auto a_voff = [&](int s, int pg) {
    int voff = kOob;
#pragma unroll
    for (int mm = 0; mm < MG; ++mm) {
      const int frag = __builtin_amdgcn_readlane(tf[pg * MG + mm], s);
      const int sv = frag >= 0 ? (frag + u3) * FB : kOob;
      voff = mi == mm ? sv : voff;
    }
    return voff + alane;
  };
  // One stage: MFMAs of stage s from (B, A); every B slot and every weight quad is
  // refilled for stage s + 2 right after its last use.  One uniform branch per MFMA group
  // and stage; the last group's pass does the refills, and both sides of its branch issue
  // the same loads in the same order.
  auto stage = [&](int s, f32x4 (&B)[NO], f32x4 (&A)[P][NQ]) {
    const int active = __builtin_amdgcn_readlane(ta, s);
    int sofs;
    const __amdgpu_buffer_rsrc_t rb2 = b_rsrc(s + 2, &sofs);
    int av[P];
#pragma unroll
    for (int pg = 0; pg < P; ++pg) av[pg] = a_voff(s + 2, pg);
    static_for<0, P>([&](auto pgc) {
      constexpr int pg = decltype(pgc)::value;
      if (active & (1 << pg)) {
        static_for<0, NO>([&](auto oc) {
          constexpr int o = decltype(oc)::value;
          const float a = A[pg][o / 4][o % 4];
#pragma unroll
          for (int w = 0; w < 4; ++w)
            acc[pg][w] = __builtin_amdgcn_mfma_f32_16x16x1f32(a, B[o][w], acc[pg][w], 0, 0, 0);
          if constexpr (pg == P - 1) {
            B[o] = load_x4(rb2, off[o], sofs);
            if constexpr (o % 4 == 3 || o == NO - 1) {
#pragma unroll
              for (int p2 = 0; p2 < P; ++p2) A[p2][o / 4] = load_x4(rw, av[p2], (o / 4) * QB);
            }
          }
        });
      } else if constexpr (pg == P - 1) {
        static_for<0, NO>([&](auto oc) {
          constexpr int o = decltype(oc)::value;
          B[o] = load_x4(rb2, off[o], sofs);
          if constexpr (o % 4 == 3 || o == NO - 1) {
#pragma unroll
            for (int p2 = 0; p2 < P; ++p2) A[p2][o / 4] = load_x4(rw, av[p2], (o / 4) * QB);
          }
        });
      }
    });
  };

  // Two register sets alternate.  The first two passes find only sentinel stages (lanes 0
  // and 1 of the table): they multiply nothing and just start the loads of the first two
  // real stages, so the loop needs no separate prologue and every wait count is exact.
  f32x4 B0[NO], B1[NO];
  f32x4 A0[P][NQ], A1[P][NQ];
#pragma unroll
  for (int o = 0; o < NO; ++o) B0[o] = B1[o] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int pg = 0; pg < P; ++pg)
#pragma unroll
    for (int q = 0; q < NQ; ++q) A0[pg][q] = A1[pg][q] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < cnt + 2; s += 2) {
    stage(s, B0, A0);
    stage(s + 1, B1, A1);
  }

  // epilogue: add the four blocks (contraction steps 0..3 mod 4).  Register t of the sum
  // holds weight row 4*(lane/16) + t of the group, lane j the columns 4j + w.
  const bool vec_ok = (p.ldO % 4 == 0) && (reinterpret_cast<uintptr_t>(p.O) % 16 == 0) && (n0 + j * 4 + 4 <= p.N);
#pragma unroll
  for (int pg = 0; pg < P; ++pg) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float v[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) v[w] = (acc[pg][w][t] + acc[pg][w][4 + t]) + (acc[pg][w][8 + t] + acc[pg][w][12 + t]);
      const int i16 = 4 * g + t, mm = i16 / RS, r = i16 % RS;
      const int u1 = p.members[cl * U + pg * MG + mm];
      if (u1 >= 0 && r < p.R) {
        const int u2 = r / p.a4, u4 = r - u2 * p.a4;
        const int64_t m = ((int64_t(u1) * p.a2 + u2) * p.a3 + u3) * p.a4 + u4;
        float *o = p.O + m * p.ldO + n0 + j * 4;
        if (vec_ok) {
          *reinterpret_cast<f32x4 *>(o) = f32x4{v[0], v[1], v[2], v[3]};
        } else {
#pragma unroll
          for (int w = 0; w < 4; ++w)
            if (n0 + j * 4 + w < p.N) o[w] = v[w];
        }
      }
    }
  }
}

typedef void (*reg_fn)(RegParams);
struct RegEntry {
  int KC, RS, P;
  reg_fn fn;
};
#define RBGP_R(KC, RS) {KC, RS, 1, spmm_reg<KC, RS, 1>}, {KC, RS, 2, spmm_reg<KC, RS, 2>}
const RegEntry kRegTable[] = {RBGP_R(8, 4),  RBGP_R(18, 2), RBGP_R(36, 2), RBGP_R(72, 2),
                              RBGP_R(18, 4), RBGP_R(36, 4), RBGP_R(72, 4),
                              RBGP_R(18, 8), RBGP_R(36, 8), RBGP_R(72, 8)};

const RegEntry *find_reg(int KC, int RS, int P) {
  for (const RegEntry &e : kRegTable)
    if (e.KC == KC && e.RS == RS && e.P == P) return &e;
  return nullptr;
}

struct RegTables {  // device tables for one cluster size U
  int U = 0, ncl = 0, smax = 0;
  int32_t *stages = nullptr, *counts = nullptr, *members = nullptr;
};

struct RegState {
  int32_t *rowtab = nullptr;
  std::map<int, RegTables> by_u;
};

template <typename T>
int upload(const std::vector<T> &h, T **d) {
  RBGP_HIP(hipMalloc(reinterpret_cast<void **>(d), h.size() * sizeof(T) + 16));
  RBGP_HIP(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
  return RBGP_OK;
}

// Group the tile rows into clusters of U whose adjacency lists overlap most
// (greedy: seed with the lowest free tile row, add the free row that enlarges the
// union of tiles least), and list for every cluster the stages it walks.
int build_tables(const rbgp_mask *m, int U, RegTables *t) {
  const rbgp_reg_plan &pl = m->reg;
  const int a1 = m->a[0], c1 = m->c[0], d1 = m->d[0], a3 = m->a[2];
  const int ncl = (a1 + U - 1) / U;
  std::vector<int32_t> members(size_t(ncl) * U, -1);
  std::vector<char> used(a1, 0);
  std::vector<std::vector<char>> has(a1, std::vector<char>(c1, 0));
  for (int u = 0; u < a1; ++u)
    for (int j = 0; j < d1; ++j) has[u][m->adj[0][size_t(u) * d1 + j]] = 1;
  for (int c = 0; c < ncl; ++c) {
    std::vector<char> uni(c1, 0);
    for (int k = 0; k < U; ++k) {
      int best = -1, best_grow = 1 << 30;
      for (int u = 0; u < a1; ++u) {
        if (used[u]) continue;
        int grow = 0;
        for (int v = 0; v < c1; ++v) grow += has[u][v] && !uni[v];
        if (grow < best_grow) { best_grow = grow; best = u; }
      }
      if (best < 0) break;
      used[best] = 1;
      members[size_t(c) * U + k] = best;
      for (int v = 0; v < c1; ++v) uni[v] |= has[best][v];
    }
  }
  std::vector<int32_t> counts(ncl, 0);
  std::vector<std::vector<int32_t>> rows(ncl);
  int smax = 0;
  for (int c = 0; c < ncl; ++c) {
    for (int v1 = 0; v1 < c1; ++v1) {
      bool any = false;
      for (int k = 0; k < U; ++k) any |= members[size_t(c) * U + k] >= 0 && has[members[size_t(c) * U + k]][v1];
      if (!any) continue;
      for (int sg = 0; sg < pl.NSTG; ++sg) {
        rows[c].push_back(int32_t((int64_t(v1) * m->c[1] + int64_t(sg) * pl.VC) * m->c[2] * m->c[3]));
        int active = 0;
        for (int k = 0; k < U; ++k)
          if (members[size_t(c) * U + k] >= 0 && has[members[size_t(c) * U + k]][v1]) active |= 1 << (k / pl.MG);
        rows[c].push_back(active);
        for (int k = 0; k < U; ++k) {
          const int u1 = members[size_t(c) * U + k];
          int frag = -1;
          if (u1 >= 0 && has[u1][v1]) {
            int j1 = 0;
            while (m->adj[0][size_t(u1) * d1 + j1] != v1) ++j1;
            frag = int32_t(((int64_t(u1) * d1 + j1) * pl.NSTG + sg) * a3);
          }
          rows[c].push_back(frag);
        }
        ++counts[c];
      }
    }
    smax = std::max(smax, counts[c]);
  }
  if (smax > 58) return RBGP_EUNSUPPORTED;   // one stage per lane plus sentinels
  std::vector<int32_t> stages(size_t(ncl) * (2 + U) * 64, -1);
  for (int c = 0; c < ncl; ++c) {
    for (int ln = 0; ln < 64; ++ln) stages[(size_t(c) * (2 + U) + 1) * 64 + ln] = 0;   // no group has work
    for (int st = 0; st < counts[c]; ++st)
      for (int f = 0; f < 2 + U; ++f)
        stages[(size_t(c) * (2 + U) + f) * 64 + 2 + st] = rows[c][size_t(st) * (2 + U) + f];
  }
  t->U = U; t->ncl = ncl; t->smax = smax;
  int rc = upload(stages, &t->stages);
  if (rc) return rc;
  rc = upload(counts, &t->counts);
  if (rc) return rc;
  return upload(members, &t->members);
}

}  // namespace

bool rbgp_reg_covers(const rbgp_mask *m) {
  const rbgp_reg_plan &p = m->reg;
  if (!p.ok) return false;
  if (int64_t(m->M) * m->rowdeg * 2 >= (int64_t(1) << 31)) return false;
  return find_reg(p.KC, p.RS, 1) != nullptr;
}

void rbgp_reg_release(void *state) {
  RegState *st = static_cast<RegState *>(state);
  if (!st) return;
  if (st->rowtab) (void)hipFree(st->rowtab);
  for (auto &kv : st->by_u) {
    if (kv.second.stages) (void)hipFree(kv.second.stages);
    if (kv.second.counts) (void)hipFree(kv.second.counts);
    if (kv.second.members) (void)hipFree(kv.second.members);
  }
  delete st;
}

int rbgp_reg_launch(const rbgp_mask *m, void **state, int tune_u, int64_t N, const void *packed, const void *I,
                    int64_t ldI, float *O, int64_t ldO, void *stream) {
  const rbgp_reg_plan &pl = m->reg;
  if (!rbgp_reg_covers(m)) return RBGP_EUNSUPPORTED;
  // I and the packed weights are addressed through 32-bit buffer offsets
  const int64_t i_bytes = ((m->K - 1) * ldI + N) * 4, w_bytes = pl.packed_elems * 4;
  if (i_bytes >= (int64_t(1) << 31) || w_bytes >= (int64_t(1) << 30)) return RBGP_EUNSUPPORTED;
  RegState *st = static_cast<RegState *>(*state);
  if (!st) {
    st = new (std::nothrow) RegState();
    if (!st) return RBGP_ENOMEM;
    *state = st;
  }
  if (!st->rowtab) {
    const int a3 = m->a[2], d3 = m->d[2], c3 = m->c[2], c4 = m->c[3];
    std::vector<int32_t> rt(size_t(a3) * pl.NO * 4, 0);
    for (int u3 = 0; u3 < a3; ++u3)
      for (int kk = 0; kk < pl.KC; ++kk) {
        const int v4 = kk % c4, j3 = (kk / c4) % d3, vv = kk / (c4 * d3);
        rt[size_t(u3) * pl.NO * 4 + kk] = (vv * c3 + m->adj[2][size_t(u3) * d3 + j3]) * c4 + v4;
      }
    int rc = upload(rt, &st->rowtab);
    if (rc) return rc;
  }
  const int cw = 64;
  const int64_t ntiles = (N + cw - 1) / cw;
  // MFMA groups per wave (cluster size U = P * MG): 2 if the launch then still has >= 1024
  // waves (one per SIMD) and the cluster's stage list fits the per-lane table, else 1
  int P = tune_u;
  const bool auto_p = P <= 0;
  if (auto_p) P = (int64_t((m->a[0] + 2 * pl.MG - 1) / (2 * pl.MG)) * m->a[2] * ntiles >= 1024) ? 2 : 1;
  const RegEntry *e = nullptr;
  RegTables *tp = nullptr;
  int U = 0;
  for (;; --P) {
    e = find_reg(pl.KC, pl.RS, P);
    if (!e) return RBGP_EUNSUPPORTED;
    U = P * pl.MG;
    tp = &st->by_u[U];
    int rc = tp->stages ? RBGP_OK : build_tables(m, U, tp);
    if (rc == RBGP_OK) break;
    if (rc != RBGP_EUNSUPPORTED || !auto_p || P == 1) return rc;
  }
  RegTables &t = *tp;
  RegParams rp;
  rp.Wp = static_cast<const float *>(packed);
  rp.I = static_cast<const float *>(I);
  rp.O = O;
  rp.rowtab = st->rowtab;
  rp.stages = t.stages; rp.counts = t.counts; rp.members = t.members;
  rp.N = N; rp.ldI = ldI; rp.ldO = ldO;
  rp.i_bytes = uint32_t(i_bytes); rp.w_bytes = uint32_t(w_bytes);
  rp.a2 = m->a[1]; rp.a3 = m->a[2]; rp.a4 = m->a[3]; rp.R = pl.R;
  rp.items_per_tile = t.ncl * m->a[2];
  const int wpw = 4;
  rp.wgs_per_tile = (rp.items_per_tile + wpw - 1) / wpw;
  rp.ntiles = int(ntiles);
#ifdef RBGP_EXPERIMENT
  rp.mode = getenv("RBGP_MODE") ? atoi(getenv("RBGP_MODE")) : 0;
#endif
#ifdef RBGP_EXPERIMENT
  rp.mode = getenv("RBGP_MODE") ? atoi(getenv("RBGP_MODE")) : 0;
#endif
  const int64_t nblocks = 8 * ((ntiles + 7) / 8) * rp.wgs_per_tile;
  if (nblocks > 0x7fffffff) return RBGP_EUNSUPPORTED;
  hipLaunchKernelGGL(e->fn, dim3(unsigned(nblocks)), dim3(wpw * 64), 0, static_cast<hipStream_t>(stream), rp);
  RBGP_HIP(hipGetLastError());
  return RBGP_OK;
}
