// Device part of the library: index tables, the pack (permutation) kernel and
// the SpMM kernels for gfx950, with their launchers and the C entry points that
// touch the GPU.
//
// O = W_s x I (Section 5, "GPU Implementation").  Two kernel families:
//
//  * GENERIC -- any four-factor mask, canonical value layout.  One thread per
//    output element walks the row's kept values through the four adjacency
//    lists.  Plain FMA; the always-available fallback.
//
//  * MFMA -- RBGP4 masks (G_r, G_b complete).  One workgroup owns the rows of
//    one tile row u_o (or a slice of its G_i groups) and TN columns of O and
//    walks the d_o nonzero tiles of that tile row (zero tiles are never
//    visited -- the role of G_o in Section 5).  Each tile is consumed in
//    |G_r.V| stages; a stage brings the |G_i.V|*|G_b.V| rows of I that the
//    stage can touch into LDS with 16-byte-per-lane direct global->LDS loads
//    (double buffered, one barrier per stage).  One wavefront owns one G_i
//    vertex u_i, i.e. the |G_r.U|*|G_b.U| rows that share a column set (row
//    repetition, Section 5), and 64*T columns.  The dense block of those rows
//    against one row of I is an outer product: v_mfma_f32_4x4x1_16b_f32 with
//    A-broadcast (cbsz=4) multiplies 4 rows x 64 columns per instruction, the
//    weight vector for 16 consecutive contraction steps sitting in one VGPR and
//    `abid` selecting the step.  No structural zero is multiplied.
#include <hip/hip_runtime.h>

#include <algorithm>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "rbgp_internal.h"
#include "rbgp_reg_common.h"

#define RBGP_HIP(call)                                                              \
  do {                                                                              \
    hipError_t e_ = (call);                                                         \
    if (e_ != hipSuccess) {                                                         \
      char buf_[256];                                                               \
      std::snprintf(buf_, sizeof buf_, "%s: %s", #call, hipGetErrorString(e_));     \
      rbgp_set_hip_error(buf_);                                                     \
      return RBGP_EHIP;                                                             \
    }                                                                               \
  } while (0)

struct rbgp_device_state {
  int device = -1;
  int32_t *adj[4] = {nullptr, nullptr, nullptr, nullptr};
  int32_t *rowoff = nullptr;             // [a_i][KS]: stage-relative I row of each contraction step
  // pack permutation per kernel family and dtype; second half: composed with the order of the
  // original mask (transposed masks, values given in the original's canonical order)
  int32_t *perm[4 * RBGP_NUM_KERNELS] = {};
  size_t perm_elems[4 * RBGP_NUM_KERNELS] = {};
  void *reg_state = nullptr;             // tables of the register-streaming family
  void *tile_state = nullptr;            // tables of the tile family
  void *sddmm_state = nullptr;           // tables and partial sums of the weight-gradient kernels
  void *staging = nullptr;               // canonical values on their way through rbgp_pack
  size_t staging_bytes = 0;
  int tune[RBGP_NUM_TUNE] = {};            // RBGP_TUNE_* values, 0 = default
};

void rbgp_device_release(rbgp_device_state *dev) {
  if (!dev) return;
  for (int i = 0; i < 4; ++i)
    if (dev->adj[i]) (void)hipFree(dev->adj[i]);
  if (dev->rowoff) (void)hipFree(dev->rowoff);
  for (int32_t *t : dev->perm)
    if (t) (void)hipFree(t);
  rbgp_reg_release(dev->reg_state);
  rbgp_tile_release(dev->tile_state);
  rbgp_sddmm_release(dev->sddmm_state);
  if (dev->staging) (void)hipFree(dev->staging);
  delete dev;
}

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// compile-time loop: f(std::integral_constant<int, I>) for I in [0, N)
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// ----------------------------------------------------------------------------
// pack: out[p] = perm[p] >= 0 ? in[perm[p]] : 0
// ----------------------------------------------------------------------------
template <typename T>
__global__ void pack_kernel(const T *__restrict__ in, const int32_t *__restrict__ perm,
                            T *__restrict__ out, int64_t n) {
  int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (p >= n) return;
  int32_t s = perm[p];
  out[p] = s >= 0 ? in[s] : T(0);
}

// ----------------------------------------------------------------------------
// GENERIC kernel
// ----------------------------------------------------------------------------
struct GenericParams {
  const int32_t *adj[4];
  int a[4], c[4], d[4];
  int64_t M, N, ldI, ldO, rowdeg;
};

bool valid_dtype(rbgp_dtype_t d) { return d == RBGP_F32 || d == RBGP_BF16_F32ACC || d == RBGP_BF16; }
bool bf16_in(rbgp_dtype_t d) { return d != RBGP_F32; }

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(uint16_t x) { return __uint_as_float(uint32_t(x) << 16); }

__device__ inline void store_out(float *o, float x) { *o = x; }
__device__ inline void store_out(uint16_t *o, float x) { *o = uint16_t(rbgp_reg::bf16_bits(x)); }

template <typename TIn, typename TOut>
__global__ __launch_bounds__(256) void spmm_generic(GenericParams p, const TIn *__restrict__ W,
                                                    const TIn *__restrict__ I, TOut *__restrict__ O) {
  const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  for (int64_t m = blockIdx.y; m < p.M; m += gridDim.y) {
    int64_t r = m;
    const int u3 = int(r % p.a[3]); r /= p.a[3];
    const int u2 = int(r % p.a[2]); r /= p.a[2];
    const int u1 = int(r % p.a[1]); r /= p.a[1];
    const int u0 = int(r);
    const TIn *w = W + m * p.rowdeg;
    float acc = 0.f;
    int64_t t = 0;
    for (int j0 = 0; j0 < p.d[0]; ++j0) {
      const int64_t k0 = p.adj[0][u0 * p.d[0] + j0];
      for (int j1 = 0; j1 < p.d[1]; ++j1) {
        const int64_t k1 = k0 * p.c[1] + p.adj[1][u1 * p.d[1] + j1];
        for (int j2 = 0; j2 < p.d[2]; ++j2) {
          const int64_t k2 = k1 * p.c[2] + p.adj[2][u2 * p.d[2] + j2];
          for (int j3 = 0; j3 < p.d[3]; ++j3, ++t) {
            const int64_t k = k2 * p.c[3] + p.adj[3][u3 * p.d[3] + j3];
            if (n < p.N) acc = __builtin_fmaf(to_f32(w[t]), to_f32(I[k * p.ldI + n]), acc);
          }
        }
      }
    }
    if (n < p.N) store_out(O + m * p.ldO + n, acc);
  }
}

// ----------------------------------------------------------------------------
// MFMA kernel
// ----------------------------------------------------------------------------
struct MfmaParams {
  const void *Wp;
  const void *I;
  float *O;               // fp32, or bf16 bits when obf16 is set (ldO counts elements of that type)
  int obf16;              // bf16 kernels: round the sums to bf16 when storing O
  const int32_t *adj0;    // [a_o][d_o]
  const int32_t *rowoff;  // [a_i][KS]
  int64_t N, ldI, ldO;
  int a1, a2, a3, a4;     // |G_o.U|, |G_r.U|, |G_i.U|, |G_b.U|
  int d1, c2;             // d_l(G_o), |G_r.V|
  int SR;                 // I rows per stage = |G_i.V| * |G_b.V|
  int R;                  // a2 * a4
  int GW, GZ;             // G_i vertices per workgroup, workgroups per tile row (GW * GZ = a3)
  int ntiles;             // ceil(N / TN)
  int buf_bytes;          // bytes of one LDS stage buffer
};

template <bool BF16>
struct InT { typedef float type; };
template <>
struct InT<true> { typedef uint16_t type; };

// KS: contraction steps of one group per stage; RB: 4-row blocks per group;
// T: columns per lane; TN: columns per workgroup.
template <int KS, int RB, int T, int TN, bool BF16>
__global__ __launch_bounds__(512) void spmm_mfma(MfmaParams p) {
  typedef typename InT<BF16>::type in_t;
  constexpr int ES = int(sizeof(in_t));
  constexpr int NCH = (KS + 15) / 16;
  constexpr int RBYTES = TN * ES;       // bytes of one staged I row
  constexpr int CPR = RBYTES / 16;      // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;         // rows covered by one wave-wide direct load
  constexpr int EPC = 16 / ES;          // elements per chunk
  static_assert(CPR >= 1 && CPR <= 64 && RPI * CPR == 64, "tile width");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwaves = __builtin_amdgcn_readfirstlane(int(blockDim.x) >> 6);

  // Workgroups are dealt round-robin to the 8 XCDs: keep every workgroup that
  // reads the same columns of I on one XCD (one L2), tile rows varying fastest.
  const int bid = blockIdx.x, xcd = bid & 7, slot = bid >> 3;
  const int MT = p.a1 * p.GZ;
  const int nt = xcd + 8 * (slot / MT), mt = slot % MT;
  if (nt >= p.ntiles) return;
  const int u1 = mt / p.GZ, gz = mt % p.GZ;
  const int gslot = wid % p.GW, nsub = wid / p.GW;
  const int u3 = gz * p.GW + gslot;
  const int64_t n0 = int64_t(nt) * TN;

  const in_t *__restrict__ Ig = static_cast<const in_t *>(p.I);
  const in_t *__restrict__ Wg = static_cast<const in_t *>(p.Wp);

  // LDS byte offset (inside a stage buffer) of the operand each lane reads at step kk
  int boff[KS];
  {
    const int32_t *ro = p.rowoff + u3 * KS;
    const int colb = (nsub * 64 * T + lane * T) * ES;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) boff[kk] = ro[kk] * RBYTES + colb;
  }

  // direct global->LDS staging: lane -> (row within the wave's slab, 16-byte chunk)
  const int ld_row = lane / CPR, ld_chunk = lane % CPR;
  const bool ld_col_ok = n0 + int64_t(ld_chunk) * EPC < p.N;
  const int ninstr = (p.SR + RPI - 1) / RPI;
  const int nstages = p.d1 * p.c2;

  // adjacency row of u_o, one entry per lane (d_o <= 128), read back with readlane
  const int adj_lo = lane < p.d1 ? p.adj0[u1 * p.d1 + lane] : 0;
  const int adj_hi = lane + 64 < p.d1 ? p.adj0[u1 * p.d1 + lane + 64] : 0;

  auto stage_issue = [&](int s, int buf) {
    const int j1 = s / p.c2, v2 = s - j1 * p.c2;
    const int v1 = j1 < 64 ? __builtin_amdgcn_readlane(adj_lo, j1) : __builtin_amdgcn_readlane(adj_hi, j1 - 64);
    const int64_t k0 = (int64_t(v1) * p.c2 + v2) * p.SR;
    const in_t *src = Ig + (k0 + ld_row) * p.ldI + n0 + ld_chunk * EPC;
    unsigned char *dst = smem + buf * p.buf_bytes;
    for (int i = wid; i < ninstr; i += nwaves) {
      const int row = i * RPI + ld_row;
      if (row < p.SR && ld_col_ok)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void *)(src + int64_t(i) * RPI * p.ldI),
            (__attribute__((address_space(3))) void *)(dst + i * 1024), 16, 0, 0);
    }
  };
  auto a_load = [&](int s, in_t (&A)[RB][NCH]) {
    const in_t *wb = Wg + ((int64_t(u1) * nstages + s) * p.a3 + u3) * (RB * NCH * 64) + lane;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) A[rb][ch] = wb[(rb * NCH + ch) * 64];
  };

  f32x4 acc[RB][T];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int t = 0; t < T; ++t) acc[rb][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  in_t Anext[RB][NCH];
  stage_issue(0, 0);
  a_load(0, Anext);

  for (int s = 0; s < nstages; ++s) {
    float A[RB][NCH];
    __builtin_amdgcn_s_waitcnt(0);  // this wave's direct loads have landed in LDS
    __syncthreads();                // ... and everybody else's; previous buffer is free
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) A[rb][ch] = to_f32(Anext[rb][ch]);
    if (s + 1 < nstages) {
      stage_issue(s + 1, (s + 1) & 1);
      a_load(s + 1, Anext);
    }
    const unsigned char *buf = smem + (s & 1) * p.buf_bytes;
    static_for<0, KS>([&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      float B[T];
      if constexpr (!BF16) {
        if constexpr (T == 1) {
          B[0] = *reinterpret_cast<const float *>(buf + boff[kk]);
        } else if constexpr (T == 2) {
          f32x2 v = *reinterpret_cast<const f32x2 *>(buf + boff[kk]);
          B[0] = v[0]; B[1] = v[1];
        } else {
          f32x4 v = *reinterpret_cast<const f32x4 *>(buf + boff[kk]);
          B[0] = v[0]; B[1] = v[1]; B[2] = v[2]; B[3] = v[3];
        }
      } else {
        if constexpr (T == 1) {
          B[0] = to_f32(*reinterpret_cast<const uint16_t *>(buf + boff[kk]));
        } else if constexpr (T == 2) {
          uint32_t v = *reinterpret_cast<const uint32_t *>(buf + boff[kk]);
          B[0] = __uint_as_float(v << 16); B[1] = __uint_as_float(v & 0xffff0000u);
        } else {
          uint2 v = *reinterpret_cast<const uint2 *>(buf + boff[kk]);
          B[0] = __uint_as_float(v.x << 16); B[1] = __uint_as_float(v.x & 0xffff0000u);
          B[2] = __uint_as_float(v.y << 16); B[3] = __uint_as_float(v.y & 0xffff0000u);
        }
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int t = 0; t < T; ++t)
          acc[rb][t] = __builtin_amdgcn_mfma_f32_4x4x1f32(A[rb][kk / 16], B[t], acc[rb][t], 4, kk % 16, 0);
    });
  }

  // epilogue: lane holds columns n0 + nsub*64*T + lane*T + t of rows rb*4 + i of its group
  const int64_t nbase = n0 + nsub * 64 * T + lane * T;
  if constexpr (BF16) {
    if (p.obf16) {
      uint16_t *const Ob = reinterpret_cast<uint16_t *>(p.O);
      const bool pair_ok = (T == 2) && (p.ldO % 2 == 0) && (reinterpret_cast<uintptr_t>(p.O) % 4 == 0) && (nbase + 2 <= p.N);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = rb * 4 + i;
          if (r >= p.R) continue;
          const int u2 = r / p.a4, u4 = r - u2 * p.a4;
          const int64_t m = ((int64_t(u1) * p.a2 + u2) * p.a3 + u3) * p.a4 + u4;
          uint16_t *o = Ob + m * p.ldO + nbase;
          if (pair_ok) {
            *reinterpret_cast<uint32_t *>(o) = rbgp_reg::bf16_pair(acc[rb][0][i], acc[rb][T - 1][i]);
          } else {
#pragma unroll
            for (int t = 0; t < T; ++t)
              if (nbase + t < p.N) o[t] = uint16_t(rbgp_reg::bf16_bits(acc[rb][t][i]));
          }
        }
      return;
    }
  }
  const bool vec_ok = (T > 1) && ((p.ldO % T) == 0) && ((reinterpret_cast<uintptr_t>(p.O) % (4 * T)) == 0) &&
                      (nbase + T <= p.N);
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = rb * 4 + i;
      if (r >= p.R) continue;
      const int u2 = r / p.a4, u4 = r - u2 * p.a4;
      const int64_t m = ((int64_t(u1) * p.a2 + u2) * p.a3 + u3) * p.a4 + u4;
      float *o = p.O + m * p.ldO + nbase;
      if (vec_ok) {
        if constexpr (T == 2) {
          *reinterpret_cast<f32x2 *>(o) = f32x2{acc[rb][0][i], acc[rb][1][i]};
        } else if constexpr (T == 4) {
          *reinterpret_cast<f32x4 *>(o) = f32x4{acc[rb][0][i], acc[rb][1][i], acc[rb][2][i], acc[rb][3][i]};
        }
      } else {
#pragma unroll
        for (int t = 0; t < T; ++t)
          if (nbase + t < p.N) o[t] = acc[rb][t][i];
      }
    }
}

typedef void (*mfma_fn)(MfmaParams);
struct MfmaEntry {
  int KS, RB, T, TN, bf16;
  mfma_fn fn;
};

#define RBGP_E(KS, RB, T, TN) \
  {KS, RB, T, TN, 0, spmm_mfma<KS, RB, T, TN, false>}, {KS, RB, T, TN, 1, spmm_mfma<KS, RB, T, TN, true>}
#define RBGP_KS(KS) RBGP_E(KS, 1, 1, 64), RBGP_E(KS, 1, 2, 128), RBGP_E(KS, 2, 1, 64), RBGP_E(KS, 2, 2, 128)

const MfmaEntry kMfmaTable[] = {RBGP_KS(2),  RBGP_KS(4),  RBGP_KS(8),  RBGP_KS(16),
                                RBGP_KS(32), RBGP_KS(18), RBGP_KS(36), RBGP_KS(72)};

const MfmaEntry *find_mfma(int KS, int RB, int T, int TN, int bf16) {
  for (const MfmaEntry &e : kMfmaTable)
    if (e.KS == KS && e.RB == RB && e.T == T && e.TN == TN && e.bf16 == bf16) return &e;
  return nullptr;
}

bool mfma_covers(const rbgp_mask *m) {
  const rbgp_mfma_plan &p = m->plan;
  if (!p.ok || m->d[0] > 128) return false;
  return find_mfma(p.KS, p.RB, 1, 64, 0) != nullptr;
}

// AUTO: the register-streaming family where it covers the mask (measured faster than the
// LDS family on every VGG19 layer shape, also where several G_i vertices share a row of I),
// else the LDS family, else GENERIC.
// Estimated seconds per column of I: one of 1024 SIMDs at ~2.07 GHz serves 64 columns per instruction.  The
// constants are fitted to the 4096^3 products of Tables 2 and 3 (27 masks, each on every family that covers it).
// Register family: a wave walks the stages of its (cluster, G_i vertex) pair; a stage of KC steps costs KC 16-row
// MFMAs of ~36 cycles (fp32), or ~8 cycles per step in bf16 (the loads of the stage; its 32-step MFMAs hide behind
// them, a second MFMA block for the remainder of a stage does not), plus what does not overlap.
double reg_seconds(const rbgp_mask *m, bool bf16) {
  if (m->regroup && (!bf16 || m->regroup_bf16)) m = m->regroup;   // (the kernels run on the regrouped mask)
  const rbgp_reg_clusters &cl = m->reg_clusters;
  int64_t walked = 0;
  for (int c = 0; c < cl.ncl; ++c) walked += cl.counts[size_t(c)];
  const int KC = m->reg.KC;
  double stage = bf16 ? 150.0 + 6.8 * KC + (KC > 32 && rbgp_bf16_tail16(KC) ? 100.0 : 0.0) : 110.0 + 36.0 * KC;
  // tile rows with the very same tiles (rows of G_r in the tile-row index) share their loads of I: the bf16 kernels
  // take two or four of them per wave (measured on the filled masks of Table 3: 182 / 122 / 100-111 us)
  if (bf16 && m->reg.MG == 1 && m->reg.fold % 2 == 0)
    stage *= m->reg.fold % 4 == 0 && cl.max_stages >= 32 && KC <= 36 ? 0.56 : 0.67;
  // (fp32, the same with stages of up to 32 steps: two such tile rows per wave and two waves per SIMD keep the matrix
  // core busy throughout -- 500-520 us for the 2 x 34.4 GFLOP of Table 3's filled masks, 32.4 cycles per MFMA)
  if (!bf16 && m->reg.MG == 1 && m->reg.fold % 2 == 0 && KC <= 32) stage = 40.0 + 33.0 * KC;
  return double(walked) * m->a[2] * stage / (64.0 * 1024.0 * 2.07e9);
}
// LDS-staged family (fp32 MFMA for both dtypes): a wave walks (tile, column of G_r) steps of RB * KS 4-row MFMAs,
// ~11.5 cycles each (the LDS read that feeds it) + ~95 cycles per step.
double lds_seconds(const rbgp_mask *m) {
  const double steps = double(m->a[0]) * m->d[0] * m->c[1] * m->a[2];
  return steps * (11.5 * m->plan.RB * m->plan.KS + 95.0) / (64.0 * 1024.0 * 2.07e9);
}
double hbm_seconds(const rbgp_mask *m) { return double(m->M + m->K) * 4.0 / 5.0e12; }

int resolve_kernel_unfilled(const rbgp_mask *m, rbgp_dtype_t dtype);

// AUTO, last step: the register family on the mask with G_i filled in where that is estimated faster than the
// family chosen for the mask itself and the product is not waiting for HBM anyway.  Measured on the 4096^3
// products of Table 3, fp32 (us): one row per column set 1538 / 848 / 833 on the register family and 2054 / 1383 /
// 1178 on the LDS family -> 622 / 595 / 580 at densities 1/4, 1/8, 1/16; two rows 824 -> 617 at 1/4 (466 and 453 at
// 1/8 and 1/16 stay on the register family); four rows stay (586 against 621).  bf16: also Table 2's cells with a
// half-full G_i (G_o at 1/8: 129 -> 51 us).  Since the two-group kernel of the filled masks runs two waves per SIMD
// (500-520 us on the one-row masks) the half-full G_i cells of fp32 take it too: 517 against 542 us on the LDS
// family with G_o at 1/2, 266 / 281 at 1/4, 142 / 150 at 1/8.
int resolve_kernel(const rbgp_mask *m, rbgp_dtype_t dtype) {
  if (m->kernel_choice == RBGP_KERNEL_MFMA_REG_FILLED) return m->filled ? RBGP_KERNEL_MFMA_REG_FILLED : RBGP_KERNEL_GENERIC;
  const int k0 = resolve_kernel_unfilled(m, dtype);
  if (m->kernel_choice != RBGP_KERNEL_AUTO || !m->filled) return k0;
  if (m->c[3] == 9 && m->d[3] == 9) return k0;   // (the mask of a lowered 3x3 convolution: rbgp_conv3x3 needs its own layout)
  if (k0 == RBGP_KERNEL_GENERIC) return RBGP_KERNEL_MFMA_REG_FILLED;
  const bool bf16 = bf16_in(dtype);
  const double t0 = k0 == RBGP_KERNEL_MFMA ? lds_seconds(m) : reg_seconds(m, bf16);
  return t0 > 2.0 * hbm_seconds(m) && reg_seconds(m->filled, bf16) < t0 ? RBGP_KERNEL_MFMA_REG_FILLED : k0;
}

int resolve_kernel_unfilled(const rbgp_mask *m, rbgp_dtype_t dtype) {
  const bool reg_ok = rbgp_reg_covers(m);
  // (the tile family has bf16 kernels only: fp32 calls on such a mask take the default choice)
  if (m->kernel_choice == RBGP_KERNEL_MFMA_TILE && bf16_in(dtype) && rbgp_plan_tile(m).ok) return RBGP_KERNEL_MFMA_TILE;
  switch (m->kernel_choice) {
    case RBGP_KERNEL_GENERIC: return RBGP_KERNEL_GENERIC;
    case RBGP_KERNEL_MFMA: return mfma_covers(m) ? RBGP_KERNEL_MFMA : RBGP_KERNEL_GENERIC;
    case RBGP_KERNEL_MFMA_REG: return reg_ok ? RBGP_KERNEL_MFMA_REG : RBGP_KERNEL_GENERIC;
    default: break;
  }
  const bool lds_ok = mfma_covers(m);
  if (reg_ok && lds_ok) {
    // The register family multiplies whole clusters of MG tile rows at every tile of their union:
    // where G_o is so sparse that the tile rows of a cluster share few tiles, most of those MFMA
    // rows are padding.  That costs nothing while the product waits for HBM (WRN-40-4 group 1:
    // 25 % useful rows, still the faster family) and decides where the matrix core is the bound
    // (the 4096^3 SDMM of Table 2 with G_o at 1/8: 29 % useful rows, 305 us against 177 us on the
    // LDS family, which has no clusters; with G_o complete 454 against 751).  So: the register
    // family unless its estimated time is both well above the HBM time of the product (HBM streams
    // ~5 TB/s) and above the LDS family's.
    // (VGG19 layers at density 1/16 with 27-42 % useful rows and an estimate up to 1.3 x the HBM time are
    // still faster on the register family, as is every other cell of that sweep.)
    // The mask of a lowered 3x3 convolution stays on the register family: rbgp_conv3x3 and the fused gradients read
    // its layout (and it was the faster family on every VGG19 cell, forward and transposed).
    if (m->c[3] == 9 && m->d[3] == 9) return RBGP_KERNEL_MFMA_REG;
    const double t_reg = reg_seconds(m, bf16_in(dtype));
    return t_reg > 4.0 * hbm_seconds(m) && lds_seconds(m) < t_reg ? RBGP_KERNEL_MFMA : RBGP_KERNEL_MFMA_REG;
  }
  if (reg_ok) return RBGP_KERNEL_MFMA_REG;
  return lds_ok ? RBGP_KERNEL_MFMA : RBGP_KERNEL_GENERIC;
}

int64_t packed_elems(const rbgp_mask *m, int kernel, rbgp_dtype_t dtype) {
  if (kernel == RBGP_KERNEL_MFMA) return m->plan.packed_elems;
  if (kernel == RBGP_KERNEL_MFMA_TILE) return rbgp_plan_tile(m).packed_elems;
  if (kernel == RBGP_KERNEL_MFMA_REG) {
    if (bf16_in(dtype)) return m->regroup && m->regroup_bf16 ? m->regroup->reg.packed_elems_bf16 : m->reg.packed_elems_bf16;
    return m->regroup ? m->regroup->reg.packed_elems : m->reg.packed_elems;
  }
  if (kernel == RBGP_KERNEL_MFMA_REG_FILLED)
    return bf16_in(dtype) ? m->filled->reg.packed_elems_bf16 : m->filled->reg.packed_elems;
  return m->nnz;
}

template <typename T>
int upload(const std::vector<T> &h, T **d) {
  RBGP_HIP(hipMalloc(reinterpret_cast<void **>(d), h.size() * sizeof(T) + 16));
  RBGP_HIP(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
  return RBGP_OK;
}

// Create the device tables of a mask on the current device (first GPU use).
int ensure_device(const rbgp_mask *m) {
  if (m->dev && m->dev->adj[0]) return RBGP_OK;
  if (!m->dev) {
    m->dev = new (std::nothrow) rbgp_device_state();
    if (!m->dev) return RBGP_ENOMEM;
  }
  rbgp_device_state *dev = m->dev;
  RBGP_HIP(hipGetDevice(&dev->device));
  // the state is touched only when every table is on the device (adj[0] marks "built")
  int32_t *adj[4] = {nullptr, nullptr, nullptr, nullptr}, *rowoff = nullptr;
  int rc = RBGP_OK;
  for (int i = 0; i < 4 && !rc; ++i) rc = upload(m->adj[i], &adj[i]);
  if (!rc && m->plan.ok) {
    const rbgp_mfma_plan &p = m->plan;
    std::vector<int32_t> ro(size_t(m->a[2]) * p.KS);
    for (int u3 = 0; u3 < m->a[2]; ++u3)
      for (int kk = 0; kk < p.KS; ++kk)
        ro[size_t(u3) * p.KS + kk] = m->adj[2][size_t(u3) * m->d[2] + kk / m->c[3]] * m->c[3] + kk % m->c[3];
    rc = upload(ro, &rowoff);
  }
  if (rc) {
    for (int32_t *t : adj)
      if (t) (void)hipFree(t);
    if (rowoff) (void)hipFree(rowoff);
    return rc;
  }
  dev->rowoff = rowoff;
  for (int i = 3; i >= 0; --i) dev->adj[i] = adj[i];
  return RBGP_OK;
}

int ensure_perm(const rbgp_mask *m, int kernel, bool bf16, bool original_order, int *slot) {
  rbgp_device_state *dev = m->dev;
  *slot = 2 * kernel + (bf16 ? 1 : 0) + (original_order ? 2 * RBGP_NUM_KERNELS : 0);
  if (dev->perm[*slot]) return RBGP_OK;
  std::vector<int32_t> perm;
  rbgp_build_pack_perm(m, kernel, bf16, perm);
  if (original_order)
    for (int32_t &s : perm)
      if (s >= 0) s = m->from_original[size_t(s)];
  dev->perm_elems[*slot] = perm.size();
  return upload(perm, &dev->perm[*slot]);
}

size_t elem_bytes(rbgp_dtype_t dt) { return bf16_in(dt) ? 2 : 4; }

}  // namespace

extern "C" {

int rbgp_mask_set_kernel(rbgp_mask_t *m, int kernel) {
  if (!m) return RBGP_EINVAL;
  if (kernel < RBGP_KERNEL_AUTO || kernel >= RBGP_NUM_KERNELS) return RBGP_EINVAL;
  if (kernel == RBGP_KERNEL_MFMA && !mfma_covers(m)) return RBGP_EUNSUPPORTED;
  if (kernel == RBGP_KERNEL_MFMA_REG && !rbgp_reg_covers(m)) return RBGP_EUNSUPPORTED;
  if (kernel == RBGP_KERNEL_MFMA_TILE && !rbgp_plan_tile(m).ok) return RBGP_EUNSUPPORTED;
  if (kernel == RBGP_KERNEL_MFMA_REG_FILLED && !m->filled) return RBGP_EUNSUPPORTED;
  m->kernel_choice = kernel;
  return RBGP_OK;
}

int rbgp_mask_kernel(const rbgp_mask_t *m, rbgp_dtype_t dtype) {
  if (!m || !valid_dtype(dtype)) return RBGP_EINVAL;
  return resolve_kernel(m, dtype);
}

int rbgp_mask_tune(rbgp_mask_t *m, int knob, int value) {
  if (!m || knob < 0 || knob >= RBGP_NUM_TUNE || value < 0) return RBGP_EINVAL;
  if (!m->dev) {
    m->dev = new (std::nothrow) rbgp_device_state();
    if (!m->dev) return RBGP_ENOMEM;
  }
  m->dev->tune[knob] = value;
  return RBGP_OK;
}

size_t rbgp_packed_bytes(const rbgp_mask_t *m, rbgp_dtype_t dtype) {
  if (!m || !valid_dtype(dtype)) return 0;
  return size_t(packed_elems(m, resolve_kernel(m, dtype), dtype)) * elem_bytes(dtype);
}

static int pack_layout_impl(const rbgp_mask_t *m, rbgp_dtype_t dtype, int32_t *out) {
  if (!m || !out || !valid_dtype(dtype)) return RBGP_EINVAL;
  std::vector<int32_t> perm;
  rbgp_build_pack_perm(m, resolve_kernel(m, dtype), bf16_in(dtype), perm);
  std::copy(perm.begin(), perm.end(), out);
  return RBGP_OK;
}

int rbgp_pack_layout(const rbgp_mask_t *m, rbgp_dtype_t dtype, int32_t *out) {
  RBGP_GUARDED(pack_layout_impl(m, dtype, out));
}

static int pack_device(const rbgp_mask_t *m, rbgp_dtype_t dtype, bool original_order, const void *dev_values,
                       void *dev_packed, void *hip_stream) {
  if (!m || !dev_values || !dev_packed) return RBGP_EINVAL;
  if (!valid_dtype(dtype)) return RBGP_EINVAL;
  if (original_order && m->from_original.empty()) return RBGP_EINVAL;
  int rc = ensure_device(m);
  if (rc) return rc;
  const int kernel = resolve_kernel(m, dtype);
  int slot;
  rc = ensure_perm(m, kernel, bf16_in(dtype), original_order, &slot);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t n = int64_t(m->dev->perm_elems[slot]);
  const dim3 grid(unsigned((n + 255) / 256)), block(256);
  if (dtype == RBGP_F32)
    pack_kernel<float><<<grid, block, 0, st>>>(static_cast<const float *>(dev_values), m->dev->perm[slot],
                                               static_cast<float *>(dev_packed), n);
  else
    pack_kernel<uint16_t><<<grid, block, 0, st>>>(static_cast<const uint16_t *>(dev_values),
                                                  m->dev->perm[slot], static_cast<uint16_t *>(dev_packed), n);
  RBGP_HIP(hipGetLastError());
  return RBGP_OK;
}

static int pack_device_impl(const rbgp_mask_t *m, rbgp_dtype_t dtype, const void *dev_values, void *dev_packed,
                     void *hip_stream) {
  return pack_device(m, dtype, false, dev_values, dev_packed, hip_stream);
}

int rbgp_pack_device(const rbgp_mask_t *m, rbgp_dtype_t dtype, const void *dev_values, void *dev_packed,
                     void *hip_stream) {
  RBGP_GUARDED(pack_device_impl(m, dtype, dev_values, dev_packed, hip_stream));
}

static int pack_transposed_device_impl(const rbgp_mask_t *mask_t, rbgp_dtype_t dtype, const void *dev_values,
                                void *dev_packed, void *hip_stream) {
  return pack_device(mask_t, dtype, true, dev_values, dev_packed, hip_stream);
}

int rbgp_pack_transposed_device(const rbgp_mask_t *mask_t, rbgp_dtype_t dtype, const void *dev_values,
                                void *dev_packed, void *hip_stream) {
  RBGP_GUARDED(pack_transposed_device_impl(mask_t, dtype, dev_values, dev_packed, hip_stream));
}

static int pack_host(const rbgp_mask_t *m, rbgp_dtype_t dtype, bool original_order, const void *host_values,
                     void *dev_packed, void *hip_stream) {
  if (!m || !host_values || !dev_packed) return RBGP_EINVAL;
  if (!valid_dtype(dtype)) return RBGP_EINVAL;
  if (original_order && m->from_original.empty()) return RBGP_EINVAL;
  int rc = ensure_device(m);
  if (rc) return rc;
  rbgp_device_state *dev = m->dev;
  const size_t bytes = size_t(m->nnz) * elem_bytes(dtype);
  if (dev->staging_bytes < bytes) {
    if (dev->staging) RBGP_HIP(hipFree(dev->staging));
    dev->staging = nullptr;
    dev->staging_bytes = 0;
    RBGP_HIP(hipMalloc(&dev->staging, bytes));
    dev->staging_bytes = bytes;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  RBGP_HIP(hipMemcpyAsync(dev->staging, host_values, bytes, hipMemcpyHostToDevice, st));
  rc = pack_device(m, dtype, original_order, dev->staging, dev_packed, hip_stream);
  if (rc) return rc;
  RBGP_HIP(hipStreamSynchronize(st));
  return RBGP_OK;
}

static int pack_impl(const rbgp_mask_t *m, rbgp_dtype_t dtype, const void *host_values, void *dev_packed,
              void *hip_stream) {
  return pack_host(m, dtype, false, host_values, dev_packed, hip_stream);
}

int rbgp_pack(const rbgp_mask_t *m, rbgp_dtype_t dtype, const void *host_values, void *dev_packed,
              void *hip_stream) {
  RBGP_GUARDED(pack_impl(m, dtype, host_values, dev_packed, hip_stream));
}

static int pack_transposed_impl(const rbgp_mask_t *mask_t, rbgp_dtype_t dtype, const void *host_values, void *dev_packed,
                         void *hip_stream) {
  return pack_host(mask_t, dtype, true, host_values, dev_packed, hip_stream);
}

int rbgp_pack_transposed(const rbgp_mask_t *mask_t, rbgp_dtype_t dtype, const void *host_values, void *dev_packed,
                         void *hip_stream) {
  RBGP_GUARDED(pack_transposed_impl(mask_t, dtype, host_values, dev_packed, hip_stream));
}

static int sddmm_impl(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N, const void *dev_dO,
               int64_t ld_dO, const void *dev_I, int64_t ldI, float *dev_dW, void *hip_stream) {
  if (!m) return RBGP_EINVAL;
  if (!valid_dtype(dtype)) return RBGP_EINVAL;
  if (M != m->M || K != m->K || N < 0 || ld_dO < N || ldI < N) return RBGP_ESHAPE;
  if (!dev_dW || (N > 0 && (!dev_dO || !dev_I))) return RBGP_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dev_dO) | reinterpret_cast<uintptr_t>(dev_I) | reinterpret_cast<uintptr_t>(dev_dW)) & 3)
    return RBGP_ESHAPE;
  int rc = ensure_device(m);
  if (rc) return rc;
  rbgp_device_state *dev = m->dev;
  const bool bf16 = bf16_in(dtype);
  // the MFMA kernel loads 16 bytes at dword-aligned addresses: bf16 rows must start on a dword
  const bool aligned = !bf16 || (ld_dO % 2 == 0 && ldI % 2 == 0);
  const bool use_mfma = m->kernel_choice != RBGP_KERNEL_GENERIC && rbgp_reg_covers(m) && aligned;
  return rbgp_sddmm_launch(m, &dev->sddmm_state, dev->adj, use_mfma, bf16, N, dev_dO, ld_dO, dev_I, ldI, dev_dW,
                           hip_stream);
}

int rbgp_sddmm(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N, const void *dev_dO,
               int64_t ld_dO, const void *dev_I, int64_t ldI, float *dev_dW, void *hip_stream) {
  RBGP_GUARDED(sddmm_impl(m, dtype, M, K, N, dev_dO, ld_dO, dev_I, ldI, dev_dW, hip_stream));
}

static int sddmm_static_impl(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N, const void *dev_dO,
                      int64_t ld_dO, const void *dev_I, int64_t ldI, float *dev_dW, void *hip_stream) {
  if (!m) return RBGP_EINVAL;
  if (!valid_dtype(dtype)) return RBGP_EINVAL;
  if (M != m->M || K != m->K || N < 0 || ld_dO < N || ldI < N) return RBGP_ESHAPE;
  if (!dev_dW || (N > 0 && (!dev_dO || !dev_I))) return RBGP_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dev_dO) | reinterpret_cast<uintptr_t>(dev_I) | reinterpret_cast<uintptr_t>(dev_dW)) & 3)
    return RBGP_ESHAPE;
  const bool bf16 = bf16_in(dtype);
  const bool aligned = !bf16 || (ld_dO % 2 == 0 && ldI % 2 == 0);
  const bool use_mfma = m->kernel_choice != RBGP_KERNEL_GENERIC && rbgp_reg_covers(m) && aligned;
  return rbgp_sddmm_static_launch(m, use_mfma, bf16, N, dev_dO, ld_dO, dev_I, ldI, dev_dW, hip_stream);
}

int rbgp_sddmm_static(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N, const void *dev_dO,
                      int64_t ld_dO, const void *dev_I, int64_t ldI, float *dev_dW, void *hip_stream) {
  RBGP_GUARDED(sddmm_static_impl(m, dtype, M, K, N, dev_dO, ld_dO, dev_I, ldI, dev_dW, hip_stream));
}

static int spmm_impl(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N, const void *dev_packed,
              const void *dev_I, int64_t ldI, void *dev_O, int64_t ldO, void *hip_stream) {
  if (!m) return RBGP_EINVAL;
  if (!valid_dtype(dtype)) return RBGP_EINVAL;
  if (M != m->M || K != m->K || N < 0 || ldI < N || ldO < N) return RBGP_ESHAPE;
  if (N == 0) return RBGP_OK;
  if (!dev_packed || !dev_I || !dev_O) return RBGP_EINVAL;
  int rc = ensure_device(m);
  if (rc) return rc;
  rbgp_device_state *dev = m->dev;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int kernel = resolve_kernel(m, dtype);
  const bool bf16 = bf16_in(dtype), out_bf16 = dtype == RBGP_BF16;
  if (out_bf16 && (reinterpret_cast<uintptr_t>(dev_O) & 1)) return RBGP_ESHAPE;

  // fp32: the same mask factored for fuller MFMA groups (its own tables, this mask's knobs).  Not bf16: there the
  // matrix core has room, the load path does not, and the regrouped mask has fewer tile rows that share their loads
  // (VGG19 backward data products: fp32 17-36 % faster, bf16 5-25 % slower).
  if (kernel == RBGP_KERNEL_MFMA_REG && m->regroup && (!bf16 || m->regroup_bf16)) {
    rc = ensure_device(m->regroup);
    if (rc) return rc;
    return rbgp_reg_launch(m->regroup, &m->regroup->dev->reg_state, dev->tune, bf16, out_bf16, N, dev_packed, dev_I,
                           ldI, dev_O, ldO, hip_stream);
  }
  if (kernel == RBGP_KERNEL_MFMA_REG)
    return rbgp_reg_launch(m, &dev->reg_state, dev->tune, bf16, out_bf16, N, dev_packed, dev_I, ldI, dev_O, ldO,
                           hip_stream);

  if (kernel == RBGP_KERNEL_MFMA_REG_FILLED) {   // the same kernels on the filled mask (its own tables, this mask's knobs)
    rc = ensure_device(m->filled);
    if (rc) return rc;
    return rbgp_reg_launch(m->filled, &m->filled->dev->reg_state, dev->tune, bf16, out_bf16, N, dev_packed, dev_I, ldI,
                           dev_O, ldO, hip_stream);
  }

  if (kernel == RBGP_KERNEL_MFMA_TILE)
    return rbgp_tile_launch(m, &dev->tile_state, out_bf16, N, dev_packed, dev_I, ldI, dev_O, ldO, hip_stream);

  if (kernel == RBGP_KERNEL_GENERIC) {
    GenericParams gp;
    for (int i = 0; i < 4; ++i) {
      gp.adj[i] = dev->adj[i];
      gp.a[i] = m->a[i];
      gp.c[i] = m->c[i];
      gp.d[i] = m->d[i];
    }
    gp.M = M; gp.N = N; gp.ldI = ldI; gp.ldO = ldO; gp.rowdeg = m->rowdeg;
    const dim3 grid(unsigned((N + 255) / 256), unsigned(M < 32768 ? M : 32768)), block(256);
    if (out_bf16)
      spmm_generic<uint16_t, uint16_t><<<grid, block, 0, st>>>(gp, static_cast<const uint16_t *>(dev_packed),
                                                               static_cast<const uint16_t *>(dev_I),
                                                               static_cast<uint16_t *>(dev_O));
    else if (bf16)
      spmm_generic<uint16_t, float><<<grid, block, 0, st>>>(gp, static_cast<const uint16_t *>(dev_packed),
                                                            static_cast<const uint16_t *>(dev_I),
                                                            static_cast<float *>(dev_O));
    else
      spmm_generic<float, float><<<grid, block, 0, st>>>(gp, static_cast<const float *>(dev_packed),
                                                         static_cast<const float *>(dev_I),
                                                         static_cast<float *>(dev_O));
    RBGP_HIP(hipGetLastError());
    return RBGP_OK;
  }

  // MFMA family
  const rbgp_mfma_plan &pl = m->plan;
  const int epc = bf16 ? 8 : 4;
  if ((reinterpret_cast<uintptr_t>(dev_I) & 15) || (ldI % epc)) return RBGP_ESHAPE;
  // tile shape: T columns per lane, TN per workgroup, GW groups (waves) per workgroup
  const int tune_t = dev->tune[RBGP_TUNE_COLS_PER_LANE], tune_tn = dev->tune[RBGP_TUNE_COLS_PER_WORKGROUP];
  int T = tune_t ? tune_t : 2;
  int TN = tune_tn ? tune_tn : 64 * T;
  if (!tune_t && !tune_tn) {
    // enough workgroups to fill 256 CUs, else narrower tiles
    const int64_t wg128 = ((N + 127) / 128) * m->a[0];
    if (wg128 < 512) { T = 1; TN = 64; }
  }
  const MfmaEntry *e = find_mfma(pl.KS, pl.RB, T, TN, bf16 ? 1 : 0);
  if (!e) return RBGP_EUNSUPPORTED;
  const int nsub = TN / (64 * T);
  int GW = dev->tune[RBGP_TUNE_GROUPS_PER_WORKGROUP] ? dev->tune[RBGP_TUNE_GROUPS_PER_WORKGROUP] : m->a[2];
  if (GW < 1) GW = 1;
  while (GW > 1 && (GW * nsub > 8 || m->a[2] % GW)) --GW;  // at most 8 waves per workgroup, GW | a_i
  if (GW * nsub > 8) return RBGP_EUNSUPPORTED;

  MfmaParams mp;
  mp.Wp = dev_packed; mp.I = dev_I; mp.O = static_cast<float *>(dev_O);
  mp.obf16 = out_bf16 ? 1 : 0;
  mp.adj0 = dev->adj[0]; mp.rowoff = dev->rowoff;
  mp.N = N; mp.ldI = ldI; mp.ldO = ldO;
  mp.a1 = m->a[0]; mp.a2 = m->a[1]; mp.a3 = m->a[2]; mp.a4 = m->a[3];
  mp.d1 = m->d[0]; mp.c2 = m->c[1];
  mp.SR = pl.SR; mp.R = pl.R;
  mp.GW = GW; mp.GZ = m->a[2] / GW;
  mp.ntiles = int((N + TN - 1) / TN);
  const int rbytes = TN * (bf16 ? 2 : 4);
  const int rpi = 1024 / rbytes;
  mp.buf_bytes = ((pl.SR + rpi - 1) / rpi) * 1024;
  const size_t lds = size_t(2) * mp.buf_bytes;
  if (lds > 160 * 1024) return RBGP_EUNSUPPORTED;
  RBGP_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(e->fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                               int(lds)));
  const int64_t MT = int64_t(mp.a1) * mp.GZ;
  const int64_t nblocks = 8 * ((mp.ntiles + 7) / 8) * MT;
  if (nblocks > 0x7fffffff) return RBGP_EUNSUPPORTED;
  hipLaunchKernelGGL(e->fn, dim3(unsigned(nblocks)), dim3(unsigned(GW * nsub * 64)), lds, st, mp);
  RBGP_HIP(hipGetLastError());
  return RBGP_OK;
}

int rbgp_spmm(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N, const void *dev_packed,
              const void *dev_I, int64_t ldI, void *dev_O, int64_t ldO, void *hip_stream) {
  RBGP_GUARDED(spmm_impl(m, dtype, M, K, N, dev_packed, dev_I, ldI, dev_O, ldO, hip_stream));
}

static int conv3x3_impl(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t channels_out, int64_t channels_in, int64_t images,
                 int64_t height, int64_t width, const void *dev_packed, const void *dev_X, void *dev_O, int64_t ldO,
                 void *hip_stream) {
  if (!m) return RBGP_EINVAL;
  if (!valid_dtype(dtype)) return RBGP_EINVAL;
  if (images <= 0 || height <= 0 || width <= 0 || (width % 4)) return RBGP_ESHAPE;
  const int64_t N = images * height * width;
  if (channels_out != m->M || 9 * channels_in != m->K || ldO < N) return RBGP_ESHAPE;
  const int kernel = resolve_kernel(m, dtype);
  if (kernel != RBGP_KERNEL_MFMA_REG && kernel != RBGP_KERNEL_MFMA_TILE) return RBGP_EUNSUPPORTED;
  if (!dev_packed || !dev_X || !dev_O) return RBGP_EINVAL;
  if (dtype == RBGP_BF16 && (reinterpret_cast<uintptr_t>(dev_O) & 1)) return RBGP_ESHAPE;
  int rc = ensure_device(m);
  if (rc) return rc;
  const rbgp_conv_geometry geom = {images, height, width};
  if (kernel == RBGP_KERNEL_MFMA_TILE)
    return rbgp_tile_launch(m, &m->dev->tile_state, dtype == RBGP_BF16, N, dev_packed, dev_X, N, dev_O, ldO, hip_stream,
                            &geom);
  return rbgp_reg_launch(m, &m->dev->reg_state, m->dev->tune, bf16_in(dtype), dtype == RBGP_BF16, N, dev_packed, dev_X,
                         N, dev_O, ldO, hip_stream, &geom);
}

int rbgp_conv3x3(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t channels_out, int64_t channels_in, int64_t images,
                 int64_t height, int64_t width, const void *dev_packed, const void *dev_X, void *dev_O, int64_t ldO,
                 void *hip_stream) {
  RBGP_GUARDED(conv3x3_impl(m, dtype, channels_out, channels_in, images, height, width, dev_packed, dev_X, dev_O, ldO, hip_stream));
}

static int conv3x3_sddmm_impl(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t channels_out, int64_t channels_in,
                       int64_t images, int64_t height, int64_t width, const void *dev_dO, int64_t ld_dO,
                       const void *dev_X, float *dev_dW, void *hip_stream) {
  if (!m) return RBGP_EINVAL;
  if (!valid_dtype(dtype)) return RBGP_EINVAL;
  const bool bf16 = bf16_in(dtype);
  if (images <= 0 || height <= 0 || width <= 0 || (width % (bf16 ? 8 : 4))) return RBGP_ESHAPE;
  const int64_t N = images * height * width;
  if (channels_out != m->M || 9 * channels_in != m->K || ld_dO < N) return RBGP_ESHAPE;
  if (m->c[3] != 9 || m->d[3] != 9 || m->kernel_choice == RBGP_KERNEL_GENERIC || !rbgp_reg_covers(m))
    return RBGP_EUNSUPPORTED;
  if (!dev_dO || !dev_X || !dev_dW) return RBGP_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dev_dO) | reinterpret_cast<uintptr_t>(dev_X) | reinterpret_cast<uintptr_t>(dev_dW)) & 3)
    return RBGP_ESHAPE;
  if (bf16 && ld_dO % 2) return RBGP_ESHAPE;
  int rc = ensure_device(m);
  if (rc) return rc;
  const rbgp_conv_geometry geom = {images, height, width};
  return rbgp_sddmm_launch(m, &m->dev->sddmm_state, m->dev->adj, true, bf16, N, dev_dO, ld_dO, dev_X, N, dev_dW,
                           hip_stream, &geom);
}

int rbgp_conv3x3_sddmm(const rbgp_mask_t *m, rbgp_dtype_t dtype, int64_t channels_out, int64_t channels_in,
                       int64_t images, int64_t height, int64_t width, const void *dev_dO, int64_t ld_dO,
                       const void *dev_X, float *dev_dW, void *hip_stream) {
  RBGP_GUARDED(conv3x3_sddmm_impl(m, dtype, channels_out, channels_in, images, height, width, dev_dO, ld_dO, dev_X, dev_dW, hip_stream));
}

}  // extern "C"
