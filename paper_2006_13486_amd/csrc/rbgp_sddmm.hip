// Gradient of the kept values of W_s for a fixed mask (Section 6: masks are predefined and stay
// fixed during training):  dW[m][t] = sum_n dO[m][n] * I[k][n]  for the t-th kept column k of
// row m -- the dense product dO x I^T sampled on the mask.
//
// MFMA kernel (RBGP4 masks covered by the register-streaming family).  The work unit is what the
// forward kernel calls a stage, seen from the other side: for one cluster of tile rows, one
// nonzero tile of G_o, VC columns of G_r and one G_i vertex u_i, the kept values form a dense
// block of (16 weight rows = the cluster's MG tile rows x RS rows) x (KCR contraction steps), and
// that block is the product of 16 rows of dO with KCR rows of I, contracted over the batch
// columns n.  One wave owns a unit and a range of columns: a lane loads 16 bytes of "its" row
// (row lane % 16 of the 16 dO rows, and of each block of 16 I rows) at column offset
// 4 (8 for bf16) * (lane / 16), which is exactly the operand layout of v_mfma_f32_16x16x4_f32
// (four of them per load, one per loaded column) / v_mfma_f32_16x16x32_bf16 (one per load);
// the accumulators hold the 16 x 16 blocks of dW.  Rows of the unit that do not exist (a member
// without the tile, R < RS, KCR not a multiple of 16) load some valid row instead and their
// results are dropped: an output element depends on its own two rows only.
// The batch is cut into `nsplit` ranges so that the chip is filled; each range writes its own
// partial dW and a second kernel adds the partials in a fixed order (reproducible sums).
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
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef f32x4 f32x4_u __attribute__((aligned(4)));
typedef bf16x8 bf16x8_u __attribute__((aligned(4)));

struct SddmmParams {
  const void *dO, *I;
  float *out;               // [nsplit][nnz] partial sums (dW itself when nsplit == 1)
  const int32_t *units;     // [nunits] cluster * 64 + stage of the cluster's stage list
  const int32_t *stages;    // [ncl][1 + MG][64], as for the forward kernels
  const int32_t *members;   // [ncl][MG]
  const int32_t *rowtab;    // [a_i][16 * NB]: stage-relative row of I of contraction step kk (padding -> 0)
  int64_t N, ld_dO, ldI, nnz;
  int64_t chunk;            // columns per range (a multiple of the columns per iteration)
  int a2, a3, a4, R, lgRS, MG, KCR, rowdeg;
};

template <bool BF16>
struct Operand;
template <>
struct Operand<false> {
  typedef f32x4 reg;
  static constexpr int CPL = 4;   // columns per lane and load
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
  static __device__ __forceinline__ void mac(const reg &a, const reg &b, f32x4 &acc) {
#pragma unroll
    for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t], acc, 0, 0, 0);
  }
};
template <>
struct Operand<true> {
  typedef bf16x8 reg;
  static constexpr int CPL = 8;
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
  static __device__ __forceinline__ void mac(const reg &a, const reg &b, f32x4 &acc) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
  }
};

// NB: blocks of 16 contraction steps per stage (KCR <= 16 * NB)
template <int NB, bool BF16>
__global__ __launch_bounds__(64) void sddmm_reg(SddmmParams p) {
  typedef Operand<BF16> Op;
  typedef typename Op::reg reg;
  constexpr int CPL = Op::CPL, CPI = 4 * CPL;   // columns per lane load / per iteration
  const int lane = threadIdx.x, j = lane & 15, q = lane >> 4;
  const int unit = blockIdx.x / p.a3, u3 = blockIdx.x % p.a3;
  const int code = p.units[unit];
  const int cl = code >> 6, s = code & 63;
  const int RS = 1 << p.lgRS;
  const int32_t *stg = p.stages + int64_t(cl) * (1 + p.MG) * 64 + s;
  const int base = stg[0];

  // this lane's row of dO (row j of the 16): member j / RS, row j % RS of its R rows
  int64_t arow = 0;
  {
    const int mm = j >> p.lgRS, ri = j & (RS - 1);
    const int mem = p.members[cl * p.MG + mm];
    if (mem >= 0 && stg[(1 + mm) * 64] >= 0 && ri < p.R)
      arow = ((int64_t(mem) * p.a2 + ri / p.a4) * p.a3 + u3) * p.a4 + ri % p.a4;
  }
  int64_t brow[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) brow[b] = base + p.rowtab[(u3 * NB + b) * 16 + j];   // padding: row 0 of the stage

  const int64_t n_lo = int64_t(blockIdx.y) * p.chunk;
  const int64_t n_hi = n_lo + p.chunk < p.N ? n_lo + p.chunk : p.N;
  const int64_t aoff = arow * p.ld_dO + q * CPL;
  int64_t boff[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) boff[b] = brow[b] * p.ldI + q * CPL;

  f32x4 acc[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};

  int64_t n = n_lo;
#pragma unroll 2
  for (; n + CPI <= n_hi; n += CPI) {
    const reg a = Op::load(p.dO, aoff + n);
    reg bv[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) bv[b] = Op::load(p.I, boff[b] + n);
#pragma unroll
    for (int b = 0; b < NB; ++b) Op::mac(a, bv[b], acc[b]);
  }
  if (n < n_hi) {   // ragged end of the batch: columns at and past n_hi count as zero on both sides
    const int64_t left = n_hi - (n + q * CPL);
    const int valid = left <= 0 ? 0 : left >= CPL ? CPL : int(left);
    const reg a = Op::load_tail(p.dO, aoff + n, valid);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const reg bv = Op::load_tail(p.I, boff[b] + n, valid);
      Op::mac(a, bv, acc[b]);
    }
  }

  // acc[b][i] = dW block element (row 4 * q + i of the 16, contraction step 16 * b + j)
  float *out = p.out + int64_t(blockIdx.y) * p.nnz;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r16 = 4 * q + i, mm = r16 >> p.lgRS, ri = r16 & (RS - 1);
    const int mem = p.members[cl * p.MG + mm];
    const int f = stg[(1 + mm) * 64];   // position of the stage among the member's weight fragments
    if (mem < 0 || f < 0 || ri >= p.R) continue;
    const int64_t row = ((int64_t(mem) * p.a2 + ri / p.a4) * p.a3 + u3) * p.a4 + ri % p.a4;
    float *dst = out + row * p.rowdeg + int64_t(f) * p.KCR;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int kk = 16 * b + j;
      if (kk < p.KCR) dst[kk] = acc[b][i];
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
  int32_t *units = nullptr, *stages = nullptr, *members = nullptr, *rowtab = nullptr;
  int nunits = 0;
  float *partial = nullptr;
  size_t partial_bytes = 0;
};

template <typename T>
int upload(const std::vector<T> &h, T **d) {
  RBGP_HIP(hipMalloc(reinterpret_cast<void **>(d), h.size() * sizeof(T) + 16));
  RBGP_HIP(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
  return RBGP_OK;
}

typedef void (*sddmm_fn)(SddmmParams);
sddmm_fn find_kernel(int NB, bool bf16) {
  switch (NB) {
    case 1: return bf16 ? sddmm_reg<1, true> : sddmm_reg<1, false>;
    case 2: return bf16 ? sddmm_reg<2, true> : sddmm_reg<2, false>;
    case 3: return bf16 ? sddmm_reg<3, true> : sddmm_reg<3, false>;
    case 4: return bf16 ? sddmm_reg<4, true> : sddmm_reg<4, false>;
    case 5: return bf16 ? sddmm_reg<5, true> : sddmm_reg<5, false>;
  }
  return nullptr;
}

int build_state(const rbgp_mask *m, SddmmState *st) {
  const rbgp_reg_plan &pl = m->reg;
  const rbgp_reg_clusters &cl = m->reg_clusters;
  const int NB = (pl.KCR + 15) / 16;
  std::vector<int32_t> units;
  for (int c = 0; c < cl.ncl; ++c)
    for (int s = 0; s < cl.counts[size_t(c)]; ++s) units.push_back(c * 64 + s);
  const int a3 = m->a[2], d3 = m->d[2], c3 = m->c[2], c4 = m->c[3];
  std::vector<int32_t> rt(size_t(a3) * NB * 16, 0);
  for (int u3 = 0; u3 < a3; ++u3)
    for (int kk = 0; kk < pl.KCR; ++kk) {
      const int v4 = kk % c4, j3 = (kk / c4) % d3, vv = kk / (c4 * d3);
      rt[(size_t(u3) * NB) * 16 + kk] = (vv * c3 + m->adj[2][size_t(u3) * d3 + j3]) * c4 + v4;
    }
  int rc = upload(units, &st->units);
  if (!rc) rc = upload(cl.stages, &st->stages);
  if (!rc) rc = upload(cl.members, &st->members);
  if (!rc) rc = upload(rt, &st->rowtab);
  st->nunits = int(units.size());
  return rc;
}

}  // namespace

void rbgp_sddmm_release(void *state) {
  SddmmState *st = static_cast<SddmmState *>(state);
  if (!st) return;
  if (st->units) (void)hipFree(st->units);
  if (st->stages) (void)hipFree(st->stages);
  if (st->members) (void)hipFree(st->members);
  if (st->rowtab) (void)hipFree(st->rowtab);
  if (st->partial) (void)hipFree(st->partial);
  delete st;
}

int rbgp_sddmm_launch(const rbgp_mask *m, void **state, const int32_t *const dev_adj[4], bool use_mfma, bool bf16,
                      int64_t N, const void *dO, int64_t ld_dO, const void *I, int64_t ldI, float *dW, void *stream) {
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int64_t nnz = m->nnz;
  if (N == 0) {
    sddmm_zero<<<dim3(unsigned((nnz + 255) / 256)), dim3(256), 0, hs>>>(dW, nnz);
    RBGP_HIP(hipGetLastError());
    return RBGP_OK;
  }
  if (!use_mfma) {
    GenericParams gp;
    for (int i = 0; i < 4; ++i) {
      gp.adj[i] = dev_adj[i];
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
  SddmmState *st = static_cast<SddmmState *>(*state);
  if (!st) {
    st = new (std::nothrow) SddmmState();
    if (!st) return RBGP_ENOMEM;
    *state = st;
  }
  if (!st->units) {
    int rc = build_state(m, st);
    if (rc) return rc;
  }
  const int NB = (pl.KCR + 15) / 16;
  sddmm_fn fn = find_kernel(NB, bf16);
  if (!fn) return RBGP_EUNSUPPORTED;
  // ranges of the batch: enough waves for several per SIMD (1024 SIMDs), at least two iterations each
  const int cpi = bf16 ? 32 : 16;
  const int64_t blocks = int64_t(st->nunits) * m->a[2];
  int64_t nsplit = (8192 + blocks - 1) / blocks;
  nsplit = std::max<int64_t>(1, std::min(nsplit, (N + 2 * cpi - 1) / (2 * cpi)));
  nsplit = std::min<int64_t>(nsplit, 1024);
  const int64_t chunk = ((N + nsplit - 1) / nsplit + cpi - 1) / cpi * cpi;
  nsplit = (N + chunk - 1) / chunk;
  if (nsplit > 1) {
    const size_t need = size_t(nsplit) * size_t(nnz) * sizeof(float);
    if (st->partial_bytes < need) {
      if (st->partial) RBGP_HIP(hipFree(st->partial));   // (waits for launches that still use it)
      st->partial = nullptr;
      st->partial_bytes = 0;
      RBGP_HIP(hipMalloc(reinterpret_cast<void **>(&st->partial), need));
      st->partial_bytes = need;
    }
  }
  SddmmParams p;
  p.dO = dO; p.I = I;
  p.out = nsplit > 1 ? st->partial : dW;
  p.units = st->units; p.stages = st->stages; p.members = st->members; p.rowtab = st->rowtab;
  p.N = N; p.ld_dO = ld_dO; p.ldI = ldI; p.nnz = nnz; p.chunk = chunk;
  p.a2 = pl.A2; p.a3 = m->a[2]; p.a4 = m->a[3]; p.R = pl.R;
  p.lgRS = 0;
  while ((1 << p.lgRS) < pl.RS) ++p.lgRS;
  p.MG = pl.MG; p.KCR = pl.KCR; p.rowdeg = int(m->rowdeg);
  fn<<<dim3(unsigned(blocks), unsigned(nsplit)), dim3(64), 0, hs>>>(p);
  RBGP_HIP(hipGetLastError());
  if (nsplit > 1) {
    sddmm_reduce<<<dim3(unsigned((nnz + 255) / 256)), dim3(256), 0, hs>>>(st->partial, dW, nnz, int(nsplit));
    RBGP_HIP(hipGetLastError());
  }
  return RBGP_OK;
}
