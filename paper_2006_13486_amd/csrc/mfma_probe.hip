// Probe of the matrix-core instruction forms on gfx950, used to choose the kernels' MFMA:
//  * issue rate of the fp32 and bf16 MFMA forms with one and two waves per SIMD,
//  * register layout of v_mfma_f32_16x16x1_4b_f32 (checked against its definition),
//  * cost of back-to-back launches of an empty kernel (dispatch floor of one stream).
// Build: python -m paper_2006_13486_amd.build probe ; run: paper_2006_13486_amd/mfma_probe
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); return 1; } } while (0)

template <int KIND>
__global__ __launch_bounds__(256) void k(float* out, int iters, float a0, float b0) {
  float a = a0 + threadIdx.x, b = b0 + threadIdx.x;
  if constexpr (KIND == 0) {         // 4x4x1 16 blocks, cbsz=4
    f32x4 acc[8] = {};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, acc[j], 4, 3, 0);
    }
    float s = 0; for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][3];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 1) {  // 4x4x1 no broadcast
    f32x4 acc[8] = {};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0; for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][3];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 2) {  // 16x16x4 f32
    f32x4 acc[8] = {};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0; for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][3];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 3) {  // 32x32x2 f32
    f32x16 acc[4] = {};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0; for (int j = 0; j < 4; ++j) s += acc[j][0] + acc[j][15];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 4) {  // 16x16x1 4 blocks f32
    f32x16 acc[4] = {};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x1f32(a, b, acc[j], 2, 1, 0);
    }
    float s = 0; for (int j = 0; j < 4; ++j) s += acc[j][0] + acc[j][15];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 5) {  // 4x4x4 16 blocks bf16_1k
    f32x4 acc[8] = {};
    s16x4 av = {short(threadIdx.x), 1, 2, 3}, bv = {3, 2, 1, short(threadIdx.x)};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(av, bv, acc[j], 4, 3, 0);
    }
    float s = 0; for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][3];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 6) {  // 16x16x16 bf16_1k
    f32x4 acc[8] = {};
    s16x4 av = {short(threadIdx.x), 1, 2, 3}, bv = {3, 2, 1, short(threadIdx.x)};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, bv, acc[j], 0, 0, 0);
    }
    float s = 0; for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][3];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 7) {  // 16x16x32 bf16 (gfx950)
    f32x4 acc[8] = {};
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    bf16x8 av, bv;
    for (int q = 0; q < 8; ++q) { av[q] = (__bf16)(float)(threadIdx.x + q); bv[q] = (__bf16)(float)(q); }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc[j], 0, 0, 0);
    }
    float s = 0; for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][3];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 8) {  // 32x32x16 bf16 (gfx950)
    f32x16 acc[4] = {};
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    bf16x8 av, bv;
    for (int q = 0; q < 8; ++q) { av[q] = (__bf16)(float)(threadIdx.x + q); bv[q] = (__bf16)(float)(q); }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[j], 0, 0, 0);
    }
    float s = 0; for (int j = 0; j < 4; ++j) s += acc[j][0] + acc[j][15];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  } else if constexpr (KIND == 9) {  // plain v_fma_f32, 16 chains
    float acc[16];
    for (int j = 0; j < 16; ++j) acc[j] = j;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[j] = __builtin_fmaf(a, acc[j], b);
    }
    float s = 0; for (int j = 0; j < 16; ++j) s += acc[j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
  }
}

__global__ void layout_kernel(float* out) {
  int l = threadIdx.x;
  float a = 1.0f + (l / 16) * 100 + (l % 16);            // A_b[i] = 1 + 100 b + i
  float b = 1.0f + (l / 16) * 0.5f + (l % 16) * 0.01f;   // B_b[j] = 1 + .5 b + .01 j
  f32x16 acc = {};
  acc = __builtin_amdgcn_mfma_f32_16x16x1f32(a, b, acc, 0, 0, 0);
  for (int v = 0; v < 16; ++v) out[v * 64 + l] = acc[v];
}
__global__ void empty_kernel(float* p) { if (threadIdx.x == 1000) p[0] = 1; }

template <int KIND>
int run(const char* name, double flops_per_inst, int per_iter, float* out, int blocks, int iters) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  hipLaunchKernelGGL(k<KIND>, dim3(blocks), dim3(256), 0, 0, out, 10, 1.0f, 2.0f);
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0, 0));
  hipLaunchKernelGGL(k<KIND>, dim3(blocks), dim3(256), 0, 0, out, iters, 1.0f, 2.0f);
  CHECK(hipEventRecord(e1, 0));
  CHECK(hipEventSynchronize(e1));
  float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
  double insts_per_simd = double(iters) * per_iter * (blocks / 256.0);   // waves per SIMD = blocks/256
  double cyc = ms * 1e-3 * 2.4e9 / insts_per_simd;
  double tflops = double(blocks) * 4 * iters * per_iter * flops_per_inst / (ms * 1e-3) / 1e12;
  printf("%-28s blocks=%4d  %8.3f ms  %6.2f cycles/inst/SIMD @2.4GHz  %8.1f TFLOP/s\n", name, blocks, ms, cyc, tflops);
  return 0;
}

int main() {
  float* out; CHECK(hipMalloc(&out, 1024 * 256 * 4));
  const int iters = 20000;
  for (int blocks : {256, 512}) {
    run<0>("f32 4x4x1_16B cbsz4", 512, 8, out, blocks, iters);
    run<1>("f32 4x4x1_16B", 512, 8, out, blocks, iters);
    run<2>("f32 16x16x4", 2048, 8, out, blocks, iters);
    run<3>("f32 32x32x2", 4096, 4, out, blocks, iters);
    run<4>("f32 16x16x1_4B cbsz2", 2048, 4, out, blocks, iters);
    run<5>("bf16 4x4x4_16B cbsz4", 2048, 8, out, blocks, iters);
    run<6>("bf16 16x16x16", 8192, 8, out, blocks, iters);
    run<7>("bf16 16x16x32", 16384, 8, out, blocks, iters);
    run<8>("bf16 32x32x16", 32768, 4, out, blocks, iters);
    run<9>("f32 v_fma (64 lanes)", 128, 16, out, blocks, iters);
  }
  // layout of the four-block 16x16x1 form: D_b[i][j] expected in VGPR 4b + i%4 of lane 16*(i/4) + j
  hipLaunchKernelGGL(layout_kernel, dim3(1), dim3(64), 0, 0, out);
  static float h[1024];
  CHECK(hipMemcpy(h, out, sizeof h, hipMemcpyDeviceToHost));
  int bad = 0;
  for (int b = 0; b < 4; ++b) for (int i = 0; i < 16; ++i) for (int j = 0; j < 16; ++j) {
    float want = (1.0f + b * 100 + i) * (1.0f + b * 0.5f + j * 0.01f);
    if (h[(4 * b + i % 4) * 64 + 16 * (i / 4) + j] != want) ++bad;
  }
  printf("16x16x1_4B layout check: %d mismatches of 1024\n", bad);
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  CHECK(hipEventRecord(e0, 0));
  for (int i = 0; i < 2000; ++i) hipLaunchKernelGGL(empty_kernel, dim3(256), dim3(256), 0, 0, out);
  CHECK(hipEventRecord(e1, 0)); CHECK(hipEventSynchronize(e1));
  float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
  printf("empty kernel, 2000 back-to-back launches: %.2f us per launch\n", ms * 1e3 / 2000);
  return bad != 0;
}
