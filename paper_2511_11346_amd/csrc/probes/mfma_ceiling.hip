// Measures what the matrix pipes of this GPU sustain with NO memory traffic:
// every wave issues independent bf16 MFMAs on register operands (32x32x16, and 16x16x32
// for comparison), 8 waves per CU, once with constant operands and once with random ones.  On MI355X the
// random-operand figure is set by the power limit (the core clock drops), and it
// is the practical ceiling for any bf16 GEMM-shaped kernel on real data.
// Prints one JSON line.  Build: hipcc --offload-arch=gfx950 -O3 mfma_ceiling.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// the same flops per iteration from 16x16x32 instructions: 5 x 4 independent accumulators
__global__ __launch_bounds__(512) void k_mfma16(const i32x4* data, float* out, int iters, long long* clk) {
  f32x4 acc[20];
  for (int a = 0; a < 20; a++)
    for (int i = 0; i < 4; i++) acc[a][i] = 0.f;
  i32x4 xa[5], xb[4];
  for (int i = 0; i < 5; i++) xa[i] = data[(threadIdx.x * 7 + i) & 1023];
  for (int i = 0; i < 4; i++) xb[i] = data[(threadIdx.x * 7 + 5 + i) & 1023];
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int p = 0; p < 4; p++)
#pragma unroll
      for (int v = 0; v < 5; v++)
        acc[p * 5 + v] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, xa[v]), __builtin_bit_cast(bf16x8, xb[p]), acc[p * 5 + v], 0, 0, 0);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) { clk[0] = clock64() - c0; clk[1] = wall_clock64() - w0; }
  float s = 0;
  for (int a = 0; a < 20; a++)
    for (int i = 0; i < 4; i++) s += acc[a][i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(512) void k_mfma(const i32x4* data, float* out, int iters, long long* clk) {
  f32x16 acc[10];
  for (int a = 0; a < 10; a++)
    for (int i = 0; i < 16; i++) acc[a][i] = 0.f;
  i32x4 xa[5], xb[2];
  for (int i = 0; i < 5; i++) xa[i] = data[(threadIdx.x * 7 + i) & 1023];
  for (int i = 0; i < 2; i++) xb[i] = data[(threadIdx.x * 7 + 5 + i) & 1023];
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int p = 0; p < 2; p++)
#pragma unroll
      for (int v = 0; v < 5; v++)
        acc[p * 5 + v] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, xa[v]), __builtin_bit_cast(bf16x8, xb[p]), acc[p * 5 + v], 0, 0, 0);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) { clk[0] = clock64() - c0; clk[1] = wall_clock64() - w0; }
  float s = 0;
  for (int a = 0; a < 10; a++)
    for (int i = 0; i < 16; i++) s += acc[a][i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

int main() {
  const int blocks = 2048, iters = 4000;
  float* d; long long* clk; i32x4* data;
  CHECK(hipMalloc(&d, (size_t)blocks * 512 * 4));
  CHECK(hipMalloc(&clk, 16));
  CHECK(hipMalloc(&data, 1024 * 16));
  static unsigned short h[1024 * 8];
  double tf[4], mhz[4];
  srand(1);
  for (int mode = 0; mode < 4; ++mode) {
    auto kern = mode < 2 ? k_mfma : k_mfma16;
    const bool random = mode & 1;
    for (int i = 0; i < 1024 * 8; i++) {
      const float f = random ? ((rand() / (float)RAND_MAX) - 0.5f) * 0.1f : 1.0f;
      unsigned u; memcpy(&u, &f, 4); h[i] = (unsigned short)(u >> 16);
    }
    CHECK(hipMemcpy(data, h, sizeof(h), hipMemcpyHostToDevice));
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a)); CHECK(hipEventCreate(&b));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), 0, 0, data, d, 10, clk);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(a));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), 0, 0, data, d, iters, clk);
    CHECK(hipEventRecord(b)); CHECK(hipEventSynchronize(b));
    float ms; CHECK(hipEventElapsedTime(&ms, a, b));
    long long hc[2]; CHECK(hipMemcpy(hc, clk, 16, hipMemcpyDeviceToHost));
    tf[mode] = (double)blocks * 8 * iters * 10 * 32 * 32 * 16 * 2 / ms / 1e9;   // 20 x 16x16x32 = the same
    mhz[mode] = 100.0 * hc[0] / hc[1];   // wall clock ticks at 100 MHz
  }
  printf("{\"probe\": \"mfma_ceiling\", \"constant_operands_tflops\": %.0f, \"constant_operands_core_mhz\": %.0f, "
         "\"random_operands_tflops\": %.0f, \"random_operands_core_mhz\": %.0f, "
         "\"mfma_16x16x32\": {\"constant_operands_tflops\": %.0f, \"constant_operands_core_mhz\": %.0f, "
         "\"random_operands_tflops\": %.0f, \"random_operands_core_mhz\": %.0f}}\n",
         tf[0], mhz[0], tf[1], mhz[1], tf[2], mhz[2], tf[3], mhz[3]);
  return 0;
}
