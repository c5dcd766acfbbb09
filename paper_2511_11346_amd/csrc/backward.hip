// Small kernels of the training step: layout changes between the two big
// contractions and the reverse pass through the circuit layers (Sec. 4.1 loss:
// a linear combination of prefix log-marginals, loss = sum_j g_j P_j with
// g_j = coef_{j+1} - coef_j, coef_n = 0).
#include "mtpc_internal.h"

namespace mtpc {
namespace {

__device__ __forceinline__ unsigned short to_bf16_rne(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float wsum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
__device__ __forceinline__ float wmax(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}

// 64 x 64 element tiles through LDS; T is the 2- or 4-byte element type.
template <typename T>
__global__ __launch_bounds__(256) void k_transpose(const TransposeArgs a) {
  __shared__ T tile[64][64 + (sizeof(T) == 2 ? 2 : 1)];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;       // 4 rows per pass
  const T* src = (const T*)a.src;
  T* dst = (T*)a.dst;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int r = r0 + ty + 4 * k, c = c0 + tx;
    T val = 0;
    if (r < a.R && c < a.C) val = src[(long long)r * a.ld_src + c];
    tile[ty + 4 * k][tx] = val;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int c = c0 + ty + 4 * k, r = r0 + tx;
    if (c < a.C && r < a.Rpad) dst[(long long)c * a.ld_dst + a.col0 + r] = tile[tx][ty + 4 * k];
  }
}

// One wave per evidence row; lane l holds units l and l + 64.
__global__ __launch_bounds__(256) void k_circuit_bwd(const CircuitBwdArgs a) {
  __shared__ float sP[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long row = (long long)blockIdx.x * 4 + wave;
  const int n = a.n, r = a.r;
  const bool u0 = lane < r, u1 = lane + 64 < r;
  auto put_dsl = [&](float v0, float v1) {          // transposed, in the dtype of h
    if (a.dslT == nullptr || row >= a.ldb) return;
    if (a.bf16) {
      unsigned short* d = (unsigned short*)a.dslT;
      if (u0) d[(long long)lane * a.ldb + row] = to_bf16_rne(v0);
      if (u1) d[(long long)(lane + 64) * a.ldb + row] = to_bf16_rne(v1);
    } else {
      float* d = (float*)a.dslT;
      if (u0) d[(long long)lane * a.ldb + row] = v0;
      if (u1) d[(long long)(lane + 64) * a.ldb + row] = v1;
    }
  };
  if (row >= a.rows) {                              // padding columns of the transposed output
    put_dsl(0.f, 0.f);
    return;
  }
  const float* e = a.e + row * n * r;
  const float* coef = a.coef + row * n;
  float* Ge = a.Ge + row * n * r;
  auto g_of = [&](int j) { return (j + 1 < n ? coef[j + 1] : 0.f) - coef[j]; };
  const float ninf = neg_inf();

  if (a.family == MTPC_FF) {
    // P_j = e_0 + .. + e_j: d loss / d e_i = sum_{j >= i} g_j = -coef_i
    float P = 0.f, loss = 0.f;
    for (int j = 0; j < n; ++j) {
      P += e[j];
      loss += g_of(j) * P;
      if (lane == 0) Ge[j] = -coef[j];
    }
    if (lane == 0) a.loss[row] = loss;
    return;
  }
  const float* lw = a.logw + row * r;
  const float w0 = u0 ? lw[lane] : ninf, w1 = u1 ? lw[lane + 64] : ninf;

  if (a.family == MTPC_CP) {
    // s_j[z] = log omega_z + sum_{i<=j} e_i[z],  P_j = LSE_z s_j,  dP_j/de_i[z] = softmax(s_j)[z] (i <= j)
    float s0 = w0, s1 = w1, loss = 0.f;
    for (int j = 0; j < n; ++j) {
      if (u0) s0 += e[j * r + lane];
      if (u1) s1 += e[j * r + lane + 64];
      const float m = wmax(fmaxf(s0, s1));
      const float P = m + __logf(wsum((u0 ? __expf(s0 - m) : 0.f) + (u1 ? __expf(s1 - m) : 0.f)));
      if (lane == 0) sP[wave][j] = P;
      loss += g_of(j) * P;
    }
    __builtin_amdgcn_wave_barrier();
    float a0 = 0.f, a1 = 0.f;                       // sum_{j >= i} g_j softmax(s_j)
    for (int j = n - 1; j >= 0; --j) {
      const float P = sP[wave][j], g = g_of(j);
      if (u0) { a0 += g * __expf(s0 - P); Ge[j * r + lane] = a0; s0 -= e[j * r + lane]; }
      if (u1) { a1 += g * __expf(s1 - P); Ge[j * r + lane + 64] = a1; s1 -= e[j * r + lane + 64]; }
    }
    // log omega = log_softmax(sum-unit logits): d/dlogit_z = G_z - omega_z sum_z' G_z'
    const float tot = wsum((u0 ? a0 : 0.f) + (u1 ? a1 : 0.f));
    put_dsl(a0 - __expf(w0) * tot, a1 - __expf(w1) * tot);
    if (lane == 0) a.loss[row] = loss;
    return;
  }
}

}  // namespace

hipError_t launch_transpose(const TransposeArgs& a, int dtype, hipStream_t st) {
  if (a.C < 1 || a.Rpad < 1) return hipSuccess;
  const dim3 grid((a.C + 63) / 64, (a.Rpad + 63) / 64);
  if (dtype == MTPC_BF16) hipLaunchKernelGGL(k_transpose<unsigned short>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(k_transpose<float>, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_circuit_bwd(const CircuitBwdArgs& a, hipStream_t st) {
  const long long rows = a.dslT ? a.ldb : a.rows;
  hipLaunchKernelGGL(k_circuit_bwd, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace mtpc
