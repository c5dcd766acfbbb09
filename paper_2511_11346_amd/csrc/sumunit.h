// Sum-unit weights of one position (Sec. 3.3: log omega = log_softmax(Wsum h)), as a piece of
// device code that the kernels needing them for a handful of positions share: the stand-alone
// kernel, the one that goes on to draw the latents, and the verification step.
#pragma once

#include "mtpc_internal.h"

namespace mtpc {

typedef __attribute__((ext_vector_type(4))) int i32x4_t;

// dot of two rows of 8-element (bf16) or 4-element (fp32) 16-byte chunks
template <bool BF16>
__device__ __forceinline__ float dot_chunk(const i32x4_t& a, const i32x4_t& b) {
  float s = 0.f;
  if constexpr (BF16) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint32_t ua = (uint32_t)a[t], ub = (uint32_t)b[t];
      s = fmaf(__uint_as_float(ua << 16), __uint_as_float(ub << 16), s);
      s = fmaf(__uint_as_float(ua & 0xFFFF0000u), __uint_as_float(ub & 0xFFFF0000u), s);
    }
  } else {
#pragma unroll
    for (int t = 0; t < 4; ++t) s = fmaf(__int_as_float(a[t]), __int_as_float(b[t]), s);
  }
  return s;
}

// log omega[b][:] into sc[0..r) (LDS, 128 floats) by a workgroup of NW waves: they split the r rows
// of Wsum, the position's hidden vector stays in registers (up to 8 chunks of 16 bytes per lane per
// pass: d <= 4096 bf16 / 2048 fp32 in one pass), Q rows at a time so that many loads are in flight
// (a workgroup that does nothing else takes 16 waves: one compute unit then has all of a 32 x 4096
// Wsum in flight at once instead of in two rounds).  Ends with a barrier: every thread may read sc
// afterwards.
template <bool BF16, int NW = 4>
__device__ __forceinline__ void sumunit_position(const void* h, long long ld_h, const void* Wsum, int b, int d, int r,
                                                 float* sc) {
  constexpr int ESZ = BF16 ? 2 : 4;
  constexpr int EPC = 16 / ESZ;
  constexpr int Q = NW > 4 ? 2 : 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const char* hb = (const char*)h + (long long)b * ld_h * ESZ;
  const int nch = d / EPC;
  for (int c0 = 0; c0 < nch; c0 += 512) {
    i32x4_t hv[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int c = c0 + t * 64 + lane;
      const i32x4_t x = *(const i32x4_t*)(hb + (long long)min(c, nch - 1) * 16);
      hv[t] = c < nch ? x : i32x4_t{0, 0, 0, 0};
    }
    for (int j0 = wave * Q; j0 < r; j0 += NW * Q) {
      float acc[Q];
#pragma unroll
      for (int q = 0; q < Q; ++q) acc[q] = 0.f;
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const int j = min(j0 + q, r - 1);
        const char* wr = (const char*)Wsum + (long long)j * d * ESZ;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          // unconditional (clamped) loads so that all of them are in flight together;
          // chunks beyond d meet a zero hv
          const int c = min(c0 + t * 64 + lane, nch - 1);
          acc[q] += dot_chunk<BF16>(*(const i32x4_t*)(wr + (long long)c * 16), hv[t]);
        }
      }
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const float v = group_sum(acc[q], 64);
        if (lane == 0 && j0 + q < r) { if (c0 == 0) sc[j0 + q] = v; else sc[j0 + q] += v; }
      }
    }
  }
  __syncthreads();
  if (wave == 0) {
    const float s0 = lane < r ? sc[lane] : neg_inf();
    const float s1 = lane + 64 < r ? sc[lane + 64] : neg_inf();
    const float m = group_max(fmaxf(s0, s1), 64);
    float e = 0.f;
    if (s0 > neg_inf()) e += __expf(s0 - m);
    if (s1 > neg_inf()) e += __expf(s1 - m);
    e = group_sum(e, 64);
    const float lse = m + __logf(e);
    if (lane < r) sc[lane] = s0 - lse;
    if (lane + 64 < r) sc[lane + 64] = s1 - lse;
  }
  __syncthreads();
}

}  // namespace mtpc
