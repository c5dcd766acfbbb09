// MFMA kernels of the training step (Sec. 4.1 loss):
//   k_unembed_grad  recomputes the logits of one (i, j) slab for a tile of positions
//                   exactly as the forward kernel does, normalises them in registers
//                   and writes the gradient of the loss w.r.t. the logits,
//                   Ge[b,i,j] * (onehot(x_bi) - softmax), in the dtype of h; the logits
//                   themselves are never stored.
//   k_gemm_tn       C = A B^T with both operands K-contiguous: the two contractions
//                   that turn the logit gradient into dh (over n*r*v) and dW (over B).
#include "tile.h"

namespace mtpc {

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16>
__global__ __launch_bounds__(WV * WB * 64)
void k_unembed_grad(const GradLogitsArgs a) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr bool M16 = use_m16<WV, WB, SB, NS, BF16>();
  using FR = Frag<M16>;
  constexpr int NPB = PB * FR::SUB, NVB = VB * FR::SUB;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int lcol = FR::lcol(lane), lgrp = FR::lgrp(lane);
  const int nslab = a.n * a.r;
  const int nbt = (int)((a.ldb + TL::TP - 1) / TL::TP);
  int slab, bt;
  tile_of_block(blockIdx.x, nbt, nslab, slab, bt);
  const int b0 = bt * TL::TP;
  const int wi = slab / a.r, wj = slab - wi * a.r;
  if (b0 >= a.B) {
    // a tile of padding columns only (B is not a multiple of the tile): zeros
    for (int idx = tid; idx < a.v * TL::TP; idx += TL::NT) {
      const int row = idx / TL::TP, b = b0 + idx % TL::TP;
      if (b < a.ldb) {
        const long long o = ((long long)slab * a.v + row) * a.ldb + b;
        if constexpr (BF16) ((unsigned short*)a.dLT)[o] = 0; else ((float*)a.dLT)[o] = 0.f;
      }
    }
    return;
  }

  typename FR::blk_t acc[NPB][NVB];
  tile_gemm<WV, WB, VB, PB, SB, NS, BF16, false, M16>(a.W, a.d, a.h, a.ld_h, a.B, a.d, a.v, slab, b0, smem, acc);
  const int rbase = wv * VB * 32 + 4 * lgrp;
  float mx[NPB], lse[NPB];
  tile_lse<WV, WB, VB, PB, SB, NS, M16>(acc, a.v, (float2*)(smem + TL::RED_OFF), mx, lse);

  float g[NPB];
  int x[NPB];
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb) {
    const int b = b0 + wb * PB * 32 + pb * FR::BR + lcol;
    g[pb] = 0.f;
    x[pb] = -1;
    if (b < a.B) {
      x[pb] = a.targets[(long long)b * a.n + wi];
      // a summed-out variable (-1) has constant evidence: no gradient reaches its logits
      g[pb] = (x[pb] == -1) ? 0.f : a.Ge[((long long)b * a.n + wi) * a.r + wj];
    }
  }
  // the column blocks of a row back to back: together they fill whole lines
#pragma unroll
  for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
    for (int i = 0; i < FR::NI; ++i) {
      const int row = rbase + vb * FR::BR + FR::roff(i);
      if (row >= a.v) continue;
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb) {
        const int b = b0 + wb * PB * 32 + pb * FR::BR + lcol;
        if (b >= a.ldb) continue;
        float val = 0.f;
        if (b < a.B && x[pb] != -1) val = g[pb] * ((row == x[pb] ? 1.f : 0.f) - __expf(acc[pb][vb][i] - lse[pb]));
        const long long o = ((long long)slab * a.v + row) * a.ldb + b;
        if constexpr (BF16) ((unsigned short*)a.dLT)[o] = f32_to_bf16_rne(val);
        else ((float*)a.dLT)[o] = val;
      }
    }
}

template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16>
static hipError_t launch_grad_cfg(const GradLogitsArgs& a, hipStream_t st) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr auto kern = k_unembed_grad<WV, WB, VB, PB, SB, NS, BF16>;
  if (hipError_t e = allow_lds<kern>(TL::SMEM); e != hipSuccess) return e;
  const int nbt = (int)((a.ldb + TL::TP - 1) / TL::TP);
  hipLaunchKernelGGL(kern, dim3(nbt * a.n * a.r), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

template <bool BF16>
static hipError_t launch_grad_dt(const GradLogitsArgs& a, hipStream_t st) {
  if (a.v > 256) return launch_grad_cfg<2, 4, 5, 2, 64, 4, BF16>(a, st);
  if (a.v > 128) return launch_grad_cfg<2, 4, 4, 2, 64, 4, BF16>(a, st);
  return launch_grad_cfg<2, 4, 2, 2, 64, 4, BF16>(a, st);
}

hipError_t launch_unembed_grad(const GradLogitsArgs& a, int dtype, hipStream_t st) {
  return dtype == MTPC_BF16 ? launch_grad_dt<true>(a, st) : launch_grad_dt<false>(a, st);
}

// ---------------------------------------------------------------------------
template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16, bool ASTAGED>
__global__ __launch_bounds__(WV * WB * 64)
void k_gemm_tn(const GemmArgs a) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr bool M16 = use_m16<WV, WB, SB, NS, BF16>();
  using FR = Frag<M16>;
  constexpr int NPB = PB * FR::SUB, NVB = VB * FR::SUB;
  constexpr int ESZ = BF16 ? 2 : 4;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int lcol = FR::lcol(lane), lgrp = FR::lgrp(lane);
  const int nslab = (a.M + TL::TV - 1) / TL::TV;
  const int nbt = (a.N + TL::TP - 1) / TL::TP;
  const int tiles = nbt * nslab;
  const int total = tiles * max(a.ksplit, 1);
  // One workgroup per CU walks the tiles blockIdx.x, blockIdx.x + gridDim.x, ... and opens the feed of the
  // next tile before it stores the one it has multiplied (the stores touch no ring memory): the first
  // stages of the next ring arrive while the 320 x 256 results leave.
  struct Where { int slab, b0, rows, ks, k0, klen; };
  auto where = [&](int w) {
    Where t;
    int bt;
    t.ks = w / tiles;                                // K split handled by this tile
    tile_of_block(w - t.ks * tiles, nbt, nslab, t.slab, bt);
    t.b0 = bt * TL::TP;
    t.rows = min(TL::TV, a.M - t.slab * TL::TV);
    t.k0 = t.ks * a.kchunk;
    t.klen = min(a.kchunk, a.K - t.k0);
    return t;
  };
  TileFeed<WV, WB, VB, PB, SB, NS, BF16, false, M16, ASTAGED> feed;
  auto open = [&](const Where& t) {
    // (the chunk [k0, k0 + klen) of a stage-major operand is the run of its stages k0 * ESZ / 64 onwards)
    const char* bs = (a.Bs != nullptr && SB == 64) ? (const char*)a.Bs + (long long)t.k0 * ESZ / 64 * a.N * 64 : nullptr;
    if constexpr (ASTAGED)
      feed.open((const char*)a.As + (long long)t.k0 * ESZ / 64 * a.As_rows * 64, 0, (const char*)a.Bm + (long long)t.k0 * ESZ,
                a.ldb, a.N, t.klen, t.rows, 0, t.b0, smem, nullptr, 0, 1, bs, a.As_rows, t.slab * TL::TV);
    else
      feed.open((const char*)a.A + ((long long)t.slab * TL::TV * a.lda + t.k0) * ESZ, a.lda,
                (const char*)a.Bm + (long long)t.k0 * ESZ, a.ldb, a.N, t.klen, t.rows, 0, t.b0, smem, nullptr, 0, 1, bs);
  };
  Where cur = where(blockIdx.x);
  open(cur);
  for (int w = blockIdx.x;;) {
    typename FR::blk_t acc[NPB][NVB];
    tile_gemm_run(feed, cur.klen, smem, acc);
    const int wnext = w + (int)gridDim.x;
    Where nxt = cur;
    if (wnext < total) {
      nxt = where(wnext);
      open(nxt);
    }
    const int slab = cur.slab, b0 = cur.b0, rows = cur.rows, ks = cur.ks;
    const int rbase = wv * VB * 32 + 4 * lgrp;
    // A full tile that lies inside one destination (the common case): one base pointer per
    // column, rows at constant multiples of ldc.
    bool stored = false;
    {
      const long long gr0 = (long long)slab * TL::TV;
      float* base = nullptr;
      if (rows == TL::TV) {
        if (a.ksplit > 1) base = a.partial + ((long long)ks * a.M + gr0) * a.ldc;
        else if (gr0 + TL::TV <= a.split) base = a.C + gr0 * a.ldc;
      }
      if (base != nullptr) {
        // the column blocks of a row back to back: together they fill whole lines
        const int col0 = b0 + wb * PB * 32 + lcol;
        float* cp = base + (long long)rbase * a.ldc + col0;
#pragma unroll
        for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
          for (int i = 0; i < FR::NI; ++i)
#pragma unroll
            for (int pb = 0; pb < NPB; ++pb)
              if (col0 + pb * FR::BR < a.N)
                cp[(long long)(vb * FR::BR + FR::roff(i)) * a.ldc + pb * FR::BR] = acc[pb][vb][i];
        stored = true;
      }
    }
    if (!stored) {
      // one destination row at a time (keeps the address arithmetic out of the 160 live accumulators)
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int i = 0; i < FR::NI; ++i) {
          const int row = rbase + vb * FR::BR + FR::roff(i);
          if (row >= rows) continue;
          const long long gr = (long long)slab * TL::TV + row;
          float* rp = nullptr;
          if (a.ksplit > 1) rp = a.partial + ((long long)ks * a.M + gr) * a.ldc;
          else if (gr < a.split) rp = a.C + gr * a.ldc;
          else if (gr < a.split + a.n2) rp = a.C2 + (gr - a.split) * a.ldc;
          else if (gr >= a.split3) rp = a.C3 + (gr - a.split3) * a.ldc;
          if (rp == nullptr) continue;
#pragma unroll
          for (int pb = 0; pb < NPB; ++pb) {
            const int col = b0 + wb * PB * 32 + pb * FR::BR + lcol;
            if (col < a.N) rp[col] = acc[pb][vb][i];
          }
        }
    }
    if (wnext >= total) break;
    w = wnext;
    cur = nxt;
  }
}

template <int WV, int WB, int VB, int PB, bool BF16, bool ASTAGED = false>
static hipError_t launch_gemm_cfg(const GemmArgs& a, hipStream_t st) {
  using TL = Tile<WV, WB, VB, PB, 64, 4>;
  if constexpr (!ASTAGED)
    if (a.As != nullptr) return launch_gemm_cfg<WV, WB, VB, PB, BF16, true>(a, st);
  constexpr auto kern = k_gemm_tn<WV, WB, VB, PB, 64, 4, BF16, ASTAGED>;
  if (hipError_t e = allow_lds<kern>(TL::SMEM); e != hipSuccess) return e;
  const int nslab = (a.M + TL::TV - 1) / TL::TV, nbt = (a.N + TL::TP - 1) / TL::TP;
  int grid = nslab * nbt * max(a.ksplit, 1);
  // one workgroup per CU (the ring takes most of a CU's LDS), a multiple of the 8 XCDs the ids are dealt over
  int cus = 0;
  if (hipError_t e = cu_count(&cus); e != hipSuccess) return e;
  if (cus >= 8) grid = std::min(grid, cus / 8 * 8);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

// C[i] = sum over the K splits of partial[ks][i], in the order ks = 0, 1, ...
__global__ __launch_bounds__(256) void k_reduce_splits(const float* partial, long long count, int ksplit, float* C) {
  const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= count) return;
  f32x4_t s = *(const f32x4_t*)(partial + i);
  for (int ks = 1; ks < ksplit; ++ks) {
    const f32x4_t p = *(const f32x4_t*)(partial + (long long)ks * count + i);
    s[0] += p[0]; s[1] += p[1]; s[2] += p[2]; s[3] += p[3];
  }
  *(f32x4_t*)(C + i) = s;
}

template <bool BF16>
static hipError_t launch_gemm_dt(const GemmArgs& a, hipStream_t st) {
  // 320 x 256 workgroup tiles (the forward kernel's shape; measured 7 % faster per output
  // row) or 256 x 256 ones, whichever needs less time by a count of rounds over the 256
  // CUs: whole rounds while there are few workgroups, fractional once there are many
  auto cost = [&](int rows, double gain) {
    const double wgs = (double)((a.M + rows - 1) / rows) * ((a.N + 255) / 256);
    const double rounds = wgs >= 1024 ? wgs / 256.0 : (double)(long long)((wgs + 255) / 256);
    return rounds * rows * gain;
  };
  if (a.ksplit == 1 && cost(320, 0.93) < cost(256, 1.0)) return launch_gemm_cfg<2, 4, 5, 2, BF16>(a, st);
  return launch_gemm_cfg<2, 4, 4, 2, BF16>(a, st);
}

hipError_t launch_gemm_tn(const GemmArgs& a0, int dtype, hipStream_t st) {
  if (a0.M < 1 || a0.N < 1) return hipSuccess;
  GemmArgs a = a0;
  if (a.ksplit <= 1 || a.partial == nullptr) { a.ksplit = 1; a.kchunk = a.K; }
  const hipError_t e = dtype == MTPC_BF16 ? launch_gemm_dt<true>(a, st) : launch_gemm_dt<false>(a, st);
  if (e != hipSuccess || a.ksplit == 1) return e;
  const long long count = (long long)a.M * a.ldc;     // ldc a multiple of 4 (d is a multiple of 32)
  hipLaunchKernelGGL(k_reduce_splits, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0, st, a.partial, count,
                     a.ksplit, a.C);
  return hipGetLastError();
}

}  // namespace mtpc
