// Fused unembedding kernel of the MtPC head for gfx950 (Sec. 3.3):
//   l[b,i,j,:] = W[i,j] h[b]   (MFMA, fp32 accumulate)
//   LSE over the vocabulary in registers, then either the evidence
//   e[b,i,j] = l[x] - LSE at the target token or an inverse-CDF token draw.
// The (B, n, r, v) logits live only in accumulator registers.
//
// Tiling.  One workgroup computes D = W_slab (v rows) x h_tile^T (TP positions):
// the vocabulary is the MFMA M dimension, positions the N dimension, so that the
// 32x32 accumulator block of a lane holds 16 vocabulary rows of ONE position and
// the softmax reduction is almost entirely lane-local.  Wave grid WV (vocab) x WB
// (positions); a wave owns VB x PB blocks of 32x32.
// K is consumed in stages of 64 bytes per row (32 bf16 / 16 fp32), staged through
// LDS (double buffered, 80-byte row pitch: conflict-free 16-byte reads).
#include "mtpc_internal.h"

namespace mtpc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;

constexpr int STAGE_BYTES = 64;   // bytes of K per row per stage
constexpr int CPR = 4;            // 16-byte chunks per row per stage
constexpr int PITCH = 80;         // LDS row pitch in bytes
constexpr int NSLOT = 16;         // positions sampled per pass of the draw loop

template <int WV, int WB, int VB, int PB>
struct Tile {
  static constexpr int NW = WV * WB;
  static constexpr int NT = NW * 64;
  static constexpr int TV = WV * VB * 32;
  static constexpr int TP = WB * PB * 32;
  static constexpr int ROWS = TV + TP;
  static constexpr int NCHUNK = ROWS * CPR;
  static constexpr int LPT = (NCHUNK + NT - 1) / NT;
  static constexpr int STAGE = ROWS * PITCH;
  static constexpr int VPL = (TV + 63) / 64;           // values per lane in the draw scan
  static constexpr int RED_OFF = 2 * STAGE;            // float2 red[WV][TP]
  static constexpr int MISC_OFF = RED_OFF + WV * TP * 8;   // int cnt, list[TP], slot[TP]
  static constexpr int SMEM = MISC_OFF + 16 + TP * 8;
  static_assert(NSLOT * VPL * 64 * 4 <= 2 * STAGE, "draw buffer must fit in the stage buffers");
};

template <bool BF16>
__device__ __forceinline__ void mma_step(f32x16_t& acc, const i32x4_t& a, const i32x4_t& b) {
  if constexpr (BF16) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                  __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
  } else {
    f32x4_t af = __builtin_bit_cast(f32x4_t, a), bf = __builtin_bit_cast(f32x4_t, b);
#pragma unroll
    for (int t = 0; t < 4; ++t)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[t], acc, 0, 0, 0);
  }
}

// Map the hardware workgroup id to a (slab, position tile) pair.  Workgroup ids
// are dealt round-robin to the 8 XCDs, each with its own L2: give every XCD a
// contiguous range of logical ids, and walk logical ids through groups of 4
// slabs x all position tiles so that concurrently running workgroups of an XCD
// share a few W slabs and a few h tiles.
__device__ __forceinline__ void tile_of_block(int w, int nbt, int nslab, int& slab, int& bt) {
  const int total = nbt * nslab;
  const int per = total >> 3;
  int lid = (w < per * 8) ? (w & 7) * per + (w >> 3) : w;
  constexpr int GS = 4;
  const int gsz = GS * nbt;
  const int g = lid / gsz, rem = lid - g * gsz;
  const int gs = min(GS, nslab - g * GS);
  bt = rem / gs;
  slab = g * GS + (rem - bt * gs);
}

// D = W_slab x h_tile^T for one workgroup; on return every wave holds its VB x PB
// accumulator blocks and all waves have passed a barrier (LDS stages are free).
template <int WV, int WB, int VB, int PB, bool BF16>
__device__ __forceinline__ void tile_gemm(const void* Wp, const void* hp, long long ld_h, int B, int d,
                                          int v, int slab, int b0, char* smem,
                                          f32x16_t (&acc)[PB][VB]) {
  using TL = Tile<WV, WB, VB, PB>;
  constexpr int ESZ = BF16 ? 2 : 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int l31 = lane & 31, lhalf = lane >> 5;

  // global -> LDS staging descriptors (rows beyond v / B are clamped: they stay
  // in bounds and their results are masked or never written)
  const char* gp[TL::LPT];
  int lofs[TL::LPT];
#pragma unroll
  for (int q = 0; q < TL::LPT; ++q) {
    int c = tid + q * TL::NT;
    if (c >= TL::NCHUNK) c = TL::NCHUNK - 1;
    const int row = c / CPR, ch = c % CPR;
    const char* base;
    if (row < TL::TV) {
      const long long grow = (long long)slab * v + min(row, v - 1);
      base = (const char*)Wp + grow * (long long)d * ESZ;
    } else {
      const long long brow = min(b0 + row - TL::TV, B - 1);
      base = (const char*)hp + brow * ld_h * ESZ;
    }
    gp[q] = base + ch * 16;
    lofs[q] = row * PITCH + ch * 16;
  }
  constexpr bool LAST_PARTIAL = (TL::NCHUNK % TL::NT) != 0;
  const bool last_on = !LAST_PARTIAL || (tid + (TL::LPT - 1) * TL::NT < TL::NCHUNK);

#pragma unroll
  for (int pb = 0; pb < PB; ++pb)
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[pb][vb][i] = 0.f;

  const int KI = d * ESZ / STAGE_BYTES;
  i32x4_t stg[TL::LPT];

  auto gload = [&]() {
#pragma unroll
    for (int q = 0; q < TL::LPT; ++q) {
      if (q < TL::LPT - 1 || last_on) stg[q] = *(const i32x4_t*)gp[q];
      gp[q] += STAGE_BYTES;
    }
  };
  auto lstore = [&](int buf) {
    char* s = smem + buf * TL::STAGE;
#pragma unroll
    for (int q = 0; q < TL::LPT; ++q)
      if (q < TL::LPT - 1 || last_on) *(i32x4_t*)(s + lofs[q]) = stg[q];
  };

  const int a_off = (wv * VB * 32 + l31) * PITCH + lhalf * 16;
  const int b_off = (TL::TV + wb * PB * 32 + l31) * PITCH + lhalf * 16;

  gload();
  lstore(0);
  __syncthreads();
  for (int it = 0; it < KI; ++it) {
    const int cur = it & 1;
    const bool more = it + 1 < KI;
    if (more) gload();
    const char* s = smem + cur * TL::STAGE;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      i32x4_t af[VB], bfr[PB];
#pragma unroll
      for (int vb = 0; vb < VB; ++vb)
        af[vb] = *(const i32x4_t*)(s + a_off + vb * 32 * PITCH + ks * 32);
#pragma unroll
      for (int pb = 0; pb < PB; ++pb)
        bfr[pb] = *(const i32x4_t*)(s + b_off + pb * 32 * PITCH + ks * 32);
#pragma unroll
      for (int pb = 0; pb < PB; ++pb)
#pragma unroll
        for (int vb = 0; vb < VB; ++vb) mma_step<BF16>(acc[pb][vb], af[vb], bfr[pb]);
    }
    if (more) lstore(cur ^ 1);
    __syncthreads();
  }
}

// Softmax statistics of every position column of the tile: max and log-sum-exp
// over the v vocabulary rows.  Lane (l31, lhalf) of wave (wv, wb) holds, for
// position column p = wb*PB*32 + pb*32 + l31, the vocabulary rows
//   row(vb, i) = wv*VB*32 + vb*32 + 8*(i/4) + 4*lhalf + (i%4).
// Contains one workgroup barrier; `red` must not be reused before the next one.
template <int WV, int WB, int VB, int PB>
__device__ __forceinline__ void tile_lse(const f32x16_t (&acc)[PB][VB], int v, float2* red,
                                         float (&mx)[PB], float (&lse)[PB]) {
  using TL = Tile<WV, WB, VB, PB>;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int l31 = lane & 31, lhalf = lane >> 5;
  const int rbase = wv * VB * 32 + 4 * lhalf;
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    float m = neg_inf();
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = rbase + vb * 32 + 8 * (i >> 2) + (i & 3);
        if (row < v) m = fmaxf(m, acc[pb][vb][i]);
      }
    m = fmaxf(m, __shfl_xor(m, 32));
    const float ms = (m == neg_inf()) ? 0.f : m;
    float s = 0.f;
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = rbase + vb * 32 + 8 * (i >> 2) + (i & 3);
        if (row < v) s += __expf(acc[pb][vb][i] - ms);
      }
    s += __shfl_xor(s, 32);
    if (lhalf == 0) red[wv * TL::TP + wb * PB * 32 + pb * 32 + l31] = make_float2(m, s);
  }
  __syncthreads();
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    const int p = wb * PB * 32 + pb * 32 + l31;
    float M = neg_inf();
#pragma unroll
    for (int w = 0; w < WV; ++w) M = fmaxf(M, red[w * TL::TP + p].x);
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < WV; ++w) {
      const float2 t = red[w * TL::TP + p];
      if (t.y > 0.f) s += t.y * __expf(t.x - M);
    }
    mx[pb] = M;
    lse[pb] = M + __logf(s);
  }
}

template <int WV, int WB, int VB, int PB, bool BF16, bool SAMPLE>
__global__ __launch_bounds__(WV * WB * 64)
void k_unembed(const UnembedArgs a) {
  using TL = Tile<WV, WB, VB, PB>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int l31 = lane & 31, lhalf = lane >> 5;
  const int nslab = a.n * a.r;
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  int slab, bt;
  tile_of_block(blockIdx.x, nbt, nslab, slab, bt);
  const int b0 = bt * TL::TP;
  const int wi = slab / a.r, wj = slab - wi * a.r;

  f32x16_t acc[PB][VB];
  tile_gemm<WV, WB, VB, PB, BF16>(a.W, a.h, a.ld_h, a.B, a.d, a.v, slab, b0, smem, acc);

  const int rbase = wv * VB * 32 + 4 * lhalf;
  float mx[PB], lse[PB];
  tile_lse<WV, WB, VB, PB>(acc, a.v, (float2*)(smem + TL::RED_OFF), mx, lse);

  // evidence at the target tokens
  if (a.targets != nullptr) {
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const int b = b0 + wb * PB * 32 + pb * 32 + l31;
      if (b < a.B) {
        for (int t = 0; t < a.T; ++t) {
          const long long rowid = (long long)b * a.T + t;
          const int x = a.targets[rowid * a.n + wi];
          float* dst = a.e + (rowid * a.n + wi) * a.r + wj;
          if (x < 0 || x >= a.v) {
            if (wv == 0 && lhalf == 0) *dst = (x == -1) ? 0.f : __builtin_nanf("");
          } else {
            const int xr = x - rbase;
            float val = 0.f;
            bool hit = false;
#pragma unroll
            for (int vb = 0; vb < VB; ++vb)
#pragma unroll
              for (int i = 0; i < 16; ++i)
                if (xr == vb * 32 + 8 * (i >> 2) + (i & 3)) { val = acc[pb][vb][i]; hit = true; }
            if (hit) *dst = val - lse[pb];
          }
        }
      }
    }
  }
  if (a.lse != nullptr && wv == 0 && lhalf == 0) {
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const int b = b0 + wb * PB * 32 + pb * 32 + l31;
      if (b < a.B) a.lse[((long long)b * a.n + wi) * a.r + wj] = lse[pb];
    }
  }

  if constexpr (SAMPLE) {
    if (a.zleaf == nullptr) return;
    // ---- which positions of this tile draw token wi from component wj?
    int* misc = (int*)(smem + TL::MISC_OFF);
    int* s_cnt = misc;
    int* s_list = misc + 4;
    int* s_slot = s_list + TL::TP;
    float* probs = (float*)smem;   // stage buffers are free now
    if (tid == 0) *s_cnt = 0;
    __syncthreads();
    for (int p = tid; p < TL::TP; p += TL::NT) {
      const int b = b0 + p;
      bool need = false;
      if (b < a.B)
        for (int s = 0; s < a.S; ++s)
          need |= (a.zleaf[((long long)b * a.S + s) * a.n + wi] == wj);
      if (need) s_list[atomicAdd(s_cnt, 1)] = p;
    }
    __syncthreads();
    const int cnt = *s_cnt;
    for (int c0 = 0; c0 < cnt; c0 += NSLOT) {
      const int nsl = min(NSLOT, cnt - c0);
      for (int p = tid; p < TL::TP; p += TL::NT) s_slot[p] = -1;
      __syncthreads();
      if (tid < nsl) s_slot[s_list[c0 + tid]] = tid;
      __syncthreads();
      // dump exp(l - max) of the selected positions in vocabulary order
#pragma unroll
      for (int pb = 0; pb < PB; ++pb) {
        const int sl = s_slot[wb * PB * 32 + pb * 32 + l31];
        if (sl >= 0) {
#pragma unroll
          for (int vb = 0; vb < VB; ++vb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int row = rbase + vb * 32 + 8 * (i >> 2) + (i & 3);
              probs[sl * (TL::VPL * 64) + row] = (row < a.v) ? expf(acc[pb][vb][i] - mx[pb]) : 0.f;
            }
        }
      }
      __syncthreads();
      for (int k = wave; k < nsl; k += TL::NW) {
        const int p = s_list[c0 + k];
        const int b = b0 + p;
        float vals[TL::VPL];
        float ls = 0.f;
#pragma unroll
        for (int q = 0; q < TL::VPL; ++q) {
          vals[q] = probs[k * (TL::VPL * 64) + lane * TL::VPL + q];
          ls += vals[q];
        }
        float incl = ls;   // inclusive scan over lanes
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const float t = __shfl_up(incl, o);
          if (lane >= o) incl += t;
        }
        const float Z = __shfl(incl, 63);
        for (int s = 0; s < a.S; ++s) {
          const long long di = ((long long)b * a.S + s) * a.n + wi;
          if (a.zleaf[di] != wj) continue;
          const float u = philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, (uint32_t)s,
                                         (uint32_t)wi);
          const float tgt = u * Z;
          const unsigned long long cross = __ballot(tgt < incl);
          int tok;
          if (cross != 0ull) {
            const int L = __ffsll((long long)cross) - 1;
            float run = incl - ls;
            tok = lane * TL::VPL + TL::VPL - 1;
            bool found = false;
#pragma unroll
            for (int q = 0; q < TL::VPL; ++q) {
              run += vals[q];
              if (!found && tgt < run) { tok = lane * TL::VPL + q; found = true; }
            }
            if (lane == L) a.drafts[di] = tok;
          } else {
            // rounding left u*Z >= total: the last token with positive mass
            int last = -1;
#pragma unroll
            for (int q = 0; q < TL::VPL; ++q)
              if (vals[q] > 0.f) last = lane * TL::VPL + q;
            const unsigned long long pos = __ballot(last >= 0);
            const int L = 63 - __clzll((long long)pos);
            if (lane == L) a.drafts[di] = last;
          }
        }
      }
      __syncthreads();
    }
  }
}

// Univariate marginals (App. B.1 with every other variable summed out):
//   M[b,i,a] = log sum_j m[b,i,j] phi[b,i,j,a],  m = marginal of the latent that
// indexes leaf i.  One workgroup owns window position i for a tile of positions
// and walks the r slabs, adding exp(l - LSE_j + log m_j) into a second register
// tile, so each slab's logits are again consumed in registers.
template <int WV, int WB, int VB, int PB, bool BF16>
__global__ __launch_bounds__(WV * WB * 64)
void k_univariate(const UnivariateArgs a) {
  using TL = Tile<WV, WB, VB, PB>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int l31 = lane & 31, lhalf = lane >> 5;
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  const int wi = blockIdx.x / nbt, bt = blockIdx.x - wi * nbt;
  const int b0 = bt * TL::TP;
  const int rbase = wv * VB * 32 + 4 * lhalf;

  f32x16_t run[PB][VB];
#pragma unroll
  for (int pb = 0; pb < PB; ++pb)
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) run[pb][vb][i] = 0.f;

  for (int j = 0; j < a.r; ++j) {
    f32x16_t acc[PB][VB];
    tile_gemm<WV, WB, VB, PB, BF16>(a.W, a.h, a.ld_h, a.B, a.d, a.v, wi * a.r + j, b0, smem, acc);
    float mx[PB], lse[PB];
    tile_lse<WV, WB, VB, PB>(acc, a.v, (float2*)(smem + TL::RED_OFF), mx, lse);
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const int b = min(b0 + wb * PB * 32 + pb * 32 + l31, a.B - 1);
      const float lm = a.logm ? a.logm[((long long)b * a.n + wi) * a.r + j] : 0.f;
      const float shift = lm - lse[pb];
#pragma unroll
      for (int vb = 0; vb < VB; ++vb)
#pragma unroll
        for (int i = 0; i < 16; ++i) run[pb][vb][i] += __expf(acc[pb][vb][i] + shift);
    }
    __syncthreads();   // `red` is rewritten by the next slab
  }
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    const int b = b0 + wb * PB * 32 + pb * 32 + l31;
    if (b >= a.B) continue;
    float* dst = a.out + ((long long)b * a.n + wi) * a.v;
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = rbase + vb * 32 + 8 * (i >> 2) + (i & 3);
        if (row < a.v) dst[row] = __logf(run[pb][vb][i]);
      }
  }
}

template <int WV, int WB, int VB, int PB, bool BF16>
static hipError_t launch_uni_cfg(const UnivariateArgs& a, hipStream_t st) {
  using TL = Tile<WV, WB, VB, PB>;
  auto kern = k_univariate<WV, WB, VB, PB, BF16>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       TL::SMEM);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  hipLaunchKernelGGL(kern, dim3(nbt * a.n), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

hipError_t launch_univariate(const UnivariateArgs& a, int dtype, hipStream_t st) {
  const bool bf = dtype == MTPC_BF16;
  if (a.B > 32) {
    if (a.v > 256) return bf ? launch_uni_cfg<2, 4, 5, 1, true>(a, st) : launch_uni_cfg<2, 4, 5, 1, false>(a, st);
    if (a.v > 128) return bf ? launch_uni_cfg<2, 4, 4, 1, true>(a, st) : launch_uni_cfg<2, 4, 4, 1, false>(a, st);
    return bf ? launch_uni_cfg<2, 4, 2, 1, true>(a, st) : launch_uni_cfg<2, 4, 2, 1, false>(a, st);
  }
  if (a.v > 256) return bf ? launch_uni_cfg<5, 1, 2, 1, true>(a, st) : launch_uni_cfg<5, 1, 2, 1, false>(a, st);
  if (a.v > 128) return bf ? launch_uni_cfg<4, 1, 2, 1, true>(a, st) : launch_uni_cfg<4, 1, 2, 1, false>(a, st);
  return bf ? launch_uni_cfg<2, 1, 2, 1, true>(a, st) : launch_uni_cfg<2, 1, 2, 1, false>(a, st);
}

template <int WV, int WB, int VB, int PB, bool BF16, bool SAMPLE>
static hipError_t launch_cfg(const UnembedArgs& a, hipStream_t st) {
  using TL = Tile<WV, WB, VB, PB>;
  auto kern = k_unembed<WV, WB, VB, PB, BF16, SAMPLE>;
  static bool attr_done = false;   // raising the dynamic LDS limit is idempotent
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       TL::SMEM);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  const int grid = nbt * a.n * a.r;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

template <bool BF16, bool SAMPLE>
static hipError_t launch_dt(const UnembedArgs& a, hipStream_t st) {
  // Vocabulary tile: 5 blocks of 32 per wave pair covers v <= 320; v <= 256 and
  // v <= 128 take narrower tiles.  Positions: 256-wide tiles for training-sized
  // batches, 64- or 32-wide tiles (W streamed once) for decode-sized ones.
  if (a.B > 64) {
    if (a.v > 256) return launch_cfg<2, 4, 5, 2, BF16, SAMPLE>(a, st);
    if (a.v > 128) return launch_cfg<2, 4, 4, 2, BF16, SAMPLE>(a, st);
    return launch_cfg<2, 4, 2, 2, BF16, SAMPLE>(a, st);
  }
  if (a.B > 32) {
    if (a.v > 256) return launch_cfg<5, 1, 2, 2, BF16, SAMPLE>(a, st);
    if (a.v > 128) return launch_cfg<4, 1, 2, 2, BF16, SAMPLE>(a, st);
    return launch_cfg<2, 1, 2, 2, BF16, SAMPLE>(a, st);
  }
  if (a.v > 256) return launch_cfg<5, 1, 2, 1, BF16, SAMPLE>(a, st);
  if (a.v > 128) return launch_cfg<4, 1, 2, 1, BF16, SAMPLE>(a, st);
  return launch_cfg<2, 1, 2, 1, BF16, SAMPLE>(a, st);
}

hipError_t launch_unembed(const UnembedArgs& a, int dtype, hipStream_t st) {
  const bool sample = a.zleaf != nullptr;
  if (dtype == MTPC_BF16)
    return sample ? launch_dt<true, true>(a, st) : launch_dt<true, false>(a, st);
  return sample ? launch_dt<false, true>(a, st) : launch_dt<false, false>(a, st);
}

}  // namespace mtpc
