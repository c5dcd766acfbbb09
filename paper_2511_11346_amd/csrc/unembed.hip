// Fused unembedding kernel of the MtPC head for gfx950 (Sec. 3.3):
//   l[b,i,j,:] = W[i,j] h[b]   (MFMA, fp32 accumulate)
//   LSE over the vocabulary in registers, then either the evidence
//   e[b,i,j] = l[x] - LSE at the target token or an inverse-CDF token draw.
// The (B, n, r, v) logits live only in accumulator registers.
//
// Tiling.  One workgroup computes D = W_slab (v rows) x h_tile^T (TP positions):
// the vocabulary is the MFMA M dimension, positions the N dimension, so that the
// accumulator block of a lane holds 16 (32x32 MFMA) or 4 (16x16) vocabulary rows of ONE
// position and the softmax reduction is almost entirely lane-local.  Wave grid WV (vocab)
// x WB (positions); a wave owns VB x PB blocks of 32x32 (see Frag for the two layouts).
// K is consumed in stages of SB bytes per row (SB = 64 or 128).  Both operand
// tiles go from global memory straight into LDS (buffer_load_dwordx4 ... lds) through
// a ring of NS stages with unpadded, XOR-swizzled rows; fragments are read with
// conflict-free 16-byte LDS loads one half-step ahead of the MFMAs using them.
#include "tile.h"

namespace mtpc {

// ---- token draws on a finished tile -------------------------------------------------------
// A wave holds exp(l - max) of one position in vocabulary order, VPL consecutive tokens per
// lane (`vals`), `ls` their sum, `incl` the inclusive scan of ls over lanes, Z the total.
// Inverse CDF (Alg. 1): the smallest k with u * Z < cdf[k]; if rounding leaves u * Z >= Z,
// the last token with positive mass.  Returns the token in the lane for which `writer` is set.
template <int VPL>
__device__ __forceinline__ int wave_draw_token(const float (&vals)[VPL], float ls, float incl, float Z, float u,
                                               int lane, bool& writer) {
  const float tgt = u * Z;
  const unsigned long long cross = __ballot(tgt < incl);
  if (cross != 0ull) {
    const int L = __ffsll((long long)cross) - 1;
    float run = incl - ls;
    int tok = lane * VPL + VPL - 1;
    bool found = false;
#pragma unroll
    for (int q = 0; q < VPL; ++q) {
      run += vals[q];
      if (!found && tgt < run) { tok = lane * VPL + q; found = true; }
    }
    writer = lane == L;
    return tok;
  }
  int last = -1;
#pragma unroll
  for (int q = 0; q < VPL; ++q)
    if (vals[q] > 0.f) last = lane * VPL + q;
  const unsigned long long pos = __ballot(last >= 0);
  writer = lane == 63 - __clzll((long long)pos);
  return last;
}

// the most likely token of the position a wave holds (ties: the smallest id); all lanes get it
template <int VPL>
__device__ __forceinline__ int wave_argmax_token(const float (&vals)[VPL], int lane) {
  float best = -1.f;
  int arg = 0;
#pragma unroll
  for (int q = 0; q < VPL; ++q)
    if (vals[q] > best) { best = vals[q]; arg = lane * VPL + q; }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float ob = __shfl_xor(best, o);
    const int oa = __shfl_xor(arg, o);
    if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
  }
  return arg;
}

// Draw stage of a tile whose LSE statistics are known.  The tile-local positions that draw
// are listed in LDS (s_list[0..cnt), written before the preceding barrier).  NSL positions
// at a time: their accumulator columns are dumped as exp(l - max) in vocabulary order into
// the (now free) stage buffers, then one wave per position scans its row and calls
// body(p, vals, ls, incl, Z).
template <class TL, int VB, int PB, int NSL, bool M16, class Body>
__device__ __forceinline__ void tile_draws(const typename Frag<M16>::blk_t (&acc)[PB * Frag<M16>::SUB][VB * Frag<M16>::SUB],
                                           const float (&mx)[PB * Frag<M16>::SUB], int v, char* smem, int cnt, Body body) {
  using FR = Frag<M16>;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave % (TL::TV / (VB * 32)), wb = wave / (TL::TV / (VB * 32));
  const int lcol = FR::lcol(lane);
  const int rbase = wv * VB * 32 + 4 * FR::lgrp(lane);
  int* s_list = (int*)(smem + TL::MISC_OFF) + 4;
  int* s_slot = s_list + TL::TP;
  float* probs = (float*)smem;
  constexpr int SLOT = TL::VPL * 64 + 1;     // odd stride: the lanes of a wave dump different slots into different banks
  static_assert(NSL * SLOT * 4 <= TL::RED_OFF, "draw buffer must fit in the stage buffers");
  for (int c0 = 0; c0 < cnt; c0 += NSL) {
    const int nsl = min(NSL, cnt - c0);
    for (int p = tid; p < TL::TP; p += TL::NT) s_slot[p] = -1;
    __syncthreads();
    if (tid < nsl) s_slot[s_list[c0 + tid]] = tid;
    __syncthreads();
#pragma unroll
    for (int pb = 0; pb < PB * FR::SUB; ++pb) {
      const int sl = s_slot[wb * PB * 32 + pb * FR::BR + lcol];
      if (sl >= 0) {
#pragma unroll
        for (int vb = 0; vb < VB * FR::SUB; ++vb)
#pragma unroll
          for (int i = 0; i < FR::NI; ++i) {
            const int row = rbase + vb * FR::BR + FR::roff(i);
            probs[sl * SLOT + row] = (row < v) ? expf(acc[pb][vb][i] - mx[pb]) : 0.f;
          }
      }
    }
    __syncthreads();
    for (int k = wave; k < nsl; k += TL::NW) {
      float vals[TL::VPL];
      float ls = 0.f;
#pragma unroll
      for (int q = 0; q < TL::VPL; ++q) {
        vals[q] = probs[k * SLOT + lane * TL::VPL + q];
        ls += vals[q];
      }
      float incl = ls;   // inclusive scan over lanes
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const float t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
      }
      const float Z = __shfl(incl, 63);
      body(s_list[c0 + k], vals, ls, incl, Z);
    }
    __syncthreads();
  }
}

// Draws for every position column of a tile at once, from the accumulators (16x16 blocks): one token per
// column p with need(p), by inverse CDF (Alg. 1: the smallest token k with u Z < cdf[k]; the last token with
// positive mass if rounding leaves u Z >= Z) or, greedy, the most likely token (ties: the smallest id).
// A column's v values lie in 4 lane groups x VB*2 blocks x WV waves; each lane forms the prefix of its own
// rows (sums over the lane groups by lane permutes, over the blocks in registers, over the waves through
// LDS) and looks for the crossing among its rows; the smallest crossing row of a column wins (LDS minimum).
// Three workgroup barriers per call, all waves busy, nothing dumped to LDS but one sum per column and wave.
// Wide wave tiles (more than three blocks of columns) form the terms of a block a second time after the
// barrier instead of keeping those of all blocks in registers.
// The stage buffers must be free.  uni(p) gives the uniform of column p, out(p, token) takes the result.
template <class TL, int WV, int VB, int NPB, class Need, class Uni, class Out>
__device__ __forceinline__ void tile_draws_cols(const f32x4_t (&acc)[NPB][VB * 2], const float (&mx)[NPB], int v,
                                                char* smem, bool greedy, Need need, Uni uni, Out out) {
  constexpr int NVB = VB * 2;
  constexpr bool KEEP = NPB <= 3;
  constexpr int NK = KEEP ? NPB : 1;
  static_assert(NPB * 16 == TL::WP, "the wave's blocks of 16 position columns");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int lcol = lane & 15, lgrp = lane >> 4;
  const int rbase = wv * VB * 32 + 4 * lgrp;
  float* wsum = (float*)smem;                                        // [WV][TP] sum of a wave's rows of a column
  int* cand = (int*)(wsum + WV * TL::TP);                            // [TP] smallest crossing row
  int* lastp = cand + TL::TP;                                        // [TP] last row with positive mass
  unsigned long long* best = (unsigned long long*)(lastp + TL::TP);  // [TP] greedy: (value, -row)
  static_assert((WV + 2) * TL::TP * 4 + TL::TP * 8 <= TL::RED_OFF, "fits in the stage buffers");
  for (int p = tid; p < TL::TP; p += TL::NT) {
    cand[p] = 0x7fffffff;
    lastp[p] = -1;
    best[p] = 0ull;
  }
  // the terms of block pb: e = exp(l - max) of this lane's rows, ex = what the lane groups below this one
  // hold of a block of 16 rows, tot = the block's sum; returns the sum of the wave's rows of the column
  auto terms = [&](int pb, float (&e)[NVB][4], float (&ex)[NVB], float (&tot)[NVB]) {
    float colsum = 0.f;
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb) {
#pragma unroll
      for (int t = 0; t < 4; ++t) e[vb][t] = (rbase + vb * 16 + t < v) ? expf(acc[pb][vb][t] - mx[pb]) : 0.f;
      const float s4 = ((e[vb][0] + e[vb][1]) + e[vb][2]) + e[vb][3];
      // inclusive scan over the four lane groups that hold this column (lanes lcol + 16 g)
      const float u1 = __shfl_up(s4, 16);
      const float i1 = lgrp >= 1 ? s4 + u1 : s4;
      const float u2 = __shfl_up(i1, 32);
      const float incl = lgrp >= 2 ? i1 + u2 : i1;
      ex[vb] = incl - s4;
      tot[vb] = __shfl(incl, 48 + lcol);
      colsum += tot[vb];
    }
    return colsum;
  };
  float e[NK][NVB][4], ex[NK][NVB], tot[NK][NVB];
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb) {
    const float colsum = terms(pb, e[KEEP ? pb : 0], ex[KEEP ? pb : 0], tot[KEEP ? pb : 0]);
    if (lgrp == 0) wsum[wv * TL::TP + wb * TL::WP + pb * 16 + lcol] = colsum;
  }
  __syncthreads();
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb) {
    const int col = wb * TL::WP + pb * 16 + lcol;
    constexpr int k0 = 0;
    const int k = KEEP ? pb : k0;
    if constexpr (!KEEP) (void)terms(pb, e[0], ex[0], tot[0]);
    if (greedy) {
      float bv = -1.f;
      int br = 0;
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int t = 0; t < 4; ++t)
          if (e[k][vb][t] > bv) { bv = e[k][vb][t]; br = rbase + vb * 16 + t; }
      atomicMax(&best[col], ((unsigned long long)__float_as_uint(bv) << 32) | (unsigned)(0x7fffffff - br));
    } else {
      float below = 0.f, Z = 0.f;
#pragma unroll
      for (int w = 0; w < WV; ++w) {
        const float x = wsum[w * TL::TP + col];
        if (w < wv) below += x;
        Z += x;
      }
      const float tgt = uni(col) * Z;
      float run = below;
      int first = 0x7fffffff, last = -1;
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb) {
        float c = run + ex[k][vb];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          c += e[k][vb][t];
          const int row = rbase + vb * 16 + t;
          if (tgt < c) first = min(first, row);
          if (e[k][vb][t] > 0.f) last = row;
        }
        run += tot[k][vb];
      }
      if (first != 0x7fffffff) atomicMin(&cand[col], first);
      atomicMax(&lastp[col], last);
    }
  }
  __syncthreads();
  if (wv == 0 && lgrp == 0) {
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) {
      const int col = wb * TL::WP + pb * 16 + lcol;
      if (need(col)) {
        int tok;
        if (greedy) tok = 0x7fffffff - (int)(unsigned)(best[col] & 0xffffffffull);
        else tok = cand[col] != 0x7fffffff ? cand[col] : lastp[col];
        out(col, tok);
      }
    }
  }
  __syncthreads();
}

// Which instantiations of k_unembed walk several tiles per workgroup: the ones whose epilogue leaves the
// ring alone (no draws) on the tiles of training-sized batches.
template <int WB, bool SAMPLE>
constexpr bool unembed_walks_tiles() { return !SAMPLE && WB != 1; }

template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16, bool SAMPLE, bool WPACK = false>
__global__ __launch_bounds__(WV * WB * 64)
void k_unembed(const UnembedArgs a) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr bool M16 = use_m16<WV, WB, SB, NS, BF16>();
  using FR = Frag<M16>;
  constexpr int NPB = PB * FR::SUB, NVB = VB * FR::SUB;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int lcol = FR::lcol(lane), lgrp = FR::lgrp(lane);
  const int nslab = a.n * a.r;
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  // The evidence kernel of a training-sized batch is launched with one workgroup per CU (unembed_walks_tiles):
  // a workgroup walks the tiles blockIdx.x, blockIdx.x + gridDim.x, ... (the grid is a multiple of the number
  // of XCDs, so all of them lie in this XCD's range of logical tiles) and opens the feed of the next tile
  // before the epilogue of the one it has multiplied: the first stages of the next ring arrive while the
  // softmax statistics are taken, instead of after a workgroup launch with the matrix pipe idle.
  // Every other instantiation has one tile per workgroup and leaves the loop after it.
  constexpr bool WALK = unembed_walks_tiles<WB, SAMPLE>();
  using Feed = TileFeed<WV, WB, VB, PB, SB, NS, BF16, false, M16, WPACK, WB == 1>;
  const void* const hstaged = (WB != 1 && SB == H_STAGE_BYTES) ? a.hs : nullptr;
  const int ntiles = nbt * nslab;
  int slab, bt;
  tile_of_block(blockIdx.x, nbt, nslab, slab, bt);
  Feed feed;
  // the decode-sized tiles (one wave column) are launched with one tile of positions: W is a stream
  feed.open(WPACK ? a.Wp : a.W, a.d, a.h, a.ld_h, a.B, a.d, a.v, slab, bt * TL::TP, smem, nullptr, 0, 1, hstaged);
  for (int w = blockIdx.x;;) {
  const int b0 = bt * TL::TP;
  const int wi = slab / a.r, wj = slab - wi * a.r;

  // Target tokens of the tile's positions, first XW windows of each: fetched now, while nothing
  // depends on them, parked in LDS after the product (the list / slot area the draws use, idle
  // in this instantiation).  Read in the epilogue they would be one dependent memory round
  // trip per position column and window, with the matrix pipe idle.
  constexpr int XW = 2, XR = (XW * TL::TP + TL::NT - 1) / TL::NT;
  int* s_x = (int*)(smem + TL::MISC_OFF) + 4;        // [XW][TP]
  int xpre[XR];
  int nxw = 0;
  if constexpr (!SAMPLE) if (a.targets != nullptr) {
    nxw = min(a.T + a.T2, XW);
#pragma unroll
    for (int q = 0; q < XR; ++q) {
      const int idx = tid + q * TL::NT, t = idx / TL::TP, p = idx - t * TL::TP;
      const long long b = b0 + p;
      xpre[q] = -1;
      if (t < nxw && b < a.B)
        xpre[q] = t < a.T ? a.targets[(b * a.T + t) * a.n + wi] : a.targets2[(b * a.T2 + (t - a.T)) * a.n + wi];
    }
  }

  typename FR::blk_t acc[NPB][NVB];
  tile_gemm_run(feed, a.d, smem, acc);
  const int wnext = w + (int)gridDim.x;
  int slab_next = 0, bt_next = 0;
  if constexpr (WALK)
    if (wnext < ntiles) {
      tile_of_block(wnext, nbt, nslab, slab_next, bt_next);
      feed.open(WPACK ? a.Wp : a.W, a.d, a.h, a.ld_h, a.B, a.d, a.v, slab_next, bt_next * TL::TP, smem, nullptr, 0, 1, hstaged);
    }

  if constexpr (!SAMPLE) if (a.targets != nullptr) {
#pragma unroll
    for (int q = 0; q < XR; ++q) {
      const int idx = tid + q * TL::NT;
      if (idx < nxw * TL::TP) s_x[idx] = xpre[q];
    }
  }
  // this lane holds, of position column wb*PB*32 + pb*BR + lcol, rows rbase + vb*BR + roff(i)
  const int rbase = wv * VB * 32 + 4 * lgrp;
  float mx[NPB], lse[NPB];
  tile_lse<WV, WB, VB, PB, SB, NS, M16>(acc, a.v, (float2*)(smem + TL::RED_OFF), mx, lse);   // (one barrier: s_x is visible)

  // evidence at the target tokens (the sampling instantiation never has targets)
  if constexpr (!SAMPLE) if (a.targets != nullptr) {
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) {
      const int b = b0 + wb * PB * 32 + pb * FR::BR + lcol;
      if (b < a.B) {
        const int TT = a.T + a.T2;
        for (int t = 0; t < TT; ++t) {
          const long long rowid = (long long)b * TT + t;
          const int x = t < XW ? s_x[t * TL::TP + (b - b0)]
                        : t < a.T ? a.targets[((long long)b * a.T + t) * a.n + wi]
                                  : a.targets2[((long long)b * a.T2 + (t - a.T)) * a.n + wi];
          float* dst = a.e + (rowid * a.n + wi) * a.r + wj;
          if (x < 0 || x >= a.v) {
            if (wv == 0 && lgrp == 0) *dst = (x == -1) ? 0.f : __builtin_nanf("");
          } else {
            // first the block of the target row, then its register by the bits of the offset
            // (a few dozen selects instead of a compare and a select for every register)
            const int xr = x - rbase;
            if constexpr (M16) {
              // rows rbase + 16 vb + t (t in 0..3)
              if (xr >= 0 && xr < VB * 32 && (xr & 12) == 0) {
                const int xvb = xr >> 4;
                f32x4_t blk = acc[pb][0];
#pragma unroll
                for (int vb = 1; vb < NVB; ++vb) blk = (xvb == vb) ? acc[pb][vb] : blk;
                const bool t0 = xr & 1, t1 = xr & 2;
                const float c0 = t0 ? blk[1] : blk[0], c1 = t0 ? blk[3] : blk[2];
                *dst = (t1 ? c1 : c0) - lse[pb];
              }
            } else {
              // rows rbase + 32 vb + 8 q + t (q, t in 0..3)
              if (xr >= 0 && xr < VB * 32 && (xr & 4) == 0) {
                const int xvb = xr >> 5;
                f32x16_t blk = acc[pb][0];
#pragma unroll
                for (int vb = 1; vb < VB; ++vb) blk = (xvb == vb) ? acc[pb][vb] : blk;
                const bool t0 = xr & 1, t1 = xr & 2, q0 = xr & 8, q1 = xr & 16;
                const float b0 = t0 ? blk[1] : blk[0], b1 = t0 ? blk[3] : blk[2];
                const float b2 = t0 ? blk[5] : blk[4], b3 = t0 ? blk[7] : blk[6];
                const float b4 = t0 ? blk[9] : blk[8], b5 = t0 ? blk[11] : blk[10];
                const float b6 = t0 ? blk[13] : blk[12], b7 = t0 ? blk[15] : blk[14];
                const float c0 = t1 ? b1 : b0, c1 = t1 ? b3 : b2, c2 = t1 ? b5 : b4, c3 = t1 ? b7 : b6;
                const float lo = q0 ? c1 : c0, hi = q0 ? c3 : c2;
                *dst = (q1 ? hi : lo) - lse[pb];
              }
            }
          }
        }
      }
    }
  }
  if constexpr (!SAMPLE) if (a.phiT != nullptr) {
    // keep the normalised probabilities for the training step (transposed: positions contiguous;
    // the column blocks of a row are stored back to back, together they fill whole lines).
    // phi = 2^((l - lse) log2 e): one fused multiply-add and one v_exp per probability
    constexpr float LOG2E = 1.4426950408889634f;
    const int bl = b0 + wb * PB * 32 + lcol;
    float* col = a.phiT + ((long long)slab * a.v + rbase) * a.ld_phi + bl;
    float shift[NPB];
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) shift[pb] = -lse[pb] * LOG2E;
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
      for (int i = 0; i < FR::NI; ++i) {
        const int off = vb * FR::BR + FR::roff(i);
        if (rbase + off >= a.v) continue;
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb)
          if (bl + pb * FR::BR < a.B)
            col[off * a.ld_phi + pb * FR::BR] = __builtin_amdgcn_exp2f(fmaf(acc[pb][vb][i], LOG2E, shift[pb]));
      }
  }
  if (a.logphi != nullptr) {
    // table log phi[b][wi][wj][:] for the scoring and verification steps.  Registers
    // 4q..4q+3 of a block hold four consecutive vocabulary rows of one position: one
    // 16-byte store each (the row of a position is 4v bytes long and 16-byte aligned
    // when v is a multiple of 4; otherwise element by element)
    const bool vec = (a.v & 3) == 0;
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) {
      const int b = b0 + wb * PB * 32 + pb * FR::BR + lcol;
      if (b >= a.B) continue;
      float* dst = a.logphi + (((long long)b * a.n + wi) * a.r + wj) * a.v;
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int q = 0; q < FR::NI / 4; ++q) {
          const int row = rbase + vb * FR::BR + FR::roff(4 * q);
          if (vec) {
            if (row < a.v)
              *(f32x4_t*)(dst + row) = f32x4_t{acc[pb][vb][4 * q] - lse[pb], acc[pb][vb][4 * q + 1] - lse[pb],
                                               acc[pb][vb][4 * q + 2] - lse[pb], acc[pb][vb][4 * q + 3] - lse[pb]};
          } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
              if (row + t < a.v) dst[row + t] = acc[pb][vb][4 * q + t] - lse[pb];
          }
        }
    }
  }
  if constexpr (SAMPLE && M16 && WB != 1) {
    // training-sized tiles: the tokens of all columns at once, one pass per draft (only tiles in which some
    // position draws token wi of that draft from component wj)
    if (a.zleaf == nullptr) return;
    for (int s = 0; s < a.S; ++s) {
      auto need = [&](int p) {
        const long long b = b0 + p;
        return b < a.B && a.zleaf[(b * a.S + s) * a.n + wi] == wj;
      };
      bool any = false;
      for (int p = tid; p < TL::TP; p += TL::NT) any |= need(p);
      if (!__syncthreads_or(any)) continue;
      tile_draws_cols<TL, WV, VB, NPB>(
          acc, mx, a.v, smem, a.greedy != 0, need,
          [&](int p) { return philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)(b0 + p), (uint32_t)s, (uint32_t)wi); },
          [&](int p, int tok) { a.drafts[((long long)(b0 + p) * a.S + s) * a.n + wi] = tok; });
    }
  } else if constexpr (SAMPLE) {
    if (a.zleaf == nullptr) return;
    // ---- which positions of this tile draw token wi from component wj?
    int* misc = (int*)(smem + TL::MISC_OFF);
    int* s_cnt = misc;
    int* s_list = misc + 4;
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
    tile_draws<TL, VB, PB, NSLOT, M16>(acc, mx, a.v, smem, cnt, [&](int p, const float (&vals)[TL::VPL], float ls, float incl,
                                                        float Z) {
      const int b = b0 + p;
      for (int s = 0; s < a.S; ++s) {
        const long long di = ((long long)b * a.S + s) * a.n + wi;
        if (a.zleaf[di] != wj) continue;
        int tok;
        bool writer;
        if (a.greedy) {
          tok = wave_argmax_token<TL::VPL>(vals, lane);
          writer = lane == 0;
        } else {
          const float u = philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, (uint32_t)s, (uint32_t)wi);
          tok = wave_draw_token<TL::VPL>(vals, ls, incl, Z, u, lane, writer);
        }
        if (writer) a.drafts[di] = tok;
      }
    });
  }
  if (!WALK || wnext >= ntiles) break;
  w = wnext;
  slab = slab_next;
  bt = bt_next;
  }
}

// stage geometry of the gathered draw tiles and the positions drawn per pass of their draw loop
constexpr int GATHER_SB = GATHER_STAGE_BYTES, GATHER_NS = 4, GATHER_NSL = 16;
// Token draws of Alg. 1 for training-sized batches: only the input unit a token is drawn
// from is evaluated.  The (b, s, i) triples were bucketed by (i, z) = (token, selected
// unit); a workgroup takes up to TP rows of one bucket, gathers their h rows, multiplies
// them with the one slab W[i][z] and draws every row's token - 1/r of the products a
// pass over all slabs needs.
template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16, bool WPACK, int PH>
__global__ __launch_bounds__(WV * WB * 64)
void k_draw_gather(const DrawGatherArgs a) {
  using TL = Tile<WV, WB, VB, PB, SB, NS, PH>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  // each XCD owns a contiguous range of logical tiles, so that the tiles of a bucket
  // (which share a W slab) run under one L2
  // (the grid is an upper bound; the ranges are cut from the number of tiles there are, so that
  // every XCD gets its share of them)
  const int ngroups = a.n * a.r;
  const int total = a.tile_off[ngroups];
  const int w = blockIdx.x;
  if (w >= total) return;
  const int per = total >> 3;
  const int lid = (w < per * 8) ? (w & 7) * per + (w >> 3) : w;
  const int g = a.tile_bucket[lid];                  // tile_off[g] <= lid < tile_off[g+1]
  const int first = a.row_off[g] + (lid - a.tile_off[g]) * TL::TP;
  const int nrows = min(a.row_off[g + 1] - first, TL::TP);     // >= 1 by construction of tile_off
  const int* rows = a.list + first;
  const int wi = g / a.r;

  constexpr bool M16 = use_m16<WV, WB, SB, NS, BF16>();
  constexpr int NPB = PB * Frag<M16>::SUB + PH;
  typename Frag<M16>::blk_t acc[NPB][VB * Frag<M16>::SUB];
  tile_gemm<WV, WB, VB, PB, SB, NS, BF16, true, M16, WPACK, false, PH>(WPACK ? a.Wp : a.W, a.d, a.h, a.ld_h, a.B, a.d, a.v, g, 0, smem,
                                                                       acc, rows, nrows, a.S);
  float mx[NPB], lse[NPB];
  tile_lse<WV, WB, VB, PB, SB, NS, M16, PH>(acc, a.v, (float2*)(smem + TL::RED_OFF), mx, lse);

  if constexpr (M16) {
    const int S = a.S;
    tile_draws_cols<TL, WV, VB, NPB>(
        acc, mx, a.v, smem, a.greedy != 0, [&](int p) { return p < nrows; },
        [&](int p) {
          const int rid = rows[min(p, nrows - 1)];       // b * S + s
          const int b = rid / S, sd = rid - b * S;
          return philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, (uint32_t)sd, (uint32_t)wi);
        },
        [&](int p, int tok) { a.drafts[(long long)rows[p] * a.n + wi] = tok; });
  } else {
    int* s_list = (int*)(smem + TL::MISC_OFF) + 4;
    for (int p = tid; p < nrows; p += TL::NT) s_list[p] = p;
    __syncthreads();
    tile_draws<TL, VB, PB, GATHER_NSL, M16>(acc, mx, a.v, smem, nrows, [&](int p, const float (&vals)[TL::VPL], float ls,
                                                                           float incl, float Z) {
      const int rid = rows[p];                         // b * S + s
      const int b = rid / a.S, s = rid - b * a.S;
      int tok;
      bool writer;
      if (a.greedy) {
        tok = wave_argmax_token<TL::VPL>(vals, lane);
        writer = lane == 0;
      } else {
        const float u = philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, (uint32_t)s, (uint32_t)wi);
        tok = wave_draw_token<TL::VPL>(vals, ls, incl, Z, u, lane, writer);
      }
      if (writer) a.drafts[(long long)rid * a.n + wi] = tok;
    });
  }
}

template <int WV, int WB, int VB, int PB, int PH, bool BF16, bool WPACK = false>
static hipError_t launch_draw_gather_cfg(const DrawGatherArgs& a, hipStream_t st) {
  using TL = Tile<WV, WB, VB, PB, GATHER_SB, GATHER_NS, PH>;
  static_assert(TL::TP == DRAW_GATHER_TILE || TL::TP == DRAW_GATHER_TILE_WIDE, "the tile heights the bucketing is run with");
  if constexpr (!WPACK)
    if (a.Wp != nullptr) return launch_draw_gather_cfg<WV, WB, VB, PB, PH, BF16, true>(a, st);
  constexpr auto kern = k_draw_gather<WV, WB, VB, PB, GATHER_SB, GATHER_NS, BF16, WPACK, PH>;
  if (hipError_t e = allow_lds<kern>(TL::SMEM); e != hipSuccess) return e;
  const long long rows = (long long)a.B * a.S * a.n;
  const int grid = (int)(rows / TL::TP) + a.n * a.r;             // >= sum over buckets of ceil(rows_g / TP)
  hipLaunchKernelGGL(kern, dim3(grid), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

template <bool BF16>
static hipError_t launch_draw_gather_dt(const DrawGatherArgs& a, hipStream_t st) {
  if constexpr (BF16)                                // (the wide tile counts its columns in blocks of 16)
    if (a.tile == DRAW_GATHER_TILE_WIDE) {
      if (a.v > 256) return launch_draw_gather_cfg<2, 4, 5, 1, 1, BF16>(a, st);
      if (a.v > 128) return launch_draw_gather_cfg<2, 4, 4, 1, 1, BF16>(a, st);
      return launch_draw_gather_cfg<2, 4, 2, 1, 1, BF16>(a, st);
    }
  if (a.tile != DRAW_GATHER_TILE) return hipErrorInvalidValue;
  if (a.v > 256) return launch_draw_gather_cfg<2, 4, 5, 1, 0, BF16>(a, st);
  if (a.v > 128) return launch_draw_gather_cfg<2, 4, 4, 1, 0, BF16>(a, st);
  return launch_draw_gather_cfg<2, 4, 2, 1, 0, BF16>(a, st);
}

hipError_t launch_draw_gather(const DrawGatherArgs& a, int dtype, hipStream_t st) {
  return dtype == MTPC_BF16 ? launch_draw_gather_dt<true>(a, st) : launch_draw_gather_dt<false>(a, st);
}

// Sum-unit parameters for many positions (Sec. 3.3): log omega[b,:] =
// log_softmax(Wsum h[b]).  Same tile machinery with Wsum as the only "slab" (r rows)
// and narrow position tiles, so that B/32 workgroups share the work.
template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16>
__global__ __launch_bounds__(WV * WB * 64)
void k_sumunit_mfma(const void* h, long long ld_h, const void* Wsum, int B, int d, int r, float* logw) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int l31 = lane & 31, lhalf = lane >> 5;
  const int b0 = blockIdx.x * TL::TP;
  f32x16_t acc[PB][VB];
  tile_gemm<WV, WB, VB, PB, SB, NS, BF16>(Wsum, d, h, ld_h, B, d, r, 0, b0, smem, acc);
  float mx[PB], lse[PB];
  tile_lse<WV, WB, VB, PB, SB, NS>(acc, r, (float2*)(smem + TL::RED_OFF), mx, lse);
  const int rbase = wv * VB * 32 + 4 * lhalf;
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    const int b = b0 + wb * PB * 32 + pb * 32 + l31;
    if (b >= B) continue;
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = rbase + vb * 32 + 8 * (i >> 2) + (i & 3);
        if (row < r) logw[(long long)b * r + row] = acc[pb][vb][i] - lse[pb];
      }
  }
}

template <int WV, int VB, int SB, int NS, bool BF16>
static hipError_t launch_sumunit_mfma_cfg(const void* h, long long ld_h, const void* Wsum, int B, int d,
                                          int r, float* logw, hipStream_t st) {
  using TL = Tile<WV, 1, VB, 1, SB, NS>;   // WV * VB * 32 rows (>= r) x 32 positions, WV waves
  constexpr auto kern = k_sumunit_mfma<WV, 1, VB, 1, SB, NS, BF16>;
  if (hipError_t e = allow_lds<kern>(TL::SMEM); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((B + TL::TP - 1) / TL::TP), dim3(TL::NT), TL::SMEM, st, h, ld_h, Wsum, B,
                     d, r, logw);
  return hipGetLastError();
}

// The kernel streams h once with one small workgroup per 32 positions, so what limits it is
// the number of bytes of h it keeps in flight: 128-byte stages when the rows allow it, no more
// rows of Wsum in a stage than r needs (they are loaded beside h), and the LDS that saves spent
// on a deeper ring.
template <bool BF16>
static hipError_t launch_sumunit_mfma_dt(const void* h, long long ld_h, const void* Wsum, int B, int d,
                                         int r, float* logw, hipStream_t st) {
  if ((d * (BF16 ? 2 : 4)) % 128 == 0) {
    if (r <= 32) return launch_sumunit_mfma_cfg<1, 1, 128, 8, BF16>(h, ld_h, Wsum, B, d, r, logw, st);
    if (r <= 64) return launch_sumunit_mfma_cfg<2, 1, 128, 6, BF16>(h, ld_h, Wsum, B, d, r, logw, st);
    return launch_sumunit_mfma_cfg<2, 2, 128, 4, BF16>(h, ld_h, Wsum, B, d, r, logw, st);
  }
  return launch_sumunit_mfma_cfg<2, 2, 64, 4, BF16>(h, ld_h, Wsum, B, d, r, logw, st);
}

hipError_t launch_sumunit_mfma(const void* h, long long ld_h, const void* Wsum, int B, int d, int r,
                               int dtype, float* logw, hipStream_t st) {
  return dtype == MTPC_BF16 ? launch_sumunit_mfma_dt<true>(h, ld_h, Wsum, B, d, r, logw, st)
                            : launch_sumunit_mfma_dt<false>(h, ld_h, Wsum, B, d, r, logw, st);
}

// Contextual sum layers (Sec. 3.3, sum unit parameters): every sum unit (layer l,
// incoming state k) of every position gets its own weights softmax(R[l][k] h[b] +
// bias[l][k]).  The tile machinery again: a "slab" is one sum unit (r rows of R).
template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16>
__global__ __launch_bounds__(WV * WB * 64)
void k_ctx_layers(const CtxLayerArgs a) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr int ESZ = BF16 ? 2 : 4;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int l31 = lane & 31, lhalf = lane >> 5;
  const int nslab = a.L * a.r;
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  int slab, bt;
  tile_of_block(blockIdx.x, nbt, nslab, slab, bt);
  const int b0 = bt * TL::TP;
  const int l = slab / a.r, k = slab - l * a.r;
  const char* Rlk = (const char*)a.R + ((long long)l * a.R_layer_stride + (long long)k * a.r * a.d) * ESZ;

  f32x16_t acc[PB][VB];
  tile_gemm<WV, WB, VB, PB, SB, NS, BF16>(Rlk, a.d, a.h, a.ld_h, a.B, a.d, a.r, 0, b0, smem, acc);
  const int rbase = wv * VB * 32 + 4 * lhalf;
  if (a.bias != nullptr) {
    const float* bl = a.bias + (long long)l * a.bias_layer_stride + (long long)k * a.r;
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = rbase + vb * 32 + 8 * (i >> 2) + (i & 3);
        const float bv = row < a.r ? bl[row] : 0.f;
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[pb][vb][i] += bv;
      }
  }
  float mx[PB], lse[PB];
  tile_lse<WV, WB, VB, PB, SB, NS>(acc, a.r, (float2*)(smem + TL::RED_OFF), mx, lse);
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    const int b = b0 + wb * PB * 32 + pb * 32 + l31;
    if (b >= a.B) continue;
    const long long base = ((long long)b * a.L + l) * a.r * a.r;
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = rbase + vb * 32 + 8 * (i >> 2) + (i & 3);
        if (row < a.r) {
          const float p = __expf(acc[pb][vb][i] - lse[pb]);
          if (a.out_nat) a.out_nat[base + (long long)k * a.r + row] = p;
          if (a.out_tr) a.out_tr[base + (long long)row * a.r + k] = p;
        }
      }
  }
}

// The same for r a power of two in 8..128 and natural layout only: R is taken as one
// dense [L*r*r][d] matrix cut into 256-row slabs, so no matrix-pipe row is wasted on
// padding.  A sum unit is an aligned run of r rows; in the accumulator layout those are
// whole 32-row blocks of one wave (r >= 32) or register groups of a block (r < 32) plus
// the partner lane 32 away, so its softmax needs one cross-lane exchange and no LDS.
template <int R, bool BF16>
__global__ __launch_bounds__(512)
void k_ctx_layers_dense(const CtxLayerArgs a) {
  constexpr int WV = 2, WB = 4, VB = 4, PB = 2, SB = 64, NS = 4;
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr int ESZ = BF16 ? 2 : 4;
  constexpr int UB = R >= 32 ? R / 32 : 1;          // blocks per unit
  constexpr int RG = R >= 32 ? 16 : R / 2;          // registers per unit within a block
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int l31 = lane & 31, lhalf = lane >> 5;
  const int Mr = a.L * a.r * a.r;
  const int nslab = (Mr + TL::TV - 1) / TL::TV;
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  int slab, bt;
  tile_of_block(blockIdx.x, nbt, nslab, slab, bt);
  const int b0 = bt * TL::TP;
  const int rows = min(TL::TV, Mr - slab * TL::TV);
  f32x16_t acc[PB][VB];
  tile_gemm<WV, WB, VB, PB, SB, NS, BF16>((const char*)a.R + (long long)slab * TL::TV * a.d * ESZ, a.d, a.h,
                                          a.ld_h, a.B, a.d, rows, 0, b0, smem, acc);
  const int rbase = wv * VB * 32 + 4 * lhalf;
  if (a.bias != nullptr) {
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = rbase + vb * 32 + 8 * (i >> 2) + (i & 3);
        const float bv = row < rows ? a.bias[(long long)slab * TL::TV + row] : 0.f;
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[pb][vb][i] += bv;
      }
  }
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    const int b = b0 + wb * PB * 32 + pb * 32 + l31;
#pragma unroll
    for (int vb0 = 0; vb0 < VB; vb0 += UB)
#pragma unroll
      for (int i0 = 0; i0 < 16; i0 += RG) {
        float m = neg_inf();
#pragma unroll
        for (int vb = vb0; vb < vb0 + UB; ++vb)
#pragma unroll
          for (int i = i0; i < i0 + RG; ++i) m = fmaxf(m, acc[pb][vb][i]);
        m = fmaxf(m, __shfl_xor(m, 32));
        float s = 0.f;
#pragma unroll
        for (int vb = vb0; vb < vb0 + UB; ++vb)
#pragma unroll
          for (int i = i0; i < i0 + RG; ++i) {
            acc[pb][vb][i] = __expf(acc[pb][vb][i] - m);
            s += acc[pb][vb][i];
          }
        s += __shfl_xor(s, 32);
        const float inv = 1.f / s;
#pragma unroll
        for (int vb = vb0; vb < vb0 + UB; ++vb)
#pragma unroll
          for (int i = i0; i < i0 + RG; ++i) acc[pb][vb][i] *= inv;
      }
    if (b < a.B) {
      float* dst = a.out_nat + (long long)b * Mr + (long long)slab * TL::TV;
#pragma unroll
      for (int vb = 0; vb < VB; ++vb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = rbase + vb * 32 + 8 * q;
          if (row < rows)
            *(f32x4_t*)(dst + row) = f32x4_t{acc[pb][vb][4 * q], acc[pb][vb][4 * q + 1], acc[pb][vb][4 * q + 2],
                                             acc[pb][vb][4 * q + 3]};
        }
    }
  }
}

template <int R, bool BF16>
static hipError_t launch_ctx_dense(const CtxLayerArgs& a, hipStream_t st) {
  using TL = Tile<2, 4, 4, 2, 64, 4>;
  constexpr auto kern = k_ctx_layers_dense<R, BF16>;
  if (hipError_t e = allow_lds<kern>(TL::SMEM); e != hipSuccess) return e;
  const int Mr = a.L * a.r * a.r;
  const int nbt = (a.B + TL::TP - 1) / TL::TP, nslab = (Mr + TL::TV - 1) / TL::TV;
  hipLaunchKernelGGL(kern, dim3(nbt * nslab), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

template <bool BF16>
static hipError_t launch_ctx_dense_dt(const CtxLayerArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_ctx_dense<8, BF16>(a, st);
    case 16: return launch_ctx_dense<16, BF16>(a, st);
    case 32: return launch_ctx_dense<32, BF16>(a, st);
    case 64: return launch_ctx_dense<64, BF16>(a, st);
    default: return launch_ctx_dense<128, BF16>(a, st);
  }
}

template <int WV, int WB, int VB, int PB, bool BF16>
static hipError_t launch_ctx_cfg(const CtxLayerArgs& a, hipStream_t st) {
  using TL = Tile<WV, WB, VB, PB, 64, 4>;
  constexpr auto kern = k_ctx_layers<WV, WB, VB, PB, 64, 4, BF16>;
  if (hipError_t e = allow_lds<kern>(TL::SMEM); e != hipSuccess) return e;
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  hipLaunchKernelGGL(kern, dim3(nbt * a.L * a.r), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

hipError_t launch_ctx_layers(const CtxLayerArgs& a, int dtype, hipStream_t st) {
  const bool bf = dtype == MTPC_BF16;
  const long long rr = (long long)a.r * a.r;
  const bool pow2 = a.r >= 8 && a.r <= 128 && (a.r & (a.r - 1)) == 0;
  const bool dense_R = a.L == 1 || a.R_layer_stride == rr * a.d;
  const bool dense_bias = a.bias == nullptr || a.L == 1 || a.bias_layer_stride == rr;
  if (a.B > 64 && pow2 && dense_R && dense_bias && a.out_nat != nullptr && a.out_tr == nullptr)
    return bf ? launch_ctx_dense_dt<true>(a, st) : launch_ctx_dense_dt<false>(a, st);
  if (a.B > 64) {     // 64- or 128-row unit tiles x 256 positions
    if (a.r > 64) return bf ? launch_ctx_cfg<2, 4, 2, 2, true>(a, st) : launch_ctx_cfg<2, 4, 2, 2, false>(a, st);
    return bf ? launch_ctx_cfg<2, 4, 1, 2, true>(a, st) : launch_ctx_cfg<2, 4, 1, 2, false>(a, st);
  }
  return bf ? launch_ctx_cfg<2, 1, 2, 2, true>(a, st) : launch_ctx_cfg<2, 1, 2, 2, false>(a, st);
}

// Univariate marginals (App. B.1 with every other variable summed out):
//   M[b,i,a] = log sum_j m[b,i,j] phi[b,i,j,a],  m = marginal of the latent that
// indexes leaf i.  One workgroup owns window position i for a tile of positions
// and walks the r slabs, adding exp(l - LSE_j + log m_j) into a second register
// tile, so each slab's logits are again consumed in registers.
template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16>
__global__ __launch_bounds__(WV * WB * 64)
void k_univariate(const UnivariateArgs a) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr bool M16 = use_m16<WV, WB, SB, NS, BF16>();
  using FR = Frag<M16>;
  constexpr int NPB = PB * FR::SUB, NVB = VB * FR::SUB;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wv = wave % WV, wb = wave / WV;
  const int lcol = FR::lcol(lane);
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  const int wi = blockIdx.x / nbt, bt = blockIdx.x - wi * nbt;
  const int b0 = bt * TL::TP;
  const int rbase = wv * VB * 32 + 4 * FR::lgrp(lane);

  typename FR::blk_t run[NPB][NVB];
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
      for (int i = 0; i < FR::NI; ++i) run[pb][vb][i] = 0.f;

  for (int j = 0; j < a.r; ++j) {
    typename FR::blk_t acc[NPB][NVB];
    tile_gemm<WV, WB, VB, PB, SB, NS, BF16, false, M16>(a.W, a.d, a.h, a.ld_h, a.B, a.d, a.v, wi * a.r + j, b0, smem, acc);
    float mx[NPB], lse[NPB];
    tile_lse<WV, WB, VB, PB, SB, NS, M16>(acc, a.v, (float2*)(smem + TL::RED_OFF), mx, lse);
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) {
      const int b = min(b0 + wb * PB * 32 + pb * FR::BR + lcol, a.B - 1);
      const float lm = a.logm ? a.logm[((long long)b * a.n + wi) * a.r + j] : 0.f;
      // m_j phi_j = 2^((l - lse_j + log m_j) log2 e): one fused multiply-add and one v_exp per logit
      constexpr float LOG2E = 1.4426950408889634f;
      const float shift = (lm - lse[pb]) * LOG2E;
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int i = 0; i < FR::NI; ++i) run[pb][vb][i] += __builtin_amdgcn_exp2f(fmaf(acc[pb][vb][i], LOG2E, shift));
    }
    __syncthreads();   // `red` is rewritten by the next slab
  }
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb) {
    const int b = b0 + wb * PB * 32 + pb * FR::BR + lcol;
    if (b >= a.B) continue;
    float* dst = a.out + ((long long)b * a.n + wi) * a.v;
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
      for (int i = 0; i < FR::NI; ++i) {
        const int row = rbase + vb * FR::BR + FR::roff(i);
        if (row < a.v) dst[row] = __logf(run[pb][vb][i]);
      }
  }
}

template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16>
static hipError_t launch_uni_cfg(const UnivariateArgs& a, hipStream_t st) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr auto kern = k_univariate<WV, WB, VB, PB, SB, NS, BF16>;
  if (hipError_t e = allow_lds<kern>(TL::SMEM); e != hipSuccess) return e;
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  hipLaunchKernelGGL(kern, dim3(nbt * a.n), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

template <bool BF16>
static hipError_t launch_uni_dt(const UnivariateArgs& a, hipStream_t st) {
  if (a.B > 32) {
    if (a.v > 256) return launch_uni_cfg<2, 4, 5, 1, 64, 4, BF16>(a, st);
    if (a.v > 128) return launch_uni_cfg<2, 4, 4, 1, 64, 4, BF16>(a, st);
    return launch_uni_cfg<2, 4, 2, 1, 64, 4, BF16>(a, st);
  }
  if (a.v > 256) return launch_uni_cfg<5, 1, 2, 1, 64, 4, BF16>(a, st);
  if (a.v > 128) return launch_uni_cfg<4, 1, 2, 1, 64, 4, BF16>(a, st);
  return launch_uni_cfg<2, 1, 2, 1, 64, 4, BF16>(a, st);
}

hipError_t launch_univariate(const UnivariateArgs& a, int dtype, hipStream_t st) {
  return dtype == MTPC_BF16 ? launch_uni_dt<true>(a, st) : launch_uni_dt<false>(a, st);
}

template <int WV, int WB, int VB, int PB, int SB, int NS, bool BF16, bool SAMPLE, bool WPACK = false>
static hipError_t launch_cfg(const UnembedArgs& a, hipStream_t st) {
  using TL = Tile<WV, WB, VB, PB, SB, NS>;
  constexpr auto kern = k_unembed<WV, WB, VB, PB, SB, NS, BF16, SAMPLE, WPACK>;
  if (hipError_t e = allow_lds<kern>(TL::SMEM); e != hipSuccess) return e;
  const int nbt = (a.B + TL::TP - 1) / TL::TP;
  int grid = nbt * a.n * a.r;
  if constexpr (unembed_walks_tiles<WB, SAMPLE>()) {
    // one workgroup per CU (the ring takes most of a CU's LDS, so no two share one), a multiple of the
    // 8 XCDs the workgroup ids are dealt over
    int cus = 0;
    if (hipError_t e = cu_count(&cus); e != hipSuccess) return e;
    if (cus >= 8) grid = std::min(grid, cus / 8 * 8);
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(TL::NT), TL::SMEM, st, a);
  return hipGetLastError();
}

// Decode-shaped tiles (B <= 64: WV waves over the vocabulary, W streamed once) are bound by HBM:
// 128-byte stages in a 3-stage ring when the rows allow it (whole cache lines per row and stage,
// 90 KB in flight per CU; 1.5-2.5 % faster than 64-byte stages in a 4-stage ring).
template <int WV, int PB, bool BF16, bool SAMPLE>
static hipError_t launch_dec(const UnembedArgs& a, int row_bytes, hipStream_t st) {
  static_assert(PACK_STAGE_BYTES == 128, "the stage-major copy of W is cut for the 128-byte stages");
  if (row_bytes % 128 == 0) {
    if (a.Wp != nullptr && a.Wp_stage == 128) return launch_cfg<WV, 1, 2, PB, 128, 3, BF16, SAMPLE, true>(a, st);
    return launch_cfg<WV, 1, 2, PB, 128, 3, BF16, SAMPLE>(a, st);
  }
  return launch_cfg<WV, 1, 2, PB, 64, 4, BF16, SAMPLE>(a, st);
}

template <bool BF16, bool SAMPLE>
static hipError_t launch_dt(const UnembedArgs& a, hipStream_t st) {
  // Vocabulary tile: 5 blocks of 32 per wave pair covers v <= 320; v <= 256 and
  // v <= 128 take narrower tiles.  Positions: 256-wide tiles for training-sized
  // batches, 64- or 32-wide tiles (W streamed once) for decode-sized ones.
  const int row_bytes = a.d * (BF16 ? 2 : 4);
  if (a.B > 64) {
    if (a.Wp != nullptr && a.Wp_stage == 64) {      // the copy of W in the 64-byte stages of these tiles
      if (a.v > 256) return launch_cfg<2, 4, 5, 2, 64, 4, BF16, SAMPLE, true>(a, st);
      if (a.v > 128) return launch_cfg<2, 4, 4, 2, 64, 4, BF16, SAMPLE, true>(a, st);
      return launch_cfg<2, 4, 2, 2, 64, 4, BF16, SAMPLE, true>(a, st);
    }
    if (a.v > 256) return launch_cfg<2, 4, 5, 2, 64, 4, BF16, SAMPLE>(a, st);
    if (a.v > 128) return launch_cfg<2, 4, 4, 2, 64, 4, BF16, SAMPLE>(a, st);
    return launch_cfg<2, 4, 2, 2, 64, 4, BF16, SAMPLE>(a, st);
  }
  if (a.B > 32) {
    if (a.v > 256) return launch_dec<5, 2, BF16, SAMPLE>(a, row_bytes, st);
    if (a.v > 128) return launch_dec<4, 2, BF16, SAMPLE>(a, row_bytes, st);
    return launch_dec<2, 2, BF16, SAMPLE>(a, row_bytes, st);
  }
  if (a.v > 256) return launch_dec<5, 1, BF16, SAMPLE>(a, row_bytes, st);
  if (a.v > 128) return launch_dec<4, 1, BF16, SAMPLE>(a, row_bytes, st);
  return launch_dec<2, 1, BF16, SAMPLE>(a, row_bytes, st);
}

// Stage-major copy of a matrix: one thread moves 16 bytes; a workgroup's reads cover 256 / (SB / 16) rows of
// one stage (SB contiguous bytes each), its writes one contiguous run.
__global__ __launch_bounds__(256) void k_pack_rows(const char* __restrict__ src, char* __restrict__ dst, long long slabs, int v,
                                                   int row_bytes, long long row_stride, int stage_bytes) {
  const int cps = stage_bytes / 16;
  const long long per_slab = (long long)v * row_bytes / 16;            // 16-byte chunks of a slab
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;       // chunk index in the packed order
  if (t >= slabs * per_slab) return;
  const long long slab = t / per_slab, u = t - slab * per_slab;
  const int stage = (int)(u / ((long long)v * cps)), w = (int)(u - (long long)stage * v * cps);
  const int row = w / cps, ch = w - row * cps;
  const i32x4_t x = *(const i32x4_t*)(src + (slab * v + row) * row_stride + (long long)stage * stage_bytes + ch * 16);
  *(i32x4_t*)(dst + t * 16) = x;
}

hipError_t launch_pack_rows(const void* src, void* dst, long long slabs, int v, int row_bytes, long long row_stride,
                            int stage_bytes, hipStream_t st) {
  const long long chunks = slabs * v * (row_bytes / 16);
  hipLaunchKernelGGL(k_pack_rows, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, (const char*)src, (char*)dst,
                     slabs, v, row_bytes, row_stride, stage_bytes);
  return hipGetLastError();
}

hipError_t launch_unembed(const UnembedArgs& a, int dtype, hipStream_t st) {
  const bool sample = a.zleaf != nullptr;
  if (dtype == MTPC_BF16)
    return sample ? launch_dt<true, true>(a, st) : launch_dt<true, false>(a, st);
  return sample ? launch_dt<false, true>(a, st) : launch_dt<false, false>(a, st);
}

}  // namespace mtpc

