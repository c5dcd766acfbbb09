// Verification step of a speculative-decoding cycle (Alg. 2 from the acceptance
// loop on, and the greedy variant of Sec. 3.4).  One workgroup per position:
//   1. the acceptance tests, all at once (the conditional of a drafted token is a
//      difference of two prefix log-marginals), first failure = rejected position j;
//   2. the circuit's conditional q(. | x_1..x_j) over the whole vocabulary: a
//      mixture of the input units of position j whose weights lambda are the
//      circuit's message into that leaf given the accepted tokens (CP: posterior
//      of the component; HMM: one-step prediction of the forward message; binary
//      tree: product of layer-transposed messages down the path to the leaf, with
//      fully observed left siblings evaluated bottom-up and right siblings = 1);
//   3. one draw from max(0, p - q) / Z (or from p after n acceptances).
// Everything is O(n r^2 + r v) per position and latency-bound; matrix-vector
// products use all 256 threads so that every layer costs one memory round trip.
#include <climits>

#include "mtpc_internal.h"
#include "sumunit.h"

namespace mtpc {
namespace {

// Draft index of the verification step's random numbers: drafting calls use 0 .. S-1 with S a
// signed 32-bit count, so this counter word is never theirs and equal (seed, offset) cannot hand
// an acceptance test the uniform that drew the token it tests.
constexpr uint32_t VERIFY_DRAFT_INDEX = 0xffffffffu;

__device__ __forceinline__ float wmax(float x) { return group_max(x, 64); }
__device__ __forceinline__ float wsum(float x) { return group_sum(x, 64); }
// block-wide reductions of 256 threads; `red` holds 4 floats
__device__ __forceinline__ float block_max(float x, float* red) {
  x = wmax(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_sum(float x, float* red) {
  x = wsum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// out[t] = log sum_k exp(c[k]) M[k*r + t] for t = threadIdx.x < r (others get -inf).
// c: r log-domain values in LDS; M: r x r linear probabilities in global memory,
// t contiguous.  The 256 threads form 256/G column groups that split the k range,
// sixteen loads in flight each.  x (128), part (256), red (4) are LDS scratch.
__device__ float matvec_log(const float* c, const float* __restrict__ M, int r, int G, float* x, float* part,
                            float* red) {
  const int tid = threadIdx.x;
  const float mx = block_max(tid < r ? c[tid] : neg_inf(), red);
  const float ms = (mx == neg_inf()) ? 0.f : mx;
  if (tid < r) x[tid] = __expf(c[tid] - ms);
  __syncthreads();
  const int parts = 256 / G, t = tid % G, pt = tid / G;
  const int per = (r + parts - 1) / parts;
  const int k0 = pt * per, k1 = min(r, k0 + per);
  const int tc = min(t, r - 1);
  float acc = 0.f;
  for (int kb = k0; kb < k1; kb += 16) {
    float w[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) w[u] = M[(long long)min(kb + u, r - 1) * r + tc];
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (kb + u < k1) acc = fmaf(x[kb + u], w[u], acc);
  }
  part[tid] = acc;
  __syncthreads();
  float s = 0.f;
  if (tid < r)
    for (int q = 0; q < parts; ++q) s += part[q * G + tid];
  return tid < r ? ms + __logf(s) : neg_inf();          // log 0 = -inf
}

// The same product in two halves, for chains of products whose layers are known in advance:
// mv_load fetches this thread's 16 weights of a layer (its column t, its part of the k range;
// needs ceil(r / (256 / G)) <= 16), mv_apply multiplies.  Loading the next layer before
// applying the current one takes the L2 round trip out of the chain.
struct MvWeights { float w[16]; };

__device__ __forceinline__ void mv_load(const float* __restrict__ M, int r, int G, MvWeights& o) {
  const int tid = threadIdx.x, parts = 256 / G, t = tid % G, pt = tid / G;
  const int per = (r + parts - 1) / parts, k0 = pt * per, tc = min(t, r - 1);
#pragma unroll
  for (int u = 0; u < 16; ++u) o.w[u] = M[(long long)min(k0 + u, r - 1) * r + tc];
}

__device__ float mv_apply(const float* c, const MvWeights& wt, int r, int G, float* x, float* part, float* red) {
  const int tid = threadIdx.x;
  const float mx = block_max(tid < r ? c[tid] : neg_inf(), red);
  const float ms = (mx == neg_inf()) ? 0.f : mx;
  if (tid < r) x[tid] = __expf(c[tid] - ms);
  __syncthreads();
  const int parts = 256 / G, pt = tid / G;
  const int per = (r + parts - 1) / parts;
  const int k0 = pt * per, k1 = min(r, k0 + per);
  float acc = 0.f;
#pragma unroll
  for (int u = 0; u < 16; ++u)
    if (k0 + u < k1) acc = fmaf(x[k0 + u], wt.w[u], acc);
  part[tid] = acc;
  __syncthreads();
  float s = 0.f;
  if (tid < r)
    for (int q = 0; q < parts; ++q) s += part[q * G + tid];
  return tid < r ? ms + __logf(s) : neg_inf();          // log 0 = -inf
}

__global__ __launch_bounds__(256) void k_verify(const VerifyArgs a, int G) {
  extern __shared__ float vsm[];
  __shared__ float s_red[4], s_x[128], s_c[128], s_part[256], s_ratio[64], s_alpha[64];
  __shared__ int s_arg[65], s_j, s_lo, s_hi;
  __shared__ float s_lw[128];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = a.n, r = a.r, v = a.v;
  float* s_e = vsm;                                          // [n][r] evidence of the drafted tokens
  float* s_nodes = s_e + n * r;                              // [n-1][r] binary tree: node values
  float* s_m = s_nodes + (a.family == MTPC_BTREE ? (n - 1) * r : 0);   // [v] weights of the final draw
  const int* x = a.drafts + (long long)b * n;
  const float* phi = a.logphi + (long long)b * n * r * v;
  const float* pv = a.p + (long long)b * (n + 1) * v;
  // ids outside [0, v) are the caller's error; clamping keeps every access in bounds
  auto tok_at = [&](int i) { return min(max(x[i], 0), v - 1); };

  // ---- 1. acceptance tests ---------------------------------------------------
  if (a.mode == MTPC_VERIFY_GREEDY) {
    for (int s = wave; s <= n; s += 4) {                     // argmax of p[s], smallest id on ties
      float best = neg_inf();
      int arg = INT_MAX;
      for (int t = lane; t < v; t += 64) {
        const float val = pv[(long long)s * v + t];
        if (val > best) { best = val; arg = t; }
      }
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) {
        const float ob = __shfl_xor(best, o);
        const int oa = __shfl_xor(arg, o);
        if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
      }
      if (lane == 0) s_arg[s] = arg == INT_MAX ? 0 : arg;
    }
    __syncthreads();
    if (wave == 0) {
      const bool rej = lane < n && x[min(lane, n - 1)] != s_arg[min(lane, n - 1)];
      const unsigned long long m = __ballot(rej);
      const int j = m ? __ffsll((long long)m) - 1 : n;
      if (lane == 0) { a.accepted[b] = j; a.token[b] = s_arg[j]; }
    }
    return;
  }
  if (tid < n) {
    const float lq = a.prefix[(long long)b * n + tid] - (tid > 0 ? a.prefix[(long long)b * n + tid - 1] : 0.f);
    s_ratio[tid] = pv[(long long)tid * v + tok_at(tid)] / __expf(lq);
    s_alpha[tid] = philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, VERIFY_DRAFT_INDEX, (uint32_t)tid);
  }
  __syncthreads();
  if (wave == 0) {
    const bool rej = lane < n && s_alpha[min(lane, n - 1)] > s_ratio[min(lane, n - 1)];
    const unsigned long long m = __ballot(rej);
    if (lane == 0) s_j = m ? __ffsll((long long)m) - 1 : n;
  }
  __syncthreads();
  const int j = s_j;

  // ---- 2. weights of the final draw into s_m ---------------------------------
  if (j == n) {
    for (int t = tid; t < v; t += 256) s_m[t] = pv[(long long)n * v + t];
  } else {
    // evidence of the accepted tokens: e[i][z] = log phi[i][z][x_i], i < j
    for (int i0 = tid; i0 < j * r; i0 += 4 * 256) {
      float tmp[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = min(i0 + u * 256, j * r - 1);
        tmp[u] = phi[(long long)idx * v + tok_at(idx / r)];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i0 + u * 256 < j * r) s_e[i0 + u * 256] = tmp[u];
    }
    __syncthreads();
    const float* lw = a.logw ? a.logw + (long long)b * r : nullptr;
    if (a.h != nullptr && a.family != MTPC_FF) {             // sum units of this position, computed here
      if (a.bf16) sumunit_position<true>(a.h, a.ld_h, a.Wsum, b, a.d, r, s_lw);
      else sumunit_position<false>(a.h, a.ld_h, a.Wsum, b, a.d, r, s_lw);
      lw = s_lw;
    }
    const long long lstep = a.L > 1 ? (long long)r * r : 0;
    const long long lbase = a.contextual ? (long long)b * a.L * r * r : 0;
    const bool ahead = (r + 256 / G - 1) / (256 / G) <= 16;     // a thread's share of a layer fits mv_load
    // log-domain message into leaf j -> s_c
    if (a.family == MTPC_FF) {
      if (tid < r) s_c[tid] = 0.f;
    } else if (a.family == MTPC_CP) {
      if (tid < r) {
        float acc = lw[tid];
        for (int i = 0; i < j; ++i) acc += s_e[i * r + tid];
        s_c[tid] = acc;
      }
    } else if (a.family == MTPC_HMM) {
      if (tid < r) s_c[tid] = lw[tid] + (j > 0 ? s_e[tid] : 0.f);
      __syncthreads();
      MvWeights cur, nxt;
      if (ahead && j >= 1) mv_load(a.lay_nat + lbase, r, G, cur);
      for (int i = 1; i <= j; ++i) {                         // predict state i from state i-1
        float o;
        if (ahead) {
          if (i < j) mv_load(a.lay_nat + lbase + i * lstep, r, G, nxt);
          o = mv_apply(s_c, cur, r, G, s_x, s_part, s_red);
          cur = nxt;
        } else {
          o = matvec_log(s_c, a.lay_nat + lbase + (i - 1) * lstep, r, G, s_x, s_part, s_red);
        }
        if (i < j && tid < r) o += s_e[i * r + tid];         // ... and observe token i if accepted
        if (tid < r) s_c[tid] = o;
        __syncthreads();
      }
    } else {
      // binary tree, heap order: inner nodes 0..n-2, leaf i at n-1+i
      auto value = [&](int c, int t) {                       // fully observed child c, unit t
        return c >= n - 1 ? s_e[(c - (n - 1)) * r + t] : s_nodes[c * r + t];
      };
      int lg = 0;
      while ((1 << lg) < n) ++lg;
      auto next_left = [&](int m) {                          // next inner node below m whose leaves all lie left of leaf j
        for (--m; m >= 1; --m) {
          const int lev = 31 - __clz(m + 1);
          const int span = n >> lev;
          if ((m + 1 - (1 << lev)) * span + span - 1 < j) return m;
        }
        return 0;
      };
      MvWeights cur, nxt;
      int m = next_left(n - 1);
      if (ahead && m) mv_load(a.lay_tr + lbase + (m - 1) * lstep, r, G, cur);
      while (m) {                                            // bottom-up over those subtrees
        const int mn = next_left(m);
        if (ahead && mn) mv_load(a.lay_tr + lbase + (mn - 1) * lstep, r, G, nxt);
        if (tid < r) s_c[tid] = value(2 * m + 1, tid) + value(2 * m + 2, tid);
        __syncthreads();
        const float o = ahead ? mv_apply(s_c, cur, r, G, s_x, s_part, s_red)
                              : matvec_log(s_c, a.lay_tr + lbase + (m - 1) * lstep, r, G, s_x, s_part, s_red);
        if (tid < r) s_nodes[m * r + tid] = o;
        __syncthreads();
        cur = nxt;
        m = mn;
      }
      // top-down along the path: D_child[t] = (sum_k D_node[k] A_node[k][t]) * sibling[t]
      for (int lev = 0; lev < lg; ++lev) {
        // child of the path node at this level: the node (or leaf) one level down that covers leaf j
        const int c = lev + 1 < lg ? (1 << (lev + 1)) - 1 + (j >> (lg - lev - 1)) : n - 1 + j;
        const int node = (c - 1) >> 1;
        // the node of the next level is this level's child c: its layer can be fetched now
        if (ahead && lev + 1 < lg) mv_load(a.lay_nat + lbase + (c - 1) * lstep, r, G, nxt);
        float o;
        if (node == 0) o = tid < r ? lw[tid] : neg_inf();
        else if (ahead) o = mv_apply(s_c, cur, r, G, s_x, s_part, s_red);
        else o = matvec_log(s_c, a.lay_nat + lbase + (node - 1) * lstep, r, G, s_x, s_part, s_red);
        cur = nxt;
        if ((c & 1) == 0 && tid < r) o += value(c - 1, tid);  // left sibling: leaves < j, observed
        __syncthreads();
        if (tid < r) s_c[tid] = o;                            // right sibling: nothing observed, = 1
        __syncthreads();
      }
    }
    __syncthreads();
    // lambda = softmax(s_c) (linear) -> s_x
    {
      const float cv = tid < r ? s_c[tid] : neg_inf();
      const float mx = block_max(cv, s_red);
      const float ex = tid < r ? __expf(cv - mx) : 0.f;
      const float tot = block_sum(ex, s_red);
      if (tid < r) s_x[tid] = ex / tot;
      __syncthreads();
    }
    // q(a | x_1..x_j) = sum_z lambda_z phi[j][z][a];  weights max(0, p - q)
    for (int t0 = tid; t0 < v; t0 += 256) {
      const float* col = phi + (long long)j * r * v + t0;
      float q = 0.f;
      for (int z0 = 0; z0 < r; z0 += 8) {
        float lp[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) lp[u] = col[(long long)min(z0 + u, r - 1) * v];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (z0 + u < r) q = fmaf(s_x[z0 + u], __expf(lp[u]), q);
      }
      s_m[t0] = fmaxf(0.f, pv[(long long)j * v + t0] - q);
    }
  }
  __syncthreads();

  // ---- 3. inverse-CDF draw from s_m / Z ---------------------------------------
  const int C = (v + 255) / 256;                             // consecutive ids per thread
  float total = 0.f, excl = 0.f;
  for (int pass = 0; pass < 2; ++pass) {
    float ls = 0.f;
    for (int q = 0; q < C; ++q) {
      const int t = tid * C + q;
      if (t < v) ls += s_m[t];
    }
    float incl = ls;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const float up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    __syncthreads();
    if (lane == 63) s_red[wave] = incl;
    __syncthreads();
    float base = 0.f;
    for (int w = 0; w < wave; ++w) base += s_red[w];
    total = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
    excl = base + incl - ls;
    if (total > 0.f || j == n || pass == 1) break;
    // p == q at the rejected position: the adjusted distribution is undefined, draw from p
    __syncthreads();
    for (int t = tid; t < v; t += 256) s_m[t] = pv[(long long)j * v + t];
    __syncthreads();
  }
  if (tid == 0) { s_lo = INT_MAX; s_hi = -1; }
  __syncthreads();
  const float u = philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, VERIFY_DRAFT_INDEX, (uint32_t)n);
  const float tgt = u * total;
  {
    float run = excl;
    int first = INT_MAX, lastpos = -1;
    for (int q = 0; q < C; ++q) {
      const int t = tid * C + q;
      if (t < v) {
        const float w = s_m[t];
        run += w;
        if (first == INT_MAX && tgt < run) first = t;
        if (w > 0.f) lastpos = t;
      }
    }
    if (first != INT_MAX) atomicMin(&s_lo, first);
    if (lastpos >= 0) atomicMax(&s_hi, lastpos);
  }
  __syncthreads();
  if (tid == 0) {
    a.accepted[b] = j;
    a.token[b] = s_lo != INT_MAX ? s_lo : max(s_hi, 0);
  }
}

}  // namespace

hipError_t launch_verify(const VerifyArgs& a, hipStream_t st) {
  int G = 1;
  while (G < a.r) G <<= 1;                                   // r <= 128 -> at least two column groups
  const size_t smem = ((size_t)a.n * a.r + (a.family == MTPC_BTREE ? (size_t)(a.n - 1) * a.r : 0) + a.v) * 4;
  if (hipError_t e = allow_lds<k_verify>(96 * 1024); e != hipSuccess) return e;
  hipLaunchKernelGGL(k_verify, dim3(a.B), dim3(256), smem, st, a, G);
  return hipGetLastError();
}

}  // namespace mtpc
