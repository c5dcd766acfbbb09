// Small kernels of the MtPC head: sum-unit parameters, the circuit's sum/product
// layers on the evidence e[rows][n][r], latent draws of the ancestral sampler,
// latent marginals, and the gather-style evidence used to score a few drafts.
// All of them touch O(B n r) or O(L r^2) data; none is a roofline concern.
#include "mtpc_internal.h"

namespace mtpc {

typedef __attribute__((ext_vector_type(4))) int i32x4_t;

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
// reductions inside aligned groups of G lanes (G a power of two <= 64)
__device__ __forceinline__ float group_max(float x, int G) {
  for (int o = G >> 1; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float group_sum(float x, int G) {
  for (int o = G >> 1; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

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

// ---------------------------------------------------------------------------
// log omega[b,:] = log_softmax(Wsum h[b])   (Sec. 3.3, sum unit parameters)
// one wave per position; r <= 128 scores kept two per lane
// ---------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void k_sumunit(const void* h, long long ld_h, const void* Wsum,
                                                 int B, int d, int r, float* logw) {
  constexpr int ESZ = BF16 ? 2 : 4;
  constexpr int EPC = 16 / ESZ;
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= B) return;
  const char* hb = (const char*)h + (long long)b * ld_h * ESZ;
  const int nch = d / EPC;
  float s0 = neg_inf(), s1 = neg_inf();
  for (int j = 0; j < r; ++j) {
    const char* wr = (const char*)Wsum + (long long)j * d * ESZ;
    float acc = 0.f;
    for (int c = lane; c < nch; c += 64)
      acc += dot_chunk<BF16>(*(const i32x4_t*)(wr + c * 16), *(const i32x4_t*)(hb + c * 16));
    acc = wave_sum(acc);
    if ((j & 63) == lane) { if (j < 64) s0 = acc; else s1 = acc; }
  }
  float m = fmaxf(s0, s1);
  m = group_max(m, 64);
  float e = 0.f;
  if (s0 > neg_inf()) e += __expf(s0 - m);
  if (s1 > neg_inf()) e += __expf(s1 - m);
  e = group_sum(e, 64);
  const float lse = m + __logf(e);
  if (lane < r) logw[(long long)b * r + lane] = s0 - lse;
  if (lane + 64 < r) logw[(long long)b * r + lane + 64] = s1 - lse;
}

hipError_t launch_sumunit(const void* h, long long ld_h, const void* Wsum, int B, int d, int r,
                          int dtype, float* logw, hipStream_t st) {
  dim3 grid((B + 3) / 4), block(256);
  if (dtype == MTPC_BF16)
    hipLaunchKernelGGL(k_sumunit<true>, grid, block, 0, st, h, ld_h, Wsum, B, d, r, logw);
  else
    hipLaunchKernelGGL(k_sumunit<false>, grid, block, 0, st, h, ld_h, Wsum, B, d, r, logw);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// softmax over the last axis of every r x r sum layer -> linear probabilities
// one wave per sum unit (row k of layer l of position-block b)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_normalise_layers(const float* logits, long long ls,
                                                          long long bs, int nb, int L, int r,
                                                          int transpose, float* out) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long nrows = (long long)nb * L * r;
  if (row >= nrows) return;
  const int k = (int)(row % r);
  const int l = (int)((row / r) % L);
  const long long b = row / ((long long)r * L);
  const float* src = logits + b * bs + (long long)l * ls + (long long)k * r;
  const float x0 = lane < r ? src[lane] : neg_inf();
  const float x1 = lane + 64 < r ? src[lane + 64] : neg_inf();
  const float m = group_max(fmaxf(x0, x1), 64);
  const float ms = (m == neg_inf()) ? 0.f : m;
  const float e0 = x0 > neg_inf() ? expf(x0 - ms) : 0.f;
  const float e1 = x1 > neg_inf() ? expf(x1 - ms) : 0.f;
  const float tot = group_sum(e0 + e1, 64);
  const float inv = tot > 0.f ? 1.f / tot : 0.f;
  float* dst = out + (b * L + l) * (long long)r * r;
  if (lane < r) dst[transpose ? (long long)lane * r + k : (long long)k * r + lane] = e0 * inv;
  if (lane + 64 < r)
    dst[transpose ? (long long)(lane + 64) * r + k : (long long)k * r + lane + 64] = e1 * inv;
}

hipError_t launch_normalise_layers(const float* logits, long long layer_stride, long long batch_stride,
                                   int nb, int L, int r, int transpose, float* out, hipStream_t st) {
  const long long nrows = (long long)nb * L * r;
  if (nrows == 0) return hipSuccess;
  hipLaunchKernelGGL(k_normalise_layers, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, st, logits,
                     layer_stride, batch_stride, nb, L, r, transpose, out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// circuit layers.  A group of G lanes (G = smallest power of two >= min(r, 64))
// owns one evidence row; lane g holds the units j = g and g + 64 (r <= 128).
// Sum layers are evaluated in the linear domain after a max shift:
//   log sum_j w[j] exp(c[j]) = m + log sum_j w[j] exp(c[j] - m).
// ---------------------------------------------------------------------------
struct Pair { float a, b; };   // units g and g+64 of a lane

__device__ __forceinline__ float pair_lse(Pair x, int g, int r, int G) {
  // LSE over the r units of a group (missing units hold -inf)
  float m = group_max(fmaxf(x.a, x.b), G);
  if (m == neg_inf()) return m;
  float s = 0.f;
  if (g < r) s += __expf(x.a - m);
  if (g + 64 < r) s += __expf(x.b - m);
  s = group_sum(s, G);
  return m + __logf(s);
}

// out[k] = log sum_j Wl[j][k] exp(c[j]) for the lane's k = g (and g+64); Wl is a
// normalised layer stored [j][k] (k contiguous).  `sh` is this group's r floats of LDS.
__device__ __forceinline__ Pair sum_layer(Pair c, const float* __restrict__ Wl, float* sh, int g,
                                          int r, int G) {
  const float m = group_max(fmaxf(c.a, c.b), G);
  Pair o;
  if (m == neg_inf()) { o.a = o.b = m; return o; }   // uniform inside the group
  if (g < r) sh[g] = __expf(c.a - m);
  if (g + 64 < r) sh[g + 64] = __expf(c.b - m);
  __builtin_amdgcn_wave_barrier();
  float s0 = 0.f, s1 = 0.f;
  const bool two = g + 64 < r;
  for (int j = 0; j < r; ++j) {
    const float p = sh[j];
    if (g < r) s0 = fmaf(p, Wl[(long long)j * r + g], s0);
    if (two) s1 = fmaf(p, Wl[(long long)j * r + g + 64], s1);
  }
  __builtin_amdgcn_wave_barrier();
  o.a = g < r ? m + __logf(s0) : neg_inf();
  o.b = two ? m + __logf(s1) : neg_inf();
  return o;
}

__device__ __forceinline__ Pair load_pair(const float* p, int g, int r, float fill) {
  Pair x;
  x.a = g < r ? p[g] : fill;
  x.b = g + 64 < r ? p[g + 64] : fill;
  return x;
}
__device__ __forceinline__ Pair add_pair(Pair x, Pair y) { return Pair{x.a + y.a, x.b + y.b}; }
__device__ __forceinline__ void store_pair(float* p, Pair x, int g, int r) {
  if (g < r) p[g] = x.a;
  if (g + 64 < r) p[g + 64] = x.b;
}

// dynamic LDS: per group  r floats (exchange) + (n-1)*r floats (BTree node values)
__global__ __launch_bounds__(256) void k_circuit(const CircuitArgs a, int G, int groups_per_block,
                                                 int sh_per_group) {
  extern __shared__ float csm[];
  const int gl = threadIdx.x / G;           // group inside the block
  const int g = threadIdx.x % G;
  const long long row = (long long)blockIdx.x * groups_per_block + gl;
  // whole groups leave together; nothing below synchronises across groups
  if (gl >= groups_per_block || row >= a.rows) return;
  const long long rr = row;
  const int n = a.n, r = a.r;
  const float* e = a.e + rr * n * r;
  const long long b = rr / a.T;
  const float ninf = neg_inf();
  float* sh = csm + (size_t)gl * sh_per_group;
  float* nodes = sh + r;                    // BTree only
  const float* lay = a.layers;
  if (a.contextual && lay) lay += b * (long long)a.L * r * r;
  const long long lstep = (a.L > 1) ? (long long)r * r : 0;
  // An id outside [-1, v) leaves NaN in every unit of its window position; max
  // reductions would drop it, so poison every output that observes that position.
  int first_bad = n;
  for (int i = n - 1; i >= 0; --i)
    if (e[i * r] != e[i * r]) first_bad = i;
  auto emit = [&](int i, float v) {      // value of the prefix ending at token i
    if (g != 0) return;
    if (i >= first_bad) v = __builtin_nanf("");
    if (a.prefix) a.out[row * n + i] = v;
    else if (i == n - 1) a.out[row] = v;
  };

  if (a.family == MTPC_FF) {
    float acc = 0.f;
    for (int i = 0; i < n; ++i) {
      acc += e[i * r];
      emit(i, acc);
    }
    return;
  }
  const Pair lw = load_pair(a.logw + b * r, g, r, ninf);

  if (a.family == MTPC_CP) {
    Pair acc = lw;
    for (int i = 0; i < n; ++i) {
      acc = add_pair(acc, load_pair(e + i * r, g, r, ninf));
      if (a.prefix || i == n - 1) {
        const float v = pair_lse(acc, g, r, G);
        emit(i, v);
      }
    }
    return;
  }

  if (a.family == MTPC_HMM) {
    // forward messages of Eq. HMM: alpha_0 = log omega + e_0,
    // alpha_i[j'] = e_i[j'] + log sum_j exp(alpha_{i-1}[j]) T_{i-1}[j][j']
    Pair alpha = add_pair(lw, load_pair(e, g, r, ninf));
    for (int i = 0; i < n; ++i) {
      if (i > 0) {
        const Pair t = sum_layer(alpha, lay + (long long)(i - 1) * lstep, sh, g, r, G);
        alpha = add_pair(t, load_pair(e + i * r, g, r, ninf));
      }
      if (a.prefix || i == n - 1) {
        const float v = pair_lse(alpha, g, r, G);
        emit(i, v);
      }
    }
    return;
  }

  // ---- binary tree (Eq. BTree), heap order: inner nodes 0..n-2, leaf i at n-1+i.
  // nodes[m*r + k] = C_m[k] for inner m >= 1 with every leaf below it observed.
  auto full_value = [&](int c) -> Pair {   // c: heap index of a child
    return c >= n - 1 ? load_pair(e + (c - (n - 1)) * r, g, r, ninf)
                      : load_pair(nodes + (size_t)c * r, g, r, ninf);
  };
  for (int m = n - 2; m >= 1; --m) {
    const Pair prod = add_pair(full_value(2 * m + 1), full_value(2 * m + 2));
    const Pair c = sum_layer(prod, lay + (long long)(m - 1) * lstep, sh, g, r, G);
    store_pair(nodes + (size_t)m * r, c, g, r);
    __builtin_amdgcn_wave_barrier();
  }
  if (!a.prefix) {
    const Pair prod = add_pair(add_pair(full_value(1), full_value(2)), lw);
    const float v = pair_lse(prod, g, r, G);
    emit(n - 1, v);
    return;
  }
  // prefix marginals: tokens 0..i observed, the rest summed out.  A subtree with
  // no observed leaf evaluates to 1 (log 0 = 0 in every unit); a subtree fully
  // observed is the stored value; only the nodes on the path from leaf i to the
  // root whose range straddles the boundary are re-evaluated.
  for (int i = 0; i < n; ++i) {
    Pair pv = Pair{0.f, 0.f};       // value of the straddling child on the path so far
    int idx = n - 1 + i;            // heap index walking up from leaf i
    int size = 1;                   // leaves under idx
    while (idx > 0) {
      const int m = (idx - 1) >> 1;
      size <<= 1;                   // leaves under m
      // leaf range of m: first = (m - (n/size - 1)) * size
      const int first = (m - (n / size - 1)) * size;
      const int last = first + size - 1;
      if (m > 0 && last <= i) { idx = m; continue; }    // fully observed: stored value
      const int cl = 2 * m + 1, cr = cl + 1;
      const int half = size >> 1;
      const int l_last = first + half - 1, r_first = first + half, r_last = last;
      // left child always starts at or before i
      const Pair lv = (l_last <= i) ? full_value(cl) : pv;
      const Pair rv = (r_first > i) ? Pair{0.f, 0.f} : (r_last <= i ? full_value(cr) : pv);
      const Pair prod = add_pair(lv, rv);
      if (m > 0) {
        pv = sum_layer(prod, lay + (long long)(m - 1) * lstep, sh, g, r, G);
      } else {
        const float v = pair_lse(add_pair(prod, lw), g, r, G);
        emit(i, v);
      }
      idx = m;
    }
  }
}

hipError_t launch_circuit(const CircuitArgs& a, hipStream_t st) {
  int G = 1;
  while (G < a.r && G < 64) G <<= 1;
  int sh_per_group = a.r + (a.family == MTPC_BTREE ? (a.n - 1) * a.r : 0);
  int gpb = 256 / G;
  while (gpb > 1 && (size_t)gpb * sh_per_group * 4 > 48 * 1024) gpb >>= 1;
  const size_t smem = (size_t)gpb * sh_per_group * 4;
  const unsigned grid = (unsigned)((a.rows + gpb - 1) / gpb);
  hipLaunchKernelGGL(k_circuit, dim3(grid), dim3(256), smem, st, a, G, gpb, sh_per_group);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// latent draws (Alg. 1): one thread per draft; CDFs accumulated in double
// ---------------------------------------------------------------------------
__device__ __forceinline__ int draw_linear(const float* p, int r, float u) {
  double acc = 0.0;
  int last = 0;
  for (int k = 0; k < r; ++k) {
    const float pk = p[k];
    acc += (double)pk;
    if (pk > 0.f) last = k;
    if ((double)u < acc) return k;
  }
  return last;
}
__device__ __forceinline__ int draw_log(const float* lp, int r, float u) {
  double acc = 0.0;
  int last = 0;
  for (int k = 0; k < r; ++k) {
    const float pk = expf(lp[k]);
    acc += (double)pk;
    if (pk > 0.f) last = k;
    if ((double)u < acc) return k;
  }
  return last;
}

__global__ __launch_bounds__(256) void k_latents(const LatentArgs a) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)a.B * a.S) return;
  const int b = (int)(t / a.S), s = (int)(t % a.S);
  const int n = a.n, r = a.r;
  int* zl = a.zleaf + t * n;
  if (a.family == MTPC_FF) {
    for (int i = 0; i < n; ++i) zl[i] = 0;
    return;
  }
  const float* lay = a.layers;
  if (a.contextual && lay) lay += (long long)b * a.L * r * r;
  const long long lstep = (a.L > 1) ? (long long)r * r : 0;
  auto U = [&](int lat) {
    return philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, (uint32_t)s, (uint32_t)(n + lat));
  };
  const int z0 = draw_log(a.logw + (long long)b * r, r, U(0));
  if (a.family == MTPC_CP) {
    for (int i = 0; i < n; ++i) zl[i] = z0;
    if (a.latents) a.latents[t] = z0;
  } else if (a.family == MTPC_HMM) {
    int z = z0;
    zl[0] = z;
    if (a.latents) a.latents[t * n] = z;
    for (int i = 1; i < n; ++i) {
      z = draw_linear(lay + (long long)(i - 1) * lstep + (long long)z * r, r, U(i));
      zl[i] = z;
      if (a.latents) a.latents[t * n + i] = z;
    }
  } else {
    // BTree: node m's latent given its parent's (heap order); the state that
    // indexes leaf i is the latent of its parent node (n-2+i)/2.  `latents` is
    // always a valid buffer here (the caller's or library scratch).
    int* L = a.latents + t * (n - 1);
    L[0] = z0;
    for (int m = 1; m < n - 1; ++m)
      L[m] = draw_linear(lay + (long long)(m - 1) * lstep + (long long)L[(m - 1) >> 1] * r, r, U(m));
    for (int i = 0; i < n; ++i) zl[i] = L[(n - 2 + i) >> 1];
  }
}

hipError_t launch_latents(const LatentArgs& a, hipStream_t st) {
  const long long tot = (long long)a.B * a.S;
  hipLaunchKernelGGL(k_latents, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// log marginal of the latent that indexes leaf i (for univariate marginals):
// CP: omega; HMM: omega T_1 ... T_i; BTree: top-down products to the leaf's parent
// one thread per (position, unit); r <= 128 values exchanged through LDS
// ---------------------------------------------------------------------------
__global__ void k_latent_marginals(const LatentMarginalArgs a) {
  extern __shared__ float lsm[];          // 2 * n * r floats: node marginals (linear)
  const int b = blockIdx.x, j = threadIdx.x, n = a.n, r = a.r;
  const float* lay = a.layers;
  if (a.contextual && lay) lay += (long long)b * a.L * r * r;
  const long long lstep = (a.L > 1) ? (long long)r * r : 0;
  float* out = a.logm + (long long)b * n * r;
  const float w = (j < r) ? expf(a.logw[(long long)b * r + j]) : 0.f;
  if (a.family == MTPC_CP) {
    if (j < r) for (int i = 0; i < n; ++i) out[i * r + j] = a.logw[(long long)b * r + j];
    return;
  }
  if (a.family == MTPC_HMM) {
    float* cur = lsm;
    float* nxt = lsm + r;
    if (j < r) { cur[j] = w; out[j] = logf(w); }
    __syncthreads();
    for (int i = 1; i < n; ++i) {
      float s = 0.f;
      if (j < r) {
        const float* T = lay + (long long)(i - 1) * lstep;
        for (int k = 0; k < r; ++k) s = fmaf(cur[k], T[(long long)k * r + j], s);
        nxt[j] = s;
        out[i * r + j] = logf(s);
      }
      __syncthreads();
      float* t = cur; cur = nxt; nxt = t;
    }
    return;
  }
  // BTree: marginal of every inner node's latent, heap order
  if (j < r) lsm[j] = w;
  __syncthreads();
  for (int m = 1; m < n - 1; ++m) {
    if (j < r) {
      const float* A = lay + (long long)(m - 1) * lstep;
      const float* par = lsm + (size_t)((m - 1) >> 1) * r;
      float s = 0.f;
      for (int k = 0; k < r; ++k) s = fmaf(par[k], A[(long long)k * r + j], s);
      lsm[(size_t)m * r + j] = s;
    }
    __syncthreads();
  }
  if (j < r)
    for (int i = 0; i < n; ++i) out[i * r + j] = logf(lsm[(size_t)((n - 2 + i) >> 1) * r + j]);
}

hipError_t launch_latent_marginals(const LatentMarginalArgs& a, hipStream_t st) {
  int threads = 64;
  while (threads < a.r) threads <<= 1;
  const size_t smem = (size_t)(a.n > 2 ? a.n : 2) * a.r * 4;
  hipLaunchKernelGGL(k_latent_marginals, dim3(a.B), dim3(threads), smem, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// gather evidence: e[(b,s)][i][j] = <W[i][j][x_bsi], h[b]> - lse[b][i][j]
// one wave per (b, s, i, group of 4 components)
// ---------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void k_gather_evidence(const GatherArgs a) {
  constexpr int ESZ = BF16 ? 2 : 4;
  constexpr int EPC = 16 / ESZ;
  const int lane = threadIdx.x & 63;
  const int jg = (a.r + 3) / 4;
  const long long wid = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long total = (long long)a.B * a.S * a.n * jg;
  if (wid >= total) return;
  const int q = (int)(wid % jg);
  const long long bsi = wid / jg;
  const int i = (int)(bsi % a.n);
  const long long bs = bsi / a.n;
  const int b = (int)(bs / a.S);
  const int x = a.x[bsi];
  const char* hb = (const char*)a.h + (long long)b * a.ld_h * ESZ;
  const int nch = a.d / EPC;
  for (int jj = 0; jj < 4; ++jj) {
    const int j = q * 4 + jj;
    if (j >= a.r) break;
    float* dst = a.e + (bs * a.n + i) * a.r + j;
    if (x < 0 || x >= a.v) {
      if (lane == 0) *dst = (x == -1) ? 0.f : __builtin_nanf("");
      continue;
    }
    const char* wr = (const char*)a.W + ((((long long)i * a.r + j) * a.v + x) * (long long)a.d) * ESZ;
    float acc = 0.f;
    for (int c = lane; c < nch; c += 64)
      acc += dot_chunk<BF16>(*(const i32x4_t*)(wr + c * 16), *(const i32x4_t*)(hb + c * 16));
    acc = wave_sum(acc);
    if (lane == 0) *dst = acc - a.lse[((long long)b * a.n + i) * a.r + j];
  }
}

hipError_t launch_gather_evidence(const GatherArgs& a, int dtype, hipStream_t st) {
  const long long total = (long long)a.B * a.S * a.n * ((a.r + 3) / 4);
  dim3 grid((unsigned)((total + 3) / 4)), block(256);
  if (dtype == MTPC_BF16) hipLaunchKernelGGL(k_gather_evidence<true>, grid, block, 0, st, a);
  else hipLaunchKernelGGL(k_gather_evidence<false>, grid, block, 0, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
__global__ void k_philox_uniforms(int B, int S, int slots, uint32_t seed_lo, uint32_t seed_hi,
                                  uint32_t offset, float* out) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long tot = (long long)B * S * slots;
  if (t >= tot) return;
  const int slot = (int)(t % slots);
  const long long bs = t / slots;
  out[t] = philox_uniform(seed_lo, seed_hi, offset, (uint32_t)(bs / S), (uint32_t)(bs % S), (uint32_t)slot);
}

hipError_t launch_philox_uniforms(int B, int S, int slots, uint32_t seed_lo, uint32_t seed_hi,
                                  uint32_t offset, float* out, hipStream_t st) {
  const long long tot = (long long)B * S * slots;
  hipLaunchKernelGGL(k_philox_uniforms, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, B, S,
                     slots, seed_lo, seed_hi, offset, out);
  return hipGetLastError();
}

}  // namespace mtpc
