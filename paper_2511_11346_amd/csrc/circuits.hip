// Small kernels of the MtPC head: sum-unit parameters, the circuit's sum/product
// layers on the evidence e[rows][n][r], latent draws of the ancestral sampler,
// latent marginals, and the table lookup that scores drafts.
// All of them touch O(B n r) or O(L r^2) data; none is a roofline concern.
#include <type_traits>

#include "mtpc_internal.h"
#include "sumunit.h"

namespace mtpc {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ float wave_sum(float x) { return group_sum(x, 64); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// First window position of an evidence row e[n][r] whose unit 0 is NaN (n if
// none).  The lanes of a group probe different positions, eight loads in flight
// each, so the scan costs one memory round trip instead of n.
__device__ __forceinline__ int first_nan_position(const float* e, int n, int r, int g, int G) {
  int fb = n;
  for (int i0 = 0; i0 < n; i0 += 8 * G) {
    float t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = e[(long long)min(i0 + u * G + g, n - 1) * r];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (t[u] != t[u]) fb = min(fb, min(i0 + u * G + g, n - 1));
  }
  return group_min(fb, G);
}

__device__ void draft_latents(const LatentArgs& a, int b, int s, const float* lw, int lane);

// ---------------------------------------------------------------------------
// log omega[b,:] = log_softmax(Wsum h[b])   (Sec. 3.3, sum unit parameters)
// Few positions: one workgroup of 16 waves per position (sumunit_position).  With la.zleaf set the
// workgroup goes on to draw the latents of the position's drafts from the weights it has just
// computed (Alg. 1, top-down; one wave per draft) - one launch and one dependent round trip less
// on the decode path.  Many positions go through the MFMA tile kernel instead.
// ---------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(1024) void k_sumunit(const void* h, long long ld_h, const void* Wsum,
                                                  int B, int d, int r, float* logw, const LatentArgs la) {
  __shared__ float sc[128];
  const int b = blockIdx.x;
  sumunit_position<BF16, 16>(h, ld_h, Wsum, b, d, r, sc);
  if ((int)threadIdx.x < r) logw[(long long)b * r + threadIdx.x] = sc[threadIdx.x];
  if (la.zleaf != nullptr)
    for (int s = threadIdx.x >> 6; s < la.S; s += 16) draft_latents(la, b, s, sc, threadIdx.x & 63);
}

static hipError_t launch_sumunit_small(const void* h, long long ld_h, const void* Wsum, int B, int d, int r,
                                       int dtype, float* logw, const LatentArgs& la, hipStream_t st) {
  dim3 grid(B), block(1024);
  if (dtype == MTPC_BF16)
    hipLaunchKernelGGL(k_sumunit<true>, grid, block, 0, st, h, ld_h, Wsum, B, d, r, logw, la);
  else
    hipLaunchKernelGGL(k_sumunit<false>, grid, block, 0, st, h, ld_h, Wsum, B, d, r, logw, la);
  return hipGetLastError();
}

hipError_t launch_sumunit(const void* h, long long ld_h, const void* Wsum, int B, int d, int r,
                          int dtype, float* logw, hipStream_t st) {
  if (B > SUMUNIT_SMALL_B) return launch_sumunit_mfma(h, ld_h, Wsum, B, d, r, dtype, logw, st);
  LatentArgs none{};
  return launch_sumunit_small(h, ld_h, Wsum, B, d, r, dtype, logw, none, st);
}

// sum units and latent draws in one launch (B <= SUMUNIT_SMALL_B, a family with sum units; the
// normalised layers the draws of the HMM / binary tree read must be complete before it)
hipError_t launch_sumunit_latents(const void* h, long long ld_h, const void* Wsum, int d, int dtype, float* logw,
                                  const LatentArgs& la, hipStream_t st) {
  return launch_sumunit_small(h, ld_h, Wsum, la.B, d, la.r, dtype, logw, la, st);
}

// ---------------------------------------------------------------------------
// softmax over the last axis of every r x r sum layer -> linear probabilities
// one wave per sum unit (row k of layer l of position-block b); the natural copy
// [k][j], the transposed one [j][k], or both from one launch
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_normalise_layers(const float* logits, long long ls,
                                                          long long bs, int nb, int L, int r,
                                                          float* out_nat, float* out_tr) {
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
  const long long base = (b * L + l) * (long long)r * r;
  if (out_nat) {
    if (lane < r) out_nat[base + (long long)k * r + lane] = e0 * inv;
    if (lane + 64 < r) out_nat[base + (long long)k * r + lane + 64] = e1 * inv;
  }
  if (out_tr) {
    if (lane < r) out_tr[base + (long long)lane * r + k] = e0 * inv;
    if (lane + 64 < r) out_tr[base + (long long)(lane + 64) * r + k] = e1 * inv;
  }
}

hipError_t launch_normalise_layers(const float* logits, long long layer_stride, long long batch_stride,
                                   int nb, int L, int r, float* out_nat, float* out_tr, hipStream_t st) {
  const long long nrows = (long long)nb * L * r;
  if (nrows == 0 || (!out_nat && !out_tr)) return hipSuccess;
  hipLaunchKernelGGL(k_normalise_layers, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, st, logits,
                     layer_stride, batch_stride, nb, L, r, out_nat, out_tr);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// circuit layers.  A group of G lanes (G = smallest power of two >= min(r, 64))
// owns RB consecutive evidence rows; lane g holds the units j = g and g + 64
// (r <= 128) of each.  Sum layers are evaluated in the linear domain after a max
// shift:  log sum_j w[j] exp(c[j]) = m + log sum_j w[j] exp(c[j] - m),
// and every weight fetched from the (L2-resident) layer serves all RB rows.
// Rows that share a batch must share their layers, so contextual layers run RB=1.
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

template <int RB> struct Rows { Pair v[RB]; };

// out[q][k] = log sum_j Wl[j][k] exp(c[q][j]) for the lane's k = g (and g+64); Wl is
// a normalised layer stored [j][k] (k contiguous).  `sh` holds this group's
// r * RB floats, laid out [j][q] so that one LDS read serves all RB rows.
template <int RB>
__device__ __forceinline__ Rows<RB> sum_layer(const Rows<RB>& c, const float* __restrict__ Wl, float* sh,
                                              int g, int r, int G) {
  float m[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) {
    m[q] = group_max(fmaxf(c.v[q].a, c.v[q].b), G);
    const float ms = (m[q] == neg_inf()) ? 0.f : m[q];
    if (g < r) sh[g * RB + q] = __expf(c.v[q].a - ms);             // exp(-inf) = 0
    if (g + 64 < r) sh[(g + 64) * RB + q] = __expf(c.v[q].b - ms);
  }
  __builtin_amdgcn_wave_barrier();
  float s0[RB], s1[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) s0[q] = s1[q] = 0.f;
  const bool one = g < r, two = g + 64 < r;
  const int gc = one ? g : 0;
  for (int j0 = 0; j0 < r; j0 += 8) {
    // eight weights per lane in flight at once (clamped rows get weight zero)
    float w0[8], w1[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int j = min(j0 + u, r - 1);
      w0[u] = Wl[(long long)j * r + gc];
      w1[u] = two ? Wl[(long long)j * r + g + 64] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool live = one && j0 + u < r;
      const float a0 = live ? w0[u] : 0.f, a1 = live ? w1[u] : 0.f;
      const int j = min(j0 + u, r - 1);
#pragma unroll
      for (int q = 0; q < RB; ++q) {
        const float p = sh[j * RB + q];
        s0[q] = fmaf(p, a0, s0[q]);
        s1[q] = fmaf(p, a1, s1[q]);
      }
    }
  }
  __builtin_amdgcn_wave_barrier();
  Rows<RB> o;
#pragma unroll
  for (int q = 0; q < RB; ++q) {
    o.v[q].a = one ? m[q] + __logf(s0[q]) : neg_inf();           // -inf + log 0 = -inf
    o.v[q].b = two ? m[q] + __logf(s1[q]) : neg_inf();
  }
  return o;
}

// dynamic LDS: per group  RB*r floats (exchange) + (n-1)*RB*r floats (BTree node values)
template <int RB>
__global__ __launch_bounds__(256) void k_circuit(const CircuitArgs a, int G, int groups_per_block,
                                                 int sh_per_group) {
  extern __shared__ float csm[];
  const int gl = threadIdx.x / G;           // group inside the block
  const int g = threadIdx.x % G;
  const long long row0 = ((long long)blockIdx.x * groups_per_block + gl) * RB;
  // whole groups leave together; nothing below synchronises across groups
  if (gl >= groups_per_block || row0 >= a.rows) return;
  const int n = a.n, r = a.r;
  const float ninf = neg_inf();
  float* sh = csm + (size_t)gl * sh_per_group;
  float* nodes = sh + RB * r;               // BTree only: nodes[(m*RB + q)*r + k]
  const long long lstep = (a.L > 1) ? (long long)r * r : 0;
  const float* lay = a.layers;
  if (a.contextual && lay) lay += (row0 / a.T) * (long long)a.L * r * r;   // RB == 1 here

  // rows beyond the end repeat the last row (loads stay in bounds) and are not stored
  long long row[RB];
  const float* e[RB];
  int first_bad[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) {
    row[q] = row0 + q;
    const long long rc = row[q] < a.rows ? row[q] : a.rows - 1;
    e[q] = a.e + rc * n * r;
    // An id outside [-1, v) leaves NaN in every unit of its window position; max
    // reductions would drop it, so poison every output that observes that position.
    first_bad[q] = n;
  }
  if constexpr (RB == 1) {
    // few rows: the call is latency-bound, so fetch the whole evidence row with all
    // loads in flight at once and serve the layer-by-layer accesses from LDS
    float* stage = csm + (size_t)groups_per_block * sh_per_group + (size_t)gl * n * r;
    const int tot = n * r;
    for (int t0 = 0; t0 < tot; t0 += 8 * G) {
      float tmp[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) tmp[u] = e[0][min(t0 + u * G + g, tot - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (t0 + u * G + g < tot) stage[t0 + u * G + g] = tmp[u];
    }
    __builtin_amdgcn_wave_barrier();
    e[0] = stage;
  }
#pragma unroll
  for (int q = 0; q < RB; ++q) first_bad[q] = first_nan_position(e[q], n, r, g, G);
  auto emit = [&](int q, int i, float v) {      // value of the prefix ending at token i of row q
    if (g != 0 || row[q] >= a.rows) return;
    if (i >= first_bad[q]) v = __builtin_nanf("");
    if (a.prefix) a.out[row[q] * n + i] = v;
    else if (i == n - 1) a.out[row[q]] = v;
  };

  if (a.family == MTPC_FF) {
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      // a running sum of up to 64 terms near -6 each: kept in double, so that the fp32 result
      // carries one rounding instead of one per token (an ulp is 3e-5 at 400)
      double acc = 0.0;
      for (int i = 0; i < n; ++i) {
        acc += (double)e[q][i * r];
        emit(q, i, (float)acc);
      }
    }
    return;
  }
  Rows<RB> lw;
#pragma unroll
  for (int q = 0; q < RB; ++q) {
    const long long rc = row[q] < a.rows ? row[q] : a.rows - 1;
    lw.v[q] = load_pair(a.logw + (rc / a.T) * r, g, r, ninf);
  }
  auto leaf = [&](int i) {                  // evidence of token i for all rows
    Rows<RB> x;
#pragma unroll
    for (int q = 0; q < RB; ++q) x.v[q] = load_pair(e[q] + i * r, g, r, ninf);
    return x;
  };
  auto add = [&](const Rows<RB>& x, const Rows<RB>& y) {
    Rows<RB> o;
#pragma unroll
    for (int q = 0; q < RB; ++q) o.v[q] = add_pair(x.v[q], y.v[q]);
    return o;
  };
  auto emit_lse = [&](int i, const Rows<RB>& x) {
#pragma unroll
    for (int q = 0; q < RB; ++q) emit(q, i, pair_lse(x.v[q], g, r, G));
  };
  // The chains (CP, HMM) take one step per token.  Their messages are kept relative to their
  // largest unit and the magnitude taken out is summed in double, so that the fp32 result carries
  // the rounding of one step, not of n (an ulp is 3e-5 at the |log q| = 350 of a 64-token window).
  double scale[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) scale[q] = 0.0;
  auto renorm = [&](Rows<RB>& x) {
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      const float m = group_max(fmaxf(x.v[q].a, x.v[q].b), G);
      if (m == ninf) continue;                           // probability zero so far: nothing to take out
      x.v[q].a -= m;
      x.v[q].b -= m;
      scale[q] += (double)m;
    }
  };
  auto emit_scaled = [&](int i, const Rows<RB>& x) {     // x fresh from renorm: its largest unit is 0
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      float s = 0.f;
      if (g < r) s += __expf(x.v[q].a);
      if (g + 64 < r) s += __expf(x.v[q].b);
      s = group_sum(s, G);                               // all units -inf: log 0 = -inf
      emit(q, i, (float)(scale[q] + (double)__logf(s)));
    }
  };

  if (a.family == MTPC_CP) {
    Rows<RB> acc = lw;
    for (int i = 0; i < n; ++i) {
      acc = add(acc, leaf(i));
      renorm(acc);                                      // every step, so that the log-likelihood call
      if (a.prefix || i == n - 1) emit_scaled(i, acc);  // returns the bits of the last prefix marginal
    }
    return;
  }

  if (a.family == MTPC_HMM) {
    // forward messages of Eq. HMM: alpha_0 = log omega + e_0,
    // alpha_i[j'] = e_i[j'] + log sum_j exp(alpha_{i-1}[j]) T_{i-1}[j][j']
    Rows<RB> alpha = add(lw, leaf(0));
    for (int i = 0; i < n; ++i) {
      if (i > 0) alpha = add(sum_layer<RB>(alpha, lay + (long long)(i - 1) * lstep, sh, g, r, G), leaf(i));
      renorm(alpha);
      if (a.prefix || i == n - 1) emit_scaled(i, alpha);
    }
    return;
  }

  // ---- binary tree (Eq. BTree), heap order: inner nodes 0..n-2, leaf i at n-1+i.
  // nodes[(m*RB+q)*r + k] = C_m[k] of row q for inner m >= 1 with every leaf below it observed.
  auto full_value = [&](int c) {            // c: heap index of a child
    if (c >= n - 1) return leaf(c - (n - 1));
    Rows<RB> x;
#pragma unroll
    for (int q = 0; q < RB; ++q) x.v[q] = load_pair(nodes + ((size_t)c * RB + q) * r, g, r, ninf);
    return x;
  };
  for (int m = n - 2; m >= 1; --m) {
    const Rows<RB> c = sum_layer<RB>(add(full_value(2 * m + 1), full_value(2 * m + 2)),
                                     lay + (long long)(m - 1) * lstep, sh, g, r, G);
#pragma unroll
    for (int q = 0; q < RB; ++q) store_pair(nodes + ((size_t)m * RB + q) * r, c.v[q], g, r);
    __builtin_amdgcn_wave_barrier();
  }
  if (!a.prefix) {
    emit_lse(n - 1, add(add(full_value(1), full_value(2)), lw));
    return;
  }
  // prefix marginals: tokens 0..i observed, the rest summed out.  A subtree with
  // no observed leaf evaluates to 1 (log 0 = 0 in every unit); a subtree fully
  // observed is the stored value; only the nodes on the path from leaf i to the
  // root whose range straddles the boundary are re-evaluated.
  Rows<RB> zero;
#pragma unroll
  for (int q = 0; q < RB; ++q) zero.v[q] = Pair{0.f, 0.f};
  for (int i = 0; i < n; ++i) {
    Rows<RB> pv = zero;             // value of the straddling child on the path so far
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
      const Rows<RB> lv = (l_last <= i) ? full_value(cl) : pv;
      const Rows<RB> rv = (r_first > i) ? zero : (r_last <= i ? full_value(cr) : pv);
      const Rows<RB> prod = add(lv, rv);
      if (m > 0) pv = sum_layer<RB>(prod, lay + (long long)(m - 1) * lstep, sh, g, r, G);
      else emit_lse(i, add(prod, lw));
      idx = m;
    }
  }
}

template <int RB>
static hipError_t launch_circuit_rb(const CircuitArgs& a, hipStream_t st) {
  int G = 1;
  while (G < a.r && G < 64) G <<= 1;
  const int sh_per_group = RB * (a.r + (a.family == MTPC_BTREE ? (a.n - 1) * a.r : 0));
  int gpb = 256 / G;
  const int stage_per_group = RB == 1 ? a.n * a.r : 0;      // LDS copy of the evidence row
  while (gpb > 1 && (size_t)gpb * (sh_per_group + stage_per_group) * 4 > 48 * 1024) gpb >>= 1;
  // one group at the largest sizes (n = 64, r = 128, RB = 1): 32.5 KiB + 32 KiB <= 64 KiB
  const size_t smem = (size_t)gpb * (sh_per_group + stage_per_group) * 4;
  const long long ngroups = ((long long)a.rows + RB - 1) / RB;
  const unsigned grid = (unsigned)((ngroups + gpb - 1) / gpb);
  hipLaunchKernelGGL(k_circuit<RB>, dim3(grid), dim3(256), smem, st, a, G, gpb, sh_per_group);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Binary tree with layers shared by all rows (static A).  The order in which
// nodes are evaluated does not depend on the data, so a workgroup first writes
// the evaluation as a short program (one step per sum-layer application) and then
// all its groups walk that program together: the layer of step t+1 is fetched
// into LDS while step t is multiplied, and no group waits on global memory for
// weights.  A group of G lanes owns RB = 4 rows, r <= 64.
// ---------------------------------------------------------------------------
// One sum layer for the RB rows of a group with the layer in LDS and one unit per
// lane (r <= 64):  c[q] <- log sum_j Wl[j][g] exp(c[q][j]).  Lanes g >= r hold -inf.
template <int RB>
__device__ __forceinline__ void sum_layer_lds(float (&c)[RB], const float* Wl, float* sh, int g, int r, int G) {
  float m[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) m[q] = group_max(c[q], G);
  const bool live = g < r;
  const int gc = live ? g : 0;
  float ex[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) ex[q] = __expf(c[q] - ((m[q] == neg_inf()) ? 0.f : m[q]));   // exp(-inf) = 0
  if (live) {
#pragma unroll
    for (int q = 0; q < RB; ++q) sh[g * RB + q] = ex[q];
  }
  __builtin_amdgcn_wave_barrier();
  float s[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) s[q] = 0.f;
  for (int j0 = 0; j0 < r; j0 += 8) {
    // sixteen LDS reads in flight: eight weights and the eight RB-wide exchange rows
    float w[8], p[8][RB];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int j = min(j0 + u, r - 1);
      w[u] = Wl[j * r + gc];
#pragma unroll
      for (int q = 0; q < RB; ++q) p[u][q] = sh[j * RB + q];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float wu = (j0 + u < r) ? w[u] : 0.f;
#pragma unroll
      for (int q = 0; q < RB; ++q) s[q] = fmaf(p[u][q], wu, s[q]);
    }
  }
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int q = 0; q < RB; ++q) c[q] = live ? m[q] + __logf(s[q]) : neg_inf();   // -inf + log 0 = -inf
}

template <int RB>
__global__ __launch_bounds__(256) void k_btree_static(const CircuitArgs a, int G) {
  extern __shared__ __align__(16) float bsm[];
  const int n = a.n, r = a.r;
  const int groups = 256 / G;
  const int gl = threadIdx.x / G, g = threadIdx.x % G;
  const float ninf = neg_inf();
  const bool live = g < r;
  const int gc = live ? g : 0;
  // LDS: [2][r*r] layer ring | per group: RB*r exchange + (n-1)*RB*r node values | program
  const int rr = r * r;
  const size_t per_group = (size_t)RB * r * n;
  float* layer = bsm;
  float* sh = bsm + 2 * rr + gl * per_group;
  float* nodes = sh + RB * r;                   // nodes[(m*RB + q)*r + k]
  TreeStep* prog = (TreeStep*)(bsm + 2 * rr + groups * per_group);
  __shared__ int s_nsteps;
  if (threadIdx.x == 0) s_nsteps = build_tree_program(prog, n, a.prefix);
  __syncthreads();
  const int nsteps = s_nsteps;

  const long long row0 = ((long long)blockIdx.x * groups + gl) * RB;
  long long row[RB];
  const float* e[RB];
  int first_bad[RB];
  float lw[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) {
    row[q] = row0 + q;
    const long long rc = row[q] < a.rows ? row[q] : a.rows - 1;     // clamped: loads stay in bounds
    e[q] = a.e + rc * n * r;
    const float x = a.logw[(rc / a.T) * r + gc];
    lw[q] = live ? x : ninf;
    first_bad[q] = first_nan_position(e[q], n, r, g, G);
  }
  // leaf operands come from global memory: they are fetched one step ahead
  float nxl[RB], nxr[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) nxl[q] = nxr[q] = 0.f;
  auto prefetch = [&](int t) {
    if (t >= nsteps) return;
    const TreeStep s = prog[t];
    if (s.lsrc >= n - 1) {
#pragma unroll
      for (int q = 0; q < RB; ++q) nxl[q] = e[q][(s.lsrc - (n - 1)) * r + gc];
    }
    if (s.rsrc >= n - 1) {
#pragma unroll
      for (int q = 0; q < RB; ++q) nxr[q] = e[q][(s.rsrc - (n - 1)) * r + gc];
    }
  };
  auto operand = [&](int src, const float (&pv)[RB], const float (&pre)[RB], float (&x)[RB]) {
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      float v;
      if (src == -1) v = pv[q];
      else if (src == -2) v = 0.f;
      else if (src >= n - 1) v = pre[q];
      else v = nodes[((size_t)src * RB + q) * r + gc];
      x[q] = live ? v : ninf;
    }
  };
  // The layer of step t (transposed layout [j][k], at most 16 floats per thread)
  // goes to ring slot t & 1 in two halves: loads issued before step t-1 is
  // evaluated, LDS stores after it, so the loads' latency hides behind that step.
  const long long lstep = (a.L > 1) ? (long long)rr : 0;
  float stage[16];
  auto layer_of = [&](int t) -> const float* {
    if (t >= nsteps) return nullptr;
    const int m = prog[t].m;
    return m == 0 ? nullptr : a.layers + (long long)(m - 1) * lstep;
  };
  auto fetch_load = [&](int t) {
    const float* src = layer_of(t);
    if (!src) return;
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (u * 256 < rr) stage[u] = src[min((int)threadIdx.x + u * 256, rr - 1)];
  };
  auto fetch_store = [&](int t) {
    if (!layer_of(t)) return;
    float* dst = layer + (t & 1) * rr;
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if ((int)threadIdx.x + u * 256 < rr) dst[threadIdx.x + u * 256] = stage[u];
  };
  fetch_load(0);
  prefetch(0);
  fetch_store(0);
  float pv[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) pv[q] = 0.f;
  for (int t = 0; t < nsteps; ++t) {
    __syncthreads();             // layer t is complete in slot t & 1; slot (t+1) & 1 is no longer read
    const TreeStep st = prog[t];
    float c[RB];
    {
      float lv[RB], rv[RB];
      operand(st.lsrc, pv, nxl, lv);
      operand(st.rsrc, pv, nxr, rv);
#pragma unroll
      for (int q = 0; q < RB; ++q) c[q] = lv[q] + rv[q];
    }
    fetch_load(t + 1);
    prefetch(t + 1);
    if (st.m == 0) {             // root: mixture with log omega
      const int i = -2 - st.out;
      float x[RB], m[RB], s[RB];
#pragma unroll
      for (int q = 0; q < RB; ++q) { x[q] = c[q] + lw[q]; m[q] = group_max(x[q], G); }
#pragma unroll
      for (int q = 0; q < RB; ++q) s[q] = group_sum((live && m[q] != ninf) ? __expf(x[q] - m[q]) : 0.f, G);
#pragma unroll
      for (int q = 0; q < RB; ++q) {
        float v = (m[q] == ninf) ? ninf : m[q] + __logf(s[q]);
        if (g == 0 && row[q] < a.rows) {
          if (i >= first_bad[q]) v = __builtin_nanf("");
          if (a.prefix) a.out[row[q] * n + i] = v; else a.out[row[q]] = v;
        }
      }
    } else {
      sum_layer_lds<RB>(c, layer + (t & 1) * rr, sh, g, r, G);
      if (st.out >= 0) {
        if (live) {
#pragma unroll
          for (int q = 0; q < RB; ++q) nodes[((size_t)st.out * RB + q) * r + g] = c[q];
        }
        __builtin_amdgcn_wave_barrier();
      } else {
#pragma unroll
        for (int q = 0; q < RB; ++q) pv[q] = c[q];
      }
    }
    fetch_store(t + 1);
  }
}

// ---------------------------------------------------------------------------
// Binary tree with layers shared by all rows and r = 16, 32 or 64 units: the sum layers on the
// matrix pipe.  A sum layer applied to many rows is the product  S[k][row] = sum_j A[k][j] X[j][row]
// with X = exp(children's values - their row maximum) (Eq. BTree in the linear domain after a max
// shift); a workgroup owns 16 rows and walks the same step program as k_btree_static with
// v_mfma_f32_16x16x4_f32 (fp32 operands and accumulation).  Lane (row = l % 16, g = l / 16) holds,
// of its row, the units j = 16 b + 4 g + i (b < R / 16, i < 4): that is at once the B-operand
// layout of the product (k-index g), the layout its result comes back in (rows 4 g + i of output
// block b) and four contiguous floats per block in memory.
// The workgroup has one wave per block of 16 output units (R / 16 waves, each on a SIMD of its own):
// every wave forms the whole operand vector X (the exponentials are repeated, the products are
// not), multiplies it with its own 16 rows of the layer, and stores its 16 results; one barrier
// per step makes them visible.  The path value of a prefix walk alternates between two slots, so
// that a wave may store the new one while another still reads the old one.  The wave's rows of
// a step's layer (natural layout A[k][j], 16-byte loads) and the step's leaf evidence are fetched
// two steps ahead, into two register sets used alternately; the steps themselves sit in scalar
// registers, and the lanes of a row combine their maxima and sums with the vector unit's lane swaps.
// LDS: (n-1) node values and 2 path values x 16 rows x (R + 4) floats, and the program.
// ---------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(4 * R) void k_btree_mfma(const CircuitArgs a) {
  constexpr int NB = R / 16;        // blocks of 16 units = waves
  constexpr int RS = R + 4;         // row stride of a stored value (floats; 16-byte aligned rows)
  extern __shared__ __align__(16) float msm[];
  const int n = a.n;
  const int lane = threadIdx.x & 63, rl = lane & 15, g = lane >> 4;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* nodes = msm;                                   // [n+1][16][RS]: nodes 0..n-2, path values n-1 and n
  TreeStep* prog = (TreeStep*)(msm + (size_t)(n + 1) * 16 * RS);
  __shared__ int s_nsteps;
  if (threadIdx.x == 0) s_nsteps = build_tree_program(prog, n, a.prefix);
  __syncthreads();
  const int nsteps = __builtin_amdgcn_readfirstlane(s_nsteps);
  const long long row = (long long)blockIdx.x * 16 + rl;
  const long long rc = row < a.rows ? row : (long long)a.rows - 1;       // clamped: loads stay in bounds
  const float* e = a.e + rc * n * R + 4 * g;
  const float* lay = a.layers_nat + (size_t)(16 * wv + rl) * R + 4 * g;   // this wave's 16 rows of a layer
  const size_t lstep = a.L > 1 ? (size_t)R * R : 0;
  float* mine = nodes + (size_t)rl * RS + 4 * g;
  const float ninf = neg_inf();

  f32x4_t lw[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) lw[b] = *(const f32x4_t*)(a.logw + (rc / a.T) * R + 16 * b + 4 * g);

  // A step of the program, the same for every lane: kept in scalar registers.
  struct Step { int m, lsrc, rsrc, out; };
  auto read_step = [&](int t) {
    const int2 raw = *(const int2*)(prog + min(t, nsteps - 1));          // four shorts
    const int w0 = __builtin_amdgcn_readfirstlane(raw.x), w1 = __builtin_amdgcn_readfirstlane(raw.y);
    return Step{(short)(w0 & 0xffff), w0 >> 16, (short)(w1 & 0xffff), w1 >> 16};
  };
  // Operands of the two steps after the current one, in two register sets used alternately: leaf
  // evidence (from HBM: a full step of look-ahead is not enough to cover that) and this wave's
  // rows of the step's layer.
  f32x4_t nxl[2][NB], nxr[2][NB], An[2][NB];
  auto prefetch = [&](auto set, int t, const Step& s) {
    constexpr int P = decltype(set)::value;
    if (t >= nsteps) return;
    if (s.lsrc >= n - 1) {
#pragma unroll
      for (int b = 0; b < NB; ++b) nxl[P][b] = *(const f32x4_t*)(e + (size_t)(s.lsrc - (n - 1)) * R + 16 * b);
    }
    if (s.rsrc >= n - 1) {
#pragma unroll
      for (int b = 0; b < NB; ++b) nxr[P][b] = *(const f32x4_t*)(e + (size_t)(s.rsrc - (n - 1)) * R + 16 * b);
    }
    if (s.m > 0) {
      const float* A = lay + (size_t)(s.m - 1) * lstep;
#pragma unroll
      for (int b2 = 0; b2 < NB; ++b2) An[P][b2] = *(const f32x4_t*)(A + 16 * b2);
    }
  };
#pragma unroll
  for (int q = 0; q < 2; ++q)
#pragma unroll
    for (int b = 0; b < NB; ++b) nxl[q][b] = nxr[q][b] = An[q][b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // The lanes that share a row (l, l ^ 16, l ^ 32, l ^ 48) combine their values with the two lane
  // swaps of the vector unit: after swapping the odd 16-lane rows of one copy with the even rows of
  // another, the two copies hold both members of every pair; then the same for the 32-lane halves.
  auto both16 = [](float x, float& p, float& q) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    p = __uint_as_float(r[0]); q = __uint_as_float(r[1]);
  };
  auto both32 = [](float x, float& p, float& q) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    p = __uint_as_float(r[0]); q = __uint_as_float(r[1]);
  };
  auto row_max = [&](float x) { float p, q; both16(x, p, q); x = fmaxf(p, q); both32(x, p, q); return fmaxf(p, q); };
  auto row_sum = [&](float x) { float p, q; both16(x, p, q); x = p + q; both32(x, p, q); return p + q; };

  int pcur = 0;                      // slot (n - 1 + pcur) holds the current path value
  Step cur = read_step(0), nx1 = read_step(1);
  prefetch(std::integral_constant<int, 0>{}, 0, cur);
  prefetch(std::integral_constant<int, 1>{}, 1, nx1);

  // one step with the register set `set`; refills that set for step t + 2
  auto step = [&](auto set, int t) {
    constexpr int P = decltype(set)::value;
    const Step st = cur;
    const Step nx2 = read_step(t + 2);
    f32x4_t c[NB], Ac[NB];
    {
      const int lslot = st.lsrc == -1 ? n - 1 + pcur : st.lsrc;
      const int rslot = st.rsrc == -1 ? n - 1 + pcur : st.rsrc;
      f32x4_t lv[NB], rv[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        if (st.lsrc == -2) lv[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        else if (st.lsrc >= n - 1) lv[b] = nxl[P][b];
        else lv[b] = *(const f32x4_t*)(mine + (size_t)lslot * 16 * RS + 16 * b);
        if (st.rsrc == -2) rv[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        else if (st.rsrc >= n - 1) rv[b] = nxr[P][b];
        else rv[b] = *(const f32x4_t*)(mine + (size_t)rslot * 16 * RS + 16 * b);
        c[b] = lv[b] + rv[b];
        Ac[b] = An[P][b];
      }
    }
    prefetch(set, t + 2, nx2);
    cur = nx1;
    nx1 = nx2;
    if (st.m == 0) {
#pragma unroll
      for (int b = 0; b < NB; ++b) c[b] += lw[b];
    }
    float m = ninf;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) m = fmaxf(m, c[b][i]);
    m = row_max(m);
    const float ms = (m == ninf) ? 0.f : m;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) c[b][i] = __expf(c[b][i] - ms);        // exp(-inf) = 0; NaN stays NaN
    if (st.m == 0) {             // root: mixture with log omega (every wave computes it, the first one stores)
      float sum = 0.f;
#pragma unroll
      for (int b = 0; b < NB; ++b) sum += (c[b][0] + c[b][1]) + (c[b][2] + c[b][3]);
      sum = row_sum(sum);
      const float v = ms + __logf(sum);                                  // log 0 = -inf
      if (wv == 0 && g == 0 && row < a.rows) {
        if (a.prefix) a.out[row * n + (-2 - st.out)] = v; else a.out[row] = v;
      }
      return;                    // nothing stored in LDS: no barrier needed
    }
    f32x4_t S = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b2 = 0; b2 < NB; ++b2)
#pragma unroll
      for (int i = 0; i < 4; ++i) S = __builtin_amdgcn_mfma_f32_16x16x4f32(Ac[b2][i], c[b2][i], S, 0, 0, 0);
    f32x4_t res;
#pragma unroll
    for (int i = 0; i < 4; ++i) res[i] = ms + __logf(S[i]);
    // a node's slot is written once, before any step reads it; the path value goes to the slot
    // that no wave reads during this step
    const int oslot = st.out >= 0 ? st.out : n - 1 + (pcur ^ 1);
    *(f32x4_t*)(mine + (size_t)oslot * 16 * RS + 16 * wv) = res;
    if (st.out < 0) pcur ^= 1;
    if constexpr (NB > 1) __syncthreads();
  };
  for (int t = 0; t < nsteps; t += 2) {
    step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < nsteps) step(std::integral_constant<int, 1>{}, t + 1);
  }
}

static size_t btree_mfma_smem(const CircuitArgs& a) {
  if (a.layers_nat == nullptr || (a.r != 16 && a.r != 32 && a.r != 64)) return 0;
  return (size_t)(a.n + 1) * 16 * (a.r + 4) * 4 + (size_t)tree_program_steps(a.n, a.prefix) * sizeof(TreeStep);
}

template <int R>
static hipError_t launch_btree_mfma_r(const CircuitArgs& a, size_t smem, hipStream_t st) {
  if (hipError_t e = allow_lds<k_btree_mfma<R>>(150 * 1024); e != hipSuccess) return e;
  hipLaunchKernelGGL(k_btree_mfma<R>, dim3((unsigned)((a.rows + 15) / 16)), dim3(4 * R), smem, st, a);
  return hipGetLastError();
}

static hipError_t launch_btree_mfma(const CircuitArgs& a, size_t smem, hipStream_t st) {
  if (a.r == 64) return launch_btree_mfma_r<64>(a, smem, st);
  if (a.r == 32) return launch_btree_mfma_r<32>(a, smem, st);
  return launch_btree_mfma_r<16>(a, smem, st);
}

// rows per group of the program-driven tree kernel: 4 when that still gives every CU
// two workgroups, else 2 (twice the workgroups, half the LDS each)
static int btree_static_rb(const CircuitArgs& a) {
  int G = 1;
  while (G < a.r && G < 64) G <<= 1;
  return a.rows >= 8ll * (256 / G) * 512 ? 4 : 2;
}

// LDS the program-driven tree kernel needs (0: shape not supported by it)
static size_t btree_static_smem(const CircuitArgs& a) {
  if (a.r > 64) return 0;
  int G = 1;
  while (G < a.r && G < 64) G <<= 1;
  const int groups = 256 / G;
  return (2ull * a.r * a.r + (size_t)groups * btree_static_rb(a) * a.r * a.n) * 4 +
         (size_t)tree_program_steps(a.n, a.prefix) * sizeof(TreeStep);
}

static hipError_t launch_btree_static(const CircuitArgs& a, hipStream_t st) {
  int G = 1;
  while (G < a.r && G < 64) G <<= 1;
  const int groups = 256 / G;
  const int RB = btree_static_rb(a);
  const size_t smem = btree_static_smem(a);
  if (hipError_t e = RB == 4 ? allow_lds<k_btree_static<4>>(160 * 1024 - 64) : allow_lds<k_btree_static<2>>(160 * 1024 - 64);
      e != hipSuccess)
    return e;
  const long long ngroups = ((long long)a.rows + RB - 1) / RB;
  const dim3 grid((unsigned)((ngroups + groups - 1) / groups));
  if (RB == 4) hipLaunchKernelGGL(k_btree_static<4>, grid, dim3(256), smem, st, a, G);
  else hipLaunchKernelGGL(k_btree_static<2>, grid, dim3(256), smem, st, a, G);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Few rows (decode-sized calls): the HMM chain and the binary tree are chains of
// dependent r x r products, and with one group per row every product waits for its
// layer to come from L2.  Here ONE WORKGROUP owns a row: all layers of the row, its
// evidence and log omega are fetched into LDS with every load in flight at once, then
//  - binary tree: the nodes of a level are evaluated side by side by the workgroup's
//    groups (one barrier per level), and the n prefix marginals - each a walk from a
//    leaf to the root of at most log2 n products - are dealt to the groups;
//  - HMM: one group runs the forward recursion out of LDS.
// One unit per lane (r <= 64).  LDS: layers L*r*r + evidence n*r + nodes (n-1)*r +
// log omega r + one exchange row of r floats per group.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_circuit_row(const CircuitArgs a, int G) {
  extern __shared__ __align__(16) float rsm[];
  const int n = a.n, r = a.r, tid = threadIdx.x;
  const int NG = 256 / G, gi = tid / G, g = tid % G;
  const long long row = blockIdx.x;
  const long long pos = row / a.T;
  const int Lst = a.L;                                   // stored layers (1: shared by all steps / nodes)
  const int lstep = Lst > 1 ? r * r : 0;
  float* s_lay = rsm;                                    // [Lst][j][k]
  float* s_ev = s_lay + (size_t)Lst * r * r;             // [n][r]
  float* s_nodes = s_ev + (size_t)n * r;                 // [n-1][r] (binary tree)
  float* s_lw = s_nodes + (size_t)(n - 1) * r;           // [r]
  float* s_sh = s_lw + r + (size_t)gi * r;               // this group's exchange row
  int* s_bad = (int*)(s_lw + r + (size_t)NG * r);

  const float* lay = a.layers;
  if (a.contextual && lay) lay += pos * (long long)Lst * r * r;
  const float* ev = a.e + row * (long long)n * r;
  const int nlay = lay ? Lst * r * r : 0;
  if ((nlay & 3) == 0 && (((size_t)lay) & 15) == 0) {
    // 16-byte loads, four per thread in flight
    const float4* src = (const float4*)lay;
    float4* dst = (float4*)s_lay;
    const int nq = nlay >> 2;
    for (int t0 = 0; t0 < nq; t0 += 4 * 256) {
      float4 tmp[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) tmp[u] = src[min(t0 + u * 256 + tid, nq - 1)];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (t0 + u * 256 + tid < nq) dst[t0 + u * 256 + tid] = tmp[u];
    }
  } else {
    for (int t0 = 0; t0 < nlay; t0 += 8 * 256) {         // eight loads per thread in flight
      float tmp[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) tmp[u] = lay[min(t0 + u * 256 + tid, nlay - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (t0 + u * 256 + tid < nlay) s_lay[t0 + u * 256 + tid] = tmp[u];
    }
  }
  for (int t = tid; t < n * r; t += 256) s_ev[t] = ev[t];
  if (tid < r) s_lw[tid] = a.logw[pos * r + tid];
  __syncthreads();
  // an id outside [-1, v) left NaN in every unit of its window position: poison what observes it
  if (gi == 0) {
    const int fb = first_nan_position(s_ev, n, r, g, G);
    if (g == 0) *s_bad = fb;
  }
  __syncthreads();
  const int first_bad = *s_bad;
  const float ninf = neg_inf();
  auto emit = [&](int i, float v) {
    if (g != 0) return;
    if (i >= first_bad) v = __builtin_nanf("");
    if (a.prefix) a.out[row * n + i] = v;
    else if (i == n - 1) a.out[row] = v;
  };
  auto lse = [&](float x) {
    const float m = group_max(x, G);
    if (m == ninf) return m;
    return m + __logf(group_sum(g < r ? __expf(x - m) : 0.f, G));
  };
  auto leaf = [&](int i) { return g < r ? s_ev[i * r + g] : ninf; };
  const float lw = g < r ? s_lw[g] : ninf;

  if (a.family == MTPC_HMM) {
    if (gi != 0) return;                                 // (no workgroup barrier below)
    // the message stays relative to its largest unit, the magnitude taken out is summed in double
    float alpha[1] = {lw + leaf(0)};
    double scale = 0.0;
    for (int i = 0; i < n; ++i) {
      if (i > 0) {
        sum_layer_lds<1>(alpha, s_lay + (size_t)(i - 1) * lstep, s_sh, g, r, G);
        alpha[0] += leaf(i);
      }
      const float m = group_max(alpha[0], G);
      if (m != ninf) { alpha[0] -= m; scale += (double)m; }
      if (a.prefix || i == n - 1)                        // largest unit 0 (or all -inf: log 0)
        emit(i, (float)(scale + (double)__logf(group_sum(g < r ? __expf(alpha[0]) : 0.f, G))));
    }
    return;
  }

  // ---- binary tree, heap order: inner nodes 0..n-2, leaf i at n-1+i
  auto full_value = [&](int c) {                         // child fully observed
    if (c >= n - 1) return leaf(c - (n - 1));
    return g < r ? s_nodes[c * r + g] : ninf;
  };
  for (int lo = (n >> 1) - 1; lo >= 1; lo = (lo - 1) >> 1) {   // levels bottom-up: nodes lo .. 2*lo
    for (int m = lo + gi; m <= 2 * lo; m += NG) {
      float c[1] = {full_value(2 * m + 1) + full_value(2 * m + 2)};
      sum_layer_lds<1>(c, s_lay + (size_t)(m - 1) * lstep, s_sh, g, r, G);
      if (g < r) s_nodes[m * r + g] = c[0];
    }
    __syncthreads();
  }
  if (!a.prefix) {
    if (gi == 0) emit(n - 1, lse(full_value(1) + full_value(2) + lw));
    return;
  }
  // prefix i: a subtree without observed leaf is 1, a fully observed one its stored value;
  // only the nodes whose leaf range straddles the boundary are evaluated again
  for (int i = gi; i < n; i += NG) {
    float pv = 0.f;                 // value of the straddling child on the path so far
    int idx = n - 1 + i, size = 1;
    while (idx > 0) {
      const int m = (idx - 1) >> 1;
      size <<= 1;
      const int first = (m - (n / size - 1)) * size, last = first + size - 1;
      if (m > 0 && last <= i) { idx = m; continue; }
      const int cl = 2 * m + 1, cr = cl + 1, half = size >> 1;
      const int l_last = first + half - 1, r_first = first + half;
      const float lv = (l_last <= i) ? full_value(cl) : pv;
      const float rv = (r_first > i) ? (g < r ? 0.f : ninf) : (last <= i ? full_value(cr) : pv);
      float c[1] = {lv + rv};
      if (m > 0) {
        sum_layer_lds<1>(c, s_lay + (size_t)(m - 1) * lstep, s_sh, g, r, G);
        pv = c[0];
      } else {
        emit(i, lse(c[0] + lw));
      }
      idx = m;
    }
  }
}

// LDS of k_circuit_row in bytes (0: the shape is not served)
static size_t circuit_row_smem(const CircuitArgs& a, int G) {
  if (a.r > 64 || (a.family != MTPC_HMM && a.family != MTPC_BTREE)) return 0;
  const int L = a.family == MTPC_HMM ? a.n - 1 : a.n - 2;
  if (L > 0 && !a.layers) return 0;
  const size_t fl = (size_t)(L > 0 ? a.L : 0) * a.r * a.r + (size_t)a.n * a.r + (size_t)(a.n - 1) * a.r + a.r +
                    (size_t)(256 / G) * a.r + 4;
  return fl * 4;
}

static hipError_t launch_circuit_row(const CircuitArgs& a, int G, size_t smem, hipStream_t st) {
  static size_t attr = 0;                                // largest dynamic LDS size granted so far
  if (smem > attr) {
    hipError_t e = hipFuncSetAttribute((const void*)k_circuit_row, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)smem);
    if (e != hipSuccess) return e;
    attr = smem;
  }
  hipLaunchKernelGGL(k_circuit_row, dim3((unsigned)a.rows), dim3(256), smem, st, a, G);
  return hipGetLastError();
}

hipError_t launch_circuit(const CircuitArgs& a, hipStream_t st) {
  // decode-sized calls of the families with r x r layers: one workgroup per row
  if (a.rows <= 2048 && (a.family == MTPC_HMM || a.family == MTPC_BTREE)) {
    int G = 1;
    while (G < a.r && G < 64) G <<= 1;
    const size_t need = circuit_row_smem(a, G);
    if (need != 0 && need <= 144 * 1024) return launch_circuit_row(a, G, need, st);
  }
  // batching rows pays when sum layers are shared and there are rows to batch;
  // the batched BTree node store must still fit one group into 48 KiB of LDS
  // (measured: the tree's many dependent node evaluations gain from sharing weight
  // loads; the HMM chain prefers more, narrower groups)
  if (a.family == MTPC_BTREE && !a.contextual && a.n > 2 && a.rows >= 256) {
    const size_t mfma = btree_mfma_smem(a);
    if (mfma != 0 && mfma <= 150 * 1024) return launch_btree_mfma(a, mfma, st);
    const size_t need = btree_static_smem(a);
    if (need != 0 && need <= 150 * 1024) return launch_btree_static(a, st);
  }
  const size_t one_group4 = 4ull * 4 * (a.r + (size_t)(a.n - 1) * a.r);
  if (a.family == MTPC_BTREE && !a.contextual && a.rows >= 1024 && one_group4 <= 48 * 1024)
    return launch_circuit_rb<4>(a, st);
  return launch_circuit_rb<1>(a, st);
}

// ---------------------------------------------------------------------------
// latent draws (Alg. 1): one wave per draft.  Lane l holds the weights of units l
// and l+64; the CDF is an inclusive scan in double, the draw the first lane whose
// partial sum exceeds the uniform (the smallest k with u < p_0+..+p_k), else the
// last unit with positive weight.  The result is wave-uniform, so the next sum
// unit's row is again one coalesced load.
// ---------------------------------------------------------------------------
// Inclusive scan over the 64 lanes in double.  Inside a row of 16 lanes the four steps are DPP
// row shifts (lanes without a source read zero), then the row totals travel over the LDS crossbar:
// the last lane of the previous row, and after that the last lane of the row before it, which by
// then holds the total of two rows.
template <int CTRL>
__device__ __forceinline__ double dpp_move_f64(double x) {
  const long long v = __double_as_longlong(x);
  const unsigned lo = (unsigned)dpp_move<CTRL>((int)(unsigned)(v & 0xffffffffll));
  const unsigned hi = (unsigned)dpp_move<CTRL>((int)(unsigned)((unsigned long long)v >> 32));
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ double wave_scan_incl(double x, int lane) {
  x += dpp_move_f64<0x111>(x);      // row_shr:1
  x += dpp_move_f64<0x112>(x);      // row_shr:2
  x += dpp_move_f64<0x114>(x);      // row_shr:4
  x += dpp_move_f64<0x118>(x);      // row_shr:8
  const int row = lane >> 4;
  const double t1 = __shfl(x, max(16 * row - 1, 0));
  if (row >= 1) x += t1;
  const double t2 = __shfl(x, max(16 * row - 17, 0));
  if (row >= 2) x += t2;
  return x;
}
__device__ __forceinline__ int wave_draw(float p0, float p1, int r, float u, int lane) {
  const bool in0 = lane < r, in1 = lane + 64 < r;
  const double c0 = wave_scan_incl(in0 ? (double)p0 : 0.0, lane);
  unsigned long long m = __ballot(in0 && (double)u < c0);
  if (m) return __ffsll((long long)m) - 1;
  if (r > 64) {
    const double c1 = __shfl(c0, 63) + wave_scan_incl(in1 ? (double)p1 : 0.0, lane);
    m = __ballot(in1 && (double)u < c1);
    if (m) return 64 + __ffsll((long long)m) - 1;
    m = __ballot(in1 && p1 > 0.f);
    if (m) return 64 + 63 - __clzll((long long)m);
  }
  m = __ballot(in0 && p0 > 0.f);
  return m ? 63 - __clzll((long long)m) : 0;
}

// index of the largest of the r weights (lane holds units lane and lane + 64); ties: smallest index
__device__ __forceinline__ int wave_argmax(float p0, float p1, int r, int lane) {
  float best = lane < r ? p0 : -1.f;
  int arg = lane;
  if (lane + 64 < r && p1 > best) { best = p1; arg = lane + 64; }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float ob = __shfl_xor(best, o);
    const int oa = __shfl_xor(arg, o);
    if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
  }
  return arg;
}

// the latents of draft (b, s) by one wave; lw: the position's log omega (global or LDS)
__device__ void draft_latents(const LatentArgs& a, int b, int s, const float* lw, int lane) {
  const long long t = (long long)b * a.S + s;
  const int n = a.n, r = a.r;
  int* zl = a.zleaf + t * n;
  const float* lay = a.layers;
  if (a.contextual && lay) lay += (long long)b * a.L * r * r;
  const long long lstep = (a.L > 1) ? (long long)r * r : 0;
  auto U = [&](int lat) {
    return philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, (uint32_t)s, (uint32_t)(n + lat));
  };
  auto draw_row = [&](const float* row, int lat) {      // row of normalised linear weights
    const float p0 = lane < r ? row[lane] : 0.f;
    const float p1 = lane + 64 < r ? row[lane + 64] : 0.f;
    return a.greedy ? wave_argmax(p0, p1, r, lane) : wave_draw(p0, p1, r, U(lat), lane);
  };
  const float q0 = lane < r ? expf(lw[lane]) : 0.f, q1 = lane + 64 < r ? expf(lw[lane + 64]) : 0.f;
  const int z0 = a.greedy ? wave_argmax(q0, q1, r, lane) : wave_draw(q0, q1, r, U(0), lane);
  if (a.family == MTPC_CP) {
    for (int i = lane; i < n; i += 64) zl[i] = z0;
    if (a.latents && lane == 0) a.latents[t] = z0;
  } else if (a.family == MTPC_HMM) {
    int z = z0;
    for (int i = 0; i < n; ++i) {
      if (i > 0) z = draw_row(lay + (long long)(i - 1) * lstep + (long long)z * r, i);
      if (lane == 0) { zl[i] = z; if (a.latents) a.latents[t * n + i] = z; }
    }
  } else {
    // BTree: node m's latent given its parent's (heap order); the state that
    // indexes leaf i is the latent of its parent node (n-2+i)/2.  `latents` is
    // always a valid buffer here (the caller's or library scratch); lane m % 64
    // keeps node m's latent for its children.
    int* L = a.latents + t * (n - 1);
    int mine = z0;                                      // latent of node `lane` (n - 1 <= 63 nodes)
    for (int m = 1; m < n - 1; ++m) {
      const int zp = __shfl(mine, (m - 1) >> 1);
      const int z = draw_row(lay + (long long)(m - 1) * lstep + (long long)zp * r, m);
      if (lane == m) mine = z;
    }
    if (lane < n - 1) L[lane] = mine;
    for (int i = lane; i < n; i += 64) zl[i] = __shfl(mine, (n - 2 + i) >> 1);
  }
}

__global__ __launch_bounds__(256) void k_latents(const LatentArgs a) {
  const int lane = threadIdx.x & 63;
  if (a.zero != nullptr)
    for (long long g = (long long)blockIdx.x * 256 + threadIdx.x; g < a.nzero; g += (long long)gridDim.x * 256) a.zero[g] = 0;
  const long long t = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);     // draft index
  if (t >= (long long)a.B * a.S) return;
  const int b = (int)(t / a.S), s = (int)(t % a.S);
  if (a.family == MTPC_FF) {
    int* zl = a.zleaf + t * a.n;
    for (int i = lane; i < a.n; i += 64) zl[i] = 0;
    return;
  }
  draft_latents(a, b, s, a.logw + (long long)b * a.r, lane);
}

hipError_t launch_latents(const LatentArgs& a, hipStream_t st) {
  const long long tot = (long long)a.B * a.S;
  hipLaunchKernelGGL(k_latents, dim3((unsigned)((tot + 3) / 4)), dim3(256), 0, st, a);
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
// evidence of drafted tokens read from the table of normalised input units the sampling
// pass wrote: e[(b*S+s)][i][j] = logphi[b][i][j][x]
__global__ __launch_bounds__(256) void k_gather_table(const GatherArgs a, const float* logphi) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long total = (long long)a.B * a.S * a.n * a.r;
  if (t >= total) return;
  const int j = (int)(t % a.r);
  const long long bsi = t / a.r;
  const int i = (int)(bsi % a.n);
  const long long b = bsi / a.n / a.S;
  const int x = a.x[bsi];
  float v;
  if (x >= 0 && x < a.v) v = logphi[((b * a.n + i) * a.r + j) * a.v + x];
  else v = (x == -1) ? 0.f : __builtin_nanf("");
  a.e[t] = v;
}

hipError_t launch_gather_table(const GatherArgs& a, const float* logphi, hipStream_t st) {
  const long long total = (long long)a.B * a.S * a.n * a.r;
  hipLaunchKernelGGL(k_gather_table, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, logphi);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Token draws of Alg. 1 from the table of normalised input units (large batches: the fused
// kernel only writes the table, the draws read one row each).  One wave per token; lane l
// holds tokens 5l..5l+4 (v <= 320), the CDF is an ordered scan over lanes, the draw the
// smallest k with u * total < cdf[k], else the last token with positive mass.
__global__ __launch_bounds__(256) void k_draw_table(const DrawArgs a) {
  constexpr int VPL = 5;
  const int lane = threadIdx.x & 63;
  const long long di = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);   // (b, s, i) flattened
  if (di >= (long long)a.B * a.S * a.n) return;
  const int i = (int)(di % a.n);
  const long long bs = di / a.n;
  const long long b = bs / a.S;
  const int s = (int)(bs - b * a.S);
  const int z = a.zleaf[di];
  // rows of the full table, or (compact) one row of unnormalised logits per token
  const float* row = a.compact ? a.logphi + di * a.v : a.logphi + ((b * a.n + i) * a.r + z) * a.v;
  float lg[VPL], vals[VPL];
  float mx = neg_inf();
#pragma unroll
  for (int q = 0; q < VPL; ++q) {
    const int k = lane * VPL + q;
    lg[q] = k < a.v ? row[k] : neg_inf();
    mx = fmaxf(mx, lg[q]);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  if (!a.compact) mx = 0.f;   // rows of the table are normalised (and may be all -inf)
  float ls = 0.f;
#pragma unroll
  for (int q = 0; q < VPL; ++q) {
    vals[q] = lane * VPL + q < a.v ? expf(lg[q] - mx) : 0.f;
    ls += vals[q];
  }
  if (a.greedy) {
    float best = neg_inf();   // lanes past the vocabulary keep -inf and never win
    int arg = 0;
#pragma unroll
    for (int q = 0; q < VPL; ++q)
      if (lg[q] > best) { best = lg[q]; arg = lane * VPL + q; }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      const float ob = __shfl_xor(best, o);
      const int oa = __shfl_xor(arg, o);
      if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    }
    if (lane == 0) a.drafts[di] = arg;
    return;
  }
  float incl = ls;   // inclusive scan over lanes
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  const float Z = __shfl(incl, 63);
  const float u = philox_uniform(a.seed_lo, a.seed_hi, a.offset, (uint32_t)b, (uint32_t)s, (uint32_t)i);
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
    if (lane == L) a.drafts[di] = tok;
  } else {
    int last = -1;
#pragma unroll
    for (int q = 0; q < VPL; ++q)
      if (vals[q] > 0.f) last = lane * VPL + q;
    const unsigned long long pos = __ballot(last >= 0);
    const int L = 63 - __clzll((long long)pos);
    if (lane == L) a.drafts[di] = last;
  }
}

// ---------------------------------------------------------------------------
// Very few drafts (2 B S <= r): a draft only needs the logits of the one input unit each of
// its tokens is drawn from, n of the n*r slabs of W.  One workgroup computes 16 logits of one
// token, W[i][z][16 rows] . h[b], as plain dot products (its 4 waves take 4 rows each, the
// hidden vector stays in registers); the rows go to a compact table [B*S*n][v] that
// k_draw_table reads.  B*S*n*v*d products and as many bytes of W instead of a pass over all of it.
// ---------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void k_rows_logits(const RowLogitArgs a) {
  constexpr int ESZ = BF16 ? 2 : 4;
  constexpr int EPC = 16 / ESZ;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long di = blockIdx.x;                       // (b, s, i) flattened
  const int i = (int)(di % a.n);
  const long long b = di / a.n / a.S;
  const int z = min(max(a.zleaf[di], 0), a.r - 1);
  const char* hb = (const char*)a.h + b * a.ld_h * ESZ;
  const char* Wz = (const char*)a.W + ((long long)(i * a.r + z) * a.v) * a.d * ESZ;
  const int row0 = blockIdx.y * 16 + wave * 4;
  const int nch = a.d / EPC;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < nch; c0 += 512) {
    i32x4_t hv[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int c = c0 + t * 64 + lane;
      const i32x4_t x = *(const i32x4_t*)(hb + (long long)min(c, nch - 1) * 16);
      hv[t] = c < nch ? x : i32x4_t{0, 0, 0, 0};
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const char* wr = Wz + (long long)min(row0 + q, a.v - 1) * a.d * ESZ;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        // unconditional (clamped) loads so that all of them are in flight together;
        // chunks beyond d meet a zero hv
        const int c = min(c0 + t * 64 + lane, nch - 1);
        acc[q] += dot_chunk<BF16>(*(const i32x4_t*)(wr + (long long)c * 16), hv[t]);
      }
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float val = wave_sum(acc[q]);
    if (lane == 0 && row0 + q < a.v) a.out[di * a.v + row0 + q] = val;
  }
}

hipError_t launch_rows_logits(const RowLogitArgs& a, int dtype, hipStream_t st) {
  const dim3 grid((unsigned)((long long)a.B * a.S * a.n), (unsigned)((a.v + 15) / 16));
  if (dtype == MTPC_BF16) hipLaunchKernelGGL(k_rows_logits<true>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(k_rows_logits<false>, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Gradient of the sum-unit matrix (Sec. 4.1 loss): dWsum[j][c] = sum_b g[j][b] hT[c][b], with the
// gradient of the sum-unit logits g [r][ldb] and the transposed hidden states hT [d][ldb] both
// contiguous over the (zero-padded) positions.  r*d dot products of length B: a workgroup takes
// 4 columns c, each of its waves 4 rows j at a time; sums in a fixed order.
template <bool BF16>
__global__ __launch_bounds__(256) void k_dwsum(const void* gT, const void* hT, long long ldb, int r, int d,
                                               float* out) {
  constexpr int ESZ = BF16 ? 2 : 4;
  constexpr int CT = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = blockIdx.x * CT;
  const long long pitch = ldb * ESZ;
  const int nch = (int)(pitch / 16);
  for (int j0 = wave * 4; j0 < r; j0 += 16) {
    float acc[4][CT];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int q = 0; q < CT; ++q) acc[u][q] = 0.f;
#pragma unroll 2
    for (int t = lane; t < nch; t += 64) {
      i32x4_t hv[CT];
#pragma unroll
      for (int q = 0; q < CT; ++q) hv[q] = *(const i32x4_t*)((const char*)hT + (long long)min(c0 + q, d - 1) * pitch + (long long)t * 16);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const i32x4_t gv = *(const i32x4_t*)((const char*)gT + (long long)min(j0 + u, r - 1) * pitch + (long long)t * 16);
#pragma unroll
        for (int q = 0; q < CT; ++q) acc[u][q] += dot_chunk<BF16>(gv, hv[q]);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int q = 0; q < CT; ++q) {
        const float val = wave_sum(acc[u][q]);
        if (lane == 0 && j0 + u < r && c0 + q < d) out[(long long)(j0 + u) * d + c0 + q] = val;
      }
  }
}

hipError_t launch_dwsum(const void* gT, const void* hT, long long ldb, int r, int d, int dtype, float* out,
                        hipStream_t st) {
  const dim3 grid((unsigned)((d + 3) / 4));
  if (dtype == MTPC_BF16) hipLaunchKernelGGL(k_dwsum<true>, grid, dim3(256), 0, st, gT, hT, ldb, r, d, out);
  else hipLaunchKernelGGL(k_dwsum<false>, grid, dim3(256), 0, st, gT, hT, ldb, r, d, out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Univariate marginals (App. B.1) from the table of normalised input units:
//   M[b][i][a] = log sum_j exp(logm[b][i][j] + log phi[b][i][j][a]).
// One wave per (b, i); lane l holds tokens l, l + 64, ...; the r rows of the table are read
// once, front to back (whole 256-byte segments), into a running maximum and a sum relative to it.
__global__ __launch_bounds__(256) void k_univariate_table(const float* logphi, const float* logm, float* out,
                                                          long long tokens, int r, int v) {
  constexpr int VPL = 5;                      // v <= 320
  const int lane = threadIdx.x & 63;
  const long long t = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);       // (b, i) flattened
  if (t >= tokens) return;
  const float* rows = logphi + t * r * v;
  float m[VPL], s[VPL];
#pragma unroll
  for (int q = 0; q < VPL; ++q) { m[q] = neg_inf(); s[q] = 0.f; }
  constexpr int JB = 4;                       // rows fetched together
  for (int j0 = 0; j0 < r; j0 += JB) {
    float x[JB][VPL];
#pragma unroll
    for (int u = 0; u < JB; ++u) {
      const int j = min(j0 + u, r - 1);
      const float lm = (j0 + u < r) ? (logm ? logm[t * r + j] : 0.f) : neg_inf();
#pragma unroll
      for (int q = 0; q < VPL; ++q) {
        const int k = lane + 64 * q;
        x[u][q] = lm + rows[(long long)j * v + min(k, v - 1)];
      }
    }
#pragma unroll
    for (int q = 0; q < VPL; ++q) {
      float mm = m[q];
#pragma unroll
      for (int u = 0; u < JB; ++u) mm = fmaxf(mm, x[u][q]);
      if (mm == neg_inf()) continue;          // only terms of probability zero so far
      float ss = s[q] * __expf(m[q] - mm);    // (m = -inf: s = 0, exp(-inf) = 0)
#pragma unroll
      for (int u = 0; u < JB; ++u) ss += __expf(x[u][q] - mm);
      m[q] = mm;
      s[q] = ss;
    }
  }
#pragma unroll
  for (int q = 0; q < VPL; ++q) {
    const int k = lane + 64 * q;
    if (k < v) out[t * v + k] = s[q] > 0.f ? m[q] + __logf(s[q]) : neg_inf();
  }
}

hipError_t launch_univariate_table(const UnivariateArgs& a, const float* logphi, hipStream_t st) {
  const long long tokens = (long long)a.B * a.n;
  hipLaunchKernelGGL(k_univariate_table, dim3((unsigned)((tokens + 3) / 4)), dim3(256), 0, st, logphi, a.logm, a.out,
                     tokens, a.r, a.v);
  return hipGetLastError();
}

hipError_t launch_draw_table(const DrawArgs& a, hipStream_t st) {
  const long long rows = (long long)a.B * a.S * a.n;
  hipLaunchKernelGGL(k_draw_table, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Bucketing of the token draws by (token index, selected input unit).  Three small kernels:
// clear the counters; count (the value an atomic returns is the triple's rank in its
// bucket); one workgroup turns the counts into row and tile offsets; fill the lists.
__global__ __launch_bounds__(256) void k_bucket_clear(int* count, int ng) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < ng) count[t] = 0;
}

// Ranks are taken inside a workgroup first (LDS counters), then every non-empty bucket of
// the workgroup reserves its range with one global atomic: B*S*n / 1024 * (buckets hit)
// global atomics instead of B*S*n on n*r addresses.
__global__ __launch_bounds__(1024) void k_bucket_count(const BucketArgs a) {
  extern __shared__ int s_count[];                   // [n*r]
  const int ng = a.n * a.r;
  for (int g = threadIdx.x; g < ng; g += 1024) s_count[g] = 0;
  __syncthreads();
  const long long t = (long long)blockIdx.x * 1024 + threadIdx.x;
  const bool live = t < (long long)a.B * a.S * a.n;
  int g = 0, rank = 0;
  if (live) {
    const int i = (int)(t % a.n);
    g = i * a.r + min(max(a.zleaf[t], 0), a.r - 1);
    rank = atomicAdd(&s_count[g], 1);
  }
  __syncthreads();
  for (int k = threadIdx.x; k < ng; k += 1024) {
    const int c = s_count[k];
    if (c > 0) s_count[k] = atomicAdd(&a.count[k], c);
  }
  __syncthreads();
  if (live) a.slot[t] = s_count[g] + rank;
}

__global__ __launch_bounds__(256) void k_bucket_offsets(const BucketArgs a) {
  __shared__ int s_rows[256], s_tiles[256];
  const int ng = a.n * a.r, tid = threadIdx.x;
  const int per = (ng + 255) / 256;                  // consecutive buckets per thread
  const int g0 = min(tid * per, ng), g1 = min(g0 + per, ng);
  int rows = 0, tiles = 0;
  for (int g = g0; g < g1; ++g) {
    const int c = a.count[g];
    rows += c;
    tiles += (c + a.tile - 1) / a.tile;
  }
  s_rows[tid] = rows;
  s_tiles[tid] = tiles;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {                // inclusive scan
    const int r2 = tid >= o ? s_rows[tid - o] : 0, t2 = tid >= o ? s_tiles[tid - o] : 0;
    __syncthreads();
    s_rows[tid] += r2;
    s_tiles[tid] += t2;
    __syncthreads();
  }
  int ro = s_rows[tid] - rows, to = s_tiles[tid] - tiles;
  for (int g = g0; g < g1; ++g) {
    const int c = a.count[g];
    a.row_off[g] = ro;
    a.tile_off[g] = to;
    ro += c;
    to += (c + a.tile - 1) / a.tile;
  }
  if (tid == 255) {
    a.row_off[ng] = s_rows[255];
    a.tile_off[ng] = s_tiles[255];
  }
}

__global__ __launch_bounds__(256) void k_bucket_fill(const BucketArgs a) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)a.B * a.S * a.n) return;
  const int i = (int)(t % a.n);
  const int z = min(max(a.zleaf[t], 0), a.r - 1);
  const int g = i * a.r + z, slot = a.slot[t];
  a.list[a.row_off[g] + slot] = (int)(t / a.n);
  if (slot % a.tile == 0) a.tile_bucket[a.tile_off[g] + slot / a.tile] = g;   // the first row of a tile names its bucket
}

hipError_t launch_buckets(const BucketArgs& a, hipStream_t st) {
  const int ng = a.n * a.r;
  const long long rows = (long long)a.B * a.S * a.n;
  const unsigned gb = (unsigned)((rows + 255) / 256);
  if (!a.cleared) hipLaunchKernelGGL(k_bucket_clear, dim3((ng + 255) / 256), dim3(256), 0, st, a.count, ng);
  hipLaunchKernelGGL(k_bucket_count, dim3((unsigned)((rows + 1023) / 1024)), dim3(1024), (size_t)ng * 4, st, a);
  hipLaunchKernelGGL(k_bucket_offsets, dim3(1), dim3(256), 0, st, a);
  hipLaunchKernelGGL(k_bucket_fill, dim3(gb), dim3(256), 0, st, a);
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
