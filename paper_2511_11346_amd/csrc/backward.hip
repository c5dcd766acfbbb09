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
__device__ __forceinline__ float wsum(float x) { return group_sum(x, 64); }
__device__ __forceinline__ float wmax(float x) { return group_max(x, 64); }

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
  for (int k0 = 0; k0 < 16; ++k0) {
    const int c = c0 + ty + 4 * k0, r = r0 + tx;
    if (c < a.C && r < a.Rpad) {
      constexpr int EPS = 64 / (int)sizeof(T);         // elements of a row per stage
      const long long k = a.col0 + r;
      if (a.stage_rows) dst[(k / EPS * a.stage_rows + c) * EPS + k % EPS] = tile[tx][ty + 4 * k0];
      else dst[(long long)c * a.ld_dst + k] = tile[tx][ty + 4 * k0];
    }
  }
}

// The same with 16-byte accesses on both sides (VE = 16 / sizeof(T) elements per thread);
// needs 16-byte aligned rows on both sides (checked by the launcher).
template <typename T>
__global__ __launch_bounds__(256) void k_transpose_vec(const TransposeArgs a) {
  constexpr int VE = 16 / sizeof(T);
  constexpr int TPR = 64 / VE;                       // threads per tile row
  struct alignas(16) Vec { T v[VE]; };
  __shared__ T tile[64][64 + VE + (sizeof(T) == 2 ? 2 : 1)];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int tx = threadIdx.x % TPR, ty = threadIdx.x / TPR;
  const T* src = (const T*)a.src;
  T* dst = (T*)a.dst;
  for (int rr = ty; rr < 64; rr += 256 / TPR) {
    const int r = r0 + rr, c = c0 + tx * VE;
    Vec x;
#pragma unroll
    for (int t = 0; t < VE; ++t) x.v[t] = 0;
    if (r < a.R) {
      if (c + VE <= a.C) x = *(const Vec*)(src + (long long)r * a.ld_src + c);
      else
        for (int t = 0; t < VE; ++t)
          if (c + t < a.C) x.v[t] = src[(long long)r * a.ld_src + c + t];
    }
#pragma unroll
    for (int t = 0; t < VE; ++t) tile[rr][tx * VE + t] = x.v[t];
  }
  __syncthreads();
  for (int cc = ty; cc < 64; cc += 256 / TPR) {
    const int c = c0 + cc, r = r0 + tx * VE;
    if (c >= a.C) continue;
    Vec x;
#pragma unroll
    for (int t = 0; t < VE; ++t) x.v[t] = tile[tx * VE + t][cc];
    constexpr int EPS = 64 / (int)sizeof(T);           // elements of a row per stage (a multiple of VE)
    const long long k = a.col0 + r;
    T* o = a.stage_rows ? dst + (k / EPS * a.stage_rows + c) * EPS + k % EPS : dst + (long long)c * a.ld_dst + k;
    if (r + VE <= a.Rpad) *(Vec*)o = x;
    else
      for (int t = 0; t < VE; ++t)
        if (r + t < a.Rpad) o[t] = x.v[t];
  }
}

// 64 (m) x 128 (b) tiles: logit gradient from the stored probabilities, written in both
// layouts (dLT along b straight away, dL along m after a transpose through LDS).  A thread
// moves four neighbouring elements at a time (16-byte loads, 8- or 16-byte stores).
template <typename T>
__global__ __launch_bounds__(256) void k_grad_from_phi(const GradPhiArgs a) {
  struct alignas(4 * sizeof(T)) Quad { T v[4]; };
  __shared__ T tile[64][128 + 4];
  const long long m0 = (long long)blockIdx.y * 64;
  const int b0 = blockIdx.x * 128;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 column quads x 8 rows per pass
  const int b = b0 + 4 * tx;                                    // first of the thread's four positions
  T* dLT = (T*)a.dLT;
  T* dL = (T*)a.dL;
  auto conv = [](float x) -> T {
    if constexpr (sizeof(T) == 2) return to_bf16_rne(x); else return x;
  };
  const bool col_ok = b < a.ldb;                                // ldb is a multiple of 4: all four or none
  int cur_slab = -1, x[4] = {-1, -1, -1, -1};
  float g[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
  for (int k = 0; k < 8; ++k) {
    const int ml = ty + 8 * k;
    const long long m = m0 + ml;
    Quad out;
#pragma unroll
    for (int c = 0; c < 4; ++c) out.v[c] = conv(0.f);
    if (m < a.M && col_ok) {
      const int slab = (int)(m / a.v), av = (int)(m - (long long)slab * a.v);
      if (slab != cur_slab) {                      // rows of a tile mostly share their slab
        cur_slab = slab;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          x[c] = -1; g[c] = 0.f;
          if (b + c < a.B) {
            x[c] = a.targets[(long long)(b + c) * a.n + slab / a.r];
            g[c] = a.Ge[(long long)(b + c) * a.n * a.r + slab];
          }
        }
      }
      // (the probabilities are read once, here: as a stream)
      typedef __attribute__((ext_vector_type(4))) float f32x4_t;
      const f32x4_t ph = __builtin_nontemporal_load((const f32x4_t*)(a.phiT + m * a.ld_phi + b));
      const float pv[4] = {ph[0], ph[1], ph[2], ph[3]};
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (b + c < a.B && x[c] != -1) out.v[c] = conv(g[c] * ((av == x[c] ? 1.f : 0.f) - pv[c]));
      constexpr int EPS = 64 / (int)sizeof(T);     // elements of a row per stage (b is a multiple of 4)
      if (a.staged) *(Quad*)(dLT + ((long long)(b / EPS) * a.M + m) * EPS + b % EPS) = out;
      else *(Quad*)(dLT + m * a.ldb + b) = out;
    } else if (m < a.Mx && col_ok) {
      out = *(const Quad*)(dLT + m * a.ldb + b);   // sum-unit rows, written by the reverse pass
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) tile[ml][4 * tx + c] = out.v[c];
  }
  __syncthreads();
  const int mq = threadIdx.x & 15, br = threadIdx.x >> 4;        // 16 row quads x 16 positions per pass
#pragma unroll 2
  for (int k = 0; k < 8; ++k) {
    const int bl = br + 16 * k;
    const long long m = m0 + 4 * mq;
    if (b0 + bl < a.B && m < a.dl_end) {                        // dl_end is a multiple of 4
      Quad out;
#pragma unroll
      for (int c = 0; c < 4; ++c) out.v[c] = tile[4 * mq + c][bl];
      constexpr int EPS = 64 / (int)sizeof(T);
      if (a.staged) *(Quad*)(dL + ((m / EPS) * a.B + (b0 + bl)) * EPS + m % EPS) = out;
      else *(Quad*)(dL + (long long)(b0 + bl) * a.ldM + m) = out;
    }
  }
}

// acc_u = sum_k sh[k] * M[k*r + unit_u] for the lane's units (lane, lane + 64); M is an
// r x r matrix in global memory read along its contiguous axis, eight rows in flight.
__device__ __forceinline__ void wave_matvec(const float* __restrict__ M, const float* sh, int r, int lane,
                                            float& acc0, float& acc1) {
  const bool u1 = lane + 64 < r;
  const int c0 = min(lane, r - 1), c1 = min(lane + 64, r - 1);
  acc0 = acc1 = 0.f;
  for (int k0 = 0; k0 < r; k0 += 8) {
    float w0[8], w1[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const long long k = min(k0 + u, r - 1);
      w0[u] = M[k * r + c0];
      w1[u] = u1 ? M[k * r + c1] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (k0 + u < r) {
        const float x = sh[k0 + u];
        acc0 = fmaf(x, w0[u], acc0);
        acc1 = fmaf(x, w1[u], acc1);
      }
  }
}

// One wave per evidence row; lane l holds units l and l + 64.
__global__ __launch_bounds__(256) void k_circuit_bwd(const CircuitBwdArgs a) {
  __shared__ float sP[4][64];
  __shared__ float sX[4][128];
  __shared__ float sPi[4][128], sC[4][128];
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

  if (a.family == MTPC_HMM) {
    // forward messages (Eq. HMM) alpha_j, kept in Ge[j] until the reverse pass replaces them
    // by their adjoints.  With pi_j = softmax(alpha_j), pred_j = pi_j T_j (predicted next
    // state) and gam_j = adj(alpha_{j+1}) / pred_j:
    //   adj(alpha_j) = g_j pi_j + pi_j * (T_j gam_j),   d loss / d log T_j[z][z'] = pi_j[z] T_j[z][z'] gam_j[z'].
    float* sh = sX[wave];
    const long long lstep = a.L > 1 ? (long long)r * r : 0;
    const long long lrow = a.contextual ? row * a.L * r * r : 0;       // this position's own layers
    const float* lay_nat = a.lay_nat + lrow;
    const float* lay_tr = a.lay_tr ? a.lay_tr + lrow : nullptr;   // shared layers only
    float al0 = w0 + (u0 ? e[lane] : 0.f), al1 = w1 + (u1 ? e[lane + 64] : 0.f);
    float loss = 0.f;
    for (int j = 0; j < n; ++j) {
      if (j > 0) {
        const float m = wmax(fmaxf(al0, al1));
        const float ms = m == ninf ? 0.f : m;
        if (u0) sh[lane] = __expf(al0 - ms);
        if (u1) sh[lane + 64] = __expf(al1 - ms);
        __builtin_amdgcn_wave_barrier();
        float s0, s1;
        wave_matvec(lay_nat + (j - 1) * lstep, sh, r, lane, s0, s1);
        __builtin_amdgcn_wave_barrier();
        al0 = u0 ? ms + __logf(s0) + e[j * r + lane] : ninf;
        al1 = u1 ? ms + __logf(s1) + e[j * r + lane + 64] : ninf;
      }
      if (u0) Ge[j * r + lane] = al0;
      if (u1) Ge[j * r + lane + 64] = al1;
      const float m = wmax(fmaxf(al0, al1));
      const float P = m + __logf(wsum((u0 ? __expf(al0 - m) : 0.f) + (u1 ? __expf(al1 - m) : 0.f)));
      if (lane == 0) sP[wave][j] = P;
      loss += g_of(j) * P;
    }
    __builtin_amdgcn_wave_barrier();
    float ad0 = 0.f, ad1 = 0.f;                     // adjoint of alpha_{j+1}
    float nx0 = 0.f, nx1 = 0.f;                     // alpha_{j+1} - e_{j+1}
    for (int j = n - 1; j >= 0; --j) {
      const float P = sP[wave][j], g = g_of(j);
      const float cur0 = u0 ? Ge[j * r + lane] : ninf, cur1 = u1 ? Ge[j * r + lane + 64] : ninf;
      const float pi0 = u0 ? __expf(cur0 - P) : 0.f, pi1 = u1 ? __expf(cur1 - P) : 0.f;
      float n0 = g * pi0, n1 = g * pi1;
      if (j < n - 1) {
        const float pr0 = __expf(nx0 - P), pr1 = __expf(nx1 - P);          // predicted next state
        const float gm0 = (u0 && pr0 > 0.f) ? ad0 / pr0 : 0.f, gm1 = (u1 && pr1 > 0.f) ? ad1 / pr1 : 0.f;
        if (u0) sh[lane] = gm0;
        if (u1) sh[lane + 64] = gm1;
        __builtin_amdgcn_wave_barrier();
        float c0, c1;
        if (!a.contextual) {
          wave_matvec(lay_tr + j * lstep, sh, r, lane, c0, c1);            // (T_j gam)[z] via T_j^T
        } else {
          // this position's own transition matrix (natural layout only): lanes run over z',
          // the loop over z; (T gam)_z is a wave reduction, and the softmax backward of
          // pi_z T[z][z'] gam_z' is pi_z T[z][z'] (gam_z' - (T gam)_z), written along z'
          if (u0) sPi[wave][lane] = pi0;
          if (u1) sPi[wave][lane + 64] = pi1;
          __builtin_amdgcn_wave_barrier();
          const float* Tj = lay_nat + j * lstep;
          // one matrix per step: written once, in the dtype of h, straight into the logit-gradient
          // block; a matrix shared by the steps (or a caller's per-position buffer): fp32 accumulation
          const long long o = row * a.ld_dlog + (long long)j * r * r;
          float* acc32 = a.dlog32 ? a.dlog32 + row * (long long)a.L * r * r + j * lstep : nullptr;
          for (int z = 0; z < r; ++z) {
            const float t0 = u0 ? Tj[z * r + lane] : 0.f, t1 = u1 ? Tj[z * r + lane + 64] : 0.f;
            const float cz = wsum(t0 * gm0 + t1 * gm1);
            const float pz = sPi[wave][z];
            if (lane == 0) sC[wave][z] = cz;
            if (u0) {
              const float val = pz * t0 * (gm0 - cz);
              if (acc32) acc32[z * r + lane] += val;
              else if (a.bf16) ((unsigned short*)a.dlog)[o + z * r + lane] = to_bf16_rne(val);
              else ((float*)a.dlog)[o + z * r + lane] = val;
            }
            if (u1) {
              const float val = pz * t1 * (gm1 - cz);
              if (acc32) acc32[z * r + lane + 64] += val;
              else if (a.bf16) ((unsigned short*)a.dlog)[o + z * r + lane + 64] = to_bf16_rne(val);
              else ((float*)a.dlog)[o + z * r + lane + 64] = val;
            }
          }
          __builtin_amdgcn_wave_barrier();
          c0 = u0 ? sC[wave][lane] : 0.f;
          c1 = u1 ? sC[wave][lane + 64] : 0.f;
        }
        __builtin_amdgcn_wave_barrier();
        n0 += pi0 * c0;
        n1 += pi1 * c1;
        if (a.pi != nullptr) {
          float* pp = a.pi + (row * (n - 1) + j) * r;
          float* gp = a.gam + (row * (n - 1) + j) * r;
          if (u0) { pp[lane] = pi0; gp[lane] = gm0; }
          if (u1) { pp[lane + 64] = pi1; gp[lane + 64] = gm1; }
        }
      }
      nx0 = u0 ? cur0 - e[j * r + lane] : ninf;
      nx1 = u1 ? cur1 - e[j * r + lane + 64] : ninf;
      ad0 = n0; ad1 = n1;
      if (u0) Ge[j * r + lane] = n0;
      if (u1) Ge[j * r + lane + 64] = n1;
    }
    if (a.dlog != nullptr && a.dlog32 == nullptr)   // padding columns of the block
      for (int c = (n - 1) * r * r + lane; c < a.dlog_cols; c += 64) {
        if (a.bf16) ((unsigned short*)a.dlog)[row * a.ld_dlog + c] = 0;
        else ((float*)a.dlog)[row * a.ld_dlog + c] = 0.f;
      }
    const float tot = wsum((u0 ? ad0 : 0.f) + (u1 ? ad1 : 0.f));
    put_dsl(ad0 - __expf(w0) * tot, ad1 - __expf(w1) * tot);
    if (lane == 0) a.loss[row] = loss;
    return;
  }
}

// Binary tree (Eq. BTree), one wave per evidence row.  The forward pass walks the
// tree program (full node values bottom-up, then the path of every prefix) and keeps
// the output of every step; the reverse pass walks it backwards.  For a step
// c[k] = log sum_j A[k][j] exp(x[j]) with x the sum of its two operands:
//   xi[j] = exp(x[j] - max x),  delta[k] = adj(c)[k] exp(max x - c[k]),
//   adj(x)[j] = xi[j] sum_k A[k][j] delta[k],   d loss / d log A[k][j] = delta[k] A[k][j] xi[j],
// and adj(x) goes to both operands (leaf: evidence gradient; stored node: its
// adjoint; path value: the adjoint consumed by the previous step of the path).
__global__ __launch_bounds__(256) void k_btree_bwd(const CircuitBwdArgs a, int nsteps_max) {
  extern __shared__ TreeStep bprog[];
  __shared__ float sX[4][128];
  __shared__ float sPi[4][128];
  __shared__ int s_nsteps;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long row = (long long)blockIdx.x * 4 + wave;
  const int n = a.n, r = a.r;
  const bool u0 = lane < r, u1 = lane + 64 < r;
  if (threadIdx.x == 0) s_nsteps = build_tree_program(bprog, n, 1);
  __syncthreads();
  const int T = s_nsteps;
  auto put_dsl = [&](float v0, float v1) {
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
  if (row >= a.rows) {
    put_dsl(0.f, 0.f);
    return;
  }
  const float ninf = neg_inf();
  const float* e = a.e + row * n * r;
  const float* coef = a.coef + row * n;
  float* Ge = a.Ge + row * n * r;
  float* ct = a.ct + row * nsteps_max * r;           // output of every step
  float* ad = a.adj + row * (long long)(n - 1) * r;   // adjoints of the stored node values
  float* sh = sX[wave];
  const float* lw = a.logw + row * r;
  const float w0 = u0 ? lw[lane] : ninf, w1 = u1 ? lw[lane + 64] : ninf;
  const long long lstep = a.L > 1 ? (long long)r * r : 0;
  const long long lrow = a.contextual ? row * a.L * r * r : 0;        // this position's own layers
  auto g_of = [&](int j) { return (j + 1 < n ? coef[j + 1] : 0.f) - coef[j]; };
  // value of an operand for the lane's two units; path values live in ct[t-1]
  auto operand = [&](int src, int t, float& x0, float& x1) {
    if (src == -2) { x0 = u0 ? 0.f : ninf; x1 = u1 ? 0.f : ninf; return; }
    const float* p;
    if (src == -1) p = ct + (long long)(t - 1) * r;
    else if (src >= n - 1) p = e + (long long)(src - (n - 1)) * r;
    else p = ct + (long long)(n - 2 - src) * r;      // node m is the output of up-pass step n-2-m
    x0 = u0 ? p[lane] : ninf;
    x1 = u1 ? p[lane + 64] : ninf;
  };

  // ---- forward
  float loss = 0.f;
  for (int t = 0; t < T; ++t) {
    const TreeStep st = bprog[t];
    float l0, l1, r0, r1;
    operand(st.lsrc, t, l0, l1);
    operand(st.rsrc, t, r0, r1);
    float x0 = l0 + r0, x1 = l1 + r1;
    if (st.m == 0) {
      x0 += w0; x1 += w1;
      const float m = wmax(fmaxf(x0, x1));
      const float P = m + __logf(wsum((u0 ? __expf(x0 - m) : 0.f) + (u1 ? __expf(x1 - m) : 0.f)));
      loss += g_of(-2 - st.out) * P;
      if (lane == 0) ct[(long long)t * r] = P;       // the root step keeps its scalar
      continue;
    }
    const float m = wmax(fmaxf(x0, x1));
    const float ms = m == ninf ? 0.f : m;
    if (u0) sh[lane] = __expf(x0 - ms);
    if (u1) sh[lane + 64] = __expf(x1 - ms);
    __builtin_amdgcn_wave_barrier();
    float s0, s1;
    if (!a.contextual) {
      wave_matvec(a.lay_tr + (st.m - 1) * lstep, sh, r, lane, s0, s1);     // sum_j A[k][j] xi[j] via A^T
    } else {
      // this position's own layer, natural layout only: lanes run over j, one wave reduction per k
      const float* A = a.lay_nat + lrow + (st.m - 1) * lstep;
      const float xa = u0 ? sh[lane] : 0.f, xb = u1 ? sh[lane + 64] : 0.f;
      s0 = s1 = 0.f;
      for (int k = 0; k < r; ++k) {
        const float v = wsum((u0 ? A[k * r + lane] * xa : 0.f) + (u1 ? A[k * r + lane + 64] * xb : 0.f));
        if (k == lane) s0 = v;
        if (k == lane + 64) s1 = v;
      }
    }
    __builtin_amdgcn_wave_barrier();
    if (u0) ct[(long long)t * r + lane] = ms + __logf(s0);
    if (u1) ct[(long long)t * r + lane + 64] = ms + __logf(s1);
  }
  // ---- reverse
  for (int idx = lane; idx < (n - 1) * r; idx += 64) ad[idx] = 0.f;
  for (int idx = lane; idx < n * r; idx += 64) Ge[idx] = 0.f;
  __builtin_amdgcn_wave_barrier();
  float gw0 = 0.f, gw1 = 0.f;                        // gradient w.r.t. log omega
  float pv0 = 0.f, pv1 = 0.f;                        // adjoint of the path value of the step above
  auto scatter = [&](int src, float a0, float a1) {
    if (src == -2) return;
    if (src == -1) { pv0 = a0; pv1 = a1; return; }
    float* p = src >= n - 1 ? Ge + (long long)(src - (n - 1)) * r : ad + (long long)(src - 1) * r;
    if (u0) p[lane] += a0;
    if (u1) p[lane + 64] += a1;
  };
  for (int t = T - 1; t >= 0; --t) {
    const TreeStep st = bprog[t];
    float l0, l1, r0, r1;
    operand(st.lsrc, t, l0, l1);
    operand(st.rsrc, t, r0, r1);
    float x0 = l0 + r0, x1 = l1 + r1;
    float xb0, xb1;                                  // adjoint of x
    if (st.m == 0) {
      const float P = ct[(long long)t * r], g = g_of(-2 - st.out);
      xb0 = u0 ? g * __expf(x0 + w0 - P) : 0.f;
      xb1 = u1 ? g * __expf(x1 + w1 - P) : 0.f;
      gw0 += xb0; gw1 += xb1;
    } else {
      float cb0, cb1;                                // adjoint of this step's output
      if (st.out >= 0) {
        cb0 = u0 ? ad[(long long)(st.out - 1) * r + lane] : 0.f;
        cb1 = u1 ? ad[(long long)(st.out - 1) * r + lane + 64] : 0.f;
      } else {
        cb0 = pv0; cb1 = pv1;
      }
      const float m = wmax(fmaxf(x0, x1));
      const float ms = m == ninf ? 0.f : m;
      const float xi0 = u0 ? __expf(x0 - ms) : 0.f, xi1 = u1 ? __expf(x1 - ms) : 0.f;
      const float c0 = u0 ? ct[(long long)t * r + lane] : 0.f, c1 = u1 ? ct[(long long)t * r + lane + 64] : 0.f;
      const float d0 = (u0 && cb0 != 0.f) ? cb0 * __expf(ms - c0) : 0.f;
      const float d1 = (u1 && cb1 != 0.f) ? cb1 * __expf(ms - c1) : 0.f;
      if (u0) sh[lane] = d0;
      if (u1) sh[lane + 64] = d1;
      __builtin_amdgcn_wave_barrier();
      float s0, s1;
      if (!a.contextual) {
        wave_matvec(a.lay_nat + (st.m - 1) * lstep, sh, r, lane, s0, s1);   // sum_k A[k][j] delta[k]
      } else {
        // one pass over this position's layer gives both sum_k A[k][j] delta[k] and the softmax
        // backward of its logits, delta_k A[k][j] (xi_j - (A xi)_k) with (A xi)_k = exp(c_k - max x),
        // accumulated in fp32 per position (a layer is applied by several steps)
        if (u0) sPi[wave][lane] = c0 == ninf ? 0.f : __expf(c0 - ms);
        if (u1) sPi[wave][lane + 64] = c1 == ninf ? 0.f : __expf(c1 - ms);
        __builtin_amdgcn_wave_barrier();
        const float* A = a.lay_nat + lrow + (st.m - 1) * lstep;
        float* dl = a.dlog32 + row * (long long)a.L * r * r + (st.m - 1) * lstep;
        s0 = s1 = 0.f;
        for (int k = 0; k < r; ++k) {
          const float dk = sh[k], sk = sPi[wave][k];
          if (u0) {
            const float w = A[k * r + lane];
            s0 = fmaf(w, dk, s0);
            dl[k * r + lane] += dk * w * (xi0 - sk);
          }
          if (u1) {
            const float w = A[k * r + lane + 64];
            s1 = fmaf(w, dk, s1);
            dl[k * r + lane + 64] += dk * w * (xi1 - sk);
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
      xb0 = xi0 * s0; xb1 = xi1 * s1;
      if (a.pi != nullptr) {
        float* pp = a.pi + (row * nsteps_max + t) * r;
        float* gp = a.gam + (row * nsteps_max + t) * r;
        if (u0) { pp[lane] = d0; gp[lane] = xi0; }
        if (u1) { pp[lane + 64] = d1; gp[lane + 64] = xi1; }
      }
    }
    __builtin_amdgcn_wave_barrier();
    scatter(st.lsrc, xb0, xb1);
    scatter(st.rsrc, xb0, xb1);
    __builtin_amdgcn_wave_barrier();
  }
  const float tot = wsum((u0 ? gw0 : 0.f) + (u1 ? gw1 : 0.f));
  put_dsl(gw0 - __expf(w0) * tot, gw1 - __expf(w1) * tot);
  if (lane == 0) a.loss[row] = loss;
}

// part[by][j][z][z'] = sum over the rows of block by of pi[b][j][z] * gam[b][j][z'] for step j.
// Thread t owns outputs t, t + 256, ...: NO of them.  Nothing is accumulated across workgroups
// here: k_layer_reduce adds the partial tiles in a fixed order, so that the layer gradients are
// the same bits on every run.
template <int NO>
__global__ __launch_bounds__(256) void k_layer_outer(const float* pi, const float* gam, int rows, int steps,
                                                     int r, int rows_per_block, float* part) {
  __shared__ float sp[16][128], sg[16][128];
  const int j = blockIdx.x, tid = threadIdx.x;
  const long long b0 = (long long)blockIdx.y * rows_per_block;
  const long long b1 = min((long long)rows, b0 + rows_per_block);
  float acc[NO];
#pragma unroll
  for (int q = 0; q < NO; ++q) acc[q] = 0.f;
  for (long long c0 = b0; c0 < b1; c0 += 16) {
    __syncthreads();
    for (int idx = tid; idx < 16 * r; idx += 256) {
      const long long b = c0 + idx / r;
      const int z = idx % r;
      const bool ok = b < b1;
      sp[idx / r][z] = ok ? pi[(b * steps + j) * r + z] : 0.f;
      sg[idx / r][z] = ok ? gam[(b * steps + j) * r + z] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NO; ++q) {
      const int o = tid + q * 256;
      if (o < r * r) {
        const int z = o / r, zz = o - z * r;
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < 16; ++t) s = fmaf(sp[t][z], sg[t][zz], s);
        acc[q] += s;
      }
    }
  }
  float* dst = part + ((long long)blockIdx.y * steps + j) * r * r;
#pragma unroll
  for (int q = 0; q < NO; ++q) {
    const int o = tid + q * 256;
    if (o < r * r) dst[o] = acc[q];
  }
}

// G[l][o] = sum over the steps j that apply layer l (ascending), and for each over the row blocks
// (ascending), of part[by][j][o].  HMM: step j applies layer j (layer 0 when one matrix is shared).
// Tree mode (tree_n > 0): step j applies the layer of node prog[j].m (root steps: none).
__global__ __launch_bounds__(256) void k_layer_reduce(const float* part, int steps, int nby, int r, int L,
                                                      float* G, int tree_n) {
  extern __shared__ TreeStep oprog[];
  __shared__ int s_cnt;
  const int rr = r * r;
  if (tree_n > 0) {
    if (threadIdx.x == 0) s_cnt = build_tree_program(oprog, tree_n, 1);
    __syncthreads();
  }
  const int nsteps = tree_n > 0 ? s_cnt : steps;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)L * rr) return;
  const int l = (int)(idx / rr), o = (int)(idx - (long long)l * rr);
  float s = 0.f;
  for (int j = 0; j < nsteps; ++j) {
    int layer = tree_n > 0 ? oprog[j].m - 1 : j;
    if (layer < 0) continue;
    if (L == 1) layer = 0;
    if (layer != l) continue;
    for (int by = 0; by < nby; ++by) s += part[((long long)by * steps + j) * rr + o];
  }
  G[idx] = s;
}

// softmax backward of every layer row: dlogit[l][z][:] = T (.) (G - sum_z' T G); one wave per row
__global__ __launch_bounds__(256) void k_layer_finish(const float* G, const float* T, int nrows, int r,
                                                      float* dlayers) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= nrows) return;
  const bool u0 = lane < r, u1 = lane + 64 < r;
  const float t0 = u0 ? T[row * r + lane] : 0.f, t1 = u1 ? T[row * r + lane + 64] : 0.f;
  const float g0 = u0 ? G[row * r + lane] : 0.f, g1 = u1 ? G[row * r + lane + 64] : 0.f;
  const float s = wsum(t0 * g0 + t1 * g1);
  if (u0) dlayers[row * r + lane] = t0 * (g0 - s);
  if (u1) dlayers[row * r + lane + 64] = t1 * (g1 - s);
}

// part[by][c] = sum_b src[b][c] over the rows of block by (src in the dtype of h, fp32 sums);
// k_colsum_reduce adds the blocks in ascending order (no atomics: the same bits on every run)
template <typename T>
__global__ __launch_bounds__(256) void k_colsum(const T* src, long long ld, int rows, int cols, float* part) {
  __shared__ float red[4][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63), ty = threadIdx.x >> 6;
  const int b0 = blockIdx.y * 256;
  float s = 0.f;
  if (c < cols)
    for (int b = b0 + ty; b < min(rows, b0 + 256); b += 4) {
      if constexpr (sizeof(T) == 2) s += __uint_as_float(((unsigned)src[(long long)b * ld + c]) << 16);
      else s += src[(long long)b * ld + c];
    }
  red[ty][threadIdx.x & 63] = s;
  __syncthreads();
  if (ty == 0 && c < cols)
    part[(long long)blockIdx.y * cols + c] =
        (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

__global__ __launch_bounds__(256) void k_colsum_reduce(const float* part, int nby, int cols, float* out) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= cols) return;
  float s = 0.f;
  for (int by = 0; by < nby; ++by) s += part[(long long)by * cols + c];
  out[c] = s;
}

// dst[b][c] (dtype of h, row stride ld) = src[b][c] for c < cols, 0 for cols <= c < cols_pad
template <typename T>
__global__ __launch_bounds__(256) void k_convert_block(const float* src, int rows, int cols, int cols_pad, T* dst,
                                                       long long ld) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)rows * cols_pad) return;
  const long long b = t / cols_pad;
  const int c = (int)(t - b * cols_pad);
  const float v = c < cols ? src[b * cols + c] : 0.f;
  if constexpr (sizeof(T) == 2) dst[b * ld + c] = to_bf16_rne(v); else dst[b * ld + c] = v;
}

__global__ __launch_bounds__(256) void k_fill_zero(float* p, long long n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

}  // namespace

hipError_t launch_transpose(const TransposeArgs& a, int dtype, hipStream_t st) {
  if (a.C < 1 || a.Rpad < 1) return hipSuccess;
  const dim3 grid((a.C + 63) / 64, (a.Rpad + 63) / 64);
  const int esz = dtype == MTPC_BF16 ? 2 : 4, ve = 16 / esz;
  const bool vec = a.ld_src % ve == 0 && a.ld_dst % ve == 0 && a.col0 % ve == 0 &&
                   (((uintptr_t)a.src | (uintptr_t)a.dst) & 15) == 0;
  if (vec) {
    if (dtype == MTPC_BF16) hipLaunchKernelGGL(k_transpose_vec<unsigned short>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(k_transpose_vec<float>, grid, dim3(256), 0, st, a);
  } else {
    if (dtype == MTPC_BF16) hipLaunchKernelGGL(k_transpose<unsigned short>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(k_transpose<float>, grid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

hipError_t launch_grad_from_phi(const GradPhiArgs& a, int dtype, hipStream_t st) {
  const dim3 grid((unsigned)((a.ldb + 127) / 128), (unsigned)((a.ldM + 63) / 64));
  if (dtype == MTPC_BF16) hipLaunchKernelGGL(k_grad_from_phi<unsigned short>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(k_grad_from_phi<float>, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_circuit_bwd(const CircuitBwdArgs& a, hipStream_t st) {
  const long long rows = a.dslT ? a.ldb : a.rows;
  const int r = a.r;
  const bool tree = a.family == MTPC_BTREE;
  const int T = tree ? tree_program_steps(a.n, 1) : a.n - 1;
  const size_t prog_bytes = tree ? (size_t)T * sizeof(TreeStep) : 0;
  const bool ctx = a.contextual && a.dlog != nullptr;        // layers computed from h (R): bias gradient = column sums
  const bool layers = !a.contextual && a.dlayers != nullptr && ((a.family == MTPC_HMM && a.n > 1) || (tree && a.n > 2));
  if (a.contextual && a.dlog32 != nullptr) {       // per-position fp32 accumulators
    const long long cnt = (long long)a.rows * a.L * r * r;
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st, a.dlog32, cnt);
  }
  if (tree) hipLaunchKernelGGL(k_btree_bwd, dim3((unsigned)((rows + 3) / 4)), dim3(256), prog_bytes, st, a, T);
  else hipLaunchKernelGGL(k_circuit_bwd, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, a);
  if (layers) {
    const int steps = T, rpb = LAYER_GRAD_ROWS;
    const int nby = (a.rows + rpb - 1) / rpb;
    const dim3 grid(steps, (unsigned)nby);
    const int no = (r * r + 255) / 256;
    if (no <= 1) hipLaunchKernelGGL(k_layer_outer<1>, grid, dim3(256), 0, st, a.pi, a.gam, a.rows, steps, r, rpb, a.Gpart);
    else if (no <= 4) hipLaunchKernelGGL(k_layer_outer<4>, grid, dim3(256), 0, st, a.pi, a.gam, a.rows, steps, r, rpb, a.Gpart);
    else if (no <= 16) hipLaunchKernelGGL(k_layer_outer<16>, grid, dim3(256), 0, st, a.pi, a.gam, a.rows, steps, r, rpb, a.Gpart);
    else hipLaunchKernelGGL(k_layer_outer<64>, grid, dim3(256), 0, st, a.pi, a.gam, a.rows, steps, r, rpb, a.Gpart);
    const long long cnt = (long long)a.L * r * r;
    hipLaunchKernelGGL(k_layer_reduce, dim3((unsigned)((cnt + 255) / 256)), dim3(256), prog_bytes, st, a.Gpart, steps, nby,
                       r, a.L, a.G, tree ? a.n : 0);
    const int nrows = a.L * r;
    hipLaunchKernelGGL(k_layer_finish, dim3((nrows + 3) / 4), dim3(256), 0, st, a.G, a.lay_nat, nrows, r, a.dlayers);
  }
  if (ctx && a.dlog32 != nullptr) {
    const int cols = a.L * r * r;
    const long long cnt = (long long)a.rows * a.dlog_cols;
    const dim3 g((unsigned)((cnt + 255) / 256));
    if (a.bf16) hipLaunchKernelGGL(k_convert_block<unsigned short>, g, dim3(256), 0, st, a.dlog32, a.rows, cols,
                                   a.dlog_cols, (unsigned short*)a.dlog, a.ld_dlog);
    else hipLaunchKernelGGL(k_convert_block<float>, g, dim3(256), 0, st, a.dlog32, a.rows, cols, a.dlog_cols,
                            (float*)a.dlog, a.ld_dlog);
  }
  if (ctx && a.dlayers != nullptr) {               // bias gradient = column sums of the logit gradients
    const int cols = a.L * r * r;
    const int nby = (a.rows + LAYER_GRAD_ROWS - 1) / LAYER_GRAD_ROWS;
    const dim3 grid((cols + 63) / 64, nby);
    if (a.bf16) hipLaunchKernelGGL(k_colsum<unsigned short>, grid, dim3(256), 0, st, (const unsigned short*)a.dlog,
                                   a.ld_dlog, a.rows, cols, a.Gpart);
    else hipLaunchKernelGGL(k_colsum<float>, grid, dim3(256), 0, st, (const float*)a.dlog, a.ld_dlog, a.rows, cols,
                            a.Gpart);
    hipLaunchKernelGGL(k_colsum_reduce, dim3((cols + 255) / 256), dim3(256), 0, st, a.Gpart, nby, cols, a.dlayers);
  }
  return hipGetLastError();
}

}  // namespace mtpc
