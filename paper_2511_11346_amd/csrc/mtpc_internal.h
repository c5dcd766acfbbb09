// Internal declarations shared by the HIP translation units of libmtpc.
// Not part of the public ABI (see include/mtpc.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "mtpc.h"

namespace mtpc {

// Arguments of the fused unembedding kernel (Sec. 3.3: phi_ij = softmax(W_ij e_t)).
// One workgroup owns ALL v logits of one (i, j) slab for a tile of positions, so
// the softmax over the vocabulary finishes in registers and only O(B n r) values
// are written.
struct UnembedArgs {
  const void* h;        // [B][ld_h]
  long long ld_h;       // elements
  const void* W;        // [n*r][v][d]
  const void* Wp;       // stage-major copy of W (mtpc_pack_weights) or nullptr, in stages of Wp_stage bytes; read
  int Wp_stage;         // instead of W by the tiles whose stages have that size: 128 bytes for B <= 64, else 64
  const void* hs;       // stage-major copy of h in 64-byte stages, [d*esz/64][B][64 bytes] (launch_pack_rows), or
                        // nullptr; read instead of h by the 256-position tiles (B > 64): a stage of a tile is then
                        // one run of 16 KB and the L2 is asked for whole 128-byte lines
  int B, d, v, n, r;
  // evidence: e[(b*T+t)][i][j] = l[x] - LSE for target window t of position b
  const int* targets;   // [B][T][n] or nullptr
  int T;
  const int* targets2;  // [B][T2][n]: a second set of windows per position (rows T..T+T2-1 of a position), or nullptr
  int T2;
  float* e;             // [B*(T+T2)][n][r]
  // sampling: token i of draft (b, s) is drawn from slab (i, zleaf[b][s][i])
  const int* zleaf;     // [B][S][n] or nullptr
  int S;
  int* drafts;          // [B][S][n]
  uint32_t seed_lo, seed_hi, offset;
  int greedy;           // 1: every draw is replaced by the most likely outcome (no random numbers)
  float* logphi;        // [B][n][r][v] normalised logits of every slab, or nullptr
  float* phiT;          // [n*r*v][ld_phi] softmax probabilities, transposed, or nullptr (evidence kernel only)
  long long ld_phi;
};

// Univariate marginals: M[b][i][a] = log sum_j m[b][i][j] phi[b][i][j][a].
struct UnivariateArgs {
  const void* h;
  long long ld_h;
  const void* W;
  int B, d, v, n, r;
  const float* logm;    // [B][n][r] log marginal of the latent indexing leaf i (nullptr: r == 1)
  float* out;           // [B][n][v]
};

// dWsum[j][c] = sum_b gT[j][b] hT[c][b]; gT [r][ldb], hT [d][ldb] in the dtype of h, ldb a multiple of 32
hipError_t launch_dwsum(const void* gT, const void* hT, long long ldb, int r, int d, int dtype, float* out,
                        hipStream_t st);
// The same from the table of normalised input units log phi[B][n][r][v] (a.h, a.W unused):
// M[b][i][a] = log sum_j exp(logm[b][i][j] + logphi[b][i][j][a]).
hipError_t launch_univariate_table(const UnivariateArgs& a, const float* logphi, hipStream_t st);

// Contextual sum layers: P[b][l][k][:] = softmax(R[l][k] h[b] + bias[l][k][:]) as linear
// probabilities, natural [b][l][k][j] and/or transposed [b][l][j][k] layout.
struct CtxLayerArgs {
  const void* h;
  long long ld_h;
  const void* R;          // [L][r][r][d]
  long long R_layer_stride;   // elements, 0 = shared
  const float* bias;      // [L][r][r] or nullptr
  long long bias_layer_stride;
  int B, d, r, L;         // L = layers to produce
  float* out_nat;         // [B][L][r][r] or nullptr
  float* out_tr;          // [B][L][r][r] transposed or nullptr
};
hipError_t launch_ctx_layers(const CtxLayerArgs& a, int dtype, hipStream_t st);

hipError_t launch_unembed(const UnembedArgs& a, int dtype, hipStream_t st);
// dst[slab][stage][row][stage_bytes] = the stage_bytes of row `row` of slab `slab` of W that K stage `stage` covers
// Stage-major copy of `slabs` matrices of v rows (row_bytes used bytes, row_stride bytes apart): per matrix
// [row_bytes / stage_bytes][v][stage_bytes].  W for the decode tiles (128-byte stages), h for the
// 256-position tiles (one matrix, 64-byte stages).
hipError_t launch_pack_rows(const void* src, void* dst, long long slabs, int v, int row_bytes, long long row_stride,
                            int stage_bytes, hipStream_t st);
constexpr int H_STAGE_BYTES = 64;
constexpr int PACK_STAGE_BYTES = 128;
hipError_t launch_univariate(const UnivariateArgs& a, int dtype, hipStream_t st);

// ---- small kernels (circuits.hip) -----------------------------------------
// log omega[b][:] = log_softmax(Wsum h[b])
hipError_t launch_sumunit(const void* h, long long ld_h, const void* Wsum, int B, int d, int r,
                          int dtype, float* logw, hipStream_t st);
// same result through the MFMA tile kernel (unembed.hip); used when B is large
hipError_t launch_sumunit_mfma(const void* h, long long ld_h, const void* Wsum, int B, int d, int r,
                               int dtype, float* logw, hipStream_t st);
// softmax over the last axis of r x r logits -> linear probabilities.
// in: logits[(b*bs) + l*ls + k*r + j]; out_nat[((b*L + l)*r + k)*r + j] and / or the same
// transposed, out_tr[((b*L + l)*r + j)*r + k] (either may be nullptr).
hipError_t launch_normalise_layers(const float* logits, long long layer_stride, long long batch_stride,
                                   int nb, int L, int r, float* out_nat, float* out_tr, hipStream_t st);

struct CircuitArgs {
  int family;           // mtpc_family
  int rows;             // B*T evidence rows
  int T;                // rows per position (logw / contextual layers are indexed by row / T)
  int n, r;
  const float* e;       // [rows][n][r]
  const float* logw;    // [B][r] (nullptr for FF)
  const float* layers;  // normalised linear probabilities, HMM: [nb][L][j][j'], BTree: [nb][L][j][k] (transposed)
  const float* layers_nat;  // BTree with shared layers: the same in natural layout [L][k][j], or nullptr
  int L;                // number of stored layers (1 = homogeneous)
  int contextual;       // 1: layers has a leading position axis
  float* out;           // prefix ? [rows][n] : [rows]
  int prefix;
};
hipError_t launch_circuit(const CircuitArgs& a, hipStream_t st);

// latent draws of Alg. 1 (top-down over sum units)
struct LatentArgs {
  int family, B, S, n, r;
  const float* logw;    // [B][r]
  const float* layers;  // normalised linear, natural layout [nb][L][k][j]
  int L, contextual;
  uint32_t seed_lo, seed_hi, offset;
  int greedy;           // 1: every sum unit takes its largest weight
  int* zleaf;           // [B][S][n] state that indexes leaf i
  int* latents;         // [B][S][n_lat] or nullptr
  int* zero;            // launch_latents only: nzero ints it also sets to zero (the counters of the
  int nzero;            // bucketing that follows, which saves that a launch of its own), or nullptr
};
hipError_t launch_latents(const LatentArgs& a, hipStream_t st);
// batches up to this many positions compute their sum units one workgroup per position
constexpr int SUMUNIT_SMALL_B = 128;
// the same draws in the launch that computes log omega (B <= SUMUNIT_SMALL_B, families with sum
// units): writes logw [B][r] and the latents; the normalised layers must be complete before it
hipError_t launch_sumunit_latents(const void* h, long long ld_h, const void* Wsum, int d, int dtype, float* logw,
                                  const LatentArgs& a, hipStream_t st);

// log marginal of the latent that indexes each leaf: logm[b][i][j]
struct LatentMarginalArgs {
  int family, B, n, r;
  const float* logw;
  const float* layers;  // natural layout
  int L, contextual;
  float* logm;          // [B][n][r]
};
hipError_t launch_latent_marginals(const LatentMarginalArgs& a, hipStream_t st);

// evidence of drafted tokens from the table the sampling pass wrote:
// e[(b*S+s)][i][j] = logphi[b][i][j][x] with x = drafts[b][s][i]
struct GatherArgs {
  int B, S, v, n, r;
  const int* x;         // [B][S][n]
  float* e;             // [B*S][n][r]
};
hipError_t launch_gather_table(const GatherArgs& a, const float* logphi, hipStream_t st);

// token draws of Alg. 1 from the table of normalised input units: token i of draft (b,s)
// comes from the row log phi[b][i][zleaf[b][s][i]][:]
struct DrawArgs {
  int B, S, v, n, r;
  const float* logphi;  // [B][n][r][v]
  const int* zleaf;     // [B][S][n] selected input unit of every token
  int* drafts;          // [B][S][n]
  uint32_t seed_lo, seed_hi, offset;
  int greedy;           // most likely token instead of a draw (smallest id on ties)
  int compact;          // logphi is [B*S*n][v]: one row of (unnormalised) logits per token
};
hipError_t launch_draw_table(const DrawArgs& a, hipStream_t st);

// logits of the selected input unit of every token: out[(b,s,i)][:] = W[i][zleaf[b][s][i]] h[b]
struct RowLogitArgs {
  const void* h;
  long long ld_h;
  const void* W;
  int B, S, d, v, n, r;
  const int* zleaf;     // [B][S][n]
  float* out;           // [B*S*n][v]
};
hipError_t launch_rows_logits(const RowLogitArgs& a, int dtype, hipStream_t st);

// Buckets of the (b, s, i) triples by (i, selected input unit): bucket g = i*r + z holds
// list[row_off[g] .. row_off[g+1]) = the draft rows b*S+s whose token i comes from unit z
// (in no particular order), and is covered by tiles tile_off[g] .. tile_off[g+1]-1 of
// `tile` rows each.
struct BucketArgs {
  int B, S, n, r, tile;
  const int* zleaf;     // [B][S][n]
  int* count;           // [n*r] scratch
  int cleared;          // count is already zero (launch_latents did it)
  int* slot;            // [B*S*n] scratch: rank of a triple inside its bucket
  int* row_off;         // [n*r + 1]
  int* tile_off;        // [n*r + 1]
  int* tile_bucket;     // [B*S*n / tile + n*r] bucket of every tile
  int* list;            // [B*S*n]
};
hipError_t launch_buckets(const BucketArgs& a, hipStream_t st);

// token draws through the buckets: one slab per tile, h rows gathered
struct DrawGatherArgs {
  const void* h;
  long long ld_h;
  const void* W;
  const void* Wp;       // stage-major copy of W in the 64-byte stages of these tiles, or nullptr
  int B, S, d, v, n, r;
  const int* row_off;
  const int* tile_off;
  const int* tile_bucket;
  const int* list;
  int* drafts;          // [B][S][n]
  uint32_t seed_lo, seed_hi, offset;
  int greedy;
  int tile;             // rows per tile the buckets were cut into: DRAW_GATHER_TILE or (bf16) DRAW_GATHER_TILE_WIDE
};
hipError_t launch_draw_gather(const DrawGatherArgs& a, int dtype, hipStream_t st);
constexpr int DRAW_GATHER_TILE = 128;   // rows per tile of the gathered draw kernel
// ... and of its wider bf16 tile, for buckets that would leave a nearly empty last tile of 128 rows behind
// (a tile costs nearly the same whatever it holds, so what counts is the number of rounds over the CUs)
constexpr int DRAW_GATHER_TILE_WIDE = 192;
constexpr int GATHER_STAGE_BYTES = 64;  // ... and the bytes of a row it takes per stage

// Verification step of a speculative-decoding cycle (Alg. 2, acceptance loop on)
struct VerifyArgs {
  int family, B, n, r, v, mode;
  const float* logphi;  // [B][n][r][v]
  const int* drafts;    // [B][n]
  const float* prefix;  // [B][n]
  const float* p;       // [B][n+1][v]
  const float* logw;    // [B][r] (nullptr for FF, or when the kernel computes it itself, see h)
  const void* h;        // with h set (B <= SUMUNIT_SMALL_B): log omega = log_softmax(Wsum h[b]) is computed
  long long ld_h;       // by the position's own workgroup
  const void* Wsum;
  int d, bf16;
  const float* lay_nat; // normalised linear layers [nb][L][k][j]
  const float* lay_tr;  // the same transposed [nb][L][j][k] (BTree only)
  int L, contextual;
  uint32_t seed_lo, seed_hi, offset;
  int* accepted;        // [B]
  int* token;           // [B]
};
hipError_t launch_verify(const VerifyArgs& a, hipStream_t st);

// ---- training step (grad.hip, backward.hip) ----------------------------------
// Recompute pass: dLT[(i*r+j)*v + a][b] = Ge[b][i][j] * (1[a == x_bi] - phi[b,i,j,a]) in the
// dtype of h; columns b in [B, ldb) are written as zero.
struct GradLogitsArgs {
  const void* h; long long ld_h; const void* W;
  int B, d, v, n, r;
  const int* targets;   // [B][n]
  const float* Ge;      // [B][n][r] gradient of the loss w.r.t. the evidence
  void* dLT;            // [n*r*v][ldb]
  long long ldb;        // >= B, a multiple of 32
};
hipError_t launch_unembed_grad(const GradLogitsArgs& a, int dtype, hipStream_t st);

// Logit gradient from stored probabilities: for m = (i*r+j)*v + a < M
//   val = Ge[b][i][j] * (1[a == x_bi] - phiT[m][b]);   rows M <= m < Mx of dLT are passed through.
// Writes dLT[m][b] (m < M, b < ldb, zero for b >= B) and dL[b][m] (b < B, m < ldM, zero for m >= Mx).
struct GradPhiArgs {
  const float* phiT; long long ld_phi;
  const int* targets; const float* Ge;
  int B, n, r, v;
  long long M, Mx, ldM, ldb;
  long long dl_end;     // dL is written for m < dl_end (a multiple of 4); columns beyond belong to others
  void* dLT; void* dL;
  // 1: both are written stage-major in 64-byte stages, as the contractions read their 320-row operands:
  // rows m < M of dLT as [ldb * esz / 64][M][64 bytes] (the sum-unit rows M..Mx-1 stay where they are, behind
  // it), dL as [ldM * esz / 64][B][64 bytes] (then dl_end = ldM: every column is written here)
  int staged;
};
hipError_t launch_grad_from_phi(const GradPhiArgs& a, int dtype, hipStream_t st);

// C[M][N] (fp32, row stride ldc; optionally split by rows over two buffers) = A[M][K] * B[N][K]^T, both operands K-contiguous
// with row strides lda / ldb (elements); K a multiple of 32 (bf16) or 16 (fp32).
struct GemmArgs {
  const void* A; long long lda; int M;
  const void* Bm; long long ldb; int N;
  const void* Bs;       // Bm stage-major, [K * esz / 64][N][64 bytes] (read instead of Bm), or nullptr
  const void* As;       // A stage-major, [K * esz / 64][As_rows][64 bytes] with As_rows >= M (read instead of A), or nullptr
  int As_rows;
  int K;
  float* C; long long ldc;
  // output rows are dealt to up to three buffers: [0, split) -> C, [split, split + n2) -> C2,
  // [split3, M) -> C3; rows in between are computed and dropped
  int split; int n2; float* C2;
  int split3; float* C3;
  // split over K (few output tiles, long K): ksplit > 1 workgroups per tile each take kchunk
  // columns and write their partial tile to partial[ks][M][ldc]; a second kernel adds the
  // partials in a fixed order into C (single output buffer only)
  int ksplit; int kchunk; float* partial;
};
hipError_t launch_gemm_tn(const GemmArgs& a, int dtype, hipStream_t st);
// number of K splits that fills the 256 CUs best for an M x N output (1: none)
inline int gemm_ksplit(int M, int N, int K) {
  const long long tiles = (long long)((M + 255) / 256) * ((N + 255) / 256);
  if (tiles >= 384) return 1;
  const int cand[] = {1, 2, 3, 4, 6, 8, 12, 16};
  int best = 1;
  double best_cost = 1e30;
  for (int ks : cand) {
    if (ks > 1 && K / ks < 2048) break;
    // rounds over the CUs, each 1/ks long, plus a little for writing and adding the partials
    const double cost = (double)((tiles * ks + 255) / 256) / ks + 0.02 * ks;
    if (cost < best_cost - 1e-9) { best_cost = cost; best = ks; }
  }
  return best;
}

// dst[c][col0 + r] = src[r][c] for r < R, c < C; dst[c][col0 + r] = 0 for R <= r < Rpad.
struct TransposeArgs {
  const void* src; long long ld_src; int R, C;
  void* dst; long long ld_dst; long long col0; int Rpad;
  // 0: dst[c][col0 + r].  Else the destination is stage-major in 64-byte stages with this many rows,
  // [columns * esz / 64][stage_rows][64 bytes] (the form the contraction kernels read an operand in)
  int stage_rows;
};
hipError_t launch_transpose(const TransposeArgs& a, int dtype, hipStream_t st);

// Reverse pass through the circuit: from the evidence and the loss coefficients to
// the gradient w.r.t. the evidence, the sum-unit logits (written transposed, in the
// dtype of h, as r rows of ldb columns) and the layer logits; also the loss itself.
struct CircuitBwdArgs {
  int family, rows, n, r;
  const float* e;        // [rows][n][r]
  const float* logw;     // [rows][r] (nullptr for FF)
  const float* coef;     // [rows][n]
  const float* lay_nat;  // normalised linear layers [L][k][j] (static only)
  const float* lay_tr;   // the same transposed [L][j][k]
  int L;
  float* pi;             // scratch [rows][steps][r] (layer gradients only; steps = n-1 for the HMM)
  float* gam;            // scratch [rows][steps][r]
  float* G;              // scratch [L][r][r]
  float* Gpart;          // scratch: per block of LAYER_GRAD_ROWS rows, [steps][r][r] outer-product partials
                         // (shared layers) or [L*r*r] column sums (bias gradient of layers computed from h)
  // layers of every position (computed from h): lay_nat / lay_tr hold [rows][L][r][r] and the
  // gradient w.r.t. the logits of position b goes to dlog[b*ld_dlog + (l*r + z)*r + z'] in the
  // dtype of h (dlog_cols columns, zero beyond L*r*r); dlayers then receives the column sums
  int contextual;
  void* dlog; long long ld_dlog; int dlog_cols;
  float* dlog32;         // fp32 accumulators [rows][L*r*r] (tree; a matrix shared by all steps; a caller's
                         // per-position gradient buffer), converted into dlog at the end when dlog is set
  float* ct;             // binary tree: scratch [rows][steps][r], output of every program step
  float* adj;            // binary tree: scratch [rows][n-1][r], adjoints of the node values
  float* Ge;             // [rows][n][r]
  void* dslT;            // [r][ldb] or nullptr
  long long ldb;
  int bf16;
  float* loss;           // [rows]
  float* dlayers;        // [L][r][r] gradient w.r.t. the layer logits (accumulated), or nullptr
};
hipError_t launch_circuit_bwd(const CircuitBwdArgs& a, hipStream_t st);
constexpr int LAYER_GRAD_ROWS = 256;   // rows whose contribution to a layer gradient one workgroup sums

// Raises a kernel's dynamic-LDS limit the first time the kernel is launched on a device.  This
// is the library's only process-wide state: one bit per kernel and device, set once the call
// has succeeded; threads that race here make the same idempotent call.
template <auto Kern>
inline hipError_t allow_lds(int bytes) {
  static std::atomic<unsigned long long> done{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = (dev >= 0 && dev < 64) ? 1ull << dev : 0ull;
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute((const void*)Kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// Compute units of the current device (asked once per device).
inline hipError_t cu_count(int* n) {
  static std::atomic<int> known[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool slot = dev >= 0 && dev < 64;
  int v = slot ? known[dev].load(std::memory_order_acquire) : 0;
  if (v == 0) {
    e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (slot) known[dev].store(v, std::memory_order_release);
  }
  *n = v;
  return hipSuccess;
}

hipError_t launch_philox_uniforms(int B, int S, int slots, uint32_t seed_lo, uint32_t seed_hi,
                                  uint32_t offset, float* out, hipStream_t st);

// ---- device helpers --------------------------------------------------------
#if defined(__HIPCC__)
// Philox4x32-10 (Salmon et al., SC'11): 10 rounds of two 32x32->64 multiplies.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
  const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int rnd = 0; rnd < 10; ++rnd) {
    if (rnd > 0) { k0 += W0; k1 += W1; }
    uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Uniform of (position b, draft s, slot t): counter (t/4, b, s, offset), word t%4,
// u = (word >> 8) * 2^-24 in [0, 1).
__device__ __forceinline__ float philox_uniform(uint32_t seed_lo, uint32_t seed_hi, uint32_t offset,
                                                uint32_t b, uint32_t s, uint32_t slot) {
  uint32_t w[4];
  philox4x32_10(slot >> 2, b, s, offset, seed_lo, seed_hi, w);
  uint32_t sel = slot & 3u;
  uint32_t word = sel == 0 ? w[0] : sel == 1 ? w[1] : sel == 2 ? w[2] : w[3];
  return (float)(word >> 8) * 5.9604644775390625e-8f;
}

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

// Reductions inside aligned groups of G lanes (G a power of two <= 64); every lane of the group
// gets the result.  The steps inside a row of 16 lanes are data-parallel-primitive moves on the
// operand path (swap neighbours, swap pairs, mirror 8, mirror 16: once the smaller blocks agree, a
// mirror pairs each block with the other one), only the steps across rows go through the LDS
// crossbar - a chain of circuit steps is a chain of these reductions, and a crossbar step costs
// about ten times a move.  All source lanes lie inside the group, so groups that have left do not
// matter.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int x) {
  return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, true);
}
template <class Op>
__device__ __forceinline__ float group_reduce(float x, int G, Op op) {
  if (G >= 2) x = op(x, __int_as_float(dpp_move<0xB1>(__float_as_int(x))));     // quad_perm [1,0,3,2]
  if (G >= 4) x = op(x, __int_as_float(dpp_move<0x4E>(__float_as_int(x))));     // quad_perm [2,3,0,1]
  if (G >= 8) x = op(x, __int_as_float(dpp_move<0x141>(__float_as_int(x))));    // row_half_mirror
  if (G >= 16) x = op(x, __int_as_float(dpp_move<0x140>(__float_as_int(x))));   // row_mirror
  if (G >= 32) x = op(x, __shfl_xor(x, 16));
  if (G >= 64) x = op(x, __shfl_xor(x, 32));
  return x;
}
__device__ __forceinline__ float group_max(float x, int G) {
  return group_reduce(x, G, [](float a, float b) { return fmaxf(a, b); });
}
__device__ __forceinline__ float group_sum(float x, int G) {
  return group_reduce(x, G, [](float a, float b) { return a + b; });
}
__device__ __forceinline__ int group_min(int x, int G) {
  if (G >= 2) x = min(x, dpp_move<0xB1>(x));
  if (G >= 4) x = min(x, dpp_move<0x4E>(x));
  if (G >= 8) x = min(x, dpp_move<0x141>(x));
  if (G >= 16) x = min(x, dpp_move<0x140>(x));
  if (G >= 32) x = min(x, __shfl_xor(x, 16));
  if (G >= 64) x = min(x, __shfl_xor(x, 32));
  return x;
}

// ---- evaluation order of the binary tree (Eq. BTree) ---------------------------
// The order in which the tree's nodes are evaluated does not depend on the data: a
// kernel writes it once as a short program, one step per sum-layer application.
struct TreeStep {
  short m;        // inner node whose layer is applied (0: root, uses log omega instead of a layer)
  short lsrc;     // left operand: >= 0 heap index of a fully observed child, -1 path value, -2 all-ones
  short rsrc;     // right operand, same coding
  short out;      // >= 0: store as full value of node `out`; -1: becomes the path value; -2 - i: emit prefix i
};

__device__ inline int build_tree_program(TreeStep* prog, int n, int prefix) {
  int t = 0;
  for (int m = n - 2; m >= 1; --m) prog[t++] = TreeStep{(short)m, (short)(2 * m + 1), (short)(2 * m + 2), (short)m};
  if (!prefix) {
    prog[t++] = TreeStep{0, 1, 2, (short)(-2 - (n - 1))};
    return t;
  }
  for (int i = 0; i < n; ++i) {
    int idx = n - 1 + i, size = 1;
    while (idx > 0) {
      const int m = (idx - 1) >> 1;
      size <<= 1;
      const int first = (m - (n / size - 1)) * size, last = first + size - 1;
      if (m > 0 && last <= i) { idx = m; continue; }          // fully observed: stored value
      const int half = size >> 1;
      const int l_last = first + half - 1, r_first = first + half;
      const short ls = (l_last <= i) ? (short)(2 * m + 1) : (short)-1;
      const short rs = (r_first > i) ? (short)-2 : (last <= i ? (short)(2 * m + 2) : (short)-1);
      prog[t++] = TreeStep{(short)m, ls, rs, (short)(m > 0 ? -1 : -2 - i)};
      idx = m;
    }
  }
  return t;
}
#endif

inline int tree_program_steps(int n, int prefix) {
  if (!prefix) return n - 2 + 1;
  int lg = 0;
  while ((1 << lg) < n) ++lg;
  return n - 2 + n * lg;          // upper bound: at most log2(n) steps per prefix
}

}  // namespace mtpc
