// Host-only stand-ins for the kernel launchers of libmtpc, for the sanitizer build of the ABI layer
// (api.hip: validation, workspace plans, offset arithmetic).  Nothing is launched.  Every launcher
// checks that each buffer it is handed, with the extent its kernel would touch, lies inside one of
// the address ranges the driver registered (the workspace of exactly the size mtpc_workspace_bytes
// promised, and the caller's own buffers at their exact sizes): an offset computed too far, a
// buffer carved too small or an overlap with the end of the workspace aborts the run.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "mtpc_internal.h"

namespace host_check {
struct Range { unsigned long long lo, hi; const char* name; };
std::vector<Range> g_ranges;
int g_launches = 0;
const char* g_case = "";

void reset(const char* what) { g_ranges.clear(); g_launches = 0; g_case = what; }
void add(const void* p, unsigned long long bytes, const char* name) {
  g_ranges.push_back({(unsigned long long)p, (unsigned long long)p + bytes, name});
}
void need(const void* p, unsigned long long bytes, const char* what) {
  if (p == nullptr) {
    std::fprintf(stderr, "[%s] %s: null pointer handed to a launcher\n", g_case, what);
    std::abort();
  }
  const unsigned long long lo = (unsigned long long)p, hi = lo + bytes;
  for (const Range& r : g_ranges)
    if (lo >= r.lo && hi <= r.hi) return;
  std::fprintf(stderr, "[%s] %s: [%llx, %llx) (%llu bytes) is inside no registered buffer\n", g_case, what, lo, hi, bytes);
  for (const Range& r : g_ranges) std::fprintf(stderr, "    %-12s [%llx, %llx)\n", r.name, r.lo, r.hi);
  std::abort();
}
void opt(const void* p, unsigned long long bytes, const char* what) { if (p) need(p, bytes, what); }
}  // namespace host_check

namespace mtpc {
using host_check::need;
using host_check::opt;
typedef unsigned long long u64;

static u64 esz(int dtype) { return dtype == MTPC_BF16 ? 2 : 4; }
static u64 strided(u64 rows, long long ld, u64 cols, u64 es) { return rows ? ((rows - 1) * (u64)ld + cols) * es : 0; }
static int nlat(int family, int n) { return family == MTPC_FF ? 0 : family == MTPC_CP ? 1 : family == MTPC_HMM ? n : n - 1; }
static hipError_t ok() { ++host_check::g_launches; return hipSuccess; }

hipError_t launch_sumunit(const void* h, long long ld_h, const void* Wsum, int B, int d, int r, int dtype, float* logw,
                          hipStream_t) {
  need(h, strided(B, ld_h, d, esz(dtype)), "sumunit h");
  need(Wsum, (u64)r * d * esz(dtype), "sumunit Wsum");
  need(logw, (u64)B * r * 4, "sumunit logw");
  return ok();
}
hipError_t launch_sumunit_mfma(const void* h, long long ld_h, const void* Wsum, int B, int d, int r, int dtype,
                               float* logw, hipStream_t st) {
  return launch_sumunit(h, ld_h, Wsum, B, d, r, dtype, logw, st);
}
hipError_t launch_normalise_layers(const float* logits, long long ls, long long bs, int nb, int L, int r, float* out_nat,
                                   float* out_tr, hipStream_t) {
  need(logits, ((u64)(nb - 1) * bs + (u64)(L - 1) * ls + (u64)r * r) * 4, "normalise logits");
  opt(out_nat, (u64)nb * L * r * r * 4, "normalise out_nat");
  opt(out_tr, (u64)nb * L * r * r * 4, "normalise out_tr");
  return ok();
}
hipError_t launch_ctx_layers(const CtxLayerArgs& a, int dtype, hipStream_t) {
  need(a.h, strided(a.B, a.ld_h, a.d, esz(dtype)), "ctx h");
  need(a.R, ((u64)(a.L - 1) * a.R_layer_stride + (u64)a.r * a.r * a.d) * esz(dtype), "ctx R");
  opt(a.bias, ((u64)(a.L - 1) * a.bias_layer_stride + (u64)a.r * a.r) * 4, "ctx bias");
  opt(a.out_nat, (u64)a.B * a.L * a.r * a.r * 4, "ctx out_nat");
  opt(a.out_tr, (u64)a.B * a.L * a.r * a.r * 4, "ctx out_tr");
  return ok();
}
hipError_t launch_unembed(const UnembedArgs& a, int dtype, hipStream_t) {
  need(a.h, strided(a.B, a.ld_h, a.d, esz(dtype)), "unembed h");
  need(a.W, (u64)a.n * a.r * a.v * a.d * esz(dtype), "unembed W");
  opt(a.Wp, (u64)a.n * a.r * a.v * a.d * esz(dtype), "unembed stage-major W");
  opt(a.hs, (u64)a.B * a.d * esz(dtype), "unembed stage-major h");
  if (a.targets) {
    need(a.targets, (u64)a.B * a.T * a.n * 4, "unembed targets");
    opt(a.targets2, (u64)a.B * a.T2 * a.n * 4, "unembed targets2");
    need(a.e, (u64)a.B * (a.T + a.T2) * a.n * a.r * 4, "unembed e");
  }
  if (a.zleaf) {
    need(a.zleaf, (u64)a.B * a.S * a.n * 4, "unembed zleaf");
    need(a.drafts, (u64)a.B * a.S * a.n * 4, "unembed drafts");
  }
  opt(a.logphi, (u64)a.B * a.n * a.r * a.v * 4, "unembed logphi");
  opt(a.phiT, (u64)a.n * a.r * a.v * a.ld_phi * 4, "unembed phiT");
  return ok();
}
hipError_t launch_univariate(const UnivariateArgs& a, int dtype, hipStream_t) {
  need(a.h, strided(a.B, a.ld_h, a.d, esz(dtype)), "univariate h");
  need(a.W, (u64)a.n * a.r * a.v * a.d * esz(dtype), "univariate W");
  opt(a.logm, (u64)a.B * a.n * a.r * 4, "univariate logm");
  need(a.out, (u64)a.B * a.n * a.v * 4, "univariate out");
  return ok();
}
hipError_t launch_univariate_table(const UnivariateArgs& a, const float* logphi, hipStream_t) {
  need(logphi, (u64)a.B * a.n * a.r * a.v * 4, "univariate table");
  opt(a.logm, (u64)a.B * a.n * a.r * 4, "univariate logm");
  need(a.out, (u64)a.B * a.n * a.v * 4, "univariate out");
  return ok();
}
hipError_t launch_circuit(const CircuitArgs& a, hipStream_t) {
  const u64 pos = (u64)a.rows / a.T;
  need(a.e, (u64)a.rows * a.n * a.r * 4, "circuit e");
  if (a.family != MTPC_FF) need(a.logw, pos * a.r * 4, "circuit logw");
  if (a.layers) need(a.layers, (a.contextual ? pos : 1) * (u64)a.L * a.r * a.r * 4, "circuit layers");
  if (a.layers_nat) need(a.layers_nat, (u64)a.L * a.r * a.r * 4, "circuit layers (natural layout)");
  need(a.out, (u64)a.rows * (a.prefix ? a.n : 1) * 4, "circuit out");
  return ok();
}
hipError_t launch_latents(const LatentArgs& a, hipStream_t) {
  if (a.family != MTPC_FF) need(a.logw, (u64)a.B * a.r * 4, "latents logw");
  if (a.layers) need(a.layers, (a.contextual ? (u64)a.B : 1) * a.L * a.r * a.r * 4, "latents layers");
  need(a.zleaf, (u64)a.B * a.S * a.n * 4, "latents zleaf");
  if (nlat(a.family, a.n) > 0) need(a.latents, (u64)a.B * a.S * nlat(a.family, a.n) * 4, "latents out");
  opt(a.zero, (u64)a.nzero * 4, "latents: counters to clear");
  return ok();
}
hipError_t launch_sumunit_latents(const void* h, long long ld_h, const void* Wsum, int d, int dtype, float* logw,
                                  const LatentArgs& a, hipStream_t st) {
  if (a.B > SUMUNIT_SMALL_B || a.family == MTPC_FF) { std::fprintf(stderr, "fused sum units + latents outside their range\n"); std::abort(); }
  launch_sumunit(h, ld_h, Wsum, a.B, d, a.r, dtype, logw, st);
  --host_check::g_launches;
  return launch_latents(a, st);
}
hipError_t launch_latent_marginals(const LatentMarginalArgs& a, hipStream_t) {
  need(a.logw, (u64)a.B * a.r * 4, "latent marginals logw");
  if (a.layers) need(a.layers, (a.contextual ? (u64)a.B : 1) * a.L * a.r * a.r * 4, "latent marginals layers");
  need(a.logm, (u64)a.B * a.n * a.r * 4, "latent marginals logm");
  return ok();
}
hipError_t launch_gather_table(const GatherArgs& a, const float* logphi, hipStream_t) {
  need(logphi, (u64)a.B * a.n * a.r * a.v * 4, "gather table");
  need(a.x, (u64)a.B * a.S * a.n * 4, "gather x");
  need(a.e, (u64)a.B * a.S * a.n * a.r * 4, "gather e");
  return ok();
}
hipError_t launch_draw_table(const DrawArgs& a, hipStream_t) {
  need(a.logphi, a.compact ? (u64)a.B * a.S * a.n * a.v * 4 : (u64)a.B * a.n * a.r * a.v * 4, "draw table");
  need(a.zleaf, (u64)a.B * a.S * a.n * 4, "draw zleaf");
  need(a.drafts, (u64)a.B * a.S * a.n * 4, "draw drafts");
  return ok();
}
hipError_t launch_rows_logits(const RowLogitArgs& a, int dtype, hipStream_t) {
  need(a.h, strided(a.B, a.ld_h, a.d, esz(dtype)), "rows h");
  need(a.W, (u64)a.n * a.r * a.v * a.d * esz(dtype), "rows W");
  need(a.zleaf, (u64)a.B * a.S * a.n * 4, "rows zleaf");
  need(a.out, (u64)a.B * a.S * a.n * a.v * 4, "rows out");
  return ok();
}
static void bucket_arrays(const int* row_off, const int* tile_off, const int* tile_bucket, const int* list, u64 B, u64 S,
                          u64 n, u64 r, u64 tile) {
  need(row_off, (n * r + 1) * 4, "bucket row_off");
  need(tile_off, (n * r + 1) * 4, "bucket tile_off");
  need(tile_bucket, (B * S * n / tile + n * r) * 4, "bucket tile_bucket");
  need(list, B * S * n * 4, "bucket list");
}
hipError_t launch_buckets(const BucketArgs& a, hipStream_t) {
  need(a.zleaf, (u64)a.B * a.S * a.n * 4, "bucket zleaf");
  need(a.count, (u64)a.n * a.r * 4, "bucket count");
  need(a.slot, (u64)a.B * a.S * a.n * 4, "bucket slot");
  bucket_arrays(a.row_off, a.tile_off, a.tile_bucket, a.list, a.B, a.S, a.n, a.r, a.tile);
  return ok();
}
hipError_t launch_draw_gather(const DrawGatherArgs& a, int dtype, hipStream_t) {
  need(a.h, strided(a.B, a.ld_h, a.d, esz(dtype)), "draw gather h");
  need(a.W, (u64)a.n * a.r * a.v * a.d * esz(dtype), "draw gather W");
  opt(a.Wp, (u64)a.n * a.r * a.v * a.d * esz(dtype), "draw gather stage-major W");
  if (a.tile != DRAW_GATHER_TILE && !(dtype == MTPC_BF16 && a.tile == DRAW_GATHER_TILE_WIDE)) {
    std::fprintf(stderr, "[%s] draw gather: tile height %d\n", host_check::g_case, a.tile);
    std::abort();
  }
  bucket_arrays(a.row_off, a.tile_off, a.tile_bucket, a.list, a.B, a.S, a.n, a.r, a.tile);
  need(a.drafts, (u64)a.B * a.S * a.n * 4, "draw gather drafts");
  return ok();
}
hipError_t launch_verify(const VerifyArgs& a, hipStream_t) {
  need(a.drafts, (u64)a.B * a.n * 4, "verify drafts");
  need(a.p, (u64)a.B * (a.n + 1) * a.v * 4, "verify p");
  if (a.mode == MTPC_VERIFY_SAMPLING) {
    need(a.logphi, (u64)a.B * a.n * a.r * a.v * 4, "verify logphi");
    need(a.prefix, (u64)a.B * a.n * 4, "verify prefix");
    if (a.family != MTPC_FF) {
      if (a.h) {
        need(a.h, strided(a.B, a.ld_h, a.d, a.bf16 ? 2 : 4), "verify h");
        need(a.Wsum, (u64)a.r * a.d * (a.bf16 ? 2 : 4), "verify Wsum");
      } else {
        need(a.logw, (u64)a.B * a.r * 4, "verify logw");
      }
    }
    const u64 lay = (a.contextual ? (u64)a.B : 1) * a.L * a.r * a.r * 4;
    if (a.lay_nat) need(a.lay_nat, lay, "verify lay_nat");
    if (a.lay_tr) need(a.lay_tr, lay, "verify lay_tr");
  }
  need(a.accepted, (u64)a.B * 4, "verify accepted");
  need(a.token, (u64)a.B * 4, "verify token");
  return ok();
}
hipError_t launch_unembed_grad(const GradLogitsArgs& a, int dtype, hipStream_t) {
  need(a.h, strided(a.B, a.ld_h, a.d, esz(dtype)), "grad h");
  need(a.W, (u64)a.n * a.r * a.v * a.d * esz(dtype), "grad W");
  need(a.targets, (u64)a.B * a.n * 4, "grad targets");
  need(a.Ge, (u64)a.B * a.n * a.r * 4, "grad Ge");
  need(a.dLT, (u64)a.n * a.r * a.v * a.ldb * esz(dtype), "grad dLT");
  return ok();
}
hipError_t launch_grad_from_phi(const GradPhiArgs& a, int dtype, hipStream_t) {
  need(a.phiT, (u64)a.M * a.ld_phi * 4, "grad phiT");
  need(a.targets, (u64)a.B * a.n * 4, "grad targets");
  need(a.Ge, (u64)a.B * a.n * a.r * 4, "grad Ge");
  need(a.dLT, (u64)a.Mx * a.ldb * esz(dtype), "grad dLT");
  need(a.dL, (u64)a.B * a.ldM * esz(dtype), "grad dL");
  return ok();
}
hipError_t launch_gemm_tn(const GemmArgs& a, int dtype, hipStream_t) {
  need(a.A, strided(a.M, a.lda, a.K, esz(dtype)), "gemm A");
  need(a.Bm, strided(a.N, a.ldb, a.K, esz(dtype)), "gemm B");
  opt(a.Bs, (u64)a.N * a.K * esz(dtype), "gemm B, stage-major");
  if (a.As) {
    if (a.As_rows < a.M) { std::fprintf(stderr, "gemm: stage-major A with too few rows\n"); std::abort(); }
    need(a.As, (u64)a.As_rows * a.K * esz(dtype), "gemm A, stage-major");
  }
  const int r1 = a.M < a.split ? a.M : a.split;
  need(a.C, strided(r1, a.ldc, a.N, 4), "gemm C");
  if (a.n2 > 0) need(a.C2, strided(a.n2, a.ldc, a.N, 4), "gemm C2");
  if (a.split3 < a.M) need(a.C3, strided(a.M - a.split3, a.ldc, a.N, 4), "gemm C3");
  if (a.ksplit > 1) need(a.partial, (u64)a.ksplit * a.M * a.ldc * 4, "gemm partial");
  return ok();
}
hipError_t launch_transpose(const TransposeArgs& a, int dtype, hipStream_t) {
  if (a.C < 1 || a.Rpad < 1) return hipSuccess;
  need(a.src, strided(a.R, a.ld_src, a.C, esz(dtype)), "transpose src");
  if (a.stage_rows) {                     // stage-major destination: whole 64-byte stages of stage_rows rows
    const u64 eps = 64 / esz(dtype);
    if (a.stage_rows < a.C) { std::fprintf(stderr, "transpose: bad stage-major destination\n"); std::abort(); }
    need(a.dst, ((u64)a.col0 + a.Rpad + eps - 1) / eps * a.stage_rows * 64, "transpose dst, stage-major");
  } else {
    need((const char*)a.dst + (u64)a.col0 * esz(dtype), strided(a.C, a.ld_dst, a.Rpad, esz(dtype)), "transpose dst");
  }
  return ok();
}
hipError_t launch_circuit_bwd(const CircuitBwdArgs& a, hipStream_t) {
  const u64 rows = a.rows;
  const bool tree = a.family == MTPC_BTREE;
  const u64 steps = tree ? tree_program_steps(a.n, 1) : a.n - 1;
  need(a.e, rows * a.n * a.r * 4, "bwd e");
  need(a.coef, rows * a.n * 4, "bwd coef");
  need(a.Ge, rows * a.n * a.r * 4, "bwd Ge");
  need(a.loss, rows * 4, "bwd loss");
  if (a.family != MTPC_FF) {
    need(a.logw, rows * a.r * 4, "bwd logw");
    need(a.dslT, (u64)a.r * a.ldb * (a.bf16 ? 2 : 4), "bwd dslT");
  }
  const u64 lay = (a.contextual ? rows : 1) * a.L * a.r * a.r * 4;
  if (a.lay_nat) need(a.lay_nat, lay, "bwd lay_nat");
  if (a.lay_tr) need(a.lay_tr, lay, "bwd lay_tr");
  if (a.pi) {
    need(a.pi, rows * steps * a.r * 4, "bwd pi");
    need(a.gam, rows * steps * a.r * 4, "bwd gam");
    need(a.G, (u64)a.L * a.r * a.r * 4, "bwd G");
    need(a.Gpart, (rows + LAYER_GRAD_ROWS - 1) / LAYER_GRAD_ROWS * steps * a.r * a.r * 4, "bwd Gpart");
    need(a.dlayers, (u64)a.L * a.r * a.r * 4, "bwd dlayers");
  }
  if (a.dlog) {
    need(a.dlog, strided(rows, a.ld_dlog, a.dlog_cols, a.bf16 ? 2 : 4), "bwd dlog");
    if (a.dlayers) {
      need(a.dlayers, (u64)a.L * a.r * a.r * 4, "bwd bias gradient");
      need(a.Gpart, (rows + LAYER_GRAD_ROWS - 1) / LAYER_GRAD_ROWS * (u64)a.L * a.r * a.r * 4, "bwd column partials");
    }
  }
  if (a.dlog32) need(a.dlog32, rows * a.L * a.r * a.r * 4, "bwd dlog32");
  if (tree) {
    need(a.ct, rows * steps * a.r * 4, "bwd ct");
    need(a.adj, rows * (a.n - 1) * a.r * 4, "bwd adj");
  }
  return ok();
}
hipError_t launch_dwsum(const void* gT, const void* hT, long long ldb, int r, int d, int dtype, float* out, hipStream_t) {
  need(gT, (u64)r * ldb * esz(dtype), "dwsum gT");
  need(hT, (u64)d * ldb * esz(dtype), "dwsum hT");
  need(out, (u64)r * d * 4, "dwsum out");
  return ok();
}
hipError_t launch_pack_rows(const void* src, void* dst, long long slabs, int v, int row_bytes, long long row_stride,
                            int stage_bytes, hipStream_t) {
  if (row_bytes % stage_bytes != 0 || row_stride < row_bytes) { std::fprintf(stderr, "pack: ragged stages\n"); std::abort(); }
  need(src, (u64)(slabs * v - 1) * row_stride + row_bytes, "pack source");
  need(dst, (u64)slabs * v * row_bytes, "pack destination");
  return ok();
}
hipError_t launch_philox_uniforms(int B, int S, int slots, uint32_t, uint32_t, uint32_t, float* out, hipStream_t) {
  need(out, (u64)B * S * slots * 4, "philox out");
  return ok();
}

}  // namespace mtpc
