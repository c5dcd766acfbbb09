// C ABI of libmtpc (include/mtpc.h): argument validation, workspace carve-up and
// the launch sequence of each operation.  Host code only.
#include <cmath>
#include <cstring>
#include <mutex>

#include "mtpc_internal.h"

// Scratch of mtpc_sample_static: one array per GPU the library is loaded on, held until the
// process ends.  In host code this name only stands for the symbol; the array's address on a
// device comes from hipGetSymbolAddress (see static_scratch below) and is what kernels get.
constexpr size_t STATIC_SCRATCH_BYTES = MTPC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace mtpc {
namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct Events { void* start; void* stop; };
enum { PROF_UNEMBED = 0, PROF_CIRCUIT = 1 };
thread_local Events g_prof[2] = {{nullptr, nullptr}, {nullptr, nullptr}};

int n_latents(int family, int n) {
  switch (family) {
    case MTPC_FF: return 0;
    case MTPC_CP: return 1;
    case MTPC_HMM: return n;
    default: return n - 1;
  }
}
int n_layers(int family, int n) {
  if (family == MTPC_HMM) return n - 1;
  if (family == MTPC_BTREE) return n - 2;
  return 0;
}

// Decode-sized batches (B <= 64, bound by the one read of W): the sampling pass also writes
// the table of normalised input units (B*n*r*v floats) and the drafts are scored from it,
// instead of a second pass over W.  Larger batches draw through buckets of (token, selected
// unit) - 1/r of a pass when the buckets are full - and score their drafts with one evidence
// pass, unless the caller asks for the table.  In between (buckets of fewer than 64 rows on
// average) a bucket tile costs as much as a slab of the full pass: when scores are wanted too,
// the one sampling pass that also leaves the table is cheaper than buckets plus a second pass.
// With one unit per layer (r = 1, the fully factorised head) there is nothing to skip and the
// narrower bucket tiles only cost: it always takes the one sampling pass.
bool decode_sized(const mtpc_head* hd) { return hd->B <= 64; }
bool buckets_pay(const mtpc_head* hd, int S, bool want_scores) {
  if (decode_sized(hd) || hd->r < 2) return false;
  return !want_scores || (long long)hd->B * S >= 64LL * hd->r;
}
// Rows per tile of the gathered draws.  A tile takes nearly the same time whatever it holds (its K loop is
// bound by what every stage costs, not by the products), so what counts is the number of rounds the tiles
// make over the CUs: buckets of B S / r rows on average (+- a few standard deviations of the multinomial
// spread) are cut into 128-row tiles or, bf16 only, into 192-row tiles that cost about 1.4 times as much.
int draw_gather_tile(const mtpc_head* hd, int S) {
  if (hd->dtype != MTPC_BF16) return DRAW_GATHER_TILE;
  int cus = 0;
  if (cu_count(&cus) != hipSuccess || cus < 1) cus = 256;
  const double m = (double)hd->B * S / hd->r, top = m + 1.5 * std::sqrt(m);
  const double nb = (double)hd->n * hd->r;
  auto rounds = [&](int tile) { return std::ceil(nb * std::ceil(top / tile) / cus); };
  return 1.4 * rounds(DRAW_GATHER_TILE_WIDE) < rounds(DRAW_GATHER_TILE) ? DRAW_GATHER_TILE_WIDE : DRAW_GATHER_TILE;
}
// A handful of drafts without scores (2 B S <= r, say batch-1 greedy speculative decoding): only
// the n slabs a draft's tokens are drawn from are read, as plain dot products.
bool few_drafts(const mtpc_head* hd, int S) { return 2LL * hd->B * S <= hd->r; }
bool table_fits(const mtpc_head* hd) {
  return (unsigned long long)hd->B * hd->n * hd->r * hd->v * 4ull <= (8ull << 30);
}
bool table_in_workspace(const mtpc_head* hd, int S) {      // for a sampling call that wants scores
  if (buckets_pay(hd, S, true)) return false;
  return table_fits(hd);                                   // else a second pass
}

// The 256-position tiles of the fused kernel read h from a stage-major copy when one can be made: whole
// 64-byte stages per row, and all of it behind one 32-bit buffer resource.
bool stage_major_h_pays(const mtpc_head* hd) {
  const unsigned long long row = (unsigned long long)hd->d * (hd->dtype == MTPC_BF16 ? 2 : 4);
  return hd->B > 64 && row % H_STAGE_BYTES == 0 && row * (unsigned long long)hd->B < (1ull << 32);
}

// most windows per position whose rows B*T*n still index with an int
long long hd_rows_limit(const mtpc_head* hd) {
  if (!hd || hd->B < 1 || hd->n < 1) return 0x7fffffffLL;      // rejected later by check_head
  return 0x7fffffffLL / hd->n / hd->B;
}

struct Plan {           // byte offsets into the workspace
  size_t logw, lay_nat, lay_circ, e, zleaf, lat, logm, table, total;
  size_t hs;            // stage-major copy of h for the 256-position tiles of the fused kernel
  bool has_hs;
  size_t lean_total;    // univariate marginals: the plan without the table
  size_t bk_count, bk_slot, bk_rowoff, bk_tileoff, bk_tilebucket, bk_list;
  size_t rowlogits;     // compact table of the few-drafts path   // buckets of the token draws (large batches)
  int nb, Lst;          // position blocks and stored layers of the normalised copies
  bool has_nat;         // the natural-layout copy of the layers has a place of its own
  bool has_table;       // room for the table of input units (sampling with scores, see decode_sized;
                        // univariate marginals of a head with sum units whose table is at most 8 GiB)
};

mtpc_status check_head(int family, const mtpc_head* hd) {
  if (!hd) return MTPC_ERR_NULL;
  if (!hd->h || !hd->W) return MTPC_ERR_NULL;
  if (family != MTPC_FF && !hd->Wsum) return MTPC_ERR_NULL;
  if (hd->B < 1 || hd->d < 1 || hd->n < 1 || hd->r < 1 || hd->v < 1) return MTPC_ERR_SHAPE;
  if (hd->ld_h < hd->d) return MTPC_ERR_SHAPE;
  if (family == MTPC_FF && hd->r != 1) return MTPC_ERR_SHAPE;
  if (hd->dtype != MTPC_F32 && hd->dtype != MTPC_BF16) return MTPC_ERR_UNSUPPORTED;
  if (hd->d % 32 != 0 || hd->n > 64 || hd->r > 128 || hd->v > 320) return MTPC_ERR_UNSUPPORTED;
  if (family == MTPC_BTREE && (hd->n < 2 || (hd->n & (hd->n - 1)) != 0)) return MTPC_ERR_UNSUPPORTED;
  const size_t esz = hd->dtype == MTPC_BF16 ? 2 : 4;
  if (((uintptr_t)hd->h | (uintptr_t)hd->W | (uintptr_t)hd->Wsum | (uintptr_t)hd->W_stage_major) & 15) return MTPC_ERR_UNSUPPORTED;
  if (((size_t)hd->ld_h * esz) & 15) return MTPC_ERR_UNSUPPORTED;
  if (hd->W_stage_major && hd->W_stage_bytes != 0 && hd->W_stage_bytes != 64 && hd->W_stage_bytes != 128)
    return MTPC_ERR_UNSUPPORTED;
  if ((long long)hd->n * hd->r * hd->v > 0x7fffffffLL) return MTPC_ERR_UNSUPPORTED;
  // a tile (up to 256 rows of h, 320 of W) is addressed through one 32-bit buffer resource
  if ((unsigned long long)hd->ld_h * esz > (1ull << 24) || (unsigned long long)hd->d * esz > (1ull << 23))
    return MTPC_ERR_UNSUPPORTED;
  return MTPC_OK;
}

mtpc_status check_layers(int family, const mtpc_head* hd, const mtpc_sumlayers* ly) {
  if (n_layers(family, hd->n) <= 0) return MTPC_OK;
  if (!ly || (!ly->logits && !ly->R)) return MTPC_ERR_NULL;
  const long long rr = (long long)hd->r * hd->r;
  if (ly->R != nullptr) {          // contextual: logits (optional) are the bias
    if (ly->batch_stride != 0) return MTPC_ERR_SHAPE;
    if (ly->R_layer_stride != 0 && ly->R_layer_stride < rr * hd->d) return MTPC_ERR_SHAPE;
    if ((uintptr_t)ly->R & 15) return MTPC_ERR_UNSUPPORTED;
    if (ly->logits && ly->layer_stride != 0 && ly->layer_stride < rr) return MTPC_ERR_SHAPE;
    return MTPC_OK;
  }
  if (!ly->logits) return MTPC_ERR_NULL;
  if (ly->layer_stride != 0 && ly->layer_stride < rr) return MTPC_ERR_SHAPE;
  if (ly->batch_stride < 0) return MTPC_ERR_SHAPE;
  return MTPC_OK;
}

Plan make_plan(int family, int op, const mtpc_head* hd, const mtpc_sumlayers* ly, int S, int mode,
               bool want_prefix, bool caller_table = false) {
  Plan p{};
  const size_t B = hd->B, n = hd->n, r = hd->r;
  const int L = n_layers(family, hd->n);
  const bool ctx = L > 0 && ly && ly->R != nullptr;      // layers computed from h: one set per position
  if (ctx) {
    const bool bias_shared = !ly->logits || ly->layer_stride == 0;
    p.Lst = (ly->R_layer_stride == 0 && bias_shared) ? 1 : L;
    p.nb = hd->B;
  } else {
    p.Lst = (L > 0 && ly && ly->layer_stride == 0) ? 1 : L;
    p.nb = (L > 0 && ly && ly->batch_stride != 0) ? hd->B : 1;
  }
  const size_t lay_bytes = L > 0 ? up((size_t)p.nb * p.Lst * r * r * 4) : 0;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += up(bytes); return o; };
  p.logw = take(B * r * 4);
  p.has_hs = (op == MTPC_OP_LOGLIK || op == MTPC_OP_MARGINALS || op == MTPC_OP_WINDOWS) && stage_major_h_pays(hd);
  p.hs = p.has_hs ? take(B * (size_t)hd->d * (hd->dtype == MTPC_BF16 ? 2 : 4)) : 0;
  const bool sample = op == MTPC_OP_SAMPLE;
  const bool uni = op == MTPC_OP_MARGINALS && mode == MTPC_MARG_UNIVARIATE;
  const bool verify = op == MTPC_OP_VERIFY;
  const bool table_op = op == MTPC_OP_TABLE || op == MTPC_OP_WINDOWS;   // S windows per position
  // (the tree's matrix-pipe circuit kernel reads shared layers in natural layout)
  const bool need_nat = L > 0 && (family == MTPC_HMM || sample || uni || verify || (family == MTPC_BTREE && !ctx && p.nb == 1));
  const bool need_tr = L > 0 && family == MTPC_BTREE && (!sample || want_prefix) && !uni;
  p.has_nat = need_nat;
  p.lay_nat = need_nat ? take(lay_bytes) : 0;
  p.lay_circ = need_tr ? take(lay_bytes) : p.lay_nat;
  const size_t rows = (sample || table_op) ? B * (size_t)S : B;
  p.e = (uni || verify || (sample && !want_prefix)) ? 0 : take(rows * n * r * 4);
  // (a sampling call that is handed a table to fill scores its drafts from that one)
  p.has_table = sample && want_prefix && !caller_table && table_in_workspace(hd, S);
  p.table = p.has_table ? take(B * n * r * (size_t)hd->v * 4) : 0;
  p.rowlogits = (sample && few_drafts(hd, S)) ? take(B * (size_t)S * n * hd->v * 4) : 0;
  if (sample && !decode_sized(hd)) {
    p.bk_count = take(n * r * 4);
    p.bk_rowoff = take((n * r + 1) * 4);
    p.bk_tileoff = take((n * r + 1) * 4);
    p.bk_tilebucket = take((B * (size_t)S * n / DRAW_GATHER_TILE + n * r) * 4);
    p.bk_slot = take(B * (size_t)S * n * 4);
    p.bk_list = take(B * (size_t)S * n * 4);
  }
  p.zleaf = sample ? take(B * (size_t)S * n * 4) : 0;
  p.lat = sample ? take(B * (size_t)S * (size_t)(n_latents(family, hd->n) + 1) * 4) : 0;
  p.logm = uni ? take(B * n * r * 4) : 0;
  p.lean_total = off;
  if (uni && r > 1 && table_fits(hd)) {       // last, so that a caller may leave it out (see prepare)
    p.has_table = true;
    p.table = take(B * n * r * (size_t)hd->v * 4);
  }
  // a sampling call whose fused kernel runs on the 256-position tiles: the stage-major copy of h, last, so
  // that a caller with a workspace of the older size still runs (see prepare)
  if (sample && stage_major_h_pays(hd) && (want_prefix || caller_table || !buckets_pay(hd, S, want_prefix))) {
    p.has_hs = true;
    p.hs = take(B * (size_t)hd->d * (hd->dtype == MTPC_BF16 ? 2 : 4));
  }
  p.total = off;
  return p;
}

struct ProfScope {
  hipStream_t st;
  const Events& ev;
  explicit ProfScope(hipStream_t s, int which = PROF_UNEMBED) : st(s), ev(g_prof[which]) {
    if (ev.start && ev.stop) (void)hipEventRecord((hipEvent_t)ev.start, st);
  }
  ~ProfScope() {
    if (ev.start && ev.stop) (void)hipEventRecord((hipEvent_t)ev.stop, st);
  }
};

// the circuit kernel of a call, bracketed by the profiling events when they are set
hipError_t profiled_circuit(const CircuitArgs& c, hipStream_t st) {
  ProfScope prof(st, PROF_CIRCUIT);
  return launch_circuit(c, st);
}

#define HIP_TRY(x) do { if ((x) != hipSuccess) return MTPC_ERR_HIP; } while (0)

mtpc_status prepare(int family, int op, const mtpc_head* hd, const mtpc_sumlayers* ly, int S, int mode,
                    bool want_prefix, Plan& plan, bool caller_table = false) {
  mtpc_status st = check_head(family, hd);
  if (st != MTPC_OK) return st;
  st = check_layers(family, hd, ly);
  if (st != MTPC_OK) return st;
  if ((op == MTPC_OP_SAMPLE || op == MTPC_OP_TABLE || op == MTPC_OP_WINDOWS) && S < 1) return MTPC_ERR_SHAPE;
  plan = make_plan(family, op, hd, ly, S, mode, want_prefix, caller_table);
  if (!hd->workspace) return MTPC_ERR_NULL;
  if ((uintptr_t)hd->workspace & 15) return MTPC_ERR_WORKSPACE;
  if (hd->workspace_bytes < plan.total) {
    // univariate marginals run without the table when the workspace has no room for it
    const bool uni = op == MTPC_OP_MARGINALS && mode == MTPC_MARG_UNIVARIATE;
    if (op == MTPC_OP_SAMPLE && plan.has_hs && hd->workspace_bytes >= plan.hs) {
      plan.has_hs = false;         // sampling without the stage-major copy of h (the last carve)
      plan.total = plan.hs;
      return MTPC_OK;
    }
    if (!uni || !plan.has_table || hd->workspace_bytes < plan.lean_total) return MTPC_ERR_WORKSPACE;
    plan.has_table = false;
    plan.total = plan.lean_total;
  }
  return MTPC_OK;
}

// the operands every launch of the fused kernel shares
UnembedArgs unembed_args(const mtpc_head* hd) {
  UnembedArgs u{};
  u.h = hd->h; u.ld_h = hd->ld_h; u.W = hd->W; u.Wp = hd->W_stage_major;
  u.Wp_stage = hd->W_stage_bytes == 0 ? PACK_STAGE_BYTES : hd->W_stage_bytes;
  u.B = hd->B; u.d = hd->d; u.v = hd->v; u.n = hd->n; u.r = hd->r;
  return u;
}

// the stage-major copy of h into the workspace (when the plan has room for it) and into the arguments
hipError_t stage_major_h(const mtpc_head* hd, bool have, size_t off, UnembedArgs& u, hipStream_t st) {
  if (!have) return hipSuccess;
  const int esz = hd->dtype == MTPC_BF16 ? 2 : 4;
  void* dst = (char*)hd->workspace + off;
  u.hs = dst;
  return launch_pack_rows(hd->h, dst, 1, hd->B, hd->d * esz, (long long)hd->ld_h * esz, H_STAGE_BYTES, st);
}

// sum-unit parameters shared by all ops
// `draws` (sampling calls of a few positions): the launch that computes the sum units goes on to
// draw the latents, after the layers those draws read; returns with *draws_done set then.
// `own_sumunit`: the consumer computes its sum units itself (verification of a few positions).
mtpc_status launch_params(int family, const mtpc_head* hd, const mtpc_sumlayers* ly, const Plan& p,
                          bool nat, bool circ, hipStream_t st, const LatentArgs* draws = nullptr,
                          bool* draws_done = nullptr, bool own_sumunit = false) {
  char* ws = (char*)hd->workspace;
  nat = nat && p.has_nat;
  const bool fuse = draws != nullptr && family != MTPC_FF && hd->B <= SUMUNIT_SMALL_B;
  if (draws_done) *draws_done = fuse;
  if (family != MTPC_FF && !fuse && !own_sumunit)
    HIP_TRY(launch_sumunit(hd->h, hd->ld_h, hd->Wsum, hd->B, hd->d, hd->r, hd->dtype,
                           (float*)(ws + p.logw), st));
  const int L = n_layers(family, hd->n);
  if (L > 0 && ly->R != nullptr) {
    CtxLayerArgs c{};
    c.h = hd->h; c.ld_h = hd->ld_h; c.R = ly->R; c.R_layer_stride = ly->R_layer_stride;
    c.bias = ly->logits; c.bias_layer_stride = ly->layer_stride;
    c.B = hd->B; c.d = hd->d; c.r = hd->r; c.L = p.Lst;
    // HMM layers are consumed in natural layout everywhere; the BTree contraction wants [j][k]
    c.out_nat = (nat || (circ && family == MTPC_HMM)) ? (float*)(ws + p.lay_nat) : nullptr;
    c.out_tr = (circ && family == MTPC_BTREE) ? (float*)(ws + p.lay_circ) : nullptr;
    if (c.out_nat || c.out_tr) HIP_TRY(launch_ctx_layers(c, hd->dtype, st));
  } else if (L > 0) {
    float* out_nat = nat ? (float*)(ws + p.lay_nat) : nullptr;
    float* out_tr = (circ && family == MTPC_BTREE) ? (float*)(ws + p.lay_circ) : nullptr;
    HIP_TRY(launch_normalise_layers(ly->logits, ly->layer_stride, ly->batch_stride, p.nb, p.Lst, hd->r,
                                    out_nat, out_tr, st));
  }
  if (fuse)
    HIP_TRY(launch_sumunit_latents(hd->h, hd->ld_h, hd->Wsum, hd->d, hd->dtype, (float*)(ws + p.logw), *draws, st));
  return MTPC_OK;
}

CircuitArgs circuit_args(int family, const mtpc_head* hd, const Plan& p, int rows, int T, float* out,
                         int prefix) {
  char* ws = (char*)hd->workspace;
  CircuitArgs c{};
  c.family = family; c.rows = rows; c.T = T; c.n = hd->n; c.r = hd->r;
  c.e = (const float*)(ws + p.e);
  c.logw = family == MTPC_FF ? nullptr : (const float*)(ws + p.logw);
  c.layers = n_layers(family, hd->n) > 0 ? (const float*)(ws + p.lay_circ) : nullptr;
  c.layers_nat = (c.layers && family == MTPC_BTREE && p.nb == 1 && p.has_nat) ? (const float*)(ws + p.lay_nat) : nullptr;
  c.L = p.Lst; c.contextual = p.nb > 1; c.out = out; c.prefix = prefix;
  return c;
}

// loglik and prefix marginals: params -> fused unembedding (evidence) -> circuit
mtpc_status run_evidence_op(int family, const mtpc_head* hd, const mtpc_sumlayers* ly,
                            const int32_t* targets, float* out, int prefix) {
  if (!targets || !out) return MTPC_ERR_NULL;
  Plan p;
  mtpc_status s = prepare(family, prefix ? MTPC_OP_MARGINALS : MTPC_OP_LOGLIK, hd, ly, 1,
                          MTPC_MARG_PREFIX, false, p);
  if (s != MTPC_OK) return s;
  hipStream_t st = (hipStream_t)hd->stream;
  char* ws = (char*)hd->workspace;
  s = launch_params(family, hd, ly, p, family != MTPC_FF && family != MTPC_CP, true, st);
  if (s != MTPC_OK) return s;
  UnembedArgs u = unembed_args(hd);
  u.targets = targets; u.T = 1; u.e = (float*)(ws + p.e);
  HIP_TRY(stage_major_h(hd, p.has_hs, p.hs, u, st));
  {
    ProfScope prof(st);
    HIP_TRY(launch_unembed(u, hd->dtype, st));
  }
  HIP_TRY(profiled_circuit(circuit_args(family, hd, p, hd->B, 1, out, prefix), st));
  return MTPC_OK;
}

mtpc_status run_univariate(int family, const mtpc_head* hd, const mtpc_sumlayers* ly, float* out) {
  if (!out) return MTPC_ERR_NULL;
  Plan p;
  mtpc_status s = prepare(family, MTPC_OP_MARGINALS, hd, ly, 1, MTPC_MARG_UNIVARIATE, false, p);
  if (s != MTPC_OK) return s;
  hipStream_t st = (hipStream_t)hd->stream;
  char* ws = (char*)hd->workspace;
  s = launch_params(family, hd, ly, p, true, false, st);
  if (s != MTPC_OK) return s;
  UnivariateArgs u{};
  u.h = hd->h; u.ld_h = hd->ld_h; u.W = hd->W;
  u.B = hd->B; u.d = hd->d; u.v = hd->v; u.n = hd->n; u.r = hd->r;
  u.out = out;
  if (family != MTPC_FF) {
    LatentMarginalArgs m{};
    m.family = family; m.B = hd->B; m.n = hd->n; m.r = hd->r;
    m.logw = (const float*)(ws + p.logw);
    m.layers = n_layers(family, hd->n) > 0 ? (const float*)(ws + p.lay_nat) : nullptr;
    m.L = p.Lst; m.contextual = p.nb > 1;
    m.logm = (float*)(ws + p.logm);
    HIP_TRY(launch_latent_marginals(m, st));
    u.logm = m.logm;
  }
  // One pass of the evidence kernel that only writes log phi (the head without sum units: straight
  // into `out`, which is that table), then the mixture over the r units per token.  A table
  // above 8 GiB is not kept: the slabs of a token are then mixed in registers, on smaller tiles.
  if (family == MTPC_FF || p.has_table) {
    UnembedArgs t = unembed_args(hd);
    t.logphi = family == MTPC_FF ? out : (float*)(ws + p.table);
    HIP_TRY(stage_major_h(hd, p.has_hs, p.hs, t, st));
    {
      ProfScope prof(st);
      HIP_TRY(launch_unembed(t, hd->dtype, st));
    }
    if (family != MTPC_FF) HIP_TRY(launch_univariate_table(u, t.logphi, st));
    return MTPC_OK;
  }
  {
    ProfScope prof(st);
    HIP_TRY(launch_univariate(u, hd->dtype, st));
  }
  return MTPC_OK;
}

mtpc_status run_marginals(int family, const mtpc_head* hd, const mtpc_sumlayers* ly,
                          const int32_t* targets, int32_t mode, float* out) {
  if (mode == MTPC_MARG_PREFIX) return run_evidence_op(family, hd, ly, targets, out, 1);
  if (mode == MTPC_MARG_UNIVARIATE) return run_univariate(family, hd, ly, out);
  return MTPC_ERR_UNSUPPORTED;
}

mtpc_status run_sample(int family, const mtpc_head* hd, const mtpc_sumlayers* ly, int32_t S,
                       uint64_t seed, uint32_t offset, int32_t* drafts, int32_t* latents,
                       float* prefix_logq, float* logphi, bool greedy = false) {
  if (!drafts) return MTPC_ERR_NULL;
  const bool want_prefix = prefix_logq != nullptr;
  Plan p;
  mtpc_status s = prepare(family, MTPC_OP_SAMPLE, hd, ly, S, 0, want_prefix, p, logphi != nullptr);
  if (s != MTPC_OK) return s;
  if ((long long)hd->B * S > 0x7fffffffLL / hd->n) return MTPC_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)hd->stream;
  char* ws = (char*)hd->workspace;
  const uint32_t seed_lo = (uint32_t)(seed & 0xffffffffu), seed_hi = (uint32_t)(seed >> 32);

  // Where the tokens are drawn (see decode_sized):
  //   InKernel  - in the epilogue of the fused kernel, which evaluates every slab
  //   Buckets   - k_draw_gather on the one slab each token needs
  //   FromTable - the fused kernel only writes the caller's table, k_draw_table reads it
  // and how the drafts are scored: from the table when there is one, else by one more
  // fused pass with the drafts as targets.
  //   Rows      - k_rows_logits on the n slabs a draft needs, k_draw_table on the compact result
  enum class Draw { InKernel, Buckets, FromTable, Rows };
  const void* hs_ready = nullptr;            // the stage-major copy of h, once a launch of this call has made it
  const size_t esz = hd->dtype == MTPC_BF16 ? 2 : 4;
  const bool span_ok = (unsigned long long)hd->B * (unsigned long long)hd->ld_h * esz <= 0xffffffffull;
  const Draw draw = (!want_prefix && !logphi && few_drafts(hd, S)) ? Draw::Rows
                    : decode_sized(hd) ? Draw::InKernel
                    : logphi         ? Draw::FromTable
                    : span_ok && buckets_pay(hd, S, want_prefix) ? Draw::Buckets   // (h through one 4 GiB resource)
                                     : Draw::InKernel;

  LatentArgs la{};
  la.family = family; la.B = hd->B; la.S = S; la.n = hd->n; la.r = hd->r;
  la.logw = family == MTPC_FF ? nullptr : (const float*)(ws + p.logw);
  la.layers = n_layers(family, hd->n) > 0 ? (const float*)(ws + p.lay_nat) : nullptr;
  la.L = p.Lst; la.contextual = p.nb > 1;
  la.seed_lo = seed_lo; la.seed_hi = seed_hi; la.offset = offset; la.greedy = greedy;
  la.zleaf = (int*)(ws + p.zleaf);
  la.latents = latents ? latents : (int*)(ws + p.lat);
  if (draw == Draw::Buckets) {                            // the launch that draws the latents also clears the bucket counters
    la.zero = (int*)(ws + p.bk_count);
    la.nzero = hd->n * hd->r;
  }
  bool drawn = false;
  s = launch_params(family, hd, ly, p, true, want_prefix, st, &la, &drawn);
  if (s != MTPC_OK) return s;
  if (!drawn) HIP_TRY(launch_latents(la, st));


  const bool table_scores = want_prefix && draw != Draw::Buckets && (logphi != nullptr || p.has_table);
  float* table = logphi ? logphi : (table_scores ? (float*)(ws + p.table) : nullptr);

  if (draw == Draw::Rows) {
    RowLogitArgs rl{};
    rl.h = hd->h; rl.ld_h = hd->ld_h; rl.W = hd->W;
    rl.B = hd->B; rl.S = S; rl.d = hd->d; rl.v = hd->v; rl.n = hd->n; rl.r = hd->r;
    rl.zleaf = la.zleaf; rl.out = (float*)(ws + p.rowlogits);
    HIP_TRY(launch_rows_logits(rl, hd->dtype, st));
    DrawArgs dr{};
    dr.B = hd->B; dr.S = S; dr.v = hd->v; dr.n = hd->n; dr.r = hd->r;
    dr.logphi = rl.out; dr.zleaf = la.zleaf; dr.drafts = drafts; dr.compact = 1;
    dr.seed_lo = seed_lo; dr.seed_hi = seed_hi; dr.offset = offset; dr.greedy = greedy;
    HIP_TRY(launch_draw_table(dr, st));
  } else if (draw == Draw::Buckets) {
    BucketArgs bk{};
    bk.B = hd->B; bk.S = S; bk.n = hd->n; bk.r = hd->r; bk.tile = draw_gather_tile(hd, S);
    bk.zleaf = la.zleaf;
    bk.count = (int*)(ws + p.bk_count); bk.slot = (int*)(ws + p.bk_slot);
    bk.cleared = !drawn;         // (a launch that made the sum units and drew the latents at once did not)
    bk.row_off = (int*)(ws + p.bk_rowoff); bk.tile_off = (int*)(ws + p.bk_tileoff);
    bk.tile_bucket = (int*)(ws + p.bk_tilebucket);
    bk.list = (int*)(ws + p.bk_list);
    HIP_TRY(launch_buckets(bk, st));
    DrawGatherArgs dg{};
    dg.h = hd->h; dg.ld_h = hd->ld_h; dg.W = hd->W;
    dg.Wp = (hd->W_stage_major && hd->W_stage_bytes == GATHER_STAGE_BYTES) ? hd->W_stage_major : nullptr;
    dg.B = hd->B; dg.S = S; dg.d = hd->d; dg.v = hd->v; dg.n = hd->n; dg.r = hd->r;
    dg.row_off = bk.row_off; dg.tile_off = bk.tile_off; dg.tile_bucket = bk.tile_bucket; dg.list = bk.list;
    dg.drafts = drafts;
    dg.seed_lo = seed_lo; dg.seed_hi = seed_hi; dg.offset = offset; dg.greedy = greedy;
    dg.tile = bk.tile;
    HIP_TRY(launch_draw_gather(dg, hd->dtype, st));
  } else {
    UnembedArgs u = unembed_args(hd);
    u.logphi = table;
    HIP_TRY(stage_major_h(hd, p.has_hs, p.hs, u, st));
    hs_ready = u.hs;
    if (draw == Draw::InKernel) {
      u.zleaf = la.zleaf; u.S = S; u.drafts = drafts;
      u.seed_lo = seed_lo; u.seed_hi = seed_hi; u.offset = offset; u.greedy = greedy;
    }
    {
      ProfScope prof(st);
      HIP_TRY(launch_unembed(u, hd->dtype, st));
    }
    if (draw == Draw::FromTable) {
      DrawArgs dr{};
      dr.B = hd->B; dr.S = S; dr.v = hd->v; dr.n = hd->n; dr.r = hd->r;
      dr.logphi = table; dr.zleaf = la.zleaf; dr.drafts = drafts;
      dr.seed_lo = seed_lo; dr.seed_hi = seed_hi; dr.offset = offset; dr.greedy = greedy;
      HIP_TRY(launch_draw_table(dr, st));
    }
  }
  if (want_prefix && !table_scores) {
    UnembedArgs u2 = unembed_args(hd);
    u2.targets = drafts; u2.T = S; u2.e = (float*)(ws + p.e);
    if (hs_ready != nullptr) u2.hs = hs_ready;
    else HIP_TRY(stage_major_h(hd, p.has_hs, p.hs, u2, st));
    ProfScope prof(st);
    HIP_TRY(launch_unembed(u2, hd->dtype, st));
  }
  if (want_prefix) {
    if (table_scores) {
      GatherArgs g{};
      g.B = hd->B; g.S = S; g.v = hd->v; g.n = hd->n; g.r = hd->r;
      g.x = drafts; g.e = (float*)(ws + p.e);
      HIP_TRY(launch_gather_table(g, table, st));
    }
    HIP_TRY(profiled_circuit(circuit_args(family, hd, p, hd->B * S, S, prefix_logq, 1), st));
  }
  return MTPC_OK;
}

// log-likelihoods / prefix marginals of several windows per position, given as two sets
// (say targets and drafts): params -> ONE fused unembedding pass -> circuit
mtpc_status run_window_scores(int family, const mtpc_head* hd, const mtpc_sumlayers* ly, const int32_t* x,
                              int32_t T, const int32_t* x2, int32_t T2, int32_t mode, float* out) {
  if (!x || !out || (T2 > 0 && !x2)) return MTPC_ERR_NULL;
  if (T < 1 || T2 < 0) return MTPC_ERR_SHAPE;
  if (mode != MTPC_SCORE_JOINT && mode != MTPC_SCORE_PREFIX) return MTPC_ERR_UNSUPPORTED;
  const long long TT = (long long)T + T2;
  if (TT > 0x7fffffffLL || (long long)hd_rows_limit(hd) < TT) return MTPC_ERR_UNSUPPORTED;
  Plan p;
  mtpc_status s = prepare(family, MTPC_OP_WINDOWS, hd, ly, (int)TT, 0, false, p);
  if (s != MTPC_OK) return s;
  hipStream_t st = (hipStream_t)hd->stream;
  char* ws = (char*)hd->workspace;
  s = launch_params(family, hd, ly, p, family != MTPC_FF && family != MTPC_CP, true, st);
  if (s != MTPC_OK) return s;
  UnembedArgs u = unembed_args(hd);
  u.targets = x; u.T = T; u.targets2 = x2; u.T2 = T2; u.e = (float*)(ws + p.e);
  HIP_TRY(stage_major_h(hd, p.has_hs, p.hs, u, st));
  {
    ProfScope prof(st);
    HIP_TRY(launch_unembed(u, hd->dtype, st));
  }
  HIP_TRY(profiled_circuit(circuit_args(family, hd, p, hd->B * (int)TT, (int)TT, out, mode == MTPC_SCORE_PREFIX), st));
  return MTPC_OK;
}

// log-likelihoods / prefix marginals of T windows per position from the table of input units
// a sampling call left: params -> gather -> circuit, no pass over W
mtpc_status run_table_scores(int family, const mtpc_head* hd, const mtpc_sumlayers* ly, const float* logphi,
                             const int32_t* x, int32_t T, int32_t mode, float* out) {
  if (!logphi || !x || !out) return MTPC_ERR_NULL;
  if (mode != MTPC_SCORE_JOINT && mode != MTPC_SCORE_PREFIX) return MTPC_ERR_UNSUPPORTED;
  Plan p;
  mtpc_status s = prepare(family, MTPC_OP_TABLE, hd, ly, T, 0, false, p);
  if (s != MTPC_OK) return s;
  if ((long long)hd->B * T > 0x7fffffffLL / hd->n) return MTPC_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)hd->stream;
  char* ws = (char*)hd->workspace;
  s = launch_params(family, hd, ly, p, family != MTPC_FF && family != MTPC_CP, true, st);
  if (s != MTPC_OK) return s;
  GatherArgs g{};
  g.B = hd->B; g.S = T; g.v = hd->v; g.n = hd->n; g.r = hd->r;
  g.x = x; g.e = (float*)(ws + p.e);
  HIP_TRY(launch_gather_table(g, logphi, st));
  HIP_TRY(profiled_circuit(circuit_args(family, hd, p, hd->B * T, T, out, mode == MTPC_SCORE_PREFIX), st));
  return MTPC_OK;
}

mtpc_status run_verify(int family, const mtpc_head* hd, const mtpc_sumlayers* ly, const float* logphi,
                       const int32_t* drafts, const float* prefix_logq, const float* pver, int32_t mode,
                       uint64_t seed, uint32_t offset, int32_t* accepted, int32_t* token) {
  if (!drafts || !pver || !accepted || !token) return MTPC_ERR_NULL;
  if (mode != MTPC_VERIFY_SAMPLING && mode != MTPC_VERIFY_GREEDY) return MTPC_ERR_UNSUPPORTED;
  if (mode == MTPC_VERIFY_SAMPLING && (!prefix_logq || !logphi)) return MTPC_ERR_NULL;
  Plan p;
  mtpc_status s = prepare(family, MTPC_OP_VERIFY, hd, ly, 1, 0, false, p);
  if (s != MTPC_OK) return s;
  hipStream_t st = (hipStream_t)hd->stream;
  char* ws = (char*)hd->workspace;
  const int L = n_layers(family, hd->n);
  // a few positions: each position's workgroup computes its own sum units
  const bool own = family != MTPC_FF && hd->B <= SUMUNIT_SMALL_B;
  if (mode == MTPC_VERIFY_SAMPLING) {
    s = launch_params(family, hd, ly, p, true, family == MTPC_BTREE, st, nullptr, nullptr, own);
    if (s != MTPC_OK) return s;
  }
  VerifyArgs a{};
  a.family = family; a.B = hd->B; a.n = hd->n; a.r = hd->r; a.v = hd->v; a.mode = mode;
  a.logphi = logphi; a.drafts = drafts; a.prefix = prefix_logq; a.p = pver;
  a.logw = (family == MTPC_FF || own) ? nullptr : (const float*)(ws + p.logw);
  if (own) { a.h = hd->h; a.ld_h = hd->ld_h; a.Wsum = hd->Wsum; a.d = hd->d; a.bf16 = hd->dtype == MTPC_BF16; }
  a.lay_nat = L > 0 ? (const float*)(ws + p.lay_nat) : nullptr;
  a.lay_tr = (L > 0 && family == MTPC_BTREE) ? (const float*)(ws + p.lay_circ) : nullptr;
  a.L = p.Lst; a.contextual = p.nb > 1;
  a.seed_lo = (uint32_t)(seed & 0xffffffffu); a.seed_hi = (uint32_t)(seed >> 32); a.offset = offset;
  a.accepted = accepted; a.token = token;
  HIP_TRY(launch_verify(a, st));
  return MTPC_OK;
}

// Workspace of the training step (byte offsets) and its padded strides.
// Rows m of the logit gradient (columns of its transpose): [0, M) unembedding logits,
// [M, M + r) sum-unit logits, then - only when the layers are computed from h - a gap up
// to Mlay (a multiple of 64) and L*r*r layer logits; ldM pads the total to a multiple of 32.
struct BwdPlan {
  size_t logw, e, Ge, dLT, dL, WT, hT, lay_nat, lay_tr, pi, gam, G, Gpart, ct, adj, phi, partial, dlog32, total;
  size_t hs;                // stage-major copy of h for the forward pass
  bool has_hs;
  size_t hTs;               // stage-major copy of hT for the dW contraction
  bool has_hTs;
  int ksplit, kchunk;       // split of the dh contraction over K (few output tiles)
  bool keep_phi;            // probabilities kept by the forward pass (else the logits are recomputed)
  bool ctx;                 // layers computed from h, one set per position
  bool perpos;              // layer logits given per position by the caller
  int Lst;                  // stored layers (1: one matrix shared by all steps)
  int steps;                // reverse-pass steps with a layer (HMM: n-1; tree: program length)
  long long M, Mx, Mlay, Mtot, ldM, ldb;
};

BwdPlan make_bwd_plan(int family, const mtpc_head* hd, const mtpc_sumlayers* ly, bool keep_phi) {
  BwdPlan q{};
  q.keep_phi = keep_phi;
  const size_t esz = hd->dtype == MTPC_BF16 ? 2 : 4;
  const size_t B = hd->B, n = hd->n, r = hd->r;
  const int L = n_layers(family, hd->n);
  q.ctx = L > 0 && ly && ly->R != nullptr;
  q.perpos = L > 0 && ly && !q.ctx && ly->batch_stride != 0;
  if (q.ctx) q.Lst = (ly->R_layer_stride == 0 && (!ly->logits || ly->layer_stride == 0)) ? 1 : L;
  else q.Lst = (L > 0 && ly && ly->layer_stride == 0) ? 1 : L;
  q.M = (long long)hd->n * hd->r * hd->v;
  q.Mx = q.M + (family == MTPC_FF ? 0 : hd->r);      // the sum-unit rows ride along in both contractions
  q.Mlay = q.ctx ? (q.Mx + 63) / 64 * 64 : q.Mx;
  q.Mtot = q.ctx ? q.Mlay + (long long)q.Lst * hd->r * hd->r : q.Mx;
  q.ldM = (q.Mtot + 31) / 32 * 32;
  q.ldb = ((long long)hd->B + 31) / 32 * 32;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += up(bytes); return o; };
  q.logw = take(B * r * 4);
  q.e = take(B * n * r * 4);
  q.Ge = take(B * n * r * 4);
  q.dLT = take((size_t)(q.ctx ? q.ldM : q.Mx) * q.ldb * esz);
  q.dL = take(B * q.ldM * esz);
  q.WT = take((size_t)hd->d * q.ldM * esz);
  q.hT = take((size_t)hd->d * q.ldb * esz);
  q.has_hs = stage_major_h_pays(hd);
  q.hs = q.has_hs ? take(B * (size_t)hd->d * esz) : 0;
  q.has_hTs = (unsigned long long)hd->d * q.ldb * esz < (1ull << 32);
  q.hTs = q.has_hTs ? take((size_t)hd->d * q.ldb * esz) : 0;
  q.steps = family == MTPC_BTREE ? tree_program_steps(hd->n, 1) : L;
  if (L > 0) {
    const size_t lay = ((q.ctx || q.perpos) ? B : 1) * (size_t)q.Lst * r * r * 4;
    q.lay_nat = take(lay);
    if (!q.ctx && !q.perpos) {
      q.lay_tr = take(lay);
      q.pi = take(B * q.steps * r * 4);
      q.gam = take(B * q.steps * r * 4);
      q.G = take((size_t)q.Lst * r * r * 4);
      q.Gpart = take(((B + LAYER_GRAD_ROWS - 1) / LAYER_GRAD_ROWS) * (size_t)q.steps * r * r * 4);
    } else if (q.ctx) {                        // bias gradient: column sums per block of rows
      q.Gpart = take(((B + LAYER_GRAD_ROWS - 1) / LAYER_GRAD_ROWS) * (size_t)q.Lst * r * r * 4);
    }
  }
  if (family == MTPC_BTREE) {
    q.ct = take(B * q.steps * r * 4);
    q.adj = take(B * (n - 1) * r * 4);
  }
  // fp32 accumulation of per-position layer-logit gradients: the tree, or one R for all steps
  if (q.ctx && (family == MTPC_BTREE || (q.Lst == 1 && L > 1))) q.dlog32 = take(B * (size_t)q.Lst * r * r * 4);
  if (keep_phi) q.phi = take((size_t)q.M * q.ldb * 4);
  q.ksplit = gemm_ksplit(hd->B, hd->d, (int)q.ldM);
  q.kchunk = (int)q.ldM;
  if (q.ksplit > 1) {
    q.kchunk = (int)(((q.ldM + q.ksplit - 1) / q.ksplit + 63) / 64 * 64);
    q.ksplit = (int)((q.ldM + q.kchunk - 1) / q.kchunk);
    q.partial = take((size_t)q.ksplit * B * hd->d * 4);
  }
  q.total = off;
  return q;
}

// loss and gradients: forward (evidence, probabilities) -> circuit reverse pass -> logit
// gradient in both layouts -> the two contractions
mtpc_status run_backward(int family, const mtpc_head* hd, const mtpc_sumlayers* ly, const int32_t* targets,
                         const float* coef, float* loss, float* dh, float* dW, float* dWsum, float* dlayers,
                         float* dR) {
  if (!targets || !coef || !loss || !dh || !dW) return MTPC_ERR_NULL;
  if (family != MTPC_FF && !dWsum) return MTPC_ERR_NULL;
  mtpc_status s = check_head(family, hd);
  if (s != MTPC_OK) return s;
  s = check_layers(family, hd, ly);
  if (s != MTPC_OK) return s;
  const int L = n_layers(family, hd->n);
  const bool ctx = L > 0 && ly->R != nullptr;
  if (L > 0) {
    if (ctx) {
      // layers computed from h: R and bias either both one per step / inner node (contiguous)
      // or both shared by all of them
      const long long rr = (long long)hd->r * hd->r;
      const bool per_layer = ly->R_layer_stride == rr * hd->d && (!ly->logits || ly->layer_stride == rr);
      const bool shared = ly->R_layer_stride == 0 && (!ly->logits || ly->layer_stride == 0);
      if (L > 1 && !per_layer && !shared) return MTPC_ERR_UNSUPPORTED;
      if (ly->batch_stride != 0) return MTPC_ERR_SHAPE;
      if (!dR || (ly->logits && !dlayers)) return MTPC_ERR_NULL;
    } else {
      if (!dlayers) return MTPC_ERR_NULL;
      // per position: dense [B][Lst][r][r] logits only
      if (ly->batch_stride != 0) {
        const long long rr = (long long)hd->r * hd->r;
        const long long per = (ly->layer_stride == 0 ? 1 : L) * rr;
        if (ly->batch_stride != per || (ly->layer_stride != 0 && ly->layer_stride != rr)) return MTPC_ERR_UNSUPPORTED;
      }
    }
  }
  // with the larger workspace the forward pass keeps its probabilities (n*r*v*B fp32) and the
  // logit gradient is an elementwise pass; with the smaller one the logits are recomputed
  BwdPlan q = make_bwd_plan(family, hd, ly, true);
  if (!hd->workspace) return MTPC_ERR_NULL;
  if ((uintptr_t)hd->workspace & 15) return MTPC_ERR_WORKSPACE;
  if (hd->workspace_bytes < q.total) q = make_bwd_plan(family, hd, ly, false);
  if (hd->workspace_bytes < q.total) return MTPC_ERR_WORKSPACE;
  if (q.ldM * 4 > 0x7fffffffLL / 320 || q.ldb * 4 > 0x7fffffffLL / 320) return MTPC_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)hd->stream;
  char* ws = (char*)hd->workspace;
  const size_t esz = hd->dtype == MTPC_BF16 ? 2 : 4;
  const long long rr = (long long)hd->r * hd->r;

  // ---- parameters and forward pass
  if (family != MTPC_FF)
    HIP_TRY(launch_sumunit(hd->h, hd->ld_h, hd->Wsum, hd->B, hd->d, hd->r, hd->dtype, (float*)(ws + q.logw), st));
  if (ctx) {
    CtxLayerArgs cl{};
    cl.h = hd->h; cl.ld_h = hd->ld_h; cl.R = ly->R; cl.R_layer_stride = ly->R_layer_stride;
    cl.bias = ly->logits; cl.bias_layer_stride = ly->layer_stride;
    cl.B = hd->B; cl.d = hd->d; cl.r = hd->r; cl.L = q.Lst;
    cl.out_nat = (float*)(ws + q.lay_nat); cl.out_tr = nullptr;
    HIP_TRY(launch_ctx_layers(cl, hd->dtype, st));
  } else if (q.perpos) {
    HIP_TRY(launch_normalise_layers(ly->logits, ly->layer_stride, ly->batch_stride, hd->B, q.Lst, hd->r,
                                    (float*)(ws + q.lay_nat), nullptr, st));
  } else if (L > 0) {
    HIP_TRY(launch_normalise_layers(ly->logits, ly->layer_stride, 0, 1, q.Lst, hd->r,
                                    (float*)(ws + q.lay_nat), (float*)(ws + q.lay_tr), st));
  }
  UnembedArgs u = unembed_args(hd);
  u.targets = targets; u.T = 1; u.e = (float*)(ws + q.e);
  if (q.keep_phi) { u.phiT = (float*)(ws + q.phi); u.ld_phi = q.ldb; }
  HIP_TRY(stage_major_h(hd, q.has_hs, q.hs, u, st));
  HIP_TRY(launch_unembed(u, hd->dtype, st));

  // ---- reverse pass through the circuit
  CircuitBwdArgs c{};
  c.family = family; c.rows = hd->B; c.n = hd->n; c.r = hd->r;
  c.e = (const float*)(ws + q.e);
  c.logw = family == MTPC_FF ? nullptr : (const float*)(ws + q.logw);
  c.coef = coef; c.Ge = (float*)(ws + q.Ge);
  c.dslT = family == MTPC_FF ? nullptr : (void*)(ws + q.dLT + (size_t)q.M * q.ldb * esz);
  c.ldb = q.ldb; c.bf16 = hd->dtype == MTPC_BF16; c.loss = loss;
  if (L > 0) {
    c.lay_nat = (const float*)(ws + q.lay_nat);
    c.lay_tr = (ctx || q.perpos) ? nullptr : (const float*)(ws + q.lay_tr);
    c.L = q.Lst;
    c.dlayers = dlayers;
    if (ctx) {
      c.contextual = 1;
      c.dlog = ws + q.dL + (size_t)q.Mlay * esz; c.ld_dlog = q.ldM; c.dlog_cols = (int)(q.ldM - q.Mlay);
      if (q.dlog32) c.dlog32 = (float*)(ws + q.dlog32);
      c.Gpart = (float*)(ws + q.Gpart);
    } else if (q.perpos) {
      // the caller's [B][Lst][r][r] gradient buffer is the accumulator itself
      c.contextual = 1; c.dlog = nullptr; c.dlog32 = dlayers; c.dlayers = nullptr;
    } else {
      c.pi = (float*)(ws + q.pi); c.gam = (float*)(ws + q.gam); c.G = (float*)(ws + q.G);
      c.Gpart = (float*)(ws + q.Gpart);
    }
  }
  if (family == MTPC_BTREE) {
    c.ct = (float*)(ws + q.ct); c.adj = (float*)(ws + q.adj);
  }
  HIP_TRY(launch_circuit_bwd(c, st));

  // ---- logit gradient in both layouts: dLT [.][ldb] and dL = dLT^T [B][ldM]
  // (stage-major, as the contractions read their 320-row operands, when this kernel writes every element of
  // both - no layer-logit columns from elsewhere - and one 32-bit buffer resource spans each)
  const bool grads_staged = q.keep_phi && !ctx && (unsigned long long)q.M * q.ldb * esz < (1ull << 32) &&
                            (unsigned long long)hd->B * q.ldM * esz < (1ull << 32);
  TransposeArgs t{};
  if (q.keep_phi) {
    GradPhiArgs g{};
    g.phiT = (const float*)(ws + q.phi); g.ld_phi = q.ldb; g.targets = targets; g.Ge = c.Ge;
    g.B = hd->B; g.n = hd->n; g.r = hd->r; g.v = hd->v;
    g.M = q.M; g.Mx = q.Mx; g.ldM = q.ldM; g.ldb = q.ldb;
    g.dl_end = ctx ? q.Mlay : q.ldM;           // the layer-logit columns are written by the reverse pass
    g.dLT = ws + q.dLT; g.dL = ws + q.dL;
    g.staged = grads_staged;
    HIP_TRY(launch_grad_from_phi(g, hd->dtype, st));
  } else {
    GradLogitsArgs g{};
    g.h = hd->h; g.ld_h = hd->ld_h; g.W = hd->W;
    g.B = hd->B; g.d = hd->d; g.v = hd->v; g.n = hd->n; g.r = hd->r;
    g.targets = targets; g.Ge = c.Ge; g.dLT = ws + q.dLT; g.ldb = q.ldb;
    {
      ProfScope prof(st);
      HIP_TRY(launch_unembed_grad(g, hd->dtype, st));
    }
    t.src = ws + q.dLT; t.ld_src = q.ldb; t.R = (int)q.Mx; t.C = hd->B;
    t.dst = ws + q.dL; t.ld_dst = q.ldM; t.col0 = 0; t.Rpad = (int)(ctx ? q.Mlay : q.ldM);
    HIP_TRY(launch_transpose(t, hd->dtype, st));
  }
  if (ctx) {                                 // layer-logit block: written per position, transposed here
    t.src = ws + q.dL + (size_t)q.Mlay * esz; t.ld_src = q.ldM; t.R = hd->B; t.C = (int)(q.ldM - q.Mlay);
    t.dst = ws + q.dLT + (size_t)q.Mlay * q.ldb * esz; t.ld_dst = q.ldb; t.col0 = 0; t.Rpad = (int)q.ldb;
    HIP_TRY(launch_transpose(t, hd->dtype, st));
  }
  // ---- WT = [W; Wsum; (gap); R]^T [d][ldM], hT = h^T [d][ldb]
  // WT is read by the dh contraction only, as its 256-row operand: written stage-major straight away
  // (64-byte stages, [ldM * esz / 64][d][64 bytes]) when one 32-bit buffer resource spans it
  const bool wt_staged = (unsigned long long)hd->d * q.ldM * esz < (1ull << 32);
  t.stage_rows = wt_staged ? hd->d : 0;
  t.src = hd->W; t.ld_src = hd->d; t.R = (int)q.M; t.C = hd->d;
  t.dst = ws + q.WT; t.ld_dst = q.ldM; t.col0 = 0; t.Rpad = (int)(family == MTPC_FF ? q.ldM : q.M);
  HIP_TRY(launch_transpose(t, hd->dtype, st));
  if (family != MTPC_FF) {
    t.src = hd->Wsum; t.ld_src = hd->d; t.R = hd->r; t.C = hd->d;
    t.col0 = q.M; t.Rpad = (int)((ctx ? q.Mlay : q.ldM) - q.M);
    HIP_TRY(launch_transpose(t, hd->dtype, st));
  }
  if (ctx) {
    t.src = ly->R; t.ld_src = hd->d; t.R = (int)(q.Lst * rr); t.C = hd->d;
    t.col0 = q.Mlay; t.Rpad = (int)(q.ldM - q.Mlay);
    HIP_TRY(launch_transpose(t, hd->dtype, st));
  }
  t.stage_rows = 0;                           // hT also feeds the small dWsum kernel: plain, plus a stage-major copy
  t.src = hd->h; t.ld_src = hd->ld_h; t.R = hd->B; t.C = hd->d;
  t.dst = ws + q.hT; t.ld_dst = q.ldb; t.col0 = 0; t.Rpad = (int)q.ldb;
  HIP_TRY(launch_transpose(t, hd->dtype, st));
  if (q.has_hTs)
    HIP_TRY(launch_pack_rows(ws + q.hT, ws + q.hTs, 1, hd->d, (int)(q.ldb * esz), q.ldb * (long long)esz, H_STAGE_BYTES, st));

  // ---- the two contractions
  GemmArgs m{};
  m.A = ws + q.dL; m.lda = q.ldM; m.M = hd->B;                   // dh[b][k] = sum_m dL[b][m] WT[k][m]
  m.Bm = ws + q.WT; m.ldb = q.ldM; m.N = hd->d; m.K = (int)q.ldM;
  m.Bs = wt_staged ? ws + q.WT : nullptr;
  m.As = grads_staged ? ws + q.dL : nullptr; m.As_rows = hd->B;
  m.C = dh; m.ldc = hd->d; m.split = hd->B; m.n2 = 0; m.C2 = nullptr; m.split3 = 0x7fffffff; m.C3 = nullptr;
  m.ksplit = q.ksplit; m.kchunk = q.kchunk; m.partial = q.ksplit > 1 ? (float*)(ws + q.partial) : nullptr;
  HIP_TRY(launch_gemm_tn(m, hd->dtype, st));
  m.ksplit = 1; m.partial = nullptr;
  // dW[m][k] = sum_b dLT[m][b] hT[k][b].  With layers computed from h the r rows of dWsum and,
  // after a gap, those of dR ride along; otherwise the r rows would add one nearly empty row of
  // tiles (n r v is a multiple of the tile height for the 320-token vocabulary: one more round over
  // the CUs), so they get a small kernel of their own.
  const bool own_dwsum = family != MTPC_FF && !ctx;
  m.A = ws + q.dLT; m.lda = q.ldb; m.M = (int)(own_dwsum ? q.M : q.Mtot);
  m.Bm = ws + q.hT; m.ldb = q.ldb; m.N = hd->d; m.K = (int)q.ldb;
  m.Bs = q.has_hTs ? ws + q.hTs : nullptr;
  m.As = grads_staged ? ws + q.dLT : nullptr; m.As_rows = (int)q.M;
  m.C = dW; m.ldc = hd->d;
  m.split = (int)q.M; m.n2 = (family == MTPC_FF || own_dwsum) ? 0 : hd->r; m.C2 = dWsum;
  m.split3 = ctx ? (int)q.Mlay : 0x7fffffff; m.C3 = dR;
  HIP_TRY(launch_gemm_tn(m, hd->dtype, st));
  if (own_dwsum)
    HIP_TRY(launch_dwsum(ws + q.dLT + (size_t)q.M * q.ldb * esz, ws + q.hT, q.ldb, hd->r, hd->d, hd->dtype, dWsum, st));
  return MTPC_OK;
}

// Address of the static scratch array on the current device, looked up once per device.
mtpc_status static_scratch(void** out) {
  constexpr int MAX_DEV = 64;
  static std::mutex mu;
  static void* ptrs[MAX_DEV] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MTPC_ERR_HIP;
  if (dev < 0 || dev >= MAX_DEV) return MTPC_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (ptrs[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return MTPC_ERR_HIP;
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return MTPC_OK;
}

}  // namespace
}  // namespace mtpc

using namespace mtpc;

extern "C" {

const char* mtpc_status_string(mtpc_status s) {
  switch (s) {
    case MTPC_OK: return "ok";
    case MTPC_ERR_NULL: return "a required pointer is NULL";
    case MTPC_ERR_SHAPE: return "a size is non-positive or inconsistent";
    case MTPC_ERR_UNSUPPORTED: return "outside the supported sizes, dtypes or alignment";
    case MTPC_ERR_WORKSPACE: return "workspace too small or misaligned";
    case MTPC_ERR_HIP: return "a HIP call failed";
  }
  return "unknown status";
}

size_t mtpc_workspace_bytes(int32_t family, int32_t op, const mtpc_head* head,
                            const mtpc_sumlayers* layers, int32_t S, int32_t mode) {
  if (family < MTPC_FF || family > MTPC_BTREE || op < MTPC_OP_LOGLIK || op > MTPC_OP_WINDOWS) return 0;
  if (!head || head->B < 1 || head->d < 1 || head->n < 1 || head->r < 1 || head->v < 1) return 0;
  if (op == MTPC_OP_BACKWARD) return make_bwd_plan(family, head, layers, mode != MTPC_BWD_RECOMPUTE).total;
  const bool per_draft = op == MTPC_OP_SAMPLE || op == MTPC_OP_TABLE || op == MTPC_OP_WINDOWS;
  if (per_draft && S < 1) return 0;
  // sized for the most demanding variant of the op (sample: with prefix scores)
  Plan p = make_plan(family, op, head, layers, per_draft ? S : 1, mode, true);
  return p.total;
}

mtpc_status mtpc_ff_loglik(const mtpc_head* head, const int32_t* targets, float* loglik) {
  return run_evidence_op(MTPC_FF, head, nullptr, targets, loglik, 0);
}
mtpc_status mtpc_cp_loglik(const mtpc_head* head, const int32_t* targets, float* loglik) {
  return run_evidence_op(MTPC_CP, head, nullptr, targets, loglik, 0);
}
mtpc_status mtpc_hmm_loglik(const mtpc_head* head, const mtpc_sumlayers* T, const int32_t* targets,
                            float* loglik) {
  return run_evidence_op(MTPC_HMM, head, T, targets, loglik, 0);
}
mtpc_status mtpc_btree_loglik(const mtpc_head* head, const mtpc_sumlayers* A, const int32_t* targets,
                              float* loglik) {
  return run_evidence_op(MTPC_BTREE, head, A, targets, loglik, 0);
}

mtpc_status mtpc_ff_marginals(const mtpc_head* head, const int32_t* targets, int32_t mode, float* out) {
  return run_marginals(MTPC_FF, head, nullptr, targets, mode, out);
}
mtpc_status mtpc_cp_marginals(const mtpc_head* head, const int32_t* targets, int32_t mode, float* out) {
  return run_marginals(MTPC_CP, head, nullptr, targets, mode, out);
}
mtpc_status mtpc_hmm_marginals(const mtpc_head* head, const mtpc_sumlayers* T, const int32_t* targets,
                               int32_t mode, float* out) {
  return run_marginals(MTPC_HMM, head, T, targets, mode, out);
}
mtpc_status mtpc_btree_marginals(const mtpc_head* head, const mtpc_sumlayers* A, const int32_t* targets,
                                 int32_t mode, float* out) {
  return run_marginals(MTPC_BTREE, head, A, targets, mode, out);
}

mtpc_status mtpc_ff_sample(const mtpc_head* head, int32_t S, uint64_t seed, uint32_t offset,
                           int32_t* drafts, int32_t* latents, float* prefix_logq, float* logphi) {
  return run_sample(MTPC_FF, head, nullptr, S, seed, offset, drafts, latents, prefix_logq, logphi);
}
mtpc_status mtpc_cp_sample(const mtpc_head* head, int32_t S, uint64_t seed, uint32_t offset,
                           int32_t* drafts, int32_t* latents, float* prefix_logq, float* logphi) {
  return run_sample(MTPC_CP, head, nullptr, S, seed, offset, drafts, latents, prefix_logq, logphi);
}
mtpc_status mtpc_hmm_sample(const mtpc_head* head, const mtpc_sumlayers* T, int32_t S, uint64_t seed,
                            uint32_t offset, int32_t* drafts, int32_t* latents, float* prefix_logq,
                            float* logphi) {
  return run_sample(MTPC_HMM, head, T, S, seed, offset, drafts, latents, prefix_logq, logphi);
}
mtpc_status mtpc_btree_sample(const mtpc_head* head, const mtpc_sumlayers* A, int32_t S, uint64_t seed,
                              uint32_t offset, int32_t* drafts, int32_t* latents, float* prefix_logq,
                              float* logphi) {
  return run_sample(MTPC_BTREE, head, A, S, seed, offset, drafts, latents, prefix_logq, logphi);
}

mtpc_status mtpc_sample_static(int32_t family, const mtpc_head* head, const mtpc_sumlayers* layers, int32_t S,
                               uint64_t seed, uint32_t offset, int32_t* drafts, int32_t* latents,
                               float* prefix_logq, float* logphi) {
  if (family < MTPC_FF || family > MTPC_BTREE) return MTPC_ERR_UNSUPPORTED;
  if (!head) return MTPC_ERR_NULL;
  mtpc_head hd = *head;                       // the caller's workspace fields are not used
  void* ptr = nullptr;
  const mtpc_status s = static_scratch(&ptr);
  if (s != MTPC_OK) return s;
  hd.workspace = ptr;
  hd.workspace_bytes = STATIC_SCRATCH_BYTES;  // a call that needs more returns MTPC_ERR_WORKSPACE
  return run_sample(family, &hd, layers, S, seed, offset, drafts, latents, prefix_logq, logphi);
}

mtpc_status mtpc_ff_greedy_draft(const mtpc_head* head, int32_t* drafts, int32_t* latents, float* prefix_logq,
                                 float* logphi) {
  return run_sample(MTPC_FF, head, nullptr, 1, 0, 0, drafts, latents, prefix_logq, logphi, true);
}
mtpc_status mtpc_cp_greedy_draft(const mtpc_head* head, int32_t* drafts, int32_t* latents, float* prefix_logq,
                                 float* logphi) {
  return run_sample(MTPC_CP, head, nullptr, 1, 0, 0, drafts, latents, prefix_logq, logphi, true);
}
mtpc_status mtpc_hmm_greedy_draft(const mtpc_head* head, const mtpc_sumlayers* T, int32_t* drafts,
                                  int32_t* latents, float* prefix_logq, float* logphi) {
  return run_sample(MTPC_HMM, head, T, 1, 0, 0, drafts, latents, prefix_logq, logphi, true);
}
mtpc_status mtpc_btree_greedy_draft(const mtpc_head* head, const mtpc_sumlayers* A, int32_t* drafts,
                                    int32_t* latents, float* prefix_logq, float* logphi) {
  return run_sample(MTPC_BTREE, head, A, 1, 0, 0, drafts, latents, prefix_logq, logphi, true);
}

mtpc_status mtpc_ff_verify(const mtpc_head* head, const float* logphi, const int32_t* drafts,
                           const float* prefix_logq, const float* p, int32_t mode, uint64_t seed,
                           uint32_t offset, int32_t* accepted, int32_t* token) {
  return run_verify(MTPC_FF, head, nullptr, logphi, drafts, prefix_logq, p, mode, seed, offset, accepted, token);
}
mtpc_status mtpc_cp_verify(const mtpc_head* head, const float* logphi, const int32_t* drafts,
                           const float* prefix_logq, const float* p, int32_t mode, uint64_t seed,
                           uint32_t offset, int32_t* accepted, int32_t* token) {
  return run_verify(MTPC_CP, head, nullptr, logphi, drafts, prefix_logq, p, mode, seed, offset, accepted, token);
}
mtpc_status mtpc_hmm_verify(const mtpc_head* head, const mtpc_sumlayers* T, const float* logphi,
                            const int32_t* drafts, const float* prefix_logq, const float* p,
                            int32_t mode, uint64_t seed, uint32_t offset, int32_t* accepted,
                            int32_t* token) {
  return run_verify(MTPC_HMM, head, T, logphi, drafts, prefix_logq, p, mode, seed, offset, accepted, token);
}
mtpc_status mtpc_btree_verify(const mtpc_head* head, const mtpc_sumlayers* A, const float* logphi,
                              const int32_t* drafts, const float* prefix_logq, const float* p,
                              int32_t mode, uint64_t seed, uint32_t offset, int32_t* accepted,
                              int32_t* token) {
  return run_verify(MTPC_BTREE, head, A, logphi, drafts, prefix_logq, p, mode, seed, offset, accepted, token);
}

mtpc_status mtpc_ff_window_scores(const mtpc_head* head, const int32_t* x, int32_t T, const int32_t* x2,
                                  int32_t T2, int32_t mode, float* out) {
  return run_window_scores(MTPC_FF, head, nullptr, x, T, x2, T2, mode, out);
}
mtpc_status mtpc_cp_window_scores(const mtpc_head* head, const int32_t* x, int32_t T, const int32_t* x2,
                                  int32_t T2, int32_t mode, float* out) {
  return run_window_scores(MTPC_CP, head, nullptr, x, T, x2, T2, mode, out);
}
mtpc_status mtpc_hmm_window_scores(const mtpc_head* head, const mtpc_sumlayers* T_layers, const int32_t* x,
                                   int32_t T, const int32_t* x2, int32_t T2, int32_t mode, float* out) {
  return run_window_scores(MTPC_HMM, head, T_layers, x, T, x2, T2, mode, out);
}
mtpc_status mtpc_btree_window_scores(const mtpc_head* head, const mtpc_sumlayers* A, const int32_t* x,
                                     int32_t T, const int32_t* x2, int32_t T2, int32_t mode, float* out) {
  return run_window_scores(MTPC_BTREE, head, A, x, T, x2, T2, mode, out);
}

mtpc_status mtpc_ff_table_scores(const mtpc_head* head, const float* logphi, const int32_t* x, int32_t T,
                                 int32_t mode, float* out) {
  return run_table_scores(MTPC_FF, head, nullptr, logphi, x, T, mode, out);
}
mtpc_status mtpc_cp_table_scores(const mtpc_head* head, const float* logphi, const int32_t* x, int32_t T,
                                 int32_t mode, float* out) {
  return run_table_scores(MTPC_CP, head, nullptr, logphi, x, T, mode, out);
}
mtpc_status mtpc_hmm_table_scores(const mtpc_head* head, const mtpc_sumlayers* T_layers, const float* logphi,
                                  const int32_t* x, int32_t T, int32_t mode, float* out) {
  return run_table_scores(MTPC_HMM, head, T_layers, logphi, x, T, mode, out);
}
mtpc_status mtpc_btree_table_scores(const mtpc_head* head, const mtpc_sumlayers* A, const float* logphi,
                                    const int32_t* x, int32_t T, int32_t mode, float* out) {
  return run_table_scores(MTPC_BTREE, head, A, logphi, x, T, mode, out);
}

mtpc_status mtpc_ff_loss_backward(const mtpc_head* head, const int32_t* targets, const float* coef,
                                  float* loss, float* dh, float* dW) {
  return run_backward(MTPC_FF, head, nullptr, targets, coef, loss, dh, dW, nullptr, nullptr, nullptr);
}
mtpc_status mtpc_cp_loss_backward(const mtpc_head* head, const int32_t* targets, const float* coef,
                                  float* loss, float* dh, float* dW, float* dWsum) {
  return run_backward(MTPC_CP, head, nullptr, targets, coef, loss, dh, dW, dWsum, nullptr, nullptr);
}
mtpc_status mtpc_hmm_loss_backward(const mtpc_head* head, const mtpc_sumlayers* T, const int32_t* targets,
                                   const float* coef, float* loss, float* dh, float* dW, float* dWsum,
                                   float* dlayers, float* dR) {
  return run_backward(MTPC_HMM, head, T, targets, coef, loss, dh, dW, dWsum, dlayers, dR);
}
mtpc_status mtpc_btree_loss_backward(const mtpc_head* head, const mtpc_sumlayers* A, const int32_t* targets,
                                     const float* coef, float* loss, float* dh, float* dW, float* dWsum,
                                     float* dlayers, float* dR) {
  return run_backward(MTPC_BTREE, head, A, targets, coef, loss, dh, dW, dWsum, dlayers, dR);
}

mtpc_status mtpc_pack_weights(const mtpc_head* head, void* W_stage_major) {
  if (!head || !W_stage_major) return MTPC_ERR_NULL;
  mtpc_head probe = *head;
  probe.W_stage_major = nullptr;
  if (!probe.Wsum) probe.Wsum = probe.W;                 // (not read here; a head without sum units has none)
  mtpc_status s = check_head(MTPC_CP, &probe);
  if (s != MTPC_OK) return s;
  if ((uintptr_t)W_stage_major & 15) return MTPC_ERR_UNSUPPORTED;
  const long long row_bytes = (long long)head->d * (head->dtype == MTPC_BF16 ? 2 : 4);
  const int stage = head->W_stage_bytes == 0 ? PACK_STAGE_BYTES : head->W_stage_bytes;
  if ((stage != 64 && stage != 128) || row_bytes % stage != 0) return MTPC_ERR_UNSUPPORTED;
  if (launch_pack_rows(head->W, W_stage_major, (long long)head->n * head->r, head->v, (int)row_bytes, row_bytes,
                       stage, (hipStream_t)head->stream) != hipSuccess)
    return MTPC_ERR_HIP;
  return MTPC_OK;
}

mtpc_status mtpc_philox_uniforms(int32_t B, int32_t S, int32_t slots, uint64_t seed, uint32_t offset,
                                 float* out, void* stream) {
  if (!out) return MTPC_ERR_NULL;
  if (B < 1 || S < 1 || slots < 1) return MTPC_ERR_SHAPE;
  if (launch_philox_uniforms(B, S, slots, (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32),
                             offset, out, (hipStream_t)stream) != hipSuccess)
    return MTPC_ERR_HIP;
  return MTPC_OK;
}

void mtpc_profile_unembed(void* start_event, void* stop_event) {
  g_prof[PROF_UNEMBED].start = start_event;
  g_prof[PROF_UNEMBED].stop = stop_event;
}

void mtpc_profile_circuit(void* start_event, void* stop_event) {
  g_prof[PROF_CIRCUIT].start = start_event;
  g_prof[PROF_CIRCUIT].stop = stop_event;
}

}  // extern "C"
