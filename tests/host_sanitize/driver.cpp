// Drives every entry point of the C ABI (include/mtpc.h) on the host alone, against the stand-in
// launchers of stubs.cpp, in a build with AddressSanitizer and UndefinedBehaviorSanitizer on the
// host side.  Buffers are address ranges that are never dereferenced (no kernel runs); what is
// exercised is argument validation, the workspace plans and all the offset arithmetic between an
// entry point and its launches, from tiny shapes to the largest legal ones.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "mtpc.h"

namespace host_check {
void reset(const char* what);
void add(const void* p, unsigned long long bytes, const char* name);
extern int g_launches;
}  // namespace host_check

namespace {

typedef unsigned long long u64;
u64 g_next = 0x100000000000ull;
struct Buf { void* p; u64 bytes; const char* name; };
std::vector<Buf> g_bufs;      // the caller's buffers of the current case
int g_checked = 0;

void* fake(u64 bytes, const char* name) {
  void* p = (void*)g_next;
  g_next += (bytes + (1ull << 33)) & ~0xfffull;
  g_bufs.push_back({p, bytes, name});
  return p;
}

void begin(const std::string& what, const mtpc_head& hd) {
  static std::string keep;
  keep = what;
  host_check::reset(keep.c_str());
  for (const Buf& b : g_bufs) host_check::add(b.p, b.bytes, b.name);
  if (hd.workspace) host_check::add(hd.workspace, hd.workspace_bytes, "workspace");
}

void expect(int got, int want, const std::string& what) {
  ++g_checked;
  if (got != want) {
    std::fprintf(stderr, "%s: status %d (%s), expected %d\n", what.c_str(), got, mtpc_status_string((mtpc_status)got), want);
    std::exit(1);
  }
}

enum LayerMode { PER_LAYER, SHARED, PER_POSITION, CTX_PER_LAYER, CTX_SHARED };

struct Case {
  int family, dtype, B, d, n, r, v, S;
  LayerMode lm;
  long long ld_h;
};

int n_layers(int family, int n) { return family == MTPC_HMM ? n - 1 : family == MTPC_BTREE ? n - 2 : 0; }
int n_lat(int family, int n) { return family == MTPC_FF ? 0 : family == MTPC_CP ? 1 : family == MTPC_HMM ? n : n - 1; }

void run_case(const Case& c, bool with_backward) {
  g_bufs.clear();
  const u64 es = c.dtype == MTPC_BF16 ? 2 : 4;
  const u64 B = c.B, d = c.d, n = c.n, r = c.r, v = c.v, S = c.S;
  char tag[160];
  std::snprintf(tag, sizeof tag, "family %d dtype %d B %d d %d n %d r %d v %d S %d layers %d", c.family, c.dtype, c.B, c.d,
                c.n, c.r, c.v, c.S, (int)c.lm);
  const std::string T(tag);
  mtpc_head hd{};
  hd.B = c.B; hd.d = c.d; hd.n = c.n; hd.r = c.r; hd.v = c.v; hd.dtype = c.dtype;
  hd.ld_h = c.ld_h ? c.ld_h : c.d;
  hd.h = fake(((B - 1) * (u64)hd.ld_h + d) * es, "h");
  hd.W = fake(n * r * v * d * es, "W");
  hd.Wsum = c.family == MTPC_FF ? nullptr : fake(r * d * es, "Wsum");
  const int L = n_layers(c.family, c.n);
  mtpc_sumlayers ly{};
  const mtpc_sumlayers* lyp = nullptr;
  u64 dlayers_bytes = 0, dR_bytes = 0;
  if (L > 0) {
    const u64 rr = r * r;
    const bool shared = c.lm == SHARED || c.lm == CTX_SHARED;
    const u64 Lst = shared ? 1 : L;
    if (c.lm == PER_POSITION) {
      ly.logits = (const float*)fake(B * Lst * rr * 4, "layer logits");
      ly.layer_stride = rr; ly.batch_stride = Lst * rr;
      dlayers_bytes = B * Lst * rr * 4;
    } else {
      ly.logits = (const float*)fake(Lst * rr * 4, "layer logits");
      ly.layer_stride = shared ? 0 : rr; ly.batch_stride = 0;
      dlayers_bytes = Lst * rr * 4;
    }
    if (c.lm == CTX_PER_LAYER || c.lm == CTX_SHARED) {
      ly.R = fake(Lst * rr * d * es, "R");
      ly.R_layer_stride = shared ? 0 : rr * d;
      dR_bytes = Lst * rr * d * 4;
    }
    lyp = &ly;
  }
  const int stage = B <= 64 ? 128 : 64;  // the stage size the pass over W uses for this batch
  if ((d * es) % stage == 0) {          // the stage-major copy of W, handed to every later call of the case
    void* packed = fake(n * r * v * d * es, "stage-major W");
    hd.W_stage_bytes = stage;
    begin(T + " pack W", hd);
    expect(mtpc_pack_weights(&hd, packed), MTPC_OK, T + " pack W");
    hd.W_stage_major = packed;
    hd.W_stage_bytes = 96;
    begin(T + " stage size that does not exist", hd);
    expect(mtpc_pack_weights(&hd, packed), MTPC_ERR_UNSUPPORTED, T + " stage size that does not exist");
    hd.W_stage_bytes = stage;
  } else {
    void* packed = fake(n * r * v * d * es, "stage-major W");
    begin(T + " pack W, ragged rows", hd);
    expect(mtpc_pack_weights(&hd, packed), MTPC_ERR_UNSUPPORTED, T + " pack W, ragged rows");
  }
  int32_t* targets = (int32_t*)fake(B * n * 4, "targets");
  float* out1 = (float*)fake(B * 4, "loglik");
  float* outP = (float*)fake(B * n * 4, "prefix marginals");
  float* outU = (float*)fake(B * n * v * 4, "univariate marginals");
  int32_t* drafts = (int32_t*)fake(B * S * n * 4, "drafts");
  int32_t* latents = (int32_t*)fake(B * S * (n_lat(c.family, c.n) + 1) * 4, "latents");
  float* scores = (float*)fake(B * S * n * 4, "draft scores");
  float* table = (float*)fake(B * n * r * v * 4, "logphi table");
  float* winout = (float*)fake(B * (S + 1) * n * 4, "window scores");
  float* pver = (float*)fake(B * (n + 1) * v * 4, "verifier p");
  int32_t* acc = (int32_t*)fake(B * 4, "accepted");
  int32_t* tok = (int32_t*)fake(B * 4, "token");
  void* wsbase = (void*)g_next;
  g_next += 1ull << 42;

  auto with_ws = [&](int op, int Sarg, int mode, u64 shrink = 0) {
    const size_t need = mtpc_workspace_bytes(c.family, op, &hd, lyp, Sarg, mode);
    if (need == 0) { std::fprintf(stderr, "%s: workspace query for op %d returned 0\n", tag, op); std::exit(1); }
    hd.workspace = wsbase;
    hd.workspace_bytes = need - shrink;
  };
  auto call4 = [&](auto ff, auto cp, auto hmm, auto bt, auto... args) -> int {
    switch (c.family) {
      case MTPC_FF: return ff(&hd, args...);
      case MTPC_CP: return cp(&hd, args...);
      case MTPC_HMM: return hmm(&hd, lyp, args...);
      default: return bt(&hd, lyp, args...);
    }
  };
  const bool ctx = c.lm == CTX_PER_LAYER || c.lm == CTX_SHARED;

  with_ws(MTPC_OP_LOGLIK, 1, 0);
  begin(T + " loglik", hd);
  expect(call4(mtpc_ff_loglik, mtpc_cp_loglik, mtpc_hmm_loglik, mtpc_btree_loglik, (const int32_t*)targets, out1), MTPC_OK, T + " loglik");
  // one byte less than promised must be refused, before anything is launched
  hd.workspace_bytes -= 1;
  begin(T + " loglik, short workspace", hd);
  expect(call4(mtpc_ff_loglik, mtpc_cp_loglik, mtpc_hmm_loglik, mtpc_btree_loglik, (const int32_t*)targets, out1),
         MTPC_ERR_WORKSPACE, T + " loglik, short workspace");
  if (host_check::g_launches != 0) { std::fprintf(stderr, "%s: launched with a short workspace\n", tag); std::exit(1); }

  with_ws(MTPC_OP_MARGINALS, 1, MTPC_MARG_PREFIX);
  begin(T + " prefix marginals", hd);
  expect(call4(mtpc_ff_marginals, mtpc_cp_marginals, mtpc_hmm_marginals, mtpc_btree_marginals, (const int32_t*)targets,
               (int32_t)MTPC_MARG_PREFIX, outP), MTPC_OK, T + " prefix marginals");
  with_ws(MTPC_OP_MARGINALS, 1, MTPC_MARG_UNIVARIATE);
  begin(T + " univariate marginals", hd);
  expect(call4(mtpc_ff_marginals, mtpc_cp_marginals, mtpc_hmm_marginals, mtpc_btree_marginals, (const int32_t*)nullptr,
               (int32_t)MTPC_MARG_UNIVARIATE, outU), MTPC_OK, T + " univariate marginals");
  if (r > 1 && B * n * r * v * 4 <= (8ull << 30)) {      // the same without room for the table
    with_ws(MTPC_OP_MARGINALS, 1, MTPC_MARG_UNIVARIATE, B * n * r * v * 4);
    begin(T + " univariate marginals, lean", hd);
    expect(call4(mtpc_ff_marginals, mtpc_cp_marginals, mtpc_hmm_marginals, mtpc_btree_marginals, (const int32_t*)nullptr,
                 (int32_t)MTPC_MARG_UNIVARIATE, outU), MTPC_OK, T + " univariate marginals, lean");
  }

  with_ws(MTPC_OP_SAMPLE, c.S, 0);
  for (int variant = 0; variant < 4; ++variant) {
    float* sc = (variant & 1) ? scores : nullptr;
    float* tb = (variant & 2) ? table : nullptr;
    begin(T + " sample v" + std::to_string(variant), hd);
    expect(call4(mtpc_ff_sample, mtpc_cp_sample, mtpc_hmm_sample, mtpc_btree_sample, (int32_t)c.S, (uint64_t)0x123456789abcdefull,
                 (uint32_t)7, drafts, (variant == 0 ? (int32_t*)nullptr : latents), sc, tb), MTPC_OK, T + " sample");
  }
  with_ws(MTPC_OP_SAMPLE, 1, 0);
  {
    // (greedy drafts are [B][n]: S = 1)
    begin(T + " greedy draft", hd);
    expect(call4(mtpc_ff_greedy_draft, mtpc_cp_greedy_draft, mtpc_hmm_greedy_draft, mtpc_btree_greedy_draft, drafts, latents,
                 scores, table), MTPC_OK, T + " greedy draft");
  }
  with_ws(MTPC_OP_WINDOWS, c.S + 1, 0);
  begin(T + " window scores", hd);
  expect(call4(mtpc_ff_window_scores, mtpc_cp_window_scores, mtpc_hmm_window_scores, mtpc_btree_window_scores,
               (const int32_t*)targets, (int32_t)1, (const int32_t*)drafts, (int32_t)c.S, (int32_t)MTPC_SCORE_PREFIX, winout),
         MTPC_OK, T + " window scores");
  with_ws(MTPC_OP_TABLE, c.S, 0);
  begin(T + " table scores", hd);
  expect(call4(mtpc_ff_table_scores, mtpc_cp_table_scores, mtpc_hmm_table_scores, mtpc_btree_table_scores,
               (const float*)table, (const int32_t*)drafts, (int32_t)c.S, (int32_t)MTPC_SCORE_JOINT, winout), MTPC_OK, T + " table scores");
  with_ws(MTPC_OP_VERIFY, 1, 0);
  for (int mode : {MTPC_VERIFY_SAMPLING, MTPC_VERIFY_GREEDY}) {
    begin(T + " verify", hd);
    expect(call4(mtpc_ff_verify, mtpc_cp_verify, mtpc_hmm_verify, mtpc_btree_verify, (const float*)table,
                 (const int32_t*)drafts, (const float*)scores, (const float*)pver, (int32_t)mode, (uint64_t)1, (uint32_t)2, acc, tok),
           MTPC_OK, T + " verify");
  }
  if (with_backward) {
    float* coef = (float*)fake(B * n * 4, "coef");
    float* loss = (float*)fake(B * 4, "loss");
    float* dh = (float*)fake(B * d * 4, "dh");
    float* dW = (float*)fake(n * r * v * d * 4, "dW");
    float* dWsum = c.family == MTPC_FF ? nullptr : (float*)fake(r * d * 4, "dWsum");
    float* dlayers = dlayers_bytes ? (float*)fake(dlayers_bytes, "dlayers") : nullptr;
    float* dR = dR_bytes ? (float*)fake(dR_bytes, "dR") : nullptr;
    for (int mode : {MTPC_BWD_KEEP_PROBS, MTPC_BWD_RECOMPUTE}) {
      with_ws(MTPC_OP_BACKWARD, 1, mode);
      begin(T + " loss_backward", hd);
      int st;
      switch (c.family) {
        case MTPC_FF: st = mtpc_ff_loss_backward(&hd, targets, coef, loss, dh, dW); break;
        case MTPC_CP: st = mtpc_cp_loss_backward(&hd, targets, coef, loss, dh, dW, dWsum); break;
        case MTPC_HMM: st = mtpc_hmm_loss_backward(&hd, lyp, targets, coef, loss, dh, dW, dWsum, dlayers, dR); break;
        default: st = mtpc_btree_loss_backward(&hd, lyp, targets, coef, loss, dh, dW, dWsum, dlayers, dR); break;
      }
      expect(st, MTPC_OK, T + " loss_backward mode " + std::to_string(mode));
    }
  }
  (void)ctx;
}

void argument_errors() {
  g_bufs.clear();
  mtpc_head hd{};
  hd.B = 4; hd.d = 64; hd.n = 4; hd.r = 2; hd.v = 16; hd.dtype = MTPC_BF16;
  hd.h = fake(4 * 64 * 2, "h"); hd.ld_h = 64; hd.W = fake(4 * 2 * 16 * 64 * 2, "W"); hd.Wsum = fake(2 * 64 * 2, "Wsum");
  hd.workspace = fake(1 << 20, "ws"); hd.workspace_bytes = 1 << 20;
  int32_t* tg = (int32_t*)fake(64, "tg");
  float* out = (float*)fake(64, "out");
  begin("argument errors", hd);
  auto with = [&](auto edit) { mtpc_head h2 = hd; edit(h2); return h2; };
  mtpc_head t;
  expect(mtpc_cp_loglik(nullptr, tg, out), MTPC_ERR_NULL, "null head");
  expect(mtpc_cp_loglik(&hd, nullptr, out), MTPC_ERR_NULL, "null targets");
  t = with([](mtpc_head& h) { h.h = nullptr; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_NULL, "null h");
  t = with([](mtpc_head& h) { h.B = 0; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_SHAPE, "B = 0");
  t = with([](mtpc_head& h) { h.B = -5; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_SHAPE, "B < 0");
  t = with([](mtpc_head& h) { h.ld_h = 32; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_SHAPE, "ld_h < d");
  t = with([](mtpc_head& h) { h.d = 48; h.ld_h = 48; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_UNSUPPORTED, "d % 32");
  t = with([](mtpc_head& h) { h.n = 65; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_UNSUPPORTED, "n > 64");
  t = with([](mtpc_head& h) { h.r = 129; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_UNSUPPORTED, "r > 128");
  t = with([](mtpc_head& h) { h.v = 321; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_UNSUPPORTED, "v > 320");
  t = with([](mtpc_head& h) { h.dtype = 7; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_UNSUPPORTED, "dtype");
  t = with([](mtpc_head& h) { h.B = 0x7fffffff; h.n = 64; h.r = 128; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_WORKSPACE, "huge B");
  t = with([](mtpc_head& h) { h.workspace = nullptr; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_NULL, "null workspace");
  t = with([](mtpc_head& h) { h.workspace_bytes = 8; }); expect(mtpc_cp_loglik(&t, tg, out), MTPC_ERR_WORKSPACE, "tiny workspace");
  t = with([](mtpc_head& h) { h.n = 6; }); expect(mtpc_btree_loglik(&t, nullptr, tg, out), MTPC_ERR_UNSUPPORTED, "tree over 6 tokens");
  expect(mtpc_hmm_loglik(&hd, nullptr, tg, out), MTPC_ERR_NULL, "hmm without layers");
  // sizes that leave the 32-bit row index: refused, never wrapped
  t = with([](mtpc_head& h) { h.B = 1 << 20; h.n = 64; h.workspace_bytes = ~(size_t)0 >> 1; });
  expect(mtpc_cp_sample(&t, 64, 0, 0, (int32_t*)tg, nullptr, nullptr, nullptr), MTPC_ERR_UNSUPPORTED, "B S n beyond 2^31");
  expect(mtpc_cp_window_scores(&t, tg, 0x7fffffff, tg, 0x7fffffff, MTPC_SCORE_JOINT, out), MTPC_ERR_UNSUPPORTED, "T + T2 overflow");
  expect(mtpc_cp_table_scores(&t, out, tg, 1 << 20, MTPC_SCORE_JOINT, out), MTPC_ERR_UNSUPPORTED, "B T n beyond 2^31");
  expect(mtpc_philox_uniforms(1, 1, 0, 0, 0, out, nullptr), MTPC_ERR_SHAPE, "no slots");
  if (mtpc_workspace_bytes(MTPC_CP, MTPC_OP_SAMPLE, &hd, nullptr, 0, 0) != 0 ||
      mtpc_workspace_bytes(9, MTPC_OP_SAMPLE, &hd, nullptr, 1, 0) != 0 ||
      mtpc_workspace_bytes(MTPC_CP, 99, &hd, nullptr, 1, 0) != 0 || mtpc_workspace_bytes(MTPC_CP, MTPC_OP_LOGLIK, nullptr, nullptr, 1, 0) != 0) {
    std::fprintf(stderr, "workspace query accepted invalid arguments\n");
    std::exit(1);
  }
  if (host_check::g_launches != 0) { std::fprintf(stderr, "an argument error launched something\n"); std::exit(1); }
}

}  // namespace

int main() {
  argument_errors();
  const LayerMode modes[] = {PER_LAYER, SHARED, PER_POSITION, CTX_PER_LAYER, CTX_SHARED};
  // small and ragged shapes, every family and layer form, both dtypes, with the training step
  for (int dtype : {MTPC_F32, MTPC_BF16}) {
    run_case({MTPC_FF, dtype, 70, 64, 5, 1, 100, 3, PER_LAYER, 96}, true);
    run_case({MTPC_CP, dtype, 300, 128, 8, 16, 320, 2, PER_LAYER, 0}, true);
    run_case({MTPC_CP, dtype, 1, 32, 1, 1, 1, 1, PER_LAYER, 0}, true);
    for (LayerMode lm : modes) {
      run_case({MTPC_HMM, dtype, 65, 64, 6, 7, 130, 2, lm, 0}, true);
      run_case({MTPC_HMM, dtype, 3, 96, 1, 5, 33, 1, lm, 0}, true);          // a window of one token: no layer at all
      run_case({MTPC_BTREE, dtype, 97, 64, 16, 8, 257, 2, lm, 0}, true);
      run_case({MTPC_BTREE, dtype, 9, 32, 2, 3, 7, 4, lm, 0}, true);         // two leaves: root only
    }
  }
  // the named workloads at full size, with the training step
  run_case({MTPC_CP, MTPC_F32, 64, 256, 4, 8, 256, 4, PER_LAYER, 0}, true);
  run_case({MTPC_FF, MTPC_BF16, 8192, 4096, 8, 1, 320, 1, PER_LAYER, 0}, true);
  run_case({MTPC_CP, MTPC_BF16, 8192, 4096, 8, 16, 320, 1, PER_LAYER, 0}, true);
  run_case({MTPC_HMM, MTPC_BF16, 8192, 4096, 8, 32, 320, 1, SHARED, 0}, true);
  run_case({MTPC_HMM, MTPC_BF16, 8192, 4096, 8, 32, 320, 1, CTX_PER_LAYER, 0}, true);
  run_case({MTPC_BTREE, MTPC_BF16, 4096, 3072, 16, 64, 320, 1, PER_LAYER, 0}, true);
  run_case({MTPC_BTREE, MTPC_F32, 2048, 3072, 16, 32, 268, 1, CTX_PER_LAYER, 0}, true);
  for (int B : {1, 8, 64}) run_case({MTPC_CP, MTPC_BF16, B, 4096, 16, 32, 320, 1, PER_LAYER, 0}, false);
  // the largest legal sizes: row indices next to 2^31, the 8 GiB table of the univariate pass,
  // the longest window with the most units, the longest rows
  run_case({MTPC_CP, MTPC_BF16, 1 << 20, 32, 64, 2, 2, 30, PER_LAYER, 0}, false);
  run_case({MTPC_BTREE, MTPC_BF16, 8192, 64, 16, 64, 256, 1, PER_LAYER, 0}, true);
  run_case({MTPC_BTREE, MTPC_F32, 4096, 256, 64, 128, 320, 2, PER_LAYER, 0}, false);   // (the training step stops at n r v + r + L r r <= 1,677,696)
  run_case({MTPC_BTREE, MTPC_BF16, 4096, 256, 64, 128, 320, 2, PER_LAYER, 0}, false);
  run_case({MTPC_BTREE, MTPC_BF16, 300, 128, 64, 64, 320, 1, PER_LAYER, 0}, true);    // the longest logit row the training step takes
  run_case({MTPC_HMM, MTPC_BF16, 4096, 256, 64, 128, 320, 2, PER_POSITION, 0}, false);
  run_case({MTPC_HMM, MTPC_BF16, 500, 256, 64, 64, 320, 2, PER_POSITION, 0}, true);
  run_case({MTPC_HMM, MTPC_F32, 70, 512, 64, 128, 320, 1, CTX_PER_LAYER, 0}, false);
  run_case({MTPC_HMM, MTPC_F32, 70, 512, 64, 32, 320, 1, CTX_PER_LAYER, 0}, true);
  run_case({MTPC_CP, MTPC_F32, 3, 2097152, 1, 2, 3, 1, PER_LAYER, 4194304}, true);
  run_case({MTPC_CP, MTPC_BF16, 100000, 8192, 64, 128, 320, 1, PER_LAYER, 0}, false);
  std::printf("host sanitizer run: %d calls checked\n", g_checked);
  return 0;
}
