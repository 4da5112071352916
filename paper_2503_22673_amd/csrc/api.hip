// C interface: argument checks, the host half of packing, the workspace plan
// and the launch sequence of one training step.
#include "common.h"
#include "host_logic.h"
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <vector>
#include <algorithm>
#include <cmath>
#include <mutex>

static_assert((size_t)AS_GEMM_TAIL_SCRATCH_BYTES == kGemmTailFloats * 4, "header and kernel agree on the tail scratch");
static thread_local std::string g_tls_err;

int as_fail(as_ctx* ctx, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
  g_tls_err = buf;
  if (ctx) ctx->err = buf;
  return code;
}

// ------------------------------------------------------------------ context
static const char* kTargetName[AS_N_TARGETS] = {"q", "k", "v", "o", "gate", "up", "down", "router"};

extern "C" int as_create(as_ctx** out, const as_model_config* cfg, int device) {
  if (!out || !cfg) return as_fail(nullptr, AS_ERR_NULL, "as_create: NULL argument");
  std::string err;
  int rc = check_config(cfg, &err);
  if (rc) return as_fail(nullptr, rc, "%s", err.c_str());
  as_ctx* c = new as_ctx();
  c->cfg = *cfg;
  c->device = device;
  *out = c;
  return AS_OK;
}

// Brackets may nest (a launcher that calls other launchers): only the outermost pair records.
void prof_begin(as_ctx* ctx, hipStream_t st, int cls, double flops) {
  if (!ctx || !ctx->prof_on) return;
  if (ctx->prof_depth++ > 0) return;
  if (ctx->prof_only >= 0 && cls != ctx->prof_only) { ctx->prof_skipping = true; return; }
  if (ctx->prof_used >= 65536) return;
  if (ctx->prof_used >= ctx->prof.size()) {
    as_ctx::ProfRec r; r.flops = 0; r.cls = 0;
    if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) { ctx->prof_on = false; return; }
    ctx->prof.push_back(r);
  }
  as_ctx::ProfRec& r = ctx->prof[ctx->prof_used];
  r.flops = flops; r.cls = cls;
  (void)hipEventRecord(r.a, st);
}
void prof_end(as_ctx* ctx, hipStream_t st) {
  if (!ctx || !ctx->prof_on) return;
  if (--ctx->prof_depth > 0) return;
  if (ctx->prof_skipping) { ctx->prof_skipping = false; return; }
  if (ctx->prof_used >= 65536 || ctx->prof_used >= ctx->prof.size()) return;
  (void)hipEventRecord(ctx->prof[ctx->prof_used].b, st);
  ctx->prof_used++;
}

extern "C" int as_profile(as_ctx* ctx, int enable) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_profile: NULL context");
  AS_HIP(ctx, hipSetDevice(ctx->device));
  AS_HIP(ctx, hipDeviceSynchronize());
  ctx->prof_on = enable != 0;
  ctx->prof_used = 0; ctx->prof_depth = 0; ctx->prof_skipping = false;
  return AS_OK;
}

extern "C" int as_profile_only(as_ctx* ctx, int kernel_class) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_profile_only: NULL context");
  if (kernel_class >= AS_K_N_CLASSES) return as_fail(ctx, AS_ERR_SHAPE, "as_profile_only: unknown kernel class");
  if (ctx->prof_on) return as_fail(ctx, AS_ERR_SHAPE, "as_profile_only: set the class before as_profile(ctx, 1)");
  ctx->prof_only = kernel_class < 0 ? -1 : kernel_class;
  return AS_OK;
}

extern "C" int as_profile_read(as_ctx* ctx, int kernel_class, int64_t* launches, double* ms, double* flops) {
  if (!ctx || !launches || !ms || !flops) return as_fail(ctx, AS_ERR_NULL, "as_profile_read: NULL argument");
  if (kernel_class < 0 || kernel_class >= AS_K_N_CLASSES) return as_fail(ctx, AS_ERR_SHAPE, "as_profile_read: unknown kernel class");
  AS_HIP(ctx, hipSetDevice(ctx->device));
  AS_HIP(ctx, hipDeviceSynchronize());
  int64_t n = 0; double t = 0, f = 0;
  size_t used = ctx->prof_used < ctx->prof.size() ? ctx->prof_used : ctx->prof.size();
  for (size_t i = 0; i < used; i++) {
    const as_ctx::ProfRec& r = ctx->prof[i];
    if (r.cls != kernel_class) continue;
    float e = 0.f;
    AS_HIP(ctx, hipEventElapsedTime(&e, r.a, r.b));
    n++; t += e; f += r.flops;
  }
  *launches = n; *ms = t; *flops = f;
  return AS_OK;
}

extern "C" int as_probe_lds_feed(as_ctx* ctx, int32_t loads_in_flight, const void* d_buf, size_t span_bytes, int32_t iters,
                                 int32_t blocks, int32_t* d_sink, double* gbps, void* stream) {
  if (!ctx || !d_buf || !d_sink || !gbps) return as_fail(ctx, AS_ERR_NULL, "as_probe_lds_feed: NULL argument");
  if (span_bytes < 65536 || (span_bytes & (span_bytes - 1)) || iters < 1 || blocks < 1 || iters > (1 << 20) || blocks > (1 << 16))
    return as_fail(ctx, AS_ERR_SHAPE, "as_probe_lds_feed: span a power of two >= 64 KB, iters in [1, 2^20], blocks in [1, 2^16]");
  hipStream_t st = (hipStream_t)stream;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  hipEvent_t a, b;
  AS_HIP(ctx, hipEventCreate(&a)); AS_HIP(ctx, hipEventCreate(&b));
  int rc = launch_feed_probe(ctx, loads_in_flight, d_buf, span_bytes, iters / 8 + 1, blocks, d_sink, st);   // warm-up
  if (!rc) { (void)hipEventRecord(a, st); rc = launch_feed_probe(ctx, loads_in_flight, d_buf, span_bytes, iters, blocks, d_sink, st); (void)hipEventRecord(b, st); }
  hipError_t e = hipEventSynchronize(b);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
  (void)hipEventDestroy(a); (void)hipEventDestroy(b);
  if (rc) return rc;
  if (e != hipSuccess) return as_fail(ctx, AS_ERR_HIP, "as_probe_lds_feed: %s", hipGetErrorString(e));
  *gbps = (double)blocks * iters * 8.0 * loads_in_flight * 1024.0 / (ms * 1e-3) / 1e9;
  return AS_OK;
}

extern "C" int as_probe_mfma_peak(as_ctx* ctx, int32_t iters, int32_t blocks, float* d_sink, double* tflops, void* stream) {
  if (!ctx || !d_sink || !tflops) return as_fail(ctx, AS_ERR_NULL, "as_probe_mfma_peak: NULL argument");
  if (iters < 1 || blocks < 1 || iters > (1 << 24) || blocks > (1 << 20)) return as_fail(ctx, AS_ERR_SHAPE, "as_probe_mfma_peak: iters in [1, 2^24], blocks in [1, 2^20]");
  hipStream_t st = (hipStream_t)stream;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  hipEvent_t a, b;
  AS_HIP(ctx, hipEventCreate(&a)); AS_HIP(ctx, hipEventCreate(&b));
  int rc = launch_mfma_peak(ctx, iters, blocks, d_sink, st);            // warm-up
  if (!rc) { (void)hipEventRecord(a, st); rc = launch_mfma_peak(ctx, iters, blocks, d_sink, st); (void)hipEventRecord(b, st); }
  hipError_t e = hipEventSynchronize(b);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
  (void)hipEventDestroy(a); (void)hipEventDestroy(b);
  if (rc) return rc;
  if (e != hipSuccess) return as_fail(ctx, AS_ERR_HIP, "as_probe_mfma_peak: %s", hipGetErrorString(e));
  *tflops = (double)blocks * 8.0 * iters * 8.0 * 32768.0 / (ms * 1e-3) / 1e12;
  return AS_OK;
}

extern "C" void as_destroy(as_ctx* ctx) {
  if (!ctx) return;
  for (auto& r : ctx->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  if (ctx->d_stage) (void)hipFree(ctx->d_stage);
  if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
  delete ctx;
}

extern "C" const char* as_last_error(const as_ctx* ctx) {
  return ctx ? ctx->err.c_str() : g_tls_err.c_str();
}

// ------------------------------------------------------------------- pack

static int ensure_stage(as_ctx* ctx, size_t bytes) {
  if (bytes > ctx->d_stage_bytes) {
    if (ctx->d_stage) (void)hipFree(ctx->d_stage);
    ctx->d_stage = nullptr; ctx->d_stage_bytes = 0;
    AS_HIP(ctx, hipMalloc(&ctx->d_stage, bytes));
    ctx->d_stage_bytes = bytes;
  }
  if (bytes > ctx->h_stage_bytes) {
    if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
    ctx->h_stage = nullptr; ctx->h_stage_bytes = 0;
    AS_HIP(ctx, hipHostMalloc(&ctx->h_stage, bytes, hipHostMallocDefault));
    ctx->h_stage_bytes = bytes;
  }
  return AS_OK;
}

extern "C" int as_pack_policy(as_ctx* ctx, const int32_t* turn_tokens, const int32_t* turn_offsets,
                              const uint8_t* turn_roles, const int32_t* traj_offsets, int32_t n_traj,
                              int32_t row_len, int32_t max_rows, int32_t pad_id, int32_t truncate, int32_t policy,
                              int32_t* d_tokens, int32_t* d_cu_seqlens, uint8_t* d_loss_mask,
                              int32_t* n_rows_out, int32_t* n_segments_out, int32_t* n_traj_consumed_out,
                              uint8_t* h_seg_skip_out, int32_t* h_traj_row_out, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_pack: NULL context");
  if (!turn_offsets || !traj_offsets || !n_rows_out || !n_segments_out || !n_traj_consumed_out)
    return as_fail(ctx, AS_ERR_NULL, "as_pack: NULL offsets or counters");
  if (n_traj > 0 && traj_offsets[n_traj] > 0 && (!turn_roles || (turn_offsets[traj_offsets[n_traj]] > 0 && !turn_tokens)))
    return as_fail(ctx, AS_ERR_NULL, "as_pack: NULL turn arrays");
  if (!d_cu_seqlens || (max_rows > 0 && row_len > 0 && (!d_tokens || !d_loss_mask)))
    return as_fail(ctx, AS_ERR_NULL, "as_pack: NULL output");
  std::vector<Piece> pieces; std::vector<int32_t> cu; std::vector<uint8_t> skip;
  int32_t rows = 0, consumed = 0;
  std::string err;
  int rc = pack_plan(ctx->cfg.vocab, turn_tokens, turn_offsets, turn_roles, traj_offsets, n_traj, row_len, max_rows,
                     truncate, policy, pieces, cu, skip, &rows, &consumed, h_traj_row_out, &err);
  if (rc) return as_fail(ctx, rc, "%s", err.c_str());
  hipStream_t st = (hipStream_t)stream;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  const int32_t n_tok = n_traj > 0 ? turn_offsets[traj_offsets[n_traj]] : 0;
  const size_t np = pieces.size();
  // staging layout: tokens | piece_dst | piece_src | cu | piece_mask
  size_t o_tok = 0, o_dst = o_tok + (size_t)n_tok * 4, o_src = o_dst + np * 4, o_cu = o_src + np * 4,
         o_msk = o_cu + cu.size() * 4, total = o_msk + np;
  total = (total + 255) & ~(size_t)255;
  rc = ensure_stage(ctx, total);
  if (rc) return rc;
  char* h = (char*)ctx->h_stage; char* d = (char*)ctx->d_stage;
  if (n_tok) memcpy(h + o_tok, turn_tokens, (size_t)n_tok * 4);
  for (size_t i = 0; i < np; i++) {
    ((int32_t*)(h + o_dst))[i] = pieces[i].dst;
    ((int32_t*)(h + o_src))[i] = pieces[i].src;
    ((uint8_t*)(h + o_msk))[i] = pieces[i].mask;
  }
  memcpy(h + o_cu, cu.data(), cu.size() * 4);
  AS_HIP(ctx, hipMemcpyAsync(d, h, total, hipMemcpyHostToDevice, st));
  AS_HIP(ctx, hipMemcpyAsync(d_cu_seqlens, d + o_cu, cu.size() * 4, hipMemcpyDeviceToDevice, st));
  if (np) {
    rc = launch_pack(ctx, (const int32_t*)(d + o_tok), (const int32_t*)(d + o_dst), (const int32_t*)(d + o_src),
                     (const uint8_t*)(d + o_msk), (int)np, rows * row_len, pad_id, d_tokens, d_loss_mask, st);
    if (rc) return rc;
  }
  AS_HIP(ctx, hipStreamSynchronize(st));       // the staging buffer is free again
  *n_rows_out = rows; *n_segments_out = (int32_t)cu.size() - 1; *n_traj_consumed_out = consumed;
  if (h_seg_skip_out && !skip.empty()) memcpy(h_seg_skip_out, skip.data(), skip.size());
  return AS_OK;
}

extern "C" int as_pack(as_ctx* ctx, const int32_t* turn_tokens, const int32_t* turn_offsets,
                       const uint8_t* turn_roles, const int32_t* traj_offsets, int32_t n_traj,
                       int32_t row_len, int32_t max_rows, int32_t pad_id, int32_t truncate,
                       int32_t* d_tokens, int32_t* d_cu_seqlens, uint8_t* d_loss_mask,
                       int32_t* n_rows_out, int32_t* n_segments_out, int32_t* n_traj_consumed_out,
                       uint8_t* h_seg_skip_out, void* stream) {
  return as_pack_policy(ctx, turn_tokens, turn_offsets, turn_roles, traj_offsets, n_traj, row_len, max_rows, pad_id, truncate,
                        AS_PACK_NEXT_FIT, d_tokens, d_cu_seqlens, d_loss_mask, n_rows_out, n_segments_out, n_traj_consumed_out,
                        h_seg_skip_out, nullptr, stream);
}

// --------------------------------------------------------- workspace plan
struct Bump {
  char* base; size_t off;
  void* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

struct LoraSlot {       // prepared copies of one adapter (type T)
  bool on = false;
  int din = 0, dout = 0;
  void *A = nullptr;    // [rp, din]   rows beyond rank are zero   (lives inside a concatenated group)
  void *At = nullptr;   // [din, group_cols] column block of the group transpose
  void *Bs = nullptr;   // [dout, rp]  = scale * B, zero padded
  void *Bst = nullptr;  // [rp, dout]
  int slot = 0;         // position inside its group (qkv / o / gate-up / down)
};

struct Acts {           // activations of one layer kept for its backward
  float *rstd1, *rstd2, *lse;
  void *a, *qkv, *o, *h_mid, *b, *gu, *m;
  void *u_qkv, *u_o, *u_gu, *u_d;
  // mixture-of-experts layers: gu / m hold the 2N (token, slot) rows grouped by expert
  float *rl, *wsel;                      // router logits [N, E], routing weights [N, 2]
  int32_t *sel, *eoff, *pos, *perm;      // chosen experts [N, 2], expert row offsets [E+1], pair -> row, row -> pair
  void *y_perm, *u_r;                    // expert outputs [2N, d], router adapter activations [N, rp]
};

struct Plan {
  int N, Np, d, D, Dkv, QKV, F, V, L, rp, es, Mc;
  bool head_fused;                       // vocabulary head without stored logits (statistics and gradient rows come out of the GEMM epilogues)
  float* gemm_tail;                      // scratch of the projection GEMMs' split last round (kGemmTailFloats floats, bf16 tier)
  float *part, *zlab, *lse_rows;         // its per-block softmax statistics [Mc, V / 128, 2], label logits and log-sum-exps per target   // Np: token count rounded up to 64 (row length of token-major transposes)
  int cap;                               // token rows every activation buffer holds (rows * row_len of the plan)
  int n_qkv, n_gu;                       // adapters inside the q/k/v and gate/up groups
  int32_t *seg_start, *seg_end, *tgt_idx, *tgt_pos, *labels, *count, *iscratch;
  int32_t* step_tab; size_t step_tab_ints;   // per-step host table: segment table, sources, attention launch orders, kept-segment map, pairs
  int32_t *tok_c; uint8_t* mask_c;       // tokens and mask with the skipped segments squeezed out
  const int32_t *order_q = nullptr, *order_k = nullptr;   // attention launch orders of this step (longest workgroups first)
  float *rope_cos, *rope_sin, *loss_rows, *rstd_f, *logits, *delta, *partial, *gpart;
  float *row_w, *w_kept, *logp_ws;       // preference loss: factor of each target row, of each kept segment; log-probability sums when the caller keeps none
  std::vector<void*> h;                  // L+1 residual-stream snapshots
  std::vector<Acts> acts;
  void *hf, *P, *dhf, *headT, *Pt, *hfT;
  void *dh, *dh2, *dm, *dgu, *db, *d_o, *dqkv, *da;
  void *du_qkv, *du_o, *du_gu, *du_d;
  void *wT, *xT, *dyT, *uT, *duT, *attT;
  void* wdq;                             // one dequantised projection matrix (NF4 base)
  void *xbp, *dlogit, *du_r, *wrT;       // MoE scratch: permuted rows [2N, d], router logit gradient [N, E], [N, rp], router weight transpose [d, E]
  std::vector<LoraSlot> lora;            // L * AS_N_TARGETS
  std::vector<void*> A_qkv, At_qkv, A_gu, At_gu;   // per layer concatenated groups
  size_t partial_floats;
};

static int pick_splitk(int mode, int M, int N, int K) {
  int bm = 64, bn = 64;
  if (mode == AS_BF16) { if (N <= 128 && M > 128) { bm = 256; bn = 64; } else if (M <= 128) { bm = 64; bn = 256; } else { bm = 256; bn = 256; } }
  int64_t blocks = cdiv(M, bm) * cdiv(N, bn);
  int64_t s = cdiv(512, blocks);
  int64_t smax = std::max<int64_t>(1, K / 256);
  return (int)std::max<int64_t>(1, std::min(s, smax));
}

static void target_dims(const as_model_config& c, int t, int* din, int* dout) {
  int D = c.n_q_heads * c.head_dim, Dkv = c.n_kv_heads * c.head_dim;
  switch (t) {
    case AS_T_Q: *din = c.d_model; *dout = D; break;
    case AS_T_K: case AS_T_V: *din = c.d_model; *dout = Dkv; break;
    case AS_T_O: *din = D; *dout = c.d_model; break;
    case AS_T_GATE: case AS_T_UP: *din = c.d_model; *dout = c.ffn; break;
    case AS_T_ROUTER: *din = c.d_model; *dout = c.n_experts; break;
    default: *din = c.ffn; *dout = c.d_model; break;
  }
}

static void make_plan(const as_ctx* ctx, int64_t rows, int64_t row_len, Bump& w, Plan& P) {
  const as_model_config& c = ctx->cfg;
  const bool full = c.train_mode == AS_FULL;
  P.N = (int)(rows * row_len); P.cap = P.N; P.d = c.d_model; P.D = c.n_q_heads * c.head_dim; P.Dkv = c.n_kv_heads * c.head_dim;
  P.QKV = P.D + 2 * P.Dkv; P.F = c.ffn; P.V = c.vocab; P.L = c.n_layers;
  P.es = c.mode == AS_FP32 ? 4 : 2;
  P.rp = full ? 0 : (c.mode == AS_BF16 ? (int)cdiv(c.lora_rank, 64) * 64 : (int)cdiv(c.lora_rank, 16) * 16);   // whole 64-wide K steps for the MFMA tiles
  P.head_fused = c.mode == AS_BF16 && P.V % 256 == 0 && P.d % 64 == 0;
  P.Mc = P.head_fused ? (int)std::min<int64_t>(8192, cdiv(std::max(P.N, 1), 256) * 256) : (int)std::min<int64_t>(4096, cdiv(std::max(P.N, 1), 64) * 64);
  P.Np = (int)cdiv(P.N, 64) * 64;
  const size_t N = (size_t)P.N, es = (size_t)P.es;
  const bool moe = c.n_experts > 0;
  const size_t NF = moe ? 2 * N : N, E = (size_t)c.n_experts;      // rows of the FFN intermediates
  auto on = [&](int t) { return !full && ((c.lora_targets >> t) & 1u); };
  P.n_qkv = on(AS_T_Q) + on(AS_T_K) + on(AS_T_V);
  P.n_gu = on(AS_T_GATE) + on(AS_T_UP);
  const size_t rp = (size_t)P.rp;

  P.seg_start = (int32_t*)w.take(N * 4); P.seg_end = (int32_t*)w.take(N * 4);
  P.tgt_idx = (int32_t*)w.take(N * 4); P.tgt_pos = (int32_t*)w.take(N * 4); P.labels = (int32_t*)w.take(N * 4);
  P.count = (int32_t*)w.take(256);
  P.step_tab_ints = 6 * N + 64;                           // (S+1) + S + N/32 + N/256 + S + 2 P with S, P <= N
  P.step_tab = (int32_t*)w.take(P.step_tab_ints * 4);
  P.gemm_tail = (float*)w.take(c.mode == AS_BF16 ? kGemmTailFloats * 4 : 0);
  P.tok_c = (int32_t*)w.take(N * 4); P.mask_c = (uint8_t*)w.take(N);
  P.iscratch = (int32_t*)w.take(full ? 2 * N * 4 : 0);
  P.rope_cos = (float*)w.take((size_t)row_len * (c.head_dim / 2) * 4);
  P.rope_sin = (float*)w.take((size_t)row_len * (c.head_dim / 2) * 4);
  P.loss_rows = (float*)w.take(N * 4);
  P.row_w = (float*)w.take(N * 4); P.w_kept = (float*)w.take(N * 4); P.logp_ws = (float*)w.take(N * 4);
  P.rstd_f = (float*)w.take(N * 4);
  P.h.resize(P.L + 1);
  for (int l = 0; l <= P.L; l++) P.h[l] = w.take(N * P.d * es);
  // recompute 0: every layer keeps all its activations; 1: one shared set, the layer's forward is
  // re-run before its backward; 2: every layer keeps the GEMM and attention outputs, and only the
  // cheap ones (both norm outputs, the SwiGLU product) live in one shared set and are rebuilt.
  const int n_sets = c.recompute == 1 ? 1 : P.L;
  P.acts.resize(n_sets);
  void *sh_a = nullptr, *sh_b = nullptr, *sh_m = nullptr;
  if (c.recompute == 2) { sh_a = w.take(N * P.d * es); sh_b = w.take(N * P.d * es); sh_m = w.take(NF * P.F * es); }
  for (int s = 0; s < n_sets; s++) {
    Acts& a = P.acts[s];
    a.rstd1 = (float*)w.take(N * 4); a.rstd2 = (float*)w.take(N * 4);
    a.lse = (float*)w.take(N * c.n_q_heads * 4);
    a.qkv = w.take(N * P.QKV * es); a.o = w.take(N * P.D * es);
    a.h_mid = w.take(N * P.d * es);
    a.gu = w.take(NF * 2 * P.F * es);
    if (c.recompute == 2) { a.a = sh_a; a.b = sh_b; a.m = sh_m; }
    else { a.a = w.take(N * P.d * es); a.b = w.take(N * P.d * es); a.m = w.take(NF * P.F * es); }
    a.u_qkv = w.take(N * P.n_qkv * rp * es); a.u_o = w.take(on(AS_T_O) ? N * rp * es : 0);
    a.u_gu = w.take(N * P.n_gu * rp * es); a.u_d = w.take(on(AS_T_DOWN) ? N * rp * es : 0);
    a.rl = (float*)w.take(N * E * 4); a.wsel = (float*)w.take(moe ? N * 2 * 4 : 0);
    a.sel = (int32_t*)w.take(moe ? N * 2 * 4 : 0); a.eoff = (int32_t*)w.take(moe ? (E + 1) * 4 : 0);
    a.pos = (int32_t*)w.take(moe ? N * 2 * 4 : 0); a.perm = (int32_t*)w.take(moe ? N * 2 * 4 : 0);
    a.y_perm = w.take(moe ? 2 * N * P.d * es : 0); a.u_r = w.take(on(AS_T_ROUTER) ? N * rp * es : 0);
  }
  // 256 rows more than tokens: the head's products run over whole 256-row tiles of the (device-counted) target rows
  P.hf = w.take((N + 256) * P.d * es); P.dhf = w.take((N + 256) * P.d * es);
  P.logits = (float*)w.take(P.head_fused ? 0 : (size_t)P.Mc * P.V * 4);
  P.part = (float*)w.take(P.head_fused ? (size_t)P.Mc * (P.V / 128) * 8 : 0);
  P.zlab = (float*)w.take(P.head_fused ? N * 4 : 0); P.lse_rows = (float*)w.take(P.head_fused ? N * 4 : 0);
  P.P = w.take((size_t)P.Mc * P.V * es);
  P.headT = w.take((size_t)P.V * P.d * es);
  P.Pt = w.take(full ? (size_t)P.Mc * P.V * es : 0);
  P.hfT = w.take(full ? (size_t)P.Mc * P.d * es : 0);
  P.delta = (float*)w.take(N * c.n_q_heads * 4);
  P.dh = w.take(N * P.d * es); P.dh2 = w.take(N * P.d * es);
  P.dm = w.take(NF * P.F * es); P.dgu = w.take(NF * 2 * P.F * es); P.db = w.take(N * P.d * es);
  P.d_o = w.take(N * P.D * es); P.dqkv = w.take(N * P.QKV * es); P.da = w.take(N * P.d * es);
  P.du_qkv = w.take(N * P.n_qkv * rp * es); P.du_o = w.take(on(AS_T_O) ? N * rp * es : 0);
  P.du_gu = w.take(N * P.n_gu * rp * es); P.du_d = w.take(on(AS_T_DOWN) ? N * rp * es : 0);
  size_t wmax = std::max({(size_t)P.QKV * P.d, (size_t)P.d * P.D, (size_t)2 * P.F * P.d, (size_t)P.d * P.F});
  P.wT = w.take(wmax * (moe ? E : 1) * es);            // sparse models: the transposed matrices of all experts at once
  P.wdq = w.take(c.weight_format == AS_W_NF4 ? std::max((size_t)P.F * P.d, (size_t)P.D * P.d) * es : 0);
  P.xbp = w.take(moe ? 2 * N * P.d * es : 0); P.dlogit = w.take(N * E * es);
  P.du_r = w.take(on(AS_T_ROUTER) ? N * rp * es : 0); P.wrT = w.take((size_t)P.d * E * es);
  const bool need_T = full || (c.lora_targets & 0xff);
  size_t xmax = std::max({(size_t)P.d, (size_t)P.D, (size_t)P.F});
  size_t ymax = std::max({(size_t)P.QKV, moe ? E : (size_t)2 * P.F, (size_t)P.d});
  const size_t Np = (size_t)P.Np;
  P.xT = w.take(need_T ? xmax * Np * es : 0);
  P.dyT = w.take(need_T ? ymax * Np * es : 0);
  size_t umax = (size_t)std::max({P.n_qkv, P.n_gu, 1}) * rp;
  P.uT = w.take(umax * Np * es); P.duT = w.take(umax * Np * es);
  P.gpart = (float*)w.take(full ? (size_t)256 * P.d * 4 : 0);
  // token-major K, Q, dO (V in forward), then the per-query-head float partials of dK and dV
  P.attT = w.take(c.mode == AS_BF16 ? (size_t)(2 * P.D + P.Dkv) * Np * es + (size_t)2 * P.D * Np * 4 : 0);

  // prepared adapter copies
  P.lora.assign((size_t)P.L * AS_N_TARGETS, LoraSlot());
  P.A_qkv.assign(P.L, nullptr); P.At_qkv.assign(P.L, nullptr); P.A_gu.assign(P.L, nullptr); P.At_gu.assign(P.L, nullptr);
  size_t part = 0;
  for (int l = 0; l < P.L && !full; l++) {
    P.A_qkv[l] = w.take((size_t)P.n_qkv * rp * P.d * es); P.At_qkv[l] = w.take((size_t)P.d * P.n_qkv * rp * es);
    P.A_gu[l] = w.take((size_t)P.n_gu * rp * P.d * es); P.At_gu[l] = w.take((size_t)P.d * P.n_gu * rp * es);
    int sq = 0, sg = 0;
    for (int t = 0; t < AS_N_TARGETS; t++) {
      LoraSlot& s = P.lora[(size_t)l * AS_N_TARGETS + t];
      s.on = on(t);
      if (!s.on) continue;
      target_dims(c, t, &s.din, &s.dout);
      if (t <= AS_T_V) { s.slot = sq++; s.A = P.A_qkv[l] ? (char*)P.A_qkv[l] + (size_t)s.slot * rp * P.d * es : nullptr;
                         s.At = P.At_qkv[l] ? (char*)P.At_qkv[l] + (size_t)s.slot * rp * es : nullptr; }
      else if (t == AS_T_GATE || t == AS_T_UP) { s.slot = sg++; s.A = P.A_gu[l] ? (char*)P.A_gu[l] + (size_t)s.slot * rp * P.d * es : nullptr;
                         s.At = P.At_gu[l] ? (char*)P.At_gu[l] + (size_t)s.slot * rp * es : nullptr; }
      else { s.slot = 0; s.A = w.take(rp * s.din * es); s.At = w.take((size_t)s.din * rp * es); }
      s.Bs = w.take((size_t)s.dout * rp * es); s.Bst = w.take(rp * s.dout * es);
      if (l == 0) {
        int r = c.lora_rank;
        part = std::max(part, (size_t)pick_splitk(c.mode, s.dout, r, P.N) * s.dout * r);
        part = std::max(part, (size_t)pick_splitk(c.mode, r, s.din, P.N) * r * s.din);
        if (c.mode == AS_BF16 && r <= 64) {
          part = std::max(part, lora_grad_tn_partial_floats(P.N, s.dout, r));
          part = std::max(part, lora_grad_tn_partial_floats(P.N, s.din, r));
        }
      }
    }
  }
  P.partial_floats = part;
  P.partial = (float*)w.take(part * 4);
}

extern "C" int as_workspace_bytes(const as_ctx* ctx, int64_t max_rows, int64_t row_len, size_t* bytes) {
  if (!ctx || !bytes) return as_fail(nullptr, AS_ERR_NULL, "as_workspace_bytes: NULL argument");
  if (max_rows < 1 || row_len < 1 || max_rows * row_len > (int64_t)1 << 30)
    return as_fail(const_cast<as_ctx*>(ctx), AS_ERR_SHAPE, "as_workspace_bytes: rows*row_len must be in [1, 2^30]");
  Bump w{nullptr, 0}; Plan P;
  make_plan(ctx, max_rows, row_len, w, P);
  *bytes = (w.off + 255) & ~(size_t)255;
  return AS_OK;
}

// ----------------------------------------------------------- training step
namespace {
// What the step computes from the per-target losses -log p.
enum { LOSS_MEAN = 0,      // their mean over the targets (supervised fine-tuning), forward and backward
       LOSS_SEQ_LOGP = 1,  // per-segment sums pi_s = sum log p, forward only
       LOSS_DPO = 2 };     // the pair preference loss on those sums against reference sums, forward and backward
struct LossSpec {
  int kind = LOSS_MEAN;
  const int32_t* h_pairs = nullptr; int n_pairs = 0;
  const float* d_ref_logp = nullptr; float beta = 0.f;
  float* d_logp = nullptr; float* d_stats = nullptr;
  // filled by the step
  const int32_t *d_pairs = nullptr, *d_kept_of = nullptr, *d_cu = nullptr;   // pair table, caller's segment -> kept segment, kept segment table
  int n_seg = 0, n_kept = 0;
};

struct Step {
  as_ctx* ctx; const as_model_config& c; Plan& P; hipStream_t st; int mode; int gv; int av;
  const as_weights* W; const as_lora* lora; const as_grads* G; int max_seg;
  LossSpec LS;
  size_t es() const { return (size_t)P.es; }
  void* off(void* p, size_t elems) const { return (char*)p + elems * es(); }
  const void* off(const void* p, size_t elems) const { return (const char*)p + elems * es(); }

  // C = A1 B1^T (+ A2 B2^T) (+ R)
  int gemm(int M, int N, const void* A1, int64_t lda1, const void* B1, int64_t ldb1, int K1,
           const void* A2, int64_t lda2, const void* B2, int64_t ldb2, int K2,
           const void* R, int64_t ldr, void* C, int64_t ldc, int c_f32 = 0, float alpha = 1.f,
           int accumulate = 0, const int* m_dev = nullptr, int m_off = 0, bool allow_split = false) {
    GemmParams g; memset(&g, 0, sizeof g);
    g.seg[0] = {A1, B1, lda1, ldb1, K1}; g.nseg = 1;
    if (A2 && K2 > 0) { g.seg[1] = {A2, B2, lda2, ldb2, K2}; g.nseg = 2; }
    g.M = M; g.N = N; g.m_dev = m_dev; g.C = C; g.ldc = ldc; g.c_f32 = c_f32; g.alpha = alpha;
    g.rows_cap = rows_cap_once; rows_cap_once = 0;
    g.R = R; g.ldr = ldr; g.accumulate = accumulate; g.splitk = 1; g.partial = nullptr; g.tail_part = P.gemm_tail;
    if (allow_split) {
      int sk = pick_splitk(mode, M, N, K1);
      if (sk > 1 && (size_t)sk * M * N <= P.partial_floats) { g.splitk = sk; g.partial = P.partial; }
    }
    return launch_gemm_off(ctx, mode, gv, g, m_off, st);
  }

  // set right before a gemm() whose row operands are all token-row workspace buffers (they hold P.cap rows)
  int rows_cap_once = 0;
  LoraSlot& slot(int l, int t) { return P.lora[(size_t)l * AS_N_TARGETS + t]; }

  // The dense [rows, cols] matrix of a frozen projection: the caller's pointer, or, for an NF4 base, the
  // workspace slot it is dequantised into right before its use (one slot: the stream orders the reuse).
  int wq_rc = AS_OK;
  const void* dense(const void* w, const float* absmax, int rows, int cols) {
    if (c.weight_format != AS_W_NF4) return w;
    int rc = launch_nf4_dequantize(ctx, mode, (const uint8_t*)w, absmax, (int64_t)rows * cols, P.wdq, st);
    if (rc && !wq_rc) wq_rc = rc;
    return P.wdq;
  }

  // Projections that read the same input and write side by side (q | k | v, gate | up) go out as one launch when their
  // matrices can be used where they are (dense format) and either all or none of them carry an adapter.
  bool side_by_side_ok(int l, const int* tgt, int nt) {
    if (c.weight_format == AS_W_NF4) return false;
    int on = 0;
    for (int i = 0; i < nt; i++) on += slot(l, tgt[i]).on ? 1 : 0;
    return on == 0 || on == nt;
  }
  int gemm_side_by_side(int l, const int* tgt, int nt, const void* x, int K, const void* const* w, const int* nout,
                        const void* u, int ldu, void* C, int ldc) {
    GemmParams g; memset(&g, 0, sizeof g);
    const bool on = slot(l, tgt[0]).on;
    g.seg[0] = {x, w[0], K, K, K}; g.nseg = 1;
    if (on) { g.seg[1] = {u, slot(l, tgt[0]).Bs, ldu, P.rp, P.rp}; g.nseg = 2; }
    g.ncg = nt;
    int end = 0;
    for (int i = 0; i < nt; i++) {
      end += nout[i]; g.cg_end[i] = end; g.cg_B1[i] = w[i];
      g.cg_B2[i] = on ? slot(l, tgt[i]).Bs : nullptr; g.cg_a2[i] = on ? slot(l, tgt[i]).slot * P.rp : 0;
    }
    g.M = P.N; g.N = end; g.C = C; g.ldc = ldc; g.alpha = 1.f; g.splitk = 1; g.rows_cap = P.cap; g.tail_part = P.gemm_tail;
    return launch_gemm_off(ctx, mode, gv, g, 0, st);
  }

  int prep_lora(int l) {
    const as_layer_lora& Lr = lora->layers[l];
    const float s = c.lora_alpha / (float)c.lora_rank;
    const int r = c.lora_rank, rp = P.rp;
    for (int t = 0; t < AS_N_TARGETS; t++) {
      LoraSlot& sl = slot(l, t);
      if (!sl.on) continue;
      int64_t ld_at = (t <= AS_T_V) ? (int64_t)P.n_qkv * rp : (t == AS_T_GATE || t == AS_T_UP) ? (int64_t)P.n_gu * rp : rp;
      // A [r, din] -> A copy [rp, din] and its transpose block [din, rp] inside a [din, group] matrix
      int rc = launch_lora_prep_ex(Lr.a[t], r, sl.din, rp, sl.din, 1.f, sl.A, sl.din, sl.At, ld_at);
      if (rc) return rc;
      // B [dout, r] -> s*B [dout, rp] and transpose [rp, dout]
      rc = launch_lora_prep_ex(Lr.b[t], sl.dout, r, sl.dout, rp, s, sl.Bs, rp, sl.Bst, sl.dout);
      if (rc) return rc;
    }
    return AS_OK;
  }
  int launch_lora_prep_ex(const float* in, int rows, int cols, int rows_pad, int cols_pad, float scale,
                          void* out, int64_t ldo, void* out_t, int64_t ldo_t);

  int forward_layer(int l, Acts& a) {
    const as_layer_weights& w = W->layers[l];
    const int N = P.N, d = P.d, D = P.D, Dkv = P.Dkv, QKV = P.QKV, F = P.F, rp = P.rp;
    const void* h_in = P.h[l]; void* h_out = P.h[l + 1];
    int rc;
    if ((rc = launch_rmsnorm_fwd(ctx, mode, N, d, h_in, nullptr, nullptr, w.g1, c.rms_eps, a.a, a.rstd1, st))) return rc;
    const int ldu = P.n_qkv * rp;
    if (P.n_qkv && (rc = gemm(N, ldu, a.a, d, P.A_qkv[l], d, d, nullptr, 0, nullptr, 0, 0, nullptr, 0, a.u_qkv, ldu))) return rc;
    const void* wq[3] = {w.wq, w.wk, w.wv}; const float* aq[3] = {w.aq, w.ak, w.av};
    const int nout[3] = {D, Dkv, Dkv}; const int coff[3] = {0, D, D + Dkv};
    const int tq[3] = {AS_T_Q, AS_T_K, AS_T_V};
    if (side_by_side_ok(l, tq, 3)) {
      if ((rc = gemm_side_by_side(l, tq, 3, a.a, d, wq, nout, a.u_qkv, ldu, a.qkv, QKV))) return rc;
    } else
    for (int i = 0; i < 3; i++) {
      LoraSlot& s = slot(l, i);
      rows_cap_once = P.cap;
      rc = gemm(N, nout[i], a.a, d, dense(wq[i], aq[i], nout[i], d), d, d, s.on ? off(a.u_qkv, (size_t)s.slot * rp) : nullptr, ldu, s.Bs, rp, s.on ? rp : 0,
                nullptr, 0, off(a.qkv, coff[i]), QKV);
      if (rc) return rc;
    }
    if ((rc = launch_rope(ctx, mode, N, c.n_q_heads + c.n_kv_heads, c.head_dim, a.qkv, QKV, P.seg_start, P.rope_cos, P.rope_sin, 0, st))) return rc;
    AttnParams ap; memset(&ap, 0, sizeof ap);
    ap.n = N; ap.Hq = c.n_q_heads; ap.Hkv = c.n_kv_heads; ap.dh = c.head_dim; ap.seg_start = P.seg_start; ap.seg_end = P.seg_end;
    ap.q = a.qkv; ap.k = off(a.qkv, D); ap.v = off(a.qkv, D + Dkv); ap.ldq = QKV; ap.ldkv = QKV; ap.o = a.o; ap.lse = a.lse; ap.max_seg = max_seg; ap.t_scratch = P.attT;
    ap.order_q = P.order_q; ap.order_k = P.order_k;
    if ((rc = launch_attention_fwd(ctx, mode, av, ap, st))) return rc;
    { LoraSlot& s = slot(l, AS_T_O);
      if (s.on && (rc = gemm(N, rp, a.o, D, s.A, D, D, nullptr, 0, nullptr, 0, 0, nullptr, 0, a.u_o, rp))) return rc;
      rows_cap_once = P.cap;
      if ((rc = gemm(N, d, a.o, D, dense(w.wo, w.ao, d, D), D, D, s.on ? a.u_o : nullptr, rp, s.Bs, rp, s.on ? rp : 0, h_in, d, a.h_mid, d))) return rc; }
    if ((rc = launch_rmsnorm_fwd(ctx, mode, N, d, a.h_mid, nullptr, nullptr, w.g2, c.rms_eps, a.b, a.rstd2, st))) return rc;
    if (c.n_experts) return forward_moe(l, a);
    const int ldg = P.n_gu * rp;
    if (P.n_gu && (rc = gemm(N, ldg, a.b, d, P.A_gu[l], d, d, nullptr, 0, nullptr, 0, 0, nullptr, 0, a.u_gu, ldg))) return rc;
    const void* wg[2] = {w.wgate, w.wup}; const float* ag[2] = {w.agate, w.aup};
    const int tg[2] = {AS_T_GATE, AS_T_UP}; const int ng[2] = {F, F};
    if (side_by_side_ok(l, tg, 2)) {
      if ((rc = gemm_side_by_side(l, tg, 2, a.b, d, wg, ng, a.u_gu, ldg, a.gu, 2 * F))) return rc;
    } else
    for (int i = 0; i < 2; i++) {
      LoraSlot& s = slot(l, AS_T_GATE + i);
      rows_cap_once = P.cap;
      rc = gemm(N, F, a.b, d, dense(wg[i], ag[i], F, d), d, d, s.on ? off(a.u_gu, (size_t)s.slot * rp) : nullptr, ldg, s.Bs, rp, s.on ? rp : 0,
                nullptr, 0, off(a.gu, (size_t)i * F), 2 * F);
      if (rc) return rc;
    }
    if ((rc = launch_swiglu_fwd(ctx, mode, N, F, a.gu, a.m, st))) return rc;
    { LoraSlot& s = slot(l, AS_T_DOWN);
      if (s.on && (rc = gemm(N, rp, a.m, F, s.A, F, F, nullptr, 0, nullptr, 0, 0, nullptr, 0, a.u_d, rp))) return rc;
      rows_cap_once = P.cap;
      if ((rc = gemm(N, d, a.m, F, dense(w.wdown, w.adown, d, F), F, F, s.on ? a.u_d : nullptr, rp, s.Bs, rp, s.on ? rp : 0, a.h_mid, d, h_out, d))) return rc; }
    return AS_OK;
  }

  // every expert's product over its own rows: rows eoff[e] .. eoff[e+1] of A and C times the e-th of the stacked
  // matrices at B (b_stride elements apart); one launch where the kernel allows, else one per expert
  int gemm_experts(const int32_t* eoff, int N, const void* A, int64_t lda, const void* B, int64_t b_stride, int64_t ldb, int K, void* C, int64_t ldc) {
    GemmParams g; memset(&g, 0, sizeof g);
    g.seg[0] = {A, B, lda, ldb, K}; g.nseg = 1;
    g.M = P.N; g.N = N; g.C = C; g.ldc = ldc; g.alpha = 1.f; g.splitk = 1;
    g.grp_off = eoff; g.grp_n = c.n_experts; g.grp_b_stride = b_stride; g.grp_rows = 2.0 * P.N;
    g.rows_cap = 2 * P.N;                                  // A and C are (token, slot) buffers: 2 N rows
    return launch_gemm_off(ctx, mode, gv, g, 0, st);
  }

  // Sparse FFN (top-2 of E experts): router, grouping of the (token, slot) pairs by expert, one
  // SwiGLU FFN per expert over its rows, weighted sum back in token order on top of the residual.
  int forward_moe(int l, Acts& a) {
    const as_layer_weights& w = W->layers[l];
    const int N = P.N, d = P.d, F = P.F, rp = P.rp, E = c.n_experts;
    int rc;
    LoraSlot& s = slot(l, AS_T_ROUTER);
    if (s.on && (rc = gemm(N, rp, a.b, d, s.A, d, d, nullptr, 0, nullptr, 0, 0, nullptr, 0, a.u_r, rp))) return rc;
    if ((rc = gemm(N, E, a.b, d, w.wrouter, d, d, s.on ? a.u_r : nullptr, rp, s.Bs, rp, s.on ? rp : 0, nullptr, 0, a.rl, E, 1))) return rc;
    if ((rc = launch_moe_route(ctx, a.rl, N, E, a.sel, a.wsel, st))) return rc;
    if ((rc = launch_moe_permute(ctx, a.sel, N, E, a.eoff, a.pos, a.perm, st))) return rc;
    if ((rc = launch_moe_gather(ctx, mode, a.b, a.perm, nullptr, 2 * N, d, P.xbp, st))) return rc;
    const void* wg[2] = {w.wgate, w.wup};
    for (int i = 0; i < 2; i++)
      if ((rc = gemm_experts(a.eoff, F, P.xbp, d, wg[i], (int64_t)F * d, d, d, off(a.gu, (size_t)i * F), 2 * F))) return rc;
    if ((rc = launch_swiglu_fwd(ctx, mode, 2 * N, F, a.gu, a.m, st))) return rc;
    if ((rc = gemm_experts(a.eoff, d, a.m, F, w.wdown, (int64_t)d * F, F, F, a.y_perm, d))) return rc;
    return launch_moe_combine(ctx, mode, a.h_mid, a.y_perm, a.pos, a.wsel, N, d, P.h[l + 1], st);
  }

  // P.dh (gradient of the layer output) -> P.db (gradient of the second norm's output)
  int backward_moe(int l, Acts& a) {
    const as_layer_weights& w = W->layers[l];
    const int N = P.N, d = P.d, F = P.F, rp = P.rp, E = c.n_experts;
    int rc;
    if ((rc = launch_moe_dlogit(ctx, mode, P.dh, a.y_perm, a.pos, a.sel, a.wsel, N, d, E, P.dlogit, st))) return rc;
    if ((rc = launch_moe_gather(ctx, mode, P.dh, a.perm, a.wsel, 2 * N, d, P.xbp, st))) return rc;        // w * dy, grouped
    // the transposed matrices of all experts side by side (the workspace slot holds E of them), then one product each
    for (int e = 0; e < E; e++)
      if ((rc = transpose(d, F, off(w.wdown, (size_t)e * d * F), F, off(P.wT, (size_t)e * F * d), d))) return rc;      // [F, d]
    if ((rc = gemm_experts(a.eoff, F, P.xbp, d, P.wT, (int64_t)F * d, d, d, P.dm, F))) return rc;
    if ((rc = launch_swiglu_bwd(ctx, mode, 2 * N, F, P.dm, a.gu, P.dgu, nullptr, st))) return rc;
    for (int e = 0; e < E; e++) {
      void* wt = off(P.wT, (size_t)e * 2 * F * d);
      if ((rc = transpose(F, d, off(w.wgate, (size_t)e * F * d), d, wt, 2 * F))) return rc;               // [d, 2F]
      if ((rc = transpose(F, d, off(w.wup, (size_t)e * F * d), d, off(wt, (size_t)F), 2 * F))) return rc;
    }
    if ((rc = gemm_experts(a.eoff, d, P.dgu, 2 * F, P.wT, (int64_t)2 * F * d, 2 * F, 2 * F, P.xbp, d))) return rc;     // grouped gradient of the expert inputs
    if ((rc = launch_moe_combine(ctx, mode, nullptr, P.xbp, a.pos, nullptr, N, d, P.da, st))) return rc;  // back to token order
    // router: db = (expert part) + dlogit Wr + du_r A
    LoraSlot& s = slot(l, AS_T_ROUTER);
    if ((rc = transpose(E, d, w.wrouter, d, P.wrT, E))) return rc;                                        // [d, E]
    if (s.on && (rc = gemm(N, rp, P.dlogit, E, s.Bst, E, E, nullptr, 0, nullptr, 0, 0, nullptr, 0, P.du_r, rp))) return rc;
    if ((rc = gemm(N, d, P.dlogit, E, P.wrT, E, E, s.on ? P.du_r : nullptr, rp, s.At, rp, s.on ? rp : 0, P.da, d, P.db, d))) return rc;
    if (s.on) {
      if (!tn_path()) {
        if ((rc = transpose_tok(E, P.dlogit, E, P.dyT))) return rc;
        if ((rc = transpose_tok(d, a.b, d, P.xT))) return rc;
      }
      if ((rc = transpose_tok(rp, a.u_r, rp, P.uT))) return rc;
      if ((rc = transpose_tok(rp, P.du_r, rp, P.duT))) return rc;
      if ((rc = lora_grads(l, AS_T_ROUTER, P.dlogit, E, a.b, d, P.dyT, P.xT))) return rc;
    }
    return AS_OK;
  }

  // the activations that are cheaper to rebuild than to keep: both norm outputs here; the SwiGLU product
  // is rewritten by the layer's SwiGLU backward kernel, which reads gate | up anyway
  int rebuild_cheap(int l, Acts& a) {
    const as_layer_weights& w = W->layers[l];
    int rc;
    if ((rc = launch_rmsnorm_fwd(ctx, mode, P.N, P.d, P.h[l], nullptr, nullptr, w.g1, c.rms_eps, a.a, a.rstd1, st))) return rc;
    return launch_rmsnorm_fwd(ctx, mode, P.N, P.d, a.h_mid, nullptr, nullptr, w.g2, c.rms_eps, a.b, a.rstd2, st);
  }

  // nothing to compute: loss, count and every gradient are exactly zero
  int zero_outputs(float* d_loss, float* d_loss_sum, int32_t* d_count) {
    int rc;
    if (d_loss && (rc = launch_fill_zero(ctx, d_loss, 4, st))) return rc;
    if (d_loss_sum && (rc = launch_fill_zero(ctx, d_loss_sum, 4, st))) return rc;
    if (d_count && (rc = launch_fill_zero(ctx, d_count, 4, st))) return rc;
    if (!G) return AS_OK;
    const size_t d = P.d, D = P.D, Dkv = P.Dkv, F = P.F;
    for (int l = 0; l < P.L; l++) {
      if (c.train_mode == AS_LORA) {
        for (int t = 0; t < AS_N_TARGETS; t++) {
          if (!((c.lora_targets >> t) & 1u)) continue;
          int din, dout; target_dims(c, t, &din, &dout);
          if ((rc = launch_fill_zero(ctx, G->lora_layers[l].a[t], (size_t)c.lora_rank * din * 4, st))) return rc;
          if ((rc = launch_fill_zero(ctx, G->lora_layers[l].b[t], (size_t)dout * c.lora_rank * 4, st))) return rc;
        }
      } else {
        const as_layer_weight_grads& g = G->w_layers[l];
        float* ptr[9] = {g.g1, g.wq, g.wk, g.wv, g.wo, g.g2, g.wgate, g.wup, g.wdown};
        size_t cnt[9] = {d, D * d, Dkv * d, Dkv * d, d * D, d, F * d, F * d, d * F};
        for (int i = 0; i < 9; i++) if ((rc = launch_fill_zero(ctx, ptr[i], cnt[i] * 4, st))) return rc;
      }
    }
    if (c.train_mode == AS_FULL) {
      if ((rc = launch_fill_zero(ctx, G->embed, (size_t)P.V * d * 4, st)) || (rc = launch_fill_zero(ctx, G->head, (size_t)P.V * d * 4, st)) ||
          (rc = launch_fill_zero(ctx, G->g_final, d * 4, st))) return rc;
    }
    return AS_OK;
  }

  int transpose(int rows, int cols, const void* in, int64_t ldi, void* out, int64_t ldo) {
    return launch_transpose(ctx, mode, rows, rows, cols, in, ldi, out, ldo, nullptr, 0, st);
  }
  // [N tokens, cols] -> [cols, Np]: token-major copy whose rows are padded with zeros to Np
  int transpose_tok(int cols, const void* in, int64_t ldi, void* out) {
    return launch_transpose(ctx, mode, P.N, P.Np, cols, in, ldi, out, P.Np, nullptr, 0, st);
  }

  // adapter gradients of one projection: dB = s dy^T u, dA = du^T x.  bf16 with rank <= 64: one
  // streaming pass over dy and over x (row-major, as they are) against the token-major copies of u
  // and du.  Otherwise: GEMMs on the token-major copies dyT [dout, Np], xT [din, Np].
  bool tn_path() const { return mode == AS_BF16 && c.lora_rank <= 64; }
  int lora_grads(int l, int t, const void* dy, int64_t lddy, const void* x, int64_t ldx, const void* dyT_rows, const void* xT) {
    LoraSlot& s = slot(l, t);
    if (!s.on) return AS_OK;
    const int Np = P.Np, r = c.lora_rank, rp = P.rp;
    const float sc = c.lora_alpha / (float)c.lora_rank;
    const as_layer_lora_grads& g = G->lora_layers[l];
    const void* uT = off(P.uT, (size_t)s.slot * rp * Np);
    const void* duT = off(P.duT, (size_t)s.slot * rp * Np);
    if (tn_path()) {
      int rc = launch_lora_grad_tn(ctx, dy, lddy, uT, Np, P.N, s.dout, r, sc, g.b[t], r, 1, P.partial, P.partial_floats, st);
      if (rc) return rc;
      return launch_lora_grad_tn(ctx, x, ldx, duT, Np, P.N, s.din, r, 1.f, g.a[t], 1, s.din, P.partial, P.partial_floats, st);
    }
    int rc = gemm(s.dout, r, dyT_rows, Np, uT, Np, Np, nullptr, 0, nullptr, 0, 0, nullptr, 0, g.b[t], r, 1, sc, 0, nullptr, 0, true);
    if (rc) return rc;
    return gemm(r, s.din, duT, Np, xT, Np, Np, nullptr, 0, nullptr, 0, 0, nullptr, 0, g.a[t], s.din, 1, 1.f, 0, nullptr, 0, true);
  }
  int weight_grad(float* dW, int dout, int din, const void* dyT_rows, const void* xT) {
    const int N = P.Np;
    return gemm(dout, din, dyT_rows, N, xT, N, N, nullptr, 0, nullptr, 0, 0, nullptr, 0, dW, din, 1);
  }

  // dh_out in P.dh -> dh_in in P.dh (P.dh2 holds the mid-layer gradient)
  int backward_layer(int l, Acts& a) {
    const as_layer_weights& w = W->layers[l];
    const bool full = c.train_mode == AS_FULL;
    const int N = P.N, d = P.d, D = P.D, Dkv = P.Dkv, QKV = P.QKV, F = P.F, rp = P.rp;
    int rc;
    if (c.n_experts) { if ((rc = backward_moe(l, a))) return rc; }
    else {
    // ---- down projection
    { LoraSlot& s = slot(l, AS_T_DOWN);
      if ((rc = transpose(d, F, dense(w.wdown, w.adown, d, F), F, P.wT, d))) return rc;                       // [F, d]
      if (s.on && (rc = gemm(N, rp, P.dh, d, s.Bst, d, d, nullptr, 0, nullptr, 0, 0, nullptr, 0, P.du_d, rp))) return rc;
      rows_cap_once = P.cap;
      if ((rc = gemm(N, F, P.dh, d, P.wT, d, d, s.on ? P.du_d : nullptr, rp, s.At, rp, s.on ? rp : 0, nullptr, 0, P.dm, F))) return rc;
      // ---- SwiGLU (in recompute mode 2 it also rewrites the forward product, which the gradients below need)
      const bool rewrite_m = c.recompute == 2 && l != c.n_layers - 1 && (full || s.on);
      if ((rc = launch_swiglu_bwd(ctx, mode, N, F, P.dm, a.gu, P.dgu, rewrite_m ? a.m : nullptr, st))) return rc;
      if (full || (s.on && !tn_path())) {
        if ((rc = transpose_tok(d, P.dh, d, P.dyT))) return rc;
        if ((rc = transpose_tok(F, a.m, F, P.xT))) return rc;
      }
      if (s.on) {
        if ((rc = transpose_tok(rp, a.u_d, rp, P.uT))) return rc;
        if ((rc = transpose_tok(rp, P.du_d, rp, P.duT))) return rc;
        if ((rc = lora_grads(l, AS_T_DOWN, P.dh, d, a.m, F, P.dyT, P.xT))) return rc;
      }
      if (full && (rc = weight_grad(G->w_layers[l].wdown, d, F, P.dyT, P.xT))) return rc; }
    // ---- gate / up projections
    { const int ldg = P.n_gu * rp;
      const void* wg[2] = {w.wgate, w.wup}; const float* ag[2] = {w.agate, w.aup};
      for (int i = 0; i < 2; i++) {
        LoraSlot& s = slot(l, AS_T_GATE + i);
        if ((rc = transpose(F, d, dense(wg[i], ag[i], F, d), d, off(P.wT, (size_t)i * F), 2 * F))) return rc;        // [d, 2F]
        if (s.on && (rc = gemm(N, rp, off(P.dgu, (size_t)i * F), 2 * F, s.Bst, F, F, nullptr, 0, nullptr, 0, 0, nullptr, 0,
                               off(P.du_gu, (size_t)s.slot * rp), ldg))) return rc;
      }
      rows_cap_once = P.cap;
      if ((rc = gemm(N, d, P.dgu, 2 * F, P.wT, 2 * F, 2 * F, P.n_gu ? P.du_gu : nullptr, ldg, P.At_gu[l], ldg, ldg,
                     nullptr, 0, P.db, d))) return rc;
      if (full || (P.n_gu && !tn_path())) {
        if ((rc = transpose_tok(2 * F, P.dgu, 2 * F, P.dyT))) return rc;
        if ((rc = transpose_tok(d, a.b, d, P.xT))) return rc;
      }
      if (P.n_gu) {
        if ((rc = transpose_tok(ldg, a.u_gu, ldg, P.uT))) return rc;
        if ((rc = transpose_tok(ldg, P.du_gu, ldg, P.duT))) return rc;
        for (int i = 0; i < 2; i++)
          if ((rc = lora_grads(l, AS_T_GATE + i, off(P.dgu, (size_t)i * F), 2 * F, a.b, d, off(P.dyT, (size_t)i * F * P.Np), P.xT))) return rc;
      }
      if (full) {
        if ((rc = weight_grad(G->w_layers[l].wgate, F, d, P.dyT, P.xT))) return rc;
        if ((rc = weight_grad(G->w_layers[l].wup, F, d, off(P.dyT, (size_t)F * P.Np), P.xT))) return rc;
      } }
    }
    // ---- second norm
    if (full && (rc = launch_rmsnorm_dgain(ctx, mode, N, d, P.db, nullptr, a.h_mid, a.rstd2, P.gpart, 256, G->w_layers[l].g2, st))) return rc;
    if ((rc = launch_rmsnorm_bwd(ctx, mode, N, d, P.db, nullptr, a.h_mid, w.g2, a.rstd2, P.dh, P.dh2, st))) return rc;
    // ---- output projection
    { LoraSlot& s = slot(l, AS_T_O);
      if ((rc = transpose(d, D, dense(w.wo, w.ao, d, D), D, P.wT, d))) return rc;                          // [D, d]
      if (s.on && (rc = gemm(N, rp, P.dh2, d, s.Bst, d, d, nullptr, 0, nullptr, 0, 0, nullptr, 0, P.du_o, rp))) return rc;
      rows_cap_once = P.cap;
      if ((rc = gemm(N, D, P.dh2, d, P.wT, d, d, s.on ? P.du_o : nullptr, rp, s.At, rp, s.on ? rp : 0, nullptr, 0, P.d_o, D))) return rc;
      if (full || (s.on && !tn_path())) {
        if ((rc = transpose_tok(d, P.dh2, d, P.dyT))) return rc;
        if ((rc = transpose_tok(D, a.o, D, P.xT))) return rc;
      }
      if (s.on) {
        if ((rc = transpose_tok(rp, a.u_o, rp, P.uT))) return rc;
        if ((rc = transpose_tok(rp, P.du_o, rp, P.duT))) return rc;
        if ((rc = lora_grads(l, AS_T_O, P.dh2, d, a.o, D, P.dyT, P.xT))) return rc;
      }
      if (full && (rc = weight_grad(G->w_layers[l].wo, d, D, P.dyT, P.xT))) return rc; }
    // ---- attention
    { AttnParams ap; memset(&ap, 0, sizeof ap);
      ap.n = N; ap.Hq = c.n_q_heads; ap.Hkv = c.n_kv_heads; ap.dh = c.head_dim; ap.seg_start = P.seg_start; ap.seg_end = P.seg_end;
      ap.q = a.qkv; ap.k = off(a.qkv, D); ap.v = off(a.qkv, D + Dkv); ap.ldq = QKV; ap.ldkv = QKV; ap.o = a.o; ap.lse = a.lse;
      ap.d_o = P.d_o; ap.dq = P.dqkv; ap.dk = off(P.dqkv, D); ap.dv = off(P.dqkv, D + Dkv); ap.delta = P.delta; ap.max_seg = max_seg; ap.t_scratch = P.attT;
      ap.order_q = P.order_q; ap.order_k = P.order_k;
      // the MFMA kernels rotate dq and dk back themselves (one rounding, no extra pass); else a pass of its own does
      const bool fused_rope = attention_bwd_is_mfma(mode, av, ap);
      if (fused_rope) { ap.rope_cos = P.rope_cos; ap.rope_sin = P.rope_sin; }
      if ((rc = launch_attention_bwd(ctx, mode, av, ap, st))) return rc;
      if (!fused_rope && (rc = launch_rope(ctx, mode, N, c.n_q_heads + c.n_kv_heads, c.head_dim, P.dqkv, QKV, P.seg_start, P.rope_cos, P.rope_sin, 1, st))) return rc; }
    // ---- q / k / v projections
    { const int ldu = P.n_qkv * rp;
      const void* wq[3] = {w.wq, w.wk, w.wv}; const float* aq[3] = {w.aq, w.ak, w.av};
      const int nout[3] = {D, Dkv, Dkv}; const int coff[3] = {0, D, D + Dkv};
      // with frozen embeddings nothing below the first layer's first norm takes a gradient
      const bool need_da = full || l > 0;
      for (int i = 0; i < 3; i++) {
        LoraSlot& s = slot(l, i);
        if (need_da && (rc = transpose(nout[i], d, dense(wq[i], aq[i], nout[i], d), d, off(P.wT, coff[i]), QKV))) return rc;          // [d, QKV]
        if (s.on && (rc = gemm(N, rp, off(P.dqkv, coff[i]), QKV, s.Bst, nout[i], nout[i], nullptr, 0, nullptr, 0, 0, nullptr, 0,
                               off(P.du_qkv, (size_t)s.slot * rp), ldu))) return rc;
      }
      rows_cap_once = P.cap;
      if (need_da && (rc = gemm(N, d, P.dqkv, QKV, P.wT, QKV, QKV, P.n_qkv ? P.du_qkv : nullptr, ldu, P.At_qkv[l], ldu, ldu,
                                nullptr, 0, P.da, d))) return rc;
      if (full || (P.n_qkv && !tn_path())) {
        if ((rc = transpose_tok(QKV, P.dqkv, QKV, P.dyT))) return rc;
        if ((rc = transpose_tok(d, a.a, d, P.xT))) return rc;
      }
      if (P.n_qkv) {
        if ((rc = transpose_tok(ldu, a.u_qkv, ldu, P.uT))) return rc;
        if ((rc = transpose_tok(ldu, P.du_qkv, ldu, P.duT))) return rc;
        for (int i = 0; i < 3; i++)
          if ((rc = lora_grads(l, i, off(P.dqkv, coff[i]), QKV, a.a, d, off(P.dyT, (size_t)coff[i] * P.Np), P.xT))) return rc;
      }
      if (full) {
        float* gw[3] = {G->w_layers[l].wq, G->w_layers[l].wk, G->w_layers[l].wv};
        for (int i = 0; i < 3; i++) if ((rc = weight_grad(gw[i], nout[i], d, off(P.dyT, (size_t)coff[i] * P.Np), P.xT))) return rc;
      } }
    // ---- first norm
    if (!full && l == 0) return AS_OK;
    if (full && (rc = launch_rmsnorm_dgain(ctx, mode, N, d, P.da, nullptr, P.h[l], a.rstd1, P.gpart, 256, G->w_layers[l].g1, st))) return rc;
    return launch_rmsnorm_bwd(ctx, mode, N, d, P.da, nullptr, P.h[l], w.g1, a.rstd1, P.dh2, P.dh, st);
  }

  // one product of the head over the target rows r0 .. r0 + rows - 1 (their number lives on the device), with one of the
  // epilogues that keep the logits out of memory
  int head_gemm(int epi, int rows, int r0, const float* row_w, void* C) {
    GemmParams g; memset(&g, 0, sizeof g);
    g.seg[0] = {off(P.hf, (size_t)r0 * P.d), W->head, P.d, P.d, P.d}; g.nseg = 1;
    g.M = rows; g.N = P.V; g.m_dev = P.count; g.C = C; g.ldc = P.V; g.alpha = 1.f; g.splitk = 1;
    g.epi = epi; g.epi_part = P.part; g.epi_lse = P.lse_rows + r0; g.epi_lab = P.labels + r0;
    g.epi_w = row_w ? row_w + r0 : nullptr; g.epi_cnt = P.count;
    return launch_gemm_off(ctx, mode, gv, g, r0, st);
  }

  // ---- vocabulary head over the compacted target rows P.hf (their number lives on the device) ----
  // Without stored logits (bf16, vocabulary a multiple of 256): per chunk of target rows, the product hf W^T is run with an
  // epilogue that keeps only per-block softmax statistics, a row pass turns them into log-sum-exp and loss, and the product
  // is run again with an epilogue that writes (softmax - onehot) * factor as bf16: that matrix times W gives the gradient.
  // Otherwise (fp32 tier, odd sizes): a float logits chunk, a row pass, the same second product.
  bool head_fused = false;
  int head_chunk_rows(int r0) const { return head_fused ? std::min(P.Mc, (int)cdiv(P.N - r0, 256) * 256) : std::min(P.Mc, P.N - r0); }
  int head_begin(bool grads) {
    int rc;
    if (grads && (rc = transpose(P.V, P.d, W->head, P.d, P.headT, P.V))) return rc;                     // [d, V]
    head_fused = P.head_fused;
    if (!head_fused) return AS_OK;
    GemmParams g; memset(&g, 0, sizeof g);
    g.seg[0] = {P.hf, W->head, P.d, P.d, P.d}; g.nseg = 1; g.M = std::min(P.Mc, (int)cdiv(P.N, 256) * 256); g.N = P.V; g.m_dev = P.count;
    g.C = P.P; g.ldc = P.V; g.splitk = 1;
    if (!gemm_rs_applies(mode, g)) return as_fail(ctx, AS_ERR_SHAPE, "the head matrix must be 16-byte aligned");
    return launch_label_logit(ctx, P.hf, W->head, P.d, P.labels, P.count, P.N, P.zlab, st);
  }
  int head_losses(int r0, int rows) {                        // per-target losses of one chunk
    int rc;
    if (head_fused) {
      if ((rc = head_gemm(GEMM_EPI_STATS, rows, r0, nullptr, nullptr))) return rc;
      return launch_ce_finish(ctx, P.part, P.V / 128, r0, rows, P.count, P.zlab, P.lse_rows, P.loss_rows, st);
    }
    if ((rc = gemm(rows, P.V, off(P.hf, (size_t)r0 * P.d), P.d, W->head, P.d, P.d, nullptr, 0, nullptr, 0, 0, nullptr, 0, P.logits, P.V, 1, 1.f, 0, P.count, r0))) return rc;
    return launch_ce_rows(ctx, mode, P.logits, rows, P.V, r0, P.labels, P.count, P.loss_rows, nullptr, nullptr, st);
  }
  // gradient rows dhf = ((softmax - onehot) * factor) W, factor = row_w or 1 / count; with_losses: the losses too (else they
  // are there already); dw_head: the head's own gradient (full fine-tuning), summed over the chunks
  int head_grad_rows(const float* row_w, bool with_losses, float* dw_head) {
    const int N = P.N, d = P.d, V = P.V, Mc = P.Mc;
    int rc;
    for (int ch = 0, chunks = (int)cdiv(N, Mc); ch < chunks; ch++) {
      const int r0 = ch * Mc, rows = head_chunk_rows(r0);
      const void* hf_c = off(P.hf, (size_t)r0 * d);
      if (head_fused) {
        if (with_losses && (rc = head_losses(r0, rows))) return rc;
        if ((rc = head_gemm(GEMM_EPI_PROB, rows, r0, row_w, P.P))) return rc;
      } else {
        if ((rc = gemm(rows, V, hf_c, d, W->head, d, d, nullptr, 0, nullptr, 0, 0, nullptr, 0, P.logits, V, 1, 1.f, 0, P.count, r0))) return rc;
        if ((rc = launch_ce_rows(ctx, mode, P.logits, rows, V, r0, P.labels, P.count, P.loss_rows, row_w, P.P, st))) return rc;
      }
      if ((rc = gemm(rows, d, P.P, V, P.headT, V, V, nullptr, 0, nullptr, 0, 0, nullptr, 0, off(P.dhf, (size_t)r0 * d), d, 0, 1.f, 0, P.count, r0))) return rc;
      if (dw_head) {
        // dW_head += P_c^T hf_c  (rows past the live count are read as zero)
        // the contraction length is padded to whole 64-token steps (zero rows past the chunk), so that the MFMA kernel takes it
        const int rows64 = (int)cdiv(rows, 64) * 64;
        if ((rc = launch_transpose(ctx, mode, rows, rows64, V, P.P, V, P.Pt, Mc, P.count, r0, st))) return rc;
        if ((rc = launch_transpose(ctx, mode, rows, rows64, d, hf_c, d, P.hfT, Mc, P.count, r0, st))) return rc;
        if ((rc = gemm(V, d, P.Pt, Mc, P.hfT, Mc, rows64, nullptr, 0, nullptr, 0, 0, nullptr, 0, dw_head, d, 1, 1.f, ch > 0))) return rc;
      }
    }
    return AS_OK;
  }

  int head_and_loss(float* d_loss, float* d_loss_sum) {
    const bool full = c.train_mode == AS_FULL;
    const int N = P.N, d = P.d;
    int rc;
    // hf = RMSNorm(h_L) on the target rows only
    if ((rc = launch_rmsnorm_fwd(ctx, mode, N, d, P.h[P.L], P.tgt_idx, P.count, W->g_final, c.rms_eps, P.hf, P.rstd_f, st))) return rc;
    if ((rc = head_begin(LS.kind != LOSS_SEQ_LOGP))) return rc;
    const float* row_w = nullptr;
    if (LS.kind != LOSS_MEAN) {
      // The factor of a target's gradient row depends on the sums over all targets, and the logits are never
      // kept: a first pass over the head yields the per-target losses only, a second one (below) the gradient.
      for (int r0 = 0; r0 < N; r0 += P.Mc) if ((rc = head_losses(r0, head_chunk_rows(r0)))) return rc;
      float* logp = LS.d_logp ? LS.d_logp : P.logp_ws;
      if ((rc = launch_seq_logp(ctx, P.loss_rows, P.tgt_idx, P.count, LS.d_cu, LS.d_kept_of, LS.n_seg, logp, st))) return rc;
      if (LS.kind == LOSS_SEQ_LOGP) return AS_OK;
      if ((rc = launch_dpo_pairs(ctx, LS.d_pairs, LS.n_pairs, logp, LS.d_ref_logp, LS.beta, LS.n_seg, LS.d_kept_of, LS.n_kept, P.w_kept, LS.d_stats, st))) return rc;
      if ((rc = launch_dpo_row_weights(ctx, P.tgt_idx, P.count, LS.d_cu, LS.n_kept, P.w_kept, N, P.row_w, st))) return rc;
      row_w = P.row_w;
    }
    if ((rc = head_grad_rows(row_w, LS.kind == LOSS_MEAN, full ? G->head : nullptr))) return rc;
    if (LS.kind == LOSS_MEAN && (rc = launch_loss_finalize(ctx, P.loss_rows, P.count, d_loss, d_loss_sum, st))) return rc;
    // back through the final norm, scattered to all rows (zero where a row is no target)
    if (full && (rc = launch_rmsnorm_dgain(ctx, mode, N, d, P.dhf, P.tgt_pos, P.h[P.L], P.rstd_f, P.gpart, 256, G->g_final, st))) return rc;
    return launch_rmsnorm_bwd(ctx, mode, N, d, P.dhf, P.tgt_pos, P.h[P.L], W->g_final, P.rstd_f, nullptr, P.dh, st);
  }
};

int Step::launch_lora_prep_ex(const float* in, int rows, int cols, int rows_pad, int cols_pad, float scale,
                              void* out, int64_t ldo, void* out_t, int64_t ldo_t) {
  return launch_lora_prep2(ctx, mode, in, rows, cols, rows_pad, cols_pad, scale, out, ldo, out_t, ldo_t, st);
}
}  // namespace

// Small per-step table (compacted segment boundaries, launch orders, pair list) host -> device into the caller's
// workspace.  The source is ordinary host memory: the copy call returns once it has taken the data over, so nothing of
// the library's has to outlive the call.
static int stage_step_table(as_ctx* ctx, const void* src, size_t bytes, void* dst, hipStream_t st) {
  AS_HIP(ctx, hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, st));
  return AS_OK;
}

static int run_step(as_ctx* ctx, const char* who, const as_weights* weights, const as_lora* lora,
                    const int32_t* d_tokens, const int32_t* d_cu_seqlens,
                    const int32_t* h_cu_seqlens, int32_t n_segments, const uint8_t* h_seg_skip,
                    const uint8_t* d_loss_mask, int32_t n_rows, int32_t row_len,
                    float* d_loss, float* d_loss_sum, int32_t* d_count,
                    const as_grads* grads, void* d_workspace, size_t workspace_bytes,
                    void* stream, LossSpec LS) {
  const as_model_config& c = ctx->cfg;
  const bool full = c.train_mode == AS_FULL;
  if (!weights || !weights->layers || !weights->embed || !weights->head || !weights->g_final)
    return as_fail(ctx, AS_ERR_NULL, "%s: NULL weights", who);
  const bool fwd_only = LS.kind == LOSS_SEQ_LOGP;
  const bool adapters_off = fwd_only && !full && !lora;          // log-probabilities of the base model under the adapters
  if (!d_tokens || !d_cu_seqlens || !h_cu_seqlens || !d_loss_mask || (!fwd_only && !grads))
    return as_fail(ctx, AS_ERR_NULL, "%s: NULL argument", who);
  if (LS.kind == LOSS_MEAN && (!d_loss || !d_loss_sum || !d_count)) return as_fail(ctx, AS_ERR_NULL, "%s: NULL output", who);
  if (LS.kind == LOSS_SEQ_LOGP && !LS.d_logp) return as_fail(ctx, AS_ERR_NULL, "%s: NULL output", who);
  if (LS.kind == LOSS_DPO) {
    if (!LS.d_stats || !LS.d_ref_logp || (LS.n_pairs > 0 && !LS.h_pairs)) return as_fail(ctx, AS_ERR_NULL, "%s: NULL argument", who);
    if (LS.n_pairs < 0 || (int64_t)LS.n_pairs > (int64_t)n_rows * row_len) return as_fail(ctx, AS_ERR_SHAPE, "%s: n_pairs must be in [0, n_rows*row_len]", who);
    if (!(LS.beta >= 0.f) || !std::isfinite(LS.beta)) return as_fail(ctx, AS_ERR_SHAPE, "%s: beta must be finite and >= 0", who);
    for (int p = 0; p < LS.n_pairs; p++) {
      const int a = LS.h_pairs[2 * p], b = LS.h_pairs[2 * p + 1];
      if (a < 0 || a >= n_segments || b < 0 || b >= n_segments || a == b)
        return as_fail(ctx, AS_ERR_SHAPE, "%s: pair %d = (%d, %d) must name two different segments in [0, %d)", who, p, a, b, n_segments);
    }
  }
  if (n_rows < 1 || row_len < 1 || (int64_t)n_rows * row_len > (int64_t)1 << 30)
    return as_fail(ctx, AS_ERR_SHAPE, "%s: n_rows*row_len must be in [1, 2^30]", who);
  for (int l = 0; l < c.n_layers; l++) {
    const as_layer_weights& w = weights->layers[l];
    if (!w.g1 || !w.wq || !w.wk || !w.wv || !w.wo || !w.g2 || !w.wgate || !w.wup || !w.wdown)
      return as_fail(ctx, AS_ERR_NULL, "%s: NULL weight in layer %d", who, l);
    if (c.n_experts && !w.wrouter) return as_fail(ctx, AS_ERR_NULL, "%s: NULL router weight in layer %d", who, l);
    if (c.weight_format == AS_W_NF4 && (!w.aq || !w.ak || !w.av || !w.ao || !w.agate || !w.aup || !w.adown))
      return as_fail(ctx, AS_ERR_NULL, "%s: NULL block maxima of an NF4 weight in layer %d", who, l);
  }
  if (!full && !adapters_off) {
    if (!lora || !lora->layers || (!fwd_only && !grads->lora_layers)) return as_fail(ctx, AS_ERR_NULL, "%s: LoRA mode needs adapters and their gradient buffers", who);
    for (int l = 0; l < c.n_layers; l++)
      for (int t = 0; t < AS_N_TARGETS; t++)
        if ((c.lora_targets >> t) & 1u)
          if (!lora->layers[l].a[t] || !lora->layers[l].b[t] || (!fwd_only && (!grads->lora_layers[l].a[t] || !grads->lora_layers[l].b[t])))
            return as_fail(ctx, AS_ERR_NULL, "%s: NULL adapter or gradient for target %s in layer %d", who, kTargetName[t], l);
  } else if (full && !fwd_only) {
    if (!grads->w_layers || !grads->embed || !grads->head || !grads->g_final) return as_fail(ctx, AS_ERR_NULL, "%s: full mode needs weight gradient buffers", who);
    for (int l = 0; l < c.n_layers; l++) {
      const as_layer_weight_grads& g = grads->w_layers[l];
      if (!g.g1 || !g.wq || !g.wk || !g.wv || !g.wo || !g.g2 || !g.wgate || !g.wup || !g.wdown)
        return as_fail(ctx, AS_ERR_NULL, "%s: NULL weight gradient in layer %d", who, l);
    }
  }
  const int64_t N = (int64_t)n_rows * row_len;
  int max_seg = 0;
  std::string cu_err;
  int rc = check_cu(h_cu_seqlens, n_segments, N, row_len, &max_seg, &cu_err);
  if (rc) return as_fail(ctx, rc, "%s", cu_err.c_str());
  if (!d_workspace || ((uintptr_t)d_workspace & 255)) return as_fail(ctx, AS_ERR_WORKSPACE, "%s: workspace must be non-NULL and 256-byte aligned", who);
  Bump wsp{(char*)d_workspace, 0}; Plan P;
  make_plan(ctx, n_rows, row_len, wsp, P);
  if (adapters_off) { P.n_qkv = P.n_gu = 0; for (LoraSlot& sl : P.lora) sl.on = false; }
  if (wsp.off > workspace_bytes) return as_fail(ctx, AS_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", who, workspace_bytes, wsp.off);

  hipStream_t st = (hipStream_t)stream;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  // Segments the caller marks as carrying no loss-bearing token (pad tails, trajectories without an
  // assistant turn) cannot touch the loss or any gradient: segments never see each other and the
  // weights they would read are not being differentiated through them.  They are squeezed out.
  int n = (int)N, n_seg_eff = n_segments;
  const int32_t* d_cu_eff = d_cu_seqlens;
  std::vector<int32_t> cu_h(h_cu_seqlens, h_cu_seqlens + n_segments + 1), src;   // segment table the kernels will see
  bool compact = false;
  if (h_seg_skip) {
    for (int s = 0; s < n_segments; s++) compact = compact || h_seg_skip[s];
    if (compact) {
      cu_h.assign(1, 0);
      max_seg = 0;
      for (int s = 0; s < n_segments; s++) {
        if (h_seg_skip[s]) continue;
        const int len = h_cu_seqlens[s + 1] - h_cu_seqlens[s];
        src.push_back(h_cu_seqlens[s]); cu_h.push_back(cu_h.back() + len); max_seg = std::max(max_seg, len);
      }
      n_seg_eff = (int)src.size(); n = cu_h.back();
    }
  }
  // The attention kernels' workgroups differ in length by the position of their rows inside a segment
  // (a late query tile visits many key tiles, an early key block is visited by many query tiles), and the
  // workgroups of one segment stream the same tiles.  The launch order lists the segments longest first and,
  // inside a segment, the long workgroups first: neighbours in the order then share their operand tiles in
  // the L2 of the XCD they run on, and the launch ends on the short workgroups of the short segments.
  const bool orders = c.mode == AS_BF16 && (c.head_dim == 64 || c.head_dim == 128) && n > 0;
  const bool seq = LS.kind != LOSS_MEAN;
  if (seq || (n_seg_eff > 0 && (compact || orders))) {
    std::vector<int32_t> tab = cu_h;                       // [cu (S'+1) | src_start (S') | order_q | order_k | kept_of (S) | pairs (2P)]
    tab.insert(tab.end(), src.begin(), src.end());
    size_t off_q = 0, off_k = 0;
    if (orders) {
      const int QT = attention_query_tile(c.n_q_heads, c.n_kv_heads), KPB = 256;
      const int nq = (int)cdiv(n, QT), nk = (int)cdiv(n, KPB);
      auto seg_of = [&](int t) { return (int)(std::upper_bound(cu_h.begin(), cu_h.end(), t) - cu_h.begin()) - 1; };
      std::vector<int32_t> wq(nq), wk(nk), sq(nq), sk(nk), oq(nq), ok(nk);
      for (int i = 0; i < nq; i++) { sq[i] = seg_of(i * QT); wq[i] = std::min(i * QT + QT - 1, n - 1) / 64 - cu_h[sq[i]] / 64 + 1; oq[i] = i; }
      for (int i = 0; i < nk; i++) { sk[i] = seg_of(std::min(i * KPB + KPB - 1, n - 1)); wk[i] = (cu_h[sk[i] + 1] - 1) / 64 - (i * KPB) / 64 + 1; ok[i] = i; }
      auto seg_len = [&](int s) { return cu_h[s + 1] - cu_h[s]; };
      auto before = [&](const std::vector<int32_t>& sg, const std::vector<int32_t>& w, int a, int b) {
        if (sg[a] != sg[b]) { const int la = seg_len(sg[a]), lb = seg_len(sg[b]); return la != lb ? la > lb : sg[a] < sg[b]; }
        return w[a] > w[b];
      };
      std::stable_sort(oq.begin(), oq.end(), [&](int a, int b) { return before(sq, wq, a, b); });
      std::stable_sort(ok.begin(), ok.end(), [&](int a, int b) { return before(sk, wk, a, b); });
      off_q = tab.size(); tab.insert(tab.end(), oq.begin(), oq.end());
      off_k = tab.size(); tab.insert(tab.end(), ok.begin(), ok.end());
    }
    size_t off_kept = 0, off_pairs = 0;
    if (seq) {
      off_kept = tab.size();
      for (int s = 0, k = 0; s < n_segments; s++) tab.push_back(compact && h_seg_skip[s] ? -1 : k++);
      off_pairs = tab.size();
      if (LS.n_pairs > 0) tab.insert(tab.end(), LS.h_pairs, LS.h_pairs + 2 * (size_t)LS.n_pairs);
    }
    if (tab.size() > P.step_tab_ints) return as_fail(ctx, AS_ERR_WORKSPACE, "%s: per-step table of %zu entries exceeds the planned %zu", who, tab.size(), P.step_tab_ints);
    rc = stage_step_table(ctx, tab.data(), tab.size() * 4, P.step_tab, st);
    if (rc) return rc;
    const int32_t* d_tab = P.step_tab;
    if (seq) { LS.d_cu = d_tab; LS.d_kept_of = d_tab + off_kept; LS.d_pairs = d_tab + off_pairs; LS.n_seg = n_segments; LS.n_kept = n_seg_eff; }
    if (compact) {
      if ((rc = launch_compact(ctx, d_tokens, d_loss_mask, d_tab, d_tab + n_seg_eff + 1, n_seg_eff, n, P.tok_c, P.mask_c, st))) return rc;
      d_tokens = P.tok_c; d_loss_mask = P.mask_c; d_cu_eff = d_tab;
    }
    if (orders) { P.order_q = d_tab + off_q; P.order_k = d_tab + off_k; }
  }
  P.N = n; P.Np = (int)cdiv(n, 64) * 64;
  if (seq) d_count = P.count;
  Step S{ctx, c, P, st, c.mode, 0, 0, weights, lora, fwd_only ? nullptr : grads, max_seg, LS};
  if (n == 0) {
    // nothing to differentiate: every sum is empty (log-probability 0), the pair loss follows from the references alone
    if (seq) {
      float* logp = LS.d_logp ? LS.d_logp : P.logp_ws;
      if ((rc = launch_fill_float(ctx, logp, n_segments, 0.f, st))) return rc;
      if (LS.kind == LOSS_DPO && (rc = launch_dpo_pairs(ctx, LS.d_pairs, LS.n_pairs, logp, LS.d_ref_logp, LS.beta, n_segments, LS.d_kept_of, 0, P.w_kept, LS.d_stats, st))) return rc;
      return S.zero_outputs(nullptr, nullptr, nullptr);
    }
    return S.zero_outputs(d_loss, d_loss_sum, d_count);
  }
  if ((rc = launch_segment_info(ctx, d_cu_eff, n_seg_eff, n, P.seg_start, P.seg_end, st))) return rc;
  if ((rc = launch_rope_table(ctx, max_seg, c.head_dim, c.rope_base, P.rope_cos, P.rope_sin, st))) return rc;
  if ((rc = launch_select_targets(ctx, P.seg_start, d_loss_mask, d_tokens, n, P.tgt_idx, P.tgt_pos, P.labels, d_count, st))) return rc;
  P.count = d_count;
  if (!full && !adapters_off) for (int l = 0; l < c.n_layers; l++) if ((rc = S.prep_lora(l))) return rc;
  if ((rc = launch_embed(ctx, c.mode, d_tokens, n, c.d_model, weights->embed, P.h[0], st))) return rc;
  for (int l = 0; l < c.n_layers; l++)
    if ((rc = S.forward_layer(l, P.acts[c.recompute == 1 ? 0 : l]))) return rc;
  if ((rc = S.head_and_loss(d_loss, d_loss_sum))) return rc;
  if (fwd_only) return S.wq_rc;
  for (int l = c.n_layers - 1; l >= 0; l--) {
    Acts& a = P.acts[c.recompute == 1 ? 0 : l];
    if (c.recompute == 1 && l != c.n_layers - 1 && (rc = S.forward_layer(l, a))) return rc;   // re-run the layer from its saved input
    if (c.recompute == 2 && l != c.n_layers - 1 && (rc = S.rebuild_cheap(l, a))) return rc;
    if ((rc = S.backward_layer(l, a))) return rc;
  }
  if (full && (rc = launch_embed_bwd(ctx, c.mode, d_tokens, n, c.d_model, c.vocab, P.dh, P.iscratch, grads->embed, st))) return rc;
  return S.wq_rc;
}

extern "C" int as_train_step(as_ctx* ctx, const as_weights* weights, const as_lora* lora,
                             const int32_t* d_tokens, const int32_t* d_cu_seqlens,
                             const int32_t* h_cu_seqlens, int32_t n_segments, const uint8_t* h_seg_skip,
                             const uint8_t* d_loss_mask, int32_t n_rows, int32_t row_len,
                             float* d_loss, float* d_loss_sum, int32_t* d_count,
                             const as_grads* grads, void* d_workspace, size_t workspace_bytes,
                             void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_train_step: NULL context");
  return run_step(ctx, "as_train_step", weights, lora, d_tokens, d_cu_seqlens, h_cu_seqlens, n_segments, h_seg_skip, d_loss_mask,
                  n_rows, row_len, d_loss, d_loss_sum, d_count, grads, d_workspace, workspace_bytes, stream, LossSpec());
}

extern "C" int as_sequence_logps(as_ctx* ctx, const as_weights* weights, const as_lora* lora,
                                 const int32_t* d_tokens, const int32_t* d_cu_seqlens,
                                 const int32_t* h_cu_seqlens, int32_t n_segments, const uint8_t* h_seg_skip,
                                 const uint8_t* d_loss_mask, int32_t n_rows, int32_t row_len,
                                 float* d_logp, void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_sequence_logps: NULL context");
  LossSpec LS; LS.kind = LOSS_SEQ_LOGP; LS.d_logp = d_logp;
  return run_step(ctx, "as_sequence_logps", weights, lora, d_tokens, d_cu_seqlens, h_cu_seqlens, n_segments, h_seg_skip, d_loss_mask,
                  n_rows, row_len, nullptr, nullptr, nullptr, nullptr, d_workspace, workspace_bytes, stream, LS);
}

extern "C" int as_dpo_step(as_ctx* ctx, const as_weights* weights, const as_lora* lora,
                           const int32_t* d_tokens, const int32_t* d_cu_seqlens,
                           const int32_t* h_cu_seqlens, int32_t n_segments, const uint8_t* h_seg_skip,
                           const uint8_t* d_loss_mask, int32_t n_rows, int32_t row_len,
                           const int32_t* h_pairs, int32_t n_pairs, const float* d_ref_logp, float beta,
                           float* d_stats, float* d_logp,
                           const as_grads* grads, void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_dpo_step: NULL context");
  LossSpec LS; LS.kind = LOSS_DPO; LS.h_pairs = h_pairs; LS.n_pairs = n_pairs; LS.d_ref_logp = d_ref_logp; LS.beta = beta;
  LS.d_stats = d_stats; LS.d_logp = d_logp;
  return run_step(ctx, "as_dpo_step", weights, lora, d_tokens, d_cu_seqlens, h_cu_seqlens, n_segments, h_seg_skip, d_loss_mask,
                  n_rows, row_len, nullptr, nullptr, nullptr, grads, d_workspace, workspace_bytes, stream, LS);
}

static int check_mode(as_ctx* ctx, int mode);

// ------------------------------------------------------ head as a building block
// the head's scratch buffers alone, carved from a workspace (same sizes as inside the step's plan)
static void make_head_plan(const as_ctx* ctx, int mode, int64_t n_rows, Bump& w, Plan& P) {
  const as_model_config& c = ctx->cfg;
  P.N = (int)n_rows; P.cap = P.N; P.d = c.d_model; P.V = c.vocab; P.L = 0; P.es = mode == AS_FP32 ? 4 : 2; P.gemm_tail = nullptr;
  P.head_fused = mode == AS_BF16 && P.V % 256 == 0 && P.d % 64 == 0;
  P.Mc = P.head_fused ? (int)std::min<int64_t>(8192, cdiv(std::max(P.N, 1), 256) * 256) : (int)std::min<int64_t>(4096, cdiv(std::max(P.N, 1), 64) * 64);
  const size_t es = (size_t)P.es, N = (size_t)P.N;
  P.logits = (float*)w.take(P.head_fused ? 0 : (size_t)P.Mc * P.V * 4);
  P.part = (float*)w.take(P.head_fused ? (size_t)P.Mc * (P.V / 128) * 8 : 0);
  P.zlab = (float*)w.take(P.head_fused ? N * 4 : 0); P.lse_rows = (float*)w.take(P.head_fused ? N * 4 : 0);
  P.P = w.take((size_t)P.Mc * P.V * es);
  P.headT = w.take((size_t)P.V * P.d * es);
}

extern "C" int as_op_head_loss_workspace(const as_ctx* ctx, int mode, int64_t n_rows, size_t* bytes) {
  if (!ctx || !bytes) return as_fail(nullptr, AS_ERR_NULL, "as_op_head_loss_workspace: NULL argument");
  if ((mode != AS_FP32 && mode != AS_BF16) || n_rows < 1 || n_rows > (int64_t)1 << 30) return as_fail(const_cast<as_ctx*>(ctx), AS_ERR_SHAPE, "as_op_head_loss_workspace: mode / row count");
  Bump w{nullptr, 0}; Plan P;
  make_head_plan(ctx, mode, n_rows, w, P);
  *bytes = (w.off + 255) & ~(size_t)255;
  return AS_OK;
}

extern "C" int as_op_head_loss(as_ctx* ctx, int mode, int64_t n_rows, const void* hf, const void* head, const int32_t* labels,
                               const int32_t* d_count, const float* row_w, float* loss_rows, void* dhf,
                               void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_op_head_loss: NULL context");
  int rc = check_mode(ctx, mode); if (rc) return rc;
  if (!hf || !head || !labels || !d_count || !loss_rows || !dhf) return as_fail(ctx, AS_ERR_NULL, "as_op_head_loss: NULL operand");
  if (n_rows < 1 || n_rows > (int64_t)1 << 30) return as_fail(ctx, AS_ERR_SHAPE, "as_op_head_loss: row count must be in [1, 2^30]");
  if (!d_workspace || ((uintptr_t)d_workspace & 255)) return as_fail(ctx, AS_ERR_WORKSPACE, "as_op_head_loss: workspace must be non-NULL and 256-byte aligned");
  Bump wsp{(char*)d_workspace, 0}; Plan P;
  make_head_plan(ctx, mode, n_rows, wsp, P);
  if (wsp.off > workspace_bytes) return as_fail(ctx, AS_ERR_WORKSPACE, "as_op_head_loss: workspace has %zu bytes, %zu needed", workspace_bytes, wsp.off);
  P.hf = const_cast<void*>(hf); P.dhf = dhf; P.labels = const_cast<int32_t*>(labels); P.count = const_cast<int32_t*>(d_count); P.loss_rows = loss_rows;
  as_weights W; memset(&W, 0, sizeof W); W.head = head;
  hipStream_t st = (hipStream_t)stream;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  Step S{ctx, ctx->cfg, P, st, mode, 0, 0, &W, nullptr, nullptr, 0, LossSpec()};
  if ((rc = S.head_begin(true))) return rc;
  return S.head_grad_rows(row_w, true, nullptr);
}

// -------------------------------------------------------------------- AdamW
extern "C" int as_adamw_update(as_ctx* ctx, float* const* d_master, void* const* d_params_lowp,
                               const float* const* d_grads, float* const* d_m, float* const* d_v,
                               const int64_t* numel, const uint8_t* apply_wd, int32_t n_tensors,
                               int64_t step, float lr, float beta1, float beta2, float eps,
                               float weight_decay, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_adamw_update: NULL context");
  if (n_tensors < 0) return as_fail(ctx, AS_ERR_SHAPE, "as_adamw_update: n_tensors < 0");
  if (n_tensors && (!d_master || !d_grads || !d_m || !d_v || !numel || !apply_wd)) return as_fail(ctx, AS_ERR_NULL, "as_adamw_update: NULL table");
  if (step < 1) return as_fail(ctx, AS_ERR_SHAPE, "as_adamw_update: step counts from 1");
  if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f)) return as_fail(ctx, AS_ERR_SHAPE, "as_adamw_update: betas must be in [0,1), eps >= 0");
  for (int i = 0; i < n_tensors; i++) {
    if (numel[i] < 0) return as_fail(ctx, AS_ERR_SHAPE, "as_adamw_update: negative numel for tensor %d", i);
    if (numel[i] && (!d_master[i] || !d_grads[i] || !d_m[i] || !d_v[i])) return as_fail(ctx, AS_ERR_NULL, "as_adamw_update: NULL buffer for tensor %d", i);
  }
  AS_HIP(ctx, hipSetDevice(ctx->device));
  const float bc1 = (float)(1.0 - pow((double)beta1, (double)step)), bc2 = (float)(1.0 - pow((double)beta2, (double)step));
  // batches of up to kAdamBatch tensors, each described in its launch's own argument: no table in device memory
  hipStream_t st = (hipStream_t)stream;
  AdamBatch bt; bt.n = 0; bt.n_chunks = 0;
  for (int i = 0; i < n_tensors; i++) {
    if (numel[i] == 0) continue;
    const int64_t nc = cdiv(numel[i], 65536);
    if (nc > INT32_MAX / 2) return as_fail(ctx, AS_ERR_SHAPE, "as_adamw_update: tensor %d is too large", i);
    if (bt.n == kAdamBatch || (int64_t)bt.n_chunks + nc > INT32_MAX / 2) {
      int rc = launch_adamw_batch(ctx, bt, lr, beta1, beta2, eps, bc1, bc2, st);
      if (rc) return rc;
      bt.n = 0; bt.n_chunks = 0;
    }
    bt.t[bt.n++] = {d_master[i], d_params_lowp ? (bf16_t*)d_params_lowp[i] : nullptr, d_grads[i], d_m[i], d_v[i], numel[i],
                    apply_wd[i] ? weight_decay : 0.f, bt.n_chunks};
    bt.n_chunks += (int)nc;
  }
  return launch_adamw_batch(ctx, bt, lr, beta1, beta2, eps, bc1, bc2, st);
}

// ---------------------------------------------------------- building blocks
static int check_mode(as_ctx* ctx, int mode) {
  if (mode != AS_FP32 && mode != AS_BF16) return as_fail(ctx, AS_ERR_CONFIG, "mode must be AS_FP32 or AS_BF16");
  return AS_OK;
}

extern "C" int as_nf4_quantize(as_ctx* ctx, int mode, const void* d_w, int64_t numel, uint8_t* d_codes, float* d_absmax, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_nf4_quantize: NULL context");
  int rc = check_mode(ctx, mode); if (rc) return rc;
  if (numel < 0) return as_fail(ctx, AS_ERR_SHAPE, "as_nf4_quantize: negative element count");
  if (numel && (!d_w || !d_codes || !d_absmax)) return as_fail(ctx, AS_ERR_NULL, "as_nf4_quantize: NULL argument");
  AS_HIP(ctx, hipSetDevice(ctx->device));
  return launch_nf4_quantize(ctx, mode, d_w, numel, d_codes, d_absmax, (hipStream_t)stream);
}

extern "C" int as_nf4_dequantize(as_ctx* ctx, int mode, const uint8_t* d_codes, const float* d_absmax, int64_t numel, void* d_out, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_nf4_dequantize: NULL context");
  int rc = check_mode(ctx, mode); if (rc) return rc;
  if (numel < 0) return as_fail(ctx, AS_ERR_SHAPE, "as_nf4_dequantize: negative element count");
  if (numel && (!d_codes || !d_absmax || !d_out)) return as_fail(ctx, AS_ERR_NULL, "as_nf4_dequantize: NULL argument");
  AS_HIP(ctx, hipSetDevice(ctx->device));
  return launch_nf4_dequantize(ctx, mode, d_codes, d_absmax, numel, d_out, (hipStream_t)stream);
}

extern "C" int as_op_gemm(as_ctx* ctx, int mode, int variant, int64_t M, int64_t N,
                          const void* A1, int64_t lda1, const void* B1, int64_t ldb1, int64_t K1,
                          const void* A2, int64_t lda2, const void* B2, int64_t ldb2, int64_t K2,
                          float alpha, const void* R, int64_t ldr, void* C, int64_t ldc, int c_is_f32,
                          void* d_tail_scratch, size_t tail_scratch_bytes, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_op_gemm: NULL context");
  if (d_tail_scratch && (tail_scratch_bytes < (size_t)AS_GEMM_TAIL_SCRATCH_BYTES || ((uintptr_t)d_tail_scratch & 255)))
    return as_fail(ctx, AS_ERR_WORKSPACE, "as_op_gemm: tail scratch must be 256-byte aligned and hold AS_GEMM_TAIL_SCRATCH_BYTES");
  int rc = check_mode(ctx, mode); if (rc) return rc;
  if (!A1 || !B1 || !C) return as_fail(ctx, AS_ERR_NULL, "as_op_gemm: NULL operand");
  if (M < 0 || N < 0 || K1 < 0 || K2 < 0 || M > INT32_MAX || N > INT32_MAX || K1 > INT32_MAX || K2 > INT32_MAX)
    return as_fail(ctx, AS_ERR_SHAPE, "as_op_gemm: sizes must be in [0, 2^31)");
  if (lda1 < K1 || ldb1 < K1 || ldc < N || (R && ldr < N) || (A2 && (lda2 < K2 || ldb2 < K2 || !B2)))
    return as_fail(ctx, AS_ERR_SHAPE, "as_op_gemm: leading dimension smaller than the row length");
  GemmParams g; memset(&g, 0, sizeof g);
  g.seg[0] = {A1, B1, lda1, ldb1, (int)K1}; g.nseg = 1;
  if (A2 && K2 > 0) { g.seg[1] = {A2, B2, lda2, ldb2, (int)K2}; g.nseg = 2; }
  g.M = (int)M; g.N = (int)N; g.C = C; g.ldc = ldc; g.c_f32 = c_is_f32; g.alpha = alpha; g.R = R; g.ldr = ldr; g.splitk = 1;
  g.tail_part = (float*)d_tail_scratch; g.rows_cap = d_tail_scratch ? (int)M : 0;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  return launch_gemm(ctx, mode, variant, g, (hipStream_t)stream);
}

extern "C" int as_op_gemm_rows(as_ctx* ctx, int mode, int variant, int64_t M, int64_t N,
                               const void* A, int64_t lda, const void* B, int64_t ldb, int64_t K,
                               float alpha, const void* R, int64_t ldr, void* C, int64_t ldc, int c_is_f32,
                               const int32_t* d_rows, int64_t row_off, const int32_t* d_group_off, int group, int n_groups,
                               int64_t group_b_stride, int64_t rows_cap, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_op_gemm_rows: NULL context");
  int rc = check_mode(ctx, mode); if (rc) return rc;
  if (!A || !B || !C) return as_fail(ctx, AS_ERR_NULL, "as_op_gemm_rows: NULL operand");
  if (!d_rows && !d_group_off) return as_fail(ctx, AS_ERR_NULL, "as_op_gemm_rows: a device row count or a group table is required");
  if (M < 0 || N < 0 || K < 0 || M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || row_off < 0 || row_off > INT32_MAX ||
      rows_cap < 0 || rows_cap > INT32_MAX || group < 0 || n_groups < 0 || group_b_stride < 0)
    return as_fail(ctx, AS_ERR_SHAPE, "as_op_gemm_rows: sizes must be in [0, 2^31)");
  if (n_groups > 0 && (!d_group_off || d_rows || row_off)) return as_fail(ctx, AS_ERR_SHAPE, "as_op_gemm_rows: all groups at once need the group table alone");
  if (lda < K || ldb < K || ldc < N || (R && ldr < N))
    return as_fail(ctx, AS_ERR_SHAPE, "as_op_gemm_rows: leading dimension smaller than the row length");
  GemmParams g; memset(&g, 0, sizeof g);
  g.seg[0] = {A, B, lda, ldb, (int)K}; g.nseg = 1;
  g.M = (int)M; g.N = (int)N; g.C = C; g.ldc = ldc; g.c_f32 = c_is_f32; g.alpha = alpha; g.R = R; g.ldr = ldr; g.splitk = 1;
  g.m_dev = d_rows; g.grp_off = d_group_off; g.grp = group; g.rows_cap = (int)rows_cap; g.grp_n = n_groups; g.grp_b_stride = group_b_stride;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  return launch_gemm_off(ctx, mode, variant, g, (int)row_off, (hipStream_t)stream);
}

extern "C" int as_op_rmsnorm_fwd(as_ctx* ctx, int mode, int64_t n, int64_t d, const void* x, const void* g,
                                 float eps, void* y, float* rstd, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_op_rmsnorm_fwd: NULL context");
  int rc = check_mode(ctx, mode); if (rc) return rc;
  if (!x || !g || !y || !rstd) return as_fail(ctx, AS_ERR_NULL, "as_op_rmsnorm_fwd: NULL operand");
  if (n < 0 || d < 1 || n > INT32_MAX || d > INT32_MAX) return as_fail(ctx, AS_ERR_SHAPE, "as_op_rmsnorm_fwd: bad sizes");
  AS_HIP(ctx, hipSetDevice(ctx->device));
  return launch_rmsnorm_fwd(ctx, mode, (int)n, (int)d, x, nullptr, nullptr, g, eps, y, rstd, (hipStream_t)stream);
}

extern "C" int as_op_rmsnorm_bwd(as_ctx* ctx, int mode, int64_t n, int64_t d, const void* dy, const void* x,
                                 const void* g, const float* rstd, const void* add, void* dx, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_op_rmsnorm_bwd: NULL context");
  int rc = check_mode(ctx, mode); if (rc) return rc;
  if (!dy || !x || !g || !rstd || !dx) return as_fail(ctx, AS_ERR_NULL, "as_op_rmsnorm_bwd: NULL operand");
  if (n < 0 || d < 1 || n > INT32_MAX || d > INT32_MAX) return as_fail(ctx, AS_ERR_SHAPE, "as_op_rmsnorm_bwd: bad sizes");
  AS_HIP(ctx, hipSetDevice(ctx->device));
  return launch_rmsnorm_bwd(ctx, mode, (int)n, (int)d, dy, nullptr, x, g, rstd, add, dx, (hipStream_t)stream);
}

static int attn_common(as_ctx* ctx, int mode, int64_t n, int64_t ldq, int64_t ldkv, AttnParams* ap) {
  int rc = check_mode(ctx, mode); if (rc) return rc;
  const as_model_config& c = ctx->cfg;
  if (n < 0 || n > INT32_MAX) return as_fail(ctx, AS_ERR_SHAPE, "attention: bad token count");
  if (ldq < (int64_t)c.n_q_heads * c.head_dim || ldkv < (int64_t)c.n_kv_heads * c.head_dim)
    return as_fail(ctx, AS_ERR_SHAPE, "attention: row stride smaller than heads*head_dim");
  memset(ap, 0, sizeof *ap);
  ap->n = (int)n; ap->Hq = c.n_q_heads; ap->Hkv = c.n_kv_heads; ap->dh = c.head_dim; ap->ldq = ldq; ap->ldkv = ldkv;
  ap->max_seg = (int)std::min<int64_t>(n, 16384);
  return AS_OK;
}

extern "C" int as_op_attention_fwd(as_ctx* ctx, int mode, int variant, int64_t n, const int32_t* seg_start,
                                   const void* q, int64_t ldq, const void* k, const void* v, int64_t ldkv,
                                   void* o, float* lse, void* t_scratch, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_op_attention_fwd: NULL context");
  if (!seg_start || !q || !k || !v || !o || !lse) return as_fail(ctx, AS_ERR_NULL, "as_op_attention_fwd: NULL operand");
  AttnParams ap; int rc = attn_common(ctx, mode, n, ldq, ldkv, &ap); if (rc) return rc;
  ap.seg_start = seg_start; ap.q = q; ap.k = k; ap.v = v; ap.o = o; ap.lse = lse; ap.t_scratch = t_scratch;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  return launch_attention_fwd(ctx, mode, variant, ap, (hipStream_t)stream);
}

static int attention_bwd_op(as_ctx* ctx, const char* who, int mode, int variant, int64_t n, const int32_t* seg_start,
                            const int32_t* seg_end, const void* q, int64_t ldq, const void* k,
                            const void* v, int64_t ldkv, const void* o, const float* lse,
                            const void* d_o, void* dq, void* dk, void* dv, float* delta_scratch,
                            void* t_scratch, void* stream) {
  if (!seg_start || !seg_end || !q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !delta_scratch)
    return as_fail(ctx, AS_ERR_NULL, "%s: NULL operand", who);
  AttnParams ap; int rc = attn_common(ctx, mode, n, ldq, ldkv, &ap); if (rc) return rc;
  ap.seg_start = seg_start; ap.seg_end = seg_end; ap.q = q; ap.k = k; ap.v = v; ap.o = const_cast<void*>(o); ap.lse = const_cast<float*>(lse);
  ap.d_o = d_o; ap.dq = dq; ap.dk = dk; ap.dv = dv; ap.delta = delta_scratch; ap.t_scratch = t_scratch;
  AS_HIP(ctx, hipSetDevice(ctx->device));
  return launch_attention_bwd(ctx, mode, variant, ap, (hipStream_t)stream);
}

extern "C" int as_op_attention_bwd(as_ctx* ctx, int mode, int variant, int64_t n, const int32_t* seg_start,
                                   const int32_t* seg_end, const void* q, int64_t ldq, const void* k,
                                   const void* v, int64_t ldkv, const void* o, const float* lse,
                                   const void* d_o, void* dq, void* dk, void* dv, float* delta_scratch,
                                   void* t_scratch, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_op_attention_bwd: NULL context");
  return attention_bwd_op(ctx, "as_op_attention_bwd", mode, variant, n, seg_start, seg_end, q, ldq, k, v, ldkv, o, lse, d_o, dq, dk, dv,
                          delta_scratch, t_scratch, stream);
}

// ---- the same without any allocation: both scratch buffers live in a device array of the library ----
// In host code the array's name only stands for the symbol; its device address is asked for once per device,
// with that device current, and kept.  Every GPU has a copy of its own.
static __device__ __align__(256) unsigned char scratch[AS_STATIC_SCRATCH_BYTES];
static constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];            // guarded by g_scratch_mu
static std::mutex g_scratch_mu;

static int static_scratch(as_ctx* ctx, void** out) {
  if (ctx->device < 0 || ctx->device >= kMaxDevices) return as_fail(ctx, AS_ERR_SHAPE, "static scratch: device index %d out of range", ctx->device);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[ctx->device]) {
    AS_HIP(ctx, hipSetDevice(ctx->device));
    void* ptr = nullptr;
    AS_HIP(ctx, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    g_scratch_ptr[ctx->device] = ptr;
  }
  *out = g_scratch_ptr[ctx->device];
  return AS_OK;
}

extern "C" int as_op_attention_bwd_static(as_ctx* ctx, int mode, int variant, int64_t n, const int32_t* seg_start,
                                          const int32_t* seg_end, const void* q, int64_t ldq, const void* k,
                                          const void* v, int64_t ldkv, const void* o, const float* lse,
                                          const void* d_o, void* dq, void* dk, void* dv, void* stream) {
  if (!ctx) return as_fail(nullptr, AS_ERR_NULL, "as_op_attention_bwd_static: NULL context");
  int rc = check_mode(ctx, mode); if (rc) return rc;
  if (n < 0 || n > INT32_MAX) return as_fail(ctx, AS_ERR_SHAPE, "as_op_attention_bwd_static: bad token count");
  const as_model_config& c = ctx->cfg;
  // delta [n, Hq] floats, then (256-byte aligned) the token-major copies and partial sums of as_op_attention_bwd
  const size_t es = mode == AS_FP32 ? 4 : 2, n64 = (size_t)cdiv(n, 64) * 64;
  const size_t delta_bytes = ((size_t)n * c.n_q_heads * 4 + 255) & ~(size_t)255;
  const size_t need = delta_bytes + (size_t)(6 * c.n_q_heads + c.n_kv_heads) * c.head_dim * n64 * es;
  if (need > (size_t)AS_STATIC_SCRATCH_BYTES)
    return as_fail(ctx, AS_ERR_WORKSPACE, "as_op_attention_bwd_static: %lld tokens need %zu bytes of scratch, the library holds %zu",
                   (long long)n, need, (size_t)AS_STATIC_SCRATCH_BYTES);
  void* base = nullptr;
  if ((rc = static_scratch(ctx, &base))) return rc;
  return attention_bwd_op(ctx, "as_op_attention_bwd_static", mode, variant, n, seg_start, seg_end, q, ldq, k, v, ldkv, o, lse, d_o, dq, dk, dv,
                          (float*)base, (char*)base + delta_bytes, stream);
}
