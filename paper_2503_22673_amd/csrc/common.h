// Shared declarations of the gfx950 fine-tuning library: element types,
// error plumbing, the context, and the launchers each .hip file exports to
// the C interface in api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string>
#include <vector>
#include <algorithm>
#include <atomic>
#include "actionstudio.h"

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define AS_WAVE 64

struct as_ctx {
  as_model_config cfg;
  int device;
  std::string err;
  // staging owned by the context (as_pack only)
  void* d_stage = nullptr; size_t d_stage_bytes = 0;
  void* h_stage = nullptr; size_t h_stage_bytes = 0;
  // optional per-launch timing (as_profile): event pairs around kernels of the tracked classes
  struct ProfRec { hipEvent_t a, b; double flops; int cls; };
  bool prof_on = false; int prof_depth = 0;
  int prof_only = -1; bool prof_skipping = false;   // >= 0: only this class is bracketed
  std::vector<ProfRec> prof; size_t prof_used = 0;
};
// Brackets one kernel launch with events when profiling is on (no-ops otherwise).
void prof_begin(as_ctx* ctx, hipStream_t st, int cls, double flops);
void prof_end(as_ctx* ctx, hipStream_t st);

int as_fail(as_ctx* ctx, int code, const char* fmt, ...);
#define AS_HIP(ctx, call) do { hipError_t e_ = (call); if (e_ != hipSuccess) \
  return as_fail((ctx), AS_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); } while (0)
#define AS_LAUNCH_CHECK(ctx) AS_HIP(ctx, hipGetLastError())
// Raises a kernel's dynamic LDS limit once per device (the attribute belongs to the code object loaded on that device).
#define AS_SET_SMEM(ctx, kern, bytes) do { static std::atomic<uint64_t> done_{0}; const uint64_t bit_ = 1ull << ((ctx)->device & 63); \
  if (!(done_.load(std::memory_order_relaxed) & bit_)) { \
    AS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(bytes))); \
    done_.fetch_or(bit_, std::memory_order_relaxed); } } while (0)

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

template <typename T> __device__ __forceinline__ float to_f(T x);
template <> __device__ __forceinline__ float to_f<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f(float x);
template <> __device__ __forceinline__ float from_f<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float x) { return (bf16_t)x; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- GEMM (gemm.hip) ------------------------------------------------------
// C[M,N] = alpha * sum_s A_s[M,K_s] B_s[N,K_s]^T (+ R), optional split over K.
struct GemmSeg { const void* A; const void* B; int64_t lda, ldb; int K; };
struct GemmParams {
  GemmSeg seg[2]; int nseg;
  int M, N;
  const int* m_dev;        // if set, the row count is read from the device (<= M)
  void* C; int64_t ldc; int c_f32;
  float alpha;
  const void* R; int64_t ldr;
  int accumulate;          // C += result (float output only)
  int splitk; float* partial;   // splitk > 1: partial [splitk, M, N] float, reduced afterwards
  // grouped rows (mixture of experts): with grp_off set, the product covers rows
  // [grp_off[grp], grp_off[grp+1]) of A, R and C (device-side table), at most M of them
  const int* grp_off; int grp;
  double grp_rows;            // expected live rows of the launch (timing records only)
  // grp_n > 0: ALL groups 0 .. grp_n - 1 in one launch (grp is ignored); group e multiplies with the matrix that
  // starts grp_b_stride elements after that of group e - 1 (B of segment 0; one segment only)
  int grp_n; int64_t grp_b_stride;
  // rows that every row operand (A of each segment, R, C) really has allocated, or 0: lets a kernel that works in
  // whole 256-row tiles run over the ragged last tile too (rows past M are computed from whatever is there and
  // written to rows past M of C; no row of the result depends on another row)
  int rows_cap;
  // Column groups: several weight matrices whose outputs sit side by side in C (q | k | v, gate | up) as ONE launch: fewer,
  // larger grids (every launch ends on a partial round of tiles) and the shared row panel of A is read once per tile row.
  // Group g covers columns [cg_end[g-1], cg_end[g]) (multiples of 256); its rows of B come from cg_B1[g] (segment 0) and
  // cg_B2[g] (segment 1), both indexed from the group's first column, and segment 1 reads A at column offset cg_a2[g]
  // (each projection has its own adapter activations).  ncg == 0: seg[].B as usual.
  int ncg; int cg_end[3]; const void* cg_B1[3]; const void* cg_B2[3]; int cg_a2[3];
  // Vocabulary head without stored logits (hand-scheduled kernel only; rows and row arrays are those of A):
  //  epi == GEMM_EPI_STATS: nothing is written to C; for every row and every 128-column block of the result the maximum and
  //    the sum of exp(value - maximum) go to epi_part[(row * (N / 128) + block) * 2 + {0, 1}];
  //  epi == GEMM_EPI_PROB:  C = w_row * (exp(value - epi_lse[row]) - [column == epi_lab[row]]), w_row = epi_w[row] when
  //    given, else 1 / *epi_cnt: the gradient of the masked loss with respect to the logits, straight from the accumulators.
  // Last partial round of tiles (hand-scheduled kernel, plain rows): with tail_first >= 0 the tiles tail_first .. of the launch
  // are each computed by TWO workgroups, one per half of the contraction, as float partials in tail_part
  // [tile - tail_first][half][256 x 256]; a second small launch adds the halves in order and applies the epilogue.
  // A launch of 3696 tiles on 256 CUs then ends after 14.5 rounds instead of 15.  Set by the launcher.
  int tail_first; float* tail_part;
  int epi; const float* epi_lse; const int32_t* epi_lab; const float* epi_w; const int32_t* epi_cnt; float* epi_part;
};
enum { GEMM_EPI_NONE = 0, GEMM_EPI_STATS = 1, GEMM_EPI_PROB = 2 };
// the hand-scheduled kernel would take this product (whole 256 x 256 tiles, K in 64-wide steps, alignment)
bool gemm_rs_applies(int mode, const GemmParams& p);
// floats of scratch (GemmParams::tail_part given by the caller through `tail_ws`) that let the launcher split the last round
constexpr size_t kGemmTailFloats = (size_t)128 * 2 * 256 * 256;
int launch_gemm(as_ctx* ctx, int mode, int variant, const GemmParams& p, hipStream_t st);
// live rows = *p.m_dev - m_off, clamped to [0, p.M]
int launch_gemm_off(as_ctx* ctx, int mode, int variant, const GemmParams& p, int m_off, hipStream_t st);

int launch_feed_probe(as_ctx* ctx, int k, const void* buf, size_t span, int iters, int blocks, int* sink, hipStream_t st);
int launch_mfma_peak(as_ctx* ctx, int iters, int blocks, float* sink, hipStream_t st);

// ---- adapter gradients (lora_grad.hip) ---------------------------------------
// C[m*sm + j*sj] = alpha * sum_t X[t, m] * UT[j, t]  (bf16 X row-major, UT token-major, float C)
size_t lora_grad_tn_partial_floats(int n, int M, int r);
int launch_lora_grad_tn(as_ctx* ctx, const void* X, int64_t ldx, const void* UT, int64_t ldu, int n, int M, int r,
                        float alpha, float* C, int64_t sm, int64_t sj, float* partial, size_t partial_floats, hipStream_t st);

// ---- attention (attention.hip) -----------------------------------------------
struct AttnParams {
  int n, Hq, Hkv, dh;
  const int32_t* seg_start; const int32_t* seg_end;
  const void *q, *k, *v; int64_t ldq, ldkv;
  void* o; float* lse;
  const void* d_o; void *dq, *dk, *dv; float* delta;
  int max_seg;             // longest segment (host knowledge, sizes LDS of the plain kernels)
  // MFMA kernels: scratch for token-major copies ([column][token], row length ldT = tokens rounded up
  // to 64): forward needs Hkv*dh rows (V^T), backward (2*Hq + Hkv)*dh rows (K^T, Q^T, dO^T)
  void* t_scratch;
  const void *qT, *kT, *vT, *doT; int64_t ldT;   // filled by the launchers
  // optional launch orders (device arrays, longest workgroups first): order_q[i] = query tile of workgroup i
  // (tiles of attention_query_tile() tokens), order_k[i] = key block (256 keys) of workgroup i in the dK / dV launches
  const int32_t* order_q; const int32_t* order_k;
  // backward, MFMA kernels only: when set, dq and dk leave the kernels already rotated back (the inverse of the rotary
  // embedding applied to q and k before attention): tables [position][dh / 2] of cos and sin, position = t - seg_start[t]
  const float* rope_cos; const float* rope_sin;
};
// the MFMA backward kernels will take this call (then the rotation above is available)
bool attention_bwd_is_mfma(int mode, int variant, const AttnParams& p);
int launch_attention_fwd(as_ctx* ctx, int mode, int variant, const AttnParams& p, hipStream_t st);
int attention_query_tile(int n_q_heads, int n_kv_heads);   // tokens per workgroup of the forward and dQ MFMA kernels
int launch_attention_bwd(as_ctx* ctx, int mode, int variant, const AttnParams& p, hipStream_t st);

// ---- element-wise and friends (elementwise.hip) ---------------------------------
int launch_pack(as_ctx* ctx, const int32_t* d_src_tokens, const int32_t* d_piece_dst,
                const int32_t* d_piece_src, const uint8_t* d_piece_mask, int n_pieces, int n_out,
                int pad_id, int32_t* d_tokens, uint8_t* d_mask, hipStream_t st);
// tok_c[i], mask_c[i] = tok[src], mask[src] with src = src_start[s] + (i - cu_c[s]) for the kept segment s holding i
int launch_compact(as_ctx* ctx, const int32_t* tok, const uint8_t* mask, const int32_t* cu_c, const int32_t* src_start,
                   int n_seg, int n, int32_t* tok_c, uint8_t* mask_c, hipStream_t st);
int launch_segment_info(as_ctx* ctx, const int32_t* d_cu, int n_seg, int n, int32_t* seg_start,
                        int32_t* seg_end, hipStream_t st);
int launch_rope_table(as_ctx* ctx, int max_pos, int dh, float base, float* cosb, float* sinb, hipStream_t st);
int launch_embed(as_ctx* ctx, int mode, const int32_t* tok, int n, int d, const void* E, void* h, hipStream_t st);
int launch_rmsnorm_fwd(as_ctx* ctx, int mode, int n, int d, const void* x, const int32_t* row_idx,
                       const int* n_dev, const void* g, float eps, void* y, float* rstd, hipStream_t st);
// dx[t] = vjp(dy[row_of(t)]) + add[t]; src_pos (optional) maps t -> row of dy or -1 (then dx = add or 0)
int launch_rmsnorm_bwd(as_ctx* ctx, int mode, int n, int d, const void* dy, const int32_t* src_pos,
                       const void* x, const void* g, const float* rstd, const void* add, void* dx,
                       hipStream_t st);
int launch_rmsnorm_dgain(as_ctx* ctx, int mode, int n, int d, const void* dy, const int32_t* src_pos,
                         const void* x, const float* rstd, float* partial, int n_part, float* dg,
                         hipStream_t st);
int launch_rope(as_ctx* ctx, int mode, int n, int n_heads, int dh, void* x, int64_t ldx,
                const int32_t* seg_start, const float* cosb, const float* sinb, int inverse, hipStream_t st);
// NF4 block quantisation (quant.hip)
int launch_nf4_quantize(as_ctx* ctx, int mode, const void* w, int64_t numel, uint8_t* codes, float* absmax, hipStream_t st);
int launch_nf4_dequantize(as_ctx* ctx, int mode, const uint8_t* codes, const float* absmax, int64_t numel, void* out, hipStream_t st);
// mixture-of-experts routing and row grouping (moe.hip)
int launch_moe_route(as_ctx* ctx, const float* logit, int n, int E, int32_t* sel, float* w, hipStream_t st);
int launch_moe_permute(as_ctx* ctx, const int32_t* sel, int n, int E, int32_t* eoff, int32_t* pos, int32_t* perm, hipStream_t st);
int launch_moe_gather(as_ctx* ctx, int mode, const void* src, const int32_t* perm, const float* w, int rows, int d, void* out, hipStream_t st);
int launch_moe_combine(as_ctx* ctx, int mode, const void* res, const void* y, const int32_t* pos, const float* w, int n, int d,
                       void* out, hipStream_t st);
int launch_moe_dlogit(as_ctx* ctx, int mode, const void* dy, const void* y, const int32_t* pos, const int32_t* sel, const float* w,
                      int n, int d, int Epad, void* dlogit, hipStream_t st);
int launch_swiglu_fwd(as_ctx* ctx, int mode, int64_t n, int F, const void* gu, void* m, hipStream_t st);
int launch_swiglu_bwd(as_ctx* ctx, int mode, int64_t n, int F, const void* dm, const void* gu, void* dgu, void* m_out, hipStream_t st);
// out[c, r] = in[r, c] for r < rows_pad, reading zero for r >= rows (and, with rows_dev, for rows at
// or past *rows_dev - row_off)
int launch_transpose(as_ctx* ctx, int mode, int rows, int rows_pad, int cols, const void* in, int64_t ldi, void* out,
                     int64_t ldo, const int* rows_dev, int row_off, hipStream_t st);
int launch_transpose_qs(as_ctx* ctx, int mode, int rows, int rows_pad, int cols, const void* in, int64_t ldi, void* out,
                        int64_t ldo, hipStream_t st);
// out[rows_pad, cols_pad] (type T, row stride ldo) = scale * in[rows, cols] (float), zero in the
// padding; out_t (row stride ldo_t) receives the transpose.  Either output may be NULL.
int launch_lora_prep2(as_ctx* ctx, int mode, const float* in, int rows, int cols, int rows_pad, int cols_pad,
                      float scale, void* out, int64_t ldo, void* out_t, int64_t ldo_t, hipStream_t st);
int launch_fill_zero(as_ctx* ctx, void* p, size_t bytes, hipStream_t st);
int launch_select_targets(as_ctx* ctx, const int32_t* seg_start, const uint8_t* mask, const int32_t* tok,
                          int n, int32_t* tgt_idx, int32_t* tgt_pos, int32_t* labels, int32_t* count,
                          hipStream_t st);
// one row of logits per target: loss_t, and P = (softmax - onehot) / count written as T
int launch_ce_rows(as_ctx* ctx, int mode, const float* logits, int rows_cap, int V, int row0,
                   const int32_t* labels, const int32_t* count, float* loss_rows, const float* row_w, void* P, hipStream_t st);
// preference loss (dpo.hip)
int launch_seq_logp(as_ctx* ctx, const float* loss_rows, const int32_t* tgt_idx, const int32_t* count, const int32_t* cu,
                    const int32_t* kept_of, int n_seg, float* logp, hipStream_t st);
int launch_dpo_pairs(as_ctx* ctx, const int32_t* pairs, int n_pairs, const float* logp, const float* ref, float beta, int n_seg,
                     const int32_t* kept_of, int n_kept, float* w_kept, float* stats, hipStream_t st);
int launch_dpo_row_weights(as_ctx* ctx, const int32_t* tgt_idx, const int32_t* count, const int32_t* cu, int n_kept,
                           const float* w_kept, int n, float* row_w, hipStream_t st);
int launch_fill_float(as_ctx* ctx, float* p, int n, float v, hipStream_t st);
// head without stored logits: z_lab[row] = hf[row] . W[labels[row]] for rows < *count; then per row the log-sum-exp from the
// per-block statistics of the GEMM and loss = lse - z_lab
int launch_label_logit(as_ctx* ctx, const void* hf, const void* W, int d, const int32_t* labels, const int32_t* count, int rows_cap,
                       float* zlab, hipStream_t st);
int launch_ce_finish(as_ctx* ctx, const float* part, int nblk, int row0, int rows_cap, const int32_t* count, const float* zlab,
                     float* lse, float* loss_rows, hipStream_t st);
int launch_loss_finalize(as_ctx* ctx, const float* loss_rows, const int32_t* count, float* loss,
                         float* loss_sum, hipStream_t st);
int launch_splitk_reduce(as_ctx* ctx, const float* partial, int splitk, int64_t mn, int N, float alpha,
                         float* C, int64_t ldc, hipStream_t st);
// one tensor of a multi-tensor update, and one 64 K-element chunk of work
struct AdamTensor { float* w; bf16_t* w_lowp; const float* g; float* m; float* v; int64_t n; float wd; int first_chunk; };
// a batch of tensors travels as a kernel argument: no table in device memory, nothing to allocate or to keep alive
constexpr int kAdamBatch = 64;
struct AdamBatch { AdamTensor t[kAdamBatch]; int n; int n_chunks; };
int launch_adamw_batch(as_ctx* ctx, const AdamBatch& b, float lr, float b1, float b2, float eps, float bc1, float bc2, hipStream_t st);
int launch_embed_bwd(as_ctx* ctx, int mode, const int32_t* tok, int n, int d, int V, const void* dh,
                     int32_t* scratch, float* dE, hipStream_t st);
