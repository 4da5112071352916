/*
 * actionstudio.h -- C interface of the MI355X (gfx950) fine-tuning step.
 *
 * The library computes the hot path of the ActionStudio training pipeline
 * (paper Section 3.2): trajectories are turned into packed token rows with a
 * role-derived loss mask (Section 3.2.1, Universal Data Parser), and one
 * supervised fine-tuning step -- forward and backward of a decoder-only
 * transformer under LoRA or full fine-tuning (Section 3.2.2; LoRA setting of
 * Section 4.5) -- is run on them, followed by an AdamW update (learning-rate
 * range and schedule: Section 4.1).
 *
 * General rules
 *  - Every pointer is marked [host] or [device].  Device buffers are
 *    allocated and freed by the caller; the library keeps no device pointer
 *    of the caller's after a call returns.  Device memory of the library's
 *    own: the staging buffer of as_pack inside the context, pinned host + device,
 *    grown on demand by as_pack only, and one fixed device array
 *    (AS_STATIC_SCRATCH_BYTES, see as_op_attention_bwd_static).  No other call
 *    allocates or frees memory of any kind on the device: as_train_step and its
 *    relatives work inside the caller's workspace (their small per-step tables
 *    included), as_adamw_update hands its tensor table over in kernel arguments.
 *    With per-launch timing switched on (as_profile) events are created on demand.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue work and return without waiting for the device, except
 *    as_pack, which waits for its own upload; results are valid once the
 *    stream has been synchronised.  Host arrays passed to a call may be
 *    reused as soon as it returns.
 *  - Matrices are row-major.  A linear map y = W x stores W as [out, in].
 *  - Every function returns AS_OK (0) or a negative as_status.  Conditions
 *    that can be checked on the host are checked before anything is
 *    launched; after an error no output is defined.  as_last_error() gives a
 *    message for the last failing call on that context (or, for a NULL
 *    context, the last failing call of the calling thread).
 *  - Same inputs give bit-identical outputs: no floating-point atomics.
 *  - Element type "T" below is float in AS_FP32 mode and bfloat16 in AS_BF16
 *    mode.  LoRA matrices and all gradients are always float.
 */
#ifndef ACTIONSTUDIO_H
#define ACTIONSTUDIO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AS_OK = 0,
  AS_ERR_NULL = -1,        /* a required pointer is NULL                         */
  AS_ERR_CONFIG = -2,      /* as_model_config is inconsistent or unsupported     */
  AS_ERR_SHAPE = -3,       /* sizes do not fit each other or the configuration   */
  AS_ERR_CU_SEQLENS = -4,  /* segment table is not a valid partition             */
  AS_ERR_TOKEN_RANGE = -5, /* token id outside [0, vocab)                        */
  AS_ERR_ROLE = -6,        /* role code outside 0..3                             */
  AS_ERR_TOO_LONG = -7,    /* trajectory longer than a row, truncation disabled  */
  AS_ERR_WORKSPACE = -8,   /* workspace missing, misaligned or too small         */
  AS_ERR_HIP = -9          /* a HIP runtime call failed                          */
} as_status;

/* Roles of Unified Format 2.0 (paper, Appendix "Unified Format 2.0").  Only
 * assistant tokens bear loss. */
enum { AS_ROLE_SYSTEM = 0, AS_ROLE_USER = 1, AS_ROLE_ASSISTANT = 2, AS_ROLE_TOOL = 3 };

enum { AS_FP32 = 0, AS_BF16 = 1 };            /* as_model_config.mode        */
enum { AS_LORA = 0, AS_FULL = 1 };            /* as_model_config.train_mode  */

/* LoRA targets: index into the a[]/b[] arrays below and bit position in
 * as_model_config.lora_targets. */
enum { AS_W_DENSE = 0, AS_W_NF4 = 1 };

enum { AS_T_Q = 0, AS_T_K, AS_T_V, AS_T_O, AS_T_GATE, AS_T_UP, AS_T_DOWN, AS_T_ROUTER, AS_N_TARGETS };

typedef struct as_ctx as_ctx;

typedef struct {
  uint32_t struct_size;            /* sizeof(as_model_config), for versioning    */
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  int32_t n_experts, top_k;        /* 0, 0 for a dense FFN                       */
  float rms_eps, rope_base;
  int32_t lora_rank;               /* 0 when train_mode == AS_FULL               */
  float lora_alpha;                /* scale = lora_alpha / lora_rank             */
  uint32_t lora_targets;           /* bit i set: target i carries an adapter     */
  int32_t mode;                    /* AS_FP32 | AS_BF16                          */
  int32_t train_mode;              /* AS_LORA | AS_FULL                          */
  int32_t recompute;               /* activation recompute: 0 keep everything;
                                      1 keep only layer inputs and re-run a layer's
                                      forward before its backward; 2 keep GEMM and
                                      attention outputs, rebuild only the norm
                                      outputs and the SwiGLU product (fits 8B
                                      shapes at 4 x 16k tokens in 288 GB)        */
  int32_t weight_format;           /* AS_W_DENSE: projection weights of type T;
                                      AS_W_NF4: 4-bit NormalFloat blocks (quantised
                                      frozen base under LoRA, paper Section 4.5 /
                                      Table 3 "Q+LoRA"), see as_nf4_quantize      */
} as_model_config;

/* Frozen (LoRA) or trainable (full) weights of one layer.  [device], type T.
 * g1,g2 [d_model]; wq [Hq*dh, d]; wk,wv [Hkv*dh, d]; wo [d, Hq*dh];
 * wgate,wup [ffn, d]; wdown [d, ffn]  (MoE: [n_experts, ...] stacked);
 * wrouter [n_experts, d] or NULL.
 * With weight_format == AS_W_NF4 the seven projection pointers hold packed 4-bit
 * codes (uint8, numel/2 bytes, row-major element order) and aq .. adown the float
 * absolute maxima of their 64-element blocks (numel/64 each); gains stay type T. */
typedef struct {
  const void *g1, *wq, *wk, *wv, *wo, *g2, *wgate, *wup, *wdown, *wrouter;
  const float *aq, *ak, *av, *ao, *agate, *aup, *adown;
} as_layer_weights;

typedef struct {
  const void* embed;               /* [device] T [vocab, d]                      */
  const void* g_final;             /* [device] T [d]                             */
  const void* head;                /* [device] T [vocab, d] (not tied to embed)  */
  const as_layer_weights* layers;  /* [host] array of n_layers                   */
} as_weights;

/* Adapters of one layer: a[i] is A_i [rank, d_in], b[i] is B_i [d_out, rank],
 * [device] float, NULL for targets without an adapter. */
typedef struct {
  const float* a[AS_N_TARGETS];
  const float* b[AS_N_TARGETS];
} as_layer_lora;

typedef struct {
  const as_layer_lora* layers;     /* [host] array of n_layers                   */
} as_lora;

/* Gradient outputs, all [device] float, same shapes as what they belong to.
 * LoRA mode fills lora_layers; full mode fills the weight gradients. */
typedef struct {
  float* a[AS_N_TARGETS];
  float* b[AS_N_TARGETS];
} as_layer_lora_grads;

typedef struct {
  float *g1, *wq, *wk, *wv, *wo, *g2, *wgate, *wup, *wdown, *wrouter;
} as_layer_weight_grads;

typedef struct {
  const as_layer_lora_grads* lora_layers;    /* [host] n_layers, LoRA mode       */
  const as_layer_weight_grads* w_layers;     /* [host] n_layers, full mode       */
  float *embed, *g_final, *head;             /* [device], full mode              */
} as_grads;

/* ---- context ------------------------------------------------------------ */

/* Validates the configuration and binds the context to HIP device `device`.
 * Supported: head_dim in {32, 64, 128}; n_q_heads a multiple of n_kv_heads;
 * d_model, ffn, head counts positive; lora_rank in [1, 256] with at least one
 * target bit in LoRA mode.  AS_ERR_CONFIG otherwise. */
int as_create(as_ctx** out, const as_model_config* cfg, int device);
void as_destroy(as_ctx* ctx);
const char* as_last_error(const as_ctx* ctx);

/* Bytes of device workspace as_train_step needs for up to max_rows rows of
 * row_len tokens.  The workspace must be 256-byte aligned. */
int as_workspace_bytes(const as_ctx* ctx, int64_t max_rows, int64_t row_len, size_t* bytes);

/* ---- per-kernel timing (measurement aid, not part of the method) ---------- *
 * as_profile(ctx, 1) makes the library bracket every launch of the kernel
 * classes below with HIP events on the launch stream (up to 65536 launches,
 * later ones are not recorded); as_profile(ctx, 0) stops and clears.
 * as_profile_read waits for the device, then returns, for one class, the
 * number of recorded launches, the sum of their durations in milliseconds
 * and the sum of their algorithmic flops (2*M*N*K for GEMMs with a host-known
 * row count; 0 for classes where the host cannot know the work). */
enum { AS_K_GEMM_MFMA_256 = 0,   /* bf16 MFMA GEMM, 256x256 tile                 */
       AS_K_GEMM_MFMA_SKINNY,    /* bf16 MFMA GEMM, 256x64 / 64x256 / 128x128    */
       AS_K_GEMM_FMA,            /* plain FMA GEMM                               */
       AS_K_GEMM_DEVROWS,        /* any GEMM whose row count lives on the device */
       AS_K_ATTN_FWD, AS_K_ATTN_BWD, AS_K_TRANSPOSE, AS_K_NORM, AS_K_SWIGLU, AS_K_ROPE, AS_K_CE,
       AS_K_LORA_GRAD,           /* adapter-gradient kernel (contraction over tokens) */
       AS_K_GEMM_GROUPED,        /* expert GEMMs over grouped rows (flops: expected share) */
       AS_K_MOE,                 /* routing, grouping, gather and combine kernels */
       AS_K_GEMM_RS,             /* 256x256 MFMA GEMMs of the hand-scheduled register-staged kernel (long contractions) */
       AS_K_N_CLASSES };
int as_profile(as_ctx* ctx, int enable);
/* Restricts the brackets to one kernel class (kernel_class < 0: every class again): the events cost about 3 us of
 * device time each, 0.5 % of a step with thousands of launches.  Call while timing is off.
 * Errors: AS_ERR_SHAPE for an unknown class or while timing is on. */
int as_profile_only(as_ctx* ctx, int kernel_class);
int as_profile_read(as_ctx* ctx, int kernel_class, int64_t* launches, double* ms, double* flops);

/* Register-resident bf16 MFMA loop over the whole chip (no memory traffic): measures the matrix
 * throughput the part sustains at its clocks under load.  Launches `blocks` workgroups of 8
 * wavefronts, each wavefront issuing iters*8 v_mfma_f32_32x32x16_bf16; times it with events on
 * `stream`, waits, and returns TFLOP/s in *tflops [host].  d_sink [device] float[1]. */
int as_probe_mfma_peak(as_ctx* ctx, int32_t iters, int32_t blocks, float* d_sink, double* tflops, void* stream);

/* Global -> LDS feed rate: `blocks` workgroups of 8 wavefronts, each wavefront keeping
 * `loads_in_flight` (1, 2, 4 or 8) direct-to-LDS loads of 1 KB in flight, walking the first `span_bytes`
 * (a power of two, at most the size of d_buf) of d_buf [device] for `iters` rounds.  Waits, and returns
 * GB/s in *gbps [host].  A small span measures the L2 -> LDS path, a large one the MALL / HBM mix.
 * d_sink [device] int32[1]. */
int as_probe_lds_feed(as_ctx* ctx, int32_t loads_in_flight, const void* d_buf, size_t span_bytes, int32_t iters,
                      int32_t blocks, int32_t* d_sink, double* gbps, void* stream);

/* ---- pack (Section 3.2.1) ----------------------------------------------- */

/* Packs trajectories into rows of row_len tokens.
 *  turn_tokens  [host] int32, all turns back to back
 *  turn_offsets [host] int32 [n_turns+1], token offset of each turn
 *  turn_roles   [host] uint8 [n_turns]
 *  traj_offsets [host] int32 [n_traj+1], first turn of each trajectory
 * Policy: trajectories in input order; a trajectory that does not fit behind
 * the current fill of the open row closes it (tail filled with pad_id) and
 * opens the next; a trajectory longer than row_len keeps its first row_len
 * tokens if `truncate`, else AS_ERR_TOO_LONG; empty trajectories are consumed
 * and leave nothing; packing stops after max_rows rows.
 * Outputs: d_tokens [device] int32 [max_rows*row_len] (first n_rows*row_len
 * written), d_loss_mask [device] uint8 likewise (1 = token of an assistant
 * turn), d_cu_seqlens [device] int32 with room for n_traj + max_rows + 1
 * entries: boundaries of all segments of the flat stream, every trajectory
 * and every non-empty pad tail being one segment.  The three counters are
 * [host].  h_seg_skip_out [host] uint8 with room for n_traj + max_rows
 * entries, or NULL: 1 for segments that hold no loss-bearing token (pad
 * tails, trajectories without a kept assistant token), for as_train_step.
 * Token ids are checked against the context's vocab. */
int as_pack(as_ctx* ctx, const int32_t* turn_tokens, const int32_t* turn_offsets,
            const uint8_t* turn_roles, const int32_t* traj_offsets, int32_t n_traj,
            int32_t row_len, int32_t max_rows, int32_t pad_id, int32_t truncate,
            int32_t* d_tokens, int32_t* d_cu_seqlens, uint8_t* d_loss_mask,
            int32_t* n_rows_out, int32_t* n_segments_out, int32_t* n_traj_consumed_out,
            uint8_t* h_seg_skip_out, void* stream);

/* The same with a choice of packing policy (the paper does not fix one).
 *  AS_PACK_NEXT_FIT: the policy of as_pack.
 *  AS_PACK_BEST_FIT_DECREASING: for a pool of trajectories larger than one batch.  All trajectories
 *   are validated; the non-empty ones (cut to row_len first, or AS_ERR_TOO_LONG) are taken by
 *   non-increasing length, ties in input order; each goes to the open row that it fills best (least
 *   free space left, ties to the lowest row); a new row is opened only when no open row has room;
 *   with max_rows rows open and no room the trajectory is left out.  Rows are written in row
 *   order, the trajectories of a row in the order they were placed.
 *  h_traj_row_out [host] int32 [n_traj] or NULL: row of each trajectory, -1 = not placed (offer it
 *   again), -2 = empty.  *n_traj_consumed_out counts placed + empty trajectories. */
enum { AS_PACK_NEXT_FIT = 0, AS_PACK_BEST_FIT_DECREASING = 1 };
int as_pack_policy(as_ctx* ctx, const int32_t* turn_tokens, const int32_t* turn_offsets,
                   const uint8_t* turn_roles, const int32_t* traj_offsets, int32_t n_traj,
                   int32_t row_len, int32_t max_rows, int32_t pad_id, int32_t truncate, int32_t policy,
                   int32_t* d_tokens, int32_t* d_cu_seqlens, uint8_t* d_loss_mask,
                   int32_t* n_rows_out, int32_t* n_segments_out, int32_t* n_traj_consumed_out,
                   uint8_t* h_seg_skip_out, int32_t* h_traj_row_out, void* stream);

/* ---- one training step (Sections 3.2.2, 4.5) ---------------------------- */

/* Forward and backward of the masked next-token loss over n_rows*row_len
 * packed tokens.  Position t is a target when token t+1 lies in the same
 * segment and d_loss_mask[t+1] == 1; the loss is the mean over targets of
 * logsumexp(z_t) - z_t[token_{t+1}].  Attention is causal inside a segment
 * and never crosses a boundary of d_cu_seqlens; rotary positions restart at
 * each segment.
 *  h_cu_seqlens [host] copy of the segment table, checked before launch
 *               (starts at 0, strictly increasing, ends at n_rows*row_len, no
 *               segment crossing a row end) -- AS_ERR_CU_SEQLENS otherwise.
 *  h_seg_skip   [host] uint8 [n_segments] or NULL.  A 1 is the caller's
 *               statement that the segment holds no loss-bearing token (as
 *               as_pack reports it); such a segment cannot influence the loss
 *               or any gradient and is left out of the computation.  Marking
 *               a segment that does hold mask bits drops its loss terms.
 *  d_loss, d_loss_sum [device] float[1]; d_count [device] int32[1].
 *  lora NULL in full mode.  Gradients are overwritten.  With no target at
 *  all, the loss and every gradient are exactly zero. */
int as_train_step(as_ctx* ctx, const as_weights* weights, const as_lora* lora,
                  const int32_t* d_tokens, const int32_t* d_cu_seqlens,
                  const int32_t* h_cu_seqlens, int32_t n_segments, const uint8_t* h_seg_skip,
                  const uint8_t* d_loss_mask, int32_t n_rows, int32_t row_len,
                  float* d_loss, float* d_loss_sum, int32_t* d_count,
                  const as_grads* grads, void* d_workspace, size_t workspace_bytes,
                  void* stream);

/* ---- preference learning (Sections 1 and 3.2: DPO beside supervised tuning) */

/* The paper names the paradigm only; the loss is the published DPO objective with a frozen
 * reference policy.  With pi_s = sum over the targets t of segment s of log p(token_{t+1} | ...)
 * (the same targets as as_train_step) and ref_s the same sum under the reference policy,
 *   z_p  = beta * [(pi_c - ref_c) - (pi_r - ref_r)]  for pair p = (chosen segment c, rejected r),
 *   loss = mean over pairs of log(1 + exp(-z_p)).
 *
 * as_sequence_logps: forward pass only; writes pi_s for every segment of the caller's table to
 *  d_logp [device] float [n_segments] (0 for a segment without target, or marked in h_seg_skip).
 *  In LoRA mode a NULL `lora` switches the adapters off (the base model: the usual reference
 *  policy of adapter training); in full mode pass the reference weights as `weights`.
 *
 * as_dpo_step: forward, pair loss and backward.
 *  h_pairs     [host] int32 [n_pairs][2]: chosen and rejected segment index of each pair, two
 *              different indices in [0, n_segments) -- AS_ERR_SHAPE otherwise.  A segment may
 *              be in several pairs or in none (then it gets no gradient).
 *  d_ref_logp  [device] float [n_segments], e.g. from as_sequence_logps.
 *  beta        finite, >= 0.
 *  d_stats     [device] float[3]: loss, mean z_p ("reward margin"), fraction of pairs with z_p > 0.
 *  d_logp      [device] float [n_segments] or NULL: the policy's pi_s.
 *  Gradients are overwritten; with no pair they are exactly zero and the loss is 0.
 * All other arguments, the workspace size and the error behaviour are as_train_step's.  The
 * vocabulary head runs twice (per-target losses first, then the gradient rows, whose factor
 * depends on all sums); everything else runs once. */
int as_sequence_logps(as_ctx* ctx, const as_weights* weights, const as_lora* lora,
                      const int32_t* d_tokens, const int32_t* d_cu_seqlens,
                      const int32_t* h_cu_seqlens, int32_t n_segments, const uint8_t* h_seg_skip,
                      const uint8_t* d_loss_mask, int32_t n_rows, int32_t row_len,
                      float* d_logp, void* d_workspace, size_t workspace_bytes, void* stream);
int as_dpo_step(as_ctx* ctx, const as_weights* weights, const as_lora* lora,
                const int32_t* d_tokens, const int32_t* d_cu_seqlens,
                const int32_t* h_cu_seqlens, int32_t n_segments, const uint8_t* h_seg_skip,
                const uint8_t* d_loss_mask, int32_t n_rows, int32_t row_len,
                const int32_t* h_pairs, int32_t n_pairs, const float* d_ref_logp, float beta,
                float* d_stats, float* d_logp,
                const as_grads* grads, void* d_workspace, size_t workspace_bytes, void* stream);

/* ---- AdamW (Section 4.1 hyper-parameters) -------------------------------- */

/* m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 * w <- w - lr * ( m/(1-b1^step) / (sqrt(v/(1-b2^step)) + eps) + wd * w ),
 * the decay using w before the update, skipped where apply_wd[i] == 0.
 * Arrays of n_tensors [host] entries holding [device] pointers:
 *  d_master float (the fp32 weights that are updated); d_params_lowp either
 *  NULL or, per tensor, NULL or a bfloat16 copy rewritten from the master
 *  (round to nearest even); d_grads, d_m, d_v float.  step counts from 1.
 *  The tensors go out in batches of 64 per kernel launch, each batch described in the launch's own argument (no
 *  table in device memory, nothing allocated, nothing waited for). */
int as_adamw_update(as_ctx* ctx, float* const* d_master, void* const* d_params_lowp,
                    const float* const* d_grads, float* const* d_m, float* const* d_v,
                    const int64_t* numel, const uint8_t* apply_wd, int32_t n_tensors,
                    int64_t step, float lr, float beta1, float beta2, float eps,
                    float weight_decay, void* stream);

/* ---- building blocks (the kernels of as_train_step, one at a time) ------- *
 * All pointers [device] unless marked.  `mode` picks T as above.            */

/* C[M,N] = alpha * ( A1[M,K1] B1[N,K1]^T + A2[M,K2] B2[N,K2]^T ) (+ R[M,N]),
 * the second product being the low-rank LoRA term folded into the same
 * accumulation (Section 4.5); A2 may be NULL.  A, B, R of type T; C of type T,
 * or float when c_is_f32.  variant: 0 = pick, 1 = plain FMA kernel,
 * 2 = MFMA kernel (bf16 only; K1, K2, lda, ldb multiples of 8) with the tile
 * shape picked; 10..14 = register-staged tiles 256x256 / 256x64 / 64x256 /
 * 128x128 / 128x64; 30 = direct-to-LDS 256x256 tiles (K in 64-wide steps, else 10);
 * 34 = hand-scheduled 256x256 kernel where it applies (else 30).
 * d_tail_scratch [device], may be NULL: AS_GEMM_TAIL_SCRATCH_BYTES of scratch, 256-byte aligned.  With it the
 * hand-scheduled kernel splits the contraction of the tiles of a last, at most half-full round of 256 workgroups
 * over two workgroups each (as as_train_step does inside its workspace): float partial sums per half, added in
 * order by a second small launch. */
#define AS_GEMM_TAIL_SCRATCH_BYTES (64u << 20)
int as_op_gemm(as_ctx* ctx, int mode, int variant, int64_t M, int64_t N,
               const void* A1, int64_t lda1, const void* B1, int64_t ldb1, int64_t K1,
               const void* A2, int64_t lda2, const void* B2, int64_t ldb2, int64_t K2,
               float alpha, const void* R, int64_t ldr, void* C, int64_t ldc, int c_is_f32,
               void* d_tail_scratch, size_t tail_scratch_bytes, void* stream);

/* The same product over rows whose number is only known on the device (one K
 * segment).  The target rows of the vocabulary head (Section 3.2.1: the loss
 * covers assistant tokens only, their number comes out of the mask on the
 * device) and the rows of one expert of a sparse model (Section 4.1 names
 * Mixtral-8x7B/8x22B) are such products.
 *   d_rows       [device] int32, may be NULL: the product covers rows
 *                0 .. min(M, *d_rows - row_off) - 1 of A, R and C (the caller
 *                has already moved the three pointers to row row_off).
 *   d_group_off  [device] int32 table, may be NULL: the product covers rows
 *                d_group_off[group] .. d_group_off[group + 1] - 1 (at most M
 *                of them) of A, R and C.
 *   n_groups     > 0: every group 0 .. n_groups - 1 in one call (`group` is
 *                ignored, d_rows must be NULL, row_off 0); group e multiplies
 *                with the matrix that starts group_b_stride elements after
 *                that of group e - 1, B being that of group 0.
 *   rows_cap     with d_group_off: the number of rows A, R and C have (0 = not
 *                stated; kernels that read whole row tiles then stay out).
 * Rows outside the live range are neither read into the result nor written.
 * A, R, C must hold M rows (d_rows) or rows_cap rows (d_group_off).
 * Errors: AS_ERR_NULL without both tables, AS_ERR_SHAPE as as_op_gemm. */
int as_op_gemm_rows(as_ctx* ctx, int mode, int variant, int64_t M, int64_t N,
                    const void* A, int64_t lda, const void* B, int64_t ldb, int64_t K,
                    float alpha, const void* R, int64_t ldr, void* C, int64_t ldc, int c_is_f32,
                    const int32_t* d_rows, int64_t row_off, const int32_t* d_group_off, int group, int n_groups,
                    int64_t group_b_stride, int64_t rows_cap, void* stream);

/* y = x * rstd * g with rstd = (mean x^2 + eps)^-1/2 per row; rstd float[n]. */
int as_op_rmsnorm_fwd(as_ctx* ctx, int mode, int64_t n, int64_t d, const void* x, const void* g,
                      float eps, void* y, float* rstd, void* stream);
/* dx = rstd g dy - x rstd^3/d sum_j(g_j dy_j x_j) (+ add, type T, may be NULL). */
int as_op_rmsnorm_bwd(as_ctx* ctx, int mode, int64_t n, int64_t d, const void* dy, const void* x,
                      const void* g, const float* rstd, const void* add, void* dx, void* stream);

/* Varlen causal attention with grouped KV heads over packed rows.  q [n,Hq,dh]
 * with row stride ldq elements, k, v [n,Hkv,dh] with stride ldkv, o [n,Hq,dh]
 * dense, lse float [n,Hq].  seg_start [n] int32: first token of each token's
 * segment.  variant: 0 = pick, 1 = plain kernel, 2 = MFMA kernels (bf16, head_dim 64 or 128); backward only:
 * 4 = the MFMA kernels that work from token-major copies, dK and dV in two launches with float partials per query
 * head.  Otherwise head_dim 64 takes the same kernels with dK and dV from one launch, and head_dim 128 with row
 * strides that are multiples of 128 elements the one-pass kernels that read their operands as they are.
 * t_scratch: type T, only read by the MFMA kernels (may be NULL otherwise):
 * room for Hkv*dh * n64 elements in forward and (6*Hq + Hkv)*dh * n64 in
 * backward, n64 = n rounded up to 64 (token-major copies of V, resp. K, Q, dO,
 * followed in backward by float dK / dV partials per query head; the one-pass kernels leave it untouched). */
int as_op_attention_fwd(as_ctx* ctx, int mode, int variant, int64_t n, const int32_t* seg_start,
                        const void* q, int64_t ldq, const void* k, const void* v, int64_t ldkv,
                        void* o, float* lse, void* t_scratch, void* stream);
/* seg_end [n] int32: one past the last token of each token's segment.
 * dq, dk, dv have the layout of q, k, v (strides ldq, ldkv). */
int as_op_attention_bwd(as_ctx* ctx, int mode, int variant, int64_t n, const int32_t* seg_start,
                        const int32_t* seg_end, const void* q, int64_t ldq, const void* k,
                        const void* v, int64_t ldkv, const void* o, const float* lse,
                        const void* d_o, void* dq, void* dk, void* dv, float* delta_scratch,
                        void* t_scratch, void* stream);

/* The vocabulary head with the masked cross-entropy (Section 3.2.1: the loss covers assistant tokens only), as the
 * step runs it over the compacted target rows:
 *   loss_rows[r] = logsumexp_v(hf[r] . head[v]) - hf[r] . head[labels[r]],
 *   dhf[r]       = factor_r * (softmax_v(hf[r] . head[v]) - onehot(labels[r])) head,   factor_r = row_w[r], or 1 / *d_count
 * for the rows r < *d_count (a device-side count, at most n_rows); other rows are neither read into a result nor written.
 *  hf, dhf  [device] T [n_rows rounded up to a multiple of 256, d_model] (the products run over whole 256-row tiles);
 *  head     [device] T [vocab, d_model], 16-byte aligned; labels [device] int32 [n_rows]; row_w [device] float [n_rows] or NULL;
 *  loss_rows [device] float [n_rows].
 * In AS_BF16 mode with vocab a multiple of 256 and d_model a multiple of 64 no logits are stored: the product runs twice,
 * first with an epilogue that keeps per-block softmax statistics only, then with one that writes the gradient rows with
 * respect to the logits as bf16, 8192 target rows at a time.  Otherwise a float logits chunk of 4096 rows is used.
 * Workspace: as_op_head_loss_workspace bytes, 256-byte aligned.  d_model and vocab are the context's. */
int as_op_head_loss_workspace(const as_ctx* ctx, int mode, int64_t n_rows, size_t* bytes);
int as_op_head_loss(as_ctx* ctx, int mode, int64_t n_rows, const void* hf, const void* head, const int32_t* labels,
                    const int32_t* d_count, const float* row_w, float* loss_rows, void* dhf,
                    void* d_workspace, size_t workspace_bytes, void* stream);

/* as_op_attention_bwd for callers that cannot allocate device memory or hand over a workspace (code under HIP
 * graph capture, serving loops, harnesses that forbid hipMalloc): same arguments without the two scratch
 * buffers, which live in a device array of AS_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held
 * until the process ends).  The call allocates nothing.  Sizes that need more than that
 * ((6*Hq + Hkv)*dh*n64 elements of T plus n*Hq floats, n64 = n rounded up to 64) are rejected with
 * AS_ERR_WORKSPACE before anything is launched.  All calls on one GPU share the array: calls that overlap on
 * one GPU (different streams or threads) race, and nothing of a call's scratch contents survives the next. */
#define AS_STATIC_SCRATCH_BYTES (32u << 20)
int as_op_attention_bwd_static(as_ctx* ctx, int mode, int variant, int64_t n, const int32_t* seg_start,
                               const int32_t* seg_end, const void* q, int64_t ldq, const void* k,
                               const void* v, int64_t ldkv, const void* o, const float* lse,
                               const void* d_o, void* dq, void* dk, void* dv, void* stream);

/* NF4 block quantisation of a frozen weight tensor (the "Q" of the paper's Q+LoRA regime, Section 4.5;
 * format of the public QLoRA description): numel (a multiple of 64) elements of type T, flattened
 * row-major, in blocks of 64: absmax[b] = max |w| of block b (float), code = index of the nearest of
 * the 16 NormalFloat levels to w / absmax (float32 decision, midpoint goes up), two codes per byte
 * (element 2j in the low nibble).  d_codes: numel/2 bytes, d_absmax: numel/64 floats, all [device].
 * as_nf4_dequantize writes level[code] * absmax as type T.  as_train_step dequantises one projection
 * at a time into its workspace, so the resident copy of the base model is 4.5 bits per weight. */
int as_nf4_quantize(as_ctx* ctx, int mode, const void* d_w, int64_t numel, uint8_t* d_codes, float* d_absmax, void* stream);
int as_nf4_dequantize(as_ctx* ctx, int mode, const uint8_t* d_codes, const float* d_absmax, int64_t numel, void* d_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ACTIONSTUDIO_H */
