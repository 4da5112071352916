// Preference learning (DPO; the paper's Sections 1 and 3.2 name it beside supervised fine-tuning, the
// loss is the published DPO objective with a frozen reference policy): the small kernels between the
// two passes over the vocabulary head.  Pass one yields -log p of every target; these kernels turn them
// into per-segment sums pi_s, the pair loss and, per target row, the factor its (softmax - one-hot) row is
// scaled with in pass two.  Every sum runs in a fixed order, in double.
#include "common.h"

// first target row whose token position is >= pos (rows are in token order)
__device__ inline int lower_row(const int32_t* __restrict__ tgt_idx, int cnt, int pos) {
  int lo = 0, hi = cnt;
  while (lo < hi) { const int mid = (lo + hi) >> 1; if (tgt_idx[mid] < pos) lo = mid + 1; else hi = mid; }
  return lo;
}

// pi_s = - sum of the target losses of segment s.  One workgroup per segment of the caller's table;
// kept_of[s] is the segment's index in the table the kernels run on (-1: left out, pi = 0).
__global__ __launch_bounds__(256) void seq_logp_kernel(const float* __restrict__ loss_rows, const int32_t* __restrict__ tgt_idx,
                                                       const int32_t* __restrict__ count, const int32_t* __restrict__ cu,
                                                       const int32_t* __restrict__ kept_of, float* __restrict__ logp) {
  __shared__ double sh[256];
  const int s = blockIdx.x, ks = kept_of ? kept_of[s] : s;
  double acc = 0.0;
  if (ks >= 0) {
    const int cnt = *count;
    const int r0 = lower_row(tgt_idx, cnt, cu[ks]), r1 = lower_row(tgt_idx, cnt, cu[ks + 1]);
    const int per = (r1 - r0 + 255) / 256, b = r0 + threadIdx.x * per, e = min(r1, b + per);
    for (int i = b; i < e; i++) acc += (double)loss_rows[i];
  }
  sh[threadIdx.x] = acc;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) logp[s] = (float)(-sh[0]);
}

// z_p = beta [(pi_c - ref_c) - (pi_r - ref_r)];  loss = mean_p log(1 + exp(-z_p));
// d loss / d pi_c = -beta sigmoid(-z_p) / P, d loss / d pi_r = +beta sigmoid(-z_p) / P.
// One workgroup.  stats = {loss, mean z, fraction of pairs with z > 0}.  w_kept[k] receives MINUS the
// derivative with respect to pi of kept segment k (the factor of its targets' loss rows), summed over the
// pairs the segment is in, in pair order.
__global__ __launch_bounds__(1024) void dpo_pairs_kernel(const int32_t* __restrict__ pairs, int n_pairs, const float* __restrict__ logp,
                                                         const float* __restrict__ ref, float beta, int n_seg,
                                                         const int32_t* __restrict__ kept_of, float* __restrict__ w_kept,
                                                         float* __restrict__ stats) {
  __shared__ double sh[3][1024];
  const int tid = threadIdx.x;
  auto z_of = [&](int p) {
    const int c = pairs[2 * p], r = pairs[2 * p + 1];
    return (double)beta * (((double)logp[c] - (double)ref[c]) - ((double)logp[r] - (double)ref[r]));
  };
  const int per = (n_pairs + 1023) / 1024, b = min(n_pairs, tid * per), e = min(n_pairs, b + per);
  double l = 0.0, m = 0.0, a = 0.0;
  for (int p = b; p < e; p++) {
    const double z = z_of(p);
    l += z > 0 ? log1p(exp(-z)) : -z + log1p(exp(z));
    m += z; a += z > 0 ? 1.0 : 0.0;
  }
  sh[0][tid] = l; sh[1][tid] = m; sh[2][tid] = a;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (tid < off) for (int k = 0; k < 3; k++) sh[k][tid] += sh[k][tid + off];
    __syncthreads();
  }
  if (tid < 3) stats[tid] = n_pairs > 0 ? (float)(sh[tid][0] / (double)n_pairs) : 0.f;
  for (int s = tid; s < n_seg; s += 1024) {
    const int ks = kept_of ? kept_of[s] : s;
    if (ks < 0) continue;
    double w = 0.0;
    for (int p = 0; p < n_pairs; p++) {
      const int c = pairs[2 * p], r = pairs[2 * p + 1];
      if (c != s && r != s) continue;
      const double g = (double)beta / (1.0 + exp(z_of(p))) / (double)n_pairs;      // beta sigmoid(-z) / P
      if (c == s) w += g;
      if (r == s) w -= g;
    }
    w_kept[ks] = (float)w;
  }
}

// row_w[i] = w_kept[segment of target row i]
__global__ void dpo_row_weights_kernel(const int32_t* __restrict__ tgt_idx, const int32_t* __restrict__ count,
                                       const int32_t* __restrict__ cu, int n_kept, const float* __restrict__ w_kept,
                                       float* __restrict__ row_w) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= *count) return;
  const int t = tgt_idx[i];
  int lo = 0, hi = n_kept;                          // last k with cu[k] <= t
  while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (cu[mid] <= t) lo = mid; else hi = mid; }
  row_w[i] = w_kept[lo];
}

__global__ void fill_float_kernel(float* __restrict__ p, int n, float v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

int launch_seq_logp(as_ctx* ctx, const float* loss_rows, const int32_t* tgt_idx, const int32_t* count, const int32_t* cu,
                    const int32_t* kept_of, int n_seg, float* logp, hipStream_t st) {
  if (n_seg <= 0) return AS_OK;
  seq_logp_kernel<<<n_seg, 256, 0, st>>>(loss_rows, tgt_idx, count, cu, kept_of, logp);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_dpo_pairs(as_ctx* ctx, const int32_t* pairs, int n_pairs, const float* logp, const float* ref, float beta, int n_seg,
                     const int32_t* kept_of, int n_kept, float* w_kept, float* stats, hipStream_t st) {
  if (n_kept > 0) {
    fill_float_kernel<<<(n_kept + 255) / 256, 256, 0, st>>>(w_kept, n_kept, 0.f);
    AS_LAUNCH_CHECK(ctx);
  }
  dpo_pairs_kernel<<<1, 1024, 0, st>>>(pairs, n_pairs, logp, ref, beta, n_seg, kept_of, w_kept, stats);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_dpo_row_weights(as_ctx* ctx, const int32_t* tgt_idx, const int32_t* count, const int32_t* cu, int n_kept,
                           const float* w_kept, int n, float* row_w, hipStream_t st) {
  if (n <= 0) return AS_OK;
  dpo_row_weights_kernel<<<(n + 255) / 256, 256, 0, st>>>(tgt_idx, count, cu, n_kept, w_kept, row_w);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_fill_float(as_ctx* ctx, float* p, int n, float v, hipStream_t st) {
  if (n <= 0) return AS_OK;
  fill_float_kernel<<<(n + 255) / 256, 256, 0, st>>>(p, n, v);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}
