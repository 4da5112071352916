// Varlen causal attention with grouped KV heads over packed rows: a query at
// token t sees keys seg_start[t] .. t only, so nothing crosses a trajectory
// boundary.  Query head j reads KV head j / (Hq/Hkv).
//
// Plain kernels (any type; the fp32 tier): one wavefront per (token, head),
// scores of the whole visible range kept in LDS.
#include "common.h"

// --------------------------------------------------------------- plain fwd
template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_plain(AttnParams p, float scale) {
  extern __shared__ float sm[];
  float* qs = sm;                  // [dh]
  float* sc = sm + p.dh;           // [max_seg]
  const int t = blockIdx.x, j = blockIdx.y, lane = threadIdx.x, dh = p.dh;
  const int g = j / (p.Hq / p.Hkv);
  const int s0 = p.seg_start[t], len = t - s0 + 1;
  const T* q = (const T*)p.q + (int64_t)t * p.ldq + j * dh;
  const T* kb = (const T*)p.k + (int64_t)s0 * p.ldkv + g * dh;
  const T* vb = (const T*)p.v + (int64_t)s0 * p.ldkv + g * dh;
  for (int c = lane; c < dh; c += 64) qs[c] = to_f<T>(q[c]);
  __syncthreads();
  float mx = -INFINITY;
  for (int u = lane; u < len; u += 64) {
    const T* kr = kb + (int64_t)u * p.ldkv;
    float d = 0.f;
    for (int c = 0; c < dh; c++) d = fmaf(qs[c], to_f<T>(kr[c]), d);
    d *= scale;
    sc[u] = d;
    mx = fmaxf(mx, d);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int u = lane; u < len; u += 64) { float e = expf(sc[u] - mx); sc[u] = e; sum += e; }
  sum = wave_sum(sum);
  __syncthreads();
  T* o = (T*)p.o + ((int64_t)t * p.Hq + j) * dh;
  for (int c = lane; c < dh; c += 64) {
    float acc = 0.f;
    for (int u = 0; u < len; u++) acc = fmaf(sc[u], to_f<T>(vb[(int64_t)u * p.ldkv + c]), acc);
    o[c] = from_f<T>(acc / sum);
  }
  if (lane == 0) p.lse[(int64_t)t * p.Hq + j] = mx + logf(sum);
}

// --------------------------------------------------------------- plain bwd
// dq for one (token, head); also writes delta = sum_c dO*O for the dK/dV pass.
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dq_plain(AttnParams p, float scale) {
  extern __shared__ float sm[];
  float* qs = sm; float* dos = sm + p.dh; float* sc = sm + 2 * p.dh;
  const int t = blockIdx.x, j = blockIdx.y, lane = threadIdx.x, dh = p.dh;
  const int g = j / (p.Hq / p.Hkv);
  const int s0 = p.seg_start[t], len = t - s0 + 1;
  const T* q = (const T*)p.q + (int64_t)t * p.ldq + j * dh;
  const T* o = (const T*)p.o + ((int64_t)t * p.Hq + j) * dh;
  const T* d_o = (const T*)p.d_o + ((int64_t)t * p.Hq + j) * dh;
  const T* kb = (const T*)p.k + (int64_t)s0 * p.ldkv + g * dh;
  const T* vb = (const T*)p.v + (int64_t)s0 * p.ldkv + g * dh;
  float dl = 0.f;
  for (int c = lane; c < dh; c += 64) {
    float a = to_f<T>(d_o[c]);
    qs[c] = to_f<T>(q[c]); dos[c] = a;
    dl += a * to_f<T>(o[c]);
  }
  dl = wave_sum(dl);
  const float lse = p.lse[(int64_t)t * p.Hq + j];
  if (lane == 0) p.delta[(int64_t)t * p.Hq + j] = dl;
  __syncthreads();
  for (int u = lane; u < len; u += 64) {
    const T* kr = kb + (int64_t)u * p.ldkv; const T* vr = vb + (int64_t)u * p.ldkv;
    float d = 0.f, dp = 0.f;
    for (int c = 0; c < dh; c++) { d = fmaf(qs[c], to_f<T>(kr[c]), d); dp = fmaf(dos[c], to_f<T>(vr[c]), dp); }
    float pr = expf(d * scale - lse);
    sc[u] = pr * (dp - dl);
  }
  __syncthreads();
  T* dq = (T*)p.dq + (int64_t)t * p.ldq + j * dh;
  for (int c = lane; c < dh; c += 64) {
    float acc = 0.f;
    for (int u = 0; u < len; u++) acc = fmaf(sc[u], to_f<T>(kb[(int64_t)u * p.ldkv + c]), acc);
    dq[c] = from_f<T>(acc * scale);
  }
}

// dk, dv for one (token u, KV head): sums over the query heads of the group in
// head order and over later tokens of the segment in token order.
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_plain(AttnParams p, float scale) {
  extern __shared__ float sm[];
  float* ks = sm; float* vs = sm + p.dh; float* sp = sm + 2 * p.dh; float* sd = sp + p.max_seg;
  const int u = blockIdx.x, g = blockIdx.y, lane = threadIdx.x, dh = p.dh;
  const int grp = p.Hq / p.Hkv;
  const int e = p.seg_end[u], len = e - u;
  const T* k = (const T*)p.k + (int64_t)u * p.ldkv + g * dh;
  const T* v = (const T*)p.v + (int64_t)u * p.ldkv + g * dh;
  for (int c = lane; c < dh; c += 64) { ks[c] = to_f<T>(k[c]); vs[c] = to_f<T>(v[c]); }
  float dk0 = 0.f, dk1 = 0.f, dv0 = 0.f, dv1 = 0.f;     // dh <= 128: columns lane and lane + 64
  for (int jj = 0; jj < grp; jj++) {
    const int j = g * grp + jj;
    __syncthreads();
    for (int i = lane; i < len; i += 64) {
      const int t = u + i;
      const T* qr = (const T*)p.q + (int64_t)t * p.ldq + j * dh;
      const T* dor = (const T*)p.d_o + ((int64_t)t * p.Hq + j) * dh;
      float d = 0.f, dp = 0.f;
      for (int c = 0; c < dh; c++) { d = fmaf(to_f<T>(qr[c]), ks[c], d); dp = fmaf(to_f<T>(dor[c]), vs[c], dp); }
      float pr = expf(d * scale - p.lse[(int64_t)t * p.Hq + j]);
      sp[i] = pr;
      sd[i] = pr * (dp - p.delta[(int64_t)t * p.Hq + j]);
    }
    __syncthreads();
    for (int i = 0; i < len; i++) {
      const int t = u + i;
      const T* qr = (const T*)p.q + (int64_t)t * p.ldq + j * dh;
      const T* dor = (const T*)p.d_o + ((int64_t)t * p.Hq + j) * dh;
      float pi = sp[i], di = sd[i];
      if (lane < dh) { dv0 = fmaf(pi, to_f<T>(dor[lane]), dv0); dk0 = fmaf(di, to_f<T>(qr[lane]), dk0); }
      if (lane + 64 < dh) { dv1 = fmaf(pi, to_f<T>(dor[lane + 64]), dv1); dk1 = fmaf(di, to_f<T>(qr[lane + 64]), dk1); }
    }
  }
  T* dk = (T*)p.dk + (int64_t)u * p.ldkv + g * dh;
  T* dv = (T*)p.dv + (int64_t)u * p.ldkv + g * dh;
  if (lane < dh) { dk[lane] = from_f<T>(dk0 * scale); dv[lane] = from_f<T>(dv0); }
  if (lane + 64 < dh) { dk[lane + 64] = from_f<T>(dk1 * scale); dv[lane + 64] = from_f<T>(dv1); }
}

static int check_plain(as_ctx* ctx, const AttnParams& p, size_t smem) {
  if (p.dh > 128) return as_fail(ctx, AS_ERR_SHAPE, "attention: head_dim <= 128");
  if (smem > 160 * 1024) return as_fail(ctx, AS_ERR_SHAPE, "attention (plain kernels): segment too long for LDS");
  return AS_OK;
}

template <typename K>
static int set_smem(as_ctx* ctx, K kern, size_t smem) {
  if (smem > 48 * 1024)
    AS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
  return AS_OK;
}

int launch_attention_fwd_mfma(as_ctx* ctx, const AttnParams& p, int variant, hipStream_t st);
int launch_attention_bwd_mfma(as_ctx* ctx, const AttnParams& p, int variant, hipStream_t st);
bool attention_mfma_ok(const AttnParams& p);

int launch_attention_fwd(as_ctx* ctx, int mode, int variant, const AttnParams& p, hipStream_t st) {
  if (p.n <= 0) return AS_OK;
  bool mf = mode == AS_BF16 && variant != 1 && attention_mfma_ok(p);
  if (variant >= 2 && !mf) return as_fail(ctx, AS_ERR_SHAPE, "attention: MFMA kernel needs bf16, head_dim 64/128, aligned strides");
  if (mf) { prof_begin(ctx, st, AS_K_ATTN_FWD, 0.0); int r = launch_attention_fwd_mfma(ctx, p, variant, st); prof_end(ctx, st); return r; }
  size_t smem = (size_t)(p.dh + p.max_seg) * sizeof(float);
  int rc = check_plain(ctx, p, smem); if (rc) return rc;
  float scale = 1.f / sqrtf((float)p.dh);
  dim3 grid(p.n, p.Hq);
  if (mode == AS_FP32) { rc = set_smem(ctx, attn_fwd_plain<float>, smem); if (rc) return rc;
                         attn_fwd_plain<float><<<grid, 64, smem, st>>>(p, scale); }
  else { rc = set_smem(ctx, attn_fwd_plain<bf16_t>, smem); if (rc) return rc;
         attn_fwd_plain<bf16_t><<<grid, 64, smem, st>>>(p, scale); }
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

bool attention_bwd_is_mfma(int mode, int variant, const AttnParams& p) { return mode == AS_BF16 && variant != 1 && attention_mfma_ok(p); }

int launch_attention_bwd(as_ctx* ctx, int mode, int variant, const AttnParams& p, hipStream_t st) {
  if (p.n <= 0) return AS_OK;
  bool mf = mode == AS_BF16 && variant != 1 && attention_mfma_ok(p);
  if (!mf && p.rope_cos) return as_fail(ctx, AS_ERR_SHAPE, "attention: only the MFMA kernels rotate their gradients");
  if (variant >= 2 && !mf) return as_fail(ctx, AS_ERR_SHAPE, "attention: MFMA kernel needs bf16, head_dim 64/128, aligned strides");
  if (mf) { prof_begin(ctx, st, AS_K_ATTN_BWD, 0.0); int r = launch_attention_bwd_mfma(ctx, p, variant, st); prof_end(ctx, st); return r; }
  size_t smem1 = (size_t)(2 * p.dh + p.max_seg) * sizeof(float);
  size_t smem2 = (size_t)(2 * p.dh + 2 * p.max_seg) * sizeof(float);
  int rc = check_plain(ctx, p, smem2); if (rc) return rc;
  float scale = 1.f / sqrtf((float)p.dh);
  dim3 g1(p.n, p.Hq), g2(p.n, p.Hkv);
  if (mode == AS_FP32) {
    rc = set_smem(ctx, attn_bwd_dq_plain<float>, smem1); if (rc) return rc;
    rc = set_smem(ctx, attn_bwd_dkv_plain<float>, smem2); if (rc) return rc;
    attn_bwd_dq_plain<float><<<g1, 64, smem1, st>>>(p, scale);
    AS_LAUNCH_CHECK(ctx);
    attn_bwd_dkv_plain<float><<<g2, 64, smem2, st>>>(p, scale);
  } else {
    rc = set_smem(ctx, attn_bwd_dq_plain<bf16_t>, smem1); if (rc) return rc;
    rc = set_smem(ctx, attn_bwd_dkv_plain<bf16_t>, smem2); if (rc) return rc;
    attn_bwd_dq_plain<bf16_t><<<g1, 64, smem1, st>>>(p, scale);
    AS_LAUNCH_CHECK(ctx);
    attn_bwd_dkv_plain<bf16_t><<<g2, 64, smem2, st>>>(p, scale);
  }
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}
