// Mixture-of-experts plumbing around the grouped expert GEMMs (Mixtral-style layers, paper
// Section 4.1 model list): top-2 routing, the stable permutation that groups (token, slot) pairs by
// expert, gathers, the weighted combine and their backward counterparts.  All orders are fixed
// (token order inside an expert, slot 0 before slot 1), so results are reproducible bit for bit.
#include "common.h"

#define DISPATCH_T(mode, ...) do { if ((mode) == AS_FP32) { typedef float T; __VA_ARGS__; } \
  else { typedef bf16_t T; __VA_ARGS__; } } while (0)

// The two largest router logits of each token (ties go to the lower expert index) and the softmax
// over those two.  One thread per token; logits are float.
__global__ void moe_route_kernel(const float* __restrict__ logit, int n, int E, int32_t* __restrict__ sel,
                                 float* __restrict__ w) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  const float* l = logit + (int64_t)t * E;
  int i0 = 0; float v0 = l[0];
  for (int e = 1; e < E; e++) if (l[e] > v0) { v0 = l[e]; i0 = e; }
  int i1 = -1; float v1 = -INFINITY;
  for (int e = 0; e < E; e++) if (e != i0 && l[e] > v1) { v1 = l[e]; i1 = e; }
  float e1 = expf(v1 - v0);                       // v0 >= v1
  float inv = 1.f / (1.f + e1);
  sel[2 * t] = i0; sel[2 * t + 1] = i1;
  w[2 * t] = inv; w[2 * t + 1] = e1 * inv;
}

// Stable counting sort of the 2n (token, slot) pairs by expert, done by one workgroup: thread i owns
// a contiguous slab of tokens, per-expert counts are scanned across threads in LDS.
// eoff[e] = first permuted row of expert e, pos[2t+s] = permuted row of the pair, perm = inverse.
__global__ __launch_bounds__(1024) void moe_permute_kernel(const int32_t* __restrict__ sel, int n, int E,
                                                           int32_t* __restrict__ eoff, int32_t* __restrict__ pos,
                                                           int32_t* __restrict__ perm) {
  extern __shared__ int32_t cnt[];                // [E][1024], then [E+1] expert bases
  int32_t* ebase = cnt + E * 1024;
  const int tid = threadIdx.x;
  const int per = (n + 1023) / 1024, b = min(n, tid * per), e_ = min(n, b + per);
  for (int e = 0; e < E; e++) cnt[e * 1024 + tid] = 0;
  for (int t = b; t < e_; t++) { cnt[sel[2 * t] * 1024 + tid]++; cnt[sel[2 * t + 1] * 1024 + tid]++; }
  __syncthreads();
  for (int e = 0; e < E; e++) {                   // exclusive scan over threads, expert by expert
    int32_t* c = cnt + e * 1024;
    int mine = c[tid];
    for (int off = 1; off < 1024; off <<= 1) {
      int v = tid >= off ? c[tid - off] : 0;
      __syncthreads();
      c[tid] += v;
      __syncthreads();
    }
    int incl = c[tid];
    __syncthreads();
    c[tid] = incl - mine;
    if (tid == 1023) ebase[e + 1] = incl;          // total of expert e (for now)
    __syncthreads();
  }
  if (tid == 0) {
    ebase[0] = 0;
    for (int e = 0; e < E; e++) ebase[e + 1] += ebase[e];
    for (int e = 0; e <= E; e++) eoff[e] = ebase[e];
  }
  __syncthreads();
  for (int t = b; t < e_; t++)
    for (int s = 0; s < 2; s++) {
      const int e = sel[2 * t + s];
      const int p = ebase[e] + cnt[e * 1024 + tid]++;
      pos[2 * t + s] = p;
      perm[p] = 2 * t + s;
    }
}

// out[i] = (w ? w[perm[i]] : 1) * src[perm[i] / 2]     (rows of d elements)
template <typename T>
__global__ void moe_gather_kernel(const T* __restrict__ src, const int32_t* __restrict__ perm, const float* __restrict__ w,
                                  int rows, int d, T* __restrict__ out) {
  const int i = blockIdx.x;
  if (i >= rows) return;
  const int pr = perm[i];
  const float sc = w ? w[pr] : 1.f;
  const T* s = src + (int64_t)(pr >> 1) * d;
  T* o = out + (int64_t)i * d;
  for (int j = threadIdx.x; j < d; j += blockDim.x) o[j] = w ? from_f<T>(sc * to_f<T>(s[j])) : s[j];
}

// out[t] = res[t] + w[2t] y[pos[2t]] + w[2t+1] y[pos[2t+1]]
template <typename T>
__global__ void moe_combine_kernel(const T* __restrict__ res, const T* __restrict__ y, const int32_t* __restrict__ pos,
                                   const float* __restrict__ w, int n, int d, T* __restrict__ out) {
  const int t = blockIdx.x;
  if (t >= n) return;
  const T* y0 = y + (int64_t)pos[2 * t] * d; const T* y1 = y + (int64_t)pos[2 * t + 1] * d;
  const float w0 = w ? w[2 * t] : 1.f, w1 = w ? w[2 * t + 1] : 1.f;
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    float v = res ? to_f<T>(res[(int64_t)t * d + j]) : 0.f;
    v += w0 * to_f<T>(y0[j]);
    v += w1 * to_f<T>(y1[j]);
    out[(int64_t)t * d + j] = from_f<T>(v);
  }
}

// Gradient of the routing weights and of the router logits: dw_s = <dy[t], y[pos_s]>,
// dl_s = w_s (dw_s - sum_s' w_s' dw_s'); dlogit[t, :] is zero except at the two selected experts.
template <typename T>
__global__ void moe_dlogit_kernel(const T* __restrict__ dy, const T* __restrict__ y, const int32_t* __restrict__ pos,
                                  const int32_t* __restrict__ sel, const float* __restrict__ w, int n, int d, int Epad,
                                  T* __restrict__ dlogit) {
  const int t = blockIdx.x * (blockDim.x / AS_WAVE) + threadIdx.x / AS_WAVE, lane = threadIdx.x % AS_WAVE;
  if (t >= n) return;
  const T* g = dy + (int64_t)t * d;
  const T* y0 = y + (int64_t)pos[2 * t] * d; const T* y1 = y + (int64_t)pos[2 * t + 1] * d;
  float a0 = 0.f, a1 = 0.f;
  for (int j = lane; j < d; j += AS_WAVE) { float gj = to_f<T>(g[j]); a0 += gj * to_f<T>(y0[j]); a1 += gj * to_f<T>(y1[j]); }
  a0 = wave_sum(a0); a1 = wave_sum(a1);
  const float w0 = w[2 * t], w1 = w[2 * t + 1], mean = w0 * a0 + w1 * a1;
  const int s0 = sel[2 * t], s1 = sel[2 * t + 1];
  for (int e = lane; e < Epad; e += AS_WAVE)
    dlogit[(int64_t)t * Epad + e] = from_f<T>(e == s0 ? w0 * (a0 - mean) : e == s1 ? w1 * (a1 - mean) : 0.f);
}

int launch_moe_route(as_ctx* ctx, const float* logit, int n, int E, int32_t* sel, float* w, hipStream_t st) {
  if (n <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_MOE, 0.0);
  moe_route_kernel<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(logit, n, E, sel, w);
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_moe_permute(as_ctx* ctx, const int32_t* sel, int n, int E, int32_t* eoff, int32_t* pos, int32_t* perm, hipStream_t st) {
  size_t smem = ((size_t)E * 1024 + E + 1) * sizeof(int32_t);
  if (smem > 160 * 1024) return as_fail(ctx, AS_ERR_SHAPE, "moe: too many experts for the permutation kernel");
  if (smem > 48 * 1024)
    AS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(moe_permute_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
  prof_begin(ctx, st, AS_K_MOE, 0.0);
  moe_permute_kernel<<<1, 1024, smem, st>>>(sel, n, E, eoff, pos, perm);
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_moe_gather(as_ctx* ctx, int mode, const void* src, const int32_t* perm, const float* w, int rows, int d, void* out, hipStream_t st) {
  if (rows <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_MOE, 0.0);
  DISPATCH_T(mode, (moe_gather_kernel<T><<<rows, 256, 0, st>>>((const T*)src, perm, w, rows, d, (T*)out)));
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_moe_combine(as_ctx* ctx, int mode, const void* res, const void* y, const int32_t* pos, const float* w, int n, int d,
                       void* out, hipStream_t st) {
  if (n <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_MOE, 0.0);
  DISPATCH_T(mode, (moe_combine_kernel<T><<<n, 256, 0, st>>>((const T*)res, (const T*)y, pos, w, n, d, (T*)out)));
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_moe_dlogit(as_ctx* ctx, int mode, const void* dy, const void* y, const int32_t* pos, const int32_t* sel, const float* w,
                      int n, int d, int Epad, void* dlogit, hipStream_t st) {
  if (n <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_MOE, 0.0);
  DISPATCH_T(mode, (moe_dlogit_kernel<T><<<(unsigned)cdiv(n, 4), 256, 0, st>>>((const T*)dy, (const T*)y, pos, sel, w, n, d, Epad, (T*)dlogit)));
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}
