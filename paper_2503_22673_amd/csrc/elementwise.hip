// HBM-bound kernels of the fine-tuning step: packing, embedding gather,
// RMSNorm, RoPE, SwiGLU, transposes, LoRA operand preparation, target
// selection, the cross-entropy row pass, reductions and AdamW.
// One wavefront (64 lanes) owns one token row wherever a row reduction is
// needed, so reductions are shuffles only; rows are read with 16-byte loads.
#include "common.h"

#define DISPATCH_T(mode, ...) do { if ((mode) == AS_FP32) { typedef float T; __VA_ARGS__; } \
  else { typedef bf16_t T; __VA_ARGS__; } } while (0)

template <typename T> struct Vec;
template <> struct Vec<float> { static constexpr int N = 4; typedef f32x4 type; };
template <> struct Vec<bf16_t> { static constexpr int N = 8; typedef bf16x8 type; };

template <typename T> __device__ __forceinline__ void load_vec(const T* p, float* out) {
  typename Vec<T>::type v = *reinterpret_cast<const typename Vec<T>::type*>(p);
#pragma unroll
  for (int i = 0; i < Vec<T>::N; i++) out[i] = to_f<T>(v[i]);
}
template <typename T> __device__ __forceinline__ void store_vec(T* p, const float* in) {
  typename Vec<T>::type v;
#pragma unroll
  for (int i = 0; i < Vec<T>::N; i++) v[i] = from_f<T>(in[i]);
  *reinterpret_cast<typename Vec<T>::type*>(p) = v;
}
template <typename T> static bool vec_ok(const void* p, int64_t ld) {
  return ((uintptr_t)p % 16 == 0) && (ld % Vec<T>::N == 0);
}

// ------------------------------------------------------------------ pack
// The host has cut the batch into pieces (a kept part of a turn, or a pad
// tail); piece_dst holds their start offsets in the output, ascending.
__global__ void pack_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ piece_dst,
                            const int32_t* __restrict__ piece_src, const uint8_t* __restrict__ piece_mask,
                            int n_pieces, int n_out, int pad_id, int32_t* __restrict__ tok,
                            uint8_t* __restrict__ mask) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_out) return;
  int lo = 0, hi = n_pieces - 1;            // last piece with piece_dst[p] <= t
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (piece_dst[mid] <= t) lo = mid; else hi = mid - 1;
  }
  int s = piece_src[lo];
  tok[t] = s < 0 ? pad_id : src[s + (t - piece_dst[lo])];
  mask[t] = piece_mask[lo];
}

int launch_pack(as_ctx* ctx, const int32_t* d_src_tokens, const int32_t* d_piece_dst,
                const int32_t* d_piece_src, const uint8_t* d_piece_mask, int n_pieces, int n_out,
                int pad_id, int32_t* d_tokens, uint8_t* d_mask, hipStream_t st) {
  if (n_out <= 0) return AS_OK;
  pack_kernel<<<cdiv(n_out, 256), 256, 0, st>>>(d_src_tokens, d_piece_dst, d_piece_src, d_piece_mask,
                                                n_pieces, n_out, pad_id, d_tokens, d_mask);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

__global__ void compact_kernel(const int32_t* __restrict__ tok, const uint8_t* __restrict__ mask,
                               const int32_t* __restrict__ cu_c, const int32_t* __restrict__ src_start, int n_seg, int n,
                               int32_t* __restrict__ tok_c, uint8_t* __restrict__ mask_c) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int lo = 0, hi = n_seg - 1;               // last s with cu_c[s] <= i
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (cu_c[mid] <= i) lo = mid; else hi = mid - 1;
  }
  int src = src_start[lo] + (i - cu_c[lo]);
  tok_c[i] = tok[src];
  mask_c[i] = mask[src];
}

int launch_compact(as_ctx* ctx, const int32_t* tok, const uint8_t* mask, const int32_t* cu_c, const int32_t* src_start,
                   int n_seg, int n, int32_t* tok_c, uint8_t* mask_c, hipStream_t st) {
  if (n <= 0) return AS_OK;
  compact_kernel<<<cdiv(n, 256), 256, 0, st>>>(tok, mask, cu_c, src_start, n_seg, n, tok_c, mask_c);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

__global__ void segment_info_kernel(const int32_t* __restrict__ cu, int n_seg, int n,
                                    int32_t* __restrict__ seg_start, int32_t* __restrict__ seg_end) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  int lo = 0, hi = n_seg - 1;               // last s with cu[s] <= t
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid - 1;
  }
  seg_start[t] = cu[lo];
  seg_end[t] = cu[lo + 1];
}

int launch_segment_info(as_ctx* ctx, const int32_t* d_cu, int n_seg, int n, int32_t* seg_start,
                        int32_t* seg_end, hipStream_t st) {
  if (n <= 0) return AS_OK;
  segment_info_kernel<<<cdiv(n, 256), 256, 0, st>>>(d_cu, n_seg, n, seg_start, seg_end);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ------------------------------------------------------------------ RoPE
// cos/sin of p * base^(-2i/dh), evaluated in double and rounded once.
__global__ void rope_table_kernel(int max_pos, int half, int dh, double base, float* __restrict__ cosb,
                                  float* __restrict__ sinb) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= max_pos * half) return;
  int p = idx / half, i = idx % half;
  double theta = pow(base, -2.0 * (double)i / (double)dh);
  double s, c;
  sincos((double)p * theta, &s, &c);
  cosb[idx] = (float)c;
  sinb[idx] = (float)s;
}

int launch_rope_table(as_ctx* ctx, int max_pos, int dh, float base, float* cosb, float* sinb, hipStream_t st) {
  int half = dh / 2;
  int64_t tot = (int64_t)max_pos * half;
  if (tot <= 0) return AS_OK;
  rope_table_kernel<<<cdiv(tot, 256), 256, 0, st>>>(max_pos, half, dh, (double)base, cosb, sinb);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// Rotates pairs (i, i + dh/2) of every head in place; the position of token t
// is t - seg_start[t].  One thread per (token, head, 2 adjacent i).
template <typename T>
__global__ void rope_kernel(int n, int n_heads, int dh, T* __restrict__ x, int64_t ldx,
                            const int32_t* __restrict__ seg_start, const float* __restrict__ cosb,
                            const float* __restrict__ sinb, float sign) {
  int half = dh >> 1;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t tot = (int64_t)n * n_heads * half;
  if (idx >= tot) return;
  int i = idx % half;
  int64_t r = idx / half;
  int hd = r % n_heads;
  int t = r / n_heads;
  int p = t - seg_start[t];
  float c = cosb[(int64_t)p * half + i], s = sign * sinb[(int64_t)p * half + i];
  T* row = x + (int64_t)t * ldx + (int64_t)hd * dh;
  float x1 = to_f<T>(row[i]), x2 = to_f<T>(row[i + half]);
  row[i] = from_f<T>(x1 * c - x2 * s);
  row[i + half] = from_f<T>(x1 * s + x2 * c);
}

// Same rotation, one thread per (token, head, Vec<T>::N adjacent i): 16-byte loads and stores.
template <typename T>
__global__ void rope_vec_kernel(int n, int n_heads, int dh, T* __restrict__ x, int64_t ldx,
                                const int32_t* __restrict__ seg_start, const float* __restrict__ cosb,
                                const float* __restrict__ sinb, float sign) {
  constexpr int VN = Vec<T>::N;
  const int half = dh >> 1, per = half / VN;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)n * n_heads * per) return;
  const int i = (int)(idx % per) * VN;
  const int64_t r = idx / per;
  const int hd = (int)(r % n_heads), t = (int)(r / n_heads);
  const int p = t - seg_start[t];
  T* row = x + (int64_t)t * ldx + (int64_t)hd * dh;
  float x1[VN], x2[VN], o1[VN], o2[VN];
  load_vec<T>(row + i, x1); load_vec<T>(row + i + half, x2);
#pragma unroll
  for (int k = 0; k < VN; k += 4) {
    const f32x4 c = *reinterpret_cast<const f32x4*>(cosb + (int64_t)p * half + i + k);
    const f32x4 s = *reinterpret_cast<const f32x4*>(sinb + (int64_t)p * half + i + k);
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const float sq = sign * s[q];
      o1[k + q] = x1[k + q] * c[q] - x2[k + q] * sq;
      o2[k + q] = x1[k + q] * sq + x2[k + q] * c[q];
    }
  }
  store_vec<T>(row + i, o1); store_vec<T>(row + i + half, o2);
}

int launch_rope(as_ctx* ctx, int mode, int n, int n_heads, int dh, void* x, int64_t ldx,
                const int32_t* seg_start, const float* cosb, const float* sinb, int inverse, hipStream_t st) {
  int64_t tot = (int64_t)n * n_heads * (dh / 2);
  if (tot <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_ROPE, 0.0);
  DISPATCH_T(mode, {
    constexpr int VN = Vec<T>::N;
    if ((dh / 2) % VN == 0 && vec_ok<T>(x, ldx) && ((uintptr_t)cosb % 16) == 0 && ((uintptr_t)sinb % 16) == 0)
      rope_vec_kernel<T><<<cdiv(tot / VN, 256), 256, 0, st>>>(n, n_heads, dh, (T*)x, ldx, seg_start, cosb, sinb, inverse ? -1.f : 1.f);
    else
      rope_kernel<T><<<cdiv(tot, 256), 256, 0, st>>>(n, n_heads, dh, (T*)x, ldx, seg_start, cosb, sinb, inverse ? -1.f : 1.f); });
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// --------------------------------------------------------------- embedding
template <typename T>
__global__ void embed_kernel(const int32_t* __restrict__ tok, int n, int d, const T* __restrict__ E,
                             T* __restrict__ h, int vec) {
  int t = blockIdx.x;
  const T* src = E + (int64_t)tok[t] * d;
  T* dst = h + (int64_t)t * d;
  if (vec) {
    constexpr int VN = Vec<T>::N;
    for (int j = threadIdx.x * VN; j < d; j += blockDim.x * VN)
      *reinterpret_cast<typename Vec<T>::type*>(dst + j) = *reinterpret_cast<const typename Vec<T>::type*>(src + j);
  } else {
    for (int j = threadIdx.x; j < d; j += blockDim.x) dst[j] = src[j];
  }
}

int launch_embed(as_ctx* ctx, int mode, const int32_t* tok, int n, int d, const void* E, void* h, hipStream_t st) {
  if (n <= 0) return AS_OK;
  DISPATCH_T(mode, { int vec = vec_ok<T>(E, d) && vec_ok<T>(h, d);
                     embed_kernel<T><<<n, 256, 0, st>>>(tok, n, d, (const T*)E, (T*)h, vec); });
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ----------------------------------------------------------------- RMSNorm
// One wavefront per row, four rows per block.
template <typename T>
__global__ void rmsnorm_fwd_kernel(int n, int d, const T* __restrict__ x, const int32_t* __restrict__ row_idx,
                                   const int* __restrict__ n_dev, const T* __restrict__ g, float eps,
                                   T* __restrict__ y, float* __restrict__ rstd, int vec) {
  int row = blockIdx.x * (blockDim.x / AS_WAVE) + threadIdx.x / AS_WAVE;
  int lane = threadIdx.x % AS_WAVE;
  int nn = n_dev ? min(n, *n_dev) : n;
  if (row >= nn) return;
  const T* xr = x + (int64_t)(row_idx ? row_idx[row] : row) * d;
  T* yr = y + (int64_t)row * d;
  constexpr int VN = Vec<T>::N, KEEP = 8, STEP = AS_WAVE * VN;
  typedef typename Vec<T>::type VT;
  VT kept[KEEP];                         // the first KEEP 16-byte pieces of the row stay in registers for the second pass (bf16: 4096 columns)
  float ss = 0.f;
  if (vec) {
#pragma unroll
    for (int c = 0; c < KEEP; c++) {
      const int j = c * STEP + lane * VN;
      if (j < d) {
        kept[c] = *reinterpret_cast<const VT*>(xr + j);
#pragma unroll
        for (int i = 0; i < VN; i++) { const float v = to_f<T>(kept[c][i]); ss += v * v; }
      }
    }
    for (int j = KEEP * STEP + lane * VN; j < d; j += STEP) {
      float v[VN]; load_vec<T>(xr + j, v);
#pragma unroll
      for (int i = 0; i < VN; i++) ss += v[i] * v[i];
    }
  } else {
    for (int j = lane; j < d; j += AS_WAVE) { float v = to_f<T>(xr[j]); ss += v * v; }
  }
  ss = wave_sum(ss);
  float r = rsqrtf(ss / (float)d + eps);
  // one Newton step: rsqrtf is an approximation, the fp32 tier needs ~1e-7
  { float a = ss / (float)d + eps; r = r * (1.5f - 0.5f * a * r * r); }
  if (lane == 0) rstd[row] = r;
  if (vec) {
#pragma unroll
    for (int c = 0; c < KEEP; c++) {
      const int j = c * STEP + lane * VN;
      if (j < d) {
        float v[VN], gg[VN]; load_vec<T>(g + j, gg);
#pragma unroll
        for (int i = 0; i < VN; i++) v[i] = to_f<T>(kept[c][i]) * r * gg[i];
        store_vec<T>(yr + j, v);
      }
    }
    for (int j = KEEP * STEP + lane * VN; j < d; j += STEP) {
      float v[VN], gg[VN]; load_vec<T>(xr + j, v); load_vec<T>(g + j, gg);
#pragma unroll
      for (int i = 0; i < VN; i++) v[i] = v[i] * r * gg[i];
      store_vec<T>(yr + j, v);
    }
  } else {
    for (int j = lane; j < d; j += AS_WAVE) yr[j] = from_f<T>(to_f<T>(xr[j]) * r * to_f<T>(g[j]));
  }
}

int launch_rmsnorm_fwd(as_ctx* ctx, int mode, int n, int d, const void* x, const int32_t* row_idx,
                       const int* n_dev, const void* g, float eps, void* y, float* rstd, hipStream_t st) {
  if (n <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_NORM, 0.0);
  DISPATCH_T(mode, { int vec = vec_ok<T>(x, d) && vec_ok<T>(y, d) && vec_ok<T>(g, d);
                     rmsnorm_fwd_kernel<T><<<cdiv(n, 4), 256, 0, st>>>(n, d, (const T*)x, row_idx, n_dev,
                                                                       (const T*)g, eps, (T*)y, rstd, vec); });
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

template <typename T>
__global__ void rmsnorm_bwd_kernel(int n, int d, const T* __restrict__ dy, const int32_t* __restrict__ src_pos,
                                   const T* __restrict__ x, const T* __restrict__ g,
                                   const float* __restrict__ rstd, const T* __restrict__ add,
                                   T* __restrict__ dx, int vec) {
  int row = blockIdx.x * (blockDim.x / AS_WAVE) + threadIdx.x / AS_WAVE;
  int lane = threadIdx.x % AS_WAVE;
  if (row >= n) return;
  constexpr int VN = Vec<T>::N;
  int64_t src = src_pos ? src_pos[row] : row;
  T* dxr = dx + (int64_t)row * d;
  const T* ar = add ? add + (int64_t)row * d : nullptr;
  if (src < 0) {                         // no upstream gradient for this row
    for (int j = lane; j < d; j += AS_WAVE) dxr[j] = ar ? ar[j] : from_f<T>(0.f);
    return;
  }
  const T* dyr = dy + src * d;
  const T* xr = x + (int64_t)row * d;
  float r = rstd[src_pos ? src : row];
  float dot = 0.f;
  constexpr int KEEP = 8, STEP = AS_WAVE * VN;
  typedef typename Vec<T>::type VT;
  VT kdy[KEEP], kx[KEEP];                // the first KEEP 16-byte pieces of both rows stay in registers for the second pass
  if (vec) {
#pragma unroll
    for (int q = 0; q < KEEP; q++) {
      const int j = q * STEP + lane * VN;
      if (j < d) {
        kdy[q] = *reinterpret_cast<const VT*>(dyr + j); kx[q] = *reinterpret_cast<const VT*>(xr + j);
        float c[VN]; load_vec<T>(g + j, c);
#pragma unroll
        for (int i = 0; i < VN; i++) dot += to_f<T>(kdy[q][i]) * to_f<T>(kx[q][i]) * c[i];
      }
    }
    for (int j = KEEP * STEP + lane * VN; j < d; j += STEP) {
      float a[VN], b[VN], c[VN]; load_vec<T>(dyr + j, a); load_vec<T>(xr + j, b); load_vec<T>(g + j, c);
#pragma unroll
      for (int i = 0; i < VN; i++) dot += a[i] * b[i] * c[i];
    }
  } else {
    for (int j = lane; j < d; j += AS_WAVE) dot += to_f<T>(dyr[j]) * to_f<T>(xr[j]) * to_f<T>(g[j]);
  }
  dot = wave_sum(dot);
  float k = r * r * r * dot / (float)d;
  if (vec) {
#pragma unroll
    for (int q = 0; q < KEEP; q++) {
      const int j = q * STEP + lane * VN;
      if (j < d) {
        float c[VN], o[VN]; load_vec<T>(g + j, c);
        if (ar) load_vec<T>(ar + j, o);
#pragma unroll
        for (int i = 0; i < VN; i++) o[i] = (ar ? o[i] : 0.f) + (r * c[i] * to_f<T>(kdy[q][i]) - to_f<T>(kx[q][i]) * k);
        store_vec<T>(dxr + j, o);
      }
    }
    for (int j = KEEP * STEP + lane * VN; j < d; j += STEP) {
      float a[VN], b[VN], c[VN], o[VN]; load_vec<T>(dyr + j, a); load_vec<T>(xr + j, b); load_vec<T>(g + j, c);
      if (ar) load_vec<T>(ar + j, o);
#pragma unroll
      for (int i = 0; i < VN; i++) o[i] = (ar ? o[i] : 0.f) + (r * c[i] * a[i] - b[i] * k);
      store_vec<T>(dxr + j, o);
    }
  } else {
    for (int j = lane; j < d; j += AS_WAVE) {
      float v = r * to_f<T>(g[j]) * to_f<T>(dyr[j]) - to_f<T>(xr[j]) * k;
      dxr[j] = from_f<T>((ar ? to_f<T>(ar[j]) : 0.f) + v);
    }
  }
}

int launch_rmsnorm_bwd(as_ctx* ctx, int mode, int n, int d, const void* dy, const int32_t* src_pos,
                       const void* x, const void* g, const float* rstd, const void* add, void* dx,
                       hipStream_t st) {
  if (n <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_NORM, 0.0);
  DISPATCH_T(mode, { int vec = vec_ok<T>(dy, d) && vec_ok<T>(x, d) && vec_ok<T>(g, d) && vec_ok<T>(dx, d) &&
                               (!add || vec_ok<T>(add, d));
                     rmsnorm_bwd_kernel<T><<<cdiv(n, 4), 256, 0, st>>>(n, d, (const T*)dy, src_pos, (const T*)x,
                         (const T*)g, rstd, (const T*)add, (T*)dx, vec); });
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// Gain gradient dg_j = sum_t dy[t,j] x[t,j] rstd[t]: each block sums a slab of
// rows into partial[block, :], a second pass adds the slabs in block order.
template <typename T>
__global__ void rmsnorm_dgain_part(int n, int d, const T* __restrict__ dy, const int32_t* __restrict__ src_pos,
                                   const T* __restrict__ x, const float* __restrict__ rstd,
                                   float* __restrict__ partial, int rows_per) {
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  int r0 = blockIdx.y * rows_per, r1 = min(n, r0 + rows_per);
  float acc = 0.f;
  for (int t = r0; t < r1; t++) {
    int64_t src = src_pos ? src_pos[t] : t;
    if (src < 0) continue;
    acc += to_f<T>(dy[src * d + j]) * to_f<T>(x[(int64_t)t * d + j]) * rstd[src_pos ? src : t];
  }
  partial[(int64_t)blockIdx.y * d + j] = acc;
}
__global__ void sum_partials_kernel(const float* __restrict__ partial, int n_part, int64_t len,
                                    float alpha, float* __restrict__ out) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= len) return;
  float acc = 0.f;
  for (int p = 0; p < n_part; p++) acc += partial[(int64_t)p * len + j];
  out[j] = alpha * acc;
}

int launch_rmsnorm_dgain(as_ctx* ctx, int mode, int n, int d, const void* dy, const int32_t* src_pos,
                         const void* x, const float* rstd, float* partial, int n_part, float* dg,
                         hipStream_t st) {
  if (n <= 0 || n_part <= 0) return AS_OK;
  int rows_per = (int)cdiv(n, n_part);
  dim3 grid(cdiv(d, 256), n_part);
  DISPATCH_T(mode, (rmsnorm_dgain_part<T><<<grid, 256, 0, st>>>(n, d, (const T*)dy, src_pos, (const T*)x, rstd,
                                                                 partial, rows_per)));
  AS_LAUNCH_CHECK(ctx);
  sum_partials_kernel<<<cdiv(d, 256), 256, 0, st>>>(partial, n_part, d, 1.f, dg);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ------------------------------------------------------------------ SwiGLU
// gu holds [gate | up] side by side, row length 2F.
template <typename T>
__global__ void swiglu_fwd_kernel(int64_t n, int F, const T* __restrict__ gu, T* __restrict__ m, int vec) {
  constexpr int VN = Vec<T>::N;
  int64_t per_row = vec ? F / VN : F;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n * per_row) return;
  int64_t t = idx / per_row; int j = (idx % per_row) * (vec ? VN : 1);
  const T* gr = gu + t * 2 * F;
  if (vec) {
    float a[VN], b[VN], o[VN]; load_vec<T>(gr + j, a); load_vec<T>(gr + F + j, b);
#pragma unroll
    for (int i = 0; i < VN; i++) o[i] = a[i] / (1.f + __expf(-a[i])) * b[i];
    store_vec<T>(m + t * F + j, o);
  } else {
    float a = to_f<T>(gr[j]), b = to_f<T>(gr[F + j]);
    m[t * F + j] = from_f<T>(a / (1.f + __expf(-a)) * b);
  }
}

template <typename T>
__global__ void swiglu_bwd_kernel(int64_t n, int F, const T* __restrict__ dm, const T* __restrict__ gu,
                                  T* __restrict__ dgu, T* __restrict__ m_out, int vec) {
  constexpr int VN = Vec<T>::N;
  int64_t per_row = vec ? F / VN : F;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n * per_row) return;
  int64_t t = idx / per_row; int j = (idx % per_row) * (vec ? VN : 1);
  const T* gr = gu + t * 2 * F;
  T* dr = dgu + t * 2 * F;
  if (vec) {
    float a[VN], b[VN], c[VN], og[VN], ou[VN];
    load_vec<T>(gr + j, a); load_vec<T>(gr + F + j, b); load_vec<T>(dm + t * F + j, c);
#pragma unroll
    for (int i = 0; i < VN; i++) {
      float sg = 1.f / (1.f + __expf(-a[i]));
      og[i] = c[i] * b[i] * sg * (1.f + a[i] * (1.f - sg));
      ou[i] = c[i] * a[i] * sg;
    }
    store_vec<T>(dr + j, og); store_vec<T>(dr + F + j, ou);
    if (m_out) {                                       // the forward product again, in the forward kernel's arithmetic
      float o[VN];
#pragma unroll
      for (int i = 0; i < VN; i++) o[i] = a[i] / (1.f + __expf(-a[i])) * b[i];
      store_vec<T>(m_out + t * F + j, o);
    }
  } else {
    float a = to_f<T>(gr[j]), b = to_f<T>(gr[F + j]), c = to_f<T>(dm[t * F + j]);
    float sg = 1.f / (1.f + __expf(-a));
    dr[j] = from_f<T>(c * b * sg * (1.f + a * (1.f - sg)));
    dr[F + j] = from_f<T>(c * a * sg);
    if (m_out) m_out[t * F + j] = from_f<T>(a / (1.f + __expf(-a)) * b);
  }
}

int launch_swiglu_fwd(as_ctx* ctx, int mode, int64_t n, int F, const void* gu, void* m, hipStream_t st) {
  if (n <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_SWIGLU, 0.0);
  DISPATCH_T(mode, { int vec = vec_ok<T>(gu, F) && vec_ok<T>(m, F);
                     int64_t tot = n * (vec ? F / Vec<T>::N : F);
                     swiglu_fwd_kernel<T><<<cdiv(tot, 256), 256, 0, st>>>(n, F, (const T*)gu, (T*)m, vec); });
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}
// m_out (may be NULL): also writes silu(gate) * up, bit for bit what launch_swiglu_fwd writes
int launch_swiglu_bwd(as_ctx* ctx, int mode, int64_t n, int F, const void* dm, const void* gu, void* dgu, void* m_out, hipStream_t st) {
  if (n <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_SWIGLU, 0.0);
  DISPATCH_T(mode, { int vec = vec_ok<T>(gu, F) && vec_ok<T>(dm, F) && vec_ok<T>(dgu, F) && (!m_out || vec_ok<T>(m_out, F));
                     int64_t tot = n * (vec ? F / Vec<T>::N : F);
                     swiglu_bwd_kernel<T><<<cdiv(tot, 256), 256, 0, st>>>(n, F, (const T*)dm, (const T*)gu, (T*)dgu, (T*)m_out, vec); });
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// --------------------------------------------------------------- transpose
// out[c, r] = in[r, c] through a padded 64x64 LDS tile; rows past the
// device-side row count (if given) read as zero.
// QS: inside every group of 16 output positions the two middle quads are exchanged (position order
// 0-3, 8-11, 4-7, 12-15 of the source rows), which is the order one lane half of a 32x32x16 MFMA
// holds its 8 contraction indices in: such a fragment is then one 16-byte read.
template <typename T, bool QS>
__global__ void transpose_kernel(int rows, int rows_pad, int cols, const T* __restrict__ in, int64_t ldi,
                                 T* __restrict__ out, int64_t ldo, const int* __restrict__ rows_dev, int row_off) {
  __shared__ T tile[64][65];
  int live = rows_dev ? min(rows, *rows_dev - row_off) : rows;
  int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  int tx = threadIdx.x % 64, ty = threadIdx.x / 64;       // 256 threads: 4 rows at a time
  for (int i = ty; i < 64; i += 4) {
    int r = r0 + i, c = c0 + tx;
    tile[i][tx] = (r < live && c < cols) ? in[(int64_t)r * ldi + c] : from_f<T>(0.f);
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    int c = c0 + i, r = r0 + tx;
    const int src = QS ? ((tx & ~12) | ((tx & 4) << 1) | ((tx & 8) >> 1)) : tx;
    if (c < cols && r < rows_pad) out[(int64_t)c * ldo + r] = tile[src][i];
  }
}

// bf16, 16-byte accesses on both sides: a 64x64 tile is read as 8-element row chunks and written as
// 8-element chunks of the output rows (gathered from an LDS tile column).  Needs cols, ldi, ldo, rows_pad
// multiples of 8 (rows_pad of 64 in fact: whole output chunks) and 16-byte aligned bases.
template <bool QS>
__global__ void transpose_vec_kernel(int rows, int rows_pad, int cols, const bf16_t* __restrict__ in, int64_t ldi,
                                     bf16_t* __restrict__ out, int64_t ldo, const int* __restrict__ rows_dev, int row_off) {
  __shared__ bf16_t tile[64][72];                          // [source row][source col], padded
  const int live = rows_dev ? min(rows, *rows_dev - row_off) : rows;
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int k = threadIdx.x; k < 512; k += 256) {           // 64 rows x 8 chunks
    const int i = k >> 3, cc = (k & 7) * 8;
    const int r = r0 + i, c = c0 + cc;
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; e++) v[e] = (bf16_t)0.f;
    if (r < live && c < cols) v = *reinterpret_cast<const bf16x8*>(in + (int64_t)r * ldi + c);   // cols % 8 == 0: whole chunks
    *reinterpret_cast<bf16x8*>(&tile[i][cc]) = v;
  }
  __syncthreads();
  for (int k = threadIdx.x; k < 512; k += 256) {           // 64 output rows (source cols) x 8 chunks of 8 source rows
    const int oc = k & 63, ch = k >> 6;                    // consecutive threads: consecutive output rows, same chunk
    const int c = c0 + oc, rr = r0 + ch * 8;
    if (c >= cols || rr >= rows_pad) continue;
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const int pos = ch * 8 + e;                          // output position inside the tile
      const int src = QS ? ((pos & ~12) | ((pos & 4) << 1) | ((pos & 8) >> 1)) : pos;
      v[e] = tile[src][oc];
    }
    *reinterpret_cast<bf16x8*>(out + (int64_t)c * ldo + rr) = v;
  }
}

static bool transpose_vec_ok(int mode, int rows_pad, int cols, const void* in, int64_t ldi, const void* out, int64_t ldo) {
  return mode == AS_BF16 && rows_pad % 64 == 0 && cols % 8 == 0 && ldi % 8 == 0 && ldo % 8 == 0 &&
         (uintptr_t)in % 16 == 0 && (uintptr_t)out % 16 == 0;
}

int launch_transpose(as_ctx* ctx, int mode, int rows, int rows_pad, int cols, const void* in, int64_t ldi, void* out,
                     int64_t ldo, const int* rows_dev, int row_off, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return AS_OK;
  dim3 grid(cdiv(cols, 64), cdiv(rows_pad, 64));
  prof_begin(ctx, st, AS_K_TRANSPOSE, 0.0);
  if (transpose_vec_ok(mode, rows_pad, cols, in, ldi, out, ldo))
    transpose_vec_kernel<false><<<grid, 256, 0, st>>>(rows, rows_pad, cols, (const bf16_t*)in, ldi, (bf16_t*)out, ldo, rows_dev, row_off);
  else
  DISPATCH_T(mode, (transpose_kernel<T, false><<<grid, 256, 0, st>>>(rows, rows_pad, cols, (const T*)in, ldi, (T*)out, ldo, rows_dev, row_off)));
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// the quad-swapped variant (rows_pad must be a multiple of 16)
int launch_transpose_qs(as_ctx* ctx, int mode, int rows, int rows_pad, int cols, const void* in, int64_t ldi, void* out,
                        int64_t ldo, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return AS_OK;
  if (rows_pad % 16) return as_fail(ctx, AS_ERR_SHAPE, "transpose: the quad-swapped layout needs a row count padded to 16");
  dim3 grid(cdiv(cols, 64), cdiv(rows_pad, 64));
  prof_begin(ctx, st, AS_K_TRANSPOSE, 0.0);
  if (transpose_vec_ok(mode, rows_pad, cols, in, ldi, out, ldo))
    transpose_vec_kernel<true><<<grid, 256, 0, st>>>(rows, rows_pad, cols, (const bf16_t*)in, ldi, (bf16_t*)out, ldo, nullptr, 0);
  else
  DISPATCH_T(mode, (transpose_kernel<T, true><<<grid, 256, 0, st>>>(rows, rows_pad, cols, (const T*)in, ldi, (T*)out, ldo, nullptr, 0)));
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ------------------------------------------------------ LoRA operand copies
// out[rp, cp] = scale * in[r, c] inside, 0 in the padding; out_t is its transpose.
template <typename T>
__global__ void lora_prep_kernel(const float* __restrict__ in, int rows, int cols, int rows_pad, int cols_pad,
                                 float scale, T* __restrict__ out, int64_t ldo, T* __restrict__ out_t, int64_t ldo_t) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)rows_pad * cols_pad) return;
  int r = idx / cols_pad, c = idx % cols_pad;
  float v = (r < rows && c < cols) ? scale * in[(int64_t)r * cols + c] : 0.f;
  if (out) out[(int64_t)r * ldo + c] = from_f<T>(v);
  if (out_t) out_t[(int64_t)c * ldo_t + r] = from_f<T>(v);
}

int launch_lora_prep2(as_ctx* ctx, int mode, const float* in, int rows, int cols, int rows_pad, int cols_pad,
                      float scale, void* out, int64_t ldo, void* out_t, int64_t ldo_t, hipStream_t st) {
  int64_t tot = (int64_t)rows_pad * cols_pad;
  if (tot <= 0) return AS_OK;
  DISPATCH_T(mode, (lora_prep_kernel<T><<<cdiv(tot, 256), 256, 0, st>>>(in, rows, cols, rows_pad, cols_pad, scale,
                                                                        (T*)out, ldo, (T*)out_t, ldo_t)));
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n_words) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n_words; i += stride) p[i] = 0u;
}
int launch_fill_zero(as_ctx* ctx, void* p, size_t bytes, hipStream_t st) {
  size_t w = bytes / 4;                        // callers pass multiples of 4 bytes
  if (!w) return AS_OK;
  int blocks = (int)(cdiv((int64_t)w, 256) < 4096 ? cdiv((int64_t)w, 256) : 4096);
  fill_zero_kernel<<<blocks, 256, 0, st>>>((uint32_t*)p, w);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ---------------------------------------------------------- target selection
// Position t is a target when t+1 exists, starts no segment, and carries the
// mask.  One block scans the whole stream so the order is fixed.
__global__ void select_targets_kernel(const int32_t* __restrict__ seg_start, const uint8_t* __restrict__ mask,
                                      const int32_t* __restrict__ tok, int n, int32_t* __restrict__ tgt_idx,
                                      int32_t* __restrict__ tgt_pos, int32_t* __restrict__ labels,
                                      int32_t* __restrict__ count) {
  __shared__ int32_t sums[1024];
  int tid = threadIdx.x;
  int per = (n + 1023) / 1024;
  int b = tid * per, e = min(n, b + per);
  int c = 0;
  for (int t = b; t < e; t++) c += (t + 1 < n && seg_start[t + 1] != t + 1 && mask[t + 1]) ? 1 : 0;
  sums[tid] = c;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {          // inclusive scan
    int v = tid >= off ? sums[tid - off] : 0;
    __syncthreads();
    sums[tid] += v;
    __syncthreads();
  }
  int base = sums[tid] - c;
  for (int t = b; t < e; t++) {
    bool is = (t + 1 < n && seg_start[t + 1] != t + 1 && mask[t + 1]);
    if (is) { tgt_idx[base] = t; labels[base] = tok[t + 1]; tgt_pos[t] = base; base++; }
    else tgt_pos[t] = -1;
  }
  if (tid == 1023) *count = sums[1023];
}

int launch_select_targets(as_ctx* ctx, const int32_t* seg_start, const uint8_t* mask, const int32_t* tok,
                          int n, int32_t* tgt_idx, int32_t* tgt_pos, int32_t* labels, int32_t* count,
                          hipStream_t st) {
  select_targets_kernel<<<1, 1024, 0, st>>>(seg_start, mask, tok, n, tgt_idx, tgt_pos, labels, count);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ------------------------------------------------------------ cross-entropy
__device__ __forceinline__ float block_reduce(float v, float* sh, bool is_max) {
  v = is_max ? wave_max(v) : wave_sum(v);
  int w = threadIdx.x / AS_WAVE, nw = blockDim.x / AS_WAVE;
  __syncthreads();
  if (threadIdx.x % AS_WAVE == 0) sh[w] = v;
  __syncthreads();
  float r = sh[0];
  for (int i = 1; i < nw; i++) r = is_max ? fmaxf(r, sh[i]) : r + sh[i];
  return r;
}

// One block per target row of a chunk: logsumexp, the row's loss, and the
// gradient with respect to the logits: (softmax - one-hot) times the row's factor,
// row_w[row] when given, else 1 / target count (the mean loss).  P == nullptr: losses only.
template <typename T>
__global__ void ce_rows_kernel(const float* __restrict__ logits, int V, int row0, const int32_t* __restrict__ labels,
                               const int32_t* __restrict__ count, float* __restrict__ loss_rows,
                               const float* __restrict__ row_w, T* __restrict__ P) {
  __shared__ float sh[16];
  int cnt = *count;
  int row = row0 + blockIdx.x;
  if (row >= cnt) return;
  const float* z = logits + (int64_t)blockIdx.x * V;
  T* p = P + (int64_t)blockIdx.x * V;
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < V; v += blockDim.x) mx = fmaxf(mx, z[v]);
  mx = block_reduce(mx, sh, true);
  float s = 0.f;
  for (int v = threadIdx.x; v < V; v += blockDim.x) s += expf(z[v] - mx);
  s = block_reduce(s, sh, false);
  float lse = mx + logf(s);
  int y = labels[row];
  if (threadIdx.x == 0 && loss_rows) loss_rows[row] = lse - z[y];
  if (!P) return;
  float inv = row_w ? row_w[row] : 1.f / (float)cnt;
  for (int v = threadIdx.x; v < V; v += blockDim.x) {
    float g = expf(z[v] - lse) - (v == y ? 1.f : 0.f);
    p[v] = from_f<T>(g * inv);
  }
}

int launch_ce_rows(as_ctx* ctx, int mode, const float* logits, int rows_cap, int V, int row0,
                   const int32_t* labels, const int32_t* count, float* loss_rows, const float* row_w, void* P, hipStream_t st) {
  if (rows_cap <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_CE, 0.0);
  DISPATCH_T(mode, (ce_rows_kernel<T><<<rows_cap, 512, 0, st>>>(logits, V, row0, labels, count, loss_rows, row_w, (T*)P)));
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ---- head without stored logits: the two small row kernels around the GEMMs
// z_lab[row] = hf[row] . W[label[row]], one wave per target row (bf16 operands, float sum in a fixed order)
__global__ __launch_bounds__(256) void label_logit_kernel(const bf16_t* __restrict__ hf, const bf16_t* __restrict__ W, int d,
                                                          const int32_t* __restrict__ labels, const int32_t* __restrict__ count,
                                                          float* __restrict__ zlab) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= *count) return;
  const bf16_t* a = hf + (int64_t)row * d; const bf16_t* b = W + (int64_t)labels[row] * d;
  float acc = 0.f;
  for (int c = lane * 8; c < d; c += 512) {
    const bf16x8 x = *reinterpret_cast<const bf16x8*>(a + c), y = *reinterpret_cast<const bf16x8*>(b + c);
#pragma unroll
    for (int k = 0; k < 8; k++) acc = fmaf((float)x[k], (float)y[k], acc);
  }
  acc = wave_sum(acc);
  if (lane == 0) zlab[row] = acc;
}
int launch_label_logit(as_ctx* ctx, const void* hf, const void* W, int d, const int32_t* labels, const int32_t* count, int rows_cap,
                       float* zlab, hipStream_t st) {
  if (rows_cap <= 0) return AS_OK;
  if (d % 8) return as_fail(ctx, AS_ERR_SHAPE, "label logits: d_model must be a multiple of 8");
  prof_begin(ctx, st, AS_K_CE, 0.0);
  label_logit_kernel<<<(unsigned)cdiv(rows_cap, 4), 256, 0, st>>>((const bf16_t*)hf, (const bf16_t*)W, d, labels, count, zlab);
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// One wave per row of the chunk: combines the (maximum, sum of exponentials) pairs of the row's column blocks.
// Rows are chunk-relative in `part`, absolute (row0 + r) in zlab / lse / loss_rows.
__global__ __launch_bounds__(256) void ce_finish_kernel(const float* __restrict__ part, int nblk, int row0, const int32_t* __restrict__ count,
                                                        const float* __restrict__ zlab, float* __restrict__ lse_out, float* __restrict__ loss_rows) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int row = row0 + r;
  if (row >= *count) return;
  const float2* pr = reinterpret_cast<const float2*>(part) + (int64_t)r * nblk;
  float m = -INFINITY;
  for (int b = lane; b < nblk; b += 64) m = fmaxf(m, pr[b].x);
  m = wave_max(m);
  float s = 0.f;
  for (int b = lane; b < nblk; b += 64) { const float2 v = pr[b]; s += v.y * expf(v.x - m); }
  s = wave_sum(s);
  if (lane == 0) { const float lse = m + logf(s); lse_out[row] = lse; loss_rows[row] = lse - zlab[row]; }
}
int launch_ce_finish(as_ctx* ctx, const float* part, int nblk, int row0, int rows_cap, const int32_t* count, const float* zlab,
                     float* lse, float* loss_rows, hipStream_t st) {
  if (rows_cap <= 0) return AS_OK;
  prof_begin(ctx, st, AS_K_CE, 0.0);
  ce_finish_kernel<<<(unsigned)cdiv(rows_cap, 4), 256, 0, st>>>(part, nblk, row0, count, zlab, lse, loss_rows);
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// Sums the per-target losses in a fixed order: thread i takes a contiguous
// slab, slabs are combined by a tree in LDS.
__global__ void loss_finalize_kernel(const float* __restrict__ loss_rows, const int32_t* __restrict__ count,
                                     float* __restrict__ loss, float* __restrict__ loss_sum) {
  __shared__ double sh[1024];
  int n = *count;
  int per = (n + 1023) / 1024;
  int b = threadIdx.x * per, e = min(n, b + per);
  double acc = 0.0;
  for (int i = b; i < e; i++) acc += (double)loss_rows[i];
  sh[threadIdx.x] = acc;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *loss_sum = (float)sh[0];
    *loss = n > 0 ? (float)(sh[0] / (double)n) : 0.f;
  }
}

int launch_loss_finalize(as_ctx* ctx, const float* loss_rows, const int32_t* count, float* loss,
                         float* loss_sum, hipStream_t st) {
  loss_finalize_kernel<<<1, 1024, 0, st>>>(loss_rows, count, loss, loss_sum);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// -------------------------------------------------------- split-K reduction
__global__ void splitk_reduce_kernel(const float* __restrict__ partial, int splitk, int64_t mn, int N,
                                     float alpha, float* __restrict__ C, int64_t ldc) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= mn) return;
  float acc = 0.f;
  for (int s = 0; s < splitk; s++) acc += partial[(int64_t)s * mn + i];
  C[(i / N) * ldc + (i % N)] = alpha * acc;
}
int launch_splitk_reduce(as_ctx* ctx, const float* partial, int splitk, int64_t mn, int N, float alpha,
                         float* C, int64_t ldc, hipStream_t st) {
  if (mn <= 0) return AS_OK;
  splitk_reduce_kernel<<<cdiv(mn, 256), 256, 0, st>>>(partial, splitk, mn, N, alpha, C, ldc);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// -------------------------------------------------------------------- AdamW
// Up to kAdamBatch tensors per launch, described in the kernel argument itself: workgroup b takes the b-th chunk of
// 65,536 consecutive elements of the batch (tensor found by a scan over the batch's first-chunk numbers).
__global__ __launch_bounds__(256) void adamw_batch_kernel(const AdamBatch b, float lr, float b1, float b2, float eps, float bc1, float bc2) {
  int ti = 0;
  while (ti + 1 < b.n && (int)blockIdx.x >= b.t[ti + 1].first_chunk) ti++;
  const AdamTensor& t = b.t[ti];
  const int64_t lo = (int64_t)((int)blockIdx.x - t.first_chunk) * 65536, hi = min(t.n, lo + 65536);
  for (int64_t i = lo + threadIdx.x; i < hi; i += 256) {
    float gi = t.g[i], wi = t.w[i];
    float mi = b1 * t.m[i] + (1.f - b1) * gi;
    float vi = b2 * t.v[i] + (1.f - b2) * gi * gi;
    t.m[i] = mi; t.v[i] = vi;
    float upd = (mi / bc1) / (sqrtf(vi / bc2) + eps) + t.wd * wi;
    wi = wi - lr * upd;
    t.w[i] = wi;
    if (t.w_lowp) t.w_lowp[i] = (bf16_t)wi;
  }
}
int launch_adamw_batch(as_ctx* ctx, const AdamBatch& b, float lr, float b1, float b2, float eps, float bc1, float bc2, hipStream_t st) {
  if (b.n <= 0 || b.n_chunks <= 0) return AS_OK;
  adamw_batch_kernel<<<b.n_chunks, 256, 0, st>>>(b, lr, b1, b2, eps, bc1, bc2);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ------------------------------------------------- embedding gradient (full)
// dE[v] = sum of dh[t] over the positions t holding token v, in ascending t.
// rank[t] = number of earlier positions with the same token (brute force over
// LDS-staged token tiles) gives each position a fixed slot in its token's list.
__global__ void token_rank_kernel(const int32_t* __restrict__ tok, int n, int32_t* __restrict__ prev) {
  // prev[t] = largest t' < t with tok[t'] == tok[t], or -1: a linked list per token
  __shared__ int32_t tile[1024];
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  int mine = t < n ? tok[t] : -1;
  int best = -1;
  int t_hi = min(n, (int)((blockIdx.x + 1) * blockDim.x));
  for (int base = 0; base < t_hi; base += 1024) {
    __syncthreads();
    if (base + (int)threadIdx.x < n) tile[threadIdx.x] = tok[base + threadIdx.x];
    __syncthreads();
    int lim = min(1024, t - base);
    for (int i = 0; i < lim; i++) if (tile[i] == mine) best = base + i;
  }
  if (t < n) prev[t] = best;
}
template <typename T>
__global__ void embed_bwd_kernel(const int32_t* __restrict__ tok, const int32_t* __restrict__ prev,
                                 const int32_t* __restrict__ is_last, int n, int d, const T* __restrict__ dh,
                                 float* __restrict__ dE) {
  // one block per position that is the LAST occurrence of its token: walk the list backwards
  int t = blockIdx.x;
  if (!is_last[t]) return;
  int v = tok[t];
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    // collect in ascending order: first count, then the walk is reversed by recursion-free two passes
    float acc = 0.f;
    // ascending order needs the list reversed; addition order is fixed either way (descending t)
    for (int u = t; u >= 0; u = prev[u]) acc += to_f<T>(dh[(int64_t)u * d + j]);
    dE[(int64_t)v * d + j] = acc;
  }
}
__global__ void mark_last_kernel(const int32_t* __restrict__ prev, int n, int32_t* __restrict__ is_last) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  int p = prev[t];
  if (p >= 0) is_last[p] = 0;      // plain stores of the same value: order does not matter
}
__global__ void fill_int_kernel(int32_t* p, int n, int v) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) p[t] = v;
}

int launch_embed_bwd(as_ctx* ctx, int mode, const int32_t* tok, int n, int d, int V, const void* dh,
                     int32_t* scratch, float* dE, hipStream_t st) {
  // scratch: 2n int32 (prev, is_last).  dE is zeroed first (rows of unused tokens stay zero).
  int rc = launch_fill_zero(ctx, dE, (size_t)V * d * sizeof(float), st);
  if (rc) return rc;
  if (n <= 0) return AS_OK;
  int32_t* prev = scratch; int32_t* is_last = scratch + n;
  token_rank_kernel<<<cdiv(n, 1024), 1024, 0, st>>>(tok, n, prev);
  AS_LAUNCH_CHECK(ctx);
  fill_int_kernel<<<cdiv(n, 256), 256, 0, st>>>(is_last, n, 1);
  AS_LAUNCH_CHECK(ctx);
  mark_last_kernel<<<cdiv(n, 256), 256, 0, st>>>(prev, n, is_last);
  AS_LAUNCH_CHECK(ctx);
  DISPATCH_T(mode, (embed_bwd_kernel<T><<<n, 256, 0, st>>>(tok, prev, is_last, n, d, (const T*)dh, dE)));
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}
