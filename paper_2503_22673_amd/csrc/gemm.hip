// C[M,N] = alpha * sum_s A_s[M,K_s] * B_s[N,K_s]^T (+ R): the projection GEMMs
// of the fine-tuning step.  The second K segment carries the low-rank LoRA
// product (x A^T)(s B)^T, so the adapter costs one extra pass over r columns
// inside the same accumulators instead of a second GEMM and an add.
//
// Two kernels:
//  * gemm_fma_kernel   -- any type, any shape; 64x64 tile, fp32 FMAs.  The
//    fp32 tier runs on it.
//  * gemm_mfma_kernel  -- bf16 in, fp32 accumulate, v_mfma_f32_32x32x16_bf16.
//    Tiles are staged global -> registers -> LDS (two LDS stages, one barrier
//    per 64-wide K step), rows padded by 16 bytes so that the 16-byte fragment
//    reads of 16 lanes hit 64 distinct banks.  Workgroup ids are first
//    de-interleaved over the 8 XCDs (ids are dealt round-robin to XCDs, each
//    with a private L2) and then walked in groups of 8 row-tiles so that the
//    tiles resident on one XCD share A and B panels.
#include "common.h"

// ------------------------------------------------------------------ helpers
struct KRange { int beg, end; };   // k-tile range of one segment for this split
__device__ __forceinline__ KRange split_range(int K, int BK, int splitk, int z) {
  int tiles = (K + BK - 1) / BK;
  int per = (tiles + splitk - 1) / splitk;
  KRange r; r.beg = min(tiles, z * per); r.end = min(tiles, r.beg + per);
  return r;
}

// Live row count of this launch and, for grouped rows, the first row of the group (rb): rows of A, R
// and C are then rb + (0 .. M-1).  mmax is the largest row index a clamped load may touch.
__device__ __forceinline__ int gemm_rows(const GemmParams& p, int m_off, int& rb, int& mmax) {
  int M = p.m_dev ? min(p.M, *p.m_dev - m_off) : p.M;
  rb = 0; mmax = p.M - 1;
  if (p.grp_off) {
    rb = p.grp_off[p.grp];
    M = min(M, p.grp_off[p.grp + 1] - rb);
    mmax = max(M, 1) - 1;
  }
  return M;
}

template <typename T>
__device__ __forceinline__ void store_out(const GemmParams& p, int z, int row, int col, float v, int rb) {
  if (p.splitk > 1) { p.partial[((int64_t)z * p.M + row) * p.N + col] = v; return; }
  v *= p.alpha;
  row += rb;
  if (p.R) v += to_f<T>(((const T*)p.R)[(int64_t)row * p.ldr + col]);
  if (p.c_f32) {
    float* c = (float*)p.C + (int64_t)row * p.ldc + col;
    *c = p.accumulate ? *c + v : v;
  } else {
    ((T*)p.C)[(int64_t)row * p.ldc + col] = from_f<T>(v);
  }
}

// ------------------------------------------------------------- plain kernel
template <typename T>
__global__ __launch_bounds__(256) void gemm_fma_kernel(GemmParams p, int m_off) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  int rb, mmax;
  int M = gemm_rows(p, m_off, rb, mmax);
  int row0 = blockIdx.y * BM, col0 = blockIdx.x * BN, z = blockIdx.z;
  if (row0 >= M) return;
  int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  int lr = tid / 4, lk = (tid % 4) * 4;                 // loader: one row, 4 consecutive k
  for (int s = 0; s < p.nseg; s++) {
    const T* A = (const T*)p.seg[s].A; const T* B = (const T*)p.seg[s].B;
    int64_t lda = p.seg[s].lda, ldb = p.seg[s].ldb; int K = p.seg[s].K;
    KRange kr = split_range(K, BK, p.splitk, z);
    for (int kt = kr.beg; kt < kr.end; kt++) {
      int k0 = kt * BK;
#pragma unroll
      for (int q = 0; q < 4; q++) {
        int k = k0 + lk + q;
        int ar = row0 + lr, br = col0 + lr;
        As[lk + q][lr] = (ar < M && k < K) ? to_f<T>(A[(int64_t)(rb + ar) * lda + k]) : 0.f;
        Bs[lk + q][lr] = (br < p.N && k < K) ? to_f<T>(B[(int64_t)br * ldb + k]) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < BK; k++) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; i++) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
          for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int r = row0 + ty * 4 + i, c = col0 + tx * 4 + j;
      if (r < M && c < p.N) store_out<T>(p, z, r, c, acc[i][j], rb);
    }
}

// -------------------------------------------------------------- MFMA kernel
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Epilogue shared by the MFMA kernels.  Lane l holds column l%32 and rows 8*(e/4) + 4*(l/32) + e%4 of
// each 32x32 block.  The output kind is uniform for the launch, so it is tested once, outside the
// element loops; `full` tiles skip the bounds tests.
template <int TM, int TN>
__device__ __forceinline__ void gemm_epilogue(const GemmParams& p, f32x16 (&acc)[TM][TN], int M, int z, int row0, int col0,
                                              int rb0, int cb0, bool full, int rb) {
  auto each = [&](auto f) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const int c = cb0 + j * 32;
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int r = rb0 + i * 32 + 8 * (e >> 2) + (e & 3);
          if (full || (r < M && c < p.N)) f(r + rb, c, acc[i][j][e]);
        }
      }
  };
  if (p.splitk > 1) {
    float* part = p.partial + (int64_t)z * p.M * p.N;
    each([&](int r, int c, float v) { part[(int64_t)(r - rb) * p.N + c] = v; });
  } else if (p.c_f32) {
    float* C = (float*)p.C; const float alpha = p.alpha; const bf16_t* R = (const bf16_t*)p.R;
    if (p.accumulate || R)
      each([&](int r, int c, float v) {
        float* q = C + (int64_t)r * p.ldc + c;
        float x = alpha * v + (R ? (float)R[(int64_t)r * p.ldr + c] : 0.f);
        *q = p.accumulate ? *q + x : x;
      });
    else each([&](int r, int c, float v) { C[(int64_t)r * p.ldc + c] = alpha * v; });
  } else if (p.R) {
    bf16_t* C = (bf16_t*)p.C; const bf16_t* R = (const bf16_t*)p.R; const float alpha = p.alpha;
    each([&](int r, int c, float v) { C[(int64_t)r * p.ldc + c] = (bf16_t)(alpha * v + (float)R[(int64_t)r * p.ldr + c]); });
  } else {
    bf16_t* C = (bf16_t*)p.C; const float alpha = p.alpha;
    each([&](int r, int c, float v) { C[(int64_t)r * p.ldc + c] = (bf16_t)(alpha * v); });
  }
}

// EDGE = false: every K segment is a multiple of 64, so tile loads need no k guard.
template <int BM, int BN, int WM, int WN, bool EDGE>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_kernel(GemmParams p, int m_off, int tiles_m, int tiles_n) {
  constexpr int BK = 64, LS = BK + 8, NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int CA = BM * 8 / NT, CB = BN * 8 / NT;      // 16-byte chunks per thread and tile
  static_assert(CA >= 1 && CB >= 1, "tile too small for the thread count");
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sA = (bf16_t*)smem;                            // [2][BM][LS]
  bf16_t* sB = sA + 2 * BM * LS;                         // [2][BN][LS]

  int rb, mmax;
  const int M = gemm_rows(p, m_off, rb, mmax);
  // XCD de-interleave, then grouped walk over the tile grid (over the live row tiles only when
  // the row count is a device-side value)
  if (p.m_dev || p.grp_off) tiles_m = min(tiles_m, (max(M, 0) + BM - 1) / BM);
  int nblk = tiles_m * tiles_n, pid = blockIdx.x, z = blockIdx.y;
  if (pid >= nblk) return;
  int q8 = nblk / 8, rem = nblk % 8, xcd = pid % 8, loc = pid / 8;
  int logical = xcd * q8 + min(xcd, rem) + loc;
  constexpr int GROUP = 8;
  int in_group = GROUP * tiles_n, grp = logical / in_group, first_m = grp * GROUP;
  int gsize = min(tiles_m - first_m, GROUP);
  int tile_m = first_m + (logical % in_group) % gsize, tile_n = (logical % in_group) / gsize;
  const int row0 = tile_m * BM, col0 = tile_n * BN;
  if (row0 >= M) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  KRange kr0 = split_range(p.seg[0].K, BK, p.splitk, z);
  KRange kr1 = {0, 0};
  if (p.nseg > 1) kr1 = split_range(p.seg[1].K, BK, p.splitk, z);
  const int nt0 = kr0.end - kr0.beg, nt = nt0 + (kr1.end - kr1.beg);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  u32x4 ra[CA], rbv[CB];
  // per-thread row offsets inside the tile are fixed; only the k offset moves
  int64_t offA[CA], offB[CB];
  {
    const int mclamp = mmax, nclamp = p.N - 1;
#pragma unroll
    for (int i = 0; i < CA; i++) { int c = tid + i * NT; offA[i] = (int64_t)(rb + min(row0 + (c >> 3), mclamp)); }
#pragma unroll
    for (int i = 0; i < CB; i++) { int c = tid + i * NT; offB[i] = (int64_t)min(col0 + (c >> 3), nclamp); }
  }
  const int kc = (tid & 7) * 8;                          // NT is a multiple of 8: same k chunk for every i

  auto fetch = [&](int it) {
    const bool first = it < nt0;
    const bf16_t* A = (const bf16_t*)(first ? p.seg[0].A : p.seg[1].A);
    const bf16_t* B = (const bf16_t*)(first ? p.seg[0].B : p.seg[1].B);
    const int64_t lda = first ? p.seg[0].lda : p.seg[1].lda, ldb = first ? p.seg[0].ldb : p.seg[1].ldb;
    const int K = first ? p.seg[0].K : p.seg[1].K;
    const int k = (first ? kr0.beg + it : kr1.beg + it - nt0) * BK + kc;
    const bool in = !EDGE || k < K;
    const int ks = in ? k : 0;                           // a valid address either way
#pragma unroll
    for (int i = 0; i < CA; i++) {
      u32x4 v = *reinterpret_cast<const u32x4*>(A + offA[i] * lda + ks);
      ra[i] = in ? v : (u32x4){0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < CB; i++) {
      u32x4 v = *reinterpret_cast<const u32x4*>(B + offB[i] * ldb + ks);
      rbv[i] = in ? v : (u32x4){0u, 0u, 0u, 0u};
    }
  };
  auto stash = [&](int buf) {
    bf16_t* a = sA + buf * BM * LS; bf16_t* b = sB + buf * BN * LS;
#pragma unroll
    for (int i = 0; i < CA; i++) { int c = tid + i * NT; *reinterpret_cast<u32x4*>(a + (c >> 3) * LS + kc) = ra[i]; }
#pragma unroll
    for (int i = 0; i < CB; i++) { int c = tid + i * NT; *reinterpret_cast<u32x4*>(b + (c >> 3) * LS + kc) = rbv[i]; }
  };

  if (nt > 0) { fetch(0); stash(0); }
  __syncthreads();
  for (int it = 0; it < nt; it++) {
    const int buf = it & 1;
    if (it + 1 < nt) fetch(it + 1);
    const bf16_t* a = sA + buf * BM * LS + (wm * TM * 32 + (lane & 31)) * LS + (lane >> 5) * 8;
    const bf16_t* b = sB + buf * BN * LS + (wn * TN * 32 + (lane & 31)) * LS + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ks++) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; i++) af[i] = *reinterpret_cast<const bf16x8*>(a + i * 32 * LS + ks * 16);
#pragma unroll
      for (int j = 0; j < TN; j++) bfr[j] = *reinterpret_cast<const bf16x8*>(b + j * 32 * LS + ks * 16);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (it + 1 < nt) stash(buf ^ 1);
    __syncthreads();
  }

  gemm_epilogue<TM, TN>(p, acc, M, z, row0, col0, row0 + wm * TM * 32 + 4 * (lane >> 5), col0 + wn * TN * 32 + (lane & 31),
                        (row0 + BM <= M) && (col0 + BN <= p.N), rb);
}

// Same tiling, but tiles travel global -> LDS directly (global_load_lds_dwordx4: a wavefront
// deposits 64 x 16 bytes contiguously, i.e. 8 rows of 8 chunks), so no VGPR staging and no LDS
// stores.  The destination cannot be padded, so chunks are XOR-swizzled instead: LDS slot
// (row, c) holds the row's chunk c ^ ((row >> 1) & 7); each lane picks the matching global chunk.  Fragment
// reads of 8 consecutive rows then touch 8 different 16-byte columns: no bank conflicts.
// Fragments are double-buffered in registers.  The barrier of a K step sits before the last of its four
// 16-wide slices: by then every fragment of the current tile is in registers, so the next tile's loads can
// be issued into the buffer just released and the first fragments of the next tile are read while the last
// slice's MFMAs run, instead of right after a barrier with nothing to overlap them.
// Needs every K segment to be a multiple of 64.
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_dlds_kernel(GemmParams p, int m_off, int tiles_m, int tiles_n) {
  constexpr int BK = 64, NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int LA = BM / 8 / NW, LB = BN / 8 / NW;      // 1 KB wave-loads per wave and tile
  static_assert(LA >= 1 && LB >= 1, "tile too small for the wave count");
  static_assert(BK / 16 == 4, "the loop is written for four K slices");
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sA = (bf16_t*)smem;                            // [2][BM][64]
  bf16_t* sB = sA + 2 * BM * BK;                         // [2][BN][64]

  int rb, mmax;
  const int M = gemm_rows(p, m_off, rb, mmax);
  // the row count may live on the device (target rows, rows of one expert): map the workgroups
  // over the live row tiles only, so that they still spread over all XCDs
  if (p.m_dev || p.grp_off) tiles_m = min(tiles_m, (max(M, 0) + BM - 1) / BM);
  int nblk = tiles_m * tiles_n, pid = blockIdx.x, z = blockIdx.y;
  if (pid >= nblk) return;
  int q8 = nblk / 8, rem = nblk % 8, xcd = pid % 8, loc = pid / 8;
  int logical = xcd * q8 + min(xcd, rem) + loc;
  constexpr int GROUP = 8;
  int in_group = GROUP * tiles_n, grp = logical / in_group, first_m = grp * GROUP;
  int gsize = min(tiles_m - first_m, GROUP);
  int tile_m = first_m + (logical % in_group) % gsize, tile_n = (logical % in_group) / gsize;
  const int row0 = tile_m * BM, col0 = tile_n * BN;
  if (row0 >= M) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  KRange kr0 = split_range(p.seg[0].K, BK, p.splitk, z);
  KRange kr1 = {0, 0};
  if (p.nseg > 1) kr1 = split_range(p.seg[1].K, BK, p.splitk, z);
  const int nt0 = kr0.end - kr0.beg, nt = nt0 + (kr1.end - kr1.beg);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  // loader: wave-load i of this wave covers tile rows (wave*L + i)*8 .. +7; lane l sits at row l/8,
  // LDS chunk l%8, and fetches global chunk (l%8) ^ swz(row)
  const int lrow = lane >> 3;
  int rowA[LA], rowB[LB];
  {
    const int mclamp = mmax, nclamp = p.N - 1;
#pragma unroll
    for (int i = 0; i < LA; i++) rowA[i] = rb + min(row0 + (wave * LA + i) * 8 + lrow, mclamp);
#pragma unroll
    for (int i = 0; i < LB; i++) rowB[i] = min(col0 + (wave * LB + i) * 8 + lrow, nclamp);
  }
  // per-lane row pointers of the first K segment are kept in registers (no 64-bit multiplies per step)
  const bf16_t* pA[LA]; const bf16_t* pB[LB];
#pragma unroll
  for (int i = 0; i < LA; i++) pA[i] = (const bf16_t*)p.seg[0].A + (int64_t)rowA[i] * p.seg[0].lda + (((lane & 7) ^ swz((wave * LA + i) * 8 + lrow)) * 8);
#pragma unroll
  for (int i = 0; i < LB; i++) pB[i] = (const bf16_t*)p.seg[0].B + (int64_t)rowB[i] * p.seg[0].ldb + (((lane & 7) ^ swz((wave * LB + i) * 8 + lrow)) * 8);
  auto fetch = [&](int it, int buf) {
    const bool first = it < nt0;
    bf16_t* a = sA + buf * BM * BK + wave * LA * 8 * BK;
    bf16_t* b = sB + buf * BN * BK + wave * LB * 8 * BK;
    if (first) {
      const int k1 = (kr0.beg + it) * BK;
#pragma unroll
      for (int i = 0; i < LA; i++)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(pA[i] + k1),
                                         (__attribute__((address_space(3))) void*)(a + i * 8 * BK), 16, 0, 0);
#pragma unroll
      for (int i = 0; i < LB; i++)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(pB[i] + k1),
                                         (__attribute__((address_space(3))) void*)(b + i * 8 * BK), 16, 0, 0);
      return;
    }
    const bf16_t* A = (const bf16_t*)p.seg[1].A; const bf16_t* B = (const bf16_t*)p.seg[1].B;
    const int64_t lda = p.seg[1].lda, ldb = p.seg[1].ldb;
    const int k = (kr1.beg + it - nt0) * BK;
#pragma unroll
    for (int i = 0; i < LA; i++)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(A + (int64_t)rowA[i] * lda + k + (((lane & 7) ^ swz((wave * LA + i) * 8 + lrow)) * 8)),
                                       (__attribute__((address_space(3))) void*)(a + i * 8 * BK), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < LB; i++)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(B + (int64_t)rowB[i] * ldb + k + (((lane & 7) ^ swz((wave * LB + i) * 8 + lrow)) * 8)),
                                       (__attribute__((address_space(3))) void*)(b + i * 8 * BK), 16, 0, 0);
  };

  // reader: row = base + l%32, logical chunk 2*ks + l/32 lives at chunk (2*ks + l/32) ^ swz(row)
  const int x7 = swz(lane & 31), hh = lane >> 5;
  int coff[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ks++) coff[ks] = ((2 * ks + hh) ^ x7) * 8;

  if (nt > 0) fetch(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0f70);                    // vmcnt(0): the first tile has landed
  __syncthreads();
  bf16x8 af[2][TM], bfr[2][TN];
  auto rd = [&](int buf, int ks, int slot) {
    const bf16_t* a = sA + buf * BM * BK + (wm * TM * 32 + (lane & 31)) * BK;
    const bf16_t* b = sB + buf * BN * BK + (wn * TN * 32 + (lane & 31)) * BK;
#pragma unroll
    for (int i = 0; i < TM; i++) af[slot][i] = *reinterpret_cast<const bf16x8*>(a + i * 32 * BK + coff[ks]);
#pragma unroll
    for (int j = 0; j < TN; j++) bfr[slot][j] = *reinterpret_cast<const bf16x8*>(b + j * 32 * BK + coff[ks]);
  };
  auto mm = [&](int slot) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[slot][i], bfr[slot][j], acc[i][j], 0, 0, 0);
  };
  auto weave = [&]() {                                   // one LDS read between MFMAs, then the rest of the MFMAs
#pragma unroll
    for (int r = 0; r < TM + TN; r++) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TM + TN), 0);
  };
  if (nt > 1) fetch(1, 1);
  if (nt > 0) rd(0, 0, 0);
  for (int it = 0; it < nt; it++) {
    const int buf = it & 1;
    rd(buf, 1, 1); mm(0); weave();
    rd(buf, 2, 0); mm(1); weave();
    rd(buf, 3, 1); mm(0); weave();
    __builtin_amdgcn_s_waitcnt(0x0070);                  // vmcnt(0) lgkmcnt(0)
    __syncthreads();                                     // tile it is in registers everywhere, tile it+1 has landed
    // straight-line tail (the last two steps re-request the final tile into a buffer nobody reads
    // again, and read fragments nobody uses), so that loads, LDS reads and MFMAs can interleave
    fetch(min(it + 2, nt - 1), buf);
    rd(buf ^ 1, 0, 0);
    mm(1);
#pragma unroll
    for (int r = 0; r < TM + TN; r++) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x020, LA + LB, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TM + TN), 0);
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);                    // the re-requested tile must land before the workgroup's LDS is released
  gemm_epilogue<TM, TN>(p, acc, M, z, row0, col0, row0 + wm * TM * 32 + 4 * (lane >> 5), col0 + wn * TN * 32 + (lane & 31),
                        (row0 + BM <= M) && (col0 + BN <= p.N), rb);
}

// Epilogue for accumulator blocks that were computed transposed (B fragment as the first MFMA operand): a lane owns
// row (lane % 32) of every 32 x 32 block and, per accumulator quad b4, the four consecutive columns
// 8 b4 + 4 (lane / 32) .. + 3.  Whole tiles only, no split-K.  One row pointer per 32-row block and immediate column
// offsets: nothing to keep in registers besides the accumulators (the element-wise epilogue above, unrolled over
// 256 accumulators per lane, spills, and on this chip a spill reload waits for every store in flight).
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
template <int TM, int TN, bool MASK = false>
__device__ __forceinline__ void gemm_epilogue_rows(const GemmParams& p, f32x16 (&acc)[TM][TN], int row_lane, int col_lane,
                                                   int row_lo = 0, int row_hi = 0) {
  const float alpha = p.alpha;
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int64_t r = row_lane + 32 * i;
    if (MASK && (r < row_lo || r >= row_hi)) continue;   // with MASK only rows row_lo .. row_hi - 1 are written (and read)
    if (p.c_f32) {
      float* c = (float*)p.C + r * p.ldc + col_lane;
      const bf16_t* rr = p.R ? (const bf16_t*)p.R + r * p.ldr + col_lane : nullptr;
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int b4 = 0; b4 < 4; b4++) {
          f32x4 v;
#pragma unroll
          for (int k = 0; k < 4; k++) v[k] = alpha * acc[i][j][4 * b4 + k];
          if (rr) { const bf16x4_t x = *reinterpret_cast<const bf16x4_t*>(rr + 32 * j + 8 * b4);
#pragma unroll
            for (int k = 0; k < 4; k++) v[k] += (float)x[k]; }
          f32x4* q = reinterpret_cast<f32x4*>(c + 32 * j + 8 * b4);
          if (p.accumulate) { const f32x4 o = *q;
#pragma unroll
            for (int k = 0; k < 4; k++) v[k] += o[k]; }
          *q = v;
        }
    } else {
      bf16_t* c = (bf16_t*)p.C + r * p.ldc + col_lane;
      const bf16_t* rr = p.R ? (const bf16_t*)p.R + r * p.ldr + col_lane : nullptr;
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int b4 = 0; b4 < 4; b4++) {
          f32x4 v;
#pragma unroll
          for (int k = 0; k < 4; k++) v[k] = alpha * acc[i][j][4 * b4 + k];
          if (rr) { const bf16x4_t x = *reinterpret_cast<const bf16x4_t*>(rr + 32 * j + 8 * b4);
#pragma unroll
            for (int k = 0; k < 4; k++) v[k] += (float)x[k]; }
          bf16x4_t w;
#pragma unroll
          for (int k = 0; k < 4; k++) w[k] = (bf16_t)v[k];
          *reinterpret_cast<bf16x4_t*>(c + 32 * j + 8 * b4) = w;
        }
    }
  }
}

// The same accumulator layout, bf16 output, through LDS: stored 8 bytes per lane as above, a store instruction touches
// 32 rows with 16 bytes each, and the epilogue of a 256 x 256 tile costs 8-10 % of a tile with a contraction of 4096.
// Here every wave writes its 128 x 128 block (with the residual added and rounded once, as above) into its own part of
// the tile memory, which is free once every wave has left the loop, and reads it back 16 bytes per lane, so that a store
// instruction writes four whole 256-byte row pieces.  Rows are 272 bytes apart in LDS.  The residual takes the same way
// in: loaded 16 bytes per lane, parked at the place of the result, picked up by the lane that owns the element.
// PROB: the values are turned into w_row * (exp(value - lse_row) - [column is the row's label]) before they are rounded
// (the gradient of the masked cross-entropy with respect to the logits, written instead of the logits themselves).
template <int TM, int TN, bool MASK = false, bool PROB = false>
__device__ __forceinline__ void gemm_epilogue_staged(const GemmParams& p, f32x16 (&acc)[TM][TN], unsigned char* smem, int wave, int lane,
                                                     int row_w0, int col_w0, int row_lo = 0, int row_hi = 0) {
  constexpr int LROW = 272, ROWS = TM * 32;
  static_assert(TN * 32 == 128, "a block row is 256 bytes: 16 lanes of 16 bytes");
  unsigned char* my = smem + wave * (ROWS * LROW);
  const int l31 = lane & 31, hh = lane >> 5, r4 = lane >> 4, c16 = lane & 15;
  const float alpha = p.alpha;
  __syncthreads();                                       // the other waves have read their last fragments
  if (p.R) {
    const bf16_t* rr = (const bf16_t*)p.R + (int64_t)(row_w0 + r4) * p.ldr + col_w0 + c16 * 8;
#pragma unroll 8
    for (int it = 0; it < ROWS / 4; it++) {
      const int r = row_w0 + 4 * it + r4;
      if (!MASK || (r >= row_lo && r < row_hi))          // with MASK only rows row_lo .. row_hi - 1 are read and written
        *reinterpret_cast<u32x4*>(my + (4 * it + r4) * LROW + c16 * 16) = *reinterpret_cast<const u32x4*>(rr + (int64_t)(4 * it) * p.ldr);
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);                  // lgkmcnt(0): LDS operations of a wave complete in order; this is for the compiler's sake
    asm volatile("" ::: "memory");
  }
#pragma unroll
  for (int i = 0; i < TM; i++) {
    float neg_lse2 = 0.f, wrow = 0.f; int clab = -1;
    if (PROB) {                                          // rows outside the live range compute with the last live row's values and are not written
      const int r = MASK ? min(max(row_w0 + 32 * i + l31, row_lo), row_hi - 1) : row_w0 + 32 * i + l31;
      neg_lse2 = -1.4426950408889634f * p.epi_lse[r];
      wrow = p.epi_w ? p.epi_w[r] : 1.f / (float)*p.epi_cnt;
      clab = p.epi_lab[r] - col_w0 - 4 * hh;               // position of the label among this lane's columns of the block, if any
    }
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int b4 = 0; b4 < 4; b4++) {
        bf16x4_t* q = reinterpret_cast<bf16x4_t*>(my + (32 * i + l31) * LROW + (32 * j + 8 * b4 + 4 * hh) * 2);
        f32x4 v;
#pragma unroll
        for (int k = 0; k < 4; k++) v[k] = alpha * acc[i][j][4 * b4 + k];
        if (PROB) {
#pragma unroll
          for (int k = 0; k < 4; k++)
            v[k] = wrow * (__builtin_amdgcn_exp2f(fmaf(v[k], 1.4426950408889634f, neg_lse2)) - (clab == 32 * j + 8 * b4 + k ? 1.f : 0.f));
        }
        if (p.R) { const bf16x4_t x = *q;
#pragma unroll
          for (int k = 0; k < 4; k++) v[k] += (float)x[k]; }
        bf16x4_t w;
#pragma unroll
        for (int k = 0; k < 4; k++) w[k] = (bf16_t)v[k];
        *q = w;
      }
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);
  asm volatile("" ::: "memory");
  bf16_t* c = (bf16_t*)p.C + (int64_t)(row_w0 + r4) * p.ldc + col_w0 + c16 * 8;
#pragma unroll 8
  for (int it = 0; it < ROWS / 4; it++) {
    const int r = row_w0 + 4 * it + r4;
    if (!MASK || (r >= row_lo && r < row_hi))
      *reinterpret_cast<u32x4*>(c + (int64_t)(4 * it) * p.ldc) = *reinterpret_cast<const u32x4*>(my + (4 * it + r4) * LROW + c16 * 16);
  }
}

// Softmax statistics of a wave's 128 x 128 block of logits, straight from the accumulators (same lane layout as above: a lane
// owns row lane % 32 of every 32-row block and half of the block's 128 columns, the other half sits in lane ^ 32): per row the
// maximum and the sum of exp(value - maximum) over the 128 columns.  Nothing of the logits is written.
template <int TM, int TN, bool MASK>
__device__ __forceinline__ void gemm_epilogue_stats(const GemmParams& p, f32x16 (&acc)[TM][TN], int row_lane, int blk, int hh, int row_lo, int row_hi) {
  const float alpha = p.alpha;
  const int nblk = p.N / 128;
#pragma unroll
  for (int i = 0; i < TM; i++) {
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) m = fmaxf(m, alpha * acc[i][j][e]);
    const float mo = __shfl_xor(m, 32, 64);
    const float mx = fmaxf(m, mo);
    const float nm2 = -1.4426950408889634f * mx;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) s += __builtin_amdgcn_exp2f(fmaf(alpha * acc[i][j][e], 1.4426950408889634f, nm2));
    s += __shfl_xor(s, 32, 64);
    const int r = row_lane + 32 * i;
    if (hh == 0 && (!MASK || (r >= row_lo && r < row_hi))) {
      float2* q = reinterpret_cast<float2*>(p.epi_part) + (int64_t)r * nblk + blk;
      *q = make_float2(mx, s);
    }
  }
}

// Register-staged pipeline with a hand-scheduled loop, four waves of 128 x 128 (one per SIMD: the 256 accumulator
// registers of a wave live in the accumulation half of the register file, the vector half holds two register
// stages of tile data and two fragment sets).  In the kernels above a tile's loads are issued one K step before
// the tile is needed, because LDS holds two stages and the landing stage is the only place a direct-to-LDS load
// can go; a load that misses the L2 comes back later than that, and the workgroup waits for it at the barrier.
// Here a tile travels global -> registers -> LDS and its loads are issued 1.75 K steps before its LDS store.
// With one wave per SIMD every wait in the instruction stream idles the matrix pipe, so the loop is written out
// instruction by instruction (gen_gemm_rs_loop.py -> gemm_rs_loop.inc).  LDS layout and fragment order are those
// of the direct-to-LDS kernel.  Covers whole 256 x 256 tiles, K segments that are multiples of 64, host-side
// row counts, no split-K; the launcher sends everything else to the other kernels.
// LIVE = 1: the row count is a device-side value and / or the rows are those of one group (expert).  Tiles past the live
// rows exit; a tile still computes 256 rows, moved up if need be so that they lie inside the `limit` rows the operands
// are known to have (M for a plain row count, rows_cap for grouped rows), and writes the rows that are its own and live.
#include "gemm_rs_loop.inc"
// EPI: the epilogue is a compile-time choice (GEMM_EPI_*), so that the head's epilogues, which need registers of their own,
// cost the projection GEMMs nothing.
template <int LIVE, int EPI = GEMM_EPI_NONE>
__global__ __launch_bounds__(256) void gemm_mfma_rs_kernel(GemmParams p, int m_off, int tiles_m, int tiles_n) {
  constexpr int BM = 256, BN = 256, BK = 64, TM = 4, TN = 4;
  extern __shared__ __align__(16) unsigned char smem[];
  int rb = 0, mlive = p.M;
  if (LIVE) {
    if (p.grp_n > 0) {                                   // the live row tiles of all groups, one group after the other
      int total = 0;
      for (int e = 0; e < p.grp_n; e++) total += (p.grp_off[e + 1] - p.grp_off[e] + BM - 1) / BM;
      tiles_m = min(tiles_m, total);
    } else {
      int mmax;
      mlive = gemm_rows(p, m_off, rb, mmax);
      tiles_m = min(tiles_m, (max(mlive, 0) + BM - 1) / BM);
    }
  }
  int nblk = tiles_m * tiles_n, pid = blockIdx.x;
  int khalf = -1;                                        // >= 0: this workgroup computes one half of the contraction of a tail tile
  if (!LIVE && EPI == GEMM_EPI_NONE && p.tail_first >= 0 && pid >= p.tail_first) { khalf = (pid - p.tail_first) & 1; pid = p.tail_first + ((pid - p.tail_first) >> 1); }
  if (pid >= nblk) return;
  int q8 = nblk / 8, rem = nblk % 8, xcd = pid % 8, loc = pid / 8;
  int logical = xcd * q8 + min(xcd, rem) + loc;
  // the 32 workgroups an XCD runs at a time cover 4 row tiles x 8 column tiles: the row panels (activations, read from
  // HBM the first time) are the expensive L2 misses, the column panels (weights, hot in the memory-side cache because
  // every XCD reads them) the cheap ones; measured against 8 x 4: +2..6 %, against 16 x 2: +14 %
  constexpr int GROUP = 4;
  int in_group = GROUP * tiles_n, grp = logical / in_group, first_m = grp * GROUP;
  int gsize = min(tiles_m - first_m, GROUP);
  int tile_m = first_m + (logical % in_group) % gsize, tile_n = (logical % in_group) / gsize;
  int b_group = 0;
  if (LIVE && p.grp_n > 0) {                             // which group this row tile belongs to, and which of its tiles it is
    int e = 0, rows_e = p.grp_off[1] - p.grp_off[0], nt_e = (rows_e + BM - 1) / BM;
    while (tile_m >= nt_e && e + 1 < p.grp_n) {
      tile_m -= nt_e; e++;
      rows_e = p.grp_off[e + 1] - p.grp_off[e]; nt_e = (rows_e + BM - 1) / BM;
    }
    rb = p.grp_off[e]; mlive = rows_e; b_group = e;
  }
  const int row_lo = rb + tile_m * BM, row_hi = rb + mlive;                  // LIVE: the rows this tile writes
  const int row0 = LIVE ? min(row_lo, (p.grp_off ? p.rows_cap : p.M) - BM) : tile_m * BM, col0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, l31 = lane & 31, hh = lane >> 5, lrow = lane >> 3, lch = lane & 7;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int nt0 = p.seg[0].K / BK, nt = nt0 + (p.nseg > 1 ? p.seg[1].K / BK : 0);
  const GemmSeg s0 = p.seg[0], s1 = p.nseg > 1 ? p.seg[1] : p.seg[0];
  int64_t k_skip = 0;                                    // elements of segment 0 this workgroup starts behind
  if (khalf >= 0) {                                      // first half: steps [0, nt / 2) of segment 0; second half: the rest of it and segment 1
    const int sp = nt / 2;                               // the launcher made sure that sp <= nt0
    if (khalf == 0) { nt0 = sp; nt = sp; } else { k_skip = (int64_t)sp * BK; nt0 -= sp; nt -= sp; }
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  if (nt > 0) {
    // per-lane addresses of the loop, handed over through this lane's 64-byte line of LDS scratch
    const int x7 = (l31 >> 1) & 7;
    u32x4 line[4];
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
      const unsigned c = (unsigned)(((2 * ks + hh) ^ x7) * 16);
      line[0][ks] = (unsigned)((wm * 128 + l31) * 128) + c;                    // fragment reads of A
      line[1][ks] = 65536u + (unsigned)((wn * 128 + l31) * 128) + c;           // ... of B
    }
    const unsigned wrow = (unsigned)((wave * 64 + lrow) * 128);
    line[2][0] = wrow + (unsigned)((lch ^ (lrow >> 1)) * 16);                  // LDS stores, even / odd load
    line[2][1] = wrow + (unsigned)((lch ^ ((lrow >> 1) | 4)) * 16);
    line[2][2] = line[2][0] + 65536u; line[2][3] = line[2][1] + 65536u;
    line[3][0] = (unsigned)((lrow * s0.lda + lch * 8) * 2); line[3][1] = (unsigned)((lrow * s0.ldb + lch * 8) * 2);
    line[3][2] = (unsigned)((lrow * s1.lda + lch * 8) * 2); line[3][3] = (unsigned)((lrow * s1.ldb + lch * 8) * 2);
    u32x4* scratch = reinterpret_cast<u32x4*>(smem + 131072 + tid * 64);
#pragma unroll
    for (int i = 0; i < 4; i++) scratch[i] = line[i];
    const unsigned scratch_addr = 131072u + (unsigned)tid * 64u;
    // wave-uniform operand bases: first of the wave's 64 rows of the tile, first K step
    const bf16_t* b0p = (const bf16_t*)s0.B + (int64_t)b_group * p.grp_b_stride; const bf16_t* b1p = (const bf16_t*)s1.B;
    int colg = col0, a2off = 0;
    if (p.ncg > 0) {                                     // which weight matrix this column tile belongs to
      int cgi = 0;
      while (cgi + 1 < p.ncg && col0 >= p.cg_end[cgi]) cgi++;
      colg = col0 - (cgi ? p.cg_end[cgi - 1] : 0);
      b0p = (const bf16_t*)p.cg_B1[cgi]; b1p = (const bf16_t*)(p.nseg > 1 ? p.cg_B2[cgi] : p.cg_B1[cgi]); a2off = p.nseg > 1 ? p.cg_a2[cgi] : 0;
    }
    const uint64_t A0 = (uint64_t)((const bf16_t*)s0.A + (int64_t)(row0 + wave * 64) * s0.lda + k_skip);
    const uint64_t B0 = (uint64_t)(b0p + (int64_t)(colg + wave * 64) * s0.ldb + k_skip);
    const uint64_t A1 = (uint64_t)((const bf16_t*)s1.A + a2off + (int64_t)(row0 + wave * 64) * s1.lda);
    const uint64_t B1 = (uint64_t)(b1p + (int64_t)(colg + wave * 64) * s1.ldb);
    const int sA0 = (int)(16 * s0.lda), sB0 = (int)(16 * s0.ldb), sA1 = (int)(16 * s1.lda), sB1 = (int)(16 * s1.ldb);   // 8 rows, bytes
    asm volatile(GEMM_RS_LOOP_ASM
                 : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]),
                   "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]),
                   "+a"(acc[2][0]), "+a"(acc[2][1]), "+a"(acc[2][2]), "+a"(acc[2][3]),
                   "+a"(acc[3][0]), "+a"(acc[3][1]), "+a"(acc[3][2]), "+a"(acc[3][3])
                 : "v"(scratch_addr), "s"(A0), "s"(B0), "s"(A1), "s"(B1), "s"(sA0), "s"(sB0), "s"(sA1), "s"(sB1), "s"(nt0), "s"(nt)
                 : GEMM_RS_LOOP_CLOBBERS);
  }
  // bf16 results with 16-byte rows leave through LDS (whole 256-byte row pieces per store), the rest row by row
  if (!LIVE && EPI == GEMM_EPI_NONE && khalf >= 0) {     // raw float sums of this half into the tile's scratch
    GemmParams q = p;
    q.C = p.tail_part + ((int64_t)(pid - p.tail_first) * 2 + khalf) * (BM * BN); q.ldc = BN; q.c_f32 = 1; q.alpha = 1.f; q.R = nullptr; q.accumulate = 0;
    gemm_epilogue_rows<TM, TN, false>(q, acc, wm * TM * 32 + l31, wn * TN * 32 + 4 * hh);
    return;
  }
  if constexpr (EPI == GEMM_EPI_STATS) { gemm_epilogue_stats<TM, TN, LIVE != 0>(p, acc, row0 + wm * TM * 32 + l31, (col0 + wn * TN * 32) / 128, hh, row_lo, row_hi); return; }
  if constexpr (EPI == GEMM_EPI_PROB) { gemm_epilogue_staged<TM, TN, LIVE != 0, true>(p, acc, smem, wave, lane, row0 + wm * TM * 32, col0 + wn * TN * 32, row_lo, row_hi); return; }
  const bool staged = !p.c_f32 && !(p.ldc % 8) && (!p.R || (!(p.ldr % 8) && !((uintptr_t)p.R % 16)));
  if (staged) gemm_epilogue_staged<TM, TN, LIVE != 0>(p, acc, smem, wave, lane, row0 + wm * TM * 32, col0 + wn * TN * 32, row_lo, row_hi);
  else gemm_epilogue_rows<TM, TN, LIVE != 0>(p, acc, row0 + wm * TM * 32 + l31, col0 + wn * TN * 32 + 4 * hh, row_lo, row_hi);
}

template <int BM, int BN, int WM, int WN>
static int launch_dlds_cfg(as_ctx* ctx, const GemmParams& p, int m_off, hipStream_t st) {
  size_t smem = (size_t)2 * (BM + BN) * 64 * sizeof(bf16_t);
  auto k0 = gemm_mfma_dlds_kernel<BM, BN, WM, WN>;
  AS_SET_SMEM(ctx, k0, smem);
  int tm = (int)cdiv(p.M, BM), tn = (int)cdiv(p.N, BN);
  dim3 grid(tm * tn, p.splitk > 1 ? p.splitk : 1);
  k0<<<grid, WM * WN * 64, smem, st>>>(p, m_off, tm, tn);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// Second launch for the tiles of a split last round: sum of the two halves (first half first), then the usual epilogue.
// Four workgroups per tile (64 rows each: a last round is at most 128 tiles), the same workgroup -> tile mapping as the
// main kernel; a thread owns 4 consecutive columns.
__global__ __launch_bounds__(256) void gemm_tail_fixup_kernel(GemmParams p, int tiles_m, int tiles_n) {
  constexpr int BM = 256, BN = 256, GROUP = 4;
  const int tile = blockIdx.x >> 2, r_first = (blockIdx.x & 3) * (BM / 4);
  const int nblk = tiles_m * tiles_n, pid = p.tail_first + tile;
  if (pid >= nblk) return;
  const int q8 = nblk / 8, rem = nblk % 8, xcd = pid % 8, loc = pid / 8;
  const int logical = xcd * q8 + min(xcd, rem) + loc;
  const int in_group = GROUP * tiles_n, grp = logical / in_group, first_m = grp * GROUP;
  const int gsize = min(tiles_m - first_m, GROUP);
  const int tile_m = first_m + (logical % in_group) % gsize, tile_n = (logical % in_group) / gsize;
  const float* h0 = p.tail_part + (int64_t)tile * 2 * (BM * BN); const float* h1 = h0 + BM * BN;
  const int c = (threadIdx.x & 63) * 4;
  for (int r = r_first + (threadIdx.x >> 6); r < r_first + BM / 4; r += 4) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(h0 + r * BN + c), b = *reinterpret_cast<const f32x4*>(h1 + r * BN + c);
    const int64_t row = (int64_t)tile_m * BM + r; const int col = tile_n * BN + c;
    f32x4 v;
#pragma unroll
    for (int k = 0; k < 4; k++) v[k] = p.alpha * (a[k] + b[k]);
    if (p.R) { const bf16x4_t x = *reinterpret_cast<const bf16x4_t*>((const bf16_t*)p.R + row * p.ldr + col);
#pragma unroll
      for (int k = 0; k < 4; k++) v[k] += (float)x[k]; }
    if (p.c_f32) {
      f32x4* q = reinterpret_cast<f32x4*>((float*)p.C + row * p.ldc + col);
      if (p.accumulate) { const f32x4 o = *q;
#pragma unroll
        for (int k = 0; k < 4; k++) v[k] += o[k]; }
      *q = v;
    } else {
      bf16x4_t w;
#pragma unroll
      for (int k = 0; k < 4; k++) w[k] = (bf16_t)v[k];
      *reinterpret_cast<bf16x4_t*>((bf16_t*)p.C + row * p.ldc + col) = w;
    }
  }
}

// whole 256 x 256 tiles of a plain launch (host-side row count, no split-K, K segments in 64-wide steps, 16-byte rows)
static bool rs_ok(const GemmParams& p) {
  if (p.splitk > 1 || p.M < 256 || (p.N % 256)) return false;
  if (p.grp_off && p.rows_cap < 256) return false;       // grouped rows: the caller states how many rows the operands have
  if (p.grp_n > 0 && (p.nseg != 1 || p.m_dev)) return false;
  // the epilogue stores four consecutive columns of a row at a time
  if ((p.ldc % 4) || ((uintptr_t)p.C % 16) || (p.R && ((p.ldr % 4) || ((uintptr_t)p.R % 8)))) return false;
  for (int s = 0; s < p.nseg; s++)
    if ((p.seg[s].K % 64) || p.seg[s].K < 64 || p.seg[s].lda * 16 > INT32_MAX || p.seg[s].ldb * 16 > INT32_MAX) return false;
  int nt = 0; for (int s = 0; s < p.nseg; s++) nt += (int)(p.seg[s].K / 64);
  return nt >= 1;
}

static bool rs_live(const GemmParams& p) { return p.m_dev || p.grp_off; }
static bool mfma_ok(const GemmParams& p);
bool gemm_rs_applies(int mode, const GemmParams& p) { return mode == AS_BF16 && mfma_ok(p) && rs_ok(p); }

static int launch_rs_cfg(as_ctx* ctx, const GemmParams& p_in, int m_off, hipStream_t st) {
  GemmParams p = p_in;
  constexpr size_t smem = 131072 + 256 * 64;             // two stages of A and B tiles + a 64-byte line per lane (the staged epilogue: 4 x 128 rows of 272 bytes)
  AS_SET_SMEM(ctx, gemm_mfma_rs_kernel<0>, smem);
  AS_SET_SMEM(ctx, gemm_mfma_rs_kernel<1>, smem);
  AS_SET_SMEM(ctx, (gemm_mfma_rs_kernel<1, GEMM_EPI_STATS>), smem);
  AS_SET_SMEM(ctx, (gemm_mfma_rs_kernel<1, GEMM_EPI_PROB>), smem);
  const int tn = p.N / 256;
  if (p.epi != GEMM_EPI_NONE && !p.m_dev) return as_fail(ctx, AS_ERR_SHAPE, "gemm: the head epilogues run over a device-side row count");
  if (rs_live(p)) {                                      // every row tile the live rows can reach; the kernel drops the rest
    const int tm = p.grp_n > 0 ? (int)cdiv(p.rows_cap, 256) + p.grp_n : (int)cdiv(p.M, 256);
    if (p.epi == GEMM_EPI_STATS) gemm_mfma_rs_kernel<1, GEMM_EPI_STATS><<<dim3(tm * tn), 256, smem, st>>>(p, m_off, tm, tn);
    else if (p.epi == GEMM_EPI_PROB) gemm_mfma_rs_kernel<1, GEMM_EPI_PROB><<<dim3(tm * tn), 256, smem, st>>>(p, m_off, tm, tn);
    else gemm_mfma_rs_kernel<1><<<dim3(tm * tn), 256, smem, st>>>(p, m_off, tm, tn);
  } else {
    // whole row tiles only: the ragged last one too when the operands have the rows, else the caller handles the rest
    const int tm = p.rows_cap >= (int)cdiv(p.M, 256) * 256 ? (int)cdiv(p.M, 256) : p.M / 256;
    // Split the contraction of the last partial round's tiles over two workgroups each when that round would leave at
    // least half of the CUs idle, the launch has full rounds before it (short launches keep one summation order with the
    // other kernels) and the contraction is long enough to be worth a second small launch.
    const int T = tm * tn, cus = 256, full = T / cus * cus, rest = T - full;
    const int nt0 = (int)(p.seg[0].K / 64), nt = nt0 + (p.nseg > 1 ? (int)(p.seg[1].K / 64) : 0);
    p.tail_first = -1;
    if (p.tail_part && p.epi == GEMM_EPI_NONE && full > 0 && rest > 0 && rest <= 128 && nt >= 32 && nt / 2 <= nt0) p.tail_first = full;
    else p.tail_part = nullptr;
    gemm_mfma_rs_kernel<0><<<dim3(p.tail_first >= 0 ? full + 2 * rest : T), 256, smem, st>>>(p, 0, tm, tn);
    if (p.tail_first >= 0) { AS_LAUNCH_CHECK(ctx); gemm_tail_fixup_kernel<<<dim3(4 * rest), 256, 0, st>>>(p, tm, tn); }
  }
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

template <int BM, int BN, int WM, int WN>
static int launch_mfma_cfg(as_ctx* ctx, const GemmParams& p, int m_off, hipStream_t st) {
  constexpr int LS = 72;
  size_t smem = (size_t)2 * (BM + BN) * LS * sizeof(bf16_t);
  bool edge = false;
  for (int s = 0; s < p.nseg; s++) edge = edge || (p.seg[s].K % 64 != 0);
  auto k0 = gemm_mfma_kernel<BM, BN, WM, WN, false>;
  auto k1 = gemm_mfma_kernel<BM, BN, WM, WN, true>;
  AS_SET_SMEM(ctx, k0, smem);
  AS_SET_SMEM(ctx, k1, smem);
  int tm = (int)cdiv(p.M, BM), tn = (int)cdiv(p.N, BN);
  dim3 grid(tm * tn, p.splitk > 1 ? p.splitk : 1);
  if (edge) k1<<<grid, WM * WN * 64, smem, st>>>(p, m_off, tm, tn);
  else k0<<<grid, WM * WN * 64, smem, st>>>(p, m_off, tm, tn);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

static bool mfma_ok(const GemmParams& p) {
  if (p.R && (p.ldr % 1)) return false;
  for (int s = 0; s < p.nseg; s++) {
    const GemmSeg& g = p.seg[s];
    if (g.K % 8 || g.lda % 8 || g.ldb % 8) return false;
    if (((uintptr_t)g.A | (uintptr_t)g.B) % 16) return false;
  }
  return true;
}

// Tile configuration of the MFMA kernels.  Register-staged (any K that is a multiple of 8): 0 = 256x256 (8 waves,
// 128x64 each), 1 = 256x64, 2 = 64x256, 3 = 128x128, 4 = 128x64.  20 = direct-to-LDS 256x256 with 8 waves (K in 64-wide steps);
// 24 = the hand-scheduled register-staged 256x256 kernel with 4 waves.
static int pick_cfg(const GemmParams& p) {
  // narrow outputs (the adapters' rank-wide products) stream A once at HBM speed: 128 x 128 tiles measured 2-33 % ahead of
  // 256 x 64 here (58,880 rows; N = 128: 121 against 181 us, where two 64-wide column tiles read A twice); up to 64
  // columns a 128 x 64 tile loads half the B rows per step (a CU's load path carries A and B alike): 3-6 % ahead
  if (p.N <= 64 && p.M > 128) return 4;
  if (p.N <= 128 && p.M > 128) return 3;
  if (p.M <= 128) return 2;
  if ((int64_t)cdiv(p.M, 256) * cdiv(p.N, 256) * p.splitk < 128) return 3;
  // The hand-scheduled register-staged kernel is ahead on every shape it covers (9-13 % on the shapes of an 8B model)
  if (rs_ok(p)) return 24;
  return 20;                                             // direct-to-LDS tiles when K allows, else staged (0)
}

// m_dev semantics: the live row count is *m_dev - m_off (clamped to [0, M]).
// variant: 0 pick, 1 plain FMA kernel, 2 MFMA kernel with the default tile choice, 10 + c forces tile configuration c.
int launch_gemm_off(as_ctx* ctx, int mode, int variant, const GemmParams& p_in, int m_off, hipStream_t st) {
  GemmParams p = p_in;
  if (p.M <= 0 || p.N <= 0) return AS_OK;
  if (p.nseg < 1 || p.nseg > 2) return as_fail(ctx, AS_ERR_SHAPE, "gemm: 1 or 2 K segments");
  if (p.splitk < 1) p.splitk = 1;
  if (p.splitk > 1 && !p.partial) return as_fail(ctx, AS_ERR_WORKSPACE, "gemm: split-K needs a partial buffer");
  if (p.accumulate && !p.c_f32) return as_fail(ctx, AS_ERR_SHAPE, "gemm: accumulate needs float output");
  if (p.grp_off && p.splitk > 1) return as_fail(ctx, AS_ERR_SHAPE, "gemm: grouped rows and split-K do not combine");
  if (p.grp_n > 0) {
    if (!p.grp_off || p.nseg != 1 || p.m_dev || m_off) return as_fail(ctx, AS_ERR_SHAPE, "gemm: all groups in one launch need a group table and one K segment");
    const int c0 = variant >= 10 ? variant - 10 : pick_cfg(p);
    if (!(mode == AS_BF16 && variant != 1 && mfma_ok(p) && c0 == 24 && rs_ok(p))) {       // one launch per group
      const size_t esz = mode == AS_BF16 ? 2 : 4;
      for (int e = 0; e < p.grp_n; e++) {
        GemmParams q = p; q.grp_n = 0; q.grp = e; q.grp_rows = p.grp_rows / p.grp_n;
        q.seg[0].B = (const char*)p.seg[0].B + (size_t)e * p.grp_b_stride * esz;
        const int rc1 = launch_gemm_off(ctx, mode, variant, q, 0, st);
        if (rc1) return rc1;
      }
      return AS_OK;
    }
  }
  if (p.epi != GEMM_EPI_NONE) {
    if (!gemm_rs_applies(mode, p) || variant == 1 || (variant >= 10 && variant != 34)) return as_fail(ctx, AS_ERR_SHAPE, "gemm: the head epilogues need the hand-scheduled kernel (bf16, N a multiple of 256, K in 64-wide steps)");
    if (p.epi == GEMM_EPI_STATS && !p.epi_part) return as_fail(ctx, AS_ERR_NULL, "gemm: statistics epilogue without a buffer");
    if (p.epi == GEMM_EPI_PROB && (!p.epi_lse || !p.epi_lab || (!p.epi_w && !p.epi_cnt) || p.c_f32 || p.R || (p.ldc % 8))) return as_fail(ctx, AS_ERR_SHAPE, "gemm: probability epilogue needs lse, labels, a row factor and bf16 output");
  }
  if (p.ncg > 0) {
    if (p.ncg > 3 || p.grp_off || p.m_dev || p.splitk > 1 || p.cg_end[p.ncg - 1] != p.N) return as_fail(ctx, AS_ERR_SHAPE, "gemm: column groups need plain rows and ends that add up to N");
    bool fused = mode == AS_BF16 && variant != 1 && mfma_ok(p) && (variant >= 10 ? variant - 10 : pick_cfg(p)) == 24 && rs_ok(p) &&
                 p.rows_cap >= (int)cdiv(p.M, 256) * 256;      // the hand-scheduled kernel over every row tile
    for (int g = 0; g < p.ncg && fused; g++) fused = p.cg_end[g] % 256 == 0 && !((uintptr_t)p.cg_B1[g] % 16) && (p.nseg < 2 || !((uintptr_t)p.cg_B2[g] % 16));
    if (!fused) {                                        // one launch per group
      const size_t esz = mode == AS_BF16 ? 2 : 4;
      for (int g = 0, c0 = 0; g < p.ncg; c0 = p.cg_end[g], g++) {
        GemmParams q = p; q.ncg = 0; q.N = p.cg_end[g] - c0;
        q.seg[0].B = p.cg_B1[g];
        if (p.nseg > 1) { q.seg[1].B = p.cg_B2[g]; q.seg[1].A = (const char*)p.seg[1].A + (size_t)p.cg_a2[g] * esz; }
        q.C = (char*)p.C + (size_t)c0 * (p.c_f32 ? 4 : esz);
        if (p.R) q.R = (const char*)p.R + (size_t)c0 * esz;
        const int rc1 = launch_gemm_off(ctx, mode, variant, q, m_off, st);
        if (rc1) return rc1;
      }
      return AS_OK;
    }
  }
  if (variant < 0 || (variant > 2 && variant != 10 && variant != 11 && variant != 12 && variant != 13 && variant != 14 && variant != 30 && variant != 34)) return as_fail(ctx, AS_ERR_SHAPE, "gemm: unknown variant");
  bool use_mfma = (mode == AS_BF16) && variant != 1 && mfma_ok(p);
  if (variant >= 2 && !use_mfma) return as_fail(ctx, AS_ERR_SHAPE, "gemm: MFMA kernel needs bf16 and 8-element alignment");
  int rc = AS_OK;
  double ksum = 0; for (int s = 0; s < p.nseg; s++) ksum += p.seg[s].K;
  int cfg = variant >= 10 ? variant - 10 : pick_cfg(p);
  if (p.epi != GEMM_EPI_NONE) cfg = 24;                    // only the hand-scheduled kernel has those epilogues (checked above)
  if (cfg >= 20) for (int s = 0; s < p.nseg; s++) if (p.seg[s].K % 64) cfg = 0;     // direct-to-LDS tiles need whole 64-wide K steps
  const bool big = use_mfma && (cfg == 0 || cfg >= 20);
  const bool rs = use_mfma && cfg == 24 && rs_ok(p) && !rs_live(p) && !m_off;     // live-row launches keep their own timing classes
  prof_begin(ctx, st, rs ? AS_K_GEMM_RS : p.grp_off ? AS_K_GEMM_GROUPED : p.m_dev ? AS_K_GEMM_DEVROWS : !use_mfma ? AS_K_GEMM_FMA : big ? AS_K_GEMM_MFMA_256 : AS_K_GEMM_MFMA_SKINNY,
             p.grp_off ? 2.0 * p.grp_rows * p.N * ksum : p.m_dev ? 0.0 : 2.0 * p.M * p.N * ksum);
  if (use_mfma) {
    switch (cfg) {
      case 1: rc = launch_mfma_cfg<256, 64, 4, 1>(ctx, p, m_off, st); break;
      case 2: rc = launch_mfma_cfg<64, 256, 1, 4>(ctx, p, m_off, st); break;
      case 3: rc = launch_mfma_cfg<128, 128, 2, 2>(ctx, p, m_off, st); break;
      case 4: rc = launch_mfma_cfg<128, 64, 2, 2>(ctx, p, m_off, st); break;
      case 20: rc = launch_dlds_cfg<256, 256, 2, 4>(ctx, p, m_off, st); break;
      case 24: {                                           // whole row tiles by the register-staged kernel, the ragged rest by the default one
        if (!rs_ok(p) || (m_off && !p.m_dev)) { rc = launch_dlds_cfg<256, 256, 2, 4>(ctx, p, m_off, st); break; }
        rc = launch_rs_cfg(ctx, p, m_off, st);
        if (rs_live(p)) break;                             // covers its ragged tiles itself
        const int done = p.rows_cap >= (int)cdiv(p.M, 256) * 256 ? p.M : p.M / 256 * 256;
        if (!rc && done < p.M) {
          GemmParams t = p;
          t.M = p.M - done;
          for (int s = 0; s < t.nseg; s++) t.seg[s].A = (const bf16_t*)t.seg[s].A + (int64_t)done * t.seg[s].lda;
          t.C = t.c_f32 ? (void*)((float*)t.C + (int64_t)done * t.ldc) : (void*)((bf16_t*)t.C + (int64_t)done * t.ldc);
          if (t.R) t.R = (const bf16_t*)t.R + (int64_t)done * t.ldr;
          rc = launch_dlds_cfg<256, 256, 2, 4>(ctx, t, 0, st);
        }
        break; }
      default: rc = launch_mfma_cfg<256, 256, 2, 4>(ctx, p, m_off, st); break;
    }
  } else {
    dim3 grid((unsigned)cdiv(p.N, 64), (unsigned)cdiv(p.M, 64), (unsigned)p.splitk);
    if (mode == AS_FP32) gemm_fma_kernel<float><<<grid, 256, 0, st>>>(p, m_off);
    else gemm_fma_kernel<bf16_t><<<grid, 256, 0, st>>>(p, m_off);
    AS_LAUNCH_CHECK(ctx);
  }
  prof_end(ctx, st);
  if (rc) return rc;
  if (p.splitk > 1) {
    if (!p.c_f32) return as_fail(ctx, AS_ERR_SHAPE, "gemm: split-K writes float output");
    rc = launch_splitk_reduce(ctx, p.partial, p.splitk, (int64_t)p.M * p.N, p.N, p.alpha, (float*)p.C, p.ldc, st);
  }
  return rc;
}

int launch_gemm(as_ctx* ctx, int mode, int variant, const GemmParams& p, hipStream_t st) {
  return launch_gemm_off(ctx, mode, variant, p, 0, st);
}

// ------------------------------------------------- matrix-core peak probe
// Register-resident MFMA loop: no memory traffic at all, eight independent accumulators per
// wavefront, two wavefronts per SIMD.  What this sustains is the ceiling any GEMM on the chip can
// reach at the clocks the part holds under matrix load.
__global__ __launch_bounds__(512) void mfma_peak_kernel(int iters, float* sink) {
  bf16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; j++) { a[j] = (bf16_t)(0.001f * (threadIdx.x + j)); b[j] = (bf16_t)(0.002f * (threadIdx.x - j)); }
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[i][e] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++) s += acc[i][0] + acc[i][15];
  if (s == 123.456f) sink[0] = s;          // never true; keeps the loop alive
}

int launch_mfma_peak(as_ctx* ctx, int iters, int blocks, float* sink, hipStream_t st) {
  mfma_peak_kernel<<<blocks, 512, 0, st>>>(iters, sink);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

// ------------------------------------------------ global -> LDS feed probe
// Every wavefront keeps K 1-KB direct-to-LDS loads in flight, waits for them, and repeats, walking a
// region of `span` bytes (power of two).  With a span that fits L2 this measures the L2 -> LDS path,
// with a larger one the MALL / HBM mix.  A 256x256x64 bf16 GEMM tile step needs 64 KB per CU.
template <int K>
__global__ __launch_bounds__(512) void feed_probe_kernel(const char* src, size_t span_mask, int iters, int* sink) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t base = (size_t)blockIdx.x * 7919u * 65536u;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < K; i++) {
      const size_t off = (base + ((size_t)it * 8 * K + wave * K + i) * 1024 + lane * 16) & span_mask;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + off),
                                       (__attribute__((address_space(3))) void*)(smem + (wave * K + i) * 1024), 16, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __builtin_amdgcn_s_barrier();
  }
  if (iters < 0 && smem[threadIdx.x] == 123) sink[0] = 1;
}

int launch_feed_probe(as_ctx* ctx, int k, const void* buf, size_t span, int iters, int blocks, int* sink, hipStream_t st) {
  const size_t mask = (span - 1) & ~(size_t)15;
#define FEED(K) { AS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(feed_probe_kernel<K>), hipFuncAttributeMaxDynamicSharedMemorySize, 8 * K * 1024)); \
                  feed_probe_kernel<K><<<blocks, 512, 8 * K * 1024, st>>>((const char*)buf, mask, iters, sink); }
  switch (k) { case 1: FEED(1) break; case 2: FEED(2) break; case 4: FEED(4) break; case 8: FEED(8) break;
               default: return as_fail(ctx, AS_ERR_SHAPE, "feed probe: loads in flight per wave must be 1, 2, 4 or 8"); }
#undef FEED
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}
