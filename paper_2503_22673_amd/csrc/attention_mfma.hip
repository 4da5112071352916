// Flash-style varlen causal attention on the matrix cores (bf16 in, fp32
// accumulate), head_dim 64 or 128, grouped KV heads.
//
// Orientation.  Scores are produced transposed, S^T = K Q^T, so that in the
// accumulator layout of v_mfma_f32_32x32x16_bf16 a lane owns ONE query (its
// column) and 16 keys (its registers): the running max / sum of the online
// softmax are per-lane scalars plus one exchange between the two lane halves,
// and the probabilities, rounded to bf16, are already laid out as the B
// operand of the next product O^T = V^T P^T (contraction over the keys a lane
// holds).  The same holds in the backward kernels for dS.  The operand that is
// contracted over its row index (V in forward; K, Q, dO in backward) is taken
// from a token-major copy ([column][token], made by a transpose pass right
// before the launch) so that its fragments are two 8-byte LDS reads.
//
// Tiles are cut on the flat token stream (64 keys per step); a query t sees
// key u iff seg_start[t] <= u <= t, equivalently u <= t < seg_end[u], so no
// tile logic depends on where trajectories begin.
//
// Backward is split in two kernels so that every gradient has one owner and
// is summed in a fixed order: dQ per query tile (loop over key tiles), dK/dV
// per key tile (loop over the query heads of the group, then query tiles).
#include "common.h"
#include <type_traits>

namespace {

constexpr int BKEY = 64;      // keys (or queries) per staged tile
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
// v_exp_f32 without the denormal-range fix-up of exp2f: arguments here are <= 0 or masked to -inf
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int e = 0; e < 16; e++) z[e] = 0.f;
  return z;
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int sl) {
  bf16x8 v;
#pragma unroll
  for (int j = 0; j < 8; j++) v[j] = (bf16_t)a[8 * sl + j];
  return v;
}

// ------------------------------------------------------------------ forward
//  * K and V^T tiles go from global memory straight into LDS (no staging registers, no store pass), two
//    stages deep, so a step costs one barrier; rows are unpadded and the 16-byte chunks of a row are
//    XOR-swizzled with the row index so that fragment reads stay spread over the banks;
//  * the causal / segment mask is evaluated only on tiles that touch the diagonal or a segment start
//    (a wave-uniform test), every other tile takes a mask-free path;
//  * the 1/sqrt(d) log2(e) factor is folded into the exponent's fused multiply-add;
//  * the running maximum is only raised when a tile exceeds it by more than 2^8 (the accumulators are
//    float, the probabilities stay below 256), so rescaling the output accumulators is rare and sits
//    behind a wave-uniform branch.
template <int ROWBYTES> __device__ __forceinline__ int swz_row(int row) { return ROWBYTES == 256 ? (row & 15) : ((row >> 1) & 7); }

// [ROWS][COLS] bf16 tile -> LDS, 1 KB per wave instruction.  The per-lane part of the addresses (row inside the tile,
// swizzled chunk) is computed once per kernel (tile_offsets); a tile load is then a wave-uniform base, advanced with
// scalar arithmetic, plus those 32-bit offsets.  Computing the addresses afresh for every tile cost about 140 vector
// instructions per tile and wave, as many cycles of the vector unit as the softmax itself.
template <int ROWS, int COLS, int NW> struct TileShape {
  static constexpr int CPR = COLS / 8, RPL = 64 / CPR, NL = ROWS / RPL, PER = NL / NW;
  static_assert(NL % NW == 0, "tile rows must split evenly over the waves");
};
template <typename T> __device__ __forceinline__ const T* uniform_ptr(const T* ptr) {
  const uint64_t v = (uint64_t)ptr;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const T*)(((uint64_t)hi << 32) | lo);
}
template <int ROWS, int COLS, int NW>
__device__ __forceinline__ void tile_offsets(int64_t ld, int wave, int lane, uint32_t (&voff)[TileShape<ROWS, COLS, NW>::PER]) {
  using S = TileShape<ROWS, COLS, NW>;
#pragma unroll
  for (int i = 0; i < S::PER; i++) {
    const int w = wave * S::PER + i;
    const int row = w * S::RPL + lane / S::CPR, c = lane % S::CPR;
    voff[i] = (uint32_t)((row * ld + ((c ^ swz_row<COLS * 2>(row)) * 8)) * 2);      // bytes; the launcher keeps tiles under 4 GB
  }
}
// tile whose first element is `tile` (wave-uniform), every row in bounds
template <int ROWS, int COLS, int NW>
__device__ __forceinline__ void tile_to_lds_fast(const bf16_t* tile, const uint32_t (&voff)[TileShape<ROWS, COLS, NW>::PER], bf16_t* s, int wave) {
  using S = TileShape<ROWS, COLS, NW>;
  const char* b = (const char*)uniform_ptr(tile);
#pragma unroll
  for (int i = 0; i < S::PER; i++)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(b + voff[i]),
                                     (__attribute__((address_space(3))) void*)(s + (wave * S::PER + i) * 512), 16, 0, 0);
}
// row-major tensor, tile rows row0 .. row0 + ROWS - 1; rows past row_max (only the last tile of the stream has any) are clamped
template <int ROWS, int COLS, int NW>
__device__ __forceinline__ void tile_to_lds(const bf16_t* base, int64_t ld, int row0, int row_max, const uint32_t (&voff)[TileShape<ROWS, COLS, NW>::PER],
                                            bf16_t* s, int wave, int lane) {
  using S = TileShape<ROWS, COLS, NW>;
  if (row0 + ROWS - 1 <= row_max) { tile_to_lds_fast<ROWS, COLS, NW>(base + (int64_t)row0 * ld, voff, s, wave); return; }
#pragma unroll
  for (int i = 0; i < S::PER; i++) {
    const int w = wave * S::PER + i;
    const int row = w * S::RPL + lane / S::CPR, c = lane % S::CPR;
    const bf16_t* src = base + (int64_t)min(row0 + row, row_max) * ld + ((c ^ swz_row<COLS * 2>(row)) * 8);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(s + w * 512), 16, 0, 0);
  }
}

// Wave = QB blocks of 32 queries of one head; workgroup = HPW heads x (NWV / HPW) query groups, NWV = 8 / QB waves.
// QB = 1 keeps a wave under 256 registers, so two waves share a SIMD and one's softmax runs under the other's MFMAs.
// Workgroups go to the eight XCDs round-robin by linear index, and each XCD has an L2 of its own.  The work
// items of a launch form `ngrp` groups (a head or a group of heads) of `per` items each; the items of a
// group stream the same operand tiles, so a whole group is kept on one XCD: XCD x takes the groups x, x + 8, ...
// one after the other, each in the order given (longest first).  Without a multiple of eight groups the
// mapping falls back to group-major order.
__device__ inline void xcd_group_map(int wg, int per, int ngrp, int& group, int& item) {
  if (ngrp % 8 == 0) { const int slot = wg >> 3; group = (slot / per) * 8 + (wg & 7); item = slot % per; }
  else { group = wg / per; item = wg % per; }
}

template <int DH, int HPW, int QB, int NWV>
__global__ __launch_bounds__(NWV * 64, QB == 1 ? 2 : 1) void attn_fwd2_mfma(AttnParams p, float sl2) {
  constexpr int KS = DH / 16, CB = DH / 32, WQ = 32 * QB, QT = WQ * (NWV / HPW);
  constexpr int KT_E = BKEY * DH, ST_E = 2 * KT_E;        // elements of one tile / of one stage (K tile + V^T tile)
  extern __shared__ __align__(16) unsigned char dyn_smem[];
  bf16_t* sm = (bf16_t*)dyn_smem;
  const int tid = threadIdx.x, lane = tid & 63, l31 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform values stay in scalar registers and branches on them are real branches
  const int n = p.n, grp = p.Hq / p.Hkv;
  int hg, qi;
  const int nqt = (n + QT - 1) / QT;
  xcd_group_map(blockIdx.x, nqt, p.Hq / HPW, hg, qi);
  const int j = hg * HPW + (wave % HPW), g = j / grp;
  const int t_wg = (p.order_q ? p.order_q[qi] : nqt - 1 - qi) * QT;   // long rows first
  const int t_base = t_wg + (wave / HPW) * WQ;
  const bf16_t* Q = (const bf16_t*)p.q; const bf16_t* K = (const bf16_t*)p.k; const bf16_t* VT = (const bf16_t*)p.vT;

  bf16x8 qf[QB][KS];
  int tq[QB], ss[QB];
#pragma unroll
  for (int qb = 0; qb < QB; qb++) {
    tq[qb] = t_base + qb * 32 + l31;
    int tc = min(tq[qb], n - 1);
    ss[qb] = p.seg_start[tc];
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
      qf[qb][ks] = *reinterpret_cast<const bf16x8*>(Q + (int64_t)tc * p.ldq + j * DH + ks * 16 + h * 8);
  }
  const int ss_hi = __builtin_amdgcn_readfirstlane(p.seg_start[min(t_base + WQ - 1, n - 1)]);  // the latest segment start any query of this wave has
  f32x16 o[QB][CB];
  float mref[QB], l[QB];
#pragma unroll
  for (int qb = 0; qb < QB; qb++) { mref[qb] = -INFINITY; l[qb] = 0.f;
#pragma unroll
    for (int cb = 0; cb < CB; cb++) o[qb][cb] = zero16(); }

  const int kv_first = __builtin_amdgcn_readfirstlane(p.seg_start[min(t_wg, n - 1)] / BKEY);
  const int kv_last = min(t_wg + QT - 1, n - 1) / BKEY;
  uint32_t offR[TileShape<BKEY, DH, NWV>::PER], offT[TileShape<DH, BKEY, NWV>::PER];
  tile_offsets<BKEY, DH, NWV>(p.ldkv, wave, lane, offR); tile_offsets<DH, BKEY, NWV>(p.ldT, wave, lane, offT);
  auto stage = [&](int kt, int b) {
    tile_to_lds<BKEY, DH, NWV>(K + g * DH, p.ldkv, kt * BKEY, n - 1, offR, sm + b * ST_E, wave, lane);
    tile_to_lds_fast<DH, BKEY, NWV>(VT + (int64_t)g * DH * p.ldT + kt * BKEY, offT, sm + b * ST_E + KT_E, wave);
  };
  const int swK = swz_row<DH * 2>(l31), swV = swz_row<128>(l31);
  stage(kv_first, 0);
  for (int kt = kv_first; kt <= kv_last; kt++) {
    const int b = (kt - kv_first) & 1;
    __builtin_amdgcn_s_waitcnt(0x0f70);      // this wave's part of tile kt has landed
    __syncthreads();                         // ... everyone's has, and everyone is done with tile kt-1
    if (kt < kv_last) stage(kt + 1, b ^ 1);
    const int k0 = kt * BKEY;
    if (k0 > t_base + WQ - 1 || t_base >= n) continue;          // tile lies after every query of this wave
    const bf16_t* sK = sm + b * ST_E; const bf16_t* sVt = sK + KT_E;
    f32x16 s[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; qb++) { s[qb][0] = zero16(); s[qb][1] = zero16(); }
    // fragments are read PFD MFMA steps ahead of their use (LDS latency is several MFMA times)
    constexpr int PFD = 6, NQK = 2 * KS, NPV = 4 * CB;
    auto kfrag = [&](int i) { const int ks = i >> 1, kb = i & 1;
      return *reinterpret_cast<const bf16x8*>(sK + (kb * 32 + l31) * DH + (((ks * 2 + h) ^ swK) * 8)); };
    auto vfrag = [&](int i) { const int x = i / CB, cb = i % CB;   // quad-swapped token order: chunk 2x + h of the row holds this lane half's 8 keys
      return *reinterpret_cast<const bf16x8*>(sVt + (cb * 32 + l31) * BKEY + (((2 * x + h) ^ swV) * 8)); };
    {
      bf16x8 kq[PFD];
#pragma unroll
      for (int i = 0; i < PFD; i++) kq[i] = kfrag(i);
#pragma unroll
      for (int i = 0; i < NQK; i++) {
        const bf16x8 a = kq[i % PFD];
        if (i + PFD < NQK) kq[i % PFD] = kfrag(i + PFD);
#pragma unroll
        for (int qb = 0; qb < QB; qb++) s[qb][i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][i >> 1], s[qb][i & 1], 0, 0, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, PFD, 0);
#pragma unroll
      for (int i = 0; i < NQK - PFD; i++) {
        __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, PFD * QB, 0);
    }
    bf16x8 vq[PFD];                                          // the first V fragments do not depend on the softmax
#pragma unroll
    for (int i = 0; i < PFD; i++) vq[i] = vfrag(i);
    const bool full = (k0 + 63 <= t_base) && (k0 >= ss_hi);  // every key of the tile is visible to every query of the wave
    bf16x8 pb[QB][4];
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
      if (!full) {
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int e = 0; e < 16; e++) {
            int key = k0 + kb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
            s[qb][kb][e] = (key >= ss[qb] && key <= tq[qb]) ? s[qb][kb][e] : -INFINITY;
          }
      }
      float mx = s[qb][0][0];
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int e = 0; e < 16; e++) mx = fmaxf(mx, s[qb][kb][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sl2;
      const bool raise = mx > mref[qb] + 8.f;
      if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        const float m_new = raise ? mx : mref[qb];
        const float alpha = raise ? fast_exp2(mref[qb] - m_new) : 1.f;
        mref[qb] = m_new;
        l[qb] *= alpha;
#pragma unroll
        for (int cb = 0; cb < CB; cb++)
#pragma unroll
          for (int e = 0; e < 16; e++) o[qb][cb][e] *= alpha;
      }
      const float neg_m = (mref[qb] == -INFINITY) ? 0.f : -mref[qb];
      float rs = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int e = 0; e < 16; e++) { float pv = fast_exp2(fmaf(s[qb][kb][e], sl2, neg_m)); s[qb][kb][e] = pv; rs += pv; }
      rs += __shfl_xor(rs, 32, 64);
      l[qb] += rs;
#pragma unroll
      for (int kb = 0; kb < 2; kb++) { pb[qb][kb * 2] = pack8(s[qb][kb], 0); pb[qb][kb * 2 + 1] = pack8(s[qb][kb], 1); }
    }
#pragma unroll
    for (int i = 0; i < NPV; i++) {                          // i = x * CB + cb, x = kb*2 + sl: 16 keys each
      const bf16x8 a = vq[i % PFD];
      if (i + PFD < NPV) vq[i % PFD] = vfrag(i + PFD);
#pragma unroll
      for (int qb = 0; qb < QB; qb++) o[qb][i % CB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][i / CB], o[qb][i % CB], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NPV - PFD; i++) {
      __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, PFD * QB, 0);
  }
  bf16_t* O = (bf16_t*)p.o;
#pragma unroll
  for (int qb = 0; qb < QB; qb++) {
    if (tq[qb] >= n) continue;
    float inv = 1.f / l[qb];
    bf16_t* orow = O + ((int64_t)tq[qb] * p.Hq + j) * DH;
#pragma unroll
    for (int cb = 0; cb < CB; cb++)
#pragma unroll
      for (int b4 = 0; b4 < 4; b4++) {
        bf16x4 w;
#pragma unroll
        for (int i = 0; i < 4; i++) w[i] = (bf16_t)(o[qb][cb][b4 * 4 + i] * inv);
        *reinterpret_cast<bf16x4*>(orow + cb * 32 + 8 * b4 + 4 * h) = w;
      }
    if (h == 0) p.lse[(int64_t)tq[qb] * p.Hq + j] = (mref[qb] + log2f(l[qb])) * 0.6931471805599453f;
  }
}

// Stores a lane's column of a transposed [head_dim x tokens] accumulator block as one bf16 row of dh values, scaled; with
// rotary tables the row is first rotated back by the token's position (component i pairs with i + dh / 2; both sit in the
// same lane, CB / 2 accumulator blocks apart), so that the gradient is rounded once, after the rotation.
template <int DH>
__device__ __forceinline__ void store_grad_row(const f32x16 (&acc)[DH / 32], float scale, bf16_t* row, int h, const float* rc, const float* rs, int pos) {
  constexpr int CB = DH / 32, HB = CB / 2;
  if (rc) {
    const float* c0 = rc + (int64_t)pos * (DH / 2); const float* s0 = rs + (int64_t)pos * (DH / 2);
#pragma unroll
    for (int cb = 0; cb < HB; cb++)
#pragma unroll
      for (int b4 = 0; b4 < 4; b4++) {
        const int i0 = cb * 32 + 8 * b4 + 4 * h;
        const f32x4 c = *reinterpret_cast<const f32x4*>(c0 + i0), sn = *reinterpret_cast<const f32x4*>(s0 + i0);
        bf16x4 w1, w2;
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const float x1 = acc[cb][b4 * 4 + i] * scale, x2 = acc[cb + HB][b4 * 4 + i] * scale;
          w1[i] = (bf16_t)(x1 * c[i] + x2 * sn[i]);
          w2[i] = (bf16_t)(x2 * c[i] - x1 * sn[i]);
        }
        *reinterpret_cast<bf16x4*>(row + i0) = w1;
        *reinterpret_cast<bf16x4*>(row + DH / 2 + i0) = w2;
      }
    return;
  }
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int b4 = 0; b4 < 4; b4++) {
      bf16x4 w;
#pragma unroll
      for (int i = 0; i < 4; i++) w[i] = (bf16_t)(acc[cb][b4 * 4 + i] * scale);
      *reinterpret_cast<bf16x4*>(row + cb * 32 + 8 * b4 + 4 * h) = w;
    }
}

// ---------------------------------------------------------- backward: delta
__global__ void attn_delta_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ d_o, int64_t rows, int dh,
                                  float* __restrict__ delta) {
  int64_t r = (int64_t)blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
  int lane = threadIdx.x & 63;
  if (r >= rows) return;
  float acc = 0.f;
  for (int c = lane; c < dh; c += 64) acc += (float)o[r * dh + c] * (float)d_o[r * dh + c];
  acc = wave_sum(acc);
  if (lane == 0) delta[r] = acc;
}

// the same with 16 bytes per lane: DH / 8 neighbouring lanes share a row (DH / 8 a power of two, at most 64)
template <int DH>
__global__ __launch_bounds__(256) void attn_delta_vec_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ d_o, int64_t rows,
                                                             float* __restrict__ delta) {
  constexpr int LPR = DH / 8;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x, r = t / LPR;
  float acc = 0.f;
  if (r < rows) {
    const u32x4 a = *reinterpret_cast<const u32x4*>(o + t * 8), b = *reinterpret_cast<const u32x4*>(d_o + t * 8);
#pragma unroll
    for (int k = 0; k < 4; k++)                          // a bf16 is the upper half of a float
      acc += __uint_as_float(a[k] << 16) * __uint_as_float(b[k] << 16) + __uint_as_float(a[k] & 0xffff0000u) * __uint_as_float(b[k] & 0xffff0000u);
  }
#pragma unroll
  for (int off = 1; off < LPR; off <<= 1) acc += __shfl_xor(acc, off);
  if (r < rows && (threadIdx.x & (LPR - 1)) == 0) delta[r] = acc;
}

template <int DH>
static void launch_delta(const AttnParams& p, int64_t rows, hipStream_t st) {
  constexpr int LPR = DH / 8;
  if constexpr (DH % 8 == 0 && (LPR & (LPR - 1)) == 0 && LPR <= 64) {
    if (!((uintptr_t)p.o % 16) && !((uintptr_t)p.d_o % 16)) {
      attn_delta_vec_kernel<DH><<<(unsigned)cdiv(rows * LPR, 256), 256, 0, st>>>((const bf16_t*)p.o, (const bf16_t*)p.d_o, rows, p.delta);
      return;
    }
  }
  attn_delta_kernel<<<(unsigned)cdiv(rows, 4), 256, 0, st>>>((const bf16_t*)p.o, (const bf16_t*)p.d_o, rows, DH, p.delta);
}

// ----------------------------------------------- backward, second generation
// Same split and orientation as the kernels above, with the changes of attn_fwd2_mfma: tiles straight
// into LDS, two stages, one barrier per step; token-major copies in quad-swapped order (16-byte fragment
// reads); mask only on tiles that touch the diagonal or a segment boundary; scale folded into the
// exponent's multiply-add.
template <int DH, int HPW>
__global__ __launch_bounds__(512) void attn_bwd_dq2_mfma(AttnParams p, float scale, float sl2) {
  constexpr int KS = DH / 16, CB = DH / 32, NWV = 8, QT = 32 * (NWV / HPW);
  constexpr int KT_E = BKEY * DH, ST_E = 3 * KT_E;        // K tile, V tile, K^T tile
  extern __shared__ __align__(16) unsigned char dyn_smem[];
  bf16_t* sm = (bf16_t*)dyn_smem;
  const int tid = threadIdx.x, lane = tid & 63, l31 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = p.n, grp = p.Hq / p.Hkv;
  int hg, qi;
  const int nqt = (n + QT - 1) / QT;
  xcd_group_map(blockIdx.x, nqt, p.Hq / HPW, hg, qi);
  const int j = hg * HPW + (wave % HPW), g = j / grp;
  const int t_wg = (p.order_q ? p.order_q[qi] : nqt - 1 - qi) * QT;   // long rows first
  const int t_base = t_wg + (wave / HPW) * 32;
  const bf16_t* Q = (const bf16_t*)p.q; const bf16_t* K = (const bf16_t*)p.k; const bf16_t* V = (const bf16_t*)p.v;
  const bf16_t* dO = (const bf16_t*)p.d_o; const bf16_t* KT = (const bf16_t*)p.kT;
  const int tq = t_base + l31, tc = min(tq, n - 1), ss = p.seg_start[tc];
  bf16x8 qf[KS], dof[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    qf[ks] = *reinterpret_cast<const bf16x8*>(Q + (int64_t)tc * p.ldq + j * DH + ks * 16 + h * 8);
    dof[ks] = *reinterpret_cast<const bf16x8*>(dO + ((int64_t)tc * p.Hq + j) * DH + ks * 16 + h * 8);
  }
  const float neg_lse2 = -p.lse[(int64_t)tc * p.Hq + j] * 1.4426950408889634f;
  const float dl = p.delta[(int64_t)tc * p.Hq + j];
  const int ss_hi = __builtin_amdgcn_readfirstlane(p.seg_start[min(t_base + 31, n - 1)]);
  f32x16 dq[CB];
#pragma unroll
  for (int cb = 0; cb < CB; cb++) dq[cb] = zero16();

  const int kv_first = __builtin_amdgcn_readfirstlane(p.seg_start[min(t_wg, n - 1)] / BKEY);
  const int kv_last = min(t_wg + QT - 1, n - 1) / BKEY;
  uint32_t offR[TileShape<BKEY, DH, NWV>::PER], offT[TileShape<DH, BKEY, NWV>::PER];
  tile_offsets<BKEY, DH, NWV>(p.ldkv, wave, lane, offR); tile_offsets<DH, BKEY, NWV>(p.ldT, wave, lane, offT);
  auto stage = [&](int kt, int b) {
    bf16_t* d = sm + b * ST_E;
    tile_to_lds<BKEY, DH, NWV>(K + g * DH, p.ldkv, kt * BKEY, n - 1, offR, d, wave, lane);
    tile_to_lds<BKEY, DH, NWV>(V + g * DH, p.ldkv, kt * BKEY, n - 1, offR, d + KT_E, wave, lane);
    tile_to_lds_fast<DH, BKEY, NWV>(KT + (int64_t)g * DH * p.ldT + kt * BKEY, offT, d + 2 * KT_E, wave);
  };
  const int swK = swz_row<DH * 2>(l31), swT = swz_row<128>(l31);
  stage(kv_first, 0);
  for (int kt = kv_first; kt <= kv_last; kt++) {
    const int b = (kt - kv_first) & 1;
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();
    if (kt < kv_last) stage(kt + 1, b ^ 1);
    const int k0 = kt * BKEY;
    if (k0 > t_base + 31 || t_base >= n) continue;
    const bf16_t* sK = sm + b * ST_E; const bf16_t* sV = sK + KT_E; const bf16_t* sKt = sK + 2 * KT_E;
    f32x16 s[2], dp[2];
    s[0] = zero16(); s[1] = zero16(); dp[0] = zero16(); dp[1] = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
        const int off = (kb * 32 + l31) * DH + (((ks * 2 + h) ^ swK) * 8);
        bf16x8 a = *reinterpret_cast<const bf16x8*>(sK + off);
        bf16x8 bb = *reinterpret_cast<const bf16x8*>(sV + off);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
        dp[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb, dof[ks], dp[kb], 0, 0, 0);
      }
    if (!((k0 + 63 <= t_base) && (k0 >= ss_hi))) {          // the tile touches the diagonal or a segment start
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          int key = k0 + kb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
          s[kb][e] = (key >= ss && key <= tq) ? s[kb][e] : -INFINITY;
        }
    }
    bf16x8 dsb[4];
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
#pragma unroll
      for (int e = 0; e < 16; e++) s[kb][e] = fast_exp2(fmaf(s[kb][e], sl2, neg_lse2)) * (dp[kb][e] - dl);
      dsb[kb * 2] = pack8(s[kb], 0); dsb[kb * 2 + 1] = pack8(s[kb], 1);
    }
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
      for (int cb = 0; cb < CB; cb++) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(sKt + (cb * 32 + l31) * BKEY + (((2 * x + h) ^ swT) * 8));
        dq[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsb[x], dq[cb], 0, 0, 0);
      }
  }
  if (tq < n) store_grad_row<DH>(dq, scale, (bf16_t*)p.dq + (int64_t)tq * p.ldq + j * DH, h, p.rope_cos, p.rope_sin, tq - ss);
}

// Wave = 32 keys of one KV head (a lane owns one key), workgroup = 8 waves = 256 keys and ONE query head of
// the group; loops over 64-query tiles.  With several query heads per KV head each launch
// writes float partials [query head][token][dh] that a second pass sums in head order: one workgroup
// looping over all heads of the group would be several times longer than the average workgroup, and the
// launch as long as its longest workgroup.  dK and dV come from two launches (WHICH = 0: dK,
// needs S, dP and the dK product; WHICH = 1: dV, needs S and the dV product): with both sets of
// accumulators in one wave the kernel needs more than 256 registers, which costs the second wave per
// SIMD and a stream of accumulator-register copies; recomputing S in a second launch is cheaper.
template <int DH, int WHICH>
__global__ __launch_bounds__(512) void attn_bwd_dkv2_mfma(AttnParams p, float scale, float sl2, float* __restrict__ part) {
  constexpr int KS = DH / 16, CB = DH / 32, NWV = 8, KPB = 32 * NWV;
  constexpr int KT_E = BKEY * DH;
  constexpr bool DO_K = WHICH != 1, DO_V = WHICH != 0;    // WHICH 2: both gradients from one S (head_dim 64: the registers allow it)
  constexpr int NT = (DO_K ? 3 : 1) + (DO_V ? 1 : 0);     // dK: Q, dO, Q^T tiles; dV: Q, dO^T tiles; both: Q, dO, Q^T, dO^T
  constexpr int ST_E = NT * KT_E + 4 * BKEY;              // + 64 lse and 64 delta floats (2 bf16 slots each)
  extern __shared__ __align__(16) unsigned char dyn_smem[];
  bf16_t* sm = (bf16_t*)dyn_smem;
  const int tid = threadIdx.x, lane = tid & 63, l31 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = p.n, grp = p.Hq / p.Hkv;
  int jj, ki;
  xcd_group_map(blockIdx.x, (n + KPB - 1) / KPB, p.Hq, jj, ki);
  const int g = jj / grp;
  const int u_wg = (p.order_k ? p.order_k[ki] : ki) * KPB, u_base = u_wg + wave * 32;
  const bf16_t* Q = (const bf16_t*)p.q; const bf16_t* K = (const bf16_t*)p.k; const bf16_t* V = (const bf16_t*)p.v;
  const bf16_t* dO = (const bf16_t*)p.d_o; const bf16_t* QTm = (const bf16_t*)p.qT; const bf16_t* DOT = (const bf16_t*)p.doT;
  const int u = u_base + l31, uc = min(u, n - 1);
  const int uend = (u < n) ? p.seg_end[uc] : 0;                 // queries u <= t < uend see this key
  bf16x8 kf[KS], vf[DO_K ? KS : 1];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    kf[ks] = *reinterpret_cast<const bf16x8*>(K + (int64_t)uc * p.ldkv + g * DH + ks * 16 + h * 8);
    if constexpr (DO_K) vf[ks] = *reinterpret_cast<const bf16x8*>(V + (int64_t)uc * p.ldkv + g * DH + ks * 16 + h * 8);
  }
  f32x16 acc[CB], acc2[WHICH == 2 ? CB : 1];                    // dK^T or dV^T, [dh rows, key lane]; both: dK^T and dV^T
#pragma unroll
  for (int cb = 0; cb < CB; cb++) acc[cb] = zero16();
  if constexpr (WHICH == 2) {
#pragma unroll
    for (int cb = 0; cb < CB; cb++) acc2[cb] = zero16();
  }
  const int q_first = u_wg / BKEY;
  const int q_last = __builtin_amdgcn_readfirstlane((p.seg_end[min(u_wg + KPB - 1, n - 1)] - 1) / BKEY);
  // this wave's keys are visible from queries in [u_base, w_end); all of them from queries in [u_base + 31, w_end_min)
  const int w_end = (u_base < n) ? __builtin_amdgcn_readfirstlane(p.seg_end[min(u_base + 31, n - 1)]) : 0;
  const int w_end_min = (u_base < n) ? __builtin_amdgcn_readfirstlane(p.seg_end[min(u_base, n - 1)]) : 0;
  const int total = q_last - q_first + 1;
  // Query tiles are taken from the segment's end downwards: the workgroups of one head and segment that start
  // together then read the same tiles at the same time, whatever their own first tile is.
  uint32_t offQ[TileShape<BKEY, DH, NWV>::PER], offD[TileShape<BKEY, DH, NWV>::PER], offT[TileShape<DH, BKEY, NWV>::PER];
  tile_offsets<BKEY, DH, NWV>(p.ldq, wave, lane, offQ); tile_offsets<BKEY, DH, NWV>((int64_t)p.Hq * DH, wave, lane, offD);
  tile_offsets<DH, BKEY, NWV>(p.ldT, wave, lane, offT);
  auto stage = [&](int it, int b) {
    const int t0 = (q_last - it) * BKEY;
    bf16_t* d = sm + b * ST_E;
    tile_to_lds<BKEY, DH, NWV>(Q + jj * DH, p.ldq, t0, n - 1, offQ, d, wave, lane);
    if constexpr (DO_K) {
      tile_to_lds<BKEY, DH, NWV>(dO + jj * DH, (int64_t)p.Hq * DH, t0, n - 1, offD, d + KT_E, wave, lane);
      tile_to_lds_fast<DH, BKEY, NWV>(QTm + (int64_t)jj * DH * p.ldT + t0, offT, d + 2 * KT_E, wave);
    }
    if constexpr (DO_V) tile_to_lds_fast<DH, BKEY, NWV>(DOT + (int64_t)jj * DH * p.ldT + t0, offT, d + (NT - 1) * KT_E, wave);
    if (wave < (DO_K ? 2 : 1)) {                           // 64 lse (wave 0) and 64 delta (wave 1) values, 4 bytes a lane
      const float* src = (wave == 0 ? p.lse : p.delta) + (int64_t)min(t0 + lane, n - 1) * p.Hq + jj;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(d + NT * KT_E + wave * 2 * BKEY), 4, 0, 0);
    }
  };
  const int swR = swz_row<DH * 2>(l31), swT = swz_row<128>(l31);
  if (total > 0) stage(0, 0);
  for (int it = 0; it < total; it++) {
    const int b = it & 1;
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();
    if (it + 1 < total) stage(it + 1, b ^ 1);
    const int t0 = (q_last - it) * BKEY;
    if (t0 + 63 < u_base || t0 >= w_end) continue;             // no query of the tile sees a key of this wave
    const bf16_t* sQ = sm + b * ST_E;
    const bf16_t* sdO = sQ + KT_E;                              // with dK only
    const bf16_t* sT = sQ + (DO_K ? 2 : 1) * KT_E;              // Q^T (dK) or dO^T (dV)
    const bf16_t* sT2 = sQ + (NT - 1) * KT_E;                   // dO^T when both
    const float* sLse = (const float*)(sQ + NT * KT_E); const float* sDel = sLse + BKEY;
    f32x16 s[2], dp[DO_K ? 2 : 1];
    s[0] = zero16(); s[1] = zero16();
    if constexpr (DO_K) { dp[0] = zero16(); dp[1] = zero16(); }
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
#pragma unroll
      for (int qb = 0; qb < 2; qb++) {
        const int off = (qb * 32 + l31) * DH + (((ks * 2 + h) ^ swR) * 8);
        bf16x8 a = *reinterpret_cast<const bf16x8*>(sQ + off);
        s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[ks], s[qb], 0, 0, 0);
        if constexpr (DO_K) {
          bf16x8 bb = *reinterpret_cast<const bf16x8*>(sdO + off);
          dp[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb, vf[ks], dp[qb], 0, 0, 0);
        }
      }
    if (!((t0 >= u_base + 31) && (t0 + 63 < w_end_min))) {     // the tile touches the diagonal or a segment end
#pragma unroll
      for (int qb = 0; qb < 2; qb++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int t = t0 + qb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
          s[qb][e] = (t >= u && t < uend) ? s[qb][e] : -INFINITY;
        }
    }
    bf16x8 bop[4], bop2[WHICH == 2 ? 4 : 1];                    // dS (dK) or P (dV) as B operands; both: dS and P
#pragma unroll
    for (int qb = 0; qb < 2; qb++) {
#pragma unroll
      for (int b4 = 0; b4 < 4; b4++) {
        const int qi0 = qb * 32 + 8 * b4 + 4 * h;            // 4 consecutive queries: one 16-byte read each
        const f32x4 ls = *reinterpret_cast<const f32x4*>(&sLse[qi0]);
        f32x4 dl;
        if constexpr (DO_K) dl = *reinterpret_cast<const f32x4*>(&sDel[qi0]);
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const int e = b4 * 4 + i;
          const float pr = fast_exp2(fmaf(s[qb][e], sl2, -1.4426950408889634f * ls[i]));
          if constexpr (WHICH == 2) { dp[qb][e] = pr * (dp[qb][e] - dl[i]); s[qb][e] = pr; }
          else if constexpr (WHICH == 0) s[qb][e] = pr * (dp[qb][e] - dl[i]); else s[qb][e] = pr;
        }
      }
      if constexpr (WHICH == 2) {
        bop[qb * 2] = pack8(dp[qb], 0); bop[qb * 2 + 1] = pack8(dp[qb], 1);
        bop2[qb * 2] = pack8(s[qb], 0); bop2[qb * 2 + 1] = pack8(s[qb], 1);
      } else { bop[qb * 2] = pack8(s[qb], 0); bop[qb * 2 + 1] = pack8(s[qb], 1); }
    }
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
      for (int cb = 0; cb < CB; cb++) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(sT + (cb * 32 + l31) * BKEY + (((2 * x + h) ^ swT) * 8));
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bop[x], acc[cb], 0, 0, 0);
        if constexpr (WHICH == 2) {
          const bf16x8 a2 = *reinterpret_cast<const bf16x8*>(sT2 + (cb * 32 + l31) * BKEY + (((2 * x + h) ^ swT) * 8));
          acc2[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, bop2[x], acc2[cb], 0, 0, 0);
        }
      }
  }
  if (u >= n) return;
  auto put = [&](const f32x16 (&r)[CB], int which) {
    if (grp > 1) {
      float* row = part + (((int64_t)which * p.Hq + jj) * n + u) * DH;
#pragma unroll
      for (int cb = 0; cb < CB; cb++)
#pragma unroll
        for (int b4 = 0; b4 < 4; b4++) {
          f32x4 w;
#pragma unroll
          for (int i = 0; i < 4; i++) w[i] = r[cb][b4 * 4 + i];
          *reinterpret_cast<f32x4*>(row + cb * 32 + 8 * b4 + 4 * h) = w;
        }
    } else {
      bf16_t* row = (bf16_t*)(which == 0 ? p.dk : p.dv) + (int64_t)u * p.ldkv + g * DH;
      store_grad_row<DH>(r, which == 0 ? scale : 1.f, row, h, which == 0 ? p.rope_cos : nullptr, p.rope_sin, u - p.seg_start[u]);
    }
  };
  put(acc, WHICH == 1 ? 1 : 0);
  if constexpr (WHICH == 2) put(acc2, 1);
}

// dQ with one wave per SIMD (head_dim 128, four query heads per KV head): wave = 64 queries of one head (a lane owns two
// queries), workgroup = the 4 heads of a group on the same 64 tokens, so a K / V tile is staged once per group.  The
// dQ^T accumulators (128 registers) and the wave's Q and dO fragments (128) fill the accumulation half of the register
// file; a tile step is one generated instruction sequence (gen_attn_dq_tile.py -> attn_dq_tile.inc), one asm statement
// per loop trip.  K and V tiles sit in LDS once, row major, three stages deep; dQ^T += K^T dS^T reads K through the
// transposing LDS loads, so no token-major copy of K is needed.  Every wave issues eight loads per tile.
#include "attn_dq_tile.inc"
__global__ __launch_bounds__(256) void attn_bwd_dq3_mfma(AttnParams p, float scale, float sl2) {
  constexpr int DH = 128, KS = DH / 16, CB = DH / 32, QT = 64;
  constexpr int KT_B = BKEY * DH * 2, ST_B = 2 * KT_B;   // bytes of a tile, of a stage (K, V)
  extern __shared__ __align__(256) unsigned char dyn_smem256[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)dyn_smem256;
  if (lds0 & 255) return;                                       // never the case: the array is the kernel's only LDS
  const int tid = threadIdx.x, lane = tid & 63, l31 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = p.n, grp = p.Hq / p.Hkv;
  int hg, qi;
  const int nqt = (n + QT - 1) / QT;
  xcd_group_map(blockIdx.x, nqt, p.Hq / 4, hg, qi);
  const int j = hg * 4 + wave, g = j / grp;
  const int t_wg = (p.order_q ? p.order_q[qi] : nqt - 1 - qi) * QT;   // long rows first
  const bf16_t* Q = (const bf16_t*)p.q; const bf16_t* K = (const bf16_t*)p.k; const bf16_t* V = (const bf16_t*)p.v;
  const bf16_t* dO = (const bf16_t*)p.d_o;
  const int ss_hi = __builtin_amdgcn_readfirstlane(p.seg_start[min(t_wg + QT - 1, n - 1)]);
  f32x16 dq[2][CB];
#pragma unroll
  for (int qb = 0; qb < 2; qb++)
#pragma unroll
    for (int cb = 0; cb < CB; cb++) dq[qb][cb] = zero16();
  const int kv_first = __builtin_amdgcn_readfirstlane(p.seg_start[min(t_wg, n - 1)] / BKEY);
  const int kv_last = min(t_wg + QT - 1, n - 1) / BKEY;
  const int total = kv_last - kv_first + 1;
  // LDS position of chunk c of row r: c ^ f(r), f = the low four row bits in the order (1, 0, 2, 3)
  auto swz = [](int row) { return ((row & 3) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1); };
  const int l4 = lane >> 4, lc = lane & 15;
  const uint32_t off0 = (uint32_t)((((int64_t)(wave * 16 + l4)) * p.ldkv + ((lc ^ swz(l4)) * 8)) * 2);
  auto stage = [&](int it, int st) {                           // the loads of key tile kv_first + it, from here (first two tiles, ragged tiles)
    const int k0 = (kv_first + it) * BKEY;
    unsigned char* d = dyn_smem256 + st * ST_B;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int row = wave * 16 + 4 * i + l4, tok = min(k0 + row, n - 1), ch = (lc ^ swz(row)) * 8;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(K + (int64_t)tok * p.ldkv + g * DH + ch),
                                       (__attribute__((address_space(3))) void*)(d + (wave * 4 + i) * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int row = wave * 16 + 4 * i + l4, tok = min(k0 + row, n - 1), ch = (lc ^ swz(row)) * 8;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(V + (int64_t)tok * p.ldkv + g * DH + ch),
                                       (__attribute__((address_space(3))) void*)(d + KT_B + (wave * 4 + i) * 1024), 16, 0, 0);
    }
  };
  const int sl = lane & 15, mh = (lane >> 4) & 1, row0 = 4 * h + (sl >> 2);
  const uint32_t aR0 = lds0 + l31 * 256 + ((h ^ swz(l31)) * 16);
  const uint32_t aT0 = lds0 + row0 * 256 + (((2 * mh + ((sl & 3) >> 1)) ^ swz(row0)) * 16) + (sl & 1) * 8;
  if (total > 0) stage(0, 0);                                  // the first tiles travel while the wave fetches its own rows
  if (total > 1) stage(1, 1);
  int tq[2], ss[2];
  float nl2[2], dl[2];
  bf16x8 qf[2][KS], dof[2][KS];
#pragma unroll
  for (int qb = 0; qb < 2; qb++) {
    tq[qb] = t_wg + qb * 32 + l31;
    const int tc = min(tq[qb], n - 1);
    ss[qb] = p.seg_start[tc];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      qf[qb][ks] = *reinterpret_cast<const bf16x8*>(Q + (int64_t)tc * p.ldq + j * DH + ks * 16 + h * 8);
      dof[qb][ks] = *reinterpret_cast<const bf16x8*>(dO + ((int64_t)tc * p.Hq + j) * DH + ks * 16 + h * 8);
    }
    nl2[qb] = -p.lse[(int64_t)tc * p.Hq + j] * 1.4426950408889634f;
    dl[qb] = p.delta[(int64_t)tc * p.Hq + j];
  }
  int st = 0;
  for (int it = 0; it < total; it++) {
    if (it + 1 < total) __builtin_amdgcn_s_waitcnt(0x0f78); else __builtin_amdgcn_s_waitcnt(0x0f70);   // all but the next tile's eight loads
    __syncthreads();
    const int k0 = (kv_first + it) * BKEY;
    const int nx = it + 2, k0n = (kv_first + nx) * BKEY, stn = st == 0 ? 2 : st - 1;      // (it + 2) % 3
    const bool has = nx < total, fast = has && k0n + BKEY - 1 <= n - 1;
    if (has && !fast) stage(nx, stn);
    // 1: every query of the wave sees every key of the tile; 2: the tile touches the diagonal or a segment start
    const int kind = (k0 + 63 <= t_wg && k0 >= ss_hi) ? 1 : 2;
    const int mode = kind | (fast ? 4 : 0);
    const uint32_t sb = st * ST_B, sbn = stn * ST_B;
    const uint32_t aR = aR0 + sb, aT = aT0 + sb;
    const int tb0 = k0 + 4 * h - ss[0], tb1 = k0 + 4 * h - ss[1], lim0 = tq[0] - ss[0], lim1 = tq[1] - ss[1];
    const int k0c = has ? k0n : 0;
    const uint64_t gk = (uint64_t)(K + g * DH + (int64_t)k0c * p.ldkv), gv = (uint64_t)(V + g * DH + (int64_t)k0c * p.ldkv);
    const uint32_t str = (uint32_t)(4 * p.ldkv * 2);
    const uint32_t m0t = lds0 + sbn + wave * 4096;
    asm volatile(ATTN_DQ_TILE_ASM
                 : "+a"(dq[0][0]), "+a"(dq[0][1]), "+a"(dq[0][2]), "+a"(dq[0][3]), "+a"(dq[1][0]), "+a"(dq[1][1]), "+a"(dq[1][2]), "+a"(dq[1][3])
                 : "a"(qf[0][0]), "a"(qf[0][1]), "a"(qf[0][2]), "a"(qf[0][3]), "a"(qf[0][4]), "a"(qf[0][5]), "a"(qf[0][6]), "a"(qf[0][7]),
                   "a"(qf[1][0]), "a"(qf[1][1]), "a"(qf[1][2]), "a"(qf[1][3]), "a"(qf[1][4]), "a"(qf[1][5]), "a"(qf[1][6]), "a"(qf[1][7]),
                   "a"(dof[0][0]), "a"(dof[0][1]), "a"(dof[0][2]), "a"(dof[0][3]), "a"(dof[0][4]), "a"(dof[0][5]), "a"(dof[0][6]), "a"(dof[0][7]),
                   "a"(dof[1][0]), "a"(dof[1][1]), "a"(dof[1][2]), "a"(dof[1][3]), "a"(dof[1][4]), "a"(dof[1][5]), "a"(dof[1][6]), "a"(dof[1][7]),
                   "v"(aR), "v"(aT), "s"(sl2), "v"(nl2[0]), "v"(nl2[1]), "v"(dl[0]), "v"(dl[1]), "v"(tb0), "v"(tb1), "v"(lim0), "v"(lim1), "s"(mode),
                   "s"(gk), "s"(gv), "s"(str), "v"(off0), "s"(m0t)
                 : ATTN_DQ_TILE_CLOBBERS);
    st = st == 2 ? 0 : st + 1;
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");            // the accumulators are read next: wait states of the last MFMA
#pragma unroll
  for (int qb = 0; qb < 2; qb++)
    if (tq[qb] < n) store_grad_row<DH>(dq[qb], scale, (bf16_t*)p.dq + (int64_t)tq[qb] * p.ldq + j * DH, h, p.rope_cos, p.rope_sin, tq[qb] - ss[qb]);
}

// dK and dV in ONE pass (head_dim 128): S, the exponentials and dP are computed once, and the query heads of a KV head
// are taken one after the other into the same accumulators (head order, then tile order: a fixed summation order, no
// partial sums in memory).  Wave = 32 keys, workgroup = 4 waves = 128 keys, one wave per SIMD: both accumulator sets (2 x 64 registers) and the wave's K and V
// fragments sit in the accumulation half of the register file.  With one wave per SIMD only the wave's own instruction
// order can overlap matrix work, vector work and the arrival of the next tiles, so a tile step is one generated
// instruction sequence (gen_attn_dkv_tile.py -> attn_dkv_tile.inc: plain and masked, with and without the loads of the
// tile two steps ahead).  It is ONE asm statement per loop trip, so that the accumulators stay where they are between
// trips.  Q and dO tiles sit in LDS once, row major, three stages deep; the products that contract over the queries
// read them through the transposing LDS loads, so this kernel needs no token-major copy of Q or dO.
// Every wave issues nine loads per tile (four kilobytes of Q, four of dO, and the tile's lse values (even waves) or
// delta values (odd waves); those of waves 2 and 3 land in spare space), so that one count serves all waves.
#include "attn_dkv_tile.inc"
__global__ __launch_bounds__(256) void attn_bwd_dkv3_mfma(AttnParams p, float scale, float sl2) {
  constexpr int DH = 128, KS = DH / 16, CB = DH / 32, NWV = 4, KPB = 32 * NWV, NST = 3;
  constexpr int KT_B = BKEY * DH * 2;                     // bytes of a tile
  constexpr int ST_B = 2 * KT_B + 1024;                   // Q, dO, 64 lse, 64 delta floats, 512 spare bytes
  static_assert(ST_B % 256 == 0, "slice and column-block addresses are formed by XOR on a 256-byte aligned row address");
  extern __shared__ __align__(256) unsigned char dyn_smem256[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)dyn_smem256;
  if (lds0 & 255) return;                                       // never the case: the array is the kernel's only LDS
  const int tid = threadIdx.x, lane = tid & 63, l31 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = p.n, grp = p.Hq / p.Hkv;
  int g, ki;
  xcd_group_map(blockIdx.x, 2 * ((n + 255) / 256), p.Hkv, g, ki);
  const int u_wg = (p.order_k ? p.order_k[ki >> 1] * 2 + (ki & 1) : ki) * KPB, u_base = u_wg + wave * 32;
  if (u_wg >= n) return;                                        // the second half of a last, half-empty block of 256
  const bf16_t* Q = (const bf16_t*)p.q; const bf16_t* K = (const bf16_t*)p.k; const bf16_t* V = (const bf16_t*)p.v;
  const bf16_t* dO = (const bf16_t*)p.d_o;
  const int64_t ldo = (int64_t)p.Hq * DH;
  const int u = u_base + l31, uc = min(u, n - 1);
  const int uend = (u < n) ? p.seg_end[uc] : 0;                 // queries u <= t < uend see this key
  const int vis = (u < n) ? uend - u : 0;
  f32x16 accK[CB], accV[CB];                                    // dK^T and dV^T, [dh rows, key lane]
#pragma unroll
  for (int cb = 0; cb < CB; cb++) { accK[cb] = zero16(); accV[cb] = zero16(); }
  const int q_first = u_wg / BKEY;
  const int q_last = __builtin_amdgcn_readfirstlane((p.seg_end[min(u_wg + KPB - 1, n - 1)] - 1) / BKEY);
  const int w_end = (u_base < n) ? __builtin_amdgcn_readfirstlane(p.seg_end[min(u_base + 31, n - 1)]) : 0;
  const int w_end_min = (u_base < n) ? __builtin_amdgcn_readfirstlane(p.seg_end[min(u_base, n - 1)]) : 0;
  const int total = q_last - q_first + 1;                       // query tiles per head
  const int steps = total * grp;                                // the query heads of the group one after the other: step = (head, tile)
  // LDS position of chunk c of row r: c ^ f(r), f = the low four row bits in the order (1, 0, 2, 3)
  auto swz = [](int row) { return ((row & 3) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1); };
  // a load instruction of a wave fills one kilobyte = four rows; lane -> row lane / 16, position lane % 16
  const int l4 = lane >> 4, lc = lane & 15;
  const uint32_t offQ0 = (uint32_t)((((int64_t)(wave * 16 + l4)) * p.ldq + ((lc ^ swz(l4)) * 8)) * 2);
  const uint32_t offD0 = (uint32_t)((((int64_t)(wave * 16 + l4)) * ldo + ((lc ^ swz(l4)) * 8)) * 2);
  const float* stat = (wave & 1) ? p.delta : p.lse;             // this wave's ninth load
  auto stat_ptr = [&](int jj, int t0) { return stat + (int64_t)min(t0 + lane, n - 1) * p.Hq + jj; };
  auto stage = [&](int hh, int it, int st) {                   // the loads of tile `it` of head hh, from here (first two steps, ragged tiles)
    const int t0 = (q_last - it) * BKEY, jj = g * grp + hh;
    unsigned char* d = dyn_smem256 + st * ST_B;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int row = wave * 16 + 4 * i + l4, tok = min(t0 + row, n - 1), ch = (lc ^ swz(row)) * 8;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Q + (int64_t)tok * p.ldq + jj * DH + ch),
                                       (__attribute__((address_space(3))) void*)(d + (wave * 4 + i) * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int row = wave * 16 + 4 * i + l4, tok = min(t0 + row, n - 1), ch = (lc ^ swz(row)) * 8;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(dO + (int64_t)tok * ldo + jj * DH + ch),
                                       (__attribute__((address_space(3))) void*)(d + KT_B + (wave * 4 + i) * 1024), 16, 0, 0);
    }
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)stat_ptr(jj, t0),
                                     (__attribute__((address_space(3))) void*)(d + 2 * KT_B + wave * 256), 4, 0, 0);
  };
  // this lane's row in a tile (256-byte rows, chunk h: slice ks is that address XOR 32 ks); its corner of the
  // 4 row x 16 column patch of a transposing read (lanes 0..15 of a block: row s / 4, columns 4 (s % 4) ..; blocks:
  // columns 16 (b & 1) .., rows 4 (b / 2) ..; the column block is an XOR of 64 cb, rows 8.. an XOR of 16 plus 2048);
  // its four lse / delta values per eight queries
  const int sl = lane & 15, mh = (lane >> 4) & 1, row0 = 4 * h + (sl >> 2);
  const uint32_t aR0 = lds0 + l31 * 256 + ((h ^ swz(l31)) * 16);
  const uint32_t aT0 = lds0 + row0 * 256 + (((2 * mh + ((sl & 3) >> 1)) ^ swz(row0)) * 16) + (sl & 1) * 8;
  const uint32_t aL0 = lds0 + 2 * KT_B + 16 * h;
  if (steps > 0) stage(0, 0, 0);                               // the first tiles travel while the wave fetches its own rows
  if (steps > 1) { if (total > 1) stage(0, 1, 1); else stage(1, 0, 1); }
  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    kf[ks] = *reinterpret_cast<const bf16x8*>(K + (int64_t)uc * p.ldkv + g * DH + ks * 16 + h * 8);
    vf[ks] = *reinterpret_cast<const bf16x8*>(V + (int64_t)uc * p.ldkv + g * DH + ks * 16 + h * 8);
  }
  int st = 0, it = 0, hn = total > 2 ? 0 : (total == 2 ? 1 : 2), itn = total > 2 ? 2 : 0;   // (head, tile) of this step; of the step after next
  for (int step = 0; step < steps; step++) {
    if (step + 1 < steps) __builtin_amdgcn_s_waitcnt(0x0f79); else __builtin_amdgcn_s_waitcnt(0x0f70);   // all but the next step's nine loads
    __syncthreads();
    const int t0 = (q_last - it) * BKEY;
    const int t0n = (q_last - itn) * BKEY, stn = st == 0 ? 2 : st - 1;                     // stage (step + 2) % 3
    const bool has = step + 2 < steps, fast = has && t0n + BKEY - 1 <= n - 1;
    if (has && !fast) stage(hn, itn, stn);
    // 0: no query of the tile sees a key of this wave; 1: every query sees every key; 2: the tile touches the diagonal or a segment end
    const int kind = (t0 + 63 < u_base || t0 >= w_end) ? 0 : ((t0 >= u_base + 31) && (t0 + 63 < w_end_min)) ? 1 : 2;
    const int mode = kind | (fast ? 4 : 0);
    const uint32_t sb = st * ST_B, sbn = stn * ST_B;
    const uint32_t aR = aR0 + sb, aT = aT0 + sb, aL = aL0 + sb;
    const int tb = t0 + 4 * h - u;
    const int t0c = has ? t0n : 0;
    const int jn = g * grp + (has ? hn : 0);
    const uint64_t gq = (uint64_t)(Q + jn * DH + (int64_t)t0c * p.ldq), gd = (uint64_t)(dO + jn * DH + (int64_t)t0c * ldo);
    const uint32_t strq = (uint32_t)(4 * p.ldq * 2), strd = (uint32_t)(4 * ldo * 2);
    const uint32_t m0t = lds0 + sbn + wave * 4096, m0l = lds0 + sbn + 2 * KT_B + wave * 256;
    const uint64_t vl = (uint64_t)stat_ptr(jn, t0c);
    asm volatile(ATTN_DKV_TILE_ASM
                 : "+a"(accK[0]), "+a"(accK[1]), "+a"(accK[2]), "+a"(accK[3]), "+a"(accV[0]), "+a"(accV[1]), "+a"(accV[2]), "+a"(accV[3])
                 : "a"(kf[0]), "a"(kf[1]), "a"(kf[2]), "a"(kf[3]), "a"(kf[4]), "a"(kf[5]), "a"(kf[6]), "a"(kf[7]),
                   "a"(vf[0]), "a"(vf[1]), "a"(vf[2]), "a"(vf[3]), "a"(vf[4]), "a"(vf[5]), "a"(vf[6]), "a"(vf[7]),
                   "v"(aR), "v"(aT), "v"(aL), "s"(sl2), "v"(tb), "v"(vis), "s"(mode),
                   "s"(gq), "s"(gd), "s"(strq), "s"(strd), "v"(offQ0), "v"(offD0), "s"(m0t), "v"(vl), "s"(m0l)
                 : ATTN_DKV_TILE_CLOBBERS);
    st = st == 2 ? 0 : st + 1;
    if (++it == total) it = 0;
    if (++itn == total) { itn = 0; hn++; }
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");            // the accumulators are read next: wait states of the last MFMA
  if (u >= n) return;
  const int pos = u - p.seg_start[u];
  store_grad_row<DH>(accK, scale, (bf16_t*)p.dk + (int64_t)u * p.ldkv + g * DH, h, p.rope_cos, p.rope_sin, pos);
  store_grad_row<DH>(accV, 1.f, (bf16_t*)p.dv + (int64_t)u * p.ldkv + g * DH, h, nullptr, p.rope_sin, pos);
}

// dk[u, g, :] = scale * sum over the query heads of group g, in head order, of the dK partials; dv likewise (scale 1).
// With rotary tables dk is rotated back by the token's position before its one rounding: a thread then owns 4 columns
// i .. i + 3 of the lower half and their partners i + dh / 2.
__global__ void attn_dkv_reduce_kernel(const float* __restrict__ part, int n, int Hq, int Hkv, int dh, float scale,
                                       bf16_t* __restrict__ dk, bf16_t* __restrict__ dv, int64_t ldkv,
                                       const int32_t* __restrict__ seg_start, const float* __restrict__ rc, const float* __restrict__ rs) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;        // one thread: 4 columns of one (which, token, kv head)
  const int c4 = dh / 4, grp = Hq / Hkv;
  const int64_t per = (int64_t)n * Hkv * c4;
  if (idx >= 2 * per) return;
  const int which = (int)(idx / per);
  const int64_t r = idx % per;
  const int c = (int)(r % c4) * 4, g = (int)((r / c4) % Hkv);
  const int64_t u = r / ((int64_t)c4 * Hkv);
  auto sum4 = [&](int col) {
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int z = 0; z < grp; z++) sum += *reinterpret_cast<const f32x4*>(part + (((int64_t)which * Hq + g * grp + z) * n + u) * dh + col);
    return sum;
  };
  bf16x4 w;
  if (which == 0 && rc) {
    const int half = dh / 2;
    if (c >= half) return;                                  // the thread of column c also writes column c + dh / 2
    const f32x4 x1 = sum4(c), x2 = sum4(c + half);
    const int pos = (int)u - seg_start[u];
    const f32x4 cs = *reinterpret_cast<const f32x4*>(rc + (int64_t)pos * half + c), sn = *reinterpret_cast<const f32x4*>(rs + (int64_t)pos * half + c);
    bf16x4 w2;
#pragma unroll
    for (int i = 0; i < 4; i++) { w[i] = (bf16_t)(scale * (x1[i] * cs[i] + x2[i] * sn[i])); w2[i] = (bf16_t)(scale * (x2[i] * cs[i] - x1[i] * sn[i])); }
    *reinterpret_cast<bf16x4*>(dk + u * ldkv + g * dh + c) = w;
    *reinterpret_cast<bf16x4*>(dk + u * ldkv + g * dh + c + half) = w2;
    return;
  }
  const f32x4 sum = sum4(c);
  const float sc = which == 0 ? scale : 1.f;
#pragma unroll
  for (int i = 0; i < 4; i++) w[i] = (bf16_t)(sum[i] * sc);
  *reinterpret_cast<bf16x4*>((which == 0 ? dk : dv) + u * ldkv + g * dh + c) = w;
}

int heads_per_group(int grp) { return grp % 4 == 0 ? 4 : (grp % 2 == 0 ? 2 : 1); }
int heads_per_wg(const AttnParams& p) {
  int grp = p.Hq / p.Hkv;
  return grp % 4 == 0 ? 4 : (grp % 2 == 0 ? 2 : 1);
}

template <int DH, int HPW, int QB, int NWV = 8 / QB>
int launch_fwd2(as_ctx* ctx, const AttnParams& p_in, float sl2, hipStream_t st) {
  AttnParams p = p_in;
  if (32 * QB * (NWV / HPW) != attention_query_tile(p.Hq, p.Hkv)) p.order_q = nullptr;   // the order table is cut for another tile size
  constexpr size_t smem = (size_t)2 * 2 * BKEY * DH * sizeof(bf16_t);       // two stages of a K tile and a V^T tile
  AS_SET_SMEM(ctx, (attn_fwd2_mfma<DH, HPW, QB, NWV>), smem);
  constexpr int QT = 32 * QB * (NWV / HPW);
  attn_fwd2_mfma<DH, HPW, QB, NWV><<<(unsigned)(cdiv(p.n, QT) * (p.Hq / HPW)), NWV * 64, smem, st>>>(p, sl2);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

template <int DH>
int fwd_dh(as_ctx* ctx, const AttnParams& p_in, int variant, hipStream_t st) {
  AttnParams p = p_in;
  const int Np = (int)cdiv(p.n, 64) * 64, Dkv = p.Hkv * DH;
  if (!p.t_scratch) return as_fail(ctx, AS_ERR_WORKSPACE, "attention: the MFMA kernels need the token-major scratch buffer");
  p.ldT = Np; p.vT = p.t_scratch;
  int rc = launch_transpose_qs(ctx, AS_BF16, p.n, Np, Dkv, p.v, p.ldkv, p.t_scratch, Np, st);   // V^T [Dkv, Np]
  if (rc) return rc;
  const float sl2 = 1.4426950408889634f / sqrtf((float)DH);
  const int hpw = heads_per_wg(p);
  return hpw == 4 ? launch_fwd2<DH, 4, 1>(ctx, p, sl2, st) : hpw == 2 ? launch_fwd2<DH, 2, 1>(ctx, p, sl2, st) : launch_fwd2<DH, 1, 1>(ctx, p, sl2, st);
}

template <int DH, int HPW>
int launch_dq2(as_ctx* ctx, const AttnParams& p, float scale, float sl2, hipStream_t st) {
  constexpr size_t smem = (size_t)2 * 3 * BKEY * DH * sizeof(bf16_t);       // two stages of K, V and K^T tiles
  AS_SET_SMEM(ctx, (attn_bwd_dq2_mfma<DH, HPW>), smem);
  attn_bwd_dq2_mfma<DH, HPW><<<(unsigned)(cdiv(p.n, 32 * (8 / HPW)) * (p.Hq / HPW)), 512, smem, st>>>(p, scale, sl2);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

template <int DH, int WHICH>
int launch_dkv2(as_ctx* ctx, const AttnParams& p, float scale, float sl2, float* part, hipStream_t st) {
  constexpr size_t smem = (size_t)2 * ((WHICH == 0 ? 3 : WHICH == 1 ? 2 : 4) * BKEY * DH + 4 * BKEY) * sizeof(bf16_t);
  AS_SET_SMEM(ctx, (attn_bwd_dkv2_mfma<DH, WHICH>), smem);
  attn_bwd_dkv2_mfma<DH, WHICH><<<(unsigned)(cdiv(p.n, 256) * p.Hq), 512, smem, st>>>(p, scale, sl2, part);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_dq3(as_ctx* ctx, const AttnParams& p, float scale, float sl2, hipStream_t st) {
  constexpr size_t smem = (size_t)3 * 2 * BKEY * 128 * sizeof(bf16_t);      // three stages of a K and a V tile
  AS_SET_SMEM(ctx, attn_bwd_dq3_mfma, smem);
  attn_bwd_dq3_mfma<<<(unsigned)(cdiv(p.n, 64) * (p.Hq / 4)), 256, smem, st>>>(p, scale, sl2);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_dkv3(as_ctx* ctx, const AttnParams& p, float scale, float sl2, hipStream_t st) {
  constexpr size_t smem = (size_t)3 * (2 * BKEY * 128 * sizeof(bf16_t) + 1024);   // three stages of a Q and a dO tile, lse, delta
  AS_SET_SMEM(ctx, attn_bwd_dkv3_mfma, smem);
  attn_bwd_dkv3_mfma<<<(unsigned)(2 * cdiv(p.n, 256) * p.Hkv), 256, smem, st>>>(p, scale, sl2);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

template <int DH>
int bwd_dh(as_ctx* ctx, const AttnParams& p_in, int variant, hipStream_t st) {
  AttnParams p = p_in;
  const int Np = (int)cdiv(p.n, 64) * 64, Dkv = p.Hkv * DH, D = p.Hq * DH;
  if (!p.t_scratch) return as_fail(ctx, AS_ERR_WORKSPACE, "attention: the MFMA kernels need the token-major scratch buffer");
  bf16_t* ts = (bf16_t*)p.t_scratch;
  p.ldT = Np; p.kT = ts; p.qT = ts + (size_t)Dkv * Np; p.doT = ts + (size_t)(Dkv + D) * Np;
  int rc;
  const float scale = 1.f / sqrtf((float)DH), sl2 = 1.4426950408889634f * scale;
  const int64_t rows = (int64_t)p.n * p.Hq;
  {
    // one pass for dK and dV (head_dim 128, row strides a multiple of 256 bytes): reads Q and dO as they are
    const bool one_pass = DH == 128 && variant != 4 && p.ldq % 128 == 0;
    const int hpw = heads_per_wg(p);
    // dQ with one wave per SIMD: four query heads per KV head, K / V row strides a multiple of 256 bytes; reads K as it is
    const bool dq_one_wave = one_pass && hpw == 4 && p.ldkv % 128 == 0;
    if (!dq_one_wave && (rc = launch_transpose_qs(ctx, AS_BF16, p.n, Np, Dkv, p.k, p.ldkv, ts, Np, st))) return rc;           // K^T
    if (!one_pass) {
      if ((rc = launch_transpose_qs(ctx, AS_BF16, p.n, Np, D, p.q, p.ldq, ts + (size_t)Dkv * Np, Np, st))) return rc;       // Q^T
      if ((rc = launch_transpose_qs(ctx, AS_BF16, p.n, Np, D, p.d_o, D, ts + (size_t)(Dkv + D) * Np, Np, st))) return rc;   // dO^T
    }
    launch_delta<DH>(p, rows, st);
    AS_LAUNCH_CHECK(ctx);
    if (dq_one_wave) rc = launch_dq3(ctx, p, scale, sl2, st);
    else if (hpw == 4) rc = launch_dq2<DH, 4>(ctx, p, scale, sl2, st); else if (hpw == 2) rc = launch_dq2<DH, 2>(ctx, p, scale, sl2, st);
    else rc = launch_dq2<DH, 1>(ctx, p, scale, sl2, st);
    if (rc) return rc;
    float* part = (float*)(ts + (size_t)(Dkv + 2 * D) * Np);       // [2][Hq][n][dh] floats behind the token-major copies
    if (one_pass) return launch_dkv3(ctx, p, scale, sl2, st);     // sums over the query heads itself
    // head_dim 64: both gradients in one launch (S and the exponentials once); at head_dim 128 two waves per SIMD do not have the registers for it
    if constexpr (DH == 64) {
      if (variant != 4) { if ((rc = launch_dkv2<DH, 2>(ctx, p, scale, sl2, part, st))) return rc; }
      else if ((rc = launch_dkv2<DH, 0>(ctx, p, scale, sl2, part, st)) || (rc = launch_dkv2<DH, 1>(ctx, p, scale, sl2, part, st))) return rc;
    } else if ((rc = launch_dkv2<DH, 0>(ctx, p, scale, sl2, part, st)) || (rc = launch_dkv2<DH, 1>(ctx, p, scale, sl2, part, st))) return rc;
    if (p.Hq > p.Hkv) {
      const int64_t threads = 2 * (int64_t)p.n * p.Hkv * (DH / 4);
      attn_dkv_reduce_kernel<<<(unsigned)cdiv(threads, 256), 256, 0, st>>>(part, p.n, p.Hq, p.Hkv, DH, scale, (bf16_t*)p.dk, (bf16_t*)p.dv, p.ldkv,
                                                                             p.seg_start, p.rope_cos, p.rope_sin);
      AS_LAUNCH_CHECK(ctx);
    }
    return AS_OK;
  }
  return AS_OK;
}

}  // namespace

int attention_query_tile(int n_q_heads, int n_kv_heads) { return 32 * (8 / heads_per_group(n_q_heads / n_kv_heads)); }

bool attention_mfma_ok(const AttnParams& p) {
  if (p.dh != 64 && p.dh != 128) return false;
  if (p.ldq % 8 || p.ldkv % 8) return false;
  if (p.n > (1 << 23) || p.ldq > (1 << 24) || p.ldkv > (1 << 24)) return false;   // tile offsets are 32-bit byte counts
  uintptr_t a = (uintptr_t)p.q | (uintptr_t)p.k | (uintptr_t)p.v | (uintptr_t)p.o | (uintptr_t)p.d_o |
                (uintptr_t)p.dq | (uintptr_t)p.dk | (uintptr_t)p.dv;
  return a % 16 == 0;
}

int launch_attention_fwd_mfma(as_ctx* ctx, const AttnParams& p, int variant, hipStream_t st) {
  return p.dh == 128 ? fwd_dh<128>(ctx, p, variant, st) : fwd_dh<64>(ctx, p, variant, st);
}

int launch_attention_bwd_mfma(as_ctx* ctx, const AttnParams& p, int variant, hipStream_t st) {
  return p.dh == 128 ? bwd_dh<128>(ctx, p, variant, st) : bwd_dh<64>(ctx, p, variant, st);
}
