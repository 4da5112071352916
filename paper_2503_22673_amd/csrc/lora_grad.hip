// Adapter gradients: C[m, j] = alpha * sum_t X[t, m] * U[t, j], a product contracted over TOKENS,
// i.e. over the row index of both operands (dB = s dy^T u with X = dy, U = u; dA^T = x^T du with
// X = x, U = du).  X is a big row-major activation ([tokens, M] bf16, up to 14336 columns), U is
// 64 columns wide at most, so the kernel is a single streaming pass over X at HBM speed.
//
// Matrix cores want the contraction index contiguous per lane.  Instead of transposing X through
// memory, each lane loads an 8-token x 8-column block (eight 16-byte loads, 256 B contiguous per
// 16 lanes and token) and transposes it in registers (v_perm), which yields the A operands of eight
// v_mfma_f32_16x16x32_bf16 -- one per column of the block; MFMA row m then stands for column
// c0 + 8 m + q of X.  U comes from its small token-major copy ([j][token]), one 16-byte load per
// lane and 16-column block.  Token ranges (splits) go to a partial buffer reduced in split order.
#include "common.h"

namespace {
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

struct TnParams {
  const bf16_t* X; int64_t ldx;      // [n, M] row-major
  const bf16_t* UT; int64_t ldu;     // [>= 16*NB rows, tokens rounded up to 64] token-major, zero past n and past r
  int n, M, r;
  float* partial;                    // [splits, M, r]
  int steps_per_split, total_steps;  // 32-token steps
};

#include "lora_grad_loop.inc"
template <int NB>
__global__ __launch_bounds__(256) void lora_grad_tn_kernel(TnParams p) {
  const int tid = threadIdx.x, lane = tid & 63, lm = lane & 15, lg = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // the four waves of a workgroup take four neighbouring 128-column slabs and the same tokens, so that
  // the workgroup reads 1 KB of every token row at a time
  const int slab = blockIdx.x * 4 + wave, split = blockIdx.y;
  if (slab * 128 >= p.M) return;
  const int col = slab * 128 + 8 * lm;
  const bool col_ok = col < p.M;
  f32x4 acc[8][NB];
#pragma unroll
  for (int q = 0; q < 8; q++)
#pragma unroll
    for (int nb = 0; nb < NB; nb++) acc[q][nb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const int s_end = min((split + 1) * p.steps_per_split, p.total_steps);
  auto load = [&](int step, u32x4 (&x)[8], bf16x8 (&b)[NB]) {
    const int t0 = step * 32 + 8 * lg;
#pragma unroll
    for (int r = 0; r < 8; r++) {
      const int t = t0 + r;
      const bool ok = col_ok && t < p.n;
      const u32x4 v = *reinterpret_cast<const u32x4*>(p.X + (int64_t)(ok ? t : 0) * p.ldx + (ok ? col : 0));
      x[r] = ok ? v : (u32x4){0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int nb = 0; nb < NB; nb++) b[nb] = *reinterpret_cast<const bf16x8*>(p.UT + (int64_t)(nb * 16 + lm) * p.ldu + t0);
  };
  auto compute = [&](const u32x4 (&x)[8], const bf16x8 (&b)[NB]) {
#pragma unroll
    for (int q = 0; q < 8; q++) {
      // column q of the 8x8 block: dword d of the operand = (x[2d][q], x[2d+1][q])
      u32x4 a;
#pragma unroll
      for (int d = 0; d < 4; d++)
        a[d] = __builtin_amdgcn_perm(x[2 * d + 1][q >> 1], x[2 * d][q >> 1], (q & 1) ? 0x07060302u : 0x05040100u);
      const bf16x8 av = __builtin_bit_cast(bf16x8, a);
#pragma unroll
      for (int nb = 0; nb < NB; nb++) acc[q][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b[nb], acc[q][nb], 0, 0, 0);
    }
  };
  int step = split * p.steps_per_split;
  // Whole steps of a full-width slab with all four column blocks of the narrow operand run in the generated loop
  // (gen_lora_grad_loop.py: four register sets, three steps in flight); what is left -- a last step that runs past the
  // tokens, narrower operands, a ragged slab -- takes the loop below.
  if constexpr (NB == 4) {
    const int s_full = min(s_end, p.n / 32);
    if (p.M % 128 == 0 && s_full > step) {
      uint32_t vx[8], vu[4];
#pragma unroll
      for (int r = 0; r < 8; r++) vx[r] = (uint32_t)((((int64_t)(8 * lg + r)) * p.ldx + col) * 2);
#pragma unroll
      for (int nb = 0; nb < 4; nb++) vu[nb] = (uint32_t)((((int64_t)(nb * 16 + lm)) * p.ldu + 8 * lg) * 2);
      const uint64_t gx = (uint64_t)(p.X + (int64_t)step * 32 * p.ldx), gu = (uint64_t)(p.UT + (int64_t)step * 32);
      const uint32_t stride = (uint32_t)(32 * p.ldx * 2), nsteps = (uint32_t)(s_full - step);
      asm volatile(LORA_GRAD_LOOP_ASM
                   : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]),
                     "+a"(acc[2][0]), "+a"(acc[2][1]), "+a"(acc[2][2]), "+a"(acc[2][3]), "+a"(acc[3][0]), "+a"(acc[3][1]), "+a"(acc[3][2]), "+a"(acc[3][3]),
                     "+a"(acc[4][0]), "+a"(acc[4][1]), "+a"(acc[4][2]), "+a"(acc[4][3]), "+a"(acc[5][0]), "+a"(acc[5][1]), "+a"(acc[5][2]), "+a"(acc[5][3]),
                     "+a"(acc[6][0]), "+a"(acc[6][1]), "+a"(acc[6][2]), "+a"(acc[6][3]), "+a"(acc[7][0]), "+a"(acc[7][1]), "+a"(acc[7][2]), "+a"(acc[7][3])
                   : "v"(vx[0]), "v"(vx[1]), "v"(vx[2]), "v"(vx[3]), "v"(vx[4]), "v"(vx[5]), "v"(vx[6]), "v"(vx[7]),
                     "v"(vu[0]), "v"(vu[1]), "v"(vu[2]), "v"(vu[3]), "s"(gx), "s"(gu), "s"(stride), "s"(nsteps)
                   : LORA_GRAD_LOOP_CLOBBERS);
      step = s_full;
    }
  }
  // two register sets: the block of the next step is in flight while this one is multiplied
  u32x4 xa[8], xb[8];
  bf16x8 ba[NB], bb[NB];
  if (step < s_end) load(step, xa, ba);
  for (; step < s_end; step += 2) {
    if (step + 1 < s_end) load(step + 1, xb, bb);
    compute(xa, ba);
    if (step + 1 >= s_end) break;
    if (step + 2 < s_end) load(step + 2, xa, ba);
    compute(xb, bb);
  }
  // accumulator row 4*lg + i of MFMA q is column c0 + 8*(4*lg + i) + q; its column is j = nb*16 + lm
  float* out = p.partial + (int64_t)split * p.M * p.r;
#pragma unroll
  for (int q = 0; q < 8; q++)
#pragma unroll
    for (int nb = 0; nb < NB; nb++) {
      const int j = nb * 16 + lm;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int m = slab * 128 + 8 * (4 * lg + i) + q;
        if (m < p.M && j < p.r) out[(int64_t)m * p.r + j] = acc[q][nb][i];
      }
    }
}

__global__ void tn_reduce_kernel(const float* __restrict__ partial, int splits, int M, int r, float alpha,
                                 float* __restrict__ C, int64_t sm, int64_t sj) {
  // a thread owns four consecutive elements (M is a multiple of 8) and adds the splits in order; eight loads in flight
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4, total = (int64_t)M * r;
  if (i >= total) return;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  int s = 0;
  for (; s + 8 <= splits; s += 8) {
    f32x4 v[8];
#pragma unroll
    for (int k = 0; k < 8; k++) v[k] = *reinterpret_cast<const f32x4*>(partial + (int64_t)(s + k) * total + i);
#pragma unroll
    for (int k = 0; k < 8; k++) acc += v[k];
  }
  for (; s < splits; s++) acc += *reinterpret_cast<const f32x4*>(partial + (int64_t)s * total + i);
#pragma unroll
  for (int k = 0; k < 4; k++) C[((i + k) / r) * sm + ((i + k) % r) * sj] = alpha * acc[k];
}
}  // namespace

// One workgroup fits a CU (the accumulators fill the register file): the token range is split so that the launch is one
// round of at most 256 workgroups (14336 columns: 28 x 9 = 252 workgroups; with 28 x 10 the last 24 ran alone and the
// launch took half as long again).
static int tn_splits(int n, int M) {
  const int steps = (int)cdiv(n, 32), wg_cols = (int)cdiv(cdiv(M, 128), 4);
  return (int)std::max<int64_t>(1, std::min<int64_t>(256 / wg_cols, cdiv(steps, 16)));
}

size_t lora_grad_tn_partial_floats(int n, int M, int r) { return (size_t)tn_splits(n, M) * M * r; }

// C[m * sm + j * sj] = alpha * sum_t X[t, m] * UT[j, t];  r <= 64, M a multiple of 8, ldx a multiple of 8.
int launch_lora_grad_tn(as_ctx* ctx, const void* X, int64_t ldx, const void* UT, int64_t ldu, int n, int M, int r,
                        float alpha, float* C, int64_t sm, int64_t sj, float* partial, size_t partial_floats, hipStream_t st) {
  if (n <= 0 || M <= 0 || r <= 0) return AS_OK;
  if (r > 64 || (M % 8) || (ldx % 8) || (ldu % 8) || ((uintptr_t)X % 16) || ((uintptr_t)UT % 16) || ((uintptr_t)partial % 16))
    return as_fail(ctx, AS_ERR_SHAPE, "lora_grad_tn: rank <= 64 and 8-element alignment needed");
  const int steps = (int)cdiv(n, 32), slabs = (int)cdiv(M, 128);
  const int splits = tn_splits(n, M);
  if ((size_t)splits * M * r > partial_floats) return as_fail(ctx, AS_ERR_WORKSPACE, "lora_grad_tn: partial buffer too small");
  TnParams p{(const bf16_t*)X, ldx, (const bf16_t*)UT, ldu, n, M, r, partial, (int)cdiv(steps, splits), steps};
  const int nb = (int)cdiv(r, 16);
  dim3 grid((unsigned)cdiv(slabs, 4), splits);
  prof_begin(ctx, st, AS_K_LORA_GRAD, 2.0 * n * (double)M * r);
#define TN_LAUNCH(NB) { lora_grad_tn_kernel<NB><<<grid, 256, 0, st>>>(p); }
  switch (nb) { case 1: TN_LAUNCH(1) break; case 2: TN_LAUNCH(2) break; case 3: TN_LAUNCH(3) break; default: TN_LAUNCH(4) break; }
#undef TN_LAUNCH
  AS_LAUNCH_CHECK(ctx);
  tn_reduce_kernel<<<(unsigned)cdiv((int64_t)M * r, 1024), 256, 0, st>>>(partial, splits, M, r, alpha, C, sm, sj);
  prof_end(ctx, st);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}
