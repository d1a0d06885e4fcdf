// Register-staged LDS-tiled MFMA body: the fully masked body the ring kernels run on tiles with
// ragged N or K (every access bounds-checked, any alignment of the output rows).
#ifndef NIMBLE_GEMM_TILE_KERNEL_H_
#define NIMBLE_GEMM_TILE_KERNEL_H_
#include "device_common.h"

namespace nimble {

// ---------------------------------------------------------------------------
// LDS-tiled MFMA kernel.
//   LDS tile layout: row-major rows of 64 bf16 (8 chunks of 16 bytes); chunk c
//   of row r is stored at chunk slot c ^ ((r >> 1) & 7).  The LDS serves a
//   16-byte-per-lane access 16 lanes at a time over 64 banks (256 bytes), so 16
//   consecutive rows at one logical chunk must land on 16 distinct 16-byte
//   slots modulo 256 bytes: rows r and r+1 differ in bit 7 of the address, and
//   the XOR spreads the 8 row pairs over the 8 chunk slots.  The row-wise
//   writes (8 lanes per row) are conflict free under any such permutation.
//   MFMA operand roles: the A operand (32 rows i) is a slab of B = weights
//   (output features n), the B operand (32 columns j) is a slab of A =
//   activations (rows m).  A lane then owns four consecutive n of one row m in
//   every group of four accumulator registers, which gives packed stores.
// ---------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN, bool EDGE>
__device__ __forceinline__ void gemm_tile_body(const GemmArgs& g, const int m0, const int n0,
                                               uint4* smem) {
  uint4(*As)[BM * 8] = reinterpret_cast<uint4(*)[BM * 8]>(smem);
  uint4(*Bs)[BN * 8] = reinterpret_cast<uint4(*)[BN * 8]>(smem + 2 * BM * 8);
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_LD = BM * 8 / NT, B_LD = BN * 8 / NT;
  static_assert(A_LD >= 1 && B_LD >= 1, "tile too small for the workgroup");
  static_assert(TM >= 1 && TN >= 1, "wave tile too small");
  constexpr int ROWS_PER_PASS = NT / 8;
  static_assert(ROWS_PER_PASS % 16 == 0, "the LDS swizzle needs passes of whole 16-row groups");

  const int z = blockIdx.z;
  const u16* __restrict__ A = (const u16*)g.a + (long long)z * g.sa;
  const u16* __restrict__ B = (const u16*)g.b + (long long)z * g.sb;
  const int M = g.M, N = g.N, K = g.K;

  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // recomputed per tile, see gemm_ring_body
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // global -> LDS assignment: thread handles chunk (tid & 7) of rows (tid >> 3) + i * ROWS_PER_PASS
  const int ld_row = tid >> 3, ld_c = tid & 7;
  const int ld_slot = ld_row * 8 + (ld_c ^ ((ld_row >> 1) & 7));  // ROWS_PER_PASS is a multiple of 16
  const u16* a_src[A_LD];
  const u16* b_src[B_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    int row = m0 + ld_row + i * ROWS_PER_PASS;
    if (EDGE) row = row < M ? row : M - 1;
    a_src[i] = A + (long long)row * g.lda + ld_c * 8;
  }
#pragma unroll
  for (int i = 0; i < B_LD; ++i) {
    int row = n0 + ld_row + i * ROWS_PER_PASS;
    if (EDGE) row = row < N ? row : N - 1;
    b_src[i] = B + (long long)row * g.ldb + ld_c * 8;
  }

  // fragment read offsets (in 16-byte chunks)
  const int fr_row = lane & 31;
  const int fr_a = (wm * WM + fr_row) * 8;
  const int fr_b = (wn * WN + fr_row) * 8;
  const int fr_half = lane >> 5;
  const int fr_x = (lane >> 1) & 7;

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  uint4 ra[A_LD], rb[B_LD];
  const int KT = (K + 63) >> 6;

  auto load_global = [&](int kt) {
    const int k0 = kt << 6;
    const bool kvalid = !EDGE || (k0 + ld_c * 8 < K);
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      ra[i] = kvalid ? *(const uint4*)(a_src[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < B_LD; ++i)
      rb[i] = kvalid ? *(const uint4*)(b_src[i] + k0) : make_uint4(0, 0, 0, 0);
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_LD; ++i) As[buf][ld_slot + i * ROWS_PER_PASS * 8] = ra[i];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) Bs[buf][ld_slot + i * ROWS_PER_PASS * 8] = rb[i];
  };

  load_global(0);
  store_lds(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) load_global(kt + 1);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int phys = (kk * 2 + fr_half) ^ fr_x;
      bf16x8 xa[TM], wb[TN];
#pragma unroll
      for (int j = 0; j < TM; ++j) xa[j] = as_bf16x8(As[buf][fr_a + j * 32 * 8 + phys]);
#pragma unroll
      for (int i = 0; i < TN; ++i) wb[i] = as_bf16x8(Bs[buf][fr_b + i * 32 * 8 + phys]);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[i], xa[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_lds(buf ^ 1);
    __syncthreads();
  }

  // epilogue: lane owns row m, and for accumulator group q the columns
  // n_base + q*8 + (lane>>5)*4 + 0..3
  const float alpha = g.alpha;
  const int epi = g.epilogue;
  const u16* __restrict__ bias = (const u16*)g.bias;
  const bool vec_ok = !EDGE || ((g.ldc & 3) == 0);
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int m = m0 + wm * WM + j * 32 + fr_row;
    if (EDGE && m >= M) continue;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * WN + i * 32 + q * 8 + fr_half * 4;
        if (EDGE && n >= N) continue;
        float v[4];
        const bool full4 = !EDGE || (n + 3 < N);
        if (full4) {
          float b4[4] = {0.f, 0.f, 0.f, 0.f};
          if (epi != NIMBLE_EPI_NONE) {
            const uint2 bb = *(const uint2*)(bias + n);
            b4[0] = bf2f((u16)(bb.x & 0xffff));
            b4[1] = bf2f((u16)(bb.x >> 16));
            b4[2] = bf2f((u16)(bb.y & 0xffff));
            b4[3] = bf2f((u16)(bb.y >> 16));
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = epilogue(acc[i][j][q * 4 + e], alpha, b4[e], epi);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float be = (epi != NIMBLE_EPI_NONE && n + e < N) ? bf2f(bias[n + e]) : 0.f;
            v[e] = epilogue(acc[i][j][q * 4 + e], alpha, be, epi);
          }
        }
        const long long off = (long long)z * g.sc + (long long)m * g.ldc + n;
        if (g.out_f32) {
          float* C = (float*)g.c + off;
          if (full4 && vec_ok) {
            *(float4*)C = make_float4(v[0], v[1], v[2], v[3]);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < N) C[e] = v[e];
          }
        } else {
          u16* C = (u16*)g.c + off;
          if (full4 && vec_ok) {
            uint2 pk;
            pk.x = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
            pk.y = (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16);
            *(uint2*)C = pk;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < N) C[e] = f2bf(v[e]);
          }
        }
      }
    }
  }
}

}  // namespace nimble
#endif
