// gfx950 kernels behind the dispatch function (Section 3.5) and the device
// entry points of the C ABI.  bf16 operands, f32 accumulation on the matrix
// cores (v_mfma_f32_32x32x16_bf16 / v_mfma_f32_16x16x32_bf16), f32 epilogue.
//
// Kernel family
//   gemm_ring_kernel<BM,BN,WGM,WGN,RESIDUE>  large tiles (128x128, 256x128, 256x256).
//       Interior tiles: a ring of four 32-wide K stages filled by direct
//       global->LDS loads (no register staging), 16x16x32 MFMA with the next
//       stage's fragments read while the current stage multiplies, and an
//       epilogue that transposes through LDS so that every store is a full
//       128-byte line.  RESIDUE=false is the copy for r = 0: no bounds code at
//       all.  RESIDUE=true is the copy for r != 0: workgroups whose tile touches
//       an edge (decided once per workgroup) run a clamped and masked body.
//   gemm_tile_kernel<BM,BN,WGM,WGN,RESIDUE>  small tiles (32x128, 64x128),
//       register-staged double-buffered K tiles of 64, 32x32x16 MFMA.
//   skinny_kernel<MT,LSTM>   M <= 64 per workgroup: the weights are streamed from
//       HBM exactly once straight into MFMA operands, the four waves of a
//       workgroup split K and reduce through LDS.  LSTM=true gathers the four
//       gate rows of four hidden units and applies the cell update in the
//       epilogue.
//   generic_kernel            any shape and stride, one thread per output.
//   softmax_rows_kernel       f32 scores -> bf16 probabilities, one wave per row.
//   attention64_kernel        fused softmax(alpha Q.K^T).V for head dimension 64.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "nimble_internal.h"

namespace nimble {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;

__device__ __forceinline__ float bf2f(u16 b) { return __uint_as_float(((uint32_t)b) << 16); }

// float32 -> bfloat16, round to nearest, ties to even.
__device__ __forceinline__ u16 f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (u16)(u >> 16);
}

// erf(|x|) by the rational-times-Gaussian form of Abramowitz & Stegun 7.1.26
// (|error| <= 1.5e-7), on the hardware exp2 and reciprocal: about a dozen
// instructions where the library erff costs several times that, which matters
// when the epilogue runs once per output element.
// gelu(v) = v/2 (1 + erf(v / sqrt 2)) = v/2 + |v/2| erf(|v| / sqrt 2)
__device__ __forceinline__ float gelu_erf(float v) {
  const float ax = fabsf(v) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  p *= t;
  const float e = __builtin_amdgcn_exp2f(v * v * -0.72134752044448170f);  // exp(-v^2 / 2)
  const float r = fmaf(-p, e, 1.0f);                                       // erf(|v| / sqrt 2)
  const float hv = 0.5f * v;
  return fmaf(fabsf(hv), r, hv);
}

__device__ __forceinline__ float sigmoidf(float z) { return 1.0f / (1.0f + expf(-z)); }

__device__ __forceinline__ float epilogue(float acc, float alpha, float bias, int epi) {
  float v = alpha * acc;
  if (epi != NIMBLE_EPI_NONE) v += bias;
  if (epi == NIMBLE_EPI_BIAS_GELU_ERF) v = gelu_erf(v);
  return v;
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Two float32 -> two bfloat16 (round to nearest even) in one v_cvt_pk_bf16_f32; lo in bits 0..15.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Direct global -> LDS load of 16 bytes per lane: lane i's data lands at LDS byte
// address lds_addr + 16 i (lds_addr is wave-uniform and goes through M0).  It is
// tracked by vmcnt only; the caller waits with s_waitcnt vmcnt before a barrier
// makes the data visible to the other waves.  Written as inline assembly so that
// the compiler does not serialise it against LDS reads of the other ring slots.
__device__ __forceinline__ void dma16(const void* g, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n" ::"v"(g), "s"(lds_addr)
               : "memory", "m0");
}
// Same, addressed as a wave-uniform 64-bit base (in SGPRs) plus a 32-bit per-lane
// byte offset, which keeps per-lane 64-bit pointers out of the vector registers.
__device__ __forceinline__ void dma16_so(uint32_t voff, const void* sbase, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n" ::"v"(voff), "s"(sbase),
               "s"(lds_addr)
               : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// ---------------------------------------------------------------------------
// Workgroup id -> macro tile.  Workgroups are handed to the 8 XCDs round robin;
// give each XCD a contiguous run of tile ids so that the tiles sharing rows of
// A and B meet in that XCD's L2, and walk the tiles in groups of `group_m`
// tile rows so that the set in flight is a compact block.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n,
                                              int group_m, int& tm, int& tn) {
  const int q = nblocks >> 3, rem = nblocks & 7;
  const int xcd = bid & 7, local = bid >> 3;
  const int pid = xcd * q + (xcd < rem ? xcd : rem) + local;
  const int in_group = group_m * tiles_n;
  const int gid = pid / in_group;
  const int first_m = gid * group_m;
  const int gsize = (tiles_m - first_m) < group_m ? (tiles_m - first_m) : group_m;
  const int rest = pid - gid * in_group;
  tm = first_m + rest % gsize;
  tn = rest / gsize;
}

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

  const int tid = threadIdx.x;
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

// RESIDUE=false is the copy for r = 0 (and N, K multiples of the tile): no
// bounds code exists in it.  RESIDUE=true is the copy the dispatch function
// picks for r != 0: only the workgroups whose tile touches an edge run the
// clamped and masked body, decided once per workgroup; every interior tile
// runs the same unchecked body as the r = 0 copy.
template <int BM, int BN, int WGM, int WGN, bool RESIDUE>
__global__ void __launch_bounds__(WGM* WGN * 64)
    gemm_tile_kernel(GemmArgs g, int tiles_m, int tiles_n, int group_m) {
  __shared__ __attribute__((aligned(16))) uint4 smem[2 * (BM + BN) * 8];
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, gridDim.x, tiles_m, tiles_n, group_m, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  if (RESIDUE) {
    const bool edge = (m0 + BM > g.M) || (n0 + BN > g.N) || ((g.K & 63) != 0) || ((g.ldc & 3) != 0);
    if (edge) {
      gemm_tile_body<BM, BN, WGM, WGN, true>(g, m0, n0, smem);
      return;
    }
  }
  gemm_tile_body<BM, BN, WGM, WGN, false>(g, m0, n0, smem);
}

// ---------------------------------------------------------------------------
// Interior body of the large tiles.
//   LDS: a ring of S = 4 stages, each BM + BN rows of 32 bf16 (4 chunks of 16
//   bytes); chunk c of row r sits at slot c ^ ((r >> 2) & 3), so that the 16
//   rows one quarter-wave reads at one logical chunk cover all 64 banks.
//   Every wave issues its share of each stage as 16-byte-per-lane direct
//   global->LDS loads (a wave instruction fills 16 rows x 64 bytes = 1 KiB of
//   contiguous LDS); the swizzle is applied on the global side by choosing
//   which chunk a lane fetches.
//   Step ks: wait until this wave's loads of stage ks+1 have landed, barrier
//   (now every wave's have, and every wave has finished reading stage ks-1),
//   refill the slot of stage ks-1 with stage ks+3, read the fragments of stage
//   ks+1 into the second register set, run the MFMAs of stage ks.
//   MFMA 16x16x32: the A operand is 16 weight rows (n), the B operand 16
//   activation rows (m); a lane ends up with 4 consecutive n of one row m.
// ---------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN, bool MEDGE, bool PINGPONG>
__device__ __forceinline__ void gemm_ring_body(const GemmArgs& g, const int m0, const int n0,
                                               uint4* smem) {
  constexpr int S = 4;
  constexpr int NT = WGM * WGN * 64;
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 16, TN = WN / 16;
  constexpr int A_LD = BM * 4 / NT, B_LD = BN * 4 / NT;
  constexpr int LD = A_LD + B_LD;
  static_assert(A_LD >= 1 && B_LD >= 1, "tile too small for the workgroup");
  static_assert(WN == 64, "the LDS epilogue assumes 64 output columns per wave");
  static_assert(NW * WM * WN * 2 <= S * (BM + BN) * 64, "epilogue staging does not fit in the ring");
  uint4(*As)[BM * 4] = reinterpret_cast<uint4(*)[BM * 4]>(smem);
  uint4(*Bs)[BN * 4] = reinterpret_cast<uint4(*)[BN * 4]>(smem + S * BM * 4);

  // gridDim.y > 1: K is cut into gridDim.y slices of whole stages; slice blockIdx.y writes its
  // f32 partial sums to its own [M,N] plane of the output (g.c is then the split-K workspace)
  const int z = blockIdx.z;
  const int stages_all = g.K >> 5;
  const int stages_per = (stages_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int stage0 = (int)blockIdx.y * stages_per;
  const int KS = (stages_all - stage0) < stages_per ? (stages_all - stage0) : stages_per;
  const u16* __restrict__ A = (const u16*)g.a + (long long)z * g.sa + (stage0 << 5);
  const u16* __restrict__ B = (const u16*)g.b + (long long)z * g.sb + (stage0 << 5);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // loads: pass i covers chunk ids i*NT + tid: row = i*(NT/4) + (tid >> 2), slot = tid & 3.
  // Address = uniform base of (tile row 0, pass i, stage k0) + per-lane byte offset.
  // MEDGE (the last tile along M when r != 0): rows past M-1 are fetched from row M-1, so
  // every load stays in bounds; their products land in rows the epilogue never stores.
  const int ld_row = tid >> 2;
  const int ld_c = (tid & 3) ^ ((ld_row >> 2) & 3);
  uint32_t a_off[A_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    int row = ld_row + i * (NT / 4);
    if (MEDGE) row = (m0 + row < g.M) ? row : (g.M - 1 - m0);
    a_off[i] = (uint32_t)(row * g.lda + ld_c * 8) * 2u;
  }
  const uint32_t b_off = (uint32_t)(ld_row * g.ldb + ld_c * 8) * 2u;
  const u16* a_base = A + (long long)m0 * g.lda;
  const u16* b_base = B + (long long)n0 * g.ldb;
  const long long b_pass = (long long)(NT / 4) * g.ldb;
  const uint32_t a_dst = __builtin_amdgcn_readfirstlane(lds_addr_of(&As[0][wave * 64]));
  const uint32_t b_dst = __builtin_amdgcn_readfirstlane(lds_addr_of(&Bs[0][wave * 64]));
  auto dma = [&](int ks, int slot) {
    const int k0 = ks << 5;
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      dma16_so(a_off[i], a_base + k0, a_dst + slot * (BM * 64) + i * NT * 16);
#pragma unroll
    for (int i = 0; i < B_LD; ++i)
      dma16_so(b_off, b_base + i * b_pass + k0, b_dst + slot * (BN * 64) + i * NT * 16);
  };

  // fragment reads: lane -> row (lane & 15), logical chunk (lane >> 4)
  const int fr_row = lane & 15;
  const int fr_q = lane >> 4;
  const int fr_phys = fr_q ^ ((fr_row >> 2) & 3);
  const int fr_a = (wm * WM + fr_row) * 4 + fr_phys;
  const int fr_b = (wn * WN + fr_row) * 4 + fr_phys;

  f32x4 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (s < KS) dma(s, s);

  if (KS - 1 >= S - 2)
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * LD) : "memory");  // stage 0 landed
  else
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  if constexpr (PINGPONG) {
    // Waves w and w + NW/2 share a SIMD.  The workgroup runs in two groups half a step out of
    // phase: while group P multiplies stage s, group Q issues its loads and reads its fragments
    // of stage s, then they swap.  A wave never has memory instructions and MFMAs queued
    // together, and the matrix core of each SIMD always has one wave feeding it.
    //   P:    mem(0) | mfma(0) | mem(1) | mfma(1) | ...        ("|" = workgroup barrier)
    //   Q:  |        | mem(0)  | mfma(0)| mem(1)  | ...
    // mem(s) refills the slot of stage s-1 (both groups finished reading it before the barrier
    // that starts the phase) with stage s+3, then reads the fragments of stage s.  Before the
    // barrier that precedes P's mem(s+1) every wave has waited for its own loads of stage s+1.
    const bool is_q = wave >= NW / 2;
    bf16x8 xa[TM], wb[TN];
    if (is_q) __syncthreads();
    for (int base = 0; base < KS; base += S) {
#pragma unroll
      for (int u = 0; u < S; ++u) {
        const int ks = base + u;
        if (ks < KS) {
          const int slot = u % S, slot_free = (u + S - 1) % S;
          if (ks + S - 1 < KS) dma(ks + S - 1, slot_free);
#pragma unroll
          for (int j = 0; j < TM; ++j) xa[j] = as_bf16x8(As[slot][fr_a + j * 64]);
#pragma unroll
          for (int i = 0; i < TN; ++i) wb[i] = as_bf16x8(Bs[slot][fr_b + i * 64]);
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          if (is_q && ks + 1 < KS) {
            if (ks + S - 1 < KS)
              asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * LD) : "memory");
            else
              asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          }
          __builtin_amdgcn_sched_barrier(0);
          __syncthreads();
          __builtin_amdgcn_sched_barrier(0);
          __builtin_amdgcn_s_setprio(2);
#pragma unroll
          for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb[i], xa[j], acc[i][j], 0, 0, 0);
          __builtin_amdgcn_s_setprio(0);
          if (!is_q && ks + 1 < KS) {
            if (ks + S - 1 < KS)
              asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * LD) : "memory");
            else
              asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          }
          __builtin_amdgcn_sched_barrier(0);
          __syncthreads();
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (!is_q) __syncthreads();
  } else {
    bf16x8 xa[2][TM], wb[2][TN];
#pragma unroll
    for (int j = 0; j < TM; ++j) xa[0][j] = as_bf16x8(As[0][fr_a + j * 64]);
#pragma unroll
    for (int i = 0; i < TN; ++i) wb[0][i] = as_bf16x8(Bs[0][fr_b + i * 64]);

    for (int base = 0; base < KS; base += S) {
#pragma unroll
      for (int u = 0; u < S; ++u) {  // unrolled: ring slot and register set are compile-time
        const int ks = base + u;
        if (ks < KS) {
          const int cur = u & 1;
          const int slot_next = (u + 1) % S, slot_free = (u + S - 1) % S;
          if (ks + 1 < KS) {
            // stage ks+1 may have min(S-3, KS-ks-2) younger stages still in flight behind it
            if (KS - ks - 2 >= S - 3)
              asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 3) * LD) : "memory");
            else
              asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (ks + S - 1 < KS) dma(ks + S - 1, slot_free);
#pragma unroll
            for (int j = 0; j < TM; ++j) xa[cur ^ 1][j] = as_bf16x8(As[slot_next][fr_a + j * 64]);
#pragma unroll
            for (int i = 0; i < TN; ++i) wb[cur ^ 1][i] = as_bf16x8(Bs[slot_next][fr_b + i * 64]);
          }
#pragma unroll
          for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
              acc[i][j] =
                  __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb[cur][i], xa[cur][j], acc[i][j], 0, 0, 0);
        }
      }
    }
  }

  // epilogue.  acc[i][j][v] is row m = wm*WM + 16 j + fr_row, column n = wn*WN + 16 i + 4 fr_q + v.
  const float alpha = g.alpha;
  const int epi = g.epilogue;
  float bias4[TN][4];
#pragma unroll
  for (int i = 0; i < TN; ++i) {
#pragma unroll
    for (int v = 0; v < 4; ++v) bias4[i][v] = 0.f;
    if (epi != NIMBLE_EPI_NONE) {
      const uint2 bb = *(const uint2*)((const u16*)g.bias + n0 + wn * WN + i * 16 + fr_q * 4);
      bias4[i][0] = bf2f((u16)(bb.x & 0xffff));
      bias4[i][1] = bf2f((u16)(bb.x >> 16));
      bias4[i][2] = bf2f((u16)(bb.y & 0xffff));
      bias4[i][3] = bf2f((u16)(bb.y >> 16));
    }
  }
  if (g.out_f32) {
    float* C = (float*)g.c + (long long)z * g.sc + (long long)blockIdx.y * g.M * g.ldc;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      const int m = m0 + wm * WM + j * 16 + fr_row;
      if (MEDGE && m >= g.M) continue;
#pragma unroll
      for (int i = 0; i < TN; ++i) {
        const int n = n0 + wn * WN + i * 16 + fr_q * 4;
        float4 o;
        o.x = epilogue(acc[i][j][0], alpha, bias4[i][0], epi);
        o.y = epilogue(acc[i][j][1], alpha, bias4[i][1], epi);
        o.z = epilogue(acc[i][j][2], alpha, bias4[i][2], epi);
        o.w = epilogue(acc[i][j][3], alpha, bias4[i][3], epi);
        *(float4*)(C + (long long)m * g.ldc + n) = o;
      }
    }
    return;
  }
  // bf16: every wave stages its [WM][64] block in LDS (rows of 128 bytes, chunk c of
  // row r at slot c ^ ((r >> 1) & 7)) and writes it back out as full 128-byte lines
  __syncthreads();  // all fragment reads of the ring are done
  unsigned char* region = (unsigned char*)smem + wave * (WM * WN * 2);
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int row = j * 16 + fr_row;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
      const int col = i * 16 + fr_q * 4;
      const int chunk = (col >> 3) ^ ((row >> 1) & 7);
      uint2 pk;
      pk.x = pack_bf16x2(epilogue(acc[i][j][0], alpha, bias4[i][0], epi),
                         epilogue(acc[i][j][1], alpha, bias4[i][1], epi));
      pk.y = pack_bf16x2(epilogue(acc[i][j][2], alpha, bias4[i][2], epi),
                         epilogue(acc[i][j][3], alpha, bias4[i][3], epi));
      *(uint2*)(region + row * 128 + chunk * 16 + (col & 4) * 2) = pk;
    }
  }
  // the region is private to the wave: no workgroup barrier, the compiler orders the LDS accesses
  u16* C = (u16*)g.c + (long long)z * g.sc;
#pragma unroll
  for (int p = 0; p < WM / 8; ++p) {
    const int row = p * 8 + (lane >> 3);
    const int c = lane & 7;
    const uint4 v = *(const uint4*)(region + row * 128 + ((c ^ ((row >> 1) & 7)) * 16));
    if (MEDGE && m0 + wm * WM + row >= g.M) continue;
    *(uint4*)(C + (long long)(m0 + wm * WM + row) * g.ldc + n0 + wn * WN + c * 8) = v;
  }
}

template <int BM, int BN, int WGM, int WGN, bool RESIDUE>
__global__ void __launch_bounds__(WGM* WGN * 64)
    gemm_ring_kernel(GemmArgs g, int tiles_m, int tiles_n, int group_m) {
  // the two-group schedule pays off when a wave's multiply phase is long: 128x64 wave tiles
  constexpr bool kPingPong = (BM / WGM) * (BN / WGN) >= 128 * 64 && WGM * WGN == 8;
  __shared__ __attribute__((aligned(16))) uint4 smem[2 * (BM + BN) * 8];
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, gridDim.x, tiles_m, tiles_n, group_m, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  if (RESIDUE) {
    // the packed epilogue needs 16-byte aligned output rows; K must be whole 32-wide stages
    const bool ragged = (n0 + BN > g.N) || ((g.K & 31) != 0) || ((g.ldc & 7) != 0);
    if (ragged) {  // ragged N or K, or output rows not 16-byte aligned: the fully masked body
      gemm_tile_body<BM, BN, WGM, WGN, true>(g, m0, n0, smem);
      return;
    }
    if (m0 + BM > g.M) {  // the last tile along M: same pipeline, clamped loads, masked stores
      gemm_ring_body<BM, BN, WGM, WGN, true, kPingPong>(g, m0, n0, smem);
      return;
    }
  }
  gemm_ring_body<BM, BN, WGM, WGN, false, kPingPong>(g, m0, n0, smem);
}

// ---------------------------------------------------------------------------
// Skinny kernel: at most 64 rows of activations per workgroup, 16 weight rows.
// Every weight element is read from HBM once, by exactly one lane, straight
// into an MFMA operand (no LDS staging: there is no reuse to stage for).
// ---------------------------------------------------------------------------
struct SkinnyArgs {
  const u16* x;     // [M, K]  (LSTM: [B, Ix])
  const u16* h;     // LSTM only: [B, H]
  const u16* w;     // [N, K]  (LSTM: [4H, Ix+H])
  const u16* bias;  // [N]
  void* y;          // [M, N] bf16 or f32 (LSTM: h_out [B,H] bf16)
  const float* c_prev;  // LSTM only
  float* c_out;         // LSTM only
  int M, N, K;      // LSTM: M = B, N = 4H, K = Ix + H
  int Ix, H;        // LSTM only
  int epilogue, out_f32;
};

template <int MT, bool LSTM>
__global__ void __launch_bounds__(256) skinny_kernel(SkinnyArgs s) {
  __shared__ float red[4][MT][16][17];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, gq = lane >> 4;
  const int M = s.M, N = s.N, K = s.K;
  const int mbase = blockIdx.y * 64;

  // operands of the epilogue, fetched first so their latency hides behind the weight stream
  float pre_bias[4] = {0.f, 0.f, 0.f, 0.f};
  float pre_c = 0.f;
  if (LSTM) {
    const int t = tid >> 6, mm = (tid & 63) >> 2, u = tid & 3;
    const int m = mbase + t * 16 + mm, unit = blockIdx.x * 4 + u;
    if (t < MT && m < M && unit < s.H) {
#pragma unroll
      for (int q = 0; q < 4; ++q) pre_bias[q] = bf2f(s.bias[q * s.H + unit]);
      pre_c = s.c_prev[(long long)m * s.H + unit];
    }
  } else {
    const int n = blockIdx.x * 16 + (tid & 15);
    if (n < N && s.epilogue != NIMBLE_EPI_NONE) pre_bias[0] = bf2f(s.bias[n]);
  }

  // weight row of this lane
  long long wrow;
  if (LSTM) {
    int unit = blockIdx.x * 4 + (r & 3);
    unit = unit < s.H ? unit : s.H - 1;
    wrow = (long long)(r >> 2) * s.H + unit;
  } else {
    int n = blockIdx.x * 16 + r;
    wrow = n < N ? n : N - 1;
  }
  const u16* __restrict__ wp = s.w + wrow * K + gq * 8;

  // activation rows of this lane, one per 16-row tile
  const u16* xp[MT];
  const u16* hp[MT];
  bool mvalid[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int m = mbase + t * 16 + r;
    mvalid[t] = m < M;
    const int mc = mvalid[t] ? m : 0;
    if (LSTM) {
      xp[t] = s.x + (long long)mc * s.Ix;
      hp[t] = s.h + (long long)mc * s.H - s.Ix;  // indexed with the k of the concatenation
    } else {
      xp[t] = s.x + (long long)mc * K;
      hp[t] = nullptr;
    }
  }

  f32x4 acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // this wave's contiguous range of 32-wide k steps
  const int steps = (K + 31) >> 5;
  const int per_wave = (steps + 3) >> 2;
  const int s_begin = wave * per_wave;
  const int s_end = (s_begin + per_wave) < steps ? (s_begin + per_wave) : steps;

  constexpr int U = 8;
  for (int s0 = s_begin; s0 < s_end; s0 += U) {
    uint4 wv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = (s0 + u) * 32 + gq * 8;
      const bool ok = (s0 + u < s_end) && (k < K);
      wv[u] = ok ? *(const uint4*)(wp + (long long)(s0 + u) * 32) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      uint4 xv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = (s0 + u) * 32 + gq * 8;
        const bool ok = mvalid[t] && (s0 + u < s_end) && (k < K);
        const u16* src = (LSTM && k >= s.Ix) ? hp[t] : xp[t];
        xv[u] = ok ? *(const uint4*)(src + k) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wv[u]), as_bf16x8(xv[u]), acc[t],
                                                         0, 0, 0);
    }
  }

  // accumulator of lane (r, gq), register v: weight row i = 4 gq + v, activation row j = r
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][t][r][gq * 4 + v] = acc[t][v];
  __syncthreads();

  if (LSTM) {
    // thread -> (tile t, row m, hidden unit u); the four gates sit at columns gate*4 + u
    const int t = tid >> 6;
    if (t < MT) {
      const int mm = (tid & 63) >> 2, u = tid & 3;
      const int m = mbase + t * 16 + mm;
      const int unit = blockIdx.x * 4 + u;
      if (m < M && unit < s.H) {
        float gate[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = q * 4 + u;
          const float sum = (red[0][t][mm][col] + red[1][t][mm][col]) +
                            (red[2][t][mm][col] + red[3][t][mm][col]);
          gate[q] = sum + pre_bias[q];
        }
        const long long o = (long long)m * s.H + unit;
        const float cn = sigmoidf(gate[1]) * pre_c + sigmoidf(gate[0]) * tanhf(gate[2]);
        s.c_out[o] = cn;
        ((u16*)s.y)[o] = f2bf(sigmoidf(gate[3]) * tanhf(cn));
      }
    }
  } else {
    const int mm = tid >> 4, nn = tid & 15;
    const int n = blockIdx.x * 16 + nn;
    if (n < N) {
      const float b = pre_bias[0];
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const int m = mbase + t * 16 + mm;
        if (m < M) {
          const float sum = (red[0][t][mm][nn] + red[1][t][mm][nn]) +
                            (red[2][t][mm][nn] + red[3][t][mm][nn]);
          const float v = epilogue(sum, 1.0f, b, s.epilogue);
          const long long o = (long long)m * N + n;
          if (s.out_f32)
            ((float*)s.y)[o] = v;
          else
            ((u16*)s.y)[o] = f2bf(v);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Fully bounds-checked kernel for any shape, stride and B layout.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) generic_kernel(GemmArgs g) {
  const int n = blockIdx.x * 16 + (threadIdx.x & 15);
  const int m = blockIdx.y * 16 + (threadIdx.x >> 4);
  const int z = blockIdx.z;
  if (m >= g.M || n >= g.N) return;
  const u16* __restrict__ a = (const u16*)g.a + (long long)z * g.sa + (long long)m * g.lda;
  const u16* __restrict__ b = (const u16*)g.b + (long long)z * g.sb;
  float acc = 0.f;
  if (g.b_is_kn) {
    for (int k = 0; k < g.K; ++k) acc = fmaf(bf2f(a[k]), bf2f(b[(long long)k * g.ldb + n]), acc);
  } else {
    b += (long long)n * g.ldb;
    for (int k = 0; k < g.K; ++k) acc = fmaf(bf2f(a[k]), bf2f(b[k]), acc);
  }
  const float bias = (g.epilogue != NIMBLE_EPI_NONE) ? bf2f(((const u16*)g.bias)[n]) : 0.f;
  const float v = epilogue(acc, g.alpha, bias, g.epilogue);
  const long long o = (long long)z * g.sc + (long long)m * g.ldc + n;
  if (g.out_f32)
    ((float*)g.c)[o] = v;
  else
    ((u16*)g.c)[o] = f2bf(v);
}

// ---------------------------------------------------------------------------
// Row softmax, f32 in, bf16 out; one wave per row, four rows per workgroup.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__global__ void __launch_bounds__(256)
    softmax_rows_kernel(const float* __restrict__ s, u16* __restrict__ p, long long rows, int cols) {
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  const float* sr = s + row * cols;
  u16* pr = p + row * cols;
  float mx = -INFINITY;
  for (int j = lane; j < cols; j += 64) mx = fmaxf(mx, sr[j]);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < cols; j += 64) sum += expf(sr[j] - mx);
  sum = wave_sum(sum);
  const float inv = 1.0f / sum;
  for (int j = lane; j < cols; j += 64) pr[j] = f2bf(expf(sr[j] - mx) * inv);
}

// ---------------------------------------------------------------------------
// Fused attention for head dimension 64: O = softmax(alpha Q.K^T) V per head, in one launch,
// the scores never leave the chip.  A workgroup owns 64 query rows of one head (16 per wave)
// and walks the keys in blocks of 64 with a running row maximum and row sum.
//   scores:  MFMA 16x16x32 with 16 key rows on the A side and the wave's 16 query rows on
//            the B side: a lane holds, for its query row m = lane & 15, the keys
//            16 t + 4 (lane >> 4) + v of key tile t (v = 0..3).
//   P.V:     k runs over keys.  The sum over k does not care about order, so the 8 k-slots
//            of lane group g in MFMA u are DEFINED as the 8 keys that group already holds:
//            32u + 4g + (0..3) and 32u + 16 + 4g + (0..3).  P then goes from the score
//            accumulators to the MFMA operand without leaving the lane; V is staged in LDS
//            transposed ([d][key]) so the matching 8 values are two 8-byte reads.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
    attention64_kernel(const u16* __restrict__ q, const u16* __restrict__ k, const u16* __restrict__ v,
                       u16* __restrict__ o, int L, float alpha) {
  constexpr int D = 64, BJ = 64, VT_LD = 68;  // V^T rows padded to 68 elements against bank conflicts
  __shared__ __attribute__((aligned(16))) uint4 Ks[BJ * 8];  // [key][8 chunks], chunk c at c ^ ((key >> 1) & 7)
  __shared__ __attribute__((aligned(16))) u16 Vt[D * VT_LD];  // [d][key]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, g = lane >> 4;
  const long long head = (long long)blockIdx.y * L * D;
  const int m_row = blockIdx.x * 64 + wave * 16 + r;
  const int m_ld = m_row < L ? m_row : L - 1;

  // the wave's query fragments: row m, d = 32 kk + 8 g .. + 7
  bf16x8 qf[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
    qf[kk] = as_bf16x8(*(const uint4*)(q + head + (long long)m_ld * D + kk * 32 + g * 8));

  f32x4 oacc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) oacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float row_max = -INFINITY, row_sum = 0.f;  // row_sum: this lane's share, reduced at the end

  for (int j0 = 0; j0 < L; j0 += BJ) {
    __syncthreads();  // the previous block's fragments have been read
    // stage K (row-major, swizzled) and V (transposed): 512 chunks of 16 bytes each, 2 per thread
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = tid + i * 256;
      const int row = idx >> 3, c = idx & 7;
      const int jr = (j0 + row < L) ? (j0 + row) : (L - 1);
      const uint4 kc = *(const uint4*)(k + head + (long long)jr * D + c * 8);
      Ks[row * 8 + (c ^ ((row >> 1) & 7))] = kc;
      const uint4 vc = *(const uint4*)(v + head + (long long)jr * D + c * 8);
      const u16* ve = (const u16*)&vc;
#pragma unroll
      for (int e = 0; e < 8; ++e) Vt[(c * 8 + e) * VT_LD + row] = ve[e];
    }
    __syncthreads();

    // scores of the wave's 16 rows against the 64 keys of the block
    f32x4 sacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      sacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int krow = t * 16 + r;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const bf16x8 kf = as_bf16x8(Ks[krow * 8 + ((kk * 4 + g) ^ ((krow >> 1) & 7))]);
        sacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[kk], sacc[t], 0, 0, 0);
      }
    }
    // scale, mask keys past L, block maximum of the row (4 lanes share a row)
    float bmax = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = j0 + t * 16 + g * 4 + e;
        const float sv = (j < L) ? alpha * sacc[t][e] : -INFINITY;
        sacc[t][e] = sv;
        bmax = fmaxf(bmax, sv);
      }
    bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
    const float new_max = fmaxf(row_max, bmax);  // finite: key j0 < L is in every block
    const float rescale = __expf(row_max - new_max);
    row_max = new_max;
    row_sum *= rescale;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float pv = __expf(sacc[t][e] - new_max);
        sacc[t][e] = pv;
        row_sum += pv;
        oacc[t][e] *= rescale;
      }
    // O += P.V: MFMA u consumes key tiles 2u and 2u+1
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      uint4 pw;
      pw.x = pack_bf16x2(sacc[2 * u][0], sacc[2 * u][1]);
      pw.y = pack_bf16x2(sacc[2 * u][2], sacc[2 * u][3]);
      pw.z = pack_bf16x2(sacc[2 * u + 1][0], sacc[2 * u + 1][1]);
      pw.w = pack_bf16x2(sacc[2 * u + 1][2], sacc[2 * u + 1][3]);
      const bf16x8 pf = as_bf16x8(pw);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const u16* vrow = Vt + (t * 16 + r) * VT_LD + u * 32 + g * 4;
        const uint2 lo = *(const uint2*)vrow, hi = *(const uint2*)(vrow + 16);
        const bf16x8 vf = as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y));
        oacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, oacc[t], 0, 0, 0);
      }
    }
  }
  row_sum += __shfl_xor(row_sum, 16, 64);
  row_sum += __shfl_xor(row_sum, 32, 64);
  const float inv = 1.0f / row_sum;
  if (m_row < L) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      uint2 pk;
      pk.x = pack_bf16x2(oacc[t][0] * inv, oacc[t][1] * inv);
      pk.y = pack_bf16x2(oacc[t][2] * inv, oacc[t][3] * inv);
      *(uint2*)(o + head + (long long)m_row * D + t * 16 + g * 4) = pk;
    }
  }
}

// ---------------------------------------------------------------------------
// Second half of a K-split launch: add the `slices` f32 partial planes, apply the epilogue,
// write the output.  One thread per 4 consecutive columns (N is a multiple of 128 here).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
    splitk_reduce_kernel(const float* __restrict__ ws, int slices, long long plane, int M, int N,
                         const u16* __restrict__ bias, int epi, void* __restrict__ out, int out_f32) {
  const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (idx >= (long long)M * N) return;
  float4 acc = *(const float4*)(ws + idx);
  for (int s = 1; s < slices; ++s) {
    const float4 v = *(const float4*)(ws + (long long)s * plane + idx);
    acc.x += v.x;
    acc.y += v.y;
    acc.z += v.z;
    acc.w += v.w;
  }
  float b4[4] = {0.f, 0.f, 0.f, 0.f};
  if (epi != NIMBLE_EPI_NONE) {
    const uint2 bb = *(const uint2*)(bias + (int)(idx % N));
    b4[0] = bf2f((u16)(bb.x & 0xffff));
    b4[1] = bf2f((u16)(bb.x >> 16));
    b4[2] = bf2f((u16)(bb.y & 0xffff));
    b4[3] = bf2f((u16)(bb.y >> 16));
  }
  const float v0 = epilogue(acc.x, 1.0f, b4[0], epi), v1 = epilogue(acc.y, 1.0f, b4[1], epi);
  const float v2 = epilogue(acc.z, 1.0f, b4[2], epi), v3 = epilogue(acc.w, 1.0f, b4[3], epi);
  if (out_f32) {
    *(float4*)((float*)out + idx) = make_float4(v0, v1, v2, v3);
  } else {
    uint2 pk;
    pk.x = pack_bf16x2(v0, v1);
    pk.y = pack_bf16x2(v2, v3);
    *(uint2*)((u16*)out + idx) = pk;
  }
}

// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------
static int check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return NIMBLE_OK;
  return fail(NIMBLE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

template <int BM, int BN, int WGM, int WGN>
static int launch_tile(const GemmArgs& g, const nimble_plan& p, hipStream_t st) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  int group_m = BM >= 128 ? 4 : 8;
  if (group_m > tiles_m) group_m = tiles_m;
  dim3 grid(p.grid[0], 1, p.grid[2]), block(WGM * WGN * 64);
  if (p.residue_copy)
    hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WGM, WGN, true>), grid, block, 0, st, g, tiles_m,
                       tiles_n, group_m);
  else
    hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WGM, WGN, false>), grid, block, 0, st, g, tiles_m,
                       tiles_n, group_m);
  return check_hip(hipGetLastError(), "tile kernel launch");
}

template <int BM, int BN, int WGM, int WGN>
static int launch_ring(const GemmArgs& g, const nimble_plan& p, hipStream_t st) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  int group_m = 4;
  if (group_m > tiles_m) group_m = tiles_m;
  dim3 grid(p.grid[0], p.split_k > 1 ? p.split_k : 1, p.grid[2]), block(WGM * WGN * 64);
  if (p.residue_copy)
    hipLaunchKernelGGL((gemm_ring_kernel<BM, BN, WGM, WGN, true>), grid, block, 0, st, g, tiles_m,
                       tiles_n, group_m);
  else
    hipLaunchKernelGGL((gemm_ring_kernel<BM, BN, WGM, WGN, false>), grid, block, 0, st, g, tiles_m,
                       tiles_n, group_m);
  return check_hip(hipGetLastError(), "ring kernel launch");
}

template <bool LSTM>
static int launch_skinny(const SkinnyArgs& s, const nimble_plan& p, hipStream_t st) {
  dim3 grid(p.grid[0], p.grid[1], 1), block(256);
  const int rows = s.M < 64 ? s.M : 64;
  const int mt = (rows + 15) / 16;
  switch (mt) {
    case 1: hipLaunchKernelGGL((skinny_kernel<1, LSTM>), grid, block, 0, st, s); break;
    case 2: hipLaunchKernelGGL((skinny_kernel<2, LSTM>), grid, block, 0, st, s); break;
    case 3: hipLaunchKernelGGL((skinny_kernel<3, LSTM>), grid, block, 0, st, s); break;
    default: hipLaunchKernelGGL((skinny_kernel<4, LSTM>), grid, block, 0, st, s); break;
  }
  return check_hip(hipGetLastError(), "skinny kernel launch");
}

static int launch_gemm(const GemmArgs& g, const nimble_plan& p, hipStream_t st) {
  switch (p.variant) {
    case NIMBLE_VAR_GENERIC: {
      dim3 grid(p.grid[0], p.grid[1], p.grid[2]), block(256);
      hipLaunchKernelGGL(generic_kernel, grid, block, 0, st, g);
      return check_hip(hipGetLastError(), "generic kernel launch");
    }
    case NIMBLE_VAR_SKINNY16: {
      SkinnyArgs s{};
      s.x = (const u16*)g.a;
      s.w = (const u16*)g.b;
      s.bias = (const u16*)g.bias;
      s.y = g.c;
      s.M = g.M;
      s.N = g.N;
      s.K = g.K;
      s.epilogue = g.epilogue;
      s.out_f32 = g.out_f32;
      return launch_skinny<false>(s, p, st);
    }
    case NIMBLE_VAR_T32x128: return launch_tile<32, 128, 1, 4>(g, p, st);
    case NIMBLE_VAR_T64x128: return launch_tile<64, 128, 2, 2>(g, p, st);
    case NIMBLE_VAR_T128x128: return launch_ring<128, 128, 2, 2>(g, p, st);
    case NIMBLE_VAR_T256x128: return launch_ring<256, 128, 4, 2>(g, p, st);
    case NIMBLE_VAR_T256x256: return launch_ring<256, 256, 2, 4>(g, p, st);
    default: return fail(NIMBLE_ERR_ARG, "unknown variant %d", p.variant);
  }
}

static inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

}  // namespace nimble

using namespace nimble;

extern "C" {

// One planned launch of dense; a K-split plan runs the slices into the workspace and then the
// reduction kernel.
static int run_dense(const GemmArgs& g, const nimble_plan& p, void* workspace, hipStream_t st) {
  if (p.split_k <= 1 || p.variant < NIMBLE_VAR_T128x128) return launch_gemm(g, p, st);
  GemmArgs part = g;
  part.c = workspace;
  part.out_f32 = 1;
  part.epilogue = NIMBLE_EPI_NONE;
  part.alpha = 1.0f;
  part.bias = nullptr;
  int rc = launch_gemm(part, p, st);
  if (rc != NIMBLE_OK) return rc;
  const long long quads = ((long long)g.M * g.N + 3) / 4;
  dim3 grid((unsigned)((quads + 255) / 256)), block(256);
  hipLaunchKernelGGL(splitk_reduce_kernel, grid, block, 0, st, (const float*)workspace, p.split_k,
                     (long long)g.M * g.N, g.M, g.N, (const u16*)g.bias, g.epilogue, g.c, g.out_f32);
  return check_hip(hipGetLastError(), "split-K reduction launch");
}

int nimble_dense_dyn(const void* x, const void* w, const void* bias, void* y, int64_t M,
                     int64_t N, int64_t K, int epilogue, int out_dtype, int force_variant,
                     void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  if (M < 0 || N < 0 || K < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (epilogue < NIMBLE_EPI_NONE || epilogue > NIMBLE_EPI_BIAS_GELU_ERF)
    return fail(NIMBLE_ERR_ARG, "unknown epilogue %d", epilogue);
  if (out_dtype != NIMBLE_BF16 && out_dtype != NIMBLE_F32)
    return fail(NIMBLE_ERR_DTYPE, "unknown dtype %d", out_dtype);
  if (workspace_bytes > 0 && !workspace) return fail(NIMBLE_ERR_NULL, "workspace_bytes > 0 with a null workspace");
  if (workspace && misaligned(workspace)) return fail(NIMBLE_ERR_ALIGN, "workspace must be 16-byte aligned");
  // the dispatch function plans within the scratch the caller brought: no scratch, no K split
  PlanOptions opt;
  opt.max_workspace = workspace_bytes;
  nimble_plan p;
  int rc = plan_dense(1, M, N, K, epilogue, force_variant, opt, &p);
  if (rc != NIMBLE_OK) return rc;
  if (M == 0 || N == 0) return NIMBLE_OK;
  if (!x || !w || !y) return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if (epilogue != NIMBLE_EPI_NONE && !bias) return fail(NIMBLE_ERR_NULL, "epilogue needs a bias");
  if (misaligned(x) || misaligned(w) || misaligned(y) || (bias && misaligned(bias)))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  GemmArgs g{};
  g.a = x;
  g.b = w;
  g.bias = bias;
  g.c = y;
  g.M = (int)M;
  g.N = (int)N;
  g.K = (int)K;
  g.lda = (int)K;
  g.ldb = (int)K;
  g.ldc = (int)N;
  g.alpha = 1.0f;
  g.epilogue = epilogue;
  g.out_f32 = out_dtype == NIMBLE_F32;
  g.batch = 1;
  if (p.split_rows <= 0) return run_dense(g, p, workspace, (hipStream_t)stream);

  // two launches: rows [0, split_rows) through the r = 0 copy, then the remaining rows through
  // whatever the dispatch function picks for their number (planned without a further row split)
  nimble_plan rp;
  PlanOptions tail_opt = opt;
  tail_opt.allow_row_split = false;
  rc = plan_dense(1, M - p.split_rows, N, K, epilogue, NIMBLE_VAR_AUTO, tail_opt, &rp);
  if (rc != NIMBLE_OK) return rc;
  GemmArgs head = g;
  head.M = (int)p.split_rows;
  rc = run_dense(head, p, workspace, (hipStream_t)stream);
  if (rc != NIMBLE_OK) return rc;
  GemmArgs tail = g;
  tail.M = (int)(M - p.split_rows);
  tail.a = (const u16*)x + p.split_rows * K;
  tail.c = g.out_f32 ? (void*)((float*)y + p.split_rows * N) : (void*)((u16*)y + p.split_rows * N);
  return run_dense(tail, rp, workspace, (hipStream_t)stream);
}

int nimble_batch_matmul_dyn(const void* a, const void* b, void* c, int64_t batch, int64_t M,
                            int64_t N, int64_t K, int trans_b, float alpha, int out_dtype,
                            void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  (void)workspace;
  if (batch < 0 || M < 0 || N < 0 || K < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (out_dtype != NIMBLE_BF16 && out_dtype != NIMBLE_F32)
    return fail(NIMBLE_ERR_DTYPE, "unknown dtype %d", out_dtype);
  nimble_plan p;
  int rc = nimble_batch_matmul_plan(batch, M, N, K, trans_b, out_dtype, &p);
  if (rc != NIMBLE_OK) return rc;
  if (batch == 0 || M == 0 || N == 0) return NIMBLE_OK;
  if (!a || !b || !c) return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if (misaligned(a) || misaligned(b) || misaligned(c))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  if (workspace_bytes < p.workspace_bytes)
    return fail(NIMBLE_ERR_WORKSPACE, "workspace of %zu bytes, plan needs %llu", workspace_bytes,
                (unsigned long long)p.workspace_bytes);
  GemmArgs g{};
  g.a = a;
  g.b = b;
  g.c = c;
  g.M = (int)M;
  g.N = (int)N;
  g.K = (int)K;
  g.lda = (int)K;
  g.ldb = trans_b ? (int)K : (int)N;
  g.ldc = (int)N;
  g.sa = (long long)M * K;
  g.sb = (long long)N * K;
  g.sc = (long long)M * N;
  g.alpha = alpha;
  g.epilogue = NIMBLE_EPI_NONE;
  g.out_f32 = out_dtype == NIMBLE_F32;
  g.b_is_kn = trans_b ? 0 : 1;
  g.batch = (int)batch;
  // batch slices of a K-contiguous operand stay 16-byte aligned only if M*K (N*K) is a multiple of 8
  if (p.variant != NIMBLE_VAR_GENERIC && (((M * K) & 7) != 0 || ((N * K) & 7) != 0)) {
    rc = plan_dense(batch, M, N, K, NIMBLE_EPI_NONE, NIMBLE_VAR_GENERIC, PlanOptions(), &p);
    if (rc != NIMBLE_OK) return rc;
  }
  return launch_gemm(g, p, (hipStream_t)stream);
}

int nimble_softmax_rows_dyn(const void* s_f32, void* p_bf16, int64_t rows, int64_t cols,
                            void* stream) {
  clear_error();
  if (rows < 0 || cols < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (cols > (1ll << 30) || rows > (1ll << 32)) return fail(NIMBLE_ERR_ARG, "extent too large");
  if (rows == 0 || cols == 0) return NIMBLE_OK;
  if (!s_f32 || !p_bf16) return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if (misaligned(s_f32) || misaligned(p_bf16))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  hipLaunchKernelGGL(softmax_rows_kernel, grid, block, 0, (hipStream_t)stream, (const float*)s_f32,
                     (u16*)p_bf16, (long long)rows, (int)cols);
  return check_hip(hipGetLastError(), "softmax kernel launch");
}

int nimble_attention_dyn(const void* q, const void* k, const void* v, void* o, int64_t heads, int64_t L,
                         int64_t D, float alpha, void* stream) {
  clear_error();
  if (heads < 0 || L < 0 || D < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (D != 64) return fail(NIMBLE_ERR_ARG, "fused attention is built for head dimension 64, got %lld", (long long)D);
  if (heads > 65535 || L > (1ll << 24)) return fail(NIMBLE_ERR_ARG, "extent too large");
  if (heads == 0 || L == 0) return NIMBLE_OK;
  if (!q || !k || !v || !o) return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  dim3 grid((unsigned)((L + 63) / 64), (unsigned)heads), block(256);
  hipLaunchKernelGGL(attention64_kernel, grid, block, 0, (hipStream_t)stream, (const u16*)q, (const u16*)k,
                     (const u16*)v, (u16*)o, (int)L, alpha);
  return check_hip(hipGetLastError(), "attention kernel launch");
}

int nimble_lstm_gates_dyn(const void* x, const void* h_prev, const void* w, const void* bias,
                          const void* c_prev, void* c_out, void* h_out, int64_t B, int64_t Ix,
                          int64_t H, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  (void)workspace;
  (void)workspace_bytes;
  nimble_plan p;
  int rc = nimble_lstm_plan(B, Ix, H, &p);
  if (rc != NIMBLE_OK) return rc;
  if (B == 0) return NIMBLE_OK;
  if (!h_prev || !w || !bias || !c_prev || !c_out || !h_out || (Ix > 0 && !x))
    return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if ((x && misaligned(x)) || misaligned(h_prev) || misaligned(w) || misaligned(bias) ||
      misaligned(c_prev) || misaligned(c_out) || misaligned(h_out))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  if (h_out == h_prev) return fail(NIMBLE_ERR_ARG, "h_out must not alias h_prev");
  SkinnyArgs s{};
  s.x = (const u16*)x;
  s.h = (const u16*)h_prev;
  s.w = (const u16*)w;
  s.bias = (const u16*)bias;
  s.y = h_out;
  s.c_prev = (const float*)c_prev;
  s.c_out = (float*)c_out;
  s.M = (int)B;
  s.N = (int)(4 * H);
  s.K = (int)(Ix + H);
  s.Ix = (int)Ix;
  s.H = (int)H;
  s.epilogue = NIMBLE_EPI_BIAS;
  return launch_skinny<true>(s, p, (hipStream_t)stream);
}

}  // extern "C"
