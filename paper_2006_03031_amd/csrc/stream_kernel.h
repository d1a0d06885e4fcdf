// Weight-streaming kernel for at most 16 rows, operands staged through per-wave LDS rings by
// direct global->LDS loads of whole 128-byte lines.
#ifndef NIMBLE_STREAM_KERNEL_H_
#define NIMBLE_STREAM_KERNEL_H_
#include "device_common.h"
#include "skinny_kernel.h"

namespace nimble {

// ---------------------------------------------------------------------------
// Why another weight-streaming kernel.  skinny_kernel loads a weight fragment straight into the
// MFMA operand layout: lane (r, q) holds 16 bytes of weight row r, so the 16 lanes the memory
// pipeline coalesces together touch 16 different rows, and one wave instruction costs 64 cache-line
// look-ups for 1 KiB (the activation fragment costs the same again once all 16 rows are real).
// That, not HBM, bounds it: 134 MB layers stream at 4.2-5.2 TB/s at one row and at 3.5 TB/s at
// sixteen rows whatever the occupancy.
// Here a wave instruction fetches 8 rows x 128 contiguous bytes (8 lanes per row: a whole line per
// row, 8 look-ups per KiB) and the data goes straight to LDS, from where the fragments are read in
// the MFMA layout (conflict-free with the ring kernels' swizzle).  Data in flight lives in LDS,
// not in registers, so a wave keeps S-1 stages (64 k each: 2 KiB of weights + 2 KiB of
// activations) on their way whatever its register budget.
//   Workgroup: 16 weight rows (LSTM: the i,f,g,o rows of 4 hidden units), NW waves, each with a
//   contiguous range of 64-wide K stages and a private ring of S slots: no barrier in the loop.
//   Stage:  2 loads of the weight tile, XR / 8 of the activation tile (XR = 16 rows, or 8 when
//   M <= 8, which leaves more of the LDS to stages in flight; rows past M re-read the block's first
//   row: their products land in accumulator columns that are never stored), 4 fragment reads,
//   2 MFMAs of 16x16x32 into two accumulators.
//   Needs K % 64 == 0 (LSTM: Ix % 64 == 0 too) and N*K*2 < 4 GiB (32-bit lane offsets); the
//   launcher sends everything else to skinny_kernel.
// ---------------------------------------------------------------------------
template <int N_>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_) : "memory");
}

__device__ __forceinline__ void wait_vmcnt_of(int n) {  // n is a constant after unrolling
  switch (n) {
#define NIMBLE_W(v) case v: wait_vmcnt<v>(); break;
#define NIMBLE_W8(b) NIMBLE_W(b) NIMBLE_W(b + 1) NIMBLE_W(b + 2) NIMBLE_W(b + 3) NIMBLE_W(b + 4) NIMBLE_W(b + 5) NIMBLE_W(b + 6) NIMBLE_W(b + 7)
    NIMBLE_W8(0) NIMBLE_W8(8) NIMBLE_W8(16) NIMBLE_W8(24) NIMBLE_W8(32) NIMBLE_W8(40) NIMBLE_W8(48) NIMBLE_W8(56)
#undef NIMBLE_W8
#undef NIMBLE_W
    default: wait_vmcnt<0>(); break;
  }
}

// Measured on a 134 MB layer (8192 x 8192) streamed from HBM, microseconds at 1 / 16 rows (skinny_kernel:
// 31.8 / 38.1): NW = 4 with S = 2, 3, 4, 6, 8: 31.8, 30.0, 27.9, 30.7, 31.1 / 34.3, 30.8, 30.5, 32.7, 33.3;
// NW = 8 with S = 2, 3, 4: 24.7, 24.5, 24.4 / 27.6, 28.0, 27.9; NW = 8, XR = 8, S = 3: 23.9 (four rows:
// 25.0).  Two groups of 16 weight rows per workgroup sharing one activation tile (half the activation
// traffic, but one workgroup per compute unit): 25.9-27.4 / 27.5-28.8, not kept.
template <bool LSTM, int S, int NW = 8, int XR = 16>
__global__ void __launch_bounds__(NW * 64) stream_kernel(SkinnyArgs s) {
  static_assert(XR == 8 || XR == 16, "the activation tile is one or two loads of 8 rows");
  constexpr int RG = 1;                             // groups of 16 weight rows per workgroup
  constexpr int LD = 2 * RG + XR / 8;               // direct loads per stage and wave
  constexpr int SLOT = (16 * RG + XR) * 128 / 16;   // uint4 per slot: weight rows, then XR activation rows, of 128 bytes
  static_assert(S >= 2 && S <= 8 && (S - 1) * LD <= 63, "the wait counter holds 6 bits");
  __shared__ __attribute__((aligned(16))) uint4 ring[NW][S][SLOT];
  static_assert(sizeof(float) * NW * RG * 16 * 17 <= sizeof(uint4) * NW * S * SLOT, "the partial sums reuse the ring");
  // (the waves' partial sums are exchanged through the ring's memory once every wave is done with it)
  float(*red)[RG][16][17] = reinterpret_cast<float(*)[RG][16][17]>(&ring[0][0][0]);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: stage addresses live in scalar registers
  const int r = lane & 15, gq = lane >> 4;
  const int M = s.M, N = s.N, K = s.K;
  const int mbase = blockIdx.y * 16;

  // operands of the epilogue, fetched first so their latency hides behind the weight stream
  float pre_bias[4] = {0.f, 0.f, 0.f, 0.f};
  float pre_c = 0.f;
  if (LSTM) {
    const int mm = (tid & 63) >> 2, u = tid & 3;
    const int m = mbase + mm, unit = blockIdx.x * 4 + u;
    if (tid < 64 && m < M && unit < s.H) {
      if (s.pre) {
#pragma unroll
        for (int q = 0; q < 4; ++q) pre_bias[q] = s.pre[((long long)m * 4 + q) * s.H + unit];
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) pre_bias[q] = bf2f(s.bias[q * s.H + unit]);
      }
      pre_c = s.c_prev[(long long)m * s.H + unit];
    }
  } else {
#pragma unroll
    for (int g = 0; g < RG; ++g) {
      const int n = (blockIdx.x * RG + g) * 16 + (tid & 15);
      if (tid < 256 && n < N && s.epilogue != NIMBLE_EPI_NONE) pre_bias[g] = bf2f(s.bias[n]);
    }
  }

  // direct loads: instruction i (0, 1) of a tile brings rows 8 i .. 8 i + 7, lane -> row 8 i + (lane >> 3),
  // physical chunk lane & 7 of that row, which holds logical chunk (lane & 7) ^ ((row >> 1) & 7)
  uint32_t w_off[2 * RG], x_off[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = 8 * i + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
#pragma unroll
    for (int g = 0; g < RG; ++g) {
      long long wrow;
      if (LSTM) {
        int unit = blockIdx.x * 4 + (row & 3);
        unit = unit < s.H ? unit : s.H - 1;
        wrow = (long long)(row >> 2) * s.H + unit;
      } else {
        const int n = (blockIdx.x * RG + g) * 16 + row;
        wrow = n < N ? n : N - 1;
      }
      w_off[2 * g + i] = (uint32_t)((wrow * K + c * 8) * 2);
    }
    const int m = mbase + row;
    const int mc = m < M ? m : mbase;
    // LSTM: the row stride of the source a stage reads from (x: Ix, h: H) is applied per stage
    x_off[i] = LSTM ? (uint32_t)(mc) : (uint32_t)(((long long)mc * K + c * 8) * 2);
  }
  const int xc0 = (lane & 7) ^ (((lane >> 3) >> 1) & 7);        // logical chunk of this lane, rows 0..7
  const int xc1 = (lane & 7) ^ (((8 + (lane >> 3)) >> 1) & 7);  // rows 8..15

  // this wave's contiguous range of 64-wide k stages
  const int stages = K >> 6;
  const int per_wave = (stages + NW - 1) / NW;
  const int st_begin = wave * per_wave;
  const int st_end = (st_begin + per_wave) < stages ? (st_begin + per_wave) : stages;
  const int n_st = st_end > st_begin ? st_end - st_begin : 0;

  const uint32_t ring_lds = __builtin_amdgcn_readfirstlane(lds_addr_of(&ring[wave][0][0]));
  auto issue = [&](int st, int slot) {  // st: stage index within K
    const int k0 = st << 6;
    const uint32_t dst = ring_lds + slot * (SLOT * 16);
#pragma unroll
    for (int u = 0; u < 2 * RG; ++u) dma16_so(w_off[u], s.w + k0, dst + u * 1024);
    constexpr uint32_t XT = RG * 2048;  // the activation tile follows the weight rows
    if (LSTM) {
      // the stage lies in x (k0 < Ix) or in h: Ix is a multiple of 64
      const bool in_x = k0 < s.Ix;
      const u16* base = in_x ? s.x + k0 : s.h + (k0 - s.Ix);
      const uint32_t ld = in_x ? (uint32_t)s.Ix : (uint32_t)s.H;
      dma16_so((x_off[0] * ld + xc0 * 8) * 2u, base, dst + XT);
      if (XR == 16) dma16_so((x_off[1] * ld + xc1 * 8) * 2u, base, dst + XT + 1024);
    } else {
      dma16_so(x_off[0], s.x + k0, dst + XT);
      if (XR == 16) dma16_so(x_off[1], s.x + k0, dst + XT + 1024);
    }
  };

  // fragment reads: lane (r, gq) -> row r, logical chunk gq (first half of the stage) or gq + 4
  // (XR = 8: lanes of rows 8..15 read rows 0..7 again; those accumulator columns are never stored)
  const int sw = (r >> 1) & 7;
  const int f0 = r * 8 + (gq ^ sw), f1 = r * 8 + ((gq + 4) ^ sw);
  const int xr = r & (XR - 1), xsw = (xr >> 1) & 7;
  const int g0 = RG * 128 + xr * 8 + (gq ^ xsw), g1 = RG * 128 + xr * 8 + ((gq + 4) ^ xsw);
  f32x4 acc[RG][2];
#pragma unroll
  for (int g = 0; g < RG; ++g) acc[g][0] = acc[g][1] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto compute = [&](int slot) {
    const uint4* t = &ring[wave][slot][0];
    const uint4 xa = t[g0], xb = t[g1];
    uint4 wa[RG], wb[RG];
#pragma unroll
    for (int g = 0; g < RG; ++g) wa[g] = t[g * 128 + f0], wb[g] = t[g * 128 + f1];
#pragma unroll
    for (int g = 0; g < RG; ++g) {
      acc[g][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[g]), as_bf16x8(xa), acc[g][0], 0, 0, 0);
      acc[g][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wb[g]), as_bf16x8(xb), acc[g][1], 0, 0, 0);
    }
    // the slot is refilled only after these reads have returned
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  };

  if (n_st >= S - 1) {
    // S-1 stages in flight; stage i of this wave lives in slot i % S
#pragma unroll
    for (int i = 0; i < S - 1; ++i) issue(st_begin + i, i);
    int slot = 0, fill = S - 1;
    for (int i = 0; i + (S - 1) < n_st; ++i) {
      issue(st_begin + i + S - 1, fill);       // the slot of stage i - 1, whose reads have returned
      wait_vmcnt<(S - 1) * LD>();                // stage i has landed
      compute(slot);
      slot = slot + 1 == S ? 0 : slot + 1;
      fill = fill + 1 == S ? 0 : fill + 1;
    }
    // the last S-1 stages: nothing more to issue, the wait count shrinks with what is left in flight
#pragma unroll
    for (int j = S - 2; j >= 0; --j) {
      wait_vmcnt_of(j * LD);
      compute(slot);
      slot = slot + 1 == S ? 0 : slot + 1;
    }
  } else {
    for (int i = 0; i < n_st; ++i) issue(st_begin + i, i);
    wait_vmcnt<0>();
    for (int i = 0; i < n_st; ++i) compute(i);
  }

  // accumulator of lane (r, gq), register v: weight row i = 4 gq + v, activation row j = r
  __syncthreads();  // every wave has read its last fragments: the ring's memory is free
#pragma unroll
  for (int g = 0; g < RG; ++g)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][g][r][gq * 4 + v] = acc[g][0][v] + acc[g][1][v];
  __syncthreads();

  if (LSTM) {
    // thread -> (row m, hidden unit u); the four gates sit at columns gate*4 + u
    if (tid < 64) {
      const int mm = tid >> 2, u = tid & 3;
      const int m = mbase + mm;
      const int unit = blockIdx.x * 4 + u;
      if (m < M && unit < s.H) {
        float gate[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = q * 4 + u;
          float sum = 0.f;
#pragma unroll
          for (int wv = 0; wv < NW; wv += 4)
            sum += (red[wv][0][mm][col] + red[wv + 1][0][mm][col]) + (red[wv + 2][0][mm][col] + red[wv + 3][0][mm][col]);
          gate[q] = sum + pre_bias[q];
        }
        const long long o = (long long)m * s.H + unit;
        float cn;
        const float hn = lstm_cell(gate, pre_c, cn);
        s.c_out[o] = cn;
        ((u16*)s.y)[o] = f2bf(hn);
      }
    }
  } else if (tid < 256) {
    const int mm = tid >> 4, nn = tid & 15;
    const int m = mbase + mm;
#pragma unroll
    for (int g = 0; g < RG; ++g) {
      const int n = (blockIdx.x * RG + g) * 16 + nn;
      if (n < N && m < M) {
        float sum = 0.f;
#pragma unroll
        for (int wv = 0; wv < NW; wv += 4)
          sum += (red[wv][g][mm][nn] + red[wv + 1][g][mm][nn]) + (red[wv + 2][g][mm][nn] + red[wv + 3][g][mm][nn]);
        const float v = epilogue(sum, s.alpha, pre_bias[g], s.epilogue);
        const long long o = (long long)m * N + n;
        if (s.out_f32)
          ((float*)s.y)[o] = v;
        else
          ((u16*)s.y)[o] = f2bf(v);
      }
    }
  }
}

}  // namespace nimble
#endif
