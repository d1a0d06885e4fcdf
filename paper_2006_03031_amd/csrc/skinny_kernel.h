// Weight-streaming kernel for at most 64 rows per workgroup, with the fused LSTM cell epilogue.
#ifndef NIMBLE_SKINNY_KERNEL_H_
#define NIMBLE_SKINNY_KERNEL_H_
#include "device_common.h"

namespace nimble {

// ---------------------------------------------------------------------------
// Skinny kernel: at most 64 rows of activations per workgroup, 16 weight rows.
// Every weight element is read by exactly one lane of a workgroup, straight into
// an MFMA operand (no LDS staging: there is no reuse to stage for).
// Tried and not kept: issuing the next eight steps' loads ahead of the current
// MFMAs (needs unconditional, clamped loads so that the compiler can count them;
// 160 registers and three waves per SIMD instead of four: 10-15 % slower).
// ---------------------------------------------------------------------------
struct SkinnyArgs {
  const u16* x;     // [M, K]  (LSTM: [B, Ix])
  const u16* h;     // LSTM only: [B, H]
  const u16* w;     // [N, K]  (LSTM: [4H, Ix+H])
  const u16* bias;  // [N]
  void* y;          // [M, N] bf16 or f32 (LSTM: h_out [B,H] bf16)
  const float* c_prev;  // LSTM only
  float* c_out;         // LSTM only
  const float* pre;     // LSTM only, may be null: [B, 4H] input share of the gates (bias included);
                        // then x is absent (Ix = 0) and bias is not read
  int M, N, K;      // LSTM: M = B, N = 4H, K = Ix + H
  int Ix, H;        // LSTM only
  int epilogue, out_f32;
  float alpha;      // scale of the product (dense and LSTM: 1; batch_matmul with one batch: its alpha)
};

// U = 32-wide k steps whose loads a wave issues together before it multiplies.  8 keeps four
// waves per SIMD; 16 (launched for up to 16 rows when the grid has no more workgroups than the
// chip has compute units and K > 1024, i.e. a wave has more than eight steps) doubles the bytes a
// compute unit keeps in flight when it holds a single workgroup: 33 MB layers streamed from HBM
// 7-9 % faster, 134 MB layers (two workgroups per compute unit) unchanged at one row and 7-10 %
// slower at 8-16 rows, K = 768 layers 3 % slower (the steps past the end still cost an MFMA
// each), hence the conditions.
template <int MT, bool LSTM, int U = 8>
__global__ void __launch_bounds__(256) skinny_kernel(SkinnyArgs s) {
  __shared__ float red[4][MT][16][17];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, gq = lane >> 4;
  const int M = s.M, N = s.N, K = s.K;
  const int mbase = blockIdx.y * (16 * MT);  // the launch gives every workgroup along y 16 MT rows

  // operands of the epilogue, fetched first so their latency hides behind the weight stream
  float pre_bias[4] = {0.f, 0.f, 0.f, 0.f};
  float pre_c = 0.f;
  if (LSTM) {
    const int t = tid >> 6, mm = (tid & 63) >> 2, u = tid & 3;
    const int m = mbase + t * 16 + mm, unit = blockIdx.x * 4 + u;
    if (t < MT && m < M && unit < s.H) {
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
        float cn;
        const float hn = lstm_cell(gate, pre_c, cn);
        s.c_out[o] = cn;
        ((u16*)s.y)[o] = f2bf(hn);
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
          const float v = epilogue(sum, s.alpha, b, s.epilogue);
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

}  // namespace nimble
#endif
