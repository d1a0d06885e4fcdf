// Fully bounds-checked GEMM for any shape, row softmax, fused attention for head dimension 64.
#ifndef NIMBLE_MISC_KERNELS_H_
#define NIMBLE_MISC_KERNELS_H_
#include "device_common.h"

namespace nimble {

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

// b [T, K, N] -> bt [T, N, K] (bf16), 32 x 32 tiles through LDS: the NN batch_matmul is run as
// the NT one on the transposed operand, which lives in the caller's workspace.
__global__ void __launch_bounds__(256)
    transpose_kn_kernel(const u16* __restrict__ b, u16* __restrict__ bt, int K, int N) {
  __shared__ u16 tile[32][33];
  const long long plane = (long long)K * N;
  const u16* src = b + blockIdx.z * plane;
  u16* dst = bt + blockIdx.z * plane;
  const int k0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int k = k0 + ty + 8 * r, n = n0 + tx;
    if (k < K && n < N) tile[ty + 8 * r][tx] = src[(long long)k * N + n];
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int n = n0 + ty + 8 * r, k = k0 + tx;
    if (n < N && k < K) dst[(long long)n * K + k] = tile[tx][ty + 8 * r];
  }
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
// and walks the keys in blocks of 64 or 128 with a running row maximum and row sum.
//   scores:  MFMA 16x16x32 with 16 key rows on the A side and the wave's 16 query rows on
//            the B side: a lane holds, for its query row m = lane & 15, the keys
//            16 t + 4 (lane >> 4) + v of key tile t (v = 0..3).
//   P.V:     k runs over keys.  The sum over k does not care about order, so the 8 k-slots
//            of lane group g in MFMA u are DEFINED as the 8 keys that group already holds:
//            32u + 4g + (0..3) and 32u + 16 + 4g + (0..3).  P then goes from the score
//            accumulators to the MFMA operand without leaving the lane; V is staged in LDS
//            transposed ([d][key]) so the matching 8 values are two 8-byte reads.
// ---------------------------------------------------------------------------
// BJ: keys per block, 64 or 128.  A block is a chain of dependent steps (fetch, stage, barrier, 2 MFMAs
// deep of scores, exponentials, 2 MFMAs deep of P.V) walked by a workgroup of one wave per SIMD, and it is
// bound by the instructions a wave has to issue: timed inside the kernel at 64 keys, 0.46 us until K and V are
// staged, 0.26 us of scores, 0.26 us of softmax, 0.38 us of P.V, 0.2 us in the two barriers.  What helped
// (12 heads, microseconds at L = 128 / 256 / 512, from 5.1 / 7.6 / 12.9): 128 keys per block, twice the
// independent work in every step of the chain (4.8 / 7.1 / 11.8); then the softmax in base 2 on the raw scores
// (one fused multiply-add and one exp2 per score, the mask only in the last block, the running output
// rescaled only when a maximum moved) and all of a block's K and V loads issued together (the compiler had
// put three of the eight one behind the other): 4.3 / 6.1 / 9.8.  What did not: K and V fetched into registers one or
// two blocks ahead; conflict-free transposing writes of V (two keys per 32-bit word: -3 % to +6 %); the keys
// split over two or four groups of four waves per workgroup with their own staging areas, merged through LDS
// at the end (two groups 5.1 / 6.5 / 9.3, four groups 7.2 / 8.4 / 11.4: more waves per SIMD do not help a
// chain that is bound by instruction issue, and the larger workgroup starts later).
template <int BJ>
__global__ void __launch_bounds__(256)
    attention64_kernel(const u16* __restrict__ q, const u16* __restrict__ k, const u16* __restrict__ v,
                       u16* __restrict__ o, int L, float alpha) {
  constexpr int D = 64, VT_LD = BJ + 4;  // V^T rows padded by 4 elements against bank conflicts
  constexpr int NT = BJ / 16;            // key tiles of 16 per block
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
  float row_max = -INFINITY, row_sum = 0.f;  // row_max in raw-score units; row_sum: this lane's share, reduced at the end
  const float a2 = alpha * 1.4426950408889634f;

  for (int j0 = 0; j0 < L; j0 += BJ) {
    __syncthreads();  // the previous block's fragments have been read
    {
      // stage K (row-major, swizzled) and V (transposed): BJ * 8 chunks of 16 bytes each, BJ / 32 per thread;
      // all loads first
      uint4 kc[BJ / 32], vc[BJ / 32];
#pragma unroll
      for (int i = 0; i < BJ / 32; ++i) {
        const int idx = tid + i * 256;
        const int row = idx >> 3, c = idx & 7;
        const int jr = (j0 + row < L) ? (j0 + row) : (L - 1);
        kc[i] = *(const uint4*)(k + head + (long long)jr * D + c * 8);
        vc[i] = *(const uint4*)(v + head + (long long)jr * D + c * 8);
      }
      // (left to itself the compiler issues some of these loads one at a time, each behind the LDS writes of
      // the one before: three trips to L2 in a row per block of 128 keys)
#pragma unroll
      for (int i = 0; i < BJ / 32; ++i) {
        keep_in_registers(kc[i]);
        keep_in_registers(vc[i]);
      }
#pragma unroll
      for (int i = 0; i < BJ / 32; ++i) {
        const int idx = tid + i * 256;
        const int row = idx >> 3, c = idx & 7;
        Ks[row * 8 + (c ^ ((row >> 1) & 7))] = kc[i];
        const u16* ve = (const u16*)&vc[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) Vt[(c * 8 + e) * VT_LD + row] = ve[e];
      }
    }
    __syncthreads();

    // scores of the wave's 16 rows against the keys of the block
    f32x4 sacc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      sacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int krow = t * 16 + r;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const bf16x8 kf = as_bf16x8(Ks[krow * 8 + ((kk * 4 + g) ^ ((krow >> 1) & 7))]);
        sacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[kk], sacc[t], 0, 0, 0);
      }
    }
    // Softmax in base 2 on the raw scores (alpha > 0, checked by the entry point): p = 2^(a2 s - a2 max) with
    // a2 = alpha log2 e is one fused multiply-add and one exp2 per score; the running maximum is kept in
    // raw-score units.  Keys past L exist only in the last block; the running output is rescaled only when some
    // row's maximum moved (a factor of exactly 1 otherwise).
    if (j0 + BJ > L) {  // uniform
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (j0 + t * 16 + g * 4 + e >= L) sacc[t][e] = -INFINITY;
    }
    float bmax = -INFINITY;  // block maximum of the row (4 lanes share a row)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int e = 0; e < 4; ++e) bmax = fmaxf(bmax, sacc[t][e]);
    bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
    const float new_max = fmaxf(row_max, bmax);  // finite: key j0 < L is in every block
    if (__any(new_max != row_max)) {
      const float rescale = __builtin_amdgcn_exp2f((row_max - new_max) * a2);  // 2^-inf = 0 in the first block
      row_sum *= rescale;
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) oacc[t][e] *= rescale;
    }
    row_max = new_max;
    const float nm2 = -new_max * a2;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[t][e], a2, nm2));
        sacc[t][e] = pv;
        row_sum += pv;
      }
    // O += P.V: MFMA u consumes key tiles 2u and 2u+1
#pragma unroll
    for (int u = 0; u < NT / 2; ++u) {
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

}  // namespace nimble
#endif
