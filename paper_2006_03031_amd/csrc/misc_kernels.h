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

}  // namespace nimble
#endif
