// Device-side helpers shared by every kernel: bf16 conversion, the dense epilogue, direct
// global->LDS loads, the workgroup-to-tile map.
#ifndef NIMBLE_DEVICE_COMMON_H_
#define NIMBLE_DEVICE_COMMON_H_
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

// gelu(v) = v/2 (1 + erf(v / sqrt 2)), evaluated as v * sigmoid(a v + b v^3 + c v^5) with
// a = 1.5950, b = 0.074011, c = -0.00070303 (a least-squares fit of the odd quintic to the erf form
// on |v| <= 9, the constants below being -log2(e) times these; largest deviation 2.5e-5, an order of
// magnitude below the bfloat16 spacing of the result; v^2 is clamped at 81, beyond which the
// sigmoid is 0 or 1): seven ordinary instructions plus the hardware exp2 and reciprocal.  The
// epilogue of a GELU layer is bound by exactly these instructions (128 outputs per lane with
// nothing to overlap them): the three-term rational-times-Gaussian erf of Abramowitz & Stegun
// 7.1.25 (same accuracy, eleven instructions) was the previous form, 7.1.26 and the library erff
// cost more still.  Reading the function from a 1024-segment table of chords in LDS (five ordinary
// instructions and one data-dependent 8-byte read per element) was measured too: 2-6 % slower per
// kernel, the reads' bank conflicts cost more than the arithmetic they replace.
__device__ __forceinline__ float gelu_erf(float v) {
  const float t = fminf(v * v, 81.0f);
  float p = fmaf(0.0010142630f, t, -0.10677572f);  // -log2(e) (a + b t + c t^2)
  p = fmaf(p, t, -2.3011212f);
  const float e = __builtin_amdgcn_exp2f(p * v);    // exp(-(a v + b v^3 + c v^5))
  return v * __builtin_amdgcn_rcpf(1.0f + e);
}

// The LSTM cell's nonlinearities on the hardware's exp2 and reciprocal (about 1 ulp each):
// sigma(z) = 1 / (1 + 2^(-z log2 e)), tanh(z) = 1 - 2 / (1 + 2^(2 z log2 e)); both saturate correctly
// (2^x -> inf gives 1/inf = 0).  The absolute error is a few 1e-7: far inside the bf16 rounding of h
// and the f32 bar of c.  The library forms (a division sequence, a branching tanh) are 150-250
// dependent instructions per cell, which is most of what a one-row step does after its last MFMA.
__device__ __forceinline__ float sigmoidf(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}
__device__ __forceinline__ float tanh_fast(float z) {
  return fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.8853900817779268f * z)), 1.0f);
}
// One cell update from the four gate pre-activations (i, f, g, o): returns h, writes c.  Every LSTM
// kernel goes through this one function, with the fused multiply-add spelled out, so that they agree
// bit for bit.
// (The one-launch token loop spreads the four gates of a cell over four lanes and then does exactly
// these operations on the gathered values.)
__device__ __forceinline__ float lstm_cell(const float (&gate)[4], float c_prev, float& c_new) {
  const float a_i = sigmoidf(gate[0]), a_f = sigmoidf(gate[1]), a_g = tanh_fast(gate[2]), a_o = sigmoidf(gate[3]);
  c_new = fmaf(a_f, c_prev, a_i * a_g);
  return a_o * tanh_fast(c_new);
}
// Makes a value opaque to the compiler at this point: what was loaded before a loop stays in its
// registers instead of being loaded again inside the loop.
__device__ __forceinline__ void keep_in_registers(uint4& v) {
  asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
}

// `bias` is 0 when the epilogue has none, so one fused multiply-add serves every case.
__device__ __forceinline__ float epilogue(float acc, float alpha, float bias, int epi) {
  const float v = fmaf(alpha, acc, bias);
  return epi == NIMBLE_EPI_BIAS_GELU_ERF ? gelu_erf(v) : v;
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
// acc += a . b on the matrix core with the accumulator held in place in the accumulation
// registers.  Written as a volatile statement: the order in the source is the order issued, and
// the register allocator cannot decide to shuffle accumulators between register files.
__device__ __forceinline__ void mfma_acc(f32x4& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// The compiler does not know that the statement above is a matrix instruction, so it adds none of
// the wait states a matrix result needs before anything else reads its registers (a copy, a
// spill store, the epilogue's arithmetic), and it may place such a reader directly behind the
// statement.  The last MFMA of a tile's last stage therefore carries the wait states itself, in
// the same statement so that nothing can come in between: `last` (wave-uniform) != 0 runs 32 idle
// cycles, by the end of which this result and those of all earlier MFMAs have been written.
__device__ __forceinline__ void mfma_acc_last(f32x4& acc, const bf16x8& a, const bf16x8& b, int last) {
  asm volatile(
      "v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0\n\t"
      "s_cmp_eq_u32 %3, 0\n\t"
      "s_cbranch_scc1 .Lnimble_mfma_done_%=\n\t"
      "s_nop 15\n\t"
      "s_nop 15\n"
      ".Lnimble_mfma_done_%=:"
      : "+a"(acc)
      : "v"(a), "v"(b), "s"(__builtin_amdgcn_readfirstlane(last))
      : "scc");
}

// The direct global -> LDS load addressed as a wave-uniform 64-bit base (in SGPRs) plus a 32-bit
// per-lane byte offset, which keeps per-lane 64-bit pointers out of the vector registers.
__device__ __forceinline__ void dma16_so(uint32_t voff, const void* sbase, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n" ::"v"(voff), "s"(sbase),
               "s"(lds_addr)
               : "memory", "m0");
}
// One dword per lane: a wave instruction fills 256 contiguous bytes of LDS.
__device__ __forceinline__ void dma4_so(uint32_t voff, const void* sbase, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1\n" ::"v"(voff), "s"(sbase),
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

}  // namespace nimble
#endif
