// Token loop of one LSTM sequence in a single launch: recurrent weights resident in registers, the
// hidden state handed from step to step through tagged words in memory, every wait bounded.
#ifndef NIMBLE_LSTM_SEQ_KERNEL_H_
#define NIMBLE_LSTM_SEQ_KERNEL_H_
#include "device_common.h"

namespace nimble {

// ---------------------------------------------------------------------------
// The evaluation section's LSTM remark: a cell step is too small to fill the chip, so a sequence is
// bound by what separates the steps.  As one launch per step that is the 2-3 us between dependent
// kernels; here the steps of a sequence run inside one launch.
//   Inputs: pre [T, B, 4H] f32, the inputs' share of the gates with the bias added (one dense call
//   over all T*B tokens ahead of the loop), w_h [4H, H] bf16, h_0 [B, H] bf16, c_0 [B, H] f32.
//   Grid: H / 16 workgroups of 8 waves; a workgroup owns 16 hidden units = 64 gate rows (G = 4 groups
//   of the i, f, g, o rows of 4 units) and keeps those rows of w_h in registers for the whole
//   sequence (wave w: the 64-wide K stages w * per_wave ...: 8 registers per group and stage).  Per
//   step a wave fetches its K range of h_{t-1}, multiplies, leaves its partial sums in LDS; after one
//   barrier four neighbouring lanes per (row, unit) add them up and apply the nonlinearity, one gate
//   each, and the first of them updates the cell.  c_t stays in that lane's register.
//   Hand-over of h_t: a workgroup publishes its 32 units per row as 32-bit words, bf16 value in the
//   high half and a step tag (1..65535, never 0) in the low half, with device-scope stores into
//   buffer t & 1 of two; a consumer wave loads exactly the words its MFMAs need, device scope, and
//   repeats until every tag is this step's.  Data and arrival are one word: no counter, no fence,
//   one store and one load on the critical path (a counter barrier over 16 workgroups was measured
//   at 0.85 us per step bare and 1.56 us with the data exchanged behind it).  Two buffers suffice:
//   h_t overwrites h_{t-2}, which every workgroup has finished reading before it publishes h_{t-1},
//   without which nobody can compute h_t.  Tags t and t-2 always differ (the tag period is odd).
//   The words are cleared, and buffer 0 filled with h_0, by lstm_seq_init_kernel ahead of the launch
//   on the same stream: a stale tag of an earlier launch can never be taken for this one's.
//   Every wait is bounded: a wave polls at most max_polls times per step, checking the give-up word
//   each time; a wave that runs out sets it, and every workgroup leaves at its next check.  So the
//   grid drains whatever happens (fewer workgroups resident than launched, a stalled neighbour),
//   the host reads the word afterwards and runs the sequence step by step instead.  max_polls = 0
//   gives up at the first wait: the host-side way to exercise that path.
//   Arithmetic: identical, bit for bit, to the per-step kernel on the same shapes (stream_kernel
//   with 8 waves: the same K stages per wave, the same two accumulators per stage pair, the same
//   order of adding the waves' partial sums, the same cell function).
//   Measured, microseconds per step at 1 / 2 / 4 rows (a captured graph of per-step launches: 2.65-2.72 at
//   H = 512, 2.85-2.95 at H = 1024): H = 512: 1.89 / 2.02 / 2.41; H = 1024: 2.71 / 3.20 / 3.98.  With 8 groups
//   per workgroup (half the workgroups) 2.14 / 2.15 / 2.55 and 2.91 / 3.18 / 4.27, with 2 groups 2.08 / 2.25 /
//   2.73: fewer groups shorten a workgroup's MFMAs and sums, more workgroups lengthen everybody's fetch.
//   A step at one row is one trip to the memory side and back (0.75 us from the store to the polled
//   words), the MFMAs and partial sums, the barrier, the cell arithmetic; with more rows the fetch
//   reads that many more words per workgroup, which the per-step kernel gets from one L2, and up to 16 rows
//   (built first) it cost 4.7 us per step: hence the limit of 4 rows.  Tried and not kept: every wave
//   multiplying its own 16 gate rows over the whole of K from a copy of h in LDS and updating its cells
//   itself (no partial sums, no single epilogue: 4.1 us per step, the eight waves' reads of all of h cost
//   more LDS time than the sums saved); all workgroups on one XCD (every 8th of a grid 8 times as large)
//   exchanging the words with workgroup-scope loads: the words never became visible, the loop gave up as
//   designed.
// ---------------------------------------------------------------------------
struct LstmSeqArgs {
  const float* pre;   // [T, B, 4H]
  const u16* w_h;     // [4H, H]
  const u16* h0;      // [B, H]
  const float* c0;    // [B, H]
  u16* h_seq;         // [T, B, H]
  float* c_out;       // [B, H]
  uint32_t* ctl;      // 64 words: [0] give-up word, [1] workgroups that ran all T steps
  uint32_t* exch;     // [2][B][H] tagged words
  int T, B, H;
  uint32_t max_polls;
};

__device__ __forceinline__ uint32_t lstm_seq_tag(int t) { return (uint32_t)(t % 65535) + 1u; }

// Clears the control words and buffer 1, fills buffer 0 with h_0 tagged as step 0.
__global__ void __launch_bounds__(256) lstm_seq_init_kernel(LstmSeqArgs a) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int n = a.B * a.H;
  if (i < 64) a.ctl[i] = 0u;
  if (i < n) {
    a.exch[i] = ((uint32_t)a.h0[i] << 16) | lstm_seq_tag(0);
    a.exch[n + i] = 0u;
  }
}

// PW: K stages of 64 per wave, ceil(H / 64 / 8); G: groups of 16 gate rows (4 units) per workgroup
template <int PW, int G>
__global__ void __launch_bounds__(512) lstm_seq_kernel(LstmSeqArgs a) {
  constexpr int SCOPE = __HIP_MEMORY_SCOPE_AGENT;
  constexpr int U = 4 * G;  // units per workgroup
  // partial sums [buffer][wave][group][row][gate row of the group], a group's block padded by 4 floats so that
  // the 8 groups' columns fall into different banks; a lane writes its 4 sums as one 16-byte word
  constexpr int GS = 16 * 16 + 4;
  __shared__ __attribute__((aligned(16))) float red[2][8][G * GS];
  __shared__ int s_abort[2];  // by step parity: a wave already polling for step t+1 never writes the word step t reads

  const int wg = (int)blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, gq = lane >> 4;
  const int T = a.T, B = a.B, H = a.H;

  // this wave's K stages: the per-step kernel's partition
  const int stages = H >> 6;
  const int per_wave = (stages + 7) / 8;
  const int st_begin = wave * per_wave;
  const int st_end = (st_begin + per_wave) < stages ? (st_begin + per_wave) : stages;
  const int n_st = st_end > st_begin ? st_end - st_begin : 0;  // <= PW (the launcher picks PW = per_wave)

  // recurrent weights of this workgroup's 128 gate rows over this wave's stages, in the MFMA operand
  // layout: lane (r, gq) holds 8 k of tile row r = gate r >> 2 of unit 4 g + (r & 3)
  uint4 wa[G][PW], wb[G][PW];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const int unit = wg * U + g * 4 + (r & 3);
    const u16* wrow = a.w_h + ((long long)(r >> 2) * H + unit) * H;
#pragma unroll
    for (int s = 0; s < PW; ++s) {
      if (s < n_st) {
        const int k = (st_begin + s) * 64 + gq * 8;
        wa[g][s] = *(const uint4*)(wrow + k);
        wb[g][s] = *(const uint4*)(wrow + k + 32);
      } else {
        wa[g][s] = wb[g][s] = make_uint4(0, 0, 0, 0);
      }
      // (left to itself the compiler loads the weights anew in every step instead of keeping them)
      keep_in_registers(wa[g][s]);
      keep_in_registers(wb[g][s]);
    }
  }

  // cell update: thread -> (row mm < 4, unit u of the workgroup's 32, gate q): four neighbouring lanes share a
  // cell, each adds up and activates one gate; the lane of gate 0 owns c and writes h
  const int mm = tid / (4 * U), u = (tid >> 2) & (U - 1), q = tid & 3;
  const int unit = wg * U + u;
  const bool owner = mm < B;
  float c = (owner && q == 0) ? a.c0[(long long)mm * H + unit] : 0.f;

  if (tid < 2) s_abort[tid] = 0;
  __syncthreads();

  const int xrow = r < B ? r : 0;  // rows past B read row 0: their accumulator columns are never used
  const long long plane = (long long)B * H;

  // The inputs' share of the gates streams from memory, a fresh line per step: it is fetched one step
  // ahead, and behind the wave's poll loads (loads return in order: in front of them it would hold
  // every poll back by a trip to HBM).
  float pr = 0.f, pr_next = 0.f;
  if (owner) pr = a.pre[((long long)mm * 4 + q) * H + unit];
  for (int t = 1; t <= T; ++t) {
    // h_{t-1}: this wave's k range of row xrow, polled until every word carries the tag of step t-1
    const uint32_t want = lstm_seq_tag(t - 1);
    const uint32_t* src = a.exch + (long long)((t - 1) & 1) * plane + (long long)xrow * H;
    uint4 xa[PW], xb[PW];
    bool gave_up = false;
    if (n_st > 0) {
      uint32_t polls = 0;
      for (;;) {
        // (wave-uniform: every lane counts alike and reads the same give-up word)
        if (polls >= a.max_polls) {
          gave_up = true;
          break;
        }
        ++polls;
        // the give-up word travels with the data words, not ahead of them: one round trip per poll
        const uint32_t others_gave_up = __hip_atomic_load(a.ctl, __ATOMIC_RELAXED, SCOPE);
        uint32_t bad = 0;
#pragma unroll
        for (int s = 0; s < PW; ++s) {
          if (s < n_st) {
            const unsigned long long* p =
                (const unsigned long long*)(src + (st_begin + s) * 64 + gq * 8);
            unsigned long long v[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              v[j] = __hip_atomic_load(p + j, __ATOMIC_RELAXED, SCOPE);           // k + 0..7
              v[4 + j] = __hip_atomic_load(p + 16 + j, __ATOMIC_RELAXED, SCOPE);  // k + 32..39
            }
            uint32_t pk[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const uint32_t lo = (uint32_t)v[j], hi = (uint32_t)(v[j] >> 32);
              bad |= ((lo ^ want) | (hi ^ want)) & 0xffffu;
              pk[j] = (lo >> 16) | (hi & 0xffff0000u);
            }
            xa[s] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
            xb[s] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
          } else {
            xa[s] = xb[s] = make_uint4(0, 0, 0, 0);
          }
        }
        if (__all(bad == 0u)) break;
        if (others_gave_up != 0u) {
          gave_up = true;
          break;
        }
      }
      if (gave_up) {
        if (lane == 0) __hip_atomic_store(a.ctl, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_abort[t & 1] = 1;
      }
    } else {
#pragma unroll
      for (int s = 0; s < PW; ++s) xa[s] = xb[s] = make_uint4(0, 0, 0, 0);
    }

    if (owner && t < T) pr_next = a.pre[(((long long)t * B + mm) * 4 + q) * H + unit];
    // gates' recurrent share: per group two accumulators (first and second half of each stage); all
    // MFMAs first, so that none waits for another's result
    float* rd = red[t & 1][0];
    if (!gave_up) {
      f32x4 acc[G][2];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        acc[g][0] = acc[g][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < PW; ++s) {
          if (s < n_st) {
            acc[g][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[g][s]), as_bf16x8(xa[s]), acc[g][0], 0, 0, 0);
            acc[g][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wb[g][s]), as_bf16x8(xb[s]), acc[g][1], 0, 0, 0);
          }
        }
      }
      // accumulator of lane (r, gq), register v: gate row 4 gq + v of the group, activation row r
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float4 p;
        p.x = acc[g][0][0] + acc[g][1][0];
        p.y = acc[g][0][1] + acc[g][1][1];
        p.z = acc[g][0][2] + acc[g][1][2];
        p.w = acc[g][0][3] + acc[g][1][3];
        if (r < B) *(float4*)(rd + wave * (G * GS) + g * GS + r * 16 + gq * 4) = p;  // rows past B are never read
      }
    }
    __syncthreads();
    if (s_abort[t & 1]) break;  // uniform: written before the barrier, read after it

    {
      // this lane's gate: the waves' partial sums in the per-step kernel's order, the inputs' share, the
      // gate's nonlinearity (the operations of lstm_cell, one gate per lane)
      const int g = u >> 2, uu = u & 3;
      const int row = owner ? mm : 0;
      float sum = 0.f;
#pragma unroll
      for (int wv = 0; wv < 8; wv += 4) {
        const float* e = rd + wv * (G * GS) + g * GS + row * 16 + q * 4 + uu;
        sum += (e[0] + e[G * GS]) + (e[2 * G * GS] + e[3 * G * GS]);
      }
      const float z = sum + pr;
      const float act = q == 2 ? tanh_fast(z) : sigmoidf(z);
      // the four gates of the cell sit in four neighbouring lanes
      const float a_i = __shfl(act, 0, 4), a_f = __shfl(act, 1, 4), a_g = __shfl(act, 2, 4), a_o = __shfl(act, 3, 4);
      // the next step's share of the inputs has had this whole step to arrive; taking it over here, ahead of
      // the stores, keeps any wait for it off the path from the store below to the next step's first poll
      pr = pr_next;
      asm volatile("" : "+v"(pr));
      if (owner && q == 0) {
        c = fmaf(a_f, c, a_i * a_g);
        const u16 hb = f2bf(a_o * tanh_fast(c));
        __hip_atomic_store(a.exch + (long long)(t & 1) * plane + (long long)mm * H + unit,
                           ((uint32_t)hb << 16) | lstm_seq_tag(t), __ATOMIC_RELAXED, SCOPE);
        a.h_seq[((long long)(t - 1) * B + mm) * H + unit] = hb;
      }
    }
    // (the partial sums alternate between two buffers: a wave can write step t+1's only after this
    // step's barrier, and step t+2's only after the barrier of t+1, which every thread reaches after
    // it has read step t's)
  }

  if (!(s_abort[0] | s_abort[1])) {
    if (owner && q == 0) a.c_out[(long long)mm * H + unit] = c;
    if (tid == 0) __hip_atomic_fetch_add(a.ctl + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

}  // namespace nimble
#endif
