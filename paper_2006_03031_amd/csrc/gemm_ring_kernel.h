// Large-tile MFMA kernel: ring of direct global->LDS stages, 16x16x32 MFMA, LDS-transposed epilogue,
// split-K reduction.
#ifndef NIMBLE_GEMM_RING_KERNEL_H_
#define NIMBLE_GEMM_RING_KERNEL_H_
#include <type_traits>

#include "device_common.h"
#include "gemm_tile_kernel.h"

namespace nimble {

// ---------------------------------------------------------------------------
// Interior body of the large tiles.
//   LDS: a ring of S = 4 stages, each BM + BN rows of 32 bf16 (4 chunks of 16
//   bytes); chunk c of row r sits at slot c ^ ((r >> 1) & 3).  A fragment read
//   (lane -> row lane & 15, chunk lane >> 4) then takes 4.3 clocks per wave
//   instruction, the same as a linear read; without the swizzle, or with
//   c ^ (r & 3) or c ^ ((r >> 2) & 3), it was measured at 6.3 (bank conflicts).
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
//   RING_WIDE: stages of 64 k instead of 32.  A row then contributes a whole 128-byte line per
//   stage; with 64-byte pieces every line is asked for twice (once per stage) and the L2s serve
//   one request per channel and clock whatever its size: all compute units together pulled
//   13.5-15.5 TB/s into LDS in 64-byte pieces and 22-26 TB/s in whole lines (loads only, no
//   MFMA), and the 32-wide ring ran within 10 % of the former.  Rows are 8 chunks, chunk c of row
//   r at slot c ^ ((r >> 1) & 7); S = 2 or 3 slots; one barrier per 64 k, placed between the two
//   32-wide halves of a stage: by then every wave has issued (and waited for) its last reads of
//   the slot of stage s, so the slot is refilled with stage s+S, and stage s+1 has landed, whose
//   first fragments are read during the second half's MFMAs.
enum { RING_PINGPONG = 1, RING_SOLO = 2, RING_WIDE = 3 };

// What one tile of a workgroup's walk hands to the next (PF bodies only).
//   PF: the epilogue stages its output through a small LDS area of its own behind the ring instead
//   of through the ring, so the ring is free as soon as the last MFMA has its operands: the body
//   issues the next tile's bias and first S stages before its own epilogue, and the next body
//   starts on a ring that filled while the epilogue ran.  Loads and stores complete in the order
//   a wave issued them, so the next body's waits allow for the epilogue's stores (issued after
//   those loads) by count and its first S-1 stages run while the stores drain.
struct RingLink {
  bool filled = false;  // this tile's bias and first S stages were issued by the previous body
  int stores = -1;      // stores that body issued after them (-1: not known exactly)
  bool next = false;    // a tile follows whose first stages this body may issue
  int next_m0 = 0, next_n0 = 0;
  int parity = 0;       // bias slot of this tile (the next tile's is the other one)
};

template <int BM, int BN, int WGM, int WGN, int S, bool MEDGE, int MODE, bool PF = false>
__device__ __forceinline__ int gemm_ring_body(const GemmArgs& g, const int m0, const int n0,
                                              uint4* smem, const RingLink lk = RingLink{}) {
  constexpr bool WIDE = MODE == RING_WIDE;
  static_assert(!PF || WIDE, "only the 64-wide ring hands tiles over");
  static_assert(WIDE ? (S == 2 || S == 3) : (S >= 4 || (MODE == RING_SOLO && S == 3)),
                "the pipeline keeps S-2 stages in flight");
  constexpr int CH = WIDE ? 8 : 4;      // 16-byte chunks per row and stage
  constexpr int KSH = WIDE ? 6 : 5;     // log2 of the stage width in k
  constexpr int NT = WGM * WGN * 64;
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 16, TN = WN / 16;
  // one pass of the workgroup's loads covers PASS rows; a tile height that is not a whole number
  // of passes rounds up: the ring holds BMP rows of A per stage and the extra rows are loaded
  // from the tile's last row (in bounds, never read back), so that every wave issues the same
  // number of loads per stage and one wait count serves them all
  constexpr int PASS = NT / CH;
  constexpr int A_LD = (BM + PASS - 1) / PASS, B_LD = BN / PASS;
  constexpr int BMP = A_LD * PASS;
  constexpr int LD = A_LD + B_LD;
  static_assert(BN % PASS == 0 && B_LD >= 1, "tile too narrow for the workgroup");
  static_assert(WM % 16 == 0 && WM >= 16, "a wave owns whole 16-row MFMA tiles");
  static_assert(WN % 64 == 0, "the LDS epilogue stages 64-column blocks");
  static_assert(PF || NW * WM * WN * 2 <= S * (BMP + BN) * CH * 16, "epilogue staging does not fit in the ring");
  // stores of the bf16 epilogue per wave (whole-wave instructions), see RingLink
  constexpr int NST = (WN / 64) * (WM / 8);
  static_assert(!PF || NST + (S - 1) * LD + 1 <= 63, "the wait counter holds 63");
  uint4(*As)[BMP * CH] = reinterpret_cast<uint4(*)[BMP * CH]>(smem);
  uint4(*Bs)[BN * CH] = reinterpret_cast<uint4(*)[BN * CH]>(smem + S * BMP * CH);

  // gridDim.y > 1: K is cut into gridDim.y slices of whole stages; slice blockIdx.y writes its
  // f32 partial sums to its own [M,N] plane of the output (g.c is then the split-K workspace)
  const int z = blockIdx.z;
  const int stages_all = g.K >> KSH;
  const int stages_per = (stages_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int stage0 = (int)blockIdx.y * stages_per;
  const int KS = (stages_all - stage0) < stages_per ? (stages_all - stage0) : stages_per;
  const u16* __restrict__ A = (const u16*)g.a + (long long)z * g.sa + (stage0 << KSH);
  const u16* __restrict__ B = (const u16*)g.b + (long long)z * g.sb + (stage0 << KSH);
  // (the thread index goes through an empty volatile statement: a workgroup calls this body once
  // per tile, and without it the compiler keeps every per-lane address computed from it alive
  // from one tile to the next, which pushed the 256x256 tile 50-90 registers over its budget)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // loads: pass i covers chunk ids i*NT + tid: row = i*(NT/4) + (tid >> 2), slot = tid & 3.
  // Address = uniform base of (tile row 0, pass i, stage k0) + per-lane byte offset.
  // MEDGE (the last tile along M when r != 0): rows past M-1 are fetched from row M-1, so
  // every load stays in bounds; their products land in rows the epilogue never stores.
  const int ld_row = tid / CH;
  const int ld_c = (tid & (CH - 1)) ^ ((ld_row >> 1) & (CH - 1));
  uint32_t a_off[A_LD];
  auto set_a_off = [&](const int tile_m0, const bool clamp) {
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
      int row = ld_row + i * PASS;
      if (BM % PASS != 0) row = row < BM ? row : BM - 1;
      if (clamp) row = (tile_m0 + row < g.M) ? row : (g.M - 1 - tile_m0);
      a_off[i] = (uint32_t)(row * g.lda + ld_c * 8) * 2u;
    }
  };
  set_a_off(m0, MEDGE);
  const uint32_t b_off = (uint32_t)(ld_row * g.ldb + ld_c * 8) * 2u;
  const u16* a_base = A + (long long)m0 * g.lda;
  const u16* b_base = B + (long long)n0 * g.ldb;
  const long long b_pass = (long long)PASS * g.ldb;
  const uint32_t a_dst = __builtin_amdgcn_readfirstlane(lds_addr_of(&As[0][wave * 64]));
  const uint32_t b_dst = __builtin_amdgcn_readfirstlane(lds_addr_of(&Bs[0][wave * 64]));
  auto dma = [&](int ks, int slot) {
    const int k0 = ks << KSH;
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      dma16_so(a_off[i], a_base + k0, a_dst + slot * (BMP * CH * 16) + i * NT * 16);
#pragma unroll
    for (int i = 0; i < B_LD; ++i)
      dma16_so(b_off, b_base + i * b_pass + k0, b_dst + slot * (BN * CH * 16) + i * NT * 16);
  };

  // fragment reads: lane -> row (lane & 15), logical chunk (lane >> 4)
  const int fr_row = lane & 15;
  const int fr_q = lane >> 4;
  // (rows 16 apart share the swizzle term; the wide ring's second half adds 4 to the logical chunk)
  const int fr_phys = fr_q ^ ((fr_row >> 1) & (CH - 1));
  const int fr_a = (wm * WM + fr_row) * CH + fr_phys;
  const int fr_b = (wn * WN + fr_row) * CH + fr_phys;

  f32x4 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // The tile's BN bias values are fetched now, ahead of every other load, into LDS behind the ring,
  // so that the epilogue does not begin with a round trip to memory: the first BN/128 waves each
  // bring 256 bytes with one direct global->LDS load.  Loads complete in order, so the wait for
  // stage 0 below covers it, and the barrier after that wait publishes it.  (No register is
  // involved: a load into a register that the compiler cannot see complete may be spilled or
  // copied before its data has arrived.)  The 288- and 320-row tiles leave no LDS for it and load
  // the bias in the epilogue.
  constexpr bool BIAS_LDS = PF || S * (BMP + BN) * CH * 16 + BN * 2 <= 160 * 1024;
  // (PF: two bias slots, used by alternate tiles, then the waves' staging areas)
  u16* bias_lds = reinterpret_cast<u16*>(smem + S * (BMP + BN) * CH) + (PF ? lk.parity * BN : 0);
  const bool park_bias = BIAS_LDS && g.epilogue != NIMBLE_EPI_NONE && !g.out_f32;
  auto fetch_bias = [&](const int tile_n0, u16* dst) {
    if (park_bias && wave < BN / 128) {  // whole waves
      const int wu = __builtin_amdgcn_readfirstlane(wave);
      dma4_so((uint32_t)lane * 4u, (const u16*)g.bias + tile_n0 + wu * 128,
              __builtin_amdgcn_readfirstlane(lds_addr_of(dst)) + wu * 256);
    }
  };
  // whether the waits of this tile's first S-1 stages may leave the previous epilogue's stores in flight
  const bool lax = PF && lk.filled && lk.stores == NST;

  if constexpr (WIDE) {
    if (!PF || !lk.filled) {
      fetch_bias(n0, bias_lds);
#pragma unroll
      for (int s = 0; s < S; ++s) dma(s < KS ? s : KS - 1, s);  // always S stages in flight
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 1) * LD) : "memory");  // stage 0 landed
    } else if (lax) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NST + (S - 1) * LD) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 1) * LD) : "memory");
    }
  } else {
    fetch_bias(n0, bias_lds);
#pragma unroll
    for (int s = 0; s < S - 1; ++s) {
      if constexpr (MODE == RING_SOLO)
        dma(s < KS ? s : KS - 1, s);  // always S-1 stages in flight (see the stage code below)
      else if (s < KS)
        dma(s, s);
    }
    if (MODE == RING_SOLO || KS - 1 >= S - 2)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * LD) : "memory");  // stage 0 landed
    else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();

  if constexpr (MODE == RING_PINGPONG) {
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
  } else if constexpr (MODE == RING_SOLO) {
    // One wave per SIMD, so nothing else hides this wave's LDS latency: the fragments of stage
    // s+1 are read into the second register set in between the MFMAs of stage s, and the steady
    // state is straight-line code (no branch inside a stage), so that the compiler's wait-count
    // insertion can see that the MFMAs of stage s depend only on reads that completed before the
    // barrier and lets them start at once.
    bf16x8 xa[2][TM], wb[2][TN];
    const uint4* a_rd = &As[0][fr_a];
    const uint4* b_rd = &Bs[0][fr_b];
#pragma unroll
    for (int j = 0; j < TM; ++j) xa[0][j] = as_bf16x8(a_rd[j * 64]);
#pragma unroll
    for (int i = 0; i < TN; ++i) wb[0][i] = as_bf16x8(b_rd[i * 64]);
    // Every stage runs the same code, also the last S-1 of a tile: past the end of K the loads
    // fetch the last stage again (in bounds, into a slot nobody reads any more) and the
    // fragment reads fetch stale data that is never multiplied.  That keeps the count of loads
    // in flight the same at every stage, so one wait count serves them all.
    auto stage = [&](const int ks, auto cur_tag) {
      constexpr int CUR = decltype(cur_tag)::value;
      // stage ks+1 has landed once only the S-3 younger stages are in flight
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 3) * LD) : "memory");
      __syncthreads();
      const int ld = ks + S - 1;
      dma(ld < KS ? ld : KS - 1, ld % S);  // into the slot of stage ks-1, read before this barrier
      const int nslot = (ks + 1) % S;
      const uint4* a_nx = a_rd + nslot * (BMP * 4);
      const uint4* b_nx = b_rd + nslot * (BN * 4);
#pragma unroll
      for (int i = 0; i < TN; ++i) {
        // the two reads stay in front of this weight tile's MFMAs: the empty statement below
        // is a compiler barrier for memory operations, and the MFMAs are volatile statements
        wb[CUR ^ 1][i] = as_bf16x8(b_nx[i * 64]);
#pragma unroll
        for (int x = i * TM / TN; x < (i + 1) * TM / TN; ++x)  // this tile's share of the TM reads
          xa[CUR ^ 1][x] = as_bf16x8(a_nx[x * 64]);
        asm volatile("" ::: "memory");
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          if (i == TN - 1 && j == TM - 1)
            mfma_acc_last(acc[i][j], wb[CUR][i], xa[CUR][j], ks + 1 >= KS);
          else
            mfma_acc(acc[i][j], wb[CUR][i], xa[CUR][j]);
        }
      }
    };
    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;
    int ks = 0;
    for (; ks + 1 < KS; ks += 2) {
      stage(ks, T0{});
      stage(ks + 1, T1{});
    }
    if (ks < KS) stage(ks, T0{});  // odd number of stages
    // loads past the end of K may still be in flight into the ring the epilogue is about to reuse
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  } else if constexpr (MODE == RING_WIDE) {
    // Same straight-line schedule as above on stages of 64 k: two halves of 32 k per stage, the
    // fragments of the next half read into the other register set in between the MFMAs of the
    // current one, one barrier per stage.
    bf16x8 xa[2][TM], wb[2][TN];
    const uint4* a_rd = &As[0][fr_a];
    const uint4* b_rd = &Bs[0][fr_b];
#pragma unroll
    for (int j = 0; j < TM; ++j) xa[0][j] = as_bf16x8(a_rd[j * 16 * CH]);
#pragma unroll
    for (int i = 0; i < TN; ++i) wb[0][i] = as_bf16x8(b_rd[i * 16 * CH]);
    // reads of the other half of a row: logical chunk + 4, i.e. physical chunk ^ 4
    const int half = ((fr_phys ^ 4) - fr_phys);
    // load u of a stage (0 .. LD-1): the A passes first, then the B passes
    auto dma_one = [&](int k0, int slot_, int u) {
      if (u < A_LD)
        dma16_so(a_off[u], a_base + k0, a_dst + slot_ * (BMP * CH * 16) + u * NT * 16);
      else
        dma16_so(b_off, b_base + (u - A_LD) * b_pass + k0, b_dst + slot_ * (BN * CH * 16) + (u - A_LD) * NT * 16);
    };
    // second halves (CUR == 1) also issue the ring loads of one stage, spread over their weight
    // tiles (ld_k0 < 0 in a two-slot ring: past the end of K, nothing to load)
    auto half_step = [&](const uint4* a_nx, const uint4* b_nx, auto cur_tag, int ld_k0, int ld_slot, int last) {
      constexpr int CUR = decltype(cur_tag)::value;
#pragma unroll
      for (int i = 0; i < TN; ++i) {
        wb[CUR ^ 1][i] = as_bf16x8(b_nx[i * 16 * CH]);
#pragma unroll
        for (int x = i * TM / TN; x < (i + 1) * TM / TN; ++x) xa[CUR ^ 1][x] = as_bf16x8(a_nx[x * 16 * CH]);
        if (CUR == 1 && (S != 2 || ld_k0 >= 0)) {  // uniform
#pragma unroll
          for (int u = i * LD / TN; u < (i + 1) * LD / TN; ++u) dma_one(ld_k0, ld_slot, u);
        }
        asm volatile("" ::: "memory");
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          if (CUR == 1 && i == TN - 1 && j == TM - 1)
            mfma_acc_last(acc[i][j], wb[CUR][i], xa[CUR][j], last);
          else
            mfma_acc(acc[i][j], wb[CUR][i], xa[CUR][j]);
        }
      }
    };
    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;
    int slot = 0;
    for (int ks = 0; ks < KS; ++ks) {
      // first half: multiply k 0..31 of stage ks, read its k 32..63
      half_step(a_rd + slot * (BMP * CH) + half, b_rd + slot * (BN * CH) + half, T0{}, 0, 0, 0);
      // every read of this stage's slot has been issued; once they have returned and every wave
      // is here the slot can be refilled, and stage ks+1 has landed when only the S-2 younger
      // stages are in flight
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (PF && lax && ks < S - 1)  // (uniform) the stores of the previous epilogue are younger than stage ks+1
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NST + (S - 2) * LD) : "memory");
      else
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * LD) : "memory");
      __syncthreads();
      // Past the end of K.  S = 2: nothing is loaded (the wait above is for zero loads in flight
      // whether or not a younger stage was issued), which spares the L2->LDS path two stages' worth
      // of traffic per tile.  S = 3: the last stage again, into a slot nobody reads any more, so
      // that the count of loads in flight, and with it the wait count, is the same at every stage;
      // choosing the wait count per stage instead puts a branch into the stage and ran 3-4 % slower.
      // (A second copy of the stage code without loads for the last two stages, instead of the
      // test on ld_k0, cost the 256x256 tile 20 spilled registers and 6 % at ragged M.)
      const int ld = ks + S;
      const int ld_k0 = ld < KS ? (ld << KSH) : (S == 2 ? -1 : ((KS - 1) << KSH));
      const int ld_slot = slot;
      slot = slot + 1 == S ? 0 : slot + 1;
      // second half: multiply k 32..63 of stage ks, read k 0..31 of stage ks+1, refill the freed slot
      half_step(a_rd + slot * (BMP * CH), b_rd + slot * (BN * CH), T1{}, ld_k0, ld_slot, ks + 1 >= KS);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // (S = 3: the loads past the end of K)
  }

  // PF: every wave is past its last fragment read once it is past this barrier; the ring then takes the
  // next tile's first stages while the epilogue below runs out of registers and the staging areas
  if constexpr (PF) {
    __syncthreads();
    if (lk.next) {
      set_a_off(lk.next_m0, true);
      a_base = A + (long long)lk.next_m0 * g.lda;
      b_base = B + (long long)lk.next_n0 * g.ldb;
      fetch_bias(lk.next_n0, reinterpret_cast<u16*>(smem + S * (BMP + BN) * CH) + (lk.parity ^ 1) * BN);
#pragma unroll
      for (int s = 0; s < S; ++s) dma(s < KS ? s : KS - 1, s);
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
      const uint2 bb = park_bias ? *(const uint2*)(bias_lds + wn * WN + i * 16 + fr_q * 4)
                                 : *(const uint2*)((const u16*)g.bias + n0 + wn * WN + i * 16 + fr_q * 4);
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
    return -1;
  }
  u16* C = (u16*)g.c + (long long)z * g.sc;
  constexpr int NH = WN / 64;
  if constexpr (PF) {
    // bf16 through the wave's own staging area, 16 rows at a time: [NH][16 rows][128 bytes], chunk c of
    // row r at slot c ^ ((r >> 1) & 7), written back out as full 128-byte lines.  (Wave-private: no
    // workgroup barrier; a wave's LDS accesses execute in order.)
    unsigned char* region = (unsigned char*)(smem + S * (BMP + BN) * CH) + 2 * BN * 2 + wave * (16 * WN * 2);
#pragma unroll
    for (int j = 0; j < TM; ++j) {
#pragma unroll
      for (int i = 0; i < TN; ++i) {
        const int col = (i & 3) * 16 + fr_q * 4;
        const int chunk = (col >> 3) ^ ((fr_row >> 1) & 7);
        uint2 pk;
        pk.x = pack_bf16x2(epilogue(acc[i][j][0], alpha, bias4[i][0], epi),
                           epilogue(acc[i][j][1], alpha, bias4[i][1], epi));
        pk.y = pack_bf16x2(epilogue(acc[i][j][2], alpha, bias4[i][2], epi),
                           epilogue(acc[i][j][3], alpha, bias4[i][3], epi));
        *(uint2*)(region + (i >> 2) * (16 * 128) + fr_row * 128 + chunk * 16 + (col & 4) * 2) = pk;
      }
#pragma unroll
      for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          const int row = p * 8 + (lane >> 3);
          const int c = lane & 7;
          const uint4 v = *(const uint4*)(region + h * (16 * 128) + row * 128 + ((c ^ ((row >> 1) & 7)) * 16));
          if (MEDGE && m0 + wm * WM + j * 16 + row >= g.M) continue;
          *(uint4*)(C + (long long)(m0 + wm * WM + j * 16 + row) * g.ldc + n0 + wn * WN + h * 64 + c * 8) = v;
        }
    }
    return MEDGE ? -1 : NST;
  }
  // bf16: every wave stages its [WM][WN] block in LDS as WN/64 blocks of [WM][64] (rows of 128
  // bytes, chunk c of row r at slot c ^ ((r >> 1) & 7)) and writes it back out as full 128-byte lines
  __syncthreads();  // all fragment reads of the ring are done
  unsigned char* region = (unsigned char*)smem + wave * (WM * WN * 2);
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int row = j * 16 + fr_row;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
      const int col = (i & 3) * 16 + fr_q * 4;
      const int chunk = (col >> 3) ^ ((row >> 1) & 7);
      uint2 pk;
      pk.x = pack_bf16x2(epilogue(acc[i][j][0], alpha, bias4[i][0], epi),
                         epilogue(acc[i][j][1], alpha, bias4[i][1], epi));
      pk.y = pack_bf16x2(epilogue(acc[i][j][2], alpha, bias4[i][2], epi),
                         epilogue(acc[i][j][3], alpha, bias4[i][3], epi));
      *(uint2*)(region + (i >> 2) * (WM * 128) + row * 128 + chunk * 16 + (col & 4) * 2) = pk;
    }
  }
  // the region is private to the wave: no workgroup barrier, the compiler orders the LDS accesses
#pragma unroll
  for (int h = 0; h < NH; ++h)
#pragma unroll
    for (int p = 0; p < WM / 8; ++p) {
      const int row = p * 8 + (lane >> 3);
      const int c = lane & 7;
      const uint4 v = *(const uint4*)(region + h * (WM * 128) + row * 128 + ((c ^ ((row >> 1) & 7)) * 16));
      if (MEDGE && m0 + wm * WM + row >= g.M) continue;
      uint4* dst = (uint4*)(C + (long long)(m0 + wm * WM + row) * g.ldc + n0 + wn * WN + h * 64 + c * 8);
      *dst = v;
    }
  return -1;
}

// S = number of ring stages.  4 keeps two workgroups of the 128x128 tile on a compute unit.  A
// deeper ring (8 stages for 128x128, 6 for 256x128) was measured and changed nothing: a lone
// workgroup is bound by the ~37 bytes per clock one compute unit pulls through the direct
// global->LDS path, not by the latency of the loads.  Two 4-wave workgroups of a 256x128 tile
// per compute unit (3-stage rings, one register set) were measured too: same steady-state rate as
// the 8-wave ping-pong, slower at whole rounds, so that shape is not built.
// BM may be any multiple of 16 * WGM: the 256-wide tile is built at 128..256 rows so that the
// dispatch function can pick the height at which the run-time M fills whole rounds of the chip.
template <int BM, int BN, int WGM, int WGN, bool RESIDUE, int S = 4, bool WIDE = false>
__global__ void __launch_bounds__(WGM* WGN * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
    gemm_ring_kernel(GemmArgs g, int tiles_m, int tiles_n, int group_m) {
  // WIDE: stages of 64 k (K must be a multiple of 64; the launcher sees to that), S = 2 or 3.
  // Else stages of 32 k: the straight-line schedule with two fragment sets wherever accumulators
  // and both sets fit in a wave's 256 registers (wave tiles up to 128 rows by 64 columns); the
  // two-group ping-pong with one set for the 288- and 320-row heights of the 256-wide tile
  constexpr int kMode = WIDE ? RING_WIDE : (WGM == 2 && WGN == 4 && BM > 256 ? RING_PINGPONG : RING_SOLO);
  constexpr int kCh = WIDE ? 8 : 4;
  constexpr int kPass = WGM * WGN * 64 / kCh;  // rows per load pass: the ring holds whole passes of A
  constexpr int kBmp = (BM + kPass - 1) / kPass * kPass;
  // the ring (which also holds the masked body's two 64-wide tiles), then BN bias values where they fit
  constexpr int kRing = S * (kBmp + BN) * kCh;
  static_assert(kRing >= 2 * (BM + BN) * 8, "the masked body needs two 64-wide tiles");
  // Wherever two bias slots and a 16-row staging area per wave fit behind a 64-wide ring, a tile's
  // epilogue leaves the ring alone and the next tile's first stages load while it runs (RingLink).
  constexpr int kStage = WGM * WGN * 16 * (BN / WGN) * 2 / 16;  // uint4
  // (never at the price of a workgroup fewer per compute unit)
  constexpr int kOldBytes = kRing * 16 + (kRing * 16 + BN * 2 <= 160 * 1024 ? BN * 2 : 0);
  constexpr int kPfBytes = (kRing + 2 * (BN / 8) + kStage) * 16;
  constexpr bool kPF = WIDE && kPfBytes <= 160 * 1024 && (160 * 1024 / kPfBytes == 160 * 1024 / kOldBytes);
  constexpr int kBias = kPF ? 2 * (BN / 8) + kStage : (kRing * 16 + BN * 2 <= 160 * 1024 ? BN / 8 : 0);
  __shared__ __attribute__((aligned(16))) uint4 smem[kRing + kBias];
  // A workgroup walks the tiles blockIdx.x, blockIdx.x + gridDim.x, ...: the launcher starts at most
  // as many workgroups as the chip holds at once, so a launch of several rounds pays the 2-3 us it
  // takes to retire a workgroup and start the next one on its compute unit only once.  (gridDim.x
  // is a multiple of 8 whenever a workgroup gets more than one tile, so a workgroup's tiles stay in
  // the run of tile ids of its own XCD.)
  const int tiles_total = tiles_m * tiles_n;
  // launch-wide reasons for the fully masked body: K not whole stages, output rows not 16-byte aligned
  const bool ragged_launch = RESIDUE && (((g.K & (WIDE ? 63 : 31)) != 0) || ((g.ldc & 7) != 0));
  RingLink lk;
  for (int t = blockIdx.x; t < tiles_total; t += gridDim.x) {
    // the previous tile's epilogue is done with the LDS (a handed-over ring was free before it began)
    if (t != (int)blockIdx.x && !lk.filled) __syncthreads();
    int tile_m, tile_n;
    tile_of_block(t, tiles_total, tiles_m, tiles_n, group_m, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    if constexpr (kPF) {
      const int t2 = t + (int)gridDim.x;
      lk.next = false;
      if (t2 < tiles_total && !ragged_launch) {
        int m2, n2;
        tile_of_block(t2, tiles_total, tiles_m, tiles_n, group_m, m2, n2);
        lk.next_m0 = m2 * BM;
        lk.next_n0 = n2 * BN;
        lk.next = !RESIDUE || lk.next_n0 + BN <= g.N;  // never ahead of a fully masked tile
      }
    }
    if (RESIDUE) {
      // the packed epilogue needs 16-byte aligned output rows; K must be whole stages
      const bool ragged = ragged_launch || (n0 + BN > g.N);
      if (ragged) {  // ragged N or K, or output rows not 16-byte aligned: the fully masked body
        // (the reduced tile heights are only dispatched to shapes without ragged N or K)
        if constexpr (BM % 128 == 0 || BN == 128) gemm_tile_body<BM, BN, WGM, WGN, true>(g, m0, n0, smem);
        lk.filled = false;
        continue;
      }
      if (m0 + BM > g.M) {  // the last tile along M: same pipeline, clamped loads, masked stores
        lk.stores = gemm_ring_body<BM, BN, WGM, WGN, S, true, kMode, kPF>(g, m0, n0, smem, lk);
        lk.filled = kPF && lk.next;
        lk.parity ^= 1;
        continue;
      }
    }
    lk.stores = gemm_ring_body<BM, BN, WGM, WGN, S, false, kMode, kPF>(g, m0, n0, smem, lk);
    lk.filled = kPF && lk.next;
    lk.parity ^= 1;
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

}  // namespace nimble
#endif
