// Device entry points of the C ABI and the launchers behind the dispatch function
// (Section 3.5).  bf16 operands, f32 accumulation on the matrix cores, f32 epilogue.
//
// Kernel family (one header each under csrc/)
//   gemm_ring_kernel.h   gemm_ring_kernel<BM,BN,WGM,WGN,RESIDUE>: every tiled variant (32x128,
//       64x128, 128x128, 256x128, and the 256-wide tile at heights 128..320).  A ring of four
//       32-wide K stages filled by direct global->LDS loads, 16x16x32 MFMA with in-place
//       accumulators, the next stage's fragments read in between the MFMAs, an epilogue that
//       transposes through LDS so every store is a full 128-byte line.  RESIDUE=false is the
//       copy for r = 0: no bounds code at all.  RESIDUE=true is the copy for r != 0: decided
//       once per workgroup, the last tile along M runs the same pipeline with clamped loads
//       and masked stores, ragged N/K tiles run the fully masked body.  Also the split-K
//       reduction kernel.
//   gemm_tile_kernel.h   gemm_tile_body: that fully masked body (register-staged K tiles of 64,
//       32x32x16 MFMA, every access bounds-checked).
//   skinny_kernel.h      skinny_kernel<MT,LSTM>: M <= 64 per workgroup, the weights are
//       streamed from HBM exactly once straight into MFMA operands, the four waves of a
//       workgroup split K and reduce through LDS.  LSTM=true gathers the four gate rows of
//       four hidden units and applies the cell update in the epilogue.
//   stream_kernel.h      stream_kernel<LSTM,S,NW,XR>: the weight-streaming kernel for up to 16 rows per
//       workgroup and K in whole 64-wide stages: operands staged through per-wave LDS rings by
//       direct global->LDS loads of whole 128-byte lines (what bounds skinny_kernel is cache-line
//       look-ups, 64 per KiB with its register-layout loads).
//   misc_kernels.h       generic_kernel (any shape and stride, one thread per output),
//       softmax_rows_kernel (f32 scores -> bf16 probabilities), attention64_kernel (fused
//       softmax(alpha Q.K^T).V for head dimension 64).
//   probe_kernels.h      calibration probes: a register-only MFMA loop and a streaming read.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <mutex>

#include "device_common.h"
#include "gemm_ring_kernel.h"
#include "gemm_tile_kernel.h"
#include "misc_kernels.h"
#include "nimble_internal.h"
#include "nimble_probe.h"
#include "lstm_seq_kernel.h"
#include "probe_kernels.h"
#include "skinny_kernel.h"
#include "stream_kernel.h"

namespace nimble {

// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------
static int check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return NIMBLE_OK;
  return fail(NIMBLE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// WS: slots of the 64-wide ring (0: the tile is only built on the 32-wide ring).  The 64-wide
// ring runs whenever K is whole 64-wide stages and every K slice gets at least one of them.
template <int BM, int BN, int WGM, int WGN, int WS = 2, int S = 4>
static int launch_ring(const GemmArgs& g, const nimble_plan& p, hipStream_t st) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  // tile rows per L2 group: 4 measured best of 1..32 on the BERT-large FFN shapes (NIMBLE_GROUP_M is a
  // tuning knob, read once)
  static const int group_m_default = [] {
    const char* env = std::getenv("NIMBLE_GROUP_M");
    const int v = env ? std::atoi(env) : 0;
    return v > 0 ? v : 4;
  }();
  int group_m = group_m_default;
  if (group_m > tiles_m) group_m = tiles_m;
  const int slices = p.split_k > 1 ? p.split_k : 1;
  // at most as many workgroups as are resident at once (one per compute unit for the 8-wave
  // tiles, two for the smaller ones); each walks its share of the tiles
  unsigned wgs = p.grid[0];
  {
    static const bool one_tile_each = std::getenv("NIMBLE_NO_PERSIST") != nullptr;  // measurement knob
    const unsigned resident = (unsigned)(kComputeUnits * kTilesPerCU[p.variant]);
    if (!one_tile_each && slices == 1 && p.grid[2] == 1 && wgs > resident) wgs = resident;
  }
  dim3 grid(wgs, slices, p.grid[2]), block(WGM * WGN * 64);
  if constexpr (WS > 0) {
    static const bool ring32_only = std::getenv("NIMBLE_RING32") != nullptr;  // measurement knob
    const int stages = g.K >> 6, per = (stages + slices - 1) / slices;
    if (!ring32_only && g.K > 0 && (g.K & 63) == 0 && per * (slices - 1) < stages) {
      if (p.residue_copy)
        hipLaunchKernelGGL((gemm_ring_kernel<BM, BN, WGM, WGN, true, WS, true>), grid, block, 0, st, g, tiles_m,
                           tiles_n, group_m);
      else
        hipLaunchKernelGGL((gemm_ring_kernel<BM, BN, WGM, WGN, false, WS, true>), grid, block, 0, st, g, tiles_m,
                           tiles_n, group_m);
      return check_hip(hipGetLastError(), "ring kernel launch");
    }
  }
  if (p.residue_copy)
    hipLaunchKernelGGL((gemm_ring_kernel<BM, BN, WGM, WGN, true, S>), grid, block, 0, st, g, tiles_m,
                       tiles_n, group_m);
  else
    hipLaunchKernelGGL((gemm_ring_kernel<BM, BN, WGM, WGN, false, S>), grid, block, 0, st, g, tiles_m,
                       tiles_n, group_m);
  return check_hip(hipGetLastError(), "ring kernel launch");
}

// Whether the LDS-staged streaming kernel can run a weight-streaming launch: one 16-row tile per
// workgroup, K in whole 64-wide stages (the LSTM cell: its x | h boundary too), 32-bit lane offsets.
static bool stream_kernel_ok(bool lstm, int rows_per_block, int64_t N, int64_t K, int64_t Ix) {
  return rows_per_block <= 16 && stream_kernel_shape_ok(N, K) && (!lstm || (Ix & 63) == 0);
}

template <bool LSTM>
static int launch_skinny(const SkinnyArgs& s, const nimble_plan& p, hipStream_t st) {
  dim3 grid(p.grid[0], p.grid[1], 1), block(256);
  // 16-row tiles per workgroup: the rows spread evenly over the plan's row blocks (at most 4 each)
  const int mt = (s.M + 16 * (int)p.grid[1] - 1) / (16 * (int)p.grid[1]);
  if (stream_kernel_ok(LSTM, 16 * mt, s.N, s.K, s.Ix)) {
    // eight waves with three stages each; up to 8 rows the activation tile is 8 rows (measured on a
    // 134 MB layer from HBM: 23.9 us at one row, 25.0 at four; the 16-row tile 24.7 and 25.6, and 27.9 at
    // sixteen rows; four waves per workgroup 27.9-30.5 us whatever the ring depth)
    // More workgroups than compute units on a cache-resident layer (several 16-row blocks): small
    // workgroups of four waves with two stages each, four to a compute unit, so that one's start-up and
    // reduction overlap the others' streaming (2304 x 768 at 128 rows: 5.2 us against 7.8 with the
    // shape below and 6.3 with eight waves and two stages; the LSTM cell at 64 rows 3.9 against 5.3).
    const bool many = (uint64_t)grid.x * grid.y > (uint64_t)kComputeUnits &&
                      (double)s.N * (double)s.K * 2.0 <= kCachedWeightBytes;
    if (many)
      hipLaunchKernelGGL((stream_kernel<LSTM, 2, 4, 16>), grid, dim3(256), 0, st, s);
    else if (s.M <= 8)
      hipLaunchKernelGGL((stream_kernel<LSTM, 3, 8, 8>), grid, dim3(512), 0, st, s);
    else
      hipLaunchKernelGGL((stream_kernel<LSTM, 3, 8, 16>), grid, dim3(512), 0, st, s);
    return check_hip(hipGetLastError(), "stream kernel launch");
  }
  switch (mt) {
    case 1:
      // a grid that leaves compute units with one workgroup at most, and more than one batch of
      // eight steps per wave: twice the loads per batch
      if (!LSTM && (uint64_t)p.grid[0] * p.grid[1] <= (uint64_t)kComputeUnits && s.K > 1024)
        hipLaunchKernelGGL((skinny_kernel<1, false, 16>), grid, block, 0, st, s);
      else
        hipLaunchKernelGGL((skinny_kernel<1, LSTM>), grid, block, 0, st, s);
      break;
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
      s.alpha = g.alpha;
      return launch_skinny<false>(s, p, st);
    }
    case NIMBLE_VAR_T32x128: return launch_ring<32, 128, 1, 2, 3>(g, p, st);
    case NIMBLE_VAR_T64x128: return launch_ring<64, 128, 2, 2, 3>(g, p, st);
    case NIMBLE_VAR_T128x128: return launch_ring<128, 128, 2, 2>(g, p, st);
    case NIMBLE_VAR_T256x128:
      return launch_ring<256, 128, 4, 2, 3>(g, p, st);
    case NIMBLE_VAR_T256x256:
      switch (p.bm) {  // the tile height the dispatch function chose for this M
        case 320: return launch_ring<320, 256, 2, 4, 0>(g, p, st);
        case 288: return launch_ring<288, 256, 2, 4, 0>(g, p, st);
        case 256: return launch_ring<256, 256, 2, 4>(g, p, st);
        case 224: return launch_ring<224, 256, 2, 4>(g, p, st);
        case 192: return launch_ring<192, 256, 2, 4>(g, p, st);
        case 160: return launch_ring<160, 256, 2, 4>(g, p, st);
        case 128: return launch_ring<128, 256, 2, 4>(g, p, st);
        default: return fail(NIMBLE_ERR_ARG, "t256x256 is not built with tiles of %d rows", p.bm);
      }
    default: return fail(NIMBLE_ERR_ARG, "unknown variant %d", p.variant);
  }
}

static inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Built-in scratch of nimble_dense_noalloc_dyn: the f32 partial sums of a K split live here instead
// of in memory the caller brings.  Every GPU the library runs on holds its own copy of the array
// (at its own address) from the moment the code object is loaded there until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress, never a device address:
// kernels are given the pointer that call returns.
static __device__ __align__(256) unsigned char scratch[NIMBLE_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];   // per device, looked up once with that device current
static std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch`, or null after fail().
static void* scratch_of_current_device() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(NIMBLE_ERR_HIP, "hipGetDevice: %s (device %d)", hipGetErrorString(e), dev);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      fail(NIMBLE_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace nimble

using namespace nimble;

extern "C" {

// One planned launch of dense; a K-split plan runs the slices into the workspace and then the
// reduction kernel.
static int run_dense(const GemmArgs& g, const nimble_plan& p, void* workspace, hipStream_t st) {
  if (p.split_k <= 1 || p.variant < NIMBLE_VAR_T32x128) return launch_gemm(g, p, st);
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

int nimble_dense_dyn(const void* x, const void* w, const void* bias, void* y, int64_t M, int64_t N,
                     int64_t K, int epilogue, int out_dtype, void* workspace, size_t workspace_bytes,
                     void* stream) {
  return nimble_dense_variant_dyn(x, w, bias, y, M, N, K, epilogue, out_dtype, NIMBLE_VAR_AUTO, workspace,
                                  workspace_bytes, stream);
}

int nimble_dense_noalloc_dyn(const void* x, const void* w, const void* bias, void* y, int64_t M, int64_t N,
                             int64_t K, int epilogue, int out_dtype, void* stream) {
  clear_error();
  if (epilogue < NIMBLE_EPI_NONE || epilogue > NIMBLE_EPI_BIAS_GELU_ERF)
    return fail(NIMBLE_ERR_ARG, "unknown epilogue %d", epilogue);
  if (out_dtype != NIMBLE_BF16 && out_dtype != NIMBLE_F32) return fail(NIMBLE_ERR_DTYPE, "unknown dtype %d", out_dtype);
  // the plan a caller would get who brings whatever scratch the dispatch function asks for: if it
  // fits the built-in scratch, planning within the built-in scratch gives the same plan
  PlanOptions opt;
  opt.max_workspace = ~0ull;
  nimble_plan p;
  int rc = plan_dense(1, M, N, K, epilogue, NIMBLE_VAR_AUTO, opt, &p);
  if (rc != NIMBLE_OK) return rc;
  if (p.workspace_bytes > (uint64_t)NIMBLE_NOALLOC_SCRATCH_BYTES)
    return fail(NIMBLE_ERR_WORKSPACE,
                "dense %lld x %lld x %lld needs %llu bytes of scratch, the built-in scratch holds %llu: "
                "use nimble_dense_dyn with a workspace",
                (long long)M, (long long)N, (long long)K, (unsigned long long)p.workspace_bytes,
                (unsigned long long)NIMBLE_NOALLOC_SCRATCH_BYTES);
  if (M == 0 || N == 0) return NIMBLE_OK;
  void* ws = scratch_of_current_device();
  if (!ws) return NIMBLE_ERR_HIP;
  // nothing in the scratch needs clearing: every slice of a K split writes its whole plane of
  // partial sums before the reduction kernel reads it
  return nimble_dense_variant_dyn(x, w, bias, y, M, N, K, epilogue, out_dtype, NIMBLE_VAR_AUTO, ws,
                                  (size_t)NIMBLE_NOALLOC_SCRATCH_BYTES, stream);
}

int nimble_dense_variant_dyn(const void* x, const void* w, const void* bias, void* y, int64_t M,
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
  if (batch < 0 || M < 0 || N < 0 || K < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (out_dtype != NIMBLE_BF16 && out_dtype != NIMBLE_F32)
    return fail(NIMBLE_ERR_DTYPE, "unknown dtype %d", out_dtype);
  if (workspace_bytes > 0 && !workspace) return fail(NIMBLE_ERR_NULL, "workspace_bytes > 0 with a null workspace");
  if (workspace && misaligned(workspace)) return fail(NIMBLE_ERR_ALIGN, "workspace must be 16-byte aligned");
  nimble_plan p;
  int rc = nimble_batch_matmul_plan(batch, M, N, K, trans_b, out_dtype, &p);
  if (rc != NIMBLE_OK) return rc;
  if (batch == 0 || M == 0 || N == 0) return NIMBLE_OK;
  if (!a || !b || !c) return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if (misaligned(a) || misaligned(b) || misaligned(c))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  // the NN product on the tiled kernels needs b transposed into the workspace: without enough of
  // it the bounds-checked kernel does the job (the plan is made within the scratch the caller brought)
  bool transpose_b = false;
  if (!trans_b && p.variant >= NIMBLE_VAR_T32x128) {
    if (workspace_bytes >= p.workspace_bytes && batch <= 65535) {
      transpose_b = true;
    } else {
      rc = plan_dense(batch, M, N, K, NIMBLE_EPI_NONE, NIMBLE_VAR_GENERIC, PlanOptions(), &p);
      if (rc != NIMBLE_OK) return rc;
    }
  }
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
  if (transpose_b) {
    dim3 tgrid((unsigned)((N + 31) / 32), (unsigned)((K + 31) / 32), (unsigned)batch);
    hipLaunchKernelGGL(transpose_kn_kernel, tgrid, dim3(256), 0, (hipStream_t)stream, (const u16*)b, (u16*)workspace,
                       (int)K, (int)N);
    rc = check_hip(hipGetLastError(), "transpose launch");
    if (rc != NIMBLE_OK) return rc;
    g.b = workspace;
    g.ldb = (int)K;
    g.b_is_kn = 0;
  }
  // batch slices of a K-contiguous operand stay 16-byte aligned only if M*K (N*K) is a multiple of 8
  if (p.variant != NIMBLE_VAR_GENERIC && (((M * K) & 7) != 0 || ((N * K) & 7) != 0)) {
    rc = plan_dense(batch, M, N, K, NIMBLE_EPI_NONE, NIMBLE_VAR_GENERIC, PlanOptions(), &p);
    if (rc != NIMBLE_OK) return rc;
  }
  // one launch over all rows: a plan that splits rows or K would run the r = 0 copy past M
  if (p.split_rows != 0 || (p.split_k > 1 && p.variant >= NIMBLE_VAR_T32x128))
    return fail(NIMBLE_ERR_ARG, "batch_matmul plan is not a single launch");
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
  if (!(alpha > 0.0f)) return fail(NIMBLE_ERR_ARG, "fused attention needs a positive score scale, got %g", (double)alpha);
  if (heads > 65535 || L > (1ll << 24)) return fail(NIMBLE_ERR_ARG, "extent too large");
  if (heads == 0 || L == 0) return NIMBLE_OK;
  if (!q || !k || !v || !o) return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  dim3 grid((unsigned)((L + 63) / 64), (unsigned)heads);
  static const bool blocks64 = std::getenv("NIMBLE_ATT_BLOCK64") != nullptr;  // measurement knob
  const u16 *qp = (const u16*)q, *kp = (const u16*)k, *vp = (const u16*)v;
  if (L <= 64 || blocks64)
    hipLaunchKernelGGL(attention64_kernel<64>, grid, dim3(256), 0, (hipStream_t)stream, qp, kp, vp, (u16*)o, (int)L, alpha);
  else
    hipLaunchKernelGGL(attention64_kernel<128>, grid, dim3(256), 0, (hipStream_t)stream, qp, kp, vp, (u16*)o, (int)L, alpha);
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
  s.alpha = 1.0f;
  return launch_skinny<true>(s, p, (hipStream_t)stream);
}

int nimble_lstm_gates_pre_dyn(const void* pre, const void* h_prev, const void* w_h, const void* c_prev,
                              void* c_out, void* h_out, int64_t B, int64_t H, void* stream) {
  clear_error();
  nimble_plan p;
  int rc = nimble_lstm_plan(B, 0, H, &p);
  if (rc != NIMBLE_OK) return rc;
  if (B == 0) return NIMBLE_OK;
  if (!pre || !h_prev || !w_h || !c_prev || !c_out || !h_out) return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if (misaligned(pre) || misaligned(h_prev) || misaligned(w_h) || misaligned(c_prev) || misaligned(c_out) ||
      misaligned(h_out))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  if (h_out == h_prev) return fail(NIMBLE_ERR_ARG, "h_out must not alias h_prev");
  SkinnyArgs s{};
  s.h = (const u16*)h_prev;
  s.w = (const u16*)w_h;
  s.pre = (const float*)pre;
  s.y = h_out;
  s.c_prev = (const float*)c_prev;
  s.c_out = (float*)c_out;
  s.M = (int)B;
  s.N = (int)(4 * H);
  s.K = (int)H;
  s.Ix = 0;
  s.H = (int)H;
  s.epilogue = NIMBLE_EPI_BIAS;
  s.alpha = 1.0f;
  return launch_skinny<true>(s, p, (hipStream_t)stream);
}

int nimble_lstm_seq_pre_dyn(const void* pre, const void* w_h, const void* h0, const void* c0, void* h_seq,
                            void* c_out, int64_t T, int64_t B, int64_t H, void* workspace,
                            size_t workspace_bytes, uint32_t max_polls, void* stream) {
  clear_error();
  if (T < 0 || B < 0 || H < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (!nimble_lstm_seq_supported(B, H))
    return fail(NIMBLE_ERR_SHAPE, "lstm sequence: one launch runs 1 <= B <= 4 and H = 64..1024 in multiples of 64");
  if (T > (int64_t)1 << 24) return fail(NIMBLE_ERR_ARG, "lstm sequence: more than 2^24 steps");
  if (T == 0) return NIMBLE_OK;
  if (!pre || !w_h || !h0 || !c0 || !h_seq || !c_out || !workspace) return fail(NIMBLE_ERR_NULL, "null tensor pointer");
  if (misaligned(pre) || misaligned(w_h) || misaligned(h0) || misaligned(c0) || misaligned(h_seq) ||
      misaligned(c_out) || misaligned(workspace))
    return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  if (workspace_bytes < nimble_lstm_seq_workspace_bytes(B, H))
    return fail(NIMBLE_ERR_WORKSPACE, "lstm sequence: workspace of %zu bytes, %zu needed", workspace_bytes,
                nimble_lstm_seq_workspace_bytes(B, H));
  LstmSeqArgs a{};
  a.pre = (const float*)pre;
  a.w_h = (const u16*)w_h;
  a.h0 = (const u16*)h0;
  a.c0 = (const float*)c0;
  a.h_seq = (u16*)h_seq;
  a.c_out = (float*)c_out;
  a.ctl = (uint32_t*)workspace;
  a.exch = (uint32_t*)workspace + 64;
  a.T = (int)T;
  a.B = (int)B;
  a.H = (int)H;
  a.max_polls = max_polls;
  hipStream_t st = (hipStream_t)stream;
  const int words = (int)(B * H) > 64 ? (int)(B * H) : 64;
  hipLaunchKernelGGL(lstm_seq_init_kernel, dim3((words + 255) / 256), dim3(256), 0, st, a);
  int rc = check_hip(hipGetLastError(), "lstm sequence fill launch");
  if (rc != NIMBLE_OK) return rc;
  // H / 16 workgroups (at most 64; 128 with the knob at 2): fewer than the chip holds at once
  static const int groups = [] {  // measurement knob: groups of 4 units per workgroup
    const char* e = std::getenv("NIMBLE_LSTM_SEQ_G");
    const int v = e ? std::atoi(e) : 0;
    return (v == 2 || v == 4 || v == 8) ? v : 4;
  }();
  const bool one_stage = H <= 512;
  switch (groups) {
    case 2:
      if (one_stage) hipLaunchKernelGGL((lstm_seq_kernel<1, 2>), dim3((unsigned)(H / 8)), dim3(512), 0, st, a);
      else hipLaunchKernelGGL((lstm_seq_kernel<2, 2>), dim3((unsigned)(H / 8)), dim3(512), 0, st, a);
      break;
    case 8:
      if (one_stage) hipLaunchKernelGGL((lstm_seq_kernel<1, 8>), dim3((unsigned)(H / 32)), dim3(512), 0, st, a);
      else hipLaunchKernelGGL((lstm_seq_kernel<2, 8>), dim3((unsigned)(H / 32)), dim3(512), 0, st, a);
      break;
    default:
      if (one_stage) hipLaunchKernelGGL((lstm_seq_kernel<1, 4>), dim3((unsigned)(H / 16)), dim3(512), 0, st, a);
      else hipLaunchKernelGGL((lstm_seq_kernel<2, 4>), dim3((unsigned)(H / 16)), dim3(512), 0, st, a);
      break;
  }
  return check_hip(hipGetLastError(), "lstm sequence launch");
}

int nimble_lstm_seq_status(const void* workspace, void* stream, int* gave_up) {
  clear_error();
  if (!workspace || !gave_up) return fail(NIMBLE_ERR_NULL, "null pointer");
  uint32_t word = 0;
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e == hipSuccess) e = hipMemcpy(&word, workspace, sizeof(word), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail(NIMBLE_ERR_HIP, "lstm sequence status: %s", hipGetErrorString(e));
  *gave_up = word != 0;
  return NIMBLE_OK;
}

int nimble_probe_mfma_bf16(const void* seed, void* sink, int waves_per_simd, int iters, double* flops,
                           void* stream) {
  clear_error();
  if (!seed || !sink || !flops) return fail(NIMBLE_ERR_NULL, "null pointer");
  if (misaligned(seed) || misaligned(sink)) return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  if (iters < 1 || iters > (1 << 24)) return fail(NIMBLE_ERR_ARG, "iters out of range");
  const dim3 grid(256);
  const uint4* sd = (const uint4*)seed;
  float* sk = (float*)sink;
  switch (waves_per_simd) {
    // (accumulator tiles per wave: as many as the wave's share of the register file holds)
    case 1: hipLaunchKernelGGL((probe_mfma_kernel<256, 64>), grid, dim3(256), 0, (hipStream_t)stream, sd, sk, iters); break;
    case 2: hipLaunchKernelGGL((probe_mfma_kernel<512, 32>), grid, dim3(512), 0, (hipStream_t)stream, sd, sk, iters); break;
    case 4: hipLaunchKernelGGL((probe_mfma_kernel<1024, 16>), grid, dim3(1024), 0, (hipStream_t)stream, sd, sk, iters); break;
    default: return fail(NIMBLE_ERR_ARG, "waves_per_simd must be 1, 2 or 4");
  }
  // per wave and pass: 64 / waves_per_simd MFMAs of 16 x 16 x 32 multiply-adds
  *flops = 256.0 * 4.0 * waves_per_simd * (double)iters * (64.0 / waves_per_simd) * (2.0 * 16 * 16 * 32);
  return check_hip(hipGetLastError(), "probe launch");
}

int nimble_probe_hbm_read(const void* buf, size_t bytes, void* sink, void* stream) {
  clear_error();
  if (!buf || !sink) return fail(NIMBLE_ERR_NULL, "null pointer");
  if (misaligned(buf) || misaligned(sink)) return fail(NIMBLE_ERR_ALIGN, "device pointers must be 16-byte aligned");
  if (bytes % 16 != 0) return fail(NIMBLE_ERR_ARG, "bytes must be a multiple of 16");
  const long long n16 = (long long)(bytes / 16);
  if (n16 == 0) return NIMBLE_OK;
  const long long blocks = (n16 + 1023) / 1024;
  if (blocks > 0x7fffffffll) return fail(NIMBLE_ERR_ARG, "buffer too large");
  hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)buf, n16, (uint4*)sink);
  return check_hip(hipGetLastError(), "probe launch");
}

}  // extern "C"

