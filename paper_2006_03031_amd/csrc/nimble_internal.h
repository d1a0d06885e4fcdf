// Internal declarations shared by the host dispatcher and the kernel launchers.
#ifndef NIMBLE_INTERNAL_H_
#define NIMBLE_INTERNAL_H_

#include "nimble.h"

namespace nimble {

struct VariantInfo {
  const char* name;
  int bm, bn, bk, threads;
};
extern const VariantInfo kVariants[NIMBLE_VAR_COUNT];

// The chip this library is written for: MI355X, 256 compute units in 8 XCDs.
constexpr int kComputeUnits = 256;
// Workgroups of a tiled variant that share a compute unit (LDS and registers permitting).
constexpr int kTilesPerCU[NIMBLE_VAR_COUNT] = {1, 1, 2, 2, 2, 1, 1};

// Record a message for nimble_last_error() and return `code`.
int fail(int code, const char* fmt, ...);
void clear_error();

bool tiled_variant_ok(int variant, int64_t M, int64_t N, int64_t K);
// bm = 0 or the variant's own height: always; else the heights the variant is also built at.
bool tile_rows_ok(int variant, int bm, int64_t N, int64_t K);

// Weights above this size are taken to come from HBM on every call (the L2s hold 32 MB, the
// memory-side cache 256 MB shared with everything else in flight); smaller layers are priced
// as cache-resident, which is what a layer loop or a token loop sees.
constexpr double kCachedWeightBytes = 64e6;

// Whether a weight-streaming launch of 16-row blocks over an [N, K] weight can run the LDS-staged
// streaming kernel (the LSTM cell needs Ix % 64 == 0 besides).
bool stream_kernel_shape_ok(int64_t N, int64_t K);

struct PlanOptions {
  uint64_t max_workspace = 0;   // bytes of caller scratch available (split-K partial sums)
  bool allow_row_split = true;  // may dispatch x = bm*k + r as two launches
  int force_split_k = 0;        // > 0 with a forced variant: cut K into exactly this many slices
  bool use_table = true;        // consult the tuned dispatch table before the cost model
};

// Dispatch table shared by dense (batch = 1) and batch_matmul.
int plan_dense(int64_t batch, int64_t M, int64_t N, int64_t K, int epilogue, int force_variant,
               const PlanOptions& opt, nimble_plan* p);

// One C = epi(alpha * A.B^T + bias) problem as the kernels see it.  A is
// [M,K] with row stride lda, B is [N,K] with row stride ldb (or, when
// b_is_kn, [K,N] with row stride ldb), C is [M,N] with row stride ldc; strides
// in elements; batch strides sa/sb/sc in elements.
struct GemmArgs {
  const void* a;
  const void* b;
  const void* bias;
  void* c;
  int M, N, K;
  int lda, ldb, ldc;
  long long sa, sb, sc;
  float alpha;
  int epilogue;
  int out_f32;
  int b_is_kn;
  int batch;
};

}  // namespace nimble
#endif
