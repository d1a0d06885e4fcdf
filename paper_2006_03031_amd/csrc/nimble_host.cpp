// Host side of the dynamic-shape path: shape functions (Section 3.2), storage
// sizes (Section 3.3), the residue split and the dispatch function's table
// (Section 3.5).  Integer arithmetic only; no HIP call in this file.
#include "nimble_internal.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>

namespace nimble {

static thread_local char g_err[256] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = '\0'; }

const VariantInfo kVariants[NIMBLE_VAR_COUNT] = {
    // name       bm   bn   bk  threads
    {"generic", 16, 16, 1, 256},
    {"skinny16", 16, 16, 32, 256},
    {"t32x128", 32, 128, 64, 256},
    {"t64x128", 64, 128, 64, 256},
    {"t128x128", 128, 128, 64, 256},
    {"t256x128", 256, 128, 64, 256},
    {"t256x256", 256, 256, 64, 256},
};

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Number of compute units of one MI355X.
static const int64_t kCUs = 256;

// Relative cost of one macro tile per unit of K: area divided by how well the
// variant keeps the matrix cores busy (measured per-variant efficiencies).
static double tile_cost(int variant) {
  switch (variant) {
    case NIMBLE_VAR_T32x128: return 32.0 * 128 / 0.25;
    case NIMBLE_VAR_T64x128: return 64.0 * 128 / 0.40;
    case NIMBLE_VAR_T128x128: return 128.0 * 128 / 0.70;
    case NIMBLE_VAR_T256x128: return 256.0 * 128 / 0.90;
    case NIMBLE_VAR_T256x256: return 256.0 * 256 / 1.00;
    default: return 1e30;
  }
}

bool tiled_variant_ok(int variant, int64_t M, int64_t N, int64_t K) {
  (void)M;
  (void)N;
  if (variant < NIMBLE_VAR_T32x128 || variant > NIMBLE_VAR_T256x256) return false;
  return K > 0 && K % 8 == 0;  // rows must stay 16-byte aligned
}

static void fill_tiled(nimble_plan* p, int variant, int64_t batch, int64_t M, int64_t N, int64_t K) {
  const VariantInfo& v = kVariants[variant];
  p->variant = variant;
  p->bm = v.bm;
  p->bn = v.bn;
  p->bk = v.bk;
  p->k = M / v.bm;
  p->r = (int32_t)(M % v.bm);
  p->residue_copy = (p->r != 0 || N % v.bn != 0 || K % v.bk != 0) ? 1 : 0;
  p->split_k = 1;
  p->grid[0] = (uint32_t)(ceil_div(M, v.bm) * ceil_div(N, v.bn));
  p->grid[1] = 1;
  p->grid[2] = (uint32_t)batch;
  p->block = (uint32_t)v.threads;
  p->workspace_bytes = 0;
}

// Choose the tiled variant whose estimated time is least.  The busiest compute
// unit executes ceil(tiles / CUs) tiles, so a dynamic M just past a tile
// boundary can cost a whole extra tile per CU with big tiles; smaller tiles
// quantise more finely but run the matrix cores less efficiently.
static int choose_tiled(int64_t batch, int64_t M, int64_t N, int64_t K) {
  int best = -1;
  double best_cost = 0;
  for (int v = NIMBLE_VAR_T32x128; v <= NIMBLE_VAR_T256x256; ++v) {
    if (!tiled_variant_ok(v, M, N, K)) continue;
    const VariantInfo& vi = kVariants[v];
    if (v > NIMBLE_VAR_T32x128 && M <= kVariants[v - 1].bm) break;  // tile taller than needed
    const int64_t tiles = batch * ceil_div(M, vi.bm) * ceil_div(N, vi.bn);
    const double cost = (double)ceil_div(tiles, kCUs) * tile_cost(v);
    if (best < 0 || cost < best_cost) {
      best = v;
      best_cost = cost;
    }
  }
  return best;
}

int plan_dense(int64_t batch, int64_t M, int64_t N, int64_t K, int force_variant, nimble_plan* p) {
  std::memset(p, 0, sizeof(*p));
  if (M < 0 || N < 0 || K < 0 || batch < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (M > (1ll << 30) || N > (1ll << 30) || K > (1ll << 30) || batch > 65535)
    return fail(NIMBLE_ERR_ARG, "extent too large");
  if (M * N > (1ll << 40)) return fail(NIMBLE_ERR_ARG, "output too large");
  int variant = force_variant;
  if (variant == NIMBLE_VAR_AUTO) {
    const char* env = std::getenv("NIMBLE_FORCE_VARIANT");
    if (env && *env) variant = std::atoi(env);
  }
  if (variant < NIMBLE_VAR_AUTO || variant >= NIMBLE_VAR_COUNT)
    return fail(NIMBLE_ERR_ARG, "unknown variant %d", variant);

  const bool aligned_k = (K > 0 && K % 8 == 0);
  if (variant == NIMBLE_VAR_AUTO) {
    if (!aligned_k || M == 0 || N == 0) {
      variant = NIMBLE_VAR_GENERIC;
    } else if (M <= 64 && batch == 1) {
      variant = NIMBLE_VAR_SKINNY16;
    } else {
      variant = choose_tiled(batch, M, N, K);
      if (variant < 0) variant = NIMBLE_VAR_GENERIC;
    }
  }

  if (variant == NIMBLE_VAR_GENERIC) {
    const VariantInfo& v = kVariants[variant];
    p->variant = variant;
    p->bm = v.bm;
    p->bn = v.bn;
    p->bk = v.bk;
    p->k = M / v.bm;
    p->r = (int32_t)(M % v.bm);
    p->residue_copy = 1;
    p->split_k = 1;
    p->grid[0] = (uint32_t)ceil_div(N, v.bn);
    p->grid[1] = (uint32_t)ceil_div(M, v.bm);
    p->grid[2] = (uint32_t)batch;
    p->block = 256;
    return NIMBLE_OK;
  }
  if (variant == NIMBLE_VAR_SKINNY16) {
    if (!aligned_k) return fail(NIMBLE_ERR_ARG, "skinny16 needs K %% 8 == 0");
    if (batch != 1) return fail(NIMBLE_ERR_ARG, "skinny16 is not batched");
    const VariantInfo& v = kVariants[variant];
    p->variant = variant;
    p->bm = v.bm;
    p->bn = v.bn;
    p->bk = v.bk;
    p->k = M / v.bm;
    p->r = (int32_t)(M % v.bm);
    p->residue_copy = (p->r != 0 || N % v.bn != 0 || K % v.bk != 0) ? 1 : 0;
    p->split_k = 4;  // the four waves of a workgroup each take a quarter of K
    p->grid[0] = (uint32_t)ceil_div(N, v.bn);
    p->grid[1] = (uint32_t)ceil_div(M, 64);  // up to four 16-row tiles per workgroup
    p->grid[2] = 1;
    p->block = 256;
    return NIMBLE_OK;
  }
  if (!tiled_variant_ok(variant, M, N, K))
    return fail(NIMBLE_ERR_ARG, "variant %s cannot run K=%lld", kVariants[variant].name, (long long)K);
  fill_tiled(p, variant, batch, M, N, K);
  return NIMBLE_OK;
}

static size_t dtype_size(int dtype) {
  switch (dtype) {
    case NIMBLE_BF16: return 2;
    case NIMBLE_F32: return 4;
    default: return 0;
  }
}

}  // namespace nimble

using namespace nimble;

extern "C" {

int nimble_dense_shape(const int64_t* x_shape, int x_rank, const int64_t* w_shape, int w_rank,
                       int64_t* out_shape) {
  clear_error();
  if (!x_shape || !w_shape || !out_shape) return fail(NIMBLE_ERR_NULL, "null shape pointer");
  if (x_rank != 2 || w_rank != 2)
    return fail(NIMBLE_ERR_RANK, "dense expects ranks (2,2), got (%d,%d)", x_rank, w_rank);
  if (x_shape[0] < 0 || x_shape[1] < 0 || w_shape[0] < 0 || w_shape[1] < 0)
    return fail(NIMBLE_ERR_ARG, "negative extent");
  if (x_shape[1] != w_shape[1])
    return fail(NIMBLE_ERR_SHAPE, "dense: K of x (%lld) != K of w (%lld)", (long long)x_shape[1],
                (long long)w_shape[1]);
  out_shape[0] = x_shape[0];
  out_shape[1] = w_shape[0];
  return NIMBLE_OK;
}

int nimble_batch_matmul_shape(const int64_t* a_shape, int a_rank, const int64_t* b_shape,
                              int b_rank, int trans_b, int64_t* out_shape) {
  clear_error();
  if (!a_shape || !b_shape || !out_shape) return fail(NIMBLE_ERR_NULL, "null shape pointer");
  if (a_rank != 3 || b_rank != 3)
    return fail(NIMBLE_ERR_RANK, "batch_matmul expects ranks (3,3), got (%d,%d)", a_rank, b_rank);
  for (int i = 0; i < 3; ++i)
    if (a_shape[i] < 0 || b_shape[i] < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  const int64_t kb = trans_b ? b_shape[2] : b_shape[1];
  const int64_t nb = trans_b ? b_shape[1] : b_shape[2];
  if (a_shape[0] != b_shape[0])
    return fail(NIMBLE_ERR_SHAPE, "batch_matmul: batch %lld != %lld", (long long)a_shape[0],
                (long long)b_shape[0]);
  if (a_shape[2] != kb)
    return fail(NIMBLE_ERR_SHAPE, "batch_matmul: K %lld != %lld", (long long)a_shape[2], (long long)kb);
  out_shape[0] = a_shape[0];
  out_shape[1] = a_shape[1];
  out_shape[2] = nb;
  return NIMBLE_OK;
}

int nimble_lstm_shape(const int64_t* x_shape, const int64_t* h_shape, const int64_t* c_shape,
                      const int64_t* w_shape, int64_t* h_out_shape, int64_t* c_out_shape) {
  clear_error();
  if (!x_shape || !h_shape || !c_shape || !w_shape || !h_out_shape || !c_out_shape)
    return fail(NIMBLE_ERR_NULL, "null shape pointer");
  for (int i = 0; i < 2; ++i)
    if (x_shape[i] < 0 || h_shape[i] < 0 || c_shape[i] < 0 || w_shape[i] < 0)
      return fail(NIMBLE_ERR_ARG, "negative extent");
  const int64_t B = x_shape[0], Ix = x_shape[1], H = h_shape[1];
  if (h_shape[0] != B || c_shape[0] != B) return fail(NIMBLE_ERR_SHAPE, "lstm: batch extents differ");
  if (c_shape[1] != H) return fail(NIMBLE_ERR_SHAPE, "lstm: c is not (B,H)");
  if (w_shape[0] != 4 * H || w_shape[1] != Ix + H)
    return fail(NIMBLE_ERR_SHAPE, "lstm: w is not (4H, Ix+H)");
  h_out_shape[0] = c_out_shape[0] = B;
  h_out_shape[1] = c_out_shape[1] = H;
  return NIMBLE_OK;
}

int64_t nimble_storage_bytes(const int64_t* shape, int rank, int dtype) {
  clear_error();
  if (rank < 0 || (rank > 0 && !shape)) return fail(NIMBLE_ERR_NULL, "null shape pointer");
  const size_t es = dtype_size(dtype);
  if (es == 0) return fail(NIMBLE_ERR_DTYPE, "unknown dtype %d", dtype);
  int64_t n = 1;
  for (int i = 0; i < rank; ++i) {
    if (shape[i] < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
    if (shape[i] != 0 && n > std::numeric_limits<int64_t>::max() / (8 * shape[i]))
      return fail(NIMBLE_ERR_ARG, "size overflows int64");
    n *= shape[i];
  }
  return n * (int64_t)es;
}

int64_t nimble_storage_alignment(void) { return 64; }

int nimble_residue_split(int64_t x, int64_t tile, int64_t* k, int64_t* r) {
  clear_error();
  if (!k || !r) return fail(NIMBLE_ERR_NULL, "null output pointer");
  if (x < 0 || tile <= 0) return fail(NIMBLE_ERR_ARG, "need x >= 0 and tile > 0");
  *k = x / tile;
  *r = x % tile;
  return NIMBLE_OK;
}

int nimble_dense_plan(int64_t M, int64_t N, int64_t K, int epilogue, int out_dtype,
                      int force_variant, nimble_plan* plan) {
  clear_error();
  if (!plan) return fail(NIMBLE_ERR_NULL, "null plan");
  if (epilogue < NIMBLE_EPI_NONE || epilogue > NIMBLE_EPI_BIAS_GELU_ERF)
    return fail(NIMBLE_ERR_ARG, "unknown epilogue %d", epilogue);
  if (dtype_size(out_dtype) == 0) return fail(NIMBLE_ERR_DTYPE, "unknown dtype %d", out_dtype);
  return plan_dense(1, M, N, K, force_variant, plan);
}

int nimble_batch_matmul_plan(int64_t batch, int64_t M, int64_t N, int64_t K, int trans_b,
                             int out_dtype, nimble_plan* plan) {
  clear_error();
  if (!plan) return fail(NIMBLE_ERR_NULL, "null plan");
  if (dtype_size(out_dtype) == 0) return fail(NIMBLE_ERR_DTYPE, "unknown dtype %d", out_dtype);
  if (!trans_b) {
    // b is (T,K,N): rows of b are not K-contiguous; the bounds-checked kernel reads it strided
    return plan_dense(batch, M, N, K, NIMBLE_VAR_GENERIC, plan);
  }
  const int force = (batch > 1 || M > 64) ? NIMBLE_VAR_AUTO : NIMBLE_VAR_AUTO;
  int rc = plan_dense(batch, M, N, K, force, plan);
  if (rc == NIMBLE_OK && plan->variant == NIMBLE_VAR_SKINNY16 && batch != 1)
    rc = plan_dense(batch, M, N, K, NIMBLE_VAR_GENERIC, plan);
  return rc;
}

int nimble_lstm_plan(int64_t B, int64_t Ix, int64_t H, nimble_plan* plan) {
  clear_error();
  if (!plan) return fail(NIMBLE_ERR_NULL, "null plan");
  std::memset(plan, 0, sizeof(*plan));
  if (B < 0 || Ix < 0 || H < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (Ix % 8 != 0 || H % 8 != 0 || H == 0)
    return fail(NIMBLE_ERR_ARG, "lstm needs Ix and H to be multiples of 8 (H > 0)");
  if (B > (1ll << 24) || Ix > (1ll << 24) || H > (1ll << 24)) return fail(NIMBLE_ERR_ARG, "extent too large");
  plan->variant = NIMBLE_VAR_SKINNY16;
  plan->bm = 16;
  plan->bn = 16;  // four hidden units times four gates
  plan->bk = 32;
  plan->k = B / 16;
  plan->r = (int32_t)(B % 16);
  plan->residue_copy = plan->r != 0;
  plan->split_k = 4;
  plan->grid[0] = (uint32_t)ceil_div(H, 4);
  plan->grid[1] = (uint32_t)ceil_div(B, 64);
  plan->grid[2] = 1;
  plan->block = 256;
  return NIMBLE_OK;
}

const char* nimble_variant_name(int variant) {
  if (variant < 0 || variant >= NIMBLE_VAR_COUNT) return nullptr;
  return kVariants[variant].name;
}

const char* nimble_last_error(void) { return g_err; }

}  // extern "C"
