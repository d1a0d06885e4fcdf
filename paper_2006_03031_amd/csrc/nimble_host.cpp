// Host side of the dynamic-shape path: shape functions (Section 3.2), storage
// sizes (Section 3.3), the residue split and the dispatch function's table
// (Section 3.5).  Integer arithmetic only; no HIP call in this file.
#include "nimble_internal.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <map>
#include <tuple>
#include <vector>

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
    {"t32x128", 32, 128, 32, 128},
    {"t64x128", 64, 128, 32, 256},
    {"t128x128", 128, 128, 32, 256},
    {"t256x128", 256, 128, 32, 512},
    {"t256x256", 256, 256, 32, 512},
};

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Number of compute units of one MI355X.
static const int64_t kCUs = kComputeUnits;

// Estimated time of one macro tile, in arbitrary units: the tile's area times
// (K plus a fixed per-tile overhead expressed in units of K: pipeline fill and
// the epilogue, which is larger with GELU), divided by how well the variant
// keeps the matrix cores busy in steady state (measured per variant at
// M = 8192 on the BERT-large FFN shapes).
static double tile_cost(int variant, int64_t K, int epilogue, int bm = 0) {
  double eff;
  switch (variant) {
    case NIMBLE_VAR_T32x128: eff = 0.202; break;
    case NIMBLE_VAR_T64x128: eff = 0.450; break;
    case NIMBLE_VAR_T128x128: eff = 0.560; break;
    case NIMBLE_VAR_T256x128: eff = 1.031; break;
    case NIMBLE_VAR_T256x256: eff = 1.10; break;
    default: return 1e30;
  }
  const double k0 = (epilogue == NIMBLE_EPI_BIAS_GELU_ERF) ? 256.0 : 128.0;
  // a tile of another height loads the same weight panel for fewer or more rows: measured
  // time(bm) / time(256) = 0.09 + 0.91 bm/256 for the 256-wide tile (bm = 128..320)
  const double height = (bm > 0 && bm != kVariants[variant].bm)
                            ? 0.0925 + 0.9075 * (double)bm / (double)kVariants[variant].bm : 1.0;
  return (double)kVariants[variant].bm * kVariants[variant].bn * ((double)K + k0) * height / eff;
}

// Heights the 256-wide tile is built at: 2 wave rows of 4..10 MFMA tiles of 16 rows.
static const int kTileRows256[] = {320, 288, 256, 224, 192, 160, 128};

bool tile_rows_ok(int variant, int bm, int64_t N, int64_t K) {
  if (bm == 0 || bm == kVariants[variant].bm) return true;
  if (variant != NIMBLE_VAR_T256x256) return false;
  if (N % 256 != 0 || K % 32 != 0) return false;  // the reduced heights have no ragged N/K body
  for (int h : kTileRows256)
    if (h == bm) return true;
  return false;
}

bool tiled_variant_ok(int variant, int64_t M, int64_t N, int64_t K) {
  (void)M;
  (void)N;
  if (variant < NIMBLE_VAR_T32x128 || variant > NIMBLE_VAR_T256x256) return false;
  // rows must stay 16-byte aligned; per-lane byte offsets inside a tile are 32-bit
  return K > 0 && K % 8 == 0 && K <= (1ll << 22);
}

// One unit of tile_cost in microseconds (a 256x256 tile at K = 1024 with GELU takes about 37 us
// when the whole chip is busy).
static const double kUsPerUnit = 4.4e-7;
// Gap between two dependent launches on one stream, microseconds.
static const double kLaunchGapUs = 3.5;
// The same gap as it shows between a K-split kernel and its reduction, whose launch the
// hardware queue has already decoded while the first kernel runs.
static const double kSplitGapUs = 1.80;


// Estimated time of one launch of tiled variant v over `rows` rows with K cut into `sk`
// slices, microseconds.  The tiles run in rounds of one per compute unit.  A full round runs
// at the chip's power-limited rate; the last, partial round runs faster per tile the fewer
// units it occupies.  So a dynamic M just past a tile boundary costs most of an extra round
// with big tiles, while smaller tiles quantise more finely but run the matrix cores less
// efficiently.  Cutting K multiplies the tiles and shortens each; the partial sums then cross
// HBM once more and a second small kernel adds them up.  The constants are a fit to graph-timed
// launches of every variant and K split over the BERT-base/large and LSTM layer shapes at
// 17 .. 2048 rows; over that set the choices made here cost 0.6 % more than the best ones.
static double tiled_cost_us(int v, int64_t batch, int64_t rows, int64_t N, int64_t K, int epilogue,
                            int sk = 1, int bm = 0) {
  const VariantInfo& vi = kVariants[v];
  const int64_t tiles = batch * ceil_div(rows, bm > 0 ? bm : vi.bm) * ceil_div(N, vi.bn) * sk;
  const int64_t k_slice = ceil_div(ceil_div(K, 32), sk) * 32;
  // a workgroup cannot go faster than its loads arrive through the direct global->LDS path:
  // a 32-wide stage of (bm + bn) rows costs a lone workgroup 0.13 .. 0.3 us.  A GELU epilogue
  // adds about a microsecond to such a latency-bound tile.
  static const double kStageFloorUs[NIMBLE_VAR_COUNT] = {0, 0, 0.1665, 0.161, 0.382, 0.237, 0.345};
  // time of a tile in a nearly empty last round relative to a full one
  static const double kLoneTile[NIMBLE_VAR_COUNT] = {0, 0, 0.185, 0.388, 0.678, 0.598, 0.659};
  const int64_t stages = ceil_div(k_slice, 32);
  const bool gelu = sk == 1 && epilogue == NIMBLE_EPI_BIAS_GELU_ERF;
  const double latency_floor = (double)stages * kStageFloorUs[v] + (gelu ? 0.05 : 0.0);
  const double t_full = tile_cost(v, k_slice, sk > 1 ? NIMBLE_EPI_NONE : epilogue, bm) * kUsPerUnit;
  // a round is one tile per compute unit for the 8-wave tiles, two for the smaller ones
  const int64_t slots = kCUs * kTilesPerCU[v];
  const int64_t full_rounds = tiles / slots, rem = tiles % slots;
  double us = (double)full_rounds * (t_full > latency_floor ? t_full : latency_floor);
  if (rem > 0) {
    const double occ = (double)rem / (double)slots;
    const double t_part = t_full * (kLoneTile[v] + (1.0 - kLoneTile[v]) * occ);
    us += t_part > latency_floor ? t_part : latency_floor;
  }
  // all workgroups together pull about 14 TB/s from the L2s into LDS with real operand data:
  // many small tiles re-fetch the operand panels often enough to hit that before anything else
  const double dma_us = (double)tiles * (double)stages * (double)((bm > 0 ? bm : vi.bm) + vi.bn) * 64.0 / 13.9e6;
  if (us < dma_us) us = dma_us;
  // a layer too large to stay in the caches streams its weights from HBM: about 4.2 TB/s with
  // one workgroup per compute unit, 6.4 TB/s from two up
  if ((double)N * (double)K * 2.0 > kCachedWeightBytes) {
    double fill = (double)tiles / (double)kCUs - 1.0;
    fill = fill < 0.0 ? 0.0 : (fill > 1.0 ? 1.0 : fill);
    const double hbm_us = (double)N * (double)K * 2.0 / (4.19e6 + 2.21e6 * fill);
    if (us < hbm_us) us = hbm_us;
  }
  // the reduction: a dependent launch, a fixed cost per slice, and the partial sums' traffic
  if (sk > 1) us += kSplitGapUs + 0.259 * (double)sk + (double)(sk + 1) * (double)rows * (double)N * 4.0 / 3.97e6;
  return us;
}

// Launch-to-first-result time of one kernel, which the tiled estimates above leave out (it is
// the same for every single-launch choice) and the weight-streaming estimate includes.
static const double kLaunchUs = 3.5;

// Whether a weight-streaming launch of 16-row blocks runs the LDS-staged streaming kernel (the
// launcher applies the same test): K in whole 64-wide stages, 32-bit byte offsets into the weights.
// NIMBLE_NO_STREAM (a measurement knob) turns that kernel off in both places.
bool stream_kernel_shape_ok(int64_t N, int64_t K) {
  static const bool off = std::getenv("NIMBLE_NO_STREAM") != nullptr;
  return !off && K >= 64 && K % 64 == 0 && (uint64_t)N * (uint64_t)K * 2u < (1ull << 32);
}

// Row blocks of a weight-streaming launch: a workgroup takes 16 weight rows and 16..64
// activation rows.  Where the streaming kernel runs and the layer stays in the caches, every
// workgroup takes 16 activation rows (each block re-reads the weights, which then come from L2:
// the BERT-base and LSTM layers at 17..64 rows run 5-25 % faster that way than in blocks of 32..64
// rows on the register-layout kernel).  Otherwise: a narrow layer (few weight rows) fills the chip
// only when the activation rows are spread over several workgroups, each re-reading its weight
// rows (they meet in L2); a wide layer already has a workgroup per compute unit and keeps one block
// per 64 rows so that the weights cross HBM once.
static int64_t skinny_row_blocks(int64_t rows, int64_t N, int64_t K, bool stream_ok) {
  if (stream_ok && (double)N * (double)K * 2.0 <= kCachedWeightBytes) return rows > 16 ? ceil_div(rows, 16) : 1;
  int64_t blocks = kCUs / ceil_div(N, 16);
  const int64_t most = ceil_div(rows, 16), fewest = ceil_div(rows, 64);
  if (blocks > most) blocks = most;
  if (blocks < fewest) blocks = fewest;
  return blocks < 1 ? 1 : blocks;
}

// The weight-streaming kernels, launch latency included.
// Streaming kernel (blocks of 16 rows): whichever is longer of the weight stream and the waves'
// walk over their K stages, round of workgroups after round.  Measured: a 134 MB layer from HBM
// 24.0 us at 1..8 rows and 27.9 at 16; cache-resident layers 2.5-2.8 us at K = 768..1024, 3.3-4.1 at
// K = 3072..4096 (0.14-0.20 us per stage of a wave's eight-way share of K); 17..64 rows on the 8 MB
// layers 3.6-4.9 us; 128 rows on 768 -> 768, 3072 -> 768 and 4096 -> 1024: 3.3, 5.7 and 6.7 us, where the
// best tile with K cut takes 6.9, 10.5 and 11.3; 256 rows on 768 -> 2304: 7.8 us (the 64-row tile 7.1).
// Register-layout kernel (any K): the activations are re-read once per 16 weight rows, which shows
// from 32 rows on; N / 16 workgroups only, so a short, wide layer leaves most of the chip idle.
// Fitted to 8 MB .. 134 MB layers at M = 1 .. 64.
static double skinny_cost_us(int64_t rows, int64_t N, int64_t K) {
  const double bytes = (double)N * (double)K * 2.0;
  const bool cached = bytes <= kCachedWeightBytes;
  if (stream_kernel_shape_ok(N, K) && (rows <= 16 || cached)) {
    // every 16-row block re-reads the weights: from L2 at about 15 TB/s when the layer is cache-resident
    const int64_t blocks16 = ceil_div(rows, 16);
    const int64_t wgs = ceil_div(N, 16) * blocks16;
    const double rate = cached ? 15e6 : (rows <= 8 ? 6.2e6 : 5.26e6);  // bytes per microsecond
    const double stream = bytes * (double)blocks16 / rate;
    double walk;
    if (wgs <= kCUs || !cached) {
      // one round of eight-wave workgroups: 0.45 us plus a wave's walk over its eighth of the K stages
      const int64_t rounds = ceil_div(wgs, kCUs);
      walk = (double)rounds * (0.45 + (double)ceil_div(ceil_div(K, 64), 8) * (rows <= 8 ? 0.14 : 0.20));
    } else {
      // four-wave workgroups, four to a compute unit: each holds its place for about 2 us plus 0.11 us per
      // stage of a wave's quarter of K
      walk = (double)wgs * (2.0 + 0.11 * (double)ceil_div(ceil_div(K, 64), 4)) / (4.0 * (double)kCUs);
      if (walk < 0.8) walk = 0.8;
    }
    return kLaunchUs + (stream > walk ? stream : walk);
  }
  const int64_t nblocks = skinny_row_blocks(rows, N, K, false);
  const double mt = (double)ceil_div(rows, 16 * nblocks);
  const double blocks = (double)ceil_div(rows, 64);
  const double rate = !cached ? 5.94e6 : 6.79e6;  // bytes per microsecond
  const double stream = bytes / rate * (1.0 + 0.553 * (double)rows / (double)nblocks / 16.0);
  const double walk = (double)ceil_div(K, 128) * mt * 0.126;
  return kLaunchUs + blocks * (stream > walk ? stream : walk);
}

static bool split_k_ok(int v, int64_t batch, int64_t N, int64_t K, int sk) {
  if (sk == 1) return true;
  if (v < NIMBLE_VAR_T32x128 || batch != 1) return false;         // tiled kernels, dense only
  if (N % kVariants[v].bn != 0 || K % 32 != 0) return false;       // no ragged N/K tiles
  const int64_t stages = K / 32, per = ceil_div(stages, sk);
  return per >= 4 && per * (sk - 1) < stages;                      // every slice gets work
}

// Tuned overrides, keyed by (N, K, epilogue).
static std::map<std::tuple<int64_t, int64_t, int>, std::vector<nimble_table_entry>> g_tables;

static const nimble_table_entry* table_lookup(int64_t M, int64_t N, int64_t K, int epilogue) {
  auto it = g_tables.find(std::make_tuple(N, K, epilogue));
  if (it == g_tables.end()) return nullptr;
  for (const nimble_table_entry& e : it->second)
    if (M >= e.m_lo && M <= e.m_hi) return &e;
  return nullptr;
}

struct Launch {
  int variant = -1;
  int split_k = 1;
  int bm = 0;  // tile height when it differs from the variant's own
  double us = 0;
};

// Best single launch for `rows` rows: the least estimated time among weight streaming (up to
// 64 rows) and every tiled variant and K split that fits the workspace.
static Launch best_launch(int64_t batch, int64_t rows, int64_t N, int64_t K, int epilogue,
                          uint64_t max_workspace, bool allow_skinny) {
  Launch best;
  double skinny_us = -1.0;
  // weight streaming: up to 64 rows, and beyond that in 16-row blocks of the streaming kernel while
  // the layer is small enough for the blocks' re-reads to come from L2
  if (allow_skinny && batch == 1 &&
      (rows <= 64 || (rows <= 512 && stream_kernel_shape_ok(N, K) && (double)N * (double)K * 2.0 <= kCachedWeightBytes))) {
    skinny_us = skinny_cost_us(rows, N, K);
  }
  for (int v = NIMBLE_VAR_T32x128; v <= NIMBLE_VAR_T256x256; ++v) {
    if (!tiled_variant_ok(v, rows, N, K)) continue;
    if (v > NIMBLE_VAR_T32x128 && rows <= kVariants[v - 1].bm) break;  // tile taller than needed
    for (int sk = 1; sk <= 16; sk *= 2) {
      if (!split_k_ok(v, batch, N, K, sk)) continue;
      if (sk > 1 && (uint64_t)sk * (uint64_t)rows * (uint64_t)N * 4u > max_workspace) continue;
      const double us = tiled_cost_us(v, batch, rows, N, K, epilogue, sk);
      if (best.variant < 0 || us < best.us) {
        best.variant = v;
        best.split_k = sk;
        best.bm = 0;
        best.us = us;
      }
    }
    // the same tile at a reduced height: with the run-time M known, pick the height at which
    // the tile rows fill whole rounds of the chip instead of leaving a mostly empty last round
    static const bool heights_on = !(std::getenv("NIMBLE_TILE_ROWS") && std::atoi(std::getenv("NIMBLE_TILE_ROWS")) == 0);
    if (v == NIMBLE_VAR_T256x256 && batch == 1 && heights_on)
      for (int bm : kTileRows256) {
        if (bm == kVariants[v].bm || rows <= bm || !tile_rows_ok(v, bm, N, K)) continue;
        const double us = tiled_cost_us(v, batch, rows, N, K, epilogue, 1, bm);
        if (us < best.us) {
          best.variant = v;
          best.split_k = 1;
          best.bm = bm;
          best.us = us;
        }
      }
  }
  // up to 64 rows the small tiles (with K cut) compete with weight streaming (compared launch included);
  // up to 16 rows the streaming kernel was the fastest choice on every layer measured
  if (skinny_us >= 0.0 && (best.variant < 0 || skinny_us <= best.us + kLaunchUs ||
                           (rows <= 16 && stream_kernel_shape_ok(N, K)))) {
    best = Launch();
    best.variant = NIMBLE_VAR_SKINNY16;
    best.us = skinny_us;
  }
  return best;
}

static void fill_tiled(nimble_plan* p, int variant, int split_k, int64_t batch, int64_t M, int64_t N,
                       int64_t K, int bm = 0) {
  VariantInfo v = kVariants[variant];
  if (bm > 0) v.bm = bm;
  p->variant = variant;
  p->bm = v.bm;
  p->bn = v.bn;
  p->bk = v.bk;
  p->k = M / v.bm;
  p->r = (int32_t)(M % v.bm);
  p->residue_copy = (p->r != 0 || N % v.bn != 0 || K % v.bk != 0) ? 1 : 0;
  p->split_k = split_k;
  p->grid[0] = (uint32_t)(ceil_div(M, v.bm) * ceil_div(N, v.bn));
  p->grid[1] = (uint32_t)split_k;
  p->grid[2] = (uint32_t)batch;
  p->block = (uint32_t)v.threads;
  p->workspace_bytes = split_k > 1 ? (uint64_t)split_k * (uint64_t)M * (uint64_t)N * 4u : 0;
}

int plan_dense(int64_t batch, int64_t M, int64_t N, int64_t K, int epilogue, int force_variant,
               const PlanOptions& opt, nimble_plan* p) {
  std::memset(p, 0, sizeof(*p));
  p->residue_variant = NIMBLE_VAR_AUTO;
  if (M < 0 || N < 0 || K < 0 || batch < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  if (M > (1ll << 30) || N > (1ll << 30) || K > (1ll << 30) || batch > 65535)
    return fail(NIMBLE_ERR_ARG, "extent too large");
  if (M * N > (1ll << 40)) return fail(NIMBLE_ERR_ARG, "output too large");
  int variant = force_variant;
  if (variant == NIMBLE_VAR_AUTO) {
    // measurement knob, read once: a force_variant value applied to every automatic plan
    static const int env_variant = [] {
      const char* env = std::getenv("NIMBLE_FORCE_VARIANT");
      return (env && *env) ? std::atoi(env) : (int)NIMBLE_VAR_AUTO;
    }();
    variant = env_variant;
  }
  const bool forced = variant != NIMBLE_VAR_AUTO;
  // a forced variant may carry a forced K split in bits 8..15 (NIMBLE_FORCE_SPLIT_K) and a
  // forced tile height in bits 16..23 (NIMBLE_FORCE_TILE_ROWS)
  int forced_sk = opt.force_split_k;
  int tile_rows = 0;
  if (variant >= 0) {
    if ((variant >> 8) & 0xff) forced_sk = (variant >> 8) & 0xff;
    tile_rows = ((variant >> 16) & 0xff) * 16;
    variant &= 0xff;
  }
  if (variant < NIMBLE_VAR_AUTO || variant >= NIMBLE_VAR_COUNT)
    return fail(NIMBLE_ERR_ARG, "unknown variant %d", variant);

  const bool aligned_k = (K > 0 && K % 8 == 0);
  int64_t split_rows = 0;
  int residue_variant = NIMBLE_VAR_AUTO;
  int split_k = 1;
  if (variant == NIMBLE_VAR_AUTO) {
    if (!aligned_k || M == 0 || N == 0) {
      variant = NIMBLE_VAR_GENERIC;
    } else if (const nimble_table_entry* e = (batch == 1 && opt.use_table) ? table_lookup(M, N, K, epilogue) : nullptr;
               e && (e->variant == NIMBLE_VAR_SKINNY16 ||
                     (tiled_variant_ok(e->variant, M, N, K) && split_k_ok(e->variant, 1, N, K, e->split_k) &&
                      (e->split_k <= 1 ||
                       (uint64_t)e->split_k * (uint64_t)M * (uint64_t)N * 4u <= opt.max_workspace)))) {
      variant = e->variant;  // tuned: one launch of this configuration
      split_k = e->split_k > 1 ? e->split_k : 1;
    } else {
      const Launch single = best_launch(batch, M, N, K, epilogue, opt.max_workspace, true);
      variant = single.variant < 0 ? NIMBLE_VAR_GENERIC : single.variant;
      split_k = single.split_k;
      tile_rows = single.bm;
      // Alternative: two launches.  Whole tile rows (all k of them, or as many as fill whole
      // rounds of the chip) run the r = 0 copy of a big-tile variant: no bounds code, no
      // partial round.  The remaining rows, residue included, run whatever suits their
      // number.  Taken when the estimate beats the best single launch.
      if (opt.allow_row_split && variant >= NIMBLE_VAR_T32x128 && batch == 1) {
        double best_us = single.us;
        for (int v = NIMBLE_VAR_T128x128; v <= NIMBLE_VAR_T256x256; ++v) {
          const VariantInfo& vi = kVariants[v];
          if (N % vi.bn != 0 || K % vi.bk != 0) continue;
          const int64_t tiles_n = N / vi.bn;
          int64_t cuts[2] = {(M / vi.bm) * vi.bm, 0};
          const int64_t slots = kCUs * kTilesPerCU[v];
          if (slots % tiles_n == 0) {
            const int64_t rows_per_round = (slots / tiles_n) * vi.bm;
            cuts[1] = (M / rows_per_round) * rows_per_round;
          }
          for (int c = 0; c < 2; ++c) {
            const int64_t head = cuts[c], rest = M - head;
            if (head <= 0 || rest <= 0 || (c == 1 && head == cuts[0])) continue;
            const Launch tail = best_launch(1, rest, N, K, epilogue, opt.max_workspace, true);
            if (tail.variant < 0) continue;
            const double us = tiled_cost_us(v, 1, head, N, K, epilogue) + kLaunchGapUs + tail.us;
            if (us < best_us) {
              best_us = us;
              variant = v;
              split_k = 1;
              tile_rows = 0;
              split_rows = head;
              residue_variant = tail.variant;
            }
          }
        }
      }
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
    p->grid[0] = (uint32_t)ceil_div(N, v.bn);
    p->grid[1] = (uint32_t)skinny_row_blocks(M, N, K, stream_kernel_shape_ok(N, K));  // up to four 16-row tiles per workgroup
    p->grid[2] = 1;
    // the waves of a workgroup split K among them: eight in the streaming kernel (16-row blocks,
    // 64-wide stages; four when a cache-resident layer gives more workgroups than compute units),
    // four in the register-layout kernel
    const bool streaming = stream_kernel_shape_ok(N, K) && ceil_div(M, (int64_t)p->grid[1]) <= 16;
    const bool many = (uint64_t)p->grid[0] * p->grid[1] > (uint64_t)kCUs && (double)N * (double)K * 2.0 <= kCachedWeightBytes;
    p->split_k = streaming && !many ? 8 : 4;
    p->bk = streaming ? 64 : v.bk;
    p->block = streaming && !many ? 512 : 256;
    return NIMBLE_OK;
  }
  if (!tiled_variant_ok(variant, M, N, K))
    return fail(NIMBLE_ERR_ARG, "variant %s cannot run K=%lld", kVariants[variant].name, (long long)K);
  if (!tile_rows_ok(variant, tile_rows, N, K))
    return fail(NIMBLE_ERR_ARG, "variant %s is not built with tiles of %d rows for N=%lld K=%lld",
                kVariants[variant].name, tile_rows, (long long)N, (long long)K);
  if (tile_rows > 0 && tile_rows != kVariants[variant].bm && forced_sk > 1)
    return fail(NIMBLE_ERR_ARG, "a reduced tile height cannot be combined with a K split");
  if (forced && forced_sk > 0) {
    if (!split_k_ok(variant, batch, N, K, forced_sk))
      return fail(NIMBLE_ERR_ARG, "variant %s cannot cut K=%lld into %d slices", kVariants[variant].name,
                  (long long)K, forced_sk);
    if (forced_sk > 1 && (uint64_t)forced_sk * (uint64_t)M * (uint64_t)N * 4u > opt.max_workspace)
      return fail(NIMBLE_ERR_WORKSPACE, "cutting K into %d slices needs %llu bytes of workspace", forced_sk,
                  (unsigned long long)((uint64_t)forced_sk * (uint64_t)M * (uint64_t)N * 4u));
    split_k = forced_sk;
  }
  fill_tiled(p, variant, split_k, batch, split_rows > 0 ? split_rows : M, N, K, tile_rows);
  if (split_rows > 0) {
    // k and r describe the whole call; grid and residue_copy describe the first launch; the second
    // launch is planned here exactly as the entry point plans it, so that what is reported (its
    // variant, its K split, the scratch the call needs) is what runs
    PlanOptions tail_opt = opt;
    tail_opt.allow_row_split = false;
    nimble_plan tail;
    const int rc = plan_dense(1, M - split_rows, N, K, epilogue, NIMBLE_VAR_AUTO, tail_opt, &tail);
    if (rc != NIMBLE_OK) return rc;
    p->k = M / p->bm;
    p->r = (int32_t)(M % p->bm);
    p->split_rows = split_rows;
    p->residue_variant = tail.variant;
    p->residue_split_k = tail.split_k;
    if (tail.workspace_bytes > p->workspace_bytes) p->workspace_bytes = tail.workspace_bytes;
    (void)residue_variant;
  }
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

int nimble_lstm_pre_shape(const int64_t* pre_shape, const int64_t* h_shape, const int64_t* c_shape,
                          const int64_t* wh_shape, int64_t* h_out_shape, int64_t* c_out_shape) {
  clear_error();
  if (!pre_shape || !h_shape || !c_shape || !wh_shape || !h_out_shape || !c_out_shape)
    return fail(NIMBLE_ERR_NULL, "null shape pointer");
  for (int i = 0; i < 2; ++i)
    if (pre_shape[i] < 0 || h_shape[i] < 0 || c_shape[i] < 0 || wh_shape[i] < 0)
      return fail(NIMBLE_ERR_ARG, "negative extent");
  const int64_t B = h_shape[0], H = h_shape[1];
  if (pre_shape[0] != B || c_shape[0] != B) return fail(NIMBLE_ERR_SHAPE, "lstm: batch extents differ");
  if (pre_shape[1] != 4 * H) return fail(NIMBLE_ERR_SHAPE, "lstm: pre is not (B,4H)");
  if (c_shape[1] != H) return fail(NIMBLE_ERR_SHAPE, "lstm: c is not (B,H)");
  if (wh_shape[0] != 4 * H || wh_shape[1] != H) return fail(NIMBLE_ERR_SHAPE, "lstm: w_h is not (4H,H)");
  h_out_shape[0] = c_out_shape[0] = B;
  h_out_shape[1] = c_out_shape[1] = H;
  return NIMBLE_OK;
}

int nimble_lstm_seq_shape(const int64_t* pre_shape, const int64_t* h0_shape, const int64_t* c0_shape,
                          const int64_t* wh_shape, int64_t* h_seq_shape, int64_t* c_out_shape) {
  clear_error();
  if (!pre_shape || !h0_shape || !c0_shape || !wh_shape || !h_seq_shape || !c_out_shape)
    return fail(NIMBLE_ERR_NULL, "null shape pointer");
  for (int i = 0; i < 3; ++i)
    if (pre_shape[i] < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  for (int i = 0; i < 2; ++i)
    if (h0_shape[i] < 0 || c0_shape[i] < 0 || wh_shape[i] < 0) return fail(NIMBLE_ERR_ARG, "negative extent");
  const int64_t T = pre_shape[0], B = h0_shape[0], H = h0_shape[1];
  if (pre_shape[1] != B || c0_shape[0] != B) return fail(NIMBLE_ERR_SHAPE, "lstm sequence: batch extents differ");
  if (pre_shape[2] != 4 * H) return fail(NIMBLE_ERR_SHAPE, "lstm sequence: pre is not (T,B,4H)");
  if (c0_shape[1] != H) return fail(NIMBLE_ERR_SHAPE, "lstm sequence: c0 is not (B,H)");
  if (wh_shape[0] != 4 * H || wh_shape[1] != H) return fail(NIMBLE_ERR_SHAPE, "lstm sequence: w_h is not (4H,H)");
  h_seq_shape[0] = T;
  h_seq_shape[1] = c_out_shape[0] = B;
  h_seq_shape[2] = c_out_shape[1] = H;
  return NIMBLE_OK;
}

int nimble_lstm_seq_supported(int64_t B, int64_t H) {
  return B >= 1 && B <= 4 && H >= 64 && H <= 1024 && (H % 64) == 0;
}

// Measured against a captured graph of per-step launches (microseconds per step at 1 / 2 / 4 rows):
// H = 512: 1.89 / 2.02 / 2.41 against 2.65-2.72; H = 1024: 2.71 / 3.20 / 3.98 against 2.85-2.95.
int nimble_lstm_seq_preferred(int64_t B, int64_t H) {
  return nimble_lstm_seq_supported(B, H) && (H <= 512 || B == 1);
}

size_t nimble_lstm_seq_workspace_bytes(int64_t B, int64_t H) {
  if (!nimble_lstm_seq_supported(B, H)) return 0;
  return 256 + 2 * (size_t)B * (size_t)H * 4;
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
  PlanOptions opt;
  opt.max_workspace = ~0ull;  // report the plan for a caller that provides what it asks for
  return plan_dense(1, M, N, K, epilogue, force_variant, opt, plan);
}

int nimble_dense_table_set(int64_t N, int64_t K, int epilogue, const nimble_table_entry* entries,
                           int count) {
  clear_error();
  if (N < 0 || K < 0 || count < 0) return fail(NIMBLE_ERR_ARG, "negative argument");
  if (epilogue < NIMBLE_EPI_NONE || epilogue > NIMBLE_EPI_BIAS_GELU_ERF)
    return fail(NIMBLE_ERR_ARG, "unknown epilogue %d", epilogue);
  const auto key = std::make_tuple(N, K, epilogue);
  if (count == 0) {
    g_tables.erase(key);
    return NIMBLE_OK;
  }
  if (!entries) return fail(NIMBLE_ERR_NULL, "null table");
  std::vector<nimble_table_entry> t;
  for (int i = 0; i < count; ++i) {
    const nimble_table_entry& e = entries[i];
    if (e.m_lo < 0 || e.m_hi < e.m_lo) return fail(NIMBLE_ERR_ARG, "entry %d: bad M range", i);
    if (e.variant < NIMBLE_VAR_SKINNY16 || e.variant >= NIMBLE_VAR_COUNT)
      return fail(NIMBLE_ERR_ARG, "entry %d: variant %d cannot be tabled", i, e.variant);
    if (e.split_k < 0 || e.split_k > 64) return fail(NIMBLE_ERR_ARG, "entry %d: bad split_k", i);
    if (e.variant == NIMBLE_VAR_SKINNY16 && e.m_hi > 64 && !stream_kernel_shape_ok(N, K))
      return fail(NIMBLE_ERR_ARG, "entry %d: skinny16 serves M <= 64 unless K is whole 64-wide stages", i);
    t.push_back(e);
  }
  g_tables[key] = t;
  return NIMBLE_OK;
}

int nimble_batch_matmul_plan(int64_t batch, int64_t M, int64_t N, int64_t K, int trans_b,
                             int out_dtype, nimble_plan* plan) {
  clear_error();
  if (!plan) return fail(NIMBLE_ERR_NULL, "null plan");
  if (dtype_size(out_dtype) == 0) return fail(NIMBLE_ERR_DTYPE, "unknown dtype %d", out_dtype);
  // batch_matmul is always one launch over all rows: no row split (its entry point launches the
  // plan as it stands), no K split (no reduction pass for batches), no tuned dense table
  PlanOptions bmm;
  bmm.allow_row_split = false;
  bmm.use_table = false;
  if (!trans_b) {
    // b is (T,K,N): its rows are not K-contiguous.  Where the tiled kernels could run the product
    // on b transposed (K a multiple of 8 and whole 16-byte batch strides), the plan is that NT
    // launch and its workspace is the transposed copy of b; the entry point falls back to the
    // bounds-checked kernel, which reads b strided, when the caller brings less.
    // (worth the extra launch from about 32 M multiply-adds: the bounds-checked kernel takes
    // 0.35 us per million, 4 us at config 4's L = 128 and 70 us at L = 512)
    if (K > 0 && K % 8 == 0 && ((M * K) & 7) == 0 && ((N * K) & 7) == 0 && batch > 0 && M > 0 && N > 0 &&
        (double)batch * (double)M * (double)N * (double)K >= 32e6) {
      int rc = plan_dense(batch, M, N, K, NIMBLE_EPI_NONE, NIMBLE_VAR_AUTO, bmm, plan);
      if (rc != NIMBLE_OK) return rc;
      if (plan->variant >= NIMBLE_VAR_T32x128) {
        plan->workspace_bytes = (uint64_t)batch * (uint64_t)N * (uint64_t)K * 2u;
        return NIMBLE_OK;
      }
    }
    return plan_dense(batch, M, N, K, NIMBLE_EPI_NONE, NIMBLE_VAR_GENERIC, bmm, plan);
  }
  return plan_dense(batch, M, N, K, NIMBLE_EPI_NONE, NIMBLE_VAR_AUTO, bmm, plan);
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
  // row blocks as for the weight-streaming dense (4H weight rows; measured at H = 512: 2 blocks
  // of 32 rows at B = 64 take 5.6 us against 7.9 us for one block of 64)
  const bool stream_ok = stream_kernel_shape_ok(4 * H, Ix + H) && Ix % 64 == 0;
  plan->grid[1] = (uint32_t)skinny_row_blocks(B, 4 * H, Ix + H, stream_ok);
  plan->grid[2] = 1;
  plan->block = 256;
  if (stream_ok && ceil_div(B, (int64_t)plan->grid[1]) <= 16) {  // the streaming kernel: 64-wide stages
    const bool many = (uint64_t)plan->grid[0] * plan->grid[1] > (uint64_t)kCUs &&
                      (double)(4 * H) * (double)(Ix + H) * 2.0 <= kCachedWeightBytes;
    plan->split_k = many ? 4 : 8;
    plan->bk = 64;
    plan->block = many ? 256 : 512;
  }
  return NIMBLE_OK;
}

const char* nimble_variant_name(int variant) {
  if (variant < 0 || variant >= NIMBLE_VAR_COUNT) return nullptr;
  return kVariants[variant].name;
}

const char* nimble_last_error(void) { return g_err; }

}  // extern "C"
