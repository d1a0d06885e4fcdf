/*
 * nimble.h - C ABI of the dynamic-shape dense / batch_matmul / LSTM-cell path
 * for AMD Instinct MI355X (gfx950).
 *
 * The call order is the one the paper prescribes for an operator whose leading
 * dimension is Any (Section 3.2, Section 3.3 and the listing of Appendix A):
 *
 *   1. the caller reads the run-time shapes of the inputs (host metadata),
 *   2. the caller runs the operator's shape function (nimble_*_shape, host,
 *      int64) which yields the output shape and performs the type check that
 *      could not be done while the dimension was unknown,
 *   3. the caller allocates the output from that shape (nimble_storage_bytes),
 *   4. the caller invokes the operator with inputs AND outputs passed
 *      explicitly (the invoke_mut convention); inside, a dispatch function
 *      picks one pre-built kernel from the run-time M and its residue
 *      M mod tile (Section 3.5) and launches it.
 *
 * Conventions for every nimble_*_dyn entry point
 *   - all tensor pointers are DEVICE pointers owned by the caller, row-major,
 *     contiguous, 16-byte aligned (NIMBLE_ERR_ALIGN otherwise);
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream);
 *     the call enqueues work and returns, it never synchronises, allocates or
 *     frees; `workspace` is caller-owned device scratch of `workspace_bytes`
 *     (query the need with the matching nimble_*_plan; may be NULL when 0);
 *   - return value: NIMBLE_OK (0) or a negative nimble_status; on any error
 *     nothing is launched and outputs are untouched; nimble_last_error()
 *     returns a thread-local description;
 *   - an extent of 0 for the dynamic dimension (or batch) is a legal
 *     instantiation of Any: NIMBLE_OK, nothing launched;
 *   - bf16 = bfloat16 bit patterns (uint16), f32 = IEEE binary32.
 */
#ifndef NIMBLE_H_
#define NIMBLE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum nimble_status {
  NIMBLE_OK = 0,
  NIMBLE_ERR_NULL = -1,      /* a required pointer is NULL                              */
  NIMBLE_ERR_RANK = -2,      /* an input has the wrong rank                             */
  NIMBLE_ERR_SHAPE = -3,     /* run-time type-relation violation (Section 3.1, 3.2)     */
  NIMBLE_ERR_DTYPE = -4,     /* unknown dtype selector                                  */
  NIMBLE_ERR_ALIGN = -5,     /* a device pointer is not 16-byte aligned                 */
  NIMBLE_ERR_WORKSPACE = -6, /* workspace smaller than the plan requires                */
  NIMBLE_ERR_HIP = -7,       /* the HIP runtime refused the launch                      */
  NIMBLE_ERR_ARG = -8        /* negative extent, unknown epilogue or variant, overflow  */
} nimble_status;

/* Epilogue fused into the dense kernel (the shape function of the fused
 * operator is the dense one: element-wise ops are data independent, Section 3.2). */
typedef enum nimble_epilogue {
  NIMBLE_EPI_NONE = 0,          /* y = x.w^T                                     */
  NIMBLE_EPI_BIAS = 1,          /* y = x.w^T + b                                 */
  NIMBLE_EPI_BIAS_GELU_ERF = 2  /* y = gelu(x.w^T + b), gelu(v)=v/2 (1+erf(v/sqrt 2)) */
} nimble_epilogue;

typedef enum nimble_dtype { NIMBLE_BF16 = 0, NIMBLE_F32 = 1 } nimble_dtype;

/* The kernel family the dispatch function chooses from.  Every tiled variant
 * exists in two copies: one compiled for residue r = 0 (no bounds code at
 * all) and one for r != 0 (the last tile along M is clamped and masked).  When
 * it pays, the dispatch function instead splits the call in two launches: whole
 * tile rows (all k of them, or as many as fill whole rounds of the chip) go to
 * the r = 0 copy, and the remaining rows, residue included, to the variant that
 * suits their number (see nimble_plan.split_rows). */
typedef enum nimble_variant {
  NIMBLE_VAR_AUTO = -1,
  NIMBLE_VAR_GENERIC = 0,    /* any M,N,K; fully bounds checked, scalar FMA       */
  NIMBLE_VAR_SKINNY16 = 1,   /* M tile 16: weights streamed from HBM once         */
  NIMBLE_VAR_T32x128 = 2,    /* LDS-tiled MFMA, 32 x 128 macro tile               */
  NIMBLE_VAR_T64x128 = 3,
  NIMBLE_VAR_T128x128 = 4,
  NIMBLE_VAR_T256x128 = 5,
  NIMBLE_VAR_T256x256 = 6,
  NIMBLE_VAR_COUNT = 7
} nimble_variant;

/* A forced variant may also force the K split: force_variant = variant | NIMBLE_FORCE_SPLIT_K(n)
 * cuts K into n slices (tiled variants; needs n*M*N*4 bytes of workspace). */
#define NIMBLE_FORCE_SPLIT_K(n) (((n) & 0xff) << 8)
/* ... and the tile height: the 256 x 256 variant is also built with tiles of 128, 160, 192 and
 * 224 rows (N a multiple of 256, K of 32).  With the run-time M known the dispatch function picks
 * the height at which the tile rows fill whole rounds of the 256 compute units, instead of
 * paying a mostly empty last round: the residue handling of Section 3.5 applied one level up. */
#define NIMBLE_FORCE_TILE_ROWS(rows) ((((rows) / 16) & 0xff) << 16)

/* What the dispatch function decided for one run-time shape (host only). */
typedef struct nimble_plan {
  int32_t variant;        /* nimble_variant                                       */
  int32_t bm, bn, bk;     /* macro tile of the launch (bm may be a reduced height)  */
  int64_t k;              /* floor(M / bm): number of full tiles along M          */
  int32_t r;              /* M mod bm: the residue the kernel copy is chosen by   */
  int32_t residue_copy;   /* 1 when the r != 0 copy (or an N/K edge) is launched  */
  int32_t split_k;        /* K is cut into this many slices (1 = none); with > 1  */
                          /* the slices write f32 partial sums to the workspace   */
                          /* and a second kernel adds them and applies the epilogue */
  uint32_t grid[3];       /* launch grid                                          */
  uint32_t block;         /* threads per workgroup                                */
  uint64_t workspace_bytes; /* device scratch the launch needs                    */
  int64_t split_rows;     /* > 0: two launches.  Rows [0, split_rows), a whole number  */
                          /* of tiles (at most k*bm), run the r = 0 copy of `variant`; */
  int32_t residue_variant;/* the remaining rows run this variant in a second launch    */
  int32_t residue_split_k;/* ... with K cut into this many slices (workspace_bytes is   */
                          /* the larger need of the two launches)                      */
} nimble_plan;

/* ----------------------------------------------------------------------------
 * Host-only integer functions (no device access, no HIP call).
 * -------------------------------------------------------------------------- */

/* Shape function of dense, data-independent mode (Section 3.2): x is (M,K),
 * w is (N,K); writes out_shape[0..1] = (M,N).  NIMBLE_ERR_RANK unless both
 * ranks are 2, NIMBLE_ERR_ARG on a negative extent, NIMBLE_ERR_SHAPE when the
 * two K differ.  out_shape is written only on success. */
int nimble_dense_shape(const int64_t* x_shape, int x_rank, const int64_t* w_shape, int w_rank,
                       int64_t* out_shape);

/* Shape function of batch_matmul: a is (T,M,K); b is (T,N,K) when trans_b != 0,
 * else (T,K,N); writes out_shape[0..2] = (T,M,N).  Batch and K must agree
 * (NIMBLE_ERR_SHAPE).  Two dynamic extents that are the same symbol (the
 * sequence length of attention) are simply equal numbers here (Section 3.1). */
int nimble_batch_matmul_shape(const int64_t* a_shape, int a_rank, const int64_t* b_shape,
                              int b_rank, int trans_b, int64_t* out_shape);

/* Shape function of the fused LSTM cell: x (B,Ix), h (B,H), c (B,H),
 * w (4H, Ix+H) -> h_out (B,H), c_out (B,H); all ranks 2. */
int nimble_lstm_shape(const int64_t* x_shape, const int64_t* h_shape, const int64_t* c_shape,
                      const int64_t* w_shape, int64_t* h_out_shape, int64_t* c_out_shape);

/* Shape function of the LSTM cell whose input share of the gates was computed beforehand
 * (nimble_lstm_gates_pre_dyn): pre (B,4H), h (B,H), c (B,H), w_h (4H,H) -> h_out (B,H),
 * c_out (B,H); all ranks 2.  Performs the run-time type check of that operator (Section 3.2):
 * NIMBLE_ERR_SHAPE when the extents do not fit each other. */
int nimble_lstm_pre_shape(const int64_t* pre_shape, const int64_t* h_shape, const int64_t* c_shape,
                          const int64_t* wh_shape, int64_t* h_out_shape, int64_t* c_out_shape);

/* Bytes of backing storage of a tensor (Section 3.3: alloc_storage(size,
 * alignment, device)): product of extents times the element size of `dtype`.
 * Returns the byte count, or a negative nimble_status. */
int64_t nimble_storage_bytes(const int64_t* shape, int rank, int dtype);

/* Alignment, in bytes, the paper's alloc_storage examples request (64). */
int64_t nimble_storage_alignment(void);

/* Residue split of a symbolic extent (Section 3.5): x = tile*k + r,
 * k = floor(x/tile), 0 <= r < tile. */
int nimble_residue_split(int64_t x, int64_t tile, int64_t* k, int64_t* r);

/* The dispatch function of dense (Section 3.5), host part: from the run-time
 * (M,N,K) pick the variant, its residue copy, the split of K and the grid.
 * `force_variant` = NIMBLE_VAR_AUTO lets the table decide; any other value
 * requests that variant (NIMBLE_ERR_ARG if it cannot run this shape). */
int nimble_dense_plan(int64_t M, int64_t N, int64_t K, int epilogue, int out_dtype,
                      int force_variant, nimble_plan* plan);

/* Tuned dispatch table (Section 3.5, tuning for symbolic shapes: measure the candidate
 * configurations offline on a grid of M and keep the best).  An entry overrides the built-in
 * cost model for dense calls with the given (N, K, epilogue) and m_lo <= M <= m_hi: the call
 * runs `variant` with K cut into `split_k` slices (1 = no cut) as one launch.  Entries that
 * cannot run (workspace too small for the cut, K not a multiple of 8) are skipped at dispatch.
 * `count` = 0 removes the table of that (N, K, epilogue).  Host only; not thread safe against
 * concurrent dispatch.  Returns NIMBLE_OK or NIMBLE_ERR_ARG / NIMBLE_ERR_NULL. */
typedef struct nimble_table_entry {
  int64_t m_lo, m_hi;
  int32_t variant, split_k;
} nimble_table_entry;
int nimble_dense_table_set(int64_t N, int64_t K, int epilogue, const nimble_table_entry* entries,
                           int count);

/* Same for one batch_matmul (grid z = batch). */
int nimble_batch_matmul_plan(int64_t batch, int64_t M, int64_t N, int64_t K, int trans_b,
                             int out_dtype, nimble_plan* plan);

/* Same for the fused LSTM cell. */
int nimble_lstm_plan(int64_t B, int64_t Ix, int64_t H, nimble_plan* plan);

/* Name of a variant ("skinny16", "t256x128", ...), NULL if out of range. */
const char* nimble_variant_name(int variant);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char* nimble_last_error(void);

/* ----------------------------------------------------------------------------
 * Device entry points (Section 3.5 kernels behind the dispatch function).
 * -------------------------------------------------------------------------- */

/* dense with dynamic M:  y[m,n] = epi( sum_k x[m,k] * w[n,k] + bias[n] ).
 * x [M,K] bf16, w [N,K] bf16, bias [N] bf16 (may be NULL for NIMBLE_EPI_NONE),
 * y [M,N] of out_dtype.  Accumulation and epilogue in f32.  The run-time type
 * check of the shape function is repeated (NIMBLE_ERR_SHAPE is impossible
 * here since one K is passed; negative extents give NIMBLE_ERR_ARG).  The dispatch function
 * (Section 3.5) picks the kernel from the run-time M; it plans within `workspace_bytes` (no
 * scratch: no K split). */
int nimble_dense_dyn(const void* x, const void* w, const void* bias, void* y, int64_t M, int64_t N,
                     int64_t K, int epilogue, int out_dtype, void* workspace, size_t workspace_bytes,
                     void* stream);

/* nimble_dense_dyn for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same operation, same
 * dispatch, same kernels and the same result bit for bit as nimble_dense_dyn called with the
 * workspace its plan asks for; the K-split partial sums go to a scratch array built into the
 * library (NIMBLE_NOALLOC_SCRATCH_BYTES of device memory per GPU, held from the time the
 * library's code is loaded on that GPU until the process ends).  The call allocates and frees
 * nothing.  A shape whose plan (nimble_dense_plan) needs more scratch than that is refused with
 * NIMBLE_ERR_WORKSPACE and nothing is launched.  All calls on one GPU share that GPU's scratch:
 * calls that may overlap (different streams, different host threads) race on it and must use
 * nimble_dense_dyn with workspaces of their own instead; calls on one stream are ordered and safe.
 * Nothing in the scratch carries over between calls. */
#define NIMBLE_NOALLOC_SCRATCH_BYTES (32u << 20)
int nimble_dense_noalloc_dyn(const void* x, const void* w, const void* bias, void* y, int64_t M,
                             int64_t N, int64_t K, int epilogue, int out_dtype, void* stream);

/* batch_matmul with dynamic M (and N or K when they are the same symbol):
 *   trans_b != 0: c[t,m,n] = alpha * sum_k a[t,m,k] * b[t,n,k]
 *   trans_b == 0: c[t,m,n] = alpha * sum_k a[t,m,k] * b[t,k,n]
 * a, b bf16; c of out_dtype; f32 accumulation.  With trans_b == 0 the tiled kernels run on b
 * transposed into the workspace (nimble_batch_matmul_plan gives its size, batch*N*K*2 bytes,
 * when K is a multiple of 8 and a tile suits the shape); with less workspace than that, or none,
 * a bounds-checked kernel reads b as it is. */
int nimble_batch_matmul_dyn(const void* a, const void* b, void* c, int64_t batch, int64_t M,
                            int64_t N, int64_t K, int trans_b, float alpha, int out_dtype,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Row softmax between the two attention batch_matmuls: s [rows, cols] f32 ->
 * p [rows, cols] bf16, p_j = exp(s_j - max s) / sum_j exp(s_j - max s), f32 math. */
int nimble_softmax_rows_dyn(const void* s_f32, void* p_bf16, int64_t rows, int64_t cols,
                            void* stream);

/* The attention chain S = alpha q.k^T, P = softmax rows of S, O = P.v fused into one launch
 * (the fused operator's shape function is the composition of the two batch_matmul shape
 * functions, Section 3.2; both dynamic extents are the same symbol L, Section 3.1):
 *   o[t,i,:] = sum_j softmax_j(alpha * q[t,i,:].k[t,j,:]) * v[t,j,:]
 * q, k, v, o are [heads, L, D] bf16; scores and the softmax in f32, P rounded to bf16 before
 * P.v, f32 accumulation.  Built for D = 64 and alpha > 0 (NIMBLE_ERR_ARG otherwise: use the three calls). */
int nimble_attention_dyn(const void* q, const void* k, const void* v, void* o, int64_t heads,
                         int64_t L, int64_t D, float alpha, void* stream);

/* Fused LSTM cell with dynamic batch B (gate blocks of w and bias in the order
 * i, f, g, o, H rows each):
 *   G = [x | h_prev] . w^T + bias;  c_out = sig(f) c_prev + sig(i) tanh(g);
 *   h_out = sig(o) tanh(c_out).
 * x [B,Ix] bf16, h_prev [B,H] bf16, w [4H, Ix+H] bf16, bias [4H] bf16,
 * c_prev [B,H] f32, c_out [B,H] f32 (may alias c_prev), h_out [B,H] bf16 (must
 * not alias h_prev).  Ix and H must be multiples of 8.  w is read in its natural layout: the
 * kernel gathers the four gate rows of a hidden unit itself, so there is no weight-packing pass
 * (and no entry point for one). */
int nimble_lstm_gates_dyn(const void* x, const void* h_prev, const void* w, const void* bias,
                          const void* c_prev, void* c_out, void* h_out, int64_t B, int64_t Ix,
                          int64_t H, void* workspace, size_t workspace_bytes, void* stream);

/* The same cell when the inputs' share of the gates has been computed for every token of the
 * sequence in one dense call (the evaluation section's remark that the inputs' matrix
 * multiplication can be batched along the sequence: x_all [T*B, Ix] . w_x^T + bias with f32
 * output, M = T*B dynamic): per token only the recurrent half of the weight is streamed.
 *   G = pre + h_prev . w_h^T;  cell update as above.
 * pre [B,4H] f32 (bias already added; gate blocks i, f, g, o), h_prev [B,H] bf16,
 * w_h [4H,H] bf16 (the recurrent columns of the fused weight, contiguous), c_prev / c_out
 * [B,H] f32 (may alias), h_out [B,H] bf16 (must not alias h_prev).  H a multiple of 8. */
int nimble_lstm_gates_pre_dyn(const void* pre, const void* h_prev, const void* w_h,
                              const void* c_prev, void* c_out, void* h_out, int64_t B, int64_t H,
                              void* stream);

/* ---- the token loop of a sequence in one launch ----------------------------------------
 * The evaluation section's LSTM remark (a cell step cannot fill the GPU, so the loop over tokens
 * is bound by what separates the steps): T steps of nimble_lstm_gates_pre_dyn in a single launch,
 * the recurrent weights held on chip, h_t handed from step to step through memory.
 *
 * Shape function: pre (T,B,4H), h0 (B,H), c0 (B,H), w_h (4H,H) -> h_seq (T,B,H), c_out (B,H);
 * NIMBLE_ERR_SHAPE when the extents do not fit each other, NIMBLE_ERR_ARG on a negative extent. */
int nimble_lstm_seq_shape(const int64_t* pre_shape, const int64_t* h0_shape, const int64_t* c0_shape,
                          const int64_t* wh_shape, int64_t* h_seq_shape, int64_t* c_out_shape);

/* 1 when nimble_lstm_seq_pre_dyn runs (B, H): 1 <= B <= 4, H a multiple of 64, 64 <= H <= 1024
 * (H/16 workgroups of 64 gate rows, all resident at once); else 0: run the steps one by one. */
int nimble_lstm_seq_supported(int64_t B, int64_t H);

/* 1 when, besides, the one launch measured faster than one launch per step (H <= 512, or one row up to
 * H = 1024: a step is then bound by what separates the steps; with more rows or a larger H by the words
 * every workgroup has to fetch per step); the hint a caller's dispatch takes. */
int nimble_lstm_seq_preferred(int64_t B, int64_t H);

/* Bytes of device workspace the call needs: 256 bytes of control words, then two (B,H) planes of
 * 32-bit words.  0 for shapes it does not run. */
size_t nimble_lstm_seq_workspace_bytes(int64_t B, int64_t H);

/* pre [T,B,4H] f32 (inputs' share of the gates, bias added; gate blocks i, f, g, o), w_h [4H,H] bf16,
 * h0 [B,H] bf16, c0 [B,H] f32 -> h_seq [T,B,H] bf16 (h_1 .. h_T), c_out [B,H] f32 (c_T; may alias c0).
 * Device pointers, 16-byte aligned; workspace of nimble_lstm_seq_workspace_bytes(B,H) bytes, owned by the
 * caller, used by one call at a time.  Two launches are enqueued on `stream` (a fill of the workspace, the
 * loop); the call does not wait for them.  Results are bit-identical to T calls of
 * nimble_lstm_gates_pre_dyn.
 * Every wait inside the kernel is bounded: a wave polls for the other workgroups' h_t at most
 * `max_polls` times per step (0: none at all, the loop gives up at its first wait), then sets the
 * give-up word and the whole grid leaves; h_seq and c_out are then unspecified.  The caller reads the word
 * with nimble_lstm_seq_status after the stream has finished and, if it is set, runs the steps one by one.
 * Errors: NIMBLE_ERR_SHAPE for (B,H) outside nimble_lstm_seq_supported, NIMBLE_ERR_ARG for T < 0,
 * NIMBLE_ERR_WORKSPACE, NIMBLE_ERR_NULL, NIMBLE_ERR_ALIGN; nothing is launched then.  T = 0 launches
 * nothing. */
int nimble_lstm_seq_pre_dyn(const void* pre, const void* w_h, const void* h0, const void* c0, void* h_seq,
                            void* c_out, int64_t T, int64_t B, int64_t H, void* workspace,
                            size_t workspace_bytes, uint32_t max_polls, void* stream);

/* Waits for `stream`, then copies the give-up word of `workspace` to the host:
 * *gave_up = 0: every step ran; 1: the loop gave up (see above).  NIMBLE_ERR_HIP if the copy fails. */
int nimble_lstm_seq_status(const void* workspace, void* stream, int* gave_up);

#ifdef __cplusplus
}
#endif
#endif /* NIMBLE_H_ */
