/*
 * CPU oracle for the dynamic-M dense / batch_matmul / LSTM-cell path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, by-the-definition
 * statement of what each operator computes.  It is used by the tests, by the
 * smoke check and by the benchmark's CPU-baseline leg, and by nothing else.
 * It shares no code with the HIP kernels or their host dispatcher.
 *
 * Precision: float32 storage and float32 arithmetic with sequential-k
 * accumulation (the paper's tensors are float32 throughout, Section 3.1 and
 * Section 3.3; the operands handed in are bfloat16 values already widened to
 * float32, so every product is exact in float32).  Compile with
 * -ffp-contract=off so no fused multiply-add changes the stated order.
 *
 * The method of the paper (Section 3.5: residue-specialised kernels chosen by
 * a dispatch function) reaches exactly the textbook result, so the oracle is
 * the textbook definition.  The integer side (Section 3.2 shape functions,
 * Section 3.3 storage sizes, Section 3.5 residue split) is written out as the
 * paper states it.
 *
 * Parallelism: OpenMP over output rows only; each output element is computed
 * by one thread in the stated order, so results do not depend on thread count.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define ORACLE_OK 0
#define ORACLE_ERR_RANK (-2)
#define ORACLE_ERR_SHAPE (-3)
#define ORACLE_ERR_ARG (-8)

/* epilogue selectors of oracle_dense */
#define ORACLE_EPI_NONE 0      /* y = x.w^T            */
#define ORACLE_EPI_BIAS 1      /* y = x.w^T + b        */
#define ORACLE_EPI_BIAS_GELU 2 /* y = gelu(x.w^T + b)  */

/* GELU in its exact (error-function) form: 0.5 x (1 + erf(x / sqrt 2)). */
float oracle_gelu1(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f)); }

void oracle_gelu(const float *x, float *y, int64_t n) {
  for (int64_t i = 0; i < n; ++i) y[i] = oracle_gelu1(x[i]);
}

static float sigmoid1(float z) { return 1.0f / (1.0f + expf(-z)); }

/*
 * dense: Y[m,n] = epi( sum_k X[m,k] * W[n,k] + b[n] ), X is [M,K], W is [N,K]
 * (output-features major, the layout of a TVM dense weight), Y is [M,N].
 * M is the dimension that is Any at compile time (Section 3.1).
 */
int oracle_dense(const float *x, const float *w, const float *b, float *y, int64_t M, int64_t N,
                 int64_t K, int epi) {
  if (M < 0 || N < 0 || K < 0) return ORACLE_ERR_ARG;
  if (epi < ORACLE_EPI_NONE || epi > ORACLE_EPI_BIAS_GELU) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    for (int64_t n = 0; n < N; ++n) {
      float acc = 0.0f;
      for (int64_t k = 0; k < K; ++k) acc += x[m * K + k] * w[n * K + k];
      if (epi != ORACLE_EPI_NONE) acc += b[n];
      if (epi == ORACLE_EPI_BIAS_GELU) acc = oracle_gelu1(acc);
      y[m * N + n] = acc;
    }
  }
  return ORACLE_OK;
}

/*
 * batch_matmul: C[t,m,n] = alpha * sum_k A[t,m,k] * Bm[t,n,k]   (trans_b = 1)
 *               C[t,m,n] = alpha * sum_k A[t,m,k] * Bm[t,k,n]   (trans_b = 0)
 */
int oracle_batch_matmul(const float *a, const float *bm, float *c, int64_t batch, int64_t M,
                        int64_t N, int64_t K, int trans_b, float alpha) {
  if (batch < 0 || M < 0 || N < 0 || K < 0) return ORACLE_ERR_ARG;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t t = 0; t < batch; ++t) {
    for (int64_t m = 0; m < M; ++m) {
      const float *at = a + t * M * K;
      const float *bt = bm + t * N * K;
      for (int64_t n = 0; n < N; ++n) {
        float acc = 0.0f;
        if (trans_b) {
          for (int64_t k = 0; k < K; ++k) acc += at[m * K + k] * bt[n * K + k];
        } else {
          for (int64_t k = 0; k < K; ++k) acc += at[m * K + k] * bt[k * N + n];
        }
        c[(t * M + m) * N + n] = alpha * acc;
      }
    }
  }
  return ORACLE_OK;
}

/* Row softmax: p_j = exp(s_j - max_j s) / sum_j exp(s_j - max_j s). */
int oracle_softmax_rows(const float *s, float *p, int64_t rows, int64_t cols) {
  if (rows < 0 || cols < 0) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    const float *sr = s + r * cols;
    float *pr = p + r * cols;
    float mx = -INFINITY;
    for (int64_t j = 0; j < cols; ++j) mx = sr[j] > mx ? sr[j] : mx;
    float sum = 0.0f;
    for (int64_t j = 0; j < cols; ++j) {
      pr[j] = expf(sr[j] - mx);
      sum += pr[j];
    }
    for (int64_t j = 0; j < cols; ++j) pr[j] = pr[j] / sum;
  }
  return ORACLE_OK;
}

/*
 * LSTM cell with one fused weight: G = [x | h] . W^T + b with W [4H, Ix+H] and
 * gate blocks in the order i, f, g, o (H rows each);
 *   c' = sigmoid(f) * c + sigmoid(i) * tanh(g),   h' = sigmoid(o) * tanh(c').
 * g_scratch is [B, 4H] and receives the pre-activation gates.
 */
int oracle_lstm_step(const float *x, const float *h, const float *w, const float *b,
                     const float *c, float *h_out, float *c_out, float *g_scratch, int64_t B,
                     int64_t Ix, int64_t H) {
  if (B < 0 || Ix < 0 || H < 0) return ORACLE_ERR_ARG;
  const int64_t K = Ix + H, N = 4 * H;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < B; ++m) {
    for (int64_t n = 0; n < N; ++n) {
      float acc = 0.0f;
      for (int64_t k = 0; k < Ix; ++k) acc += x[m * Ix + k] * w[n * K + k];
      for (int64_t k = 0; k < H; ++k) acc += h[m * H + k] * w[n * K + Ix + k];
      g_scratch[m * N + n] = acc + b[n];
    }
    for (int64_t j = 0; j < H; ++j) {
      const float gi = g_scratch[m * N + j];
      const float gf = g_scratch[m * N + H + j];
      const float gg = g_scratch[m * N + 2 * H + j];
      const float go = g_scratch[m * N + 3 * H + j];
      const float cn = sigmoid1(gf) * c[m * H + j] + sigmoid1(gi) * tanhf(gg);
      c_out[m * H + j] = cn;
      h_out[m * H + j] = sigmoid1(go) * tanhf(cn);
    }
  }
  return ORACLE_OK;
}

/*
 * The same cell with the input's share of the gates computed beforehand for every token of the
 * sequence in one product (the evaluation section's remark on batching the inputs' matrix
 * multiplication along the sequence):  pre = x . Wx^T + b  is given,  G = pre + h . Wh^T  with
 * Wh [4H, H] the recurrent columns of the fused weight; gate order and update as above.
 */
int oracle_lstm_step_pre(const float *pre, const float *h, const float *wh, const float *c,
                         float *h_out, float *c_out, float *g_scratch, int64_t B, int64_t H) {
  if (B < 0 || H < 0) return ORACLE_ERR_ARG;
  const int64_t N = 4 * H;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < B; ++m) {
    for (int64_t n = 0; n < N; ++n) {
      float acc = 0.0f;
      for (int64_t k = 0; k < H; ++k) acc += h[m * H + k] * wh[n * H + k];
      g_scratch[m * N + n] = pre[m * N + n] + acc;
    }
    for (int64_t j = 0; j < H; ++j) {
      const float gi = g_scratch[m * N + j];
      const float gf = g_scratch[m * N + H + j];
      const float gg = g_scratch[m * N + 2 * H + j];
      const float go = g_scratch[m * N + 3 * H + j];
      const float cn = sigmoid1(gf) * c[m * H + j] + sigmoid1(gi) * tanhf(gg);
      c_out[m * H + j] = cn;
      h_out[m * H + j] = sigmoid1(go) * tanhf(cn);
    }
  }
  return ORACLE_OK;
}

/* ------------------------------------------------------------------------
 * Integer side.
 * ---------------------------------------------------------------------- */

/*
 * Data-independent shape function of dense (Section 3.2): from the run-time
 * shapes (M,K) and (N,K) compute (M,N), and verify the type relation that
 * could not be checked while M was Any: both K must agree.
 */
int oracle_dense_shape(const int64_t *x_shape, int x_rank, const int64_t *w_shape, int w_rank,
                       int64_t *out_shape) {
  if (x_rank != 2 || w_rank != 2) return ORACLE_ERR_RANK;
  if (x_shape[0] < 0 || x_shape[1] < 0 || w_shape[0] < 0 || w_shape[1] < 0) return ORACLE_ERR_ARG;
  if (x_shape[1] != w_shape[1]) return ORACLE_ERR_SHAPE;
  out_shape[0] = x_shape[0];
  out_shape[1] = w_shape[0];
  return ORACLE_OK;
}

/* batch_matmul: (T,M,K) with (T,N,K) if trans_b else (T,K,N) -> (T,M,N). */
int oracle_batch_matmul_shape(const int64_t *a_shape, int a_rank, const int64_t *b_shape,
                              int b_rank, int trans_b, int64_t *out_shape) {
  if (a_rank != 3 || b_rank != 3) return ORACLE_ERR_RANK;
  for (int i = 0; i < 3; ++i)
    if (a_shape[i] < 0 || b_shape[i] < 0) return ORACLE_ERR_ARG;
  const int64_t kb = trans_b ? b_shape[2] : b_shape[1];
  const int64_t nb = trans_b ? b_shape[1] : b_shape[2];
  if (a_shape[0] != b_shape[0]) return ORACLE_ERR_SHAPE;
  if (a_shape[2] != kb) return ORACLE_ERR_SHAPE;
  out_shape[0] = a_shape[0];
  out_shape[1] = a_shape[1];
  out_shape[2] = nb;
  return ORACLE_OK;
}

/* LSTM cell: x (B,Ix), h (B,H), c (B,H), W (4H, Ix+H) -> h' (B,H), c' (B,H). */
int oracle_lstm_shape(const int64_t *x_shape, const int64_t *h_shape, const int64_t *c_shape,
                      const int64_t *w_shape, int64_t *h_out_shape, int64_t *c_out_shape) {
  for (int i = 0; i < 2; ++i)
    if (x_shape[i] < 0 || h_shape[i] < 0 || c_shape[i] < 0 || w_shape[i] < 0) return ORACLE_ERR_ARG;
  if (x_shape[0] != h_shape[0] || x_shape[0] != c_shape[0]) return ORACLE_ERR_SHAPE;
  if (h_shape[1] != c_shape[1]) return ORACLE_ERR_SHAPE;
  if (w_shape[0] != 4 * h_shape[1]) return ORACLE_ERR_SHAPE;
  if (w_shape[1] != x_shape[1] + h_shape[1]) return ORACLE_ERR_SHAPE;
  h_out_shape[0] = c_out_shape[0] = x_shape[0];
  h_out_shape[1] = c_out_shape[1] = h_shape[1];
  return ORACLE_OK;
}

/*
 * Bytes of backing storage for a tensor (Section 3.3): the element count
 * times the element size; `alignment` is the address alignment requested of
 * the allocator, it does not change the size.  Returns -1 on a bad argument.
 */
int64_t oracle_storage_bytes(const int64_t *shape, int rank, int64_t itemsize) {
  if (rank < 0 || itemsize <= 0) return -1;
  int64_t n = 1;
  for (int i = 0; i < rank; ++i) {
    if (shape[i] < 0) return -1;
    n *= shape[i];
  }
  return n * itemsize;
}

/*
 * Residue split of a symbolic extent tiled by `tile` (Section 3.5):
 * x = tile * k + r with k = floor(x / tile) and r in [0, tile-1]; the copy of
 * the kernel to dispatch to is the one compiled for residue r.
 */
int oracle_residue_split(int64_t x, int64_t tile, int64_t *k, int64_t *r) {
  if (x < 0 || tile <= 0) return ORACLE_ERR_ARG;
  *k = x / tile;
  *r = x - tile * (*k);
  return ORACLE_OK;
}
