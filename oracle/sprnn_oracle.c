/*
 * CPU oracle for the sparse recurrent step.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain definition of what the persistent sparse recurrent
 * kernel must compute, written out slowly and without any blocking, fusion or
 * reordering.  It shares no code with the HIP path and nothing in the product
 * may call it; only tests, the smoke check and the benchmark's CPU-baseline leg
 * use it.
 *
 * What it follows:
 *   - Vanilla cell: Eq. 2 of the paper, h_t = g(U_r h_{t-1} + b'), with b' (the
 *     input projection plus bias, Section 3.1) handed in as x[t].
 *   - The method of Sections 3.3 / 4 only re-orders a sparse dot product and
 *     pads it with zeros, so its result is the plain CSR row dot product; this
 *     file therefore evaluates each row in CSR order, left to right.
 *   - Input projection: Section 3.1 rewrites Eq. 1 as Eq. 2 by computing b' = W x_t + b for all
 *     timesteps ahead of the recurrence; oracle_input_projection_f64 is that dense product, one
 *     row of W against one input vector at a time, summed left to right in binary64.
 *   - LSTM cell: Appendix B says only that every hidden unit has four gate rows
 *     with different activations; the standard cell without peepholes is used
 *     (gate row blocks i | f | g | o):
 *         c_t = sigmoid(p_f) * c_{t-1} + sigmoid(p_i) * tanh(p_g)
 *         h_t = sigmoid(p_o) * tanh(c_t)
 *     with p_* = W_* h_{t-1} + x_*[t].
 *
 *   - GRU cell: the paper names gated recurrent units as a cell its approach extends to and gives no
 *     equations; the formulation of the libraries it compares with is used (three gate rows per hidden
 *     unit, row blocks r | z | n, the recurrent bias of the candidate inside the reset product):
 *         r = sigmoid(p_r),  z = sigmoid(p_z),  n = tanh(x_n[t] + r * (U_n h_{t-1} + b_hn))
 *         h_t = (1 - z) * n + z * h_{t-1}
 *     with p_r = U_r h_{t-1} + x_r[t], p_z = U_z h_{t-1} + x_z[t]; x carries the input projection and
 *     every bias except b_hn.
 *
 *   - Backward pass through time of the vanilla cell (Appendix B.1 trains with the pruned weights in both
 *     passes): for L = sum_t <e_t, h_t> with e_t = dL/dh_t from outside,
 *         d_t = e_t + U_r^T delta_{t+1},  delta_t = g'(a_t) * d_t  (= dL/db'_t),  delta_{T+1} = 0,
 *         dL/dh_0 = U_r^T delta_1,  dL/dU_r[i][j] = sum_t sum_b delta_t[b][i] h_{t-1}[b][j]  on the pattern,
 *     with g' taken from the forward output (ReLU: h_t > 0; tanh: 1 - h_t^2; identity: 1).  Binary64.
 *
 *   - Backward pass through time of the LSTM cell above, for L = sum_t <e_t, h_t>: the chain rule applied to the
 *     two cell equations, with the gate values i, f, g, o (after their activations), c_t and h_t kept from the
 *     forward pass.  Going from t = T down to 1, with dc_{T+1} f_{T+1} = 0 and U^T dp_{T+1} = 0:
 *         dh_t = e_t + U^T dp_{t+1}                      (U is [4H][H]; dp are the gradients of the four p blocks)
 *         dc_t = dc_{t+1} f_{t+1} + dh_t o_t (1 - tanh(c_t)^2)
 *         dp_i = dc_t g_t i_t (1 - i_t),   dp_f = dc_t c_{t-1} f_t (1 - f_t),
 *         dp_g = dc_t i_t (1 - g_t^2),     dp_o = dh_t tanh(c_t) o_t (1 - o_t)
 *     dp_t = dL/db'_t; dL/dh_0 = U^T dp_1; dL/dc_0 = dc_1 f_1; dL/dU[r][k] = sum_t sum_b dp_t[b][r] h_{t-1}[b][k].
 *
 *   - Backward pass through time of the GRU cell above, for L = sum_t <e_t, h_t>: the chain rule on its equations, with
 *     r, z, n and q = U_n h_{t-1} + b_hn kept from the forward pass.  Going from t = T down to 1, with everything
 *     beyond T zero and v_t = (dp_r | dp_z | dq) the gradient of the three recurrent sums:
 *         dh_t = e_t + dh_{t+1} z_{t+1} + U^T v_{t+1}            (U is [3H][H])
 *         da = dh_t (1 - z_t) (1 - n_t^2)        (gradient of the candidate's pre-activation = dL/dx_n)
 *         dp_r = da q_t r_t (1 - r_t),   dp_z = dh_t (h_{t-1} - n_t) z_t (1 - z_t),   dq = da r_t
 *     dL/db'_t = (dp_r | dp_z | da); dL/dh_0 = dh_1 z_1 + U^T v_1; dL/dU[r][k] = sum_t sum_b v_t[b][r] h_{t-1}[b][k];
 *     dL/db_hn[j] = sum_t sum_b dq_t[b][j].
 *
 * Precision: weights are IEEE binary16 bit patterns decoded exactly to binary32
 * (Section 6 names 16-bit weights as the compressed format); activations, the
 * products and the running sums are binary32 (one rounding per multiply and per
 * add: build with -ffp-contract=off); activation functions are evaluated with
 * the C library's single-precision routines.  The *_f64 twins do every
 * operation in binary64 and keep the state in binary64; they bound the
 * rounding error of the binary32 versions.
 *
 * Pins (tests/test_oracle_pins.py): exhaustive binary16 decode against numpy,
 * dense special case against a float64 matrix product and against
 * torch.nn.RNNCell / LSTMCell, identity and permutation closed forms (bit
 * exact), all-zero weights, exact rational brute force on tiny sizes,
 * homogeneity / batch-independence / time-composition invariants, and a
 * hand-worked integer example under tests/golden/.  Input projection: float64 matrix product of
 * numpy, identity and single-entry closed forms (bit exact), exact rational brute force, a
 * hand-worked non-square example with a bias under tests/golden/, and sensitivity checks against a
 * transposed operand and a dropped bias.  GRU: torch.nn.GRUCell on dense weights, closed forms (update
 * gate saturated either way, zero weights), batch independence and time composition.  Backward pass:
 * torch autograd on the dense cell (dL/db', dL/dh_0, dL/dU on and off the pattern), finite differences, T = 1
 * closed form.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_ACT_RELU 0
#define ORACLE_ACT_TANH 1
#define ORACLE_ACT_IDENTITY 2

/* Exact decode of an IEEE 754 binary16 bit pattern (subnormals, infinities and NaNs included). */
float oracle_half_bits_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h >> 15) & 1u;
  const uint32_t expo = (uint32_t)(h >> 10) & 0x1Fu;
  const uint32_t frac = (uint32_t)h & 0x3FFu;
  float mag;
  if (expo == 0u) {
    mag = ldexpf((float)frac, -24); /* zero or subnormal: frac * 2^-24 */
  } else if (expo == 31u) {
    mag = frac ? NAN : INFINITY;
  } else {
    mag = ldexpf((float)(1024u + frac), (int)expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
  }
  return sign ? -mag : mag;
}

static float act_f32(int act, float pre) {
  switch (act) {
    case ORACLE_ACT_RELU: return (pre > 0.0f) ? pre : 0.0f;
    case ORACLE_ACT_TANH: return tanhf(pre);
    default: return pre;
  }
}

static double act_f64(int act, double pre) {
  switch (act) {
    case ORACLE_ACT_RELU: return (pre > 0.0) ? pre : 0.0;
    case ORACLE_ACT_TANH: return tanh(pre);
    default: return pre;
  }
}

static float sigmoid_f32(float z) { return 1.0f / (1.0f + expf(-z)); }
static double sigmoid_f64(double z) { return 1.0 / (1.0 + exp(-z)); }

/*
 * Vanilla cell, Eq. 2.  x is [T][B][H], h0 is [B][H] or NULL (zeros), h_out is [T][B][H].
 * threads > 1 splits the rows of one timestep over OpenMP threads (timesteps stay sequential).
 * Returns 0, or -1 on a malformed argument.
 */
int oracle_rnn_forward(int H, int B, int T, int act, const int32_t* row_ptr, const int32_t* col_idx,
                       const uint16_t* val_bits, const float* x, const float* h0, float* h_out, int threads) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !x || !h_out) return -1;
  float* zeros = (float*)calloc((size_t)B * H, sizeof(float));
  if (!zeros) return -1;
  for (int t = 0; t < T; ++t) {
    const float* h_prev = (t == 0) ? (h0 ? h0 : zeros) : h_out + (size_t)(t - 1) * B * H;
    float* h_cur = h_out + (size_t)t * B * H;
    const float* x_t = x + (size_t)t * B * H;
#pragma omp parallel for num_threads(threads) if (threads > 1) schedule(static)
    for (int i = 0; i < H; ++i) {
      for (int b = 0; b < B; ++b) {
        float acc = 0.0f;
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
          const float w = oracle_half_bits_to_float(val_bits[k]);
          const float prod = w * h_prev[(size_t)b * H + col_idx[k]];
          acc = acc + prod;
        }
        const float pre = acc + x_t[(size_t)b * H + i];
        h_cur[(size_t)b * H + i] = act_f32(act, pre);
      }
    }
  }
  free(zeros);
  return 0;
}

/* Binary64 twin of oracle_rnn_forward: same inputs, state and outputs in double. */
int oracle_rnn_forward_f64(int H, int B, int T, int act, const int32_t* row_ptr, const int32_t* col_idx,
                           const uint16_t* val_bits, const float* x, const float* h0, double* h_out, int threads) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !x || !h_out) return -1;
  double* first = (double*)calloc((size_t)B * H, sizeof(double));
  if (!first) return -1;
  if (h0) for (size_t j = 0; j < (size_t)B * H; ++j) first[j] = (double)h0[j];
  for (int t = 0; t < T; ++t) {
    const double* h_prev = (t == 0) ? first : h_out + (size_t)(t - 1) * B * H;
    double* h_cur = h_out + (size_t)t * B * H;
    const float* x_t = x + (size_t)t * B * H;
#pragma omp parallel for num_threads(threads) if (threads > 1) schedule(static)
    for (int i = 0; i < H; ++i) {
      for (int b = 0; b < B; ++b) {
        double acc = 0.0;
        for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
          acc += (double)oracle_half_bits_to_float(val_bits[k]) * h_prev[(size_t)b * H + col_idx[k]];
        }
        h_cur[(size_t)b * H + i] = act_f64(act, acc + (double)x_t[(size_t)b * H + i]);
      }
    }
  }
  free(first);
  return 0;
}

/*
 * LSTM cell.  W is [4H][H] in CSR with row blocks i | f | g | o; x is [T][B][4H] in the same block
 * order; h0, c0 are [B][H] or NULL (zeros); h_out, c_out are [T][B][H].
 */
static int lstm_forward_f32(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                            const uint16_t* val_bits, const float* x, const float* h0, const float* c0,
                            float* h_out, float* c_out, float* gates_out, int threads) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !x || !h_out || !c_out) return -1;
  float* zeros = (float*)calloc((size_t)B * H, sizeof(float));
  if (!zeros) return -1;
  for (int t = 0; t < T; ++t) {
    const float* h_prev = (t == 0) ? (h0 ? h0 : zeros) : h_out + (size_t)(t - 1) * B * H;
    const float* c_prev = (t == 0) ? (c0 ? c0 : zeros) : c_out + (size_t)(t - 1) * B * H;
    float* h_cur = h_out + (size_t)t * B * H;
    float* c_cur = c_out + (size_t)t * B * H;
    const float* x_t = x + (size_t)t * B * 4 * H;
#pragma omp parallel for num_threads(threads) if (threads > 1) schedule(static)
    for (int j = 0; j < H; ++j) {
      for (int b = 0; b < B; ++b) {
        float p[4];
        for (int g = 0; g < 4; ++g) {
          const int row = g * H + j;
          float acc = 0.0f;
          for (int32_t k = row_ptr[row]; k < row_ptr[row + 1]; ++k) {
            const float w = oracle_half_bits_to_float(val_bits[k]);
            const float prod = w * h_prev[(size_t)b * H + col_idx[k]];
            acc = acc + prod;
          }
          p[g] = acc + x_t[(size_t)b * 4 * H + row];
        }
        const float gi = sigmoid_f32(p[0]);
        const float gf = sigmoid_f32(p[1]);
        const float gg = tanhf(p[2]);
        const float go = sigmoid_f32(p[3]);
        const float keep = gf * c_prev[(size_t)b * H + j];
        const float add = gi * gg;
        const float c = keep + add;
        if (gates_out) {
          float* q = gates_out + ((size_t)t * B + b) * 4 * H + j;
          q[0] = gi; q[(size_t)H] = gf; q[(size_t)2 * H] = gg; q[(size_t)3 * H] = go;
        }
        c_cur[(size_t)b * H + j] = c;
        h_cur[(size_t)b * H + j] = go * tanhf(c);
      }
    }
  }
  free(zeros);
  return 0;
}

int oracle_lstm_forward(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                        const uint16_t* val_bits, const float* x, const float* h0, const float* c0,
                        float* h_out, float* c_out, int threads) {
  return lstm_forward_f32(H, B, T, row_ptr, col_idx, val_bits, x, h0, c0, h_out, c_out, NULL, threads);
}

/* The same forward pass, also keeping what a backward pass needs: gates_out is [T][B][4H], the gate values after
 * their activations (blocks sigmoid(p_i) | sigmoid(p_f) | tanh(p_g) | sigmoid(p_o)). */
int oracle_lstm_forward_saved(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                              const uint16_t* val_bits, const float* x, const float* h0, const float* c0,
                              float* h_out, float* c_out, float* gates_out, int threads) {
  if (!gates_out) return -1;
  return lstm_forward_f32(H, B, T, row_ptr, col_idx, val_bits, x, h0, c0, h_out, c_out, gates_out, threads);
}

/* Binary64 twin of oracle_lstm_forward. */
int oracle_lstm_forward_f64(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                            const uint16_t* val_bits, const float* x, const float* h0, const float* c0,
                            double* h_out, double* c_out, int threads) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !x || !h_out || !c_out) return -1;
  double* hfirst = (double*)calloc((size_t)B * H, sizeof(double));
  double* cfirst = (double*)calloc((size_t)B * H, sizeof(double));
  if (!hfirst || !cfirst) { free(hfirst); free(cfirst); return -1; }
  if (h0) for (size_t j = 0; j < (size_t)B * H; ++j) hfirst[j] = (double)h0[j];
  if (c0) for (size_t j = 0; j < (size_t)B * H; ++j) cfirst[j] = (double)c0[j];
  for (int t = 0; t < T; ++t) {
    const double* h_prev = (t == 0) ? hfirst : h_out + (size_t)(t - 1) * B * H;
    const double* c_prev = (t == 0) ? cfirst : c_out + (size_t)(t - 1) * B * H;
    double* h_cur = h_out + (size_t)t * B * H;
    double* c_cur = c_out + (size_t)t * B * H;
    const float* x_t = x + (size_t)t * B * 4 * H;
#pragma omp parallel for num_threads(threads) if (threads > 1) schedule(static)
    for (int j = 0; j < H; ++j) {
      for (int b = 0; b < B; ++b) {
        double p[4];
        for (int g = 0; g < 4; ++g) {
          const int row = g * H + j;
          double acc = 0.0;
          for (int32_t k = row_ptr[row]; k < row_ptr[row + 1]; ++k) {
            acc += (double)oracle_half_bits_to_float(val_bits[k]) * h_prev[(size_t)b * H + col_idx[k]];
          }
          p[g] = acc + (double)x_t[(size_t)b * 4 * H + row];
        }
        const double c = sigmoid_f64(p[1]) * c_prev[(size_t)b * H + j] + sigmoid_f64(p[0]) * tanh(p[2]);
        c_cur[(size_t)b * H + j] = c;
        h_cur[(size_t)b * H + j] = sigmoid_f64(p[3]) * tanh(c);
      }
    }
  }
  free(hfirst);
  free(cfirst);
  return 0;
}

/*
 * Input projection b' = W x + b of Section 3.1 (Eq. 1 folded into Eq. 2) for M = T*B input vectors.
 * w_bits is the dense [R][I] input weight matrix as binary16 bit patterns (row r holds the weights of
 * output r), x is [M][I] float32, bias is [R] float32 or NULL (zeros), out is [M][R] binary64.
 * Products of a binary16 and a binary32 number are exact in binary64; the sum runs over k = 0..I-1 in
 * that order and the bias is added last.
 */
int oracle_input_projection_f64(int R, int I, int M, const uint16_t* w_bits, const float* x, const float* bias,
                                double* out, int threads) {
  if (R <= 0 || I <= 0 || M < 0 || !w_bits || !x || !out) return -1;
#pragma omp parallel for num_threads(threads) if (threads > 1) schedule(static)
  for (int m = 0; m < M; ++m) {
    for (int r = 0; r < R; ++r) {
      double acc = 0.0;
      for (int k = 0; k < I; ++k) {
        const double w = (double)oracle_half_bits_to_float(w_bits[(size_t)r * I + k]);
        acc += w * (double)x[(size_t)m * I + k];
      }
      out[(size_t)m * R + r] = acc + (bias ? (double)bias[r] : 0.0);
    }
  }
  return 0;
}

/*
 * GRU cell.  U is [3H][H] in CSR with row blocks r | z | n; x is [T][B][3H] in the same block order;
 * b_hn is [H] or NULL (zeros); h0 is [B][H] or NULL (zeros); h_out is [T][B][H].
 */
static int gru_forward_f32(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                           const uint16_t* val_bits, const float* x, const float* b_hn, const float* h0,
                           float* h_out, float* gates_out, int threads) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !x || !h_out) return -1;
  float* zeros = (float*)calloc((size_t)B * H, sizeof(float));
  if (!zeros) return -1;
  for (int t = 0; t < T; ++t) {
    const float* h_prev = (t == 0) ? (h0 ? h0 : zeros) : h_out + (size_t)(t - 1) * B * H;
    float* h_cur = h_out + (size_t)t * B * H;
    const float* x_t = x + (size_t)t * B * 3 * H;
#pragma omp parallel for num_threads(threads) if (threads > 1) schedule(static)
    for (int j = 0; j < H; ++j) {
      for (int b = 0; b < B; ++b) {
        float s[3];
        for (int g = 0; g < 3; ++g) {
          const int row = g * H + j;
          float acc = 0.0f;
          for (int32_t k = row_ptr[row]; k < row_ptr[row + 1]; ++k) {
            const float w = oracle_half_bits_to_float(val_bits[k]);
            const float prod = w * h_prev[(size_t)b * H + col_idx[k]];
            acc = acc + prod;
          }
          s[g] = acc;
        }
        const float r = sigmoid_f32(s[0] + x_t[(size_t)b * 3 * H + j]);
        const float z = sigmoid_f32(s[1] + x_t[(size_t)b * 3 * H + H + j]);
        const float q = s[2] + (b_hn ? b_hn[j] : 0.0f);
        const float rq = r * q;
        const float n = tanhf(x_t[(size_t)b * 3 * H + 2 * H + j] + rq);
        const float keep = z * h_prev[(size_t)b * H + j];
        const float fresh = (1.0f - z) * n;
        if (gates_out) {
          float* o = gates_out + ((size_t)t * B + b) * 4 * H + j;
          o[0] = r; o[(size_t)H] = z; o[(size_t)2 * H] = n; o[(size_t)3 * H] = q;
        }
        h_cur[(size_t)b * H + j] = fresh + keep;
      }
    }
  }
  free(zeros);
  return 0;
}

int oracle_gru_forward(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                       const uint16_t* val_bits, const float* x, const float* b_hn, const float* h0,
                       float* h_out, int threads) {
  return gru_forward_f32(H, B, T, row_ptr, col_idx, val_bits, x, b_hn, h0, h_out, NULL, threads);
}

/* The same forward pass, also keeping what a backward pass needs: gates_out is [T][B][4H], blocks r | z | n | q with
 * q = U_n h_{t-1} + b_hn (the factor the reset gate multiplies). */
int oracle_gru_forward_saved(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                             const uint16_t* val_bits, const float* x, const float* b_hn, const float* h0,
                             float* h_out, float* gates_out, int threads) {
  if (!gates_out) return -1;
  return gru_forward_f32(H, B, T, row_ptr, col_idx, val_bits, x, b_hn, h0, h_out, gates_out, threads);
}

/* Binary64 twin of oracle_gru_forward. */
int oracle_gru_forward_f64(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                           const uint16_t* val_bits, const float* x, const float* b_hn, const float* h0,
                           double* h_out, int threads) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !x || !h_out) return -1;
  double* first = (double*)calloc((size_t)B * H, sizeof(double));
  if (!first) return -1;
  if (h0) for (size_t j = 0; j < (size_t)B * H; ++j) first[j] = (double)h0[j];
  for (int t = 0; t < T; ++t) {
    const double* h_prev = (t == 0) ? first : h_out + (size_t)(t - 1) * B * H;
    double* h_cur = h_out + (size_t)t * B * H;
    const float* x_t = x + (size_t)t * B * 3 * H;
#pragma omp parallel for num_threads(threads) if (threads > 1) schedule(static)
    for (int j = 0; j < H; ++j) {
      for (int b = 0; b < B; ++b) {
        double s[3];
        for (int g = 0; g < 3; ++g) {
          const int row = g * H + j;
          double acc = 0.0;
          for (int32_t k = row_ptr[row]; k < row_ptr[row + 1]; ++k) {
            acc += (double)oracle_half_bits_to_float(val_bits[k]) * h_prev[(size_t)b * H + col_idx[k]];
          }
          s[g] = acc;
        }
        const double r = sigmoid_f64(s[0] + (double)x_t[(size_t)b * 3 * H + j]);
        const double z = sigmoid_f64(s[1] + (double)x_t[(size_t)b * 3 * H + H + j]);
        const double n = tanh((double)x_t[(size_t)b * 3 * H + 2 * H + j] + r * (s[2] + (b_hn ? (double)b_hn[j] : 0.0)));
        h_cur[(size_t)b * H + j] = (1.0 - z) * n + z * h_prev[(size_t)b * H + j];
      }
    }
  }
  free(first);
  return 0;
}

/*
 * Backward pass through time of the vanilla cell, binary64.  U is [H][H] in CSR (the forward matrix, not its
 * transpose); h_fwd is [T][B][H] (forward outputs h_1..h_T), h0 is [B][H] or NULL (zeros), dh_ext is
 * [T][B][H] (e_t).  Outputs: d_bprime [T][B][H] (delta_t), dh0 [B][H] (may be NULL), dU [nnz] in CSR order
 * (may be NULL).
 */
int oracle_rnn_backward_f64(int H, int B, int T, int act, const int32_t* row_ptr, const int32_t* col_idx,
                            const uint16_t* val_bits, const float* h_fwd, const float* h0, const float* dh_ext,
                            double* d_bprime, double* dh0, double* dU) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !d_bprime || (T > 0 && (!h_fwd || !dh_ext))) return -1;
  const int64_t nnz = row_ptr[H];
  double* back = (double*)calloc((size_t)B * H, sizeof(double)); /* U^T delta_{t+1}, per sample */
  if (!back) return -1;
  if (dU) for (int64_t k = 0; k < nnz; ++k) dU[k] = 0.0;
  for (int t = T - 1; t >= 0; --t) {
    const float* h_t = h_fwd + (size_t)t * B * H;
    const float* h_prev = (t == 0) ? h0 : h_fwd + (size_t)(t - 1) * B * H;
    double* delta = d_bprime + (size_t)t * B * H;
    for (int b = 0; b < B; ++b) {
      for (int i = 0; i < H; ++i) {
        const double h = (double)h_t[(size_t)b * H + i];
        double slope;
        if (act == ORACLE_ACT_RELU) slope = (h > 0.0) ? 1.0 : 0.0;
        else if (act == ORACLE_ACT_TANH) slope = 1.0 - h * h;
        else slope = 1.0;
        delta[(size_t)b * H + i] = slope * ((double)dh_ext[((size_t)t * B + b) * H + i] + back[(size_t)b * H + i]);
      }
    }
    for (size_t j = 0; j < (size_t)B * H; ++j) back[j] = 0.0;
    for (int i = 0; i < H; ++i) {
      for (int32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
        const double w = (double)oracle_half_bits_to_float(val_bits[k]);
        const int j = col_idx[k];
        for (int b = 0; b < B; ++b) {
          back[(size_t)b * H + j] += w * delta[(size_t)b * H + i];
          if (dU) dU[k] += delta[(size_t)b * H + i] * (h_prev ? (double)h_prev[(size_t)b * H + j] : 0.0);
        }
      }
    }
  }
  if (dh0) for (size_t j = 0; j < (size_t)B * H; ++j) dh0[j] = back[j];
  free(back);
  return 0;
}

/*
 * Backward pass through time of the LSTM cell, binary64.  U is [4H][H] in CSR (the forward matrix, row blocks
 * i | f | g | o).  Kept from the forward pass: gates [T][B][4H] (after their activations, same blocks), c_fwd and
 * h_fwd [T][B][H]; c0, h0 [B][H] or NULL (zeros).  dh_ext is [T][B][H] (e_t).  Outputs: d_bprime [T][B][4H] (dp_t),
 * dh0, dc0 [B][H] (may be NULL), dU [nnz] in CSR order (may be NULL).
 */
int oracle_lstm_backward_f64(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                             const uint16_t* val_bits, const float* gates, const float* c_fwd, const float* c0,
                             const float* h_fwd, const float* h0, const float* dh_ext,
                             double* d_bprime, double* dh0, double* dc0, double* dU) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !d_bprime || (T > 0 && (!gates || !c_fwd || !h_fwd || !dh_ext))) return -1;
  const int64_t nnz = row_ptr[4 * H];
  double* back = (double*)calloc((size_t)B * H, sizeof(double));  /* U^T dp_{t+1} */
  double* carry = (double*)calloc((size_t)B * H, sizeof(double)); /* dc_{t+1} f_{t+1} */
  if (!back || !carry) { free(back); free(carry); return -1; }
  if (dU) for (int64_t k = 0; k < nnz; ++k) dU[k] = 0.0;
  for (int t = T - 1; t >= 0; --t) {
    const float* h_prev = (t == 0) ? h0 : h_fwd + (size_t)(t - 1) * B * H;
    const float* c_prev = (t == 0) ? c0 : c_fwd + (size_t)(t - 1) * B * H;
    double* dp = d_bprime + (size_t)t * B * 4 * H;
    for (int b = 0; b < B; ++b) {
      const float* q = gates + ((size_t)t * B + b) * 4 * H;
      for (int j = 0; j < H; ++j) {
        const double gi = q[j], gf = q[H + j], gg = q[2 * H + j], go = q[3 * H + j];
        const double tc = tanh((double)c_fwd[((size_t)t * B + b) * H + j]);
        const double cp = c_prev ? (double)c_prev[(size_t)b * H + j] : 0.0;
        const double dh = (double)dh_ext[((size_t)t * B + b) * H + j] + back[(size_t)b * H + j];
        const double dc = carry[(size_t)b * H + j] + dh * go * (1.0 - tc * tc);
        dp[(size_t)b * 4 * H + j] = dc * gg * gi * (1.0 - gi);
        dp[(size_t)b * 4 * H + H + j] = dc * cp * gf * (1.0 - gf);
        dp[(size_t)b * 4 * H + 2 * H + j] = dc * gi * (1.0 - gg * gg);
        dp[(size_t)b * 4 * H + 3 * H + j] = dh * tc * go * (1.0 - go);
        carry[(size_t)b * H + j] = dc * gf;
      }
    }
    for (size_t j = 0; j < (size_t)B * H; ++j) back[j] = 0.0;
    for (int r = 0; r < 4 * H; ++r) {
      for (int32_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
        const double w = (double)oracle_half_bits_to_float(val_bits[k]);
        const int j = col_idx[k];
        for (int b = 0; b < B; ++b) {
          back[(size_t)b * H + j] += w * dp[(size_t)b * 4 * H + r];
          if (dU) dU[k] += dp[(size_t)b * 4 * H + r] * (h_prev ? (double)h_prev[(size_t)b * H + j] : 0.0);
        }
      }
    }
  }
  if (dh0) for (size_t j = 0; j < (size_t)B * H; ++j) dh0[j] = back[j];
  if (dc0) for (size_t j = 0; j < (size_t)B * H; ++j) dc0[j] = carry[j];
  free(back);
  free(carry);
  return 0;
}

/*
 * Backward pass through time of the GRU cell, binary64.  U is [3H][H] in CSR (the forward matrix, row blocks
 * r | z | n).  Kept from the forward pass: gates [T][B][4H] (blocks r | z | n | q), h_fwd [T][B][H]; h0 [B][H] or NULL
 * (zeros).  dh_ext is [T][B][H] (e_t).  Outputs: d_bprime [T][B][3H] (dp_r | dp_z | da), d_rec [T][B][3H]
 * (dp_r | dp_z | dq: what the recurrent product and the weight gradient use), dh0 [B][H] (may be NULL), dU [nnz] in CSR
 * order (may be NULL), db_hn [H] (may be NULL).
 */
int oracle_gru_backward_f64(int H, int B, int T, const int32_t* row_ptr, const int32_t* col_idx,
                            const uint16_t* val_bits, const float* gates, const float* h_fwd, const float* h0,
                            const float* dh_ext, double* d_bprime, double* d_rec, double* dh0, double* dU, double* db_hn) {
  if (H <= 0 || B <= 0 || T < 0 || !row_ptr || !d_bprime || !d_rec || (T > 0 && (!gates || !h_fwd || !dh_ext))) return -1;
  const int64_t nnz = row_ptr[3 * H];
  double* back = (double*)calloc((size_t)B * H, sizeof(double));   /* U^T v_{t+1} */
  double* direct = (double*)calloc((size_t)B * H, sizeof(double)); /* dh_{t+1} z_{t+1} */
  if (!back || !direct) { free(back); free(direct); return -1; }
  if (dU) for (int64_t k = 0; k < nnz; ++k) dU[k] = 0.0;
  if (db_hn) for (int j = 0; j < H; ++j) db_hn[j] = 0.0;
  for (int t = T - 1; t >= 0; --t) {
    const float* h_prev = (t == 0) ? h0 : h_fwd + (size_t)(t - 1) * B * H;
    double* dx = d_bprime + (size_t)t * B * 3 * H;
    double* v = d_rec + (size_t)t * B * 3 * H;
    for (int b = 0; b < B; ++b) {
      const float* g = gates + ((size_t)t * B + b) * 4 * H;
      for (int j = 0; j < H; ++j) {
        const double r = g[j], z = g[H + j], n = g[2 * H + j], q = g[3 * H + j];
        const double hp = h_prev ? (double)h_prev[(size_t)b * H + j] : 0.0;
        const double dh = (double)dh_ext[((size_t)t * B + b) * H + j] + direct[(size_t)b * H + j] + back[(size_t)b * H + j];
        const double da = dh * (1.0 - z) * (1.0 - n * n);
        const double dpr = da * q * r * (1.0 - r);
        const double dpz = dh * (hp - n) * z * (1.0 - z);
        const double dq = da * r;
        dx[(size_t)b * 3 * H + j] = dpr;  dx[(size_t)b * 3 * H + H + j] = dpz;  dx[(size_t)b * 3 * H + 2 * H + j] = da;
        v[(size_t)b * 3 * H + j] = dpr;   v[(size_t)b * 3 * H + H + j] = dpz;   v[(size_t)b * 3 * H + 2 * H + j] = dq;
        direct[(size_t)b * H + j] = dh * z;
        if (db_hn) db_hn[j] += dq;
      }
    }
    for (size_t j = 0; j < (size_t)B * H; ++j) back[j] = 0.0;
    for (int row = 0; row < 3 * H; ++row) {
      for (int32_t k = row_ptr[row]; k < row_ptr[row + 1]; ++k) {
        const double w = (double)oracle_half_bits_to_float(val_bits[k]);
        const int j = col_idx[k];
        for (int b = 0; b < B; ++b) {
          back[(size_t)b * H + j] += w * v[(size_t)b * 3 * H + row];
          if (dU) dU[k] += v[(size_t)b * 3 * H + row] * (h_prev ? (double)h_prev[(size_t)b * H + j] : 0.0);
        }
      }
    }
  }
  if (dh0) for (size_t j = 0; j < (size_t)B * H; ++j) dh0[j] = back[j] + direct[j];
  free(back);
  free(direct);
  return 0;
}
