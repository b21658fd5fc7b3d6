// CPU oracle for single-stream SRU / QRNN inference (arXiv 1803.11389), and for
// the LSTM the paper compares them with.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
// GPU library is checked against.  It shares no code with the GPU path, is not
// linked into it, and must never be called from it.
//
// What it computes
//   * SRU layer, paper Eq. (2):   xh = W x,  f = sigma(W_f x + b_f),
//     r = sigma(W_r x + b_r),  c_t = f*c_{t-1} + (1-f)*xh,
//     h_t = r*tanh(c_t) + (1-r)*x_t.
//   * QRNN layer, paper Eq. (3), written for a causal window of k inputs
//     (the paper prints k = 2):  u_g = sum_{j<k} W_g^j x_{t-j},
//     xh = tanh(u_0), f = sigma(u_1), o = sigma(u_2),
//     c_t = f*c_{t-1} + (1-f)*xh,  h_t = o*tanh(c_t).
//   * Multi-time-step blocking, paper Section 3 and Eq. (4): the gate
//     pre-activations of T consecutive steps are produced together as one
//     matrix-matrix product, one weight row being fetched once and applied to
//     all T columns, and only then does the element-wise recurrence ripple
//     over the T steps.
//   * A stack feeds layer l's h_t to layer l+1 as x_t.
//
// Arithmetic: every sum, gate and state is IEEE double; weights are given in
// their storage type (fp32, bf16 bit patterns, or 8-bit floats with a scale per
// row) and widened exactly.  Each dot product adds its terms in ascending column
// order whatever T is, so the result is bit-identical for every block size.
// Nothing is rounded between layers.  The paper does not state the precision
// of its runs (Section 4).  For kernels that hand the block X of Eq. 4 to the
// matrix product in bfloat16, the argument round_operand = 1 of
// oracle_*_forward makes this oracle round exactly that operand the same way
// (double -> float -> bfloat16, both round-to-nearest-even) and nothing else:
// the highway term, the state and the sums stay double.  With 0 nothing is
// rounded, and every pin below is stated for it.
//
// Direction.  The paper notes that a bidirectional network is two independent
// passes over the sequence, one in each direction (Section 2.1).  With
// reverse = 1 every layer walks the sequence from its last step to its first:
// step number tau = 0 .. L-1 of the walk is time L-1-tau, "the previous step"
// is the later time (c_{t+1} in place of c_{t-1}; the QRNN window holds x_t,
// x_{t+1}, ...), c_init is the state before time L-1 is taken in, c_final the
// state after time 0, and xhist entry (l, j) is layer l's input j+1 steps before
// the walk starts (and, on return, the last k-1 inputs it took in).  h stays
// indexed by time.  Nothing else differs, so the reverse pass over x equals the
// forward pass over the time-reversed x, read backwards (a pin).
//
// Pins (tests/test_oracle_*.py; the LSTM's are in tests/test_oracle_lstm_pins.py):
// hand-worked d=2 examples for both cells,
// step-by-step brute force (oracle_*_step below, written separately),
// closed forms (f==0, f==1/2, f==1, r==0, W==0), the non-iterative solution of
// the linear recurrence, an independent library matrix product for the weight
// layout, block-size invariance, chunk chaining and boundedness.
//
// 8-bit weights (not in the paper; they serve its argument that the bytes of
// weights per step decide the speed, Sections 1 and 3): the matrix is stored as
// OCP FP8 E4M3 codes q (1 sign, 4 exponent bits with bias 7, 3 mantissa bits,
// subnormals, no infinities, S.1111.111 = NaN) row-major, padded with zeros to
// a multiple of 256 bytes, followed by one fp32 scale per row;
// W[row][col] = scale[row] * value(q[row][col]).
//
// LSTM (paper Eq. (1)), the network the method is compared with (Sections 2.2
// and 3.1):  f = sigma(W_f x + U_f h_{t-1} + b_f), i and o likewise,
// c-hat = tanh(W_c x + U_c h_{t-1} + b_c), c_t = f*c_{t-1} + i*c-hat,
// h_t = o*tanh(c_t).  Section 3.1: the products with the input, W x_t, do not
// depend on the feedback and are formed for T steps together (a weight row
// applied to all T columns, as in Eq. 4); the products with h_{t-1} follow step
// by step.  oracle_lstm_forward takes its steps in that order; every
// pre-activation is (W-row . x) + (U-row . h_{t-1}) + b with both dot products
// in ascending column order, so the result is bit-identical for every T.
//
// Storage conventions
//   LSTM W,U: row-major [4d x d] fp32, rows [0,d) = f, [d,2d) = i, [2d,3d) = o,
//             [3d,4d) = c-hat (the order Eq. 1 lists them);  b : [4d] or NULL
//   SRU  W  : row-major [3d x d],   rows [0,d) = W, [d,2d) = W_f, [2d,3d) = W_r
//   SRU  b  : [2d] = b_f | b_r  (no bias on xh, Eq. 2);  NULL means zero
//   QRNN W  : row-major [3d x k*d], column block j multiplies x_{t-j};
//             rows [0,d) = xh, [d,2d) = f, [2d,3d) = o
//   QRNN b  : [3d] or NULL (Eq. 3 has none)
//   x, h    : time-major [L x d]
//   xhist   : [n_layers x (k-1) x d]; entry (l, j) is layer l's input at lag
//             j+1 before the first step of the call (zeros when NULL)

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { WDT_F32 = 0, WDT_BF16 = 1, WDT_FP8 = 2 };

inline double widen_bf16(uint16_t bits) {
  uint32_t u = static_cast<uint32_t>(bits) << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return static_cast<double>(f);
}

// Value of an E4M3 code, from the format's definition.
inline double value_e4m3(uint8_t code) {
  const int e = (code >> 3) & 15;
  const int m = code & 7;
  double v;
  if (e == 15 && m == 7) v = std::nan("");
  else if (e == 0) v = std::ldexp(m / 8.0, 1 - 7);          // subnormal: exponent of the smallest normal, no hidden one
  else v = std::ldexp(1.0 + m / 8.0, e - 7);
  return (code & 0x80) ? -v : v;
}

// Element (row, col) of a [rows x ncol] weight matrix in storage type wdt.
inline double weight_at(const void* W, int wdt, size_t rows, size_t ncol, size_t row, size_t col) {
  const size_t idx = row * ncol + col;
  if (wdt == WDT_BF16) return widen_bf16(static_cast<const uint16_t*>(W)[idx]);
  if (wdt == WDT_FP8) {
    const size_t scale_offset = (rows * ncol + 255) / 256 * 256;
    float scale;
    std::memcpy(&scale, static_cast<const char*>(W) + scale_offset + row * sizeof(float), sizeof scale);
    return static_cast<double>(scale) * value_e4m3(static_cast<const uint8_t*>(W)[idx]);
  }
  return static_cast<double>(static_cast<const float*>(W)[idx]);
}

inline double sigma(double z) { return 1.0 / (1.0 + std::exp(-z)); }

// Nearest bfloat16 (ties to even) of the nearest float of v, as a double.
inline double to_bf16_value(double v) {
  const float f = static_cast<float>(v);
  uint32_t u;
  std::memcpy(&u, &f, sizeof u);
  if ((u & 0x7F800000u) == 0x7F800000u) return static_cast<double>(f);   // inf / nan pass through
  u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
  float r;
  std::memcpy(&r, &u, sizeof r);
  return static_cast<double>(r);
}

// X of Eq. 4 as it enters the product: as it is, or rounded to bfloat16.
inline double operand(double v, int round_operand) { return round_operand ? to_bf16_value(v) : v; }

// Row of the time-major arrays that step tau of a layer's walk over L steps reads and writes.
inline long time_of(long tau, long L, int reverse) { return reverse ? L - 1 - tau : tau; }

// U[g][i][t] = sum_col W[g*d+i][col] * X[col][t]   (Eq. 4 for all three gates)
// X is the [ncol x nt] block, column t contiguous in t for a fixed col.
// One weight is read once and applied to all nt columns (Section 3).
void gate_block(const void* W, int wdt, int d, int ncol, const double* X,
                int nt, double* U /* [3][d][nt] */) {
#pragma omp parallel for schedule(static)
  for (int row = 0; row < 3 * d; ++row) {
    double* acc = U + static_cast<size_t>(row) * nt;
    for (int t = 0; t < nt; ++t) acc[t] = 0.0;
    for (int col = 0; col < ncol; ++col) {
      const double w = weight_at(W, wdt, static_cast<size_t>(3) * d, ncol, row, col);
      const double* xc = X + static_cast<size_t>(col) * nt;
      for (int t = 0; t < nt; ++t) acc[t] += w * xc[t];
    }
  }
}

// One SRU layer over the whole sequence, T steps per block.
// xin/hout: double [L x d]; c: double [d] in/out.
void sru_layer(const void* W, int wdt, const float* bias, const double* xin,
               double* hout, double* c, int d, long L, int T, int round_operand, int reverse) {
  std::vector<double> X(static_cast<size_t>(d) * T);
  std::vector<double> U(static_cast<size_t>(3) * d * T);
  for (long t0 = 0; t0 < L; t0 += T) {
    const int nt = static_cast<int>(L - t0 < T ? L - t0 : T);
    // X = [x_{t0} ... x_{t0+nt-1}] as columns (t0, t count steps of the walk)
    for (int j = 0; j < d; ++j)
      for (int t = 0; t < nt; ++t)
        X[static_cast<size_t>(j) * nt + t] = operand(xin[time_of(t0 + t, L, reverse) * d + j], round_operand);
    gate_block(W, wdt, d, d, X.data(), nt, U.data());
    const double* Ux = U.data();
    const double* Uf = U.data() + static_cast<size_t>(d) * nt;
    const double* Ur = U.data() + static_cast<size_t>(2) * d * nt;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < d; ++i) {
      const double bf = bias ? static_cast<double>(bias[i]) : 0.0;
      const double br = bias ? static_cast<double>(bias[d + i]) : 0.0;
      double ci = c[i];
      for (int t = 0; t < nt; ++t) {
        const double xh = Ux[static_cast<size_t>(i) * nt + t];
        const double f = sigma(Uf[static_cast<size_t>(i) * nt + t] + bf);
        const double r = sigma(Ur[static_cast<size_t>(i) * nt + t] + br);
        ci = f * ci + (1.0 - f) * xh;
        const double xt = xin[time_of(t0 + t, L, reverse) * d + i];
        hout[time_of(t0 + t, L, reverse) * d + i] = r * std::tanh(ci) + (1.0 - r) * xt;
      }
      c[i] = ci;
    }
  }
}

// One QRNN layer.  hist: double [(k-1) x d] in/out (lag j+1 at row j).
void qrnn_layer(const void* W, int wdt, const float* bias, const double* xin,
                double* hout, double* c, double* hist, int d, long L, int T,
                int k, int round_operand, int reverse) {
  const int ncol = k * d;
  std::vector<double> X(static_cast<size_t>(ncol) * T);
  std::vector<double> U(static_cast<size_t>(3) * d * T);
  // input at step s of the walk (s may be negative: taken from hist)
  auto x_at = [&](long s, int m) -> double {
    if (s >= 0) return xin[time_of(s, L, reverse) * d + m];
    return hist[static_cast<size_t>(-s - 1) * d + m];
  };
  for (long t0 = 0; t0 < L; t0 += T) {
    const int nt = static_cast<int>(L - t0 < T ? L - t0 : T);
    // column t of X is [x_t ; x_{t-1} ; ... ; x_{t-k+1}]
    for (int j = 0; j < k; ++j)
      for (int m = 0; m < d; ++m)
        for (int t = 0; t < nt; ++t)
          X[(static_cast<size_t>(j) * d + m) * nt + t] = operand(x_at(t0 + t - j, m), round_operand);
    gate_block(W, wdt, d, ncol, X.data(), nt, U.data());
    const double* Uz = U.data();
    const double* Uf = U.data() + static_cast<size_t>(d) * nt;
    const double* Uo = U.data() + static_cast<size_t>(2) * d * nt;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < d; ++i) {
      const double bz = bias ? static_cast<double>(bias[i]) : 0.0;
      const double bf = bias ? static_cast<double>(bias[d + i]) : 0.0;
      const double bo = bias ? static_cast<double>(bias[2 * d + i]) : 0.0;
      double ci = c[i];
      for (int t = 0; t < nt; ++t) {
        const double z = std::tanh(Uz[static_cast<size_t>(i) * nt + t] + bz);
        const double f = sigma(Uf[static_cast<size_t>(i) * nt + t] + bf);
        const double o = sigma(Uo[static_cast<size_t>(i) * nt + t] + bo);
        ci = f * ci + (1.0 - f) * z;
        hout[time_of(t0 + t, L, reverse) * d + i] = o * std::tanh(ci);
      }
      c[i] = ci;
    }
  }
  // new history: the last k-1 inputs seen, most recent first
  if (k > 1) {
    std::vector<double> nh(static_cast<size_t>(k - 1) * d);
    for (int j = 0; j < k - 1; ++j)
      for (int m = 0; m < d; ++m) nh[static_cast<size_t>(j) * d + m] = x_at(L - 1 - j, m);
    std::memcpy(hist, nh.data(), nh.size() * sizeof(double));
  }
}

// One LSTM layer (Eq. 1) over the whole sequence, the input products of T steps at a time (Section 3.1).
// xin/hout: double [L x d]; hprev, c: double [d] in/out (h_{t-1} and c_{t-1} of the next step to come).
void lstm_layer(const float* W, const float* U, const float* bias, const double* xin, double* hout,
                double* hprev, double* c, int d, long L, int T) {
  std::vector<double> A(static_cast<size_t>(4) * d * T);   // A[row][t] = W[row] . x_{t0+t}
  std::vector<double> hnew(d);
  for (long t0 = 0; t0 < L; t0 += T) {
    const int nt = static_cast<int>(L - t0 < T ? L - t0 : T);
    // the part without feedback, all nt steps of the block: one weight fetched once and used nt times
#pragma omp parallel for schedule(static)
    for (int row = 0; row < 4 * d; ++row) {
      double* acc = A.data() + static_cast<size_t>(row) * nt;
      for (int t = 0; t < nt; ++t) acc[t] = 0.0;
      for (int col = 0; col < d; ++col) {
        const double w = static_cast<double>(W[static_cast<size_t>(row) * d + col]);
        for (int t = 0; t < nt; ++t) acc[t] += w * xin[(t0 + t) * d + col];
      }
    }
    // the part with feedback, one step after the other
    for (int t = 0; t < nt; ++t) {
#pragma omp parallel for schedule(static)
      for (int i = 0; i < d; ++i) {
        double pre[4];
        for (int g = 0; g < 4; ++g) {
          const size_t row = static_cast<size_t>(g) * d + i;
          double u = 0.0;
          for (int col = 0; col < d; ++col) u += static_cast<double>(U[row * d + col]) * hprev[col];
          pre[g] = A[row * nt + t] + u + (bias ? static_cast<double>(bias[row]) : 0.0);
        }
        const double f = sigma(pre[0]);
        const double in = sigma(pre[1]);
        const double o = sigma(pre[2]);
        const double chat = std::tanh(pre[3]);
        c[i] = f * c[i] + in * chat;
        hnew[i] = o * std::tanh(c[i]);
      }
      for (int i = 0; i < d; ++i) {
        hprev[i] = hnew[i];
        hout[(t0 + t) * d + i] = hnew[i];
      }
    }
  }
}

}  // namespace

extern "C" {

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

// Stacked SRU forward (Eq. 2 per layer, Section 3 blocking with block size T).
// W[l]: [3d x d] in storage type wdt; bias: NULL, or array whose entries may be
// NULL; x: double [L x d] (fp32 inputs are widened exactly by the caller);
// c_init: double [n_layers x d] or NULL; outputs double:
// h [L x d] (top layer), c_final [n_layers x d], h_all optional
// [n_layers x L x d] (every layer's output).  round_operand, reverse: see the
// header of this file.  Returns 0, or 1 on bad arguments.
int oracle_sru_forward(const void* const* W, const float* const* bias,
                       const double* x, const double* c_init, double* h,
                       double* c_final, double* h_all, int n_layers, int d,
                       long L, int T, int wdt, int round_operand, int reverse) {
  if (!W || !c_final || n_layers < 1 || d < 1 || L < 0 || T < 1) return 1;
  if (L > 0 && (!x || !h)) return 1;
  if (wdt != WDT_F32 && wdt != WDT_BF16 && wdt != WDT_FP8) return 1;
  const size_t n = static_cast<size_t>(L) * d;
  std::vector<double> cur(n), nxt(n);
  for (size_t i = 0; i < n; ++i) cur[i] = x[i];
  for (int l = 0; l < n_layers; ++l) {
    std::vector<double> c(d);
    for (int i = 0; i < d; ++i)
      c[i] = c_init ? c_init[static_cast<size_t>(l) * d + i] : 0.0;
    sru_layer(W[l], wdt, bias ? bias[l] : nullptr, cur.data(), nxt.data(),
              c.data(), d, L, T, round_operand, reverse);
    std::memcpy(c_final + static_cast<size_t>(l) * d, c.data(), d * sizeof(double));
    if (h_all && n) std::memcpy(h_all + static_cast<size_t>(l) * n, nxt.data(), n * sizeof(double));
    cur.swap(nxt);
  }
  if (n) std::memcpy(h, cur.data(), n * sizeof(double));
  return 0;
}

// Stacked QRNN forward (Eq. 3 per layer, window k, fo-pooling, blocked by T).
// xhist_init: double [n_layers x (k-1) x d] or NULL (zeros: causal padding);
// xhist_final: double, same shape, or NULL.
int oracle_qrnn_forward(const void* const* W, const float* const* bias,
                        const double* x, const double* c_init,
                        const double* xhist_init, double* h, double* c_final,
                        double* xhist_final, double* h_all, int n_layers,
                        int d, long L, int T, int k, int wdt, int round_operand, int reverse) {
  if (!W || !c_final || n_layers < 1 || d < 1 || L < 0 || T < 1 || k < 1) return 1;
  if (L > 0 && (!x || !h)) return 1;
  if (wdt != WDT_F32 && wdt != WDT_BF16 && wdt != WDT_FP8) return 1;
  const size_t n = static_cast<size_t>(L) * d;
  const size_t nh = static_cast<size_t>(k - 1) * d;
  std::vector<double> cur(n), nxt(n);
  for (size_t i = 0; i < n; ++i) cur[i] = x[i];
  for (int l = 0; l < n_layers; ++l) {
    std::vector<double> c(d), hist(nh ? nh : 1, 0.0);
    for (int i = 0; i < d; ++i)
      c[i] = c_init ? c_init[static_cast<size_t>(l) * d + i] : 0.0;
    if (xhist_init)
      for (size_t i = 0; i < nh; ++i) hist[i] = xhist_init[l * nh + i];
    qrnn_layer(W[l], wdt, bias ? bias[l] : nullptr, cur.data(), nxt.data(),
               c.data(), hist.data(), d, L, T, k, round_operand, reverse);
    std::memcpy(c_final + static_cast<size_t>(l) * d, c.data(), d * sizeof(double));
    if (xhist_final && nh) std::memcpy(xhist_final + l * nh, hist.data(), nh * sizeof(double));
    if (h_all && n) std::memcpy(h_all + static_cast<size_t>(l) * n, nxt.data(), n * sizeof(double));
    cur.swap(nxt);
  }
  if (n) std::memcpy(h, cur.data(), n * sizeof(double));
  return 0;
}

// ---- brute force: one layer, one time step, no blocking -------------------
// Written on its own (a matrix-vector product per gate, then Eq. 2 / Eq. 3
// once) so that the blocked functions above can be checked against it.

// x_t, c (in/out), h_t are double [d].
int oracle_sru_step(const void* W, const float* bias, const double* x_t,
                    double* c, double* h_t, int d, int wdt) {
  if (!W || !x_t || !c || !h_t || d < 1) return 1;
  for (int i = 0; i < d; ++i) {
    double ux = 0.0, uf = 0.0, ur = 0.0;
    const size_t rows = static_cast<size_t>(3) * d;
    for (int j = 0; j < d; ++j) ux += weight_at(W, wdt, rows, d, i, j) * x_t[j];
    for (int j = 0; j < d; ++j) uf += weight_at(W, wdt, rows, d, d + i, j) * x_t[j];
    for (int j = 0; j < d; ++j) ur += weight_at(W, wdt, rows, d, 2 * d + i, j) * x_t[j];
    if (bias) { uf += bias[i]; ur += bias[d + i]; }
    const double f = 1.0 / (1.0 + std::exp(-uf));
    const double r = 1.0 / (1.0 + std::exp(-ur));
    c[i] = f * c[i] + (1.0 - f) * ux;
    h_t[i] = r * std::tanh(c[i]) + (1.0 - r) * x_t[i];
  }
  return 0;
}

// xwin: double [k x d], row j = x_{t-j} (row 0 is the current input).
int oracle_qrnn_step(const void* W, const float* bias, const double* xwin,
                     double* c, double* h_t, int d, int k, int wdt) {
  if (!W || !xwin || !c || !h_t || d < 1 || k < 1) return 1;
  const size_t ld = static_cast<size_t>(k) * d;
  for (int i = 0; i < d; ++i) {
    double u[3] = {0.0, 0.0, 0.0};
    for (int g = 0; g < 3; ++g)
      for (int j = 0; j < k; ++j)
        for (int m = 0; m < d; ++m)
          u[g] += weight_at(W, wdt, static_cast<size_t>(3) * d, ld, static_cast<size_t>(g) * d + i,
                            static_cast<size_t>(j) * d + m) *
                  xwin[static_cast<size_t>(j) * d + m];
    if (bias) { u[0] += bias[i]; u[1] += bias[d + i]; u[2] += bias[2 * d + i]; }
    const double z = std::tanh(u[0]);
    const double f = 1.0 / (1.0 + std::exp(-u[1]));
    const double o = 1.0 / (1.0 + std::exp(-u[2]));
    c[i] = f * c[i] + (1.0 - f) * z;
    h_t[i] = o * std::tanh(c[i]);
  }
  return 0;
}

// Stacked LSTM forward (Eq. 1 per layer; the input products blocked by T as Section 3.1 describes).
// W[l], U[l]: fp32 [4d x d]; bias: NULL, or array whose entries may be NULL ([4d]); x: double [L x d];
// h_init, c_init: double [n_layers x d] or NULL (zeros); outputs double: h [L x d] (top layer),
// h_final, c_final [n_layers x d] (every layer's h and c after the last step), h_all optional
// [n_layers x L x d].  Returns 0, or 1 on bad arguments.
int oracle_lstm_forward(const float* const* W, const float* const* U, const float* const* bias,
                        const double* x, const double* h_init, const double* c_init, double* h,
                        double* h_final, double* c_final, double* h_all, int n_layers, int d, long L, int T) {
  if (!W || !U || !h_final || !c_final || n_layers < 1 || d < 1 || L < 0 || T < 1) return 1;
  if (L > 0 && (!x || !h)) return 1;
  const size_t n = static_cast<size_t>(L) * d;
  std::vector<double> cur(n), nxt(n);
  for (size_t i = 0; i < n; ++i) cur[i] = x[i];
  for (int l = 0; l < n_layers; ++l) {
    std::vector<double> c(d), hp(d);
    for (int i = 0; i < d; ++i) {
      c[i] = c_init ? c_init[static_cast<size_t>(l) * d + i] : 0.0;
      hp[i] = h_init ? h_init[static_cast<size_t>(l) * d + i] : 0.0;
    }
    lstm_layer(W[l], U[l], bias ? bias[l] : nullptr, cur.data(), nxt.data(), hp.data(), c.data(), d, L, T);
    std::memcpy(c_final + static_cast<size_t>(l) * d, c.data(), d * sizeof(double));
    std::memcpy(h_final + static_cast<size_t>(l) * d, hp.data(), d * sizeof(double));
    if (h_all && n) std::memcpy(h_all + static_cast<size_t>(l) * n, nxt.data(), n * sizeof(double));
    cur.swap(nxt);
  }
  if (n) std::memcpy(h, cur.data(), n * sizeof(double));
  return 0;
}

// Brute force: one LSTM layer, one time step, the eight matrix-vector products of Eq. 1 written out
// gate by gate.  x_t, h_prev: double [d]; c: in/out; h_t: out (may not alias h_prev).
int oracle_lstm_step(const float* W, const float* U, const float* bias, const double* x_t,
                     const double* h_prev, double* c, double* h_t, int d) {
  if (!W || !U || !x_t || !h_prev || !c || !h_t || d < 1 || h_t == h_prev) return 1;
  const size_t dd = static_cast<size_t>(d);
  for (int i = 0; i < d; ++i) {
    double zf = 0.0, zi = 0.0, zo = 0.0, zc = 0.0;
    for (int j = 0; j < d; ++j) zf += static_cast<double>(W[(0 * dd + i) * dd + j]) * x_t[j];
    for (int j = 0; j < d; ++j) zi += static_cast<double>(W[(1 * dd + i) * dd + j]) * x_t[j];
    for (int j = 0; j < d; ++j) zo += static_cast<double>(W[(2 * dd + i) * dd + j]) * x_t[j];
    for (int j = 0; j < d; ++j) zc += static_cast<double>(W[(3 * dd + i) * dd + j]) * x_t[j];
    double yf = 0.0, yi = 0.0, yo = 0.0, yc = 0.0;
    for (int j = 0; j < d; ++j) yf += static_cast<double>(U[(0 * dd + i) * dd + j]) * h_prev[j];
    for (int j = 0; j < d; ++j) yi += static_cast<double>(U[(1 * dd + i) * dd + j]) * h_prev[j];
    for (int j = 0; j < d; ++j) yo += static_cast<double>(U[(2 * dd + i) * dd + j]) * h_prev[j];
    for (int j = 0; j < d; ++j) yc += static_cast<double>(U[(3 * dd + i) * dd + j]) * h_prev[j];
    const double bf = bias ? bias[i] : 0.0, bi = bias ? bias[dd + i] : 0.0;
    const double bo = bias ? bias[2 * dd + i] : 0.0, bc = bias ? bias[3 * dd + i] : 0.0;
    const double f = 1.0 / (1.0 + std::exp(-(zf + yf + bf)));
    const double in = 1.0 / (1.0 + std::exp(-(zi + yi + bi)));
    const double o = 1.0 / (1.0 + std::exp(-(zo + yo + bo)));
    const double chat = std::tanh(zc + yc + bc);
    c[i] = f * c[i] + in * chat;
    h_t[i] = o * std::tanh(c[i]);
  }
  return 0;
}

// y[L x d_out] = feat[L x d_in] * P^T, P row-major [d_out x d_in], no bias, no
// activation: the input projection of the ASR-shaped workload (not part of the
// paper's method; a plain matrix product).
int oracle_linear_forward(const float* P, const float* feat, double* y,
                          int d_out, int d_in, long L) {
  if (!P || !feat || !y || d_out < 1 || d_in < 1 || L < 0) return 1;
#pragma omp parallel for schedule(static)
  for (long t = 0; t < L; ++t)
    for (int i = 0; i < d_out; ++i) {
      double acc = 0.0;
      for (int j = 0; j < d_in; ++j)
        acc += static_cast<double>(P[static_cast<size_t>(i) * d_in + j]) *
               static_cast<double>(feat[t * d_in + j]);
      y[t * d_out + i] = acc;
    }
  return 0;
}

}  // extern "C"
