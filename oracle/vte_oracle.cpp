// CPU oracle for the fixed-structure decode operators.  TEST INFRASTRUCTURE ONLY.
//
// This file is the plain mathematical definition of every operator on the
// decode hot path, evaluated in IEEE double on the exact values of the bf16
// inputs.  It deliberately does not imitate any GPU reduction tree: every sum
// is a sequential loop in index order.  It shares no code, header, table or
// helper with the HIP library and includes nothing from it.  Only tests, the
// smoke check and the benchmark's cpu_baseline leg may call it; the product
// path never does.
//
// Why these definitions: the paper names the operator families whose
// floating-point grouping reshaping disturbs (Sec. 1: LayerNorm, GEMV;
// Sec. 2.3: reductions, Split-K GEMMs; Sec. 7.1/7.2: LM-head logits and the
// greedy token) but prints no formula for any of them, so each function below
// is the textbook definition of the named operator.  The resource-adaptation
// contract (Sec. 2.2) is an equality between GPU runs and needs no oracle; the
// oracle checks that the fixed-structure kernels compute the right function.
//
// Pins (tests/test_oracle_pins.py): unit-RMS rows, one-hot rows, constant and
// alternating rows for LayerNorm, identity / permutation / all-ones weights,
// brute-force argmax on tiny vocabularies, SiLU limits, exact-integer inputs,
// forward-vs-reverse summation, float128-free rational cross-checks in Python
// fractions on tiny shapes.
// Unpinned by anything the paper prints: the number of greedy-token flips and
// the magnitude of reshaping drift (the paper shows them only in figures).
//
// Parallelism: std::thread over OUTPUT ROWS only.  Every output's k-loop stays
// sequential, so results do not depend on the thread count.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>
#include <algorithm>
#include <limits>

namespace {

// bf16 = sign(1) exponent(8) fraction(7): the upper half of an IEEE binary32.
inline double bf16_to_f64(uint16_t h) {
  uint32_t u = static_cast<uint32_t>(h) << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return static_cast<double>(f);
}

// Round a double to the nearest bf16, ties to even, in one rounding step.
// The value is scaled so that one bf16 ulp equals 1.0, rounded with
// nearbyint() (default rounding mode: to nearest even) and scaled back; both
// scalings are exact powers of two.
inline uint16_t f64_to_bf16(double d) {
  if (std::isnan(d)) return 0x7fc0;
  if (std::isinf(d)) return d > 0 ? 0x7f80 : 0xff80;
  if (d == 0.0) return std::signbit(d) ? 0x8000 : 0x0000;
  int e = std::ilogb(d);            // |d| in [2^e, 2^(e+1))
  if (e < -126) e = -126;           // subnormal bf16 share the exponent -126
  double q = std::ldexp(d, 7 - e);  // one ulp of bf16 at this exponent -> 1.0
  double r = std::nearbyint(q);
  double v = std::ldexp(r, e - 7);
  float f = static_cast<float>(v);  // exact: at most 8 significant bits
  if (std::isinf(f)) return f > 0 ? 0x7f80 : 0xff80;
  uint32_t u;
  std::memcpy(&u, &f, sizeof u);
  return static_cast<uint16_t>(u >> 16);
}

template <class F>
void parallel_rows(int64_t n, int threads, F&& body) {
  if (threads <= 1 || n <= 1) {
    for (int64_t i = 0; i < n; ++i) body(i);
    return;
  }
  int t = static_cast<int>(std::min<int64_t>(threads, n));
  std::vector<std::thread> pool;
  pool.reserve(t);
  for (int w = 0; w < t; ++w) {
    int64_t lo = n * w / t, hi = n * (w + 1) / t;
    pool.emplace_back([lo, hi, &body] {
      for (int64_t i = lo; i < hi; ++i) body(i);
    });
  }
  for (auto& th : pool) th.join();
}

// dot(W[n,:], X[b,:]) sequential in k, double.
inline double dot_row(const uint16_t* w, const uint16_t* x, int64_t K) {
  double s = 0.0;
  for (int64_t k = 0; k < K; ++k) s += bf16_to_f64(w[k]) * bf16_to_f64(x[k]);
  return s;
}

inline double silu(double g) { return g / (1.0 + std::exp(-g)); }

}  // namespace

extern "C" {

int orc_hardware_threads() {
  unsigned n = std::thread::hardware_concurrency();
  return n ? static_cast<int>(n) : 1;
}

// ---- bf16 conversions (own code) --------------------------------------------
void orc_bf16_to_f64(const uint16_t* in, int64_t n, double* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = bf16_to_f64(in[i]);
}
void orc_f64_to_bf16(const double* in, int64_t n, uint16_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = f64_to_bf16(in[i]);
}

// ---- RMSNorm: ref[r,i] = x[r,i] * gamma[i] / sqrt(mean_j x[r,j]^2 + eps) -----
void orc_rmsnorm(const uint16_t* x, const uint16_t* gamma, int64_t rows,
                 int64_t cols, double eps, double* out, int threads) {
  parallel_rows(rows, threads, [=](int64_t r) {
    const uint16_t* xr = x + r * cols;
    double ss = 0.0;
    for (int64_t j = 0; j < cols; ++j) {
      double v = bf16_to_f64(xr[j]);
      ss += v * v;
    }
    double denom = std::sqrt(ss / static_cast<double>(cols) + eps);
    for (int64_t i = 0; i < cols; ++i)
      out[r * cols + i] = bf16_to_f64(xr[i]) * bf16_to_f64(gamma[i]) / denom;
  });
}

// ---- LayerNorm (biased variance, two passes) ----------------------------------
void orc_layernorm(const uint16_t* x, const uint16_t* gamma,
                   const uint16_t* beta, int64_t rows, int64_t cols, double eps,
                   double* out, int threads) {
  parallel_rows(rows, threads, [=](int64_t r) {
    const uint16_t* xr = x + r * cols;
    double s = 0.0;
    for (int64_t j = 0; j < cols; ++j) s += bf16_to_f64(xr[j]);
    double mu = s / static_cast<double>(cols);
    double v = 0.0;
    for (int64_t j = 0; j < cols; ++j) {
      double d = bf16_to_f64(xr[j]) - mu;
      v += d * d;
    }
    double denom = std::sqrt(v / static_cast<double>(cols) + eps);
    for (int64_t i = 0; i < cols; ++i)
      out[r * cols + i] = (bf16_to_f64(xr[i]) - mu) / denom * bf16_to_f64(gamma[i]) +
                          bf16_to_f64(beta[i]);
  });
}

// ---- GEMV: Y[b,n] = sum_k W[n,k] X[b,k];  W is [N,K] row-major ---------------
void orc_gemv(const uint16_t* W, const uint16_t* X, int64_t B, int64_t N,
              int64_t K, double* Y, int threads) {
  parallel_rows(N, threads, [=](int64_t n) {
    for (int64_t b = 0; b < B; ++b) Y[b * N + n] = dot_row(W + n * K, X + b * K, K);
  });
}

// Same sum in descending k: a self-check of the summation (not a definition).
void orc_gemv_reverse(const uint16_t* W, const uint16_t* X, int64_t B, int64_t N,
                      int64_t K, double* Y, int threads) {
  parallel_rows(N, threads, [=](int64_t n) {
    for (int64_t b = 0; b < B; ++b) {
      double s = 0.0;
      for (int64_t k = K - 1; k >= 0; --k)
        s += bf16_to_f64(W[n * K + k]) * bf16_to_f64(X[b * K + k]);
      Y[b * N + n] = s;
    }
  });
}

// Sum of |W[n,k] X[b,k]|: the scale of the fp32-accumulation error bound.
void orc_gemv_abs(const uint16_t* W, const uint16_t* X, int64_t B, int64_t N,
                  int64_t K, double* Y, int threads) {
  parallel_rows(N, threads, [=](int64_t n) {
    for (int64_t b = 0; b < B; ++b) {
      double s = 0.0;
      for (int64_t k = 0; k < K; ++k)
        s += std::fabs(bf16_to_f64(W[n * K + k]) * bf16_to_f64(X[b * K + k]));
      Y[b * N + n] = s;
    }
  });
}

// ---- gate/up with SiLU: act[b,j] = silu(g) * u, g = W[j,:]·x, u = W[Nh+j,:]·x --
// g and u are the unrounded double dot products (the fused epilogue never
// rounds them to bf16).
void orc_gemv_silu_mul(const uint16_t* W, const uint16_t* X, int64_t B,
                       int64_t Nh, int64_t K, double* act, int threads) {
  parallel_rows(Nh, threads, [=](int64_t j) {
    for (int64_t b = 0; b < B; ++b) {
      double g = dot_row(W + j * K, X + b * K, K);
      double u = dot_row(W + (Nh + j) * K, X + b * K, K);
      act[b * Nh + j] = silu(g) * u;
    }
  });
}
double orc_silu(double g) { return silu(g); }

// ---- argmax with total order: larger value wins, equal values -> lower index,
// NaN never wins, all-NaN (or V == 0) -> 0.  Also returns top1 - top2.
void orc_argmax(const double* logits, int64_t B, int64_t V, int32_t* tok,
                double* margin) {
  for (int64_t b = 0; b < B; ++b) {
    const double* l = logits + b * V;
    int64_t best = -1;
    for (int64_t v = 0; v < V; ++v) {
      if (std::isnan(l[v])) continue;
      if (best < 0 || l[v] > l[best]) best = v;
    }
    tok[b] = best < 0 ? 0 : static_cast<int32_t>(best);
    if (margin) {
      double second = -std::numeric_limits<double>::infinity();
      for (int64_t v = 0; v < V; ++v)
        if (v != best && !std::isnan(l[v]) && l[v] > second) second = l[v];
      margin[b] = (best < 0 || V < 2) ? std::numeric_limits<double>::infinity()
                                      : l[best] - second;
    }
  }
}

// ---- LM head: logits (double, never rounded) + greedy token ---------------------
void orc_lmhead_argmax(const uint16_t* W, const uint16_t* H, int64_t B, int64_t V,
                       int64_t K, double* logits_or_null, int32_t* tok,
                       double* margin_or_null, int threads) {
  std::vector<double> tmp;
  double* lg = logits_or_null;
  if (!lg) {
    tmp.resize(static_cast<size_t>(B) * V);
    lg = tmp.data();
  }
  orc_gemv(W, H, B, V, K, lg, threads);
  orc_argmax(lg, B, V, tok, margin_or_null);
}

// ---- embedding gather ------------------------------------------------------------
void orc_gather(const uint16_t* E, const int32_t* tok, int64_t B, int64_t K,
                uint16_t* Hout) {
  for (int64_t b = 0; b < B; ++b)
    std::memcpy(Hout + b * K, E + static_cast<int64_t>(tok[b]) * K, sizeof(uint16_t) * K);
}

// ---- GEMM sample: C[i,j] = sum_k A[i,k] B[j,k] for listed rows x all columns ----
void orc_gemm_rows(const uint16_t* A, const uint16_t* Bm, int64_t N, int64_t K,
                   const int64_t* rows, int64_t nrows, double* out, int threads) {
  parallel_rows(nrows * N, threads, [=](int64_t t) {
    int64_t i = rows[t / N], j = t % N;
    out[t] = dot_row(A + i * K, Bm + j * K, K);
  });
}
// ... and for listed columns x all rows (out is [ncols, M]).
void orc_gemm_cols(const uint16_t* A, const uint16_t* Bm, int64_t M, int64_t K,
                   const int64_t* cols, int64_t ncols, double* out, int threads) {
  parallel_rows(ncols * M, threads, [=](int64_t t) {
    int64_t j = cols[t / M], i = t % M;
    out[t] = dot_row(A + i * K, Bm + j * K, K);
  });
}

// ---- softmax probability of a given token (Sec. 7.2: the decode replay records the
// softmax probability of the sampled token next to the token itself) -----------------
// p[b] = exp(l[b, tok[b]]) / sum_v exp(l[b, v]), evaluated as exp(l - m) with m the row
// maximum (the shift cancels; it only keeps exp in range).  logits: [B, V] float (the
// fp32 logits a launch stored, taken as exact values).  A token outside [0, V) gives 0.
void orc_softmax_prob(const float* logits, const int32_t* tok, int64_t B, int64_t V, double* p) {
  for (int64_t b = 0; b < B; ++b) {
    const float* l = logits + b * V;
    double m = -INFINITY;
    for (int64_t v = 0; v < V; ++v)
      if (static_cast<double>(l[v]) > m) m = l[v];
    double sum = 0.0;
    for (int64_t v = 0; v < V; ++v) sum += std::exp(static_cast<double>(l[v]) - m);
    const int64_t t = tok[b];
    p[b] = (t >= 0 && t < V) ? std::exp(static_cast<double>(l[t]) - m) / sum : 0.0;
  }
}

// ---- one decode step of the Llama-shaped chain -----------------------------------
// Rounds to bf16 exactly where the chain stores a bf16 tensor between two
// launches; everything between two such points is evaluated in double.
//   h0 = E[tok]; n = bf16(rmsnorm(h0)); qkv = bf16(Wqkv n); a = qkv[0:D];
//   o = bf16(Wo a); act = bf16(silu(Wg o) * (Wu o)); d = bf16(Wd act);
//   logits = Wlm d (kept in double); next = argmax.
// Every intermediate is optional output (null = not wanted).
void orc_decode_step(const uint16_t* E, const uint16_t* gamma, const uint16_t* Wqkv,
                     const uint16_t* Wo, const uint16_t* Wgu, const uint16_t* Wd,
                     const uint16_t* Wlm, const int32_t* tok, int64_t B, int64_t D,
                     int64_t Nqkv, int64_t F, int64_t V, double eps,
                     uint16_t* h0_out, uint16_t* n_out, uint16_t* qkv_out,
                     uint16_t* o_out, uint16_t* act_out, uint16_t* d_out,
                     double* logits_out, int32_t* next_tok, double* margin,
                     int threads) {
  std::vector<uint16_t> h0(B * D), nn(B * D), qkv(B * Nqkv), a(B * D), o(B * D),
      act(B * F), d(B * D);
  std::vector<double> t(static_cast<size_t>(B) * std::max({D, Nqkv, F}));
  orc_gather(E, tok, B, D, h0.data());
  orc_rmsnorm(h0.data(), gamma, B, D, eps, t.data(), threads);
  orc_f64_to_bf16(t.data(), B * D, nn.data());
  orc_gemv(Wqkv, nn.data(), B, Nqkv, D, t.data(), threads);
  orc_f64_to_bf16(t.data(), B * Nqkv, qkv.data());
  for (int64_t b = 0; b < B; ++b)
    std::memcpy(a.data() + b * D, qkv.data() + b * Nqkv, sizeof(uint16_t) * D);
  orc_gemv(Wo, a.data(), B, D, D, t.data(), threads);
  orc_f64_to_bf16(t.data(), B * D, o.data());
  orc_gemv_silu_mul(Wgu, o.data(), B, F, D, t.data(), threads);
  orc_f64_to_bf16(t.data(), B * F, act.data());
  orc_gemv(Wd, act.data(), B, D, F, t.data(), threads);
  orc_f64_to_bf16(t.data(), B * D, d.data());
  orc_lmhead_argmax(Wlm, d.data(), B, V, D, logits_out, next_tok, margin, threads);
  auto put = [](uint16_t* dst, const std::vector<uint16_t>& src) {
    if (dst) std::memcpy(dst, src.data(), src.size() * sizeof(uint16_t));
  };
  put(h0_out, h0); put(n_out, nn); put(qkv_out, qkv); put(o_out, o);
  put(act_out, act); put(d_out, d);
}

}  // extern "C"
