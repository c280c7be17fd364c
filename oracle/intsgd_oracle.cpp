// IntSGD CPU oracle -- TEST INFRASTRUCTURE ONLY.
//
// A plain, single-threaded, deliberately slow C++ implementation of one IntSGD
// step, written from the paper's definitions (arXiv 2102.08374): the randomized
// integer rounding Int(t) of Section 2, the scaled integer message and its
// aggregate / decode / SGD update of Section 2.2 and Algorithm 1, the moving
// average r_k and the adaptive scaling factor alpha_k of Section 4.1
// (Proposition 2), and the block-wise rule of Appendix A.1 (Algorithm 2).
//
// Nothing in the product library may include, link or call this file; only the
// test-suite, the smoke check and the benchmark's cpu_baseline leg use it.  It
// shares no code with the HIP path.  Every function works on a coordinate slice
// [j0, j0+len) of the flat model vector so that a test can check any part of a
// large vector: all per-coordinate quantities depend only on the GLOBAL index j.
//
// Arithmetic contract (where the paper leaves precision open, the reading is
// fixed here):
//   * scale: one IEEE fp32 multiply alpha_f * g (the paper's gradients are fp32);
//   * deterministic rounding: round-half-to-even (the paper names torch.round);
//   * randomized rounding: floor(t) + [u < t - floor(t)], u a 24-bit uniform
//     drawn from Philox4x32-10 (Salmon et al., SC'11) at counter
//     (lo32(j/4), hi32(j/4), worker, step), key (lo32(seed), hi32(seed)),
//     word j mod 4;
//   * clip: the rounded value saturates to [-L, L]; every saturated or
//     non-finite worker-coordinate is counted (Section 5.1: local values are
//     clipped so that the aggregate fits the wire type);
//   * aggregate: exact integer sum over workers (Algorithm 1, aggregation line);
//   * decode + update in fp64, one rounding to fp32 (Algorithm 1, last two lines);
//   * update norm of the STORED fp32 iterates, accumulated in fp64;
//   * r_k, alpha_k in fp64, alpha stored as fp32 (Algorithm 1 / Algorithm 2).
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

namespace {

// Philox4x32 constants from the generator's published description.
constexpr uint32_t kMul0 = 0xD2511F53u;
constexpr uint32_t kMul1 = 0xCD9E8D57u;
constexpr uint32_t kWeyl0 = 0x9E3779B9u;
constexpr uint32_t kWeyl1 = 0xBB67AE85u;

// Index l of the block that holds global coordinate j, i.e. offsets[l] <= j <
// offsets[l+1] (offsets has B+1 entries, offsets[0] = 0, strictly increasing).
uint32_t block_of(uint64_t j, const uint64_t* offsets, uint32_t B) {
  if (B <= 1 || offsets == nullptr) return 0;
  const uint64_t* first_greater = std::upper_bound(offsets, offsets + B + 1, j);
  return (uint32_t)(first_greater - offsets) - 1;
}

}  // namespace

extern "C" {

// Philox4x32 with 10 rounds: counter c[4], key k[2] -> out[4].
void oracle_philox4x32_10(const uint32_t* c, const uint32_t* k, uint32_t* out) {
  uint32_t c0 = c[0], c1 = c[1], c2 = c[2], c3 = c[3];
  uint32_t k0 = k[0], k1 = k[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += kWeyl0;
      k1 += kWeyl1;
    }
    const uint64_t p0 = (uint64_t)kMul0 * (uint64_t)c0;
    const uint64_t p1 = (uint64_t)kMul1 * (uint64_t)c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    const uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The 32 random bits that belong to (seed, step, worker, global coordinate j).
uint32_t oracle_random_word(uint64_t seed, uint32_t step, uint32_t worker, uint64_t j) {
  const uint64_t quad = j >> 2;
  const uint32_t ctr[4] = {(uint32_t)quad, (uint32_t)(quad >> 32), worker, step};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  oracle_philox4x32_10(ctr, key, out);
  return out[j & 3];
}

// Int(t) of Section 2 for one value, given its 32 random bits: floor(t)+1 with
// probability t-floor(t), else floor(t).  Returned as an (integer-valued) float.
float oracle_int_random(float t, uint32_t word) {
  const float f = std::floor(t);
  const float p = t - f;                                  // p_t = t - [t]
  const float u = (float)(word >> 8) * 0x1p-24f;          // uniform on the 2^-24 grid of [0,1)
  return f + ((u < p) ? 1.0f : 0.0f);
}

// Deterministic variant of Section 5.1: round to nearest, ties to even.
float oracle_int_nearest(float t) { return std::nearbyintf(t); }

// Saturate an integer-valued float to [-L, L]; *clipped is set when it did not fit
// (or was NaN, which maps to 0).
int32_t oracle_saturate(float r, int32_t L, int* clipped) {
  const double rd = (double)r;
  *clipped = 0;
  if (std::isnan(rd)) { *clipped = 1; return 0; }
  if (rd > (double)L) { *clipped = 1; return L; }
  if (rd < -(double)L) { *clipped = 1; return -L; }
  return (int32_t)rd;
}

// Algorithm 1 "scale and round the local gradient" (Algorithm 2 with B > 1) for
// one worker on the slice [j0, j0+len).  g and q hold len entries (slice-local);
// alpha has B entries; offsets are global.  rounding: 0 nearest-even, 1 random.
// Returns the number of clipped worker-coordinates.
uint64_t oracle_compress(const float* g, uint64_t j0, uint64_t len, const float* alpha,
                         const uint64_t* offsets, uint32_t B, int rounding, int32_t L,
                         uint64_t seed, uint32_t step, uint32_t worker, int32_t* q) {
  uint64_t count = 0;
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    const uint64_t j = j0 + t_;
    const float a = alpha[block_of(j, offsets, B)];
    const float t = a * g[t_];                            // alpha_k o g_i^k, fp32
    float r;
    if (rounding == 1) {
      r = oracle_int_random(t, oracle_random_word(seed, step, worker, j));
    } else {
      r = oracle_int_nearest(t);
    }
    int clipped;
    q[t_] = oracle_saturate(r, L, &clipped);
    count += (uint64_t)clipped;
  }
  return count;
}

// Algorithm 1 aggregation line: S[j] = sum_i q_i[j], exact.  Returns the number
// of coordinates whose exact sum does not fit int32 (0 when n*L <= INT32_MAX);
// those are stored wrapped.
uint64_t oracle_int_sum(const int32_t* const* q, uint32_t n, uint64_t len, int32_t* sum) {
  uint64_t overflow = 0;
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    int64_t s = 0;
    for (uint32_t i = 0; i < n; ++i) s += (int64_t)q[i][t_];
    if (s > INT32_MAX || s < INT32_MIN) ++overflow;
    sum[t_] = (int32_t)(uint32_t)(uint64_t)s;
  }
  return overflow;
}

// Algorithm 1: g~ = S / (n alpha_k), x^{k+1} = x^k - eta_k g~ (per block alpha in
// Algorithm 2).  fp64 throughout, one rounding to fp32.  gtilde may be null.
void oracle_decode_update(const int32_t* sum, uint64_t j0, uint64_t len, const float* alpha,
                          const uint64_t* offsets, uint32_t B, uint32_t n, double eta,
                          const float* x, float* x_new, float* gtilde) {
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    const uint64_t j = j0 + t_;
    const double a = (double)alpha[block_of(j, offsets, B)];
    const double na = (double)n * a;
    const double c = eta / na;
    const double s = (double)sum[t_];
    if (gtilde) gtilde[t_] = (float)(s / na);
    const double prod = c * s;
    x_new[t_] = (float)((double)x[t_] - prod);
  }
}

// Momentum / weight-decay form of the update line (the optimizer of Section 5's
// experiments: SGD with momentum 0.9 and weight decay 1e-4; the paper's code is
// PyTorch, whose SGD rule this is).  Per coordinate, in fp64 with each operation
// rounded on its own, the two state vectors stored in fp32:
//   g~ = S * (1 / (n alpha));  dd = g~ + wd x;  m' = fl32(mu m + dd);  x' = fl32(x - eta m').
void oracle_decode_update_momentum(const int32_t* sum, uint64_t j0, uint64_t len,
                                   const float* alpha, const uint64_t* offsets, uint32_t B,
                                   uint32_t n, double eta, double mu, double wd, const float* x,
                                   const float* m, float* x_new, float* m_new) {
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    const uint64_t j = j0 + t_;
    const double a = (double)alpha[block_of(j, offsets, B)];
    const double cg = 1.0 / ((double)n * a);
    const double gt = cg * (double)sum[t_];
    const double decay = wd * (double)x[t_];
    const double dd = gt + decay;
    const double carried = mu * (double)m[t_];
    const float mn = (float)(carried + dd);
    const double stepv = eta * (double)mn;
    m_new[t_] = mn;
    x_new[t_] = (float)((double)x[t_] - stepv);
  }
}

// ||(x^{k+1})_l - (x^k)_l||^2 per block over the slice, ADDED into normsq[B]
// (the caller zeroes it), so slices can be accumulated.
void oracle_update_norm(const float* x_new, const float* x_old, uint64_t j0, uint64_t len,
                        const uint64_t* offsets, uint32_t B, double* normsq) {
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    const uint64_t j = j0 + t_;
    const double delta = (double)x_new[t_] - (double)x_old[t_];
    normsq[block_of(j, offsets, B)] += delta * delta;
  }
}

// Moving average and scaling factor.  B == 1: Algorithm 1,
//   r = beta r + (1-beta) normsq,  alpha = sqrt(d) / sqrt(2 n r / eta^2 + eps^2).
// B > 1: Algorithm 2, per block l of size d_l,
//   alpha_l = eta sqrt(d_l) / sqrt(2 n r_l + eta^2 (d_l/d) eps^2).
// r is updated in place; alpha_d (may be null) receives the fp64 values and
// alpha_f their fp32 roundings.  Returns 0, or 1 if some denominator was zero.
int oracle_next_alpha(const double* normsq, double* r, uint32_t B, const uint64_t* offsets,
                      uint64_t d, uint32_t n, double beta, double eps, double eta,
                      double* alpha_d, float* alpha_f) {
  int bad = 0;
  for (uint32_t l = 0; l < B; ++l) {
    r[l] = beta * r[l] + (1.0 - beta) * normsq[l];
    double a;
    if (B == 1) {
      const double den = 2.0 * (double)n * r[0] / (eta * eta) + eps * eps;
      if (den == 0.0) bad = 1;
      a = std::sqrt((double)d) / std::sqrt(den);
    } else {
      const double dl = (double)(offsets[l + 1] - offsets[l]);
      const double den = 2.0 * (double)n * r[l] + eta * eta * (dl / (double)d) * eps * eps;
      if (den == 0.0) bad = 1;
      a = eta * std::sqrt(dl) / std::sqrt(den);
    }
    if (alpha_d) alpha_d[l] = a;
    alpha_f[l] = (float)a;
  }
  return bad;
}

// One whole step on a slice, in the order of Algorithm 1: every worker scales and
// rounds, the integers are summed, decoded, the model is updated, and the update
// norm of the slice is added into normsq[B].  grads: n pointers to len floats.
// sat_count: n entries, overwritten.  sum_out (len int32) may be null.
// Returns the int-sum overflow count (0 in every valid configuration).
uint64_t oracle_step(const float* const* grads, uint32_t n, uint64_t j0, uint64_t len,
                     const float* alpha, const uint64_t* offsets, uint32_t B, int rounding,
                     int32_t L, uint64_t seed, uint32_t step, double eta, const float* x,
                     float* x_new, int32_t* sum_out, uint64_t* sat_count, double* normsq) {
  std::vector<std::vector<int32_t>> q(n, std::vector<int32_t>(len));
  std::vector<const int32_t*> qp(n);
  for (uint32_t i = 0; i < n; ++i) {
    sat_count[i] = oracle_compress(grads[i], j0, len, alpha, offsets, B, rounding, L, seed,
                                   step, i, q[i].data());
    qp[i] = q[i].data();
  }
  std::vector<int32_t> local_sum;
  int32_t* s = sum_out;
  if (!s) { local_sum.resize(len); s = local_sum.data(); }
  const uint64_t overflow = oracle_int_sum(qp.data(), n, len, s);
  oracle_decode_update(s, j0, len, alpha, offsets, B, n, eta, x, x_new, nullptr);
  oracle_update_norm(x_new, x, j0, len, offsets, B, normsq);
  return overflow;
}

// IntDIANA (Appendix A.2, Algorithm 3), worker side, for one worker on a slice: the
// worker compresses the DIFFERENCE to its local shift, Q_i = Int(alpha (g_i - h_i))
// (clipped like every integer message), and moves the shift by the decoded message,
// h_i <- h_i + Q_i / alpha.  (The algorithm box writes h_i + Q(g_i); its proofs use
// g = (1/n) sum (h_i + Q(g_i)), so Q there carries the 1/alpha of eq. (Q).)
// fp32: delta = g - h_i, t = alpha delta.  fp64: h_i + q (1/alpha), stored fp32.
uint64_t oracle_diana_compress(const float* g, const float* h_local, uint64_t j0, uint64_t len,
                               const float* alpha, const uint64_t* offsets, uint32_t B,
                               int rounding, int32_t L, uint64_t seed, uint32_t step,
                               uint32_t worker, int32_t* q, float* h_local_new) {
  uint64_t count = 0;
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    const uint64_t j = j0 + t_;
    const float a = alpha[block_of(j, offsets, B)];
    const float delta = g[t_] - h_local[t_];
    const float t = a * delta;
    float r;
    if (rounding == 1) {
      r = oracle_int_random(t, oracle_random_word(seed, step, worker, j));
    } else {
      r = oracle_int_nearest(t);
    }
    int clipped;
    q[t_] = oracle_saturate(r, L, &clipped);
    count += (uint64_t)clipped;
    const double inv = 1.0 / (double)a;
    const double moved = (double)q[t_] * inv;
    h_local_new[t_] = (float)((double)h_local[t_] + moved);
  }
  return count;
}

// IntDIANA, after aggregation: g~ = h + S/(n alpha), x <- x - eta g~, h <- h + S/(n alpha)
// (Algorithm 3, estimator / update / global-shift lines).  fp64, each operation
// rounded on its own, x and h stored fp32.
void oracle_diana_update(const int32_t* sum, uint64_t j0, uint64_t len, const float* alpha,
                         const uint64_t* offsets, uint32_t B, uint32_t n, double eta,
                         const float* x, const float* h, float* x_new, float* h_new) {
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    const uint64_t j = j0 + t_;
    const double a = (double)alpha[block_of(j, offsets, B)];
    const double cg = 1.0 / ((double)n * a);
    const double ghat = cg * (double)sum[t_];
    const double gt = (double)h[t_] + ghat;
    const double stepv = eta * gt;
    x_new[t_] = (float)((double)x[t_] - stepv);
    h_new[t_] = (float)gt;
  }
}

// One whole IntDIANA step on a slice.  h_local / h_local_new: n pointers to len floats.
uint64_t oracle_diana_step(const float* const* grads, const float* const* h_local, uint32_t n,
                           uint64_t j0, uint64_t len, const float* alpha, const uint64_t* offsets,
                           uint32_t B, int rounding, int32_t L, uint64_t seed, uint32_t step,
                           double eta, const float* x, const float* h, float* x_new, float* h_new,
                           float* const* h_local_new, int32_t* sum_out, uint64_t* sat_count,
                           double* normsq) {
  std::vector<std::vector<int32_t>> q(n, std::vector<int32_t>(len));
  std::vector<const int32_t*> qp(n);
  for (uint32_t i = 0; i < n; ++i) {
    sat_count[i] = oracle_diana_compress(grads[i], h_local[i], j0, len, alpha, offsets, B,
                                         rounding, L, seed, step, i, q[i].data(), h_local_new[i]);
    qp[i] = q[i].data();
  }
  std::vector<int32_t> local_sum;
  int32_t* s = sum_out;
  if (!s) { local_sum.resize(len); s = local_sum.data(); }
  const uint64_t overflow = oracle_int_sum(qp.data(), n, len, s);
  oracle_diana_update(s, j0, len, alpha, offsets, B, n, eta, x, h, x_new, h_new);
  oracle_update_norm(x_new, x, j0, len, offsets, B, normsq);
  return overflow;
}

// The largest integer in the aggregate (Appendix A.2 reports, per iteration, the max integer
// in the aggregated vector sum_i Q(g_i); the discussion of IntDIANA is about keeping it
// bounded): max_j |S_j| per block over a slice, as a running maximum in `largest` (uint32:
// |S_j| <= n L <= 2^31 - 1, and |INT32_MIN| = 2^31 still fits).
void oracle_max_abs_sum(const int32_t* sum, uint64_t j0, uint64_t len, const uint64_t* offsets,
                        uint32_t B, uint32_t* largest) {
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    const int64_t v = (int64_t)sum[t_];
    const uint32_t mag = (uint32_t)(v < 0 ? -v : v);
    uint32_t& slot = largest[block_of(j0 + t_, offsets, B)];
    if (mag > slot) slot = mag;
  }
}

// Heuristic IntSGD scaling (Section 5.2; the SwitchML rule the paper compares with):
// alpha = (2^nb - 1) / (n 2^max_exp), max_exp the exponent of the largest absolute value
// in the package, read here as the smallest integer e with 2^e >= max|g| over all n
// workers and all coordinates of the block (so that |alpha g| <= (2^nb - 1)/n).
// Step 1, the profiling pass: running maximum of |g| per block over a slice; non-finite
// entries are skipped (they are clipped and counted later anyway).
void oracle_max_abs(const float* g, uint64_t j0, uint64_t len, const uint64_t* offsets, uint32_t B,
                    float* max_abs) {
  for (uint64_t t_ = 0; t_ < len; ++t_) {
    const float v = std::fabs(g[t_]);
    if (!std::isfinite(v)) continue;
    float& slot = max_abs[block_of(j0 + t_, offsets, B)];
    if (v > slot) slot = v;
  }
}

// Step 2: the scaling factors.  An all-zero block gets alpha = 1 (every alpha gives zero
// integers there); alpha is capped at the largest finite fp32 number.
void oracle_heuristic_alpha(const float* max_abs, uint32_t B, uint32_t n, uint32_t nb,
                            double* alpha_d, float* alpha_f) {
  for (uint32_t l = 0; l < B; ++l) {
    double a = 1.0;
    if (max_abs[l] > 0.0f) {
      int e = 0;
      const double frac = std::frexp((double)max_abs[l], &e);    // max = frac 2^e, frac in [0.5, 1)
      const int max_exp = (frac == 0.5) ? e - 1 : e;              // smallest e with 2^e >= max
      const double top = std::ldexp(1.0, (int)nb) - 1.0;
      a = std::ldexp(top / (double)n, -max_exp);
      if (a > (double)std::numeric_limits<float>::max()) a = (double)std::numeric_limits<float>::max();
    }
    if (alpha_d) alpha_d[l] = a;
    alpha_f[l] = (float)a;
  }
}

// oracle_step with the momentum / weight-decay update in place of the plain one.
uint64_t oracle_step_momentum(const float* const* grads, uint32_t n, uint64_t j0, uint64_t len,
                              const float* alpha, const uint64_t* offsets, uint32_t B,
                              int rounding, int32_t L, uint64_t seed, uint32_t step, double eta,
                              double mu, double wd, const float* x, const float* m, float* x_new,
                              float* m_new, int32_t* sum_out, uint64_t* sat_count,
                              double* normsq) {
  std::vector<std::vector<int32_t>> q(n, std::vector<int32_t>(len));
  std::vector<const int32_t*> qp(n);
  for (uint32_t i = 0; i < n; ++i) {
    sat_count[i] = oracle_compress(grads[i], j0, len, alpha, offsets, B, rounding, L, seed,
                                   step, i, q[i].data());
    qp[i] = q[i].data();
  }
  std::vector<int32_t> local_sum;
  int32_t* s = sum_out;
  if (!s) { local_sum.resize(len); s = local_sum.data(); }
  const uint64_t overflow = oracle_int_sum(qp.data(), n, len, s);
  oracle_decode_update_momentum(s, j0, len, alpha, offsets, B, n, eta, mu, wd, x, m, x_new, m_new);
  oracle_update_norm(x_new, x, j0, len, offsets, B, normsq);
  return overflow;
}

}  // extern "C"
