// CO2 outer-update oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, slow, single-threaded CPU statement of what one CO2 worker computes
// once its tau local steps have finished (CO2 paper, Algorithm 1, the three
// update lines after the wait on the previous asynchronous all-reduce;
// Definition 3.1 / Eq. 3 for the staleness gap; Section 3.3 for Clip), plus the
// base optimizer's local update (Algorithm 1, "LU" line, with AdamW as the base
// optimizer, Section 4.1).  Only tests, the smoke check and the bench's CPU
// baseline may call it.  It shares no code, header, table or helper with the
// HIP library and is compiled by g++ with -O2 -ffp-contract=off so that every
// fp32 product and sum below is rounded once, as written.
//
// Two evaluations are given for every update:
//   *_f32 : the arithmetic type of the device path (fp32 elementwise work,
//           fp64 for the two norms and the per-segment scalar Lambda);
//   *_f64 : everything in fp64 ("truth"), used to bound the fp32 evaluation's
//           own rounding error.
//
// Readings taken where the paper is silent:
//   * ||.|| in Eq. 3 is the L2 norm over one parameter tensor ("segment"),
//     and Lambda is broadcast over that tensor's coordinates.  S = n gives the
//     per-coordinate reading, S = 1 the global one.
//   * Numerator ||x_{t,0} - x_{t-1,0}||: by Algorithm 1's last line one round
//     earlier this difference is -alpha*Clip(m_{t-1}, phi), so it is formed as
//     alpha * ||Clip(m_{t-1}, phi)|| from the momentum *before* its update.
//   * Denominator tau*||x_{t-1,1} - x_{t-1,0}||: the per-segment first-inner-
//     step norms are an input (first_step_norm); when absent, the norm of the
//     worker's own previous pseudo-gradient (deltas[0]) stands for the whole
//     product tau*||first step||.
//   * A coefficient c scales the ratio: Lambda = c*ratio + 1 (c = 1 is the
//     paper, c = 0 is its "w/o penalty" ablation).  A zero denominator gives
//     Lambda = 1.
//   * Outer round t = 0 skips the gap, momentum and iterate lines (Section
//     3.1): x_{1,0} = x_{0,0}, m stays 0.
//
// parity pins: tests/test_oracle_*.py (hand-expanded examples, closed forms,
// invariants, library momentum SGD / AdamW / lerp / clip_grad_norm_).  Nothing
// here is "parity unpinned".

#include <cmath>
#include <cstddef>
#include <cstdint>

namespace {

// Section 3.3: Clip(chi, phi) = max{-phi, min{chi, phi}}, coordinate-wise.
template <typename T>
inline T clip_coord(T chi, T phi) {
  T lo = (chi < phi) ? chi : phi;      // min{chi, phi}
  return (lo > -phi) ? lo : -phi;      // max{-phi, .}
}

inline int check_table(int64_t n, int32_t S, const int64_t* seg_off) {
  if (n < 0 || S < 1 || seg_off == nullptr) return -1;
  if (seg_off[0] != 0 || seg_off[S] != n) return -1;
  for (int32_t s = 0; s < S; ++s)
    if (seg_off[s + 1] < seg_off[s]) return -1;
  return 0;
}

}  // namespace

extern "C" {

// Per-segment sum of squares of one buffer, fp64 accumulation in ascending
// index order (the quantity under the root of either norm in Eq. 3).
// If phi > 0 the value is clipped coordinate-wise in fp32 first.
int co2_oracle_sqnorms(int64_t n, int32_t S, const int64_t* seg_off,
                       const float* buf, float phi, double* out) {
  if (check_table(n, S, seg_off) || !buf || !out) return -1;
  for (int32_t s = 0; s < S; ++s) {
    double acc = 0.0;
    for (int64_t j = seg_off[s]; j < seg_off[s + 1]; ++j) {
      float v = buf[j];
      if (phi > 0.0f) v = clip_coord<float>(v, phi);
      double dv = static_cast<double>(v);
      acc += dv * dv;
    }
    out[s] = acc;
  }
  return 0;
}

// One outer update, fp32-ordered evaluation.
//
//   x      in: x^{(i)}_{t,tau} (local params after the inner loop)
//          out: x_{t+1,0}.  May be NULL ("split form": only m and the next
//          anchor are produced; then dout must be NULL as well).
//   a_in   x_{t,0}; a_out receives x_{t+1,0} (may be the same array as a_in).
//   m      in: m_{t-1}; out: m_t.
//   d      K arrays: round t-1's pseudo-gradients x_{t-1,0} - x^{(k)}_{t-1,tau}
//          of the K workers (their mean is what the all-reduce delivers).
//   dout   out: x_{t,0} - x^{(i)}_{t,tau}, this round's pseudo-gradient (the
//          payload of the all-reduce launched now).
//   first_step_norm  NULL, or S values ||x_{t-1,1} - x_{t-1,0}||_s.
//   lambda_out, M2_out, T_out: optional S-vectors for inspection
//          (Lambda, sum Clip(m_{t-1})^2, the denominator).
//   nclipped: optional, number of coordinates with |m_t| > phi.
int co2_oracle_outer_step_f32(int64_t n, int32_t S, const int64_t* seg_off,
                              int32_t K, float alpha, float beta, float phi,
                              float c, int32_t tau, int64_t step,
                              float* x, const float* a_in, float* a_out,
                              float* m, const float* const* d, float* dout,
                              const float* first_step_norm,
                              float* lambda_out, double* M2_out, double* T_out,
                              int64_t* nclipped) {
  if (check_table(n, S, seg_off) || !a_in || !a_out || !m) return -1;
  if ((x == nullptr) != (dout == nullptr)) return -1;
  if (K < 1 || tau < 1 || !(phi > 0.0f) || step < 0) return -1;
  if (nclipped) *nclipped = 0;

  if (step == 0) {
    // First outer iteration: the AAR is launched, nothing else happens.
    for (int64_t j = 0; j < n; ++j) {
      float aj = a_in[j];
      if (x) { dout[j] = aj - x[j]; x[j] = aj; }
      a_out[j] = aj;
    }
    for (int32_t s = 0; s < S; ++s) {
      if (lambda_out) lambda_out[s] = 1.0f;
      if (M2_out) M2_out[s] = 0.0;
      if (T_out) T_out[s] = 0.0;
    }
    return 0;
  }
  if (!d) return -1;
  for (int32_t k = 0; k < K; ++k) if (!d[k]) return -1;

  const float rK = static_cast<float>(1.0 / static_cast<double>(K));

  for (int32_t s = 0; s < S; ++s) {
    const int64_t lo = seg_off[s], hi = seg_off[s + 1];

    // Eq. 3 numerator: ||x_{t,0} - x_{t-1,0}||_s = alpha*||Clip(m_{t-1},phi)||_s.
    double M2 = 0.0;
    for (int64_t j = lo; j < hi; ++j) {
      double cm = static_cast<double>(clip_coord<float>(m[j], phi));
      M2 += cm * cm;
    }
    // Eq. 3 denominator: tau*||x_{t-1,1} - x_{t-1,0}||_s.
    double T;
    if (first_step_norm) {
      T = static_cast<double>(tau) * static_cast<double>(first_step_norm[s]);
    } else {
      double P2 = 0.0;
      for (int64_t j = lo; j < hi; ++j) {
        double dv = static_cast<double>(d[0][j]);
        P2 += dv * dv;
      }
      T = std::sqrt(P2);
    }
    // Lambda_t = c * numerator / denominator + 1  (Algorithm 1, gap update).
    double Lam = 1.0;
    if (c != 0.0f && T != 0.0) {
      Lam = (static_cast<double>(c) * static_cast<double>(alpha)) * std::sqrt(M2) / T + 1.0;
    }
    const float inv = static_cast<float>(1.0 / Lam);
    if (lambda_out) lambda_out[s] = static_cast<float>(Lam);
    if (M2_out) M2_out[s] = M2;
    if (T_out) T_out[s] = T;

    for (int64_t j = lo; j < hi; ++j) {
      const float aj = a_in[j];
      // This round's local pseudo-gradient (what the new AAR carries).
      if (x) dout[j] = aj - x[j];
      // Mean of the K workers' round t-1 pseudo-gradients, left to right.
      float sum = d[0][j];
      for (int32_t k = 1; k < K; ++k) sum = sum + d[k][j];
      const float dbar = sum * rK;
      // m_t = beta*m_{t-1} + (1/Lambda_t)*(x_{t-1,0} - x_{t-1,tau}).
      const float bm = beta * m[j];
      const float pen = dbar * inv;
      const float mt = bm + pen;
      // x_{t+1,0} = x_{t,0} - alpha*Clip(m_t, phi).
      const float cm = clip_coord<float>(mt, phi);
      const float stepv = alpha * cm;
      const float xn = aj - stepv;
      if (nclipped && (mt > phi || mt < -phi)) ++*nclipped;
      m[j] = mt;
      if (x) x[j] = xn;
      a_out[j] = xn;
    }
  }
  return 0;
}

// The same update with every quantity in fp64.
int co2_oracle_outer_step_f64(int64_t n, int32_t S, const int64_t* seg_off,
                              int32_t K, double alpha, double beta, double phi,
                              double c, int32_t tau, int64_t step,
                              double* x, const double* a_in, double* a_out,
                              double* m, const double* const* d, double* dout,
                              const double* first_step_norm,
                              double* lambda_out) {
  if (check_table(n, S, seg_off) || !a_in || !a_out || !m) return -1;
  if ((x == nullptr) != (dout == nullptr)) return -1;
  if (K < 1 || tau < 1 || !(phi > 0.0) || step < 0) return -1;

  if (step == 0) {
    for (int64_t j = 0; j < n; ++j) {
      double aj = a_in[j];
      if (x) { dout[j] = aj - x[j]; x[j] = aj; }
      a_out[j] = aj;
    }
    if (lambda_out) for (int32_t s = 0; s < S; ++s) lambda_out[s] = 1.0;
    return 0;
  }
  if (!d) return -1;
  for (int32_t k = 0; k < K; ++k) if (!d[k]) return -1;

  for (int32_t s = 0; s < S; ++s) {
    const int64_t lo = seg_off[s], hi = seg_off[s + 1];
    double M2 = 0.0;
    for (int64_t j = lo; j < hi; ++j) {
      double cm = clip_coord<double>(m[j], phi);
      M2 += cm * cm;
    }
    double T;
    if (first_step_norm) {
      T = static_cast<double>(tau) * first_step_norm[s];
    } else {
      double P2 = 0.0;
      for (int64_t j = lo; j < hi; ++j) P2 += d[0][j] * d[0][j];
      T = std::sqrt(P2);
    }
    double Lam = 1.0;
    if (c != 0.0 && T != 0.0) Lam = c * alpha * std::sqrt(M2) / T + 1.0;
    if (lambda_out) lambda_out[s] = Lam;

    for (int64_t j = lo; j < hi; ++j) {
      const double aj = a_in[j];
      if (x) dout[j] = aj - x[j];
      double sum = 0.0;
      for (int32_t k = 0; k < K; ++k) sum += d[k][j];
      const double dbar = sum / static_cast<double>(K);
      const double mt = beta * m[j] + dbar / Lam;
      const double xn = aj - alpha * clip_coord<double>(mt, phi);
      m[j] = mt;
      if (x) x[j] = xn;
      a_out[j] = xn;
    }
  }
  return 0;
}

// ---------------------------------------------------------------------------
// The family of local-update outer rules CO2 is built on or compared with,
// stated in the buffers of the update above.  Three independent switches:
//
//   nonstale   The momentum line in the order of the method CO2 starts from
//              (Section 3.2, the recursion m_{t+1} = beta*m_t + (x_{t,0} - x_{t,tau})
//              written before the staleness is introduced): the mean is taken
//              over THIS round's pseudo-gradients, i.e. the worker's own
//              a - x formed in this call and the K-1 peers' in d[1..K-1]
//              (d[0] is not read).  Round 0 is then an ordinary round.  With
//              c = 0 and phi = +inf this is the slow-momentum update.
//   pull_rho   Local parameters after the update.  1: they restart from the new
//              outer iterate (Algorithm 1).  rho in (0,1): the anchor-model rule
//              of the overlap variant of local SGD the paper discusses (its
//              Discussions section): each worker keeps its own parameters and
//              is only pulled towards the anchor, x <- x - rho*(x - x_{t+1,0}),
//              while the anchor itself is updated as above.
//   norm_clip  Clipping by rescaling instead of Section 3.3's coordinate-wise
//              clamp (not in the paper; the usual alternative): per segment,
//              Clip_norm(m, phi) = m * min(1, phi/||m||_s).  The numerator of
//              Eq. 3 is then ||x_{t,0} - x_{t-1,0}||_s = alpha*min(||m_{t-1}||_s, phi).
//
// Every switch off reproduces co2_oracle_outer_step_f32 operation for operation.
//   scale_out  optional S values: the factor min(1, phi/||m_t||_s) (1 without norm_clip)
//   nclipped   coordinates with |m_t| > phi, or with norm_clip the number of
//              coordinates that lie in a rescaled segment.
int co2_oracle_outer_step_variant_f32(int64_t n, int32_t S, const int64_t* seg_off,
                                      int32_t K, float alpha, float beta, float phi,
                                      float c, int32_t tau, int64_t step,
                                      int32_t nonstale, int32_t norm_clip, float pull_rho,
                                      float* x, const float* a_in, float* a_out,
                                      float* m, const float* const* d, float* dout,
                                      const float* first_step_norm,
                                      float* lambda_out, float* scale_out,
                                      int64_t* nclipped) {
  if (check_table(n, S, seg_off) || !a_in || !a_out || !m) return -1;
  if ((x == nullptr) != (dout == nullptr)) return -1;
  if (K < 1 || tau < 1 || !(phi > 0.0f) || step < 0) return -1;
  if (!(pull_rho > 0.0f && pull_rho <= 1.0f)) return -1;
  if ((nonstale || pull_rho != 1.0f) && !x) return -1;     // both need the local parameters
  // No previous own pseudo-gradient is kept in the current-round order, so a
  // penalty there needs the first-inner-step norms.
  if (nonstale && c != 0.0f && !first_step_norm) return -1;
  if (nclipped) *nclipped = 0;

  if (step == 0 && !nonstale) {
    // Stale order, first round: only the pseudo-gradient is formed.
    for (int64_t j = 0; j < n; ++j) {
      float aj = a_in[j];
      if (x) { dout[j] = aj - x[j]; x[j] = aj; }
      a_out[j] = aj;
    }
    for (int32_t s = 0; s < S; ++s) {
      if (lambda_out) lambda_out[s] = 1.0f;
      if (scale_out) scale_out[s] = 1.0f;
    }
    return 0;
  }
  if (!d && (K > 1 || !nonstale)) return -1;
  for (int32_t k = nonstale ? 1 : 0; k < K; ++k) if (!d[k]) return -1;

  const float rK = static_cast<float>(1.0 / static_cast<double>(K));

  for (int32_t s = 0; s < S; ++s) {
    const int64_t lo = seg_off[s], hi = seg_off[s + 1];

    // Eq. 3 numerator: the displacement of the previous outer iterate.
    double M2 = 0.0;
    for (int64_t j = lo; j < hi; ++j) {
      double v = static_cast<double>(norm_clip ? m[j] : clip_coord<float>(m[j], phi));
      M2 += v * v;
    }
    double moved = std::sqrt(M2);                     // ||Clip(m_{t-1})||_s over alpha
    if (norm_clip && moved > static_cast<double>(phi)) moved = static_cast<double>(phi);
    // Eq. 3 denominator.
    double T;
    if (first_step_norm) {
      T = static_cast<double>(tau) * static_cast<double>(first_step_norm[s]);
    } else if (nonstale) {
      T = 0.0;                                        // c == 0 here: Lambda stays 1
    } else {
      double P2 = 0.0;
      for (int64_t j = lo; j < hi; ++j) {
        double dv = static_cast<double>(d[0][j]);
        P2 += dv * dv;
      }
      T = std::sqrt(P2);
    }
    double Lam = 1.0;
    if (c != 0.0f && T != 0.0) {
      Lam = (static_cast<double>(c) * static_cast<double>(alpha)) * moved / T + 1.0;
    }
    const float inv = static_cast<float>(1.0 / Lam);
    if (lambda_out) lambda_out[s] = static_cast<float>(Lam);

    // Momentum line; the squared norm of m_t is needed before the iterate
    // when clipping rescales.
    double Q = 0.0;
    for (int64_t j = lo; j < hi; ++j) {
      const float aj = a_in[j];
      if (x) dout[j] = aj - x[j];
      float sum = nonstale ? dout[j] : d[0][j];
      for (int32_t k = 1; k < K; ++k) sum = sum + d[k][j];
      const float dbar = sum * rK;
      const float bm = beta * m[j];
      const float pen = dbar * inv;
      const float mt = bm + pen;
      m[j] = mt;
      Q += static_cast<double>(mt) * static_cast<double>(mt);
    }
    float scale = 1.0f;
    if (norm_clip) {
      const double nrm = std::sqrt(Q);
      if (nrm > static_cast<double>(phi)) scale = static_cast<float>(static_cast<double>(phi) / nrm);
      if (nclipped && scale != 1.0f) *nclipped += hi - lo;
    }
    if (scale_out) scale_out[s] = scale;

    // Outer-iterate line, then what the local parameters become.
    for (int64_t j = lo; j < hi; ++j) {
      const float mt = m[j];
      const float cm = norm_clip ? mt * scale : clip_coord<float>(mt, phi);
      const float stepv = alpha * cm;
      const float xn = a_in[j] - stepv;
      if (!norm_clip && nclipped && (mt > phi || mt < -phi)) ++*nclipped;
      if (x) {
        if (pull_rho == 1.0f) {
          x[j] = xn;
        } else {
          const float gap = x[j] - xn;
          const float pull = pull_rho * gap;
          x[j] = x[j] - pull;
        }
      }
      a_out[j] = xn;
    }
  }
  return 0;
}

// ---------------------------------------------------------------------------
// Reduced-precision transport of the pseudo-gradients (the paper's Section 2,
// "Efficient Communication": compression of what the all-reduce carries is
// orthogonal to CO2 and can be combined with it).  The K incoming
// pseudo-gradients and the outgoing one are stored as bf16; all arithmetic stays
// fp32/fp64 exactly as above.

// fp32 -> bf16 bit pattern, round to nearest, ties to even; NaN stays NaN (quiet).
uint16_t co2_oracle_f32_to_bf16(float f) {
  union { float f; uint32_t u; } cv;
  cv.f = f;
  uint32_t u = cv.u;
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
  const uint32_t lsb = (u >> 16) & 1u;          // last kept bit decides ties
  u += 0x7fffu + lsb;
  return static_cast<uint16_t>(u >> 16);
}

// bf16 bit pattern -> fp32, exact.
float co2_oracle_bf16_to_f32(uint16_t b) {
  union { float f; uint32_t u; } cv;
  cv.u = static_cast<uint32_t>(b) << 16;
  return cv.f;
}

// One outer update with bf16 pseudo-gradient buffers: identical to
// co2_oracle_outer_step_f32 except that
//   d[k][j]  are bf16 bit patterns, widened exactly before use,
//   dout[j]  = bf16(a[j] - x[j])  (fp32 subtraction, then rounded once),
// and the own-delta norm of the NULL-first_step_norm case is taken over the
// widened values of d[0].
int co2_oracle_outer_step_bf16(int64_t n, int32_t S, const int64_t* seg_off,
                               int32_t K, float alpha, float beta, float phi,
                               float c, int32_t tau, int64_t step,
                               float* x, const float* a_in, float* a_out,
                               float* m, const uint16_t* const* d, uint16_t* dout,
                               const float* first_step_norm,
                               float* lambda_out, int64_t* nclipped) {
  if (check_table(n, S, seg_off) || !a_in || !a_out || !m) return -1;
  if ((x == nullptr) != (dout == nullptr)) return -1;
  if (K < 1 || tau < 1 || !(phi > 0.0f) || step < 0) return -1;
  if (nclipped) *nclipped = 0;

  if (step == 0) {
    for (int64_t j = 0; j < n; ++j) {
      float aj = a_in[j];
      if (x) { dout[j] = co2_oracle_f32_to_bf16(aj - x[j]); x[j] = aj; }
      a_out[j] = aj;
    }
    if (lambda_out) for (int32_t s = 0; s < S; ++s) lambda_out[s] = 1.0f;
    return 0;
  }
  if (!d) return -1;
  for (int32_t k = 0; k < K; ++k) if (!d[k]) return -1;

  const float rK = static_cast<float>(1.0 / static_cast<double>(K));
  for (int32_t s = 0; s < S; ++s) {
    const int64_t lo = seg_off[s], hi = seg_off[s + 1];
    double M2 = 0.0;
    for (int64_t j = lo; j < hi; ++j) {
      double cm = static_cast<double>(clip_coord<float>(m[j], phi));
      M2 += cm * cm;
    }
    double T;
    if (first_step_norm) {
      T = static_cast<double>(tau) * static_cast<double>(first_step_norm[s]);
    } else {
      double P2 = 0.0;
      for (int64_t j = lo; j < hi; ++j) {
        double dv = static_cast<double>(co2_oracle_bf16_to_f32(d[0][j]));
        P2 += dv * dv;
      }
      T = std::sqrt(P2);
    }
    double Lam = 1.0;
    if (c != 0.0f && T != 0.0) {
      Lam = (static_cast<double>(c) * static_cast<double>(alpha)) * std::sqrt(M2) / T + 1.0;
    }
    const float inv = static_cast<float>(1.0 / Lam);
    if (lambda_out) lambda_out[s] = static_cast<float>(Lam);

    for (int64_t j = lo; j < hi; ++j) {
      const float aj = a_in[j];
      if (x) dout[j] = co2_oracle_f32_to_bf16(aj - x[j]);
      float sum = co2_oracle_bf16_to_f32(d[0][j]);
      for (int32_t k = 1; k < K; ++k) sum = sum + co2_oracle_bf16_to_f32(d[k][j]);
      const float dbar = sum * rK;
      const float bm = beta * m[j];
      const float pen = dbar * inv;
      const float mt = bm + pen;
      const float cm = clip_coord<float>(mt, phi);
      const float stepv = alpha * cm;
      const float xn = aj - stepv;
      if (nclipped && (mt > phi || mt < -phi)) ++*nclipped;
      m[j] = mt;
      if (x) x[j] = xn;
      a_out[j] = xn;
    }
  }
  return 0;
}

// IEEE binary16 transport of the pseudo-gradients: the same as the bf16 case with
// the other 16-bit format (5 exponent bits, 10 fraction bits).
//
// fp32 -> binary16 bit pattern: round to nearest, ties to even; gradual underflow
// to subnormals (multiples of 2^-24) and zero; magnitudes that round to 2^16 or
// more become infinity; NaN stays a quiet NaN.
uint16_t co2_oracle_f32_to_f16(float f) {
  union { float f; uint32_t u; } cv;
  cv.f = f;
  const uint16_t sign = static_cast<uint16_t>((cv.u >> 16) & 0x8000u);
  const uint32_t mag = cv.u & 0x7fffffffu;
  if (mag > 0x7f800000u) return static_cast<uint16_t>(sign | 0x7e00u);      // NaN
  if (mag >= 0x47800000u) return static_cast<uint16_t>(sign | 0x7c00u);      // >= 2^16, infinity
  if (mag >= 0x38800000u) {                                                  // >= 2^-14: normal result
    uint32_t r = mag - 0x38000000u;               // exponent bias 127 -> 15
    const uint32_t lsb = (r >> 13) & 1u;          // last kept fraction bit decides ties
    r += 0x0fffu + lsb;
    return static_cast<uint16_t>(sign | (r >> 13));   // a carry out of the fraction reaches 0x7c00 = infinity
  }
  if (mag <= 0x33000000u) return sign;            // <= 2^-25: rounds to zero (2^-25 itself is a tie, even = 0)
  // subnormal result: count of 2^-24 units, rounded to nearest even
  const uint32_t e = mag >> 23;                   // 102 .. 112
  const uint32_t sig = (mag & 0x007fffffu) | 0x00800000u;
  const uint32_t shift = 126u - e;                // 14 .. 24
  uint32_t h = sig >> shift;
  const uint32_t rem = sig & ((1u << shift) - 1u);
  const uint32_t half = 1u << (shift - 1u);
  if (rem > half || (rem == half && (h & 1u))) ++h;
  return static_cast<uint16_t>(sign | h);         // h == 0x400 is the smallest normal, as it should be
}

// binary16 bit pattern -> fp32, exact.
float co2_oracle_f16_to_f32(uint16_t b) {
  union { float f; uint32_t u; } cv;
  const uint32_t sign = static_cast<uint32_t>(b & 0x8000u) << 16;
  const uint32_t e = (b >> 10) & 0x1fu;
  const uint32_t frac = b & 0x3ffu;
  if (e == 0x1fu) {
    cv.u = sign | 0x7f800000u | (frac << 13);
  } else if (e != 0u) {
    cv.u = sign | ((e + 112u) << 23) | (frac << 13);
  } else {
    cv.f = static_cast<float>(frac) * 5.9604644775390625e-08f;   // frac * 2^-24, exact
    cv.u |= sign;
  }
  return cv.f;
}

// One outer update with binary16 pseudo-gradient buffers: co2_oracle_outer_step_bf16
// with the conversions above.
int co2_oracle_outer_step_f16(int64_t n, int32_t S, const int64_t* seg_off,
                              int32_t K, float alpha, float beta, float phi,
                              float c, int32_t tau, int64_t step,
                              float* x, const float* a_in, float* a_out,
                              float* m, const uint16_t* const* d, uint16_t* dout,
                              const float* first_step_norm,
                              float* lambda_out, int64_t* nclipped) {
  if (check_table(n, S, seg_off) || !a_in || !a_out || !m) return -1;
  if ((x == nullptr) != (dout == nullptr)) return -1;
  if (K < 1 || tau < 1 || !(phi > 0.0f) || step < 0) return -1;
  if (nclipped) *nclipped = 0;

  if (step == 0) {
    for (int64_t j = 0; j < n; ++j) {
      float aj = a_in[j];
      if (x) { dout[j] = co2_oracle_f32_to_f16(aj - x[j]); x[j] = aj; }
      a_out[j] = aj;
    }
    if (lambda_out) for (int32_t s = 0; s < S; ++s) lambda_out[s] = 1.0f;
    return 0;
  }
  if (!d) return -1;
  for (int32_t k = 0; k < K; ++k) if (!d[k]) return -1;

  const float rK = static_cast<float>(1.0 / static_cast<double>(K));
  for (int32_t s = 0; s < S; ++s) {
    const int64_t lo = seg_off[s], hi = seg_off[s + 1];
    double M2 = 0.0;
    for (int64_t j = lo; j < hi; ++j) {
      double cm = static_cast<double>(clip_coord<float>(m[j], phi));
      M2 += cm * cm;
    }
    double T;
    if (first_step_norm) {
      T = static_cast<double>(tau) * static_cast<double>(first_step_norm[s]);
    } else {
      double P2 = 0.0;
      for (int64_t j = lo; j < hi; ++j) {
        double dv = static_cast<double>(co2_oracle_f16_to_f32(d[0][j]));
        P2 += dv * dv;
      }
      T = std::sqrt(P2);
    }
    double Lam = 1.0;
    if (c != 0.0f && T != 0.0) {
      Lam = (static_cast<double>(c) * static_cast<double>(alpha)) * std::sqrt(M2) / T + 1.0;
    }
    const float inv = static_cast<float>(1.0 / Lam);
    if (lambda_out) lambda_out[s] = static_cast<float>(Lam);

    for (int64_t j = lo; j < hi; ++j) {
      const float aj = a_in[j];
      if (x) dout[j] = co2_oracle_f32_to_f16(aj - x[j]);
      float sum = co2_oracle_f16_to_f32(d[0][j]);
      for (int32_t k = 1; k < K; ++k) sum = sum + co2_oracle_f16_to_f32(d[k][j]);
      const float dbar = sum * rK;
      const float bm = beta * m[j];
      const float pen = dbar * inv;
      const float mt = bm + pen;
      const float cm = clip_coord<float>(mt, phi);
      const float stepv = alpha * cm;
      const float xn = aj - stepv;
      if (nclipped && (mt > phi || mt < -phi)) ++*nclipped;
      m[j] = mt;
      if (x) x[j] = xn;
      a_out[j] = xn;
    }
  }
  return 0;
}

// Local update with AdamW as the base optimizer (decoupled weight decay,
// Loshchilov & Hutter): for inner step index k >= 1
//   m1 <- b1*m1 + (1-b1)*g ;  v <- b2*v + (1-b2)*g*g
//   p  <- p*(1 - lr*wd)
//   p  <- p - (lr/(1-b1^k)) * m1 / (sqrt(v)/sqrt(1-b2^k) + eps)
// Gradients arrive as bf16 bit patterns (widened exactly by a 16-bit shift).
// Optional: dout = anchor - p_out (the pseudo-gradient taken at the last inner
// step of a round) and, per segment, the sum of squares of p_out - p_in (whose
// root at the first inner step is the ||x_{t,1} - x_{t,0}|| of Eq. 3).
int co2_oracle_adamw_f32(int64_t n, const float* p_in, float* p_out,
                         const uint16_t* grad_bf16, float* exp_avg,
                         float* exp_avg_sq, float lr, float beta1, float beta2,
                         float eps, float weight_decay, int64_t k,
                         const float* anchor, float* dout,
                         int32_t S, const int64_t* seg_off, double* step_sq_out) {
  if (n < 0 || !p_in || !p_out || !grad_bf16 || !exp_avg || !exp_avg_sq || k < 1) return -1;
  if ((anchor == nullptr) != (dout == nullptr)) return -1;
  if (step_sq_out && check_table(n, S, seg_off)) return -1;

  const double bc1 = 1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(k));
  const double bc2 = 1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(k));
  const float step_size = static_cast<float>(static_cast<double>(lr) / bc1);
  const float sqrt_bc2 = static_cast<float>(std::sqrt(bc2));
  const float omb1 = 1.0f - beta1;
  const float omb2 = 1.0f - beta2;
  const float decay = 1.0f - lr * weight_decay;

  int32_t s = 0;
  double acc = 0.0;
  for (int64_t j = 0; j < n; ++j) {
    union { uint32_t u; float f; } cv;
    cv.u = static_cast<uint32_t>(grad_bf16[j]) << 16;
    const float g = cv.f;
    const float p0 = p_in[j];
    const float m1 = beta1 * exp_avg[j] + omb1 * g;
    const float v = beta2 * exp_avg_sq[j] + (omb2 * g) * g;
    const float pd = p0 * decay;
    const float denom = std::sqrt(v) / sqrt_bc2 + eps;
    const float upd = step_size * (m1 / denom);
    const float p1 = pd - upd;
    exp_avg[j] = m1;
    exp_avg_sq[j] = v;
    p_out[j] = p1;
    if (dout) dout[j] = anchor[j] - p1;
    if (step_sq_out) {
      while (s < S && j >= seg_off[s + 1]) { step_sq_out[s] = acc; acc = 0.0; ++s; }
      const double df = static_cast<double>(p1 - p0);
      acc += df * df;
    }
  }
  if (step_sq_out) {
    while (s < S) { step_sq_out[s] = acc; acc = 0.0; ++s; }
  }
  return 0;
}

int co2_oracle_adamw_f64(int64_t n, double* p, const double* grad,
                         double* exp_avg, double* exp_avg_sq, double lr,
                         double beta1, double beta2, double eps,
                         double weight_decay, int64_t k) {
  if (n < 0 || !p || !grad || !exp_avg || !exp_avg_sq || k < 1) return -1;
  const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(k));
  const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(k));
  for (int64_t j = 0; j < n; ++j) {
    const double g = grad[j];
    const double m1 = beta1 * exp_avg[j] + (1.0 - beta1) * g;
    const double v = beta2 * exp_avg_sq[j] + (1.0 - beta2) * g * g;
    double pj = p[j] * (1.0 - lr * weight_decay);
    pj -= (lr / bc1) * m1 / (std::sqrt(v) / std::sqrt(bc2) + eps);
    exp_avg[j] = m1;
    exp_avg_sq[j] = v;
    p[j] = pj;
  }
  return 0;
}

}  // extern "C"
