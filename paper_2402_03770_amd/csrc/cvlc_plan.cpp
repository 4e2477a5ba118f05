// Host-side code-length planner of libcvlc: plan construction for the three
// ways a caller can fix the plan (given fractions, given code lengths plus a
// budget, or Algorithm 1), plan validation and gamma of Eq. (5).
//
// Accounting follows Eq. (3): every coded group gets the same bit share b (the
// paper's equal packet size, scaled up to a run of packets), pays H = 128 bits
// for its header and (s + y_r) bits per update; the stream adds one 256-bit
// global header.
#include <cmath>
#include <cstring>
#include <limits>
#include <vector>

#include "cvlc_common.h"

namespace {

using cvlc::kGlobalHeaderBits;
using cvlc::kSegHeaderBits;

struct PowerLaw {  // Definition 1 with beta = 2*alpha + 1: energy of ranks (lo, hi] over the total
  double d, beta, denom;
  bool log_limit;
  PowerLaw(double d_, double alpha) : d(d_), beta(2.0 * alpha + 1.0) {
    log_limit = std::fabs(beta) < 1e-9;
    denom = log_limit ? std::log(d) : std::pow(d, beta) - 1.0;
  }
  double share(double hi, double lo) const {
    hi = hi < 1.0 ? 1.0 : hi;  // Z_0 = 0 is read as rank 1 (the power law starts at l = 1)
    lo = lo < 1.0 ? 1.0 : lo;
    if (log_limit) return (std::log(hi) - std::log(lo)) / denom;
    return (std::pow(hi, beta) - std::pow(lo, beta)) / denom;
  }
};

// PQ: Q(P, y) = P / (2^y - 1)^2 (Appendix, case study).
double pq_error(double P, double y) {
  if (!(y > 0.0)) return std::numeric_limits<double>::infinity();
  const double levels = std::exp2(y) - 1.0;
  return P / (levels * levels);
}

// QSGD: Q(P, y) = min(P / s^2, sqrt(P) / s) (Appendix, case study), s = 2^(y-1) - 1 the
// levels above zero that y bits hold beside the sign.
double qsgd_error(double P, double y) {
  if (!(y > 1.0)) return std::numeric_limits<double>::infinity();
  const double levels = std::exp2(y - 1.0) - 1.0;
  const double a = P / (levels * levels), b = std::sqrt(P) / levels;
  return a < b ? a : b;
}

struct ErrorModel {  // the bracket (Q/B^2 + 1/B_c^2) of Eq. (5)/(6), 1/B + 1/B_c = 1
  double inv_b2, inv_bc2;
  uint32_t quant;
  explicit ErrorModel(double B, uint32_t quant_ = CVLC_QUANT_PQ) : inv_b2(1.0 / (B * B)), quant(quant_) {
    const double inv_bc = 1.0 - 1.0 / B;
    inv_bc2 = inv_bc * inv_bc;
  }
  double weight(double P, double y) const {
    return (quant == CVLC_QUANT_QSGD ? qsgd_error(P, y) : pq_error(P, y)) * inv_b2 + inv_bc2;
  }
};

double gamma_integer(uint32_t d, uint32_t R, const uint32_t* P, const uint32_t* y, double alpha, double B,
                     uint32_t quant = CVLC_QUANT_PQ) {
  const PowerLaw law((double)d, alpha);
  const ErrorModel err(B, quant);
  double k = 0.0;
  for (uint32_t r = 0; r < R; ++r) k += (double)P[r];
  // ranks k+1..d are sparsified away; with k = d there are none
  double g = k >= (double)d ? 0.0 : law.share((double)d, k + 1.0);
  double z_prev = 0.0;
  for (uint32_t r = 0; r < R; ++r) {
    const double z = z_prev + (double)P[r];
    if (P[r] > 0) g += err.weight((double)P[r], (double)y[r]) * law.share(z, z_prev);
    z_prev = z;
  }
  return g;
}

int64_t group_share_bits(uint64_t budget_bits, uint32_t R) {
  if (R == 0 || budget_bits < kGlobalHeaderBits) return -1;
  return (int64_t)(32u * ((budget_bits - kGlobalHeaderBits) / (32u * (uint64_t)R)));
}

void plan_init(cvlc_plan_t* p, uint32_t d, uint32_t R, float B) {
  std::memset(p, 0, sizeof(*p));
  p->d = d;
  p->n_coded = R;
  p->s = cvlc::position_bits(d);
  p->B = B;
  p->quant = 0;
}

int plan_from_fractions(uint32_t d, uint32_t R, const uint32_t* y, const double* frac, float B, cvlc_plan_t* out) {
  plan_init(out, d, R, B);
  double cum = 0.0;
  uint64_t z_prev = 0;
  for (uint32_t r = 0; r < R; ++r) {
    if (!(frac[r] >= 0.0)) return CVLC_ERR_ARG;
    cum += frac[r];
    double zf = std::floor((double)d * cum);
    if (zf > (double)d) zf = (double)d;
    uint64_t z = (uint64_t)zf;
    if (z < z_prev) z = z_prev;
    out->code_len[r] = y[r];
    out->count[r] = (uint32_t)(z - z_prev);
    z_prev = z;
  }
  out->total_bits = cvlc_plan_total_bits(out);
  return cvlc_plan_validate(out);
}

int plan_from_budget(uint32_t d, uint64_t budget, uint32_t R, const uint32_t* y, float B, cvlc_plan_t* out) {
  if (R < 1) return CVLC_ERR_ARG;
  plan_init(out, d, R, B);
  const int64_t b = group_share_bits(budget, R);
  if (b < (int64_t)kSegHeaderBits) return CVLC_ERR_BUDGET;
  uint64_t room = d, k = 0;
  for (uint32_t r = 0; r < R; ++r) {
    if (!cvlc::code_len_supported(y[r])) return CVLC_ERR_PLAN;
    uint64_t P = (uint64_t)(b - kSegHeaderBits) / (out->s + y[r]);
    if (P > room) P = room;
    out->code_len[r] = y[r];
    out->count[r] = (uint32_t)P;
    room -= P;
    k += P;
  }
  if (k < R && d >= R) return CVLC_ERR_BUDGET;
  out->total_bits = cvlc_plan_total_bits(out);
  if (out->total_bits > budget) return CVLC_ERR_BUDGET;
  return cvlc_plan_validate(out);
}

// One instance of problem P2 for a fixed budget share: Algorithm 1.
class Algorithm1 {
 public:
  Algorithm1(uint32_t d, uint32_t R, uint32_t s, double usable_bits, double alpha, double B, uint32_t quant)
      : d_(d), R_(R), s_(s), u_(usable_bits), law_((double)d, alpha), err_(B, quant), alpha_(alpha), B_(B),
        quant_(quant), y_min_(quant == CVLC_QUANT_QSGD ? 2.0 : 1.0) {}

  // f(X, P_{r-1}, P_r) of Eq. (6) as a function of P_r.
  double pair_cost(double Pr, double X, double z_r2) const {
    const double Pr1 = X - Pr;
    const double z_r1 = z_r2 + Pr1, z_r = z_r2 + X;
    const double a = err_.weight(Pr, u_ / Pr - (double)s_) * law_.share(z_r, z_r1);
    const double b = err_.weight(Pr1, u_ / Pr1 - (double)s_) * law_.share(z_r1, z_r2);
    return a + b;
  }

  // Atomic operation: golden-section search for the minimiser of the strongly
  // convex pair cost (Lemma 3) on (X/2, X), kept inside "one update, the quantiser's
  // shortest code" (1 bit for PQ; QSGD needs a sign bit and a level bit).
  double atomic_operation(double X, double z_r2) const {
    const double p_max = u_ / ((double)s_ + y_min_);
    double lo = 0.5 * X, hi = X - 1.0;
    if (hi > p_max) hi = p_max;
    if (lo < X - p_max) lo = X - p_max;
    if (!(hi > lo)) return 0.5 * X > p_max ? p_max : 0.5 * X;
    const double g = 0.6180339887498949;
    double x1 = hi - g * (hi - lo), x2 = lo + g * (hi - lo);
    double f1 = pair_cost(x1, X, z_r2), f2 = pair_cost(x2, X, z_r2);
    for (int it = 0; it < 80; ++it) {
      if (f1 <= f2) {
        hi = x2; x2 = x1; f2 = f1;
        x1 = hi - g * (hi - lo);
        f1 = pair_cost(x1, X, z_r2);
      } else {
        lo = x1; x1 = x2; f1 = f2;
        x2 = lo + g * (hi - lo);
        f2 = pair_cost(x2, X, z_r2);
      }
    }
    return 0.5 * (lo + hi);
  }

  // SMO-style sweeps for one k, then integer code lengths (clamped to 1..16,
  // non-increasing) and refilled group sizes; returns gamma of the integer plan.
  double solve(double k, uint32_t* y, uint32_t* P) const {
    double Pc[CVLC_MAX_CODED];
    for (uint32_t r = 0; r < R_; ++r) Pc[r] = k / (double)R_;
    for (int sweep = 0; sweep < 200; ++sweep) {
      double moved = 0.0, z_r2 = 0.0;
      for (uint32_t r = 1; r < R_; ++r) {
        const double X = Pc[r - 1] + Pc[r];
        const double Pr = atomic_operation(X, z_r2);
        const double delta = std::fabs(Pr - Pc[r]);
        if (delta > moved) moved = delta;
        Pc[r] = Pr;
        Pc[r - 1] = X - Pr;
        z_r2 += Pc[r - 1];
      }
      if (moved < 0.5) break;
    }
    uint64_t room = d_;
    for (uint32_t r = 0; r < R_; ++r) {
      double yr = std::floor(u_ / Pc[r]) - (double)s_;
      if (yr < y_min_) yr = y_min_;
      if (yr > 16.0) yr = 16.0;
      uint32_t yi = (uint32_t)yr;
      if (r > 0 && yi > y[r - 1]) yi = y[r - 1];
      uint64_t Pi = (uint64_t)(u_ / (double)(s_ + yi));
      if (Pi > room) Pi = room;
      y[r] = yi;
      P[r] = (uint32_t)Pi;
      room -= Pi;
    }
    return gamma_integer(d_, R_, P, y, alpha_, B_, quant_);
  }

 private:
  uint32_t d_, R_, s_;
  double u_;
  PowerLaw law_;
  ErrorModel err_;
  double alpha_, B_;
  uint32_t quant_;
  double y_min_;
};

int plan_algorithm1(uint32_t d, uint64_t budget, uint32_t R, double alpha, float B, uint32_t quant,
                    cvlc_plan_t* out) {
  if (R < 1 || !std::isfinite(alpha) || quant > CVLC_QUANT_QSGD) return CVLC_ERR_ARG;
  plan_init(out, d, R, B);
  out->quant = quant;
  const int64_t b = group_share_bits(budget, R);
  if (b < (int64_t)kSegHeaderBits) return CVLC_ERR_BUDGET;
  const double u = (double)(b - kSegHeaderBits);
  const double k_min = (double)R;
  double k_max = (double)R * u / ((double)out->s + (quant == CVLC_QUANT_QSGD ? 2.0 : 1.0));
  if (k_max > (double)d) k_max = (double)d;
  if (k_max < k_min) return CVLC_ERR_BUDGET;
  const Algorithm1 alg(d, R, out->s, u, alpha, (double)B, quant);
  double best = std::numeric_limits<double>::infinity();
  constexpr int kGrid = 128;  // equidistant search over k
  for (int g = 0; g < kGrid; ++g) {
    const double k = k_min + (k_max - k_min) * (double)g / (double)(kGrid - 1);
    uint32_t y[CVLC_MAX_CODED], P[CVLC_MAX_CODED];
    const double gam = alg.solve(k, y, P);
    if (gam < best) {
      best = gam;
      for (uint32_t r = 0; r < R; ++r) {
        out->code_len[r] = y[r];
        out->count[r] = P[r];
      }
    }
  }
  if (!(best < std::numeric_limits<double>::infinity())) return CVLC_ERR_BUDGET;
  out->total_bits = cvlc_plan_total_bits(out);
  if (out->total_bits > budget) return CVLC_ERR_BUDGET;
  return cvlc_plan_validate(out);
}

}  // namespace

extern "C" {

uint32_t cvlc_position_bits(uint32_t d) { return cvlc::position_bits(d); }

uint64_t cvlc_plan_total_bits(const cvlc_plan_t* p) {
  if (!p) return 0;
  uint64_t words = cvlc::kGlobalHeaderWords + (uint64_t)cvlc::kSegHeaderWords * p->n_coded;
  for (uint32_t r = 0; r < p->n_coded && r < CVLC_MAX_CODED; ++r)
    words += cvlc::payload_words(p->count[r], p->s + p->code_len[r]);
  return 32u * words;
}

int cvlc_plan_validate(const cvlc_plan_t* p) {
  if (!p) return CVLC_ERR_ARG;
  if (p->d < 1 || p->d > 0x7FFFFFFFu) return CVLC_ERR_PLAN;
  if (p->n_coded > CVLC_MAX_CODED) return CVLC_ERR_PLAN;
  if (p->s != cvlc::position_bits(p->d)) return CVLC_ERR_PLAN;
  if (p->quant > CVLC_QUANT_QSGD) return CVLC_ERR_PLAN;
  if (!(p->B > 0.0f) || !std::isfinite(p->B)) return CVLC_ERR_PLAN;
  uint64_t k = 0;
  for (uint32_t r = 0; r < p->n_coded; ++r) {
    if (!cvlc::code_len_supported(p->code_len[r])) return CVLC_ERR_PLAN;
    if (p->quant == CVLC_QUANT_QSGD && p->code_len[r] < 2) return CVLC_ERR_PLAN;  // a sign bit and a level bit
    if (r > 0 && p->code_len[r] > p->code_len[r - 1]) return CVLC_ERR_PLAN;
    k += p->count[r];
  }
  if (k > p->d) return CVLC_ERR_PLAN;
  if (p->total_bits != cvlc_plan_total_bits(p)) return CVLC_ERR_PLAN;
  return CVLC_OK;
}

double cvlc_plan_gamma(const cvlc_plan_t* p, double alpha) {
  if (!p || p->n_coded > CVLC_MAX_CODED) return std::numeric_limits<double>::quiet_NaN();
  return gamma_integer(p->d, p->n_coded, p->count, p->code_len, alpha, (double)p->B, p->quant);
}

double cvlc_plan_next_scale(const cvlc_plan_t* plan) {
  double worst = 0.0;
  if (plan) {
    const uint32_t R = plan->n_coded < CVLC_MAX_CODED ? plan->n_coded : CVLC_MAX_CODED;
    for (uint32_t r = 0; r < R; ++r) {
      const uint32_t y = plan->code_len[r];
      if (y == 0 || y >= 32 || plan->count[r] == 0) continue;  // raw values carry no quantisation error
      const double Q = plan->quant == CVLC_QUANT_QSGD ? qsgd_error((double)plan->count[r], (double)y)
                                                      : pq_error((double)plan->count[r], (double)y);
      if (Q > worst) worst = Q;
    }
  }
  return worst + 1.0;
}

double cvlc_stats_gamma(const cvlc_seg_stats_t* stats, uint32_t n_coded) {
  if (!stats || n_coded > CVLC_MAX_CODED) return 0.0;
  double err = 0.0, all = 0.0;
  for (uint32_t r = 0; r <= n_coded; ++r) {
    err += stats[r].errsq;
    all += stats[r].sumsq;
  }
  return all > 0.0 ? err / all : 0.0;
}

size_t cvlc_stream_capacity(const cvlc_plan_t* p) { return p ? (size_t)(p->total_bits / 8u) : 0; }

int cvlc_plan(uint32_t d, uint64_t budget_bits, uint32_t n_coded, const uint32_t* code_len,
              const double* fractions, double alpha, float B, cvlc_plan_t* out) {
  if (!out || d < 1 || d > 0x7FFFFFFFu || n_coded > CVLC_MAX_CODED) return CVLC_ERR_ARG;
  if (!(B > 0.0f) || !std::isfinite(B)) return CVLC_ERR_ARG;
  if (fractions) {
    if (!code_len) return CVLC_ERR_ARG;
    return plan_from_fractions(d, n_coded, code_len, fractions, B, out);
  }
  if (code_len) return plan_from_budget(d, budget_bits, n_coded, code_len, B, out);
  return plan_algorithm1(d, budget_bits, n_coded, alpha, B, CVLC_QUANT_PQ, out);
}

int cvlc_plan_algorithm1(uint32_t d, uint64_t budget_bits, uint32_t n_coded, double alpha, float B, uint32_t quant,
                         cvlc_plan_t* out) {
  if (!out || d < 1 || d > 0x7FFFFFFFu || n_coded > CVLC_MAX_CODED) return CVLC_ERR_ARG;
  if (!(B > 0.0f) || !std::isfinite(B)) return CVLC_ERR_ARG;
  return plan_algorithm1(d, budget_bits, n_coded, alpha, B, quant, out);
}

const char* cvlc_status_string(int status) {
  switch (status) {
    case CVLC_OK: return "ok";
    case CVLC_ERR_ARG: return "bad argument";
    case CVLC_ERR_PLAN: return "invalid plan";
    case CVLC_ERR_BUDGET: return "budget too small";
    case CVLC_ERR_CAPACITY: return "buffer too small";
    case CVLC_ERR_NONFINITE: return "non-finite input";
    case CVLC_ERR_STREAM: return "malformed stream";
    case CVLC_ERR_DEVICE: return "HIP call failed";
    default: return "unknown status";
  }
}

}  // extern "C"

namespace cvlc {
int hip_check(hipError_t e) { return e == hipSuccess ? CVLC_OK : CVLC_ERR_DEVICE; }

namespace {
struct Bracket {
  int stage;
  hipEvent_t begin, end;
};
bool g_profiling = false;
uint32_t g_stage_mask = 0;
std::vector<Bracket> g_brackets;
}  // namespace

void profile_mark(int stage, bool begin, hipStream_t stream) {
  if (!g_profiling || !((g_stage_mask >> stage) & 1u)) return;
  if (begin) {
    Bracket b{stage, nullptr, nullptr};
    if (hipEventCreate(&b.begin) != hipSuccess || hipEventCreate(&b.end) != hipSuccess) return;
    (void)hipEventRecord(b.begin, stream);
    g_brackets.push_back(b);
  } else {
    for (size_t i = g_brackets.size(); i-- > 0;)
      if (g_brackets[i].stage == stage) {
        (void)hipEventRecord(g_brackets[i].end, stream);
        break;
      }
  }
}
}  // namespace cvlc

extern "C" {

int cvlc_profile_start(uint32_t stage_mask) {
  if (cvlc::g_profiling) return CVLC_ERR_ARG;
  cvlc::g_stage_mask = stage_mask;
  cvlc::g_brackets.clear();
  cvlc::g_profiling = true;
  return CVLC_OK;
}

int cvlc_profile_stop(float* ms_per_stage, uint32_t* brackets_per_stage) {
  if (!cvlc::g_profiling || !ms_per_stage || !brackets_per_stage) return CVLC_ERR_ARG;
  cvlc::g_profiling = false;
  for (int i = 0; i < CVLC_PROFILE_STAGES; ++i) { ms_per_stage[i] = 0.0f; brackets_per_stage[i] = 0; }
  int rc = CVLC_OK;
  for (auto& b : cvlc::g_brackets) {
    float ms = 0.0f;
    if (hipEventSynchronize(b.end) == hipSuccess && hipEventElapsedTime(&ms, b.begin, b.end) == hipSuccess) {
      ms_per_stage[b.stage] += ms;
      brackets_per_stage[b.stage] += 1;
    } else {
      rc = CVLC_ERR_DEVICE;
    }
    (void)hipEventDestroy(b.begin);
    (void)hipEventDestroy(b.end);
  }
  cvlc::g_brackets.clear();
  return rc;
}

}  // extern "C"
