/*
 * cvlc_oracle.c -- plain, slow CPU oracle of the Fed-CVLC compressor and of the
 * parameter-server decode/aggregate step.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be
 * checked against something written straight from the paper.  Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg may call it; the
 * product path never does.  It shares no code, header, table or helper with the
 * HIP implementation.
 *
 * What it computes, in the paper's order and notation:
 *   - ranking of the d model updates by |U{l}| (Definition 1),
 *   - sparsification to the top k = P_1+...+P_R and grouping of the ranked
 *     updates into R consecutive groups P_r, one code length y_r per group
 *     (Sec. IV-B three operations; Sec. IV-C, Eq. (3)-(4); Algorithm 1 last loop),
 *   - per-group centroid distribution for PQ: the group's (min, max)
 *     (Sec. IV-D item 2),
 *   - unbiased quantisation of each kept update to one of 2^{y_r} uniformly
 *     spaced centroids, rounding up or down at random (Sec. IV-B "Quantization",
 *     Appendix "Case Study", PQ),
 *   - the packet payload of (PID, CID) records, PID = s = ceil(log2 d) bits,
 *     CID = y_r bits, one code length per group (Sec. IV-C Eq. (2)-(3),
 *     Sec. IV-D items 1-3),
 *   - the PS side: map CID -> centroid, place at PID, scale by 1/B and average
 *     over the participating clients (Sec. III step 3, Sec. IV-B "Scaling"),
 *   - the code-length planner: Proposition 2 (Eq. (5)), the atomic operation on
 *     two adjacent groups (Eq. (6), Lemma 3) and Algorithm 1's sweep.
 *
 * Everything the paper leaves open (tie order, bit layout, RNG, float rounding)
 * is fixed in the comments of the function that needs it.
 *
 * Parity pins (tests that do not go through this file's own formulas):
 *   philox4x32-10 ........ published known-answer vectors
 *   ranking/grouping ..... numpy lexsort / torch.topk on crafted tie-heavy inputs
 *   quantiser ............ textbook stochastic rounding written in numpy, fed
 *                          the same uniforms; unbiasedness and MSE closed forms
 *   bit layout ........... numpy unpackbits field extraction; closed-form sizes
 *   decode/aggregate ..... dense numpy sum of single-client decodes
 *   planner (mode A, B) .. closed forms and the worked sizes of the configs
 *   planner (Algorithm 1)  exhaustion over all integer code-length vectors for
 *                          R <= 6; the sweep's fixed point against a general
 *                          constrained minimiser of Eq. (5) (Theorem 1) at
 *                          R = 4, 7, 15, 31; one-bit moves and the one-length
 *                          plans of Sec. V at the workloads' R = 7, 15, 31
 *   memory / arithmetic .. the whole file under ASan + UBSan
 * Parity unpinned: the learning results of Sec. V (they need the datasets).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAX_R 31u
#define ORC_MAGIC 0x434C5643u /* "CVLC" little endian */
#define ORC_VERSION 1u
#define ORC_GLOBAL_HEADER_WORDS 8u
#define ORC_SEG_HEADER_WORDS 4u

enum {
  ORC_OK = 0,
  ORC_ERR_ARG = -1,
  ORC_ERR_PLAN = -2,
  ORC_ERR_BUDGET = -3,
  ORC_ERR_CAPACITY = -4,
  ORC_ERR_NONFINITE = -5,
  ORC_ERR_STREAM = -6
};

typedef struct {
  uint32_t d;            /* number of model updates                           */
  uint32_t R;            /* number of coded groups (the 0-bit tail is implicit)*/
  uint32_t s;            /* position-ID width, ceil(log2 d)                    */
  uint32_t y[ORC_MAX_R]; /* code length of group r (1..16 or 32 = raw fp32)    */
  uint32_t P[ORC_MAX_R]; /* number of updates in group r                       */
  uint64_t total_bits;   /* exact stream size in bits                          */
  float B;               /* scale factor of Lemma 1                            */
  uint32_t quant;        /* 0 = PQ, 1 = QSGD                                   */
} orc_plan;

typedef struct {
  float min, max; /* signed extremes of the group (0,0 for the tail / empty)  */
  double sumsq;   /* sum of squares of the group's original values            */
  uint32_t count;
  uint32_t pad;
  double errsq;   /* sum over the group of (xtilde/B - x)^2: the left side of */
                  /* Lemma 1 for this draw; the tail is dropped whole, so its */
                  /* errsq equals its sumsq                                    */
} orc_seg_stats;

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of           */
/*   (c0,c1,c2,c3) -> (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)) */
/* with the key bumped by the Weyl constants between rounds.                  */
/* ------------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 24-bit uniform that decides the rounding direction of coordinate i of
 * one client: first output word of Philox keyed by the 64-bit seed, counter
 * (i, client, 0, 0), top 24 bits.  Keyed by the coordinate, so the draw does
 * not depend on how the coordinate was grouped. */
uint32_t orc_u24(uint64_t seed, uint32_t client, uint32_t i) {
  uint32_t ctr[4] = {i, client, 0u, 0u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  return out[0] >> 8;
}

/* ------------------------------------------------------------------------- */
/* small helpers                                                              */
/* ------------------------------------------------------------------------- */
static uint32_t f2u(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float u2f(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* s = ceil(log2 d) (Sec. IV-C, below Eq. (2)); at least one bit. */
uint32_t orc_s_bits(uint32_t d) {
  uint32_t s = 0;
  while (s < 32 && ((uint64_t)1 << s) < (uint64_t)d) ++s;
  return s < 1 ? 1 : s;
}

static int code_len_ok(uint32_t y) { return (y >= 1 && y <= 16) || y == 32; }

static uint64_t seg_payload_words(uint32_t P, uint32_t W) {
  return ((uint64_t)P * W + 31u) / 32u;
}

/* Stream size: 8 header words, 4 words per coded group, then every group's
 * records padded to a whole 32-bit word.  Headers and padding count against
 * the budget, as H does in Eq. (3). */
uint64_t orc_plan_total_bits(const orc_plan* p) {
  uint64_t words = ORC_GLOBAL_HEADER_WORDS + (uint64_t)ORC_SEG_HEADER_WORDS * p->R;
  for (uint32_t r = 0; r < p->R; ++r) words += seg_payload_words(p->P[r], p->s + p->y[r]);
  return 32u * words;
}

/* A plan is valid when the groups fit in d, code lengths do not grow with
 * rank (larger magnitude => at least as many bits, Eq. (4)) and each is one
 * of the supported lengths. */
int orc_plan_validate(const orc_plan* p) {
  if (p->d < 1 || p->d > 0x7FFFFFFFu) return ORC_ERR_PLAN;
  if (p->R > ORC_MAX_R) return ORC_ERR_PLAN;
  if (p->s != orc_s_bits(p->d)) return ORC_ERR_PLAN;
  if (p->quant > 1) return ORC_ERR_PLAN;
  if (!(p->B > 0.0f) || !isfinite(p->B)) return ORC_ERR_PLAN;
  uint64_t k = 0;
  for (uint32_t r = 0; r < p->R; ++r) {
    if (!code_len_ok(p->y[r])) return ORC_ERR_PLAN;
    if (p->quant == 1 && p->y[r] < 2) return ORC_ERR_PLAN; /* a sign bit and at least one level bit */
    if (r > 0 && p->y[r] > p->y[r - 1]) return ORC_ERR_PLAN;
    k += p->P[r];
  }
  if (k > p->d) return ORC_ERR_PLAN;
  if (p->total_bits != orc_plan_total_bits(p)) return ORC_ERR_PLAN;
  return ORC_OK;
}

static void plan_begin(orc_plan* p, uint32_t d, uint32_t R, float B) {
  memset(p, 0, sizeof(*p));
  p->d = d; p->R = R; p->s = orc_s_bits(d); p->B = B; p->quant = 0;
}

/* Planner mode A: the code lengths and the fraction of the d coordinates that
 * each coded group takes are given.  Cumulative boundary Z_r = floor(d * (f_1 +
 * ... + f_r)), P_r = Z_r - Z_{r-1}. */
int orc_plan_fractions(uint32_t d, uint32_t R, const uint32_t* y, const double* frac, float B,
                       orc_plan* out) {
  if (!y || !frac || !out || R > ORC_MAX_R || d < 1) return ORC_ERR_ARG;
  plan_begin(out, d, R, B);
  double cum = 0.0;
  uint64_t prev = 0;
  for (uint32_t r = 0; r < R; ++r) {
    if (!(frac[r] >= 0.0)) return ORC_ERR_ARG;
    cum += frac[r];
    double z = floor((double)d * cum);
    if (z > (double)d) z = (double)d;
    uint64_t Z = (uint64_t)z;
    if (Z < prev) Z = prev;
    out->y[r] = y[r];
    out->P[r] = (uint32_t)(Z - prev);
    prev = Z;
  }
  out->total_bits = orc_plan_total_bits(out);
  return orc_plan_validate(out);
}

#define ORC_GLOBAL_HEADER_BITS 256u
#define ORC_SEG_HEADER_BITS 128u /* H of Eq. (3): y_r, P_r, min, max */

/* Every coded group gets the same share b of the budget, the paper's equal
 * packet size scaled up (Sec. IV-C "we let b_r = b"): what is left after the
 * global header, split R ways and rounded down to whole words. */
static int64_t share_bits(uint64_t budget_bits, uint32_t R) {
  if (R == 0 || budget_bits < ORC_GLOBAL_HEADER_BITS) return -1;
  return (int64_t)(32u * ((budget_bits - ORC_GLOBAL_HEADER_BITS) / (32u * (uint64_t)R)));
}

/* Planner mode B: code lengths given, group sizes from the budget.  Eq. (3):
 * P_r (s + y_r) + H <= b  =>  P_r = floor((b - H)/(s + y_r)). */
int orc_plan_budget(uint32_t d, uint64_t budget_bits, uint32_t R, const uint32_t* y, float B,
                    orc_plan* out) {
  if (!y || !out || R < 1 || R > ORC_MAX_R || d < 1) return ORC_ERR_ARG;
  plan_begin(out, d, R, B);
  int64_t b = share_bits(budget_bits, R);
  if (b < (int64_t)ORC_SEG_HEADER_BITS) return ORC_ERR_BUDGET;
  uint64_t left = d;
  uint64_t k = 0;
  for (uint32_t r = 0; r < R; ++r) {
    if (!code_len_ok(y[r])) return ORC_ERR_PLAN;
    uint64_t P = (uint64_t)(b - ORC_SEG_HEADER_BITS) / (out->s + y[r]);
    if (P > left) P = left;
    out->y[r] = y[r];
    out->P[r] = (uint32_t)P;
    left -= P;
    k += P;
  }
  if (k < R && d >= R) return ORC_ERR_BUDGET; /* not even k_min = R fits */
  out->total_bits = orc_plan_total_bits(out);
  if (out->total_bits > budget_bits) return ORC_ERR_BUDGET;
  return orc_plan_validate(out);
}

/* ------------------------------------------------------------------------- */
/* Proposition 2 / Algorithm 1                                                */
/* ------------------------------------------------------------------------- */

/* PQ quantisation error of a group of P updates at y bits (Appendix "Case
 * Study"): Q = P / (2^y - 1)^2. */
static double q_pq(double P, double y) {
  if (!(y > 0.0)) return INFINITY;
  double levels = exp2(y) - 1.0;
  return P / (levels * levels);
}

/* (a^beta - b^beta)/(d^beta - 1), the share of the squared norm carried by
 * ranks (b, a] under the power law of Definition 1; ranks below 1 are read as
 * 1 (Z_0 = 0 would diverge for beta < 0) and beta -> 0 takes the log limit. */
static double energy_share(double a, double b, double d, double beta) {
  if (a < 1.0) a = 1.0;
  if (b < 1.0) b = 1.0;
  if (fabs(beta) < 1e-9) return (log(a) - log(b)) / log(d);
  return (pow(a, beta) - pow(b, beta)) / (pow(d, beta) - 1.0);
}

/* gamma of Eq. (5) for real-valued group sizes P_r with y_r = u/P_r - s, or,
 * when y_int is given, for those integer code lengths. */
/* QSGD's quantisation error (appendix case study): min(P/s^2, sqrt(P)/s), with
 * s the number of levels above zero that y bits hold beside the sign. */
static double q_qsgd(double P, double y) {
  if (!(y > 1.0)) return INFINITY;
  double levels = exp2(y - 1.0) - 1.0;
  double a = P / (levels * levels), b = sqrt(P) / levels;
  return a < b ? a : b;
}

static double gamma_eq5(uint32_t d, uint32_t R, const double* P, const uint32_t* y_int, double u,
                        uint32_t s, double beta, double B, uint32_t quant) {
  double invB2 = 1.0 / (B * B);
  double invBc = 1.0 - 1.0 / B; /* 1/B + 1/B_c = 1 */
  double k = 0.0;
  for (uint32_t r = 0; r < R; ++r) k += P[r];
  /* first term: the energy of the sparsified ranks k+1..d; there are none when k = d (the printed
   * closed form would then give minus the share of a rank d+1 that does not exist) */
  double g = k >= (double)d ? 0.0 : energy_share((double)d, k + 1.0, (double)d, beta);
  double Zprev = 0.0;
  for (uint32_t r = 0; r < R; ++r) {
    double Z = Zprev + P[r];
    if (P[r] > 0.0) {
      double y = y_int ? (double)y_int[r] : u / P[r] - (double)s;
      double Q = quant == 1 ? q_qsgd(P[r], y) : q_pq(P[r], y);
      g += (Q * invB2 + invBc * invBc) * energy_share(Z, Zprev, (double)d, beta);
    }
    Zprev = Z;
  }
  return g;
}

double orc_gamma(const orc_plan* p, double alpha) {
  double P[ORC_MAX_R];
  for (uint32_t r = 0; r < p->R; ++r) P[r] = (double)p->P[r];
  return gamma_eq5(p->d, p->R, P, p->y, 0.0, p->s, 2.0 * alpha + 1.0, (double)p->B, p->quant);
}

/* f(X, P_{r-1}, P_r) of Eq. (6) as a function of P_r, with Z_{r-2} and X fixed. */
static double q_of(uint32_t quant, double P, double y) { return quant == 1 ? q_qsgd(P, y) : q_pq(P, y); }

static double f_eq6(double Pr, double X, double Zr2, double d, double u, uint32_t s, double beta,
                    double B, uint32_t quant) {
  double invB2 = 1.0 / (B * B);
  double invBc = 1.0 - 1.0 / B;
  double Pr1 = X - Pr;
  double Zr1 = Zr2 + Pr1, Zr = Zr2 + X;
  double a = (q_of(quant, Pr, u / Pr - (double)s) * invB2 + invBc * invBc) * energy_share(Zr, Zr1, d, beta);
  double b = (q_of(quant, Pr1, u / Pr1 - (double)s) * invB2 + invBc * invBc) * energy_share(Zr1, Zr2, d, beta);
  return a + b;
}

/* The atomic operation: minimise f over P_r.  f is strongly convex (Lemma 3)
 * and its minimiser lies in (X/2, X) (end of the proof of Lemma 3), so a
 * golden-section search on that interval finds it; the interval is cut so that
 * both groups keep at least one update and the shortest code the quantiser
 * takes (1 bit for PQ; QSGD needs a sign bit and a level bit). */
static double atomic_operation(double X, double Zr2, double d, double u, uint32_t s, double beta,
                               double B, uint32_t quant) {
  double Pmax = u / ((double)s + (quant == 1 ? 2.0 : 1.0));
  double lo = 0.5 * X, hi = X - 1.0;
  if (hi > Pmax) hi = Pmax;
  if (lo < X - Pmax) lo = X - Pmax;
  if (!(hi > lo)) return 0.5 * X > Pmax ? Pmax : 0.5 * X;
  const double invphi = 0.6180339887498949;
  double x1 = hi - invphi * (hi - lo), x2 = lo + invphi * (hi - lo);
  double f1 = f_eq6(x1, X, Zr2, d, u, s, beta, B, quant), f2 = f_eq6(x2, X, Zr2, d, u, s, beta, B, quant);
  for (int it = 0; it < 80; ++it) {
    if (f1 <= f2) {
      hi = x2; x2 = x1; f2 = f1;
      x1 = hi - invphi * (hi - lo);
      f1 = f_eq6(x1, X, Zr2, d, u, s, beta, B, quant);
    } else {
      lo = x1; x1 = x2; f1 = f2;
      x2 = lo + invphi * (hi - lo);
      f2 = f_eq6(x2, X, Zr2, d, u, s, beta, B, quant);
    }
  }
  return 0.5 * (lo + hi);
}

/* Integer code lengths and group sizes from real-valued P_r: y_r = floor(u/P_r)
 * - s clamped to [1,16] ([2,16] for QSGD) and kept non-increasing, then the group is
 * refilled to P_r = floor(u/(s+y_r)) (Eq. (3) with equality as far as integers allow). */
static void integerise(uint32_t d, uint32_t R, const double* P, double u, uint32_t s, uint32_t* y,
                       uint32_t* Pint, uint32_t quant) {
  uint64_t left = d;
  for (uint32_t r = 0; r < R; ++r) {
    double yr = floor(u / P[r]) - (double)s;
    double ymin = quant == 1 ? 2.0 : 1.0;
    if (yr < ymin) yr = ymin;
    if (yr > 16.0) yr = 16.0;
    uint32_t yi = (uint32_t)yr;
    if (r > 0 && yi > y[r - 1]) yi = y[r - 1];
    uint64_t Pi = (uint64_t)(u / (double)(s + yi));
    if (Pi > left) Pi = left;
    y[r] = yi;
    Pint[r] = (uint32_t)Pi;
    left -= Pi;
  }
}

/* Step 2 of the solution of P2 (the inner loop of Algorithm 1) for one k:
 * start from P_r = k/R and sweep the atomic operation over r = 2..R until no
 * P_r moves by 0.5 (at most 200 sweeps).  P holds the real-valued group sizes
 * on return; their sum is k throughout. */
static void alg1_sweep(double k, uint32_t d, uint32_t R, double u, uint32_t s, double beta, double B,
                       uint32_t quant, double* P) {
  for (uint32_t r = 0; r < R; ++r) P[r] = k / (double)R;
  for (int sweep = 0; sweep < 200; ++sweep) {
    double moved = 0.0, Zr2 = 0.0;
    for (uint32_t r = 1; r < R; ++r) {
      double X = P[r - 1] + P[r];
      double Pr = atomic_operation(X, Zr2, (double)d, u, s, beta, B, quant);
      double delta = fabs(Pr - P[r]);
      if (delta > moved) moved = delta;
      P[r] = Pr;
      P[r - 1] = X - Pr;
      Zr2 += P[r - 1];
    }
    if (moved < 0.5) break;
  }
}

/* The sweep alone, for the tests: real-valued P_1..P_R for a given k under the
 * budget's bit share, and gamma of Eq. (5) at that point with y_r = u/P_r - s. */
int orc_alg1_sweep(uint32_t d, uint64_t budget_bits, uint32_t R, double alpha, float B, uint32_t quant,
                   double k, double* P_out, double* gamma_out) {
  if (!P_out || R < 1 || R > ORC_MAX_R || d < 1 || quant > 1 || !isfinite(alpha)) return ORC_ERR_ARG;
  int64_t b = share_bits(budget_bits, R);
  if (b < (int64_t)ORC_SEG_HEADER_BITS) return ORC_ERR_BUDGET;
  uint32_t s = orc_s_bits(d);
  double u = (double)(b - ORC_SEG_HEADER_BITS);
  double beta = 2.0 * alpha + 1.0;
  alg1_sweep(k, d, R, u, s, beta, (double)B, quant, P_out);
  if (gamma_out) *gamma_out = gamma_eq5(d, R, P_out, NULL, u, s, beta, (double)B, quant);
  return ORC_OK;
}

/* Planner mode C: Algorithm 1.  For every k on a 128-point equidistant grid of
 * [k_min, k_max] = [R, R(b-H)/(s+y_min)], y_min the quantiser's shortest code: run the sweep,
 * make the result integer and evaluate Eq. (5); keep the k with the smallest gamma. */
int orc_plan_alg1_quant(uint32_t d, uint64_t budget_bits, uint32_t R, double alpha, float B,
                        uint32_t quant, orc_plan* out) {
  if (!out || R < 1 || R > ORC_MAX_R || d < 1 || quant > 1) return ORC_ERR_ARG;
  if (!isfinite(alpha)) return ORC_ERR_ARG;
  plan_begin(out, d, R, B);
  out->quant = quant;
  int64_t b = share_bits(budget_bits, R);
  if (b < (int64_t)ORC_SEG_HEADER_BITS) return ORC_ERR_BUDGET;
  uint32_t s = out->s;
  double u = (double)(b - ORC_SEG_HEADER_BITS);
  double kmin = (double)R;
  double kmax = (double)R * u / ((double)s + (quant == 1 ? 2.0 : 1.0));
  if (kmax > (double)d) kmax = (double)d;
  if (kmax < kmin) return ORC_ERR_BUDGET;
  double beta = 2.0 * alpha + 1.0;
  double best = INFINITY;
  for (int g = 0; g < 128; ++g) {
    double k = kmin + (kmax - kmin) * (double)g / 127.0;
    double P[ORC_MAX_R];
    alg1_sweep(k, d, R, u, s, beta, (double)B, quant, P);
    uint32_t y[ORC_MAX_R], Pi[ORC_MAX_R];
    double Pd[ORC_MAX_R];
    integerise(d, R, P, u, s, y, Pi, quant);
    for (uint32_t r = 0; r < R; ++r) Pd[r] = (double)Pi[r];
    double gam = gamma_eq5(d, R, Pd, y, u, s, beta, (double)B, quant);
    if (gam < best) {
      best = gam;
      for (uint32_t r = 0; r < R; ++r) { out->y[r] = y[r]; out->P[r] = Pi[r]; }
    }
  }
  if (!(best < INFINITY)) return ORC_ERR_BUDGET;
  out->total_bits = orc_plan_total_bits(out);
  if (out->total_bits > budget_bits) return ORC_ERR_BUDGET;
  return orc_plan_validate(out);
}

int orc_plan_alg1(uint32_t d, uint64_t budget_bits, uint32_t R, double alpha, float B,
                  orc_plan* out) {
  return orc_plan_alg1_quant(d, budget_bits, R, alpha, B, 0, out);
}

/* ------------------------------------------------------------------------- */
/* ranking                                                                    */
/* ------------------------------------------------------------------------- */
typedef struct { uint32_t key, idx; } ranked;

/* |U| descending; equal magnitudes: lower index first.  The magnitude is
 * compared through the raw bits with the sign cleared, so -0 == +0 and
 * denormals are ordinary values. */
static int cmp_rank(const void* a, const void* b) {
  const ranked* x = (const ranked*)a; const ranked* y = (const ranked*)b;
  if (x->key != y->key) return x->key > y->key ? -1 : 1;
  if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1;
  return 0;
}

static int cmp_u32(const void* a, const void* b) {
  uint32_t x = *(const uint32_t*)a, y = *(const uint32_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}

/* order[l] = index of the (l+1)-th largest update, U{l+1} of Definition 1. */
int orc_rank(const float* U, uint32_t d, uint32_t* order) {
  ranked* a = (ranked*)malloc((size_t)d * sizeof(ranked));
  if (!a) return ORC_ERR_ARG;
  for (uint32_t i = 0; i < d; ++i) {
    uint32_t key = f2u(U[i]) & 0x7FFFFFFFu;
    if (key >= 0x7F800000u) { free(a); return ORC_ERR_NONFINITE; }
    a[i].key = key; a[i].idx = i;
  }
  qsort(a, d, sizeof(ranked), cmp_rank);
  for (uint32_t i = 0; i < d; ++i) order[i] = a[i].idx;
  free(a);
  return ORC_OK;
}

/* seg[i] = r in 1..R if coordinate i falls in coded group r, 0 if it is
 * sparsified away (rank > k). */
int orc_segments(const float* U, const orc_plan* p, uint32_t* seg) {
  int rc = orc_plan_validate(p);
  if (rc) return rc;
  uint32_t d = p->d;
  uint32_t* order = (uint32_t*)malloc((size_t)d * sizeof(uint32_t));
  if (!order) return ORC_ERR_ARG;
  rc = orc_rank(U, d, order);
  if (rc) { free(order); return rc; }
  memset(seg, 0, (size_t)d * sizeof(uint32_t));
  uint64_t l = 0;
  for (uint32_t r = 0; r < p->R; ++r)
    for (uint32_t e = 0; e < p->P[r]; ++e) seg[order[l++]] = r + 1;
  free(order);
  return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* quantiser                                                                  */
/* ------------------------------------------------------------------------- */

/* Spacing of the 2^y uniformly placed centroids on [m, M] and its inverse,
 * both one correctly rounded fp32 division; a group with M == m (or empty)
 * has a single centroid. */
static void centroid_grid(float m, float M, uint32_t y, float* step, float* inv) {
  float range = M - m;
  float top = (float)(((uint64_t)1 << y) - 1u);
  if (range > 0.0f) { *step = range / top; *inv = top / range; }
  else { *step = 0.0f; *inv = 0.0f; }
}

/* CID of value x in a group with extremes (m, M) at y bits: position between
 * the centroids t = (x - m) * inv in fp32, lower centroid j = floor(t), and
 * one step up with probability t - j (resolved to 2^-24 against the 24-bit
 * uniform), which makes the centroid value unbiased.  y = 32 keeps the raw
 * fp32 bits. */
uint32_t orc_quantise(float x, float m, float M, uint32_t y, uint32_t u24) {
  if (y == 32) return f2u(x);
  float step, inv;
  centroid_grid(m, M, y, &step, &inv);
  float top = (float)(((uint32_t)1 << y) - 1u);
  float t = (x - m) * inv;
  if (!(t > 0.0f)) t = 0.0f;
  if (t > top) t = top;
  float fl = floorf(t);
  uint32_t j = (uint32_t)fl;
  float p = t - fl;
  uint32_t thr = (uint32_t)(p * 16777216.0f);
  uint32_t cid = j + (u24 < thr ? 1u : 0u);
  uint32_t L1 = ((uint32_t)1 << y) - 1u;
  return cid > L1 ? L1 : cid;
}

/* Centroid value of a CID: m + CID*step with one rounding. */
float orc_dequantise(uint32_t cid, float m, float M, uint32_t y) {
  if (y == 32) return u2f(cid);
  float step, inv;
  centroid_grid(m, M, y, &step, &inv);
  return fmaf((float)cid, step, m);
}

/* ------------------------------------------------------------------------- */
/* QSGD (Alistarh et al., NeurIPS'17) as the second quantiser of Sec. IV-D:   */
/* the magnitude relative to the group's l2-norm is rounded at random to one  */
/* of the levels 0, 1/s, ..., 1 (up with probability equal to the fractional  */
/* position, so the value is unbiased) and sent with the sign.  The y bits of */
/* a record's code hold the sign in the top bit and the level below it, so    */
/* there are s = 2^(y-1) - 1 levels above zero.                               */
/* ------------------------------------------------------------------------- */

/* The norm that goes into the header must come out the same whatever order a
 * machine adds the squares in, so it is defined without floating-point sums:
 * S = sum of x_i^2 as an exact number, and the norm is the smallest fp32 value
 * n with n*n >= S (so no |x_i| exceeds it).  S is kept as a fixed-point number
 * in units of 2^-298 (the square of the smallest denormal) in 32-bit limbs. */
#define QN_LIMBS 20 /* bits 0 .. 639: squares reach bit 2*(127+149)+48 = 600, 2^31 of them 631 */

static void qn_add_square(uint64_t* limb, float x) {
  uint32_t b = f2u(x) & 0x7FFFFFFFu;
  uint32_t e = b >> 23, frac = b & 0x7FFFFFu;
  uint64_t m = e ? (frac | 0x800000u) : frac; /* |x| = m * 2^(q-149), q below */
  uint32_t q = e ? e - 1 : 0;
  uint64_t sq = m * m;                         /* < 2^48, worth sq * 2^(2q) units */
  uint32_t off = 2 * q, word = off / 32, sh = off % 32;
  limb[word] += (sq << sh) & 0xFFFFFFFFu;      /* the three 32-bit pieces of sq << sh (< 2^80) */
  limb[word + 1] += (sq >> (32 - sh)) & 0xFFFFFFFFu;
  limb[word + 2] += sh ? (sq >> (64 - sh)) : 0;
}

static void qn_carry(uint64_t* limb) { /* every limb below 2^32 afterwards */
  uint64_t carry = 0;
  for (int i = 0; i < QN_LIMBS; ++i) {
    uint64_t v = limb[i] + carry;
    limb[i] = v & 0xFFFFFFFFu;
    carry = v >> 32;
  }
}

/* n*n >= S for the fp32 bit pattern `key` (finite, sign clear), S in carried limbs. */
static int qn_square_reaches(uint32_t key, const uint64_t* S) {
  uint64_t sq[QN_LIMBS];
  memset(sq, 0, sizeof(sq));
  qn_add_square(sq, u2f(key));
  qn_carry(sq);
  for (int i = QN_LIMBS - 1; i >= 0; --i)
    if (sq[i] != S[i]) return sq[i] > S[i];
  return 1;
}

int orc_qsgd_norm(const float* x, uint32_t n, float* norm_out) {
  uint64_t S[QN_LIMBS];
  memset(S, 0, sizeof(S));
  for (uint32_t i = 0; i < n; ++i) {
    if (!isfinite(x[i])) return ORC_ERR_NONFINITE;
    qn_add_square(S, x[i]);
  }
  qn_carry(S);
  if (!qn_square_reaches(0x7F7FFFFFu, S)) return ORC_ERR_NONFINITE; /* the norm overflows fp32 */
  uint32_t lo = 0, hi = 0x7F7FFFFFu; /* smallest key whose square reaches S; squares grow with the key */
  while (lo < hi) {
    uint32_t mid = lo + (hi - lo) / 2;
    if (qn_square_reaches(mid, S)) hi = mid; else lo = mid + 1;
  }
  *norm_out = u2f(lo);
  return ORC_OK;
}

static uint32_t qsgd_levels(uint32_t y) { return ((uint32_t)1 << (y - 1)) - 1u; }

/* CID of x in a group with l2-norm `norm` at y bits: position t = |x| * (s/norm)
 * in fp32 (s/norm one correctly rounded division per group), lower level
 * floor(t), one up with probability t - floor(t) resolved against the 24-bit
 * uniform; the sign bit sits above the level.  y = 32 keeps the raw bits. */
uint32_t orc_quantise_qsgd(float x, float norm, uint32_t y, uint32_t u24) {
  if (y == 32) return f2u(x);
  float s = (float)qsgd_levels(y);
  float inv = norm > 0.0f ? s / norm : 0.0f;
  float t = fabsf(x) * inv;
  if (!(t > 0.0f)) t = 0.0f;
  if (t > s) t = s;
  float fl = floorf(t);
  uint32_t level = (uint32_t)fl;
  float p = t - fl;
  uint32_t thr = (uint32_t)(p * 16777216.0f);
  level += (u24 < thr) ? 1u : 0u;
  if (level > qsgd_levels(y)) level = qsgd_levels(y);
  return level | ((f2u(x) >> 31) << (y - 1));
}

/* Value of a CID: sign * level * (norm/s), the spacing one correctly rounded
 * division, the product one rounding. */
float orc_dequantise_qsgd(uint32_t cid, float norm, uint32_t y) {
  if (y == 32) return u2f(cid);
  float s = (float)qsgd_levels(y);
  float step = norm > 0.0f ? norm / s : 0.0f;
  float v = (float)(cid & qsgd_levels(y)) * step;
  return ((cid >> (y - 1)) & 1u) ? -v : v;
}

/* ------------------------------------------------------------------------- */
/* bit stream                                                                 */
/* ------------------------------------------------------------------------- */

/* Bit b of the stream is bit (b mod 32) of little-endian word floor(b/32).
 * Written one bit at a time on purpose. */
static void put_bits(uint32_t* words, uint64_t bitpos, uint64_t value, uint32_t nbits) {
  for (uint32_t b = 0; b < nbits; ++b)
    if ((value >> b) & 1u) words[(bitpos + b) >> 5] |= (uint32_t)1 << ((bitpos + b) & 31u);
}

static uint64_t get_bits(const uint32_t* words, uint64_t bitpos, uint32_t nbits) {
  uint64_t v = 0;
  for (uint32_t b = 0; b < nbits; ++b)
    if ((words[(bitpos + b) >> 5] >> ((bitpos + b) & 31u)) & 1u) v |= (uint64_t)1 << b;
  return v;
}

/* Order used for a group's min and max: numeric order, and -0 below +0, so
 * that the stored extremes do not depend on the order the group is visited in. */
static int value_below(float a, float b) {
  return a < b || (a == b && signbit(a) && !signbit(b));
}

/* Compress one client's update vector.
 *   words_out   cap_words 32-bit words, receives plan->total_bits/32 words
 *   stats_out   R+1 entries (groups 1..R, then the sparsified tail), or NULL
 *   seg_out     d entries, group of every coordinate (0 = dropped), or NULL
 *   cid_out     d entries, CID of every kept coordinate (0 for dropped), or NULL
 * Layout of the stream, all little-endian 32-bit words:
 *   words 0..7   magic, version | quant<<16, d, R, s, bits(B), client, total_words
 *   4 words per coded group: y_r, P_r, bits(min_r), bits(max_r)
 *   then group 1..R payloads: record e of group r in bits [e*W_r, (e+1)*W_r) of
 *   that group's word array, W_r = s + y_r, PID in the low s bits, CID above
 *   it; records in ascending PID; each group padded with zeros to a word. */
int orc_encode(const float* U, const orc_plan* p, uint64_t seed, uint32_t client,
               uint32_t* words_out, uint64_t cap_words, orc_seg_stats* stats_out,
               uint32_t* seg_out, uint32_t* cid_out) {
  if (!U || !p || !words_out) return ORC_ERR_ARG;
  int rc = orc_plan_validate(p);
  if (rc) return rc;
  uint32_t d = p->d, R = p->R, s = p->s;
  uint64_t total_words = p->total_bits / 32u;
  if (cap_words < total_words) return ORC_ERR_CAPACITY;

  uint32_t* order = (uint32_t*)malloc((size_t)d * sizeof(uint32_t));
  if (!order) return ORC_ERR_ARG;
  rc = orc_rank(U, d, order);
  if (rc) { free(order); return rc; }

  memset(words_out, 0, (size_t)total_words * 4u);
  if (seg_out) memset(seg_out, 0, (size_t)d * 4u);
  if (cid_out) memset(cid_out, 0, (size_t)d * 4u);
  words_out[0] = ORC_MAGIC;
  words_out[1] = ORC_VERSION | (p->quant << 16);
  words_out[2] = d;
  words_out[3] = R;
  words_out[4] = s;
  words_out[5] = f2u(p->B);
  words_out[6] = client;
  words_out[7] = (uint32_t)total_words;

  uint64_t l = 0; /* rank cursor */
  uint64_t payload_word = ORC_GLOBAL_HEADER_WORDS + (uint64_t)ORC_SEG_HEADER_WORDS * R;
  for (uint32_t r = 0; r < R; ++r) {
    uint32_t P = p->P[r], y = p->y[r], W = s + y;
    uint32_t* members = order + l; /* the P updates of ranks (Z_{r-1}, Z_r] */
    qsort(members, P, sizeof(uint32_t), cmp_u32); /* ascending position ID */
    float m = 0.0f, M = 0.0f;
    double sumsq = 0.0;
    for (uint32_t e = 0; e < P; ++e) {
      float x = U[members[e]];
      if (e == 0 || value_below(x, m)) m = x;
      if (e == 0 || value_below(M, x)) M = x;
      sumsq += (double)x * (double)x;
    }
    if (P > 0 && !isfinite(M - m)) { free(order); return ORC_ERR_NONFINITE; }
    float norm = 0.0f;
    if (p->quant == 1) { /* centroid distribution of QSGD: the group's l2-norm (Sec. IV-D) */
      float* vals = (float*)malloc((size_t)(P ? P : 1) * sizeof(float));
      if (!vals) { free(order); return ORC_ERR_ARG; }
      for (uint32_t e = 0; e < P; ++e) vals[e] = U[members[e]];
      rc = orc_qsgd_norm(vals, P, &norm);
      free(vals);
      if (rc) { free(order); return rc; }
    }
    uint32_t* hdr = words_out + ORC_GLOBAL_HEADER_WORDS + ORC_SEG_HEADER_WORDS * r;
    hdr[0] = y; hdr[1] = P;
    if (p->quant == 1) { hdr[2] = f2u(norm); hdr[3] = 0; }
    else { hdr[2] = f2u(m); hdr[3] = f2u(M); }
    uint32_t* seg_words = words_out + payload_word;
    double inv_B = 1.0 / (double)p->B; /* the scaling operation of Sec. IV-B: Uhat = Utilde / B */
    double errsq = 0.0;
    for (uint32_t e = 0; e < P; ++e) {
      uint32_t i = members[e];
      uint32_t u24 = orc_u24(seed, client, i);
      uint32_t cid = p->quant == 1 ? orc_quantise_qsgd(U[i], norm, y, u24) : orc_quantise(U[i], m, M, y, u24);
      float xt = p->quant == 1 ? orc_dequantise_qsgd(cid, norm, y) : orc_dequantise(cid, m, M, y);
      double err = (double)xt * inv_B - (double)U[i];
      errsq += err * err;
      uint64_t record = (uint64_t)i | ((uint64_t)cid << s);
      put_bits(seg_words, (uint64_t)e * W, record, W);
      if (seg_out) seg_out[i] = r + 1;
      if (cid_out) cid_out[i] = cid;
    }
    if (stats_out) {
      stats_out[r].min = m; stats_out[r].max = M; stats_out[r].sumsq = sumsq;
      stats_out[r].count = P; stats_out[r].pad = 0; stats_out[r].errsq = errsq;
    }
    payload_word += seg_payload_words(P, W);
    l += P;
  }
  if (stats_out) { /* the sparsified tail: what Proposition 1's first term bounds */
    double sumsq = 0.0;
    for (uint64_t t = l; t < d; ++t) { double x = U[order[t]]; sumsq += x * x; }
    stats_out[R].min = 0.0f; stats_out[R].max = 0.0f; stats_out[R].sumsq = sumsq;
    stats_out[R].count = (uint32_t)(d - l); stats_out[R].pad = 0; stats_out[R].errsq = sumsq;
  }
  free(order);
  return ORC_OK;
}

/* Parse and check one stream's headers. */
typedef struct {
  uint32_t d, R, s, client, quant;
  float B;
  uint32_t y[ORC_MAX_R], P[ORC_MAX_R];
  float m[ORC_MAX_R], M[ORC_MAX_R];
  uint64_t payload_word[ORC_MAX_R];
  uint64_t total_words;
} orc_header;

static int parse_header(const uint32_t* w, uint64_t nwords, uint32_t d_expected, orc_header* h) {
  if (nwords < ORC_GLOBAL_HEADER_WORDS) return ORC_ERR_STREAM;
  if (w[0] != ORC_MAGIC || (w[1] & 0xFFFFu) != ORC_VERSION || (w[1] >> 16) > 1) return ORC_ERR_STREAM;
  h->quant = w[1] >> 16;
  h->d = w[2]; h->R = w[3]; h->s = w[4]; h->B = u2f(w[5]); h->client = w[6]; h->total_words = w[7];
  if (h->d != d_expected || h->R > ORC_MAX_R || h->s != orc_s_bits(h->d)) return ORC_ERR_STREAM;
  if (!(h->B > 0.0f) || !isfinite(h->B)) return ORC_ERR_STREAM;
  uint64_t pos = ORC_GLOBAL_HEADER_WORDS + (uint64_t)ORC_SEG_HEADER_WORDS * h->R;
  if (nwords < pos) return ORC_ERR_STREAM;
  uint64_t k = 0;
  for (uint32_t r = 0; r < h->R; ++r) {
    const uint32_t* sh = w + ORC_GLOBAL_HEADER_WORDS + ORC_SEG_HEADER_WORDS * r;
    h->y[r] = sh[0]; h->P[r] = sh[1]; h->m[r] = u2f(sh[2]); h->M[r] = u2f(sh[3]);
    if (!code_len_ok(h->y[r])) return ORC_ERR_STREAM;
    if (h->quant == 1 && (h->y[r] < 2 || !(h->m[r] >= 0.0f) || sh[3] != 0)) return ORC_ERR_STREAM; /* {norm, 0} */
    if (!isfinite(h->m[r]) || !isfinite(h->M[r]) || !isfinite(h->M[r] - h->m[r])) return ORC_ERR_STREAM;
    k += h->P[r];
    h->payload_word[r] = pos;
    pos += seg_payload_words(h->P[r], h->s + h->y[r]);
  }
  if (k > h->d || pos != h->total_words || nwords < pos) return ORC_ERR_STREAM;
  return ORC_OK;
}

/* PS side (Sec. III step 3 with the scaling of Sec. IV-B): out[j] = sum over
 * clients of w_i * xhat_{i,j}; xhat is the centroid of the CID stored for
 * position j, 0 where the client sent nothing.  Default w_i = 1/(n * B_i).
 * Products and the running sum are kept in double, in client order, and
 * rounded to fp32 once.  accumulate != 0 starts from the values already in
 * out (streamed aggregation). */
int orc_decode_aggregate(uint32_t n, const uint32_t* const* streams, const uint64_t* nwords,
                         const float* weights, uint32_t d, float* out, int accumulate) {
  if (!out || d < 1 || (n > 0 && (!streams || !nwords))) return ORC_ERR_ARG;
  double* acc = (double*)calloc(d, sizeof(double));
  if (!acc) return ORC_ERR_ARG;
  if (accumulate) for (uint32_t j = 0; j < d; ++j) acc[j] = (double)out[j];
  for (uint32_t i = 0; i < n; ++i) {
    orc_header h;
    int rc = parse_header(streams[i], nwords[i], d, &h);
    if (rc) { free(acc); return rc; }
    double w = weights ? (double)weights[i] : 1.0 / ((double)n * (double)h.B);
    for (uint32_t r = 0; r < h.R; ++r) {
      uint32_t W = h.s + h.y[r];
      const uint32_t* seg_words = streams[i] + h.payload_word[r];
      uint32_t prev_pid = 0;
      for (uint32_t e = 0; e < h.P[r]; ++e) {
        uint64_t record = get_bits(seg_words, (uint64_t)e * W, W);
        uint32_t pid = (uint32_t)(record & (((uint64_t)1 << h.s) - 1u));
        uint32_t cid = (uint32_t)(record >> h.s);
        /* a group's records come in strictly ascending position */
        if (pid >= d || (e > 0 && pid <= prev_pid)) { free(acc); return ORC_ERR_STREAM; }
        prev_pid = pid;
        float xt = h.quant == 1 ? orc_dequantise_qsgd(cid, h.m[r], h.y[r]) : orc_dequantise(cid, h.m[r], h.M[r], h.y[r]);
        acc[pid] += w * (double)xt;
      }
    }
  }
  for (uint32_t j = 0; j < d; ++j) out[j] = (float)acc[j];
  free(acc);
  return ORC_OK;
}

/* Read the records of one stream back: pid_out/cid_out/seg_out get k entries
 * in stream order.  Returns k or a negative error. */
int64_t orc_unpack(const uint32_t* stream, uint64_t nwords, uint32_t d, uint32_t* pid_out,
                   uint32_t* cid_out, uint32_t* seg_out) {
  orc_header h;
  int rc = parse_header(stream, nwords, d, &h);
  if (rc) return rc;
  int64_t k = 0;
  for (uint32_t r = 0; r < h.R; ++r) {
    uint32_t W = h.s + h.y[r];
    for (uint32_t e = 0; e < h.P[r]; ++e) {
      uint64_t record = get_bits(stream + h.payload_word[r], (uint64_t)e * W, W);
      if (pid_out) pid_out[k] = (uint32_t)(record & (((uint64_t)1 << h.s) - 1u));
      if (cid_out) cid_out[k] = (uint32_t)(record >> h.s);
      if (seg_out) seg_out[k] = r + 1;
      ++k;
    }
  }
  return k;
}

/* ------------------------------------------------------------------------- */
/* Packets (Sec. IV-C, Eq. (3); Sec. IV-D).  A stream is cut into packets of  */
/* at most mtu bytes, every packet carrying records of one group only and a   */
/* header from which the parameter server can decode it on its own: s, y_r    */
/* and the centroid distribution, as the paper lists, plus what ties it back  */
/* to its place (group, first record) and the stream's global fields.         */
/*   word 0 "CVLP"; 1 version | quant << 16; 2 d; 3 client; 4 bits(B);        */
/*   5 r | R << 8 | y_r << 16 | s << 24; 6 P_r; 7 e0 (first record's number    */
/*   inside its group); 8, 9 the group's two centroid words;                  */
/*   then c = min(cap_r, P_r - e0) records of W_r bits from bit 0, zero padded */
/*   to a word; cap_r = floor((8 mtu - H) / W_r) with H = 320, the largest P   */
/*   that satisfies Eq. (3).  Packets are numbered group by group; an empty    */
/*   group still sends one packet (c = 0) so that its header survives.         */
/* ------------------------------------------------------------------------- */
#define ORC_PKT_MAGIC 0x504C5643u
#define ORC_PKT_HEADER_WORDS 10u

static int pkt_mtu_ok(uint32_t mtu) { return mtu % 4u == 0 && mtu >= 64u && mtu <= 65532u; }

static uint32_t pkt_cap(uint32_t mtu, uint32_t W) { return (8u * mtu - 32u * ORC_PKT_HEADER_WORDS) / W; }

static uint32_t pkt_count_of_group(uint32_t P, uint32_t cap) { return P == 0 ? 1u : (P + cap - 1u) / cap; }

int64_t orc_packet_count(const orc_plan* p, uint32_t mtu) {
  if (!p || !pkt_mtu_ok(mtu)) return ORC_ERR_ARG;
  int64_t n = 0;
  for (uint32_t r = 0; r < p->R; ++r) {
    uint32_t cap = pkt_cap(mtu, p->s + p->y[r]);
    if (cap < 1) return ORC_ERR_ARG;
    n += pkt_count_of_group(p->P[r], cap);
  }
  return n;
}

/* Cuts a stream into packets laid out at a stride of mtu bytes in packets_out
 * (zero filled behind each packet's end); sizes_out[p] receives packet p's
 * length in bytes.  Returns the number of packets or a negative error. */
int64_t orc_packetize(const uint32_t* stream, uint64_t nwords, uint32_t d, uint32_t mtu,
                      uint32_t* packets_out, uint64_t cap_packets, uint32_t* sizes_out) {
  if (!stream || !packets_out || !pkt_mtu_ok(mtu)) return ORC_ERR_ARG;
  orc_header h;
  int rc = parse_header(stream, nwords, d, &h);
  if (rc) return rc;
  uint32_t stride = mtu / 4u;
  uint64_t n = 0;
  for (uint32_t r = 0; r < h.R; ++r) {
    uint32_t W = h.s + h.y[r], cap = pkt_cap(mtu, W);
    if (cap < 1) return ORC_ERR_ARG;
    uint32_t npk = pkt_count_of_group(h.P[r], cap);
    const uint32_t* hdr = stream + ORC_GLOBAL_HEADER_WORDS + ORC_SEG_HEADER_WORDS * r;
    for (uint32_t j = 0; j < npk; ++j, ++n) {
      if (n >= cap_packets) return ORC_ERR_CAPACITY;
      uint32_t* pk = packets_out + n * stride;
      memset(pk, 0, (size_t)mtu);
      uint32_t e0 = j * cap, c = h.P[r] - e0 < cap ? h.P[r] - e0 : cap;
      pk[0] = ORC_PKT_MAGIC; pk[1] = stream[1]; pk[2] = h.d; pk[3] = h.client; pk[4] = f2u(h.B);
      pk[5] = r | (h.R << 8) | (h.y[r] << 16) | (h.s << 24);
      pk[6] = h.P[r]; pk[7] = e0; pk[8] = hdr[2]; pk[9] = hdr[3];
      for (uint32_t e = 0; e < c; ++e)
        put_bits(pk + ORC_PKT_HEADER_WORDS, (uint64_t)e * W,
                 get_bits(stream + h.payload_word[r], (uint64_t)(e0 + e) * W, W), W);
      if (sizes_out) sizes_out[n] = 4u * (ORC_PKT_HEADER_WORDS + (uint32_t)seg_payload_words(c, W));
    }
  }
  return (int64_t)n;
}

/* Puts a stream back together from all its packets, given in any order at a
 * stride of mtu bytes.  Every packet must agree with the others on the global
 * fields and on its group's fields, and every (group, packet number) must be
 * there exactly once.  Returns the stream's length in words or a negative error. */
int64_t orc_depacketize(const uint32_t* packets, uint32_t n_packets, uint32_t mtu, uint32_t d,
                        uint32_t* words_out, uint64_t cap_words) {
  if (!packets || !words_out || !pkt_mtu_ok(mtu) || n_packets < 1) return ORC_ERR_ARG;
  uint32_t stride = mtu / 4u;
  const uint32_t* first = packets;
  uint32_t R = (first[5] >> 8) & 0xFFu, s = first[5] >> 24;
  if (first[0] != ORC_PKT_MAGIC || R > ORC_MAX_R || first[2] != d || s != orc_s_bits(d)) return ORC_ERR_STREAM;
  uint32_t y[ORC_MAX_R], P[ORC_MAX_R], c0[ORC_MAX_R], c1[ORC_MAX_R], have[ORC_MAX_R];
  memset(have, 0, sizeof(have));
  for (uint32_t i = 0; i < n_packets; ++i) { /* the first packet of every group describes it */
    const uint32_t* pk = packets + (uint64_t)i * stride;
    uint32_t r = pk[5] & 0xFFu;
    if (pk[0] != ORC_PKT_MAGIC || r >= R) return ORC_ERR_STREAM;
    if (pk[7] == 0) {
      if (have[r]) return ORC_ERR_STREAM;
      have[r] = 1; y[r] = (pk[5] >> 16) & 0xFFu; P[r] = pk[6]; c0[r] = pk[8]; c1[r] = pk[9];
    }
  }
  uint64_t base[ORC_MAX_R + 1], payload[ORC_MAX_R + 1];
  base[0] = 0; payload[0] = ORC_GLOBAL_HEADER_WORDS + (uint64_t)ORC_SEG_HEADER_WORDS * R;
  for (uint32_t r = 0; r < R; ++r) {
    if (!have[r] || !code_len_ok(y[r])) return ORC_ERR_STREAM;
    uint32_t cap = pkt_cap(mtu, s + y[r]);
    if (cap < 1) return ORC_ERR_STREAM;
    base[r + 1] = base[r] + pkt_count_of_group(P[r], cap);
    payload[r + 1] = payload[r] + seg_payload_words(P[r], s + y[r]);
  }
  if (base[R] != n_packets) return ORC_ERR_STREAM;
  if (payload[R] > cap_words || payload[R] > 0xFFFFFFFFull) return ORC_ERR_CAPACITY;
  memset(words_out, 0, (size_t)payload[R] * 4u);
  words_out[0] = ORC_MAGIC; words_out[1] = first[1]; words_out[2] = d; words_out[3] = R; words_out[4] = s;
  words_out[5] = first[4]; words_out[6] = first[3]; words_out[7] = (uint32_t)payload[R];
  uint8_t* seen = (uint8_t*)calloc(n_packets, 1);
  if (!seen) return ORC_ERR_ARG;
  for (uint32_t i = 0; i < n_packets; ++i) {
    const uint32_t* pk = packets + (uint64_t)i * stride;
    uint32_t r = pk[5] & 0xFFu, W = s + y[r], cap = pkt_cap(mtu, W), e0 = pk[7];
    int ok = pk[1] == first[1] && pk[2] == d && pk[3] == first[3] && pk[4] == first[4] &&
             pk[5] == (r | (R << 8) | (y[r] << 16) | (s << 24)) && pk[6] == P[r] && pk[8] == c0[r] && pk[9] == c1[r] &&
             e0 % cap == 0 && (e0 < P[r] || (e0 == 0 && P[r] == 0));
    if (ok) {
      uint64_t slot = base[r] + e0 / cap;
      ok = !seen[slot];
      seen[slot] = 1;
    }
    if (!ok) { free(seen); return ORC_ERR_STREAM; }
    uint32_t c = P[r] - e0 < cap ? P[r] - e0 : cap;
    for (uint32_t e = 0; e < c; ++e)
      put_bits(words_out + payload[r], (uint64_t)(e0 + e) * W, get_bits(pk + ORC_PKT_HEADER_WORDS, (uint64_t)e * W, W), W);
    uint32_t* hdr = words_out + ORC_GLOBAL_HEADER_WORDS + ORC_SEG_HEADER_WORDS * r;
    hdr[0] = y[r]; hdr[1] = P[r]; hdr[2] = c0[r]; hdr[3] = c1[r];
  }
  free(seen); /* n_packets slots, each taken once: none is missing */
  return (int64_t)payload[R];
}

/* Scale factor for the next round (footnote to Proposition 1): max over the
 * coded groups of Q(P_r, y_r), plus 1, with PQ's quantisation error
 * Q(P, y) = P / (2^y - 1)^2 (appendix case study); a raw 32-bit group has no
 * quantisation error. */
double orc_next_scale(const orc_plan* p) {
  double worst = 0.0;
  for (uint32_t r = 0; r < p->R; ++r) {
    if (p->y[r] == 32 || p->P[r] == 0) continue;
    double Q = p->quant == 1 ? q_qsgd((double)p->P[r], (double)p->y[r]) : q_pq((double)p->P[r], (double)p->y[r]);
    if (Q > worst) worst = Q;
  }
  return worst + 1.0;
}

/* ||Uhat - U||^2 / ||U||^2 of one encoded vector from its statistics block (R
 * coded groups, then the tail): the quantity Propositions 1 and 2 bound by gamma. */
double orc_empirical_gamma(const orc_seg_stats* stats, uint32_t R) {
  double err = 0.0, all = 0.0;
  for (uint32_t r = 0; r <= R; ++r) { err += stats[r].errsq; all += stats[r].sumsq; }
  return all > 0.0 ? err / all : 0.0;
}

/* The points of the fit of Definition 1's exponent: ranks l = 1, 2, 4, ... and
 * l = d, ascending, with the fp32 bit pattern (sign cleared) of the l-th largest
 * magnitude U{l} at each.  Both arrays hold up to 32 entries. */
int orc_fit_points(const float* U, uint32_t d, uint32_t* ranks_out, uint32_t* keys_out, uint32_t* n_out) {
  uint32_t* order = (uint32_t*)malloc((size_t)d * sizeof(uint32_t));
  if (!order) return ORC_ERR_ARG;
  int rc = orc_rank(U, d, order);
  if (rc) { free(order); return rc; }
  uint32_t n = 0;
  for (uint64_t l = 1;; l *= 2) {
    if (l > d) l = d;
    ranks_out[n] = (uint32_t)l;
    keys_out[n] = f2u(U[order[l - 1]]) & 0x7FFFFFFFu;
    ++n;
    if (l == d) break;
  }
  free(order);
  *n_out = n;
  return ORC_OK;
}

/* alpha of Definition 1: least-squares slope of ln|U{l}| against ln l at the
 * ranks l = 1, 2, 4, ... and l = d, skipping zero magnitudes. */
int orc_fit_alpha(const float* U, uint32_t d, double* alpha_out) {
  uint32_t ranks[32], keys[32], np = 0;
  int rc = orc_fit_points(U, d, ranks, keys, &np);
  if (rc) return rc;
  double sx = 0, sy = 0, sxx = 0, sxy = 0; int n = 0;
  for (uint32_t j = 0; j < np; ++j) {
    double mag = (double)u2f(keys[j]);
    if (mag > 0.0) {
      double x = log((double)ranks[j]), yv = log(mag);
      sx += x; sy += yv; sxx += x * x; sxy += x * yv; ++n;
    }
  }
  if (n < 2) { *alpha_out = -1.0; return ORC_OK; }
  *alpha_out = ((double)n * sxy - sx * sy) / ((double)n * sxx - sx * sx);
  return ORC_OK;
}
