/*
 * Drives every entry point of the CPU oracle once on small synthetic inputs, so
 * that a build under AddressSanitizer and UndefinedBehaviorSanitizer can show
 * memory errors and undefined arithmetic in the oracle itself.  Test
 * infrastructure: compiled and run by tests/test_oracle_pins.py only.  The
 * oracle is included as source so that its static helpers are instrumented too.
 */
#include "../oracle/cvlc_oracle.c"

#include <stdio.h>

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

static uint32_t lcg_state = 12345u;
static float next_value(void) { /* heavy-tailed values of either sign, a few exact zeros and ties */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  uint32_t r = lcg_state >> 8;
  if ((r & 63u) == 0) return 0.0f;
  if ((r & 63u) == 1) return -0.0f;
  if ((r & 63u) == 2) return 0.25f;
  float mag = ldexpf((float)(r & 0xFFFFu) / 65536.0f + 1e-3f, -(int)((r >> 16) & 15u));
  return (r & 0x800000u) ? -mag : mag;
}

static int run_case(uint32_t d, uint32_t R, const uint32_t* y, const uint32_t* P, float B, uint32_t quant) {
  orc_plan p;
  memset(&p, 0, sizeof(p));
  p.d = d; p.R = R; p.s = orc_s_bits(d); p.B = B; p.quant = quant;
  for (uint32_t r = 0; r < R; ++r) { p.y[r] = y[r]; p.P[r] = P[r]; }
  p.total_bits = orc_plan_total_bits(&p);
  CHECK(orc_plan_validate(&p) == ORC_OK);
  float* U = (float*)malloc(sizeof(float) * d);
  for (uint32_t i = 0; i < d; ++i) U[i] = next_value();
  uint64_t nw = p.total_bits / 32u;
  uint32_t* words = (uint32_t*)malloc(sizeof(uint32_t) * (nw ? nw : 1));   /* exactly the stream: an overrun is seen */
  uint32_t* seg = (uint32_t*)malloc(sizeof(uint32_t) * d);
  uint32_t* cid = (uint32_t*)malloc(sizeof(uint32_t) * d);
  orc_seg_stats* stats = (orc_seg_stats*)malloc(sizeof(orc_seg_stats) * (R + 1));
  CHECK(orc_encode(U, &p, 0x123456789ABCDEFull, 7u, words, nw, stats, seg, cid) == ORC_OK);
  CHECK(orc_encode(U, &p, 1u, 0u, words, nw ? nw - 1 : 0, NULL, NULL, NULL) == ORC_ERR_CAPACITY || nw == 0);
  CHECK(orc_encode(U, &p, 0x123456789ABCDEFull, 7u, words, nw, NULL, NULL, NULL) == ORC_OK);
  CHECK(orc_segments(U, &p, seg) == ORC_OK);
  CHECK(orc_empirical_gamma(stats, R) >= 0.0);
  uint32_t k = 0;
  for (uint32_t r = 0; r < R; ++r) k += P[r];
  uint32_t* pid = (uint32_t*)malloc(sizeof(uint32_t) * (k ? k : 1));
  uint32_t* cc = (uint32_t*)malloc(sizeof(uint32_t) * (k ? k : 1));
  uint32_t* sg = (uint32_t*)malloc(sizeof(uint32_t) * (k ? k : 1));
  CHECK(orc_unpack(words, nw, d, pid, cc, sg) == (int64_t)k);
  float* out = (float*)malloc(sizeof(float) * d);
  const uint32_t* ptrs[2] = {words, words};
  uint64_t sizes[2] = {nw, nw};
  float wts[2] = {0.5f, -2.0f};
  CHECK(orc_decode_aggregate(2, ptrs, sizes, NULL, d, out, 0) == ORC_OK);
  CHECK(orc_decode_aggregate(2, ptrs, sizes, wts, d, out, 1) == ORC_OK);
  CHECK(orc_decode_aggregate(0, NULL, NULL, NULL, d, out, 0) == ORC_OK);
  /* every truncation of the stream is refused without reading past its end */
  for (uint64_t cut = 0; cut < nw; cut += (nw / 37u) + 1u) {
    uint32_t* part = (uint32_t*)malloc(sizeof(uint32_t) * (cut ? cut : 1));
    memcpy(part, words, sizeof(uint32_t) * cut);
    const uint32_t* pp[1] = {part};
    uint64_t ss[1] = {cut};
    CHECK(orc_decode_aggregate(1, pp, ss, NULL, d, out, 0) != ORC_OK);
    free(part);
  }
  /* packets */
  const uint32_t mtus[3] = {64u, 1500u, 9000u};
  for (int m = 0; m < 3; ++m) {
    int64_t np = orc_packet_count(&p, mtus[m]);
    CHECK(np >= (int64_t)R);
    uint32_t stride = mtus[m] / 4u;
    uint32_t* pk = (uint32_t*)calloc((size_t)(np ? np : 1) * stride, sizeof(uint32_t));
    uint32_t* sz = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)(np ? np : 1));
    CHECK(orc_packetize(words, nw, d, mtus[m], pk, (uint64_t)np, sz) == np);
    if (np > 0) {
      uint32_t* back = (uint32_t*)malloc(sizeof(uint32_t) * (nw ? nw : 1));
      CHECK(orc_depacketize(pk, (uint32_t)np, mtus[m], d, back, nw) == (int64_t)nw);
      CHECK(memcmp(back, words, sizeof(uint32_t) * nw) == 0);
      if (np > 1) CHECK(orc_depacketize(pk, (uint32_t)np - 1u, mtus[m], d, back, nw) < 0);
      CHECK(orc_depacketize(pk, (uint32_t)np, mtus[m], d, back, nw - 1u) < 0);
      free(back);
    }
    free(pk); free(sz);
  }
  free(U); free(words); free(seg); free(cid); free(stats); free(pid); free(cc); free(sg); free(out);
  return 0;
}

int main(void) {
  /* generator and scalar helpers */
  uint32_t ctr[4] = {0, 0, 0, 0}, key[2] = {0, 0}, o[4];
  orc_philox4x32_10(ctr, key, o);
  CHECK(o[0] == 0x6627e8d5u);
  CHECK(orc_u24(~0ull, ~0u, ~0u) < (1u << 24));
  CHECK(orc_s_bits(1) == 1 && orc_s_bits(0x7FFFFFFFu) == 31);
  CHECK(orc_quantise(0.5f, -1.0f, 1.0f, 16, 0) <= 65535u);
  CHECK(orc_dequantise(65535u, -1.0f, 1.0f, 16) == 1.0f);
  CHECK(orc_quantise_qsgd(-0.5f, 1.0f, 16, 0xFFFFFFu) >> 15 == 1u);
  CHECK(orc_dequantise_qsgd(0u, 0.0f, 2) == 0.0f);

  /* planner: the three modes, both quantisers, budgets that do not fit */
  orc_plan p;
  const uint32_t y3[3] = {8, 4, 2};
  const double f3[3] = {0.10, 0.15, 0.25};
  CHECK(orc_plan_fractions(65536u, 3, y3, f3, 1.0f, &p) == ORC_OK);
  CHECK(orc_plan_budget(1200000u, 600000u, 3, y3, 2.0f, &p) == ORC_OK);
  CHECK(orc_plan_budget(1200000u, 300u, 3, y3, 2.0f, &p) == ORC_ERR_BUDGET);
  CHECK(orc_plan_alg1(200000u, 150000u, 5, -0.6, 1.0f, &p) == ORC_OK);
  CHECK(orc_gamma(&p, -0.6) > 0.0 && orc_next_scale(&p) >= 1.0);
  CHECK(orc_plan_alg1_quant(200000u, 150000u, 31, -0.5, 3.0f, 1, &p) == ORC_OK);
  CHECK(orc_plan_alg1_quant(7u, 100000u, 3, -0.9, 1.0f, 0, &p) == ORC_OK);
  CHECK(orc_plan_alg1(200000u, 100u, 5, -0.6, 1.0f, &p) == ORC_ERR_BUDGET);
  double Psweep[31], g;
  CHECK(orc_alg1_sweep(200000u, 150000u, 31, -0.7, 1.0f, 0, 900.0, Psweep, &g) == ORC_OK);

  /* encode / decode / packets: raw, wide, 1-bit and empty groups, everything kept, nothing kept */
  { const uint32_t y[4] = {32, 16, 3, 1}, P[4] = {5, 0, 40, 100}; if (run_case(1000u, 4, y, P, 1.0f, 0)) return 1; }
  { const uint32_t y[2] = {9, 2}, P[2] = {17, 4083}; if (run_case(4100u, 2, y, P, 2.5f, 1)) return 1; }
  { const uint32_t y[1] = {7}, P[1] = {333}; if (run_case(333u, 1, y, P, 1.0f, 0)) return 1; }
  { const uint32_t y[1] = {1}, P[1] = {1}; if (run_case(1u, 1, y, P, 1.0f, 0)) return 1; }
  { if (run_case(50u, 0, NULL, NULL, 1.0f, 0)) return 1; }
  { uint32_t y[31], P[31]; for (int r = 0; r < 31; ++r) { y[r] = 16u - (uint32_t)r / 2u; P[r] = 3u + (uint32_t)r; }
    if (run_case(70001u, 31, y, P, 1.0f, 0)) return 1; }

  /* exponent fit, ranking, exact norm */
  float U[513];
  uint32_t order[513], ranks[32], keys[32], np = 0;
  for (int i = 0; i < 513; ++i) U[i] = next_value();
  CHECK(orc_rank(U, 513u, order) == ORC_OK);
  CHECK(orc_fit_points(U, 513u, ranks, keys, &np) == ORC_OK && np >= 2);
  double alpha;
  CHECK(orc_fit_alpha(U, 513u, &alpha) == ORC_OK);
  CHECK(orc_fit_alpha(U, 1u, &alpha) == ORC_OK);
  float norm;
  CHECK(orc_qsgd_norm(U, 513u, &norm) == ORC_OK && norm > 0.0f);
  U[100] = INFINITY;
  CHECK(orc_fit_points(U, 513u, ranks, keys, &np) != ORC_OK);
  puts("oracle sanitizer run: ok");
  return 0;
}
