/*
 * Sanitizer driver for the CPU oracle: built together with oracle/cg_ref.c under
 * -fsanitize=address,undefined and run by tests/test_sanitizers_cpu.py.  Every buffer is
 * allocated at its exact size so that an access outside it is reported; the problems walk
 * the branches of the oracle (padding, stride, grouping with the shuffled store, the
 * channel-wise gate, the two-sided gate, the integer path with requantisation) and the
 * hand-computed 3x3 example is checked by value.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/cg_ref.c"

static int failures = 0;
#define EXPECT(c) do { if (!(c)) { printf("FAILED line %d: %s\n", __LINE__, #c); ++failures; } } while (0)

static double *dalloc(size_t n, double v) {
  double *p = (double *)malloc((n ? n : 1) * sizeof(double));
  for (size_t i = 0; i < n; ++i) p[i] = v;
  return p;
}

/* deterministic pseudo-random values in [-1, 1) */
static uint32_t lcg = 12345u;
static double rnd(void) {
  lcg = lcg * 1664525u + 1013904223u;
  return (double)(lcg >> 8) / 8388608.0 - 1.0;
}

static void closed_form_3x3(void) {
  /* all ones, one base and one conditional channel, pad 1, E = 0, Var = 1, Delta = 5, ReLU */
  cg_ref_problem p;
  memset(&p, 0, sizeof p);
  p.n = 1; p.h = 3; p.w = 3; p.c_in = 2; p.c_out = 1; p.c_base = 1; p.kh = p.kw = 3; p.stride = 1; p.pad = 1;
  p.epilogue = CG_REF_RELU;
  double *x = dalloc(18, 1.0), *wb = dalloc(9, 1.0), *wc = dalloc(9, 1.0);
  double mean = 0, var = 1, delta = 5;
  double *y = dalloc(9, -1), *yo = dalloc(9, -1), *marg = dalloc(9, -1);
  uint8_t *d = (uint8_t *)malloc(9);
  uint32_t *bm = (uint32_t *)malloc(9 * 4), *cnt = (uint32_t *)malloc(3 * 4);
  uint64_t macs = 0;
  p.x = x; p.w_base = wb; p.w_cond = wc; p.gate_mean = &mean; p.gate_var = &var; p.delta = &delta;
  p.y = y; p.y_other = yo; p.margin = marg; p.d = d; p.bitmap = bm; p.counts = cnt; p.macs = &macs;
  EXPECT(cg_ref_forward(&p) == 0);
  const double want_y[9] = {4, 12, 4, 12, 18, 12, 4, 12, 4};
  const uint32_t want_d[9] = {0, 1, 0, 1, 1, 1, 0, 1, 0};
  for (int i = 0; i < 9; ++i) {
    EXPECT(y[i] == want_y[i]);
    EXPECT(d[i] == want_d[i]);
    EXPECT(bm[i] == want_d[i]);
  }
  EXPECT(cnt[0] == 5 && cnt[1] == 0 && cnt[2] == 5);
  /* the as-executed form agrees */
  double *y2 = dalloc(9, -1);
  p.y = y2; p.y_other = NULL; p.margin = NULL;
  EXPECT(cg_ref_forward_skip(&p) == 0);
  for (int i = 0; i < 9; ++i) EXPECT(y2[i] == want_y[i]);
  free(x); free(wb); free(wc); free(y); free(yo); free(marg); free(d); free(bm); free(cnt); free(y2);
}

static void float_problem(int n, int h, int w, int c_in, int c_out, int g, int k, int stride, int pad, int groups,
                          int shuffle, double tau_c, int two_sided) {
  cg_ref_problem p;
  memset(&p, 0, sizeof p);
  p.n = n; p.h = h; p.w = w; p.c_in = c_in; p.c_out = c_out; p.c_base = c_in / g; p.kh = p.kw = k;
  p.stride = stride; p.pad = pad; p.groups = groups; p.shuffle = shuffle; p.tau_c = tau_c; p.two_sided = two_sided;
  p.epilogue = CG_REF_RELU | CG_REF_AFFINE | CG_REF_RESIDUAL;
  const int ho = cg_ref_out_h(&p), wo = cg_ref_out_w(&p);
  const size_t nx = (size_t)n * h * w * c_in, nwb = (size_t)c_out * k * k * p.c_base,
               nwc = (size_t)c_out * k * k * (c_in - p.c_base), ny = (size_t)n * ho * wo * c_out;
  double *x = dalloc(nx, 0), *wb = dalloc(nwb, 0), *wc = dalloc(nwc, 0);
  for (size_t i = 0; i < nx; ++i) x[i] = fmax(rnd(), 0);
  for (size_t i = 0; i < nwb; ++i) wb[i] = rnd() * 0.3;
  for (size_t i = 0; i < nwc; ++i) wc[i] = rnd() * 0.3;
  double *mean = dalloc(c_out, 0.05), *var = dalloc(c_out, 0.4), *dl = dalloc(c_out, 0.1), *dh = dalloc(c_out, 1.5);
  double *s0 = dalloc(c_out, 1.1), *h0 = dalloc(c_out, -0.1), *s1 = dalloc(c_out, 0.9), *h1 = dalloc(c_out, 0.2);
  double *res = dalloc(ny, 0.25);
  double *P = dalloc(ny, 0), *R = dalloc(ny, 0), *y = dalloc(ny, 0), *yo = dalloc(ny, 0), *marg = dalloc(ny, 0);
  uint8_t *d = (uint8_t *)malloc(ny ? ny : 1);
  const size_t words = (size_t)(c_out + 31) / 32, m = (size_t)n * ho * wo;
  uint32_t *bm = (uint32_t *)malloc((m * words ? m * words : 1) * 4);
  uint32_t *cnt = (uint32_t *)malloc((2 + (size_t)n * c_out) * 4), *pre = (uint32_t *)malloc(((size_t)n * c_out + 1) * 4);
  uint64_t macs = 0;
  p.x = x; p.w_base = wb; p.w_cond = nwc ? wc : NULL; p.gate_mean = mean; p.gate_var = var; p.delta = dl;
  p.delta_hi = two_sided ? dh : NULL; p.scale0 = s0; p.shift0 = h0; p.scale1 = s1; p.shift1 = h1; p.residual = res;
  p.P = P; p.R = R; p.y = y; p.y_other = yo; p.margin = marg; p.d = d; p.bitmap = bm; p.counts = cnt; p.macs = &macs;
  p.pre_counts = pre;
  EXPECT(cg_ref_forward(&p) == 0);
  uint64_t fired = 0, pop = 0;
  for (size_t i = 0; i < ny; ++i) fired += d[i];
  for (size_t i = 0; i < m * words; ++i) pop += (uint64_t)__builtin_popcount(bm[i]);
  EXPECT(fired == pop);
  EXPECT(fired == ((uint64_t)cnt[0] | ((uint64_t)cnt[1] << 32)));
  if (tau_c == 0.0 && !two_sided && nwc) {
    double *y2 = dalloc(ny, 0);
    p.y = y2; p.y_other = NULL; p.margin = NULL; p.P = p.R = NULL; p.pre_counts = NULL;
    uint64_t macs2 = 0;
    p.macs = &macs2;
    EXPECT(cg_ref_forward_skip(&p) == 0);
    EXPECT(macs2 == macs);
    for (size_t i = 0; i < ny; ++i) EXPECT(y2[i] == y[i]);
    free(y2);
  }
  free(x); free(wb); free(wc); free(mean); free(var); free(dl); free(dh); free(s0); free(h0); free(s1); free(h1);
  free(res); free(P); free(R); free(y); free(yo); free(marg); free(d); free(bm); free(cnt); free(pre);
}

static void int_problem(int n, int h, int w, int c_in, int c_out, int g, int stride, int pad, int out_i8, int groups) {
  cg_ref_problem p;
  memset(&p, 0, sizeof p);
  p.n = n; p.h = h; p.w = w; p.c_in = c_in; p.c_out = c_out; p.c_base = c_in / g; p.kh = p.kw = 3;
  p.stride = stride; p.pad = pad; p.is_int = 1; p.out_i8 = out_i8; p.groups = groups;
  p.epilogue = CG_REF_RELU | CG_REF_RESIDUAL;
  const int ho = cg_ref_out_h(&p), wo = cg_ref_out_w(&p);
  const size_t nx = (size_t)n * h * w * c_in, nwb = (size_t)c_out * 9 * p.c_base, nwc = (size_t)c_out * 9 * (c_in - p.c_base),
               ny = (size_t)n * ho * wo * c_out;
  int8_t *x = (int8_t *)malloc(nx), *wb = (int8_t *)malloc(nwb), *wc = (int8_t *)malloc(nwc ? nwc : 1),
         *res = (int8_t *)malloc(ny ? ny : 1);
  for (size_t i = 0; i < nx; ++i) x[i] = (int8_t)(fabs(rnd()) * 127);
  for (size_t i = 0; i < nwb; ++i) wb[i] = (int8_t)(rnd() * 127);
  for (size_t i = 0; i < nwc; ++i) wc[i] = (int8_t)(rnd() * 127);
  for (size_t i = 0; i < ny; ++i) res[i] = (int8_t)(rnd() * 127);
  int32_t *thr = (int32_t *)malloc(c_out * 4), *m0 = (int32_t *)malloc(c_out * 4), *m1 = (int32_t *)malloc(c_out * 4),
          *bias = (int32_t *)malloc(c_out * 4);
  for (int c = 0; c < c_out; ++c) { thr[c] = 200 * (c % 5) - 300; m0[c] = 70 + c; m1[c] = 60 + c; bias[c] = c % 7 - 3; }
  int32_t *Pi = (int32_t *)malloc((ny ? ny : 1) * 4), *Ri = (int32_t *)malloc((ny ? ny : 1) * 4),
          *yi = (int32_t *)malloc((ny ? ny : 1) * 4), *yo = (int32_t *)malloc((ny ? ny : 1) * 4);
  uint8_t *d = (uint8_t *)malloc(ny ? ny : 1);
  const size_t words = (size_t)(c_out + 31) / 32, m = (size_t)n * ho * wo;
  uint32_t *bm = (uint32_t *)malloc((m * words ? m * words : 1) * 4), *cnt = (uint32_t *)malloc((2 + (size_t)n * c_out) * 4);
  p.xi = x; p.wi_base = wb; p.wi_cond = nwc ? wc : NULL; p.thr = thr; p.rq_mult0 = m0; p.rq_mult1 = m1; p.rq_bias = bias;
  p.rq_shift = 12; p.residual_i8 = res; p.rq_res_mult = 1 << 10;
  p.Pi = Pi; p.Ri = Ri; p.yi = yi; p.yi_other = yo; p.d = d; p.bitmap = bm; p.counts = cnt;
  EXPECT(cg_ref_forward(&p) == 0);
  for (size_t i = 0; i < ny; ++i) {
    if (out_i8) EXPECT(yi[i] >= 0 && yi[i] <= 127);
    if (nwc) EXPECT(d[i] == (Pi[i] >= thr[i % c_out]));
  }
  free(x); free(wb); free(wc); free(res); free(thr); free(m0); free(m1); free(bias); free(Pi); free(Ri); free(yi);
  free(yo); free(d); free(bm); free(cnt);
}

int main(void) {
  closed_form_3x3();
  float_problem(2, 6, 5, 8, 4, 4, 3, 1, 1, 0, 0, 0.0, 0);
  float_problem(2, 7, 6, 8, 6, 2, 3, 2, 1, 0, 0, 0.0, 0);
  float_problem(1, 5, 9, 8, 40, 4, 3, 1, 0, 0, 0, 0.0, 1);         /* two bitmap words, two-sided gate */
  float_problem(3, 4, 4, 8, 8, 4, 3, 1, 1, 4, 1, 0.0, 0);           /* grouping with the shuffled store */
  float_problem(2, 6, 6, 8, 8, 4, 3, 1, 1, 4, 0, 0.4, 0);           /* channel-wise gate */
  float_problem(2, 5, 5, 8, 8, 1, 3, 1, 1, 0, 0, 0.0, 0);           /* dense: no conditional channels */
  float_problem(4, 1, 1, 16, 8, 4, 1, 1, 0, 0, 0, 0.0, 0);          /* fully connected */
  float_problem(2, 3, 3, 8, 4, 4, 3, 1, 0, 0, 0, 0.0, 0);           /* one output pixel per image */
  int_problem(2, 6, 5, 16, 8, 4, 1, 1, 0, 0);
  int_problem(2, 7, 7, 16, 8, 4, 2, 1, 1, 0);
  int_problem(1, 5, 5, 16, 8, 4, 1, 0, 1, 4);
  if (failures) { printf("%d checks failed\n", failures); return 1; }
  printf("oracle sanitizer driver: ok\n");
  return 0;
}
