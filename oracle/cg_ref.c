/*
 * CPU oracle for the channel-gated convolution layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of the
 * layer that the GPU library is checked against.  It shares no code with the
 * GPU path and must never be called from it.  Only the tests, the smoke check
 * and the CPU-baseline leg of the benchmark may load it.
 *
 * What it computes (paper: "Channel Gating Neural Networks", Sec. 3.1-3.2):
 *
 *   split     x = [x_p, x_r] along channels, x_p = the first c_base channels,
 *             W = [W_p, W_r] likewise, so W*x = W_p*x_p + W_r*x_r   (Sec. 3.1)
 *   base      P = W_p * x_p        (always evaluated)               (Sec. 3.1)
 *   gate      d = theta(P - Delta*sqrt(Var) - E), theta(v)=1 iff v>=0
 *                                                   (Heaviside step, merged
 *                                                    BN gate of Sec. 3.2)
 *   cond.     R = W_r * x_r        (needed only where d = 1)        (Sec. 3.1)
 *   output    y = f(P) where d = 0, f(P + R) where d = 1            (Eq. 1)
 *
 * "*" is the usual deep-learning cross-correlation with symmetric zero
 * padding and floor output size; the paper does not say, this is the reading
 * taken.  f is an optional per-channel scale/shift (inference-time batch norm,
 * Sec. 3.1 footnote; one pair per branch because training uses two BNs,
 * Sec. 4), an optional residual add and an optional ReLU.
 *
 * Precision: the float path takes every input already widened to double and
 * accumulates in double.  The integer path takes int8 inputs, accumulates in
 * int32 and compares with an int32 threshold, so it is exact.
 *
 * The loops below are the definition written out: n, ho, wo, co, r, s, c.
 * OpenMP only spreads (n, ho) rows over threads; no blocking or reordering.
 *
 * Channel grouping (Sec. 3.3), groups = G > 1: input and output channels are
 * cut into G equal consecutive groups; output group i takes input group i as
 * x_p and the other input groups, in increasing order, as x_r.  w_base then
 * holds, for each output channel, the weights of its own input group, w_cond
 * those of the remaining c_in - c_base channels in that order.  With
 * shuffle != 0 the output channels are stored shuffled (Sec. 3.3, the optional
 * ShuffleNet operation): channel j of output group i goes to position j*G + i
 * of y (and reads the residual there); P, R, d, margin, bitmap and counts keep
 * the natural channel order.
 *
 * Channel-wise gate (Sec. 3.2, the weight-access extension): with tau_c > 0 an
 * output channel of an image keeps its conditional path only if at least a
 * fraction tau_c of its activations fired, S = theta(sum_{pixels} s - tau_c *
 * wo * ho) with theta(0) = 1; where S = 0 every activation of that channel and
 * image takes the d = 0 branch of Eq. 1.  d, bitmap, counts, macs and y then
 * describe the decisions after this gate; pre_counts keeps the sums it
 * thresholded.  tau_c = 0 switches it off (a sum is never negative).  The paper
 * defines the sum over one feature map; with a batch it is taken per image.
 *
 * All tensors are NHWC: x[n][h][w][c_in], outputs [n][ho][wo][c_out].
 * Weights: w_base[c_out][kh][kw][c_base], w_cond[c_out][kh][kw][c_in-c_base].
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define CG_REF_RELU 1u
#define CG_REF_AFFINE 2u
#define CG_REF_RESIDUAL 4u

typedef struct cg_ref_problem {
  int32_t n, h, w, c_in, c_out, c_base;
  int32_t kh, kw, stride, pad;
  int32_t is_int;      /* 0: float path (double inputs), 1: int8 path */
  int32_t out_i8;      /* int path: 1 = requantise to int8, 0 = raw int32 sum */
  uint32_t epilogue;   /* CG_REF_* flags */
  int32_t two_sided;   /* float path: also require z <= delta_hi (Sec. 3.2,
                          gate for saturating activations) */
  int32_t groups;      /* 0 or 1: x_p = first c_base channels for every output
                          channel; G > 1: channel grouping (Sec. 3.3) */
  int32_t shuffle;     /* grouping only: store y channel-shuffled */
  double tau_c;        /* channel-wise gate threshold, fraction of ho*wo; 0 = off */

  /* float path inputs */
  const double *x, *w_base, *w_cond;
  const double *gate_mean, *gate_var, *delta, *delta_hi; /* [c_out] */
  double gate_eps;
  const double *scale0, *shift0, *scale1, *shift1;       /* [c_out] or NULL */
  const double *residual;                                /* like y, or NULL */

  /* int path inputs */
  const int8_t *xi, *wi_base, *wi_cond;
  const int32_t *thr;                                    /* [c_out] */
  const int32_t *rq_mult0, *rq_mult1, *rq_bias;          /* [c_out] */
  int32_t rq_shift;
  const int8_t *residual_i8;
  int32_t rq_res_mult;

  /* outputs; any may be NULL */
  double *P, *R;          /* float path partial sums */
  double *y, *y_other;    /* y under the oracle's decision / under the opposite one */
  double *margin;         /* |z - Delta| in normalised units */
  int32_t *Pi, *Ri;       /* int path partial sums */
  int32_t *yi, *yi_other;
  uint8_t *d;             /* one byte per activation */
  uint32_t *bitmap;       /* [M][ceil(c_out/32)], bit (co&31) of word co>>5 */
  uint32_t *counts;       /* [2 + n*c_out]: total (lo,hi), then per (image, channel) */
  uint64_t *macs;         /* multiply-adds on in-range taps: base everywhere,
                             conditional only where the gate fired (Eq. 1) */
  uint32_t *pre_counts;   /* [n*c_out]: fired activations per (image, channel)
                             before the channel-wise gate */
} cg_ref_problem;

static int out_size(int in, int k, int stride, int pad) {
  int span = in + 2 * pad - k;
  if (span < 0) return 0;
  return span / stride + 1;
}

int cg_ref_out_h(const cg_ref_problem *p) { return out_size(p->h, p->kh, p->stride, p->pad); }
int cg_ref_out_w(const cg_ref_problem *p) { return out_size(p->w, p->kw, p->stride, p->pad); }

/* f for the float path: branch-specific affine, residual, ReLU (Eq. 1's f). */
static double finish_float(const cg_ref_problem *p, double s, int fired, int co, size_t o) {
  double a = s;
  if (p->epilogue & CG_REF_AFFINE) {
    const double *sc = fired ? p->scale1 : p->scale0;
    const double *sh = fired ? p->shift1 : p->shift0;
    a = (sc ? sc[co] : 1.0) * s + (sh ? sh[co] : 0.0);
  }
  if ((p->epilogue & CG_REF_RESIDUAL) && p->residual) a += p->residual[o];
  if ((p->epilogue & CG_REF_RELU) && a < 0.0) a = 0.0;
  return a;
}

/* f for the int path.  Without requantisation the int32 sum is the output
 * (residual add and ReLU still apply).  With it: fixed-point multiply, bias,
 * residual, round-half-up shift, clamp. */
static int32_t finish_int(const cg_ref_problem *p, int32_t s, int fired, int co, size_t o) {
  if (!p->out_i8) {
    int64_t a = s;
    if ((p->epilogue & CG_REF_RESIDUAL) && p->residual_i8)
      a += (int64_t)p->residual_i8[o] * p->rq_res_mult;
    if ((p->epilogue & CG_REF_RELU) && a < 0) a = 0;
    if (a > INT32_MAX) a = INT32_MAX;
    if (a < INT32_MIN) a = INT32_MIN;
    return (int32_t)a;
  }
  const int32_t *mu = fired ? p->rq_mult1 : p->rq_mult0;
  int64_t t = (int64_t)s * (mu ? mu[co] : 1);
  if (p->rq_bias) t += (int64_t)p->rq_bias[co] * ((int64_t)1 << p->rq_shift);
  if ((p->epilogue & CG_REF_RESIDUAL) && p->residual_i8)
    t += (int64_t)p->residual_i8[o] * p->rq_res_mult;
  if (p->rq_shift > 0) {
    t += (int64_t)1 << (p->rq_shift - 1);
    /* arithmetic shift = floor division by 2^shift */
    int64_t q = t / ((int64_t)1 << p->rq_shift);
    if (t % ((int64_t)1 << p->rq_shift) < 0) q -= 1;
    t = q;
  }
  int64_t lo = (p->epilogue & CG_REF_RELU) ? 0 : -128;
  if (t < lo) t = lo;
  if (t > 127) t = 127;
  return (int32_t)t;
}

/*
 * Returns 0 on success, 1 on an invalid problem.  counts and bitmap are
 * overwritten in full.
 */
int cg_ref_forward(const cg_ref_problem *p) {
  if (!p || p->n < 0 || p->h <= 0 || p->w <= 0 || p->c_in <= 0 || p->c_out <= 0) return 1;
  if (p->c_base <= 0 || p->c_base > p->c_in) return 1;
  if (p->kh <= 0 || p->kw <= 0 || p->stride <= 0 || p->pad < 0) return 1;
  if (p->is_int ? (!p->xi || !p->wi_base) : (!p->x || !p->w_base)) return 1;

  const int N = p->n, H = p->h, W = p->w, C = p->c_in, CO = p->c_out, CP = p->c_base;
  const int CR = C - CP;
  if (CR > 0 && (p->is_int ? !p->wi_cond : !p->w_cond)) return 1;
  const int gated = CR > 0;
  const int G = p->groups > 1 ? p->groups : 1;
  if (G > 1 && ((long long)CP * G != C || CO % G != 0)) return 1;
  if (p->shuffle && G == 1) return 1;
  const int CPG = CO / G; /* output channels per group */
  if (gated && (p->is_int ? !p->thr : (!p->gate_mean || !p->gate_var || !p->delta))) return 1;
  const int KH = p->kh, KW = p->kw, ST = p->stride, PD = p->pad;
  const int HO = cg_ref_out_h(p), WO = cg_ref_out_w(p);
  const int words = (CO + 31) / 32;
  const size_t M = (size_t)N * HO * WO;

  if (p->bitmap) memset(p->bitmap, 0, M * words * sizeof(uint32_t));
  if (p->counts) memset(p->counts, 0, (2 + (size_t)N * CO) * sizeof(uint32_t));

  uint64_t total_fired = 0, total_macs = 0;

#pragma omp parallel for collapse(2) schedule(static) reduction(+ : total_fired, total_macs)
  for (int n = 0; n < N; ++n) {
    for (int ho = 0; ho < HO; ++ho) {
      for (int wo = 0; wo < WO; ++wo) {
        const size_t m = ((size_t)n * HO + ho) * WO + wo;
        for (int co = 0; co < CO; ++co) {
          const size_t o = m * CO + co;
          const int grp = co / CPG;       /* output group = its base input group */
          const int b0 = grp * CP;        /* first channel of x_p */
          /* x_r: the channels outside [b0, b0+CP), increasing; index c sits at
           * channel c below the gap and c + CP above it */
          const size_t oy = p->shuffle ? m * CO + (size_t)(co % CPG) * G + grp : o;
          double accP = 0.0, accR = 0.0;
          int32_t iP = 0, iR = 0;
          uint64_t taps_in = 0;
          for (int r = 0; r < KH; ++r) {
            const int hi = ho * ST - PD + r;
            if (hi < 0 || hi >= H) continue;
            for (int s = 0; s < KW; ++s) {
              const int wi = wo * ST - PD + s;
              if (wi < 0 || wi >= W) continue;
              ++taps_in;
              const size_t xo = (((size_t)n * H + hi) * W + wi) * C;
              const size_t wbo = (((size_t)co * KH + r) * KW + s) * CP;
              const size_t wco = (((size_t)co * KH + r) * KW + s) * CR;
              if (p->is_int) {
                for (int c = 0; c < CP; ++c) iP += (int32_t)p->xi[xo + b0 + c] * (int32_t)p->wi_base[wbo + c];
                for (int c = 0; c < CR; ++c)
                  iR += (int32_t)p->xi[xo + (c < b0 ? c : c + CP)] * (int32_t)p->wi_cond[wco + c];
              } else {
                for (int c = 0; c < CP; ++c) accP += p->x[xo + b0 + c] * p->w_base[wbo + c];
                for (int c = 0; c < CR; ++c) accR += p->x[xo + (c < b0 ? c : c + CP)] * p->w_cond[wco + c];
              }
            }
          }

          /* gate: Heaviside step on the normalised partial sum, ties fire */
          int fired = 0;
          double marg = INFINITY;
          if (gated) {
            if (p->is_int) {
              fired = iP >= p->thr[co];
              marg = fabs((double)iP - (double)p->thr[co]);
            } else {
              const double sd = sqrt(p->gate_var[co] + p->gate_eps);
              const double dl = p->delta[co];
              if (isinf(dl)) {
                fired = dl < 0;
              } else {
                const double t = p->gate_mean[co] + dl * sd;
                fired = accP >= t;
                marg = sd > 0 ? fabs((accP - p->gate_mean[co]) / sd - dl) : fabs(accP - t);
              }
              if (p->two_sided && p->delta_hi && !isinf(p->delta_hi[co])) {
                const double th = p->gate_mean[co] + p->delta_hi[co] * sd;
                fired = fired && (accP <= th);
                const double mh = sd > 0 ? fabs((accP - p->gate_mean[co]) / sd - p->delta_hi[co]) : fabs(accP - th);
                if (mh < marg) marg = mh;
              } else if (p->two_sided && p->delta_hi && p->delta_hi[co] < 0) {
                fired = 0; /* upper threshold -inf: nothing passes */
              }
            }
          } else {
            fired = 1; /* no conditional channels: plain dense convolution */
          }

          total_macs += taps_in * (uint64_t)(CP + (fired ? CR : 0));

          if (p->is_int) {
            const int32_t s_dec = fired ? iP + iR : iP;
            const int32_t s_oth = fired ? iP : iP + iR;
            if (p->Pi) p->Pi[o] = iP;
            if (p->Ri) p->Ri[o] = iR;
            if (p->yi) p->yi[oy] = finish_int(p, s_dec, fired, co, oy);
            if (p->yi_other) p->yi_other[oy] = finish_int(p, s_oth, !fired, co, oy);
          } else {
            const double s_dec = fired ? accP + accR : accP;
            const double s_oth = fired ? accP : accP + accR;
            if (p->P) p->P[o] = accP;
            if (p->R) p->R[o] = accR;
            if (p->y) p->y[oy] = finish_float(p, s_dec, fired, co, oy);
            if (p->y_other) p->y_other[oy] = finish_float(p, s_oth, !fired, co, oy);
          }
          if (p->margin) p->margin[o] = marg;
          if (p->d) p->d[o] = (uint8_t)(gated ? fired : 0);
          if (gated && fired) {
            ++total_fired;
            if (p->bitmap) p->bitmap[m * words + (co >> 5)] |= 1u << (co & 31);
            if (p->counts) {
#pragma omp atomic
              p->counts[2 + (size_t)n * CO + co] += 1u;
            }
          }
        }
      }
    }
  }
  if (p->pre_counts && p->counts)
    memcpy(p->pre_counts, p->counts + 2, (size_t)N * CO * sizeof(uint32_t));

  /* channel-wise gate: where fewer than tau_c * ho * wo activations of an
   * (image, channel) fired, all of them fall back to the base path alone */
  if (gated && p->tau_c > 0.0) {
    if (!p->d || !p->counts) return 1; /* the pass needs the decisions and their sums */
    if (p->is_int ? (!p->yi || !p->yi_other) : (!p->y || !p->y_other)) return 1;
    const double need = p->tau_c * (double)((size_t)HO * WO);
    for (int n = 0; n < N; ++n) {
      for (int co = 0; co < CO; ++co) {
        uint32_t *cnt = &p->counts[2 + (size_t)n * CO + co];
        if ((double)*cnt >= need) continue; /* S = 1 */
        const int grp = co / CPG;
        for (int ho = 0; ho < HO; ++ho) {
          for (int wo = 0; wo < WO; ++wo) {
            const size_t m = ((size_t)n * HO + ho) * WO + wo;
            const size_t o = m * CO + co;
            if (!p->d[o]) continue;
            const size_t oy = p->shuffle ? m * CO + (size_t)(co % CPG) * G + grp : o;
            p->d[o] = 0;
            if (p->bitmap) p->bitmap[m * words + (co >> 5)] &= ~(1u << (co & 31));
            if (p->is_int) {
              const int32_t t = p->yi[oy];
              p->yi[oy] = p->yi_other[oy];
              p->yi_other[oy] = t;
            } else {
              const double t = p->y[oy];
              p->y[oy] = p->y_other[oy];
              p->y_other[oy] = t;
            }
            uint64_t taps_in = 0;
            for (int r = 0; r < KH; ++r) {
              const int hi = ho * ST - PD + r;
              if (hi < 0 || hi >= H) continue;
              for (int s = 0; s < KW; ++s) {
                const int wi = wo * ST - PD + s;
                if (wi >= 0 && wi < W) ++taps_in;
              }
            }
            total_macs -= taps_in * (uint64_t)CR;
            --total_fired;
          }
        }
        *cnt = 0;
      }
    }
  }

  if (p->counts) {
    p->counts[0] = (uint32_t)(total_fired & 0xffffffffu);
    p->counts[1] = (uint32_t)(total_fired >> 32);
  }
  if (p->macs) *p->macs = total_macs;
  return 0;
}

/*
 * The layer as Eq. 1 executes it: the base sum everywhere, the gate, and the
 * conditional sum only where the gate fired -- the work the method saves is
 * not done here either.  Same loops and order as cg_ref_forward within each of
 * the two sums, so with double accumulators y, d, bitmap, counts and macs are
 * identical to cg_ref_forward's.  Used for the CPU timing of the benchmark,
 * where it is also built with -DCG_REF_ACC=float (single-precision
 * accumulators, the float path only; integers stay exact).  Outputs: y / yi,
 * d, bitmap, counts, macs (any may be NULL).  The channel-wise gate and the
 * two-sided gate are not offered (returns 1).
 */
#ifndef CG_REF_ACC
#define CG_REF_ACC double
#endif
int cg_ref_forward_skip(const cg_ref_problem *p) {
  if (!p || p->n < 0 || p->h <= 0 || p->w <= 0 || p->c_in <= 0 || p->c_out <= 0) return 1;
  if (p->c_base <= 0 || p->c_base > p->c_in) return 1;
  if (p->kh <= 0 || p->kw <= 0 || p->stride <= 0 || p->pad < 0) return 1;
  if (p->is_int ? (!p->xi || !p->wi_base) : (!p->x || !p->w_base)) return 1;
  if (p->tau_c > 0.0 || p->two_sided) return 1;
  const int N = p->n, H = p->h, W = p->w, C = p->c_in, CO = p->c_out, CP = p->c_base;
  const int CR = C - CP;
  if (CR > 0 && (p->is_int ? !p->wi_cond : !p->w_cond)) return 1;
  const int gated = CR > 0;
  const int G = p->groups > 1 ? p->groups : 1;
  if (G > 1 && ((long long)CP * G != C || CO % G != 0)) return 1;
  if (p->shuffle && G == 1) return 1;
  const int CPG = CO / G;
  if (gated && (p->is_int ? !p->thr : (!p->gate_mean || !p->gate_var || !p->delta))) return 1;
  const int KH = p->kh, KW = p->kw, ST = p->stride, PD = p->pad;
  const int HO = cg_ref_out_h(p), WO = cg_ref_out_w(p);
  const int words = (CO + 31) / 32;
  const size_t M = (size_t)N * HO * WO;
  if (p->bitmap) memset(p->bitmap, 0, M * words * sizeof(uint32_t));
  if (p->counts) memset(p->counts, 0, (2 + (size_t)N * CO) * sizeof(uint32_t));
  uint64_t total_fired = 0, total_macs = 0;

#pragma omp parallel for collapse(2) schedule(static) reduction(+ : total_fired, total_macs)
  for (int n = 0; n < N; ++n) {
    for (int ho = 0; ho < HO; ++ho) {
      for (int wo = 0; wo < WO; ++wo) {
        const size_t m = ((size_t)n * HO + ho) * WO + wo;
        for (int co = 0; co < CO; ++co) {
          const size_t o = m * CO + co;
          const int grp = co / CPG;
          const int b0 = grp * CP;
          const size_t oy = p->shuffle ? m * CO + (size_t)(co % CPG) * G + grp : o;
          /* base path (Sec. 3.1): always */
          CG_REF_ACC accP = 0;
          int32_t iP = 0;
          uint64_t taps_in = 0;
          for (int r = 0; r < KH; ++r) {
            const int hi = ho * ST - PD + r;
            if (hi < 0 || hi >= H) continue;
            for (int s = 0; s < KW; ++s) {
              const int wi = wo * ST - PD + s;
              if (wi < 0 || wi >= W) continue;
              ++taps_in;
              const size_t xo = (((size_t)n * H + hi) * W + wi) * C;
              const size_t wbo = (((size_t)co * KH + r) * KW + s) * CP;
              if (p->is_int) {
                for (int c = 0; c < CP; ++c) iP += (int32_t)p->xi[xo + b0 + c] * (int32_t)p->wi_base[wbo + c];
              } else {
                for (int c = 0; c < CP; ++c) accP += (CG_REF_ACC)(p->x[xo + b0 + c] * p->w_base[wbo + c]);
              }
            }
          }
          /* gate (Sec. 3.2): ties fire */
          int fired = 1;
          if (gated) {
            if (p->is_int) {
              fired = iP >= p->thr[co];
            } else {
              const double dl = p->delta[co];
              if (isinf(dl))
                fired = dl < 0;
              else
                fired = (double)accP >= p->gate_mean[co] + dl * sqrt(p->gate_var[co] + p->gate_eps);
            }
          }
          /* conditional path (Eq. 1): only where the gate fired */
          CG_REF_ACC accR = 0;
          int32_t iR = 0;
          if (gated && fired) {
            for (int r = 0; r < KH; ++r) {
              const int hi = ho * ST - PD + r;
              if (hi < 0 || hi >= H) continue;
              for (int s = 0; s < KW; ++s) {
                const int wi = wo * ST - PD + s;
                if (wi < 0 || wi >= W) continue;
                const size_t xo = (((size_t)n * H + hi) * W + wi) * C;
                const size_t wco = (((size_t)co * KH + r) * KW + s) * CR;
                if (p->is_int) {
                  for (int c = 0; c < CR; ++c)
                    iR += (int32_t)p->xi[xo + (c < b0 ? c : c + CP)] * (int32_t)p->wi_cond[wco + c];
                } else {
                  for (int c = 0; c < CR; ++c)
                    accR += (CG_REF_ACC)(p->x[xo + (c < b0 ? c : c + CP)] * p->w_cond[wco + c]);
                }
              }
            }
          }
          total_macs += taps_in * (uint64_t)(CP + ((gated && fired) ? CR : 0));
          if (p->is_int) {
            if (p->yi) p->yi[oy] = finish_int(p, iP + iR, fired, co, oy);
          } else {
            if (p->y) p->y[oy] = finish_float(p, (double)accP + (double)accR, fired, co, oy);
          }
          if (p->d) p->d[o] = (uint8_t)(gated ? fired : 0);
          if (gated && fired) {
            ++total_fired;
            if (p->bitmap) p->bitmap[m * words + (co >> 5)] |= 1u << (co & 31);
            if (p->counts) {
#pragma omp atomic
              p->counts[2 + (size_t)n * CO + co] += 1u;
            }
          }
        }
      }
    }
  }
  if (p->counts) {
    p->counts[0] = (uint32_t)(total_fired & 0xffffffffu);
    p->counts[1] = (uint32_t)(total_fired >> 32);
  }
  if (p->macs) *p->macs = total_macs;
  return 0;
}

/*
 * The dense pieces of a ResNet around the gated layers (the paper's experiments
 * run ResNet-18, Sec. 5), as plain definitions in double precision, NHWC.
 */

/* y[n][ho][wo][co] = relu?(scale[co] * sum_{r,s,c} x[n][ho*st-pad+r][wo*st-pad+s][c] * w[co][r][s][c] + shift[co]),
 * taps outside the image contribute nothing; scale / shift may be NULL (1 / 0). */
int cg_ref_dense_conv(const double *x, const double *w, const double *scale, const double *shift, double *y, int n,
                      int h, int wd, int c_in, int c_out, int k, int stride, int pad, int relu) {
  if (!x || !w || !y || n < 0 || h <= 0 || wd <= 0 || c_in <= 0 || c_out <= 0 || k <= 0 || stride <= 0 || pad < 0)
    return 1;
  const int ho = out_size(h, k, stride, pad), wo = out_size(wd, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int i = 0; i < n; ++i)
    for (int oy = 0; oy < ho; ++oy)
      for (int ox = 0; ox < wo; ++ox)
        for (int co = 0; co < c_out; ++co) {
          double acc = 0.0;
          for (int r = 0; r < k; ++r) {
            const int hi = oy * stride - pad + r;
            if (hi < 0 || hi >= h) continue;
            for (int s = 0; s < k; ++s) {
              const int wi = ox * stride - pad + s;
              if (wi < 0 || wi >= wd) continue;
              for (int c = 0; c < c_in; ++c)
                acc += x[(((size_t)i * h + hi) * wd + wi) * c_in + c] * w[(((size_t)co * k + r) * k + s) * c_in + c];
            }
          }
          double a = (scale ? scale[co] : 1.0) * acc + (shift ? shift[co] : 0.0);
          if (relu && a < 0.0) a = 0.0;
          y[(((size_t)i * ho + oy) * wo + ox) * c_out + co] = a;
        }
  return 0;
}

/* 3x3 max pooling, stride 2, padding 1: the maximum over the taps inside the image. */
int cg_ref_maxpool3x3s2(const double *x, double *y, int n, int h, int wd, int c) {
  if (!x || !y || n < 0 || h <= 0 || wd <= 0 || c <= 0) return 1;
  const int ho = out_size(h, 3, 2, 1), wo = out_size(wd, 3, 2, 1);
  for (int i = 0; i < n; ++i)
    for (int oy = 0; oy < ho; ++oy)
      for (int ox = 0; ox < wo; ++ox)
        for (int ch = 0; ch < c; ++ch) {
          double m = -INFINITY;
          for (int r = 0; r < 3; ++r) {
            const int hi = oy * 2 - 1 + r;
            if (hi < 0 || hi >= h) continue;
            for (int s = 0; s < 3; ++s) {
              const int wi = ox * 2 - 1 + s;
              if (wi < 0 || wi >= wd) continue;
              const double v = x[(((size_t)i * h + hi) * wd + wi) * c + ch];
              if (v > m) m = v;
            }
          }
          y[(((size_t)i * ho + oy) * wo + ox) * c + ch] = m;
        }
  return 0;
}

/* logits[n][k] = sum_c wfc[k][c] * mean_p x[n][p][c] + bias[k] */
int cg_ref_avgpool_fc(const double *x, const double *wfc, const double *bias, double *logits, int n, int hw, int c,
                      int classes) {
  if (!x || !wfc || !logits || n < 0 || hw <= 0 || c <= 0 || classes <= 0) return 1;
  for (int i = 0; i < n; ++i)
    for (int k = 0; k < classes; ++k) {
      double s = 0.0;
      for (int ch = 0; ch < c; ++ch) {
        double m = 0.0;
        for (int p = 0; p < hw; ++p) m += x[((size_t)i * hw + p) * c + ch];
        s += wfc[(size_t)k * c + ch] * (m / hw);
      }
      logits[(size_t)i * classes + k] = s + (bias ? bias[k] : 0.0);
    }
  return 0;
}
