/*
 * CPU oracle for the pruned-CNN hot path.  TEST INFRASTRUCTURE ONLY: nothing in
 * the product path may link, load or call this file; only the tests, the smoke
 * check and the CPU-baseline leg of the benchmark do.
 *
 * Everything here is the plain definition written out: direct nested loops in
 * textbook order, NCHW / OIHW, fp32 inputs, fp64 accumulation, one final
 * rounding to fp32.  No blocking, no fusion, no reordering.  The only
 * concession to wall-clock is an OpenMP "parallel for" over independent output
 * slices (image, output channel), which does not change any sum's order.
 *
 * Paper passages followed:
 *   Section 2.1 (Pruning, Fig. 2): a layer with c_i input channels and
 *     c_{i+1} filters; removing a filter removes an output channel, removing an
 *     input channel shrinks every filter.
 *   Section 3.5 (Pruning Decision), last paragraph: filters are scored by the
 *     sum of their absolute weights and removed starting from the smallest;
 *     the next layer's input channels are removed to match.
 *   Section 3.4: a subgraph is Conv2d (+BN) (+ReLU).
 * Readings where the paper is silent (cross-correlation, zero padding, floor
 * output size, inference-mode BN with explicit eps, ties to the lower index,
 * kept list ascending) are listed in the design document.
 *
 * Pins: tests/test_oracle_*.py (hand-computed cases, closed forms, impulse
 * response, 1x1 == matmul, fold == unfold, ranking invariants, brute force).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Accumulator of the convolution loops.  double: the parity build, the only one the tests
 * compare against.  Compiled with -DORACLE_ACC_T=float the same loops accumulate in float:
 * that build exists for the CPU timing row of the benchmark alone (what the loops cost at the
 * GPU path's own accumulation width) and is never used as a reference. */
#ifndef ORACLE_ACC_T
#define ORACLE_ACC_T double
#endif

#define ACT_NONE 0
#define ACT_RELU 1
#define ACT_RELU6 2

static double act_apply(double v, int act) {
  if (act == ACT_RELU) return v > 0.0 ? v : 0.0;
  if (act == ACT_RELU6) return v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v);
  return v;
}

/* ---- Section 3.5: L1 score of each filter, summed in index order, in double ---- */
void oracle_l1_scores(const float* w, int c_out, long per_filter, double* scores) {
  for (int j = 0; j < c_out; ++j) {
    double s = 0.0;
    const float* f = w + (long)j * per_filter;
    for (long i = 0; i < per_filter; ++i) s += fabs((double)f[i]);
    scores[j] = s;
  }
}

/* ---- Section 3.5: pruning starts from the smallest score, so the survivors are
 * the `keep` largest.  order = indices by (score descending, index ascending);
 * kept = the first `keep` of order, listed in ascending index.
 * Written as a stable insertion sort so that equal scores keep index order. */
int oracle_rank(const double* scores, int c_out, int keep, int32_t* order, int32_t* kept) {
  if (keep < 1 || keep > c_out) return -1;
  for (int i = 0; i < c_out; ++i) {
    int32_t cur = i;
    int pos = i;
    while (pos > 0 && scores[order[pos - 1]] < scores[cur]) {
      order[pos] = order[pos - 1];
      --pos;
    }
    order[pos] = cur;
  }
  /* ascending list of the kept indices */
  char* flag = (char*)calloc((size_t)c_out, 1);
  if (!flag) return -2;
  for (int i = 0; i < keep; ++i) flag[order[i]] = 1;
  int n = 0;
  for (int i = 0; i < c_out; ++i)
    if (flag[i]) kept[n++] = i;
  free(flag);
  return 0;
}

/* ---- Section 2.1 / 3.5: remove filters (rows) and input channels (columns) ----
 * w: [c_out][c_in][khw]; keep_out / keep_in may be NULL (= keep all). */
void oracle_gather_weights(const float* w, int c_out, int c_in, int khw,
                           const int32_t* keep_out, int n_out,
                           const int32_t* keep_in, int n_in, float* w_out) {
  (void)c_out;
  for (int i = 0; i < n_out; ++i) {
    int o = keep_out ? keep_out[i] : i;
    for (int c = 0; c < n_in; ++c) {
      int ci = keep_in ? keep_in[c] : c;
      for (int t = 0; t < khw; ++t)
        w_out[((long)i * n_in + c) * khw + t] = w[((long)o * c_in + ci) * khw + t];
    }
  }
}

void oracle_gather_vec(const float* v, const int32_t* keep, int n_keep, float* out) {
  for (int i = 0; i < n_keep; ++i) out[i] = v[keep ? keep[i] : i];
}

/* activation channel gather: x [n][c][hw] -> y [n][n_idx][hw] */
void oracle_gather_channels(const float* x, int n, int c, long hw, const int32_t* idx,
                            int n_idx, float* y) {
  for (int b = 0; b < n; ++b)
    for (int i = 0; i < n_idx; ++i)
      memcpy(y + ((long)b * n_idx + i) * hw, x + ((long)b * c + idx[i]) * hw,
             (size_t)hw * sizeof(float));
}

/* ---- BN folding (inference BN: y = gamma (z - mean) / sqrt(var + eps) + beta) ----
 * w'' = w * s, b = beta + (conv_bias - mean) * s with s = gamma / sqrt(var + eps),
 * all in double, each result rounded to fp32 once.  BN pointers all NULL = no BN:
 * w'' = w, b = conv_bias (or 0). */
void oracle_fold_bn(const float* w, int c_out, long per_filter, const float* gamma,
                    const float* beta, const float* mean, const float* var, double eps,
                    const float* conv_bias, float* w_out, float* bias_out) {
  for (int o = 0; o < c_out; ++o) {
    double cb = conv_bias ? (double)conv_bias[o] : 0.0;
    double s = 1.0, b = cb;
    if (gamma) {
      s = (double)gamma[o] / sqrt((double)var[o] + eps);
      b = (double)beta[o] + (cb - (double)mean[o]) * s;
    }
    for (long i = 0; i < per_filter; ++i)
      w_out[(long)o * per_filter + i] = (float)((double)w[(long)o * per_filter + i] * s);
    bias_out[o] = (float)b;
  }
}

/* ---- convolution core (cross-correlation, zero padding), double result ----
 * x [n][c_in][h][w], wt [c_out][c_in/groups][kh][kw], z [n][c_out][ho][wo].
 * groups divides c_in and c_out; group g maps input channels
 * [g*cpg, (g+1)*cpg) to output channels [g*opg, (g+1)*opg). */
void oracle_conv2d_f64(const float* x, const float* wt, int n, int c_in, int h, int w,
                       int c_out, int kh, int kw, int stride, int pad, int groups,
                       double* z) {
  int ho = (h + 2 * pad - kh) / stride + 1;
  int wo = (w + 2 * pad - kw) / stride + 1;
  int cpg = c_in / groups, opg = c_out / groups;
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < n; ++b)
    for (int o = 0; o < c_out; ++o) {
      int g = o / opg;
      for (int y = 0; y < ho; ++y)
        for (int xo = 0; xo < wo; ++xo) {
          ORACLE_ACC_T acc = 0;
          for (int c = 0; c < cpg; ++c)
            for (int u = 0; u < kh; ++u) {
              int iy = y * stride + u - pad;
              if (iy < 0 || iy >= h) continue;
              for (int v = 0; v < kw; ++v) {
                int ix = xo * stride + v - pad;
                if (ix < 0 || ix >= w) continue;
                acc += (ORACLE_ACC_T)x[(((long)b * c_in + g * cpg + c) * h + iy) * w + ix] *
                       (ORACLE_ACC_T)wt[(((long)o * cpg + c) * kh + u) * kw + v];
              }
            }
          z[(((long)b * c_out + o) * ho + y) * wo + xo] = (double)acc;
        }
    }
}

/* One output element of the same convolution (+bias, +residual value, act), for
 * spot checks of tensors too large to compute whole. */
double oracle_conv2d_point(const float* x, const float* wt, int c_in, int h, int w,
                           int c_out, int kh, int kw, int stride, int pad, int groups,
                           int b, int o, int y, int xo) {
  int cpg = c_in / groups, opg = c_out / groups;
  int g = o / opg;
  double acc = 0.0;
  for (int c = 0; c < cpg; ++c)
    for (int u = 0; u < kh; ++u) {
      int iy = y * stride + u - pad;
      if (iy < 0 || iy >= h) continue;
      for (int v = 0; v < kw; ++v) {
        int ix = xo * stride + v - pad;
        if (ix < 0 || ix >= w) continue;
        acc += (double)x[(((long)b * c_in + g * cpg + c) * h + iy) * w + ix] *
               (double)wt[(((long)o * cpg + c) * kh + u) * kw + v];
      }
    }
  return acc;
}

/* ---- epilogues on the double conv result z [n][c][hw] ---- */

/* folded: y = act(z + bias[c] (+ residual)) */
void oracle_bias_act(const double* z, int n, int c, long hw, const float* bias,
                     const float* residual, int act, float* y) {
  for (int b = 0; b < n; ++b)
    for (int o = 0; o < c; ++o)
      for (long i = 0; i < hw; ++i) {
        long idx = ((long)b * c + o) * hw + i;
        double v = z[idx] + (bias ? (double)bias[o] : 0.0);
        if (residual) v += (double)residual[idx];
        y[idx] = (float)act_apply(v, act);
      }
}

/* unfolded: y = act(gamma (z + conv_bias - mean) / sqrt(var + eps) + beta (+ residual)) */
void oracle_bn_act(const double* z, int n, int c, long hw, const float* gamma,
                   const float* beta, const float* mean, const float* var, double eps,
                   const float* conv_bias, const float* residual, int act, float* y) {
  for (int b = 0; b < n; ++b)
    for (int o = 0; o < c; ++o)
      for (long i = 0; i < hw; ++i) {
        long idx = ((long)b * c + o) * hw + i;
        double v = z[idx] + (conv_bias ? (double)conv_bias[o] : 0.0);
        v = (double)gamma[o] * (v - (double)mean[o]) / sqrt((double)var[o] + eps) +
            (double)beta[o];
        if (residual) v += (double)residual[idx];
        y[idx] = (float)act_apply(v, act);
      }
}

/* ---- pooling ---- */

/* max over the in-bounds elements of each window (padding never wins) */
void oracle_maxpool(const float* x, int n, int c, int h, int w, int k, int stride, int pad,
                    float* y) {
  int ho = (h + 2 * pad - k) / stride + 1;
  int wo = (w + 2 * pad - k) / stride + 1;
  for (long bc = 0; bc < (long)n * c; ++bc)
    for (int yo = 0; yo < ho; ++yo)
      for (int xo = 0; xo < wo; ++xo) {
        int have = 0;
        float m = 0.0f;
        for (int u = 0; u < k; ++u) {
          int iy = yo * stride + u - pad;
          if (iy < 0 || iy >= h) continue;
          for (int v = 0; v < k; ++v) {
            int ix = xo * stride + v - pad;
            if (ix < 0 || ix >= w) continue;
            float e = x[(bc * h + iy) * w + ix];
            if (!have || e > m) { m = e; have = 1; }
          }
        }
        y[(bc * ho + yo) * wo + xo] = m;
      }
}

/* spatial mean per (image, channel): double sum / (h*w) */
void oracle_gavgpool(const float* x, int n, int c, long hw, float* y) {
  for (long bc = 0; bc < (long)n * c; ++bc) {
    double s = 0.0;
    for (long i = 0; i < hw; ++i) s += (double)x[bc * hw + i];
    y[bc] = (float)(s / (double)hw);
  }
}

/* ---- fully connected: y[b][o] = act(sum_f x[b][f] w[o][f] + bias[o]) ---- */
void oracle_fc(const float* x, const float* wt, const float* bias, int n, int f, int c_out,
               int act, float* y) {
  for (int b = 0; b < n; ++b)
    for (int o = 0; o < c_out; ++o) {
      double acc = 0.0;
      for (int i = 0; i < f; ++i) acc += (double)x[(long)b * f + i] * (double)wt[(long)o * f + i];
      acc += bias ? (double)bias[o] : 0.0;
      y[(long)b * c_out + o] = (float)act_apply(acc, act);
    }
}
