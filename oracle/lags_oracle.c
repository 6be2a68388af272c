/*
 * CPU oracle for the per-layer error-compensated top-k sparsifier of LAGS-SGD.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU library and
 * is never part of the product path: only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may load it.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared (never -ffast-math):
 * every float expression below is one IEEE-754 binary32 operation rounded to
 * nearest-even, with no fused multiply-add and no flush of denormals.
 *
 * What it follows (paper: "Layer-wise Adaptive Gradient Sparsification ...",
 * LAGS-SGD):
 *   - Algorithm 1 line 6: acc = residual + lr * grad       (per layer, per worker)
 *   - Eq. 4 (TopK operator) made total: exactly k entries are kept, the k
 *     entries of largest |acc|; equal magnitudes are ordered by lower index first.
 *   - Algorithm 1 line 7: residual = acc - TopK(acc, k)
 *   - Algorithm 1 lines 8-9 / Eq. 5: g = sum over workers of TopK(...), update = g / P.
 *
 * Pins (all in tests/, CPU only): brute-force subset enumeration for d <= 12,
 * hand-computed two-rounding vectors, library partition on tie-free data,
 * closed forms for the merge, the Section 4.2 RandK energy bound.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int64_t offset; /* element offset of the layer in the flat arrays */
  int64_t d;      /* elements in the layer                           */
  double rho;     /* density k/d requested for the layer             */
} oracle_layer;

/* k for a layer of d elements at density rho: at least one entry, at most d.
 * (Section 4.1 only says "top-k^(l)"; the rounding rule is this build's
 * reading: the ceiling of rho*d evaluated in double.) */
int64_t oracle_topk_count(int64_t d, double rho) {
  double x = ceil(rho * (double)d);
  int64_t k = (int64_t)x;
  if (k < 1) k = 1;
  if (k > d) k = d;
  return k;
}

static uint32_t bits_of(float x) {
  uint32_t u;
  memcpy(&u, &x, sizeof u);
  return u;
}

/* |x| as an integer that orders like the magnitude: the bit pattern without
 * the sign bit.  (+0 and -0 both map to 0; NaN patterns rank above infinity.) */
static uint32_t magnitude_key(float x) { return bits_of(x) & 0x7FFFFFFFu; }

/* Algorithm 1 line 6, elementwise: two roundings (product, then sum). */
void oracle_accumulate(const float *grad, const float *residual, int64_t d, float lr, float *acc) {
  for (int64_t i = 0; i < d; ++i) {
    float t = lr * grad[i];
    acc[i] = residual[i] + t;
  }
}

typedef struct {
  uint32_t key;
  int32_t idx;
} keyed;

/* Total order used for selection: larger magnitude first, then lower index. */
static int keyed_before(const void *pa, const void *pb) {
  const keyed *a = (const keyed *)pa, *b = (const keyed *)pb;
  if (a->key != b->key) return a->key > b->key ? -1 : 1;
  if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
  return 0;
}

/*
 * One layer of one worker (Algorithm 1 lines 6-7 with Eq. 4):
 *   acc = residual + lr*grad; sort all entries by (|acc| desc, index asc);
 *   the first k are selected; they are emitted in ascending index with the
 *   exact bits of acc; residual becomes +0.0f at selected entries and acc
 *   (bit for bit) elsewhere.
 * Returns 0, or -1 on bad arguments / out of memory.
 */
int oracle_sparsify_layer(const float *grad, float *residual, int64_t d, float lr, int64_t k,
                          int32_t *out_idx, float *out_val) {
  if (!grad || !residual || !out_idx || !out_val) return -1;
  if (d < 1 || d > 2147483647LL || k < 1 || k > d) return -1;
  float *acc = (float *)malloc((size_t)d * sizeof(float));
  keyed *order = (keyed *)malloc((size_t)d * sizeof(keyed));
  unsigned char *selected = (unsigned char *)calloc((size_t)d, 1);
  if (!acc || !order || !selected) {
    free(acc);
    free(order);
    free(selected);
    return -1;
  }
  oracle_accumulate(grad, residual, d, lr, acc);
  for (int64_t i = 0; i < d; ++i) {
    order[i].key = magnitude_key(acc[i]);
    order[i].idx = (int32_t)i;
  }
  qsort(order, (size_t)d, sizeof(keyed), keyed_before);
  for (int64_t j = 0; j < k; ++j) selected[order[j].idx] = 1;
  int64_t n = 0;
  for (int64_t i = 0; i < d; ++i) {
    if (selected[i]) {
      out_idx[n] = (int32_t)i;
      out_val[n] = acc[i];
      ++n;
      residual[i] = 0.0f;
    } else {
      residual[i] = acc[i];
    }
  }
  free(acc);
  free(order);
  free(selected);
  return n == k ? 0 : -1;
}

/*
 * All layers of one worker.  Layer l writes its k_l pairs at position
 * sum_{j<l} k_j of out_idx/out_val (indices are local to the layer).
 */
int oracle_sparsify_model(const oracle_layer *layers, int32_t n_layers, const float *grad_flat,
                          float *residual_flat, float lr, int32_t *out_idx, float *out_val) {
  if (!layers || n_layers < 0) return -1;
  int64_t out = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    int64_t k = oracle_topk_count(layers[l].d, layers[l].rho);
    int rc = oracle_sparsify_layer(grad_flat + layers[l].offset, residual_flat + layers[l].offset,
                                   layers[l].d, lr, k, out_idx + out, out_val + out);
    if (rc) return rc;
    out += k;
  }
  return 0;
}

/*
 * Algorithm 1 lines 8-9 / Eq. 5: the dense averaged update of P workers.
 * Worker p's pairs sit at idx + p*stride_k, laid out as oracle_sparsify_model
 * writes them.  Sum in worker order p = 0..P-1 starting from +0.0f, then one
 * division by (float)P for every element of every layer.  Elements of
 * update_flat outside all layers are not touched.
 */
int oracle_merge_sparse(const oracle_layer *layers, int32_t n_layers, const int32_t *idx,
                        const float *val, int32_t P, int64_t stride_k, float *update_flat) {
  if (!layers || n_layers < 0 || P < 1 || !idx || !val || !update_flat) return -1;
  int64_t out = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    int64_t d = layers[l].d;
    int64_t k = oracle_topk_count(d, layers[l].rho);
    float *u = update_flat + layers[l].offset;
    for (int64_t i = 0; i < d; ++i) u[i] = 0.0f;
    for (int32_t p = 0; p < P; ++p) {
      const int32_t *pi = idx + (int64_t)p * stride_k + out;
      const float *pv = val + (int64_t)p * stride_k + out;
      for (int64_t j = 0; j < k; ++j) {
        if (pi[j] < 0 || pi[j] >= d) return -1;
        u[pi[j]] = u[pi[j]] + pv[j];
      }
    }
    float fp = (float)P;
    for (int64_t i = 0; i < d; ++i) u[i] = u[i] / fp;
    out += k;
  }
  return 0;
}

/*
 * Algorithm 1 line 9 (Eq. 5): v = v - (1/P) * g with g the sum of the workers' selected
 * entries.  The update is formed exactly as in oracle_merge_sparse (sum in worker order
 * from +0.0f, one division by (float)P) and then subtracted from the parameters in
 * binary32, element by element, for every element of every layer.
 */
int oracle_apply_sparse(const oracle_layer *layers, int32_t n_layers, const int32_t *idx,
                        const float *val, int32_t P, int64_t stride_k, float *param_flat) {
  if (!layers || n_layers < 0 || P < 1 || !idx || !val || !param_flat) return -1;
  int64_t out = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    int64_t d = layers[l].d;
    int64_t k = oracle_topk_count(d, layers[l].rho);
    oracle_layer one = {0, d, layers[l].rho};
    float *update = (float *)malloc((size_t)d * sizeof(float));
    if (!update) return -1;
    int rc = oracle_merge_sparse(&one, 1, idx + out, val + out, P, stride_k, update);
    if (rc) {
      free(update);
      return rc;
    }
    float *v = param_flat + layers[l].offset;
    for (int64_t i = 0; i < d; ++i) v[i] = v[i] - update[i];
    free(update);
    out += k;
  }
  return 0;
}

/*
 * Section 6.2: the per-layer metric delta^(l) that checks Assumption 1, with
 * x^p = acc^p (Algorithm 1 line 6).  Numerator: || sum_p x^p - sum_p TopK(x^p) ||^2, and
 * x^p - TopK(x^p) is the new residual of worker p (Algorithm 1 line 7).  Denominator: the
 * expectation over RandK of || sum_p x^p - RandK(sum_p x^p, k) ||^2, which Section 4.2
 * gives in closed form as (1 - k/d) || sum_p x^p ||^2.  Everything in double.
 *   residual_flat  the residuals AFTER sparsification, worker p at residual_flat + p*res_stride
 *   idx, val       the selected pairs, worker p at + p*stride_k
 *   out            3 doubles per layer: numerator, ||sum_p x^p||^2, delta
 *                  (delta is NaN when the denominator is 0, e.g. k == d)
 */
int oracle_delta_monitor(const oracle_layer *layers, int32_t n_layers, const float *residual_flat,
                         int64_t res_stride, const int32_t *idx, const float *val, int32_t P,
                         int64_t stride_k, double *out3) {
  if (!layers || n_layers < 0 || P < 1 || !residual_flat || !idx || !val || !out3) return -1;
  int64_t out = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    int64_t d = layers[l].d;
    int64_t k = oracle_topk_count(d, layers[l].rho);
    double *sum_res = (double *)calloc((size_t)d, sizeof(double));
    double *sum_sel = (double *)calloc((size_t)d, sizeof(double));
    if (!sum_res || !sum_sel) {
      free(sum_res);
      free(sum_sel);
      return -1;
    }
    for (int32_t p = 0; p < P; ++p) {
      const float *r = residual_flat + (int64_t)p * res_stride + layers[l].offset;
      for (int64_t i = 0; i < d; ++i) sum_res[i] += (double)r[i];
      const int32_t *sel_i = idx + (int64_t)p * stride_k + out;
      const float *sel_v = val + (int64_t)p * stride_k + out;
      for (int64_t j = 0; j < k; ++j) {
        if (sel_i[j] < 0 || sel_i[j] >= d) {
          free(sum_res);
          free(sum_sel);
          return -1;
        }
        sum_sel[sel_i[j]] += (double)sel_v[j];
      }
    }
    double num = 0.0, sq = 0.0;
    for (int64_t i = 0; i < d; ++i) {
      double x = sum_res[i] + sum_sel[i];
      num += sum_res[i] * sum_res[i];
      sq += x * x;
    }
    double den = (1.0 - (double)k / (double)d) * sq;
    out3[3 * l + 0] = num;
    out3[3 * l + 1] = sq;
    out3[3 * l + 2] = den > 0.0 ? num / den : NAN;
    free(sum_res);
    free(sum_sel);
    out += k;
  }
  return 0;
}
