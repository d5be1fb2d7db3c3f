/*
 * CPU oracle of the KVSwap decode-step hot path -- TEST INFRASTRUCTURE ONLY.
 * See kvswap_oracle.h for conventions and pins.  Plain C, fp64, no blocking,
 * no fusion, no reordering: each function is the paper's statement of the
 * step, written as loops.
 */
#include "kvswap_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---- storage access ----------------------------------------------------- */

/* Value of an 8-bit float code, OCP "E4M3" (finite-only variant): 1 sign, 4 exponent
 * (bias 7), 3 mantissa bits; exponent 0 is subnormal (m/8 * 2^-6); the code with all
 * exponent and mantissa bits set is NaN; there are no infinities; largest value 448. */
double oracle_fp8_e4m3_value(uint8_t code) {
  const int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
  double v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0) v = ldexp((double)m / 8.0, -6);
  else v = ldexp(1.0 + (double)m / 8.0, e - 7);
  return sign ? -v : v;
}

/* Nearest finite E4M3 code to x, ties to the even mantissa, magnitudes beyond the
 * largest value saturate to +-448 (NaN -> the NaN code). */
uint8_t oracle_round_to_fp8_e4m3(double x) {
  if (isnan(x)) return 0x7F;
  const uint8_t sign = signbit(x) ? 0x80 : 0x00;
  double a = fabs(x);
  if (a >= 448.0) return sign | 0x7E;
  /* spacing of the format at a: 2^-9 below 2^-6 (subnormals and the first binade share
   * it), else 2^(floor(log2 a) - 3) */
  int e;
  (void)frexp(a, &e);                 /* a = f * 2^e, f in [0.5, 1) => floor(log2 a) = e-1 */
  int ulp_exp = (e - 1) - 3;
  if (ulp_exp < -9) ulp_exp = -9;
  double steps = nearbyint(ldexp(a, -ulp_exp)); /* nearest-even in the default mode */
  double y = ldexp(steps, ulp_exp);             /* a value of the format (may be 2^k of the next binade) */
  if (y == 0.0) return sign;
  (void)frexp(y, &e);
  int be = (e - 1) + 7;                         /* biased exponent */
  uint8_t code;
  if (be <= 0) code = (uint8_t)nearbyint(ldexp(y, 9)); /* subnormal: y = m * 2^-9 */
  else code = (uint8_t)((be << 3) | (int)nearbyint((ldexp(y, -(e - 1)) - 1.0) * 8.0));
  return sign | code;
}

static double load_elem(const void* base, int dtype, size_t i) {
  if (dtype == ORC_F32) return (double)((const float*)base)[i];
  if (dtype == ORC_FP8_E4M3) return oracle_fp8_e4m3_value(((const uint8_t*)base)[i]);
  uint32_t bits = (uint32_t)((const uint16_t*)base)[i] << 16; /* bf16 = top half of fp32 */
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/* Nearest bf16 (8 significant bits, fp32 exponent range) to x, ties to even.
 * The value is first snapped to the bf16 grid in fp64 (nearbyint rounds to
 * nearest-even in the default rounding mode), which makes the following
 * narrowing conversions exact. */
uint16_t oracle_round_to_bf16(double x) {
  if (x == 0.0 || isnan(x) || isinf(x)) {
    float f = (float)x;
    uint32_t b;
    memcpy(&b, &f, sizeof b);
    return (uint16_t)(b >> 16);
  }
  int e;
  (void)frexp(x, &e);          /* |x| = m * 2^e, m in [0.5, 1)  => floor(log2|x|) = e-1 */
  int ulp_exp = (e - 1) - 7;   /* spacing of bf16 numbers in this binade */
  if (ulp_exp < -126 - 7) ulp_exp = -126 - 7; /* subnormal range: fixed spacing */
  double y = ldexp(nearbyint(ldexp(x, -ulp_exp)), ulp_exp);
  float f = (float)y;          /* exact, or +-inf on overflow */
  uint32_t b;
  memcpy(&b, &f, sizeof b);
  return (uint16_t)(b >> 16);
}

static void store_meta(void* base, int dtype, size_t i, double x) {
  if (dtype == ORC_F32) ((float*)base)[i] = (float)x; /* C conversion: nearest-even */
  else if (dtype == ORC_FP8_E4M3) ((uint8_t*)base)[i] = oracle_round_to_fp8_e4m3(x);
  else ((uint16_t*)base)[i] = oracle_round_to_bf16(x);
}

/* The metadata is stored divided by a scale (so that it fits the range of a narrow dtype)
 * and multiplied back when it is read (Sec. 3.2: the precision of the compressed K cache
 * may be traded).  The scale is meta_scale for every selection set, or, if meta_scales is
 * given, meta_scales[set] with set = b * H_kv + k (set = b in joint mode). */
static double meta_scale(const orc_params* p, size_t set) {
  if (p->meta_scales) return p->meta_scales[set];
  return p->meta_scale != 0.0 ? p->meta_scale : 1.0;
}

static int params_ok(const orc_params* p) {
  if (!p) return 0;
  if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->head_dim < 1 ||
      p->rank < 1 || p->ctx_len < 1 || p->group_size < 1)
    return 0;
  if (p->n_q_heads % p->n_kv_heads) return 0;
  if (p->ctx_len % p->group_size) return 0;
  if (p->kv_dtype != ORC_F32 && p->kv_dtype != ORC_BF16) return 0;
  if (p->meta_dtype != ORC_F32 && p->meta_dtype != ORC_BF16 && p->meta_dtype != ORC_FP8_E4M3)
    return 0;
  if (!(p->meta_scale >= 0.0) || isinf(p->meta_scale)) return 0;
  if (p->meta_scales) {
    const long sets = p->head_mode == ORC_HEADS_JOINT ? p->batch : (long)p->batch * p->n_kv_heads;
    for (long i = 0; i < sets; ++i)
      if (!(p->meta_scales[i] > 0.0) || isinf(p->meta_scales[i])) return 0;
  }
  if (p->head_mode != ORC_HEADS_SEPARATE && p->head_mode != ORC_HEADS_JOINT) return 0;
  if (p->ctx_capacity != 0 && p->ctx_capacity < p->ctx_len) return 0;
  return 1;
}

/* rows allocated per problem in K, V and K_lr */
static size_t row_capacity(const orc_params* p) {
  return (size_t)(p->ctx_capacity > 0 ? p->ctx_capacity : p->ctx_len);
}

/* ---- K_lr = K . A  (Sec. 3.2) -------------------------------------------- */

/* joint-head design: row n of the flattened cache is (K[b,0,n,:], ..., K[b,H_kv-1,n,:]) */
static int build_metadata_joint(const orc_params* p, const void* K, const float* A,
                                void* K_lr, double* K_lr_exact, int row0, int row1) {
  const int Hk = p->n_kv_heads, d = p->head_dim, r = p->rank;
  const size_t cap = row_capacity(p);
  long b;
  int n;
#pragma omp parallel for collapse(2) schedule(static) num_threads(p->n_threads > 1 ? p->n_threads : 1)
  for (b = 0; b < p->batch; ++b) {
    for (n = row0; n < row1; ++n) {
      const size_t orow = ((size_t)b * cap + n) * r;
      for (int j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int k = 0; k < Hk; ++k) {
          const size_t krow = (((size_t)b * Hk + k) * cap + n) * d;
          for (int i = 0; i < d; ++i) /* flattened column k*d + i */
            acc += load_elem(K, p->kv_dtype, krow + i) * (double)A[((size_t)k * d + i) * r + j];
        }
        if (K_lr_exact) K_lr_exact[orow + j] = acc;
        store_meta(K_lr, p->meta_dtype, orow + j, acc / meta_scale(p, (size_t)b));
      }
    }
  }
  return 0;
}

int oracle_build_metadata_rows(const orc_params* p, const void* K, const float* A,
                               void* K_lr, double* K_lr_exact, int32_t first_row,
                               int32_t n_rows) {
  if (!params_ok(p) || !K || !A || !K_lr) return -1;
  const size_t cap = row_capacity(p);
  if (first_row < 0 || n_rows < 0 || (size_t)first_row + (size_t)n_rows > cap) return -1;
  const int row0 = first_row, row1 = first_row + n_rows;
  if (p->head_mode == ORC_HEADS_JOINT)
    return build_metadata_joint(p, K, A, K_lr, K_lr_exact, row0, row1);
  const int Hk = p->n_kv_heads, d = p->head_dim, r = p->rank;
  const long P = (long)p->batch * Hk;
  long pi;
#pragma omp parallel for schedule(dynamic) num_threads(p->n_threads > 1 ? p->n_threads : 1)
  for (pi = 0; pi < P; ++pi) {
    const int k = (int)(pi % Hk);
    const float* Ak = A + (size_t)k * d * r;
    for (int n = row0; n < row1; ++n) {
      const size_t krow = ((size_t)pi * cap + n) * d;
      const size_t orow = ((size_t)pi * cap + n) * r;
      for (int j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i)
          acc += load_elem(K, p->kv_dtype, krow + i) * (double)Ak[(size_t)i * r + j];
        if (K_lr_exact) K_lr_exact[orow + j] = acc;
        store_meta(K_lr, p->meta_dtype, orow + j, acc / meta_scale(p, (size_t)pi));
      }
    }
  }
  return 0;
}

int oracle_build_metadata(const orc_params* p, const void* K, const float* A,
                          void* K_lr, double* K_lr_exact) {
  if (!params_ok(p)) return -1;
  return oracle_build_metadata_rows(p, K, A, K_lr, K_lr_exact, 0, p->ctx_len);
}

/* ---- prediction + selection (Sec. 3.3) ----------------------------------- */

typedef struct {
  double score;
  int32_t index;
} scored_group;

/* descending score; equal scores: ascending index */
static int cmp_scored(const void* a, const void* b) {
  const scored_group* x = (const scored_group*)a;
  const scored_group* y = (const scored_group*)b;
  if (x->score > y->score) return -1;
  if (x->score < y->score) return 1;
  return (x->index > y->index) - (x->index < y->index);
}

static int cmp_i32(const void* a, const void* b) {
  const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* "Scoring and selection": group representatives of the token scores s[0..N), the M
 * best groups (ties to the lower index) in ascending index order.  g is scratch for
 * NG entries; gs_out (NG doubles) and boundary (2 doubles) are nullable. */
static void select_groups(const orc_params* p, const double* s, scored_group* g, int32_t* out,
                          double* gs_out, double* boundary) {
  const int G = p->group_size, M = p->n_select, NG = p->ctx_len / G;
  for (int j = 0; j < NG; ++j) {
    double rep;
    if (p->reduce == ORC_REDUCE_MEAN) {
      rep = 0.0;
      for (int t = 0; t < G; ++t) rep += s[(size_t)j * G + t];
      rep /= (double)G;
    } else {
      rep = s[(size_t)j * G];
      for (int t = 1; t < G; ++t)
        if (s[(size_t)j * G + t] > rep) rep = s[(size_t)j * G + t];
    }
    g[j].score = rep;
    g[j].index = j;
    if (gs_out) gs_out[j] = rep;
  }
  qsort(g, (size_t)NG, sizeof(scored_group), cmp_scored);
  for (int m = 0; m < M; ++m) out[m] = g[m].index;
  qsort(out, (size_t)M, sizeof(int32_t), cmp_i32);
  if (boundary) {
    boundary[0] = g[M - 1].score;
    boundary[1] = (M < NG) ? g[M].score : -INFINITY;
  }
}

/* joint-head design: every query head h scores the sequence's single K_lr with its
 * low-rank query q[h] . A_{g(h)}, A_k being rows k*d .. k*d+d-1 of the adapter (Eq. 1) */
static int predict_select_joint(const orc_params* p, const void* q, const void* K_lr,
                                const float* A, int32_t* idx, double* gs_out, double* s_out,
                                double* boundary) {
  const int Hq = p->n_q_heads, Hk = p->n_kv_heads, d = p->head_dim, r = p->rank;
  const int N = p->ctx_len, M = p->n_select, NG = N / p->group_size, qpk = Hq / Hk;
  int failed = 0;
  long b;
#pragma omp parallel for schedule(dynamic) num_threads(p->n_threads > 1 ? p->n_threads : 1)
  for (b = 0; b < p->batch; ++b) {
    double* q_lr = (double*)malloc(sizeof(double) * (size_t)Hq * r);
    double* s = (double*)malloc(sizeof(double) * (size_t)N);
    scored_group* g = (scored_group*)malloc(sizeof(scored_group) * (size_t)NG);
    if (!q_lr || !s || !g) {
      failed = 1;
      free(q_lr); free(s); free(g);
      continue;
    }
    for (int h = 0; h < Hq; ++h) {
      const float* Ak = A + (size_t)(h / qpk) * d * r; /* block of the shared KV head */
      const size_t qrow = ((size_t)b * Hq + h) * d;
      for (int j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i)
          acc += load_elem(q, p->kv_dtype, qrow + i) * (double)Ak[(size_t)i * r + j];
        q_lr[(size_t)h * r + j] = acc;
      }
    }
    for (int n = 0; n < N; ++n) {
      const size_t row = ((size_t)b * row_capacity(p) + n) * r;
      double tot = 0.0;
      for (int h = 0; h < Hq; ++h) {
        double acc = 0.0;
        for (int j = 0; j < r; ++j)
          acc += q_lr[(size_t)h * r + j] * (meta_scale(p, (size_t)b) * load_elem(K_lr, p->meta_dtype, row + j));
        tot += acc;
      }
      s[n] = tot;
      if (s_out) s_out[(size_t)b * N + n] = tot;
    }
    select_groups(p, s, g, idx + (size_t)b * M, gs_out ? gs_out + (size_t)b * NG : NULL,
                  boundary ? boundary + b * 2 : NULL);
    free(q_lr); free(s); free(g);
  }
  return failed ? -2 : 0;
}

int oracle_predict_select(const orc_params* p, const void* q, const void* K_lr,
                          const float* A, int32_t* idx, double* gs_out, double* s_out,
                          double* boundary) {
  if (!params_ok(p) || !q || !K_lr || !A || !idx) return -1;
  const int Hq = p->n_q_heads, Hk = p->n_kv_heads, d = p->head_dim, r = p->rank;
  const int N = p->ctx_len, G = p->group_size, M = p->n_select;
  const int NG = N / G, qpk = Hq / Hk;
  if (M < 1 || M > NG) return -1;
  if (p->head_mode == ORC_HEADS_JOINT)
    return predict_select_joint(p, q, K_lr, A, idx, gs_out, s_out, boundary);
  const long P = (long)p->batch * Hk;
  int failed = 0;
  long pi;
#pragma omp parallel for schedule(dynamic) num_threads(p->n_threads > 1 ? p->n_threads : 1)
  for (pi = 0; pi < P; ++pi) {
    const int b = (int)(pi / Hk), k = (int)(pi % Hk);
    const float* Ak = A + (size_t)k * d * r;
    double* q_lr = (double*)malloc(sizeof(double) * (size_t)qpk * r);
    double* s = (double*)malloc(sizeof(double) * (size_t)N);
    scored_group* g = (scored_group*)malloc(sizeof(scored_group) * (size_t)NG);
    if (!q_lr || !s || !g) {
      failed = 1;
      free(q_lr); free(s); free(g);
      continue;
    }
    /* low-rank query vectors of the heads that share KV head k */
    for (int hh = 0; hh < qpk; ++hh) {
      const int h = k * qpk + hh;
      const size_t qrow = ((size_t)b * Hq + h) * d;
      for (int j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i)
          acc += load_elem(q, p->kv_dtype, qrow + i) * (double)Ak[(size_t)i * r + j];
        q_lr[(size_t)hh * r + j] = acc;
      }
    }
    /* token importance: per-head low-rank logits, summed over the heads */
    for (int n = 0; n < N; ++n) {
      const size_t row = ((size_t)pi * row_capacity(p) + n) * r;
      double tot = 0.0;
      for (int hh = 0; hh < qpk; ++hh) {
        double acc = 0.0;
        for (int j = 0; j < r; ++j)
          acc += q_lr[(size_t)hh * r + j] * (meta_scale(p, (size_t)pi) * load_elem(K_lr, p->meta_dtype, row + j));
        tot += acc;
      }
      s[n] = tot;
      if (s_out) s_out[(size_t)pi * N + n] = tot;
    }
    select_groups(p, s, g, idx + (size_t)pi * M, gs_out ? gs_out + (size_t)pi * NG : NULL,
                  boundary ? boundary + pi * 2 : NULL);
    free(q_lr); free(s); free(g);
  }
  return failed ? -2 : 0;
}

/* ---- attention ----------------------------------------------------------- */

/* One softmax over the listed tokens of one (b, h) followed by the first rb_len
 * rolling-buffer tokens of its KV head: out = sum_t w_t V_t / sum_t w_t with
 * w_t = exp(scale * q.K_t - max).  rows[t] is the index of the token's row in K and V
 * counted in rows of d elements from the start of the arrays (the caller resolves cache
 * position or mapping table); rb_K / rb_V may be NULL when rb_len is 0. */
static int attend_rows(const orc_params* p, const void* q, const void* K, const void* V,
                       int b, int h, const size_t* rows, long n_tok, const void* rb_K,
                       const void* rb_V, long rb_len, long rb_capacity, double scale,
                       double* out) {
  const int Hq = p->n_q_heads, Hk = p->n_kv_heads, d = p->head_dim;
  const int k = h / (Hq / Hk);
  const size_t qrow = ((size_t)b * Hq + h) * d;
  const size_t rbbase = ((size_t)b * Hk + k) * (size_t)rb_capacity * d;
  const long total = n_tok + rb_len;
  double* z = (double*)malloc(sizeof(double) * (size_t)total);
  if (!z) return -2;
  double zmax = -INFINITY;
  for (long t = 0; t < total; ++t) {
    /* token t: a listed row, or (after all of those) a buffer row */
    const void* src = t < n_tok ? K : rb_K;
    const size_t row = t < n_tok ? rows[t] * d : rbbase + (size_t)(t - n_tok) * d;
    double acc = 0.0;
    for (int i = 0; i < d; ++i)
      acc += load_elem(q, p->kv_dtype, qrow + i) * load_elem(src, p->kv_dtype, row + i);
    z[t] = scale * acc;
    if (z[t] > zmax) zmax = z[t];
  }
  double denom = 0.0;
  for (int i = 0; i < d; ++i) out[i] = 0.0;
  for (long t = 0; t < total; ++t) {
    const double w = exp(z[t] - zmax);
    const void* src = t < n_tok ? V : rb_V;
    const size_t row = t < n_tok ? rows[t] * d : rbbase + (size_t)(t - n_tok) * d;
    denom += w;
    for (int i = 0; i < d; ++i) out[i] += w * load_elem(src, p->kv_dtype, row + i);
  }
  for (int i = 0; i < d; ++i) out[i] /= denom;
  free(z);
  return 0;
}

static double resolve_scale(const orc_params* p) {
  return p->softmax_scale != 0.0 ? p->softmax_scale : 1.0 / sqrt((double)p->head_dim);
}

int oracle_sparse_attn(const orc_params* p, const void* q, const void* K, const void* V,
                       const int32_t* idx, double* out) {
  return oracle_sparse_attn_rb(p, q, K, V, idx, NULL, NULL, 0, 0, out);
}

int oracle_sparse_attn_rb(const orc_params* p, const void* q, const void* K, const void* V,
                          const int32_t* idx, const void* rb_K, const void* rb_V,
                          int32_t rb_len, int32_t rb_capacity, double* out) {
  if (!params_ok(p) || !q || !K || !V || !idx || !out) return -1;
  if (rb_len < 0 || rb_len > rb_capacity || (rb_len > 0 && (!rb_K || !rb_V))) return -1;
  const int Hq = p->n_q_heads, Hk = p->n_kv_heads, d = p->head_dim;
  const int G = p->group_size, M = p->n_select, NG = p->ctx_len / G;
  if (M < 1 || M > NG) return -1;
  const int joint = p->head_mode == ORC_HEADS_JOINT; /* one selection per sequence */
  for (long i = 0; i < (long)p->batch * (joint ? 1 : Hk) * M; ++i)
    if (idx[i] < 0 || idx[i] >= NG) return -1;
  const double scale = resolve_scale(p);
  const long BH = (long)p->batch * Hq;
  int failed = 0;
  long bh;
#pragma omp parallel for schedule(dynamic) num_threads(p->n_threads > 1 ? p->n_threads : 1)
  for (bh = 0; bh < BH; ++bh) {
    const int b = (int)(bh / Hq), h = (int)(bh % Hq);
    const int k = h / (Hq / Hk);
    const int32_t* sel = idx + (joint ? (size_t)b : (size_t)b * Hk + k) * M;
    size_t* rows = (size_t*)malloc(sizeof(size_t) * (size_t)M * G);
    if (!rows) { failed = 1; continue; }
    const size_t base = ((size_t)b * Hk + k) * row_capacity(p); /* first row of this (b, kv head) */
    for (int m = 0; m < M; ++m)
      for (int t = 0; t < G; ++t) rows[(size_t)m * G + t] = base + (size_t)sel[m] * G + t;
    if (attend_rows(p, q, K, V, b, h, rows, (long)M * G, rb_K, rb_V, rb_len, rb_capacity, scale,
                    out + (size_t)bh * d))
      failed = 1;
    free(rows);
  }
  return failed ? -2 : 0;
}

int oracle_dense_attn(const orc_params* p, const void* q, const void* K, const void* V,
                      double* out) {
  if (!params_ok(p) || !q || !K || !V || !out) return -1;
  const int Hq = p->n_q_heads, d = p->head_dim, N = p->ctx_len;
  const double scale = resolve_scale(p);
  const long BH = (long)p->batch * Hq;
  int failed = 0;
  long bh;
#pragma omp parallel for schedule(dynamic) num_threads(p->n_threads > 1 ? p->n_threads : 1)
  for (bh = 0; bh < BH; ++bh) {
    const int b = (int)(bh / Hq), h = (int)(bh % Hq);
    size_t* rows = (size_t*)malloc(sizeof(size_t) * (size_t)N);
    if (!rows) { failed = 1; continue; }
    const size_t base = ((size_t)b * p->n_kv_heads + h / (Hq / p->n_kv_heads)) * row_capacity(p);
    for (int n = 0; n < N; ++n) rows[n] = base + (size_t)n;
    if (attend_rows(p, q, K, V, b, h, rows, N, NULL, NULL, 0, 0, scale, out + (size_t)bh * d))
      failed = 1;
    free(rows);
  }
  return failed ? -2 : 0;
}

/* ---- mapping table (Sec. 3.4.4) and selection overlap (Sec. 3.4.2) --------- */

int oracle_sparse_attn_paged(const orc_params* p, const void* q, const void* K_pool,
                             const void* V_pool, const int32_t* slot_table, int32_t n_slots,
                             const int32_t* idx, const void* rb_K, const void* rb_V,
                             int32_t rb_len, int32_t rb_capacity, double* out) {
  if (!params_ok(p) || !q || !K_pool || !V_pool || !slot_table || !idx || !out) return -1;
  if (rb_len < 0 || rb_len > rb_capacity || (rb_len > 0 && (!rb_K || !rb_V))) return -1;
  const int Hq = p->n_q_heads, Hk = p->n_kv_heads, d = p->head_dim;
  const int G = p->group_size, M = p->n_select, NG = p->ctx_len / G;
  if (M < 1 || M > NG || n_slots < 1) return -1;
  const int joint = p->head_mode == ORC_HEADS_JOINT;
  for (long i = 0; i < (long)p->batch * (joint ? 1 : Hk) * M; ++i)
    if (idx[i] < 0 || idx[i] >= NG) return -1;
  const double scale = resolve_scale(p);
  const long BH = (long)p->batch * Hq;
  int failed = 0, bad_slot = 0;
  long bh;
#pragma omp parallel for schedule(dynamic) num_threads(p->n_threads > 1 ? p->n_threads : 1)
  for (bh = 0; bh < BH; ++bh) {
    const int b = (int)(bh / Hq), h = (int)(bh % Hq);
    const int k = h / (Hq / Hk);
    const int32_t* sel = idx + (joint ? (size_t)b : (size_t)b * Hk + k) * M;
    const int32_t* table = slot_table + ((size_t)b * Hk + k) * NG;
    size_t* rows = (size_t*)malloc(sizeof(size_t) * (size_t)M * G);
    if (!rows) { failed = 1; continue; }
    int ok = 1;
    for (int m = 0; m < M; ++m) {
      const int32_t slot = table[sel[m]]; /* where logical group sel[m] physically is */
      if (slot < 0 || slot >= n_slots) { ok = 0; break; }
      for (int t = 0; t < G; ++t) rows[(size_t)m * G + t] = (size_t)slot * G + t;
    }
    if (!ok) bad_slot = 1;
    else if (attend_rows(p, q, K_pool, V_pool, b, h, rows, (long)M * G, rb_K, rb_V, rb_len,
                         rb_capacity, scale, out + (size_t)bh * d))
      failed = 1;
    free(rows);
  }
  if (bad_slot) return -1;
  return failed ? -2 : 0;
}

int oracle_selection_overlap(const orc_params* p, const int32_t* idx_prev,
                             const int32_t* idx_cur, int32_t* common) {
  if (!params_ok(p) || !idx_prev || !idx_cur || !common) return -1;
  const int M = p->n_select, NG = p->ctx_len / p->group_size;
  if (M < 1 || M > NG) return -1;
  const long sets = (long)p->batch * (p->head_mode == ORC_HEADS_JOINT ? 1 : p->n_kv_heads);
  for (long s = 0; s < sets; ++s) {
    int32_t n = 0;
    for (int i = 0; i < M; ++i)     /* every pair: the definition, no ordering assumed */
      for (int j = 0; j < M; ++j)
        if (idx_cur[s * M + i] == idx_prev[s * M + j]) ++n;
    common[s] = n;
  }
  return 0;
}
