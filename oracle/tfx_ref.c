/*
 * tfx_ref.c -- CPU oracle for the dense ops of the TensorFlow.js paper
 * (arxiv 1901.05350).  TEST INFRASTRUCTURE ONLY: this file is the yardstick the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and is never called from the product path.
 *
 * Every function is the plain definition of the op written out as nested loops:
 * fp32 inputs, one double-precision accumulator per output element, a single
 * rounding to float at the end.  No blocking, no fusion, no reordering; the only
 * parallelism is an OpenMP "parallel for" over the outermost independent loop.
 *
 * Where the paper fixes the semantics:
 *   - matMul: Section 4.1, Listing 2 -- one output value per (aRow, bCol),
 *     result = sum_i A[aRow,i] * B[i,bCol].  The listing assumes the shared
 *     dimension is a multiple of 4 "for simplicity"; no such limit here.
 *   - conv2d input index order (batch, row, column, depth) = NHWC: Section 4.1,
 *     the 4-D sampler used by the conv2d shader.
 *   - Ops are functional and never mutate their inputs: Section 3.7.
 * Where the paper is silent, the API is "largely modeled after TensorFlow"
 * (Section 3.1), so the TensorFlow conventions are used: cross-correlation (no
 * filter flip), HWIO filters, [fh,fw,inC,mult] depthwise filters with output
 * channel c*mult+q, and the SAME / VALID output-size rules.
 *
 * The 16-bit float storage variants and the element-wise addition at the end of the file
 * follow Section 4.1 (16-bit float textures; Fig. 3).
 *
 * Parity pins for every function below live in tests/test_oracle_*.py
 * (closed forms, one-hot filters, tap counts, brute force, torch/numpy float64).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

enum { REF_OK = 0, REF_ERR_NULL = -1, REF_ERR_SHAPE = -2, REF_ERR_ARG = -3 };
enum { REF_PAD_VALID = 0, REF_PAD_SAME = 1 };
enum { REF_ACT_NONE = 0, REF_ACT_RELU = 1, REF_ACT_RELU6 = 2 };

/* ---- output extent and padding of one spatial dimension -------------------
 * VALID: out = floor((in - k) / s) + 1, no padding; in < k is an error.
 * SAME : out = ceil(in / s); pad_total = max((out-1)*s + k - in, 0);
 *        pad_before = floor(pad_total / 2); the odd unit goes after
 *        (bottom / right).  TensorFlow convention (Section 3.1).            */
int tfx_ref_out_extent(int64_t in, int64_t k, int64_t s, int pad,
                       int64_t* out, int64_t* pad_before, int64_t* pad_after) {
  if (!out || !pad_before || !pad_after) return REF_ERR_NULL;
  if (in < 1 || k < 1) return REF_ERR_SHAPE;
  if (s < 1) return REF_ERR_ARG;
  if (pad == REF_PAD_VALID) {
    if (in < k) return REF_ERR_SHAPE;
    *out = (in - k) / s + 1;
    *pad_before = 0;
    *pad_after = 0;
    return REF_OK;
  }
  if (pad == REF_PAD_SAME) {
    int64_t o = (in + s - 1) / s;
    int64_t total = (o - 1) * s + k - in;
    if (total < 0) total = 0;
    *out = o;
    *pad_before = total / 2;
    *pad_after = total - total / 2;
    return REF_OK;
  }
  return REF_ERR_ARG;
}

int tfx_ref_matmul_out_shape(const int64_t a_shape[2], const int64_t b_shape[2],
                             int transpose_a, int transpose_b, int64_t out_shape[2]) {
  if (!a_shape || !b_shape || !out_shape) return REF_ERR_NULL;
  if (a_shape[0] < 1 || a_shape[1] < 1 || b_shape[0] < 1 || b_shape[1] < 1) return REF_ERR_SHAPE;
  int64_t m = transpose_a ? a_shape[1] : a_shape[0];
  int64_t ka = transpose_a ? a_shape[0] : a_shape[1];
  int64_t kb = transpose_b ? b_shape[1] : b_shape[0];
  int64_t n = transpose_b ? b_shape[0] : b_shape[1];
  if (ka != kb) return REF_ERR_SHAPE;
  out_shape[0] = m;
  out_shape[1] = n;
  return REF_OK;
}

/* x: [N,H,W,Ci]; f: [fh,fw,Ci,Co]; out: [N,oh,ow,Co]; pad_tblr: top,bottom,left,right */
int tfx_ref_conv2d_out_shape(const int64_t x_shape[4], const int64_t f_shape[4],
                             int stride_h, int stride_w, int pad,
                             int64_t out_shape[4], int64_t pad_tblr[4]) {
  if (!x_shape || !f_shape || !out_shape || !pad_tblr) return REF_ERR_NULL;
  for (int i = 0; i < 4; ++i)
    if (x_shape[i] < 1 || f_shape[i] < 1) return REF_ERR_SHAPE;
  if (x_shape[3] != f_shape[2]) return REF_ERR_SHAPE;
  int rc = tfx_ref_out_extent(x_shape[1], f_shape[0], stride_h, pad, &out_shape[1], &pad_tblr[0], &pad_tblr[1]);
  if (rc) return rc;
  rc = tfx_ref_out_extent(x_shape[2], f_shape[1], stride_w, pad, &out_shape[2], &pad_tblr[2], &pad_tblr[3]);
  if (rc) return rc;
  out_shape[0] = x_shape[0];
  out_shape[3] = f_shape[3];
  return REF_OK;
}

/* x: [N,H,W,C]; f: [fh,fw,C,mult]; out: [N,oh,ow,C*mult] */
int tfx_ref_depthwise_conv2d_out_shape(const int64_t x_shape[4], const int64_t f_shape[4],
                                       int stride_h, int stride_w, int pad,
                                       int64_t out_shape[4], int64_t pad_tblr[4]) {
  int rc = tfx_ref_conv2d_out_shape(x_shape, f_shape, stride_h, stride_w, pad, out_shape, pad_tblr);
  if (rc) return rc;
  out_shape[3] = x_shape[3] * f_shape[3];
  return REF_OK;
}

/* bias first, then activation; relu(v) = max(v,0), relu6(v) = min(max(v,0),6).
 * Both are written with comparisons that are false for a NaN, so a NaN comes out
 * as a NaN under either activation (the convention of the library the paper's API
 * follows, Section 3.1; the debug mode of Section 3.8 exists to find such values,
 * so an activation must not erase them).  -inf gives 0, +inf the upper bound. */
static double ref_activate(double v, int act) {
  if (act == REF_ACT_RELU) return v < 0.0 ? 0.0 : v;
  if (act == REF_ACT_RELU6) return v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v);
  return v;
}

/* ---- matMul (Section 4.1, Listing 2) ---------------------------------------
 * a is stored [ar,ac], b is stored [br,bc], both row-major.
 * C[i,j] = sum_k A'(i,k) * B'(k,j),  A'(i,k) = tA ? a[k,i] : a[i,k],
 *                                    B'(k,j) = tB ? b[j,k] : b[k,j].        */
int tfx_ref_matmul(const float* a, const int64_t a_shape[2], const float* b, const int64_t b_shape[2],
                   int transpose_a, int transpose_b, float* c) {
  if (!a || !b || !c || !a_shape || !b_shape) return REF_ERR_NULL;
  int64_t o[2];
  int rc = tfx_ref_matmul_out_shape(a_shape, b_shape, transpose_a, transpose_b, o);
  if (rc) return rc;
  const int64_t M = o[0], N = o[1];
  const int64_t K = transpose_a ? a_shape[0] : a_shape[1];
  const int64_t ac = a_shape[1], bc = b_shape[1];
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i) {
    for (int64_t j = 0; j < N; ++j) {
      double acc = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        double av = transpose_a ? a[k * ac + i] : a[i * ac + k];
        double bv = transpose_b ? b[j * bc + k] : b[k * bc + j];
        acc += av * bv;
      }
      c[i * N + j] = (float)acc;
    }
  }
  return REF_OK;
}

/* ---- batchMatMul: matMul independently per batch; equal batch dims ---------- */
int tfx_ref_batch_matmul(const float* a, const int64_t a_shape[3], const float* b, const int64_t b_shape[3],
                         int transpose_a, int transpose_b, float* c) {
  if (!a || !b || !c || !a_shape || !b_shape) return REF_ERR_NULL;
  if (a_shape[0] < 1 || a_shape[0] != b_shape[0]) return REF_ERR_SHAPE;
  int64_t o[2];
  int rc = tfx_ref_matmul_out_shape(a_shape + 1, b_shape + 1, transpose_a, transpose_b, o);
  if (rc) return rc;
  const int64_t sa = a_shape[1] * a_shape[2], sb = b_shape[1] * b_shape[2], sc = o[0] * o[1];
  for (int64_t bi = 0; bi < a_shape[0]; ++bi) {
    rc = tfx_ref_matmul(a + bi * sa, a_shape + 1, b + bi * sb, b_shape + 1, transpose_a, transpose_b, c + bi * sc);
    if (rc) return rc;
  }
  return REF_OK;
}

/* ---- conv2d, NHWC x HWIO, cross-correlation ---------------------------------
 * y[n,oh,ow,o] = act( sum_{kh,kw,c} X(n, oh*sh - pt + kh, ow*sw - pl + kw, c) * w[kh,kw,c,o] + bias[o] )
 * with X = 0 outside the image.  bias may be NULL (= 0).                     */
int tfx_ref_conv2d(const float* x, const int64_t x_shape[4], const float* w, const int64_t f_shape[4],
                   const float* bias, int stride_h, int stride_w, int pad, int act, float* y) {
  if (!x || !w || !y || !x_shape || !f_shape) return REF_ERR_NULL;
  if (act != REF_ACT_NONE && act != REF_ACT_RELU && act != REF_ACT_RELU6) return REF_ERR_ARG;
  int64_t o[4], p[4];
  int rc = tfx_ref_conv2d_out_shape(x_shape, f_shape, stride_h, stride_w, pad, o, p);
  if (rc) return rc;
  const int64_t N = x_shape[0], H = x_shape[1], W = x_shape[2], Ci = x_shape[3];
  const int64_t fh = f_shape[0], fw = f_shape[1], Co = f_shape[3];
  const int64_t OH = o[1], OW = o[2], pt = p[0], pl = p[2];
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t oh = 0; oh < OH; ++oh) {
      for (int64_t ow = 0; ow < OW; ++ow) {
        for (int64_t oc = 0; oc < Co; ++oc) {
          double acc = 0.0;
          for (int64_t kh = 0; kh < fh; ++kh) {
            const int64_t ih = oh * stride_h - pt + kh;
            if (ih < 0 || ih >= H) continue;
            for (int64_t kw = 0; kw < fw; ++kw) {
              const int64_t iw = ow * stride_w - pl + kw;
              if (iw < 0 || iw >= W) continue;
              const float* xp = x + ((n * H + ih) * W + iw) * Ci;
              const float* wp = w + ((kh * fw + kw) * Ci) * Co + oc;
              for (int64_t c = 0; c < Ci; ++c) acc += (double)xp[c] * (double)wp[c * Co];
            }
          }
          if (bias) acc += (double)bias[oc];
          y[((n * OH + oh) * OW + ow) * Co + oc] = (float)ref_activate(acc, act);
        }
      }
    }
  }
  return REF_OK;
}

/* ---- depthwiseConv2d, NHWC x [fh,fw,C,mult] ---------------------------------
 * y[n,oh,ow,c*mult+q] = act( sum_{kh,kw} X(n, oh*sh - pt + kh, ow*sw - pl + kw, c) * w[kh,kw,c,q]
 *                            + bias[c*mult+q] )                              */
int tfx_ref_depthwise_conv2d(const float* x, const int64_t x_shape[4], const float* w, const int64_t f_shape[4],
                             const float* bias, int stride_h, int stride_w, int pad, int act, float* y) {
  if (!x || !w || !y || !x_shape || !f_shape) return REF_ERR_NULL;
  if (act != REF_ACT_NONE && act != REF_ACT_RELU && act != REF_ACT_RELU6) return REF_ERR_ARG;
  int64_t o[4], p[4];
  int rc = tfx_ref_depthwise_conv2d_out_shape(x_shape, f_shape, stride_h, stride_w, pad, o, p);
  if (rc) return rc;
  const int64_t N = x_shape[0], H = x_shape[1], W = x_shape[2], C = x_shape[3];
  const int64_t fh = f_shape[0], fw = f_shape[1], mult = f_shape[3];
  const int64_t OH = o[1], OW = o[2], OC = o[3], pt = p[0], pl = p[2];
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t oh = 0; oh < OH; ++oh) {
      for (int64_t ow = 0; ow < OW; ++ow) {
        for (int64_t c = 0; c < C; ++c) {
          for (int64_t q = 0; q < mult; ++q) {
            double acc = 0.0;
            for (int64_t kh = 0; kh < fh; ++kh) {
              const int64_t ih = oh * stride_h - pt + kh;
              if (ih < 0 || ih >= H) continue;
              for (int64_t kw = 0; kw < fw; ++kw) {
                const int64_t iw = ow * stride_w - pl + kw;
                if (iw < 0 || iw >= W) continue;
                acc += (double)x[((n * H + ih) * W + iw) * C + c] *
                       (double)w[((kh * fw + kw) * C + c) * mult + q];
              }
            }
            if (bias) acc += (double)bias[c * mult + q];
            y[((n * OH + oh) * OW + ow) * OC + c * mult + q] = (float)ref_activate(acc, act);
          }
        }
      }
    }
  }
  return REF_OK;
}

/* ---- MobileNet tail pieces ---------------------------------------------------
 * global average pool: p[n,c] = (1/(H*W)) * sum_{h,w} a[n,h,w,c]            */
int tfx_ref_global_avg_pool(const float* a, const int64_t a_shape[4], float* p) {
  if (!a || !a_shape || !p) return REF_ERR_NULL;
  for (int i = 0; i < 4; ++i)
    if (a_shape[i] < 1) return REF_ERR_SHAPE;
  const int64_t N = a_shape[0], HW = a_shape[1] * a_shape[2], C = a_shape[3];
  for (int64_t n = 0; n < N; ++n)
    for (int64_t c = 0; c < C; ++c) {
      double acc = 0.0;
      for (int64_t i = 0; i < HW; ++i) acc += (double)a[(n * HW + i) * C + c];
      p[n * C + c] = (float)(acc / (double)HW);
    }
  return REF_OK;
}

/* row-wise softmax: exp(l - max l) / sum exp(l - max l) */
int tfx_ref_softmax(const float* logits, int64_t rows, int64_t cols, float* probs) {
  if (!logits || !probs) return REF_ERR_NULL;
  if (rows < 1 || cols < 1) return REF_ERR_SHAPE;
  for (int64_t n = 0; n < rows; ++n) {
    const float* l = logits + n * cols;
    double mx = l[0];
    for (int64_t j = 1; j < cols; ++j)
      if ((double)l[j] > mx) mx = l[j];
    double sum = 0.0;
    for (int64_t j = 0; j < cols; ++j) sum += exp((double)l[j] - mx);
    for (int64_t j = 0; j < cols; ++j) probs[n * cols + j] = (float)(exp((double)l[j] - mx) / sum);
  }
  return REF_OK;
}

/* ---- 16-bit float storage (Section 4.1: the same matMul renders to a 32-bit or to a
 * 16-bit floating point texture depending on the device) -----------------------------
 * IEEE 754 binary16: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits.
 *   e = 0      : value = (-1)^s * f * 2^-24               (zero and subnormals)
 *   1<=e<=30   : value = (-1)^s * (1024 + f) * 2^(e-25)
 *   e = 31     : infinity (f = 0) or NaN
 * Both conversions are written from that definition; the pins compare them with numpy's
 * float16 casts over all 65536 patterns and over random doubles.                      */
static double ref_half_to_double(uint16_t h) {
  const int s = (h >> 15) & 1, e = (h >> 10) & 31, f = h & 1023;
  double v;
  if (e == 0) v = ldexp((double)f, -24);
  else if (e == 31) v = f ? NAN : INFINITY;
  else v = ldexp((double)(1024 + f), e - 25);
  return s ? -v : v;
}

/* round to nearest, ties to even; values that round beyond 65504 become infinity */
static uint16_t ref_double_to_half(double v) {
  if (isnan(v)) return 0x7e00;
  const uint16_t sign = signbit(v) ? 0x8000 : 0;
  const double a = fabs(v);
  if (isinf(a)) return (uint16_t)(sign | 0x7c00);
  if (a == 0.0) return sign;
  int ex;
  (void)frexp(a, &ex);              /* a = m * 2^ex with 0.5 <= m < 1, i.e. 2^(ex-1) <= a < 2^ex */
  int e = ex - 1;                   /* unbiased exponent of a                                       */
  if (e < -14) e = -14;             /* subnormal range shares the spacing of the smallest binade    */
  const double q = ldexp(a, -(e - 10)); /* a in units of the grid spacing 2^(e-10) (exact)          */
  double r = floor(q);
  const double frac = q - r;
  if (frac > 0.5 || (frac == 0.5 && fmod(r, 2.0) == 1.0)) r += 1.0;
  /* r is an integer in [0, 2048]; r = 2048 means the value rounded up into the next binade */
  int64_t ri = (int64_t)r;
  if (ri == 2048) {
    ri = 1024;
    e += 1;
  }
  if (ri < 1024) return (uint16_t)(sign | (uint16_t)ri);          /* subnormal (e == -14) or zero   */
  if (e > 15) return (uint16_t)(sign | 0x7c00);                    /* overflow                       */
  return (uint16_t)(sign | ((uint16_t)(e + 15) << 10) | (uint16_t)(ri - 1024));
}

int tfx_ref_half_to_double(const uint16_t* h, int64_t n, double* out) {
  if (!h || !out) return REF_ERR_NULL;
  if (n < 0) return REF_ERR_SHAPE;
  for (int64_t i = 0; i < n; ++i) out[i] = ref_half_to_double(h[i]);
  return REF_OK;
}

int tfx_ref_double_to_half(const double* v, int64_t n, uint16_t* out) {
  if (!v || !out) return REF_ERR_NULL;
  if (n < 0) return REF_ERR_SHAPE;
  for (int64_t i = 0; i < n; ++i) out[i] = ref_double_to_half(v[i]);
  return REF_OK;
}

/* ---- element-wise addition (Section 4.1, Fig. 3): c[i] = a[i] + b[i] ------------------
 * The sum of two floats (or two halfs) is exact in double, so one rounding to the storage
 * type gives the correctly rounded result.                                             */
int tfx_ref_add(const float* a, const float* b, int64_t n, float* c) {
  if (n < 0) return REF_ERR_SHAPE;
  if (n > 0 && (!a || !b || !c)) return REF_ERR_NULL;
  for (int64_t i = 0; i < n; ++i) c[i] = (float)((double)a[i] + (double)b[i]);
  return REF_OK;
}

int tfx_ref_add_f16(const uint16_t* a, const uint16_t* b, int64_t n, uint16_t* c) {
  if (n < 0) return REF_ERR_SHAPE;
  if (n > 0 && (!a || !b || !c)) return REF_ERR_NULL;
  for (int64_t i = 0; i < n; ++i) c[i] = ref_double_to_half(ref_half_to_double(a[i]) + ref_half_to_double(b[i]));
  return REF_OK;
}

/* ---- batchMatMul on 16-bit float storage with fused epilogue -------------------------
 * c[b,i,j] = half( act( sum_k A'(b,i,k) * B'(b,k,j) + bias[j] ) ), operands, bias and result
 * stored as binary16, the sum taken in double (products of two halfs are exact there).
 * Shapes and transposes as tfx_ref_batch_matmul; bias [N] may be NULL.                  */
int tfx_ref_batch_matmul_f16(const uint16_t* a, const int64_t a_shape[3], const uint16_t* b,
                             const int64_t b_shape[3], int transpose_a, int transpose_b, const uint16_t* bias,
                             int act, uint16_t* c) {
  if (!a || !b || !c || !a_shape || !b_shape) return REF_ERR_NULL;
  if (act != REF_ACT_NONE && act != REF_ACT_RELU && act != REF_ACT_RELU6) return REF_ERR_ARG;
  if (a_shape[0] < 1 || a_shape[0] != b_shape[0]) return REF_ERR_SHAPE;
  int64_t o[2];
  int rc = tfx_ref_matmul_out_shape(a_shape + 1, b_shape + 1, transpose_a, transpose_b, o);
  if (rc) return rc;
  const int64_t M = o[0], N = o[1];
  const int64_t K = transpose_a ? a_shape[1] : a_shape[2];
  const int64_t ac = a_shape[2], bc = b_shape[2];
  const int64_t sa = a_shape[1] * a_shape[2], sb = b_shape[1] * b_shape[2], sc = M * N;
  for (int64_t bi = 0; bi < a_shape[0]; ++bi) {
    const uint16_t* ap = a + bi * sa;
    const uint16_t* bp = b + bi * sb;
    uint16_t* cp = c + bi * sc;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
      for (int64_t j = 0; j < N; ++j) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) {
          const double av = ref_half_to_double(transpose_a ? ap[k * ac + i] : ap[i * ac + k]);
          const double bv = ref_half_to_double(transpose_b ? bp[j * bc + k] : bp[k * bc + j]);
          acc += av * bv;
        }
        if (bias) acc += ref_half_to_double(bias[j]);
        cp[i * N + j] = ref_double_to_half(ref_activate(acc, act));
      }
    }
  }
  return REF_OK;
}

/* ---- conv2d, depthwiseConv2d and the MobileNet tail on 16-bit float storage ----------
 * Same definitions as the fp32 functions above; inputs, filters and bias are binary16, every
 * output element is the double-precision sum rounded once to binary16.  The operands are
 * decoded once into float arrays (every binary16 value is exactly a float) so that the loops
 * below read like the fp32 ones.                                                        */
#include <stdlib.h>

static float* ref_decode_halfs(const uint16_t* h, int64_t n) {
  float* f = (float*)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
  if (!f) return NULL;
  for (int64_t i = 0; i < n; ++i) f[i] = (float)ref_half_to_double(h[i]);
  return f;
}

int tfx_ref_conv2d_f16(const uint16_t* x16, const int64_t x_shape[4], const uint16_t* w16, const int64_t f_shape[4],
                       const uint16_t* bias16, int stride_h, int stride_w, int pad, int act, uint16_t* y) {
  if (!x16 || !w16 || !y || !x_shape || !f_shape) return REF_ERR_NULL;
  if (act != REF_ACT_NONE && act != REF_ACT_RELU && act != REF_ACT_RELU6) return REF_ERR_ARG;
  int64_t o[4], p[4];
  int rc = tfx_ref_conv2d_out_shape(x_shape, f_shape, stride_h, stride_w, pad, o, p);
  if (rc) return rc;
  const int64_t N = x_shape[0], H = x_shape[1], W = x_shape[2], Ci = x_shape[3];
  const int64_t fh = f_shape[0], fw = f_shape[1], Co = f_shape[3];
  const int64_t OH = o[1], OW = o[2], pt = p[0], pl = p[2];
  float* x = ref_decode_halfs(x16, N * H * W * Ci);
  float* w = ref_decode_halfs(w16, fh * fw * Ci * Co);
  float* bias = bias16 ? ref_decode_halfs(bias16, Co) : NULL;
  if (!x || !w || (bias16 && !bias)) {
    free(x); free(w); free(bias);
    return REF_ERR_NULL;
  }
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t oh = 0; oh < OH; ++oh) {
      for (int64_t ow = 0; ow < OW; ++ow) {
        for (int64_t oc = 0; oc < Co; ++oc) {
          double acc = 0.0;
          for (int64_t kh = 0; kh < fh; ++kh) {
            const int64_t ih = oh * stride_h - pt + kh;
            if (ih < 0 || ih >= H) continue;
            for (int64_t kw = 0; kw < fw; ++kw) {
              const int64_t iw = ow * stride_w - pl + kw;
              if (iw < 0 || iw >= W) continue;
              const float* xp = x + ((n * H + ih) * W + iw) * Ci;
              const float* wp = w + ((kh * fw + kw) * Ci) * Co + oc;
              for (int64_t c = 0; c < Ci; ++c) acc += (double)xp[c] * (double)wp[c * Co];
            }
          }
          if (bias) acc += (double)bias[oc];
          y[((n * OH + oh) * OW + ow) * Co + oc] = ref_double_to_half(ref_activate(acc, act));
        }
      }
    }
  }
  free(x); free(w); free(bias);
  return REF_OK;
}

int tfx_ref_depthwise_conv2d_f16(const uint16_t* x16, const int64_t x_shape[4], const uint16_t* w16,
                                 const int64_t f_shape[4], const uint16_t* bias16, int stride_h, int stride_w,
                                 int pad, int act, uint16_t* y) {
  if (!x16 || !w16 || !y || !x_shape || !f_shape) return REF_ERR_NULL;
  if (act != REF_ACT_NONE && act != REF_ACT_RELU && act != REF_ACT_RELU6) return REF_ERR_ARG;
  int64_t o[4], p[4];
  int rc = tfx_ref_depthwise_conv2d_out_shape(x_shape, f_shape, stride_h, stride_w, pad, o, p);
  if (rc) return rc;
  const int64_t N = x_shape[0], H = x_shape[1], W = x_shape[2], C = x_shape[3];
  const int64_t fh = f_shape[0], fw = f_shape[1], mult = f_shape[3];
  const int64_t OH = o[1], OW = o[2], OC = o[3], pt = p[0], pl = p[2];
  float* x = ref_decode_halfs(x16, N * H * W * C);
  float* w = ref_decode_halfs(w16, fh * fw * C * mult);
  float* bias = bias16 ? ref_decode_halfs(bias16, OC) : NULL;
  if (!x || !w || (bias16 && !bias)) {
    free(x); free(w); free(bias);
    return REF_ERR_NULL;
  }
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t oh = 0; oh < OH; ++oh) {
      for (int64_t ow = 0; ow < OW; ++ow) {
        for (int64_t c = 0; c < C; ++c) {
          for (int64_t q = 0; q < mult; ++q) {
            double acc = 0.0;
            for (int64_t kh = 0; kh < fh; ++kh) {
              const int64_t ih = oh * stride_h - pt + kh;
              if (ih < 0 || ih >= H) continue;
              for (int64_t kw = 0; kw < fw; ++kw) {
                const int64_t iw = ow * stride_w - pl + kw;
                if (iw < 0 || iw >= W) continue;
                acc += (double)x[((n * H + ih) * W + iw) * C + c] * (double)w[((kh * fw + kw) * C + c) * mult + q];
              }
            }
            if (bias) acc += (double)bias[c * mult + q];
            y[((n * OH + oh) * OW + ow) * OC + c * mult + q] = ref_double_to_half(ref_activate(acc, act));
          }
        }
      }
    }
  }
  free(x); free(w); free(bias);
  return REF_OK;
}

/* mean over the H*W positions of each channel, rounded once to binary16 */
int tfx_ref_global_avg_pool_f16(const uint16_t* x, const int64_t x_shape[4], uint16_t* y) {
  if (!x || !x_shape || !y) return REF_ERR_NULL;
  for (int i = 0; i < 4; ++i)
    if (x_shape[i] < 1) return REF_ERR_SHAPE;
  const int64_t N = x_shape[0], HW = x_shape[1] * x_shape[2], C = x_shape[3];
  for (int64_t n = 0; n < N; ++n)
    for (int64_t c = 0; c < C; ++c) {
      double acc = 0.0;
      for (int64_t p = 0; p < HW; ++p) acc += ref_half_to_double(x[(n * HW + p) * C + c]);
      y[n * C + c] = ref_double_to_half(acc / (double)HW);
    }
  return REF_OK;
}

/* row-wise softmax of binary16 logits, each probability rounded once to binary16 */
int tfx_ref_softmax_f16(const uint16_t* logits, int64_t rows, int64_t cols, uint16_t* probs) {
  if (!logits || !probs) return REF_ERR_NULL;
  if (rows < 1 || cols < 1) return REF_ERR_SHAPE;
  for (int64_t n = 0; n < rows; ++n) {
    const uint16_t* l = logits + n * cols;
    double mx = ref_half_to_double(l[0]);
    for (int64_t j = 1; j < cols; ++j) {
      const double v = ref_half_to_double(l[j]);
      if (v > mx) mx = v;
    }
    double sum = 0.0;
    for (int64_t j = 0; j < cols; ++j) sum += exp(ref_half_to_double(l[j]) - mx);
    for (int64_t j = 0; j < cols; ++j) probs[n * cols + j] = ref_double_to_half(exp(ref_half_to_double(l[j]) - mx) / sum);
  }
  return REF_OK;
}
