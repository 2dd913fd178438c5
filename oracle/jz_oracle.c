/*
 * jz_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, fp64 CPU reference for the mixed-precision training hot path of
 * "Highly Scalable Deep Learning Training System with Mixed-Precision"
 * (Jia et al., 2018): the fp16-storage convolution forward and its two
 * adjoints, and the fully connected GEMM, as used by the half-precision
 * forward/backward pass of Section 4.1 ("the operations in forward and
 * backward propagation are performed in FP16").  The paper prints no formula
 * for the convolution itself; what is written out here is the textbook CNN
 * cross-correlation (no kernel flip, zero padding, floor output size,
 * dilation 1, groups 1) and the two linear maps adjoint to it.
 *
 * Every input is an array of IEEE binary16 bit patterns.  They are widened to
 * double (exact), every product of two of them is exact in double, and only
 * the long sums round (relative error ~1e-13): this is the plain definition,
 * evaluated as exactly as a CPU conveniently can.
 *
 * The entry points ending in _f32 are the same definitions for binary32
 * inputs (the single-precision training the paper compares with in Section
 * 5.4, Table 9): the inputs are widened to double (exact) and the very same
 * loops run; products of two floats are exact in double as well (24 + 24
 * significand bits).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP path.
 *
 * Layouts: activations NHWC, filters KRSC, outputs NPQK, all innermost index
 * contiguous.  P = floor((H + 2*pad_h - R)/stride_h) + 1, likewise Q.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w;
} orc_conv;

static int out_dim(int in, int pad, int f, int st) { return (in + 2 * pad - f) / st + 1; }

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- IEEE binary16 <-> double, written from the format definition --------
 * 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits; exponent field 0 is
 * zero/subnormal (value = frac * 2^-24), 31 is Inf/NaN.  The smallest positive
 * value is 2^-24 (the underflow threshold Section 5.2 quotes). */
double orc_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1, e = (h >> 10) & 31, f = h & 1023;
  double v;
  if (e == 0)
    v = ldexp((double)f, -24);
  else if (e == 31)
    v = f ? NAN : INFINITY;
  else
    v = ldexp((double)(1024 + f), e - 25);
  return sign ? -v : v;
}

/* Round a double to binary16, round-to-nearest-even, one rounding only.
 * rint() rounds to nearest even in the default floating point environment and
 * scaling by a power of two is exact, so the integer q below is the correctly
 * rounded significand. */
uint16_t orc_double_to_half(double d) {
  uint16_t sign = signbit(d) ? 0x8000u : 0u;
  if (isnan(d)) return (uint16_t)(sign | 0x7e00u);
  double a = fabs(d);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u); /* 65520 = midpoint of 65504 and 2^16; tie goes to even = overflow */
  if (a < ldexp(1.0, -14)) {                           /* subnormal range, spacing 2^-24 */
    long q = (long)rint(ldexp(a, 24));                 /* 0..1024; 1024 is the smallest normal's bit pattern */
    return (uint16_t)(sign | (uint16_t)q);
  }
  int e2;
  (void)frexp(a, &e2); /* a = m*2^e2, m in [0.5,1)  =>  2^(e2-1) <= a < 2^e2 */
  int E = e2 - 1;
  long q = (long)rint(ldexp(a, 10 - E)); /* in [1024, 2048] */
  if (q == 2048) {
    q = 1024;
    E += 1;
  }
  return (uint16_t)(sign | (uint16_t)((E + 15) << 10) | (uint16_t)(q - 1024));
}

void orc_halves_to_doubles(const uint16_t* in, double* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = orc_half_to_double(in[i]);
}
void orc_doubles_to_halves(const double* in, uint16_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = orc_double_to_half(in[i]);
}

static double* widen(const uint16_t* in, int64_t n) {
  double* out = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  if (out) orc_halves_to_doubles(in, out, n);
  return out;
}
static double* widen_f32(const float* in, int64_t n) {
  double* out = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  if (out)
    for (int64_t i = 0; i < n; ++i) out[i] = (double)in[i];
  return out;
}

/* ---- convolution forward --------------------------------------------------
 * Y[n,p,q,k] = sum_{r,s,c} X[n, p*st_h - pad_h + r, q*st_w - pad_w + s, c] * W[k,r,s,c],
 * taps that fall outside the image contribute 0. */
static void orc_conv_fwd_on_doubles(const orc_conv* d, const double* x, const double* w, double* y) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q)
        for (int k = 0; k < K; ++k) {
          double acc = 0.0;
          for (int r = 0; r < R; ++r) {
            int h = p * d->stride_h - d->pad_h + r;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < S; ++s) {
              int ww = q * d->stride_w - d->pad_w + s;
              if (ww < 0 || ww >= W) continue;
              const double* xp = x + (((int64_t)n * H + h) * W + ww) * C;
              const double* wp = w + (((int64_t)k * R + r) * S + s) * C;
              for (int c = 0; c < C; ++c) acc += xp[c] * wp[c];
            }
          }
          y[(((int64_t)n * P + p) * Q + q) * K + k] = acc;
        }
}
int orc_conv_fwd(const orc_conv* d, const uint16_t* x16, const uint16_t* w16, double* y) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
  (void)P; (void)Q;
  double* x = widen(x16, (int64_t)N * H * W * C);
  double* w = widen(w16, (int64_t)K * R * S * C);
  if (!x || !w) { free(x); free(w); return -1; }
  orc_conv_fwd_on_doubles(d, x, w, y);
  free(x);
  free(w);
  return 0;
}

int orc_conv_fwd_f32(const orc_conv* d, const float* x32, const float* w32, double* y) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
  (void)P; (void)Q;
  double* x = widen_f32(x32, (int64_t)N * H * W * C);
  double* w = widen_f32(w32, (int64_t)K * R * S * C);
  if (!x || !w) { free(x); free(w); return -1; }
  orc_conv_fwd_on_doubles(d, x, w, y);
  free(x);
  free(w);
  return 0;
}


/* ---- backward data: the adjoint of the forward map in X ---------------------
 * Written as a scatter over exactly the index set the forward pass reads:
 * every forward term X[n,h,w,c]*W[k,r,s,c] -> Y[n,p,q,k] becomes
 * dX[n,h,w,c] += dY[n,p,q,k]*W[k,r,s,c].  No separate index algebra. */
static void orc_conv_bwd_data_on_doubles(const orc_conv* d, const double* dy, const double* w, double* dx) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
  memset(dx, 0, sizeof(double) * (size_t)N * H * W * C);
#pragma omp parallel for schedule(dynamic, 1)
  for (int n = 0; n < N; ++n) /* images are independent, so no two threads touch the same dX */
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q)
        for (int k = 0; k < K; ++k) {
          double g = dy[(((int64_t)n * P + p) * Q + q) * K + k];
          for (int r = 0; r < R; ++r) {
            int h = p * d->stride_h - d->pad_h + r;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < S; ++s) {
              int ww = q * d->stride_w - d->pad_w + s;
              if (ww < 0 || ww >= W) continue;
              double* dxp = dx + (((int64_t)n * H + h) * W + ww) * C;
              const double* wp = w + (((int64_t)k * R + r) * S + s) * C;
              for (int c = 0; c < C; ++c) dxp[c] += g * wp[c];
            }
          }
        }
}
int orc_conv_bwd_data(const orc_conv* d, const uint16_t* dy16, const uint16_t* w16, double* dx) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
  double* dy = widen(dy16, (int64_t)N * P * Q * K);
  double* w = widen(w16, (int64_t)K * R * S * C);
  if (!dy || !w) { free(dy); free(w); return -1; }
  orc_conv_bwd_data_on_doubles(d, dy, w, dx);
  free(dy);
  free(w);
  return 0;
}

int orc_conv_bwd_data_f32(const orc_conv* d, const float* dy32, const float* w32, double* dx) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
  double* dy = widen_f32(dy32, (int64_t)N * P * Q * K);
  double* w = widen_f32(w32, (int64_t)K * R * S * C);
  if (!dy || !w) { free(dy); free(w); return -1; }
  orc_conv_bwd_data_on_doubles(d, dy, w, dx);
  free(dy);
  free(w);
  return 0;
}


/* ---- backward weight: the adjoint of the forward map in W -------------------
 * dW[k,r,s,c] = sum_{n,p,q} dY[n,p,q,k] * X[n, p*st_h - pad_h + r, q*st_w - pad_w + s, c],
 * out-of-image X = 0.  No division by the batch size: any loss averaging lives
 * upstream in dY. */
static void orc_conv_bwd_weight_on_doubles(const orc_conv* d, const double* x, const double* dy, double* dw) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
#pragma omp parallel for collapse(3) schedule(static)
  for (int k = 0; k < K; ++k)
    for (int r = 0; r < R; ++r)
      for (int s = 0; s < S; ++s) {
        double* out = dw + (((int64_t)k * R + r) * S + s) * C;
        for (int c = 0; c < C; ++c) out[c] = 0.0;
        for (int n = 0; n < N; ++n)
          for (int p = 0; p < P; ++p) {
            int h = p * d->stride_h - d->pad_h + r;
            if (h < 0 || h >= H) continue;
            for (int q = 0; q < Q; ++q) {
              int ww = q * d->stride_w - d->pad_w + s;
              if (ww < 0 || ww >= W) continue;
              double g = dy[(((int64_t)n * P + p) * Q + q) * K + k];
              const double* xp = x + (((int64_t)n * H + h) * W + ww) * C;
              for (int c = 0; c < C; ++c) out[c] += g * xp[c];
            }
          }
      }
}
int orc_conv_bwd_weight(const orc_conv* d, const uint16_t* x16, const uint16_t* dy16, double* dw) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
  double* x = widen(x16, (int64_t)N * H * W * C);
  double* dy = widen(dy16, (int64_t)N * P * Q * K);
  if (!x || !dy) { free(x); free(dy); return -1; }
  orc_conv_bwd_weight_on_doubles(d, x, dy, dw);
  free(x);
  free(dy);
  return 0;
}

int orc_conv_bwd_weight_f32(const orc_conv* d, const float* x32, const float* dy32, double* dw) {
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S;
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w);
  double* x = widen_f32(x32, (int64_t)N * H * W * C);
  double* dy = widen_f32(dy32, (int64_t)N * P * Q * K);
  if (!x || !dy) { free(x); free(dy); return -1; }
  orc_conv_bwd_weight_on_doubles(d, x, dy, dw);
  free(x);
  free(dy);
  return 0;
}


static double float_to_double(float f) { return (double)f; }

/* ---- single output elements, for spot checks at sizes where the full tensor
 * would take minutes.  idx[] holds flat indices into the respective output.
 * Each routine is written once, as a macro, and instantiated for binary16 bit
 * patterns and for binary32 inputs (NAME, element type, widening function). */
#define DEFINE_ORC_CONV_FWD_AT(NAME, T, CVT) \
int NAME(const orc_conv* d, const T* x, const T* w, const int64_t* idx, int64_t n_idx, \
                    double* out) { \
  const int H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S; \
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w); \
_Pragma("omp parallel for schedule(static)") \
  for (int64_t i = 0; i < n_idx; ++i) { \
    int64_t t = idx[i]; \
    int k = (int)(t % K); t /= K; \
    int q = (int)(t % Q); t /= Q; \
    int p = (int)(t % P); t /= P; \
    int n = (int)t; \
    double acc = 0.0; \
    for (int r = 0; r < R; ++r) { \
      int h = p * d->stride_h - d->pad_h + r; \
      if (h < 0 || h >= H) continue; \
      for (int s = 0; s < S; ++s) { \
        int ww = q * d->stride_w - d->pad_w + s; \
        if (ww < 0 || ww >= W) continue; \
        const T* xp = x + (((int64_t)n * H + h) * W + ww) * C; \
        const T* wp = w + (((int64_t)k * R + r) * S + s) * C; \
        for (int c = 0; c < C; ++c) acc += CVT(xp[c]) * CVT(wp[c]); \
      } \
    } \
    out[i] = acc; \
  } \
  return 0; \
}
DEFINE_ORC_CONV_FWD_AT(orc_conv_fwd_at, uint16_t, orc_half_to_double)
DEFINE_ORC_CONV_FWD_AT(orc_conv_fwd_at_f32, float, float_to_double)


/* dX element by brute force over every forward term: a term (p,q,k,r,s) feeds
 * dX[n,h,w,c] exactly when its input coordinate equals (h,w). */
#define DEFINE_ORC_CONV_BWD_DATA_AT(NAME, T, CVT) \
int NAME(const orc_conv* d, const T* dy, const T* w, const int64_t* idx, int64_t n_idx, \
                         double* out) { \
  const int H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S; \
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w); \
_Pragma("omp parallel for schedule(static)") \
  for (int64_t i = 0; i < n_idx; ++i) { \
    int64_t t = idx[i]; \
    int c = (int)(t % C); t /= C; \
    int ww = (int)(t % W); t /= W; \
    int h = (int)(t % H); t /= H; \
    int n = (int)t; \
    double acc = 0.0; \
    for (int p = 0; p < P; ++p) \
      for (int r = 0; r < R; ++r) { \
        if (p * d->stride_h - d->pad_h + r != h) continue; \
        for (int q = 0; q < Q; ++q) \
          for (int s = 0; s < S; ++s) { \
            if (q * d->stride_w - d->pad_w + s != ww) continue; \
            const T* gp = dy + (((int64_t)n * P + p) * Q + q) * K; \
            for (int k = 0; k < K; ++k) \
              acc += CVT(gp[k]) * CVT(w[(((int64_t)k * R + r) * S + s) * C + c]); \
          } \
      } \
    out[i] = acc; \
  } \
  return 0; \
}
DEFINE_ORC_CONV_BWD_DATA_AT(orc_conv_bwd_data_at, uint16_t, orc_half_to_double)
DEFINE_ORC_CONV_BWD_DATA_AT(orc_conv_bwd_data_at_f32, float, float_to_double)


#define DEFINE_ORC_CONV_BWD_WEIGHT_AT(NAME, T, CVT) \
int NAME(const orc_conv* d, const T* x, const T* dy, const int64_t* idx, \
                           int64_t n_idx, double* out) { \
  const int N = d->N, H = d->H, W = d->W, C = d->C, K = d->K, R = d->R, S = d->S; \
  const int P = out_dim(H, d->pad_h, R, d->stride_h), Q = out_dim(W, d->pad_w, S, d->stride_w); \
_Pragma("omp parallel for schedule(dynamic, 16)") \
  for (int64_t i = 0; i < n_idx; ++i) { \
    int64_t t = idx[i]; \
    int c = (int)(t % C); t /= C; \
    int s = (int)(t % S); t /= S; \
    int r = (int)(t % R); t /= R; \
    int k = (int)t; \
    double acc = 0.0; \
    for (int n = 0; n < N; ++n) \
      for (int p = 0; p < P; ++p) { \
        int h = p * d->stride_h - d->pad_h + r; \
        if (h < 0 || h >= H) continue; \
        for (int q = 0; q < Q; ++q) { \
          int ww = q * d->stride_w - d->pad_w + s; \
          if (ww < 0 || ww >= W) continue; \
          acc += CVT(dy[(((int64_t)n * P + p) * Q + q) * K + k]) * \
                 CVT(x[(((int64_t)n * H + h) * W + ww) * C + c]); \
        } \
      } \
    out[i] = acc; \
  } \
  return 0; \
}
DEFINE_ORC_CONV_BWD_WEIGHT_AT(orc_conv_bwd_weight_at, uint16_t, orc_half_to_double)
DEFINE_ORC_CONV_BWD_WEIGHT_AT(orc_conv_bwd_weight_at_f32, float, float_to_double)


/* ---- fully connected layer -------------------------------------------------
 * x[B,I], w[O,I], y[B,O], all row-major:
 *   forward       y  = x  * w^T
 *   backward data dx = dy * w
 *   backward wgt  dw = dy^T * x            (triple loops, nothing else) */
static void orc_fc_fwd_on_doubles(int B, int I, int O, const double* x, const double* w, double* y) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < B; ++b)
    for (int o = 0; o < O; ++o) {
      double acc = 0.0;
      for (int i = 0; i < I; ++i) acc += x[(int64_t)b * I + i] * w[(int64_t)o * I + i];
      y[(int64_t)b * O + o] = acc;
    }
}
int orc_fc_fwd(int B, int I, int O, const uint16_t* x16, const uint16_t* w16, double* y) {
  double* x = widen(x16, (int64_t)B * I);
  double* w = widen(w16, (int64_t)O * I);
  if (!x || !w) { free(x); free(w); return -1; }
  orc_fc_fwd_on_doubles(B, I, O, x, w, y);
  free(x);
  free(w);
  return 0;
}

int orc_fc_fwd_f32(int B, int I, int O, const float* x32, const float* w32, double* y) {
  double* x = widen_f32(x32, (int64_t)B * I);
  double* w = widen_f32(w32, (int64_t)O * I);
  if (!x || !w) { free(x); free(w); return -1; }
  orc_fc_fwd_on_doubles(B, I, O, x, w, y);
  free(x);
  free(w);
  return 0;
}


static void orc_fc_bwd_data_on_doubles(int B, int I, int O, const double* dy, const double* w, double* dx) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < I; ++i) {
      double acc = 0.0;
      for (int o = 0; o < O; ++o) acc += dy[(int64_t)b * O + o] * w[(int64_t)o * I + i];
      dx[(int64_t)b * I + i] = acc;
    }
}
int orc_fc_bwd_data(int B, int I, int O, const uint16_t* dy16, const uint16_t* w16, double* dx) {
  double* dy = widen(dy16, (int64_t)B * O);
  double* w = widen(w16, (int64_t)O * I);
  if (!dy || !w) { free(dy); free(w); return -1; }
  orc_fc_bwd_data_on_doubles(B, I, O, dy, w, dx);
  free(dy);
  free(w);
  return 0;
}

int orc_fc_bwd_data_f32(int B, int I, int O, const float* dy32, const float* w32, double* dx) {
  double* dy = widen_f32(dy32, (int64_t)B * O);
  double* w = widen_f32(w32, (int64_t)O * I);
  if (!dy || !w) { free(dy); free(w); return -1; }
  orc_fc_bwd_data_on_doubles(B, I, O, dy, w, dx);
  free(dy);
  free(w);
  return 0;
}


static void orc_fc_bwd_weight_on_doubles(int B, int I, int O, const double* dy, const double* x, double* dw) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int o = 0; o < O; ++o)
    for (int i = 0; i < I; ++i) {
      double acc = 0.0;
      for (int b = 0; b < B; ++b) acc += dy[(int64_t)b * O + o] * x[(int64_t)b * I + i];
      dw[(int64_t)o * I + i] = acc;
    }
}
int orc_fc_bwd_weight(int B, int I, int O, const uint16_t* dy16, const uint16_t* x16, double* dw) {
  double* dy = widen(dy16, (int64_t)B * O);
  double* x = widen(x16, (int64_t)B * I);
  if (!dy || !x) { free(dy); free(x); return -1; }
  orc_fc_bwd_weight_on_doubles(B, I, O, dy, x, dw);
  free(dy);
  free(x);
  return 0;
}

int orc_fc_bwd_weight_f32(int B, int I, int O, const float* dy32, const float* x32, double* dw) {
  double* dy = widen_f32(dy32, (int64_t)B * O);
  double* x = widen_f32(x32, (int64_t)B * I);
  if (!dy || !x) { free(dy); free(x); return -1; }
  orc_fc_bwd_weight_on_doubles(B, I, O, dy, x, dw);
  free(dy);
  free(x);
  return 0;
}

