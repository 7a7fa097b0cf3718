/*
 * CPU oracle for the unit-scaled linear / FFN hot path  --  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct C.  Every floating-point result is formed in double and rounded
 * once to its storage format; every sum runs in index order.  Nothing here is shared with the HIP
 * library, and the library never calls it: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may load this file.
 *
 * What each function follows (paper = "Unit Scaling: Out-of-the-Box Low-Precision Training"):
 *   formats   Sec. 3.1 "Floating-point formats" (value formula, bias = 2^(E-1)-1) and Table A.1
 *             rows FP16, FP8 E5 (b), FP8 E4 (b); App. B for their special values.
 *   cast      Sec. 3.1 "Quantisation error" (nearest representable value, clipping at the range
 *             limit) and App. J.2 "Mixed precision" (FP8 = quantise the FP16 tensor to the FP8 set).
 *   matmul    Sec. 5.5 "Example" (alpha*X W, beta_1*G W^T, beta_2*X^T G) and Table A.2 "Linear".
 *   gelu      Table A.2 "Activations": gelu(x) = x*Phi(x); backward by the f_grad definition of
 *             Sec. 5.1 (incoming gradient times the derivative), each with its own fixed scale.
 *
 *   act       Table A.2 "Activations" (relu, tanh, sigmoid next to gelu), each with its own forward and
 *             backward scale, and App. H "Activation functions" for the aligned form f(s1*x)*s2.
 *   layernorm Table A.2 "Other": layer_norm(X, w, c)_ij = c_j + w_j (X_ij - mu_i)/sigma_i with
 *             mu_i = mean_j X_ij, sigma_i = sqrt(mean_j X_ij^2 - mu_i^2); alpha = beta_x = 1,
 *             beta_w = beta_c = b^-1/2 (weights are cut-edges, activations are not: App. I.1).
 *   diagnostics  Fig. 1 / App. K: histogram of exponent values on the FP16 grid (with the bins for zero,
 *             subnormal and infinite values of App. K); Sec. 3.1: SNR = E[X^2] / E[(q(X) - X)^2] of a cast.
 *   residual  Sec. 5.3 "Weighted addition": the fixed(tau) interpolation sqrt(1-tau)*x + sqrt(tau)*f(x),
 *             with the residual branch's weight moved out of its backward pass (the id* rewrite of
 *             that section); Table A.2 "weighted_add" for the general scale rule.
 *
 * Readings of points the paper leaves open are listed next to each function.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ODT_F32 = 0, ODT_F16 = 1, ODT_E4M3 = 2, ODT_E5M2 = 3 };

typedef struct {
  int E, M;         /* exponent / mantissa field widths */
  int bias;         /* 2^(E-1) - 1                                                   (Sec. 3.1) */
  int emax, emin;   /* largest / smallest exponent of a normal value                 (Table A.1) */
  int ieee_specials; /* 1: top exponent field is inf/NaN; 0: only all-ones pattern is NaN (App. B) */
} fmt_t;

static fmt_t fmt_of(int dt) {
  fmt_t f;
  memset(&f, 0, sizeof f);
  switch (dt) {
    case ODT_F16:  f.E = 5; f.M = 10; f.ieee_specials = 1; break;
    case ODT_E5M2: f.E = 5; f.M = 2;  f.ieee_specials = 1; break;
    case ODT_E4M3: f.E = 4; f.M = 3;  f.ieee_specials = 0; break;
    default:       f.E = 8; f.M = 23; f.ieee_specials = 1; break;
  }
  f.bias = (1 << (f.E - 1)) - 1;
  f.emin = 1 - f.bias;
  /* IEEE-like formats give up the whole top exponent field; E4 (b) keeps it as a normal binade. */
  f.emax = f.ieee_specials ? ((1 << f.E) - 2 - f.bias) : ((1 << f.E) - 1 - f.bias);
  return f;
}

/* Largest finite magnitude.  E4 (b): mantissa 111 of the top binade is NaN, so 110 is the top. */
static double fmt_max(fmt_t f) {
  double top_mant = f.ieee_specials ? (double)((1 << f.M) - 1) : (double)((1 << f.M) - 2);
  return ldexp(1.0 + top_mant / (double)(1 << f.M), f.emax);
}

/* ---- decode: the value formula of Sec. 3.1, plus subnormals and specials ------------------ */
double uso_decode_bits(uint32_t bits, int dt) {
  if (dt == ODT_F32) {
    float v;
    memcpy(&v, &bits, 4);
    return (double)v;
  }
  fmt_t f = fmt_of(dt);
  uint32_t b_mant = bits & ((1u << f.M) - 1u);
  uint32_t b_exp = (bits >> f.M) & ((1u << f.E) - 1u);
  uint32_t b_sign = (bits >> (f.M + f.E)) & 1u;
  double sign = b_sign ? -1.0 : 1.0;
  uint32_t all_ones = (1u << f.E) - 1u;
  if (f.ieee_specials && b_exp == all_ones) return b_mant ? NAN : sign * INFINITY;
  if (!f.ieee_specials && b_exp == all_ones && b_mant == (1u << f.M) - 1u) return NAN;
  if (b_exp == 0) /* subnormal: no implicit one, exponent pinned at emin */
    return sign * ldexp((double)b_mant / (double)(1u << f.M), f.emin);
  return sign * ldexp(1.0 + (double)b_mant / (double)(1u << f.M), (int)b_exp - f.bias);
}

/*
 * ---- encode: nearest representable value, ties to even, one rounding from double ---------------
 * Reading (paper: "nearest representable value", ties unstated): round-half-to-even.
 * Overflow: `saturate` != 0 clips to +-max finite (the FP8 "clipping error" of Sec. 3.1, also for
 * +-inf input); `saturate` == 0 follows IEEE and gives +-inf (FP16 tensors keep an infinity bin in
 * the paper's histograms, App. K).  NaN maps to the format's quiet NaN pattern.
 * *overflowed is set when |v| exceeded max finite before rounding (inf included).
 */
static uint32_t encode_f64(double v, int dt, int saturate, int* overflowed) {
  fmt_t f = fmt_of(dt);
  uint32_t sign = signbit(v) ? 1u : 0u;
  uint32_t sign_bits = sign << (f.M + f.E);
  uint32_t all_ones = (1u << f.E) - 1u;
  double a = fabs(v);
  double vmax = fmt_max(f);
  if (overflowed) *overflowed = 0;
  if (isnan(v)) {
    if (f.ieee_specials) return sign_bits | (all_ones << f.M) | (1u << (f.M - 1));
    return sign_bits | (all_ones << f.M) | ((1u << f.M) - 1u);
  }
  if (a > vmax && overflowed) *overflowed = 1;
  if (a == 0.0) return sign_bits;
  uint32_t max_code = f.ieee_specials ? (((all_ones - 1u) << f.M) | ((1u << f.M) - 1u))
                                      : ((all_ones << f.M) | ((1u << f.M) - 2u));
  uint32_t inf_code = all_ones << f.M; /* only meaningful for ieee_specials */
  if (isinf(v)) return sign_bits | ((saturate || !f.ieee_specials) ? max_code : inf_code);
  int e;
  (void)frexp(a, &e); /* a = frac * 2^e, frac in [0.5, 1)  =>  floor(log2 a) = e - 1 */
  e -= 1;
  if (e < f.emin) e = f.emin;           /* subnormal range shares the quantum of the lowest binade */
  double quantum_inv_exp = (double)(f.M - e);
  double q = ldexp(a, (int)quantum_inv_exp); /* a / 2^(e-M): exact scaling by a power of two     */
  double r = nearbyint(q);              /* default rounding mode = round-half-to-even            */
  /* r is an integer in [0, 2^(M+1)]: 2^M..2^(M+1)-1 normal, below 2^M subnormal, 2^(M+1) = carry  */
  if (r >= (double)(1u << (f.M + 1))) { r /= 2.0; e += 1; }
  uint32_t code;
  if (r < (double)(1u << f.M)) {
    code = (uint32_t)r;                 /* exponent field 0 */
  } else {
    if (e > f.emax) {
      code = 0xffffffffu;               /* marks overflow after rounding */
    } else {
      code = ((uint32_t)(e + f.bias) << f.M) | ((uint32_t)r - (1u << f.M));
    }
  }
  if (code == 0xffffffffu || code > max_code)
    code = (saturate || !f.ieee_specials) ? max_code : inf_code;
  return sign_bits | code;
}

uint32_t uso_encode_f64(double v, int dt, int saturate) { return encode_f64(v, dt, saturate, NULL); }

/* ---- element-wise array helpers -------------------------------------------------------------- */
static size_t dt_size(int dt) { return dt == ODT_F32 ? 4 : dt == ODT_F16 ? 2 : 1; }

static uint32_t load_bits(const void* p, int dt, size_t i) {
  switch (dt) {
    case ODT_F32: { uint32_t u; memcpy(&u, (const char*)p + 4 * i, 4); return u; }
    case ODT_F16: { uint16_t u; memcpy(&u, (const char*)p + 2 * i, 2); return u; }
    default: return ((const uint8_t*)p)[i];
  }
}
static void store_bits(void* p, int dt, size_t i, uint32_t bits) {
  switch (dt) {
    case ODT_F32: memcpy((char*)p + 4 * i, &bits, 4); break;
    case ODT_F16: { uint16_t u = (uint16_t)bits; memcpy((char*)p + 2 * i, &u, 2); break; }
    default: ((uint8_t*)p)[i] = (uint8_t)bits;
  }
}
/* round a double result to the output storage type (FP32 / FP16: IEEE, no clamp) */
static uint32_t round_out(double v, int dt) {
  if (dt == ODT_F32) { float fv = (float)v; uint32_t u; memcpy(&u, &fv, 4); return u; }
  return encode_f64(v, dt, 0, NULL);
}

void uso_decode(const void* src, int dt, size_t n, double* out) {
  for (size_t i = 0; i < n; ++i) out[i] = uso_decode_bits(load_bits(src, dt, i), dt);
}
void uso_encode(const double* src, size_t n, int dt, int saturate, void* out) {
  for (size_t i = 0; i < n; ++i) store_bits(out, dt, i, encode_f64(src[i], dt, saturate, NULL));
}

/*
 * ---- scaled, saturating cast to FP8 ------------------------------------------------------------
 * p = fp32(x * s) (the product of two <=24-bit significands is exact in double, so this is one IEEE
 * single-precision multiply), then the nearest FP8 value of p, clipped at +-max.
 * Counters (stats[0..3], added to, never cleared):
 *   [0] n_sat       |p| > max finite (inf included)             -- "outside the absolute range"
 *   [1] n_flush0    p != 0 but the code is +-0                   -- underflow
 *   [2] n_subnormal code != +-0 and |decoded| < smallest normal
 *   [3] n_nan       p is NaN
 */
void uso_cast_fp8(const void* src, int src_dt, void* dst, int dst_dt, size_t n, float scale,
                  unsigned long long* stats) {
  fmt_t f = fmt_of(dst_dt);
  double min_normal = ldexp(1.0, f.emin);
  for (size_t i = 0; i < n; ++i) {
    double x = uso_decode_bits(load_bits(src, src_dt, i), src_dt);
    float p = (float)(x * (double)scale);
    int ovf = 0;
    uint32_t code = encode_f64((double)p, dst_dt, 1, &ovf);
    ((uint8_t*)dst)[i] = (uint8_t)code;
    if (stats) {
      if (isnan(p)) { stats[3]++; continue; }
      double d = fabs(uso_decode_bits(code, dst_dt));
      if (ovf) stats[0]++;
      if (p != 0.0f && d == 0.0) stats[1]++;
      if (d != 0.0 && d < min_normal) stats[2]++;
    }
  }
}

/*
 * ---- scaled matmuls (Sec. 5.5; Table A.2 "Linear") ------------------------------------------
 * X[b,m], W[m,n], G[b,n], all row-major; operands are first decoded to double.
 *   fwd   Y [i,j] = round_out( alpha  * sum_{k<m} X[i,k] W[k,j] )
 *   dx    dX[i,k] = round_out( beta_x * sum_{j<n} G[i,j] W[k,j] )
 *   dw    dW[k,j] = round_out( beta_w * sum_{i<b} X[i,k] G[i,j] )
 * Returns 0, or 1 if the temporaries could not be allocated.
 * The scale is a float argument (the library receives it as a float too), widened to double; the
 * sum is taken in index order in double; one rounding to the output type.
 * Reading: accumulation precision is unstated in the paper; double here, so the reference is the
 * exact product up to ~1e-16 and any FP32 summation order on the GPU is judged against it.
 */
static double* decode_all(const void* src, int dt, size_t n) {
  double* d = (double*)malloc(n * sizeof(double));
  if (d) uso_decode(src, dt, n, d);
  return d;
}

/* Forward product with an optional bias row c[n] (FP16 storage; NULL = none): the FFN of App. J.1 is
 * W2 act(W1 z + b1) + b2.  Reading (the paper gives the bias no scale of its own): biases start at zero
 * ("non-bias parameters" are the ones drawn with unit variance, Sec. 5.2 recipe), so adding them leaves the
 * unit-variance output as it is and the forward pass needs no factor; the bias joins the scaled sum before the
 * single rounding:  Y[i,j] = round_out( alpha * sum_k X[i,k] W[k,j] + c[j] ). */
static int linear_fwd_impl(const void* X, int x_dt, const void* W, int w_dt, const void* c, void* Y, int y_dt,
                           long b, long m, long n, float alpha) {
  double* Xd = decode_all(X, x_dt, (size_t)b * m);
  double* Wd = decode_all(W, w_dt, (size_t)m * n);
  double* cd = c ? decode_all(c, ODT_F16, (size_t)n) : NULL;
  if (!Xd || !Wd || (c && !cd)) { free(Xd); free(Wd); free(cd); return 1; }
#pragma omp parallel
  {
    double* acc = (double*)malloc((size_t)n * sizeof(double)); /* one output row of running sums */
#pragma omp for schedule(static)
    for (long i = 0; i < b; ++i) {
      for (long j = 0; j < n; ++j) acc[j] = 0.0;
      for (long k = 0; k < m; ++k) {          /* k ascending: every acc[j] sums in index order */
        double x = Xd[i * m + k];
        for (long j = 0; j < n; ++j) acc[j] += x * Wd[k * n + j];
      }
      for (long j = 0; j < n; ++j)
        store_bits(Y, y_dt, (size_t)(i * n + j), round_out((double)alpha * acc[j] + (cd ? cd[j] : 0.0), y_dt));
    }
    free(acc);
  }
  free(Xd); free(Wd); free(cd);
  return 0;
}

int uso_linear_fwd(const void* X, int x_dt, const void* W, int w_dt, void* Y, int y_dt,
                   long b, long m, long n, float alpha) {
  return linear_fwd_impl(X, x_dt, W, w_dt, NULL, Y, y_dt, b, m, n, alpha);
}

int uso_linear_bias_fwd(const void* X, int x_dt, const void* W, int w_dt, const void* c, void* Y, int y_dt,
                        long b, long m, long n, float alpha) {
  return linear_fwd_impl(X, x_dt, W, w_dt, c, Y, y_dt, b, m, n, alpha);
}

/* Gradient of a bias row: dc[j] = round_out( beta_c * sum_{i<b} G[i,j] ), rows in index order, double sum.
 * Reading: the sum runs over the b rows (tokens) like the one in grad_W, and like the bias c of the scaled
 * layer norm (Table A.2 "Other": beta_c = b^-1/2) it gets b^-1/2; the factor is an argument. */
void uso_bias_grad(const void* G, int g_dt, void* dc, int o_dt, long b, long n, float beta_c) {
  double* acc = (double*)calloc((size_t)n, sizeof(double));
  for (long i = 0; i < b; ++i)
    for (long j = 0; j < n; ++j) acc[j] += uso_decode_bits(load_bits(G, g_dt, (size_t)(i * n + j)), g_dt);
  for (long j = 0; j < n; ++j) store_bits(dc, o_dt, (size_t)j, round_out((double)beta_c * acc[j], o_dt));
  free(acc);
}

int uso_linear_bwd_dx(const void* G, int g_dt, const void* W, int w_dt, void* dX, int o_dt,
                      long b, long m, long n, float beta_x) {
  double* Gd = decode_all(G, g_dt, (size_t)b * n);
  double* Wd = decode_all(W, w_dt, (size_t)m * n);
  if (!Gd || !Wd) { free(Gd); free(Wd); return 1; }
#pragma omp parallel for schedule(static)
  for (long i = 0; i < b; ++i) {
    for (long k = 0; k < m; ++k) {
      double acc = 0.0;
      for (long j = 0; j < n; ++j) acc += Gd[i * n + j] * Wd[k * n + j];
      store_bits(dX, o_dt, (size_t)(i * m + k), round_out((double)beta_x * acc, o_dt));
    }
  }
  free(Gd); free(Wd);
  return 0;
}

int uso_linear_bwd_dw(const void* X, int x_dt, const void* G, int g_dt, void* dW, int o_dt,
                      long b, long m, long n, float beta_w) {
  double* Xd = decode_all(X, x_dt, (size_t)b * m);
  double* Gd = decode_all(G, g_dt, (size_t)b * n);
  if (!Xd || !Gd) { free(Xd); free(Gd); return 1; }
#pragma omp parallel
  {
    double* acc = (double*)malloc((size_t)n * sizeof(double)); /* one row of dW */
#pragma omp for schedule(static)
    for (long k = 0; k < m; ++k) {
      for (long j = 0; j < n; ++j) acc[j] = 0.0;
      for (long i = 0; i < b; ++i) {          /* tokens ascending: index-order sum per element */
        double x = Xd[i * m + k];
        for (long j = 0; j < n; ++j) acc[j] += x * Gd[i * n + j];
      }
      for (long j = 0; j < n; ++j)
        store_bits(dW, o_dt, (size_t)(k * n + j), round_out((double)beta_w * acc[j], o_dt));
    }
    free(acc);
  }
  free(Xd); free(Gd);
  return 0;
}

/*
 * ---- unit-scaled GELU (Table A.2 "Activations": gelu(x) = x * Phi(x)) -----------------------
 * Reading: the exact Gaussian-CDF form, not the tanh approximation.  Phi(z) = erfc(-z/sqrt 2)/2 keeps
 * full relative accuracy in the negative tail.  Inputs and outputs are FP16 (or FP32) storage;
 * arithmetic in double; one rounding.
 *   fwd  h  = round( alpha_g * z * Phi(z) )
 *   bwd  gz = round( beta_g * (Phi(z) + z * phi(z)) * gh ),   phi = standard normal density
 */
static double Phi(double z) { return 0.5 * erfc(-z * M_SQRT1_2); }
static double phi(double z) { return exp(-0.5 * z * z) / sqrt(2.0 * M_PI); }

void uso_gelu_fwd(const void* z, void* h, size_t n, int dt, float alpha_g) {
  for (size_t i = 0; i < n; ++i) {
    double zi = uso_decode_bits(load_bits(z, dt, i), dt);
    store_bits(h, dt, i, round_out((double)alpha_g * zi * Phi(zi), dt));
  }
}
void uso_gelu_bwd(const void* z, const void* gh, void* gz, size_t n, int dt, float beta_g) {
  for (size_t i = 0; i < n; ++i) {
    double zi = uso_decode_bits(load_bits(z, dt, i), dt);
    double gi = uso_decode_bits(load_bits(gh, dt, i), dt);
    store_bits(gz, dt, i, round_out((double)beta_g * (Phi(zi) + zi * phi(zi)) * gi, dt));
  }
}

/*
 * ---- the other activations of Table A.2, aligned form of App. H ----------------------------------
 *   kind 0 gelu(x) = x*Phi(x), 1 relu(x) = max(x, 0), 2 tanh(x), 3 sigmoid(x) = 1/(1+exp(-x))
 *   fwd  h  = round( scale * f(s1 * z) )              (scale = alpha, or s2 of the aligned form)
 *   bwd  gz = round( scale * f'(s1 * z) * gh )        (scale = beta; the caller folds s1 into it)
 * Readings: relu'(0) = 0 (the derivative is taken as the indicator of x > 0, whose mean square 1/2 is what
 * App. E.1 uses for beta = sqrt 2); tanh and sigmoid by libm in double.
 */
static double act_f(int kind, double x) {
  switch (kind) {
    case 1: return x > 0.0 ? x : 0.0;
    case 2: return tanh(x);
    case 3: return 1.0 / (1.0 + exp(-x));
    default: return x * Phi(x);
  }
}
static double act_df(int kind, double x) {
  switch (kind) {
    case 1: return x > 0.0 ? 1.0 : 0.0;
    case 2: { double c = cosh(x); return 1.0 / (c * c); }
    case 3: { double s = 1.0 / (1.0 + exp(-fabs(x))); return s * (1.0 - s); }
    default: return Phi(x) + x * phi(x);
  }
}
void uso_act_fwd(const void* z, void* h, size_t n, int dt, int kind, float s1, float scale) {
  for (size_t i = 0; i < n; ++i) {
    double zi = uso_decode_bits(load_bits(z, dt, i), dt);
    store_bits(h, dt, i, round_out((double)scale * act_f(kind, (double)s1 * zi), dt));
  }
}
void uso_act_bwd(const void* z, const void* gh, void* gz, size_t n, int dt, int kind, float s1, float scale) {
  for (size_t i = 0; i < n; ++i) {
    double zi = uso_decode_bits(load_bits(z, dt, i), dt);
    double gi = uso_decode_bits(load_bits(gh, dt, i), dt);
    store_bits(gz, dt, i, round_out((double)scale * act_df(kind, (double)s1 * zi) * gi, dt));
  }
}

/*
 * ---- scaled layer norm (Table A.2 "Other") ------------------------------------------------------
 * X[b,n], w[n], c[n], Y[b,n] of storage type dt; mean[b], rstd[b] are doubles handed back for tests.
 *   fwd:  Y_ij = round( c_j + w_j * (X_ij - mu_i) * rstd_i ),  rstd_i = 1/sqrt(mean_j X_ij^2 - mu_i^2 + eps)
 *   bwd:  with xh = (X - mu) rstd and gh_ij = G_ij w_j (f_grad of the formula above, times beta):
 *         dX_ij = round( rstd_i * (gh_ij - mean_j gh_ij - xh_ij * mean_j(gh_ij xh_ij)) )           beta_x = 1
 *         dw_j  = round( beta_wc * sum_i G_ij xh_ij ),  dc_j = round( beta_wc * sum_i G_ij )       beta_wc = b^-1/2
 * Readings: the paper's variance formula as printed (second moment minus squared mean, in double); it has no
 * epsilon, so eps is an argument (0 gives the printed formula); every sum in index order.
 */
void uso_layer_norm_fwd(const void* X, const void* w, const void* c, void* Y, double* mean, double* rstd, long b, long n,
                        int dt, double eps) {
  for (long i = 0; i < b; ++i) {
    double s1 = 0.0, s2 = 0.0;
    for (long j = 0; j < n; ++j) {
      double x = uso_decode_bits(load_bits(X, dt, (size_t)(i * n + j)), dt);
      s1 += x;
      s2 += x * x;
    }
    double mu = s1 / (double)n, var = s2 / (double)n - mu * mu;
    double rs = 1.0 / sqrt(var + eps);
    if (mean) mean[i] = mu;
    if (rstd) rstd[i] = rs;
    for (long j = 0; j < n; ++j) {
      double x = uso_decode_bits(load_bits(X, dt, (size_t)(i * n + j)), dt);
      double wj = uso_decode_bits(load_bits(w, dt, (size_t)j), dt), cj = uso_decode_bits(load_bits(c, dt, (size_t)j), dt);
      store_bits(Y, dt, (size_t)(i * n + j), round_out(cj + wj * (x - mu) * rs, dt));
    }
  }
}

void uso_layer_norm_bwd(const void* X, const void* w, const void* G, void* dX, void* dw, void* dc, long b, long n, int dt,
                        double eps, float beta_wc) {
  double* aw = (double*)calloc((size_t)n, sizeof(double));
  double* ac = (double*)calloc((size_t)n, sizeof(double));
  for (long i = 0; i < b; ++i) {
    double s1 = 0.0, s2 = 0.0;
    for (long j = 0; j < n; ++j) {
      double x = uso_decode_bits(load_bits(X, dt, (size_t)(i * n + j)), dt);
      s1 += x;
      s2 += x * x;
    }
    double mu = s1 / (double)n, rs = 1.0 / sqrt(s2 / (double)n - mu * mu + eps);
    double m1 = 0.0, m2 = 0.0;
    for (long j = 0; j < n; ++j) {
      double x = uso_decode_bits(load_bits(X, dt, (size_t)(i * n + j)), dt);
      double g = uso_decode_bits(load_bits(G, dt, (size_t)(i * n + j)), dt);
      double wj = uso_decode_bits(load_bits(w, dt, (size_t)j), dt);
      double xh = (x - mu) * rs, gh = g * wj;
      m1 += gh;
      m2 += gh * xh;
      aw[j] += g * xh;
      ac[j] += g;
    }
    m1 /= (double)n;
    m2 /= (double)n;
    for (long j = 0; j < n; ++j) {
      double x = uso_decode_bits(load_bits(X, dt, (size_t)(i * n + j)), dt);
      double g = uso_decode_bits(load_bits(G, dt, (size_t)(i * n + j)), dt);
      double wj = uso_decode_bits(load_bits(w, dt, (size_t)j), dt);
      double xh = (x - mu) * rs;
      store_bits(dX, dt, (size_t)(i * n + j), round_out(rs * (g * wj - m1 - xh * m2), dt));
    }
  }
  for (long j = 0; j < n; ++j) {
    store_bits(dw, dt, (size_t)j, round_out((double)beta_wc * aw[j], dt));
    store_bits(dc, dt, (size_t)j, round_out((double)beta_wc * ac[j], dt));
  }
  free(aw);
  free(ac);
}

/*
 * ---- diagnostics: exponent histogram and signal-to-noise ratio of a cast ---------------------------
 * Histogram bins (35), by the magnitude of each value on the FP16 exponent grid of Fig. 1 / App. K:
 *   0 zero | 1 non-zero below 2^-24 (lost in FP16) | 2 FP16-subnormal range [2^-24, 2^-14) |
 *   3 + (e + 14) for 2^e <= |x| < 2^(e+1), e = -14 .. 15 | 33 |x| >= 2^16 or infinite | 34 NaN
 * Counts are added to hist (the caller clears it).
 * SNR: sums[0] += sum x^2, sums[1] += sum (q(x*scale)/scale - x)^2 with q the saturating cast of uso_cast_fp8
 * (its product rounded to FP32 first, as there); NaN inputs are skipped.  Sec. 3.1 defines SNR as sums[0]/sums[1].
 */
void uso_exponent_histogram(const void* src, int dt, size_t n, unsigned long long* hist) {
  for (size_t i = 0; i < n; ++i) {
    double a = fabs(uso_decode_bits(load_bits(src, dt, i), dt));
    int bin;
    if (a != a) bin = 34;
    else if (a == 0.0) bin = 0;
    else if (a >= 65536.0) bin = 33;
    else if (a < ldexp(1.0, -24)) bin = 1;
    else if (a < ldexp(1.0, -14)) bin = 2;
    else {
      int e;
      frexp(a, &e); /* a = f * 2^e, f in [0.5, 1): exponent of the leading bit is e - 1 */
      bin = 3 + (e - 1 + 14);
    }
    hist[bin] += 1;
  }
}

void uso_cast_snr(const void* src, int src_dt, size_t n, int dst_dt, float scale, double* sums) {
  double s0 = 0.0, s1 = 0.0;
  for (size_t i = 0; i < n; ++i) {
    double x = uso_decode_bits(load_bits(src, src_dt, i), src_dt);
    if (x != x) continue;
    float p = (float)(x * (double)scale);
    double q = uso_decode_bits(encode_f64((double)p, dst_dt, 1, NULL), dst_dt) / (double)scale;
    s0 += x * x;
    s1 += (q - x) * (q - x);
  }
  sums[0] += s0;
  sums[1] += s1;
}

/*
 * ---- weighted addition of two tensors (Sec. 5.3; Table A.2 "weighted_add") --------------------
 *   out = round( ca * a + cb * b ),  a and b of storage type dt, arithmetic in double, one rounding.
 * Used for the residual layer: forward (a, b) = (skip input x, branch output f(x)) with
 * (ca, cb) = (sqrt(1-tau), sqrt(tau)); backward (a, b) = (incoming gradient g, branch input gradient)
 * with the same weights, because the rewrite gamma*f(x) -> id*(f(id*(x, 1, gamma)), gamma, 1) applies
 * gamma = sqrt(tau) to the branch's OUTPUT in the forward pass and to the gradient leaving the branch's
 * INPUT in the backward pass, so that the gradient entering the branch is the unscaled g.
 * Reading: the weights arrive as floats (what the library gets) and are widened to double.
 */
void uso_weighted_add2(const void* a, const void* b, void* out, size_t n, int dt, float ca, float cb) {
  for (size_t i = 0; i < n; ++i) {
    double ai = uso_decode_bits(load_bits(a, dt, i), dt);
    double bi = uso_decode_bits(load_bits(b, dt, i), dt);
    store_bits(out, dt, i, round_out((double)ca * ai + (double)cb * bi, dt));
  }
}

/*
 * ---- scaled sum over the last dimension (Table A.2 "Linear": sum(x) = sum_i x_i, alpha = n^-1/2, beta = 1) -----
 *   fwd  y_i   = round( alpha * sum_{j<n} x_ij )      double sum in index order
 *   bwd  dx_ij = round( beta * g_i )                  the gradient of a sum is its incoming gradient in every place
 */
void uso_sum_fwd(const void* x, void* y, long rows, long n, float alpha) {
  for (long i = 0; i < rows; ++i) {
    double acc = 0.0;
    for (long j = 0; j < n; ++j) acc += uso_decode_bits(load_bits(x, ODT_F16, (size_t)(i * n + j)), ODT_F16);
    store_bits(y, ODT_F16, (size_t)i, round_out((double)alpha * acc, ODT_F16));
  }
}

void uso_sum_bwd(const void* g, void* dx, long rows, long n, float beta) {
  for (long i = 0; i < rows; ++i) {
    const uint32_t b = round_out((double)beta * uso_decode_bits(load_bits(g, ODT_F16, (size_t)i), ODT_F16), ODT_F16);
    for (long j = 0; j < n; ++j) store_bits(dx, ODT_F16, (size_t)(i * n + j), b);
  }
}

/*
 * ---- scaled softmax and softmax cross-entropy (Table A.2 "Other"; App. G "Softmax (followed by matmul)",
 *      "Softmax cross-entropy"; App. H "Softmax functions" for the input factor s1) --------------------
 * Rows of s values, FP16 storage, double arithmetic, one rounding per output.
 *   softmax fwd   y_j  = round( alpha * p_j ),  p = softmax(s1 * x) computed with the row maximum subtracted
 *                 (Table A.2: alpha = s, so that the output is about a vector of ones for the matmul that follows)
 *   softmax bwd   dx_j = round( beta * s1 * p_j * (g_j - sum_k p_k g_k) )      (Table A.2: beta = s)
 *                 f_grad of the unscaled softmax times beta (Sec. 5.1), p recomputed from x, not taken from
 *                 the rounded output
 *   xent          loss = -(t_c - log sum_k exp(t_k)),  t = s1 * x, c the target class      (alpha = 1)
 *                 dx_j = round( beta * s1 * (p_j - [j == c]) )   (App. G: beta = s / sqrt(s - 1); the op ends
 *                 the model, so the incoming gradient is 1)
 *                 Reading: a target outside 0 .. s-1 marks a row without a label (positions that are not
 *                 predicted): loss 0, gradient row 0.
 * s1 * x is not rounded before the exponential.
 */
static void softmax_row(const void* x, long row, long s, double s1, double* p, double* logsum, double* maxv) {
  double m = -INFINITY;
  int has_nan = 0;
  for (long j = 0; j < s; ++j) {
    double t = s1 * uso_decode_bits(load_bits(x, ODT_F16, (size_t)(row * s + j)), ODT_F16);
    p[j] = t;
    if (isnan(t)) has_nan = 1;
    if (t > m) m = t;
  }
  if (has_nan) m = NAN;
  double sum = 0.0;
  for (long j = 0; j < s; ++j) { p[j] = exp(p[j] - m); sum += p[j]; }
  for (long j = 0; j < s; ++j) p[j] /= sum;
  if (logsum) *logsum = log(sum);
  if (maxv) *maxv = m;
}

void uso_softmax_fwd(const void* x, void* y, long rows, long s, float s1, float alpha) {
#pragma omp parallel
  {
    double* p = (double*)malloc((size_t)s * sizeof(double));
#pragma omp for schedule(static)
    for (long i = 0; i < rows; ++i) {
      softmax_row(x, i, s, (double)s1, p, NULL, NULL);
      for (long j = 0; j < s; ++j) store_bits(y, ODT_F16, (size_t)(i * s + j), round_out((double)alpha * p[j], ODT_F16));
    }
    free(p);
  }
}

void uso_softmax_bwd(const void* x, const void* g, void* dx, long rows, long s, float s1, float beta) {
#pragma omp parallel
  {
    double* p = (double*)malloc((size_t)s * sizeof(double));
#pragma omp for schedule(static)
    for (long i = 0; i < rows; ++i) {
      softmax_row(x, i, s, (double)s1, p, NULL, NULL);
      double dot = 0.0;
      for (long j = 0; j < s; ++j) dot += p[j] * uso_decode_bits(load_bits(g, ODT_F16, (size_t)(i * s + j)), ODT_F16);
      for (long j = 0; j < s; ++j) {
        double gj = uso_decode_bits(load_bits(g, ODT_F16, (size_t)(i * s + j)), ODT_F16);
        store_bits(dx, ODT_F16, (size_t)(i * s + j), round_out((double)beta * (double)s1 * p[j] * (gj - dot), ODT_F16));
      }
    }
    free(p);
  }
}

void uso_softmax_xent(const void* x, const int* target, double* loss, void* dx, long rows, long s, float s1, float beta) {
#pragma omp parallel
  {
    double* p = (double*)malloc((size_t)s * sizeof(double));
#pragma omp for schedule(static)
    for (long i = 0; i < rows; ++i) {
      const long c = target[i];
      if (c < 0 || c >= s) {
        if (loss) loss[i] = 0.0;
        if (dx) for (long j = 0; j < s; ++j) store_bits(dx, ODT_F16, (size_t)(i * s + j), 0);
        continue;
      }
      double logsum, m;
      softmax_row(x, i, s, (double)s1, p, &logsum, &m);
      if (loss) {
        double tc = (double)s1 * uso_decode_bits(load_bits(x, ODT_F16, (size_t)(i * s + c)), ODT_F16);
        loss[i] = -(tc - m - logsum);
      }
      if (dx)
        for (long j = 0; j < s; ++j)
          store_bits(dx, ODT_F16, (size_t)(i * s + j),
                     round_out((double)beta * (double)s1 * (p[j] - (j == c ? 1.0 : 0.0)), ODT_F16));
    }
    free(p);
  }
}


/*
 * ---- scale selection (Sec. 5.5; Table A.2; Sec. 5.2 for the geometric-mean rule) --------------
 * mode 0: unconstrained  alpha = m^-1/2, beta_x = n^-1/2, beta_w = b^-1/2
 * mode 1: X is not a cut-edge, so alpha = beta_x = (m*n)^-1/4; beta_w unchanged
 * Returned as floats (what the library passes to its kernels).
 */
void uso_linear_scales(long b, long m, long n, int mode, float* alpha, float* beta_x, float* beta_w) {
  double a = 1.0 / sqrt((double)m), bx = 1.0 / sqrt((double)n), bw = 1.0 / sqrt((double)b);
  if (mode == 1) a = bx = sqrt(a * bx); /* geometric mean of the two constrained factors */
  *alpha = (float)a;
  *beta_x = (float)bx;
  *beta_w = (float)bw;
}

size_t uso_dtype_size(int dt) { return dt_size(dt); }
