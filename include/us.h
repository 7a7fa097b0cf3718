/*
 * us.h -- C ABI of the unit-scaled linear / FFN library for AMD MI355X (gfx950).
 *
 * The operations are the scaled ops of "Unit Scaling: Out-of-the-Box Low-Precision Training":
 * every op carries a fixed forward scale alpha and fixed backward scales beta_i (Sec. 5.1 "Scaled
 * ops"), chosen so that outputs and gradients have unit variance at initialisation (Sec. 5.2), which
 * lets all tensors live in FP16 and all matmul inputs in FP8 without a loss scale (Sec. 3.2, App. J.2).
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never allocates,
 *     frees or keeps a pointer.  Matrices are dense row-major: X[b,m], W[m,n] (fan_in x fan_out),
 *     G[b,n].  `b` is the number of tokens (batch x sequence, flattened).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     and return; there is no host synchronisation inside.
 *   - Errors are reported by status code only and are detected on the host before anything is
 *     launched: a failing call has no effect on device memory.
 *   - Tensor pointers must be 16-byte aligned; matrix dimensions must be multiples of 16.  Element
 *     counts of the element-wise calls are arbitrary.
 *   - Storage types: US_F16 = IEEE binary16; US_E4M3 / US_E5M2 = the 8-bit formats of Table A.1
 *     rows "E4 (b)" / "E5 (b)" (bias 7, max 448, one NaN, no infinity / bias 15, max 57344, IEEE
 *     specials); US_F32 = IEEE binary32.  Subnormals are honoured everywhere.
 *   - Rounding is to nearest, ties to even.  FP16/FP32 outputs overflow to infinity (IEEE); FP8
 *     outputs clip at the largest finite value.
 *   - Results are bit-identical from run to run.
 */
#ifndef US_H_
#define US_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  US_OK = 0,
  US_ERR_NULL = 1,       /* a required pointer is NULL                                   */
  US_ERR_SHAPE = 2,      /* negative dimension, or a matrix dimension not a multiple of 16 */
  US_ERR_ALIGN = 3,      /* a pointer is not 16-byte aligned                              */
  US_ERR_DTYPE = 4,      /* unsupported storage-type combination                          */
  US_ERR_WORKSPACE = 5,  /* workspace missing or smaller than us_workspace_bytes()        */
  US_ERR_LAUNCH = 6,     /* the HIP runtime refused a launch                              */
  US_ERR_VALUE = 7       /* a scalar argument outside its domain (e.g. a residual weight)   */
} us_status;

typedef enum { US_F32 = 0, US_F16 = 1, US_E4M3 = 2, US_E5M2 = 3 } us_dtype;

typedef enum {
  US_EPI_NONE = 0,
  US_EPI_GELU = 1,       /* forward: also emit the unit-scaled GELU of the output            */
  US_EPI_GELU_GRAD = 2,  /* grad_X: multiply by the unit-scaled GELU derivative of Zpre     */
  US_EPI_RESIDUAL = 3,   /* forward / grad_X: interpolate with a skip input (Sec. 5.3)      */
  /* activation of US_EPI_GELU / US_EPI_GELU_GRAD when not gelu: OR one of these onto it (Table A.2
   * "Activations"; epi_scale <= 0 then selects that activation's own unit-scaling factor)            */
  US_EPI_ACT_RELU = 0x10,
  US_EPI_ACT_TANH = 0x20,
  US_EPI_ACT_SIGMOID = 0x30,
  /* flag, OR-ed onto one of the two above: the table area of the workspace already holds the GELU
   * tables for this epi_scale (us_gelu_tables) and must not be rebuilt by the call                */
  US_EPI_TABLES_READY = 0x100
} us_epilogue;

/* The first US_TABLE_AREA_BYTES of every workspace belong to the tables of the table-driven GELU
 * epilogues (three tables at fixed offsets; a call only touches the one it uses). */
#define US_TABLE_AREA_BYTES (256 * 1024)

/* mode bits of us_ffn_fwd / us_ffn_bwd */
#define US_FFN_FP8 1            /* operands are FP8 codes (else FP16)                                   */
#define US_FFN_TABLES_READY 2   /* as US_EPI_TABLES_READY, for the GELU / GELU' inside the FFN calls  */

/* Counters of the scaled cast; device memory; added to, never cleared, by us_cast_fp8. */
typedef struct {
  unsigned long long n_sat;        /* |x*scale| above the largest finite value (inf included) */
  unsigned long long n_flush0;     /* x*scale != 0 but the code is +-0                        */
  unsigned long long n_subnormal;  /* non-zero code below the smallest normal value           */
  unsigned long long n_nan;        /* x*scale is NaN                                          */
} us_cast_stats;

const char* us_status_string(us_status s);

/* Diagnostics (host only).  Text describing the matmul kernels that the calling host thread's most recent matmul call
 * (us_linear_*, us_ffn_*, us_matmul_batched, us_attention_*) enqueued, one entry per kernel joined by " + ":
 *   kind:BMxBN:wk<wave groups>:st<stages>:<fp8|f16>:<NN|NT|TN>:<epilogue>[:f32]:s<K slices>
 * kind is "direct" (direct-to-LDS loads), "staged" (register-staged fallback for ragged reduction lengths) or "pair"
 * (grad_X and grad_W tiles in one launch).  The string belongs to the library and is valid until the thread's next
 * matmul call.  For tests and tuning: it says which tile shape a problem was given (the choice of kernel is the
 * library's; results do not depend on it beyond the order of the FP32 sums). */
const char* us_last_launch(void);

/*
 * Scale selection for matmul(X[b,m], W[m,n]) (Table A.2 "Linear"; Sec. 5.5 "Example").  Host only.
 *   mode 0: unconstrained  alpha = m^-1/2, beta_x = n^-1/2, beta_w = b^-1/2
 *   mode 1: X is not a cut-edge, so alpha and beta_x are tied to their geometric mean (m*n)^-1/4
 *           (Sec. 5.2 step 2); beta_w = b^-1/2.
 * Outputs are host pointers.  US_ERR_SHAPE if a dimension is < 1 or mode is not 0/1.
 */
us_status us_linear_scales(long b, long m, long n, int mode, float* alpha, float* beta_x, float* beta_w);

/*
 * Scaled saturating cast to FP8 (Sec. 3.1 "Quantisation error"; App. J.2: FP8 training quantises the
 * FP16 tensor to the nearest FP8 value, E4 for activations and weights, E5 for gradients).
 *   dst[i] = nearest_fp8( fp32(src[i] * scale) ), clipped to +-max finite; NaN -> NaN code.
 * src: n elements of src_dt (US_F16 or US_F32); dst: n bytes (US_E4M3 or US_E5M2).  The scale is
 * applied in FP32 before the single rounding.  stats may be NULL; otherwise the four counters are
 * incremented (device memory, caller clears).  n = 0 is a no-op.
 */
us_status us_cast_fp8(const void* src, us_dtype src_dt, void* dst, us_dtype dst_dt, size_t n,
                      float scale, us_cast_stats* stats, void* stream);

/*
 * The same cast with scale 1 for up to US_CAST_BATCH_MAX FP16 tensors in one launch (the activation,
 * weight and gradient casts of one step).  src, dst, n, dst_dt are HOST arrays of `count` entries:
 * device pointers (16-byte aligned), element counts, and US_E4M3 / US_E5M2 per tensor.  No counters.
 * US_ERR_SHAPE if count is outside 0..US_CAST_BATCH_MAX.
 */
#define US_CAST_BATCH_MAX 8
us_status us_cast_fp8_batch(int count, const void* const* src, void* const* dst, const size_t* n,
                            const us_dtype* dst_dt, void* stream);

/*
 * Forward of the scaled projection (Sec. 5.5):  Y[b,n] = alpha * X[b,m] W[m,n].
 * Operand types (x_dt, w_dt): (F16, F16) or (E4M3, E4M3).  FP32 accumulation; y_dt = F16 or F32.
 * alpha <= 0 selects m^-1/2.
 * epi = US_EPI_GELU (y_dt must be F16) additionally computes, from the ROUNDED FP16 value of Y,
 *   H = fp16( epi_scale * gelu(Y) ),  gelu(x) = x*Phi(x)   (Table A.2 "Activations"),
 * stores H to aux16 (FP16 [b,n]) if aux16 != NULL and the E4M3 cast of that FP16 H (scale 1) to aux8
 * ([b,n] bytes) if aux8 != NULL; at least one of them must be given.  epi_scale <= 0 selects the
 * unit-scaling factor 1.7009.  Y itself is always written (the backward pass needs it).
 * epi = US_EPI_RESIDUAL (y_dt must be F16) is the residual layer's weighted addition (Sec. 5.3
 * "Weighted addition", fixed(tau) with epi_scale = sqrt(tau) in (0, 1]):
 *   Y = fp16( sqrt(1 - epi_scale^2) * R + epi_scale * fp16(alpha * X W) ),
 * R = aux16, here an INPUT: the FP16 [b,n] skip tensor (Y itself is the only output; aux8 is ignored).
 * workspace may be NULL.  With epi = US_EPI_GELU, exactly one of aux16 / aux8 and a workspace of at
 * least US_TABLE_AREA_BYTES (16-byte aligned) large problems take the activation from a table over
 * the FP16 values of Y; the result is the same as without a workspace.  By default the call first
 * builds that table in the workspace (so its contents may be undefined on entry); with
 * US_EPI_GELU | US_EPI_TABLES_READY the caller vouches that us_gelu_tables filled this workspace
 * with the same epi_scale and that its first US_TABLE_AREA_BYTES were not overwritten since.
 */
us_status us_linear_fwd(const void* X, const void* W, void* Y, long b, long m, long n,
                        us_dtype x_dt, us_dtype w_dt, us_dtype y_dt, float alpha,
                        us_epilogue epi, float epi_scale, void* aux16, void* aux8,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of the scaled projection (Sec. 5.5):
 *   dX[b,m] = beta_x * G[b,n] W[m,n]^T      (skipped when dX == NULL)
 *   dW[m,n] = beta_w * X[b,m]^T G[b,n]      (skipped when dW == NULL)
 * No transposed copy of any operand is made.  Operand types: all F16, or x_dt = w_dt = E4M3 with
 * g_dt = E5M2.  out_dt = F16 or F32 for both outputs.  beta_x <= 0 selects n^-1/2, beta_w <= 0
 * selects b^-1/2.  X is only read for dW and W only for dX; the unused one may be NULL.
 * epi = US_EPI_GELU_GRAD applies to dX only (out_dt must be F16): with Zpre[b,m] (FP16, the
 * pre-activation saved by the forward pass),
 *   dX = fp16( epi_scale * gelu'(Zpre) * fp16(beta_x * G W^T) ),  gelu'(z) = Phi(z) + z*phi(z),
 * i.e. the scaled-GELU backward of Sec. 5.1 applied to the FP16-rounded matmul gradient; if aux8 !=
 * NULL the E5M2 cast of that FP16 dX is written there, and dX itself may then be NULL (only the
 * codes are stored: the values are the same).  epi_scale <= 0 selects 1.4811.
 * epi = US_EPI_RESIDUAL applies to dX only (out_dt must be F16): the backward pass of a residual layer
 * whose branch starts with this projection.  The branch weight sqrt(tau) = epi_scale in (0, 1] acts on
 * the gradient LEAVING the branch's input, not on the one entering the branch (the id* rewrite of
 * Sec. 5.3), and the skip path carries the incoming layer gradient R = Zpre (FP16 [b,m]):
 *   dX = fp16( sqrt(1 - epi_scale^2) * R + epi_scale * fp16(beta_x * G W^T) ).
 * Workspace (16-byte aligned): us_workspace_bytes(b, m, n) is the size that serves every use.  Its
 * first US_TABLE_AREA_BYTES are the table area (the table-driven GELU' epilogue gives the same results
 * as the arithmetic one and is used for large problems when the area is there; it is rebuilt by the
 * call unless epi carries US_EPI_TABLES_READY, see us_linear_fwd), the rest holds the FP32 slices of
 * the dW reduction over tokens (contents undefined on entry and exit).  A workspace is REQUIRED only
 * when dW needs slices, i.e. when us_workspace_bytes(b, m, n) > US_TABLE_AREA_BYTES: then fewer
 * bytes give US_ERR_WORKSPACE.
 */
us_status us_linear_bwd(const void* X, const void* W, const void* G, void* dX, void* dW,
                        long b, long m, long n, us_dtype x_dt, us_dtype w_dt, us_dtype g_dt,
                        us_dtype out_dt, float beta_x, float beta_w, us_epilogue epi, float epi_scale,
                        const void* Zpre, void* aux8, void* workspace, size_t workspace_bytes,
                        void* stream);

/* Bytes of workspace that serve every use by us_linear_fwd / us_linear_bwd for a [b,m] x [m,n] layer:
 * the table area plus the dW slices (0 for a non-positive dimension). */
size_t us_workspace_bytes(long b, long m, long n);

/*
 * us_linear_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace), same kernels, same
 * results bit for bit as us_linear_bwd given a workspace of us_workspace_bytes(b, m, n) bytes without
 * US_EPI_TABLES_READY (that flag is ignored here: each call rebuilds the table it uses).
 *
 * The workspace is a static device array inside the library, US_NOALLOC_SCRATCH_BYTES (16.25 MiB) on every GPU the
 * library runs on, held until the process ends.  The call allocates and frees nothing.  A shape whose grad_W needs
 * more slice memory than that (us_workspace_bytes(b, m, n) > US_NOALLOC_SCRATCH_BYTES: few output tiles and many
 * tokens, e.g. 4096 tokens into a 512 x 2048 weight) is refused with US_ERR_WORKSPACE before anything is launched;
 * use us_linear_bwd with a workspace of the caller's for those.
 *
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents; nothing in it needs to start
 * at zero (tables and slices are written completely before they are read).  Two calls whose kernels may overlap on one
 * GPU (different streams, or graphs replayed side by side) race on it: serialise them.
 */
#define US_NOALLOC_SCRATCH_BYTES (US_TABLE_AREA_BYTES + (16u << 20))
us_status us_linear_bwd_noalloc(const void* X, const void* W, const void* G, void* dX, void* dW,
                                long b, long m, long n,
                                us_dtype x_dt, us_dtype w_dt, us_dtype g_dt, us_dtype out_dt,
                                float beta_x, float beta_w, us_epilogue epi, float epi_scale,
                                const void* Zpre, void* aux8, void* stream);
size_t us_noalloc_scratch_bytes(void);

/*
 * Fill the table area of a workspace (its first US_TABLE_AREA_BYTES; workspace_bytes must be at least
 * that) with all GELU tables for the factors alpha_g / beta_g (<= 0: 1.7009 / 1.4811, Table A.2).  The
 * tables depend on nothing else, so a training loop calls this once and then passes
 * US_EPI_TABLES_READY / US_FFN_TABLES_READY; the matmul calls never write to the table area then.
 */
us_status us_gelu_tables(void* workspace, size_t workspace_bytes, float alpha_g, float beta_g, void* stream);

/*
 * Stand-alone unit-scaled GELU (Table A.2 "Activations"; backward by the f_grad rule of Sec. 5.1).
 *   fwd: h[i]  = round( alpha_g * z[i] * Phi(z[i]) )
 *   bwd: gz[i] = round( beta_g * (Phi(z[i]) + z[i]*phi(z[i])) * gh[i] )
 * dt = US_F16 or US_F32 for all arrays of a call.  alpha_g / beta_g <= 0 select 1.7009 / 1.4811.
 * In-place use (h == z, gz == gh) is allowed.
 */
us_status us_gelu_fwd(const void* z, void* h, size_t n, us_dtype dt, float alpha_g, void* stream);

us_status us_gelu_bwd(const void* z, const void* gh, void* gz, size_t n, us_dtype dt, float beta_g,
                      void* stream);

/*
 * The FFN of Fig. 3 without its residual: Linear -> unit-scaled GELU -> Linear, as one call per
 * direction, composed of the operations above with the scales of Table A.2 (alpha = fan_in^-1/2,
 * beta_x = fan_out^-1/2, beta_w = tokens^-1/2, GELU 1.7009 / 1.4811).
 *
 * mode: bit US_FFN_FP8 clear: operands are the FP16 tensors; set ("fp8" below): X8, W1_8, W2_8 are E4M3
 * and G8 is E5M2 (made by us_cast_fp8), H8 / dZ8 are written by the fused epilogues.  Bit
 * US_FFN_TABLES_READY: the workspace's table area was filled by us_gelu_tables (default factors).
 *
 * us_ffn_fwd:  Z[T,f] = fp16(d^-1/2 X W1);  H = fp16(1.7009 gelu(Z));  Y[T,d] = fp16(f^-1/2 H W2)
 *   X [T,d], W1 [d,f], W2 [f,d]: F16 (fp8 == 0) or E4M3 (fp8 != 0)
 *   Z [T,f] F16 out;  H [T,f] out: F16 when fp8 == 0, E4M3 codes when fp8 != 0;  Y [T,d] F16 out
 * us_ffn_bwd:  dH = fp16(d^-1/2 G W2^T);  dZ = fp16(1.4811 gelu'(Z) dH);  dW2 = fp16(T^-1/2 H^T G);
 *              dX = fp16(f^-1/2 dZ W1^T);  dW1 = fp16(T^-1/2 X^T dZ)
 *   G [T,d]: F16 or E5M2;  dZ16 [T,f] F16 out;  dZ8 [T,f] E5M2 out (fp8 != 0 only, else ignored).
 *   With fp8 != 0 the layer-1 matmuls read dZ8 only, so dZ16 may be NULL and is then not stored.
 *   dX [T,d], dW1 [d,f], dW2 [f,d] F16 out
 *   workspace: us_ffn_workspace_bytes(T, d, f) bytes serve both calls (optional for us_ffn_fwd, where it
 *   only enables the table-driven GELU; required for us_ffn_bwd whenever a dW needs slices).
 */
us_status us_ffn_fwd(const void* X, const void* W1, const void* W2, void* Z, void* H, void* Y,
                     long T, long d, long f, int mode, void* workspace, size_t workspace_bytes, void* stream);
us_status us_ffn_bwd(const void* X, const void* W1, const void* W2, const void* Z, const void* H,
                     const void* G, void* dZ16, void* dZ8, void* dX, void* dW1, void* dW2,
                     long T, long d, long f, int mode, void* workspace, size_t workspace_bytes,
                     void* stream);
size_t us_ffn_workspace_bytes(long T, long d, long f);

/*
 * Stand-alone unit-scaled activation, any of Table A.2's (us_activation), in the aligned form of App. H
 * "Activation functions", f_hat(x) = f(s1 x) s2:
 *   fwd: h[i]  = round( scale * f(s1 * z[i]) )             scale <= 0: the activation's alpha (s1 = 1 assumed)
 *   bwd: gz[i] = round( scale * f'(s1 * z[i]) * gh[i] )    scale <= 0: the activation's beta; relu'(0) = 0
 * s1 <= 0 selects 1.  dt = US_F16 or US_F32; in-place use is allowed.  For a given scale, kind US_ACT_GELU
 * with s1 = 1 computes what us_gelu_fwd / us_gelu_bwd compute.
 */
typedef enum { US_ACT_GELU = 0, US_ACT_RELU = 1, US_ACT_TANH = 2, US_ACT_SIGMOID = 3 } us_activation;
us_status us_act_fwd(const void* z, void* h, size_t n, us_dtype dt, us_activation kind, float s1, float scale,
                     void* stream);
us_status us_act_bwd(const void* z, const void* gh, void* gz, size_t n, us_dtype dt, us_activation kind,
                     float s1, float scale, void* stream);

/*
 * Scaled layer norm over the last dimension (Table A.2 "Other"), FP16 storage, FP32 arithmetic:
 *   fwd:  Y[i,j] = fp16( c[j] + w[j] * (X[i,j] - mu_i) * rstd_i ),  mu_i = mean_j X[i,j],
 *         rstd_i = (mean_j (X[i,j] - mu_i)^2 + eps)^-1/2            (alpha = 1; the paper's formula has eps = 0)
 *   bwd:  xh = (X - mu) rstd, gh = G * w:
 *         dX[i,j] = fp16( rstd_i * (gh[i,j] - mean_j gh[i,j] - xh[i,j] * mean_j(gh[i,j] xh[i,j])) )    (beta_x = 1)
 *         dw[j] = fp16( beta_wc * sum_i G[i,j] xh[i,j] ),  dc[j] = fp16( beta_wc * sum_i G[i,j] )
 *         beta_wc <= 0 selects b^-1/2 (Table A.2: weight and bias are cut-edges, scaled by the row count).
 * X, Y, G, dX: [b,n]; w, c, dw, dc: [n]; n a multiple of 16 and at most 4096 (a wave keeps a row in registers).
 * The backward pass recomputes the row statistics from X.  Its workspace (us_layer_norm_workspace_bytes,
 * 16-byte aligned, contents undefined on entry and exit) holds per-32-row column sums that a second kernel
 * adds in order, so the result does not depend on scheduling.
 */
us_status us_layer_norm_fwd(const void* X, const void* w, const void* c, void* Y, long b, long n, float eps,
                            void* stream);
us_status us_layer_norm_bwd(const void* X, const void* w, const void* G, void* dX, void* dw, void* dc, long b,
                            long n, float eps, float beta_wc, void* workspace, size_t workspace_bytes,
                            void* stream);
size_t us_layer_norm_workspace_bytes(long b, long n);

/*
 * Diagnostics (device memory in and out; the results are ADDED to hist / sums, which the caller clears).
 *
 * us_exponent_histogram: where a tensor's values sit on the FP16 exponent grid (the histograms of Fig. 1 and
 * App. K, with their extra bins).  src: F16 or F32, n elements; hist: US_HIST_BINS 64-bit counters:
 *   0 zero | 1 non-zero below 2^-24 | 2 FP16-subnormal range [2^-24, 2^-14) | 3 + (e + 14) for
 *   2^e <= |x| < 2^(e+1), e = -14 .. 15 | 33 |x| >= 2^16 or infinite | 34 NaN
 *
 * us_cast_snr: signal and noise of the scaled saturating cast of us_cast_fp8 (Sec. 3.1 "Quantisation error"):
 *   sums[0] += sum x^2,  sums[1] += sum (q(x*scale)/scale - x)^2   (two doubles; NaN inputs skipped; scale > 0)
 * SNR = sums[0] / sums[1].  The order of the additions is not fixed (floating-point atomics).
 */
#define US_HIST_BINS 35
us_status us_exponent_histogram(const void* src, us_dtype src_dt, size_t n, unsigned long long* hist, void* stream);
us_status us_cast_snr(const void* src, us_dtype src_dt, size_t n, us_dtype dst_dt, float scale, double* sums,
                      void* stream);

/*
 * Stand-alone weighted addition of two tensors (Table A.2 "weighted_add" with two inputs; Sec. 5.3):
 *   out[i] = round( ca * a[i] + cb * b[i] ),  dt = US_F16 or US_F32 for all three arrays; out may alias a or b.
 * The unit-scaling factor alpha = (ca^2 + cb^2)^-1/2 is the caller's to fold into ca, cb (it is 1 for the
 * interpolation weights sqrt(1-tau), sqrt(tau)).
 */
us_status us_weighted_add(const void* a, const void* b, void* out, size_t n, us_dtype dt, float ca, float cb,
                          void* stream);

/*
 * The residual FFN layer of Fig. 3 (right):  Out = sqrt(1-tau) * x + sqrt(tau) * FFN(x), 0 < tau <= 1, as
 * us_ffn_fwd / us_ffn_bwd with the interpolation fused into the second projection (forward) and into
 * grad_X of the first projection (backward).  Xskip / Gskip are the FP16 layer input / incoming
 * gradient [T,d]; X / G are the matmul operands (the same tensors when mode has no US_FFN_FP8, their
 * FP8 casts otherwise).  The branch output FFN(x) is not stored.  In the backward pass the branch
 * receives G unscaled (dZ, dW1, dW2 are those of us_ffn_bwd) and
 *   dXin = fp16( sqrt(1-tau) * Gskip + sqrt(tau) * fp16(f^-1/2 dZ W1^T) ).
 */
us_status us_ffn_res_fwd(const void* Xskip, const void* X, const void* W1, const void* W2, void* Z, void* H,
                         void* Out, long T, long d, long f, float tau, int mode, void* workspace,
                         size_t workspace_bytes, void* stream);
us_status us_ffn_res_bwd(const void* X, const void* W1, const void* W2, const void* Z, const void* H,
                         const void* Gskip, const void* G, void* dZ16, void* dZ8, void* dXin, void* dW1,
                         void* dW2, long T, long d, long f, float tau, int mode, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * Bias rows (App. J.1: ffn(z) = W2 act(W1 z + b1) + b2).  The paper gives the bias no factor of its own: biases
 * start at zero (only non-bias parameters are drawn with unit variance, Sec. 5.2), so the forward pass adds them
 * unscaled, inside the single rounding of the output, and the gradient, a sum over the b rows, gets b^-1/2 like
 * the bias of the scaled layer norm (Table A.2 "Other").
 *
 * us_linear_bias_fwd: us_linear_fwd with  Y = round( alpha * X W + bias ), the epilogue (GELU, residual) then acts on
 *   that Y.  bias: device, FP16 [n], 16-byte aligned, or NULL (then exactly us_linear_fwd).  y_dt must be US_F16
 *   when a bias is given (US_ERR_DTYPE otherwise).
 * us_bias_grad:  dc[j] = fp16( beta_c * sum_i G[i,j] ),  G [b,n] of g_dt = US_F16, US_E4M3 or US_E5M2; dc FP16 [n];
 *   n a multiple of 16 (b is free); beta_c <= 0 selects b^-1/2.  FP32 sums in a fixed order (reproducible).
 *   workspace: us_bias_grad_workspace_bytes(b, n) bytes of scratch, 16-byte aligned (US_ERR_WORKSPACE if smaller).
 * us_ffn_bias_fwd / us_ffn_bias_bwd: us_ffn_fwd / us_ffn_bwd with b1 [f], b2 [d] (either may be NULL) and their
 *   gradients db1 [f], db2 [d] (FP16 out, either may be NULL).  The bias gradients are sums of the FP16 gradients
 *   (FP8 copies exist for the matmuls only, App. J.2): db2 reads G16, the FP16 incoming gradient [T,d] (G is
 *   the matmul operand: the same tensor without US_FFN_FP8, its E5M2 cast with it; US_ERR_NULL if db2 is asked for
 *   without G16), and db1 sums the FP16 dZ inside the epilogue that produces it, so dZ16 may still be NULL with
 *   US_FFN_FP8 (the sums are the same whether or not it is stored).
 *   workspace: us_ffn_bias_workspace_bytes(T, d, f) = what us_ffn_bwd needs, rounded up to 256 bytes, plus
 *   us_bias_grad_workspace_bytes(T, max(d, f)).
 */
us_status us_linear_bias_fwd(const void* X, const void* W, const void* bias, void* Y, long b, long m, long n,
                             us_dtype x_dt, us_dtype w_dt, us_dtype y_dt, float alpha, us_epilogue epi,
                             float epi_scale, void* aux16, void* aux8, void* workspace, size_t workspace_bytes,
                             void* stream);
us_status us_bias_grad(const void* G, us_dtype g_dt, void* dc, long b, long n, float beta_c, void* workspace,
                       size_t workspace_bytes, void* stream);
size_t us_bias_grad_workspace_bytes(long b, long n);
us_status us_ffn_bias_fwd(const void* X, const void* W1, const void* b1, const void* W2, const void* b2, void* Z,
                          void* H, void* Y, long T, long d, long f, int mode, void* workspace,
                          size_t workspace_bytes, void* stream);
us_status us_ffn_bias_bwd(const void* X, const void* W1, const void* W2, const void* Z, const void* H,
                          const void* G, const void* G16, void* dZ16, void* dZ8, void* dX, void* dW1, void* dW2,
                          void* db1, void* db2, long T, long d, long f, int mode, void* workspace,
                          size_t workspace_bytes, void* stream);
size_t us_ffn_bias_workspace_bytes(long T, long d, long f);

/*
 * Scaled softmax over the last dimension (Table A.2 "Other"; App. G "Softmax (followed by matmul)"), and its
 * aligned form with an input factor s1 = 1 / temperature (App. H "Softmax functions").  X, Y, G, dX: device, FP16
 * [rows, s], 16-byte aligned, s a multiple of 8 and at most US_SOFTMAX_MAX (US_ERR_SHAPE otherwise); rows is free.
 *   fwd:  Y[i,j]  = fp16( alpha * p_ij ),  p_i = softmax(s1 * X[i,:])           alpha <= 0 selects s
 *   bwd:  dX[i,j] = fp16( beta * s1 * p_ij * (G[i,j] - sum_k p_ik G[i,k]) )     beta  <= 0 selects s
 * s1 = 0 selects 1; a negative s1 is US_ERR_VALUE.  s1 * x is not rounded before the exponential; the backward pass
 * recomputes p from X (not from the rounded Y).  A NaN or a +inf in a row makes the whole row NaN.  No masks.
 *
 * Softmax cross-entropy at the end of a model (App. G "Softmax cross-entropy": alpha = 1, beta = s / sqrt(s - 1)):
 *   loss[i] = -log softmax(s1 * X[i,:])_target[i]                (FP32 [rows], device; may be NULL)
 *   dX[i,j] = fp16( beta * s1 * (p_ij - [j == target[i]]) )      (FP16 [rows, s]; may be NULL; not both NULL)
 * target: device, int32 [rows]; a value outside 0 .. s-1 marks a row without a label: loss 0, gradient row 0.
 * s a multiple of 8 and at most US_XENT_MAX.  beta <= 0 selects s / sqrt(s - 1).
 */
#define US_SOFTMAX_MAX 4096
#define US_XENT_MAX 65536
us_status us_softmax_fwd(const void* X, void* Y, long rows, long s, float s1, float alpha, void* stream);
us_status us_softmax_bwd(const void* X, const void* G, void* dX, long rows, long s, float s1, float beta,
                         void* stream);
us_status us_softmax_xent(const void* X, const int* target, float* loss, void* dX, long rows, long s, float s1,
                          float beta, void* stream);

/*
 * A batch of equally shaped, independent scaled matmuls in one launch (the per-head products of attention):
 *   C[i] = round( scale * op(A[i]) op(B[i]) ),  i = 0 .. batch-1,  C[i] is [M,N] row-major, matrices packed one after
 *   the other.  trans_a = 0: A[i] is [M,K]; 1: A[i] is [K,M].  trans_b = 0: B[i] is [K,N]; 1: B[i] is [N,K].  Both 1 is
 *   not supported (US_ERR_SHAPE).  Operand types: F16 x F16, or the FP8 pairs of the layer products: E4M3 x E4M3
 *   (no transposition), E5M2 x E4M3 (trans_b), E4M3 x E5M2 (trans_a).  c_dt F16 or F32.  M, N, K multiples of 16,
 *   batch <= 65535, scale > 0 (US_ERR_VALUE otherwise).  FP32 accumulation over all of K in one workgroup: no workspace.
 *
 * Unit-scaled dot-product attention without mask for `heads` independent heads (batch x heads of a layer), built from
 * the call above and the scaled softmax, with the factors Table A.2 gives each op (App. F notes that the familiar
 * 1/sqrt(d) is the forward factor of the scores):
 *   fwd:  A = fp16(d^-1/2 Q K^T)   P = fp16(s * softmax(A))   O = fp16(s^-1/2 P V)
 *   bwd:  dV = fp16(s^-1/2 P^T dO)  dP = fp16(d^-1/2 dO V^T)  dA = fp16(s * p (dP - sum p dP))
 *         dQ = fp16(s^-1/2 dA K)    dK = fp16(s^-1/2 dA^T Q)
 * Q, K, V, O, dO, dQ, dK, dV: FP16 [heads, s, d]; A, P, dP, dA: FP16 [heads, s, s]; all device, 16-byte aligned; s and d
 * multiples of 16, s <= US_SOFTMAX_MAX, heads <= 65535.  A and P are stored by the forward call and read by the
 * backward call.
 */
us_status us_matmul_batched(const void* A, const void* B, void* C, long batch, long M, long N, long K, int trans_a,
                            int trans_b, us_dtype a_dt, us_dtype b_dt, us_dtype c_dt, float scale, void* stream);
us_status us_attention_fwd(const void* Q, const void* K, const void* V, void* A, void* P, void* O, long heads, long s,
                           long d, void* stream);
us_status us_attention_bwd(const void* Q, const void* K, const void* V, const void* A, const void* P, const void* dO,
                           void* dP, void* dA, void* dQ, void* dK, void* dV, long heads, long s, long d,
                           void* stream);

/*
 * Scaled sum over the last dimension (Table A.2 "Linear": sum(x), alpha = n^-1/2, beta = 1).
 *   fwd:  Y[i]    = fp16( alpha * sum_j X[i,j] )     X FP16 [rows, n] (16-byte aligned), Y FP16 [rows]; alpha <= 0: n^-1/2
 *   bwd:  dX[i,j] = fp16( beta * G[i] )              G FP16 [rows], dX FP16 [rows, n] (16-byte aligned); beta <= 0: 1
 * n a multiple of 8 (US_ERR_SHAPE otherwise); n = 0 gives Y = 0.  FP32 sum in a fixed order.
 */
us_status us_sum_fwd(const void* X, void* Y, long rows, long n, float alpha, void* stream);
us_status us_sum_bwd(const void* G, void* dX, long rows, long n, float beta, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* US_H_ */
