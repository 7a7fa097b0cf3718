// C-ABI entry points: argument checks on the host, then launches.  Nothing here allocates memory
// or synchronises with the device.
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "us_device.h"
#include "us_launch.h"

using namespace us;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool mult16(long v) { return (v & 15) == 0; }
inline bool is_fp8(us_dtype d) { return d == US_E4M3 || d == US_E5M2; }
inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline us_status from_hip(hipError_t e) { return e == hipSuccess ? US_OK : US_ERR_LAUNCH; }
// weight of the skip input of a residual interpolation whose branch weight is w (0 < w <= 1)
inline float skip_weight(float w) { return (float)sqrt(1.0 - (double)w * (double)w); }
inline bool residual_weight_ok(float w) { return w > 0.0f && w <= 1.0f; }

}  // namespace

// ---- scratch of the entry point that allocates nothing (us_linear_bwd_noalloc) -----------------------------------
// One array per GPU the library runs on, held until the process ends: the table area of the table-driven GELU'
// epilogue, then room for grad_W's FP32 K slices.  Host code never uses the array's name as an address: its device
// address is looked up once per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[US_NOALLOC_SCRATCH_BYTES];

struct ScratchAddress {
  std::once_flag once[kMaxDevices];
  hipError_t err[kMaxDevices];
  void* ptr[kMaxDevices];
  // the current device's copy of `scratch`, or NULL with *e set
  void* get(hipError_t* e) {
    int dev = 0;
    *e = hipGetDevice(&dev);
    if (*e != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *e = hipErrorInvalidDevice; return nullptr; }
    std::call_once(once[dev], [&] {
      void* p = nullptr;
      err[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      ptr[dev] = (err[dev] == hipSuccess) ? p : nullptr;
    });
    *e = err[dev];
    return ptr[dev];
  }
};
static ScratchAddress g_scratch;

extern "C" {

const char* us_last_launch(void) { return last_launch_record(); }

const char* us_status_string(us_status s) {
  switch (s) {
    case US_OK: return "ok";
    case US_ERR_NULL: return "a required pointer is NULL";
    case US_ERR_SHAPE: return "bad shape: dimensions must be non-negative multiples of 16";
    case US_ERR_ALIGN: return "pointer not 16-byte aligned";
    case US_ERR_DTYPE: return "unsupported storage-type combination";
    case US_ERR_WORKSPACE: return "workspace missing or too small";
    case US_ERR_LAUNCH: return "HIP launch failed";
    case US_ERR_VALUE: return "scalar argument outside its domain";
  }
  return "unknown status";
}

us_status us_linear_scales(long b, long m, long n, int mode, float* alpha, float* beta_x, float* beta_w) {
  if (!alpha || !beta_x || !beta_w) return US_ERR_NULL;
  if (b < 1 || m < 1 || n < 1 || (mode != 0 && mode != 1)) return US_ERR_SHAPE;
  double a = 1.0 / sqrt((double)m), bx = 1.0 / sqrt((double)n), bw = 1.0 / sqrt((double)b);
  if (mode == 1) a = bx = sqrt(a * bx);
  *alpha = (float)a;
  *beta_x = (float)bx;
  *beta_w = (float)bw;
  return US_OK;
}

us_status us_cast_fp8(const void* src, us_dtype src_dt, void* dst, us_dtype dst_dt, size_t n, float scale,
                      us_cast_stats* stats, void* stream) {
  if ((src_dt != US_F16 && src_dt != US_F32) || !is_fp8(dst_dt)) return US_ERR_DTYPE;
  if (n == 0) return US_OK;
  if (!src || !dst) return US_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst) || (reinterpret_cast<uintptr_t>(stats) & 7u)) return US_ERR_ALIGN;
  return from_hip(launch_cast(src, src_dt, dst, dst_dt, n, scale, stats, as_stream(stream)));
}

us_status us_cast_fp8_batch(int count, const void* const* src, void* const* dst, const size_t* n, const us_dtype* dst_dt,
                            void* stream) {
  if (count < 0 || count > US_CAST_BATCH_MAX) return US_ERR_SHAPE;
  if (count == 0) return US_OK;
  if (!src || !dst || !n || !dst_dt) return US_ERR_NULL;
  for (int i = 0; i < count; ++i) {
    if (!is_fp8(dst_dt[i])) return US_ERR_DTYPE;
    if (n[i] == 0) continue;
    if (!src[i] || !dst[i]) return US_ERR_NULL;
    if (!aligned16(src[i]) || !aligned16(dst[i])) return US_ERR_ALIGN;
    if (n[i] / 16 / 1024 >= 0xffffffffull / US_CAST_BATCH_MAX) return US_ERR_SHAPE;   // block index stays 32-bit
  }
  return from_hip(launch_cast_batch(count, src, dst, n, dst_dt, as_stream(stream)));
}

us_status us_gelu_fwd(const void* z, void* h, size_t n, us_dtype dt, float alpha_g, void* stream) {
  if (dt != US_F16 && dt != US_F32) return US_ERR_DTYPE;
  if (n == 0) return US_OK;
  if (!z || !h) return US_ERR_NULL;
  if (!aligned16(z) || !aligned16(h)) return US_ERR_ALIGN;
  if (!(alpha_g > 0.0f)) alpha_g = kGeluAlpha;
  return from_hip(launch_gelu_fwd(z, h, n, dt, alpha_g, as_stream(stream)));
}

us_status us_gelu_bwd(const void* z, const void* gh, void* gz, size_t n, us_dtype dt, float beta_g, void* stream) {
  if (dt != US_F16 && dt != US_F32) return US_ERR_DTYPE;
  if (n == 0) return US_OK;
  if (!z || !gh || !gz) return US_ERR_NULL;
  if (!aligned16(z) || !aligned16(gh) || !aligned16(gz)) return US_ERR_ALIGN;
  if (!(beta_g > 0.0f)) beta_g = kGeluBeta;
  return from_hip(launch_gelu_bwd(z, gh, gz, n, dt, beta_g, as_stream(stream)));
}

us_status us_gelu_tables(void* workspace, size_t workspace_bytes, float alpha_g, float beta_g, void* stream) {
  if (!workspace) return US_ERR_NULL;
  if (!aligned16(workspace)) return US_ERR_ALIGN;
  if (workspace_bytes < (size_t)kTableAreaBytes) return US_ERR_WORKSPACE;
  if (!(alpha_g > 0.0f)) alpha_g = kGeluAlpha;
  if (!(beta_g > 0.0f)) beta_g = kGeluBeta;
  char* const base = (char*)workspace;
  hipStream_t st = as_stream(stream);
  if (launch_gelu_table(base + kGeluTableOffset, alpha_g, st) != hipSuccess) return US_ERR_LAUNCH;
  if (launch_gelu_slope_table(base + kGeluSlopeTableOffset, beta_g, st) != hipSuccess) return US_ERR_LAUNCH;
  if (launch_gelu_half_table(base + kGeluHalfTableOffset, alpha_g, st) != hipSuccess) return US_ERR_LAUNCH;
  return US_OK;
}

size_t us_workspace_bytes(long b, long m, long n) {
  if (b < 1 || m < 1 || n < 1) return 0;
  return (size_t)kTableAreaBytes + gemm_workspace_bytes(m, n, b);
}

// us_linear_bias_fwd.  launch = false: the argument checks only (what a composite call runs for every one of its
// products before it enqueues the first, so that a call that fails has touched no device memory).
static us_status linear_fwd_impl(const void* X, const void* W, const void* bias, void* Y, long b, long m, long n, us_dtype x_dt,
                                 us_dtype w_dt, us_dtype y_dt, float alpha, us_epilogue epi, float epi_scale, void* aux16,
                                 void* aux8, void* workspace, size_t workspace_bytes, void* stream, bool launch) {
  const bool tables_ready = ((int)epi & US_EPI_TABLES_READY) != 0;
  const int act = ((int)epi >> 4) & 0xf;
  epi = (us_epilogue)((int)epi & 0xf);
  if (act > 3 || (act != 0 && epi != US_EPI_GELU && epi != US_EPI_GELU_GRAD)) return US_ERR_DTYPE;
  const bool f16 = (x_dt == US_F16 && w_dt == US_F16);
  const bool fp8 = (x_dt == US_E4M3 && w_dt == US_E4M3);
  if (!f16 && !fp8) return US_ERR_DTYPE;
  if (y_dt != US_F16 && y_dt != US_F32) return US_ERR_DTYPE;
  if (epi != US_EPI_NONE && epi != US_EPI_GELU && epi != US_EPI_RESIDUAL) return US_ERR_DTYPE;
  if (epi != US_EPI_NONE && y_dt != US_F16) return US_ERR_DTYPE;
  if (bias && y_dt != US_F16) return US_ERR_DTYPE;       // the bias joins the sum before the rounding to FP16
  if (epi == US_EPI_RESIDUAL && !residual_weight_ok(epi_scale)) return US_ERR_VALUE;
  if (b < 0 || m < 0 || n < 0 || !mult16(b) || !mult16(m) || !mult16(n)) return US_ERR_SHAPE;
  if (b == 0 || n == 0) return US_OK;
  if (!Y || (m > 0 && (!X || !W))) return US_ERR_NULL;
  if (epi == US_EPI_GELU && !aux16 && !aux8) return US_ERR_NULL;
  if (epi == US_EPI_RESIDUAL && !aux16) return US_ERR_NULL;
  if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || !aligned16(aux16) || !aligned16(aux8) || !aligned16(workspace) ||
      !aligned16(bias))
    return US_ERR_ALIGN;
  GemmProblem p{};
  p.bias = bias;
  p.A = X; p.B = W; p.C = Y;
  p.M = b; p.N = n; p.K = m;
  p.lda = m; p.ldb = n; p.ldc = n;
  p.a_kc = true; p.b_kc = false;
  p.a_dt = x_dt; p.b_dt = w_dt; p.c_dt = y_dt;
  p.scale = (alpha > 0.0f) ? alpha : (float)(1.0 / sqrt((double)(m > 0 ? m : 1)));
  p.epi = epi;
  p.epi_scale = (epi_scale > 0.0f) ? epi_scale : kActAlpha[act];
  p.act = act;
  if (epi == US_EPI_RESIDUAL) {
    p.skip_scale = skip_weight(epi_scale);
    p.Zpre = aux16;                                    // the skip input
  }
  p.aux16 = (epi == US_EPI_GELU) ? aux16 : nullptr;
  p.aux8 = (epi == US_EPI_GELU) ? aux8 : nullptr;
  p.table = (workspace && workspace_bytes >= (size_t)kTableAreaBytes) ? workspace : nullptr;
  p.tables_ready = tables_ready;
  if (!launch) return US_OK;
  return from_hip(launch_gemm(p, as_stream(stream)));
}

us_status us_linear_fwd(const void* X, const void* W, void* Y, long b, long m, long n, us_dtype x_dt, us_dtype w_dt,
                        us_dtype y_dt, float alpha, us_epilogue epi, float epi_scale, void* aux16, void* aux8,
                        void* workspace, size_t workspace_bytes, void* stream) {
  begin_launch_record();
  return linear_fwd_impl(X, W, nullptr, Y, b, m, n, x_dt, w_dt, y_dt, alpha, epi, epi_scale, aux16, aux8, workspace,
                         workspace_bytes, stream, true);
}

us_status us_linear_bias_fwd(const void* X, const void* W, const void* bias, void* Y, long b, long m, long n, us_dtype x_dt,
                             us_dtype w_dt, us_dtype y_dt, float alpha, us_epilogue epi, float epi_scale, void* aux16,
                             void* aux8, void* workspace, size_t workspace_bytes, void* stream) {
  begin_launch_record();
  return linear_fwd_impl(X, W, bias, Y, b, m, n, x_dt, w_dt, y_dt, alpha, epi, epi_scale, aux16, aux8, workspace,
                         workspace_bytes, stream, true);
}

// us_linear_bwd plus one internal option: colsum, FP32 [ceil(b / 32)][m], receives the column sums of the FP16 result of
// the GELU' epilogue per 32-row block (the bias gradient of the layer, before its sum over the blocks), whether or not
// that FP16 result is stored.
static us_status linear_bwd_impl(const void* X, const void* W, const void* G, void* dX, void* dW, long b, long m, long n,
                                 us_dtype x_dt, us_dtype w_dt, us_dtype g_dt, us_dtype out_dt, float beta_x, float beta_w,
                                 us_epilogue epi, float epi_scale, const void* Zpre, void* aux8, void* workspace,
                                 size_t workspace_bytes, void* stream, void* colsum, bool launch = true) {
  const bool tables_ready = ((int)epi & US_EPI_TABLES_READY) != 0;
  const int act = ((int)epi >> 4) & 0xf;
  epi = (us_epilogue)((int)epi & 0xf);
  if (act > 3 || (act != 0 && epi != US_EPI_GELU && epi != US_EPI_GELU_GRAD)) return US_ERR_DTYPE;
  const bool f16 = (x_dt == US_F16 && w_dt == US_F16 && g_dt == US_F16);
  const bool fp8 = (x_dt == US_E4M3 && w_dt == US_E4M3 && g_dt == US_E5M2);
  if (!f16 && !fp8) return US_ERR_DTYPE;
  if (out_dt != US_F16 && out_dt != US_F32) return US_ERR_DTYPE;
  if (epi != US_EPI_NONE && epi != US_EPI_GELU_GRAD && epi != US_EPI_RESIDUAL) return US_ERR_DTYPE;
  if (epi != US_EPI_NONE && out_dt != US_F16) return US_ERR_DTYPE;
  if (epi == US_EPI_RESIDUAL && !residual_weight_ok(epi_scale)) return US_ERR_VALUE;
  if (b < 0 || m < 0 || n < 0 || !mult16(b) || !mult16(m) || !mult16(n)) return US_ERR_SHAPE;
  // with the GELU' epilogue the FP16 result is optional: its E5M2 copy alone may be asked for
  const bool do_dx = (dX || (epi == US_EPI_GELU_GRAD && (aux8 || colsum))) && b > 0 && m > 0;
  const bool do_dw = dW && m > 0 && n > 0;
  if (!do_dx && !do_dw) return US_OK;
  if (do_dx && n > 0 && (!G || !W)) return US_ERR_NULL;
  if (do_dw && b > 0 && (!G || !X)) return US_ERR_NULL;
  if (do_dx && epi != US_EPI_NONE && !Zpre) return US_ERR_NULL;
  if (epi == US_EPI_RESIDUAL && do_dx && !dX) return US_ERR_NULL;
  if (!aligned16(X) || !aligned16(W) || !aligned16(G) || !aligned16(dX) || !aligned16(dW) || !aligned16(Zpre) ||
      !aligned16(aux8) || !aligned16(workspace))
    return US_ERR_ALIGN;
  // workspace layout: table area of the table-driven epilogues, then the dW slices
  const size_t slices = do_dw ? gemm_workspace_bytes(m, n, b) : 0;
  if (slices > 0 && (!workspace || workspace_bytes < (size_t)kTableAreaBytes + slices)) return US_ERR_WORKSPACE;
  void* const table = (workspace && workspace_bytes >= (size_t)kTableAreaBytes) ? workspace : nullptr;
  hipStream_t st = as_stream(stream);
  GemmProblem pdx{}, pdw{};
  if (do_dx) {
    GemmProblem& p = pdx;
    p.A = G; p.B = W; p.C = dX;
    p.M = b; p.N = m; p.K = n;
    p.lda = n; p.ldb = n; p.ldc = m;
    p.a_kc = true; p.b_kc = true;
    p.a_dt = g_dt; p.b_dt = w_dt; p.c_dt = out_dt;
    p.scale = (beta_x > 0.0f) ? beta_x : (float)(1.0 / sqrt((double)(n > 0 ? n : 1)));
    p.epi = epi;
    p.epi_scale = (epi_scale > 0.0f) ? epi_scale : kActBeta[act];
    p.act = act;
    p.Zpre = (epi != US_EPI_NONE) ? Zpre : nullptr;
    p.skip_scale = (epi == US_EPI_RESIDUAL) ? skip_weight(epi_scale) : 0.0f;
    p.aux8 = (epi == US_EPI_GELU_GRAD) ? aux8 : nullptr;
    p.colsum = (epi == US_EPI_GELU_GRAD) ? colsum : nullptr;
    p.table = table;
    p.tables_ready = tables_ready;
  }
  if (do_dw) {
    GemmProblem& p = pdw;
    p.A = X; p.B = G; p.C = dW;
    p.M = m; p.N = n; p.K = b;
    p.lda = m; p.ldb = n; p.ldc = n;
    p.a_kc = false; p.b_kc = false;
    p.a_dt = x_dt; p.b_dt = g_dt; p.c_dt = out_dt;
    p.scale = (beta_w > 0.0f) ? beta_w : (float)(1.0 / sqrt((double)(b > 0 ? b : 1)));
    p.epi = US_EPI_NONE;
    p.workspace = slices > 0 ? (void*)((char*)workspace + kTableAreaBytes) : nullptr;
    p.workspace_bytes = slices;
  }
  if (!launch) return US_OK;       // (launch = false: the argument checks only, see linear_fwd_impl)
  if (do_dx && do_dw && gemm_pair_applicable(pdx, pdw)) return from_hip(launch_gemm_pair(pdx, pdw, st));
  if (do_dx && launch_gemm(pdx, st) != hipSuccess) return US_ERR_LAUNCH;
  if (do_dw && launch_gemm(pdw, st) != hipSuccess) return US_ERR_LAUNCH;
  return US_OK;
}

us_status us_linear_bwd(const void* X, const void* W, const void* G, void* dX, void* dW, long b, long m, long n,
                        us_dtype x_dt, us_dtype w_dt, us_dtype g_dt, us_dtype out_dt, float beta_x, float beta_w,
                        us_epilogue epi, float epi_scale, const void* Zpre, void* aux8, void* workspace,
                        size_t workspace_bytes, void* stream) {
  begin_launch_record();
  return linear_bwd_impl(X, W, G, dX, dW, b, m, n, x_dt, w_dt, g_dt, out_dt, beta_x, beta_w, epi, epi_scale, Zpre, aux8,
                         workspace, workspace_bytes, stream, nullptr);
}

size_t us_noalloc_scratch_bytes(void) { return (size_t)US_NOALLOC_SCRATCH_BYTES; }

us_status us_linear_bwd_noalloc(const void* X, const void* W, const void* G, void* dX, void* dW, long b, long m, long n,
                                us_dtype x_dt, us_dtype w_dt, us_dtype g_dt, us_dtype out_dt, float beta_x, float beta_w,
                                us_epilogue epi, float epi_scale, const void* Zpre, void* aux8, void* stream) {
  begin_launch_record();
  // the tables in the scratch belong to whichever call used it last: every call rebuilds the one it needs
  epi = (us_epilogue)((int)epi & ~US_EPI_TABLES_READY);
  // what us_linear_bwd would want as workspace for this shape must fit the static array (decided on the host, before
  // any device call)
  const size_t need = (b > 0 && m > 0 && n > 0) ? us_workspace_bytes(b, m, n) : 0;
  if (need > (size_t)US_NOALLOC_SCRATCH_BYTES) return US_ERR_WORKSPACE;
  // a placeholder address stands in for the scratch while the arguments are checked: nothing is looked up or launched
  // for a call that fails
  us_status s = linear_bwd_impl(X, W, G, dX, dW, b, m, n, x_dt, w_dt, g_dt, out_dt, beta_x, beta_w, epi, epi_scale, Zpre, aux8,
                                reinterpret_cast<void*>(uintptr_t{256}), (size_t)US_NOALLOC_SCRATCH_BYTES, stream, nullptr, false);
  if (s != US_OK) return s;
  if (b <= 0 || m <= 0 || n <= 0) {      // degenerate shapes: nothing reads the scratch
    return linear_bwd_impl(X, W, G, dX, dW, b, m, n, x_dt, w_dt, g_dt, out_dt, beta_x, beta_w, epi, epi_scale, Zpre, aux8, nullptr,
                           0, stream, nullptr, true);
  }
  hipError_t e = hipSuccess;
  void* const ws = g_scratch.get(&e);
  if (!ws) return US_ERR_LAUNCH;
  return linear_bwd_impl(X, W, G, dX, dW, b, m, n, x_dt, w_dt, g_dt, out_dt, beta_x, beta_w, epi, epi_scale, Zpre, aux8, ws,
                         (size_t)US_NOALLOC_SCRATCH_BYTES, stream, nullptr, true);
}

us_status us_act_fwd(const void* z, void* h, size_t n, us_dtype dt, us_activation kind, float s1, float scale, void* stream) {
  if ((dt != US_F16 && dt != US_F32) || (int)kind < 0 || (int)kind > 3) return US_ERR_DTYPE;
  if (n == 0) return US_OK;
  if (!z || !h) return US_ERR_NULL;
  if (!aligned16(z) || !aligned16(h)) return US_ERR_ALIGN;
  return from_hip(launch_act(z, nullptr, h, n, dt, (int)kind, false, s1 > 0.0f ? s1 : 1.0f, scale > 0.0f ? scale : kActAlpha[kind],
                             as_stream(stream)));
}

us_status us_act_bwd(const void* z, const void* gh, void* gz, size_t n, us_dtype dt, us_activation kind, float s1, float scale,
                     void* stream) {
  if ((dt != US_F16 && dt != US_F32) || (int)kind < 0 || (int)kind > 3) return US_ERR_DTYPE;
  if (n == 0) return US_OK;
  if (!z || !gh || !gz) return US_ERR_NULL;
  if (!aligned16(z) || !aligned16(gh) || !aligned16(gz)) return US_ERR_ALIGN;
  return from_hip(launch_act(z, gh, gz, n, dt, (int)kind, true, s1 > 0.0f ? s1 : 1.0f, scale > 0.0f ? scale : kActBeta[kind],
                             as_stream(stream)));
}

us_status us_layer_norm_fwd(const void* X, const void* w, const void* c, void* Y, long b, long n, float eps, void* stream) {
  if (b < 0 || n < 0 || !mult16(n) || n > 4096) return US_ERR_SHAPE;
  if (!(eps >= 0.0f)) return US_ERR_VALUE;
  if (b == 0 || n == 0) return US_OK;
  if (!X || !w || !c || !Y) return US_ERR_NULL;
  if (!aligned16(X) || !aligned16(w) || !aligned16(c) || !aligned16(Y)) return US_ERR_ALIGN;
  return from_hip(launch_layer_norm_fwd(X, w, c, Y, b, n, eps, as_stream(stream)));
}

size_t us_layer_norm_workspace_bytes(long b, long n) { return (b < 1 || n < 1) ? 0 : layer_norm_workspace_bytes(b, n); }

us_status us_layer_norm_bwd(const void* X, const void* w, const void* G, void* dX, void* dw, void* dc, long b, long n, float eps,
                            float beta_wc, void* workspace, size_t workspace_bytes, void* stream) {
  if (b < 0 || n < 0 || !mult16(n) || n > 4096) return US_ERR_SHAPE;
  if (!(eps >= 0.0f)) return US_ERR_VALUE;
  if (b == 0 || n == 0) return US_OK;
  if (!X || !w || !G || !dX || !dw || !dc) return US_ERR_NULL;
  if (!aligned16(X) || !aligned16(w) || !aligned16(G) || !aligned16(dX) || !aligned16(dw) || !aligned16(dc) || !aligned16(workspace))
    return US_ERR_ALIGN;
  if (!workspace || workspace_bytes < layer_norm_workspace_bytes(b, n)) return US_ERR_WORKSPACE;
  if (!(beta_wc > 0.0f)) beta_wc = (float)(1.0 / sqrt((double)b));
  return from_hip(launch_layer_norm_bwd(X, w, G, dX, dw, dc, b, n, eps, beta_wc, workspace, as_stream(stream)));
}

us_status us_exponent_histogram(const void* src, us_dtype src_dt, size_t n, unsigned long long* hist, void* stream) {
  if (src_dt != US_F16 && src_dt != US_F32) return US_ERR_DTYPE;
  if (!hist) return US_ERR_NULL;
  if (n == 0) return US_OK;
  if (!src) return US_ERR_NULL;
  if (!aligned16(src) || (reinterpret_cast<uintptr_t>(hist) & 7u)) return US_ERR_ALIGN;
  return from_hip(launch_exponent_histogram(src, src_dt, n, hist, as_stream(stream)));
}

us_status us_cast_snr(const void* src, us_dtype src_dt, size_t n, us_dtype dst_dt, float scale, double* sums, void* stream) {
  if ((src_dt != US_F16 && src_dt != US_F32) || !is_fp8(dst_dt)) return US_ERR_DTYPE;
  if (!(scale > 0.0f)) return US_ERR_VALUE;
  if (!sums) return US_ERR_NULL;
  if (n == 0) return US_OK;
  if (!src) return US_ERR_NULL;
  if (!aligned16(src) || (reinterpret_cast<uintptr_t>(sums) & 7u)) return US_ERR_ALIGN;
  return from_hip(launch_cast_snr(src, src_dt, n, dst_dt, scale, sums, as_stream(stream)));
}

us_status us_weighted_add(const void* a, const void* b, void* out, size_t n, us_dtype dt, float ca, float cb, void* stream) {
  if (dt != US_F16 && dt != US_F32) return US_ERR_DTYPE;
  if (n == 0) return US_OK;
  if (!a || !b || !out) return US_ERR_NULL;
  if (!aligned16(a) || !aligned16(b) || !aligned16(out)) return US_ERR_ALIGN;
  return from_hip(launch_weighted_add(a, b, out, n, dt, ca, cb, as_stream(stream)));
}

us_status us_ffn_res_fwd(const void* Xskip, const void* X, const void* W1, const void* W2, void* Z, void* H, void* Out,
                         long T, long d, long f, float tau, int mode, void* workspace, size_t workspace_bytes, void* stream) {
  begin_launch_record();
  if (!(tau > 0.0f && tau <= 1.0f)) return US_ERR_VALUE;
  const bool fp8 = (mode & US_FFN_FP8) != 0;
  const int ready = (mode & US_FFN_TABLES_READY) ? US_EPI_TABLES_READY : 0;
  const us_dtype op = fp8 ? US_E4M3 : US_F16;
  // both products are checked before the first is enqueued (pass 0), then launched (pass 1)
  for (int pass = 0; pass < 2; ++pass) {
    const bool go = pass == 1;
    us_status s = linear_fwd_impl(X, W1, nullptr, Z, T, d, f, op, op, US_F16, 0.0f, (us_epilogue)(US_EPI_GELU | ready), 0.0f,
                                  fp8 ? nullptr : H, fp8 ? H : nullptr, workspace, workspace_bytes, stream, go);
    if (s != US_OK) return s;
    // layer 2 with the interpolation fused: Out = sqrt(1-tau) Xskip + sqrt(tau) fp16(f^-1/2 H W2)
    s = linear_fwd_impl(H, W2, nullptr, Out, T, f, d, op, op, US_F16, 0.0f, US_EPI_RESIDUAL, (float)sqrt((double)tau),
                        const_cast<void*>(Xskip), nullptr, nullptr, 0, stream, go);
    if (s != US_OK) return s;
  }
  return US_OK;
}

us_status us_ffn_res_bwd(const void* X, const void* W1, const void* W2, const void* Z, const void* H, const void* Gskip,
                         const void* G, void* dZ16, void* dZ8, void* dXin, void* dW1, void* dW2, long T, long d, long f,
                         float tau, int mode, void* workspace, size_t workspace_bytes, void* stream) {
  begin_launch_record();
  if (!(tau > 0.0f && tau <= 1.0f)) return US_ERR_VALUE;
  const bool fp8 = (mode & US_FFN_FP8) != 0;
  const int ready = (mode & US_FFN_TABLES_READY) ? US_EPI_TABLES_READY : 0;
  const us_dtype op = fp8 ? US_E4M3 : US_F16;
  const us_dtype gr = fp8 ? US_E5M2 : US_F16;
  if (fp8 ? !dZ8 : !dZ16) return US_ERR_NULL;
  const void* dZ = fp8 ? dZ8 : dZ16;
  for (int pass = 0; pass < 2; ++pass) {
    const bool go = pass == 1;
    // the branch sees the incoming gradient unscaled: layer 2 backward exactly as in us_ffn_bwd
    us_status s = linear_bwd_impl(H, W2, G, dZ16, dW2, T, f, d, op, op, gr, US_F16, 0.0f, 0.0f,
                                  (us_epilogue)(US_EPI_GELU_GRAD | ready), 0.0f, Z, fp8 ? dZ8 : nullptr, workspace, workspace_bytes,
                                  stream, nullptr, go);
    if (s != US_OK) return s;
    // layer 1 backward; grad_X leaves the branch through the interpolation with the skip path's gradient
    s = linear_bwd_impl(X, W1, dZ, dXin, dW1, T, d, f, op, op, gr, US_F16, 0.0f, 0.0f, US_EPI_RESIDUAL, (float)sqrt((double)tau),
                        Gskip, nullptr, workspace, workspace_bytes, stream, nullptr, go);
    if (s != US_OK) return s;
  }
  return US_OK;
}

size_t us_ffn_workspace_bytes(long T, long d, long f) {
  const size_t a = us_workspace_bytes(T, f, d);  // dW2: H[T,f]^T G[T,d]
  const size_t b = us_workspace_bytes(T, d, f);  // dW1: X[T,d]^T dZ[T,f]
  return a > b ? a : b;
}

us_status us_ffn_fwd(const void* X, const void* W1, const void* W2, void* Z, void* H, void* Y, long T, long d, long f,
                     int mode, void* workspace, size_t workspace_bytes, void* stream) {
  return us_ffn_bias_fwd(X, W1, nullptr, W2, nullptr, Z, H, Y, T, d, f, mode, workspace, workspace_bytes, stream);
}

us_status us_ffn_bias_fwd(const void* X, const void* W1, const void* b1, const void* W2, const void* b2, void* Z, void* H,
                          void* Y, long T, long d, long f, int mode, void* workspace, size_t workspace_bytes, void* stream) {
  begin_launch_record();
  const bool fp8 = (mode & US_FFN_FP8) != 0;
  const int ready = (mode & US_FFN_TABLES_READY) ? US_EPI_TABLES_READY : 0;
  const us_dtype op = fp8 ? US_E4M3 : US_F16;
  for (int pass = 0; pass < 2; ++pass) {      // pass 0 checks both products, pass 1 launches them
    const bool go = pass == 1;
    // layer 1 with the GELU fused: Z = d^-1/2 X W1 (FP16), H = 1.7009 gelu(Z) as FP16 or as E4M3 codes
    us_status s = linear_fwd_impl(X, W1, b1, Z, T, d, f, op, op, US_F16, 0.0f, (us_epilogue)(US_EPI_GELU | ready), 0.0f,
                                  fp8 ? nullptr : H, fp8 ? H : nullptr, workspace, workspace_bytes, stream, go);
    if (s != US_OK) return s;
    // layer 2: Y = f^-1/2 H W2 (+ b2)
    s = linear_fwd_impl(H, W2, b2, Y, T, f, d, op, op, US_F16, 0.0f, US_EPI_NONE, 0.0f, nullptr, nullptr, nullptr, 0, stream, go);
    if (s != US_OK) return s;
  }
  return US_OK;
}

// us_ffn_bwd; dz_colsum as in linear_bwd_impl (column sums of dZ per 32-row block, FP32 [ceil(T / 32)][f]) or NULL;
// launch = false: the argument checks of both layers only
static us_status ffn_bwd_impl(const void* X, const void* W1, const void* W2, const void* Z, const void* H, const void* G,
                              void* dZ16, void* dZ8, void* dX, void* dW1, void* dW2, long T, long d, long f, int mode,
                              void* workspace, size_t workspace_bytes, void* stream, void* dz_colsum, bool launch) {
  const bool fp8 = (mode & US_FFN_FP8) != 0;
  const int ready = (mode & US_FFN_TABLES_READY) ? US_EPI_TABLES_READY : 0;
  const us_dtype op = fp8 ? US_E4M3 : US_F16;
  const us_dtype gr = fp8 ? US_E5M2 : US_F16;
  if (fp8 ? !dZ8 : !dZ16) return US_ERR_NULL;
  const void* dZ = fp8 ? dZ8 : dZ16;
  for (int pass = 0; pass < (launch ? 2 : 1); ++pass) {
    const bool go = pass == 1;
    // layer 2 backward: dH = d^-1/2 G W2^T, fused with GELU' -> dZ (FP16 + E5M2 copy); dW2 = T^-1/2 H^T G
    us_status s = linear_bwd_impl(H, W2, G, dZ16, dW2, T, f, d, op, op, gr, US_F16, 0.0f, 0.0f,
                                  (us_epilogue)(US_EPI_GELU_GRAD | ready), 0.0f, Z,
                                  fp8 ? dZ8 : nullptr, workspace, workspace_bytes, stream, dz_colsum, go);
    if (s != US_OK) return s;
    // layer 1 backward: dX = f^-1/2 dZ W1^T; dW1 = T^-1/2 X^T dZ
    s = linear_bwd_impl(X, W1, dZ, dX, dW1, T, d, f, op, op, gr, US_F16, 0.0f, 0.0f, US_EPI_NONE, 0.0f, nullptr, nullptr,
                        workspace, workspace_bytes, stream, nullptr, go);
    if (s != US_OK) return s;
  }
  return US_OK;
}

us_status us_ffn_bwd(const void* X, const void* W1, const void* W2, const void* Z, const void* H, const void* G,
                     void* dZ16, void* dZ8, void* dX, void* dW1, void* dW2, long T, long d, long f, int mode,
                     void* workspace, size_t workspace_bytes, void* stream) {
  begin_launch_record();
  return ffn_bwd_impl(X, W1, W2, Z, H, G, dZ16, dZ8, dX, dW1, dW2, T, d, f, mode, workspace, workspace_bytes, stream, nullptr,
                      true);
}

static us_status bias_grad_impl(const void* G, us_dtype g_dt, void* dc, long b, long n, float beta_c, void* workspace,
                                size_t workspace_bytes, void* stream, bool launch) {
  if (g_dt != US_F16 && g_dt != US_E4M3 && g_dt != US_E5M2) return US_ERR_DTYPE;
  if (b < 0 || n < 0 || !mult16(n)) return US_ERR_SHAPE;
  if (n == 0) return US_OK;
  if (!dc || (b > 0 && !G)) return US_ERR_NULL;
  if (!aligned16(G) || !aligned16(dc) || !aligned16(workspace)) return US_ERR_ALIGN;
  if (b > 0 && (!workspace || workspace_bytes < bias_grad_workspace_bytes(b, n))) return US_ERR_WORKSPACE;
  if (!launch) return US_OK;
  const float beta = (beta_c > 0.0f) ? beta_c : (float)(1.0 / sqrt((double)(b > 0 ? b : 1)));
  return from_hip(launch_bias_grad(G, g_dt, dc, b, n, beta, workspace, as_stream(stream)));
}

us_status us_bias_grad(const void* G, us_dtype g_dt, void* dc, long b, long n, float beta_c, void* workspace,
                       size_t workspace_bytes, void* stream) {
  return bias_grad_impl(G, g_dt, dc, b, n, beta_c, workspace, workspace_bytes, stream, true);
}

size_t us_bias_grad_workspace_bytes(long b, long n) { return bias_grad_workspace_bytes(b, n); }

us_status us_ffn_bias_bwd(const void* X, const void* W1, const void* W2, const void* Z, const void* H, const void* G,
                          const void* G16, void* dZ16, void* dZ8, void* dX, void* dW1, void* dW2, void* db1, void* db2,
                          long T, long d, long f, int mode, void* workspace, size_t workspace_bytes, void* stream) {
  begin_launch_record();
  // the bias gradients are sums of the FP16 gradients (the FP8 copies feed the matmuls only)
  if (db2 && !G16) return US_ERR_NULL;
  if ((mode & US_FFN_FP8) ? !dZ8 : !dZ16) return US_ERR_NULL;     // the operand of the layer-1 products
  if (T < 0 || d < 0 || f < 0) return US_ERR_SHAPE;
  if (!aligned16(db1) || !aligned16(db2)) return US_ERR_ALIGN;
  // workspace: what us_ffn_bwd uses (tables, grad_W slices), then the area of the column sums
  const size_t base = (us_ffn_workspace_bytes(T, d, f) + 255) & ~(size_t)255;
  char* scratch = workspace ? (char*)workspace + base : nullptr;
  if ((db1 || db2) && T > 0) {
    if (!workspace || workspace_bytes < us_ffn_bias_workspace_bytes(T, d, f)) return US_ERR_WORKSPACE;
  }
  const size_t scratch_bytes = workspace_bytes > base ? workspace_bytes - base : 0;
  // db1: the epilogue that produces dZ adds up its columns per 32-row block on the way (whether or not the FP16 dZ is
  // stored), the sum over the blocks follows the matmuls
  const bool fused = db1 && T > 0 && f > 0;
  // every argument of every step is checked before the first launch
  us_status s = US_OK;
  if (db2) {
    s = bias_grad_impl(G16, US_F16, db2, T, d, 0.0f, scratch, scratch_bytes, stream, false);
    if (s != US_OK) return s;
  }
  s = ffn_bwd_impl(X, W1, W2, Z, H, G, dZ16, dZ8, dX, dW1, dW2, T, d, f, mode, workspace, workspace_bytes, stream,
                   fused ? scratch : nullptr, false);
  if (s != US_OK) return s;
  if (db2) {     // first: the area is free until the matmul below fills it
    s = bias_grad_impl(G16, US_F16, db2, T, d, 0.0f, scratch, scratch_bytes, stream, true);
    if (s != US_OK) return s;
  }
  s = ffn_bwd_impl(X, W1, W2, Z, H, G, dZ16, dZ8, dX, dW1, dW2, T, d, f, mode, workspace, workspace_bytes, stream,
                   fused ? scratch : nullptr, true);
  if (s != US_OK) return s;
  if (db1 && f > 0) {
    const float beta = (float)(1.0 / sqrt((double)(T > 0 ? T : 1)));
    s = from_hip(launch_bias_grad_reduce(scratch, db1, T > 0 ? (T + 31) / 32 : 0, f, beta, as_stream(stream)));
  }
  return s;
}

size_t us_ffn_bias_workspace_bytes(long T, long d, long f) {
  const size_t base = (us_ffn_workspace_bytes(T, d, f) + 255) & ~(size_t)255;
  return base + bias_grad_workspace_bytes(T, f > d ? f : d);
}

us_status us_softmax_fwd(const void* X, void* Y, long rows, long s, float s1, float alpha, void* stream) {
  if (rows < 0 || s < 0 || s % 8 != 0 || s > US_SOFTMAX_MAX) return US_ERR_SHAPE;
  if (rows == 0 || s == 0) return US_OK;
  if (!X || !Y) return US_ERR_NULL;
  if (!aligned16(X) || !aligned16(Y)) return US_ERR_ALIGN;
  if (s1 < 0.0f) return US_ERR_VALUE;
  return from_hip(launch_softmax_fwd(X, Y, rows, s, s1 > 0.0f ? s1 : 1.0f, alpha > 0.0f ? alpha : (float)s, as_stream(stream)));
}

us_status us_softmax_bwd(const void* X, const void* G, void* dX, long rows, long s, float s1, float beta, void* stream) {
  if (rows < 0 || s < 0 || s % 8 != 0 || s > US_SOFTMAX_MAX) return US_ERR_SHAPE;
  if (rows == 0 || s == 0) return US_OK;
  if (!X || !G || !dX) return US_ERR_NULL;
  if (!aligned16(X) || !aligned16(G) || !aligned16(dX)) return US_ERR_ALIGN;
  if (s1 < 0.0f) return US_ERR_VALUE;
  return from_hip(launch_softmax_bwd(X, G, dX, rows, s, s1 > 0.0f ? s1 : 1.0f, beta > 0.0f ? beta : (float)s, as_stream(stream)));
}

us_status us_softmax_xent(const void* X, const int* target, float* loss, void* dX, long rows, long s, float s1, float beta,
                          void* stream) {
  if (rows < 0 || s < 0 || s % 8 != 0 || s > US_XENT_MAX) return US_ERR_SHAPE;
  if (rows == 0 || s == 0) return US_OK;
  if (!X || !target || (!loss && !dX)) return US_ERR_NULL;
  if (!aligned16(X) || !aligned16(dX) || ((uintptr_t)target & 3) || ((uintptr_t)loss & 3)) return US_ERR_ALIGN;
  if (s1 < 0.0f) return US_ERR_VALUE;
  const float b = beta > 0.0f ? beta : (float)((double)s / sqrt((double)(s > 1 ? s - 1 : 1)));
  return from_hip(launch_softmax_xent(X, target, loss, dX, rows, s, s1 > 0.0f ? s1 : 1.0f, b, as_stream(stream)));
}

static us_status matmul_batched_impl(const void* A, const void* B, void* C, long batch, long M, long N, long K, int trans_a,
                                     int trans_b, us_dtype a_dt, us_dtype b_dt, us_dtype c_dt, float scale, void* stream) {
  if ((trans_a != 0 && trans_a != 1) || (trans_b != 0 && trans_b != 1) || (trans_a && trans_b)) return US_ERR_SHAPE;
  const bool f16 = (a_dt == US_F16 && b_dt == US_F16);
  // the FP8 pairs are those of the three layer products: forward E4M3 x E4M3, grad_X E5M2 x E4M3, grad_W E4M3 x E5M2
  const bool fp8 = !trans_a && !trans_b ? (a_dt == US_E4M3 && b_dt == US_E4M3)
                   : trans_b            ? (a_dt == US_E5M2 && b_dt == US_E4M3)
                                        : (a_dt == US_E4M3 && b_dt == US_E5M2);
  if (!f16 && !fp8) return US_ERR_DTYPE;
  if (c_dt != US_F16 && c_dt != US_F32) return US_ERR_DTYPE;
  if (batch < 0 || batch > 65535 || M < 0 || N < 0 || K < 0 || !mult16(M) || !mult16(N) || !mult16(K)) return US_ERR_SHAPE;
  if (batch == 0 || M == 0 || N == 0) return US_OK;
  if (!C || (K > 0 && (!A || !B))) return US_ERR_NULL;
  if (!aligned16(A) || !aligned16(B) || !aligned16(C)) return US_ERR_ALIGN;
  if (!(scale > 0.0f)) return US_ERR_VALUE;
  GemmProblem p{};
  p.A = A; p.B = B; p.C = C;
  p.M = M; p.N = N; p.K = K;
  p.a_kc = !trans_a;                 // A [M,K] as stored, or [K,M]
  p.b_kc = trans_b != 0;             // B [N,K] when transposed, else [K,N]
  p.lda = p.a_kc ? K : M;
  p.ldb = p.b_kc ? K : N;
  p.ldc = N;
  p.a_dt = a_dt; p.b_dt = b_dt; p.c_dt = c_dt;
  p.scale = scale;
  p.epi = US_EPI_NONE;
  p.batch = batch;
  p.batch_a = M * K; p.batch_b = N * K; p.batch_c = M * N;
  return from_hip(launch_gemm(p, as_stream(stream)));
}

us_status us_matmul_batched(const void* A, const void* B, void* C, long batch, long M, long N, long K, int trans_a, int trans_b,
                            us_dtype a_dt, us_dtype b_dt, us_dtype c_dt, float scale, void* stream) {
  begin_launch_record();
  return matmul_batched_impl(A, B, C, batch, M, N, K, trans_a, trans_b, a_dt, b_dt, c_dt, scale, stream);
}

us_status us_attention_fwd(const void* Q, const void* K, const void* V, void* A, void* P, void* O, long heads, long s, long d,
                           void* stream) {
  begin_launch_record();
  // everything the three steps below check is checked here first: a failing call launches nothing
  if (heads < 0 || heads > 65535 || s < 0 || d < 0 || !mult16(s) || !mult16(d) || s > US_SOFTMAX_MAX) return US_ERR_SHAPE;
  if (heads == 0 || s == 0 || d == 0) return US_OK;
  if (!Q || !K || !V || !A || !P || !O) return US_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(A) || !aligned16(P) || !aligned16(O)) return US_ERR_ALIGN;
  const float rs = (float)(1.0 / sqrt((double)s)), rd = (float)(1.0 / sqrt((double)d));
  // scores A = d^-1/2 Q K^T, probabilities P = s softmax(A), output O = s^-1/2 P V
  us_status st = matmul_batched_impl(Q, K, A, heads, s, s, d, 0, 1, US_F16, US_F16, US_F16, rd, stream);
  if (st != US_OK) return st;
  st = us_softmax_fwd(A, P, heads * s, s, 0.0f, 0.0f, stream);
  if (st != US_OK) return st;
  return matmul_batched_impl(P, V, O, heads, s, d, s, 0, 0, US_F16, US_F16, US_F16, rs, stream);
}

us_status us_attention_bwd(const void* Q, const void* K, const void* V, const void* A, const void* P, const void* dO, void* dP,
                           void* dA, void* dQ, void* dK, void* dV, long heads, long s, long d, void* stream) {
  begin_launch_record();
  // everything the five steps below check is checked here first: a failing call launches nothing
  if (heads < 0 || heads > 65535 || s < 0 || d < 0 || !mult16(s) || !mult16(d) || s > US_SOFTMAX_MAX) return US_ERR_SHAPE;
  if (heads == 0 || s == 0 || d == 0) return US_OK;
  if (!Q || !K || !V || !A || !P || !dO || !dP || !dA || !dQ || !dK || !dV) return US_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(A) || !aligned16(P) || !aligned16(dO) || !aligned16(dP) ||
      !aligned16(dA) || !aligned16(dQ) || !aligned16(dK) || !aligned16(dV))
    return US_ERR_ALIGN;
  const float rs = (float)(1.0 / sqrt((double)s)), rd = (float)(1.0 / sqrt((double)d));
  // dV = s^-1/2 P^T dO;  dP = d^-1/2 dO V^T;  dA = s * softmax'(A)(dP);  dQ = s^-1/2 dA K;  dK = s^-1/2 dA^T Q
  us_status st = matmul_batched_impl(P, dO, dV, heads, s, d, s, 1, 0, US_F16, US_F16, US_F16, rs, stream);
  if (st != US_OK) return st;
  st = matmul_batched_impl(dO, V, dP, heads, s, s, d, 0, 1, US_F16, US_F16, US_F16, rd, stream);
  if (st != US_OK) return st;
  st = us_softmax_bwd(A, dP, dA, heads * s, s, 0.0f, 0.0f, stream);
  if (st != US_OK) return st;
  st = matmul_batched_impl(dA, K, dQ, heads, s, d, s, 0, 0, US_F16, US_F16, US_F16, rs, stream);
  if (st != US_OK) return st;
  return matmul_batched_impl(dA, Q, dK, heads, s, d, s, 1, 0, US_F16, US_F16, US_F16, rs, stream);
}

us_status us_sum_fwd(const void* X, void* Y, long rows, long n, float alpha, void* stream) {
  if (rows < 0 || n < 0 || n % 8 != 0 || n > (1L << 30)) return US_ERR_SHAPE;
  if (rows == 0) return US_OK;
  if (!Y || (n > 0 && !X)) return US_ERR_NULL;
  if (!aligned16(X) || ((uintptr_t)Y & 1)) return US_ERR_ALIGN;
  const float a = alpha > 0.0f ? alpha : (float)(1.0 / sqrt((double)(n > 0 ? n : 1)));
  return from_hip(launch_sum_fwd(X, Y, rows, n, a, as_stream(stream)));
}

us_status us_sum_bwd(const void* G, void* dX, long rows, long n, float beta, void* stream) {
  if (rows < 0 || n < 0 || n % 8 != 0 || n > (1L << 30)) return US_ERR_SHAPE;
  if (rows == 0 || n == 0) return US_OK;
  if (!G || !dX) return US_ERR_NULL;
  if (!aligned16(dX) || ((uintptr_t)G & 1)) return US_ERR_ALIGN;
  return from_hip(launch_sum_bwd(G, dX, rows, n, beta > 0.0f ? beta : 1.0f, as_stream(stream)));
}

}  // extern "C"
