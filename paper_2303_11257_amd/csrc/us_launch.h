// Host-side launch functions implemented by the kernel translation units.  Arguments are already
// validated by the C-ABI layer; every function only enqueues work on `stream`.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

#include <mutex>

#include "../../include/us.h"

namespace us {

// What the tile-shape windows and the workgroup -> tile walk need to know about the current device: the number of
// compute units and of XCDs (accelerator dies, each with its own L2; workgroups go to them round-robin).  Queried
// once per device; MI355X's figures (256, 8) when no device can be asked (host-only use of the size functions).
struct DeviceInfo {
  int cus;
  int xcds;
};
constexpr int kMaxDevices = 64;
const DeviceInfo& device_info();

// Raising a kernel's dynamic-LDS limit is a once-per-function-and-device call: one object of this type per kernel
// instantiation (a function-local static), safe against host threads that enter the same launch together.
struct FuncConfig {
  std::once_flag once[kMaxDevices];
  hipError_t err[kMaxDevices];
  hipError_t ensure(const void* fn, int lds_bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::call_once(once[dev], [&] { err[dev] = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes); });
    return err[dev];
  }
};

// Diagnostics: which GEMM kernel(s) the calling host thread's most recent matmul call launched (tile shape, wave
// groups, stages, operand layouts, epilogue), as text.  note_gemm_launch() appends one kernel to the record that
// begin_launch_record() cleared.
void begin_launch_record();
void note_gemm_launch(const char* kind, int bm, int bn, int waves_k, int nst, bool fp8, bool a_kc, bool b_kc, int epi, bool wide,
                      int splits);
const char* last_launch_record();

hipError_t launch_cast(const void* src, us_dtype src_dt, void* dst, us_dtype dst_dt, size_t n, float scale,
                       us_cast_stats* stats, hipStream_t stream);
hipError_t launch_cast_batch(int count, const void* const* src, void* const* dst, const size_t* n, const us_dtype* dst_dt,
                             hipStream_t stream);
hipError_t launch_gelu_fwd(const void* z, void* h, size_t n, us_dtype dt, float alpha_g, hipStream_t stream);
hipError_t launch_gelu_bwd(const void* z, const void* gh, void* gz, size_t n, us_dtype dt, float beta_g,
                           hipStream_t stream);
hipError_t launch_act(const void* z, const void* gh, void* out, size_t n, us_dtype dt, int kind, bool bwd, float s1, float scale,
                      hipStream_t stream);
hipError_t launch_weighted_add(const void* a, const void* b, void* out, size_t n, us_dtype dt, float ca, float cb,
                               hipStream_t stream);

hipError_t launch_exponent_histogram(const void* src, us_dtype dt, size_t n, unsigned long long* hist, hipStream_t stream);
hipError_t launch_cast_snr(const void* src, us_dtype src_dt, size_t n, us_dtype dst_dt, float scale, double* sums, hipStream_t stream);
size_t layer_norm_workspace_bytes(long b, long n);
hipError_t launch_layer_norm_fwd(const void* X, const void* w, const void* c, void* Y, long b, long n, float eps, hipStream_t stream);
hipError_t launch_layer_norm_bwd(const void* X, const void* w, const void* G, void* dX, void* dw, void* dc, long b, long n, float eps,
                                 float beta_wc, void* workspace, hipStream_t stream);

hipError_t launch_sum_fwd(const void* X, void* Y, long rows, long n, float alpha, hipStream_t stream);
hipError_t launch_sum_bwd(const void* G, void* dX, long rows, long n, float beta, hipStream_t stream);
hipError_t launch_softmax_fwd(const void* X, void* Y, long rows, long s, float s1, float alpha, hipStream_t stream);
hipError_t launch_softmax_bwd(const void* X, const void* G, void* dX, long rows, long s, float s1, float beta, hipStream_t stream);
hipError_t launch_softmax_xent(const void* X, const int* target, float* loss, void* dX, long rows, long s, float s1, float beta,
                               hipStream_t stream);
size_t bias_grad_workspace_bytes(long b, long n);
hipError_t launch_bias_grad(const void* G, us_dtype g_dt, void* dc, long b, long n, float beta, void* workspace, hipStream_t stream);
// second half of launch_bias_grad alone: dc = fp16(beta * sum over the nblocks rows of partial[nblocks][n])
hipError_t launch_bias_grad_reduce(const void* partial, void* dc, long nblocks, long n, float beta, hipStream_t stream);

// One GEMM problem  C[M,N] = epilogue( scale * sum_k A(m,k) B(n,k) ).
//   a_kc / b_kc: operand is K-contiguous (element (r,k) at base[r*ld + k]) or K-strided
//   (element (r,k) at base[k*ld + r]).  The three layer-level products map to
//     forward  Y  = X W      : A = X (K-contig),  B = W (K-strided)
//     grad_X   dX = G W^T    : A = G (K-contig),  B = W (K-contig)
//     grad_W   dW = X^T G    : A = X (K-strided), B = G (K-strided)
struct GemmProblem {
  const void* A;
  const void* B;
  void* C;
  long M, N, K;
  long lda, ldb, ldc;      // in elements
  bool a_kc, b_kc;
  us_dtype a_dt, b_dt;     // F16/F16, or two FP8 types
  us_dtype c_dt;           // F16 or F32
  float scale;
  us_epilogue epi;
  float epi_scale;
  int act;                 // GELU / GELU_GRAD epilogues: activation kind, 0 = gelu
  float skip_scale;        // RESIDUAL: weight of the skip input (epi_scale is the weight of the matmul result)
  const void* Zpre;        // GELU_GRAD: saved pre-activation; RESIDUAL: skip input; FP16 [M,N], leading dimension ldc
  void* aux16;             // GELU: FP16 [M,N] or NULL
  void* aux8;              // GELU: E4M3 [M,N]; GELU_GRAD: E5M2 [M,N]; or NULL
  void* workspace;         // split-K partial sums (FP32), or NULL
  long batch;              // number of equally shaped, independent products (0 or 1: a single one); plain store only
  long batch_a, batch_b, batch_c;   // elements between consecutive problems
  const void* bias;        // forward product with FP16 result: optional FP16 row [N] added before the rounding, or NULL
  void* colsum;            // GELU_GRAD: optional FP32 [ceil(M / 32)][N] that receives the column sums of the FP16 result per
                           // 32-row block (every element written), or NULL
  void* table;             // table area of the workspace (us_device.h), or NULL: arithmetic epilogue
  bool tables_ready;       // the table area is already filled for this epi_scale
  size_t workspace_bytes;
};

// Number of K slices the dW reduction is cut into, and the scratch it needs (0 when 1 slice).
int gemm_splits(long M, long N, long K);
long gemm_k_per_split(long K, int splits);
size_t gemm_workspace_bytes(long M, long N, long K);

hipError_t launch_gemm(const GemmProblem& p, hipStream_t stream);

// grad_X (dx) and grad_W (dw) of one layer in a single launch with interleaved tiles; only for the
// shape / type combinations gemm_pair_applicable accepts.  Either product may run on another tile shape than
// alone, whose wave groups add their k-steps in another order: FP16 results can differ in the last place.
bool gemm_pair_applicable(const GemmProblem& dx, const GemmProblem& dw);
hipError_t launch_gemm_pair(const GemmProblem& dx, const GemmProblem& dw, hipStream_t stream);

// Fill the tables of the table-driven GELU epilogues (layouts in us_device.h).
hipError_t launch_gelu_table(void* table, float alpha_g, hipStream_t stream);
hipError_t launch_gelu_slope_table(void* table, float beta_g, hipStream_t stream);
hipError_t launch_gelu_half_table(void* table, float alpha_g, hipStream_t stream);

}  // namespace us
