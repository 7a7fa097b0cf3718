// Routing of a GEMM problem to its kernel family, and the split-K policy of the grad_W reduction.
#include <stdio.h>

#include "us_gemm_dispatch.h"

namespace us {

const DeviceInfo& device_info() {
  static const DeviceInfo fallback{256, 8};
  static DeviceInfo info[kMaxDevices];
  static std::once_flag once[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return fallback;
  std::call_once(once[dev], [dev] {
    int cus = 0, xcds = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = fallback.cus;
    if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess || xcds < 1) xcds = fallback.xcds;
    info[dev] = DeviceInfo{cus, xcds};
  });
  return info[dev];
}

namespace {
thread_local char g_record[512];
thread_local int g_record_len = 0;
}  // namespace

void begin_launch_record() {
  g_record_len = 0;
  g_record[0] = 0;
}

void note_gemm_launch(const char* kind, int bm, int bn, int waves_k, int nst, bool fp8, bool a_kc, bool b_kc, int epi, bool wide,
                      int splits) {
  static const char* const epi_name[] = {"store", "act", "act_grad", "partial", "gelu_tab", "gelu_grad_tab", "gelu_tab16", "residual"};
  const char* layout = a_kc ? (b_kc ? "NT" : "NN") : (b_kc ? "TT" : "TN");
  const int room = (int)sizeof(g_record) - g_record_len;
  if (room <= 1) return;
  const int w = snprintf(g_record + g_record_len, (size_t)room, "%s%s:%dx%d:wk%d:st%d:%s:%s:%s%s:s%d", g_record_len ? " + " : "", kind, bm,
                         bn, waves_k, nst, fp8 ? "fp8" : "f16", layout, (epi >= 0 && epi < 8) ? epi_name[epi] : "?", wide ? ":f32" : "",
                         splits);
  if (w > 0) g_record_len += (w < room ? w : room - 1);
}

const char* last_launch_record() { return g_record; }

// out[m][n] = round( scale * sum_s partial[s][m][n] ), slices added in order (deterministic).
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float* __restrict__ partial, void* out, long total,
                                                            int splits, float scale, int out_is_f32) {
  const long i4 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= total) return;
  v4f s = *reinterpret_cast<const v4f*>(partial + i4);
  for (int k = 1; k < splits; ++k) s += *reinterpret_cast<const v4f*>(partial + (size_t)k * total + i4);
  s *= scale;
  if (out_is_f32) {
    wt_store(reinterpret_cast<v4f*>((float*)out + i4), s);
  } else {
    v4h o = {to_half(s.x), to_half(s.y), to_half(s.z), to_half(s.w)};
    wt_store(reinterpret_cast<v4h*>((_Float16*)out + i4), o);
  }
}

hipError_t launch_splitk_reduce(const float* partial, void* out, long total, int splits, float scale, bool out_is_f32,
                                hipStream_t st) {
  splitk_reduce_kernel<<<(unsigned)((total / 4 + 255) / 256), 256, 0, st>>>(partial, out, total, splits, scale,
                                                                          out_is_f32 ? 1 : 0);
  return hipGetLastError();
}

// grad_W has a small output (fan_in x fan_out) and a long reduction (tokens).  When its large tiles
// cannot occupy the chip the small tile is used (two workgroups per CU: twice the CU count in slots), and if even those
// are too few the token range is cut into slices of whole 128-token stages, at least 512 tokens each.
long gemm_k_per_split(long K, int splits) {
  const long unit = 128;
  return ((K + splits - 1) / splits + unit - 1) / unit * unit;
}

int gemm_splits(long M, long N, long K) {
  if (use_big_tile(M, N, 1) || K < 1024 || use_wave_split_tile(M, N, K)) return 1;
  const long tiles = ceil_div(M, 128) * ceil_div(N, 128);
  long s = 2 * cu_count() / tiles;
  const long max_by_k = K / 512;
  if (s > max_by_k) s = max_by_k;
  if (s > 8) s = 8;
  if (s < 1) s = 1;
  const long kps = gemm_k_per_split(K, (int)s);
  return (int)((K + kps - 1) / kps);
}

size_t gemm_workspace_bytes(long M, long N, long K) {
  const int s = gemm_splits(M, N, K);
  return s <= 1 ? 0 : (size_t)s * (size_t)M * (size_t)N * sizeof(float);
}

hipError_t launch_gemm(const GemmProblem& p, hipStream_t st) {
  const bool fp8 = (p.a_dt != US_F16);
  if (p.a_kc && !p.b_kc) return fp8 ? gemm_nn_fp8(p, st) : gemm_nn_f16(p, st);
  if (p.a_kc && p.b_kc) return fp8 ? gemm_nt_fp8(p, st) : gemm_nt_f16(p, st);
  if (!p.a_kc && !p.b_kc) return fp8 ? gemm_tn_fp8(p, st) : gemm_tn_f16(p, st);
  return hipErrorInvalidValue;
}

}  // namespace us
