// Diagnostics on a tensor (Fig. 1 / App. K: histogram of exponent values on the FP16 grid; Sec. 3.1:
// signal-to-noise ratio of a cast).  Read-only, HBM-bound: 2 or 4 bytes per element.
#include "us_device.h"
#include "us_launch.h"

namespace us {

namespace {

constexpr int kThreads = 256;

// bin of |x| (layout in include/us.h): works on the FP32 bit pattern, so FP16 inputs are widened first
__device__ __forceinline__ int exponent_bin(float x) {
  const uint32_t a = __builtin_bit_cast(uint32_t, x) & 0x7fffffffu;
  if (a > 0x7f800000u) return 34;                         // NaN
  if (a == 0) return 0;
  const int e = (int)(a >> 23) - 127;                     // FP32 subnormals have e = -127: far below 2^-24
  if (e >= 16) return 33;                                 // >= 2^16, infinity included
  if (e < -24) return 1;
  if (e < -14) return 2;
  return 3 + e + 14;
}

// A unit-scale tensor puts 90 % of its values into five bins, so one shared LDS histogram would serialise on
// them: every group of four lanes (lane mod 16, per wave) counts into a copy of its own, added up at the end.
constexpr int kCopies = (kThreads / 64) * 16, kPitch = US_HIST_BINS + 2;      // odd word pitch spreads the banks

template <typename T>
__global__ void __launch_bounds__(kThreads) histogram_kernel(const T* src, size_t n, unsigned long long* hist) {
  __shared__ unsigned int local[kCopies * kPitch];
  for (int i = threadIdx.x; i < kCopies * kPitch; i += kThreads) local[i] = 0;
  __syncthreads();
  unsigned int* mine = local + ((threadIdx.x >> 6) * 16 + (threadIdx.x & 15)) * kPitch;
  constexpr int V = 16 / sizeof(T);
  typedef T vec_t __attribute__((ext_vector_type(V)));
  const size_t nvec = n / V;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x, nthr = (size_t)gridDim.x * kThreads;
  for (size_t v = tid; v < nvec; v += nthr) {
    const vec_t x = *reinterpret_cast<const vec_t*>(src + v * V);
#pragma unroll
    for (int k = 0; k < V; ++k) atomicAdd(&mine[exponent_bin((float)x[k])], 1u);
  }
  const size_t tail0 = nvec * V;
  if (tid < n - tail0) atomicAdd(&mine[exponent_bin((float)src[tail0 + tid])], 1u);
  __syncthreads();
  if (threadIdx.x < US_HIST_BINS) {
    unsigned int t = 0;
    for (int c = 0; c < kCopies; ++c) t += local[c * kPitch + threadIdx.x];
    if (t) atomicAdd(&hist[threadIdx.x], (unsigned long long)t);
  }
}

// value of the saturating cast of p to FMT, back in FP32
template <int FMT>
__device__ __forceinline__ float quantise(float p) {
  const uint32_t code = cvt_pk_fp8<FMT>(p, 0.0f);
  return FMT == US_E4M3 ? __builtin_amdgcn_cvt_f32_fp8((int)code, 0) : __builtin_amdgcn_cvt_f32_bf8((int)code, 0);
}

// *acc += v on a double in global memory: the hardware's FP64 add at system scope (performed at the memory side).  The
// device-scope form was seen once, in many runs, to lose the contributions of one eighth of the workgroups (one XCD's
// worth), which the integer atomics of this library have never done; a compare-and-swap loop is exact too but chains
// 2048 round trips (3.1 -> 0.5 TB/s on 512 MB).
__device__ __forceinline__ void atomic_add_double(double* acc, double v) {
  __hip_atomic_fetch_add(acc, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

template <typename T, int FMT>
__global__ void __launch_bounds__(kThreads) snr_kernel(const T* src, size_t n, float scale, double* sums) {
  __shared__ double part[2][kThreads / 64];
  constexpr int V = 16 / sizeof(T);
  typedef T vec_t __attribute__((ext_vector_type(V)));
  const size_t nvec = n / V;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x, nthr = (size_t)gridDim.x * kThreads;
  const double inv = 1.0 / (double)scale;
  double s0 = 0.0, s1 = 0.0;
  auto one = [&](float x) {
    if (x != x) return;
    const double q = (double)quantise<FMT>(x * scale) * inv, xd = (double)x;
    s0 += xd * xd;
    s1 += (q - xd) * (q - xd);
  };
  for (size_t v = tid; v < nvec; v += nthr) {
    const vec_t x = *reinterpret_cast<const vec_t*>(src + v * V);
#pragma unroll
    for (int k = 0; k < V; ++k) one((float)x[k]);
  }
  const size_t tail0 = nvec * V;
  if (tid < n - tail0) one((float)src[tail0 + tid]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    s0 += __shfl_xor(s0, off, 64);
    s1 += __shfl_xor(s1, off, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    part[0][threadIdx.x >> 6] = s0;
    part[1][threadIdx.x >> 6] = s1;
  }
  __syncthreads();
  if (threadIdx.x < 2) {
    double t = 0.0;
    for (int w = 0; w < kThreads / 64; ++w) t += part[threadIdx.x][w];
    atomic_add_double(&sums[threadIdx.x], t);
  }
}

int grid_for(size_t nvec) {
  size_t blocks = (nvec + kThreads - 1) / kThreads;
  if (blocks < 1) blocks = 1;
  if (blocks > 256 * 8) blocks = 256 * 8;
  return (int)blocks;
}

}  // namespace

hipError_t launch_exponent_histogram(const void* src, us_dtype dt, size_t n, unsigned long long* hist, hipStream_t st) {
  // every workgroup ends with 35 atomics on the same 35 counters: at least 64 Ki elements per workgroup keep that
  // tail short on small tensors
  const size_t by_work = n / 65536 + 1;
  int g = grid_for(dt == US_F16 ? n / 8 : n / 4);
  if ((size_t)g > by_work) g = (int)by_work;
  if (dt == US_F16) histogram_kernel<_Float16><<<g, kThreads, 0, st>>>((const _Float16*)src, n, hist);
  else histogram_kernel<float><<<g, kThreads, 0, st>>>((const float*)src, n, hist);
  return hipGetLastError();
}

hipError_t launch_cast_snr(const void* src, us_dtype src_dt, size_t n, us_dtype dst_dt, float scale, double* sums, hipStream_t st) {
  const bool e4 = dst_dt == US_E4M3;
  auto grid_snr = [](size_t nvec) { return grid_for(nvec); };
  if (src_dt == US_F16) {
    const int g = grid_snr(n / 8);
    if (e4) snr_kernel<_Float16, US_E4M3><<<g, kThreads, 0, st>>>((const _Float16*)src, n, scale, sums);
    else snr_kernel<_Float16, US_E5M2><<<g, kThreads, 0, st>>>((const _Float16*)src, n, scale, sums);
  } else {
    const int g = grid_snr(n / 4);
    if (e4) snr_kernel<float, US_E4M3><<<g, kThreads, 0, st>>>((const float*)src, n, scale, sums);
    else snr_kernel<float, US_E5M2><<<g, kThreads, 0, st>>>((const float*)src, n, scale, sums);
  }
  return hipGetLastError();
}

}  // namespace us
