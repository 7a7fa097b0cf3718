// Element-wise kernels of the unit-scaled FFN path for gfx950: the scaled saturating cast to FP8
// and the stand-alone unit-scaled GELU forward / backward.  All three are bound by HBM traffic:
// every thread moves 128-bit vectors and the arithmetic is kept to a few VALU operations per element.
#include "us_device.h"
#include "us_launch.h"

namespace us {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxCastBatch = US_CAST_BATCH_MAX;

__device__ __forceinline__ void load16(const _Float16* src, size_t i, float (&x)[16]) {
  v8h a = *reinterpret_cast<const v8h*>(src + i);
  v8h b = *reinterpret_cast<const v8h*>(src + i + 8);
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    x[k] = (float)a[k];
    x[8 + k] = (float)b[k];
  }
}
__device__ __forceinline__ void load16(const float* src, size_t i, float (&x)[16]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    v4f a = *reinterpret_cast<const v4f*>(src + i + 4 * q);
#pragma unroll
    for (int k = 0; k < 4; ++k) x[4 * q + k] = a[k];
  }
}

struct Counts {
  uint32_t sat = 0, flush0 = 0, subn = 0, nan = 0;
};

template <int FMT>
__device__ __forceinline__ void count_one(float p, uint32_t code, Counts& c) {
  constexpr float kMax = (FMT == US_E4M3) ? 448.0f : 57344.0f;
  constexpr uint32_t kFirstNormal = (FMT == US_E4M3) ? 0x08u : 0x04u;
  uint32_t mag = code & 0x7fu;
  c.sat += (__builtin_fabsf(p) > kMax) ? 1u : 0u;
  c.nan += (p != p) ? 1u : 0u;
  c.flush0 += (p != 0.0f && mag == 0u) ? 1u : 0u;       // NaN has a non-zero code, so it is not counted here
  c.subn += (mag != 0u && mag < kFirstNormal) ? 1u : 0u;
}

// dst[i] = fp8( fp32(src[i] * scale) ): 16 elements per thread per step (two or four 128-bit loads,
// one 128-bit store), grid-stride; the last n % 16 elements are handled one per thread.
template <typename SrcT, int FMT, bool STATS>
__global__ void __launch_bounds__(kThreads) cast_kernel(const SrcT* __restrict__ src, uint8_t* __restrict__ dst,
                                                        size_t n, float scale, us_cast_stats* stats) {
  const size_t nvec = n / 16;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthr = (size_t)gridDim.x * kThreads;
  Counts c;
  auto convert = [&](const float (&x)[16], size_t v) {
    v4i out;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float p0 = x[4 * q] * scale, p1 = x[4 * q + 1] * scale, p2 = x[4 * q + 2] * scale, p3 = x[4 * q + 3] * scale;
      uint32_t w = cvt4_fp8<FMT>(p0, p1, p2, p3);
      out[q] = (int)w;
      if (STATS) {
        count_one<FMT>(p0, w, c);
        count_one<FMT>(p1, w >> 8, c);
        count_one<FMT>(p2, w >> 16, c);
        count_one<FMT>(p3, w >> 24, c);
      }
    }
    wt_store(reinterpret_cast<v4i*>(dst + v * 16), out);
  };
  // two vectors per thread and step, both requested before the first is used (the counting variant runs on few
  // blocks, so the bytes in flight have to come from each thread)
  size_t v = tid;
  for (; v + nthr < nvec; v += 2 * nthr) {
    float x0[16], x1[16];
    load16(src, v * 16, x0);
    load16(src, (v + nthr) * 16, x1);
    convert(x0, v);
    convert(x1, v + nthr);
  }
  if (v < nvec) {
    float x[16];
    load16(src, v * 16, x);
    convert(x, v);
  }
  const size_t tail0 = nvec * 16;
  if (tid < n - tail0) {
    float p = (float)src[tail0 + tid] * scale;
    uint32_t w = cvt_pk_fp8<FMT>(p, 0.0f) & 0xffu;
    dst[tail0 + tid] = (uint8_t)w;
    if (STATS) count_one<FMT>(p, w, c);
  }
  if (STATS) {
    __shared__ uint32_t s[4];
    if (threadIdx.x < 4) s[threadIdx.x] = 0;
    __syncthreads();
    if (c.sat) atomicAdd(&s[0], c.sat);
    if (c.flush0) atomicAdd(&s[1], c.flush0);
    if (c.subn) atomicAdd(&s[2], c.subn);
    if (c.nan) atomicAdd(&s[3], c.nan);
    __syncthreads();
    if (threadIdx.x < 4 && s[threadIdx.x]) {
      unsigned long long* g = reinterpret_cast<unsigned long long*>(stats);
      atomicAdd(&g[threadIdx.x], (unsigned long long)s[threadIdx.x]);
    }
  }
}

// Up to kMaxCastBatch FP16 tensors cast with scale 1 in one launch (the casts of one training step:
// activations, two weight matrices and the incoming gradient are each only a few microseconds of
// work, so four launches cost more in ramp-up and tails than in traffic).  blockIdx.x is mapped to a
// tensor through the prefix sums of the per-tensor block counts; each block converts a contiguous
// run of 16-element vectors with the packed FP16 -> FP8 converter.
struct CastBatch {
  const _Float16* src[kMaxCastBatch];
  uint8_t* dst[kMaxCastBatch];
  unsigned long long n[kMaxCastBatch];
  unsigned int first_block[kMaxCastBatch + 1];
  int e5m2[kMaxCastBatch];
  int count;
};
constexpr int kBatchVecsPerBlock = 4 * kThreads;   // 16 KiB of codes per block

template <int FMT>
__device__ __forceinline__ void cast_run_half(const _Float16* __restrict__ src, uint8_t* __restrict__ dst, size_t n,
                                              size_t vec0) {
  const size_t nvec = n / 16;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const size_t v = vec0 + (size_t)u * kThreads + threadIdx.x;
    if (v < nvec) {
      const v8h a = *reinterpret_cast<const v8h*>(src + v * 16);
      const v8h b = *reinterpret_cast<const v8h*>(src + v * 16 + 8);
      v4i out;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const v2h p0 = {a[4 * q], a[4 * q + 1]}, p1 = {a[4 * q + 2], a[4 * q + 3]};
        const v2h p2 = {b[4 * q], b[4 * q + 1]}, p3 = {b[4 * q + 2], b[4 * q + 3]};
        out[q] = (int)(cvt_pk_fp8_from_half<FMT>(p0) | (cvt_pk_fp8_from_half<FMT>(p1) << 16));
        out[2 + q] = (int)(cvt_pk_fp8_from_half<FMT>(p2) | (cvt_pk_fp8_from_half<FMT>(p3) << 16));
      }
      wt_store(reinterpret_cast<v4i*>(dst + v * 16), out);
    }
  }
  // the last n % 16 elements, by the block that owns the end of the tensor
  const size_t tail0 = nvec * 16;
  if (vec0 + kBatchVecsPerBlock >= nvec && threadIdx.x < n - tail0) {
    const _Float16 h = src[tail0 + threadIdx.x];
    const v2h p = {h, h};
    dst[tail0 + threadIdx.x] = (uint8_t)cvt_pk_fp8_from_half<FMT>(p);
  }
}

__global__ void __launch_bounds__(kThreads) cast_batch_kernel(CastBatch cb) {
  int t = 0;
#pragma unroll
  for (int i = 1; i < kMaxCastBatch; ++i)
    if (i < cb.count && blockIdx.x >= cb.first_block[i]) t = i;
  const size_t vec0 = (size_t)(blockIdx.x - cb.first_block[t]) * kBatchVecsPerBlock;
  if (cb.e5m2[t]) cast_run_half<US_E5M2>(cb.src[t], cb.dst[t], cb.n[t], vec0);
  else cast_run_half<US_E4M3>(cb.src[t], cb.dst[t], cb.n[t], vec0);
}

// h = fp16/fp32( alpha_g * z * Phi(z) ), eight (FP16) or four (FP32) elements per 128-bit access.
template <typename T, bool BWD>
__global__ void __launch_bounds__(kThreads) gelu_kernel(const T* z, const T* gh, T* out, size_t n,
                                                        float s) {
  constexpr int V = 16 / sizeof(T);
  typedef T vec_t __attribute__((ext_vector_type(V)));
  const size_t nvec = n / V;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthr = (size_t)gridDim.x * kThreads;
  for (size_t v = tid; v < nvec; v += nthr) {
    vec_t zv = *reinterpret_cast<const vec_t*>(z + v * V);
    vec_t gv;
    if (BWD) gv = *reinterpret_cast<const vec_t*>(gh + v * V);
    vec_t o;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      if constexpr (sizeof(T) == 2 && BWD) {
        o[k] = gelu_grad_half(zv[k], gv[k], s);        // the same function as the matmul epilogues' GELU'
      } else {
        const float r = BWD ? gelu_grad_scaled((float)zv[k], (float)gv[k], s) : gelu_scaled((float)zv[k], s);
        if constexpr (sizeof(T) == 2) o[k] = to_half(r);
        else o[k] = r;
      }
    }
    wt_store(reinterpret_cast<vec_t*>(out + v * V), o);
  }
  const size_t tail0 = nvec * V;
  if (tid < n - tail0) {
    const float zi = (float)z[tail0 + tid];
    if constexpr (sizeof(T) == 2 && BWD) {
      out[tail0 + tid] = gelu_grad_half(z[tail0 + tid], gh[tail0 + tid], s);
    } else {
      const float r = BWD ? gelu_grad_scaled(zi, (float)gh[tail0 + tid], s) : gelu_scaled(zi, s);
      if constexpr (sizeof(T) == 2) out[tail0 + tid] = to_half(r);
      else out[tail0 + tid] = r;
    }
  }
}

// tab[i] = E4M3 code of fp16(alpha_g * gelu(z)) for the FP16 value z with bit pattern i
__global__ void __launch_bounds__(kThreads) gelu_table_kernel(uint8_t* tab, float alpha_g) {
  const uint32_t i = blockIdx.x * kThreads + threadIdx.x;       // 0 .. 65535
  const _Float16 h = to_half(gelu_scaled((float)half_from_bits(i), alpha_g));
  const v2h pair = {h, h};
  tab[i] = (uint8_t)cvt_pk_fp8_from_half<US_E4M3>(pair);
}
// tab[s * 0x4601 + a] = fp16(alpha_g * gelu(z)) for the FP16 value z with sign s and magnitude bits a <= 0x4600
__global__ void __launch_bounds__(kThreads) gelu_half_table_kernel(_Float16* tab, float alpha_g) {
  const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
  constexpr uint32_t kPer = kGeluHalfLast + 1;
  if (i >= 2 * kPer) return;
  const uint32_t bits = (i % kPer) | ((i / kPer) << 15);
  tab[i] = to_half(gelu_scaled((float)half_from_bits(bits), alpha_g));
}
// tab[i] = beta_g * gelu'(|z|) in FP32 for the FP16 magnitudes 0 .. 8.0 (bit patterns 0 .. 0x4800)
__global__ void __launch_bounds__(kThreads) gelu_slope_table_kernel(float* tab, float beta_g) {
  const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
  if (i <= (uint32_t)kGeluSlopeLast) tab[i] = gelu_slope_abs((float)half_from_bits(i), beta_g);
}

inline int grid_for(size_t nvec) {
  // enough blocks to fill 256 CUs several times over, capped so the grid-stride loop amortises launch cost
  size_t blocks = (nvec + kThreads - 1) / kThreads;
  if (blocks < 1) blocks = 1;
  if (blocks > 256 * 32) blocks = 256 * 32;
  return (int)blocks;
}

template <typename SrcT, int FMT>
hipError_t cast_dispatch(const void* src, void* dst, size_t n, float scale, us_cast_stats* stats, hipStream_t st) {
  int grid = grid_for(n / 16);
  // With counters every block ends with up to four 64-bit atomics on the same four words, and those are served one
  // after the other (about 13 ns each, measured: 4096 blocks spent 55 us there on a 17 M-element tensor): two blocks
  // per CU walk the tensor in a grid-stride loop instead.
  if (stats && grid > 2 * device_info().cus) grid = 2 * device_info().cus;
  if (stats)
    cast_kernel<SrcT, FMT, true><<<grid, kThreads, 0, st>>>((const SrcT*)src, (uint8_t*)dst, n, scale, stats);
  else
    cast_kernel<SrcT, FMT, false><<<grid, kThreads, 0, st>>>((const SrcT*)src, (uint8_t*)dst, n, scale, nullptr);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_cast(const void* src, us_dtype src_dt, void* dst, us_dtype dst_dt, size_t n, float scale,
                       us_cast_stats* stats, hipStream_t st) {
  if (src_dt == US_F16)
    return dst_dt == US_E4M3 ? cast_dispatch<_Float16, US_E4M3>(src, dst, n, scale, stats, st)
                             : cast_dispatch<_Float16, US_E5M2>(src, dst, n, scale, stats, st);
  return dst_dt == US_E4M3 ? cast_dispatch<float, US_E4M3>(src, dst, n, scale, stats, st)
                           : cast_dispatch<float, US_E5M2>(src, dst, n, scale, stats, st);
}

hipError_t launch_cast_batch(int count, const void* const* src, void* const* dst, const size_t* n, const us_dtype* dst_dt,
                             hipStream_t st) {
  CastBatch cb{};
  cb.count = count;
  unsigned int blocks = 0;
  for (int i = 0; i < count; ++i) {
    cb.src[i] = (const _Float16*)src[i];
    cb.dst[i] = (uint8_t*)dst[i];
    cb.n[i] = n[i];
    cb.e5m2[i] = (dst_dt[i] == US_E5M2) ? 1 : 0;
    cb.first_block[i] = blocks;
    const size_t nvec = n[i] / 16;
    size_t nb = (nvec + kBatchVecsPerBlock - 1) / kBatchVecsPerBlock;
    if (nb == 0 && n[i] > 0) nb = 1;                 // a tensor shorter than one vector still needs its tail
    blocks += (unsigned int)nb;
  }
  cb.first_block[count] = blocks;
  if (blocks == 0) return hipSuccess;
  cast_batch_kernel<<<blocks, kThreads, 0, st>>>(cb);
  return hipGetLastError();
}

hipError_t launch_gelu_table(void* table, float alpha_g, hipStream_t st) {
  gelu_table_kernel<<<65536 / kThreads, kThreads, 0, st>>>((uint8_t*)table, alpha_g);
  return hipGetLastError();
}

hipError_t launch_gelu_half_table(void* table, float alpha_g, hipStream_t st) {
  gelu_half_table_kernel<<<(2 * (kGeluHalfLast + 1) + kThreads - 1) / kThreads, kThreads, 0, st>>>((_Float16*)table, alpha_g);
  return hipGetLastError();
}

hipError_t launch_gelu_slope_table(void* table, float beta_g, hipStream_t st) {
  gelu_slope_table_kernel<<<(kGeluSlopeLast + kThreads) / kThreads, kThreads, 0, st>>>((float*)table, beta_g);
  return hipGetLastError();
}

hipError_t launch_gelu_fwd(const void* z, void* h, size_t n, us_dtype dt, float alpha_g, hipStream_t st) {
  if (dt == US_F16) {
    gelu_kernel<_Float16, false><<<grid_for(n / 8), kThreads, 0, st>>>((const _Float16*)z, nullptr, (_Float16*)h, n, alpha_g);
  } else {
    gelu_kernel<float, false><<<grid_for(n / 4), kThreads, 0, st>>>((const float*)z, nullptr, (float*)h, n, alpha_g);
  }
  return hipGetLastError();
}

// out = round( scale * f(s1 * z) )  or  round( scale * f'(s1 * z) * gh )  for the activations of us_device.h
template <typename T, bool BWD>
__global__ void __launch_bounds__(kThreads) act_kernel(const T* z, const T* gh, T* out, size_t n, int kind, float s1, float scale) {
  constexpr int V = 16 / sizeof(T);
  typedef T vec_t __attribute__((ext_vector_type(V)));
  const size_t nvec = n / V;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthr = (size_t)gridDim.x * kThreads;
  auto one = [&](T zi, T gi) -> T {
    if constexpr (sizeof(T) == 2 && BWD) {
      return act_grad_half(kind, s1 * (float)zi, gi, scale);
    } else {
      const float r = BWD ? act_grad_scaled(kind, s1 * (float)zi, (float)gi, scale) : act_scaled(kind, s1 * (float)zi, scale);
      if constexpr (sizeof(T) == 2) return to_half(r);
      else return r;
    }
  };
  for (size_t v = tid; v < nvec; v += nthr) {
    const vec_t zv = *reinterpret_cast<const vec_t*>(z + v * V);
    vec_t gv = zv;
    if (BWD) gv = *reinterpret_cast<const vec_t*>(gh + v * V);
    vec_t o;
#pragma unroll
    for (int k = 0; k < V; ++k) o[k] = one(zv[k], gv[k]);
    wt_store(reinterpret_cast<vec_t*>(out + v * V), o);
  }
  const size_t tail0 = nvec * V;
  if (tid < n - tail0) out[tail0 + tid] = one(z[tail0 + tid], BWD ? gh[tail0 + tid] : z[tail0 + tid]);
}

hipError_t launch_act(const void* z, const void* gh, void* out, size_t n, us_dtype dt, int kind, bool bwd, float s1, float scale,
                      hipStream_t st) {
  if (dt == US_F16) {
    const int grid = grid_for(n / 8);
    if (bwd) act_kernel<_Float16, true><<<grid, kThreads, 0, st>>>((const _Float16*)z, (const _Float16*)gh, (_Float16*)out, n, kind, s1, scale);
    else act_kernel<_Float16, false><<<grid, kThreads, 0, st>>>((const _Float16*)z, nullptr, (_Float16*)out, n, kind, s1, scale);
  } else {
    const int grid = grid_for(n / 4);
    if (bwd) act_kernel<float, true><<<grid, kThreads, 0, st>>>((const float*)z, (const float*)gh, (float*)out, n, kind, s1, scale);
    else act_kernel<float, false><<<grid, kThreads, 0, st>>>((const float*)z, nullptr, (float*)out, n, kind, s1, scale);
  }
  return hipGetLastError();
}

// out = round( ca * a + cb * b ): the product ca * a rounded to FP32, then one fused multiply-add (the
// same arithmetic as the residual epilogue of the matmul kernels).
template <typename T>
__global__ void __launch_bounds__(kThreads) weighted_add_kernel(const T* a, const T* b, T* out, size_t n, float ca, float cb) {
  constexpr int V = 16 / sizeof(T);
  typedef T vec_t __attribute__((ext_vector_type(V)));
  const size_t nvec = n / V;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthr = (size_t)gridDim.x * kThreads;
  auto one = [&](T x, T y) -> T {
    const float r = __builtin_fmaf(cb, (float)y, ca * (float)x);
    if constexpr (sizeof(T) == 2) return to_half(r);
    else return r;
  };
  for (size_t v = tid; v < nvec; v += nthr) {
    const vec_t av = *reinterpret_cast<const vec_t*>(a + v * V), bv = *reinterpret_cast<const vec_t*>(b + v * V);
    vec_t o;
#pragma unroll
    for (int k = 0; k < V; ++k) o[k] = one(av[k], bv[k]);
    wt_store(reinterpret_cast<vec_t*>(out + v * V), o);
  }
  const size_t tail0 = nvec * V;
  if (tid < n - tail0) out[tail0 + tid] = one(a[tail0 + tid], b[tail0 + tid]);
}

hipError_t launch_weighted_add(const void* a, const void* b, void* out, size_t n, us_dtype dt, float ca, float cb,
                               hipStream_t st) {
  if (dt == US_F16) {
    weighted_add_kernel<_Float16><<<grid_for(n / 8), kThreads, 0, st>>>((const _Float16*)a, (const _Float16*)b, (_Float16*)out, n, ca, cb);
  } else {
    weighted_add_kernel<float><<<grid_for(n / 4), kThreads, 0, st>>>((const float*)a, (const float*)b, (float*)out, n, ca, cb);
  }
  return hipGetLastError();
}

hipError_t launch_gelu_bwd(const void* z, const void* gh, void* gz, size_t n, us_dtype dt, float beta_g,
                           hipStream_t st) {
  if (dt == US_F16) {
    gelu_kernel<_Float16, true><<<grid_for(n / 8), kThreads, 0, st>>>((const _Float16*)z, (const _Float16*)gh, (_Float16*)gz, n, beta_g);
  } else {
    gelu_kernel<float, true><<<grid_for(n / 4), kThreads, 0, st>>>((const float*)z, (const float*)gh, (float*)gz, n, beta_g);
  }
  return hipGetLastError();
}

}  // namespace us
