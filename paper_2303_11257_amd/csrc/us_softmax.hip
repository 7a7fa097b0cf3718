// Scaled softmax over the last dimension, softmax cross-entropy and the scaled sum (Table A.2 "Other"; App. G "Softmax (followed
// by matmul)", "Softmax cross-entropy").  HBM-bound row kernels, FP16 storage, FP32 arithmetic, every tensor read
// or written once:
//   softmax forward   y = alpha * softmax(s1 x)                          4 B / element   (alpha = s by default)
//   softmax backward  dx = beta * s1 * p * (g - sum p g), p from x       6 B / element   (beta = s)
//   cross-entropy     loss = -log softmax(s1 x)_c,  dx = beta * s1 * (p - onehot(c))     4 B / element
// Softmax rows (attention: 128 .. 4096 long) are held in the registers of one wave; cross-entropy rows (a vocabulary)
// are staged in the LDS of one workgroup.
#include "us_launch.h"
#include "us_rows.h"

namespace us {

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.44269504088896340736f;

// e_j = exp(s1 x_j - max) for the row in x; returns the row sum of e (padding lanes contribute 0)
template <int NCH>
__device__ __forceinline__ float row_exp(const RowRegs<NCH>& x, int s, int lane, float s1, float (&e)[NCH][8]) {
  float m = -__builtin_inff();
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const bool valid = (k * 64 + lane) * 8 < s;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      e[k][q] = s1 * (float)x.v[k][q];
      m = valid ? __builtin_fmaxf(m, e[k][q]) : m;
    }
  }
  m = wave_max(m);
  float sum = 0.0f;
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const bool valid = (k * 64 + lane) * 8 < s;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      e[k][q] = valid ? __builtin_amdgcn_exp2f((e[k][q] - m) * kLog2e) : 0.0f;
      sum += e[k][q];
    }
  }
  return wave_sum(sum);
}

template <int NCH>
__global__ void __launch_bounds__(kThreads) softmax_fwd_kernel(const _Float16* X, _Float16* Y, long rows, int s, float s1, float alpha) {
  const int lane = threadIdx.x & 63;
  const long wave0 = (long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  const long nwaves = (long)gridDim.x * (kThreads / 64);
  for (long row = wave0; row < rows; row += nwaves) {
    RowRegs<NCH> x;
    x.load(X + row * s, s, lane);
    float e[NCH][8];
    const float inv = alpha / row_exp<NCH>(x, s, lane, s1, e);
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int col = (k * 64 + lane) * 8;
      if (col < s) {
        v8h o;
#pragma unroll
        for (int q = 0; q < 8; ++q) o[q] = to_half(e[k][q] * inv);
        wt_store(reinterpret_cast<v8h*>(Y + row * s + col), o);
      }
    }
  }
}

template <int NCH>
__global__ void __launch_bounds__(kThreads) softmax_bwd_kernel(const _Float16* X, const _Float16* G, _Float16* dX, long rows, int s,
                                                               float s1, float beta) {
  const int lane = threadIdx.x & 63;
  const long wave0 = (long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  const long nwaves = (long)gridDim.x * (kThreads / 64);
  for (long row = wave0; row < rows; row += nwaves) {
    RowRegs<NCH> x, g;
    x.load(X + row * s, s, lane);
    g.load(G + row * s, s, lane);
    float e[NCH][8];
    const float inv = 1.0f / row_exp<NCH>(x, s, lane, s1, e);
    float dot = 0.0f;
#pragma unroll
    for (int k = 0; k < NCH; ++k)
#pragma unroll
      for (int q = 0; q < 8; ++q) dot += e[k][q] * (float)g.v[k][q];
    dot = wave_sum(dot) * inv;                         // sum_k p_k g_k
    const float c = beta * s1 * inv;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int col = (k * 64 + lane) * 8;
      if (col < s) {
        v8h o;
#pragma unroll
        for (int q = 0; q < 8; ++q) o[q] = to_half(c * e[k][q] * ((float)g.v[k][q] - dot));
        wt_store(reinterpret_cast<v8h*>(dX + row * s + col), o);
      }
    }
  }
}

// reductions over the workgroup: waves in order 0 .. 3 (fixed association)
__device__ __forceinline__ float block_max(float v, float* scratch) {
  v = wave_max(v);
  __syncthreads();                                      // scratch may still be read from the previous reduction
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = scratch[0];
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) r = __builtin_fmaxf(r, scratch[w]);
  return r;
}
__device__ __forceinline__ float block_sum(float v, float* scratch) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = scratch[0];
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) r += scratch[w];
  return r;
}

// One workgroup per row; the row (s FP16 values, s a multiple of 8) stays in LDS between the passes.
__global__ void __launch_bounds__(kThreads) xent_kernel(const _Float16* X, const int* target, float* loss, _Float16* dX, long rows, int s,
                                                        float s1, float beta) {
  extern __shared__ __attribute__((aligned(16))) uint8_t xent_lds[];
  _Float16* row = reinterpret_cast<_Float16*>(xent_lds);
  __shared__ float scratch[kThreads / 64];
  const int nchunks = s / 8;
  for (long r = blockIdx.x; r < rows; r += gridDim.x) {
    const int c = target[r];
    if (c < 0 || c >= s) {                              // a row without a label (uniform over the workgroup)
      if (loss && threadIdx.x == 0) loss[r] = 0.0f;
      if (dX)
        for (int i = threadIdx.x; i < nchunks; i += kThreads)
          *reinterpret_cast<v8h*>(dX + r * s + i * 8) = v8h{0, 0, 0, 0, 0, 0, 0, 0};
      continue;
    }
    float m = -__builtin_inff();
    // eight 16-byte loads per thread are requested before the first is used: with two workgroups per CU (the rows
    // fill the LDS) the bytes in flight have to come from each thread
    for (int i0 = threadIdx.x; i0 < nchunks; i0 += 8 * kThreads) {
      v8h v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * kThreads;
        if (i < nchunks) v[u] = *reinterpret_cast<const v8h*>(X + r * s + i * 8);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * kThreads;
        if (i < nchunks) {
          *reinterpret_cast<v8h*>(row + i * 8) = v[u];
#pragma unroll
          for (int q = 0; q < 8; ++q) m = __builtin_fmaxf(m, s1 * (float)v[u][q]);
        }
      }
    }
    m = block_max(m, scratch);                          // (its barriers also publish the row in LDS)
    float sum = 0.0f;
    for (int i = threadIdx.x; i < nchunks; i += kThreads) {
      const v8h v = *reinterpret_cast<const v8h*>(row + i * 8);
#pragma unroll
      for (int q = 0; q < 8; ++q) sum += __builtin_amdgcn_exp2f((s1 * (float)v[q] - m) * kLog2e);
    }
    sum = block_sum(sum, scratch);
    if (loss && threadIdx.x == 0) loss[r] = -(s1 * (float)row[c] - m - __builtin_logf(sum));
    if (dX) {
      const float inv = 1.0f / sum, bs = beta * s1;
      for (int i = threadIdx.x; i < nchunks; i += kThreads) {
        const v8h v = *reinterpret_cast<const v8h*>(row + i * 8);
        v8h o;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const float p = __builtin_amdgcn_exp2f((s1 * (float)v[q] - m) * kLog2e) * inv;
          o[q] = to_half(bs * (p - ((i * 8 + q) == c ? 1.0f : 0.0f)));
        }
        wt_store(reinterpret_cast<v8h*>(dX + r * s + i * 8), o);
      }
    }
    __syncthreads();                                    // the row in LDS is free for the next one
  }
}

// Scaled sum over the last dimension (Table A.2 "Linear": alpha = n^-1/2, beta = 1).  One wave per row; a lane adds every
// 64th 16-byte chunk, then the lanes are added by the butterfly: a fixed order, 2 B / element read.
__global__ void __launch_bounds__(kThreads) sum_fwd_kernel(const _Float16* X, _Float16* Y, long rows, int n, float alpha) {
  const int lane = threadIdx.x & 63;
  const long wave0 = (long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  const long nwaves = (long)gridDim.x * (kThreads / 64);
  const int nchunks = n / 8;
  for (long row = wave0; row < rows; row += nwaves) {
    const _Float16* x = X + row * n;
    float acc = 0.0f;
    for (int i = lane; i < nchunks; i += 64) {
      const v8h v = *reinterpret_cast<const v8h*>(x + i * 8);
#pragma unroll
      for (int q = 0; q < 8; ++q) acc += (float)v[q];
    }
    acc = wave_sum(acc);
    if (lane == 0) Y[row] = to_half(alpha * acc);
  }
}

// Its backward pass: dx_ij = beta * g_i in every column (write-only, 2 B / element).
__global__ void __launch_bounds__(kThreads) sum_bwd_kernel(const _Float16* G, _Float16* dX, long rows, int n, float beta) {
  const int lane = threadIdx.x & 63;
  const long wave0 = (long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  const long nwaves = (long)gridDim.x * (kThreads / 64);
  const int nchunks = n / 8;
  for (long row = wave0; row < rows; row += nwaves) {
    const _Float16 b = to_half(beta * (float)G[row]);
    const v8h o = {b, b, b, b, b, b, b, b};
    for (int i = lane; i < nchunks; i += 64) *reinterpret_cast<v8h*>(dX + row * n + i * 8) = o;
  }
}

int grid_rows(long rows) {
  long g = (rows + kThreads / 64 - 1) / (kThreads / 64);
  if (g > 256 * 16) g = 256 * 16;
  return (int)(g < 1 ? 1 : g);
}

}  // namespace

hipError_t launch_sum_fwd(const void* X, void* Y, long rows, long n, float alpha, hipStream_t st) {
  sum_fwd_kernel<<<grid_rows(rows), kThreads, 0, st>>>((const _Float16*)X, (_Float16*)Y, rows, (int)n, alpha);
  return hipGetLastError();
}

hipError_t launch_sum_bwd(const void* G, void* dX, long rows, long n, float beta, hipStream_t st) {
  sum_bwd_kernel<<<grid_rows(rows), kThreads, 0, st>>>((const _Float16*)G, (_Float16*)dX, rows, (int)n, beta);
  return hipGetLastError();
}

hipError_t launch_softmax_fwd(const void* X, void* Y, long rows, long s, float s1, float alpha, hipStream_t st) {
  const _Float16* x = (const _Float16*)X;
  _Float16* y = (_Float16*)Y;
  const int nch = (int)((s / 8 + 63) / 64), grid = grid_rows(rows);
  if (nch <= 1) softmax_fwd_kernel<1><<<grid, kThreads, 0, st>>>(x, y, rows, (int)s, s1, alpha);
  else if (nch <= 2) softmax_fwd_kernel<2><<<grid, kThreads, 0, st>>>(x, y, rows, (int)s, s1, alpha);
  else if (nch <= 4) softmax_fwd_kernel<4><<<grid, kThreads, 0, st>>>(x, y, rows, (int)s, s1, alpha);
  else softmax_fwd_kernel<8><<<grid, kThreads, 0, st>>>(x, y, rows, (int)s, s1, alpha);
  return hipGetLastError();
}

hipError_t launch_softmax_bwd(const void* X, const void* G, void* dX, long rows, long s, float s1, float beta, hipStream_t st) {
  const _Float16 *x = (const _Float16*)X, *g = (const _Float16*)G;
  _Float16* dx = (_Float16*)dX;
  const int nch = (int)((s / 8 + 63) / 64), grid = grid_rows(rows);
  if (nch <= 1) softmax_bwd_kernel<1><<<grid, kThreads, 0, st>>>(x, g, dx, rows, (int)s, s1, beta);
  else if (nch <= 2) softmax_bwd_kernel<2><<<grid, kThreads, 0, st>>>(x, g, dx, rows, (int)s, s1, beta);
  else if (nch <= 4) softmax_bwd_kernel<4><<<grid, kThreads, 0, st>>>(x, g, dx, rows, (int)s, s1, beta);
  else softmax_bwd_kernel<8><<<grid, kThreads, 0, st>>>(x, g, dx, rows, (int)s, s1, beta);
  return hipGetLastError();
}

hipError_t launch_softmax_xent(const void* X, const int* target, float* loss, void* dX, long rows, long s, float s1, float beta,
                               hipStream_t st) {
  static FuncConfig cfg;
  if (hipError_t e = cfg.ensure((const void*)xent_kernel, 128 * 1024); e != hipSuccess) return e;
  const int grid = (int)(rows < 256 * 8 ? rows : 256 * 8);
  xent_kernel<<<grid, kThreads, (size_t)s * 2, st>>>((const _Float16*)X, target, loss, (_Float16*)dX, rows, (int)s, s1, beta);
  return hipGetLastError();
}

}  // namespace us
