// Gradient of a bias row: dc[j] = beta * sum over the rows of G[b,n] (App. J.1's ffn has b1, b2; beta = b^-1/2 like
// the bias of the scaled layer norm in Table A.2).  Read-only over G, HBM-bound: one pass, 2 bytes per element
// (1 for FP8 codes).  Two kernels, both with a fixed order of additions (reproducible results): column sums per
// block of 32 rows into an FP32 scratch [blocks][n], then the sum over the blocks, scaled and rounded to FP16.
#include "us_device.h"
#include "us_launch.h"

namespace us {

namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = 32;      // fewest rows a workgroup sums (sizes the scratch); more when there are many rows

template <int DT, int V>
__device__ __forceinline__ void add_chunk(float (&acc)[V], const v4i& raw) {
  if constexpr (DT == US_F16) {
    const v8h h = __builtin_bit_cast(v8h, raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += (float)h[e];
  } else {
#pragma unroll
    for (int w = 0; w < 4; ++w) {      // the byte select of the conversion is an immediate
      if constexpr (DT == US_E4M3) {
        acc[w * 4 + 0] += __builtin_amdgcn_cvt_f32_fp8(raw[w], 0);
        acc[w * 4 + 1] += __builtin_amdgcn_cvt_f32_fp8(raw[w], 1);
        acc[w * 4 + 2] += __builtin_amdgcn_cvt_f32_fp8(raw[w], 2);
        acc[w * 4 + 3] += __builtin_amdgcn_cvt_f32_fp8(raw[w], 3);
      } else {
        acc[w * 4 + 0] += __builtin_amdgcn_cvt_f32_bf8(raw[w], 0);
        acc[w * 4 + 1] += __builtin_amdgcn_cvt_f32_bf8(raw[w], 1);
        acc[w * 4 + 2] += __builtin_amdgcn_cvt_f32_bf8(raw[w], 2);
        acc[w * 4 + 3] += __builtin_amdgcn_cvt_f32_bf8(raw[w], 3);
      }
    }
  }
}

// Thread (rsub, cw): 16-byte chunk cw of the block's column range, rows row0 + rsub, row0 + rsub + RS, ...
// cpr = chunks per row, CW = chunks this block covers (at most 256), RS = 256 / CW rows side by side.
template <int DT>
__global__ void __launch_bounds__(kThreads) colsum_kernel(const uint8_t* G, float* partial, long b, long n, int cpr, int cw_count,
                                                          int rs, int rows_per_block) {
  constexpr int V = DT == US_F16 ? 8 : 16;
  __shared__ float red[kThreads * V];
  const int cw = threadIdx.x % cw_count, rsub = threadIdx.x / cw_count;
  const int chunk = blockIdx.y * 256 + cw;
  const bool active = rsub < rs && chunk < cpr;
  float acc[V] = {};
  if (active) {
    const long row0 = (long)blockIdx.x * rows_per_block;
    const long row1 = row0 + rows_per_block < b ? row0 + rows_per_block : b;
    const size_t pitch = (size_t)cpr * 16;
    const uint8_t* p = G + (size_t)chunk * 16;
    long r = row0 + rsub;
    for (; r + 3L * rs < row1; r += 4L * rs) {        // four independent loads in flight, added in row order
      v4i x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u] = *reinterpret_cast<const v4i*>(p + (size_t)(r + (long)u * rs) * pitch);
#pragma unroll
      for (int u = 0; u < 4; ++u) add_chunk<DT, V>(acc, x[u]);
    }
    for (; r < row1; r += rs) add_chunk<DT, V>(acc, *reinterpret_cast<const v4i*>(p + (size_t)r * pitch));
  }
  if (rs > 1) {                                       // row lanes 0, 1, ... of a chunk are added in that order
#pragma unroll
    for (int e = 0; e < V; ++e) red[(rsub * cw_count + cw) * V + e] = acc[e];
    __syncthreads();
    if (active && rsub == 0)
      for (int q = 1; q < rs; ++q)
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += red[(q * cw_count + cw) * V + e];
  }
  if (active && rsub == 0) {
    float* out = partial + (size_t)blockIdx.x * n + (size_t)chunk * V;
#pragma unroll
    for (int e = 0; e < V; e += 4) *reinterpret_cast<v4f*>(out + e) = v4f{acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
  }
}

// dc_j = beta * sum over blocks of partial[blk][j]: a workgroup takes 16 columns; thread (seg, col) adds the blocks
// seg, seg + 16, ..., then the 16 segment sums are added in segment order.
__global__ void __launch_bounds__(256) colsum_reduce_kernel(const float* partial, _Float16* dc, int nblocks, long n, float beta) {
  __shared__ float seg_sum[16][17];
  const int col = threadIdx.x & 15, seg = threadIdx.x >> 4;
  const long j = (long)blockIdx.x * 16 + col;
  const float* p = partial + j;
  float s = 0.0f;
  int blk = seg;
  for (; blk + 7 * 16 < nblocks; blk += 8 * 16) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[(size_t)(blk + u * 16) * n];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; blk < nblocks; blk += 16) s += p[(size_t)blk * n];
  seg_sum[seg][col] = s;
  __syncthreads();
  if (seg == 0) {
    float t = seg_sum[0][col];
#pragma unroll
    for (int k = 1; k < 16; ++k) t += seg_sum[k][col];
    dc[j] = to_half(beta * t);
  }
}

}  // namespace

size_t bias_grad_workspace_bytes(long b, long n) {
  if (b <= 0 || n <= 0) return 0;
  return (size_t)((b + kRowsPerBlock - 1) / kRowsPerBlock) * (size_t)n * sizeof(float);
}

hipError_t launch_bias_grad(const void* G, us_dtype g_dt, void* dc, long b, long n, float beta, void* workspace, hipStream_t st) {
  const int es = g_dt == US_F16 ? 2 : 1;
  const int cpr = (int)(n * es / 16);
  const int cw = cpr < 256 ? cpr : 256;
  const int rs = 256 / cw;
  // at most 2048 workgroups: beyond that each takes more rows (a multiple of the minimum, so the scratch suffices)
  long rpb = kRowsPerBlock;
  while ((b + rpb - 1) / rpb > 2048) rpb *= 2;
  const int nblocks = (int)((b + rpb - 1) / rpb);
  dim3 grid((unsigned)nblocks, (unsigned)((cpr + 255) / 256), 1);
  float* partial = (float*)workspace;
  const uint8_t* g = (const uint8_t*)G;
  if (nblocks > 0) {                       // no rows: the sums are empty and the second kernel writes zeros
    if (g_dt == US_F16) colsum_kernel<US_F16><<<grid, kThreads, 0, st>>>(g, partial, b, n, cpr, cw, rs, (int)rpb);
    else if (g_dt == US_E4M3) colsum_kernel<US_E4M3><<<grid, kThreads, 0, st>>>(g, partial, b, n, cpr, cw, rs, (int)rpb);
    else colsum_kernel<US_E5M2><<<grid, kThreads, 0, st>>>(g, partial, b, n, cpr, cw, rs, (int)rpb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  colsum_reduce_kernel<<<(unsigned)(n / 16), 256, 0, st>>>(partial, (_Float16*)dc, nblocks, n, beta);
  return hipGetLastError();
}

hipError_t launch_bias_grad_reduce(const void* partial, void* dc, long nblocks, long n, float beta, hipStream_t st) {
  colsum_reduce_kernel<<<(unsigned)(n / 16), 256, 0, st>>>((const float*)partial, (_Float16*)dc, (int)nblocks, n, beta);
  return hipGetLastError();
}

}  // namespace us
