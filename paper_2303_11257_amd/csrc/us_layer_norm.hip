// Scaled layer norm (Table A.2 "Other"): Y_ij = c_j + w_j (X_ij - mu_i) / sigma_i, alpha = beta_x = 1,
// beta_w = beta_c = b^-1/2.  HBM-bound row kernels: one wave owns a row and keeps it in registers
// (FP16 storage, FP32 arithmetic), so every tensor is read or written exactly once:
//   forward   reads X, writes Y                                   4 B / element
//   backward  reads X and G, writes dX, and leaves per-row-block column sums of G*xhat and G in a
//             workspace; a second small kernel adds the blocks in order (deterministic)      6 B / element
#include "us_launch.h"
#include "us_rows.h"

namespace us {

namespace {

constexpr int kLnThreads = 256;       // four waves, one row each at a time
constexpr int kLnRowsPerBlock = 32;   // fewest rows whose column sums one workgroup accumulates (backward; sizes the scratch)

// mean and 1/sqrt(variance + eps) of the row held in x (two passes over the registers)
template <int NCH>
__device__ __forceinline__ void row_stats(const RowRegs<NCH>& x, int n, int lane, float eps, float& mean, float& rstd) {
  float s = 0.0f;
#pragma unroll
  for (int k = 0; k < NCH; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) s += (float)x.v[k][e];
  mean = wave_sum(s) / (float)n;
  float q = 0.0f;
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const bool valid = (k * 64 + lane) * 8 < n;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float d = (float)x.v[k][e] - mean;
      q += valid ? d * d : 0.0f;
    }
  }
  rstd = 1.0f / __builtin_sqrtf(wave_sum(q) / (float)n + eps);
}

template <int NCH>
__global__ void __launch_bounds__(kLnThreads) ln_fwd_kernel(const _Float16* X, const _Float16* w, const _Float16* c, _Float16* Y,
                                                           long b, int n, float eps) {
  const int lane = threadIdx.x & 63;
  const long wave0 = (long)blockIdx.x * (kLnThreads / 64) + (threadIdx.x >> 6);
  const long nwaves = (long)gridDim.x * (kLnThreads / 64);
  RowRegs<NCH> wr, cr;
  wr.load(w, n, lane);
  cr.load(c, n, lane);
  for (long row = wave0; row < b; row += nwaves) {
    RowRegs<NCH> x;
    x.load(X + row * n, n, lane);
    float mean, rstd;
    row_stats<NCH>(x, n, lane, eps, mean, rstd);
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int col = (k * 64 + lane) * 8;
      if (col < n) {
        v8h o;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          o[e] = to_half(__builtin_fmaf(((float)x.v[k][e] - mean) * rstd, (float)wr.v[k][e], (float)cr.v[k][e]));
        wt_store(reinterpret_cast<v8h*>(Y + row * n + col), o);
      }
    }
  }
}

// Backward: dX for kLnRowsPerBlock rows per workgroup, and that block's column sums of G*xhat and G
// into partial[block][2][n] (FP32).  LDS: the four waves' sums before they are added in wave order.
template <int NCH>
__global__ void __launch_bounds__(kLnThreads) ln_bwd_kernel(const _Float16* X, const _Float16* w, const _Float16* G, _Float16* dX,
                                                           float* partial, long b, int n, float eps, int rows_per_block) {
  extern __shared__ __attribute__((aligned(16))) float red[];     // [4 waves][2][n]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long row0 = (long)blockIdx.x * rows_per_block;
  RowRegs<NCH> wr;
  wr.load(w, n, lane);
  float aw[NCH][8], ac[NCH][8];
#pragma unroll
  for (int k = 0; k < NCH; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) aw[k][e] = ac[k][e] = 0.0f;
  // the next row of this wave is requested before the current one is worked on
  RowRegs<NCH> x, g, xn, gn;
  if (row0 + wave < b) {
    xn.load(X + (row0 + wave) * n, n, lane);
    gn.load(G + (row0 + wave) * n, n, lane);
  }
  for (int r = wave; r < rows_per_block; r += kLnThreads / 64) {
    const long row = row0 + r;
    if (row >= b) break;
    x = xn;
    g = gn;
    const long next = row + kLnThreads / 64;
    if (r + kLnThreads / 64 < rows_per_block && next < b) {
      xn.load(X + next * n, n, lane);
      gn.load(G + next * n, n, lane);
    }
    float mean, rstd;
    row_stats<NCH>(x, n, lane, eps, mean, rstd);
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const bool valid = (k * 64 + lane) * 8 < n;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xh = valid ? ((float)x.v[k][e] - mean) * rstd : 0.0f;
        const float gi = (float)g.v[k][e];
        const float gh = gi * (float)wr.v[k][e];
        s1 += gh;
        s2 += gh * xh;
        aw[k][e] += gi * xh;
        ac[k][e] += gi;
      }
    }
    const float m1 = wave_sum(s1) / (float)n, m2 = wave_sum(s2) / (float)n;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int col = (k * 64 + lane) * 8;
      if (col < n) {
        v8h o;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = ((float)x.v[k][e] - mean) * rstd;
          const float gh = (float)g.v[k][e] * (float)wr.v[k][e];
          o[e] = to_half(rstd * (gh - m1 - xh * m2));
        }
        wt_store(reinterpret_cast<v8h*>(dX + row * n + col), o);
      }
    }
  }
  // the block's column sums: waves in order 0, 1, 2, 3
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int col = (k * 64 + lane) * 8;
    if (col < n) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        red[(wave * 2 + 0) * n + col + e] = aw[k][e];
        red[(wave * 2 + 1) * n + col + e] = ac[k][e];
      }
    }
  }
  __syncthreads();
  float* out = partial + (size_t)blockIdx.x * 2 * n;
  for (int i = threadIdx.x; i < 2 * n; i += kLnThreads) {
    float s = red[i];
#pragma unroll
    for (int wv = 1; wv < kLnThreads / 64; ++wv) s += red[wv * 2 * n + i];
    out[i] = s;
  }
}

// dw_j = beta * sum over blocks of partial[blk][0][j], dc_j likewise from partial[blk][1][j].  A workgroup takes
// 16 of the 2n columns; thread (seg, col) adds the blocks seg, seg + 16, ... (eight independent loads in flight),
// then the 16 segment sums are added in segment order: a fixed association, so the result is reproducible.
__global__ void __launch_bounds__(256) ln_reduce_kernel(const float* partial, _Float16* dw, _Float16* dc, int nblocks, int n,
                                                        float beta) {
  __shared__ float seg_sum[16][17];
  const int col = threadIdx.x & 15, seg = threadIdx.x >> 4;
  const int i = blockIdx.x * 16 + col;               // 0 .. 2n-1 (2n is a multiple of 16)
  const float* p = partial + i;
  const size_t stride = (size_t)2 * n;
  float s = 0.0f;
  int blk = seg;
  for (; blk + 7 * 16 < nblocks; blk += 8 * 16) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[(size_t)(blk + u * 16) * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; blk < nblocks; blk += 16) s += p[(size_t)blk * stride];
  seg_sum[seg][col] = s;
  __syncthreads();
  if (seg == 0) {
    float t = seg_sum[0][col];
#pragma unroll
    for (int k = 1; k < 16; ++k) t += seg_sum[k][col];
    const _Float16 o = to_half(beta * t);
    if (i < n) dw[i] = o;
    else dc[i - n] = o;
  }
}

int grid_rows(long b) {
  long g = (b + kLnThreads / 64 - 1) / (kLnThreads / 64);
  if (g > 256 * 16) g = 256 * 16;
  return (int)(g < 1 ? 1 : g);
}

}  // namespace

size_t layer_norm_workspace_bytes(long b, long n) {
  return (size_t)((b + kLnRowsPerBlock - 1) / kLnRowsPerBlock) * 2 * (size_t)n * sizeof(float);
}

hipError_t launch_layer_norm_fwd(const void* X, const void* w, const void* c, void* Y, long b, long n, float eps, hipStream_t st) {
  const _Float16 *x = (const _Float16*)X, *wp = (const _Float16*)w, *cp = (const _Float16*)c;
  _Float16* y = (_Float16*)Y;
  const int nch = (int)((n / 8 + 63) / 64), grid = grid_rows(b);
  if (nch <= 1) ln_fwd_kernel<1><<<grid, kLnThreads, 0, st>>>(x, wp, cp, y, b, (int)n, eps);
  else if (nch <= 2) ln_fwd_kernel<2><<<grid, kLnThreads, 0, st>>>(x, wp, cp, y, b, (int)n, eps);
  else if (nch <= 4) ln_fwd_kernel<4><<<grid, kLnThreads, 0, st>>>(x, wp, cp, y, b, (int)n, eps);
  else ln_fwd_kernel<8><<<grid, kLnThreads, 0, st>>>(x, wp, cp, y, b, (int)n, eps);
  return hipGetLastError();
}

template <int NCH>
static hipError_t launch_bwd(const _Float16* x, const _Float16* w, const _Float16* g, _Float16* dx, float* partial, long b, int n,
                             float eps, int nblocks, int rows_per_block, hipStream_t st) {
  const int lds = (kLnThreads / 64) * 2 * n * (int)sizeof(float);
  static FuncConfig cfg;
  if (hipError_t e = cfg.ensure((const void*)ln_bwd_kernel<NCH>, 160 * 1024); e != hipSuccess) return e;
  ln_bwd_kernel<NCH><<<nblocks, kLnThreads, lds, st>>>(x, w, g, dx, partial, b, n, eps, rows_per_block);
  return hipGetLastError();
}

hipError_t launch_layer_norm_bwd(const void* X, const void* w, const void* G, void* dX, void* dw, void* dc, long b, long n, float eps,
                                 float beta_wc, void* workspace, hipStream_t st) {
  const _Float16 *x = (const _Float16*)X, *wp = (const _Float16*)w, *g = (const _Float16*)G;
  const int nch = (int)((n / 8 + 63) / 64);
  // at most 4096 workgroups: beyond that each takes more rows (a multiple of the minimum, so the scratch suffices)
  long rpb = kLnRowsPerBlock;
  while ((b + rpb - 1) / rpb > 4096) rpb *= 2;
  const int nblocks = (int)((b + rpb - 1) / rpb);
  float* partial = (float*)workspace;
  hipError_t e;
  if (nch <= 1) e = launch_bwd<1>(x, wp, g, (_Float16*)dX, partial, b, (int)n, eps, nblocks, (int)rpb, st);
  else if (nch <= 2) e = launch_bwd<2>(x, wp, g, (_Float16*)dX, partial, b, (int)n, eps, nblocks, (int)rpb, st);
  else if (nch <= 4) e = launch_bwd<4>(x, wp, g, (_Float16*)dX, partial, b, (int)n, eps, nblocks, (int)rpb, st);
  else e = launch_bwd<8>(x, wp, g, (_Float16*)dX, partial, b, (int)n, eps, nblocks, (int)rpb, st);
  if (e != hipSuccess) return e;
  ln_reduce_kernel<<<(unsigned)(2 * n / 16), 256, 0, st>>>(partial, (_Float16*)dw, (_Float16*)dc, nblocks, (int)n, beta_wc);
  return hipGetLastError();
}

}  // namespace us
