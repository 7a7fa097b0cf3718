// Pieces shared by the two GEMM kernels of the gfx950 library: argument block, tile configuration,
// matrix-core wrappers, workgroup -> tile mapping, and the epilogue that turns a wave's accumulator
// block into scaled FP16 / FP32 rows (optionally through GELU or GELU') with 128-bit global stores.
#pragma once

#include "us_device.h"

namespace us {

// EPI_GELU_TAB / EPI_GELU_GRAD_TAB: same results as EPI_GELU (FP8 activation only) / EPI_GELU_GRAD,
// taken from a table over the FP16 pre-activation that the workgroup copies into LDS.
// EPI_GELU_TAB16: EPI_GELU with an FP16 activation output (and optionally its FP8 copy), from a table.
// EPI_RESIDUAL: C = fp16( skip_scale * R + epi_scale * fp16(scale * acc) ), R an FP16 [M,N] input (Zpre).
enum GemmEpi : int {
  EPI_STORE = 0, EPI_GELU = 1, EPI_GELU_GRAD = 2, EPI_PARTIAL = 3, EPI_GELU_TAB = 4, EPI_GELU_GRAD_TAB = 5, EPI_GELU_TAB16 = 6,
  EPI_RESIDUAL = 7
};

//   C[M,N] = epilogue( scale * sum_k A(m,k) * B(n,k) )
// An operand is K-contiguous (element (r,k) at base[r*ld + k]) or K-strided (element (r,k) at
// base[k*ld + r]).
struct GemmArgs {
  const uint8_t* A;
  const uint8_t* B;
  void* C;
  long M, N, K;          // K = full reduction length
  long lda, ldb, ldc;    // elements
  long k_per_split;      // reduction range of one slice (blockIdx.y); a multiple of 128 elements
  float scale, epi_scale;
  float skip_scale;      // EPI_RESIDUAL: weight of the skip input
  int act;               // EPI_GELU / EPI_GELU_GRAD (arithmetic forms): which activation, 0 = gelu (us_device.h)
  const _Float16* Zpre;  // EPI_GELU_GRAD: saved pre-activation; EPI_RESIDUAL: skip input; [M,N], leading dimension ldc
  _Float16* aux16;       // EPI_GELU: optional FP16 activation output
  uint8_t* aux8;         // optional FP8 copy of the epilogue's FP16 result
  float* partial;        // EPI_PARTIAL: [splits][M][N] FP32
  const uint8_t* table;  // EPI_*_TAB: the table in global memory (us_device.h)
  long batch_a, batch_b, batch_c;   // bytes between consecutive problems of a batch (blockIdx.z), 0 for a single one
  const _Float16* bias;  // forward product only: optional row [N] added to scale * acc before the rounding, or NULL
  float* colsum;         // EPI_GELU_GRAD / _TAB: optional FP32 [ceil(M / 32)][N], column sums of the FP16 result per 32-row block
  int xcd_gm, xcd_gn;    // XCD rectangle split of the tile grid (0,0 = one rectangle)
  int grp_w;             // width of the column bands the rectangle is walked in
  int nxcd;              // XCDs of the device (workgroup id modulo this = the XCD a workgroup runs on)
};

// Problem number blockIdx.z of a batch of equally shaped, independent products (plain-store epilogue only).
__device__ __forceinline__ void select_batch_item(GemmArgs& g) {
  const long z = blockIdx.z;
  g.A += z * g.batch_a;
  g.B += z * g.batch_b;
  g.C = (uint8_t*)g.C + z * g.batch_c;
}

// Tile configuration.  BKB = bytes of K per row and pipeline stage; NST = LDS stage buffers;
// MINB = workgroups per CU the register allocation should allow.  WAVES_K > 1: that many groups of
// WAVES_M x WAVES_N waves work on the same output tile, each on its own share of every stage's k-steps;
// their accumulators are added through LDS before the epilogue (direct kernel only).
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int BKB_, int NST_, int MINB_, int WAVES_K_ = 1>
struct GemmCfg {
  static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, BKB = BKB_, NST = NST_, MINB = MINB_;
  static constexpr int WAVES_K = WAVES_K_;
  static constexpr int WAVES_MN = WAVES_M * WAVES_N;
  static constexpr int WAVES = WAVES_MN * WAVES_K;
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int FM = WM / 32, FN = WN / 32;   // 32x32 accumulator blocks per wave
};

#define US_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

template <int FA, int FB>
__device__ __forceinline__ v16f mfma_fp8(v8i a, v8i b, v16f c) {
  // format codes of the instruction: 0 = E4M3, 1 = E5M2; unit block scales
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, FA, FB, 0, 0, 0, 0);
}

// ---- workgroup -> output tile ------------------------------------------------------------------------
// Workgroups are handed to the device's XCDs round-robin by linear id, and every XCD has its own L2.  When
// the tile grid divides evenly (host: choose_xcd_grid), XCD x gets a compact rectangle of
// (tiles_m/gm) x (tiles_n/gn) tiles; with gm == 0 the whole grid is one rectangle.  Inside a
// rectangle the tiles are walked in column bands `grp_w` tiles wide, N-fastest within a band, so the
// ~32-64 workgroups that run at the same time on one XCD form a compact block and share the A and B
// panels they stream through that XCD's L2.
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int gm, int gn, int grp_w, int nxcd,
                                              int& tm, int& tn) {
  int rm = tiles_m, rn = tiles_n, base_m = 0, base_n = 0, idx = bid;
  if (gm != 0) {
    const int xcd = bid % nxcd;
    idx = bid / nxcd;
    rm = tiles_m / gm;
    rn = tiles_n / gn;
    base_m = (xcd % gm) * rm;
    base_n = (xcd / gm) * rn;
  }
  const int band = idx / (rm * grp_w);
  const int r = idx - band * rm * grp_w;
  const int w = (rn - band * grp_w < grp_w) ? rn - band * grp_w : grp_w;   // last band may be narrower
  tm = base_m + r / w;
  tn = base_n + band * grp_w + r % w;
}

// Host side: the split gm x gn = number of XCDs that divides the tile grid and minimises the operand bytes one XCD
// touches (bm, bn: the tile's rows of A and of B); gm = gn = 0 when the grid does not divide.
inline void choose_xcd_grid(long tiles_m, long tiles_n, int nxcd, int bm, int bn, int& gm, int& gn) {
  gm = gn = 0;
  if (nxcd < 2 || (tiles_m * tiles_n) % nxcd != 0) return;
  long best = -1;
  for (int c = 1; c <= nxcd; ++c) {
    if (nxcd % c) continue;
    const int cm = c, cn = nxcd / c;
    if (tiles_m % cm || tiles_n % cn) continue;
    const long cost = tiles_m / cm * bm + tiles_n / cn * bn;     // rows of A plus rows of B that one XCD reads
    if (best < 0 || cost < best) { best = cost; gm = cm; gn = cn; }
  }
}

// Results leave through write-through stores (wt_store, us_device.h); `streaming` only documents which of them no
// kernel reads soon (FP16 / FP32 results of tens of MB) and which the next launch reads (FP8 copies, FP16 activations).
// Measured on the BERT-large step, same box: non-temporal for the former and plain stores for the latter 242 us,
// write-through for the former only 238, for everything 230.5.
template <class V>
__device__ __forceinline__ void out_store(V* p, V v, bool /*streaming*/) { wt_store(p, v); }

// FP16 result of a GELU' epilogue (the operand of the next two matmuls unless an FP8 copy is written too).
__device__ __forceinline__ void store_grad(const GemmArgs& g, long idx, v8h r) {
  v8h* p = reinterpret_cast<v8h*>((_Float16*)g.C + idx);
  out_store(p, r, g.aux8 != nullptr);
}

// ---- epilogue on eight consecutive columns of one row (FP16 strip) ---------------------------------
// z: the saved pre-activation at the same eight positions (GELU' epilogues only; fetched by the caller
// well ahead of its use).
template <int EPI, int AUX_FMT>
__device__ __forceinline__ v8h epilogue_row8(const GemmArgs& g, long idx, v8h y, v8h z, const uint8_t* lut) {
  if (EPI == EPI_GELU_TAB) {
    out_store(reinterpret_cast<v8h*>((_Float16*)g.C + idx), y, true);   // the FP16 matmul result, kept for backward
    uint32_t c[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) c[k] = *US_LDS_PTR(const uint8_t, lut + half_bits(y[k]));
    v2i w;
    w.x = (int)(c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24));
    w.y = (int)(c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24));
    out_store(reinterpret_cast<v2i*>(g.aux8 + idx), w, false);
    return y;
  }
  if (EPI == EPI_GELU_TAB16) {
    out_store(reinterpret_cast<v8h*>((_Float16*)g.C + idx), y, true);   // the FP16 matmul result, kept for backward
    v8h r;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const uint32_t zb = half_bits(y[k]);
      const uint32_t a = zb & 0x7fffu;
      const uint32_t neg = zb >> 15;
      const uint32_t i = (a < (uint32_t)kGeluHalfLast ? a : (uint32_t)kGeluHalfLast) + neg * (uint32_t)(kGeluHalfLast + 1);
      _Float16 t = half_from_bits(*US_LDS_PTR(const unsigned short, lut + i * 2));
      // beyond the table: alpha_g * z for positive z (also +inf, NaN), -0 for finite negative z, NaN for -inf
      const _Float16 far = neg ? half_from_bits(a >= 0x7c00u ? 0x7e00u : 0x8000u) : to_half(g.epi_scale * (float)y[k]);
      r[k] = (a > (uint32_t)kGeluHalfLast) ? far : t;
    }
    if (g.aux16) out_store(reinterpret_cast<v8h*>(g.aux16 + idx), r, false);
    if (g.aux8) {
      const v2h p0 = {r[0], r[1]}, p1 = {r[2], r[3]}, p2 = {r[4], r[5]}, p3 = {r[6], r[7]};
      v2i w;
      w.x = (int)(cvt_pk_fp8_from_half<AUX_FMT>(p0) | (cvt_pk_fp8_from_half<AUX_FMT>(p1) << 16));
      w.y = (int)(cvt_pk_fp8_from_half<AUX_FMT>(p2) | (cvt_pk_fp8_from_half<AUX_FMT>(p3) << 16));
      out_store(reinterpret_cast<v2i*>(g.aux8 + idx), w, false);
    }
    return r;
  }
  if (EPI == EPI_GELU_GRAD_TAB) {
    // r = fp16(slope(z) * y), slope = table[|z|] for z >= 0 and epi_scale - table[|z|] for z < 0 (FP32), the product
    // rounded once.  Two elements per 32-bit word throughout: packed mask / clamp of the table index, and the
    // mixed-precision multiply writes each FP16 result straight into its half of the output word.
    typedef unsigned short v2us __attribute__((ext_vector_type(2)));
    v4i zw, yw, rw = {0, 0, 0, 0};
    __builtin_memcpy(&zw, &z, 16);
    __builtin_memcpy(&yw, &y, 16);
    const v2us last2 = {(unsigned short)kGeluSlopeLast, (unsigned short)kGeluSlopeLast};
    v2us amax = {0, 0};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t zq = (uint32_t)zw[q];
      const uint32_t a2 = zq & 0x7fff7fffu;                                    // |z| bits of both elements
      v2us av;
      __builtin_memcpy(&av, &a2, 4);
      amax = __builtin_elementwise_max(amax, av);
      const v2us iv = __builtin_elementwise_min(av, last2);                    // beyond 8 the slope is exactly epi_scale
      float t0 = *US_LDS_PTR(const float, lut + (uint32_t)iv.x * 4);
      float t1 = *US_LDS_PTR(const float, lut + (uint32_t)iv.y * 4);
      t0 = (zq & 0x8000u) ? g.epi_scale - t0 : t0;
      t1 = ((int)zq < 0) ? g.epi_scale - t1 : t1;
      uint32_t d = 0;
      mul_to_half<0, 0>(d, t0, (uint32_t)yw[q]);
      mul_to_half<1, 1>(d, t1, (uint32_t)yw[q]);
      rw[q] = (int)d;
    }
    v8h r;
    __builtin_memcpy(&r, &rw, 16);
    // +-inf and NaN pre-activations give NaN, as the arithmetic form does: rare, so the wave looks for one first
    if (__builtin_amdgcn_ballot_w64(amax.x >= 0x7c00u || amax.y >= 0x7c00u) != 0) {
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if ((half_bits(z[k]) & 0x7fffu) >= 0x7c00u) r[k] = half_from_bits(0x7e00u);
    }
    if (g.C) store_grad(g, idx, r);
    if (g.aux8) {
      const v2h p0 = {r[0], r[1]}, p1 = {r[2], r[3]}, p2 = {r[4], r[5]}, p3 = {r[6], r[7]};
      v2i w;
      w.x = (int)(cvt_pk_fp8_from_half<AUX_FMT>(p0) | (cvt_pk_fp8_from_half<AUX_FMT>(p1) << 16));
      w.y = (int)(cvt_pk_fp8_from_half<AUX_FMT>(p2) | (cvt_pk_fp8_from_half<AUX_FMT>(p3) << 16));
      out_store(reinterpret_cast<v2i*>(g.aux8 + idx), w, false);
    }
    return r;
  }
  if (EPI == EPI_STORE) {
    out_store(reinterpret_cast<v8h*>((_Float16*)g.C + idx), y, true);
    return y;
  }
  if (EPI == EPI_RESIDUAL) {
    // weighted addition of the skip input and the FP16-rounded matmul result (the residual layer's
    // interpolation): skip * R rounded to FP32, then one fused multiply-add, then the FP16 rounding
    v8h r;
#pragma unroll
    for (int k = 0; k < 8; ++k) r[k] = to_half(__builtin_fmaf(g.epi_scale, (float)y[k], g.skip_scale * (float)z[k]));
    out_store(reinterpret_cast<v8h*>((_Float16*)g.C + idx), r, true);
    return r;
  }
  v8h r;
  if (EPI == EPI_GELU) {
    out_store(reinterpret_cast<v8h*>((_Float16*)g.C + idx), y, true);   // the FP16 matmul result, kept for backward
#pragma unroll
    for (int k = 0; k < 8; ++k) r[k] = half_from_bits(0);
    if (g.act == 0) {      // uniform branch: gelu keeps its own short path, the other activations of Table A.2 share one
#pragma unroll
      for (int k = 0; k < 8; ++k) r[k] = to_half(gelu_scaled((float)y[k], g.epi_scale));
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) r[k] = to_half(act_scaled(g.act, (float)y[k], g.epi_scale));
    }
    if (g.aux16) out_store(reinterpret_cast<v8h*>(g.aux16 + idx), r, false);
  } else {  // EPI_GELU_GRAD: y is the FP16-rounded matmul gradient
#pragma unroll
    for (int k = 0; k < 8; ++k) r[k] = half_from_bits(0);
    if (g.act == 0) {
#pragma unroll
      for (int k = 0; k < 8; ++k) r[k] = gelu_grad_half(z[k], y[k], g.epi_scale);
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) r[k] = act_grad_half(g.act, (float)z[k], y[k], g.epi_scale);
    }
    if (g.C) store_grad(g, idx, r);      // optional: the FP8 copy may be all that is wanted
  }
  if (g.aux8) {
    // FP8 copy of the FP16 value just stored: identical to casting the stored tensor afterwards
    const v2h p0 = {r[0], r[1]}, p1 = {r[2], r[3]}, p2 = {r[4], r[5]}, p3 = {r[6], r[7]};
    v2i w;
    w.x = (int)(cvt_pk_fp8_from_half<AUX_FMT>(p0) | (cvt_pk_fp8_from_half<AUX_FMT>(p1) << 16));
    w.y = (int)(cvt_pk_fp8_from_half<AUX_FMT>(p2) | (cvt_pk_fp8_from_half<AUX_FMT>(p3) << 16));
    out_store(reinterpret_cast<v2i*>(g.aux8 + idx), w, false);
  }
  return r;
}

// Strip geometry: every wave owns 32 rows x WN values of LDS (FP16, or FP32 when WIDE).
template <class Cfg, bool WIDE, int EPI = EPI_STORE>
struct EpiStrip {
  static constexpr int ES = WIDE ? 4 : 2;
  static constexpr int PITCH = Cfg::WN * ES + 16;
  static constexpr int STRIP_BYTES = 32 * PITCH * Cfg::WAVES;
  static constexpr int TABLE_BYTES = EPI == EPI_GELU_TAB ? kGeluTableBytes
                                     : EPI == EPI_GELU_GRAD_TAB ? kGeluSlopeTableBytes
                                     : EPI == EPI_GELU_TAB16 ? kGeluHalfTableBytes : 0;
  static constexpr int BYTES = STRIP_BYTES + TABLE_BYTES;     // the table sits behind the strips
};

// The matrix core is fed with the N-side fragment as first operand, so register 4q+e of lane l of a
// 32x32 accumulator block holds (row l%32, column 8q + 4(l/32) + e).  Each wave pushes 32 rows of
// its block at a time through its LDS strip and reads them back row-contiguously: all global stores
// (and the read of the saved pre-activation) are 128-bit accesses sweeping whole rows.
// Must be entered after a workgroup barrier (the strips overlay the operand tiles).  A wave works on
// the 32-row blocks I0 .. I1-1 of its accumulators (all of them unless two wave groups share a tile:
// then each group finishes one half of the rows, see the wave-split reduction of the direct kernel).
// BIAS: the kernel is a forward product with an FP16 result and may be given a bias row (GemmArgs::bias); the
// other kernels do not carry the code.
template <bool A_KC, bool B_KC, int EPI, bool WIDE>
constexpr bool epilogue_takes_bias() {
  return A_KC && !B_KC && !WIDE &&
         (EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_GELU_TAB || EPI == EPI_GELU_TAB16 || EPI == EPI_RESIDUAL);
}

template <class Cfg, int EPI, bool WIDE, int I0 = 0, int I1 = Cfg::FM, bool BIAS = false>
__device__ __forceinline__ void store_block_epilogue(const GemmArgs& g, v16f (&acc)[Cfg::FM][Cfg::FN], uint8_t* lds,
                                                     long m0, long n0, long split) {
  static_assert(WIDE ? (EPI == EPI_STORE || EPI == EPI_PARTIAL) : (EPI != EPI_PARTIAL), "");
  using S = EpiStrip<Cfg, WIDE, EPI>;
  constexpr int AUX_FMT = (EPI == EPI_GELU_GRAD || EPI == EPI_GELU_GRAD_TAB) ? US_E5M2 : US_E4M3;
  const uint8_t* lut = lds + S::STRIP_BYTES;
  static_assert(S::TABLE_BYTES == 0 || Cfg::WAVES_K == 1, "the table copy below meets all waves at a barrier");
  // Bias row: register 4q+e of accumulator block j belongs to column j*32 + 8q + 4(lane/32) + e of the wave's
  // tile, so a lane needs four consecutive bias values per (j, q).  Requested first, so that the table copy
  // below (where there is one) is in flight at the same time.
  [[maybe_unused]] v4h bias4[BIAS ? Cfg::FN : 1][4] = {};
  [[maybe_unused]] bool has_bias = false;
  if constexpr (BIAS) {
    has_bias = g.bias != nullptr;
    if (has_bias) {
      const long nb0 = n0 + ((threadIdx.x >> 6) % Cfg::WAVES_MN / Cfg::WAVES_M) * Cfg::WN + 4 * ((threadIdx.x & 63) >> 5);
#pragma unroll
      for (int j = 0; j < Cfg::FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const long n = nb0 + j * 32 + 8 * q;
          if (n < g.N) bias4[j][q] = *reinterpret_cast<const v4h*>(g.bias + n);
        }
    }
  }
  if constexpr (S::TABLE_BYTES > 0) {
    // copy the table into LDS: whole 1 KB wave loads, 16 bytes per lane, spread over the waves
    for (int c = threadIdx.x >> 6; c < S::TABLE_BYTES / 1024; c += Cfg::WAVES)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(g.table + c * 1024 + (threadIdx.x & 63) * 16),
          US_LDS_PTR(void, lds + S::STRIP_BYTES + c * 1024), 16, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of the table has landed
    __syncthreads();
  }
  constexpr int EP = S::PITCH;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int wmn = wave % Cfg::WAVES_MN;
  const int wm0 = (wmn % Cfg::WAVES_M) * Cfg::WM;
  const int wn0 = (wmn / Cfg::WAVES_M) * Cfg::WN;
  uint8_t* strip = lds + wave * (32 * EP);
  const float scale = (EPI == EPI_PARTIAL) ? 1.0f : g.scale;
  constexpr int NI = I1 - I0;                        // 32-row blocks this wave finishes
  constexpr int CPR = Cfg::WN * S::ES / 16;          // 16-byte chunks per strip row
  constexpr int PER_LANE = 32 * CPR / 64;
  // GELU' / residual: the second input of the epilogue (saved pre-activation, skip tensor) is requested
  // ahead of its use, for ZGROUP strips at a time and before any store of that group.  Loads and stores
  // share one in-order completion counter here, so a load issued between stores could only be waited for
  // together with every store before it (each one an HBM round trip); GELU' therefore fetches its whole
  // share first and never waits for a store.  The residual epilogue has little arithmetic to hide
  // behind and a tighter register budget (its kernels also hold the wave-split reduction), so it
  // fetches two strips at a time and accepts one store drain in the middle.
  constexpr bool NEEDS_Z = (EPI == EPI_GELU_GRAD || EPI == EPI_GELU_GRAD_TAB || EPI == EPI_RESIDUAL);
  constexpr int ZGROUP = !NEEDS_Z ? 1 : (EPI == EPI_RESIDUAL && NI > 2) ? 2 : NI;
  static_assert(NI % ZGROUP == 0, "");
  v8h zpre[ZGROUP][NEEDS_Z ? PER_LANE : 1] = {};
  auto fetch_group = [&](int i0) {
    if constexpr (NEEDS_Z) {
#pragma unroll
      for (int ii = 0; ii < ZGROUP; ++ii)
#pragma unroll
        for (int u = 0; u < PER_LANE; ++u) {
          const int c = lane + u * 64;
          const long m = m0 + wm0 + (I0 + i0 + ii) * 32 + c / CPR;
          const long n = n0 + wn0 + (c % CPR) * 8;
          if (m < g.M && n < g.N) zpre[ii][u] = *reinterpret_cast<const v8h*>(g.Zpre + m * g.ldc + n);
        }
    }
  };
  // Column sums of the FP16 result (the bias gradient of the layer below the activation): a lane always works on
  // the same 8 columns (CPR divides 64), so it adds its rows up in registers; the lanes of a column group are added
  // at the end and the wave writes one FP32 row per 32-row block it finished (the sum in the first, zeros in the
  // others), so that every row of GemmArgs::colsum is written exactly once per column, in an order that is fixed.
  constexpr bool CAN_COLSUM = (EPI == EPI_GELU_GRAD || EPI == EPI_GELU_GRAD_TAB) && !WIDE && (64 % CPR == 0);
  [[maybe_unused]] float cs[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
  [[maybe_unused]] bool want_colsum = false;
  if constexpr (CAN_COLSUM) want_colsum = g.colsum != nullptr;
  fetch_group(0);
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    auto to_strip = [&](auto with_bias) {
#pragma unroll
      for (int j = 0; j < Cfg::FN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = j * 32 + 8 * q + 4 * (lane >> 5);
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if constexpr (decltype(with_bias)::value)
              v[e] = __builtin_fmaf(acc[I0 + i][j][4 * q + e], scale, (float)bias4[j][q][e]);   // one rounding of the sum
            else
              v[e] = acc[I0 + i][j][4 * q + e] * scale;
          }
          uint8_t* p = strip + (lane & 31) * EP + col * S::ES;
          if (WIDE) {
            v4f o = {v[0], v[1], v[2], v[3]};
            *US_LDS_PTR(v4f, p) = o;
          } else {
            v4h o = {to_half(v[0]), to_half(v[1]), to_half(v[2]), to_half(v[3])};
            *US_LDS_PTR(v4h, p) = o;
          }
        }
      }
    };
    if constexpr (BIAS) {
      if (has_bias) to_strip(std::true_type{});
      else to_strip(std::false_type{});
    } else {
      to_strip(std::false_type{});
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // one unconditional wait for the pre-activation loads: the uses below sit in bounds-checked
    // branches, where the compiler would otherwise wait again and again, by then for the stores too
    if (NEEDS_Z && i % ZGROUP == 0) {
      if (i > 0) fetch_group(i);
      __builtin_amdgcn_s_waitcnt(0x0F70);
    }
#pragma unroll
    for (int u = 0; u < PER_LANE; ++u) {
      const int c = lane + u * 64;
      const int row = c / CPR, cc = c % CPR;
      const long m = m0 + wm0 + (I0 + i) * 32 + row;
      const long n = n0 + wn0 + cc * (16 / S::ES);
      const uint8_t* p = strip + row * EP + cc * 16;
      if (m < g.M && n < g.N) {
        if (WIDE) {
          v4f v = *US_LDS_PTR(const v4f, p);
          if (EPI == EPI_PARTIAL)
            *reinterpret_cast<v4f*>(g.partial + (size_t)split * g.M * g.N + m * g.N + n) = v;
          else
            out_store(reinterpret_cast<v4f*>((float*)g.C + m * g.ldc + n), v, true);
        } else {
          v8h y = *US_LDS_PTR(const v8h, p);
          const v8h r = epilogue_row8<EPI, AUX_FMT>(g, m * g.ldc + n, y, zpre[NEEDS_Z ? i % ZGROUP : 0][NEEDS_Z ? u : 0], lut);
          if constexpr (CAN_COLSUM) {
            if (want_colsum) {
#pragma unroll
              for (int k = 0; k < 8; ++k) cs[k] += (float)r[k];
            }
          }
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  if constexpr (CAN_COLSUM) {
    if (want_colsum) {
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int off = CPR; off < 64; off <<= 1) cs[k] += __shfl_xor(cs[k], off, 64);
      const long n = n0 + wn0 + lane * 8;                       // lanes 0 .. CPR-1 hold the wave's WN columns
      const long p0 = (m0 + wm0 + I0 * 32) / 32;                // first 32-row block this wave finished
      const long prows = (g.M + 31) / 32;
      if (lane < CPR && n < g.N) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          if (p0 + i < prows) {
            float* o = g.colsum + (p0 + i) * g.N + n;
            const v4f lo = {i == 0 ? cs[0] : 0.0f, i == 0 ? cs[1] : 0.0f, i == 0 ? cs[2] : 0.0f, i == 0 ? cs[3] : 0.0f};
            const v4f hi = {i == 0 ? cs[4] : 0.0f, i == 0 ? cs[5] : 0.0f, i == 0 ? cs[6] : 0.0f, i == 0 ? cs[7] : 0.0f};
            *reinterpret_cast<v4f*>(o) = lo;
            *reinterpret_cast<v4f*>(o + 4) = hi;
          }
        }
      }
    }
  }
}

}  // namespace us
