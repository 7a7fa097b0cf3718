// LDS-tiled MFMA GEMM for gfx950 with the unit scale (and optionally GELU / GELU') in the epilogue.
//
//   C[M,N] = epilogue( scale * sum_k A(m,k) * B(n,k) )
//
// Each operand is either K-contiguous (element (r,k) at base[r*ld + k]) or K-strided (element (r,k)
// at base[k*ld + r]); the strided case is what the forward weight and both grad_W operands look
// like in memory, and it is served without a transposed copy: the tile is staged in LDS exactly as
// it lies in HBM and the matrix-core fragments are fetched with the transposing LDS reads
// (ds_read_b64_tr_b8 / _tr_b16), which hand each lane eight (four) consecutive k of one row.
//
// Work decomposition: a workgroup of 4 waves owns a BM x BN output tile; the waves form a
// WAVES_M x WAVES_N grid and each keeps (BM/WAVES_M) x (BN/WAVES_N) accumulators in registers as
// 32x32 MFMA blocks.  K is consumed in stages of 128 bytes per row (128 FP8 or 64 FP16 values),
// double-buffered in LDS: the loads of stage s+1 are issued before the MFMAs of stage s.
//   FP8 : v_mfma_f32_32x32x64_f8f6f4 (E4M3 / E5M2 selectable per operand), 2 per stage and block
//   FP16: v_mfma_f32_32x32x16_f16, 4 per stage and block
// The matrix core is fed with the N-side fragment as its first operand, so a lane ends up with four
// consecutive columns of one output row per accumulator quad and can store 8-byte FP16 groups.
#pragma once

#include "us_device.h"

namespace us {

constexpr int kGemmThreads = 256;
constexpr int kStageBytes = 128;  // bytes of K per row and pipeline stage

enum GemmEpi : int { EPI_STORE = 0, EPI_GELU = 1, EPI_GELU_GRAD = 2, EPI_PARTIAL = 3 };

struct GemmArgs {
  const uint8_t* A;
  const uint8_t* B;
  void* C;
  long M, N, K;          // K = full reduction length
  long lda, ldb, ldc;    // elements
  long k_per_split;      // reduction range handled by one z-slice of the grid (multiple of the stage)
  float scale, epi_scale;
  int c_is_f32;
  const _Float16* Zpre;
  _Float16* aux16;
  uint8_t* aux8;
  float* partial;        // EPI_PARTIAL: [splits][M][N] FP32
};

template <int BM, int BN, bool FP8, bool A_KC, bool B_KC>
struct GemmTile {
  static constexpr int ES = FP8 ? 1 : 2;                 // element size
  static constexpr int BK = kStageBytes / ES;            // elements of K per stage
  // K-contiguous tile: rows x 128 B, padded by 16 B so that 8 consecutive rows hit distinct banks.
  static constexpr int PITCH_KC = kStageBytes + 16;
  // K-strided tile: BK rows of (rows * ES) bytes, padded by 32 B (conflict-free for the tr reads).
  static constexpr int PITCH_A_KS = BM * ES + 32;
  static constexpr int PITCH_B_KS = BN * ES + 32;
  static constexpr int A_BYTES = A_KC ? BM * PITCH_KC : BK * PITCH_A_KS;
  static constexpr int B_BYTES = B_KC ? BN * PITCH_KC : BK * PITCH_B_KS;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int A_CHUNKS = BM * kStageBytes / 16;  // 16-byte chunks per stage
  static constexpr int B_CHUNKS = BN * kStageBytes / 16;
  static constexpr int A_PER_THREAD = A_CHUNKS / kGemmThreads;
  static constexpr int B_PER_THREAD = B_CHUNKS / kGemmThreads;
};

#define US_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// ---- global -> registers -> LDS staging of one operand tile ----------------------------------------
// rows: tile rows (BM or BN) starting at row0 of `extent_r`; k0: first k of the stage; k_end: end of
// this slice's reduction range.  Chunks outside the matrix are zero.
template <int ROWS, bool KC, int ES, int NCH>
__device__ __forceinline__ void load_tile_regs(const uint8_t* __restrict__ base, long ld, long row0, long extent_r,
                                               long k0, long k_end, v4i (&regs)[NCH]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = t + i * kGemmThreads;
    long r, k;
    const uint8_t* p;
    if (KC) {
      const int row = c >> 3, kc = c & 7;  // 8 chunks of 16 B per row
      r = row0 + row;
      k = k0 + kc * (16 / ES);
      p = base + (r * ld + k) * ES;
    } else {
      constexpr int CPR = ROWS * ES / 16;  // chunks per k-row
      const int krow = c / CPR, rc = c % CPR;
      r = row0 + rc * (16 / ES);
      k = k0 + krow;
      p = base + (k * ld + r) * ES;
    }
    v4i v = {0, 0, 0, 0};
    if (r < extent_r && k < k_end) v = *reinterpret_cast<const v4i*>(p);
    regs[i] = v;
  }
}

template <int ROWS, bool KC, int ES, int PITCH, int NCH>
__device__ __forceinline__ void store_tile_lds(uint8_t* lds, const v4i (&regs)[NCH]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = t + i * kGemmThreads;
    int off;
    if (KC) {
      off = (c >> 3) * PITCH + (c & 7) * 16;
    } else {
      constexpr int CPR = ROWS * ES / 16;
      off = (c / CPR) * PITCH + (c % CPR) * 16;
    }
    *US_LDS_PTR(v4i, lds + off) = regs[i];
  }
}

// ---- LDS -> matrix-core fragment --------------------------------------------------------------------
// Fragment = 32 rows (r0..r0+31) x one MFMA's worth of k starting at byte/element ks of the stage.
// Lane l supplies row r0 + l%32 and the k-half l/32 (FP8: 32 consecutive k; FP16: 8 consecutive k).
template <bool KC, int PITCH>
__device__ __forceinline__ v8i load_frag_fp8(const uint8_t* tile, int r0, int kstep) {
  const int l = threadIdx.x & 63;
  v8i f;
  if (KC) {
    const uint8_t* p = tile + (r0 + (l & 31)) * PITCH + kstep * 64 + (l >> 5) * 32;
    v4i lo = *US_LDS_PTR(const v4i, p);
    v4i hi = *US_LDS_PTR(const v4i, p + 16);
    f = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  } else {
    // 16 lanes cooperate on an 8(k) x 16(row) byte block; lane i of the group points at k-row i/2,
    // row-half i%2, and receives the 8 k values of row (group base + i).
    const int i = l & 15;
    const uint8_t* p = tile + (kstep * 64 + (l >> 5) * 32 + (i >> 1)) * PITCH + r0 + ((l >> 4) & 1) * 16 + (i & 1) * 8;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      v2i v = __builtin_amdgcn_ds_read_tr8_b64_v2i32(US_LDS_PTR(v2i, p + q * 8 * PITCH));
      f[2 * q] = v.x;
      f[2 * q + 1] = v.y;
    }
  }
  return f;
}

template <bool KC, int PITCH>
__device__ __forceinline__ v8h load_frag_f16(const uint8_t* tile, int r0, int kstep) {
  const int l = threadIdx.x & 63;
  if (KC) {
    const uint8_t* p = tile + (r0 + (l & 31)) * PITCH + (kstep * 16 + (l >> 5) * 8) * 2;
    return *US_LDS_PTR(const v8h, p);
  } else {
    // 16 lanes cooperate on a 4(k) x 16(row) block of halves; lane i points at k-row i/4, row
    // quarter i%4, and receives the 4 k values of row (group base + i).
    const int i = l & 15;
    const uint8_t* p = tile + (kstep * 16 + (l >> 5) * 8 + (i >> 2)) * PITCH + (r0 + ((l >> 4) & 1) * 16 + (i & 3) * 4) * 2;
    v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(US_LDS_PTR(v4s, p));
    v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(US_LDS_PTR(v4s, p + 4 * PITCH));
    typedef short v8s __attribute__((ext_vector_type(8)));
    v8s s = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    v8h h;
    __builtin_memcpy(&h, &s, 16);
    return h;
  }
}

template <int FA, int FB>
__device__ __forceinline__ v16f mfma_fp8(v8i a, v8i b, v16f c) {
  // format codes of the instruction: 0 = E4M3, 1 = E5M2; unit block scales
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, FA, FB, 0, 0, 0, 0);
}

// ---- epilogue for one quad (4 consecutive columns of one row) --------------------------------------
template <int EPI, int AUX_FMT>
__device__ __forceinline__ void epilogue_quad(const GemmArgs& g, long m, long n, float v0, float v1, float v2, float v3,
                                              long split) {
  const long idx = m * g.ldc + n;
  if (EPI == EPI_PARTIAL) {
    v4f o = {v0, v1, v2, v3};
    *reinterpret_cast<v4f*>(g.partial + (size_t)split * g.M * g.N + m * g.N + n) = o;
    return;
  }
  v0 *= g.scale; v1 *= g.scale; v2 *= g.scale; v3 *= g.scale;
  if (EPI == EPI_STORE) {
    if (g.c_is_f32) {
      v4f o = {v0, v1, v2, v3};
      *reinterpret_cast<v4f*>((float*)g.C + idx) = o;
    } else {
      v4h o = {(_Float16)v0, (_Float16)v1, (_Float16)v2, (_Float16)v3};
      *reinterpret_cast<v4h*>((_Float16*)g.C + idx) = o;
    }
    return;
  }
  v4h y = {(_Float16)v0, (_Float16)v1, (_Float16)v2, (_Float16)v3};   // the stored FP16 matmul result
  v4h r;
  if (EPI == EPI_GELU) {
    *reinterpret_cast<v4h*>((_Float16*)g.C + idx) = y;
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = (_Float16)gelu_scaled((float)y[k], g.epi_scale);
    if (g.aux16) *reinterpret_cast<v4h*>(g.aux16 + idx) = r;
  } else {  // EPI_GELU_GRAD
    v4h z = *reinterpret_cast<const v4h*>(g.Zpre + idx);
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = (_Float16)gelu_grad_scaled((float)z[k], (float)y[k], g.epi_scale);
    *reinterpret_cast<v4h*>((_Float16*)g.C + idx) = r;
  }
  if (g.aux8) {
    // FP8 copy of the FP16 value just stored: identical to casting the stored tensor afterwards
    uint32_t w = cvt4_fp8<AUX_FMT>((float)r[0], (float)r[1], (float)r[2], (float)r[3]);
    *reinterpret_cast<uint32_t*>(g.aux8 + idx) = w;
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI>
__global__ void __launch_bounds__(kGemmThreads) gemm_kernel(GemmArgs g) {
  using T = GemmTile<BM, BN, FP8, A_KC, B_KC>;
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  constexpr int ES = T::ES;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int FM = WM / 32, FN = WN / 32;
  constexpr int KSTEPS = FP8 ? 2 : 4;
  constexpr int PA = A_KC ? T::PITCH_KC : T::PITCH_A_KS;
  constexpr int PB = B_KC ? T::PITCH_KC : T::PITCH_B_KS;

  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  const long tiles_m = (g.M + BM - 1) / BM;
  const long tile = blockIdx.x;
  const long m0 = (tile % tiles_m) * BM;
  const long n0 = (tile / tiles_m) * BN;
  const long split = blockIdx.y;
  const long k_begin = split * g.k_per_split;
  const long k_end = (k_begin + g.k_per_split < g.K) ? k_begin + g.k_per_split : g.K;

  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int wm0 = (wave % WAVES_M) * WM;
  const int wn0 = (wave / WAVES_M) * WN;

  v16f acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  v4i ra[T::A_PER_THREAD], rb[T::B_PER_THREAD];

  const long nstages = (k_end > k_begin) ? (k_end - k_begin + T::BK - 1) / T::BK : 0;
  if (nstages > 0) {
    load_tile_regs<BM, A_KC, ES>(g.A, g.lda, m0, g.M, k_begin, k_end, ra);
    load_tile_regs<BN, B_KC, ES>(g.B, g.ldb, n0, g.N, k_begin, k_end, rb);
    store_tile_lds<BM, A_KC, ES, PA>(lds, ra);
    store_tile_lds<BN, B_KC, ES, PB>(lds + T::A_BYTES, rb);
  }
  __syncthreads();

  for (long s = 0; s < nstages; ++s) {
    const uint8_t* cur = lds + (s & 1) * T::STAGE_BYTES;
    uint8_t* nxt = lds + ((s + 1) & 1) * T::STAGE_BYTES;
    const bool more = (s + 1 < nstages);
    if (more) {
      const long k0 = k_begin + (s + 1) * T::BK;
      load_tile_regs<BM, A_KC, ES>(g.A, g.lda, m0, g.M, k0, k_end, ra);
      load_tile_regs<BN, B_KC, ES>(g.B, g.ldb, n0, g.N, k0, k_end, rb);
    }
    const uint8_t* ta = cur;
    const uint8_t* tb = cur + T::A_BYTES;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      if constexpr (FP8) {
        v8i fa[FM], fb[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[i] = load_frag_fp8<A_KC, PA>(ta, wm0 + i * 32, ks);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[j] = load_frag_fp8<B_KC, PB>(tb, wn0 + j * 32, ks);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j) acc[i][j] = mfma_fp8<FB, FA>(fb[j], fa[i], acc[i][j]);
      } else {
        v8h fa[FM], fb[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[i] = load_frag_f16<A_KC, PA>(ta, wm0 + i * 32, ks);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[j] = load_frag_f16<B_KC, PB>(tb, wn0 + j * 32, ks);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[j], fa[i], acc[i][j], 0, 0, 0);
      }
    }
    if (more) {
      store_tile_lds<BM, A_KC, ES, PA>(nxt, ra);
      store_tile_lds<BN, B_KC, ES, PB>(nxt + T::A_BYTES, rb);
    }
    __syncthreads();
  }

  // Accumulator layout of the 32x32 block with the N-side fragment as first operand:
  // register 4q+e of lane l holds (row m = l%32, column n = 8q + 4(l/32) + e).
  constexpr int AUX_FMT = (EPI == EPI_GELU_GRAD) ? US_E5M2 : US_E4M3;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    const long m = m0 + wm0 + i * 32 + (lane & 31);
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const long n = n0 + wn0 + j * 32 + 8 * q + 4 * (lane >> 5);
        if (n < g.N)
          epilogue_quad<EPI, AUX_FMT>(g, m, n, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                                      acc[i][j][4 * q + 3], split);
      }
    }
  }
}

}  // namespace us
