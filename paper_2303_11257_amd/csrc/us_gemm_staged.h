// Register-staged GEMM kernel: handles every shape the C ABI accepts (dimensions that are multiples of
// 16, including a ragged reduction length).  It is the path for reduction lengths that are not a
// multiple of the pipeline stage; the direct-to-LDS kernel (us_gemm_direct.h) covers the rest.
//
// Global loads of stage s+1 go to registers before the MFMAs of stage s and are written to the other
// LDS buffer after them (two LDS buffers, one barrier per stage).  K-contiguous tiles are stored
// [row][BKB + 16 B pad]; K-strided tiles are stored as they lie in memory, [k][rows + 32 B pad], and
// fetched with the transposing LDS reads.
#pragma once

#include "us_gemm_common.h"

namespace us {

template <class Cfg, bool FP8, bool A_KC, bool B_KC, bool WIDE, int EPI = EPI_STORE>
struct StagedTile {
  static constexpr int ES = FP8 ? 1 : 2;
  static constexpr int BK = Cfg::BKB / ES;               // elements of K per stage
  static constexpr int PITCH_KC = Cfg::BKB + 16;
  static constexpr int PITCH_A_KS = Cfg::BM * ES + 32;
  static constexpr int PITCH_B_KS = Cfg::BN * ES + 32;
  static constexpr int A_BYTES = A_KC ? Cfg::BM * PITCH_KC : BK * PITCH_A_KS;
  static constexpr int B_BYTES = B_KC ? Cfg::BN * PITCH_KC : BK * PITCH_B_KS;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int A_PER_THREAD = Cfg::BM * Cfg::BKB / 16 / Cfg::THREADS;   // 16-byte chunks
  static constexpr int B_PER_THREAD = Cfg::BN * Cfg::BKB / 16 / Cfg::THREADS;
  static constexpr int EPI_BYTES = EpiStrip<Cfg, WIDE, EPI>::BYTES;
  static constexpr int LDS_BYTES = (2 * STAGE_BYTES > EPI_BYTES) ? 2 * STAGE_BYTES : EPI_BYTES;
  static_assert((Cfg::BM * Cfg::BKB / 16) % Cfg::THREADS == 0 && (Cfg::BN * Cfg::BKB / 16) % Cfg::THREADS == 0, "");
};

// ROWS tile rows starting at row0 (matrix extent extent_r); k0 = first k of the stage; k_end = end of
// this slice's reduction range.  Chunks outside the matrix are zero.
template <int THREADS, int ROWS, int BKB, bool KC, int ES, int NCH>
__device__ __forceinline__ void load_tile_regs(const uint8_t* __restrict__ base, long ld, long row0, long extent_r,
                                               long k0, long k_end, v4i (&regs)[NCH]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = t + i * THREADS;
    long r, k;
    if (KC) {
      constexpr int CPR = BKB / 16;        // chunks per row
      r = row0 + c / CPR;
      k = k0 + (c % CPR) * (16 / ES);
    } else {
      constexpr int CPR = ROWS * ES / 16;  // chunks per k-row
      r = row0 + (c % CPR) * (16 / ES);
      k = k0 + c / CPR;
    }
    const uint8_t* p = KC ? base + (r * ld + k) * ES : base + (k * ld + r) * ES;
    v4i v = {0, 0, 0, 0};
    if (r < extent_r && k < k_end) v = *reinterpret_cast<const v4i*>(p);
    regs[i] = v;
  }
}

template <int THREADS, int ROWS, int BKB, bool KC, int ES, int PITCH, int NCH>
__device__ __forceinline__ void store_tile_lds(uint8_t* lds, const v4i (&regs)[NCH]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = t + i * THREADS;
    constexpr int CPR = KC ? BKB / 16 : ROWS * ES / 16;
    *US_LDS_PTR(v4i, lds + (c / CPR) * PITCH + (c % CPR) * 16) = regs[i];
  }
}

// Fragment = 32 rows (r0..r0+31) x one MFMA's worth of k, number `kstep` within the stage.
// Lane l supplies row r0 + l%32 and the k-half l/32 (FP8: 32 consecutive k; FP16: 8 consecutive k).
template <bool KC, int PITCH>
__device__ __forceinline__ v8i staged_frag_fp8(const uint8_t* tile, int r0, int kstep) {
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
__device__ __forceinline__ v8h staged_frag_f16(const uint8_t* tile, int r0, int kstep) {
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

template <class Cfg, bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI, bool WIDE>
__global__ void __launch_bounds__(Cfg::THREADS, Cfg::MINB) gemm_staged_kernel(GemmArgs g) {
  using T = StagedTile<Cfg, FP8, A_KC, B_KC, WIDE, EPI>;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, WM = Cfg::WM, WN = Cfg::WN, THREADS = Cfg::THREADS, BKB = Cfg::BKB;
  constexpr int ES = T::ES;
  constexpr int FM = Cfg::FM, FN = Cfg::FN;
  constexpr int KSTEPS = FP8 ? BKB / 64 : BKB / 32;
  constexpr int PA = A_KC ? T::PITCH_KC : T::PITCH_A_KS;
  constexpr int PB = B_KC ? T::PITCH_KC : T::PITCH_B_KS;

  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  if constexpr (EPI == EPI_STORE) select_batch_item(g);

  const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
  int tm, tn;
  tile_of_block((int)blockIdx.x, tiles_m, tiles_n, g.xcd_gm, g.xcd_gn, g.grp_w, g.nxcd, tm, tn);
  const long m0 = (long)tm * BM, n0 = (long)tn * BN;
  const long split = blockIdx.y;
  const long k_begin = split * g.k_per_split;
  const long k_end = (k_begin + g.k_per_split < g.K) ? k_begin + g.k_per_split : g.K;

  const int wave = threadIdx.x >> 6;
  const int wm0 = (wave % Cfg::WAVES_M) * WM;
  const int wn0 = (wave / Cfg::WAVES_M) * WN;

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
    load_tile_regs<THREADS, BM, BKB, A_KC, ES>(g.A, g.lda, m0, g.M, k_begin, k_end, ra);
    load_tile_regs<THREADS, BN, BKB, B_KC, ES>(g.B, g.ldb, n0, g.N, k_begin, k_end, rb);
    store_tile_lds<THREADS, BM, BKB, A_KC, ES, PA>(lds, ra);
    store_tile_lds<THREADS, BN, BKB, B_KC, ES, PB>(lds + T::A_BYTES, rb);
  }
  __syncthreads();

  for (long s = 0; s < nstages; ++s) {
    const uint8_t* cur = lds + (s & 1) * T::STAGE_BYTES;
    uint8_t* nxt = lds + ((s + 1) & 1) * T::STAGE_BYTES;
    const bool more = (s + 1 < nstages);
    if (more) {
      const long k0 = k_begin + (s + 1) * T::BK;
      load_tile_regs<THREADS, BM, BKB, A_KC, ES>(g.A, g.lda, m0, g.M, k0, k_end, ra);
      load_tile_regs<THREADS, BN, BKB, B_KC, ES>(g.B, g.ldb, n0, g.N, k0, k_end, rb);
    }
    const uint8_t* ta = cur;
    const uint8_t* tb = cur + T::A_BYTES;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      if constexpr (FP8) {
        v8i fa[FM], fb[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[i] = staged_frag_fp8<A_KC, PA>(ta, wm0 + i * 32, ks);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[j] = staged_frag_fp8<B_KC, PB>(tb, wn0 + j * 32, ks);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j) acc[i][j] = mfma_fp8<FB, FA>(fb[j], fa[i], acc[i][j]);
      } else {
        v8h fa[FM], fb[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[i] = staged_frag_f16<A_KC, PA>(ta, wm0 + i * 32, ks);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[j] = staged_frag_f16<B_KC, PB>(tb, wn0 + j * 32, ks);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[j], fa[i], acc[i][j], 0, 0, 0);
      }
    }
    if (more) {
      store_tile_lds<THREADS, BM, BKB, A_KC, ES, PA>(nxt, ra);
      store_tile_lds<THREADS, BN, BKB, B_KC, ES, PB>(nxt + T::A_BYTES, rb);
    }
    __syncthreads();
  }
  // the loop's last barrier has retired every read of the operand tiles
  store_block_epilogue<Cfg, EPI, WIDE, 0, Cfg::FM, epilogue_takes_bias<A_KC, B_KC, EPI, WIDE>()>(g, acc, lds, m0, n0, split);
}

}  // namespace us
