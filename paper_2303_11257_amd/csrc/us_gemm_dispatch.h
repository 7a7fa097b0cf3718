// Host-side selection of kernel, tile shape and epilogue for one (operand layout, operand type)
// family.  Each family is instantiated in its own translation unit to keep compile times short.
#pragma once

#include "us_gemm_direct.h"
#include "us_gemm_staged.h"
#include "us_launch.h"
#include <cstdlib>

namespace us {

// Tile configurations  <BM, BN, WAVES_M, WAVES_N, BKB, NST, MINB>
//   D256: 8 waves (2 x 4, 128 x 64 accumulators per wave), one workgroup per CU, 128 KB of LDS ring
//   D128: 4 waves (2 x 2, 64 x 64 per wave), two workgroups per CU, 64 KB ring
//   S128: the register-staged kernel for reduction lengths that are not a multiple of the stage
using CfgD256 = GemmCfg<256, 256, 2, 4, 128, 2, 1>;
//   K128: grad_W only (both operands K-strided): 8 waves on one 128 x 128 tile, two groups of 2 x 2 that
//         each take half of every 256-byte stage; one workgroup per CU, no K slices in global memory
using CfgD128 = GemmCfg<128, 128, 2, 2, 128, 2, 2>;
using CfgS128 = GemmCfg<128, 128, 2, 2, 128, 2, 2>;
using CfgK128 = GemmCfg<128, 128, 2, 2, 256, 2, 1, 2>;
//   M256: 256 x 128 tile, 8 waves as two groups of 2 x 2 sharing every stage's k-steps, three stages: FP8 outputs
//         of 192-256 such tiles (one per CU), the 512-thread shape next to K128 in a paired launch, and grad_W itself
//         (both operands K-strided) on about 128 tiles in a paired launch
using CfgM256 = GemmCfg<256, 128, 2, 2, 128, 3, 1, 2>;
//   W128: forward / grad_X with so few 128 x 128 tiles that the CUs get at most one each (BERT-base: 192): 8 waves
//         on the tile, two groups sharing the k-steps of each stage, four stages; 10-16 % faster than D128 there
using CfgW128 = GemmCfg<128, 128, 2, 2, 128, 4, 1, 2>;

//   E192: 256 x 192 tile, 8 waves (4 x 2, 64 x 96 accumulators per wave), FP16 only: outputs that make one tile per CU
//         this way and only three quarters as many 256 x 256 tiles (BERT-base: 4096 x 3072 -> 16 x 16 = 256 instead of 192)
using CfgE192 = GemmCfg<256, 192, 4, 2, 128, 2, 1>;
//   H256: 128 x 256 tile, 8 waves (2 x 4, 64 x 64 per wave): the table-driven GELU' next to grad_W tiles in a paired launch
//         whose large tiles would not fit one round
using CfgH256 = GemmCfg<128, 256, 2, 4, 128, 2, 1>;

inline long ceil_div(long a, long b) { return (a + b - 1) / b; }

// All windows below are stated in units of the device's CU count (MI355X: 256), read from the device.
inline long cu_count() { return device_info().cus; }

// The large tile needs the output to cover the CUs about one and a half times, or at most once with three
// quarters of them busy (BERT-base on 256 CUs: 4096 x 3072 -> 192 tiles; backward of layer 2 there 67 -> 62 us); in
// between the small tile (two workgroups per CU, four times as many tiles) keeps more of the chip busy.
inline bool use_big_tile(long M, long N, int splits) {
  const long t = ceil_div(M, 256) * ceil_div(N, 256) * splits, cu = cu_count();
  return 2 * t >= 3 * cu || (4 * t >= 3 * cu && t <= cu);
}

// FP16 products whose output is covered exactly by 256 x 192 tiles, at most one per CU and at least seven eighths of
// the CUs busy
inline bool use_wide_tile(long M, long N) {
  const long t = ceil_div(M, 256) * ceil_div(N, 192), cu = cu_count();
  return N % 192 == 0 && t <= cu && 8 * t >= 7 * cu;
}

// grad_W whose 128 x 128 tiles just about cover the CUs once (C3: 4096 x 1024 -> 256 tiles): instead of
// cutting the long token reduction into slices that travel through HBM, two wave groups of one
// workgroup share it and add up in LDS.
inline bool use_wave_split_tile(long M, long N, long K) {
  const long tiles = ceil_div(M, 128) * ceil_div(N, 128), cu = cu_count();
  return !use_big_tile(M, N, 1) && K >= 1024 && K % 256 == 0 && 2 * tiles >= cu && tiles <= cu;
}

inline GemmArgs make_args(const GemmProblem& p, long k_per_split, int BM, int BN) {
  GemmArgs g{};
  g.A = (const uint8_t*)p.A;
  g.B = (const uint8_t*)p.B;
  g.C = p.C;
  g.M = p.M; g.N = p.N; g.K = p.K;
  g.lda = p.lda; g.ldb = p.ldb; g.ldc = p.ldc;
  g.k_per_split = k_per_split;
  g.scale = p.scale;
  g.epi_scale = p.epi_scale;
  g.skip_scale = p.skip_scale;
  g.act = p.act;
  g.Zpre = (const _Float16*)p.Zpre;
  g.aux16 = (_Float16*)p.aux16;
  g.aux8 = (uint8_t*)p.aux8;
  g.partial = (float*)p.workspace;
  g.table = (const uint8_t*)p.table;
  g.bias = (const _Float16*)p.bias;
  g.colsum = (float*)p.colsum;
  if (p.batch > 1) {
    const long es = (p.a_dt == US_F16) ? 2 : 1;
    g.batch_a = p.batch_a * es;
    g.batch_b = p.batch_b * es;
    g.batch_c = p.batch_c * (p.c_dt == US_F32 ? 4 : 2);
  }
  g.nxcd = device_info().xcds;
  choose_xcd_grid(ceil_div(p.M, BM), ceil_div(p.N, BN), g.nxcd, BM, BN, g.xcd_gm, g.xcd_gn);
  // bands 8 tiles wide: the 32 (one per CU) or 64 (two per CU) tiles that run together on an XCD form 4 x 8 or 8 x 8.
  // (Measured for the large tile: 4 wide was 3 us slower on the 8192 x 4096 x 1024 product with the GELU epilogue,
  // 16 and 32 equal to 8; the other tile shapes show no difference between 2 and 16.)
  g.grp_w = 8;
  return g;
}

template <bool DIRECT, class Cfg, bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI, bool WIDE>
hipError_t launch_one(const GemmProblem& p, int splits, long k_per_split, hipStream_t st) {
  using Tile = typename std::conditional<DIRECT, DirectTile<Cfg, FP8, A_KC, B_KC, WIDE, EPI>,
                                         StagedTile<Cfg, FP8, A_KC, B_KC, WIDE, EPI>>::type;
  constexpr int LDS = Tile::LDS_BYTES;
  void (*kern)(GemmArgs);
  if constexpr (DIRECT) kern = gemm_direct_kernel<Cfg, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>;
  else kern = gemm_staged_kernel<Cfg, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>;
  note_gemm_launch(DIRECT ? "direct" : "staged", Cfg::BM, Cfg::BN, Cfg::WAVES_K, Cfg::NST, FP8, A_KC, B_KC, EPI, WIDE, splits);
  static FuncConfig cfg;           // raising the dynamic-LDS limit: once per function and device
  if (hipError_t e = cfg.ensure((const void*)kern, LDS); e != hipSuccess) return e;
  const GemmArgs g = make_args(p, k_per_split, Cfg::BM, Cfg::BN);
  const long tiles = ceil_div(p.M, Cfg::BM) * ceil_div(p.N, Cfg::BN);
  dim3 grid((unsigned)tiles, (unsigned)splits, (unsigned)(p.batch > 1 ? p.batch : 1));
  kern<<<grid, Cfg::THREADS, LDS, st>>>(g);
  return hipGetLastError();
}

template <bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI, bool WIDE>
hipError_t launch_sized(const GemmProblem& p, int splits, long k_per_split, hipStream_t st) {
  const long bk = FP8 ? 128 : 64;                       // elements of K per stage of the direct kernels
  const bool direct_ok = p.K > 0 && p.K % bk == 0;      // slice lengths are multiples of 128 already
  if (!direct_ok) return launch_one<false, CfgS128, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(p, splits, k_per_split, st);
  const bool batched = p.batch > 1;      // the tile count that decides is the whole batch's
  if constexpr (!FP8 && (A_KC || B_KC) && EPI == EPI_STORE && !WIDE) {
    if (splits == 1 && !batched && use_wide_tile(p.M, p.N))
      return launch_one<true, CfgE192, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(p, splits, k_per_split, st);
  }
  if (use_big_tile(p.M, p.N, splits * (int)(batched ? p.batch : 1)) && (!batched || (p.M >= 256 && p.N >= 256)))
    return launch_one<true, CfgD256, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(p, splits, k_per_split, st);
  if (batched) return launch_one<true, CfgD128, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(p, splits, k_per_split, st);
  if constexpr (FP8 && (A_KC || B_KC) && (EPI == EPI_STORE || EPI == EPI_RESIDUAL) && !WIDE) {
    // an output of about one tile of 256 x 128 per CU (BERT-large: Linear 2, 8192 x 1024 -> 256): two wave groups
    // (40 against 43 us forward, 35 against 37 us in the grad_X layout; FP8 only, not measured for FP16)
    const long t_mid = ceil_div(p.M, 256) * ceil_div(p.N, 128);
    if (splits == 1 && 4 * t_mid >= 3 * cu_count() && t_mid <= cu_count() && p.K >= 1024)
      return launch_one<true, CfgM256, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(p, splits, k_per_split, st);
  }
  if constexpr ((A_KC || B_KC) && (EPI == EPI_STORE || EPI == EPI_RESIDUAL) && !WIDE) {
    if (splits == 1 && ceil_div(p.M, 128) * ceil_div(p.N, 128) <= cu_count() && p.K >= 1024)
      return launch_one<true, CfgW128, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(p, splits, k_per_split, st);
  }
  if constexpr (!A_KC && !B_KC && EPI == EPI_STORE) {
    if (splits == 1 && use_wave_split_tile(p.M, p.N, p.K))
      return launch_one<true, CfgK128, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(p, splits, k_per_split, st);
  }
  return launch_one<true, CfgD128, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(p, splits, k_per_split, st);
}

// The table-driven GELU epilogues exist for the large tile of the direct kernel only (the table
// needs 64-73 KB of LDS next to the strips).
template <bool FP8>
inline bool table_path_ok(const GemmProblem& p) {
  const long bk = FP8 ? 128 : 64;
  return p.table != nullptr && p.act == 0 && p.K > 0 && p.K % bk == 0 && use_big_tile(p.M, p.N, 1);   // the tables are gelu's
}

// ... and for the 256 x 192 tile (FP16, no column sums: a lane of its epilogue does not keep to the same columns)
inline bool wide_table_path_ok(const GemmProblem& p) {
  return p.table != nullptr && p.act == 0 && p.K > 0 && p.K % 64 == 0 && p.colsum == nullptr && use_wide_tile(p.M, p.N);
}

// Plain store epilogue: FP16 or FP32 output.
template <bool FP8, int FA, int FB, bool A_KC, bool B_KC>
hipError_t launch_store(const GemmProblem& p, hipStream_t st) {
  if (p.c_dt == US_F32) return launch_sized<FP8, FA, FB, A_KC, B_KC, EPI_STORE, true>(p, 1, p.K, st);
  return launch_sized<FP8, FA, FB, A_KC, B_KC, EPI_STORE, false>(p, 1, p.K, st);
}

hipError_t launch_splitk_reduce(const float* partial, void* out, long total, int splits, float scale, bool out_is_f32,
                                hipStream_t st);

// Families (defined one per translation unit).
hipError_t gemm_nn_f16(const GemmProblem& p, hipStream_t st);   // forward:  A K-contig, B K-strided
hipError_t gemm_nn_fp8(const GemmProblem& p, hipStream_t st);
hipError_t gemm_nt_f16(const GemmProblem& p, hipStream_t st);   // grad_X:   both K-contig
hipError_t gemm_nt_fp8(const GemmProblem& p, hipStream_t st);
hipError_t gemm_tn_f16(const GemmProblem& p, hipStream_t st);   // grad_W:   both K-strided, split-K
hipError_t gemm_tn_fp8(const GemmProblem& p, hipStream_t st);

}  // namespace us
