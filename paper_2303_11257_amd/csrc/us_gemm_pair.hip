// Both products of a layer's backward pass (grad_X and grad_W) in one launch, for the combinations of
// 512-thread tile shapes listed in gemm_pair_applicable: see gemm_pair_kernel.
#include "us_gemm_dispatch.h"

namespace us {

namespace {

template <class KA, class KB>
hipError_t launch_pair(const GemmProblem& dx, const GemmProblem& dw, hipStream_t st) {
  constexpr int LDS = KA::Tile::LDS_BYTES > KB::Tile::LDS_BYTES ? KA::Tile::LDS_BYTES : KB::Tile::LDS_BYTES;
  note_gemm_launch("pair", KA::BM, KA::BN, KA::WAVES_K, KA::NST, KA::IS_FP8, KA::A_KC_, KA::B_KC_, KA::EPI_, false, 1);
  note_gemm_launch("pair", KB::BM, KB::BN, KB::WAVES_K, KB::NST, KB::IS_FP8, KB::A_KC_, KB::B_KC_, KB::EPI_, false, 1);
  static FuncConfig cfg;
  if (hipError_t e = cfg.ensure((const void*)gemm_pair_kernel<KA, KB>, LDS); e != hipSuccess) return e;
  const GemmArgs a = make_args(dx, dx.K, KA::BM, KA::BN);
  const GemmArgs b = make_args(dw, dw.K, KB::BM, KB::BN);
  const long tiles_a = ceil_div(dx.M, KA::BM) * ceil_div(dx.N, KA::BN), tiles_b = ceil_div(dw.M, KB::BM) * ceil_div(dw.N, KB::BN);
  gemm_pair_kernel<KA, KB><<<(unsigned)(tiles_a + tiles_b), KA::THREADS, LDS, st>>>(a, b, (int)tiles_b);
  return hipGetLastError();
}

// grad_W in a pair on 256 x 128 tiles that take about half of the CUs (BERT-large: 4096 x 1024 -> 128 tiles).  Such a
// tile needs 36 % less CU time than two wave-split 128 x 128 tiles, but covers only half of the chip and runs twice as
// long: on its own that is slower, in a pair the grad_X tiles take the other CUs from the start and the launch ends
// when it would have ended with grad_W spread over all CUs, minus the CU time saved.  With fewer than 112 tiles the
// long tiles outlast the rest of the launch (BERT-base, 72 tiles: measured slower).
bool long_tile_ok(const GemmProblem& dw) {
  const long t = ceil_div(dw.M, 256) * ceil_div(dw.N, 128), cu = cu_count();
  return 16 * t >= 7 * cu && 2 * t <= cu && t % device_info().xcds == 0;
}

// grad_X without an activation derivative whose 256 x 256 tiles, together with grad_W's long tiles, give every CU one
// tile of about the same length (BERT-large layer 1: 128 + 128)
bool one_round_ok(const GemmProblem& dx, const GemmProblem& dw) {
  const long t = ceil_div(dx.M, 256) * ceil_div(dx.N, 256) + ceil_div(dw.M, 256) * ceil_div(dw.N, 128);
  return long_tile_ok(dw) && (dx.epi == US_EPI_NONE || dx.epi == US_EPI_RESIDUAL) && 8 * t >= 7 * cu_count() && t <= cu_count() &&
         dx.K >= 2048;
}

// grad_X without an epilogue on so few 128 x 128 tiles that the CUs get at most one each (wave-split small tile)
bool small_tile_ok(const GemmProblem& dx) {
  const long t = ceil_div(dx.M, 128) * ceil_div(dx.N, 128);
  return dx.epi == US_EPI_NONE && t <= cu_count() && dx.K >= 1024 && !use_big_tile(dx.M, dx.N, 1);
}

// grad_X without an epilogue whose 256 x 128 tiles, together with grad_W's tiles, give every CU at most one tile
// (BERT-base layer 1: 96 + 144): one round instead of 192 + 144 small tiles in one and a third
bool mid_one_round_ok(const GemmProblem& dx, const GemmProblem& dw) {
  const long tw = long_tile_ok(dw) ? ceil_div(dw.M, 256) * ceil_div(dw.N, 128) : ceil_div(dw.M, 128) * ceil_div(dw.N, 128);
  const long t = ceil_div(dx.M, 256) * ceil_div(dx.N, 128) + tw;
  return (dx.epi == US_EPI_NONE || dx.epi == US_EPI_RESIDUAL) && t <= cu_count() && 8 * t >= 7 * cu_count() && dx.K >= 2048;
}

// grad_X with the table-driven GELU' whose large tiles fit one round on their own but not next to grad_W's tiles
// (BERT-base layer 2: 192 + 144 on 256 CUs): twice as many tiles of 128 x 256 fill the second round's gaps
// (FP16: 62.7 -> 59.5 us; FP8 operands at the same shape: 46.6 -> 43.1 us; same box each)
bool half_tile_ok(const GemmProblem& dx, const GemmProblem& dw) {
  const long tw = long_tile_ok(dw) ? ceil_div(dw.M, 256) * ceil_div(dw.N, 128) : ceil_div(dw.M, 128) * ceil_div(dw.N, 128);
  const long t = ceil_div(dx.M, 256) * ceil_div(dx.N, 256);
  return t <= cu_count() && t + tw > cu_count();
}

template <bool FP8, class KW>
hipError_t launch_pair_kw(const GemmProblem& dx, const GemmProblem& dw, hipStream_t st) {
  constexpr int FG = FP8 ? 1 : 0;                     // gradient operand format (E5M2) where it applies
  if (dx.epi == US_EPI_GELU_GRAD && !use_big_tile(dx.M, dx.N, 1))
    return launch_pair<GemmKind<CfgM256, FP8, FG, 0, true, true, EPI_GELU_GRAD, false>, KW>(dx, dw, st);
  if (dx.epi == US_EPI_GELU_GRAD) {
    GemmProblem q = dx;
    q.table = (char*)dx.table + kGeluSlopeTableOffset;
    if (!dx.tables_ready) {
      hipError_t e = launch_gelu_slope_table(q.table, dx.epi_scale, st);
      if (e != hipSuccess) return e;
    }
    if (half_tile_ok(dx, dw))
      return launch_pair<GemmKind<CfgH256, FP8, FG, 0, true, true, EPI_GELU_GRAD_TAB, false>, KW>(q, dw, st);
    return launch_pair<GemmKind<CfgD256, FP8, FG, 0, true, true, EPI_GELU_GRAD_TAB, false>, KW>(q, dw, st);
  }
  // the large tile also when it and grad_W's long tiles fill the CUs exactly once
  const bool big = use_big_tile(dx.M, dx.N, 1) || (KW::BM == 256 && one_round_ok(dx, dw));
  if (dx.epi == US_EPI_RESIDUAL) {
    if (big) return launch_pair<GemmKind<CfgD256, FP8, FG, 0, true, true, EPI_RESIDUAL, false>, KW>(dx, dw, st);
    return launch_pair<GemmKind<CfgM256, FP8, FG, 0, true, true, EPI_RESIDUAL, false>, KW>(dx, dw, st);
  }
  if (big) return launch_pair<GemmKind<CfgD256, FP8, FG, 0, true, true, EPI_STORE, false>, KW>(dx, dw, st);
  if (mid_one_round_ok(dx, dw))
    return launch_pair<GemmKind<CfgM256, FP8, FG, 0, true, true, EPI_STORE, false>, KW>(dx, dw, st);
  if (small_tile_ok(dx)) return launch_pair<GemmKind<CfgW128, FP8, FG, 0, true, true, EPI_STORE, false>, KW>(dx, dw, st);
  return launch_pair<GemmKind<CfgM256, FP8, FG, 0, true, true, EPI_STORE, false>, KW>(dx, dw, st);
}

template <bool FP8>
hipError_t launch_pair_typed(const GemmProblem& dx, const GemmProblem& dw, hipStream_t st) {
  constexpr int FG = FP8 ? 1 : 0;
  if (long_tile_ok(dw)) return launch_pair_kw<FP8, GemmKind<CfgM256, FP8, 0, FG, false, false, EPI_STORE, false>>(dx, dw, st);
  return launch_pair_kw<FP8, GemmKind<CfgK128, FP8, 0, FG, false, false, EPI_STORE, false>>(dx, dw, st);
}

// grad_X without an epilogue whose 256 x 128 tiles cover the CUs about once
bool mid_tile_ok(const GemmProblem& dx) {
  const long t = ceil_div(dx.M, 256) * ceil_div(dx.N, 128);
  return (dx.epi == US_EPI_NONE || dx.epi == US_EPI_RESIDUAL) && 4 * t >= 3 * cu_count() && 4 * t <= 5 * cu_count();
}

}  // namespace

bool gemm_pair_applicable(const GemmProblem& dx, const GemmProblem& dw) {
  const bool fp8 = dx.a_dt != US_F16;
  if ((dw.a_dt != US_F16) != fp8) return false;
  if (!(dx.a_kc && dx.b_kc) || dw.a_kc || dw.b_kc) return false;
  if (dx.c_dt != US_F16 || dw.c_dt != US_F16 || dw.epi != US_EPI_NONE) return false;
  const long bk = fp8 ? 128 : 64;
  const bool big = use_big_tile(dx.M, dx.N, 1);
  const long t_mid = ceil_div(dx.M, 256) * ceil_div(dx.N, 128);
  // grad_X with the arithmetic activation-derivative epilogue on 256 x 128 tiles (an output too small for the large tile)
  const bool mid_act = dx.epi == US_EPI_GELU_GRAD && !big && 4 * t_mid >= 3 * cu_count() && t_mid <= 2 * cu_count();
  const bool small_pair = (small_tile_ok(dx) && !mid_tile_ok(dx)) || mid_act;
  if (dx.K <= 0 || dx.K % bk || !(big || mid_tile_ok(dx) || small_pair || one_round_ok(dx, dw) || mid_one_round_ok(dx, dw))) return false;
  if (dx.epi == US_EPI_GELU_GRAD && big && (!dx.table || dx.act != 0)) return false;   // large tile: table-driven epilogue only
  if (dx.epi != US_EPI_NONE && dx.epi != US_EPI_GELU_GRAD && dx.epi != US_EPI_RESIDUAL) return false;
  if (!use_wave_split_tile(dw.M, dw.N, dw.K)) return false;
  return long_tile_ok(dw) || (ceil_div(dw.M, 128) * ceil_div(dw.N, 128)) % device_info().xcds == 0;
}

hipError_t launch_gemm_pair(const GemmProblem& dx, const GemmProblem& dw, hipStream_t st) {
  return dx.a_dt != US_F16 ? launch_pair_typed<true>(dx, dw, st) : launch_pair_typed<false>(dx, dw, st);
}

}  // namespace us
