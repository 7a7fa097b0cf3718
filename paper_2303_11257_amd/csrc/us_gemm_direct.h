// Direct-to-LDS pipelined GEMM kernel for gfx950 (the fast path: reduction length a multiple of the
// stage, everything else may be ragged).
//
// Operand tiles travel HBM/L2 -> LDS with global_load_lds_dwordx4 (no register staging, no LDS
// store instructions): a wave instruction deposits 64 x 16 B contiguously, so tiles are unpadded and
// bank conflicts are removed by an XOR swizzle of the 16-byte chunk index instead; the swizzle is
// applied to the *global* address each lane fetches and again when fragments are read.
// NST stage buffers form a ring.  Matrix-core fragments are double-buffered in registers: the LDS reads of
// the next k-step are issued around the MFMAs of the current one (FP16: ahead of them; FP8: one fragment
// behind each of the last MFMAs), also across the stage boundary.  At that boundary a wave waits for its own LDS reads of stage s, then for its own
// loads of stage s+1 (explicit s_waitcnt vmcnt(n): younger stages stay in flight), then meets the
// other waves at one bare s_barrier; after it the buffer of stage s is free and receives the loads
// of stage s+NST, so NST stages of HBM latency are covered by MFMAs.
//
// Tile layouts in LDS (pitch P bytes, chunk = 16 B, c' = c ^ swz(row)):
//   K-contiguous operand: [row][BKB bytes]        fragments: ds_read_b128
//   K-strided operand:    [k][rows * elem size]   fragments: ds_read_b64_tr_b8 / _tr_b16 (transposing)
// Rows / columns beyond the matrix are never loaded; their LDS slots are zeroed once up front.
#pragma once

#include <type_traits>

#include "us_gemm_common.h"

namespace us {

template <class Cfg, bool FP8, bool A_KC, bool B_KC, bool WIDE, int EPI = EPI_STORE>
struct DirectTile {
  static constexpr int ES = FP8 ? 1 : 2;
  static constexpr int BK = Cfg::BKB / ES;                      // elements of K per stage
  static constexpr int PA = A_KC ? Cfg::BKB : Cfg::BM * ES;     // LDS pitch of the A / B tile
  static constexpr int PB = B_KC ? Cfg::BKB : Cfg::BN * ES;
  static constexpr int A_BYTES = Cfg::BM * Cfg::BKB;
  static constexpr int B_BYTES = Cfg::BN * Cfg::BKB;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int A_LOADS = A_BYTES / 16 / Cfg::THREADS;   // 16-byte loads per thread and stage
  static constexpr int B_LOADS = B_BYTES / 16 / Cfg::THREADS;
  static constexpr int RING_BYTES = Cfg::NST * STAGE_BYTES;
  // WAVES_K = 2: the half of every wave's accumulators that its partner finishes (FP32, one 256-byte row
  // per register) passes through LDS before the strips take the same space
  static constexpr int REDUCE_BYTES = Cfg::WAVES_K == 1 ? 0 : Cfg::WAVES * (Cfg::FM / 2) * Cfg::FN * 16 * 64 * 4;
  static constexpr int STRIP_TABLE_BYTES = EpiStrip<Cfg, WIDE, EPI>::BYTES;
  static constexpr int EPI_BYTES = REDUCE_BYTES > STRIP_TABLE_BYTES ? REDUCE_BYTES : STRIP_TABLE_BYTES;
  static constexpr int LDS_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
  static_assert(A_BYTES % (16 * Cfg::THREADS) == 0 && B_BYTES % (16 * Cfg::THREADS) == 0, "whole wave loads only");
  static_assert(Cfg::NST >= 2 && Cfg::NST <= 5, "");
  static_assert(Cfg::BKB == 64 || Cfg::BKB == 128 || (Cfg::BKB == 256 && !A_KC && !B_KC),
                "256-byte stages exist for K-strided tiles only (the K-contiguous swizzle stops at 128)");
  static_assert((FP8 ? Cfg::BKB / 64 : Cfg::BKB / 32) % Cfg::WAVES_K == 0, "whole k-steps per wave group");
  static_assert(LDS_BYTES <= 160 * 1024, "the ring must fit the CU's 160 KB of LDS");
};

// XOR mask on the 16-byte chunk index of LDS row `row`, chosen so that the fragment reads below are free of
// bank conflicts (64 banks x 4 B; b128 reads are served 16 lanes at a time, b64 reads 32 lanes).
template <bool KC, bool FP8, int PITCH>
__device__ __forceinline__ int swz(int row) {
  if constexpr (KC) {
    static_assert(PITCH == 64 || PITCH == 128, "K-contiguous pitch");
    return PITCH == 64 ? ((row >> 2) & 3) : ((row >> 1) & 7);
  } else if constexpr (FP8) {
    static_assert(PITCH == 128 || PITCH == 256, "K-strided FP8 pitch");
    return PITCH == 256 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1);
  } else {
    static_assert(PITCH == 256 || PITCH == 384 || PITCH == 512, "K-strided FP16 pitch");
    // The 32 lanes a transposing read serves together touch 64 contiguous bytes in each of four consecutive k-rows.
    // Pitches of 256 / 512 B put those rows on the same banks: each row moves by a different multiple of 64 B.  A pitch of
    // 384 B (a tile 192 values wide) already alternates between two bank halves, so one more bit separates rows 0, 1
    // from rows 2, 3 (flipping bit 2 of the chunk index stays inside the row: 24 chunks are three groups of eight).
    return PITCH == 384 ? ((row >> 1) & 1) << 2 : (row & 3) << 2;
  }
}

// Global source pointers of this thread's loads for stage 0 (pointer is null for slots outside the
// matrix), for one operand tile of ROWS rows starting at row0.
template <int THREADS, int ROWS, int BKB, bool KC, bool FP8, int PITCH, int NL>
__device__ __forceinline__ void direct_sources(const uint8_t* base, long ld, long row0, long extent_r, long k0,
                                               const uint8_t* (&src)[NL]) {
  constexpr int ES = FP8 ? 1 : 2;
  const int t = threadIdx.x;
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    const int off = (j * THREADS + t) * 16;
    const int row = off / PITCH;
    const int cc = ((off % PITCH) >> 4) ^ swz<KC, FP8, PITCH>(row);
    long r, k;
    if (KC) { r = row0 + row; k = k0 + cc * (16 / ES); }
    else    { k = k0 + row;   r = row0 + cc * (16 / ES); }
    const uint8_t* p = KC ? base + (r * ld + k) * ES : base + (k * ld + r) * ES;
    src[j] = (r < extent_r) ? p : nullptr;
  }
}

template <int THREADS, int NL>
__device__ __forceinline__ void direct_issue(const uint8_t* const (&src)[NL], long byte_advance, uint8_t* tile) {
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    uint8_t* dst = tile + (j * THREADS + wave * 64) * 16;      // wave-uniform; lane l lands at dst + 16 l
    if (src[j])
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + byte_advance),
                                       US_LDS_PTR(void, dst), 16, 0, 0);
  }
}

// LDS byte address of a pointer into the workgroup's LDS allocation.
__device__ __forceinline__ uint32_t lds_addr(const uint8_t* p) {
  return (uint32_t)(uintptr_t)US_LDS_PTR(const uint8_t, p);
}

// The transposing LDS reads are issued through inline assembly: the compiler cannot see what they
// read and would otherwise order them after ALL pending direct-to-LDS loads (s_waitcnt vmcnt(0)),
// which would serialise the pipeline.  It therefore does not count them either: every consumer of a
// fragment first passes through frag_ready() below.
template <int OFFSET>
__device__ __forceinline__ v2i ds_read_tr8(uint32_t addr) {
  v2i v;
  asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
  return v;
}
template <int OFFSET>
__device__ __forceinline__ v2i ds_read_tr16(uint32_t addr) {
  v2i v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
  return v;
}
// Wait for every LDS read issued so far and tie the fragment registers to that wait, so that no use
// of them can be scheduled above it.
__device__ __forceinline__ void lds_reads_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
template <class F, int N>
__device__ __forceinline__ void frag_ready(F (&f)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+v"(f[i]));
}

// One of this thread's loads of a stage: number j of the A tile's NA loads, then the B tile's.
template <int THREADS, int NA, int NB>
__device__ __forceinline__ void direct_issue_one(int j, const uint8_t* const (&srcA)[NA], const uint8_t* const (&srcB)[NB],
                                                 long advA, long advB, uint8_t* stage_base, int a_bytes) {
  const int wave = threadIdx.x >> 6;
  const bool is_a = j < NA;
  const int jj = is_a ? j : j - NA;
  const uint8_t* src = is_a ? srcA[jj] : srcB[jj];
  uint8_t* dst = stage_base + (is_a ? 0 : a_bytes) + (jj * THREADS + wave * 64) * 16;
  if (src)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + (is_a ? advA : advB)),
                                     US_LDS_PTR(void, dst), 16, 0, 0);
}

// Fragment = 32 rows (r0..r0+31) x one MFMA's worth of k, number `kstep` within the stage.  Lane l
// supplies row r0 + l%32 and the k-half l/32 (FP8: 32 consecutive k; FP16: 8 consecutive k).
template <bool KC, int PITCH>
__device__ __forceinline__ v8i direct_frag_fp8(const uint8_t* tile, int r0, int kstep) {
  const int l = threadIdx.x & 63;
  v8i f;
  if constexpr (KC) {
    const int r = r0 + (l & 31);
    const int c = kstep * 4 + (l >> 5) * 2;
    const int x = swz<true, true, PITCH>(r);
    const uint8_t* p = tile + r * PITCH;
    v4i lo = *US_LDS_PTR(const v4i, p + ((c ^ x) << 4));
    v4i hi = *US_LDS_PTR(const v4i, p + (((c + 1) ^ x) << 4));
    f = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  } else {
    // 16 lanes cooperate on an 8(k) x 16(row) byte block: lane i points at k-row i/2, row-half i%2,
    // and receives the 8 k values of row (group base + i).  The swizzle only depends on k mod 8
    // (or (k/2) mod 4), which the four reads of a lane share.
    const int i = l & 15;
    const int krow = kstep * 64 + (l >> 5) * 32 + (i >> 1);
    const int col = r0 + ((l >> 4) & 1) * 16 + (i & 1) * 8;
    const uint32_t a = lds_addr(tile + krow * PITCH + (((col >> 4) ^ swz<false, true, PITCH>(krow)) << 4) + (col & 15));
    const v2i v0 = ds_read_tr8<0>(a), v1 = ds_read_tr8<8 * PITCH>(a), v2 = ds_read_tr8<16 * PITCH>(a),
              v3 = ds_read_tr8<24 * PITCH>(a);
    f = {v0.x, v0.y, v1.x, v1.y, v2.x, v2.y, v3.x, v3.y};
  }
  return f;
}

template <bool KC, int PITCH>
__device__ __forceinline__ v8h direct_frag_f16(const uint8_t* tile, int r0, int kstep) {
  const int l = threadIdx.x & 63;
  if constexpr (KC) {
    const int r = r0 + (l & 31);
    const int c = kstep * 2 + (l >> 5);
    return *US_LDS_PTR(const v8h, tile + r * PITCH + ((c ^ swz<true, false, PITCH>(r)) << 4));
  } else {
    // 16 lanes cooperate on a 4(k) x 16(row) block of halves: lane i points at k-row i/4, row quarter
    // i%4, and receives the 4 k values of row (group base + i).
    const int i = l & 15;
    const int krow = kstep * 16 + (l >> 5) * 8 + (i >> 2);
    const int colb = (r0 + ((l >> 4) & 1) * 16 + (i & 3) * 4) * 2;
    const uint32_t a = lds_addr(tile + krow * PITCH + (((colb >> 4) ^ swz<false, false, PITCH>(krow)) << 4) + (colb & 15));
    const v2i lo = ds_read_tr16<0>(a), hi = ds_read_tr16<4 * PITCH>(a);
    v4i w = {lo.x, lo.y, hi.x, hi.y};
    v8h h;
    __builtin_memcpy(&h, &w, 16);
    return h;
  }
}

// s_waitcnt vmcnt(N) alone (lgkmcnt / expcnt fields left at "no wait")
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// One output tile (number `bid` in launch order, K slice `split`) by the whole workgroup; `lds` is the
// workgroup's dynamic LDS (DirectTile::LDS_BYTES).
template <class Cfg, bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI, bool WIDE>
__device__ __forceinline__ void gemm_direct_tile(const GemmArgs& g, int bid, long split, uint8_t* lds) {
  using T = DirectTile<Cfg, FP8, A_KC, B_KC, WIDE, EPI>;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, THREADS = Cfg::THREADS, BKB = Cfg::BKB, NST = Cfg::NST;
  constexpr int FM = Cfg::FM, FN = Cfg::FN;
  constexpr int ES = T::ES;
  constexpr int KSTEPS = (FP8 ? BKB / 64 : BKB / 32) / Cfg::WAVES_K;   // k-steps of a stage this wave works on
  constexpr int PA = T::PA, PB = T::PB;
  constexpr int LOADS = T::A_LOADS + T::B_LOADS;       // per thread and stage

  const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
  int tm, tn;
  tile_of_block(bid, tiles_m, tiles_n, g.xcd_gm, g.xcd_gn, g.grp_w, g.nxcd, tm, tn);
  const long m0 = (long)tm * BM, n0 = (long)tn * BN;
  const long k_begin = split * g.k_per_split;
  const long k_end = (k_begin + g.k_per_split < g.K) ? k_begin + g.k_per_split : g.K;
  const int nstages = (k_end > k_begin) ? (int)((k_end - k_begin) / T::BK) : 0;   // host guarantees divisibility

  const int wave = threadIdx.x >> 6;
  const int wmn = wave % Cfg::WAVES_MN;             // position in the output tile
  const int wk = wave / Cfg::WAVES_MN;              // share of the k-steps
  const int wm0 = (wmn % Cfg::WAVES_M) * Cfg::WM;
  const int wn0 = (wmn / Cfg::WAVES_M) * Cfg::WN;
  const int ks0 = wk * KSTEPS;

  // edge tiles: slots that are never loaded must read as zero
  const bool edge = (m0 + BM > g.M || n0 + BN > g.N);
  if (edge) {
    const v4i z = {0, 0, 0, 0};
    for (int o = threadIdx.x * 16; o < T::RING_BYTES; o += THREADS * 16) *US_LDS_PTR(v4i, lds + o) = z;
    __syncthreads();
  }

  const uint8_t* srcA[T::A_LOADS];
  const uint8_t* srcB[T::B_LOADS];
  direct_sources<THREADS, BM, BKB, A_KC, FP8, PA>(g.A, g.lda, m0, g.M, k_begin, srcA);
  direct_sources<THREADS, BN, BKB, B_KC, FP8, PB>(g.B, g.ldb, n0, g.N, k_begin, srcB);
  const long advA = A_KC ? (long)BKB : (long)T::BK * g.lda * ES;   // bytes per stage
  const long advB = B_KC ? (long)BKB : (long)T::BK * g.ldb * ES;

  v16f acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // fragment registers, two sets: one feeds the MFMAs while the other is being filled
  using FragT = typename std::conditional<FP8, v8i, v8h>::type;
  FragT fa[2][FM], fb[2][FN];
  auto load_frags = [&](FragT (&a)[FM], FragT (&b)[FN], int slot, int ks) {
    const uint8_t* ta = lds + slot * T::STAGE_BYTES;
    const uint8_t* tb = ta + T::A_BYTES;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      if constexpr (FP8) b[j] = direct_frag_fp8<B_KC, PB>(tb, wn0 + j * 32, ks0 + ks);
      else b[j] = direct_frag_f16<B_KC, PB>(tb, wn0 + j * 32, ks0 + ks);
    }
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      if constexpr (FP8) a[i] = direct_frag_fp8<A_KC, PA>(ta, wm0 + i * 32, ks0 + ks);
      else a[i] = direct_frag_f16<A_KC, PA>(ta, wm0 + i * 32, ks0 + ks);
    }
  };
  // one fragment of a k-step: numbers 0 .. FN-1 are the B fragments, FN .. FN+FM-1 the A fragments
  auto load_frag_one = [&](FragT (&a)[FM], FragT (&b)[FN], int slot, int ks, int idx) {
    const uint8_t* ta = lds + slot * T::STAGE_BYTES;
    const uint8_t* tb = ta + T::A_BYTES;
    if (idx < FN) {
      if constexpr (FP8) b[idx] = direct_frag_fp8<B_KC, PB>(tb, wn0 + idx * 32, ks0 + ks);
      else b[idx] = direct_frag_f16<B_KC, PB>(tb, wn0 + idx * 32, ks0 + ks);
    } else {
      const int i = idx - FN;
      if constexpr (FP8) a[i] = direct_frag_fp8<A_KC, PA>(ta, wm0 + i * 32, ks0 + ks);
      else a[i] = direct_frag_f16<A_KC, PA>(ta, wm0 + i * 32, ks0 + ks);
    }
  };
  auto issue_stage = [&](int stage, int slot) {
    direct_issue<THREADS>(srcA, (long)stage * advA, lds + slot * T::STAGE_BYTES);
    direct_issue<THREADS>(srcB, (long)stage * advB, lds + slot * T::STAGE_BYTES + T::A_BYTES);
  };

  // prologue: fill the ring, open stage 0, fetch its first fragments
#pragma unroll
  for (int s = 0; s < NST; ++s)
    if (s < nstages) issue_stage(s, s);
  if (nstages > 0) {
    // (on edge tiles a wave may skip loads whose lanes all lie outside the matrix, so the number of
    // younger loads is not fixed there: wait for everything)
    if (!edge && nstages >= NST) wait_vmcnt<(NST - 1) * LOADS>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    load_frags(fa[0], fb[0], 0, 0);
  }

  // The two fragment sets alternate per k-step.  With an odd number of k-steps per stage (one) the
  // loop body therefore spans two stages, so that the set index stays a compile-time constant.
  constexpr int SPI = (KSTEPS % 2) ? 2 : 1;     // stages per loop iteration
  int slot = 0;                                 // ring slot of the current stage
  bool refill = false;
  int refill_slot = 0, refill_stage = 0;
  for (int s0 = 0; s0 < nstages; s0 += SPI) {
#pragma unroll
    for (int u = 0; u < SPI * KSTEPS; ++u) {
      const int s = s0 + u / KSTEPS;
      const int ks = u % KSTEPS;
      if (SPI > 1 && s >= nstages) break;       // odd stage count: the last iteration is half empty
      FragT (&ca)[FM] = fa[u & 1];
      FragT (&cb)[FN] = fb[u & 1];
      FragT (&na)[FM] = fa[(u + 1) & 1];
      FragT (&nb)[FN] = fb[(u + 1) & 1];
      // the fragments of this k-step were requested one k-step ago
      lds_reads_done();
      frag_ready(ca);
      frag_ready(cb);
      // FP8: the next k-step's fragments are not requested ahead of this k-step's MFMAs but one fragment behind each
      // of the last FM + FN of them, so that a wave that comes out of a wait (or the barrier) feeds the matrix core
      // first (measured on one box: 2.47 -> 2.64 PFLOP/s on a 32768 x 4096 x 16384 product, BERT-large step 256 -> 247 us;
      // behind the first MFMAs instead: 2.55; two per MFMA behind the last three: 2.57; all behind the last: 2.50;
      // FP16, whose MFMAs are half as long: slower either way, so it keeps the requests in front)
      constexpr bool SPREAD = FP8;
      bool frags_pending = false;
      int fslot = slot, fks = ks + 1;
      if (ks + 1 < KSTEPS) {
        if constexpr (SPREAD) frags_pending = true;
        else load_frags(na, nb, slot, ks + 1);
      } else {
        // stage boundary: this wave holds all of stage s in registers
        if (s + 1 < nstages) {
          // own loads of stage s+1 have landed once only the NST-2 younger stages are pending
          if (!edge && s + NST <= nstages) wait_vmcnt<(NST - 2) * LOADS>();
          else wait_vmcnt<0>();
        }
        __builtin_amdgcn_s_barrier();   // stage s+1 complete for everyone; nobody reads stage s any more
        refill = (s + NST < nstages);   // the freed slot receives stage s+NST, a few loads per MFMA below
        refill_slot = slot;
        refill_stage = s + NST;
        if constexpr (EPI == EPI_GELU_GRAD || EPI == EPI_GELU_GRAD_TAB || EPI == EPI_RESIDUAL) {
          // The epilogue's second input (saved pre-activation / skip tensor): from the first boundary that refills
          // nothing any more, no wait of the main loop depends on the load counter, so one 4-byte load per 128-byte
          // line of this wave's share is sent off here (into the slot just freed, never read): the lines are in L2
          // when the epilogue asks for them instead of coming from HBM with every CU asking at once (BERT-large, backward
          // of layer 2: 97.4 -> 93.8 us, same box, same bits).
          if (s + NST == nstages) {
            constexpr int LPR = (Cfg::WN * 2 + 127) / 128;                 // lines per row of the wave's share
            constexpr int ROWS = Cfg::WM / Cfg::WAVES_K;                   // the rows this wave finishes
            const int lane = threadIdx.x & 63;
            uint8_t* dump = lds + refill_slot * T::STAGE_BYTES + wave * 256;
#pragma unroll
            for (int t = 0; t < ROWS * LPR; t += 64) {
              const int u = t + lane;
              const long m = m0 + wm0 + wk * ROWS + u / LPR;
              const long n = n0 + wn0 + (u % LPR) * 64;
              if (u < ROWS * LPR && m < g.M && n < g.N)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g.Zpre + m * g.ldc + n),
                                                 US_LDS_PTR(void, dump), 4, 0, 0);
            }
          }
        }
        if (++slot == NST) slot = 0;
        if (s + 1 < nstages) {
          if constexpr (SPREAD) { frags_pending = true; fslot = slot; fks = 0; }
          else load_frags(na, nb, slot, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the LDS requests (FP16) ahead of the MFMAs they overlap with
      // The refill loads are spread over the MFMAs of this k-step: issued in one burst by all waves
      // they would queue up in the vector-memory pipeline and hold the waves back from the matrix core.
      constexpr int NMFMA = FM * FN;
      constexpr int PER = (LOADS + NMFMA - 1) / NMFMA;
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          if constexpr (FP8) acc[i][j] = mfma_fp8<FB, FA>(cb[j], ca[i], acc[i][j]);
          else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(cb[j], ca[i], acc[i][j], 0, 0, 0);
          if constexpr (SPREAD) {
            constexpr int NFR = FM + FN;
            constexpr int FPER = (NFR + NMFMA - 1) / NMFMA;
#pragma unroll
            for (int q = 0; q < FPER; ++q) {
              const int idx = (i * FN + j) * FPER + q - (NMFMA * FPER - NFR);   // the last NFR places
              if (idx >= 0 && idx < NFR && frags_pending) load_frag_one(na, nb, fslot, fks, idx);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          if (ks + 1 == KSTEPS) {
#pragma unroll
            for (int q = 0; q < PER; ++q) {
              const int l = (i * FN + j) * PER + q;
              if (l < LOADS && refill)
                direct_issue_one<THREADS>(l, srcA, srcB, (long)refill_stage * advA, (long)refill_stage * advB,
                                          lds + refill_slot * T::STAGE_BYTES, T::A_BYTES);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      __builtin_amdgcn_sched_barrier(0);   // ... and the MFMAs ahead of the next k-step's wait
    }
  }

  __syncthreads();       // every wave is past its last fragment read before the strips overlay the ring
  if constexpr (Cfg::WAVES_K > 1) {
    // Two wave groups hold partial sums of the same tile.  Each group finishes one half of the rows:
    // it hands the other half of its accumulators to its partner through LDS and adds the partner's
    // half to its own (one addition of two terms per element, so the order does not matter and the
    // result is deterministic).  Register r of lane l travels through red[wk][wmn][r][l].
    static_assert(Cfg::WAVES_K == 2 && FM % 2 == 0, "two groups, an even number of 32-row blocks");
    constexpr int HALF = FM / 2, NR = HALF * FN * 16;
    float* red = reinterpret_cast<float*>(lds);
    const int lane = threadIdx.x & 63;
    float* mine = red + ((size_t)(wk * Cfg::WAVES_MN + wmn) * NR) * 64 + lane;
    const float* theirs = red + ((size_t)((wk ^ 1) * Cfg::WAVES_MN + wmn) * NR) * 64 + lane;
    auto send = [&](auto I0c) {          // the rows the partner finishes
      constexpr int I0 = decltype(I0c)::value;
#pragma unroll
      for (int i = 0; i < HALF; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) *US_LDS_PTR(float, mine + ((i * FN + j) * 16 + r) * 64) = acc[I0 + i][j][r];
    };
    auto receive = [&](auto I0c) {       // the rows this wave finishes
      constexpr int I0 = decltype(I0c)::value;
#pragma unroll
      for (int i = 0; i < HALF; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[I0 + i][j][r] += *US_LDS_PTR(const float, theirs + ((i * FN + j) * 16 + r) * 64);
          __builtin_amdgcn_sched_barrier(0);   // one block of 16 at a time keeps the register count down
        }
    };
    if (wk == 0) send(std::integral_constant<int, HALF>{});
    else send(std::integral_constant<int, 0>{});
    __syncthreads();
    if (wk == 0) receive(std::integral_constant<int, 0>{});
    else receive(std::integral_constant<int, HALF>{});
    __syncthreads();     // everything exchanged: the strips may overlay the exchange area
    if (wk == 0) store_block_epilogue<Cfg, EPI, WIDE, 0, HALF, epilogue_takes_bias<A_KC, B_KC, EPI, WIDE>()>(g, acc, lds, m0, n0, split);
    else store_block_epilogue<Cfg, EPI, WIDE, HALF, FM, epilogue_takes_bias<A_KC, B_KC, EPI, WIDE>()>(g, acc, lds, m0, n0, split);
    return;
  }
  store_block_epilogue<Cfg, EPI, WIDE, 0, Cfg::FM, epilogue_takes_bias<A_KC, B_KC, EPI, WIDE>()>(g, acc, lds, m0, n0, split);
}

template <class Cfg, bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI, bool WIDE>
__global__ void __launch_bounds__(Cfg::THREADS, Cfg::MINB) gemm_direct_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  if constexpr (EPI == EPI_STORE) select_batch_item(g);
  gemm_direct_tile<Cfg, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(g, (int)blockIdx.x, (long)blockIdx.y, lds);
}

// Two independent GEMMs in one launch (the two products of a layer's backward pass), for tile shapes
// with the same workgroup size: the first nb workgroups work on problem B (grad_W: few tiles, long main
// loop), the rest on problem A (grad_X).  Compared with two launches there is no drain between the
// two, and because the B tiles finish at slightly different times the A tiles start staggered: their
// epilogues (GELU' over a large output: a burst of HBM reads, vector ALU work, HBM writes) no longer
// hit every CU at the same moment, while launched on their own all CUs run in lockstep.  (Interleaving
// A and B tiles more finely was measured to be slower than either.)
// nb must be a multiple of the number of XCDs, so that both problems keep their XCD-aware tile walk.
template <class Cfg, bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI, bool WIDE>
struct GemmKind {
  using Tile = DirectTile<Cfg, FP8, A_KC, B_KC, WIDE, EPI>;
  static constexpr int THREADS = Cfg::THREADS, BM = Cfg::BM, BN = Cfg::BN;
  static constexpr int WAVES_K = Cfg::WAVES_K, NST = Cfg::NST, EPI_ = EPI;
  static constexpr bool IS_FP8 = FP8, A_KC_ = A_KC, B_KC_ = B_KC;
  __device__ static __forceinline__ void run(const GemmArgs& g, int bid, uint8_t* lds) {
    gemm_direct_tile<Cfg, FP8, FA, FB, A_KC, B_KC, EPI, WIDE>(g, bid, 0, lds);
  }
};

template <class KA, class KB>
__global__ void __launch_bounds__(KA::THREADS, 1) gemm_pair_kernel(GemmArgs a, GemmArgs b, int nb) {
  static_assert(KA::THREADS == KB::THREADS, "one workgroup size for both problems");
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int bid = (int)blockIdx.x;
  if (bid < nb) KB::run(b, bid, lds);
  else KA::run(a, bid - nb, lds);
}

}  // namespace us
