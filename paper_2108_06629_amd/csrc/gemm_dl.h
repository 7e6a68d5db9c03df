// bf16 matrix-core GEMM main loop with direct global->LDS loads and a ring of LDS stages.
//
// Used for the three products of a layer (Eq. 1, Eq. 4, Eq. 5) whenever every contiguous run of both
// operands starts on a multiple of 8 elements (16-byte chunks); other shapes take the register-staged
// loop of gemm_core.h.  Differences from that loop:
//   * tiles travel global -> LDS with buffer_load ... lds (16 bytes per lane, a wave fills 1 KB of LDS
//     in lane order): no staging registers, no LDS store instructions, and the loads of tile t+4 are
//     issued while tile t is being multiplied, so about three K steps of latency are covered;
//   * an operand whose k index is strided in memory stays in its memory order in LDS ([k][row], row
//     contiguous) and is transposed by the LDS read itself (ds_read_b64_tr_b16): within a group of 16
//     lanes, lane 4j+a supplies the address of four consecutive elements of k-row j, and lane i
//     receives element i of each of the four k-rows;
//   * K step BK (BK/16 MFMA substeps), NSTAGE stages, one barrier per step, placed before the last
//     substep: before it a wave waits for its own loads of tile t+1, after it stage t%NSTAGE is free and
//     receives tile t+NSTAGE, and the last substep's MFMAs cover the first fragment reads of tile t+1.
//     (BK, NSTAGE) = (32, 4) or (64, 2): both fill 128 KB of LDS for a 256 x 256 tile.
// The swizzle that keeps LDS reads conflict-free is applied on the global side: the lane that owns
// LDS chunk p of a row fetches global chunk p ^ f(row).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "gemm_core.h"

namespace lp {
namespace dl {

using core::bf16x8;
using core::f32x16;
using core::f32x4;
using core::kOOB;

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));


typedef __attribute__((address_space(3))) unsigned int* lds_u32_ptr;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

// One wave copies 64 x 16 bytes from a buffer to LDS: lane L's bytes land at lds_base + 16 L.
// Written as inline assembly so that the compiler does not track the asynchronous LDS write: it
// would otherwise drain *all* loads in flight (vmcnt(0)) in front of the transposing LDS reads.
// Ordering is explicit instead: wait_vmcnt + barrier before a stage is read.  lds_base is
// wave-uniform; voff is the per-lane byte offset (kOOB = out of range: zeros are written).
__device__ __forceinline__ void load_to_lds_16(__amdgpu_buffer_rsrc_t rs, unsigned voff, unsigned short* lds_base) {
  const unsigned addr = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lds_u32_ptr)lds_base);
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" : : "s"(addr), "v"(voff), "s"(rs) : "memory");
}

// ---- operand with k contiguous in memory: element (r,k) at base[r*ld + k] ------------------------
// LDS stage: [R][BK] halves; chunk p of row r holds global chunk p ^ swz(r), swz as in core::lds_off.
template <int R, int BK, int NWAVES>
struct OperandKC {
  static constexpr int STAGE_ELEMS = R * BK;
  static constexpr int CPR = BK / 8;                         // chunks per row
  static constexpr int RP = 128 / BK;                        // rows per 256 bytes
  static constexpr int ROWS_PER_LOAD = 64 / CPR;             // rows per 1 KB wave load
  static constexpr int WAVELOADS = R / ROWS_PER_LOAD;
  static constexpr int PER_WAVE = WAVELOADS / NWAVES;
  static_assert(BK == 32 || BK == 64, "");
  static_assert(WAVELOADS % NWAVES == 0, "rows must split evenly over the waves");
  __amdgpu_buffer_rsrc_t rs;
  int r0, Rtot, Ktot, ld;
  // lane-constant parts
  int lrow, lpos;
  __device__ __forceinline__ void init(const void* p, unsigned bytes, int r0_, int Rtot_, int Ktot_, int ld_) {
    rs = core::make_rsrc(p, bytes);
    r0 = r0_; Rtot = Rtot_; Ktot = Ktot_; ld = ld_;
    const int lane = threadIdx.x & 63;
    lrow = lane / CPR;
    lpos = lane % CPR;
  }
  // load i of this wave (of PER_WAVE) for the tile that starts at reduction index k0
  __device__ __forceinline__ void issue_one(int i, int k0, unsigned short* stage, int wave_u) const {
    const int g = wave_u * PER_WAVE + i;                    // group of ROWS_PER_LOAD rows
    const int trow = g * ROWS_PER_LOAD + lrow;             // row inside the tile
    const int chunk = lpos ^ ((trow / RP) % CPR);           // the swizzle of core::lds_off, applied on the global side
    const int row = r0 + trow, k = k0 + chunk * 8;
    const unsigned off = (row < Rtot && k < Ktot) ? ((unsigned)row * (unsigned)ld + (unsigned)k) * 2u : kOOB;
    load_to_lds_16(rs, off, stage + g * 512);
  }
  // all waves together fill one stage with the tile that starts at reduction index k0
  __device__ __forceinline__ void issue(int k0, unsigned short* stage, int wave_u) const {
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) issue_one(i, k0, stage, wave_u);
  }
  // The same loads for a tile whose BK reduction indices all exist: the byte offset is a per-lane
  // constant (row part, kOOB for a row past the end: adding koff keeps it out of range) plus koff(k0).
  static constexpr bool SPLIT_ISSUE = true;
  unsigned base[PER_WAVE];
  __device__ __forceinline__ void prepare(int wave_u) {
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
      const int trow = (wave_u * PER_WAVE + i) * ROWS_PER_LOAD + lrow;
      const int chunk = lpos ^ ((trow / RP) % CPR);
      const int row = r0 + trow;
      base[i] = row < Rtot ? ((unsigned)row * (unsigned)ld + (unsigned)(chunk * 8)) * 2u : kOOB;
    }
  }
  __device__ __forceinline__ unsigned koff(int k0) const { return (unsigned)k0 * 2u; }
  __device__ __forceinline__ void issue_one_full(int i, unsigned koff_, unsigned short* stage, int wave_u) const {
    load_to_lds_16(rs, base[i] + koff_, stage + (wave_u * PER_WAVE + i) * 512);
  }
  // fragment of MFMA tile rows [row0, row0+32), k substep kk: lane (r = lane&31, g = lane>>5) gets k = 16kk + 8g + 0..7
  __device__ __forceinline__ bf16x8 frag(const unsigned short* stage, int row0, int kk) const {
    const int lane = threadIdx.x & 63;
    const int row = row0 + (lane & 31), chunk = kk * 2 + (lane >> 5);
    return *(const bf16x8*)(stage + core::lds_off<BK>(row, chunk));
  }
};

// ---- operand with k strided in memory: element (r,k) at base[k*ld + r] ---------------------------
// LDS stage: [BK][R] halves, chunk p of k-row k holds global chunk p ^ swz(k).  A transposing read of
// half a wave touches four consecutive k-rows, 64 bytes of each; swz moves those four segments onto
// different quarters of the 256-byte bank line: rows of 256 or 512 bytes (R = 128, 256) all start on the
// same quarter, so row k moves by k & 3 quarters; rows of 128 bytes (R = 64) alternate between two
// quarters by themselves, so rows 2 and 3 of a group move by one.
template <int R, int BK, int NWAVES>
struct OperandKS {
  static_assert(R == 64 || R == 128 || R == 256, "row length of 8, 16 or 32 chunks");
  static __device__ __forceinline__ int swz(int k) { return R == 64 ? ((k >> 1) & 1) << 2 : (k & 3) << 2; }
  static constexpr int STAGE_ELEMS = R * BK;
  static constexpr int CPR = R / 8;                          // chunks per k-row
  static constexpr int ROWS_PER_LOAD = 64 / CPR;             // k-rows per 1 KB wave load
  static constexpr int WAVELOADS = BK / ROWS_PER_LOAD;
  static constexpr int PER_WAVE = WAVELOADS / NWAVES;
  static_assert(WAVELOADS % NWAVES == 0, "k-rows must split evenly over the waves");
  __amdgpu_buffer_rsrc_t rs;
  int r0, Rtot, Ktot, ld;
  int lk, lpos;
  __device__ __forceinline__ void init(const void* p, unsigned bytes, int r0_, int Rtot_, int Ktot_, int ld_) {
    rs = core::make_rsrc(p, bytes);
    r0 = r0_; Rtot = Rtot_; Ktot = Ktot_; ld = ld_;
    const int lane = threadIdx.x & 63;
    lk = lane / CPR;
    lpos = lane % CPR;
  }
  __device__ __forceinline__ void issue_one(int i, int k0, unsigned short* stage, int wave_u) const {
    const int g = wave_u * PER_WAVE + i;
    const int kr = g * ROWS_PER_LOAD + lk;                   // k-row inside the tile
    const int chunk = lpos ^ swz(kr);
    const int k = k0 + kr, r = r0 + chunk * 8;
    const unsigned off = (k < Ktot && r < Rtot) ? ((unsigned)k * (unsigned)ld + (unsigned)r) * 2u : kOOB;
    load_to_lds_16(rs, off, stage + g * 512);
  }
  __device__ __forceinline__ void issue(int k0, unsigned short* stage, int wave_u) const {
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) issue_one(i, k0, stage, wave_u);
  }
  // full tiles: per-lane constant (k-row inside the tile and column part) plus koff(k0), as in OperandKC
  static constexpr bool SPLIT_ISSUE = true;
  unsigned base[PER_WAVE];
  __device__ __forceinline__ void prepare(int wave_u) {
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
      const int kr = (wave_u * PER_WAVE + i) * ROWS_PER_LOAD + lk;
      const int chunk = lpos ^ swz(kr);
      const int r = r0 + chunk * 8;
      base[i] = r < Rtot ? ((unsigned)kr * (unsigned)ld + (unsigned)r) * 2u : kOOB;
    }
  }
  __device__ __forceinline__ unsigned koff(int k0) const { return (unsigned)k0 * (unsigned)ld * 2u; }
  __device__ __forceinline__ void issue_one_full(int i, unsigned koff_, unsigned short* stage, int wave_u) const {
    load_to_lds_16(rs, base[i] + koff_, stage + (wave_u * PER_WAVE + i) * 512);
  }
  __device__ __forceinline__ bf16x8 frag(const unsigned short* stage, int row0, int kk) const {
    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15, j = l16 >> 2, a = l16 & 3;
    const int col = row0 + ((lane >> 4) & 1) * 16 + a * 4;  // first of the four elements this lane points at
    const int k = kk * 16 + (lane >> 5) * 8 + j;             // k & 3 == j for both halves
    const int chunk = (col >> 3) ^ swz(j);
    const unsigned short* p = stage + k * R + chunk * 8 + (col & 7);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * R));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
};

template <bool KC, int R, int BK, int NWAVES>
struct OperandSel {
  using type = OperandKC<R, BK, NWAVES>;
};
template <int R, int BK, int NWAVES>
struct OperandSel<false, R, BK, NWAVES> {
  using type = OperandKS<R, BK, NWAVES>;
};

// s_waitcnt with vmcnt <= n (expcnt and lgkmcnt untouched)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// smem: NSTAGE * (BM + BN) * BK halves.  Multiplies the KT K-tiles that start at reduction index k_base
// (split-K: a workgroup takes a K range and the operands' Ktot is the end of that range).
template <int BM, int BN, int BK, int NSTAGE, int WM, int WN, class OA, class OB, class Epi>
__device__ __forceinline__ void gemm_tile_dl(const OA& oa_in, const OB& ob_in, int k_base, int KT, unsigned short* smem, Epi epi) {
  OA oa = oa_in;
  OB ob = ob_in;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int A_ELEMS = BM * BK, B_ELEMS = BN * BK, STAGE = A_ELEMS + B_ELEMS;
  constexpr int LOADS = OA::PER_WAVE + OB::PER_WAVE;        // buffer loads per lane per tile
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8 fa[2][TM], fb[2][TN];
  // Fragments are read in the order the MFMAs consume them (b[0], a[0..TM-1], b[1], ...: the MFMAs walk
  // down a column of the wave's tile before moving to the next), one read after each MFMA of the
  // previous substep, so every fragment has the same head start of about NMFMA - 1 matrix instructions.
  auto read_frags = [&](const unsigned short* st, int kk, bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
    b[0] = ob.frag(st + A_ELEMS, wn * (TN * 32), kk);
#pragma unroll
    for (int i = 0; i < TM; ++i) a[i] = oa.frag(st, wm * (TM * 32) + i * 32, kk);
#pragma unroll
    for (int j = 1; j < TN; ++j) b[j] = ob.frag(st + A_ELEMS, wn * (TN * 32) + j * 32, kk);
  };
  auto mfmas = [&](bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int i = 0; i < TM; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };
  // tiles past the end are "loaded" too (every chunk out of range, so zeros and no memory traffic):
  // the number of loads in flight stays the same in every iteration, which keeps the vmcnt waits exact
  auto issue = [&](int t) {
    unsigned short* st = smem + (t % NSTAGE) * STAGE;
    oa.issue(k_base + t * BK, st, wave);
    ob.issue(k_base + t * BK, st + A_ELEMS, wave);
  };

  // scheduling pattern of one substep: one LDS fragment read after each of the first MFMAs
  constexpr int NREAD = TM + TN, NMFMA = TM * TN, NPAIR = NREAD < NMFMA ? NREAD : NMFMA;
  auto interleave_reads = [&]() {
#pragma unroll
    for (int q = 0; q < NPAIR; ++q) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
  };

#pragma unroll
  for (int t = 0; t < NSTAGE; ++t) issue(t);
  wait_vmcnt<(NSTAGE - 1) * LOADS>();
  __syncthreads();
  read_frags(smem, 0, fa[0], fb[0]);

  constexpr int KS = BK / 16;   // MFMA substeps per K step
  auto substeps = [&](int t) {  // all but the last substep of tile t
    const unsigned short* cur = smem + (t % NSTAGE) * STAGE;
#pragma unroll
    for (int kk = 0; kk + 1 < KS; ++kk) {
      read_frags(cur, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
      mfmas(fa[kk & 1], fb[kk & 1]);
      interleave_reads();
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  if constexpr (OA::SPLIT_ISSUE && OB::SPLIT_ISSUE) {
    // The refill of the freed stage and the first fragment reads of tile t+1 are dealt out over the
    // MFMAs of the last substep, one slot per MFMA with the MFMA first, so that the matrix pipe has
    // work from the first cycle after the barrier while the addresses of the loads are formed.
    constexpr int NFRAG = TM + TN;
    oa.prepare(wave);
    ob.prepare(wave);
    auto last_substep = [&](int t, auto full) {
      unsigned short* st = smem + (t % NSTAGE) * STAGE;
      const unsigned short* nxt = smem + ((t + 1) % NSTAGE) * STAGE;
      const int k0 = k_base + (t + NSTAGE) * BK;
      const unsigned koa = oa.koff(k0), kob = ob.koff(k0);
      bf16x8(&ca)[TM] = fa[(KS - 1) & 1];
      bf16x8(&cb)[TN] = fb[(KS - 1) & 1];
      bf16x8(&na)[TM] = fa[KS & 1];
      bf16x8(&nb)[TN] = fb[KS & 1];
#pragma unroll
      for (int q = 0; q < NMFMA; ++q) {
        const int i = q % TM, j = q / TM;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[i], cb[j], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) {   // consumption order: b[0], a[0..TM-1], b[1..]
          if ((NFRAG <= NMFMA ? f : f * NMFMA / NFRAG) != q) continue;
          if (f == 0) nb[0] = ob.frag(nxt + A_ELEMS, wn * (TN * 32), 0);
          else if (f <= TM) na[f - 1] = oa.frag(nxt, wm * (TM * 32) + (f - 1) * 32, 0);
          else nb[f - TM] = ob.frag(nxt + A_ELEMS, wn * (TN * 32) + (f - TM) * 32, 0);
        }
#pragma unroll
        for (int l = 0; l < LOADS; ++l) {
          if ((LOADS <= NMFMA ? l : l * NMFMA / LOADS) != q) continue;
          if (l < OA::PER_WAVE) {
            if constexpr (decltype(full)::value) oa.issue_one_full(l, koa, st, wave);
            else oa.issue_one(l, k0, st, wave);
          } else {
            if constexpr (decltype(full)::value) ob.issue_one_full(l - OA::PER_WAVE, kob, st + A_ELEMS, wave);
            else ob.issue_one(l - OA::PER_WAVE, k0, st + A_ELEMS, wave);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // tiles [0, full_tiles) have all BK reduction indices; iteration t refills with tile t + NSTAGE
    const int full_tiles = (oa.Ktot - k_base) / BK;
    const int t_full = full_tiles - NSTAGE < KT ? full_tiles - NSTAGE : KT;
    int t = 0;
    for (; t < t_full; ++t) {
      substeps(t);
      wait_vmcnt<(NSTAGE - 2) * LOADS>();   // this wave's part of tile t+1 has landed
      __syncthreads();                      // ... and everyone's; nobody reads tile t's stage any more
      last_substep(t, std::true_type{});
    }
    for (; t < KT; ++t) {
      substeps(t);
      wait_vmcnt<(NSTAGE - 2) * LOADS>();
      __syncthreads();
      last_substep(t, std::false_type{});
    }
  } else {
    for (int t = 0; t < KT; ++t) {
      const unsigned short* nxt = smem + ((t + 1) % NSTAGE) * STAGE;
      substeps(t);
      wait_vmcnt<(NSTAGE - 2) * LOADS>();   // this wave's part of tile t+1 has landed
      __syncthreads();                      // ... and everyone's; nobody reads tile t's stage any more
      issue(t + NSTAGE);
      read_frags(nxt, 0, fa[KS & 1], fb[KS & 1]);
      mfmas(fa[(KS - 1) & 1], fb[(KS - 1) & 1]);
      interleave_reads();
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  wait_vmcnt<0>();   // the trailing (empty) tiles still write LDS
  __syncthreads();

  static_assert(WM * WN * 32 * (TN * 32 + 8) * 4 <= NSTAGE * STAGE * 2, "epilogue band does not fit the ring");
  core::epilogue_through_lds<TM, TN>(reinterpret_cast<float*>(smem), acc, wave, lane, wm * (TM * 32), wn * (TN * 32), epi);
}

}  // namespace dl
}  // namespace lp
