// Device-side building blocks of the bf16 matrix-core GEMMs (fully connected and implicit-GEMM
// convolution products of Eq. 1, Eq. 4, Eq. 5).
//
// Each workgroup owns a BM x BN tile of C and walks K in steps of BK.  Both operand tiles are staged
// in LDS in one canonical form, [row][k] with k contiguous, so the MFMA fragment reads are the same
// 16-byte ds_read for every product; an operand whose k index is strided in memory is transposed in
// registers (8x8 blocks of 16-bit values) on its way from global memory to LDS.  LDS rows are
// XOR-swizzled in 16-byte chunks so that the 16 lanes of a fragment read touch all banks.  Global
// loads go through buffer resources, so out-of-range chunks read as zero without branches.  Two LDS
// buffers and two fragment register sets (see gemm_tile for the schedule), one barrier per K step.
// Accumulators are 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16), TM x TN of them per wave.
//
// A "stage" object owns the addressing of one operand: gload(k0) fetches its part of the tile that
// starts at reduction index k0 into registers, sstore(lds) writes it to LDS.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

namespace lp {
namespace core {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned short bf16_bits(float v) {
  __bf16 b = (__bf16)v;  // round-to-nearest-even
  return __builtin_bit_cast(unsigned short, b);
}
__device__ __forceinline__ float bf16_to_f32(unsigned short b) { return __uint_as_float(((unsigned)b) << 16); }

// GELU (exact erf form, f(z) = z Phi(z)) for the products' epilogues, where the activation's arithmetic is exposed:
// Phi(-|z|) = erfc(|z| / sqrt 2) / 2 = t Q(t) exp(-z^2 / 2) / 2 with t = 1 / (1 + |z| / (2 sqrt 2)) and Q a degree-10
// polynomial (own least-squares fit of erfc(x) exp(x^2) / t on Chebyshev nodes in t over x >= 0: relative error of erfc
// 2e-7), one reciprocal and one exponential per element and no branches.  Over all bfloat16 inputs its rounded result
// differs from the correctly rounded one only below z = -7.7 (values of 1e-14), as often as the library erf form does.
__device__ __forceinline__ float gelu_erfc_poly(float z) {
  const float ax = fabsf(z) * 0.70710678118654752440f;
  const float t = __frcp_rn(fmaf(0.5f, ax, 1.f));
  const float e = __expf(-ax * ax);
  float q = 4.317306590e-02f;
  q = fmaf(q, t, -2.346054905e-01f); q = fmaf(q, t, 4.933857416e-01f); q = fmaf(q, t, -4.545637179e-01f);
  q = fmaf(q, t, 1.318500400e-01f); q = fmaf(q, t, -5.905090993e-02f); q = fmaf(q, t, 9.341474848e-02f);
  q = fmaf(q, t, 1.753240754e-01f); q = fmaf(q, t, 2.468838798e-01f); q = fmaf(q, t, 2.820937768e-01f);
  q = fmaf(q, t, 2.820947951e-01f);
  const float lower = 0.5f * t * q * e;          // Phi(-|z|)
  return z * (z < 0.f ? lower : 1.f - lower);
}

__device__ __forceinline__ float apply_act(float z, int act) {
  if (act == 1) return z > 0.f ? z : 0.f;                                          // ReLU
  if (act == 2) return gelu_erfc_poly(z);                                         // GELU (erf form)
  if (act == 3) return tanhf(z);
  if (act == 4) return 1.f / (1.f + expf(-z));                                      // sigmoid
  return z;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, (int)bytes, 0x00020000);
}

constexpr unsigned kOOB = 0x80000000u;  // byte offset past any buffer this library accepts: reads 0

// 8 consecutive 16-bit elements starting at element offset `eoff`; the first `nvalid` (<= 8) exist.
template <bool ALIGNED>
__device__ __forceinline__ u32x4 load8(__amdgpu_buffer_rsrc_t r, unsigned eoff, int nvalid) {
  if constexpr (ALIGNED) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, nvalid > 0 ? eoff * 2u : kOOB, 0, 0);
  } else {
    unsigned e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      e[i] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, i < nvalid ? (eoff + i) * 2u : kOOB, 0, 0);
    u32x4 v;
    v[0] = e[0] | (e[1] << 16);
    v[1] = e[2] | (e[3] << 16);
    v[2] = e[4] | (e[5] << 16);
    v[3] = e[6] | (e[7] << 16);
    return v;
  }
}

__device__ __forceinline__ int clamp8(int n) { return n < 0 ? 0 : (n > 8 ? 8 : n); }

// x[j][e] (8 rows of 8 halves)  ->  y[e][j]
__device__ __forceinline__ void transpose8x8(const u32x4 (&x)[8], u32x4 (&y)[8]) {
#pragma unroll
  for (int dp = 0; dp < 4; ++dp) {  // source dword dp holds columns e = 2dp, 2dp+1
#pragma unroll
    for (int d = 0; d < 4; ++d) {   // destination dword d holds rows j = 2d, 2d+1
      const unsigned lo = x[2 * d][dp], hi = x[2 * d + 1][dp];
      y[2 * dp][d] = (lo & 0xffffu) | (hi << 16);
      y[2 * dp + 1][d] = (lo >> 16) | (hi & 0xffff0000u);
    }
  }
}

// element offset of 16-byte chunk `chunk` of row `row` in a swizzled [rows][BK] LDS tile
template <int BK>
__device__ __forceinline__ int lds_off(int row, int chunk) {
  constexpr int CPR = BK / 8;                          // chunks per row
  constexpr int RP = (128 / BK) > 0 ? (128 / BK) : 1;  // rows per 256 bytes
  return row * BK + ((chunk ^ ((row / RP) % CPR)) * 8);
}

// ---- plain 2-D operands ---------------------------------------------------------------------------
// k contiguous in memory: element (r,k) at base[r*ld + k]
template <int R, int BK, int NT, bool ALIGNED>
struct StageKC {
  static constexpr int NCH = R * BK / 8;
  static constexpr int CH = (NCH + NT - 1) / NT;
  __amdgpu_buffer_rsrc_t rs;
  int r0, Rtot, Ktot, ld, tid;
  u32x4 v[CH];
  __device__ __forceinline__ void gload(int k0) {
#pragma unroll
    for (int it = 0; it < CH; ++it) {
      const int id = it * NT + tid;
      const int row = id / (BK / 8), kc = id % (BK / 8);
      const int gr = r0 + row, gk = k0 + kc * 8;
      const int nv = (gr < Rtot && (NCH % NT == 0 || id < NCH)) ? clamp8(Ktot - gk) : 0;
      v[it] = load8<ALIGNED>(rs, (unsigned)gr * (unsigned)ld + (unsigned)gk, nv);
    }
  }
  __device__ __forceinline__ void sstore(unsigned short* lds) {
#pragma unroll
    for (int it = 0; it < CH; ++it) {
      const int id = it * NT + tid;
      if (NCH % NT == 0 || id < NCH) *(u32x4*)(lds + lds_off<BK>(id / (BK / 8), id % (BK / 8))) = v[it];
    }
  }
};

// k strided in memory: element (r,k) at base[k*ld + r]; threads move 8(k) x 8(r) blocks
template <int R, int BK, int NT, bool ALIGNED>
struct StageKS {
  static constexpr int NB = (BK / 8) * (R / 8);
  static constexpr int IT = (NB + NT - 1) / NT;
  __amdgpu_buffer_rsrc_t rs;
  int r0, Rtot, Ktot, ld, tid;  // tid may be rotated by the caller to spread work over waves
  u32x4 v[IT][8];
  __device__ __forceinline__ void gload(int k0) {
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int id = it * NT + tid;
      if (NB % NT == 0 || id < NB) {
        const int rc = id % (R / 8), kg = id / (R / 8);
        const int gr = r0 + rc * 8;
        const int nvr = clamp8(Rtot - gr);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int gk = k0 + kg * 8 + j;
          v[it][j] = load8<ALIGNED>(rs, (unsigned)gk * (unsigned)ld + (unsigned)gr, gk < Ktot ? nvr : 0);
        }
      }
    }
  }
  __device__ __forceinline__ void sstore(unsigned short* lds) {
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int id = it * NT + tid;
      if (NB % NT == 0 || id < NB) {
        const int rc = id % (R / 8), kg = id / (R / 8);
        u32x4 y[8];
        transpose8x8(v[it], y);
#pragma unroll
        for (int e = 0; e < 8; ++e) *(u32x4*)(lds + lds_off<BK>(rc * 8 + e, kg)) = y[e];
      }
    }
  }
};

// Tile of a workgroup.  Workgroup ids that are congruent mod 8 run on the same XCD and share its L2;
// ids are handed out in increasing order, so with one resident workgroup per CU the 256 CUs work on
// ids [256 w, 256 w + 256) at about the same time.
//
// SUPER = true (tile grid a multiple of 16 x 16, one workgroup per CU): each XCD takes an 8 x 4 block
// of tiles (its 32 CUs share 8 A panels and 4 B panels through L2) and the eight XCDs' blocks form a
// 16 x 16 super-block, so operand panels that several XCDs need at the same time come out of HBM once.
// Otherwise: each XCD gets a contiguous range of logical ids, walked in groups of 8 tile rows.
template <bool SUPER>
__device__ __forceinline__ void tile_of_block(int pid, int nbm, int nbn, int& tm, int& tn) {
  const int xcd = pid % 8, loc = pid / 8;
  if (SUPER && nbm % 16 == 0 && nbn % 16 == 0) {
    const int w = loc / 32, i = loc % 32;       // super-block, tile inside the XCD's 8 x 4 block
    const int sbm = nbm / 16;
    const int sr = w % sbm, sc = w / sbm;       // super-blocks walked down the rows first
    tm = sr * 16 + (xcd % 2) * 8 + (i % 8);
    tn = sc * 16 + (xcd / 2) * 4 + (i / 8);
    return;
  }
  const int nb = nbm * nbn;
  const int per = nb / 8, rem = nb % 8;
  const int lid = xcd * per + (xcd < rem ? xcd : rem) + loc;
  constexpr int GM = 8;
  const int width = GM * nbn;
  const int first = (lid / width) * GM;
  const int gsz = (nbm - first) < GM ? (nbm - first) : GM;
  tm = first + (lid % width) % gsz;
  tn = (lid % width) / gsz;
}

// Accumulators of one wave (TM x TN blocks of 32 x 32, the layout v_mfma_f32_32x32x16 leaves them in) to memory: band by
// band of 32 rows through this wave's strip of LDS, so that a lane then owns four consecutive columns of a row and a
// wavefront writes whole 128-byte lines.  `smem` must be free (all waves past their last fragment read) and hold
// waves x 32 x (TN*32+8) floats.  epi is asked once for a view with its run-time switches turned into compile-time
// constants (with_static_act); a view that needs a second operand per output element (kHasSide: the stash of a fused
// Hadamard product) is asked for it one band ahead, so that those loads are in flight during the trip through LDS.
struct NoSide {};
template <int TM, int TN, class Epi>
__device__ __forceinline__ void epilogue_through_lds(float* smem, const f32x16 (&acc)[TM][TN], int wave, int lane, int row0, int col0,
                                                     const Epi& epi) {
  constexpr int EP_LD = TN * 32 + 8;
  constexpr int NE = 4 * TN;   // 16-byte groups of a band per lane
  float* ep = smem + wave * (32 * EP_LD);
  epi.with_static_act([&](auto store) {
    using Store = decltype(store);
    using Side = typename Store::Side;
    Side side[2][NE];
    auto fetch = [&](int i, Side (&sd)[NE]) {
#pragma unroll
      for (int q = 0; q < NE; ++q) {
        const int e = lane + 64 * q;
        sd[q] = store.side(row0 + i * 32 + e / (TN * 8), col0 + (e % (TN * 8)) * 4);
      }
    };
    if constexpr (Store::kHasSide) fetch(0, side[0]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if constexpr (Store::kHasSide) {
        if (i + 1 < TM) fetch(i + 1, side[(i + 1) & 1]);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          ep[((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * EP_LD + j * 32 + (lane & 31)] = acc[i][j][r];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      if constexpr (Store::kHasSide) {
#pragma unroll
        for (int q = 0; q < NE; ++q) {
          const int e = lane + 64 * q;
          const int row = e / (TN * 8), c4 = e % (TN * 8);
          const f32x4 v = *reinterpret_cast<const f32x4*>(ep + row * EP_LD + c4 * 4);
          store(row0 + i * 32 + row, col0 + c4 * 4, v, side[i & 1][q]);
        }
      } else {
#pragma unroll 4
        for (int e = lane; e < 32 * TN * 8; e += 64) {
          const int row = e / (TN * 8), c4 = e % (TN * 8);
          const f32x4 v = *reinterpret_cast<const f32x4*>(ep + row * EP_LD + c4 * 4);
          store(row0 + i * 32 + row, col0 + c4 * 4, v);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  });
}

// Accumulates K tiles [kt0, kt1) of the BM x BN tile and hands the result to epi(row_in_tile,
// col_in_tile, four consecutive columns).  smem: 2 * (BM + BN) * BK halves.
//
// Schedule of one K step (BK = 64 = four MFMA substeps of k = 16), written so that the matrix pipe
// never waits for a barrier with nothing queued behind it:
//   top        global loads of tile t+1 are issued into registers
//   substep 0  MFMAs on fragments fetched earlier, interleaved with the LDS reads of substep 1
//   substep 1  same, reading substep 2
//   substep 2  same, reading substep 3, then the LDS stores of tile t+1 (other buffer), two per MFMA
//   barrier    tile t+1 is now visible, and every wave already holds its last fragments of tile t
//   substep 3  MFMAs of tile t cover the first fragment reads of tile t+1
// sched_group_barrier pins the MFMA / DS interleaving; the last K step is peeled so that the loop
// body has no branches (the scheduler cannot interleave across basic blocks).
template <int BM, int BN, int BK, int WM, int WN, class SA, class SB, class Epi>
__device__ __forceinline__ void gemm_tile(SA& sa, SB& sb, int kt0, int kt1, unsigned short* smem, Epi epi) {
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int A_ELEMS = BM * BK, B_ELEMS = BN * BK;
  constexpr int KS = BK / 16;
  static_assert(KS == 4, "written for BK = 64");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WN, wn = wave % WN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frow_a = wm * (TM * 32) + (lane & 31);
  const int frow_b = wn * (TN * 32) + (lane & 31);
  const int fchunk = lane >> 5;

  bf16x8 fa[2][TM], fb[2][TN];
  auto read_frags = [&](const unsigned short* As, const unsigned short* Bs, int kk, bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i) a[i] = *(const bf16x8*)(As + lds_off<BK>(frow_a + i * 32, kk * 2 + fchunk));
#pragma unroll
    for (int j = 0; j < TN; ++j) b[j] = *(const bf16x8*)(Bs + lds_off<BK>(frow_b + j * 32, kk * 2 + fchunk));
  };
  auto mfmas = [&](bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };

  if (kt0 < kt1) {
    sa.gload(kt0 * BK);
    sb.gload(kt0 * BK);
    sa.sstore(smem);
    sb.sstore(smem + A_ELEMS);
  }
  __syncthreads();
  if (kt0 < kt1) read_frags(smem, smem + A_ELEMS, 0, fa[0], fb[0]);

  // scheduling pattern of one substep: one LDS fragment read after each of the first MFMAs
  constexpr int NREAD = TM + TN, NMFMA = TM * TN, NPAIR = NREAD < NMFMA ? NREAD : NMFMA;
  auto interleave_reads = [&]() {
#pragma unroll
    for (int q = 0; q < NPAIR; ++q) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
    if constexpr (NREAD > NPAIR) __builtin_amdgcn_sched_group_barrier(0x100, NREAD - NPAIR, 0);
  };
  auto step = [&](int kt, auto more_tag) {
    constexpr bool more = decltype(more_tag)::value;
    const int cur = (kt - kt0) & 1;
    const unsigned short* As = smem + cur * (A_ELEMS + B_ELEMS);
    const unsigned short* Bs = As + A_ELEMS;
    unsigned short* nxt = smem + (cur ^ 1) * (A_ELEMS + B_ELEMS);
    if constexpr (more) {
      sa.gload((kt + 1) * BK);
      sb.gload((kt + 1) * BK);
    }
    read_frags(As, Bs, 1, fa[1], fb[1]);
    mfmas(fa[0], fb[0]);
    interleave_reads();
    if constexpr (NMFMA > NPAIR) __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NPAIR, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(As, Bs, 2, fa[0], fb[0]);
    mfmas(fa[1], fb[1]);
    interleave_reads();
    if constexpr (NMFMA > NPAIR) __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NPAIR, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(As, Bs, 3, fa[1], fb[1]);
    mfmas(fa[0], fb[0]);
    if constexpr (more) {
      sa.sstore(nxt);
      sb.sstore(nxt + A_ELEMS);
    }
    interleave_reads();
    if constexpr (more) {
#pragma unroll
      for (int q = 0; q < TM * TN - (TM + TN); ++q) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x200, 2, 0); }
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    if constexpr (more) read_frags(nxt, nxt + A_ELEMS, 0, fa[0], fb[0]);
    mfmas(fa[1], fb[1]);
    __builtin_amdgcn_sched_barrier(0);
  };
  for (int kt = kt0; kt + 1 < kt1; ++kt) step(kt, std::true_type{});
  if (kt0 < kt1) step(kt1 - 1, std::false_type{});
  __syncthreads();

  epilogue_through_lds<TM, TN>(reinterpret_cast<float*>(smem), acc, wave, lane, wm * (TM * 32), wn * (TN * 32), epi);
}

template <int ACT>
__device__ __forceinline__ float apply_act_static(float z) {
  if constexpr (ACT == 1) return z > 0.f ? z : 0.f;
  else if constexpr (ACT == 2) return gelu_erfc_poly(z);
  else if constexpr (ACT == 3) return tanhf(z);
  else if constexpr (ACT == 4) return 1.f / (1.f + expf(-z));
  else return z;
}

// Writes four consecutive elements of a row of C in up to three forms (see lp::GemmDesc).
// vec: N, ldc and the output pointers allow 8-/16-byte stores.
// The activation is a run-time field; an epilogue that handles many elements per lane asks for a view with the
// activation as a compile-time constant once (with_static_act) instead of deciding it per element.
// HAD (the dX form only, to keep the other kernels small): the product is dA of the preceding layer and had_s that
// layer's stash S; what goes to out_z is then dY = q(q(dA) * f'(S)) (Eq. 3 moved into the product that feeds it,
// Sec. III-B), the arithmetic of the stand-alone Hadamard kernel element for element: dA is rounded to bf16 first,
// exactly as if it had been stored and read back.
template <bool HAD>
struct StoreEpilogueT {
  unsigned short* out_z;
  unsigned short* out_a;
  float* out_f32;
  int M, N, ldc, act, m0, n0;
  bool vec;
  // optional: f(z) for every bfloat16 bit pattern z (65536 entries); when set, A is looked up instead of computed
  const unsigned short* act_lut;
  // HAD: stash of the preceding layer (indexed like out_z; 8-byte aligned rows when vec), and f'(z) for every bfloat16
  // bit pattern z as fp32 (null: f' = [S > 0], the ReLU form)
  const unsigned short* had_s;
  const float* had_lut;
  // HAD with pool_wp > 0: the layer below is a 2 x 2 max-pooled ReLU layer, whose gradient is routed, not only masked.
  // Row r of this product is then the pooled pixel (b, y, x) with x = r % pool_wp, had_s is that layer's full-resolution
  // Z and out_z its full-resolution dY, both [.., 2 Hp, 2 pool_wp, ldc].
  int pool_wp;

  // ACT < 0: the activation is read from `act`; 5: table look-up
  template <int ACT>
  __device__ __forceinline__ void store(int r, int c, const f32x4& v) const {
    const int row = m0 + r, col = n0 + c;
    if (row >= M || col >= N) return;
    const size_t o = (size_t)row * ldc + col;
    unsigned short zb[4], ab[4];
    if (out_z || out_a) {
#pragma unroll
      for (int t = 0; t < 4; ++t) zb[t] = bf16_bits(v[t]);
      if (out_a) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          if constexpr (ACT < 0) ab[t] = bf16_bits(apply_act(bf16_to_f32(zb[t]), act));
          else if constexpr (ACT == 0) ab[t] = zb[t];
          else if constexpr (ACT == 5) ab[t] = act_lut[zb[t]];
          else ab[t] = bf16_bits(apply_act_static<ACT>(bf16_to_f32(zb[t])));
        }
      }
    }
    if (vec) {  // col + 3 < N follows from N % 4 == 0
      if (out_f32) *reinterpret_cast<f32x4*>(out_f32 + o) = v;
      if (out_z) *reinterpret_cast<u32x2*>(out_z + o) = u32x2{(unsigned)zb[0] | ((unsigned)zb[1] << 16), (unsigned)zb[2] | ((unsigned)zb[3] << 16)};
      if (out_a) *reinterpret_cast<u32x2*>(out_a + o) = u32x2{(unsigned)ab[0] | ((unsigned)ab[1] << 16), (unsigned)ab[2] | ((unsigned)ab[3] << 16)};
    } else {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        if (col + t < N) {
          if (out_f32) out_f32[o + t] = v[t];
          if (out_z) out_z[o + t] = zb[t];
          if (out_a) out_a[o + t] = ab[t];
        }
      }
    }
  }
  __device__ __forceinline__ void operator()(int r, int c, const f32x4& v) const { store<-1>(r, c, v); }

  // the four stash values that belong to store_had(r, c, ...); zeros where they are not read ahead
  __device__ __forceinline__ u32x2 had_side(int r, int c) const {
    const int row = m0 + r, col = n0 + c;
    if (!vec || row >= M || col >= N) return u32x2{0u, 0u};
    return *reinterpret_cast<const u32x2*>(had_s + (size_t)row * ldc + col);
  }
  template <bool LUT>
  __device__ __forceinline__ unsigned short had_one(float v, unsigned short s) const {
    const float da = bf16_to_f32(bf16_bits(v));
    const float df = LUT ? had_lut[s] : (bf16_to_f32(s) > 0.f ? 1.f : 0.f);
    return bf16_bits(da * df);
  }
  template <bool LUT>
  __device__ __forceinline__ void store_had(int r, int c, const f32x4& v, const u32x2& sd) const {
    const int row = m0 + r, col = n0 + c;
    if (row >= M || col >= N) return;
    const size_t o = (size_t)row * ldc + col;
    if (vec) {
      const unsigned short y0 = had_one<LUT>(v[0], (unsigned short)(sd[0] & 0xffffu)), y1 = had_one<LUT>(v[1], (unsigned short)(sd[0] >> 16));
      const unsigned short y2 = had_one<LUT>(v[2], (unsigned short)(sd[1] & 0xffffu)), y3 = had_one<LUT>(v[3], (unsigned short)(sd[1] >> 16));
      *reinterpret_cast<u32x2*>(out_z + o) = u32x2{(unsigned)y0 | ((unsigned)y1 << 16), (unsigned)y2 | ((unsigned)y3 << 16)};
    } else {
#pragma unroll
      for (int t = 0; t < 4; ++t)
        if (col + t < N) out_z[o + t] = had_one<LUT>(v[t], had_s[o + t]);
    }
  }

  // The four pixels of the window of pooled pixel (r, c..c+3) receive q(q(dA) * [z > 0]) at the first maximum of relu(z)
  // (row-major order inside the window, strict '>' keeps the first) and 0 elsewhere: the arithmetic of the stand-alone
  // routing kernel, element for element.  Every full-resolution pixel belongs to exactly one window, so dY is written whole.
  __device__ __forceinline__ void store_pool_route(int r, int c, const f32x4& v) const {
    const int row = m0 + r, col = n0 + c;
    if (row >= M || col >= N) return;
    const int ry = row / pool_wp, x = row - ry * pool_wp;   // ry = b * Hp + y
    const size_t base = ((size_t)4 * ry * pool_wp + 2 * x) * ldc + col;
    const size_t down = (size_t)2 * pool_wp * ldc;
    const size_t offs[4] = {base, base + ldc, base + down, base + down + ldc};
    unsigned short zb[4][4], ob[4][4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (vec) {
        const u32x2 zz = *reinterpret_cast<const u32x2*>(had_s + offs[k]);
        zb[k][0] = (unsigned short)(zz[0] & 0xffffu); zb[k][1] = (unsigned short)(zz[0] >> 16);
        zb[k][2] = (unsigned short)(zz[1] & 0xffffu); zb[k][3] = (unsigned short)(zz[1] >> 16);
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) zb[k][t] = col + t < N ? had_s[offs[k] + t] : (unsigned short)0;
      }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float best = 0.f;
      int arg = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float z = bf16_to_f32(zb[k][t]);
        const float a = z > 0.f ? z : 0.f;
        if (k == 0 || a > best) { best = a; arg = k; }
      }
      const float da = bf16_to_f32(bf16_bits(v[t]));
#pragma unroll
      for (int k = 0; k < 4; ++k) ob[k][t] = bf16_bits(k == arg ? da * (bf16_to_f32(zb[k][t]) > 0.f ? 1.f : 0.f) : 0.f);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (vec) {
        *reinterpret_cast<u32x2*>(out_z + offs[k]) = u32x2{(unsigned)ob[k][0] | ((unsigned)ob[k][1] << 16), (unsigned)ob[k][2] | ((unsigned)ob[k][3] << 16)};
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t)
          if (col + t < N) out_z[offs[k] + t] = ob[k][t];
      }
    }
  }

  template <int ACT>
  struct StaticAct {
    const StoreEpilogueT& e;
    static constexpr bool kHasSide = false;
    using Side = NoSide;
    __device__ __forceinline__ NoSide side(int, int) const { return NoSide{}; }
    __device__ __forceinline__ void operator()(int r, int c, const f32x4& v) const { e.template store<ACT>(r, c, v); }
    __device__ __forceinline__ void operator()(int r, int c, const f32x4& v, NoSide) const { e.template store<ACT>(r, c, v); }
  };
  template <bool LUT>
  struct Hadamard {
    const StoreEpilogueT& e;
    static constexpr bool kHasSide = true;
    using Side = u32x2;
    __device__ __forceinline__ u32x2 side(int r, int c) const { return e.had_side(r, c); }
    __device__ __forceinline__ void operator()(int r, int c, const f32x4& v, const u32x2& sd) const { e.template store_had<LUT>(r, c, v, sd); }
    __device__ __forceinline__ void operator()(int r, int c, const f32x4& v) const { e.template store_had<LUT>(r, c, v, e.had_side(r, c)); }
  };
  struct PoolRoute {
    const StoreEpilogueT& e;
    static constexpr bool kHasSide = false;
    using Side = NoSide;
    __device__ __forceinline__ NoSide side(int, int) const { return NoSide{}; }
    __device__ __forceinline__ void operator()(int r, int c, const f32x4& v) const { e.store_pool_route(r, c, v); }
    __device__ __forceinline__ void operator()(int r, int c, const f32x4& v, NoSide) const { e.store_pool_route(r, c, v); }
  };
  // calls f with a view of this epilogue whose activation is a compile-time constant (same arithmetic, element for element)
  template <class F>
  __device__ __forceinline__ void with_static_act(F&& f) const {
    if constexpr (HAD) {
      if (had_s) {
        if (pool_wp > 0) f(PoolRoute{*this});
        else if (had_lut) f(Hadamard<true>{*this});
        else f(Hadamard<false>{*this});
        return;
      }
    }
    switch (out_a ? act : 0) {
      case 1: f(StaticAct<1>{*this}); break;
      case 2:
        if (act_lut) f(StaticAct<5>{*this});
        else f(StaticAct<2>{*this});
        break;
      case 3: f(StaticAct<3>{*this}); break;
      case 4: f(StaticAct<4>{*this}); break;
      default: f(StaticAct<0>{*this}); break;
    }
  }
};
using StoreEpilogue = StoreEpilogueT<false>;

// Epilogue of a weight-gradient product that is consumed on the spot (Eq. 6 fused into Eq. 5): the
// tile of G never goes to memory; W <- W - lr * G on the fp32 master, and the bf16 working copy of the
// new weights is written next to it.  Same arithmetic as the stand-alone update kernel: one fma per
// weight, then round-to-nearest-even.
struct SgdEpilogue {
  float* master;
  unsigned short* work_out;
  float neg_lr;
  int M, N, ldc, m0, n0;
  bool vec;
  __device__ __forceinline__ void operator()(int r, int c, const f32x4& g) const {
    const int row = m0 + r, col = n0 + c;
    if (row >= M || col >= N) return;
    const size_t o = (size_t)row * ldc + col;
    if (vec) {  // col + 3 < N follows from N % 4 == 0
      f32x4 w = *reinterpret_cast<const f32x4*>(master + o);
#pragma unroll
      for (int t = 0; t < 4; ++t) w[t] = fmaf(neg_lr, g[t], w[t]);
      *reinterpret_cast<f32x4*>(master + o) = w;
      *reinterpret_cast<u32x2*>(work_out + o) = u32x2{(unsigned)bf16_bits(w[0]) | ((unsigned)bf16_bits(w[1]) << 16),
                                                      (unsigned)bf16_bits(w[2]) | ((unsigned)bf16_bits(w[3]) << 16)};
    } else {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        if (col + t < N) {
          const float w = fmaf(neg_lr, g[t], master[o + t]);
          master[o + t] = w;
          work_out[o + t] = bf16_bits(w);
        }
      }
    }
  }
  // The master weights of a band are fetched while the band before it is on its trip through LDS (16-byte form only:
  // the element-wise form loads them where it uses them).  Same arithmetic either way.
  static constexpr bool kHasSide = true;
  using Side = f32x4;
  __device__ __forceinline__ f32x4 side(int r, int c) const {
    const int row = m0 + r, col = n0 + c;
    f32x4 w = {0.f, 0.f, 0.f, 0.f};
    if (vec && row < M && col < N) w = *reinterpret_cast<const f32x4*>(master + (size_t)row * ldc + col);
    return w;
  }
  __device__ __forceinline__ void operator()(int r, int c, const f32x4& g, const f32x4& w0) const {
    if (!vec) { (*this)(r, c, g); return; }
    const int row = m0 + r, col = n0 + c;
    if (row >= M || col >= N) return;
    const size_t o = (size_t)row * ldc + col;
    f32x4 w;
#pragma unroll
    for (int t = 0; t < 4; ++t) w[t] = fmaf(neg_lr, g[t], w0[t]);
    *reinterpret_cast<f32x4*>(master + o) = w;
    *reinterpret_cast<u32x2*>(work_out + o) = u32x2{(unsigned)bf16_bits(w[0]) | ((unsigned)bf16_bits(w[1]) << 16),
                                                    (unsigned)bf16_bits(w[2]) | ((unsigned)bf16_bits(w[3]) << 16)};
  }
  template <class F>
  __device__ __forceinline__ void with_static_act(F&& f) const { f(*this); }
};

}  // namespace core
}  // namespace lp
