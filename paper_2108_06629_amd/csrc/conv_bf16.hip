// 3x3, stride 1, zero pad 1 convolution tasks as implicit GEMMs on the bf16 matrix cores (NHWC
// activations, weights [3][3][C_in][C_out], cross-correlation, no bias):
//
//   F   z[(b,y,x), o]   = sum_{(tap,c)} x[b, y+kh-1, x+kw-1, c] * w[(tap,c), o]          Eq. 1
//   dX  dx[(b,y,x), c]  = sum_{(tap,o)} dy[b, y-kh+1, x-kw+1, o] * w[tap, c, o]          Eq. 4
//   dW  g[(tap,c), o]   = sum_{(b,y,x)} x[b, y+kh-1, x+kw-1, c] * dy[(b,y,x), o]         Eq. 5
//
// with tap = 3*kh + kw.  No im2col buffer exists: the operand that is a shifted view of an image is
// gathered chunk by chunk while its tile is staged into LDS (zero padding = an out-of-range buffer
// offset), and everything after that is the main loop of gemm_core.h.  dW reduces over B*H*W pixels
// into a small [9*C_in, C_out] result, so it is split over K across workgroups; the fp32 partials are
// summed by a second kernel in a fixed order.
#include "conv_thin.h"
#include "gemm_core.h"
#include "gemm_dl.h"
#include "lp_kernels.h"

namespace lp {
namespace {

using namespace core;

constexpr int BM = 128, BN = 64, BK = 64, WM = 2, WN = 2, NT = WM * WN * 64;

// Division by a divisor fixed per launch: q = (n * m) >> 32 with m = floor(2^32 / d) + 1, exact while
// n * d < 2^32 (the host checks the largest n it will see); otherwise, and for d = 1, plain division.
struct FastDiv {
  unsigned d, m;
  __host__ static FastDiv make(unsigned d, unsigned long long max_n) {
    FastDiv f;
    f.d = d;
    f.m = (d > 1 && max_n * d < (1ull << 32)) ? (unsigned)((1ull << 32) / d) + 1u : 0u;
    return f;
  }
  __device__ __forceinline__ unsigned div(unsigned n) const { return m ? __umulhi(n, m) : n / d; }
};

struct ConvKArgs {
  const unsigned short* img;   // F: x, dX: dy, dW: x
  const unsigned short* mat;   // F: w, dX: w, dW: dy
  unsigned short* out_z;
  unsigned short* out_a;
  float* out_f32;
  int B, H, W, Cimg;           // channels of the gathered image
  int M, N, K;                 // GEMM view
  int Cin, Cout;
  int c0;                      // dX: first input channel of the range
  int ldc, act;
  unsigned img_bytes, mat_bytes;
  int kt_per_split;            // dW: K tiles per workgroup in y
  int vec_out;
  const unsigned short* had_s; // dX: stash of the layer below, laid out like out_z; its Hadamard product (Eq. 3) is then applied on the way out
  const float* had_lut;        // ... with f' looked up here (null: the ReLU form)
  int pool_wp;                 // ... and, when > 0, routed to the 2 x 2 windows of a pooled layer (this product's image width)
  unsigned short* pool_a;      // F (halo form): when set, also A[b, y/2, x/2, :] = max over the 2 x 2 window of relu(z), computed from the stored Z
  FastDiv divW, divH, divC;    // by W, by H, by the gathered image's channel count
};

__device__ __forceinline__ void tap_offsets(int tap, bool flip, int& dy, int& dx) {
  const int kh = tap / 3, kw = tap - kh * 3;
  dy = flip ? 1 - kh : kh - 1;
  dx = flip ? 1 - kw : kw - 1;
}

// A operand of F and dX: rows are pixels (b,y,x), k = (tap, c) with c contiguous in memory.
template <bool ALIGNED>
struct StagePixelsKC {
  static constexpr int NCH = BM * BK / 8;
  static constexpr int CH = NCH / NT;
  static_assert(NCH % NT == 0, "");
  __amdgpu_buffer_rsrc_t rs;
  int Ktot, C, H, W, tid;
  bool flip;
  FastDiv divC;
  int pix[CH], yx[CH];   // pixel index and (y << 16 | x) of this thread's rows; pix < 0: row past M
  u32x4 v[CH];
  __device__ __forceinline__ void init(const ConvKArgs& p, int m0, bool flip_) {
    rs = make_rsrc(p.img, p.img_bytes);
    Ktot = p.K; C = p.Cimg; H = p.H; W = p.W; tid = threadIdx.x; flip = flip_; divC = p.divC;
#pragma unroll
    for (int it = 0; it < CH; ++it) {
      const int row = (it * NT + tid) / (BK / 8);
      const int m = m0 + row;
      if (m < p.M) {
        const int t = (int)p.divW.div((unsigned)m), x = m - t * W;
        const int y = t - (int)p.divH.div((unsigned)t) * H;
        pix[it] = m; yx[it] = (y << 16) | x;
      } else {
        pix[it] = -1; yx[it] = 0;
      }
    }
  }
  __device__ __forceinline__ unsigned elem_off(int it, int k, bool& ok) const {
    const int tap = (int)divC.div((unsigned)k), c = k - tap * C;
    int dy, dx;
    tap_offsets(tap, flip, dy, dx);
    const int yy = (yx[it] >> 16) + dy, xx = (yx[it] & 0xffff) + dx;
    ok = pix[it] >= 0 && k < Ktot && yy >= 0 && yy < H && xx >= 0 && xx < W;
    return (unsigned)((pix[it] + dy * W + dx) * C + c);
  }
  __device__ __forceinline__ void gload(int k0) {
#pragma unroll
    for (int it = 0; it < CH; ++it) {
      const int kc = (it * NT + tid) % (BK / 8);
      const int k = k0 + kc * 8;
      if constexpr (ALIGNED) {   // C % 8 == 0: the 8 elements share one tap
        bool ok;
        const unsigned e = elem_off(it, k, ok);
        v[it] = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? e * 2u : kOOB, 0, 0);
      } else {
        unsigned h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          bool ok;
          const unsigned e = elem_off(it, k + j, ok);
          h[j] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, ok ? e * 2u : kOOB, 0, 0);
        }
        v[it] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
      }
    }
  }
  __device__ __forceinline__ void sstore(unsigned short* lds) {
#pragma unroll
    for (int it = 0; it < CH; ++it) {
      const int id = it * NT + tid;
      *(u32x4*)(lds + lds_off<BK>(id / (BK / 8), id % (BK / 8))) = v[it];
    }
  }
};

// B operand of dX: rows are input channels c, k = (tap, o) with o contiguous: w[(tap*Cin + c)*Cout + o]
struct StageWeightsDX {
  static constexpr int NCH = BN * BK / 8;
  static constexpr int CH = NCH / NT;
  static_assert(NCH % NT == 0, "");
  __amdgpu_buffer_rsrc_t rs;
  int n0, Ntot, Ktot, Cin, Cout, c0, tid;
  u32x4 v[CH];
  __device__ __forceinline__ void init(const ConvKArgs& p, int n0_) {
    rs = make_rsrc(p.mat, p.mat_bytes);
    n0 = n0_; Ntot = p.N; Ktot = p.K; Cin = p.Cin; Cout = p.Cout; c0 = p.c0; tid = threadIdx.x;
  }
  __device__ __forceinline__ void gload(int k0) {
#pragma unroll
    for (int it = 0; it < CH; ++it) {
      const int id = it * NT + tid;
      const int n = n0 + id / (BK / 8), k = k0 + (id % (BK / 8)) * 8;
      const int tap = k / Cout, o = k - tap * Cout;   // Cout % 8 == 0: one tap per chunk
      const bool ok = n < Ntot && k < Ktot;
      const unsigned e = (unsigned)((tap * Cin + c0 + n) * Cout + o);
      v[it] = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? e * 2u : kOOB, 0, 0);
    }
  }
  __device__ __forceinline__ void sstore(unsigned short* lds) {
#pragma unroll
    for (int it = 0; it < CH; ++it) {
      const int id = it * NT + tid;
      *(u32x4*)(lds + lds_off<BK>(id / (BK / 8), id % (BK / 8))) = v[it];
    }
  }
};

// A operand of dW: rows are (tap, c), k runs over pixels (b,y,x): x[b, y+kh-1, x+kw-1, c].
// Threads move 8 (pixels) x 8 (channels) blocks and transpose them in registers.
template <bool ALIGNED>
struct StagePixelsKS {
  static constexpr int NB = (BK / 8) * (BM / 8);
  static constexpr int IT = (NB + NT - 1) / NT;
  __amdgpu_buffer_rsrc_t rs;
  int m0, Mtot, Ktot, C, H, W, tid;
  FastDiv divW, divH;
  // per row of this thread's 8-row group (ALIGNED: one entry, the rows share a tap): tap offsets and channel,
  // packed as (dy + 1) | (dx + 1) << 2 | c << 4; -1: row past M
  static constexpr int NQ = ALIGNED ? 1 : 8;
  int rowinfo[IT][NQ];
  u32x4 v[IT][8];
  __device__ __forceinline__ void init(const ConvKArgs& p, int m0_) {
    rs = make_rsrc(p.img, p.img_bytes);
    m0 = m0_; Mtot = p.M; Ktot = p.K; C = p.Cimg; H = p.H; W = p.W; tid = threadIdx.x;
    divW = p.divW; divH = p.divH;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int rc = (it * NT + tid) % (BM / 8);
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const int mm = m0 + rc * 8 + q;
        const int tap = (int)p.divC.div((unsigned)mm), c = mm - tap * C;
        int dy, dx;
        tap_offsets(tap, false, dy, dx);
        rowinfo[it][q] = mm < Mtot ? ((dy + 1) | ((dx + 1) << 2) | (c << 4)) : -1;
      }
    }
  }
  __device__ __forceinline__ void gload(int k0) {
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int id = it * NT + tid;
      if (NB % NT == 0 || id < NB) {
        const int kg = id / (BM / 8);
        const int p0 = k0 + kg * 8;
        // (x, y) of the first of this thread's 8 consecutive pixels; the others by stepping
        const int t = (int)divW.div((unsigned)p0);
        int x = p0 - t * W, y = t - (int)divH.div((unsigned)t) * H;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int pxl = p0 + j;
          if constexpr (ALIGNED) {   // C % 8 == 0: the 8 rows share one tap
            const int ri = rowinfo[it][0];
            const int dy = (ri & 3) - 1, dx = ((ri >> 2) & 3) - 1, c = ri >> 4;
            const int yy = y + dy, xx = x + dx;
            const bool ok = ri >= 0 && pxl < Ktot && yy >= 0 && yy < H && xx >= 0 && xx < W;
            const unsigned e = (unsigned)((pxl + dy * W + dx) * C + c);
            v[it][j] = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? e * 2u : kOOB, 0, 0);
          } else {
            unsigned h[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              const int ri = rowinfo[it][q];
              const int dy = (ri & 3) - 1, dx = ((ri >> 2) & 3) - 1, c = ri >> 4;
              const int yy = y + dy, xx = x + dx;
              const bool ok = ri >= 0 && pxl < Ktot && yy >= 0 && yy < H && xx >= 0 && xx < W;
              const unsigned e = (unsigned)((pxl + dy * W + dx) * C + c);
              h[q] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, ok ? e * 2u : kOOB, 0, 0);
            }
            v[it][j] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
          }
          if (++x == W) { x = 0; if (++y == H) y = 0; }
        }
      }
    }
  }
  __device__ __forceinline__ void sstore(unsigned short* lds) {
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int id = it * NT + tid;
      if (NB % NT == 0 || id < NB) {
        const int rc = id % (BM / 8), kg = id / (BM / 8);
        u32x4 y[8];
        transpose8x8(v[it], y);
#pragma unroll
        for (int e = 0; e < 8; ++e) *(u32x4*)(lds + lds_off<BK>(rc * 8 + e, kg)) = y[e];
      }
    }
  }
};


// ---- direct-to-LDS forms (channel counts that are multiples of 8) ----------------------------------
// Same products on the main loop of gemm_dl.h: 128 x 64 tiles, K step 32, four LDS stages (48 KB, three
// workgroups per CU), so about three K steps of gather latency are covered -- these layers have short
// reductions (9 C_in) and little arithmetic per step, and what bounds them is how many loads are in
// flight.  A buffer_load ... lds takes its global address per lane, so the gather costs nothing extra:
// the lane that fills LDS chunk p of a row computes the address of the shifted pixel (or an out-of-range
// offset for the zero padding).
namespace cdl {

constexpr int DBM = 128, DBN = 64, DBK = 32, DSTAGES = 4, DWM = 2, DWN = 2, DNW = DWM * DWN, DNT = DNW * 64;

// A operand of F and dX: rows are pixels, k = (tap, c), c contiguous in memory.  LDS layout and fragment
// reads are those of dl::OperandKC.
struct PixelsKC : dl::OperandKC<DBM, DBK, DNW> {
  static constexpr bool SPLIT_ISSUE = false;   // gathers: addresses are not affine in the tile index
  using Base = dl::OperandKC<DBM, DBK, DNW>;
  int C, H, W;
  bool flip;
  FastDiv divC;
  bool tap_uniform;   // C is a multiple of the K step: a whole K step lies inside one tap
  int pix[Base::PER_WAVE], yx[Base::PER_WAVE], kofs[Base::PER_WAVE];
  __device__ __forceinline__ void init(const ConvKArgs& p, int m0, bool flip_, int wave_u) {
    Base::init(p.img, p.img_bytes, m0, p.M, p.K, 0);
    C = p.Cimg; H = p.H; W = p.W; flip = flip_; divC = p.divC;
    tap_uniform = C % DBK == 0;
#pragma unroll
    for (int i = 0; i < Base::PER_WAVE; ++i) {
      const int g = wave_u * Base::PER_WAVE + i;
      const int trow = g * Base::ROWS_PER_LOAD + this->lrow;
      kofs[i] = (this->lpos ^ ((trow / Base::RP) % Base::CPR)) * 8;
      const int m = m0 + trow;
      if (m < p.M) {
        const int t = (int)p.divW.div((unsigned)m), x = m - t * W;
        const int y = t - (int)p.divH.div((unsigned)t) * H;
        pix[i] = m; yx[i] = (y << 16) | x;
      } else {
        pix[i] = -1; yx[i] = 0;
      }
    }
  }
  __device__ __forceinline__ void issue(int k0, unsigned short* stage, int wave_u) const {
    if (tap_uniform) {
      // k0 is the same for the whole workgroup: tap, its offsets and the shift in memory on the scalar unit
      const int tap = (int)divC.div((unsigned)k0);
      int dy, dx;
      tap_offsets(tap, flip, dy, dx);
      const int shift = (dy * W + dx) * C + (k0 - tap * C);
      const bool k_ok = k0 < this->Ktot;   // Ktot = 9 C is a multiple of the K step too
#pragma unroll
      for (int i = 0; i < Base::PER_WAVE; ++i) {
        const int g = wave_u * Base::PER_WAVE + i;
        const int yy = (yx[i] >> 16) + dy, xx = (yx[i] & 0xffff) + dx;
        const bool ok = k_ok && pix[i] >= 0 && yy >= 0 && yy < H && xx >= 0 && xx < W;
        const unsigned off = ok ? (unsigned)(pix[i] * C + shift + kofs[i]) * 2u : kOOB;
        dl::load_to_lds_16(this->rs, off, stage + g * 512);
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < Base::PER_WAVE; ++i) {
      const int g = wave_u * Base::PER_WAVE + i;
      const int k = k0 + kofs[i];
      const int tap = (int)divC.div((unsigned)k), c = k - tap * C;
      int dy, dx;
      tap_offsets(tap, flip, dy, dx);
      const int yy = (yx[i] >> 16) + dy, xx = (yx[i] & 0xffff) + dx;
      const bool ok = pix[i] >= 0 && k < this->Ktot && yy >= 0 && yy < H && xx >= 0 && xx < W;
      const unsigned off = ok ? (unsigned)((pix[i] + dy * W + dx) * C + c) * 2u : kOOB;
      dl::load_to_lds_16(this->rs, off, stage + g * 512);
    }
  }
};

// B operand of dX: rows are input channels n (of the range that starts at c0), k = (tap, o), o contiguous:
// w[(tap * Cin + c0 + n) * Cout + o]
struct WeightsDX : dl::OperandKC<DBN, DBK, DNW> {
  static constexpr bool SPLIT_ISSUE = false;   // gathers: addresses are not affine in the tile index
  using Base = dl::OperandKC<DBN, DBK, DNW>;
  int Cin, Cout, c0;
  FastDiv divC;   // by Cout
  __device__ __forceinline__ void init(const ConvKArgs& p, int n0) {
    Base::init(p.mat, p.mat_bytes, n0, p.N, p.K, 0);
    Cin = p.Cin; Cout = p.Cout; c0 = p.c0; divC = p.divC;
  }
  __device__ __forceinline__ void issue(int k0, unsigned short* stage, int wave_u) const {
    const bool tap_uniform = Cout % DBK == 0;
    const int tap_u = (int)divC.div((unsigned)k0);   // scalar
#pragma unroll
    for (int i = 0; i < Base::PER_WAVE; ++i) {
      const int g = wave_u * Base::PER_WAVE + i;
      const int trow = g * Base::ROWS_PER_LOAD + this->lrow;
      const int chunk = this->lpos ^ ((trow / Base::RP) % Base::CPR);
      const int n = this->r0 + trow, k = k0 + chunk * 8;
      const int tap = tap_uniform ? tap_u : (int)divC.div((unsigned)k), o = k - tap * Cout;
      const unsigned off = (n < this->Rtot && k < this->Ktot) ? (unsigned)((tap * Cin + c0 + n) * Cout + o) * 2u : kOOB;
      dl::load_to_lds_16(this->rs, off, stage + g * 512);
    }
  }
};

// A operand of dW: rows are (tap, c), k runs over pixels; memory order [pixel][c] is kept in LDS and
// transposed by the LDS read, as in dl::OperandKS.
struct PixelsKS : dl::OperandKS<DBM, DBK, DNW> {
  static constexpr bool SPLIT_ISSUE = false;   // gathers: addresses are not affine in the tile index
  using Base = dl::OperandKS<DBM, DBK, DNW>;
  int C, H, W;
  FastDiv divW, divH;
  int rowinfo[Base::PER_WAVE];   // (dy + 1) | (dx + 1) << 2 | c << 4 of the 8 rows this lane fetches; -1: past M
  __device__ __forceinline__ void init(const ConvKArgs& p, int m0, int wave_u) {
    Base::init(p.img, p.img_bytes, m0, p.M, p.K, 0);
    C = p.Cimg; H = p.H; W = p.W; divW = p.divW; divH = p.divH;
#pragma unroll
    for (int i = 0; i < Base::PER_WAVE; ++i) {
      const int g = wave_u * Base::PER_WAVE + i;
      const int kr = g * Base::ROWS_PER_LOAD + this->lk;
      const int m = m0 + (this->lpos ^ Base::swz(kr)) * 8;
      const int tap = (int)p.divC.div((unsigned)m), c = m - tap * C;
      int dy, dx;
      tap_offsets(tap, false, dy, dx);
      rowinfo[i] = m < p.M ? ((dy + 1) | ((dx + 1) << 2) | (c << 4)) : -1;
    }
  }
  __device__ __forceinline__ void issue(int k0, unsigned short* stage, int wave_u) const {
#pragma unroll
    for (int i = 0; i < Base::PER_WAVE; ++i) {
      const int g = wave_u * Base::PER_WAVE + i;
      const int pxl = k0 + g * Base::ROWS_PER_LOAD + this->lk;
      const int t = (int)divW.div((unsigned)pxl), x = pxl - t * W;
      const int y = t - (int)divH.div((unsigned)t) * H;
      const int ri = rowinfo[i];
      const int dy = (ri & 3) - 1, dx = ((ri >> 2) & 3) - 1, c = ri >> 4;
      const int yy = y + dy, xx = x + dx;
      const bool ok = ri >= 0 && pxl < this->Ktot && yy >= 0 && yy < H && xx >= 0 && xx < W;
      const unsigned off = ok ? (unsigned)((pxl + dy * W + dx) * C + c) * 2u : kOOB;
      dl::load_to_lds_16(this->rs, off, stage + g * 512);
    }
  }
};

using MatKS = dl::OperandKS<DBN, DBK, DNW>;   // W of F ([9 C_in][C_out]) and dY of dW ([pixels][C_out])

__global__ void __launch_bounds__(DNT) conv_fwd_dl_kernel(ConvKArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int tm, tn;
  tile_of_block<false>(blockIdx.x, (p.M + DBM - 1) / DBM, (p.N + DBN - 1) / DBN, tm, tn);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  PixelsKC oa;
  oa.init(p, tm * DBM, false, wave);
  MatKS ob;
  ob.init(p.mat, p.mat_bytes, tn * DBN, p.N, p.K, p.Cout);
  StoreEpilogue epi{p.out_z, p.out_a, nullptr, p.M, p.N, p.ldc, p.act, tm * DBM, tn * DBN, p.vec_out != 0};
  dl::gemm_tile_dl<DBM, DBN, DBK, DSTAGES, DWM, DWN>(oa, ob, 0, (p.K + DBK - 1) / DBK, smem, epi);
}

__global__ void __launch_bounds__(DNT) conv_dx_dl_kernel(ConvKArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int tm, tn;
  tile_of_block<false>(blockIdx.x, (p.M + DBM - 1) / DBM, (p.N + DBN - 1) / DBN, tm, tn);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  PixelsKC oa;
  oa.init(p, tm * DBM, true, wave);
  WeightsDX ob;
  ob.init(p, tn * DBN);
  StoreEpilogueT<true> epi{p.out_z, nullptr, nullptr, p.M, p.N, p.ldc, 0, tm * DBM, tn * DBN, p.vec_out != 0, nullptr, p.had_s, p.had_lut, p.pool_wp};
  dl::gemm_tile_dl<DBM, DBN, DBK, DSTAGES, DWM, DWN>(oa, ob, 0, (p.K + DBK - 1) / DBK, smem, epi);
}

__global__ void __launch_bounds__(DNT) conv_dw_dl_kernel(ConvKArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  const int nbn = (p.N + DBN - 1) / DBN;
  const int tm = blockIdx.x / nbn, tn = blockIdx.x % nbn;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int KT = (p.K + DBK - 1) / DBK;
  const int kt0 = blockIdx.y * p.kt_per_split;
  const int kt1 = kt0 + p.kt_per_split < KT ? kt0 + p.kt_per_split : KT;
  const int k_end = kt1 * DBK < p.K ? kt1 * DBK : p.K;   // this workgroup's pixel range ends here: later tiles load zeros
  PixelsKS oa;
  oa.init(p, tm * DBM, wave);
  oa.Ktot = k_end;
  MatKS ob;
  ob.init(p.mat, p.mat_bytes, tn * DBN, p.N, k_end, p.Cout);
  float* out = p.out_f32 + (size_t)blockIdx.y * p.M * p.N;   // split s writes partial s (gridDim.y == 1: the result)
  StoreEpilogue epi{nullptr, nullptr, out, p.M, p.N, p.ldc, 0, tm * DBM, tn * DBN, p.vec_out != 0};
  dl::gemm_tile_dl<DBM, DBN, DBK, DSTAGES, DWM, DWN>(oa, ob, kt0 * DBK, kt1 > kt0 ? kt1 - kt0 : 0, smem, epi);
}

constexpr size_t kLdsDl = (size_t)DSTAGES * (DBM + DBN) * DBK * sizeof(unsigned short);

}  // namespace cdl


// ---- halo forms of F and dX (channel counts that are multiples of 16, images at most 32 wide) -------
// The gather kernels above fetch every pixel once per tap.  Here a tile is a run of PBM consecutive
// pixels (NHWC order) and one step of the reduction covers 16 channels of all nine taps: the LDS stage
// holds those 16 channels of the pixels [p0 - HALO, p0 + PBM + HALO) -- a contiguous range of memory,
// no gather -- and the nine taps read it shifted by dy * W + dx pixels.  Rows that a tap would take from
// outside the image (padding, the neighbouring row or image) are zeroed after the read from a per-lane
// 9-bit mask.  Next to it the stage holds the 9 x 16 rows of W that go with those channels.  Per step a
// 256-pixel tile moves 29 KB for 4.7 MFLOP, a quarter of the gather kernel's bytes per flop.
// Stage layout: one KB (a wave's 64 x 16 bytes) per load slot; slots [0, A_SLOTS) are the patch (32
// pixels of 32 bytes each), the next 18 the weights.  Patch pixel r keeps its two 16-byte chunks swapped
// when (r >> 3) & 1, which makes the 16-lane phases of a fragment read hit 16 different bank groups.
namespace halo {

using dl::lds_s16x4_ptr;
using dl::s16x4;
using dl::s16x8;

constexpr int HALO = 33, CK = 16, HBN = 64, W_SLOTS = 18, HSTAGES = 2;

template <int PBM, int WM, int WN, bool DX>
struct Tile {
  static constexpr int NW = WM * WN, TM = PBM / WM / 32, TN = HBN / WN / 32;
  static constexpr int A_SLOTS = (PBM + 2 * HALO + 31) / 32;
  static constexpr int PW = (A_SLOTS + W_SLOTS + NW - 1) / NW;      // loads per wave per step
  static constexpr int STAGE = PW * NW * 512;                       // halves
  static constexpr size_t LDS_BYTES = (size_t)HSTAGES * STAGE * 2;
  static_assert(TM >= 1 && TN >= 1 && PBM % (WM * 32) == 0, "");

  __amdgpu_buffer_rsrc_t rs_img, rs_mat;
  int W, KT;
  int base[PW], inc[PW];        // byte offset of this lane's chunk at step 0 (-1: nothing to load), bytes per step
  unsigned tapmask[TM];         // bit t: tap t of this lane's pixel in row tile i lies inside the image

  __device__ __forceinline__ void init(const ConvKArgs& p, int p0, int n0, int wave_u, int wm) {
    rs_img = make_rsrc(p.img, p.img_bytes);
    rs_mat = make_rsrc(p.mat, p.mat_bytes);
    W = p.W;
    const int C = p.Cimg;               // channels of the gathered image = length of the reduction per tap
    KT = C / CK;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < PW; ++i) {
      const int idx = wave_u * PW + i;
      if (idx < A_SLOTS) {
        const int pl = idx * 32 + (lane >> 1);
        const int q = (lane & 1) ^ ((pl >> 3) & 1);
        const int gp = p0 - HALO + pl;
        base[i] = (gp >= 0 && gp < p.M) ? (gp * C + q * 8) * 2 : -1;
        inc[i] = CK * 2;
      } else if (idx < A_SLOTS + W_SLOTS) {
        const int g = idx - A_SLOTS;
        if constexpr (!DX) {   // W[(tap, c)][o]: 8 k-rows of 64 outputs per slot, k-strided layout as in dl::OperandKS<64>
          const int kr = g * 8 + (lane >> 3);
          const int chunk = (lane & 7) ^ (((kr >> 1) & 1) << 2);
          const int tap = kr / CK, j = kr % CK;
          const int col = n0 + chunk * 8;
          base[i] = col < p.N ? ((tap * C + j) * p.Cout + col) * 2 : -1;
          inc[i] = CK * p.Cout * 2;
        } else {               // W[tap][c0 + n][o]: per tap 64 rows (input channels) of 16 outputs, rows of 32 bytes like the patch
          const int tap = g >> 1, rl = (g & 1) * 32 + (lane >> 1);
          const int q = (lane & 1) ^ ((rl >> 3) & 1);
          const int n = n0 + rl;
          base[i] = n < p.N ? ((tap * p.Cin + p.c0 + n) * p.Cout + q * 8) * 2 : -1;
          inc[i] = CK * 2;
        }
      } else {
        base[i] = -1; inc[i] = 0;
      }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = p0 + wm * (TM * 32) + i * 32 + (lane & 31);
      unsigned mask = 0;
      if (m < p.M) {
        const int t = (int)p.divW.div((unsigned)m), x = m - t * W;
        const int y = t - (int)p.divH.div((unsigned)t) * p.H;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
          int dy, dx;
          tap_offsets(tap, DX, dy, dx);
          const int yy = y + dy, xx = x + dx;
          if (yy >= 0 && yy < p.H && xx >= 0 && xx < W) mask |= 1u << tap;
        }
      }
      tapmask[i] = mask;
    }
  }
  __device__ __forceinline__ void issue(int t, unsigned short* stage, int wave_u) const {
#pragma unroll
    for (int i = 0; i < PW; ++i) {
      const int idx = wave_u * PW + i;
      const unsigned off = (base[i] >= 0 && t < KT) ? (unsigned)(base[i] + t * inc[i]) : kOOB;
      if (idx < A_SLOTS) dl::load_to_lds_16(rs_img, off, stage + idx * 512);
      else dl::load_to_lds_16(rs_mat, off, stage + idx * 512);
    }
  }
  // A fragment of row tile i (32 pixels from row0), tap `tap`: lane (r, g) reads channels 8g..8g+7 of pixel r shifted
  template <int TAP>
  __device__ __forceinline__ bf16x8 frag_a(const unsigned short* stage, int row0, int i) const {
    const int lane = threadIdx.x & 63;
    constexpr int kh = TAP / 3, kw = TAP % 3;
    constexpr int dy = DX ? 1 - kh : kh - 1, dx = DX ? 1 - kw : kw - 1;
    const int pl = HALO + row0 + (lane & 31) + dy * W + dx;
    const int slot = (lane >> 5) ^ ((pl >> 3) & 1);
    bf16x8 v = *(const bf16x8*)(stage + pl * 16 + slot * 8);
    if (!((tapmask[i] >> TAP) & 1u)) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    return v;
  }
  template <int TAP>
  __device__ __forceinline__ bf16x8 frag_b(const unsigned short* stage, int col0) const {
    const int lane = threadIdx.x & 63;
    const unsigned short* wst = stage + A_SLOTS * 512;
    if constexpr (!DX) {   // transposing read, as dl::OperandKS<64>::frag with k = 16 TAP + ...
      const int l16 = lane & 15, j = l16 >> 2, a = l16 & 3;
      const int col = col0 + ((lane >> 4) & 1) * 16 + a * 4;
      const int k = TAP * 16 + (lane >> 5) * 8 + j;
      const int chunk = (col >> 3) ^ (((j >> 1) & 1) << 2);
      const unsigned short* q = wst + k * 64 + chunk * 8 + (col & 7);
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)q);
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(q + 4 * 64));
      const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, v);
    } else {
      const int rl = col0 + (lane & 31);
      const int slot = (lane >> 5) ^ ((rl >> 3) & 1);
      return *(const bf16x8*)(wst + TAP * 1024 + rl * 16 + slot * 8);
    }
  }
};

// Main loop: the pipeline of dl::gemm_tile_dl (loads of step t + HSTAGES issued while step t is multiplied, one
// barrier per step, before its last two substeps) with nine substeps per step, one per tap.
template <int PBM, int WM, int WN, bool DX, class Epi>
__device__ __forceinline__ void run(const Tile<PBM, WM, WN, DX>& tl, unsigned short* smem, Epi epi) {
  using T = Tile<PBM, WM, WN, DX>;
  constexpr int TM = T::TM, TN = T::TN, STAGE = T::STAGE, LOADS = T::PW;
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

  // Fragments are fetched two taps ahead into three register buffers (a tap has only TM * TN MFMAs to cover
  // an LDS read with, and the small tile runs one wave per SIMD); nine taps per step keep the buffers' roles
  // the same in every step.
  bf16x8 fa[3][TM], fb[3][TN];
  auto read_frags = [&](const unsigned short* st, auto tap_tag, bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
    constexpr int TAP = decltype(tap_tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i) a[i] = tl.template frag_a<TAP>(st, wm * (TM * 32) + i * 32, i);
#pragma unroll
    for (int j = 0; j < TN; ++j) b[j] = tl.template frag_b<TAP>(st, wn * (TN * 32) + j * 32);
  };
  auto mfmas = [&](bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };
  auto issue = [&](int t) { tl.issue(t, smem + (t % HSTAGES) * STAGE, wave); };

#pragma unroll
  for (int t = 0; t < HSTAGES; ++t) issue(t);
  dl::wait_vmcnt<(HSTAGES - 1) * LOADS>();
  __syncthreads();
  read_frags(smem, std::integral_constant<int, 0>{}, fa[0], fb[0]);
  read_frags(smem, std::integral_constant<int, 1>{}, fa[1], fb[1]);

  auto step = [&](int t) {
    const unsigned short* cur = smem + (t % HSTAGES) * STAGE;
    const unsigned short* nxt = smem + ((t + 1) % HSTAGES) * STAGE;
    auto taps = [&](auto self, auto tap_tag) -> void {
      constexpr int TAP = decltype(tap_tag)::value;
      if constexpr (TAP < 7) {   // taps 0..6 fetch taps 2..8 of this step
        read_frags(cur, std::integral_constant<int, TAP + 2>{}, fa[(TAP + 2) % 3], fb[(TAP + 2) % 3]);
        mfmas(fa[TAP % 3], fb[TAP % 3]);
        self(self, std::integral_constant<int, TAP + 1>{});
      }
    };
    taps(taps, std::integral_constant<int, 0>{});
    dl::wait_vmcnt<(HSTAGES - 2) * LOADS>();   // this wave's part of step t+1 has landed
    __syncthreads();                            // ... and everyone's; every tap of step t is in registers by now
    issue(t + HSTAGES);
    read_frags(nxt, std::integral_constant<int, 0>{}, fa[0], fb[0]);
    mfmas(fa[1], fb[1]);                        // tap 7
    read_frags(nxt, std::integral_constant<int, 1>{}, fa[1], fb[1]);
    mfmas(fa[2], fb[2]);                        // tap 8
  };
  const int KT = tl.KT;
  for (int t = 0; t < KT; ++t) step(t);
  dl::wait_vmcnt<0>();   // the trailing (empty) steps still write LDS
  __syncthreads();

  static_assert((size_t)WM * WN * 32 * (TN * 32 + 8) * 4 <= T::LDS_BYTES, "epilogue band does not fit the ring");
  core::epilogue_through_lds<TM, TN>(reinterpret_cast<float*>(smem), acc, wave, lane, wm * (TM * 32), wn * (TN * 32), epi);
}

template <int PBM, int WM, int WN, bool DX>
__global__ void __launch_bounds__(WM* WN * 64) conv_halo_kernel(ConvKArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  const int nbn = (p.N + HBN - 1) / HBN;
  const int tm = blockIdx.x / nbn, tn = blockIdx.x % nbn;   // the column tiles of one pixel tile run next to each other
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  Tile<PBM, WM, WN, DX> tl;
  tl.init(p, tm * PBM, tn * HBN, wave, wave / WN);
  StoreEpilogueT<DX> epi{p.out_z, DX ? nullptr : p.out_a, nullptr, p.M, p.N, p.ldc, DX ? 0 : p.act, tm * PBM, tn * HBN, p.vec_out != 0, nullptr,
                         DX ? p.had_s : nullptr, DX ? p.had_lut : nullptr, DX ? p.pool_wp : 0};
  run<PBM, WM, WN, DX>(tl, smem, epi);
  if constexpr (!DX) {
    if (p.pool_a) {
      // ReLU and 2 x 2 max-pooling of this workgroup's own tile of Z (the launcher has checked that a tile is a whole
      // number of image row pairs): once all waves' stores of Z have completed, each lane reads the four pixels of one
      // window for eight channels back (from L2: nobody has read these lines before) and writes the pooled activation.
      // The arithmetic of the stand-alone pooling kernel: the maximum of relu of the stored bf16 values.
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      const int C = p.ldc, W = p.W, Wp = W >> 1;
      constexpr int CG = HBN / 8;                       // groups of eight channels in the tile
      for (int item = threadIdx.x; item < (PBM / 4) * CG; item += WM * WN * 64) {
        const int pp = item / CG, c = tn * HBN + (item % CG) * 8;
        const int j = pp / Wp, xp = pp - j * Wp;
        const int p00 = tm * PBM + j * 2 * W + 2 * xp;
        if (p00 >= p.M || c >= p.N) continue;
        const unsigned short* z0 = p.out_z + (size_t)p00 * C + c;
        const u32x4 zv[4] = {*reinterpret_cast<const u32x4*>(z0), *reinterpret_cast<const u32x4*>(z0 + C),
                             *reinterpret_cast<const u32x4*>(z0 + (size_t)W * C), *reinterpret_cast<const u32x4*>(z0 + (size_t)W * C + C)};
        u32x4 out;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          float best[2];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const float lo = bf16_to_f32((unsigned short)(zv[k][d] & 0xffffu)), hi = bf16_to_f32((unsigned short)(zv[k][d] >> 16));
            const float rl = lo > 0.f ? lo : 0.f, rh = hi > 0.f ? hi : 0.f;
            if (k == 0 || rl > best[0]) best[0] = rl;
            if (k == 0 || rh > best[1]) best[1] = rh;
          }
          out[d] = (unsigned)bf16_bits(best[0]) | ((unsigned)bf16_bits(best[1]) << 16);
        }
        *reinterpret_cast<u32x4*>(p.pool_a + ((size_t)(tm * PBM) / 4 + pp) * C + c) = out;
      }
    }
  }
}

// the halo forms apply when both channel counts allow 16-byte chunks and 16-channel steps, and the row fits the halo
inline bool ok(const ConvDesc& c, int c_reduce, const void* a, const void* b) {
  return c_reduce % CK == 0 && c.Cin % 8 == 0 && c.Cout % 8 == 0 && c.W + 1 <= HALO && (uintptr_t)a % 16 == 0 && (uintptr_t)b % 16 == 0;
}

template <bool DX>
hipError_t launch(const ConvKArgs& p, hipStream_t s) {
  const int nbn = (p.N + HBN - 1) / HBN;
  const long t256 = (long)((p.M + 255) / 256) * nbn;
  if (t256 >= 256) {   // 256-pixel tiles when they still give every CU a workgroup
    using T = Tile<256, 4, 2, DX>;
    auto kern = conv_halo_kernel<256, 4, 2, DX>;
    static bool attr = false;
    if (!attr) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)T::LDS_BYTES);
      if (e != hipSuccess) return e;
      attr = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)t256), dim3(512), T::LDS_BYTES, s, p);
  } else {
    using T = Tile<128, 4, 2, DX>;
    auto kern = conv_halo_kernel<128, 4, 2, DX>;
    static bool attr = false;
    if (!attr) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)T::LDS_BYTES);
      if (e != hipSuccess) return e;
      attr = true;
    }
    const long t128 = (long)((p.M + 127) / 128) * nbn;
    hipLaunchKernelGGL(kern, dim3((unsigned)t128), dim3(512), T::LDS_BYTES, s, p);
  }
  return hipGetLastError();
}

}  // namespace halo

template <bool ALIGNED_A, bool ALIGNED_B>
__global__ void __launch_bounds__(NT) conv_fwd_kernel(ConvKArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int tm, tn;
  tile_of_block<false>(blockIdx.x, (p.M + BM - 1) / BM, (p.N + BN - 1) / BN, tm, tn);
  StagePixelsKC<ALIGNED_A> sa;
  sa.init(p, tm * BM, false);
  StageKS<BN, BK, NT, ALIGNED_B> sb;
  sb.rs = make_rsrc(p.mat, p.mat_bytes);
  sb.r0 = tn * BN; sb.Rtot = p.N; sb.Ktot = p.K; sb.ld = p.Cout; sb.tid = threadIdx.x;
  StoreEpilogue epi{p.out_z, p.out_a, nullptr, p.M, p.N, p.ldc, p.act, tm * BM, tn * BN, p.vec_out != 0};
  gemm_tile<BM, BN, BK, WM, WN>(sa, sb, 0, (p.K + BK - 1) / BK, smem, epi);
}

__global__ void __launch_bounds__(NT) conv_dx_kernel(ConvKArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int tm, tn;
  tile_of_block<false>(blockIdx.x, (p.M + BM - 1) / BM, (p.N + BN - 1) / BN, tm, tn);
  StagePixelsKC<true> sa;
  sa.init(p, tm * BM, true);
  StageWeightsDX sb;
  sb.init(p, tn * BN);
  StoreEpilogueT<true> epi{p.out_z, nullptr, nullptr, p.M, p.N, p.ldc, 0, tm * BM, tn * BN, p.vec_out != 0, nullptr, p.had_s, p.had_lut, p.pool_wp};
  gemm_tile<BM, BN, BK, WM, WN>(sa, sb, 0, (p.K + BK - 1) / BK, smem, epi);
}

template <bool ALIGNED_A, bool ALIGNED_B>
__global__ void __launch_bounds__(NT) conv_dw_kernel(ConvKArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  const int nbn = (p.N + BN - 1) / BN;
  const int tm = blockIdx.x / nbn, tn = blockIdx.x % nbn;
  StagePixelsKS<ALIGNED_A> sa;
  sa.init(p, tm * BM);
  StageKS<BN, BK, NT, ALIGNED_B> sb;
  sb.rs = make_rsrc(p.mat, p.mat_bytes);
  sb.r0 = tn * BN; sb.Rtot = p.N; sb.Ktot = p.K; sb.ld = p.Cout; sb.tid = (threadIdx.x + NT / 2) % NT;
  const int KT = (p.K + BK - 1) / BK;
  const int kt0 = blockIdx.y * p.kt_per_split;
  const int kt1 = kt0 + p.kt_per_split < KT ? kt0 + p.kt_per_split : KT;
  float* out = p.out_f32 + (size_t)blockIdx.y * p.M * p.N;   // split s writes partial s (gridDim.y == 1: the result)
  StoreEpilogue epi{nullptr, nullptr, out, p.M, p.N, p.ldc, 0, tm * BM, tn * BN, p.vec_out != 0};
  gemm_tile<BM, BN, BK, WM, WN>(sa, sb, kt0, kt1, smem, epi);
}

// Sums the split-K partials of dW in a fixed order.  A block handles 32 consecutive outputs; its eight
// waves-halves each add up one eighth of the splits (a contiguous range, in order, eight loads in flight),
// and the eight sub-sums are added in order through LDS: short dependent chains even for 128 splits.
// With `master` set the sum is not stored: it is applied to the fp32 master weights (w <- fma(-lr, g, w), the arithmetic of
// the stand-alone update kernel) and the bf16 copy of the result goes to `work` (Eq. 6 moved into the task that forms G).
__global__ void __launch_bounds__(256) reduce_partials_kernel(const float* __restrict__ part, float* __restrict__ g, size_t n, int splits,
                                                              float* __restrict__ master, unsigned short* __restrict__ work, float neg_lr) {
  __shared__ float sub[8][32];
  const int o = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const size_t i = (size_t)blockIdx.x * 32 + o;
  const int per = (splits + 7) / 8;
  const int s_begin = grp * per, s_end = s_begin + per < splits ? s_begin + per : splits;
  float acc = 0.f;
  if (i < n) {
    for (int s0 = s_begin; s0 < s_end; s0 += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = s0 + u < s_end ? part[(size_t)(s0 + u) * n + i] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (s0 + u < s_end) acc += v[u];
    }
  }
  sub[grp][o] = acc;
  __syncthreads();
  if (grp == 0 && i < n) {
    float t = sub[0][o];
#pragma unroll
    for (int k = 1; k < 8; ++k) t += sub[k][o];
    if (master) {
      const float w = fmaf(neg_lr, t, master[i]);
      master[i] = w;
      work[i] = bf16_bits(w);
    } else {
      g[i] = t;
    }
  }
}

constexpr size_t kLds = 2ull * (BM + BN) * BK * sizeof(unsigned short);

template <class K>
hipError_t set_lds(K kern) {
  return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
}

// both loops use 128 x 64 tiles; a split covers at least 512 pixels
int dw_splits(const ConvDesc& c) {
  const long M = 9L * c.Cin, N = c.Cout, K = (long)c.B * c.H * c.W;
  const long tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  long s = (512 + tiles - 1) / tiles;   // aim at two workgroups per CU (measured on the six layers of the VGG-style workload: 384, 448, 576 ... 2048 are all slower)
  if (s > K / 512) s = K / 512;
  if (s > 256) s = 256;
  if (s < 1) s = 1;
  return (int)s;
}

// the direct-to-LDS kernels need 16-byte chunks of 8 channels everywhere
bool dl_ok(const ConvDesc& c, const void* a, const void* b) {
  return c.Cin % 8 == 0 && c.Cout % 8 == 0 && (uintptr_t)a % 16 == 0 && (uintptr_t)b % 16 == 0;
}

template <class K>
hipError_t set_lds_dl(K kern, bool& done) {
  if (done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)cdl::kLdsDl);
  done = e == hipSuccess;
  return e;
}

// largest dividends: a pixel index (+ one K tile of overshoot) for W and H, a (tap, channel) index (+ a tile) for C
void set_divs(ConvKArgs& p, const ConvDesc& c) {
  const unsigned long long pix = (unsigned long long)c.B * c.H * c.W + 256;
  p.divW = FastDiv::make((unsigned)c.W, pix);
  p.divH = FastDiv::make((unsigned)c.H, pix);
  p.divC = FastDiv::make((unsigned)p.Cimg, 9ull * p.Cimg + 256);
}

bool fits32(const ConvDesc& c) {
  const unsigned long long img = (unsigned long long)c.B * c.H * c.W * (c.Cin > c.Cout ? c.Cin : c.Cout) * 2;
  return img < 0x7fffffffull && c.B > 0 && c.H > 0 && c.W > 0 && c.H < 32768 && c.W < 32768 && c.Cin > 0 && c.Cout > 0;
}

}  // namespace

size_t conv_grad_weight_scratch_bytes(const ConvDesc& c) {
  const int s = dw_splits(c);
  return s > 1 ? (size_t)s * 9 * c.Cin * c.Cout * sizeof(float) : 0;
}

hipError_t launch_conv_fwd(const ConvDesc& c, bool bf16, const void* x, const void* w, void* out_z, void* out_a, int act, hipStream_t s,
                           void* pooled_a, bool* pooled_done) {
  if (pooled_done) *pooled_done = false;
  if (!bf16) return hipErrorNotSupported;
  if (!fits32(c) || !x || !w) return hipErrorInvalidValue;
  ConvKArgs p{};
  p.img = (const unsigned short*)x; p.mat = (const unsigned short*)w;
  p.out_z = (unsigned short*)out_z; p.out_a = (unsigned short*)out_a;
  p.B = c.B; p.H = c.H; p.W = c.W; p.Cimg = c.Cin; p.Cin = c.Cin; p.Cout = c.Cout;
  p.M = c.B * c.H * c.W; p.N = c.Cout; p.K = 9 * c.Cin;
  p.ldc = c.Cout; p.act = act;
  p.img_bytes = (unsigned)((size_t)p.M * c.Cin * 2); p.mat_bytes = (unsigned)((size_t)p.K * c.Cout * 2);
  p.vec_out = (c.Cout % 4 == 0) && ((uintptr_t)out_z % 8 == 0) && ((uintptr_t)out_a % 8 == 0);
  set_divs(p, c);
  const bool al_a = c.Cin % 8 == 0 && (uintptr_t)x % 16 == 0, al_b = c.Cout % 8 == 0 && (uintptr_t)w % 16 == 0;
  const int nb = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  if (conv_thin_ok(c, x, w)) return launch_conv_thin_fwd(c, x, w, out_z, out_a, act, s);
  if (halo::ok(c, c.Cin, x, w)) {
    // pooling in the same launch: ReLU layers whose tiles (128 or 256 pixels) are whole numbers of image row pairs
    if (pooled_a && pooled_done && out_z && !out_a && act == ACT_RELU && c.H % 2 == 0 && c.W % 2 == 0 && 128 % (2 * c.W) == 0 &&
        (uintptr_t)out_z % 16 == 0 && (uintptr_t)pooled_a % 16 == 0) {
      p.pool_a = (unsigned short*)pooled_a;
      *pooled_done = true;
    }
    return halo::launch<false>(p, s);
  }
  if (dl_ok(c, x, w)) {
    static bool attr_dl = false;
    if (hipError_t e = set_lds_dl(cdl::conv_fwd_dl_kernel, attr_dl)) return e;
    hipLaunchKernelGGL(cdl::conv_fwd_dl_kernel, dim3(nb), dim3(cdl::DNT), cdl::kLdsDl, s, p);
    return hipGetLastError();
  }
  static bool attr = false;
  if (!attr) {
    hipError_t e = set_lds(conv_fwd_kernel<true, true>);
    if (e == hipSuccess) e = set_lds(conv_fwd_kernel<false, true>);
    if (e == hipSuccess) e = set_lds(conv_fwd_kernel<true, false>);
    if (e == hipSuccess) e = set_lds(conv_fwd_kernel<false, false>);
    if (e != hipSuccess) return e;
    attr = true;
  }
  if (al_a && al_b) hipLaunchKernelGGL((conv_fwd_kernel<true, true>), dim3(nb), dim3(NT), kLds, s, p);
  else if (!al_a && al_b) hipLaunchKernelGGL((conv_fwd_kernel<false, true>), dim3(nb), dim3(NT), kLds, s, p);
  else if (al_a && !al_b) hipLaunchKernelGGL((conv_fwd_kernel<true, false>), dim3(nb), dim3(NT), kLds, s, p);
  else hipLaunchKernelGGL((conv_fwd_kernel<false, false>), dim3(nb), dim3(NT), kLds, s, p);
  return hipGetLastError();
}

hipError_t launch_conv_grad_act(const ConvDesc& c, bool bf16, const void* dy, const void* w, void* dx, int c0, int c1, hipStream_t s,
                                const void* had_s, const float* had_lut, bool had_pooled) {
  if (!bf16) return hipErrorNotSupported;
  if (!fits32(c) || !dy || !w || !dx || c0 < 0 || c1 > c.Cin || c0 >= c1) return hipErrorInvalidValue;
  // 16-byte chunks of dy and of w along the output channels
  if (c.Cout % 8 != 0 || (uintptr_t)dy % 16 != 0 || (uintptr_t)w % 16 != 0) return hipErrorNotSupported;
  ConvKArgs p{};
  p.img = (const unsigned short*)dy; p.mat = (const unsigned short*)w;
  p.out_z = (unsigned short*)dx + c0;
  p.B = c.B; p.H = c.H; p.W = c.W; p.Cimg = c.Cout; p.Cin = c.Cin; p.Cout = c.Cout; p.c0 = c0;
  p.M = c.B * c.H * c.W; p.N = c1 - c0; p.K = 9 * c.Cout;
  p.ldc = c.Cin; p.act = 0;
  p.img_bytes = (unsigned)((size_t)p.M * c.Cout * 2); p.mat_bytes = (unsigned)((size_t)9 * c.Cin * c.Cout * 2);
  p.vec_out = (p.N % 4 == 0) && (c.Cin % 4 == 0) && ((uintptr_t)p.out_z % 8 == 0);
  if (had_s) {
    p.had_s = (const unsigned short*)had_s + c0;
    p.had_lut = had_lut;
    p.pool_wp = had_pooled ? c.W : 0;
    if (had_pooled && had_lut) return hipErrorInvalidValue;   // routing exists in the ReLU form only
    p.vec_out = p.vec_out && ((uintptr_t)p.had_s % 8 == 0);
  }
  set_divs(p, c);
  const int nb = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  if (halo::ok(c, c.Cout, dy, w)) return halo::launch<true>(p, s);
  if (dl_ok(c, dy, w) && c0 % 8 == 0) {
    static bool attr_dl = false;
    if (hipError_t e = set_lds_dl(cdl::conv_dx_dl_kernel, attr_dl)) return e;
    hipLaunchKernelGGL(cdl::conv_dx_dl_kernel, dim3(nb), dim3(cdl::DNT), cdl::kLdsDl, s, p);
    return hipGetLastError();
  }
  static bool attr = false;
  if (!attr) {
    hipError_t e = set_lds(conv_dx_kernel);
    if (e != hipSuccess) return e;
    attr = true;
  }
  hipLaunchKernelGGL(conv_dx_kernel, dim3(nb), dim3(NT), kLds, s, p);
  return hipGetLastError();
}

hipError_t launch_conv_grad_weight(const ConvDesc& c, bool bf16, const void* x, const void* dy, float* g, float* partial, hipStream_t s,
                                   float* sgd_master, void* sgd_work, float sgd_lr) {
  if (!bf16) return hipErrorNotSupported;
  if (!fits32(c) || !x || !dy || (!g && !sgd_master)) return hipErrorInvalidValue;
  const int splits = dw_splits(c);
  if (splits > 1 && !partial) return hipErrorInvalidValue;
  // the fused update lives in the kernel that sums the split-K partials
  if (sgd_master && (splits <= 1 || !sgd_work || g)) return hipErrorInvalidValue;
  unsigned short* const work = (unsigned short*)sgd_work;
  const float neg_lr = -sgd_lr;
  if (splits > 1 && conv_thin_ok(c, x, dy)) {
    const int chunks = conv_thin_dw_chunks(c), groups = chunks < splits ? chunks : splits;   // the scratch holds `splits` partials
    if (hipError_t e = launch_conv_thin_dw(c, x, dy, partial, groups, s)) return e;
    const size_t n = (size_t)9 * c.Cin * c.Cout;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 31) / 32)), dim3(256), 0, s, (const float*)partial, g, n, groups, sgd_master, work, neg_lr);
    return hipGetLastError();
  }
  ConvKArgs p{};
  p.img = (const unsigned short*)x; p.mat = (const unsigned short*)dy;
  p.out_f32 = splits > 1 ? partial : g;
  p.B = c.B; p.H = c.H; p.W = c.W; p.Cimg = c.Cin; p.Cin = c.Cin; p.Cout = c.Cout;
  p.M = 9 * c.Cin; p.N = c.Cout; p.K = c.B * c.H * c.W;
  p.ldc = c.Cout; p.act = 0;
  p.img_bytes = (unsigned)((size_t)p.K * c.Cin * 2); p.mat_bytes = (unsigned)((size_t)p.K * c.Cout * 2);
  const bool use_dl = dl_ok(c, x, dy);
  const int bk = use_dl ? cdl::DBK : BK;
  const int KT = (p.K + bk - 1) / bk;
  p.kt_per_split = (KT + splits - 1) / splits;
  p.vec_out = (c.Cout % 4 == 0) && ((uintptr_t)p.out_f32 % 16 == 0) && (((size_t)p.M * p.N) % 4 == 0);
  set_divs(p, c);
  const bool al_a = c.Cin % 8 == 0 && (uintptr_t)x % 16 == 0, al_b = c.Cout % 8 == 0 && (uintptr_t)dy % 16 == 0;
  const int nb = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  static bool attr = false;
  if (!attr) {
    hipError_t e = set_lds(conv_dw_kernel<true, true>);
    if (e == hipSuccess) e = set_lds(conv_dw_kernel<false, true>);
    if (e == hipSuccess) e = set_lds(conv_dw_kernel<true, false>);
    if (e == hipSuccess) e = set_lds(conv_dw_kernel<false, false>);
    if (e != hipSuccess) return e;
    attr = true;
  }
  const dim3 grid(nb, splits);
  if (use_dl) {
    static bool attr_dl = false;
    if (hipError_t e = set_lds_dl(cdl::conv_dw_dl_kernel, attr_dl)) return e;
    hipLaunchKernelGGL(cdl::conv_dw_dl_kernel, grid, dim3(cdl::DNT), cdl::kLdsDl, s, p);
  } else if (al_a && al_b) hipLaunchKernelGGL((conv_dw_kernel<true, true>), grid, dim3(NT), kLds, s, p);
  else if (!al_a && al_b) hipLaunchKernelGGL((conv_dw_kernel<false, true>), grid, dim3(NT), kLds, s, p);
  else if (al_a && !al_b) hipLaunchKernelGGL((conv_dw_kernel<true, false>), grid, dim3(NT), kLds, s, p);
  else hipLaunchKernelGGL((conv_dw_kernel<false, false>), grid, dim3(NT), kLds, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || splits == 1) return e;
  const size_t n = (size_t)p.M * p.N;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 31) / 32)), dim3(256), 0, s, (const float*)partial, g, n, splits, sgd_master, work, neg_lr);
  return hipGetLastError();
}

}  // namespace lp
