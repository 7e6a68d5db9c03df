// The three products of a fully connected layer with very few outputs (D_l <= 16: a classifier head), Eq. 1, Eq. 4
// and Eq. 5.  On 64 x 64 MFMA tiles such a layer is almost all padding (a 4096 -> 10 layer at batch 128 took 12 + 5 us
// for F with its K split and reduction, 6 us for dX, 10 us for dW); here the whole weight matrix row block W[k..k+8)[0..N)
// is N consecutive 16-byte vectors, so each product is a short vector kernel:
//
//   F   one workgroup per batch row: lanes stride over k in steps of 8, fp32 partial sums, butterfly reduction per
//       wavefront, the four wavefronts added in a fixed order
//   dX  one lane per (row, 8 input features): N-term dot products against the same N vectors of W
//   dW  one lane per input feature and sixteenth of the batch rows, the sixteen parts summed in a fixed tree
//
// fp32 accumulation in a fixed order everywhere (no atomics); every output element is summed in the same order whatever
// column range of dX is asked for.  The launcher (launch_gemm_bf16) comes here for shapes gemm_skinny_shape() accepts.
#include "gemm_core.h"
#include "lp_kernels.h"

namespace lp {
namespace {

using namespace core;

__device__ __forceinline__ float bf_lo(unsigned v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf_hi(unsigned v) { return __uint_as_float(v & 0xffff0000u); }
// element e of consecutive 16-byte vectors of bf16 (e is a compile-time constant after unrolling)
template <int NV>
__device__ __forceinline__ float vec_elem(const u32x4 (&w)[NV], int e) {
  const unsigned d = w[e / 8][(e % 8) / 2];
  return (e & 1) ? bf_hi(d) : bf_lo(d);
}
__device__ __forceinline__ float vec_elem1(const u32x4& v, int e) {
  const unsigned d = v[e / 2];
  return (e & 1) ? bf_hi(d) : bf_lo(d);
}
__device__ __forceinline__ float wave_sum64(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Z[m][0..N) = X[m][0..K) . W[0..K)[0..N), A = f(Z).  K % 8 == 0; X rows and W 16-byte aligned.  One workgroup per
// batch row: lane t takes k = 8 t, 8 t + 2048, ...; a butterfly sums each wavefront, the four wavefronts' sums are added
// as (0 + 1) + (2 + 3).
template <int N>
__global__ void __launch_bounds__(256) skinny_fwd_kernel(const unsigned short* __restrict__ X, const unsigned short* __restrict__ W,
                                                         unsigned short* __restrict__ Z, unsigned short* __restrict__ A, int M, int K, int lda,
                                                         int ldc, int act, const unsigned short* __restrict__ act_lut) {
  __shared__ float part[4][N];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = blockIdx.x;   // the grid has exactly M workgroups
  float acc[N];
#pragma unroll
  for (int n = 0; n < N; ++n) acc[n] = 0.f;
  const unsigned short* x = X + (size_t)m * lda;
  for (int k = threadIdx.x * 8; k < K; k += 2048) {
    const u32x4 xv = *reinterpret_cast<const u32x4*>(x + k);
    u32x4 w[N];
#pragma unroll
    for (int n = 0; n < N; ++n) w[n] = *reinterpret_cast<const u32x4*>(W + (size_t)k * N + n * 8);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const float xk = vec_elem1(xv, kk);
#pragma unroll
      for (int n = 0; n < N; ++n) acc[n] = fmaf(xk, vec_elem<N>(w, kk * N + n), acc[n]);
    }
  }
#pragma unroll
  for (int n = 0; n < N; ++n) {
    const float v = wave_sum64(acc[n]);
    if (lane == 0) part[wave][n] = v;
  }
  __syncthreads();
  if ((int)threadIdx.x < N) {
    const int n = threadIdx.x;
    const unsigned short zb = bf16_bits((part[0][n] + part[1][n]) + (part[2][n] + part[3][n]));
    if (Z) Z[(size_t)m * ldc + n] = zb;
    if (A) A[(size_t)m * ldc + n] = (act == ACT_GELU && act_lut) ? act_lut[zb] : bf16_bits(apply_act(bf16_to_f32(zb), act));
  }
}

// dX[m][k..k+8) = sum_n dY[m][n] W[k..k+8)[n] for the C columns that start at W / dX (the caller has moved both to the
// first column of the range).  VEC: C % 8 == 0 and W, the rows of dX and of the stash are 16-byte aligned; otherwise the
// same sums from 2-byte accesses (a column range that starts or ends off a multiple of 8), so that cutting the columns
// changes no bits.  had_s: the Hadamard product of the layer below on the way out, as in StoreEpilogueT<true>.
template <int N, bool VEC>
__global__ void __launch_bounds__(256) skinny_dx_kernel(const unsigned short* __restrict__ dY, const unsigned short* __restrict__ W,
                                                        unsigned short* __restrict__ dX, int M, int C, int ldc,
                                                        const unsigned short* __restrict__ had_s, const float* __restrict__ had_lut) {
  const int groups = (C + 7) / 8;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)M * groups) return;
  const int m = (int)(i / groups), k = (int)(i % groups) * 8;
  float dy[N];
#pragma unroll
  for (int n = 0; n < N; ++n) dy[n] = bf16_to_f32(dY[(size_t)m * N + n]);
  const size_t off = (size_t)m * ldc + k;
  unsigned short o[8], sb[8];
  if constexpr (VEC) {
    u32x4 w[N];
#pragma unroll
    for (int n = 0; n < N; ++n) w[n] = *reinterpret_cast<const u32x4*>(W + (size_t)k * N + n * 8);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      float a = 0.f;
#pragma unroll
      for (int n = 0; n < N; ++n) a = fmaf(dy[n], vec_elem<N>(w, kk * N + n), a);
      o[kk] = bf16_bits(a);
    }
    if (had_s) {
      const u32x4 sv = *reinterpret_cast<const u32x4*>(had_s + off);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) sb[kk] = (unsigned short)((kk & 1) ? (sv[kk / 2] >> 16) : (sv[kk / 2] & 0xffffu));
    }
  } else {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      float a = 0.f;
      if (k + kk < C) {
#pragma unroll
        for (int n = 0; n < N; ++n) a = fmaf(dy[n], bf16_to_f32(W[(size_t)(k + kk) * N + n]), a);
      }
      o[kk] = bf16_bits(a);
      sb[kk] = (had_s && k + kk < C) ? had_s[off + kk] : (unsigned short)0;
    }
  }
  if (had_s) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const float df = had_lut ? had_lut[sb[kk]] : (bf16_to_f32(sb[kk]) > 0.f ? 1.f : 0.f);
      o[kk] = bf16_bits(bf16_to_f32(o[kk]) * df);
    }
  }
  if constexpr (VEC) {
    u32x4 ov;
#pragma unroll
    for (int q = 0; q < 4; ++q) ov[q] = (unsigned)o[2 * q] | ((unsigned)o[2 * q + 1] << 16);
    *reinterpret_cast<u32x4*>(dX + off) = ov;
  } else {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      if (k + kk < C) dX[off + kk] = o[kk];
  }
}

// G[k][0..N) = sum_m X[m][k] dY[m][0..N), fp32.  A workgroup owns 16 input features; its 16 groups of 16 lanes sum the
// batch rows m = g, g + 16, ... each, and the sixteen partial sums are added pairwise in a fixed tree.
// With `master` set G is not stored: each element is applied to the fp32 master weights (w <- fma(-lr, g, w), the arithmetic
// of the stand-alone update kernel) and the bf16 copy of the result goes to `work` (Eq. 6 moved into the task that forms G).
template <int N>
__global__ void __launch_bounds__(256) skinny_dw_kernel(const unsigned short* __restrict__ X, const unsigned short* __restrict__ dY,
                                                        float* __restrict__ G, int B, int K, int lda,
                                                        float* __restrict__ master, unsigned short* __restrict__ work, float neg_lr) {
  __shared__ float part[16][16 * N];
  const int kl = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int k0 = blockIdx.x * 16, k = k0 + kl;
  float acc[N];
#pragma unroll
  for (int n = 0; n < N; ++n) acc[n] = 0.f;
#pragma unroll 4
  for (int m = g; m < B; m += 16) {
    const float x = k < K ? bf16_to_f32(X[(size_t)m * lda + k]) : 0.f;
#pragma unroll
    for (int n = 0; n < N; ++n) acc[n] = fmaf(x, bf16_to_f32(dY[(size_t)m * N + n]), acc[n]);
  }
#pragma unroll
  for (int n = 0; n < N; ++n) part[g][kl * N + n] = acc[n];
  __syncthreads();
  for (int e = threadIdx.x; e < 16 * N; e += 256) {
    if (k0 + e / N < K) {
      float q[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) q[u] = part[u][e];
#pragma unroll
      for (int w = 8; w > 0; w >>= 1)
#pragma unroll
        for (int u = 0; u < w; ++u) q[u] = q[2 * u] + q[2 * u + 1];
      const size_t o = (size_t)k0 * N + e;
      if (master) {
        const float w = fmaf(neg_lr, q[0], master[o]);
        master[o] = w;
        work[o] = bf16_bits(w);
      } else {
        G[o] = q[0];
      }
    }
  }
}

inline bool al16(const void* p) { return ((uintptr_t)p % 16) == 0; }

template <int N>
hipError_t launch_n(int form, const GemmDesc& d, hipStream_t s) {
  if (form == 0) {
    hipLaunchKernelGGL(skinny_fwd_kernel<N>, dim3((unsigned)d.M), dim3(256), 0, s, (const unsigned short*)d.A, (const unsigned short*)d.B,
                       (unsigned short*)d.out_z, (unsigned short*)d.out_a, d.M, d.K, d.lda, d.ldc, d.act, (const unsigned short*)d.act_lut);
  } else if (form == 1) {
    const size_t n = (size_t)d.M * ((d.N + 7) / 8);
    const bool vec = d.N % 8 == 0 && al16(d.B) && al16(d.out_z) && (!d.had_s || al16(d.had_s));
    if (vec)
      hipLaunchKernelGGL((skinny_dx_kernel<N, true>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const unsigned short*)d.A, (const unsigned short*)d.B,
                         (unsigned short*)d.out_z, d.M, d.N, d.ldc, (const unsigned short*)d.had_s, d.had_s ? d.had_lut : nullptr);
    else
      hipLaunchKernelGGL((skinny_dx_kernel<N, false>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const unsigned short*)d.A, (const unsigned short*)d.B,
                         (unsigned short*)d.out_z, d.M, d.N, d.ldc, (const unsigned short*)d.had_s, d.had_s ? d.had_lut : nullptr);
  } else {
    hipLaunchKernelGGL(skinny_dw_kernel<N>, dim3((unsigned)((d.M + 15) / 16)), dim3(256), 0, s, (const unsigned short*)d.A, (const unsigned short*)d.B,
                       d.out_f32, d.K, d.M, d.lda, d.sgd_master, d.sgd_master ? (unsigned short*)d.out_z : nullptr, -d.sgd_lr);
  }
  return hipGetLastError();
}

}  // namespace

bool gemm_skinny_shape(int batch, int d_in, int d_out) { return d_out >= 1 && d_out <= 16 && d_in % 8 == 0 && batch >= 1 && batch <= 2048; }

// form: 0 = F, 1 = dX, 2 = dW; *taken = false when the operands are not laid out as the kernels need (the caller then
// runs the tiled GEMM).
hipError_t launch_gemm_skinny(const GemmDesc& d, hipStream_t s, bool* taken) {
  *taken = false;
  if (d.sgd_master && (d.a_kcontig || d.b_kcontig)) return hipSuccess;   // the update rides in the dW form only
  if (d.had_s && !(d.a_kcontig && d.b_kcontig)) return hipSuccess;   // the tiled launcher reports the misuse
  int form, batch, d_in = 0, d_out;
  if (d.a_kcontig && !d.b_kcontig) {            // F: X [batch][in] . W [in][out]
    form = 0; batch = d.M; d_in = d.K; d_out = d.N;
    if (!gemm_skinny_shape(batch, d_in, d_out) || d.ldb != d_out || d.ldc < d_out || d.lda % 8 != 0 || d.lda < d_in || !al16(d.A) || !al16(d.B) || d.out_f32 ||
        (!d.out_z && !d.out_a))
      return hipSuccess;
  } else if (d.a_kcontig && d.b_kcontig) {      // dX: dY [batch][out] . (W + c0 rows) [cols][out]^T
    form = 1; batch = d.M; d_out = d.K;
    // decided by the layer alone (ldc is its input width), never by the column range, so that a product and its parts
    // run the same arithmetic
    if (d_out < 1 || d_out > 16 || batch > 2048 || d.ldb != d_out || d.lda != d_out || d.ldc % 8 != 0 || d.ldc < d.N || !d.out_z || d.out_a || d.out_f32)
      return hipSuccess;
  } else if (!d.a_kcontig && !d.b_kcontig) {    // dW: X [batch][in]^T . dY [batch][out]
    form = 2; batch = d.K; d_in = d.M; d_out = d.N;
    // plain: G to out_f32; with the update: master weights in sgd_master, their bf16 copy to out_z, nothing else
    const bool outs_ok = d.sgd_master ? (d.out_z && !d.out_f32 && !d.out_a) : (d.out_f32 && !d.out_z && !d.out_a);
    if (!gemm_skinny_shape(batch, d_in, d_out) || d.ldb != d_out || d.ldc != d_out || d.lda < d_in || !outs_ok) return hipSuccess;
  } else {
    return hipSuccess;
  }
  *taken = true;
  switch (d_out) {
    case 1: return launch_n<1>(form, d, s);
    case 2: return launch_n<2>(form, d, s);
    case 3: return launch_n<3>(form, d, s);
    case 4: return launch_n<4>(form, d, s);
    case 5: return launch_n<5>(form, d, s);
    case 6: return launch_n<6>(form, d, s);
    case 7: return launch_n<7>(form, d, s);
    case 8: return launch_n<8>(form, d, s);
    case 9: return launch_n<9>(form, d, s);
    case 10: return launch_n<10>(form, d, s);
    case 11: return launch_n<11>(form, d, s);
    case 12: return launch_n<12>(form, d, s);
    case 13: return launch_n<13>(form, d, s);
    case 14: return launch_n<14>(form, d, s);
    case 15: return launch_n<15>(form, d, s);
    default: return launch_n<16>(form, d, s);
  }
}

}  // namespace lp
