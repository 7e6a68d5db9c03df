// fp32 GEMM for the fp32 contexts (small networks): same operand conventions as the bf16 kernel,
// fp32 matrix-core FMAs (v_mfma_f32_16x16x4_f32), 32x32 tile per 256-thread workgroup, one 16x16
// accumulator tile per wave.  Every load is individually guarded, so any shape and stride works.
#include "lp_kernels.h"

namespace lp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct GemmFArgs {
  const float* A;
  const float* B;
  float* out_z;
  float* out_a;
  float* out_f32;
  int M, N, K, lda, ldb, ldc, act;
};

__device__ __forceinline__ float apply_act_f(float z, int act) {
  if (act == ACT_RELU) return z > 0.f ? z : 0.f;
  if (act == ACT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752440f));
  if (act == ACT_TANH) return tanhf(z);
  if (act == ACT_SIGMOID) return 1.f / (1.f + expf(-z));
  return z;
}

template <bool AKC, bool BKC>
__global__ void __launch_bounds__(256) gemm_f32_kernel(GemmFArgs p) {
  constexpr int BT = 32, BK = 32;
  __shared__ float As[BT][BK + 1];
  __shared__ float Bs[BT][BK + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
  const int wr = wave >> 1, wc = wave & 1;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < p.K; k0 += BK) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int id = it * 256 + tid;
      {
        const int row = AKC ? id / BK : id % BT, k = AKC ? id % BK : id / BT;
        const int gm = m0 + row, gk = k0 + k;
        float v = 0.f;
        if (gm < p.M && gk < p.K) v = AKC ? p.A[(size_t)gm * p.lda + gk] : p.A[(size_t)gk * p.lda + gm];
        As[row][k] = v;
      }
      {
        const int row = BKC ? id / BK : id % BT, k = BKC ? id % BK : id / BT;
        const int gn = n0 + row, gk = k0 + k;
        float v = 0.f;
        if (gn < p.N && gk < p.K) v = BKC ? p.B[(size_t)gn * p.ldb + gk] : p.B[(size_t)gk * p.ldb + gn];
        Bs[row][k] = v;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK / 4; ++kk) {
      const float a = As[wr * 16 + (lane & 15)][kk * 4 + (lane >> 4)];
      const float b = Bs[wc * 16 + (lane & 15)][kk * 4 + (lane >> 4)];
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc, 0, 0, 0);
    }
    __syncthreads();
  }
  const int col = n0 + wc * 16 + (lane & 15);
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = m0 + wr * 16 + (lane >> 4) * 4 + r;
    if (row < p.M && col < p.N) {
      const size_t o = (size_t)row * p.ldc + col;
      const float v = acc[r];
      if (p.out_f32) p.out_f32[o] = v;
      if (p.out_z) p.out_z[o] = v;
      if (p.out_a) p.out_a[o] = apply_act_f(v, p.act);
    }
  }
}

}  // namespace

hipError_t launch_gemm_f32(const GemmDesc& d, hipStream_t s) {
  if (d.M <= 0 || d.N <= 0 || d.K <= 0 || !d.A || !d.B) return hipErrorInvalidValue;
  GemmFArgs a;
  a.A = (const float*)d.A;
  a.B = (const float*)d.B;
  a.out_z = (float*)d.out_z;
  a.out_a = (float*)d.out_a;
  a.out_f32 = d.out_f32;
  a.M = d.M; a.N = d.N; a.K = d.K;
  a.lda = d.lda; a.ldb = d.ldb; a.ldc = d.ldc;
  a.act = d.act;
  dim3 grid((d.N + 31) / 32, (d.M + 31) / 32);
  if (grid.y > 65535u) return hipErrorInvalidValue;
  if (d.a_kcontig && d.b_kcontig) hipLaunchKernelGGL((gemm_f32_kernel<true, true>), grid, dim3(256), 0, s, a);
  else if (d.a_kcontig && !d.b_kcontig) hipLaunchKernelGGL((gemm_f32_kernel<true, false>), grid, dim3(256), 0, s, a);
  else if (!d.a_kcontig && !d.b_kcontig) hipLaunchKernelGGL((gemm_f32_kernel<false, false>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((gemm_f32_kernel<false, true>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace lp
