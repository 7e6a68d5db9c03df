// bf16 x bf16 -> fp32 GEMM launchers for the three products of a fully connected layer
// (Eq. 1, Eq. 4, Eq. 5):
//
//     F   Z  = A_prev . W        A: k contiguous,  B = W  [K][N]: k strided
//     dX  dA = dY . W^T          A: k contiguous,  B = W  [N][K]: k contiguous
//     dW  G  = A_prev^T . dY     A: k strided,     B = dY [K][N]: k strided
//
// Two kernel bodies: gemm_core.h (operands staged through registers; any shape) and gemm_dl.h (direct
// global->LDS loads, transposing LDS reads; needs 16-byte aligned runs).  This file binds plain 2-D
// operands to them and picks a tile shape.
#include "gemm_core.h"
#include "gemm_dl.h"
#include "lp_kernels.h"

#include <mutex>

namespace lp {
namespace {

using namespace core;

struct GemmKArgs {
  const unsigned short* A;
  const unsigned short* B;
  unsigned short* out_z;
  unsigned short* out_a;
  float* out_f32;
  int M, N, K, lda, ldb, ldc, act;
  unsigned a_bytes, b_bytes;
  int vec_out;
  int kt_per_split;     // split-K: K tiles per workgroup in y (0: no split)
  float* partial;       // split-K: [gridDim.y][M][N] fp32
  float* sgd_master;    // SGD variants: fp32 master weights updated in the epilogue
  float neg_lr;
  const unsigned short* act_lut;   // optional table of the activation over all bf16 inputs (GELU)
  const unsigned short* had_s;     // dX form only: stash of the preceding layer; the Hadamard product of Eq. 3 is then applied on the way out
  const float* had_lut;            // ... with f' looked up here (null: the ReLU form)
};

template <bool KC, int R, int BK, int NT, bool ALIGNED>
struct StageSel {
  using type = StageKC<R, BK, NT, ALIGNED>;
};
template <int R, int BK, int NT, bool ALIGNED>
struct StageSel<false, R, BK, NT, ALIGNED> {
  using type = StageKS<R, BK, NT, ALIGNED>;
};

template <int BM, int BN, int BK, int WM, int WN, bool AKC, bool BKC, bool ALIGNED, bool SGD = false>
__global__ void __launch_bounds__(WM* WN * 64) gemm_bf16_kernel(GemmKArgs p) {
  constexpr int NT = WM * WN * 64;
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int tm, tn;
  tile_of_block<(BM == 256 && BN == 256)>(blockIdx.x, (p.M + BM - 1) / BM, (p.N + BN - 1) / BN, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x;

  typename StageSel<AKC, BM, BK, NT, ALIGNED>::type sa;
  sa.rs = make_rsrc(p.A, p.a_bytes);
  sa.r0 = m0; sa.Rtot = p.M; sa.Ktot = p.K; sa.ld = p.lda; sa.tid = tid;
  typename StageSel<BKC, BN, BK, NT, ALIGNED>::type sb;
  sb.rs = make_rsrc(p.B, p.b_bytes);
  sb.r0 = n0; sb.Rtot = p.N; sb.Ktot = p.K; sb.ld = p.ldb;
  sb.tid = BKC ? tid : (tid + NT / 2) % NT;  // when both operands are transposed in registers, start B's blocks on the other waves

  if constexpr (SGD) {
    SgdEpilogue epi{p.sgd_master, p.out_z, p.neg_lr, p.M, p.N, p.ldc, m0, n0, p.vec_out != 0};
    gemm_tile<BM, BN, BK, WM, WN>(sa, sb, 0, (p.K + BK - 1) / BK, smem, epi);
  } else if (p.kt_per_split > 0) {
    // split-K: K tiles [kt0, kt1) into an fp32 partial, as in the direct-to-LDS kernel
    const int KT = (p.K + BK - 1) / BK;
    const int kt0 = blockIdx.y * p.kt_per_split;
    const int kt1 = kt0 + p.kt_per_split < KT ? kt0 + p.kt_per_split : KT;
    StoreEpilogue epi{nullptr, nullptr, p.partial + (size_t)blockIdx.y * p.M * p.N, p.M, p.N, p.N, 0, m0, n0, (p.N % 4) == 0};
    gemm_tile<BM, BN, BK, WM, WN>(sa, sb, kt0, kt1, smem, epi);
  } else {
    StoreEpilogueT<AKC && BKC> epi{p.out_z, p.out_a, p.out_f32, p.M, p.N, p.ldc, p.act, m0, n0, p.vec_out != 0, p.act_lut, p.had_s, p.had_lut};
    gemm_tile<BM, BN, BK, WM, WN>(sa, sb, 0, (p.K + BK - 1) / BK, smem, epi);
  }
}

// direct-to-LDS variant (256x256 tile, K step 32, four LDS stages)
template <int BM, int BN, int BK, int NSTAGE, int WM, int WN, bool AKC, bool BKC, bool SGD = false>
__global__ void __launch_bounds__(WM* WN * 64) gemm_bf16_dl_kernel(GemmKArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int tm, tn;
  tile_of_block<(BM == 256 && BN == 256)>(blockIdx.x, (p.M + BM - 1) / BM, (p.N + BN - 1) / BN, tm, tn);
  typename dl::OperandSel<AKC, BM, BK, WM * WN>::type oa;
  typename dl::OperandSel<BKC, BN, BK, WM * WN>::type ob;
  oa.init(p.A, p.a_bytes, tm * BM, p.M, p.K, p.lda);
  ob.init(p.B, p.b_bytes, tn * BN, p.N, p.K, p.ldb);
  const int KT = (p.K + BK - 1) / BK;
  if constexpr (SGD) {
    SgdEpilogue epi{p.sgd_master, p.out_z, p.neg_lr, p.M, p.N, p.ldc, tm * BM, tn * BN, p.vec_out != 0};
    dl::gemm_tile_dl<BM, BN, BK, NSTAGE, WM, WN>(oa, ob, 0, KT, smem, epi);
    return;
  }
  if (p.kt_per_split > 0) {
    // split-K: this workgroup multiplies K tiles [kt0, kt1) and writes an fp32 partial
    const int kt0 = blockIdx.y * p.kt_per_split;
    const int kt1 = kt0 + p.kt_per_split < KT ? kt0 + p.kt_per_split : KT;
    const int k_end = kt1 * BK < p.K ? kt1 * BK : p.K;
    oa.Ktot = k_end;
    ob.Ktot = k_end;
    StoreEpilogue epi{nullptr, nullptr, p.partial + (size_t)blockIdx.y * p.M * p.N, p.M, p.N, p.N, 0, tm * BM, tn * BN, (p.N % 4) == 0};   // M*N*4 bytes per split: 16-byte aligned when N % 4 == 0
    dl::gemm_tile_dl<BM, BN, BK, NSTAGE, WM, WN>(oa, ob, kt0 * BK, kt1 > kt0 ? kt1 - kt0 : 0, smem, epi);
    return;
  }
  StoreEpilogueT<AKC && BKC> epi{p.out_z, p.out_a, p.out_f32, p.M, p.N, p.ldc, p.act, tm * BM, tn * BN, p.vec_out != 0, p.act_lut, p.had_s, p.had_lut};
  dl::gemm_tile_dl<BM, BN, BK, NSTAGE, WM, WN>(oa, ob, 0, KT, smem, epi);
}

// sums the split-K partials in a fixed order and applies the epilogue (rounding, activation);
// one thread per group of four columns of a row
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float* __restrict__ part, int splits, GemmKArgs p) {
  const int ng = (p.N + 3) / 4;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)p.M * ng) return;
  const int row = (int)(i / ng), col = (int)(i % ng) * 4;
  const size_t mn = (size_t)p.M * p.N, o = (size_t)row * p.N + col;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (p.N % 4 == 0) {
    // eight loads in flight at a time (a partial is one cache miss each); summed in split order
    for (int s0 = 0; s0 < splits; s0 += 8) {
      f32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        v[u] = s0 + u < splits ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(part + (size_t)(s0 + u) * mn + o)) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (s0 + u < splits) {
#pragma unroll
          for (int t = 0; t < 4; ++t) acc[t] += v[u][t];
        }
    }
  } else {
    for (int s0 = 0; s0 < splits; s0 += 8) {   // same order, scalar loads
      float v[8][4];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int t = 0; t < 4; ++t) v[u][t] = (s0 + u < splits && col + t < p.N) ? part[(size_t)(s0 + u) * mn + o + t] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (s0 + u < splits) {
#pragma unroll
          for (int t = 0; t < 4; ++t) acc[t] += v[u][t];
        }
    }
  }
  if (p.sgd_master) {   // a weight-gradient product that is consumed on the spot: Eq. 6 applied to the summed tile
    SgdEpilogue epi{p.sgd_master, p.out_z, p.neg_lr, p.M, p.N, p.ldc, 0, 0, p.vec_out != 0};
    epi(row, col, acc);
    return;
  }
  StoreEpilogueT<true> epi{p.out_z, p.out_a, p.out_f32, p.M, p.N, p.ldc, p.act, 0, 0, p.vec_out != 0, p.act_lut, p.had_s, p.had_lut};
  epi.with_static_act([&](auto store) { store(row, col, acc); });
}

template <int BM, int BN, int BK, int NSTAGE, int WM, int WN, bool AKC, bool BKC, bool SGD = false>
hipError_t launch_dl(const GemmKArgs& a, hipStream_t s) {
  auto kern = gemm_bf16_dl_kernel<BM, BN, BK, NSTAGE, WM, WN, AKC, BKC, SGD>;
  constexpr size_t lds = (size_t)NSTAGE * (BM + BN) * BK * sizeof(unsigned short);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int nb = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  if (a.kt_per_split > 0) {
    // one K range per workgroup row of the grid, then a reduction that applies the real epilogue
    const int KT = (a.K + BK - 1) / BK;
    const int splits = (KT + a.kt_per_split - 1) / a.kt_per_split;
    hipLaunchKernelGGL(kern, dim3(nb, splits), dim3(WM * WN * 64), lds, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t n4 = (size_t)a.M * ((a.N + 3) / 4);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, (const float*)a.partial, splits, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(kern, dim3(nb), dim3(WM * WN * 64), lds, s, a);
  return hipGetLastError();
}

// kind: 0 = register-staged loop (gemm_core.h), 1 = direct-to-LDS loop (gemm_dl.h, K step 64, two stages)
struct TileCfg {
  const char* name;
  int bm, bn, kind;
};
constexpr TileCfg kCfgs[] = {
    {"256x256x64_w2x4", 256, 256, 0},     // 0
    {"128x128x64_w2x2", 128, 128, 0},     // 1
    {"64x64x64_w2x2", 64, 64, 0},         // 2
    {"256x256x64_w2x2", 256, 256, 0},     // 3
    {"256x256x64_dl_w2x4", 256, 256, 1},  // 4
    {"128x128x64_dl_w2x2", 128, 128, 1},  // 5
};

template <int BM, int BN, int BK, int WM, int WN, bool AKC, bool BKC, bool ALIGNED, bool SGD = false>
hipError_t launch_one(const GemmKArgs& a, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, BK, WM, WN, AKC, BKC, ALIGNED, SGD>;
  constexpr size_t lds = 2ull * (BM + BN) * BK * sizeof(unsigned short);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int nb = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  if (a.kt_per_split > 0 && !SGD) {
    const int KT = (a.K + BK - 1) / BK;
    const int splits = (KT + a.kt_per_split - 1) / a.kt_per_split;
    hipLaunchKernelGGL(kern, dim3(nb, splits), dim3(WM * WN * 64), lds, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t n4 = (size_t)a.M * ((a.N + 3) / 4);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, (const float*)a.partial, splits, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(kern, dim3(nb), dim3(WM * WN * 64), lds, s, a);
  return hipGetLastError();
}

template <bool AKC, bool BKC, bool ALIGNED>
hipError_t launch_cfg(int cfg, const GemmKArgs& a, hipStream_t s) {
  switch (cfg) {
    case 0: return launch_one<256, 256, 64, 2, 4, AKC, BKC, ALIGNED>(a, s);
    case 1: return launch_one<128, 128, 64, 2, 2, AKC, BKC, ALIGNED>(a, s);
    case 2: return launch_one<64, 64, 64, 2, 2, AKC, BKC, ALIGNED>(a, s);
    case 3: return launch_one<256, 256, 64, 2, 2, AKC, BKC, ALIGNED>(a, s);
  }
  return hipErrorInvalidValue;
}

// the G product with the update fused into its epilogue (both operands k-strided)
template <bool ALIGNED>
hipError_t launch_cfg_sgd(int cfg, const GemmKArgs& a, hipStream_t s) {
  switch (cfg) {
    case 0: return launch_one<256, 256, 64, 2, 4, false, false, ALIGNED, true>(a, s);
    case 1: return launch_one<128, 128, 64, 2, 2, false, false, ALIGNED, true>(a, s);
    case 2: return launch_one<64, 64, 64, 2, 2, false, false, ALIGNED, true>(a, s);
    case 3: return launch_one<256, 256, 64, 2, 2, false, false, ALIGNED, true>(a, s);
  }
  return hipErrorInvalidValue;
}
hipError_t launch_cfg_dl_sgd(int cfg, const GemmKArgs& a, hipStream_t s) {
  switch (cfg) {
    case 4: return launch_dl<256, 256, 64, 2, 2, 4, false, false, true>(a, s);
    case 5: return launch_dl<128, 128, 64, 2, 2, 2, false, false, true>(a, s);
  }
  return hipErrorInvalidValue;
}

template <bool AKC, bool BKC>
hipError_t launch_cfg_dl(int cfg, const GemmKArgs& a, hipStream_t s) {
  switch (cfg) {
    case 4: return launch_dl<256, 256, 64, 2, 2, 4, AKC, BKC>(a, s);
    case 5: return launch_dl<128, 128, 64, 2, 2, 2, AKC, BKC>(a, s);
  }
  return hipErrorInvalidValue;
}

// how many K ranges a product on 128x128 tiles is cut into (1: not split)
int splitk_factor(int M, int N, int K) {
  const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256);
  const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
  if (t256 >= 192 || t128 >= 256 || K < 2048) return 1;
  long s = 512 / t128;               // two workgroups per CU
  // at least sixteen K steps each (shorter ranges cost more in partial-sum traffic than they gain), four
  // when the whole output is so small (64 K elements) that its partials do not matter
  const long min_k = (long)M * N <= 65536 ? 256 : 1024;
  if (s > K / min_k) s = K / min_k;
  if (s > 16) s = 16;
  return s < 2 ? 1 : (int)s;
}

}  // namespace

int gemm_bf16_splitk_splits(int M, int N, int K) { return splitk_factor(M, N, K); }

size_t gemm_bf16_splitk_bytes(int M, int N, int K) {
  const int s = splitk_factor(M, N, K);
  return s > 1 ? ((size_t)s * M * N * sizeof(float) + 255) / 256 * 256 : 0;
}

// Measurement aid: nothing but the GEMM's matrix instruction.  Each of the eight waves of a workgroup keeps the
// 4 x 2 accumulator tiles of the 256 x 256 GEMM tile (128 registers) and fixed fragments in registers and
// issues `iters` rounds of eight independent v_mfma_f32_32x32x16_bf16: what the matrix pipes sustain with no
// LDS, cache or memory activity to feed them.
namespace {
__global__ void __launch_bounds__(512) mfma_only_kernel(float* __restrict__ out, int iters, int uniform) {
  // operands: pseudo-random values in [-1, 1) (random sign, exponent and mantissa bits, as real activations
  // and weights have: what the multipliers draw depends on how many bits toggle); `uniform` = 1: all lanes
  // hold the same few small values instead
  auto value = [&](unsigned k) -> __bf16 {
    if (uniform) return (__bf16)(0.0009765625f * (float)(1 + (k & 3)));
    unsigned h = (k + 0x9e3779b9u * (blockIdx.x * 512u + threadIdx.x + 1u)) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    return (__bf16)((float)(h & 0xffff) * (1.f / 32768.f) - 1.f);
  };
  bf16x8 a[4], b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) a[i][e] = value(i * 8 + e);
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) b[j][e] = value(32 + j * 8 + e);
  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
  out[(size_t)blockIdx.x * 512 + threadIdx.x] = sum;
}
}  // namespace

hipError_t launch_mfma_only(float* out, int workgroups, int iters, bool uniform_values, hipStream_t s) {
  if (workgroups <= 0 || iters < 0 || !out) return hipErrorInvalidValue;
  hipLaunchKernelGGL(mfma_only_kernel, dim3((unsigned)workgroups), dim3(512), 0, s, out, iters, uniform_values ? 1 : 0);
  return hipGetLastError();
}

// ---- GELU and its derivative over all bfloat16 inputs ---------------------------------------------------
// A bf16 pre-activation has 65536 possible values.  In a product's epilogue the exact GELU costs about 28 vector
// instructions per element, and that arithmetic is exposed (every workgroup of a round reaches its epilogue at the
// same time); a look-up costs one gather from a table whose live part (2^-10 <= |z| < 16: some 3300 entries) sits in
// the CU's L1.  Two tables, static device arrays of the library (128 + 256 KiB per GPU, kept until the process ends),
// each filled once per device by a kernel that evaluates in fp64 and rounds to nearest even:
//   gelu_table[z]       z Phi(z) as bf16       (the F epilogue's second output)
//   gelu_grad_table[z]  Phi(z) + z phi(z) as fp32   (the factor of the Hadamard product, Eq. 3)
// Phi through erfc, so that nothing cancels for z << 0.
namespace {
static __device__ __align__(256) unsigned short gelu_table[65536];
static __device__ __align__(256) float gelu_grad_table[65536];
__global__ void __launch_bounds__(256) gelu_table_fill_kernel(unsigned short* __restrict__ t) {
  const unsigned i = blockIdx.x * 256 + threadIdx.x;
  const double z = (double)bf16_to_f32((unsigned short)i);
  t[i] = bf16_bits((float)(0.5 * z * erfc(-z * 0.70710678118654752440)));
}
__global__ void __launch_bounds__(256) gelu_grad_table_fill_kernel(float* __restrict__ t) {
  const unsigned i = blockIdx.x * 256 + threadIdx.x;
  const double z = (double)bf16_to_f32((unsigned short)i);
  const double cdf = 0.5 * erfc(-z * 0.70710678118654752440);
  const double pdf = 0.39894228040143267794 * exp(-0.5 * z * z);
  t[i] = (float)(cdf + (pdf > 0.0 ? z * pdf : 0.0));   // +-inf: 1 and 0, not inf * 0
}
constexpr int kMaxDevices = 64;
std::mutex table_mutex;
const void* table_ptr[2][kMaxDevices] = {};

// which: 0 = gelu_table, 1 = gelu_grad_table
hipError_t table_of_device(int which, const void** out, hipStream_t s) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(table_mutex);
  if (!table_ptr[which][dev]) {
    void* p = nullptr;
    e = which == 0 ? hipGetSymbolAddress(&p, HIP_SYMBOL(gelu_table)) : hipGetSymbolAddress(&p, HIP_SYMBOL(gelu_grad_table));   // this device's copy
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    if (which == 0) hipLaunchKernelGGL(gelu_table_fill_kernel, dim3(256), dim3(256), 0, s, (unsigned short*)p);
    else hipLaunchKernelGGL(gelu_grad_table_fill_kernel, dim3(256), dim3(256), 0, s, (float*)p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(s);   // kernels on any other stream may read the table from now on
    if (e != hipSuccess) return e;
    table_ptr[which][dev] = p;
  }
  *out = table_ptr[which][dev];
  return hipSuccess;
}
}  // namespace

hipError_t gelu_lut_bf16(const void** out, hipStream_t s) { return table_of_device(0, out, s); }
hipError_t gelu_grad_lut_f32(const float** out, hipStream_t s) {
  const void* p = nullptr;
  const hipError_t e = table_of_device(1, &p, s);
  if (e == hipSuccess) *out = (const float*)p;
  return e;
}

int gemm_bf16_num_cfgs() { return (int)(sizeof(kCfgs) / sizeof(kCfgs[0])); }
const char* gemm_bf16_cfg_name(int cfg) { return (cfg >= 0 && cfg < gemm_bf16_num_cfgs()) ? kCfgs[cfg].name : "?"; }

hipError_t launch_gemm_bf16(const GemmDesc& d, hipStream_t s, int tile_cfg) {
  if (d.M <= 0 || d.N <= 0 || d.K <= 0 || !d.A || !d.B) return hipErrorInvalidValue;
  const unsigned long long a_elems = d.a_kcontig ? (unsigned long long)(d.M - 1) * d.lda + d.K
                                                 : (unsigned long long)(d.K - 1) * d.lda + d.M;
  const unsigned long long b_elems = d.b_kcontig ? (unsigned long long)(d.N - 1) * d.ldb + d.K
                                                 : (unsigned long long)(d.K - 1) * d.ldb + d.N;
  // byte offsets are 32-bit inside the kernel and 0x80000000 marks "out of range"
  if (a_elems * 2 >= 0x7fffffffull || b_elems * 2 >= 0x7fffffffull) return hipErrorInvalidValue;
  if (tile_cfg < 0) {   // a layer with a handful of outputs has its own kernels (gemm_skinny.hip)
    bool taken = false;
    const hipError_t e = launch_gemm_skinny(d, s, &taken);
    if (taken || e != hipSuccess) return e;
  }

  GemmKArgs a;
  a.A = (const unsigned short*)d.A;
  a.B = (const unsigned short*)d.B;
  a.out_z = (unsigned short*)d.out_z;
  a.out_a = (unsigned short*)d.out_a;
  a.out_f32 = d.out_f32;
  a.M = d.M; a.N = d.N; a.K = d.K;
  a.lda = d.lda; a.ldb = d.ldb; a.ldc = d.ldc;
  a.act = d.act;
  a.a_bytes = (unsigned)(a_elems * 2);
  a.b_bytes = (unsigned)(b_elems * 2);
  a.vec_out = (d.N % 4 == 0) && (d.ldc % 4 == 0) && ((uintptr_t)d.out_z % 8 == 0) && ((uintptr_t)d.out_a % 8 == 0) &&
              ((uintptr_t)d.out_f32 % 16 == 0);
  a.kt_per_split = 0;
  a.partial = nullptr;
  a.sgd_master = d.sgd_master;
  a.neg_lr = -d.sgd_lr;
  a.act_lut = (d.act == ACT_GELU && d.out_a) ? (const unsigned short*)d.act_lut : nullptr;
  a.had_s = (const unsigned short*)d.had_s;
  a.had_lut = d.had_s ? d.had_lut : nullptr;
  if (d.had_s) {
    // the fused Hadamard product exists in the dX form only and writes nothing but out_z
    if (!d.a_kcontig || !d.b_kcontig || !d.out_z || d.out_a || d.out_f32 || d.sgd_master) return hipErrorInvalidValue;
    a.vec_out = a.vec_out && ((uintptr_t)d.had_s % 8 == 0);
  }
  const bool sgd = d.sgd_master != nullptr;
  if (sgd) {
    if (d.a_kcontig || d.b_kcontig || !d.out_z) return hipErrorInvalidValue;
    a.out_a = nullptr; a.out_f32 = nullptr; a.act = 0;
    a.vec_out = (d.N % 4 == 0) && (d.ldc % 4 == 0) && ((uintptr_t)d.out_z % 8 == 0) && ((uintptr_t)d.sgd_master % 16 == 0);
  }

  // 16-byte loads need every contiguous run to start on a multiple of 8 elements
  const int a_contig = d.a_kcontig ? d.K : d.M, b_contig = d.b_kcontig ? d.K : d.N;
  const bool aligned = (d.lda % 8 == 0) && (d.ldb % 8 == 0) && (a_contig % 8 == 0) && (b_contig % 8 == 0) &&
                       ((uintptr_t)d.A % 16 == 0) && ((uintptr_t)d.B % 16 == 0);
  const bool both_kc = d.a_kcontig && d.b_kcontig;

  int cfg = tile_cfg;
  if (cfg < 0) {
    // 256x256 tiles when they give (nearly) every CU one; else 128x128 (two workgroups per CU), which
    // measured faster than 64x64 down to a handful of tiles with the direct-to-LDS loop.  Aligned
    // shapes take the direct-to-LDS loop.  Otherwise the register-staged loop; with a k-strided
    // operand it transposes in registers and needs more VGPRs than two waves per SIMD leave, so
    // 256x256 then runs as four waves of 128x128; its 128x128 form needs 64 tiles to beat 64x64.
    const long t256 = (long)((d.M + 255) / 256) * ((d.N + 255) / 256);
    const long t128 = (long)((d.M + 127) / 128) * ((d.N + 127) / 128);
    if (t256 >= 192) cfg = aligned ? 4 : (both_kc ? 0 : 3);
    else if (aligned) cfg = 5;
    else cfg = t128 >= 64 ? 1 : 2;
  }
  if (cfg < 0 || cfg >= gemm_bf16_num_cfgs()) return hipErrorInvalidValue;
  // (with the update in the epilogue the same rule holds: K is cut exactly where the plain product's would be, the
  // partial sums are added in the same order, and the kernel that adds them applies the update)
  if (tile_cfg < 0 && (cfg == 5 || cfg == 1 || cfg == 2)) {
    // small tiles that do not fill the chip and a long reduction: split K over workgroups.  A caller
    // that multiplies a column range of a larger product passes the split count of the whole product,
    // so that every output element is summed in the same order however the columns are cut.
    const int splits = d.splitk_splits >= 0 ? d.splitk_splits : splitk_factor(d.M, d.N, d.K);
    if (splits > 1) {
      const bool fits = d.splitk_scratch && d.splitk_bytes >= (size_t)splits * d.M * d.N * sizeof(float) &&
                        (uintptr_t)d.splitk_scratch % 16 == 0;
      if (fits) {
        const int KT = (d.K + 63) / 64;
        a.kt_per_split = (KT + splits - 1) / splits;
        a.partial = d.splitk_scratch;
      } else if (d.splitk_splits > 1) {
        return hipErrorInvalidValue;   // a forced split count must not silently change the summation order
      }
    }
  }
  // A product with the update in its epilogue and a short reduction is bound by the 10 bytes per weight of that
  // epilogue: 128 x 128 tiles, two workgroups per CU, let one workgroup's main loop run under the other's epilogue
  // (4096 x 4096 outputs over K = 256: 40 us per launch, and the step of eight such layers 0.69 -> 0.64 ms; at K = 1024
  // the larger tile is ahead again).  Every element is summed over k in the same order in both tilings, so the bits
  // do not depend on the choice.
  if (tile_cfg < 0 && sgd && cfg == 4 && d.K <= 512) cfg = 5;
  const bool sgd_in_tile = sgd && a.kt_per_split == 0;   // otherwise the reduction kernel applies it
  if (kCfgs[cfg].kind == 1) {
    if (!aligned) return hipErrorInvalidValue;
    if (sgd_in_tile) return launch_cfg_dl_sgd(cfg, a, s);
    if (d.a_kcontig && d.b_kcontig) return launch_cfg_dl<true, true>(cfg, a, s);
    if (d.a_kcontig && !d.b_kcontig) return launch_cfg_dl<true, false>(cfg, a, s);
    if (!d.a_kcontig && !d.b_kcontig) return launch_cfg_dl<false, false>(cfg, a, s);
    return launch_cfg_dl<false, true>(cfg, a, s);
  }
  if (sgd_in_tile) return aligned ? launch_cfg_sgd<true>(cfg, a, s) : launch_cfg_sgd<false>(cfg, a, s);
  if (aligned) {
    if (d.a_kcontig && d.b_kcontig) return launch_cfg<true, true, true>(cfg, a, s);
    if (d.a_kcontig && !d.b_kcontig) return launch_cfg<true, false, true>(cfg, a, s);
    if (!d.a_kcontig && !d.b_kcontig) return launch_cfg<false, false, true>(cfg, a, s);
    return launch_cfg<false, true, true>(cfg, a, s);
  }
  if (d.a_kcontig && d.b_kcontig) return launch_cfg<true, true, false>(cfg, a, s);
  if (d.a_kcontig && !d.b_kcontig) return launch_cfg<true, false, false>(cfg, a, s);
  if (!d.a_kcontig && !d.b_kcontig) return launch_cfg<false, false, false>(cfg, a, s);
  return launch_cfg<false, true, false>(cfg, a, s);
}

}  // namespace lp
