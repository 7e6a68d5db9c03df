// Bandwidth-bound tasks of the training step: the Hadamard part of Eq. 3 (run in the stage that
// holds Z_l), the error at the output with the last layer's delta, the delayed SGD update of Eq. 6,
// and the max-pool helpers of convolution layers.  All kernels stream 16-byte vectors per lane with
// consecutive lanes on consecutive addresses; row reductions stay inside one 64-lane wavefront.
#include "lp_kernels.h"

#include <mutex>

namespace lp {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned short f2bf(float v) {
  __bf16 b = (__bf16)v;  // round-to-nearest-even
  return __builtin_bit_cast(unsigned short, b);
}
__device__ __forceinline__ float bf2f(unsigned short b) { return __uint_as_float(((unsigned)b) << 16); }

template <int ACT>
__device__ __forceinline__ float act_f(float z) {
  if (ACT == ACT_RELU) return z > 0.f ? z : 0.f;
  if (ACT == ACT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752440f));
  if (ACT == ACT_TANH) return tanhf(z);
  if (ACT == ACT_SIGMOID) return 1.f / (1.f + expf(-z));
  return z;
}
template <int ACT>
__device__ __forceinline__ float act_df(float z) {
  if (ACT == ACT_RELU) return z > 0.f ? 1.f : 0.f;
  if (ACT == ACT_GELU) {
    const float cdf = 0.5f * (1.f + erff(z * 0.70710678118654752440f));
    const float pdf = 0.39894228040143267794f * __expf(-0.5f * z * z);
    return cdf + z * pdf;
  }
  if (ACT == ACT_TANH) { const float t = tanhf(z); return 1.f - t * t; }
  if (ACT == ACT_SIGMOID) { const float s = 1.f / (1.f + expf(-z)); return s * (1.f - s); }
  return 1.f;
}

template <typename T>
struct Elem;
template <>
struct Elem<unsigned short> {
  static __device__ __forceinline__ float ld(unsigned short v) { return bf2f(v); }
  static __device__ __forceinline__ unsigned short st(float v) { return f2bf(v); }
};
template <>
struct Elem<float> {
  static __device__ __forceinline__ float ld(float v) { return v; }
  static __device__ __forceinline__ float st(float v) { return v; }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// sum over a 256-thread block, result valid in every thread; fixed order
__device__ __forceinline__ float block_sum_256(float v, float* sh4) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh4[threadIdx.x >> 6] = v;
  __syncthreads();
  return (sh4[0] + sh4[1]) + (sh4[2] + sh4[3]);
}

// ---- dY = dA (.) f'(S) ---------------------------------------------------------------------------
constexpr int EW_VEC_PER_THREAD = 4;

// ACT_LUT (not an activation of the library): f' is looked up in `lut`, fp32 entries for all 65536 bf16 patterns of S
constexpr int ACT_LUT = 100;
template <int ACT>
__device__ __forceinline__ float act_df_bf16(unsigned short s, const float* __restrict__ lut) {
  if constexpr (ACT == ACT_LUT) return lut[s];
  else return act_df<ACT>(bf2f(s));
}

template <int ACT>
__global__ void __launch_bounds__(256) act_grad_bf16_kernel(const u32x4* __restrict__ dA, const u32x4* __restrict__ S,
                                                            u32x4* __restrict__ dY, size_t nvec, size_t n, const float* __restrict__ lut) {
  const size_t base = (size_t)blockIdx.x * (256 * EW_VEC_PER_THREAD) + threadIdx.x;
  u32x4 a[EW_VEC_PER_THREAD], s[EW_VEC_PER_THREAD];
#pragma unroll
  for (int u = 0; u < EW_VEC_PER_THREAD; ++u) {
    const size_t i = base + (size_t)u * 256;
    if (i < nvec) { a[u] = __builtin_nontemporal_load(dA + i); s[u] = __builtin_nontemporal_load(S + i); }
  }
#pragma unroll
  for (int u = 0; u < EW_VEC_PER_THREAD; ++u) {
    const size_t i = base + (size_t)u * 256;
    if (i < nvec) {
      u32x4 o;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const float a0 = bf2f((unsigned short)(a[u][d] & 0xffffu)), a1 = bf2f((unsigned short)(a[u][d] >> 16));
        const unsigned short s0 = (unsigned short)(s[u][d] & 0xffffu), s1 = (unsigned short)(s[u][d] >> 16);
        o[d] = (unsigned)f2bf(a0 * act_df_bf16<ACT>(s0, lut)) | ((unsigned)f2bf(a1 * act_df_bf16<ACT>(s1, lut)) << 16);
      }
      __builtin_nontemporal_store(o, dY + i);
    }
  }
  // scalar tail (n not a multiple of 8) by the first lanes of block 0
  if (blockIdx.x == 0) {
    const size_t i = nvec * 8 + threadIdx.x;
    if (i < n) {
      const unsigned short* a16 = (const unsigned short*)dA;
      const unsigned short* s16 = (const unsigned short*)S;
      ((unsigned short*)dY)[i] = f2bf(bf2f(a16[i]) * act_df_bf16<ACT>(s16[i], lut));
    }
  }
}

// The GELU form for large tensors.  The look-up of the kernel above is a 4-byte gather per element through the vector
// memory path, which the streaming loads and stores of the same kernel also use: 0.22 ms for 134 M elements, against
// 0.15 ms when f' was computed.  Here one workgroup per CU first copies the part of the table that real pre-activations
// hit (|z| < 16: bit patterns below 0x4180 of either sign, 2 x 16768 floats = 131 KiB) into LDS and then walks the
// tensor with a grid stride; a look-up is an LDS read, anything outside the cached range goes to the table in memory.
// Same table, same product: the bits of the kernel above.
constexpr int LUT_CACHED = 0x4180;
__global__ void __launch_bounds__(1024) act_grad_bf16_lds_lut_kernel(const u32x4* __restrict__ dA, const u32x4* __restrict__ S,
                                                                     u32x4* __restrict__ dY, size_t nvec, size_t n, const float* __restrict__ lut) {
  extern __shared__ float tab[];
  for (int i = threadIdx.x; i < 2 * LUT_CACHED / 4; i += 1024) {
    const int e = i * 4;                                  // LUT_CACHED % 4 == 0: a quad never straddles the two halves
    const int bits = e < LUT_CACHED ? e : 0x8000 + (e - LUT_CACHED);
    *reinterpret_cast<f32x4*>(tab + e) = *reinterpret_cast<const f32x4*>(lut + bits);
  }
  __syncthreads();
  auto df = [&](unsigned short b) -> float {
    const int m = b & 0x7fff;
    return m < LUT_CACHED ? tab[m + (b >> 15) * LUT_CACHED] : lut[b];
  };
  // four 16-byte vectors of each operand in flight per lane: one workgroup per CU has to keep the whole of that CU's
  // share of the memory pipeline busy (128 KiB per CU)
  constexpr int U = 4;
  const size_t stride = (size_t)gridDim.x * 1024;
  for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i < nvec; i += U * stride) {
    u32x4 a[U], sv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t k = i + u * stride;
      if (k < nvec) { a[u] = __builtin_nontemporal_load(dA + k); sv[u] = __builtin_nontemporal_load(S + k); }
      else { a[u] = u32x4{0u, 0u, 0u, 0u}; sv[u] = u32x4{0u, 0u, 0u, 0u}; }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t k = i + u * stride;
      u32x4 o;
#pragma unroll
      for (int d = 0; d < 4; ++d)
        o[d] = (unsigned)f2bf(bf2f((unsigned short)(a[u][d] & 0xffffu)) * df((unsigned short)(sv[u][d] & 0xffffu))) |
               ((unsigned)f2bf(bf2f((unsigned short)(a[u][d] >> 16)) * df((unsigned short)(sv[u][d] >> 16))) << 16);
      if (k < nvec) __builtin_nontemporal_store(o, dY + k);
    }
  }
  if (blockIdx.x == 0) {   // scalar tail (n not a multiple of 8)
    const size_t i = nvec * 8 + threadIdx.x;
    if (i < n) {
      const unsigned short* a16 = (const unsigned short*)dA;
      const unsigned short* s16 = (const unsigned short*)S;
      ((unsigned short*)dY)[i] = f2bf(bf2f(a16[i]) * df(s16[i]));
    }
  }
}

template <int ACT>
__global__ void __launch_bounds__(256) act_grad_f32_kernel(const f32x4* __restrict__ dA, const f32x4* __restrict__ S,
                                                           f32x4* __restrict__ dY, size_t nvec, size_t n) {
  const size_t base = (size_t)blockIdx.x * (256 * EW_VEC_PER_THREAD) + threadIdx.x;
#pragma unroll
  for (int u = 0; u < EW_VEC_PER_THREAD; ++u) {
    const size_t i = base + (size_t)u * 256;
    if (i < nvec) {
      const f32x4 a = dA[i], s = S[i];
      f32x4 o;
#pragma unroll
      for (int d = 0; d < 4; ++d) o[d] = a[d] * act_df<ACT>(s[d]);
      dY[i] = o;
    }
  }
  if (blockIdx.x == 0) {
    const size_t i = nvec * 4 + threadIdx.x;
    if (i < n) ((float*)dY)[i] = ((const float*)dA)[i] * act_df<ACT>(((const float*)S)[i]);
  }
}

// ---- max-pool helpers (NHWC, 2x2 stride 2) -------------------------------------------------------
template <typename T, int ACT>
__global__ void __launch_bounds__(256) relu_pool_kernel(const T* __restrict__ z, T* __restrict__ a, int B, int H, int W, int C) {
  const size_t total = (size_t)B * (H / 2) * (W / 2) * C;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C);
  size_t t = i / C;
  const int x = (int)(t % (W / 2)); t /= (W / 2);
  const int y = (int)(t % (H / 2));
  const int b = (int)(t / (H / 2));
  float best = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const size_t off = (((size_t)b * H + (2 * y + (k >> 1))) * W + (2 * x + (k & 1))) * C + c;
    const float v = Elem<T>::ld(Elem<T>::st(act_f<ACT>(Elem<T>::ld(z[off]))));
    if (k == 0 || v > best) best = v;
  }
  a[i] = Elem<T>::st(best);
}

template <typename T, int ACT>
__global__ void __launch_bounds__(256) act_grad_pool_kernel(const T* __restrict__ dA, const T* __restrict__ Z, T* __restrict__ dY,
                                                            int B, int H, int W, int C) {
  const size_t total = (size_t)B * (H / 2) * (W / 2) * C;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C);
  size_t t = i / C;
  const int x = (int)(t % (W / 2)); t /= (W / 2);
  const int y = (int)(t % (H / 2));
  const int b = (int)(t / (H / 2));
  size_t off[4];
  float zv[4];
  float best = 0.f;
  int arg = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    off[k] = (((size_t)b * H + (2 * y + (k >> 1))) * W + (2 * x + (k & 1))) * C + c;
    zv[k] = Elem<T>::ld(Z[off[k]]);
    const float v = Elem<T>::ld(Elem<T>::st(act_f<ACT>(zv[k])));
    if (k == 0 || v > best) { best = v; arg = k; }   // strict '>' keeps the first maximum
  }
  const float da = Elem<T>::ld(dA[i]);
#pragma unroll
  for (int k = 0; k < 4; ++k) dY[off[k]] = Elem<T>::st(k == arg ? da * act_df<ACT>(zv[k]) : 0.f);
}

// The same two kernels for bf16 tensors whose channel count is a multiple of 8: one lane handles 8 consecutive
// channels of one pooled pixel (16-byte loads and stores, consecutive lanes on consecutive channel groups).
// Element for element the arithmetic of the scalar kernels above.
__device__ __forceinline__ void unpack8(const u32x4& v, float (&f)[8]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) { f[2 * d] = bf2f((unsigned short)(v[d] & 0xffffu)); f[2 * d + 1] = bf2f((unsigned short)(v[d] >> 16)); }
}
__device__ __forceinline__ u32x4 pack8(const float (&f)[8]) {
  u32x4 v;
#pragma unroll
  for (int d = 0; d < 4; ++d) v[d] = (unsigned)f2bf(f[2 * d]) | ((unsigned)f2bf(f[2 * d + 1]) << 16);
  return v;
}

template <int ACT>
__global__ void __launch_bounds__(256) relu_pool_vec8_kernel(const u32x4* __restrict__ z, u32x4* __restrict__ a, int B, int H, int W, int C8) {
  const size_t total = (size_t)B * (H / 2) * (W / 2) * C8;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C8);
  size_t t = i / C8;
  const int x = (int)(t % (W / 2)); t /= (W / 2);
  const int y = (int)(t % (H / 2));
  const int b = (int)(t / (H / 2));
  u32x4 zv[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) zv[k] = z[(((size_t)b * H + (2 * y + (k >> 1))) * W + (2 * x + (k & 1))) * C8 + c];
  float best[8];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float f[8];
    unpack8(zv[k], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float v = bf2f(f2bf(act_f<ACT>(f[e])));
      if (k == 0 || v > best[e]) best[e] = v;
    }
  }
  a[i] = pack8(best);
}

template <int ACT>
__global__ void __launch_bounds__(256) act_grad_pool_vec8_kernel(const u32x4* __restrict__ dA, const u32x4* __restrict__ Z, u32x4* __restrict__ dY,
                                                                 int B, int H, int W, int C8) {
  const size_t total = (size_t)B * (H / 2) * (W / 2) * C8;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C8);
  size_t t = i / C8;
  const int x = (int)(t % (W / 2)); t /= (W / 2);
  const int y = (int)(t % (H / 2));
  const int b = (int)(t / (H / 2));
  size_t off[4];
  float zf[4][8], da[8];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    off[k] = (((size_t)b * H + (2 * y + (k >> 1))) * W + (2 * x + (k & 1))) * C8 + c;
    unpack8(Z[off[k]], zf[k]);
  }
  unpack8(dA[i], da);
  float out[4][8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float best = 0.f;
    int arg = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float v = bf2f(f2bf(act_f<ACT>(zf[k][e])));
      if (k == 0 || v > best) { best = v; arg = k; }   // strict '>' keeps the first maximum
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) out[k][e] = k == arg ? da[e] * act_df<ACT>(zf[k][e]) : 0.f;
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) dY[off[k]] = pack8(out[k]);
}

// ---- loss + delta of the output layer ------------------------------------------------------------
// one wavefront per row
template <typename T>
__global__ void __launch_bounds__(256) softmax_ce_kernel(const T* __restrict__ Z, const int* __restrict__ labels, T* __restrict__ dY,
                                                         float* __restrict__ row_loss, int rows, int cols) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* z = Z + (size_t)row * cols;
  float m = -INFINITY;
  for (int c = lane; c < cols; c += 64) m = fmaxf(m, Elem<T>::ld(z[c]));
  m = wave_max(m);
  float sum = 0.f;
  for (int c = lane; c < cols; c += 64) sum += expf(Elem<T>::ld(z[c]) - m);
  sum = wave_sum(sum);
  const int y = labels[row];
  const bool y_ok = (unsigned)y < (unsigned)cols;   // a label outside the classes is not dereferenced: NaN loss
  const float inv = 1.f / sum, invB = 1.f / (float)rows;
  T* dy = dY + (size_t)row * cols;
  for (int c = lane; c < cols; c += 64) {
    const float p = expf(Elem<T>::ld(z[c]) - m) * inv;
    dy[c] = Elem<T>::st((p - (c == y ? 1.f : 0.f)) * invB);
  }
  if (lane == 0) row_loss[row] = y_ok ? (m + logf(sum)) - Elem<T>::ld(z[y]) : __builtin_nanf("");
}

// The same for rows whose length is a multiple of the 16-byte vector (8 bf16 / 4 floats) and that fit the
// registers of one wavefront (NV vectors per lane): the row is read once, with 16-byte loads, and written once.
template <typename T>
struct Vec16;
template <>
struct Vec16<unsigned short> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const u32x4& v, float* f) {
#pragma unroll
    for (int d = 0; d < 4; ++d) { f[2 * d] = bf2f((unsigned short)(v[d] & 0xffffu)); f[2 * d + 1] = bf2f((unsigned short)(v[d] >> 16)); }
  }
  static __device__ __forceinline__ u32x4 pack(const float* f) {
    u32x4 v;
#pragma unroll
    for (int d = 0; d < 4; ++d) v[d] = (unsigned)f2bf(f[2 * d]) | ((unsigned)f2bf(f[2 * d + 1]) << 16);
    return v;
  }
};
template <>
struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const u32x4& v, float* f) {
#pragma unroll
    for (int d = 0; d < 4; ++d) f[d] = __uint_as_float(v[d]);
  }
  static __device__ __forceinline__ u32x4 pack(const float* f) {
    u32x4 v;
#pragma unroll
    for (int d = 0; d < 4; ++d) v[d] = __float_as_uint(f[d]);
    return v;
  }
};

template <typename T, int NV>
__global__ void __launch_bounds__(256) softmax_ce_rowreg_kernel(const T* __restrict__ Z, const int* __restrict__ labels, T* __restrict__ dY,
                                                                float* __restrict__ row_loss, int rows, int cols) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* zrow = Z + (size_t)row * cols;
  const u32x4* z = reinterpret_cast<const u32x4*>(zrow);
  u32x4* dy = reinterpret_cast<u32x4*>(dY + (size_t)row * cols);
  const int nvec = cols / VN;
  float v[NV][VN];
  float m = -INFINITY;
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int i = lane + 64 * u;
    if (i < nvec) {
      Vec16<T>::unpack(__builtin_nontemporal_load(z + i), v[u]);
#pragma unroll
      for (int e = 0; e < VN; ++e) m = fmaxf(m, v[u][e]);
    }
  }
  m = wave_max(m);
  float sum = 0.f;
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    if (lane + 64 * u < nvec) {
#pragma unroll
      for (int e = 0; e < VN; ++e) { v[u][e] = expf(v[u][e] - m); sum += v[u][e]; }
    }
  }
  sum = wave_sum(sum);
  const int y = labels[row];
  const bool y_ok = (unsigned)y < (unsigned)cols;
  const float inv = 1.f / sum, invB = 1.f / (float)rows;
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int i = lane + 64 * u;
    if (i < nvec) {
      float o[VN];
#pragma unroll
      for (int e = 0; e < VN; ++e) o[e] = (v[u][e] * inv - (i * VN + e == y ? 1.f : 0.f)) * invB;
      __builtin_nontemporal_store(Vec16<T>::pack(o), dy + i);
    }
  }
  if (lane == 0) row_loss[row] = y_ok ? (m + logf(sum)) - Elem<T>::ld(zrow[y]) : __builtin_nanf("");
}

constexpr int MSE_PER_BLOCK = 8192;

// Each block handles MSE_PER_BLOCK consecutive elements with 16-byte vectors per lane (the loads of a lane are all
// issued before its arithmetic) and writes one partial sum of squared differences.
template <typename T>
__global__ void __launch_bounds__(256) mse_kernel(const T* __restrict__ Z, const T* __restrict__ Tg, T* __restrict__ dY,
                                                  float* __restrict__ partial, size_t n, float scale) {
  constexpr int VN = Vec16<T>::N;
  constexpr int UNROLL = MSE_PER_BLOCK / (256 * VN);
  __shared__ float sh4[4];
  const u32x4* z = reinterpret_cast<const u32x4*>(Z);
  const u32x4* tg = reinterpret_cast<const u32x4*>(Tg);
  u32x4* dy = reinterpret_cast<u32x4*>(dY);
  const size_t v0 = (size_t)blockIdx.x * (MSE_PER_BLOCK / VN) + threadIdx.x;
  const size_t nvec = n / VN;
  u32x4 zv[UNROLL], tv[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const size_t i = v0 + (size_t)u * 256;
    if (i < nvec) { zv[u] = __builtin_nontemporal_load(z + i); tv[u] = __builtin_nontemporal_load(tg + i); }
  }
  float acc = 0.f;
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const size_t i = v0 + (size_t)u * 256;
    if (i < nvec) {
      float a[VN], b[VN], o[VN];
      Vec16<T>::unpack(zv[u], a);
      Vec16<T>::unpack(tv[u], b);
#pragma unroll
      for (int e = 0; e < VN; ++e) {
        const float d = a[e] - b[e];
        acc += d * d;
        o[e] = d * scale;
      }
      __builtin_nontemporal_store(Vec16<T>::pack(o), dy + i);
    }
  }
  // the last elements of a tensor whose size is not a multiple of the vector: the block that owns them, one per lane
  const size_t tail = nvec * VN + threadIdx.x;
  if (tail < n && tail / MSE_PER_BLOCK == blockIdx.x) {
    const float d = Elem<T>::ld(Z[tail]) - Elem<T>::ld(Tg[tail]);
    acc += d * d;
    dY[tail] = Elem<T>::st(d * scale);
  }
  acc = block_sum_256(acc, sh4);
  if (threadIdx.x == 0) partial[blockIdx.x] = acc;
}

// loss = scale * sum(partials), fixed summation order
__global__ void __launch_bounds__(256) finalize_loss_kernel(const float* __restrict__ partial, size_t count, float scale,
                                                            float* __restrict__ loss) {
  __shared__ float sh4[4];
  float acc = 0.f;
  for (size_t i = threadIdx.x; i < count; i += 256) acc += partial[i];
  acc = block_sum_256(acc, sh4);
  if (threadIdx.x == 0) *loss = acc * scale;
}

// ---- Eq. 6 -----------------------------------------------------------------------------------------
template <bool BF16>
__global__ void __launch_bounds__(256) sgd_kernel(f32x4* __restrict__ master, const f32x4* __restrict__ g, u32x2* __restrict__ work,
                                                  float neg_lr, size_t nvec, size_t n) {
  const size_t base = (size_t)blockIdx.x * (256 * EW_VEC_PER_THREAD) + threadIdx.x;
  f32x4 w[EW_VEC_PER_THREAD], gg[EW_VEC_PER_THREAD];
#pragma unroll
  for (int u = 0; u < EW_VEC_PER_THREAD; ++u) {
    const size_t i = base + (size_t)u * 256;
    if (i < nvec) { gg[u] = __builtin_nontemporal_load(g + i); w[u] = master[i]; }
  }
#pragma unroll
  for (int u = 0; u < EW_VEC_PER_THREAD; ++u) {
    const size_t i = base + (size_t)u * 256;
    if (i < nvec) {
      f32x4 o;
#pragma unroll
      for (int d = 0; d < 4; ++d) o[d] = fmaf(neg_lr, gg[u][d], w[u][d]);
      // streaming stores: neither copy is read again before the next step
      __builtin_nontemporal_store(o, master + i);
      if (BF16) {
        u32x2 b;
        b[0] = (unsigned)f2bf(o[0]) | ((unsigned)f2bf(o[1]) << 16);
        b[1] = (unsigned)f2bf(o[2]) | ((unsigned)f2bf(o[3]) << 16);
        __builtin_nontemporal_store(b, work + i);
      }
    }
  }
  if (blockIdx.x == 0) {
    const size_t i = nvec * 4 + threadIdx.x;
    if (i < n) {
      float* m = (float*)master;
      const float o = fmaf(neg_lr, ((const float*)g)[i], m[i]);
      m[i] = o;
      if (BF16) ((unsigned short*)work)[i] = f2bf(o);
    }
  }
}

// Copies two buffers in one launch (the two factors of a gradient, into their ring slot).  16 bytes per
// lane; a buffer whose size is not a multiple of 16 ends with a byte-wise tail.
__global__ void __launch_bounds__(256) copy2_kernel(const u32x4* __restrict__ a, u32x4* __restrict__ da, size_t va, size_t a_bytes,
                                                    const u32x4* __restrict__ b, u32x4* __restrict__ db, size_t vb, size_t b_bytes) {
  const size_t base = (size_t)blockIdx.x * (256 * EW_VEC_PER_THREAD) + threadIdx.x;
#pragma unroll
  for (int u = 0; u < EW_VEC_PER_THREAD; ++u) {
    size_t i = base + (size_t)u * 256;
    const u32x4* src = a; u32x4* dst = da; size_t bytes = a_bytes;
    if (i >= va) { i -= va; src = b; dst = db; bytes = b_bytes; if (i >= vb) continue; }
    if ((i + 1) * 16 <= bytes) {
      __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
    } else {
      for (size_t k = i * 16; k < bytes; ++k) ((unsigned char*)dst)[k] = ((const unsigned char*)src)[k];
    }
  }
}

__global__ void __launch_bounds__(256) cast_bf16_kernel(const float* __restrict__ src, unsigned short* __restrict__ dst, size_t n) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i + 3 < n) {
    const f32x4 v = *(const f32x4*)(src + i);
    u32x2 b;
    b[0] = (unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16);
    b[1] = (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16);
    *(u32x2*)(dst + i) = b;
  } else {
    for (size_t j = i; j < n; ++j) dst[j] = f2bf(src[j]);
  }
}

inline unsigned blocks_for(size_t items, size_t per_block) { return (unsigned)((items + per_block - 1) / per_block); }

}  // namespace

hipError_t launch_act_grad(bool bf16, int act, const void* dA, const void* S, void* dY, size_t n, hipStream_t s, const float* gelu_grad_lut) {
  if (n == 0) return hipSuccess;
  if (act == ACT_IDENTITY) {
    if (dA == dY) return hipSuccess;
    return hipMemcpyAsync(dY, dA, n * (bf16 ? 2 : 4), hipMemcpyDeviceToDevice, s);
  }
  const size_t per = bf16 ? 8 : 4, nvec = n / per;
  const unsigned nb = blocks_for(nvec > 0 ? nvec : 1, 256 * EW_VEC_PER_THREAD);
  if (bf16) {
    const float* no_lut = nullptr;
    if (act == ACT_RELU) hipLaunchKernelGGL(act_grad_bf16_kernel<ACT_RELU>, dim3(nb), dim3(256), 0, s, (const u32x4*)dA, (const u32x4*)S, (u32x4*)dY, nvec, n, no_lut);
    else if (act == ACT_GELU && gelu_grad_lut && n >= ((size_t)1 << 22)) {
      // large tensors: the table's live part in LDS, one workgroup of 1024 lanes per CU
      constexpr int lds = 2 * LUT_CACHED * (int)sizeof(float);
      struct Setup { hipError_t err; int cus; };
      static const Setup setup = [] {          // once per process (one GPU per process)
        Setup u{hipSuccess, 0};
        int dev = 0;
        u.err = hipGetDevice(&dev);
        if (u.err == hipSuccess) u.err = hipDeviceGetAttribute(&u.cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (u.err == hipSuccess) u.err = hipFuncSetAttribute((const void*)act_grad_bf16_lds_lut_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (u.cus < 1) u.cus = 256;
        return u;
      }();
      if (setup.err != hipSuccess) return setup.err;
      const int cus = setup.cus;
      hipLaunchKernelGGL(act_grad_bf16_lds_lut_kernel, dim3((unsigned)cus), dim3(1024), lds, s, (const u32x4*)dA, (const u32x4*)S, (u32x4*)dY, nvec, n, gelu_grad_lut);
    }
    else if (act == ACT_GELU && gelu_grad_lut) hipLaunchKernelGGL(act_grad_bf16_kernel<ACT_LUT>, dim3(nb), dim3(256), 0, s, (const u32x4*)dA, (const u32x4*)S, (u32x4*)dY, nvec, n, gelu_grad_lut);
    else if (act == ACT_GELU) hipLaunchKernelGGL(act_grad_bf16_kernel<ACT_GELU>, dim3(nb), dim3(256), 0, s, (const u32x4*)dA, (const u32x4*)S, (u32x4*)dY, nvec, n, no_lut);
    else if (act == ACT_TANH) hipLaunchKernelGGL(act_grad_bf16_kernel<ACT_TANH>, dim3(nb), dim3(256), 0, s, (const u32x4*)dA, (const u32x4*)S, (u32x4*)dY, nvec, n, no_lut);
    else if (act == ACT_SIGMOID) hipLaunchKernelGGL(act_grad_bf16_kernel<ACT_SIGMOID>, dim3(nb), dim3(256), 0, s, (const u32x4*)dA, (const u32x4*)S, (u32x4*)dY, nvec, n, no_lut);
    else return hipErrorInvalidValue;
  } else {
    if (act == ACT_RELU) hipLaunchKernelGGL(act_grad_f32_kernel<ACT_RELU>, dim3(nb), dim3(256), 0, s, (const f32x4*)dA, (const f32x4*)S, (f32x4*)dY, nvec, n);
    else if (act == ACT_GELU) hipLaunchKernelGGL(act_grad_f32_kernel<ACT_GELU>, dim3(nb), dim3(256), 0, s, (const f32x4*)dA, (const f32x4*)S, (f32x4*)dY, nvec, n);
    else if (act == ACT_TANH) hipLaunchKernelGGL(act_grad_f32_kernel<ACT_TANH>, dim3(nb), dim3(256), 0, s, (const f32x4*)dA, (const f32x4*)S, (f32x4*)dY, nvec, n);
    else if (act == ACT_SIGMOID) hipLaunchKernelGGL(act_grad_f32_kernel<ACT_SIGMOID>, dim3(nb), dim3(256), 0, s, (const f32x4*)dA, (const f32x4*)S, (f32x4*)dY, nvec, n);
    else return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename T>
static hipError_t relu_pool_t(const void* z, void* a, int B, int H, int W, int C, int act, hipStream_t s) {
  const size_t total = (size_t)B * (H / 2) * (W / 2) * C;
  const unsigned nb = blocks_for(total, 256);
  if (act == ACT_RELU) hipLaunchKernelGGL((relu_pool_kernel<T, ACT_RELU>), dim3(nb), dim3(256), 0, s, (const T*)z, (T*)a, B, H, W, C);
  else if (act == ACT_GELU) hipLaunchKernelGGL((relu_pool_kernel<T, ACT_GELU>), dim3(nb), dim3(256), 0, s, (const T*)z, (T*)a, B, H, W, C);
  else hipLaunchKernelGGL((relu_pool_kernel<T, ACT_IDENTITY>), dim3(nb), dim3(256), 0, s, (const T*)z, (T*)a, B, H, W, C);
  return hipGetLastError();
}
hipError_t launch_relu_pool(bool bf16, const void* z, void* a, int B, int H, int W, int C, int act, hipStream_t s) {
  if (bf16 && C % 8 == 0 && (uintptr_t)z % 16 == 0 && (uintptr_t)a % 16 == 0) {
    const size_t total = (size_t)B * (H / 2) * (W / 2) * (C / 8);
    const unsigned nb = blocks_for(total, 256);
    if (act == ACT_RELU) hipLaunchKernelGGL(relu_pool_vec8_kernel<ACT_RELU>, dim3(nb), dim3(256), 0, s, (const u32x4*)z, (u32x4*)a, B, H, W, C / 8);
    else if (act == ACT_GELU) hipLaunchKernelGGL(relu_pool_vec8_kernel<ACT_GELU>, dim3(nb), dim3(256), 0, s, (const u32x4*)z, (u32x4*)a, B, H, W, C / 8);
    else hipLaunchKernelGGL(relu_pool_vec8_kernel<ACT_IDENTITY>, dim3(nb), dim3(256), 0, s, (const u32x4*)z, (u32x4*)a, B, H, W, C / 8);
    return hipGetLastError();
  }
  return bf16 ? relu_pool_t<unsigned short>(z, a, B, H, W, C, act, s) : relu_pool_t<float>(z, a, B, H, W, C, act, s);
}

template <typename T>
static hipError_t act_grad_pool_t(int act, const void* dA, const void* Z, void* dY, int B, int H, int W, int C, hipStream_t s) {
  const size_t total = (size_t)B * (H / 2) * (W / 2) * C;
  const unsigned nb = blocks_for(total, 256);
  if (act == ACT_RELU) hipLaunchKernelGGL((act_grad_pool_kernel<T, ACT_RELU>), dim3(nb), dim3(256), 0, s, (const T*)dA, (const T*)Z, (T*)dY, B, H, W, C);
  else if (act == ACT_GELU) hipLaunchKernelGGL((act_grad_pool_kernel<T, ACT_GELU>), dim3(nb), dim3(256), 0, s, (const T*)dA, (const T*)Z, (T*)dY, B, H, W, C);
  else hipLaunchKernelGGL((act_grad_pool_kernel<T, ACT_IDENTITY>), dim3(nb), dim3(256), 0, s, (const T*)dA, (const T*)Z, (T*)dY, B, H, W, C);
  return hipGetLastError();
}
hipError_t launch_act_grad_pool(bool bf16, int act, const void* dA, const void* Z, void* dY, int B, int H, int W, int C, hipStream_t s) {
  if (bf16 && C % 8 == 0 && (uintptr_t)dA % 16 == 0 && (uintptr_t)Z % 16 == 0 && (uintptr_t)dY % 16 == 0) {
    const size_t total = (size_t)B * (H / 2) * (W / 2) * (C / 8);
    const unsigned nb = blocks_for(total, 256);
    if (act == ACT_RELU) hipLaunchKernelGGL(act_grad_pool_vec8_kernel<ACT_RELU>, dim3(nb), dim3(256), 0, s, (const u32x4*)dA, (const u32x4*)Z, (u32x4*)dY, B, H, W, C / 8);
    else if (act == ACT_GELU) hipLaunchKernelGGL(act_grad_pool_vec8_kernel<ACT_GELU>, dim3(nb), dim3(256), 0, s, (const u32x4*)dA, (const u32x4*)Z, (u32x4*)dY, B, H, W, C / 8);
    else hipLaunchKernelGGL(act_grad_pool_vec8_kernel<ACT_IDENTITY>, dim3(nb), dim3(256), 0, s, (const u32x4*)dA, (const u32x4*)Z, (u32x4*)dY, B, H, W, C / 8);
    return hipGetLastError();
  }
  return bf16 ? act_grad_pool_t<unsigned short>(act, dA, Z, dY, B, H, W, C, s) : act_grad_pool_t<float>(act, dA, Z, dY, B, H, W, C, s);
}

size_t loss_partials_count(int loss_is_mse, int rows, int cols) {
  if (!loss_is_mse) return (size_t)rows;
  return ((size_t)rows * cols + MSE_PER_BLOCK - 1) / MSE_PER_BLOCK;
}

template <typename T>
static hipError_t softmax_ce_t(const void* Z, const int* labels, void* dY, float* partials, int rows, int cols, hipStream_t s) {
  constexpr int VN = 16 / (int)sizeof(T);
  const unsigned nb = (unsigned)((rows + 3) / 4);
  const bool vec = cols % VN == 0 && cols / VN <= 64 * 8 && (uintptr_t)Z % 16 == 0 && (uintptr_t)dY % 16 == 0;
  const int nv = vec ? (cols / VN + 63) / 64 : 0;   // vectors per lane
#define LP_CE(NV) hipLaunchKernelGGL((softmax_ce_rowreg_kernel<T, NV>), dim3(nb), dim3(256), 0, s, (const T*)Z, labels, (T*)dY, partials, rows, cols)
  if (nv == 1) LP_CE(1);
  else if (nv == 2) LP_CE(2);
  else if (nv >= 3 && nv <= 4) LP_CE(4);
  else if (nv >= 5 && nv <= 8) LP_CE(8);
  else hipLaunchKernelGGL(softmax_ce_kernel<T>, dim3(nb), dim3(256), 0, s, (const T*)Z, labels, (T*)dY, partials, rows, cols);
#undef LP_CE
  return hipGetLastError();
}

hipError_t launch_softmax_ce(bool bf16, const void* Z, const int* labels, void* dY, float* loss, float* partials, int rows, int cols, hipStream_t s) {
  hipError_t e = bf16 ? softmax_ce_t<unsigned short>(Z, labels, dY, partials, rows, cols, s) : softmax_ce_t<float>(Z, labels, dY, partials, rows, cols, s);
  if (e != hipSuccess || !loss) return e;
  hipLaunchKernelGGL(finalize_loss_kernel, dim3(1), dim3(256), 0, s, (const float*)partials, (size_t)rows, 1.f / (float)rows, loss);
  return hipGetLastError();
}

hipError_t launch_mse(bool bf16, const void* Z, const void* T, void* dY, float* loss, float* partials, int rows, int cols, hipStream_t s) {
  const size_t n = (size_t)rows * cols;
  const unsigned nb = (unsigned)loss_partials_count(1, rows, cols);
  const float scale = 2.f / (float)n;
  if (bf16) hipLaunchKernelGGL(mse_kernel<unsigned short>, dim3(nb), dim3(256), 0, s, (const unsigned short*)Z, (const unsigned short*)T, (unsigned short*)dY, partials, n, scale);
  else hipLaunchKernelGGL(mse_kernel<float>, dim3(nb), dim3(256), 0, s, (const float*)Z, (const float*)T, (float*)dY, partials, n, scale);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !loss) return e;
  hipLaunchKernelGGL(finalize_loss_kernel, dim3(1), dim3(256), 0, s, (const float*)partials, (size_t)nb, 1.f / (float)n, loss);
  return hipGetLastError();
}

// ---- loss partials for callers that cannot allocate ------------------------------------------------
// The partial sums of the loss kernels normally live in the caller's workspace.  This array is the same
// scratch inside the library's own image: every GPU the library runs on holds one copy (256 KiB) until the
// process ends.  In host code its name is only a handle; the device address is asked for once per device.
namespace {
constexpr size_t kStaticLossPartials = 65536;
static __device__ __align__(256) float scratch[kStaticLossPartials];
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
float* scratch_ptr[kMaxDevices] = {};
}  // namespace

size_t static_loss_partials_capacity() { return kStaticLossPartials; }

hipError_t static_loss_partials(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the copy of the device that is current
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = scratch_ptr[dev];
  return hipSuccess;
}

hipError_t launch_sgd(float* master, const float* g, void* work_out_bf16, float lr, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const size_t nvec = n / 4;
  const unsigned nb = blocks_for(nvec > 0 ? nvec : 1, 256 * EW_VEC_PER_THREAD);
  if (work_out_bf16) hipLaunchKernelGGL(sgd_kernel<true>, dim3(nb), dim3(256), 0, s, (f32x4*)master, (const f32x4*)g, (u32x2*)work_out_bf16, -lr, nvec, n);
  else hipLaunchKernelGGL(sgd_kernel<false>, dim3(nb), dim3(256), 0, s, (f32x4*)master, (const f32x4*)g, (u32x2*)nullptr, -lr, nvec, n);
  return hipGetLastError();
}

hipError_t launch_copy2(const void* a, void* da, size_t a_bytes, const void* b, void* db, size_t b_bytes, hipStream_t s) {
  // all four pointers 16-byte aligned (workspace blocks and tensors of the library are)
  const size_t va = (a_bytes + 15) / 16, vb = (b_bytes + 15) / 16;
  if (va + vb == 0) return hipSuccess;
  hipLaunchKernelGGL(copy2_kernel, dim3(blocks_for(va + vb, 256 * EW_VEC_PER_THREAD)), dim3(256), 0, s, (const u32x4*)a, (u32x4*)da, va,
                     a_bytes, (const u32x4*)b, (u32x4*)db, vb, b_bytes);
  return hipGetLastError();
}

hipError_t launch_cast_bf16(const float* src, void* dst_bf16, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(cast_bf16_kernel, dim3(blocks_for(n, 1024)), dim3(256), 0, s, src, (unsigned short*)dst_bf16, n);
  return hipGetLastError();
}

}  // namespace lp
