// 3x3 convolution tasks of a layer with very few input channels (9 * C_in <= 32: the image layer of a
// CNN), Eq. 1 and Eq. 5 as in conv_bf16.hip.  With C_in = 3 a pixel is 6 bytes, so nothing is aligned for
// the 16-byte gathers of the general kernels and their reduction of 27 would sit in a K tile of 64.  Here a
// workgroup copies the contiguous run of pixels it needs (its chunk plus a halo of HP pixels on each side)
// into LDS as it lies in memory, and the MFMA fragments are put together from 2-byte LDS reads:
//
//   F   rows = pixels, k = (tap, c) padded from 9 C_in to 32 (two MFMA k steps), columns = outputs;
//   dW  rows = (tap, c) padded to 32, k = pixels, columns = outputs; a workgroup sums over its chunks,
//       its four waves over quarters of a chunk, and writes one fp32 partial that the caller's
//       fixed-order reduction adds up.
//
// A tap that leaves the image is masked per pixel (9-bit mask), which also covers pixels past the end
// of the tensor and the halo's reach into a neighbouring image.
#include "conv_thin.h"

#include "gemm_core.h"

namespace lp {
namespace {

using namespace core;

constexpr int HP = 40;   // halo pixels per side: >= W + 1, and HP * C * 2 bytes is a multiple of 16 for every C
constexpr int KP = 32;   // 9 * C padded to two k steps of 16

struct ThinArgs {
  const unsigned short* x;     // [B, H, W, C]
  const unsigned short* mat;   // F: w [9 C, Cout]; dW: dy [B, H, W, Cout]
  unsigned short* out_z;
  unsigned short* out_a;
  float* partial;              // dW: [workgroups][9 C][Cout]
  int H, W, Cout, M;           // M = B * H * W pixels
  int act, vec_out, chunks;
  unsigned x_bytes, mat_bytes;
};

// 9-bit mask of the taps of pixel m (flattened (b, y, x)) that stay inside its image; 0 past the end
__device__ __forceinline__ unsigned tap_mask(int m, int M, int H, int W) {
  if (m >= M) return 0u;
  const int t = m / W, x = m - t * W, y = t % H;
  unsigned mask = 0;
#pragma unroll
  for (int tap = 0; tap < 9; ++tap) {
    const int yy = y + tap / 3 - 1, xx = x + tap % 3 - 1;
    if (yy >= 0 && yy < H && xx >= 0 && xx < W) mask |= 1u << tap;
  }
  return mask;
}

__device__ __forceinline__ bf16x8 pack8(const unsigned short (&e)[8]) {
  u32x4 v;
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = (unsigned)e[2 * q] | ((unsigned)e[2 * q + 1] << 16);
  return __builtin_bit_cast(bf16x8, v);
}

// copies the pixels [p0 - HP, p0 + PB + HP) to LDS in 16-byte pieces; pixels outside the tensor read as zeros
// (the buffer's range check works on whole dwords: when the tensor has an odd number of 2-byte elements the
// piece that holds its last element fetches that one again with a 2-byte load)
template <int C, int PB>
__device__ __forceinline__ void stage_patch(__amdgpu_buffer_rsrc_t rs, unsigned x_bytes, int p0, unsigned short* patch) {
  constexpr int NCH = ((PB + 2 * HP) * C * 2 + 15) / 16;
  static_assert(NCH <= 256, "one piece per thread");
  if ((int)threadIdx.x < NCH) {
    const long off = ((long)p0 - HP) * (C * 2) + 16 * (long)threadIdx.x;   // a multiple of 16: p0 % 8 == 0
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off >= 0 ? (unsigned)off : kOOB, 0, 0);
    *reinterpret_cast<u32x4*>(patch + 8 * threadIdx.x) = v;
    const long tail = (long)x_bytes - 2;
    if ((x_bytes & 2u) && off <= tail && tail < off + 16)
      patch[8 * threadIdx.x + (int)(tail - off) / 2] = __builtin_amdgcn_raw_buffer_load_b16(rs, (unsigned)tail, 0, 0);
  }
}

template <int C>
__global__ void __launch_bounds__(256) thin_fwd_kernel(ThinArgs p) {
  constexpr int PB = 256, EP_LD = 72;
  __shared__ __attribute__((aligned(16))) unsigned short patch[((PB + 2 * HP) * C + 7) / 8 * 8];
  __shared__ __attribute__((aligned(16))) unsigned short wl[KP * 64];
  __shared__ __attribute__((aligned(16))) float band[4][32 * EP_LD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, g = lane >> 5;
  const int p0 = blockIdx.x * PB;

  stage_patch<C, PB>(make_rsrc(p.x, p.x_bytes), p.x_bytes, p0, patch);
  {  // weights: k rows padded with zeros to KP, outputs to 64
    const int row = tid >> 3, ch = tid & 7;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (row < 9 * C && ch * 8 < p.Cout)
      v = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc(p.mat, p.mat_bytes), (unsigned)(row * p.Cout + ch * 8) * 2u, 0, 0);
    *reinterpret_cast<u32x4*>(wl + row * 64 + ch * 8) = v;
  }
  // this lane's eight k indices of each k step: element offset inside the patch relative to the pixel, tap bit
  int koff[2][8];
  unsigned kbit[2][8];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int kk = 16 * s + 8 * g + j;
      const int tap = kk / C, c = kk - tap * C;
      const bool valid = kk < 9 * C;
      koff[s][j] = valid ? ((tap / 3 - 1) * p.W + (tap % 3 - 1)) * C + c : 0;
      kbit[s][j] = valid ? 1u << tap : 0u;
    }
  __syncthreads();

  bf16x8 fb[2][2];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn)
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      unsigned short e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) e[j] = wl[(16 * s + 8 * g + j) * 64 + jn * 32 + r];
      fb[jn][s] = pack8(e);
    }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int pl = 64 * wave + 32 * i + r;
    const unsigned mask = tap_mask(p0 + pl, p.M, p.H, p.W);
    const unsigned short* px = patch + (HP + pl) * C;
    bf16x8 fa[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      unsigned short e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const unsigned short v = px[koff[s][j]];
        e[j] = (mask & kbit[s][j]) ? v : (unsigned short)0;
      }
      fa[s] = pack8(e);
    }
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][jn][q] = 0.f;
#pragma unroll
      for (int s = 0; s < 2; ++s) acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s], fb[jn][s], acc[i][jn], 0, 0, 0);
    }
  }

  // through LDS for row-contiguous stores, as in the GEMM epilogue
  StoreEpilogue epi{p.out_z, p.out_a, nullptr, p.M, p.Cout, p.Cout, p.act, p0, 0, p.vec_out != 0};
  float* ep = band[wave];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int q = 0; q < 16; ++q) ep[((q >> 2) * 8 + g * 4 + (q & 3)) * EP_LD + jn * 32 + r] = acc[i][jn][q];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll 4
    for (int e = lane; e < 32 * 16; e += 64) {
      const int row = e / 16, c4 = e % 16;
      const f32x4 v = *reinterpret_cast<const f32x4*>(ep + row * EP_LD + c4 * 4);
      epi(64 * wave + 32 * i + row, c4 * 4, v);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

// dynamic LDS: patch | per-pixel tap masks | dy chunk [PB][64] (later the four waves' partial sums)
template <int C>
__global__ void __launch_bounds__(256) thin_dw_kernel(ThinArgs p) {
  constexpr int PB = 512, PATCH = ((PB + 2 * HP) * C + 7) / 8 * 8;
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  unsigned short* patch = smem;
  unsigned short* pmask = patch + PATCH;
  unsigned short* dyl = pmask + PB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, g = lane >> 5;
  const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.x, p.x_bytes), rs_dy = make_rsrc(p.mat, p.mat_bytes);

  // this lane's row of the result: (tap, c) = r, or nothing for r >= 9 C
  const int tap = r / C, c = r - tap * C;
  const bool row_valid = r < 9 * C;
  const int moff = row_valid ? ((tap / 3 - 1) * p.W + (tap % 3 - 1)) * C + c : 0;
  const unsigned tbit = row_valid ? 1u << tap : 0u;

  f32x16 acc[2];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[jn][q] = 0.f;

  for (int ch = blockIdx.x; ch < p.chunks; ch += gridDim.x) {
    const int p0 = ch * PB;
    __syncthreads();   // the previous chunk has been read
    stage_patch<C, PB>(rs_x, p.x_bytes, p0, patch);
#pragma unroll
    for (int q = 0; q < PB / 256; ++q) pmask[q * 256 + tid] = (unsigned short)tap_mask(p0 + q * 256 + tid, p.M, p.H, p.W);
#pragma unroll 4
    for (int it = 0; it < PB * 8 / 256; ++it) {
      const int idx = it * 256 + tid, px = idx >> 3, ck = idx & 7;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (p0 + px < p.M && ck * 8 < p.Cout)
        v = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, (unsigned)((p0 + px) * p.Cout + ck * 8) * 2u, 0, 0);
      *reinterpret_cast<u32x4*>(dyl + px * 64 + ck * 8) = v;
    }
    __syncthreads();
#pragma unroll 2
    for (int s = 0; s < PB / 4 / 16; ++s) {   // this wave's quarter of the chunk, 16 pixels per MFMA
      const int pk0 = (PB / 4) * wave + 16 * s + 8 * g;
      unsigned short ea[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const unsigned short v = patch[(HP + pk0 + j) * C + moff];
        ea[j] = (pmask[pk0 + j] & tbit) ? v : (unsigned short)0;
      }
      const bf16x8 fa = pack8(ea);
#pragma unroll
      for (int jn = 0; jn < 2; ++jn) {
        unsigned short eb[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) eb[j] = dyl[(pk0 + j) * 64 + jn * 32 + r];
        acc[jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, pack8(eb), acc[jn], 0, 0, 0);
      }
    }
  }

  // the four waves' sums, added in wave order
  __syncthreads();
  float* red = reinterpret_cast<float*>(dyl);
#pragma unroll
  for (int jn = 0; jn < 2; ++jn)
#pragma unroll
    for (int q = 0; q < 16; ++q) red[wave * 2048 + ((q >> 2) * 8 + g * 4 + (q & 3)) * 64 + jn * 32 + r] = acc[jn][q];
  __syncthreads();
  const int n_out = 9 * C * p.Cout;
  float* out = p.partial + (size_t)blockIdx.x * n_out;
  for (int e = tid; e < n_out; e += 256) {
    const int row = e / p.Cout, col = e - row * p.Cout;
    const int o = row * 64 + col;
    out[e] = ((red[o] + red[2048 + o]) + red[4096 + o]) + red[6144 + o];
  }
}

constexpr size_t kDwLds = ((((512 + 2 * HP) * 3 + 7) / 8 * 8) + 512 + 512 * 64) * sizeof(unsigned short);

}  // namespace

bool conv_thin_ok(const ConvDesc& c, const void* x, const void* other) {
  return c.Cin == 3 && c.Cout % 8 == 0 && c.Cout <= 64 && c.W + 1 <= HP && (uintptr_t)x % 16 == 0 && (uintptr_t)other % 16 == 0;
}

hipError_t launch_conv_thin_fwd(const ConvDesc& c, const void* x, const void* w, void* out_z, void* out_a, int act, hipStream_t s) {
  if (!conv_thin_ok(c, x, w)) return hipErrorNotSupported;
  ThinArgs p{};
  p.x = (const unsigned short*)x; p.mat = (const unsigned short*)w;
  p.out_z = (unsigned short*)out_z; p.out_a = (unsigned short*)out_a;
  p.H = c.H; p.W = c.W; p.Cout = c.Cout; p.M = c.B * c.H * c.W;
  p.act = act;
  p.vec_out = ((uintptr_t)out_z % 8 == 0) && ((uintptr_t)out_a % 8 == 0);   // Cout % 8 == 0
  p.x_bytes = (unsigned)((size_t)p.M * c.Cin * 2); p.mat_bytes = (unsigned)((size_t)9 * c.Cin * c.Cout * 2);
  hipLaunchKernelGGL(thin_fwd_kernel<3>, dim3((unsigned)((p.M + 255) / 256)), dim3(256), 0, s, p);
  return hipGetLastError();
}

int conv_thin_dw_chunks(const ConvDesc& c) { return (c.B * c.H * c.W + 511) / 512; }

hipError_t launch_conv_thin_dw(const ConvDesc& c, const void* x, const void* dy, float* partial, int groups, hipStream_t s) {
  if (!conv_thin_ok(c, x, dy) || !partial || groups < 1) return hipErrorNotSupported;
  ThinArgs p{};
  p.x = (const unsigned short*)x; p.mat = (const unsigned short*)dy;
  p.partial = partial;
  p.H = c.H; p.W = c.W; p.Cout = c.Cout; p.M = c.B * c.H * c.W;
  p.chunks = conv_thin_dw_chunks(c);
  p.x_bytes = (unsigned)((size_t)p.M * c.Cin * 2); p.mat_bytes = (unsigned)((size_t)p.M * c.Cout * 2);
  static bool attr = false;
  if (!attr) {
    hipError_t e = hipFuncSetAttribute((const void*)thin_dw_kernel<3>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDwLds);
    if (e != hipSuccess) return e;
    attr = true;
  }
  hipLaunchKernelGGL(thin_dw_kernel<3>, dim3((unsigned)groups), dim3(256), kDwLds, s, p);
  return hipGetLastError();
}

}  // namespace lp
