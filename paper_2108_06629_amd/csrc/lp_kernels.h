// Internal launch interface between the C-ABI layer (lp_api.cpp) and the HIP kernels.
// Not part of the public boundary; see include/lp.h for that.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lp {

enum Act { ACT_IDENTITY = 0, ACT_RELU = 1, ACT_GELU = 2, ACT_TANH = 3, ACT_SIGMOID = 4 };

// C[M,N] = sum_k Aop(m,k) * Bop(n,k), fp32 accumulate.
//   a_kcontig:  Aop(m,k) = A[m*lda + k]   else  Aop(m,k) = A[k*lda + m]
//   b_kcontig:  Bop(n,k) = B[n*ldb + k]   else  Bop(n,k) = B[k*ldb + n]
// Outputs (any may be null): out_z = C rounded to the act type; out_a = act(out_z value) in the act
// type; out_f32 = C as float.  All outputs share ldc.
struct GemmDesc {
  const void* A = nullptr;
  const void* B = nullptr;
  int M = 0, N = 0, K = 0;
  int lda = 0, ldb = 0, ldc = 0;
  bool a_kcontig = true, b_kcontig = true;
  void* out_z = nullptr;
  void* out_a = nullptr;
  float* out_f32 = nullptr;
  int act = ACT_IDENTITY;
  // optional scratch for split-K partial sums (fp32); the launcher splits K when the output has too
  // few tiles to occupy the chip and the scratch is large enough
  float* splitk_scratch = nullptr;
  size_t splitk_bytes = 0;
  // < 0: the launcher decides from this product's shape; >= 1: exactly this many K ranges (1: none).
  // A column range of a larger product passes the count of the whole product so that the summation
  // order of an output element does not depend on how the columns are cut.
  int splitk_splits = -1;
  // fused delayed update (only with a_kcontig == b_kcontig == false, the G product): instead of storing
  // G, apply W <- W - lr G to sgd_master (fp32, [M][N] with ldc) and write the bf16 copy of the result
  // to out_z.  out_a, out_f32 and act are ignored; K is never split.
  float* sgd_master = nullptr;
  float sgd_lr = 0.f;
  // optional, for act == ACT_GELU with out_a: the table gelu_lut_bf16 returns; A is then looked up, not computed
  const void* act_lut = nullptr;
  // optional, dX form (both operands k contiguous) with out_z only: the product is dA of the preceding layer and
  // had_s that layer's stash, laid out like out_z (same ldc); out_z then receives dY = q(q(dA) * f'(S)) (Eq. 3),
  // bit for bit what launch_act_grad makes of the stored dA.  f' = [S > 0] (ReLU; S may be A or Z), or, with
  // had_lut (the table gelu_grad_lut_f32 returns), the GELU derivative of S = Z.
  const void* had_s = nullptr;
  const float* had_lut = nullptr;
};
// Device address of GELU(z) for all 65536 bfloat16 bit patterns z (bf16 entries; a static array of the library,
// one copy per GPU).  The first call on a device fills it with a kernel on `s` and waits for it: not under capture.
hipError_t gelu_lut_bf16(const void** out, hipStream_t s);
// The same for the derivative: Phi(z) + z phi(z) as fp32, the factor of the Hadamard product of a GELU layer.
hipError_t gelu_grad_lut_f32(const float** out, hipStream_t s);
// K ranges the launcher cuts a product of this shape into (1: not split), and the scratch that takes
// (0: split-K would not be used)
int gemm_bf16_splitk_splits(int M, int N, int K);
size_t gemm_bf16_splitk_bytes(int M, int N, int K);

// tile_cfg < 0: pick by problem size.  Returns hipErrorInvalidValue for impossible shapes.
hipError_t launch_gemm_bf16(const GemmDesc& d, hipStream_t s, int tile_cfg = -1);
hipError_t launch_gemm_f32(const GemmDesc& d, hipStream_t s);
// Layers with at most 16 outputs (d_in a multiple of 8, batch <= 2048) run their three products on short vector
// kernels instead of MFMA tiles; launch_gemm_bf16 goes there by itself.  gemm_skinny_shape tells which layers those are
// (their summation order differs from the tiled kernels', which matters to whoever promises equal bits).
bool gemm_skinny_shape(int batch, int d_in, int d_out);
hipError_t launch_gemm_skinny(const GemmDesc& d, hipStream_t s, bool* taken);
int gemm_bf16_num_cfgs();
const char* gemm_bf16_cfg_name(int cfg);

// 3x3 stride-1 pad-1 convolution tasks as implicit GEMMs over NHWC bf16 tensors.
struct ConvDesc {
  int B = 0, H = 0, W = 0, Cin = 0, Cout = 0;
};
// F: z[b,y,x,o] = sum xpad[b,y+kh,x+kw,c] w[kh,kw,c,o]; writes out_z and/or out_a=act(z) (full res).
// pooled_a / pooled_done (optional, with out_z and without out_a): the caller wants a[b,y/2,x/2,o] = max over the 2x2
// window of relu(z) as well; *pooled_done says whether this launch wrote it (the pixel-halo form of a ReLU layer whose
// tiles hold whole image row pairs does), otherwise launch_relu_pool is still to be called.
hipError_t launch_conv_fwd(const ConvDesc& c, bool bf16, const void* x, const void* w, void* out_z, void* out_a,
                           int act, hipStream_t s, void* pooled_a = nullptr, bool* pooled_done = nullptr);
// dX: dx[b,y,x,c] for c in [c0,c1) (dx has Cin channels).  had_s (optional): stash of the layer below, [b,y,x,Cin]
// like dx; dx then receives dY of that layer, q(q(dA) * f'(S)), as GemmDesc::had_s does for a fully connected layer
// (f' = [S > 0], or looked up in had_lut).  had_pooled: the layer below is a 2x2 max-pooled ReLU layer; had_s is then
// its full-resolution Z [b,2H,2W,Cin] and dx its full-resolution dY: each element of this product goes to the first
// maximum of its window (times [z > 0]), the other three pixels get 0, as launch_act_grad_pool routes a stored dA.
hipError_t launch_conv_grad_act(const ConvDesc& c, bool bf16, const void* dy, const void* w, void* dx, int c0, int c1,
                                hipStream_t s, const void* had_s = nullptr, const float* had_lut = nullptr, bool had_pooled = false);
// dW: g[kh,kw,c,o] fp32.  `partial` is scratch of conv_grad_weight_scratch_bytes().
// sgd_master (with g == nullptr; only where that scratch is non-empty, i.e. the product is split over K): the gradient is
// not stored but applied, w <- fma(-sgd_lr, g, w) on the fp32 master, and the bf16 copy of the result goes to sgd_work.
hipError_t launch_conv_grad_weight(const ConvDesc& c, bool bf16, const void* x, const void* dy, float* g,
                                   float* partial, hipStream_t s, float* sgd_master = nullptr, void* sgd_work = nullptr, float sgd_lr = 0.f);
size_t conv_grad_weight_scratch_bytes(const ConvDesc& c);

// dY = dA (.) f'(S), n elements.
// gelu_grad_lut (bf16 GELU only, optional): the table gelu_grad_lut_f32 returns; f' is then looked up, not computed
hipError_t launch_act_grad(bool bf16, int act, const void* dA, const void* S, void* dY, size_t n, hipStream_t s, const float* gelu_grad_lut = nullptr);
// pooled conv layer: a[b,y/2,x/2,c] = max over window of relu(z)
hipError_t launch_relu_pool(bool bf16, const void* z, void* a, int B, int H, int W, int C, int act, hipStream_t s);
// pooled conv layer backward: dy (full res) from da (pooled) and z (full res)
hipError_t launch_act_grad_pool(bool bf16, int act, const void* dA, const void* Z, void* dY, int B, int H, int W, int C,
                                hipStream_t s);

// loss + delta of the last layer.  partials: float scratch with >= loss_partials_count() entries.
size_t loss_partials_count(int loss_is_mse, int rows, int cols);
hipError_t launch_softmax_ce(bool bf16, const void* Z, const int* labels, void* dY, float* loss, float* partials,
                             int rows, int cols, hipStream_t s);
hipError_t launch_mse(bool bf16, const void* Z, const void* T, void* dY, float* loss, float* partials, int rows,
                      int cols, hipStream_t s);

// The same scratch as a static device array of the library (one copy per GPU): its device address on the current
// device (looked up on the first call per device) and its capacity in floats.
hipError_t static_loss_partials(float** out);
size_t static_loss_partials_capacity();

// master <- master - lr * g;  work_out (bf16, may be null) <- round(master)
hipError_t launch_sgd(float* master, const float* g, void* work_out_bf16, float lr, size_t n, hipStream_t s);
// dst_bf16 <- round(src)
// measurement aid: workgroups x 8 waves x iters x 8 MFMAs of 32 x 32 x 16 (65536 flop each wave-wide); out: workgroups * 512 floats
hipError_t launch_mfma_only(float* out, int workgroups, int iters, bool uniform_values, hipStream_t s);
hipError_t launch_cast_bf16(const float* src, void* dst_bf16, size_t n, hipStream_t s);
// two device-to-device copies in one launch; every pointer 16-byte aligned
hipError_t launch_copy2(const void* a, void* da, size_t a_bytes, const void* b, void* db, size_t b_bytes, hipStream_t s);

}  // namespace lp
