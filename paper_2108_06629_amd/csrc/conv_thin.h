// Convolution tasks of a layer with three input channels (conv_thin.hip); used by the dispatch in conv_bf16.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "lp_kernels.h"

namespace lp {

// C_in == 3, C_out a multiple of 8 and at most 64, rows short enough for the halo, 16-byte aligned operands
bool conv_thin_ok(const ConvDesc& c, const void* x, const void* other);
// F (Eq. 1): writes out_z and/or out_a = act(z); hipErrorNotSupported when conv_thin_ok is false
hipError_t launch_conv_thin_fwd(const ConvDesc& c, const void* x, const void* w, void* out_z, void* out_a, int act, hipStream_t s);
// dW (Eq. 5): `groups` workgroups (at most conv_thin_dw_chunks) each write one fp32 partial [9 C_in][C_out] to
// partial[group]; the caller adds the partials up
int conv_thin_dw_chunks(const ConvDesc& c);
hipError_t launch_conv_thin_dw(const ConvDesc& c, const void* x, const void* dy, float* partial, int groups, hipStream_t s);

}  // namespace lp
