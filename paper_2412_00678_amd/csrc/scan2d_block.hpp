// Layers around the scan (producers of its inputs inside a 2DMamba block, Sec. 3.2, Fig. 2; the aggregator behind the
// last block, Supp. A): host-side entries used by the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include "../../include/scan2d.h"

namespace scan2d {

// Depth-wise convolution + SiLU; SCAN2D_ERR_BAD_SHAPE for a filter shape outside the documented range.
int block_conv_silu_launch(const scan2d_desc* d, const scan2d_conv_shape* cs, const void* u, const float* w, const float* bias,
                           void* x, hipStream_t stream);

// Step, B and C projections; SCAN2D_ERR_BAD_SHAPE when R, Dc or R + 2N are outside the documented range.
int block_xproj_launch(const scan2d_desc* d, int R, const void* x, const void* Wx, const float* Wdt, void* delta_raw, void* Bm,
                       void* Cm, hipStream_t stream);

// Attention pooling of the aggregator (scan2d_pool.hip); SCAN2D_ERR_BAD_SHAPE when D is outside 1..128 or Bt above 65535.
int block_attn_pool_launch(const scan2d_desc* d, int D, const void* h, const void* V, const float* w, const uint8_t* mask,
                           float* attn, float* z, hipStream_t stream);

// Linear layer at every position of a channel-major map (scan2d_linear.hip); SCAN2D_ERR_BAD_SHAPE when Cout < 1.
int block_linear_launch(const scan2d_desc* d, int Cout, const void* in, const void* Wt, const float* bias, const void* residual,
                        void* out, hipStream_t stream);

// Normalisation over the channels of each position (scan2d_norm.hip); kind 0 = layer norm, 1 = RMS norm;
// SCAN2D_ERR_BAD_SHAPE for another kind or a negative eps.
int block_norm_launch(const scan2d_desc* d, int kind, float eps, const void* in, const float* gamma, const float* beta, void* out,
                      hipStream_t stream);

}  // namespace scan2d
