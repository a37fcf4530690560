// Producers of the scan's inputs inside a 2DMamba block (Sec. 3.2, Fig. 2): host-side entries used by the C ABI.
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

}  // namespace scan2d
