// Backward pass of the 2D selective scan: host-side entry used by the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include "../../include/scan2d.h"

namespace scan2d {

size_t bwd_workspace_bytes(const scan2d_desc* d);

// One line describing the backward plan; false when the shape has no plan.
bool bwd_describe(const scan2d_desc* d, char* text, size_t text_bytes);

int bwd_launch(const scan2d_desc* d, const void* x, const void* delta, const float* A, const void* Bm,
               const void* Cm, const float* Dskip, const uint8_t* mask, const void* dy, void* dx,
               void* ddelta, float* dA, float* dBm, float* dCm, float* dDskip, void* workspace,
               size_t workspace_bytes, hipStream_t stream);

}  // namespace scan2d
