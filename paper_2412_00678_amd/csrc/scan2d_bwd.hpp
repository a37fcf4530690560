// Backward pass of the 2D selective scan: host-side entry used by the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include "../../include/scan2d.h"

namespace scan2d {

// softplus: the workspace of scan2d_bwd_softplus (the banded form adds one fp32 map-sized buffer for the step).
// av: the instantiations with an independent decay parameter A_v for the column recurrence.
size_t bwd_workspace_bytes(const scan2d_desc* d, bool softplus = false, bool av = false);

// SCAN2D_OK when bwd_launch would accept the descriptor (plan and grid sizes), else the error it would return;
// enqueues nothing.
int bwd_check(const scan2d_desc* d, bool softplus = false, bool av = false);

// Training pair: bytes of the band checkpoints that a forward pass can leave for the backward pass (0: this shape has
// no such forward), and that forward pass (the shared-producer forward kernel in its checkpoint-and-output mode).
size_t bwd_saved_bytes(const scan2d_desc* d);
int fwd_saving_launch(const scan2d_desc* d, const void* x, const void* delta, const float* A, const void* Bm, const void* Cm,
                      const float* Dskip, const uint8_t* mask, void* y, float* saved, hipStream_t stream);

// One line describing the backward plan; false when the shape has no plan.
bool bwd_describe(const scan2d_desc* d, char* text, size_t text_bytes);

// softplus: `delta` is the raw projection, the step is softplus(delta + delta_bias[c]); ddelta is then the
// gradient of the raw projection and ddelta_bias (null iff delta_bias is) that of the bias.
int bwd_launch(const scan2d_desc* d, const void* x, const void* delta, const float* delta_bias, bool softplus,
               const float* A, const void* Bm,
               const void* Cm, const float* Dskip, const uint8_t* mask, const void* dy, void* dx,
               void* ddelta, float* ddelta_bias, float* dA, float* dBm, float* dCm, float* dDskip, void* workspace,
               size_t workspace_bytes, hipStream_t stream, const float* A_v = nullptr, float* dA_v = nullptr,
               const float* saved = nullptr,    // saved: the checkpoints left by fwd_saving_launch (no checkpoint sweep then)
               const void* z = nullptr, const void* y_scan = nullptr, void* dz = nullptr);   // see bwd_gate_in_sweep
// True where the main sweep has an instantiation that also runs the backward of the output gate (softplus step, no
// flags): bwd_launch may then be given z, y_scan and dz, with dy the gradient of the GATED output.
bool bwd_gate_in_sweep(const scan2d_desc* d);

}  // namespace scan2d
