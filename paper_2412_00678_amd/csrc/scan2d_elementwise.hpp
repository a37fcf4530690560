// Element-wise kernels beside the scan kernels: the output gate of the block, identity cells, and the
// transposes of the columns-first order.  What they have in common: the work is per position, not per
// (position, state), so doing it inside the scan kernels would either be repeated by every lane group of
// a map or cost the scan kernels registers and branches; they are bound by vector issue and registers, not
// by HBM, while a pass over a map-sized tensor here runs at the HBM copy rate.
//
// Output gate, y = y_scan * SiLU(z) (2DMamba Sec. 3.2 / Fig. 2: the Mamba block with its scan replaced by
// the 2D one).  The gate inside the scan kernels was built and measured: the extra ring of raw registers
// for z cost them a wave of occupancy, more than the extra pass over y costs here.
#pragma once

#include <hip/hip_runtime.h>

#include "../../include/scan2d.h"

namespace scan2d {

// y = y_scan * z / (1 + exp(-z)); y may alias y_scan (in place).  [Bt][Dc][H][W], storage type.
int gate_fwd_launch(const scan2d_desc* d, const void* y_scan, const void* z, void* y, hipStream_t stream);

// The backward of the gated operator is the ungated one fed dy * SiLU(z).  One pass writes that product
// (storage type) to `dyg` and the final dz = dy * y_scan * s (1 + z (1 - s)), s = 1 / (1 + exp(-z)).
size_t gate_bwd_bytes(const scan2d_desc* d);     // bytes of `dyg`, a multiple of 256
int gate_bwd_launch(const scan2d_desc* d, const void* z, const void* y_scan, const void* dy, void* dyg, void* dz,
                    hipStream_t stream);

// Identity cells (SCAN2D_FLAG_IDENTITY_CELLS): a masked cell has step 0 besides x = 0.  Element-wise kernels
// too, for the same reason: a select per element inside the scan kernels costs every caller (measured: 15 % on
// the 256x256 bf16 forward as a run-time flag), a second set of instantiations costs build time and size.
// The scan kernels run on a copy of the step (storage type, [Bt][Dc][H][W]) that holds +0 under the mask -
// or -inf when the step is the softplus of it, whose value (0) and derivative (0) are then exact.
size_t skip_bytes(const scan2d_desc* d);         // bytes of that copy (a multiple of 256); 0 without the flag
int skip_step_launch(const scan2d_desc* d, const void* delta, const uint8_t* mask, bool minus_inf, void* out, hipStream_t stream);
// ddelta = 0 under the mask, in place (the step of an identity cell is a constant).
int skip_grad_launch(const scan2d_desc* d, const uint8_t* mask, void* ddelta, hipStream_t stream);

// Columns first (SCAN2D_FLAG_COLUMNS_FIRST, the supplement's ablation of the scan order): the scan of the
// transposed maps, transposed back.  dst[p][j][i] = src[p][i][j] for `planes` planes of H x W elements of
// 1, 2 or 4 bytes; 32 x 32 tiles through LDS.
int transpose_launch(int elem_bytes, const void* src, void* dst, long long planes, int H, int W, hipStream_t stream);

// Learnable padding token (2DMamba Eq. 4): a masked cell holds pad[c] instead of a fixed zero.  Element-wise kernels
// around the unchanged scan kernels, like the identity cells: the scan runs without a mask on a copy of x that holds
// pad[c] (rounded to the storage type) under the mask; the backward then leaves the gradient of that copy in dx, from
// which dpad[c] = sum over the masked cells is taken (fixed order) before dx is set to +0 there.
int pad_fill_launch(const scan2d_desc* d, const void* x, const uint8_t* mask, const float* pad, void* out, hipStream_t stream);
// ppad: [Bt][Dc] fp32 scratch (not read when mask is null: dpad is then all zeros).
int pad_grad_launch(const scan2d_desc* d, const uint8_t* mask, void* dx, float* ppad, float* dpad, hipStream_t stream);

}  // namespace scan2d
