// Backward instantiations with an independent decay for the column recurrence (the supplement's A-bar ablation).
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernels bwd_kernels_av_f32(int NW, bool fast) { return lookup_bwd_kernels_av<float>(NW, fast); }
BwdKernels bwd_kernels_av_bf16(int NW, bool fast) { return lookup_bwd_kernels_av<bf16_t>(NW, fast); }
}
