// Instantiations of the shared-producer forward kernels that compute the softplus step and apply the output gate.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_shared_kernel_gate_f32(int LG, int K, int NW, int NG, int waves, int RPB) {
    return lookup_fwd_shared_kernel<float, true, false, false, true>(LG, K, NW, NG, waves, RPB);
}
FwdKernel fwd_shared_kernel_gate_bf16(int LG, int K, int NW, int NG, int waves, int RPB, bool ua) {
    return ua ? lookup_fwd_shared_kernel<bf16_t, true, true, false, true>(LG, K, NW, NG, waves, RPB)
              : lookup_fwd_shared_kernel<bf16_t, true, false, false, true>(LG, K, NW, NG, waves, RPB);
}
}
