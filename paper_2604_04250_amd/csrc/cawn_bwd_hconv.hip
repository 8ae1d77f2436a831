// Backward kernels behind the depth-wise harmonic convolution (Sec. 3.6 of the paper), threshold gate.
#include "cawn_bwd_kernel.hpp"

namespace cawn {

hipError_t launch_bwd_hconv(const BwdArgs &a, int conv_k, hipStream_t s)
{
    return launch_bwd_family_act<true, false, false, true>(a, conv_k, s);
}

}  // namespace cawn
