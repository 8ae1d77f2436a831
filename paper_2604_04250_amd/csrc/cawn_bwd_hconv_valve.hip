// Backward kernels behind the depth-wise harmonic convolution (Sec. 3.6 of the paper), per-head valve (Sec. 3.3).
#include "cawn_bwd_kernel.hpp"

namespace cawn {

hipError_t launch_bwd_hconv_valve(const BwdArgs &a, int conv_k, hipStream_t s)
{
    return launch_bwd_family_act<true, true, false, true>(a, conv_k, s);
}

}  // namespace cawn
