// Backward kernels behind the depth-wise harmonic convolution (Sec. 3.6 of the paper), data-dependent retention (Sec. 3.3 item 4), either gate.
#include "cawn_bwd_kernel.hpp"

namespace cawn {

hipError_t launch_bwd_hconv_ret(const BwdArgs &a, int conv_k, hipStream_t s)
{
    return a.valve ? launch_bwd_family_act<true, true, true, true>(a, conv_k, s)
                   : launch_bwd_family_act<true, false, true, true>(a, conv_k, s);
}

}  // namespace cawn
