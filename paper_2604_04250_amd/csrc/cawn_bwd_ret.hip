// Backward kernels of the data-dependent retention (Sec. 3.3 item 4 of the paper), with either gate.
#include "cawn_bwd_kernel.hpp"

namespace cawn {

hipError_t launch_bwd_ret(const BwdArgs &a, int conv_k, hipStream_t s)
{
    return a.valve ? launch_bwd_family_act<true, true, true, false>(a, conv_k, s)
                   : launch_bwd_family_act<true, false, true, false>(a, conv_k, s);
}

}  // namespace cawn
