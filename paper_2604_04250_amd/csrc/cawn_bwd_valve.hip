// Backward kernels of the per-head input valve (Sec. 3.3 of the paper) with a constant retention per lane.
#include "cawn_bwd_kernel.hpp"

namespace cawn {

hipError_t launch_bwd_valve(const BwdArgs &a, int conv_k, hipStream_t s)
{
    return a.want_param ? launch_bwd_family_act<true, true, false, false>(a, conv_k, s)
                        : launch_bwd_family_act<false, true, false, false>(a, conv_k, s);
}

}  // namespace cawn
