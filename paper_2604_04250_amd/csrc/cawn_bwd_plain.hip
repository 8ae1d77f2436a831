// Backward kernels of the threshold gate with a constant retention per lane (Sec. 3.4, Sec. 3.5 of the paper).
#include "cawn_bwd_kernel.hpp"

namespace cawn {

hipError_t launch_bwd_plain(const BwdArgs &a, int conv_k, hipStream_t s)
{
    return a.want_param ? launch_bwd_family_act<true, false, false, false>(a, conv_k, s)
                        : launch_bwd_family_act<false, false, false, false>(a, conv_k, s);
}

}  // namespace cawn
