// Forward scan kernels of the per-head input valve (Sec. 3.3 of the paper) with a constant retention per lane.
#include "cawn_fwd_kernel.hpp"

namespace cawn {

hipError_t launch_fwd_valve(const FwdArgs &a, int conv_k, bool vec, hipStream_t s)
{
    return launch_fwd_family<true, false>(a, conv_k, vec, s);
}

}  // namespace cawn
