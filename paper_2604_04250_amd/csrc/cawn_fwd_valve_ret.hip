// Forward scan kernels of the per-head valve with the data-dependent retention (Sec. 3.3 of the paper).
#include "cawn_fwd_kernel.hpp"

namespace cawn {

hipError_t launch_fwd_valve_ret(const FwdArgs &a, int conv_k, bool vec, hipStream_t s)
{
    return launch_fwd_family<true, true>(a, conv_k, vec, s);
}

}  // namespace cawn
