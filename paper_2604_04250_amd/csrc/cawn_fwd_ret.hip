// Forward scan kernels of the data-dependent retention (Sec. 3.3 item 4 of the paper), threshold gate.
#include "cawn_fwd_kernel.hpp"

namespace cawn {

hipError_t launch_fwd_ret(const FwdArgs &a, int conv_k, bool vec, hipStream_t s)
{
    return launch_fwd_family<false, true>(a, conv_k, vec, s);
}

}  // namespace cawn
