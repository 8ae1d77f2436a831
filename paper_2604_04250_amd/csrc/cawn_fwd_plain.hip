// Forward scan kernels of the threshold gate with a constant retention per lane (Sec. 3.2-3.5 of the paper).
#include "cawn_fwd_kernel.hpp"

namespace cawn {

hipError_t launch_fwd_plain(const FwdArgs &a, int conv_k, bool vec, hipStream_t s)
{
    return launch_fwd_family<false, false>(a, conv_k, vec, s);
}

}  // namespace cawn
