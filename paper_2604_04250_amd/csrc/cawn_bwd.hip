// Fused backward (Sec. 3.4 last paragraph, Sec. 3.5 of the paper): which family of kernels a call runs.
// The kernel itself is cawn_bwd_kernel.hpp; its families are instantiated in cawn_bwd_<family>.hip.
#include "cawn_bwd_kernel.hpp"

namespace cawn {

hipError_t launch_bwd(const BwdArgs &a, int conv_k, bool vec, hipStream_t s)
{
    (void)vec;      // one lane per thread in every build of the backward kernel
    static_assert(BwdV == 1, "the vectorised backward was dropped");
    if (a.hconv) {      // the harmonic convolution's tap gradients need the rebuilt state
        if (!a.want_param) return hipErrorInvalidValue;
        if (a.ret) return launch_bwd_hconv_ret(a, conv_k, s);
        return a.valve ? launch_bwd_hconv_valve(a, conv_k, s) : launch_bwd_hconv(a, conv_k, s);
    }
    if (a.ret) return launch_bwd_ret(a, conv_k, s);
    if (a.valve) return launch_bwd_valve(a, conv_k, s);
    return launch_bwd_plain(a, conv_k, s);
}

}  // namespace cawn
