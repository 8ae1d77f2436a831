// placeholder until the backward kernels land
#include "cawn_internal.hpp"
namespace cawn {
hipError_t launch_bwd(const BwdArgs &, int, bool, hipStream_t) { return hipErrorNotSupported; }
}
extern "C" int cawn_phase_accumulate_bwd(const cawn_desc *, const float *, const float *, const float *,
                              const float *, const float *, const float *, const void *, const void *,
                              const float *, const float *, const void *, float *, float *, float *, float *,
                              float *, float *, void *, void *, size_t, void *) { return CAWN_EUNSUPPORTED; }
