// Stand-ins for the kernel launchers in the HOST-ONLY build of the library (build.py:
// build_host_sanitized).  That build compiles api.hip with the host C++ compiler under
// AddressSanitizer / UndefinedBehaviorSanitizer so that the CPU tests can run the argument checks,
// the planner and the dealing under the sanitizers; it contains no device code, and every
// launcher reports hipErrorNotSupported.  Never loaded on a GPU path.
#include "../../include/mi355conv.h"
#include "conv_internal.h"

namespace mi355conv {

hipError_t prepare_gather_gemm() { return hipErrorNotSupported; }
hipError_t prepare_wgrad() { return hipErrorNotSupported; }
hipError_t prepare_wgrad_fast() { return hipErrorNotSupported; }
hipError_t launch_direct_fwd(const float *, const float *, float *, const Shape &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_direct_bwd_data(const float *, const float *, float *, const Shape &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_direct_bwd_weight(const float *, const float *, float *, const Shape &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_slice_reduce(const float *, float *, long long, int, long long, hipStream_t, const float *, float, int)
{
    return hipErrorNotSupported;
}
hipError_t launch_bias_act(float *, long long, const float *, float, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gather_gemm(const GatherGemmParams &, bool, int, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gather_elem(const GatherGemmParams &, bool, int, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_wgrad(const WgradParams &, int, int, bool, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_wgrad_fast(const WgradParams &, int, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bwd_data_small_ic(const SmallIcParams &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_wgrad_small_ic(const SmallIcParams &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_fwd_small_ic(const SmallIcParams &, hipStream_t) { return hipErrorNotSupported; }

}  // namespace mi355conv

extern "C" int conv2d_probe_mfma_rate(int, int, int, float *, void *) { return MI355CONV_ERR_HIP; }
