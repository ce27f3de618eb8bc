// The team kernel for networks with depthwise layers (inverted-residual families): depthwise, gating and
// squeeze-excite units instead of the max-pool.  A translation unit of its own, so that the two team kernels compile
// side by side.
#include "stream_units.h"

namespace sushi {

hipError_t prepare_team_kernel_mobile() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(sushi_team_kernel<OPS_MOBILE>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, RED_BYTES + RES_STORE_BYTES);
}

hipError_t team_kernel_mobile_blocks_per_cu(int *n) {
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(n, sushi_team_kernel<OPS_MOBILE>, STREAM_THREADS,
                                                        RED_BYTES + RES_STORE_BYTES);
}

hipError_t launch_team_kernel_mobile(const TeamArgs &a, int nwg, hipStream_t s) {
    hipLaunchKernelGGL(sushi_team_kernel<OPS_MOBILE>, dim3(nwg), dim3(STREAM_THREADS), RED_BYTES + RES_STORE_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace sushi
