// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <stdint.h>

#include "lp.h"

// Host-side plan: the integers of Sec. 3.3 (Eq. 7-9) and Sec. 3.4 (Eq. 11) for
// every partition, plus what the copy kernels need to address the packed buffer.
struct lp_plan {
    lp_config cfg;
    int32_t dim;          // 0 = T, 1 = H, 2 = W
    int32_t K;
    int32_t N;            // patches along dim
    int32_t L;            // core patches per partition, ceil(N / K)
    int32_t O;            // overlap patches
    int32_t extent;       // latent extent along dim
    int64_t inner;        // product of the extents after dim (elements per unit step along dim)
    int64_t outer;        // product of the extents before dim, channels included
    int64_t latent_elems; // C*T*H*W
    int64_t total_elems;  // sum of the sub-latent sizes
    lp_part_info part[LP_MAX_PARTS];
};

namespace lp {
void set_last_hip_error(int err);
}

#ifdef __HIPCC__
#include <hip/hip_runtime.h>
namespace lp {
// Launch through hipLaunchKernel so that the status is this launch's own return
// value (hipGetLastError would also report errors other code left behind).
template <typename... Args>
inline int launch_kernel(const void *fn, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, Args... args) {
    void *argv[] = {static_cast<void *>(&args)...};
    const hipError_t e = hipLaunchKernel(fn, grid, block, argv, lds_bytes, stream);
    if (e != hipSuccess) {
        set_last_hip_error(int(e));
        return LP_ERR_HIP;
    }
    return LP_OK;
}
}  // namespace lp
#endif
