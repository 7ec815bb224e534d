// Plain streaming copy: the bandwidth yardstick and counter-calibration kernel declared in
// include/signvote_bench.h.  One 16-byte non-temporal load and store per thread.
#include "../../include/signvote.h"
#include "../../include/signvote_bench.h"
#include "device_utils.h"

namespace ssv {

__global__ __launch_bounds__(kBlock) void copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, int64_t n) {
    const int64_t step = (int64_t)gridDim.x * kBlock;              // one pass unless the grid was capped
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += step) stream_store(dst + i, stream_load(src + i));
}

}  // namespace ssv

extern "C" int ssv_bench_copy(const void* src, void* dst, int64_t bytes, void* stream) {
    if (src == nullptr || dst == nullptr) return SSV_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0) return SSV_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(src) % 16 != 0 || reinterpret_cast<uintptr_t>(dst) % 16 != 0) return SSV_ERR_ALIGN;
    const int64_t n = bytes / 16;
    int64_t grid = (n + ssv::kBlock - 1) / ssv::kBlock;
    if (grid > 0x40000000LL) grid = 0x40000000LL;      // defensive: 2^30 blocks cover 4 TiB, beyond any buffer here
    (void)hipGetLastError();                           // a stale error of an earlier call is not this launch's
    hipLaunchKernelGGL(ssv::copy_kernel, dim3((unsigned)grid), dim3(ssv::kBlock), 0, static_cast<hipStream_t>(stream),
                       static_cast<const ssv::f32x4*>(src), static_cast<ssv::f32x4*>(dst), n);
    return hipGetLastError() == hipSuccess ? SSV_OK : SSV_ERR_HIP;
}
