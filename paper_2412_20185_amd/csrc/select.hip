// Step 1 of dynamic error compensation (DecDEC Section 4.1): sc_indices, the k
// input channels with the largest |x|, and x[sc_indices], as a kernel of its
// own.  The paper's kernel uses an approximate, chunked bucket Top-K (Section
// 4.3); this is the exact Top-K it uses as its quality reference (Section 5.2).
// The algorithm is in select_block.h; one workgroup does the whole selection
// (256 threads up to 8192 channels, 1024 threads above).
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "select_block.h"

namespace decdec {
namespace {

template <int THREADS, int NCH>
__global__ __launch_bounds__(THREADS) void select_topk_kernel(const uint16_t* __restrict__ x, int K, int k,
                                                             int32_t* __restrict__ idx_out,
                                                             uint16_t* __restrict__ xsel_out) {
    __shared__ SelectShared sh;
    block_select_topk<THREADS, NCH>(x, K, k, sh, idx_out, xsel_out);
}

}  // namespace

hipError_t launch_select_topk(const void* x, int K, int k, int32_t* idx_out, void* xsel_out, hipStream_t stream,
                              const KernelTimer* tm) {
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint16_t* xs = static_cast<uint16_t*>(xsel_out);
    const dim3 one(1);
    if (K <= 4096) return launch_kernel(tm, select_topk_kernel<256, 2>, one, dim3(256), 0, stream, xp, K, k, idx_out, xs);
    if (K <= 8192) return launch_kernel(tm, select_topk_kernel<256, 4>, one, dim3(256), 0, stream, xp, K, k, idx_out, xs);
    if (K <= 16384)
        return launch_kernel(tm, select_topk_kernel<1024, 2>, one, dim3(1024), 0, stream, xp, K, k, idx_out, xs);
    if (K <= 32768)
        return launch_kernel(tm, select_topk_kernel<1024, 4>, one, dim3(1024), 0, stream, xp, K, k, idx_out, xs);
    return launch_kernel(tm, select_topk_kernel<1024, 8>, one, dim3(1024), 0, stream, xp, K, k, idx_out, xs);
}

}  // namespace decdec
