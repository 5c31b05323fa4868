// Validation mode of the column-sparse attention call: the kernels trust the column numbers
// they are given (an entry outside [0, seq) would address memory outside K and V), so a
// caller that cannot vouch for its indices can ask for this check in front of the launch.
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

__global__ void __launch_bounds__(256) index_range_kernel(const int32_t* __restrict__ idx, int64_t count, int32_t n,
                                                          int32_t* __restrict__ bad_count,
                                                          const int32_t* __restrict__ varlen, int32_t batch,
                                                          int64_t per_batch, int32_t k) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int bad = 0;
    for (; i < count; i += stride) {
        const int32_t c = idx[i];
        if (varlen == nullptr) {
            bad += (c < 0 || c >= n) ? 1 : 0;
        } else {
            // variable-length batch: the leading `kept` entries of a row count, against the element's own length
            const int b = (int)(i / per_batch);
            const int pos = (int)(i % k);
            bad += (pos < varlen[batch + b] && (c < 0 || c >= varlen[b])) ? 1 : 0;
        }
    }
    // one atomic per wavefront that saw a bad entry (vector atomics; the count only needs to be non-zero)
    const unsigned long long any = __ballot(bad != 0);
    if (any != 0ull && (threadIdx.x & 63) == (unsigned)__builtin_ctzll(any)) atomicAdd(bad_count, __builtin_popcountll(any));
}

}  // namespace

hipError_t launch_index_range_check(const int32_t* idx, int64_t count, int32_t n, int32_t* bad_count,
                                    const int32_t* varlen, int32_t batch, int64_t per_batch, int32_t k, hipStream_t s) {
    hipError_t e = hipMemsetAsync(bad_count, 0, sizeof(int32_t), s);
    if (e != hipSuccess) return e;
    const int64_t blocks = (count + 255) / 256;
    const int grid = (int)(blocks < 4096 ? (blocks < 1 ? 1 : blocks) : 4096);
    hipLaunchKernelGGL(index_range_kernel, dim3(grid), dim3(256), 0, s, idx, count, n, bad_count, varlen, batch, per_batch, k);
    return hipGetLastError();
}

}  // namespace pulsecol
