// Variable-length batches: a padded batch whose elements have their own sequence lengths.
// The kernels read two words per batch element from a small device array, varlen[2 * batch]:
// the element's length (rows 0 .. len-1 of its slabs are real, the rest is padding) and `kept`, the
// number of leading entries of its column sets that count.  The kernels here maintain that array
// without any host-to-device copy: lengths travel inside the launch arguments, and `kept` is derived
// on the device -- from the keep ratio (Sec. 3.1, sparsity budget: k = max(1, floor(keep * len)) on
// the element's own length), from a caller's k, or from the column sets themselves (whose unused tail
// is filled with -1).
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

__global__ void varlen_store_kernel(int32_t* __restrict__ varlen, int32_t first, int32_t count, VarlenChunk values) {
    const int i = threadIdx.x;
    if (i < count) varlen[first + i] = values.v[i];
}

__global__ void varlen_kept_from_ratio_kernel(int32_t* __restrict__ varlen, int32_t batch, double keep_ratio) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int len = varlen[b];
    // the same rule, the same guard against the binary image of a decimal ratio, as the host's pulsecol_num_keep
    long long k = (long long)__builtin_floor(keep_ratio * (double)len + 1e-9);
    k = k < 1 ? 1 : (k > len ? len : k);
    varlen[batch + b] = (int32_t)k;
}

__global__ void varlen_kept_from_k_kernel(int32_t* __restrict__ varlen, int32_t batch, int32_t k) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int len = varlen[b];
    varlen[batch + b] = k < len ? k : len;
}

__global__ void varlen_kept_from_idx_kernel(int32_t* __restrict__ varlen, int32_t batch, const int32_t* __restrict__ idx,
                                            int64_t per_batch, int32_t k) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int32_t* row = idx + (int64_t)b * per_batch;
    const int len = varlen[b];
    const int most = k < len ? k : len;
    // valid entries come first, the padding (-1) behind them: first negative entry by bisection
    int lo = 0, hi = most;                       // the answer lies in [lo, hi]
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (row[mid] >= 0) lo = mid + 1; else hi = mid;
    }
    varlen[batch + b] = lo < 1 ? 1 : lo;         // at least one column (an all-padding row is the caller's error; keep the kernels in bounds)
}

}  // namespace

hipError_t launch_varlen_store(int32_t* varlen, int32_t first, int32_t count, const VarlenChunk& values, hipStream_t s) {
    if (count < 1 || count > 64) return hipErrorInvalidValue;
    hipLaunchKernelGGL(varlen_store_kernel, dim3(1), dim3(64), 0, s, varlen, first, count, values);
    return hipGetLastError();
}

hipError_t launch_varlen_kept_from_ratio(int32_t* varlen, int32_t batch, double keep_ratio, hipStream_t s) {
    hipLaunchKernelGGL(varlen_kept_from_ratio_kernel, dim3((batch + 63) / 64), dim3(64), 0, s, varlen, batch, keep_ratio);
    return hipGetLastError();
}

hipError_t launch_varlen_kept_from_k(int32_t* varlen, int32_t batch, int32_t k, hipStream_t s) {
    hipLaunchKernelGGL(varlen_kept_from_k_kernel, dim3((batch + 63) / 64), dim3(64), 0, s, varlen, batch, k);
    return hipGetLastError();
}

hipError_t launch_varlen_kept_from_idx(int32_t* varlen, int32_t batch, const int32_t* idx, int64_t per_batch, int32_t k,
                                       hipStream_t s) {
    hipLaunchKernelGGL(varlen_kept_from_idx_kernel, dim3((batch + 63) / 64), dim3(64), 0, s, varlen, batch, idx, per_batch, k);
    return hipGetLastError();
}

}  // namespace pulsecol
