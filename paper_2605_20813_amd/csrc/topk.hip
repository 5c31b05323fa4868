// Exact per-row top-k of fp32 scores (Sec. 3.3, TopK equation), gfx950.
//
// One workgroup per score row.  The k-th largest value is found by a 4-pass radix select on
// the order-preserving integer image of the floats (one 256-bin LDS histogram per byte, most
// significant first); the row is then swept once more in index order and every element above
// the threshold, plus the first `need` elements equal to it, is written at the position a
// ballot/popcount prefix sum gives it.  The output is therefore ascending in column index
// and, among equal scores, the lower index wins.  Integer work only: results are exact and
// identical from run to run.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int TK_THREADS = 1024;
constexpr int TK_WAVES = TK_THREADS / 64;

// floats -> unsigned keys with the same order (larger float <=> larger key)
__device__ __forceinline__ uint32_t order_key(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ void __launch_bounds__(TK_THREADS) topk_kernel(TopkParams p) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_prefix, sh_need;
    __shared__ uint32_t wave_cnt[2][TK_WAVES];

    const int row = blockIdx.x;
    const float* __restrict__ s = p.scores + (int64_t)row * p.n;
    int32_t* __restrict__ out = p.idx + (int64_t)row * p.k;
    const int n = p.n;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    // ---- radix select: after the loop `prefix` is the key of the k-th largest element and
    //      `need` how many elements equal to it belong to the top-k
    uint32_t prefix = 0, mask = 0, need = (uint32_t)p.k;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < n; j += TK_THREADS) {
            const uint32_t key = order_key(s[j]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t above = 0;
            int bin = 255;
            for (; bin > 0; --bin) {
                if (above + hist[bin] >= need) break;
                above += hist[bin];
            }
            sh_prefix = prefix | ((uint32_t)bin << shift);
            sh_need = need - above;
        }
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        mask |= 255u << shift;
    }

    // ---- ordered compaction
    uint32_t eq_seen = 0, out_pos = 0;
    for (int base = 0; base < n; base += TK_THREADS) {
        const int j = base + tid;
        uint32_t key = 0;
        const bool live = j < n;
        if (live) key = order_key(s[j]);
        const bool gt = live && key > prefix;
        const bool eq = live && key == prefix;

        const uint64_t eq_ballot = __ballot(eq);
        const uint32_t eq_lane = __popcll(eq_ballot & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[0][wave] = __popcll(eq_ballot);
        __syncthreads();
        uint32_t eq_before = eq_seen, eq_total = 0;
#pragma unroll
        for (int w = 0; w < TK_WAVES; ++w) {
            const uint32_t c = wave_cnt[0][w];
            eq_before += (w < wave) ? c : 0u;
            eq_total += c;
        }
        const bool sel = gt || (eq && (eq_before + eq_lane) < need);

        const uint64_t sel_ballot = __ballot(sel);
        const uint32_t sel_lane = __popcll(sel_ballot & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[1][wave] = __popcll(sel_ballot);
        __syncthreads();
        uint32_t sel_before = out_pos, sel_total = 0;
#pragma unroll
        for (int w = 0; w < TK_WAVES; ++w) {
            const uint32_t c = wave_cnt[1][w];
            sel_before += (w < wave) ? c : 0u;
            sel_total += c;
        }
        if (sel) {
            const uint32_t pos = sel_before + sel_lane;
            if (pos < (uint32_t)p.k) out[pos] = j;     // guard: holds by construction
        }
        eq_seen += eq_total;
        out_pos += sel_total;
        // wave_cnt[0] is rewritten only after the next barrier pair: the loop's first barrier
        // of the next iteration comes after every wave has read wave_cnt[1], and wave_cnt[0]
        // was last read before this iteration's second barrier.
    }
}

}  // namespace

hipError_t launch_topk(const TopkParams& p, hipStream_t s) {
    hipLaunchKernelGGL(topk_kernel, dim3(p.rows), dim3(TK_THREADS), 0, s, p);
    return hipGetLastError();
}

}  // namespace pulsecol
