// Roofline probes for the box the benchmark runs on: what the matrix pipe and the memory
// system deliver to the simplest possible kernel, so that the attention kernels can be read
// against measured ceilings as well as against the data-sheet peaks.
//
//   mfma_only: 256 workgroups x 4 waves (one wave per SIMD), nothing but
//              v_mfma_f32_32x32x16_bf16 on four independent accumulators; once with constant
//              operands, once with random ones (the clock the chip sustains depends on how
//              many bits toggle).
//   mfma_weights<W>: the same matrix instructions on random operands with W softmax weights per
//              instruction formed beside them (fma, exp2, add on the results of the chain before,
//              placed between the matrix instructions): W = 1 is the mix of the attention kernels
//              (one wave per SIMD), W = 2 that of the two select passes (one and two waves per
//              SIMD).  No memory, no LDS: what the issue port and the power limit leave of the
//              matrix pipe to this mix of instructions.
//   copy:      1 GiB device-to-device with 16-byte accesses; bytes read + bytes written.
//
// Prints one JSON object.  Stand-alone program (no library code), built by
// paper_2605_20813_amd/build.py and started by bench.py as a child process.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>

#define CHECK(x)                                                                              \
    do {                                                                                      \
        hipError_t e_ = (x);                                                                  \
        if (e_ != hipSuccess) {                                                               \
            fprintf(stderr, "roofline_probe: %s failed: %s\n", #x, hipGetErrorString(e_));    \
            return 1;                                                                         \
        }                                                                                     \
    } while (0)

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__device__ unsigned mix(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

constexpr int NFRAG = 8;          // operand fragments cycled through
constexpr int MFMA_PER_ITER = 4 * NFRAG;

template <bool RANDOM>
__global__ void __launch_bounds__(256) mfma_only(float* out, int iters) {
    bf16x8 a[NFRAG], b[NFRAG];
    for (int f = 0; f < NFRAG; ++f)
        for (int e = 0; e < 8; ++e) {
            const unsigned h = mix((threadIdx.x * 64 + f * 8 + e) * 2654435761u + blockIdx.x);
            const unsigned g = mix(h + 12345u);
            // sum of two uniforms: roughly bell-shaped in [-2.4, 2.4]
            const float ua = ((h & 0xffff) + (h >> 16)) * (1.0f / 65536.0f) - 1.0f;
            const float ub = ((g & 0xffff) + (g >> 16)) * (1.0f / 65536.0f) - 1.0f;
            a[f][e] = RANDOM ? (__bf16)(ua * 2.4f) : (__bf16)0.0115f;
            b[f][e] = RANDOM ? (__bf16)(ub * 2.4f) : (__bf16)0.0115f;
        }
    f32x16 c[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int f = 0; f < NFRAG; ++f)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], b[(f + i) % NFRAG], c[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) s += c[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// Two accumulation chains of 8 matrix instructions each, issued alternately (as the kernels issue the two
// products that share an operand fragment); behind every matrix instruction W weights from the chains before.
template <int W>
__global__ void __launch_bounds__(256) mfma_weights(float* out, int iters) {
    bf16x8 a[NFRAG], b[NFRAG];
    for (int f = 0; f < NFRAG; ++f)
        for (int e = 0; e < 8; ++e) {
            const unsigned h = mix((threadIdx.x * 64 + f * 8 + e) * 2654435761u + blockIdx.x);
            const unsigned g = mix(h + 12345u);
            a[f][e] = (__bf16)((((h & 0xffff) + (h >> 16)) * (1.0f / 65536.0f) - 1.0f) * 2.4f);
            b[f][e] = (__bf16)((((g & 0xffff) + (g >> 16)) * (1.0f / 65536.0f) - 1.0f) * 2.4f);
        }
    f32x16 prev0, prev1;
    for (int r = 0; r < 16; ++r) prev0[r] = prev1[r] = 0.f;
    float sum[4] = {0.f, 0.f, 0.f, 0.f};
    const float scale = 0.1275f, ref = 6.0f;
    for (int it = 0; it < iters; ++it) {
        f32x16 cur0, cur1;
        for (int r = 0; r < 16; ++r) cur0[r] = cur1[r] = 0.f;
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) {
            cur0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], b[(f + 3) % NFRAG], cur0, 0, 0, 0);
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const int r = f * W + w;
                sum[r & 3] += __builtin_amdgcn_exp2f(__builtin_fmaf(prev0[r], scale, -ref));
            }
            __builtin_amdgcn_sched_barrier(0);       // nothing moves across: one matrix instruction, then its weights
            cur1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], b[(f + 5) % NFRAG], cur1, 0, 0, 0);
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const int r = f * W + w;
                sum[(r + 2) & 3] += __builtin_amdgcn_exp2f(__builtin_fmaf(prev1[r], scale, -ref));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        prev0 = cur0;
        prev1 = cur1;
    }
    out[blockIdx.x * 256 + threadIdx.x] = (sum[0] + sum[1]) + (sum[2] + sum[3]);
}

__global__ void __launch_bounds__(256) copy16(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

template <typename F>
static int timed(F launch, int reps, float* best_ms) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    *best_ms = 1e30f;
    for (int r = 0; r < reps; ++r) {
        CHECK(hipEventRecord(e0));
        launch();
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (r > 0 && ms < *best_ms) *best_ms = ms;      // the first repetition warms up
    }
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

int main() {
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    float* out;
    CHECK(hipMalloc(&out, (size_t)cus * 256 * sizeof(float)));
    const int iters = 40000;                         // ~20-30 ms per launch
    const double flop = (double)cus * 4 * iters * MFMA_PER_ITER * (2.0 * 32 * 32 * 16);
    float ms_const, ms_rand;
    if (timed([&] { hipLaunchKernelGGL(mfma_only<false>, dim3(cus), dim3(256), 0, 0, out, iters); }, 4, &ms_const)) return 1;
    if (timed([&] { hipLaunchKernelGGL(mfma_only<true>, dim3(cus), dim3(256), 0, 0, out, iters); }, 4, &ms_rand)) return 1;

    // the instruction mixes of the attention kernels and of the select passes
    float* out2;
    CHECK(hipMalloc(&out2, (size_t)cus * 2 * 256 * sizeof(float)));
    const int witers = 50000;
    const double wflop = (double)cus * 4 * witers * 2 * NFRAG * (2.0 * 32 * 32 * 16);
    float ms_w1, ms_w2, ms_w2x2;
    if (timed([&] { hipLaunchKernelGGL(mfma_weights<1>, dim3(cus), dim3(256), 0, 0, out2, witers); }, 4, &ms_w1)) return 1;
    if (timed([&] { hipLaunchKernelGGL(mfma_weights<2>, dim3(cus), dim3(256), 0, 0, out2, witers); }, 4, &ms_w2)) return 1;
    if (timed([&] { hipLaunchKernelGGL(mfma_weights<2>, dim3(cus * 2), dim3(256), 0, 0, out2, witers); }, 4, &ms_w2x2)) return 1;
    CHECK(hipFree(out2));

    const size_t bytes = (size_t)1 << 30;
    uint4 *src, *dst;
    CHECK(hipMalloc(&src, bytes));
    CHECK(hipMalloc(&dst, bytes));
    CHECK(hipMemset(src, 1, bytes));
    float ms_copy;
    if (timed([&] { hipLaunchKernelGGL(copy16, dim3(cus * 16), dim3(256), 0, 0, src, dst, bytes / 16); }, 5, &ms_copy)) return 1;
    CHECK(hipGetLastError());

    printf("{\"compute_units\": %d, \"mfma_only_tflops_constant_operands\": %.1f, \"mfma_only_tflops_random_operands\": %.1f, "
           "\"mfma_plus_1_weight_tflops\": %.1f, \"mfma_plus_2_weights_tflops\": %.1f, "
           "\"mfma_plus_2_weights_two_waves_per_simd_tflops\": %.1f, \"copy_1gib_gbps_read_plus_write\": %.1f}\n",
           cus, flop / ms_const * 1e-9, flop / ms_rand * 1e-9, wflop / ms_w1 * 1e-9, wflop / ms_w2 * 1e-9,
           2.0 * wflop / ms_w2x2 * 1e-9, 2.0 * bytes / ms_copy * 1e-6);
    CHECK(hipFree(src));
    CHECK(hipFree(dst));
    CHECK(hipFree(out));
    return 0;
}
