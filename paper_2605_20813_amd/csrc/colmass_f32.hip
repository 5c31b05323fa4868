// Column softmax mass, fp32 inputs (Sec. 3.3, score equation, per query group G_u of a head):
//   s_{u,j} = (1/|G_u|) sum_{i in G_u} exp2(z_ij * scale * log2(e) - lse2_i)
// with lse2_i = log2 sum_j exp(z_ij * scale) from the row pass (attn_f32.hip, lse-only mode).
//
// K-stationary like the bf16 kernel, on v_mfma_f32_32x32x2_f32: a workgroup owns 128 key
// columns (4 waves x 32 keys held in registers as the A operand) and streams 32-row Q tiles
// through padded LDS.  Fixed summation order, no floating-point atomics.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int NTHREADS = 256;
constexpr int KEYS_PER_WG = 128;
constexpr int QT = 32;
constexpr int PAD = 4;
constexpr int FLUSH = 16;

template <int D>
__global__ void __launch_bounds__(NTHREADS) colmass_f32_kernel(ScoreParams p) {
    constexpr int PIECES = D / 4;
    constexpr int KK = D / 2;
    constexpr int CH = QT * PIECES / NTHREADS;
    constexpr int LDW = D + PAD;

    __shared__ __attribute__((aligned(16))) float lds_q[QT * LDW];
    __shared__ float lds_lse[QT];

    const int nkb = (p.n + KEYS_PER_WG - 1) / KEYS_PER_WG;
    int bh, kblk;
    if (!xcd_tile(blockIdx.x, nkb, p.batch * p.heads, &bh, &kblk)) return;
    const int b = bh / p.heads, h = bh - b * p.heads;
    // variable-length batches: queries and keys of this batch element end at its own length
    const int n = p.varlen != nullptr ? p.varlen[b] : p.n;
    if (kblk * KEYS_PER_WG >= n) return;    // a block of padding keys: its scores are left untouched
    const int64_t head_off = (int64_t)b * p.td.sb + (int64_t)h * p.td.sh;
    // grouped-query layout: query head h reads K/V head h / (heads / kv_heads)
    const int64_t kv_off = (int64_t)b * p.td_kv.sb + (int64_t)(h / (p.heads / p.kv_heads)) * p.td_kv.sh;
    const float* __restrict__ Q = (const float*)p.q + head_off;
    const float* __restrict__ K = (const float*)p.k + kv_off;
    const float* __restrict__ lse = p.lse + (int64_t)bh * p.n;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, lh = lane >> 5;
    const int key0 = kblk * KEYS_PER_WG + wave * 32;

    float kf[KK];    // A operand: K[key lq][d = 2*kk + lh]
    {
        int row = key0 + lq;
        row = row < n ? row : n - 1;
        const float* src = K + (int64_t)row * p.td_kv.sn + lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[kk] = src[2 * kk];
    }

    f32x4 stage[CH];
    float stage_lse = 0.f;
    auto fetch = [&](int t) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + NTHREADS * j;
            int row = t * QT + c / PIECES;
            row = row < n ? row : n - 1;
            stage[j] = *(const f32x4*)(Q + (int64_t)row * p.td.sn + (c % PIECES) * 4);
        }
        if (tid < QT) {
            const int row = t * QT + tid;
            stage_lse = row < n ? lse[row] : INFINITY;     // rows past the end contribute exp2(-inf) = 0
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + NTHREADS * j;
            *(f32x4*)(lds_q + (c / PIECES) * LDW + (c % PIECES) * 4) = stage[j];
        }
        if (tid < QT) lds_lse[tid] = stage_lse;
    };

    const int ntiles = (n + QT - 1) / QT;
    const float c2 = p.scale * kLog2e;
    f32x16 acc_short, acc_long;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc_short[r] = 0.f; acc_long[r] = 0.f; }

    fetch(0);
    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
        commit();
        __syncthreads();
        if (t + 1 < ntiles) fetch(t + 1);

        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
        const float* qrow = lds_q + lq * LDW + lh;     // B operand: Q[query lq][d = 2*kk + lh]
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) s = mfma_f32(kf[kk], qrow[2 * kk], s);
        const float l2 = lds_lse[lq];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_short[r] += exp2f(__builtin_fmaf(s[r], c2, -l2));
        if ((t % FLUSH) == FLUSH - 1) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc_long[r] += acc_short[r]; acc_short[r] = 0.f; }
        }
        // ---- last tile of a query group: combine lanes (fixed butterfly), divide by the group's
        // size, store the group's score row, start over
        const int rows_done = (t + 1) * QT;
        const bool group_end = t + 1 == ntiles || (p.groups > 1 && rows_done % p.group_size == 0);
        if (group_end) {
            const int u = p.groups > 1 ? (t * QT) / p.group_size : 0;
            const int g_first = p.groups > 1 ? u * p.group_size : 0;
            const int g_rows = (rows_done < n ? rows_done : n) - g_first;
            const float inv = 1.0f / (float)g_rows;
            float* __restrict__ out = p.scores + ((int64_t)bh * p.groups + u) * p.n;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = acc_long[r] + acc_short[r];
#pragma unroll
                for (int m = 1; m < 32; m <<= 1) v += __shfl_xor(v, m, 64);
                const int key = key0 + acc_row(r, lh);
                if (lq == 0 && key < n) out[key] = v * inv;
                acc_long[r] = 0.f;
                acc_short[r] = 0.f;
            }
        }
    }
}

template <int D>
hipError_t launch(const ScoreParams& p, hipStream_t s) {
    const int nkb = (p.n + KEYS_PER_WG - 1) / KEYS_PER_WG;
    const int bh_pad = (p.batch * p.heads + 7) / 8 * 8;
    hipLaunchKernelGGL((colmass_f32_kernel<D>), dim3(nkb * bh_pad), dim3(NTHREADS), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_colmass_f32(const ScoreParams& p, int head_dim, hipStream_t s) {
    if (head_dim == 128) return launch<128>(p, s);
    if (head_dim == 64) return launch<64>(p, s);
    return hipErrorInvalidValue;
}

}  // namespace pulsecol
