// Column softmax mass, bf16 inputs (Sec. 3.3, score equation):
//   s_{u,j} = (1/|G_u|) sum_{i in G_u} exp(z_ij - lse_i),  z_ij = q_i . k_j * scale,
// for the query groups G_u of a head (consecutive runs of group_size rows; one group = the
// whole head on the hot path),
// with the row log-sum-exp lse_i produced by the row pass (attn_bf16.hip, lse-only mode) and
// handed over in log2 units, so that p_ij = exp2(z_ij * scale * log2(e) - lse2_i).
//
// K-stationary: a workgroup owns 256 key columns (4 waves x 64); each wave keeps its K rows
// in registers as the MFMA B operand and streams every 64-row Q tile of the head through
// double-buffered LDS as the A operand.  In S[query][key] a lane owns one key column and its
// 16 registers are 16 query rows, so the column sum is an in-lane sum (four interleaved partial
// sums, each a short and a long accumulator) and the two half-waves meet once per group.
// exp2(z*c - lse_i*log2e) takes lse_i per register row, read from LDS four at a time.
// P never leaves fp32 and there are no floating-point atomics: the result is bit-identical
// from run to run.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int NTHREADS = 256;
constexpr int KEYS_PER_WG = 256;
constexpr int QT = 64;              // query rows per streamed tile
constexpr int FLUSH = 16;           // tiles between flushes of the short accumulator into the long one

template <int D>
__global__ void __launch_bounds__(NTHREADS) colmass_bf16_kernel(ScoreParams p) {
    constexpr int PIECES = D / 8;
    constexpr int KK = D / 16;
    constexpr int CH = QT * PIECES / NTHREADS;
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = QT * ROW_BYTES;

    __shared__ __attribute__((aligned(16))) unsigned char lds_q[2][TILE_BYTES];
    __shared__ __attribute__((aligned(16))) float lds_lse[2][QT];

    const int n = p.n;
    const int nkb = (n + KEYS_PER_WG - 1) / KEYS_PER_WG;
    int bh, kblk;
    if (!xcd_tile(blockIdx.x, nkb, p.batch * p.heads, &bh, &kblk)) return;
    const int b = bh / p.heads, h = bh - b * p.heads;
    const int64_t head_off = (int64_t)b * p.td.sb + (int64_t)h * p.td.sh;
    // grouped-query layout: query head h reads K/V head h / (heads / kv_heads)
    const int64_t kv_off = (int64_t)b * p.td_kv.sb + (int64_t)(h / (p.heads / p.kv_heads)) * p.td_kv.sh;
    const __bf16* __restrict__ Q = (const __bf16*)p.q + head_off;
    const __bf16* __restrict__ K = (const __bf16*)p.k + kv_off;
    const float* __restrict__ lse = p.lse + (int64_t)bh * n;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, lh = lane >> 5;
    const int key0 = kblk * KEYS_PER_WG + wave * 64;

    // ---- stationary K fragments: B operand, [key lq][d = kk*16 + 8*lh .. +7]
    bf16x8 kf[2][KK];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        int row = key0 + kb * 32 + lq;
        row = row < n ? row : n - 1;
        const __bf16* src = K + (int64_t)row * p.td_kv.sn + 8 * lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[kb][kk] = *(const bf16x8*)(src + kk * 16);
    }

    u32x4 stage[CH];
    float stage_lse = 0.f;
    // Each thread stages the same CH pieces of every tile: its pointers advance by one tile per
    // iteration (no per-tile row arithmetic); only a last, partial tile clamps its rows.
    const __bf16* qsrc[CH];
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = tid + NTHREADS * j;
        qsrc[j] = Q + (int64_t)(c / PIECES) * p.td.sn + (c % PIECES) * 8;
    }
    const int64_t tile_stride = (int64_t)QT * p.td.sn;
    const float* lse_src = lse + (tid < QT ? tid : 0);
    // (tiles are fetched in order: the pointers move on by one tile per call)
    auto fetch = [&](int t) {
        if (__builtin_expect((t + 1) * QT <= n, 1)) {
#pragma unroll
            for (int j = 0; j < CH; ++j) { stage[j] = *(const u32x4*)qsrc[j]; qsrc[j] += tile_stride; }
            if (tid < QT) stage_lse = *lse_src;
            lse_src += QT;
        } else {
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                const int c = tid + NTHREADS * j;
                int row = t * QT + c / PIECES;
                row = row < n ? row : n - 1;
                stage[j] = *(const u32x4*)(Q + (int64_t)row * p.td.sn + (c % PIECES) * 8);
            }
            if (tid < QT) {
                const int row = t * QT + tid;
                // rows past the end get +inf: exp2(z - inf) = 0, they add nothing to any column
                stage_lse = row < n ? lse[row] : INFINITY;
            }
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + NTHREADS * j;
            const int row = c / PIECES, piece = c % PIECES;
            *(u32x4*)(lds_q[buf] + row * ROW_BYTES + ((piece ^ swizzle_k<PIECES>(row)) << 4)) = stage[j];
        }
        if (tid < QT) lds_lse[buf][tid] = stage_lse;
    };

    const int ntiles = (n + QT - 1) / QT;
    fetch(0);
    commit(0);
    __syncthreads();

    const float c2 = p.scale * kLog2e;
    // per key block kb, this lane's key column; four interleaved partial sums keep the add chains independent
    float acc_short[2][4] = {}, acc_long[2][4] = {};

    // rows until the running query group ends (groups are multiples of 32 rows; one group: never)
    int rows_to_group_end = p.groups > 1 ? p.group_size : 0x7fffffff;
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) fetch(t + 1);

        f32x16 s[2][2];   // [kb][qb]: S[query rows of block qb][key lq of block kb]
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][qb][r] = 0.f;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int row = qb * 32 + lq;
            const unsigned char* rowp = lds_q[buf] + row * ROW_BYTES;
            const int sw = swizzle_k<PIECES>(row);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 qfrag = *(const bf16x8*)(rowp + (((2 * kk + lh) ^ sw) << 4));
                s[0][qb] = mfma_bf16(qfrag, kf[0][kk], s[0][qb]);
                s[1][qb] = mfma_bf16(qfrag, kf[1][kk], s[1][qb]);
            }
        }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            // register r holds query row qb*32 + 8*(r/4) + 4*lh + r%4: four consecutive rows per r/4
            f32x4 l2[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) l2[g] = *(const f32x4*)(&lds_lse[buf][qb * 32 + 8 * g + 4 * lh]);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc_short[kb][r & 3] += fast_exp2(__builtin_fmaf(s[kb][qb][r], c2, -l2[r >> 2][r & 3]));
            }
            if (qb == 1 && (t % FLUSH) == FLUSH - 1) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int c = 0; c < 4; ++c) { acc_long[kb][c] += acc_short[kb][c]; acc_short[kb][c] = 0.f; }
            }

            // ---- last rows of a query group (groups are multiples of 32 rows): add the two
            // half-waves (they hold the same key columns, other query rows), divide by the
            // group's size, store the group's score row, start over
            const int rows_done = t * QT + (qb + 1) * 32;
            rows_to_group_end -= 32;
            const bool group_end = (qb == 1 && t + 1 == ntiles) || (rows_to_group_end == 0 && rows_done < n);
            if (rows_to_group_end == 0) rows_to_group_end = p.group_size;
            if (group_end) {
                const int rows_seen = rows_done < n ? rows_done : n;
                const int u = p.groups > 1 ? (rows_seen - 1) / p.group_size : 0;
                const int g_first = p.groups > 1 ? u * p.group_size : 0;
                const int g_rows = rows_seen - g_first;
                const float inv = 1.0f / (float)g_rows;
                float* __restrict__ out = p.scores + ((int64_t)bh * p.groups + u) * n;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const float v = half_sum(((acc_long[kb][0] + acc_short[kb][0]) + (acc_long[kb][1] + acc_short[kb][1])) +
                                             ((acc_long[kb][2] + acc_short[kb][2]) + (acc_long[kb][3] + acc_short[kb][3])));
                    const int key = key0 + kb * 32 + lq;
                    if (lh == 0 && key < n) out[key] = v * inv;
#pragma unroll
                    for (int c = 0; c < 4; ++c) { acc_long[kb][c] = 0.f; acc_short[kb][c] = 0.f; }
                }
            }
        }

        if (t + 1 < ntiles) commit(buf ^ 1);
        __syncthreads();
    }
}

template <int D>
hipError_t launch(const ScoreParams& p, hipStream_t s) {
    const int nkb = (p.n + KEYS_PER_WG - 1) / KEYS_PER_WG;
    const int bh_pad = (p.batch * p.heads + 7) / 8 * 8;
    hipLaunchKernelGGL((colmass_bf16_kernel<D>), dim3(nkb * bh_pad), dim3(NTHREADS), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_colmass_bf16(const ScoreParams& p, int head_dim, hipStream_t s) {
    if (head_dim == 128) return launch<128>(p, s);
    if (head_dim == 64) return launch<64>(p, s);
    return hipErrorInvalidValue;
}

}  // namespace pulsecol
