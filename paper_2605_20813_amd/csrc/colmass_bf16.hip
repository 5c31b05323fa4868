// Column softmax mass, bf16 inputs (Sec. 3.3, score equation):
//   s_{u,j} = (1/|G_u|) sum_{i in G_u} exp(z_ij - lse_i),  z_ij = q_i . k_j * scale,
// for the query groups G_u of a head (consecutive runs of group_size rows; one group = the
// whole head on the hot path),
// with the row log-sum-exp lse_i produced by the row pass (attn_bf16.hip, lse-only mode) and
// handed over in log2 units, so that p_ij = exp2(z_ij * scale * log2(e) - lse2_i).
//
// K-stationary: a workgroup owns 256 key columns (4 waves x 64); each wave keeps its K rows
// in registers as the MFMA B operand and streams every 64-row Q tile of the head through
// LDS as the A operand: direct-to-LDS loads into one of three tile slots, issued two tiles ahead of
// their use, the rows' log-sum-exp values alongside.  In S[query][key] a lane owns one key column and its
// 16 registers are 16 query rows, so the column sum is an in-lane sum (four interleaved partial
// sums, each a short and a long accumulator) and the two half-waves meet once per group.
// exp2(z*c - lse_i*log2e) takes lse_i per register row, read from LDS four at a time.
// P never leaves fp32 and there are no floating-point atomics: the result is bit-identical
// from run to run.
// Ordinary compiler-scheduled code; the only hand-placed instructions are the waits and barriers
// that order the direct-to-LDS loads against the LDS reads.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

typedef unsigned char byte;

constexpr int NTHREADS = 256;
constexpr int KEYS_PER_WG = 256;
constexpr int QT = 64;              // query rows per streamed tile
constexpr int FLUSH = 16;           // tiles between flushes of the short accumulator into the long one

// s_waitcnt vmcnt(v) with the other counters left alone (gfx9 encoding: vmcnt in [3:0] and [15:14])
template <int v>
__device__ __forceinline__ void wait_vmcnt_at_most() {
    static_assert(v >= 0 && v < 64, "six bits");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (v & 0xF) | ((v & 0x30) << 10));
}
// nothing that touches memory moves across this point, neither in the compiler nor in its scheduler
__device__ __forceinline__ void memory_order_point() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// One Q tile and its 64 log-sum-exp values, this wave's share: CH loads of 64 x 16 bytes into the
// 1 KB chunks wave*CH + i of the slot (lane L lands at chunk byte 16*L = tile row chunk*RPC +
// L/PIECES, LDS piece L%PIECES, and fetches the global piece (L%PIECES) ^ swizzle(row) of its row:
// qoff[i] is that piece's byte offset from the tile's first row), and one load of 64 x 4 bytes for the
// tile's log-sum-exp values.  Rows past the end of the head read the last row instead; the caller
// gives them weight zero.
// (The slot pointer is a restrict parameter so that the loads carry an alias scope: the compiler
// then does not make LDS reads of the other slots wait for these loads.  A slot is ONE object,
// the tile followed by its log-sum-exp values: the compiler tells only a handful of such load
// targets apart, and beyond that number every LDS read waits for every load.)
template <int CH, int LSE_OFF>
__device__ __forceinline__ void issue_q_tile(byte* __restrict__ slot,
                                             const byte* __restrict__ Qg, const float* __restrict__ lse,
                                             int t, int n, uint32_t row_bytes, const int (&trow)[CH],
                                             const uint32_t (&qoff)[CH], int wave, int lane) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int row = t * QT + trow[i];
        // both factors are below 2^24 and the product below 2^32 (checked on the host)
        const uint32_t off = __umul24((uint32_t)(row < n ? row : n - 1), row_bytes) + qoff[i];
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Qg + off),
                                         (PULSECOL_LDS void*)(slot + (wave * CH + i) * 1024), 16, 0, 0);
    }
    // every wave brings all 64 values (the same bytes four times over): no branch in here, which
    // keeps the compiler's own bookkeeping of these loads exact
    const int row = t * QT + lane;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(lse + (uint32_t)(row < n ? row : n - 1)),
                                     (PULSECOL_LDS void*)(slot + LSE_OFF), 4, 0, 0);
}

template <int D>
__global__ void __launch_bounds__(NTHREADS) colmass_bf16_kernel(ScoreParams p) {
    constexpr int PIECES = D / 8;
    constexpr int KK = D / 16;
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = QT * ROW_BYTES;
    constexpr int RPC = 64 / PIECES;                  // tile rows per 1 KB chunk
    constexpr int CH = TILE_BYTES / 1024 / 4;         // chunks per wave and tile
    constexpr int VM_PER_TILE = CH + 1;               // vector memory operations a wave issues per tile
    static_assert(CH >= 1 && CH * 4 * 1024 == TILE_BYTES, "the waves' chunks cover the tile exactly");

    // one array per slot (tile, then its 64 log-sum-exp values): distinct objects, so that reads of
    // one slot are known not to touch another
    constexpr int SLOT_BYTES = TILE_BYTES + QT * 4;
    __shared__ __attribute__((aligned(1024))) byte lds_s0[SLOT_BYTES], lds_s1[SLOT_BYTES], lds_s2[SLOT_BYTES];

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
    const byte* __restrict__ Q = (const byte*)((const __bf16*)p.q + head_off);
    const __bf16* __restrict__ K = (const __bf16*)p.k + kv_off;
    const float* __restrict__ lse = p.lse + (int64_t)bh * p.n;
    const uint32_t row_bytes = (uint32_t)p.td.sn * 2u;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

    // ---- load geometry of this lane: chunk i of its wave covers tile row trow[i]
    int trow[CH];
    uint32_t qoff[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        trow[i] = (wave * CH + i) * RPC + lane / PIECES;
        qoff[i] = (uint32_t)((lane % PIECES) ^ swizzle_k<PIECES>(trow[i])) * 16u;
    }
    // ---- fragment addresses inside a slot: Q fragment kk of query block qb = tile row qb*32 + lq,
    // piece 2*kk + lh (rows 32 apart share a swizzle: the block is an instruction offset)
    uint32_t qaddr[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qaddr[kk] = (uint32_t)(lq * ROW_BYTES + (((2 * kk + lh) ^ swizzle_k<PIECES>(lq)) << 4));
    static_assert(PIECES <= 32, "rows 32 apart share a swizzle");

    const int ntiles = (n + QT - 1) / QT;
    const float c2 = p.scale * kLog2e;
    // per key block kb, this lane's key column; four interleaved partial sums keep the add chains independent
    float acc_short[2][4] = {}, acc_long[2][4] = {};

    // rows until the running query group ends (groups are multiples of 32 rows; one group: never)
    int rows_to_group_end = p.groups > 1 ? p.group_size : 0x7fffffff;

    auto compute_tile = [&](int t, const byte* __restrict__ slot) {
        const byte* qslot = slot;
        const float* lslot = (const float*)(slot + TILE_BYTES);
        f32x16 s[2][2];   // [kb][qb]: S[query rows of block qb][key lq of block kb]
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][qb][r] = 0.f;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 qfrag = *(const bf16x8*)(qslot + qb * 32 * ROW_BYTES + qaddr[kk]);
                s[0][qb] = mfma_bf16(qfrag, kf[0][kk], s[0][qb]);
                s[1][qb] = mfma_bf16(qfrag, kf[1][kk], s[1][qb]);
            }
        }
        // rows past the end of the head (last tile only) add nothing to any column
        const int valid = n - t * QT;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            // register r holds query row qb*32 + 8*(r/4) + 4*lh + r%4: four consecutive rows per r/4
            f32x4 l2[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) l2[g] = *(const f32x4*)(lslot + qb * 32 + 8 * g + 4 * lh);
            if (__builtin_expect(valid >= QT, 1)) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc_short[kb][r & 3] += fast_exp2(__builtin_fmaf(s[kb][qb][r], c2, -l2[r >> 2][r & 3]));
                }
            } else {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = fast_exp2(__builtin_fmaf(s[kb][qb][r], c2, -l2[r >> 2][r & 3]));
                        acc_short[kb][r & 3] += (qb * 32 + acc_row(r, lh) < valid) ? e : 0.f;
                    }
                }
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
                float* __restrict__ out = p.scores + ((int64_t)bh * p.groups + u) * p.n;
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
    };

    // ---- tiles 0 and 1 go out
    issue_q_tile<CH, TILE_BYTES>(lds_s0, Q, lse, 0, n, row_bytes, trow, qoff, wave, lane);
    issue_q_tile<CH, TILE_BYTES>(lds_s1, Q, lse, 1, n, row_bytes, trow, qoff, wave, lane);

    // Step t: tile t has landed in every wave once this wave's loads of tile t+1 are the only ones
    // it still may have in flight (vector memory completes in issue order, and whatever this step
    // issues comes later still) and all waves have said so at the barrier.  The barrier also tells
    // that every wave has finished reading tile t-1, whose slot the loads of tile t+2 now refill.
    // Loads are issued for tiles past the end as well (the head's last row, slots never read), so
    // the count in flight is the same at every step.
    auto step = [&](int t, const byte* __restrict__ cur, byte* __restrict__ fill) {
        wait_vmcnt_at_most<VM_PER_TILE>();
        memory_order_point();
        __builtin_amdgcn_s_barrier();
        memory_order_point();
        issue_q_tile<CH, TILE_BYTES>(fill, Q, lse, t + 2, n, row_bytes, trow, qoff, wave, lane);
        memory_order_point();
        compute_tile(t, cur);
    };
    for (int t = 0; t < ntiles; t += 3) {
        step(t, lds_s0, lds_s2);
        if (t + 1 >= ntiles) break;
        step(t + 1, lds_s1, lds_s0);
        if (t + 2 >= ntiles) break;
        step(t + 2, lds_s2, lds_s1);
    }
    wait_vmcnt_at_most<0>();        // nothing of this workgroup is on its way to LDS when it ends
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
