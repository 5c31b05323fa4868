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
#include <utility>

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
template <int CH>
__device__ __forceinline__ void issue_q_tile(byte* __restrict__ slot, byte* __restrict__ lse_slot,
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
                                     (PULSECOL_LDS void*)lse_slot, 4, 0, 0);
}

// LDS fragment reads as inline assembly with hand-placed waits.  (The compiler's own wait-count
// insertion drains lgkmcnt to zero in front of every LDS read while a direct-to-LDS load is in
// flight; LDS returns data in order, so "all but the N newest reads" is exact.)  For these loads the
// compiler knows neither the latency nor that the destination is written later: nothing may read
// the variable before the wait that covers it.  tests/test_asm_hazards.py checks the generated code.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128_at(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF>
__device__ __forceinline__ f32x4 lds_read_f32x4_at(uint32_t addr) {
    f32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(v) : "v"(addr), "n"(OFF));
    return v;
}
__device__ __forceinline__ void fence() { __builtin_amdgcn_sched_barrier(0); }
__device__ __forceinline__ uint32_t lds_address(const void* generic_lds_ptr) {
    return (uint32_t)(uintptr_t)(PULSECOL_LDS const void*)generic_lds_ptr;
}

// A tile is two blocks of 32 query rows; a block's scores take 2 * KK matrix instructions (KK
// fragments of the block's rows, each against the wave's two blocks of 32 keys) and 32 softmax
// weights per lane (fma, exp2, add each).  The two kinds of work are interleaved instruction by
// instruction: while the matrix instructions of a block issue, the weights of the block before it are
// formed, a few per matrix instruction, so that every wave's instruction stream feeds the matrix pipe
// and the vector pipe evenly.  (Written as two phases per block -- all matrix instructions, then all
// weights -- the two waves that share a SIMD fall into step: both in the matrix phase, then both in
// the vector phase, each pipe idle half of the time.)
template <int D>
struct ColWave {
    static constexpr int PIECES = D / 8;
    static constexpr int KK = D / 16;
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int TILE_BYTES = QT * ROW_BYTES;
    static constexpr int NPAIR = 2 * KK;                      // fragment reads (= pairs of matrix instructions) per tile
    static constexpr int AHEAD = KK / 2;                      // fragment reads in flight ahead of their use
    static constexpr int PER_SLOT = 16 / KK;                  // weights formed behind each matrix instruction
    static constexpr int LSE_RING = 4;                        // tiles whose log-sum-exp values LDS holds at a time
    static constexpr int LSE_BYTES = QT * 4;
    static constexpr int LSE_BASE = 3 * TILE_BYTES;           // the ring follows the three tile slots
    // Pairs between a log-sum-exp read and its first use.  LDS returns data in order, so the read has landed
    // once a fragment requested after it has: the fragment of the pair that uses it is requested AHEAD pairs
    // before that pair, hence AHEAD + 1.
    static constexpr int LEAD = AHEAD + 1;
    static_assert(KK == 4 || KK == 8, "head dimension 64 or 128");
    // The weights of a block are formed in register order, two key blocks per register: pair x of the KK pairs
    // of a block handles registers x * PER_SLOT .. +PER_SLOT-1, so the log-sum-exp group g (registers 4g .. 4g+3,
    // four consecutive query rows) is first needed in pair first_use(g), and is read LEAD pairs before that --
    // which for the first groups falls into the block before, while that block's own scores are still being
    // computed.
    static constexpr int first_use(int g) { return g * KK / 4; }
    // group read in the second slot of in-block pair x: for the block being consumed (>= 0), or -1
    static constexpr int lse_group_consumed(int x) {
        for (int g = 0; g < 4; ++g) if (first_use(g) - LEAD == x) return g;
        return -1;
    }
    // ... for the block being computed, which is consumed next (>= 0), or -1
    static constexpr int lse_group_computed(int x) {
        for (int g = 0; g < 4; ++g) if (first_use(g) - LEAD + KK == x) return g;
        return -1;
    }
    // log-sum-exp reads in pair q of a tile (FIRST: the head's first tile, whose first block has no block before
    // it to consume)
    template <bool FIRST>
    static constexpr int lse_reads(int q) {
        const int x = q % KK;
        return ((lse_group_consumed(x) >= 0 && !(FIRST && q < KK)) ? 1 : 0) + (lse_group_computed(x) >= 0 ? 1 : 0);
    }
    // LDS reads issued behind fragment p before pair p waits for it: the fragments requested ahead, and the
    // log-sum-exp reads of the pairs since fragment p was requested
    template <bool FIRST>
    static constexpr int newer(int p) {
        int c = (p + AHEAD - 1 < NPAIR - 1 ? p + AHEAD - 1 : NPAIR - 1) - p;
        for (int q = (p - AHEAD > 0 ? p - AHEAD : 0); q < p; ++q) c += lse_reads<FIRST>(q);
        return c;
    }
    static_assert(lse_group_consumed(0) < 0 || lse_group_computed(0) < 0, "one log-sum-exp read per pair at most");

    bf16x8 kf[2][KK];         // stationary K fragments: B operand, [key lq of block kb][d = kk*16 + 8*lh .. +7]
    f32x16 sb[2][2];          // scores [query block qb][key block kb]
    f32x4 lr[4];              // log-sum-exp (log2 units) of four query rows each, of the block whose weights are being formed
    float acc_short[2][4], acc_long[2][4];
    uint32_t qv[KK];          // LDS address of this lane's fragment kk in slot 0, first block
    uint32_t lv;              // LDS address of this lane's first log-sum-exp group in ring entry 0
    float c2;

    // weight e (0..31) of query block cq: register e / 2, key block e % 2
    __device__ __forceinline__ void weight(int cq, int e) {
        const int r = e >> 1, kb = e & 1;
        acc_short[kb][r & 3] += fast_exp2(__builtin_fmaf(sb[cq][kb][r], c2, -lr[r >> 2][r & 3]));
    }
    template <int OFF>
    __device__ __forceinline__ void read_lse(int g, uint32_t ring_addr) {
        // (one statement per group so that the destination is a whole variable)
        if (g == 0) lr[0] = lds_read_f32x4_at<LSE_BASE + OFF>(ring_addr);
        if (g == 1) lr[1] = lds_read_f32x4_at<LSE_BASE + OFF + 32>(ring_addr);
        if (g == 2) lr[2] = lds_read_f32x4_at<LSE_BASE + OFF + 64>(ring_addr);
        if (g == 3) lr[3] = lds_read_f32x4_at<LSE_BASE + OFF + 96>(ring_addr);
    }

    // Pair P of the tile in slot S: two matrix instructions on fragment P, the request for fragment P + AHEAD,
    // at most one log-sum-exp read, and (CONSUME) 2 * PER_SLOT weights of the block before.  ring_cur / ring_prev:
    // LDS addresses (lane's first group) of the log-sum-exp values of this tile and of the tile before.
    template <int S, int P, bool FIRST>
    __device__ __forceinline__ void pair(bf16x8 (&fr)[NPAIR], uint32_t ring_cur, uint32_t ring_prev) {
        constexpr int qb = P / KK, x = P % KK, cq = 1 - qb;
        constexpr bool CONSUME = !(FIRST && qb == 0);
        constexpr int SLOT = S * TILE_BYTES;
        asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(fr[P]) : "n"(newer<FIRST>(P)));
        if constexpr (x == 0) {
            f32x16 zero;
#pragma unroll
            for (int r = 0; r < 16; ++r) zero[r] = 0.f;
            sb[qb][0] = mfma_bf16(fr[P], kf[0][x], zero);
        } else {
            sb[qb][0] = mfma_bf16(fr[P], kf[0][x], sb[qb][0]);
        }
        fence();
        if constexpr (P + AHEAD < NPAIR) {
            constexpr int Q = P + AHEAD;
            fr[Q] = lds_read_b128_at<SLOT + (Q / KK) * 32 * ROW_BYTES>(qv[Q % KK]);
        }
        if constexpr (CONSUME) {
#pragma unroll
            for (int i = 0; i < PER_SLOT; ++i) weight(cq, x * 2 * PER_SLOT + i);
        }
        fence();
        if constexpr (x == 0) {
            f32x16 zero;
#pragma unroll
            for (int r = 0; r < 16; ++r) zero[r] = 0.f;
            sb[qb][1] = mfma_bf16(fr[P], kf[1][x], zero);
        } else {
            sb[qb][1] = mfma_bf16(fr[P], kf[1][x], sb[qb][1]);
        }
        fence();
        // the block being consumed: second block of the tile before (qb == 0) or first block of this tile
        if constexpr (CONSUME && lse_group_consumed(x) >= 0) {
            if constexpr (qb == 0) read_lse<32 * 4>(lse_group_consumed(x), ring_prev);
            else read_lse<0>(lse_group_consumed(x), ring_cur);
        }
        // the block being computed, whose weights the next block's pairs will form
        if constexpr (lse_group_computed(x) >= 0) read_lse<qb * 32 * 4>(lse_group_computed(x), ring_cur);
        if constexpr (CONSUME) {
#pragma unroll
            for (int i = 0; i < PER_SLOT; ++i) weight(cq, x * 2 * PER_SLOT + PER_SLOT + i);
        }
        fence();
    }
    template <int S, int P0, bool FIRST, int... Ps>
    __device__ __forceinline__ void pairs(bf16x8 (&fr)[NPAIR], uint32_t ring_cur, uint32_t ring_prev, std::integer_sequence<int, Ps...>) {
        (pair<S, P0 + Ps, FIRST>(fr, ring_cur, ring_prev), ...);
    }
    // the first AHEAD fragments of a tile (behind the barrier that says the tile has landed)
    template <int S>
    __device__ __forceinline__ void request_first(bf16x8 (&fr)[NPAIR]) {
        static_assert(AHEAD == 2 || AHEAD == 4, "written out for two and four");
        fr[0] = lds_read_b128_at<S * TILE_BYTES>(qv[0]);
        fr[1] = lds_read_b128_at<S * TILE_BYTES>(qv[1]);
        if constexpr (AHEAD == 4) {
            fr[2] = lds_read_b128_at<S * TILE_BYTES>(qv[2]);
            fr[3] = lds_read_b128_at<S * TILE_BYTES>(qv[3]);
        }
    }
    // The weights of a block outside the interleave (the last full block of a head): the groups that the
    // interleave would have read in the following block are read here.
    __device__ __forceinline__ void weights_alone(int cq, uint32_t ring_addr) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (first_use(g) - LEAD >= 0) {
                if (g == 1) lr[1] = lds_read_f32x4_at<LSE_BASE + 32 * 4 + 32>(ring_addr);
                if (g == 2) lr[2] = lds_read_f32x4_at<LSE_BASE + 32 * 4 + 64>(ring_addr);
                if (g == 3) lr[3] = lds_read_f32x4_at<LSE_BASE + 32 * 4 + 96>(ring_addr);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(lr[0]), "+v"(lr[1]), "+v"(lr[2]), "+v"(lr[3]));
#pragma unroll
        for (int e = 0; e < 32; ++e) weight(cq, e);
    }
};

template <int D>
__global__ void __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2)))
colmass_bf16_kernel(ScoreParams p) {
    using W = ColWave<D>;
    constexpr int PIECES = W::PIECES;
    constexpr int KK = W::KK;
    constexpr int ROW_BYTES = W::ROW_BYTES;
    constexpr int TILE_BYTES = W::TILE_BYTES;
    constexpr int NPAIR = W::NPAIR;
    constexpr int RPC = 64 / PIECES;                  // tile rows per 1 KB chunk
    constexpr int CH = TILE_BYTES / 1024 / 4;         // chunks per wave and tile
    constexpr int VM_PER_TILE = CH + 1;               // vector memory operations a wave issues per tile
    static_assert(CH >= 1 && CH * 4 * 1024 == TILE_BYTES, "the waves' chunks cover the tile exactly");

    // ONE array: three tile slots, then a ring of four tiles' log-sum-exp values (64 each).  Slot and block
    // are instruction offsets of the fragment reads.  The ring is one entry longer than the slots because the
    // weights of a tile's second block are formed during the first block of the next tile, after the barrier
    // that frees the tile's slot.
    __shared__ __attribute__((aligned(1024))) byte lds_all[3 * TILE_BYTES + W::LSE_RING * W::LSE_BYTES];

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

    W w;
    // ---- stationary K fragments
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        int row = key0 + kb * 32 + lq;
        row = row < n ? row : n - 1;
        const __bf16* src = K + (int64_t)row * p.td_kv.sn + 8 * lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) w.kf[kb][kk] = *(const bf16x8*)(src + kk * 16);
    }

    // ---- load geometry of this lane: chunk i of its wave covers tile row trow[i]
    int trow[CH];
    uint32_t qoff[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        trow[i] = (wave * CH + i) * RPC + lane / PIECES;
        qoff[i] = (uint32_t)((lane % PIECES) ^ swizzle_k<PIECES>(trow[i])) * 16u;
    }
    // ---- fragment addresses: Q fragment kk of query block qb = tile row qb*32 + lq, piece 2*kk + lh
    // (rows 32 apart share a swizzle: the block is an instruction offset); log-sum-exp group g of block qb =
    // rows qb*32 + 8*g + 4*lh .. +3
    const uint32_t lds0 = lds_address(lds_all);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) w.qv[kk] = lds0 + (uint32_t)(lq * ROW_BYTES + (((2 * kk + lh) ^ swizzle_k<PIECES>(lq)) << 4));
    w.lv = lds0 + (uint32_t)(16 * lh);
    static_assert(PIECES <= 32, "rows 32 apart share a swizzle");

    const int nfull = n / QT;               // whole tiles: the interleaved steps; a ragged last tile is computed apart
    const int ntiles = (n + QT - 1) / QT;
    w.c2 = p.scale * kLog2e;
    // per key block kb, this lane's key column; four interleaved partial sums keep the add chains independent
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int c = 0; c < 4; ++c) { w.acc_short[kb][c] = 0.f; w.acc_long[kb][c] = 0.f; }

    // rows until the running query group ends (groups are multiples of 32 rows; one group: never)
    int rows_to_group_end = p.groups > 1 ? p.group_size : 0x7fffffff;

    // What follows the weights of block qb of tile t: the periodic flush of the short accumulators and, at
    // the last rows of a query group (groups are multiples of 32 rows), the group's score row: add the two
    // half-waves (they hold the same key columns, other query rows), divide by the group's size, store,
    // start over.
    auto block_done = [&](int t, int qb) {
        if (qb == 1 && (t % FLUSH) == FLUSH - 1) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int c = 0; c < 4; ++c) { w.acc_long[kb][c] += w.acc_short[kb][c]; w.acc_short[kb][c] = 0.f; }
        }
        const int rows_done = t * QT + (qb + 1) * 32;
        rows_to_group_end -= 32;
        const bool group_end = (rows_done >= n) || (rows_to_group_end == 0 && rows_done < n);
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
                const float v = half_sum(((w.acc_long[kb][0] + w.acc_short[kb][0]) + (w.acc_long[kb][1] + w.acc_short[kb][1])) +
                                         ((w.acc_long[kb][2] + w.acc_short[kb][2]) + (w.acc_long[kb][3] + w.acc_short[kb][3])));
                const int key = key0 + kb * 32 + lq;
                if (lh == 0 && key < n) out[key] = v * inv;
#pragma unroll
                for (int c = 0; c < 4; ++c) { w.acc_long[kb][c] = 0.f; w.acc_short[kb][c] = 0.f; }
            }
        }
    };
    auto ring_of = [&](int t) { return w.lv + (uint32_t)((t & (W::LSE_RING - 1)) * W::LSE_BYTES); };
    auto issue = [&](int t) {
        issue_q_tile<CH>(lds_all + (t % 3) * TILE_BYTES, lds_all + W::LSE_BASE + (t & (W::LSE_RING - 1)) * W::LSE_BYTES,
                         Q, lse, t, n, row_bytes, trow, qoff, wave, lane);
    };

    // ---- tiles 0 and 1 go out
    issue(0);
    issue(1);

    // Step t (tile t in slot S = t % 3): tile t has landed in every wave once this wave's loads of tile t+1 are
    // the only ones it still may have in flight (vector memory completes in issue order, and whatever this
    // step issues comes later still) and all waves have said so at the barrier.  The barrier also tells that
    // every wave is done with the slot of tile t-1 and with the log-sum-exp values of tile t-2, which the
    // loads of tile t+2 now replace.  Loads are issued for tiles past the end as well (the head's last row,
    // slots never read), so the count in flight is the same at every step.
    auto step = [&](auto slot_c, auto first_c, int t) {
        constexpr int S = decltype(slot_c)::value;
        constexpr bool FIRST = decltype(first_c)::value;     // no block before this tile's first: nothing to consume
        wait_vmcnt_at_most<VM_PER_TILE>();
        memory_order_point();
        __builtin_amdgcn_s_barrier();
        memory_order_point();
        bf16x8 fr[NPAIR];
        w.template request_first<S>(fr);
        memory_order_point();
        issue(t + 2);
        memory_order_point();
        const uint32_t ring_cur = ring_of(t), ring_prev = ring_of(t - 1);
        // first block of the tile, with the weights of the second block of the tile before
        w.template pairs<S, 0, FIRST>(fr, ring_cur, ring_prev, std::make_integer_sequence<int, KK>{});
        if (!FIRST) block_done(t - 1, 1);
        // second block, with the weights of the first
        w.template pairs<S, KK, FIRST>(fr, ring_cur, ring_prev, std::make_integer_sequence<int, KK>{});
        block_done(t, 0);
    };
    if (nfull > 0) {
        step(std::integral_constant<int, 0>{}, std::true_type{}, 0);
        for (int t = 1; t < nfull; t += 3) {
            step(std::integral_constant<int, 1>{}, std::false_type{}, t);
            if (t + 1 >= nfull) break;
            step(std::integral_constant<int, 2>{}, std::false_type{}, t + 1);
            if (t + 2 >= nfull) break;
            step(std::integral_constant<int, 0>{}, std::false_type{}, t + 2);
        }
        // the weights of the last whole tile's second block, on their own
        w.weights_alone(1, ring_of(nfull - 1));
        block_done(nfull - 1, 1);
    }
    wait_vmcnt_at_most<0>();
    if (nfull < ntiles) {
        // ---- a ragged last tile, in plain code: rows past the end of the head add nothing to any column
        memory_order_point();
        __builtin_amdgcn_s_barrier();
        memory_order_point();
        const int t = nfull;
        const byte* qslot = lds_all + (t % 3) * TILE_BYTES;
        const float* lslot = (const float*)(lds_all + W::LSE_BASE + (t & (W::LSE_RING - 1)) * W::LSE_BYTES);
        const int valid = n - t * QT;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (qb * 32 >= valid) break;
            f32x16 s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 qfrag = *(const bf16x8*)(qslot + qb * 32 * ROW_BYTES + (w.qv[kk] - lds0));
                s[0] = mfma_bf16(qfrag, w.kf[0][kk], s[0]);
                s[1] = mfma_bf16(qfrag, w.kf[1][kk], s[1]);
            }
            f32x4 l2[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) l2[g] = *(const f32x4*)(lslot + qb * 32 + 8 * g + 4 * lh);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const float e = fast_exp2(__builtin_fmaf(s[kb][r], w.c2, -l2[r >> 2][r & 3]));
                    w.acc_short[kb][r & 3] += (qb * 32 + acc_row(r, lh) < valid) ? e : 0.f;
                }
            }
            block_done(t, qb);
        }
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
