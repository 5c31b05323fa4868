// Exact per-row top-k of fp32 scores (Sec. 3.3, TopK equation), gfx950.
//
// One workgroup per score row.  The k-th largest value is found by a radix select on the
// order-preserving integer image of the floats (LDS histograms, most significant digit first);
// then every element above the threshold, plus the first `need` elements equal to it in index
// order, is written at the position a ballot/popcount prefix sum gives it.  The output is
// therefore ascending in column index and, among equal scores, the lower index wins.  Integer
// work only: results are exact and identical from run to run.
//
// Two kernels: topk_rows_kernel reads the row once and keeps it in registers (rows of up to
// 65536 elements, a multiple of 4, 16-byte aligned: every shape of the paper's workloads; a
// resident grid whose workgroups walk over the rows and fetch the next row while writing out);
// topk_kernel streams the row from memory five times and takes everything else.
#include <type_traits>
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int TK_THREADS = 1024;
constexpr int TK_WAVES = TK_THREADS / 64;

// floats -> unsigned keys with the same order (larger float <=> larger key)
__device__ __forceinline__ uint32_t order_key_of_bits(uint32_t u) {
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ uint32_t order_key(float x) { return order_key_of_bits(__float_as_uint(x)); }

// Elements and kept columns of score row `row`: the context's n and k, or (variable-length batches)
// the length of the row's batch element and its kept count; a row whose query group lies wholly in
// the padding of its element has neither (0, 0).
__device__ __forceinline__ void row_geometry(const TopkParams& p, int row, int& n_row, int& k_row) {
    n_row = p.n;
    k_row = p.k;
    if (p.varlen != nullptr) {
        const int b = row / p.rows_per_batch;
        const int u = row % p.groups;                   // rows are ordered [batch, head, group]
        const int len = p.varlen[b];
        const int kept = p.varlen[p.batch + b];
        const bool padding = p.groups > 1 && u * p.group_size >= len;
        n_row = padding ? 0 : len;
        k_row = padding ? 0 : (kept < p.k ? kept : p.k);
    }
}
// entries [from, k) of an output row are padding: -1
__device__ __forceinline__ void pad_row(int32_t* __restrict__ out, int from, int k, int tid) {
    for (int j = from + tid; j < k; j += TK_THREADS) out[j] = -1;
}

__global__ void __launch_bounds__(TK_THREADS) topk_kernel(TopkParams p) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_prefix, sh_need;
    __shared__ uint32_t wave_cnt[2][TK_WAVES];

    const int row = blockIdx.x;
    const float* __restrict__ s = p.scores + (int64_t)row * p.stride;
    int32_t* __restrict__ out = p.idx + (int64_t)row * p.k;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    int n, k_row;
    row_geometry(p, row, n, k_row);
    pad_row(out, k_row, p.k, tid);
    if (k_row == 0) return;                             // uniform: the whole workgroup

    // ---- radix select: after the loop `prefix` is the key of the k-th largest element and
    //      `need` how many elements equal to it belong to the top-k
    uint32_t prefix = 0, mask = 0, need = (uint32_t)k_row;
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
            if (pos < (uint32_t)k_row) out[pos] = j;     // guard: holds by construction
        }
        eq_seen += eq_total;
        out_pos += sel_total;
        // wave_cnt[0] is rewritten only after the next barrier pair: the loop's first barrier
        // of the next iteration comes after every wave has read wave_cnt[1], and wave_cnt[0]
        // was last read before this iteration's second barrier.
    }
}


// ---- rows that fit the registers of one workgroup (n <= 65536, n % 4 == 0, 16-byte aligned):
// the row is read from memory ONCE, as order keys, 4 * V4 per thread; everything after that works
// on registers.  Wave w owns the contiguous segment [w*SEG, (w+1)*SEG), SEG = 256 * V4; its load
// instruction i covers 256 consecutive elements, lane l the four elements seg0 + i*256 + 4*l .. +3
// (one 16-byte load per lane, 1 KB contiguous per instruction).
//
// Radix select with 13-bit digits, starting at the highest bit in which the row's keys differ at
// all (scores of one row share their sign and most of their exponent: a fixed first digit would
// send every element to the same histogram bin, and same-address LDS atomics serialise): at most
// three passes, 8192 bins.  Then the ordered compaction: every wave knows from the per-wave
// totals where its output starts, and places its elements with ballots alone (no barrier inside).
//
// A workgroup walks over a run of consecutive rows (the query groups of one head, one after the
// other), and the k-th largest score of a row is close to that of the row before (a few percent).
// From the second row on, the select therefore starts from an estimate: every fourth key of the
// row is counted against the last row's threshold and a level below and above it, and the level
// that a quarter of k keys would exceed is interpolated.  One sweep then counts the keys above a
// bracket around the estimate and collects the keys inside it, wave by wave, into the candidate
// list.  If the k-th largest key lies inside (count above < k <= count above + list size, and no
// wave's share of the list overflowed), the radix passes run over the list alone and the full
// first pass and the list-building sweep are saved; if not, the row takes the full path.  Either
// way the threshold is the exact k-th largest key: the estimate only decides how it is found.
// The bracket's half width follows the estimate's error (see below); it doubles after a miss and
// halves after an overflow.
constexpr int TKR_DIGIT = 13;
constexpr int TKR_BINS = 1 << TKR_DIGIT;
constexpr int TKR_BPT = TKR_BINS / TK_THREADS;       // histogram bins per thread

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { const uint32_t o = __shfl_xor(v, d); v = o > v ? o : v; }
    return v;
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { const uint32_t o = __shfl_xor(v, d); v = o < v ? o : v; }
    return v;
}
// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (no LDS round trips: a
// shuffle goes through the LDS crossbar, and a row's select has a dozen reductions on its serial path):
// four shifts inside the rows of 16 lanes, then lane 15 of rows 0 and 2 onto rows 1 and 3, then lane 31
// onto rows 2 and 3.
__device__ __forceinline__ uint32_t wave_prefix_sum_u32(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);      // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);      // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);      // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);      // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);     // row_bcast:15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);     // row_bcast:31 -> rows 2, 3
    return v;
}
// the sum over the wave, the same in every lane (a scalar)
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_prefix_sum_u32(v), 63);
}

// VARLEN: variable-length batches (rows of their own length and kept count, rows of padding); the
// fixed-length instantiation carries none of that bookkeeping, which costs it registers it does not have.
constexpr int TKR_WAVE_CAND = 256;                   // a wave's share of the candidate list on the bracket path
constexpr int TKR_FEW = 32;                          // keys that one wave ranks directly instead of another radix pass
constexpr uint32_t TKR_PROBE = 1u << 20;             // distance of the probe levels from the last row's threshold, in key units
constexpr uint32_t TKR_HALF_WIDTH_MIN = 1u << 12, TKR_HALF_WIDTH_MAX = 1u << 22;

template <int V4, bool VARLEN>
__global__ void __launch_bounds__(TK_THREADS) topk_rows_kernel(TopkParams p, int rows_per_wg) {
    constexpr int SEG = 256 * V4;
    static_assert(TKR_BPT * TK_THREADS == TKR_BINS && TKR_BPT % 4 == 0, "whole 16-byte groups of bins per thread");
    __shared__ __attribute__((aligned(16))) uint32_t hist[TKR_BINS];
    __shared__ uint32_t wave_a[TK_WAVES], wave_b[TK_WAVES];
    __shared__ uint32_t sh_bin, sh_need, sh_cnt, sh_ncand;
    // the elements that fell into the first pass's bin, if they are few enough: the later passes
    // then walk over this list instead of sweeping the registers again
    constexpr int CAND_MAX = 4096;
    static_assert(TKR_WAVE_CAND * TK_WAVES == CAND_MAX, "the waves' shares make up the list");
    __shared__ uint32_t cand[CAND_MAX];
    __shared__ uint32_t seg_cnt[TK_WAVES];             // bracket path: candidates in each wave's share
    __shared__ uint32_t few[TKR_FEW];                  // the last keys of a select, ranked directly

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int first = wave * SEG + lane * 4;          // this lane's first element
    // load instructions of this lane that reach into a row of n_row elements (the row stride p.n is a
    // multiple of 4, so a 16-byte load never leaves the row's storage; with a fixed length a lane's four
    // elements are inside or outside together, with variable lengths the last group may straddle the end)
    auto groups_inside = [&](int n_row) {
        return first >= n_row ? 0 : ((n_row - first + 255) / 256 < V4 ? (n_row - first + 255) / 256 : V4);
    };
    const int row_begin = blockIdx.x * rows_per_wg;
    const int row_end = row_begin + rows_per_wg < p.rows ? row_begin + rows_per_wg : p.rows;
    if (row_begin >= row_end) return;                  // uniform (the grid is sized so that it does not happen)
    int n = p.n, k_row = p.k;
    if constexpr (VARLEN) row_geometry(p, row_begin, n, k_row);
    int nv = groups_inside(n);
    // the last row's threshold key and the bracket's half width, in key units (2^17: about one percent of a score)
    uint32_t guess = 0u, half_width = 1u << 17;
    bool have_guess = false;

    // The workgroup walks over rows row_begin .. row_end - 1; the scores of the next row are
    // requested while the running row is written out (each register group as soon as the
    // compaction is done with it), so that only the first row's load is waited for in full.
    // key[][] holds the row: as float bit patterns from the load until the row's turn comes, as
    // order keys from then on
    uint32_t key[V4][4];
    const uint32_t* __restrict__ bits = (const uint32_t*)p.scores;
#pragma unroll
    for (int i = 0; i < V4; ++i) {
        u32x4 v = {0u, 0u, 0u, 0u};                          // outside the row: never looked at, every use is guarded by nv
        if (i < nv) v = *(const u32x4*)(bits + (int64_t)row_begin * p.stride + first + i * 256);
#pragma unroll
        for (int c = 0; c < 4; ++c) key[i][c] = v[c];
    }

  for (int row = row_begin; row < row_end; ++row) {
    int32_t* __restrict__ out = p.idx + (int64_t)row * p.k;
    // The thread's number, hidden from the compiler's loop-invariant hoisting once per row: it would compute
    // everything that follows from it (the 64 column numbers of the lane, LDS addresses, lane masks) in front of
    // the loop and, with no registers for them, keep them in scratch.
    int tid_hidden = threadIdx.x;
    asm volatile("" : "+v"(tid_hidden));
    const int tid = tid_hidden;
    const int lane = tid & 63, wave = tid >> 6;
    const int first_r = wave * SEG + lane * 4;
    const bool more = row + 1 < row_end;
    const uint32_t* __restrict__ next_bits = bits + (int64_t)(more ? row + 1 : row) * p.stride + first_r;
    // this row's geometry was settled when its load was issued; the next row's decides what is fetched for it
    int n_next = p.n, k_next = p.k;
    if constexpr (VARLEN) { if (more) row_geometry(p, row + 1, n_next, k_next); }
    const int nv_next = more ? (VARLEN ? groups_inside(n_next) : nv) : 0;
    if constexpr (VARLEN) pad_row(out, k_row, p.k, tid);
    if (VARLEN && k_row == 0) {
        // a row of padding (uniform over the workgroup): nothing to select, only the next row's load
#pragma unroll
        for (int i = 0; i < V4; ++i) {
            if (i < nv_next) {
                const u32x4 v = *(const u32x4*)(next_bits + i * 256);
#pragma unroll
                for (int c = 0; c < 4; ++c) key[i][c] = v[c];
            }
        }
        n = n_next; k_row = k_next; nv = nv_next;
        continue;
    }
    const bool straddles = VARLEN && (n & 3) != 0;    // uniform: variable-length rows only

#pragma unroll
    for (int i = 0; i < V4; ++i) {
#pragma unroll
        for (int c = 0; c < 4; ++c) key[i][c] = order_key_of_bits(key[i][c]);
    }
    // bits of a ballot that belong to the lanes in front of this one, counted on top of `acc`
    auto count_before = [](uint64_t ballot, uint32_t acc) {
        return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, acc));
    };

    // ---- the bracket around the last row's threshold (see the head of this kernel)
    uint32_t prefix = 0u, need = (uint32_t)k_row;
    int hi = -1;
    bool bracketed = false;
    uint32_t above_wave = 0u;                          // bracket path: this wave's keys above the bracket
    uint32_t listed_last = 0u;                         // ... and the row's
    uint32_t est = 0u;
    bool placed = false;
    if (!VARLEN && have_guess) {
        // (1) Where this row's k-th largest key lies relative to the last row's: every fourth key of the row is
        // counted against three levels, the last threshold and a million key units (about 8 % of a score) below
        // and above it.  Between the two levels that enclose a quarter of k, the level is interpolated on the
        // logarithm of the counts: the number of keys above a level falls off roughly exponentially with the
        // level near the top of a row, and a straight line between the counts is off by a fifth of the interval.
        const uint32_t g_lo = guess > TKR_PROBE ? guess - TKR_PROBE : 0u;
        const uint32_t g_hi = guess < 0xFFFFFFFFu - TKR_PROBE ? guess + TKR_PROBE : 0xFFFFFFFFu;
        uint32_t cnt = 0u, cnt_mid = 0u;               // cnt: keys above g_lo in the low half, above g_hi in the high half
#pragma unroll
        for (int i = 0; i < V4; ++i) {
            if (i < nv) {
                cnt += (key[i][0] > g_lo ? 1u : 0u) + (key[i][0] > g_hi ? 0x10000u : 0u);
                cnt_mid += key[i][0] > guess ? 1u : 0u;
            }
        }
        cnt = wave_sum_u32(cnt);                       // at most 16 * 64 per wave and half, 16384 per row
        cnt_mid = wave_sum_u32(cnt_mid);
        if (lane == 0) { wave_a[wave] = cnt; wave_b[wave] = cnt_mid; }
        __syncthreads();
        uint32_t all = 0u, all_mid = 0u;
#pragma unroll
        for (int w = 0; w < TK_WAVES; ++w) { all += wave_a[w]; all_mid += wave_b[w]; }
        __syncthreads();                               // wave_a / wave_b are reused below
        const uint32_t c_lo = 4u * (all & 0xFFFFu), c_hi = 4u * (all >> 16), c_mid = 4u * all_mid;
        if (c_lo >= (uint32_t)k_row && (uint32_t)k_row > c_hi) {
            const bool upper = c_mid >= (uint32_t)k_row;           // the level lies between the last threshold and g_hi
            const uint32_t from = upper ? guess : g_lo, to = upper ? g_hi : guess;
            const float a = (float)(upper ? c_mid : c_lo), b = (float)(upper ? c_hi : c_mid);
            const float la = __log2f(a), lb = __log2f(b > 0.5f ? b : 0.5f), lk = __log2f((float)k_row);
            const float frac = la > lb ? (la - lk) / (la - lb) : 0.f;
            est = __builtin_amdgcn_readfirstlane(from + (uint32_t)(frac * (float)(to - from)));      // (uniform: kept in a scalar register)
            placed = true;
        }
    }
    if (placed) {
        // (2) the bracket around the estimate
        const uint32_t lo_key = est > half_width ? est - half_width : 0u;
        const uint32_t hi_key = est < 0xFFFFFFFFu - half_width ? est + half_width : 0xFFFFFFFFu;
        const uint32_t span = hi_key - lo_key;         // > 0: half_width >= 1
        uint32_t above = 0u, off = 0u;                 // off: candidates of this wave so far (uniform)
#pragma unroll
        for (int i = 0; i < V4; ++i) {
            if (i < nv) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t kx = key[i][c];
                    above += kx > hi_key ? 1u : 0u;
                    const bool hit = kx - lo_key <= span;
                    const uint64_t hit_b = __ballot(hit);
                    if (hit_b != 0ull) {
                        const uint32_t at = count_before(hit_b, off);
                        if (hit && at < (uint32_t)TKR_WAVE_CAND) cand[wave * TKR_WAVE_CAND + at] = kx;
                        off += __popcll(hit_b);
                    }
                }
            }
        }
        above = wave_sum_u32(above);
        if (lane == 0) { wave_a[wave] = above; seg_cnt[wave] = off; }
        __syncthreads();
        uint32_t all_above = 0u, all_listed = 0u;
        bool overflow = false;
#pragma unroll
        for (int w = 0; w < TK_WAVES; ++w) {
            all_above += wave_a[w];
            all_listed += seg_cnt[w];
            overflow = overflow || seg_cnt[w] > (uint32_t)TKR_WAVE_CAND;
        }
        __syncthreads();                               // wave_a is reused below
        listed_last = all_listed;
        if (!overflow && all_above < (uint32_t)k_row && (uint32_t)k_row <= all_above + all_listed) {
            bracketed = true;
            above_wave = above;
            need = (uint32_t)k_row - all_above;
            // every key on the list agrees with the bracket's ends above their highest differing bit
            hi = 31 - __clz((int)(lo_key ^ hi_key));
            prefix = hi >= 31 ? 0u : ((lo_key >> (hi + 1)) << (hi + 1));
        } else if (overflow) {
            half_width = half_width > 2u * TKR_HALF_WIDTH_MIN ? half_width >> 1 : TKR_HALF_WIDTH_MIN;
        } else {
            half_width = half_width < TKR_HALF_WIDTH_MAX ? half_width << 1 : TKR_HALF_WIDTH_MAX;
        }
    }

    if (!bracketed) {
        uint32_t kmax = 0u, kmin = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 0; i < V4; ++i) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (i < nv && (!straddles || first_r + i * 256 + c < n)) {
                    kmax = key[i][c] > kmax ? key[i][c] : kmax;
                    kmin = key[i][c] < kmin ? key[i][c] : kmin;
                }
            }
        }
        kmax = wave_max_u32(kmax);
        kmin = wave_min_u32(kmin);
        if (lane == 0) { wave_a[wave] = kmax; wave_b[wave] = kmin; }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < TK_WAVES; ++w) {
            kmax = wave_a[w] > kmax ? wave_a[w] : kmax;
            kmin = wave_b[w] < kmin ? wave_b[w] : kmin;
        }
        __syncthreads();                                   // wave_a / wave_b are reused below
        if (straddles) {
            // the elements a 16-byte load brought in from behind the row's end take the row's smallest key: they
            // follow every real element in index order, so the selection (k_row <= n real elements) never reaches them
#pragma unroll
            for (int i = 0; i < V4; ++i) {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (i < nv && first_r + i * 256 + c >= n) key[i][c] = kmin;
            }
        }
        // Bits above `hi` are the same in every key of the row.
        hi = 31 - __clz((int)(kmax ^ kmin));           // -1 if all keys are equal
        prefix = hi >= 31 ? 0u : ((kmax >> (hi + 1)) << (hi + 1));
    }

    // ---- radix select: afterwards `prefix` is the key of the k-th largest element and `need`
    //      how many elements equal to it belong to the top-k.
    // register groups of this lane that still hold an element matching the prefix: all of them in
    // the first pass, next to none later (a bin of the first pass holds n/8192 elements on
    // average), so that the later passes skip almost all of their work, whole waves at a time
    uint32_t live = nv >= 32 ? 0xFFFFFFFFu : ((1u << nv) - 1u);
    bool first_pass = !bracketed, listed = bracketed;
    uint32_t ncand = 0;
    while (hi >= 0) {
        const int width = hi + 1 < TKR_DIGIT ? hi + 1 : TKR_DIGIT;
        const int shift = hi + 1 - width;
#pragma unroll
        for (int b = 0; b < TKR_BPT / 4; ++b) *(u32x4*)&hist[TKR_BPT * tid + 4 * b] = u32x4{0u, 0u, 0u, 0u};
        __syncthreads();
        const uint32_t limit = 1u << width;
        if (first_pass) {
            // every key agrees with the prefix above the first digit by construction: no test per
            // element (a test per element is a predicated region per element, and those, not the
            // atomics, are what a sweep over the registers costs)
#pragma unroll
            for (int i = 0; i < V4; ++i) {
                if (i < nv) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) atomicAdd(&hist[(key[i][c] ^ prefix) >> shift], 1u);
                }
            }
        } else if (bracketed) {
            // the list lies in the waves' shares, seg_cnt[w] entries at the front of share w
#pragma unroll
            for (int j = tid; j < CAND_MAX; j += TK_THREADS) {
                if ((uint32_t)(j % TKR_WAVE_CAND) < seg_cnt[j / TKR_WAVE_CAND]) {
                    const uint32_t x = (cand[j] ^ prefix) >> shift;
                    if (x < limit) atomicAdd(&hist[x], 1u);
                }
            }
        } else if (listed) {
            for (uint32_t j = tid; j < ncand; j += TK_THREADS) {
                const uint32_t x = (cand[j] ^ prefix) >> shift;
                if (x < limit) atomicAdd(&hist[x], 1u);
            }
        } else if (__ballot(live != 0u) != 0ull) {
            uint32_t still = 0u;
#pragma unroll
            for (int i = 0; i < V4; ++i) {
                const bool mine = (live >> i) & 1u;
                if (__ballot(mine) == 0ull) continue;        // nobody in the wave: skip the group outright
                if (mine) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        // the digit, if all bits above it agree with the prefix (whose lower bits are zero)
                        const uint32_t x = (key[i][c] ^ prefix) >> shift;
                        if (x < limit) { atomicAdd(&hist[x], 1u); still |= 1u << i; }
                    }
                }
            }
            live = still;
        }
        __syncthreads();
        // the digit of the k-th largest: the highest bin b with count(bins >= b) >= need.
        // Thread t looks at bins TKR_BPT*t .. +TKR_BPT-1; `above` = count of all bins beyond them.
        uint32_t mine = 0;
#pragma unroll
        for (int b = 0; b < TKR_BPT / 4; ++b) {
            const u32x4 v = *(const u32x4*)&hist[TKR_BPT * tid + 4 * b];
            mine += (v[0] + v[1]) + (v[2] + v[3]);
        }
        // inclusive suffix sum over the lanes of the wave: the wave's total less the lanes in front
        const uint32_t upto = wave_prefix_sum_u32(mine);
        const uint32_t wave_total = (uint32_t)__builtin_amdgcn_readlane((int)upto, 63);
        const uint32_t suffix = wave_total - upto + mine;
        if (lane == 0) wave_a[wave] = wave_total;
        __syncthreads();
        uint32_t above = suffix - mine;
#pragma unroll
        for (int w = 0; w < TK_WAVES; ++w) above += (w > wave) ? wave_a[w] : 0u;
        if (above < need && above + mine >= need) {        // one thread: the bin is among its own
            // (its counts are read again here rather than kept in registers across the scan)
            for (int b = TKR_BPT - 1; b >= 0; --b) {
                const uint32_t hb = hist[TKR_BPT * tid + b];
                if (above + hb >= need) {
                    sh_bin = TKR_BPT * tid + b; sh_need = need - above; sh_cnt = hb; sh_ncand = 0u;
                    break;
                }
                above += hb;
            }
        }
        __syncthreads();
        prefix |= sh_bin << shift;
        need = sh_need;
        hi = shift - 1;
        const uint32_t in_bin = sh_cnt;
        if (!first_pass && hi >= 0 && in_bin <= (uint32_t)TKR_FEW && (listed || bracketed)) {
            // A handful of keys left on the list: instead of another pass they are put side by side and one
            // wave ranks them directly.  (sh_ncand was set to zero together with sh_bin.)
            auto offer = [&](uint32_t kx) {
                if (((kx ^ prefix) >> (hi + 1)) == 0u) {
                    const uint32_t at = atomicAdd(&sh_ncand, 1u);
                    if (at < (uint32_t)TKR_FEW) few[at] = kx;               // guard: holds by construction (in_bin counted them)
                }
            };
            if (bracketed) {
#pragma unroll
                for (int j = tid; j < CAND_MAX; j += TK_THREADS)
                    if ((uint32_t)(j % TKR_WAVE_CAND) < seg_cnt[j / TKR_WAVE_CAND]) offer(cand[j]);
            } else {
                for (uint32_t j = tid; j < ncand; j += TK_THREADS) offer(cand[j]);
            }
            __syncthreads();
            if (wave == 0) {
                const uint32_t mine = few[(uint32_t)lane < in_bin ? lane : 0];
                uint32_t gt = 0u, ge = 0u;
                for (uint32_t j = 0; j < in_bin; ++j) {
                    const uint32_t other = few[j];
                    gt += other > mine ? 1u : 0u;
                    ge += other >= mine ? 1u : 0u;
                }
                // the key with fewer than `need` keys above it and at least `need` keys not below it
                // (every lane that holds it writes the same two words)
                if ((uint32_t)lane < in_bin && gt < need && need <= ge) { sh_bin = mine; sh_need = need - gt; }
            }
            __syncthreads();
            prefix = sh_bin;
            need = sh_need;
            hi = -1;
        }
        if (first_pass && hi >= 0 && sh_cnt <= (uint32_t)CAND_MAX) {
            // one more sweep over the registers, the last: whoever agrees with the prefix down to
            // the first digit goes on the list (in any order: the passes only count)
#pragma unroll
            for (int i = 0; i < V4; ++i) {
                bool hit[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) hit[c] = ((key[i][c] ^ prefix) >> shift) == 0u;
                if (i < nv && (hit[0] || hit[1] || hit[2] || hit[3])) {         // rare: one region per group
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (hit[c]) {
                            const uint32_t at = atomicAdd(&sh_ncand, 1u);
                            if (at < (uint32_t)CAND_MAX) cand[at] = key[i][c];      // guard: holds by construction (sh_cnt counted them)
                        }
                }
            }
            listed = true;
            ncand = sh_cnt;
            // (the next pass's first barrier stands between these writes and its reads of the list)
        }
        first_pass = false;
        // (hist, wave_a, sh_bin are rewritten only behind the next pass's first barrier or, after
        //  the last pass, behind the barrier below)
    }

    if (bracketed) {
        // the half width follows the estimate's error: it shrinks by an eighth per row and is raised at once
        // to two and a half times the last error
        const uint32_t err = prefix > est ? prefix - est : est - prefix;
        uint32_t next = half_width - (half_width >> 3);
        const uint32_t floor_hw = err < TKR_HALF_WIDTH_MAX ? err * 2u + (err >> 1) : TKR_HALF_WIDTH_MAX;
        next = next > floor_hw ? next : floor_hw;
        half_width = __builtin_amdgcn_readfirstlane(next < TKR_HALF_WIDTH_MIN ? TKR_HALF_WIDTH_MIN : (next > TKR_HALF_WIDTH_MAX ? TKR_HALF_WIDTH_MAX : next));
        // ... and a wave's share of the list is short: no wider than what gave three quarters of the list's room
        if (listed_last > 3u * TK_THREADS) half_width -= half_width >> 2;
    }
    guess = __builtin_amdgcn_readfirstlane(prefix);
    have_guess = !VARLEN;          // (the variable-length instantiation has no registers to spare for the estimate)

    // ---- ordered compaction.  Per wave: elements above the threshold and elements equal to it
    // (on the bracket path: the keys above the bracket are counted already, the rest is on the
    // wave's share of the list).
    uint32_t n_gt = 0, n_eq = 0;
    if (bracketed) {
        for (uint32_t j = lane; j < seg_cnt[wave]; j += 64) {
            const uint32_t kx = cand[wave * TKR_WAVE_CAND + j];
            n_gt += kx > prefix ? 1u : 0u;
            n_eq += kx == prefix ? 1u : 0u;
        }
        n_gt += lane == 0 ? above_wave : 0u;
    } else {
#pragma unroll
        for (int i = 0; i < V4; ++i) {
            if (i < nv) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    n_gt += key[i][c] > prefix ? 1u : 0u;
                    n_eq += key[i][c] == prefix ? 1u : 0u;
                }
            }
        }
    }
    n_gt = wave_sum_u32(n_gt);
    n_eq = wave_sum_u32(n_eq);
    __syncthreads();
    if (lane == 0) { wave_a[wave] = n_gt; wave_b[wave] = n_eq; }
    __syncthreads();
    // the first `need` equal elements in index order are taken: waves in front of this one
    // have used up eq_seen of them and written out_pos entries
    uint32_t eq_seen = 0, out_pos = 0;
#pragma unroll
    for (int w = 0; w < TK_WAVES; ++w) {
        if (w < wave) {
            const uint32_t e = wave_b[w];
            const uint32_t left = need > eq_seen ? need - eq_seen : 0u;
            out_pos += wave_a[w] + (e < left ? e : left);
            eq_seen += e;
        }
    }
    // the same in every lane: kept in scalar registers, like the running counts below
    eq_seen = __builtin_amdgcn_readfirstlane(eq_seen);
    out_pos = __builtin_amdgcn_readfirstlane(out_pos);
    const bool wave_has_eq = __builtin_amdgcn_readfirstlane(n_eq) != 0u;
    // Lane masks throughout: a comparison is one instruction that leaves its mask in scalar registers, the
    // logic on the masks is scalar work beside the vector pipe, and nothing is evaluated under a narrowed
    // execution mask except the stores themselves.  Two versions of the loop: most waves hold no element
    // equal to the threshold (ties at the k-th value are rare) and run the one that does not look for any.
    auto compact_group = [&](int i, auto with_eq_c) {
        constexpr bool WITH_EQ = decltype(with_eq_c)::value;
        const bool in = i < nv;
        bool sel[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) sel[c] = in & (key[i][c] > prefix);
        if constexpr (WITH_EQ) {
            bool eq[4];
            uint32_t eq_rank = eq_seen;                     // equal elements of the lanes in front ...
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                eq[c] = in & (key[i][c] == prefix);
                const uint64_t eq_b = __ballot(eq[c]);
                eq_rank = count_before(eq_b, eq_rank);
                eq_seen += __popcll(eq_b);
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                sel[c] = sel[c] | (eq[c] & (eq_rank < need));
                eq_rank += eq[c] ? 1u : 0u;                 // ... and of this lane's earlier elements
            }
        }
        uint32_t pos = out_pos, sel_all = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint64_t sel_b = __ballot(sel[c]);
            pos = count_before(sel_b, pos);
            sel_all += __popcll(sel_b);
        }
        // (guard: holds by construction; no store can land behind the row's k_row entries.  Folded into the
        //  masks: a branch here would make the compiler carry the masks through vector registers.)
        const bool fits = out_pos + sel_all <= (uint32_t)k_row;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (sel[c] & fits) out[pos] = first_r + i * 256 + c;
            pos += sel[c] ? 1u : 0u;
        }
        out_pos += sel_all;
    };
#pragma unroll
    for (int i = 0; i < V4; ++i) {
        if (wave * SEG + i * 256 < n) {                  // uniform: nothing of this wave lies beyond
            if (wave_has_eq) compact_group(i, std::true_type{});
            else compact_group(i, std::false_type{});
        }
        // the compaction is done with this register group: refill it with the next row's scores
        if (i < nv_next) {
            const u32x4 v = *(const u32x4*)(next_bits + i * 256);
#pragma unroll
            for (int c = 0; c < 4; ++c) key[i][c] = v[c];
        }
    }
    if constexpr (VARLEN) { n = n_next; k_row = k_next; nv = nv_next; }
    __syncthreads();                                   // wave_a / wave_b are rewritten by the next row
  }
}

template <int V4, bool VARLEN>
hipError_t launch_rows_as(const TopkParams& p, hipStream_t s) {
    // as many workgroups as the chip holds at a time (1024 threads at more than 64 registers: one
    // per CU); each walks over its run of consecutive rows
    const int resident = compute_units();
    const int rows_per_wg = (p.rows + resident - 1) / resident;
    const int grid = (p.rows + rows_per_wg - 1) / rows_per_wg;
    hipLaunchKernelGGL((topk_rows_kernel<V4, VARLEN>), dim3(grid), dim3(TK_THREADS), 0, s, p, rows_per_wg);
    return hipGetLastError();
}

template <int V4>
hipError_t launch_rows(const TopkParams& p, hipStream_t s) {
    if (p.varlen != nullptr) return launch_rows_as<V4, true>(p, s);
    return launch_rows_as<V4, false>(p, s);
}

// Block masses, in place.  One workgroup per score row; a sweep of the workgroup covers 1024 consecutive scores with one
// 16-byte load per lane, so 16 neighbouring lanes hold one key block of 64 scores; its sum is the lane's four values
// added in order, then four exchange steps inside the 16 lanes (a fixed tree: bit-identical from run to run).  The sum
// of block j goes to element j of the same row.  Element j is read in sweep j / 1024 and the sum of sweep t lands in
// elements [16 t, 16 t + 16), so a store can only overtake a load of a sweep that is not later than its own: a barrier
// between the loads and the stores of every batch of sweeps orders the in-place update.
constexpr int BS_THREADS = 256;
constexpr int BS_UNROLL = 8;        // sweeps whose loads are issued together

__global__ void __launch_bounds__(BS_THREADS) block_sums_kernel(const float* __restrict__ scores, float* __restrict__ out,
                                                                int32_t n, int64_t stride) {
    const float4* __restrict__ row = reinterpret_cast<const float4*>(scores + (int64_t)blockIdx.x * stride);
    float* __restrict__ dst = out + (int64_t)blockIdx.x * stride;
    const int sweeps = n / (4 * BS_THREADS);                 // whole sweeps; the rest (a multiple of 64 scores) follows
    const int tid = threadIdx.x;
    auto fold = [](float4 v) {
        float a = (v.x + v.y) + (v.z + v.w);
        a += __shfl_xor(a, 1);
        a += __shfl_xor(a, 2);
        a += __shfl_xor(a, 4);
        a += __shfl_xor(a, 8);
        return a;
    };
    int t = 0;
    for (; t + BS_UNROLL <= sweeps; t += BS_UNROLL) {
        float4 v[BS_UNROLL];
#pragma unroll
        for (int u = 0; u < BS_UNROLL; ++u) v[u] = row[(int64_t)(t + u) * BS_THREADS + tid];
        float a[BS_UNROLL];
#pragma unroll
        for (int u = 0; u < BS_UNROLL; ++u) a[u] = fold(v[u]);
        __syncthreads();
        if ((tid & 15) == 0) {
#pragma unroll
            for (int u = 0; u < BS_UNROLL; ++u) dst[(t + u) * (BS_THREADS / 16) + (tid >> 4)] = a[u];
        }
    }
    // what is left: fewer than BS_UNROLL whole sweeps, then a part of a sweep
    for (; t <= sweeps; ++t) {
        const int e = (t * BS_THREADS + tid) * 4;            // first score of this lane
        const bool live = e < n;
        float4 v = live ? row[(int64_t)t * BS_THREADS + tid] : float4{0.f, 0.f, 0.f, 0.f};
        const float a = fold(v);
        __syncthreads();
        if (live && (tid & 15) == 0) dst[t * (BS_THREADS / 16) + (tid >> 4)] = a;
    }
}

}  // namespace

hipError_t launch_block_sums(const float* scores, float* out, int32_t rows, int32_t n, int64_t stride, int32_t block, hipStream_t s) {
    // 16 lanes x 16 bytes = one key block; rows start on 16-byte boundaries
    if (rows < 1 || block != 64 || n < block || n % block != 0 || stride % 4 != 0) return hipErrorInvalidValue;
    if ((reinterpret_cast<uintptr_t>(scores) & 15u) != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(block_sums_kernel, dim3(rows), dim3(BS_THREADS), 0, s, scores, out, n, stride);
    return hipGetLastError();
}

hipError_t launch_topk(const TopkParams& p, hipStream_t s) {
    if (p.rows < 1 || p.n < 1 || p.k < 1 || p.k > p.n) return hipErrorInvalidValue;
    // rows that one workgroup can hold in registers, and that 16-byte loads can read
    if (p.stride < p.n) return hipErrorInvalidValue;
    if (p.n <= 65536 && p.n % 4 == 0 && p.stride % 4 == 0 && (reinterpret_cast<uintptr_t>(p.scores) & 15u) == 0) {
        const int per_wave = (p.n + TK_WAVES - 1) / TK_WAVES;      // elements a wave has to hold
        if (per_wave <= 256) return launch_rows<1>(p, s);
        if (per_wave <= 512) return launch_rows<2>(p, s);
        if (per_wave <= 1024) return launch_rows<4>(p, s);
        if (per_wave <= 2048) return launch_rows<8>(p, s);
        return launch_rows<16>(p, s);
    }
    hipLaunchKernelGGL(topk_kernel, dim3(p.rows), dim3(TK_THREADS), 0, s, p);
    return hipGetLastError();
}

}  // namespace pulsecol
