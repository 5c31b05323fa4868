// bf16 attention kernels for gfx950: column-sparse attention (Sec. 3.4 and the appendix
// listing "Column-Sparse Attention Forward"), the dense baseline (Sec. 3.1) and the row
// log-sum-exp pass of the identification step (Sec. 3.3: the softmax matrix P needs the
// row normalisers before column masses can be summed).
//
// One workgroup = 256 query rows (4 waves x 64 rows), one tile = 64 K/V rows, processed as
// two half-tiles of 32.  Q stays in registers (AGPRs) as the MFMA B operand for the whole
// kernel.  K and V rows are gathered straight into LDS (global_load_lds_dwordx4: 16 lanes
// cover one 256-byte row, the XOR swizzle is applied on the global side) into four tile
// slots per operand, three tiles ahead, and read back as MFMA A operands (V through the
// transposing LDS read).  Every lane owns one query column of S^T / O^T, so the online-softmax
// state is two scalars per lane and query block.  P is rounded to bf16 only as the MFMA
// operand; l is summed from the fp32 P.  The output accumulator lives in AGPRs and is touched
// by the matrix pipe only.
//
// Software pipeline (one wave per SIMD, so overlap has to come from the instruction
// stream): half-step j issues the MFMAs of  S(j+1) = K(j+1) Q^T  and  O += V(j-1) P(j-1)
// while the VALU turns S(j) into P(j).  The half-step is written as a sequence of slots, one
// MFMA each, fenced so that the compiler keeps the hand-made interleaving.  A wave issues in
// order, and with one wave per SIMD every instruction between two MFMAs costs issue time
// (about 12 ticks for the MFMA itself, 8 for an exp, 4 for anything else, against the 32 ticks
// the matrix pipe is busy), except that the first non-VALU instruction behind an MFMA is
// free.  So every slot is: the MFMA (the first of a group of pairs with the wait for the
// group's fragments fused in front), then the slot's LDS read / gather instruction / scalar
// work, then one tick of the softmax work (fma, add, pack, exp); a gather is split over two
// slots; loads are spread over the whole iteration; the steady loop is unrolled by the four
// tile slots so that LDS addresses are a base register plus an immediate.  One workgroup runs
// per CU, so nothing covers its start and end: the first half-step waits only for the Q block
// (staged through LDS) and the first K tile, and the last tile still goes through a scheduled
// iteration.  The reference maximum is raised
// lazily and after the fact: P is formed against the current reference, and only when a
// lane's row sum of the half-tile exceeds 2^kTau (or is not finite) does the wave take the
// slow path that finds the true maximum, moves the reference by a whole number of log2
// units, rescales l and the accumulator by that exact power of two and recomputes P.  The
// result is exact either way (numerator and denominator carry the same factor); the fast
// path needs no row maximum at all.
//
// The MFMAs are inline assembly (to pin operands to AGPRs), so the compiler does not know
// their latency: every place where the VALU reads an MFMA result is either separated from
// the producer by several later MFMAs of the same in-order stream or preceded by
// mfma_settle().  Some loads are inline assembly too (row numbers, LDS fragments), so that
// their waits can be placed by hand; for those the compiler knows neither the latency nor that
// the destination is written later.  The rules that keep this sound: such a load is one
// statement whose output is the whole variable, nothing reads the variable before the wait
// that covers it, and every such variable is named by a statement behind that wait (which
// keeps its registers reserved).  tests/test_asm_hazards.py checks the generated code.
#include <type_traits>
#include <utility>

#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int BM = kBlockM_bf16;
constexpr int BN = kBlockN_bf16;
constexpr int NTHREADS = 256;
constexpr int NBUF = 4;            // LDS tile slots for K and for V: tile t lives in slot t % NBUF, and the
                                   // steady loop is unrolled NBUF times so that every slot is an immediate
constexpr int NBUF_K = NBUF;
constexpr int NBUF_V = NBUF;
constexpr int PRO_TILES = 3;       // K tiles requested by the prologue (the loop loads tile PRO_TILES first)
constexpr float kTau = 8.0f;       // log2 of the growth allowed before the reference max is raised
constexpr float kGrowthLimit = 256.0f;   // 2^kTau

typedef unsigned char byte;

__device__ __forceinline__ void fence() { __builtin_amdgcn_sched_barrier(0); }

// S = a * q (fresh accumulator) and S += a * q, with q held in AGPRs
__device__ __forceinline__ void mfma_qk_first(f32x16& s, bf16x8 a, bf16x8 q) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(a), "a"(q));
}
__device__ __forceinline__ void mfma_qk(f32x16& s, bf16x8 a, bf16x8 q) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(a), "a"(q));
}
// O += a * p with O held in AGPRs
__device__ __forceinline__ void mfma_pv(f32x16& o, bf16x8 a, bf16x8 p) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o) : "v"(a), "v"(p));
}
// The same three, preceded by "wait until at most N LDS reads are outstanding": used by the
// first MFMA that consumes a fragment requested a few slots earlier.
template <int N>
__device__ __forceinline__ void mfma_qk_first_after(f32x16& s, bf16x8 a, bf16x8 q) {
    asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(a), "a"(q), "n"(N));
}
template <int N>
__device__ __forceinline__ void mfma_qk_after(f32x16& s, bf16x8 a, bf16x8 q) {
    asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(a), "a"(q), "n"(N));
}
template <int N>
__device__ __forceinline__ void mfma_pv_after(f32x16& o, bf16x8 a, bf16x8 p) {
    asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o) : "v"(a), "v"(p), "n"(N));
}
// Waits out the write-back of every matrix instruction issued so far (the longest
// MFMA-result-to-VALU hazard on gfx950 is 18 wait states).  The values the VALU is about to
// read are routed through the statement so that no use of them can be placed before it.
__device__ __forceinline__ void mfma_settle(f32x16& s0, f32x16& s1) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+v"(s0), "+v"(s1));
}
template <int N>
__device__ __forceinline__ void mfma_settle_acc(f32x16 (&o)[2][N]) {
    static_assert(N == 1 || N == 2 || N == 4, "accumulator blocks");
    if constexpr (N == 4)
        asm volatile("s_nop 15\n\ts_nop 15" : "+a"(o[0][0]), "+a"(o[0][1]), "+a"(o[0][2]), "+a"(o[0][3]),
                                               "+a"(o[1][0]), "+a"(o[1][1]), "+a"(o[1][2]), "+a"(o[1][3]));
    else if constexpr (N == 2)
        asm volatile("s_nop 15\n\ts_nop 15" : "+a"(o[0][0]), "+a"(o[0][1]), "+a"(o[1][0]), "+a"(o[1][1]));
    else
        asm volatile("s_nop 15\n\ts_nop 15" : "+a"(o[0][0]), "+a"(o[1][0]));
}
// element pair `i` (two bf16 in one 32-bit register) of a fragment
__device__ __forceinline__ void set_pair(bf16x8& f, int i, uint32_t w) {
    u32x4 t = __builtin_bit_cast(u32x4, f);
    t[i] = w;
    f = __builtin_bit_cast(bf16x8, t);
}

// LDS fragment reads of the scheduled half-step, as inline assembly with hand-placed waits.
// (The compiler's own wait-count insertion drains lgkmcnt to zero whenever a direct-to-LDS
// load is in flight; LDS returns data in order, so "all but the N newest reads" is exact.)
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128_at(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF>
__device__ __forceinline__ bf16x4 lds_read_tr_at(uint32_t addr) {
    bf16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=&v"(v) : "v"(addr), "n"(OFF));
    return v;
}
// 64-bit half `h` of a fragment
__device__ __forceinline__ void set_half(bf16x8& f, int h, bf16x4 v) {
    f = h == 0 ? __builtin_shufflevector(v, __builtin_shufflevector(f, f, 4, 5, 6, 7), 0, 1, 2, 3, 4, 5, 6, 7)
               : __builtin_shufflevector(__builtin_shufflevector(f, f, 0, 1, 2, 3), v, 0, 1, 2, 3, 4, 5, 6, 7);
}
__device__ __forceinline__ uint32_t lds_address(const void* generic_lds_ptr) {
    return (uint32_t)(uintptr_t)(PULSECOL_LDS const void*)generic_lds_ptr;
}

// s_waitcnt vmcnt(v) with the other counters left alone (gfx9 encoding: vmcnt in [3:0] and [15:14])
template <int v>
__device__ __forceinline__ void wait_vmcnt_at_most() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (v & 0xF) | ((v & 0x30) << 10));
}

constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }

template <int D, int MODE>
struct AttnWave {
    static constexpr int PIECES = D / 8;                 // 16-byte pieces per row
    static constexpr int KK = D / 16;                    // contraction steps of Q K^T
    static constexpr int DB = D / 32;                    // 32-wide blocks of the head dimension
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int TILE_BYTES = BN * ROW_BYTES;
    static constexpr int HALF_BYTES = 32 * ROW_BYTES;
    static constexpr int ROWS_PER_CHUNK = 64 / PIECES;   // one direct-to-LDS load instruction moves 64 x 16 bytes
    static constexpr int CH = BN / ROWS_PER_CHUNK / 4;   // such instructions per wave and tile (per operand)
    static constexpr bool HAS_V = (MODE != kLseOnly);
    static constexpr bool BLOCKS = (MODE == kBlock);       // block-sparse: a tile is one block of BN consecutive keys
    static constexpr bool GATHER = (MODE == kSparse || MODE == kBlock);
    static constexpr int ODB = HAS_V ? DB : 1;
    static constexpr int NPV = HAS_V ? 2 * DB : 0;       // V fragments (= MFMA pairs) of a half-step
    static constexpr int NP = KK + NPV;                  // MFMA pairs of a half-step
    static constexpr int NS = 2 * NP;                    // MFMA slots of a half-step
    static constexpr int EXP_TICKS = 34;                 // 32 values through a 3-stage pipeline
    // One wait per WAIT_PAIRS MFMA pairs, for the fragments of all of them (a wait costs issue
    // time); fragment reads run AHEAD pairs ahead of their use, so that the last fragment of a
    // group still has AHEAD - WAIT_PAIRS + 1 pairs to arrive.
    // (The row pass has no P V stream behind which the next half-step's first fragments could be
    // requested; it reads them right behind its barrier and waits for each by itself.)
    static constexpr int WAIT_PAIRS = !HAS_V ? 1 : (KK >= 8 ? 4 : 2);
    static constexpr int AHEAD = WAIT_PAIRS + 2;
    // ticks issued before slot s: spread over all slots but the last one, so that the row sums
    // are complete (and their check can be computed) one slot before the half-step ends
    static constexpr int exp_ticks_before(int s) {
        const int t = ceil_div(EXP_TICKS * s, NS - 1);
        return t < EXP_TICKS ? t : EXP_TICKS;
    }
    // Load schedule of an iteration, one instruction pair (address, load) per entry, spread out
    // so that the vector memory pipe sees a steady trickle instead of a burst: first half-step,
    // K load j: address behind the second MFMA of pair 1 + j*LOAD_STRIDE, load behind the first
    // MFMA of the next pair; second half-step, V load j: the same at pair j*LOAD_STRIDE.
    static constexpr int LOAD_STRIDE = (NP - 2) / CH;
    static constexpr int k_addr_pair(int j) { return 1 + j * LOAD_STRIDE; }
    static constexpr int v_addr_pair(int j) { return j * LOAD_STRIDE; }
    // index of the load whose address / load instruction sits in pair p, or -1
    static constexpr int k_addr_at(int p) { return (p >= 1 && (p - 1) % LOAD_STRIDE == 0 && (p - 1) / LOAD_STRIDE < CH) ? (p - 1) / LOAD_STRIDE : -1; }
    static constexpr int v_addr_at(int p) { return (p % LOAD_STRIDE == 0 && p / LOAD_STRIDE < CH) ? p / LOAD_STRIDE : -1; }
    // V loads issued before the barrier of the second half-step (it sits in pair KK, in front of
    // that pair's load)
    static constexpr int v_loads_before_barrier() {
        int c = 0;
        for (int j = 0; j < CH; ++j) c += (v_addr_pair(j) + 1 < KK) ? 1 : 0;
        return c;
    }
    // loads of the running iteration in flight at its barrier: everything older has to be complete
    static constexpr int VM_PER_ISSUE = CH + (HAS_V ? v_loads_before_barrier() : 0);

    // lane geometry
    int lane, wave, lq, lh;
    // problem
    int n, ns, ntiles, nhalf;
    bool ragged;
    uint32_t row_bytes;   // byte stride between sequence positions of K / V in global memory
    uint32_t row_mul;     // what a tile's row word is multiplied by: row_bytes, or (block-sparse) the bytes of a key block
    uint32_t wave_lds;    // LDS address of this wave's first 1 KB chunk in tile slot 0 of K
    uint32_t dma_off;     // global byte offset of the load whose first half has been issued
    const byte* K;
    const byte* V;
    const byte* idx;      // int32 column numbers of this head
    // registers that live across the whole kernel
    bf16x8 qf[2][KK];     // AGPRs
    f32x16 o_acc[2][ODB]; // AGPRs
    float c2;
    float mc[2];          // reference maximum in log2 units (raw maximum * c2), equal in both half-waves
    float l_run[2];       // per-lane partial row sum (this lane's keys only)
    // global byte offset that load instruction i adds to row word * row_mul: this lane's piece inside a row, plus
    // (block-sparse) the row's offset inside its key block
    uint32_t koff[CH], voff[CH];
    uint32_t kaddr[KK];   // LDS byte offset (inside a tile slot, first half) of this lane's K fragment kk
    uint32_t vaddr[ODB];  // same for the first 4-row group of the V fragment of d-block db
    int lrow;
    uint32_t lane_rows_off;   // byte offset, inside a tile's 64 column numbers, of this lane's CH consecutive ones

    __device__ __forceinline__ void init_addresses() {
        lrow = lane / PIECES;
        lane_rows_off = (uint32_t)(wave * 16 + lrow * CH) * 4u;
        const int lslot = lane % PIECES;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int row = (wave * CH + i) * ROWS_PER_CHUNK + lrow;
            koff[i] = (uint32_t)(lslot ^ swizzle_k<PIECES>(row)) * 16u;
            voff[i] = (uint32_t)(lslot ^ swizzle_v<PIECES>(row)) * 16u;
            if (BLOCKS) {
                // load i of this lane brings the key at position wave*16 + lrow*CH + i of the block
                const uint32_t in_block = (uint32_t)(wave * 16 + lrow * CH + i) * row_bytes;
                koff[i] += in_block;
                voff[i] += in_block;
            }
        }
        row_mul = BLOCKS ? row_bytes * (uint32_t)BN : row_bytes;
        // K fragment kk: tile row lq (+32 for the second half), piece 2*kk + lh
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            kaddr[kk] = (uint32_t)(lq * ROW_BYTES + (((2 * kk + lh) ^ swizzle_k<PIECES>(lq)) << 4));
        // V fragment: contraction element e of a lane <-> tile row half*32 + hf*16 + 8*(e/4) + 4*lh + e%4.
        // The transposing read takes the address of row 4*lh + j16/4 (and +8), 8 bytes at
        // d = db*32 + 16*((lane/16)&1) + 4*(j16%4), j16 = lane%16.
        const int j16 = lane & 15;
        const int row0 = 4 * lh + (j16 >> 2);
        const int colpiece = ((lane >> 4) & 1) * 2 + ((j16 & 3) >> 1);
        const int inpiece = (j16 & 1) * 8;
#pragma unroll
        for (int db = 0; db < ODB; ++db)
            vaddr[db] = (uint32_t)(row0 * ROW_BYTES + inpiece + (((db * 4 + colpiece) ^ swizzle_v<PIECES>(row0)) << 4));
    }

    // ------------------------------------------------------------------ gathers
    // byte offset of a 16-byte piece of K/V row `row` from the head's base: both factors are
    // below 2^24 (checked on the host), so the full-rate 24-bit multiply-add does it
    __device__ __forceinline__ uint32_t row_offset(int row, uint32_t piece_off) const {
        return __umul24((uint32_t)row, row_mul) + piece_off;
    }
    // Which sequence position goes where: load instruction i of a wave fills LDS tile row
    // (wave*CH + i)*ROWS_PER_CHUNK + lrow, and it takes position wave*16 + lrow*CH + i of the
    // tile's 64 (K and V alike, so scores and values still meet; only tail masking has to know).
    // A lane's CH positions are then consecutive, and their row numbers are ONE load of CH
    // entries of the pattern, starting at entry `first_entry`: the lane's first position, pulled
    // back so that all CH entries lie inside the pattern.  In the last tile a lane whose positions
    // straddle or pass the end thereby fetches entries that belong to earlier positions a second
    // time; entry_is_new() tells them apart and mask_tail() gives those positions weight zero.
    // (Block-sparse: the one word of a tile is the number of its key block, the same for every lane and load.)
    typedef int row_vector_t __attribute__((ext_vector_type(CH)));
    typedef std::conditional_t<BLOCKS, int, row_vector_t> rows_t;
    static __device__ __forceinline__ int row_word(const rows_t& rows, int i) {
        if constexpr (BLOCKS) return rows; else return rows[i];
    }
    __device__ __forceinline__ int first_entry(int first_pos) const {
        const int last = ns > CH ? ns - CH : 0;
        return first_pos < last ? first_pos : last;
    }
    // position p (element p % CH of its lane) holds an entry of its own, inside the pattern
    __device__ __forceinline__ bool entry_is_new(int p) const {
        const int p0 = p - p % CH;
        const int e = first_entry(p0) + p % CH;
        return e >= p0 && e < ns;
    }
    __device__ __forceinline__ void load_rows(int t, rows_t& dst) const { load_rows(idx, t, dst); }
    // ... from the pattern `idx` (the set of another query block than the running one)
    __device__ __forceinline__ void load_rows(const byte* idx, int t, rows_t& dst) const {
        static_assert(CH * ROWS_PER_CHUNK == 16, "a wave fills 16 rows of a tile");
        t = t < ntiles ? t : ntiles - 1;          // past the end: repeat the last tile (never read back)
        if constexpr (BLOCKS) {
            dst = *(const int*)(idx + (uint32_t)t * 4u);
            return;
        } else {
        const int e0 = first_entry(t * BN + wave * 16 + lrow * CH);
        if (GATHER) {
            if (__builtin_expect(ns >= CH, 1)) {
                typedef int unaligned_rows_t __attribute__((ext_vector_type(CH), aligned(4)));
                dst = *(const unaligned_rows_t*)(idx + (uint32_t)e0 * 4u);
            } else {
#pragma unroll
                for (int i = 0; i < CH; ++i) dst[i] = *(const int*)(idx + (uint32_t)(e0 + i < ns ? e0 + i : ns - 1) * 4u);
            }
        } else {
#pragma unroll
            for (int i = 0; i < CH; ++i) dst[i] = e0 + i < ns ? e0 + i : ns - 1;
        }
        }
    }
    // The same for the scheduled half-steps (which only run when the pattern has more than one
    // tile, so ns > CH), with a load the compiler does not see: it would otherwise wait for ALL
    // outstanding vector memory operations (the direct-to-LDS loads included) in front of the
    // first use.  The row numbers are used one iteration later; the wait in front of the running
    // iteration's barrier already covers them (they are older than every direct-to-LDS load that
    // wait leaves in flight).  The destination is the whole variable, written by this one
    // statement on every path: nothing may copy it before the data has arrived, and the
    // registers must stay reserved until then (the kernel names them in a final wait).
    __device__ __forceinline__ void load_rows_async(int t, rows_t& dst) const {
        if (!GATHER) { load_rows(t, dst); return; }
        t = t < ntiles ? t : ntiles - 1;
        if constexpr (BLOCKS) {
            const uint32_t off = (uint32_t)t * 4u;
            asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(off), "s"(idx));
        } else {
            const uint32_t want = (uint32_t)(t * (BN * 4)) + lane_rows_off, last = (uint32_t)(ns - CH) * 4u;
            const uint32_t off = want < last ? want : last;
            static_assert(CH == 2 || CH == 4, "row numbers per lane and tile");
            if constexpr (CH == 4) asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(off), "s"(idx));
            else asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(dst) : "v"(off), "s"(idx));
        }
    }
    // position inside its tile of the key in LDS tile row `row`
    static __device__ __forceinline__ int tile_pos(int row) {
        return (row & ~15) + (row % ROWS_PER_CHUNK) * CH + (row & 15) / ROWS_PER_CHUNK;
    }
    // Load instruction i of a wave fills the 1 KB chunk cid = wave*CH + i of a tile slot: lane L
    // lands at chunk byte 16*L, i.e. tile row cid*ROWS_PER_CHUNK + L/PIECES, LDS piece L%PIECES,
    // and therefore fetches the global piece (L%PIECES) ^ swizzle(row) of that row.
    // (Every pointer is a restrict parameter so that the loads carry alias scopes: the compiler
    // then knows that LDS reads of other slots need not wait for these loads.)
    __device__ __forceinline__ void issue_k_tile(byte* __restrict__ kslot, const byte* __restrict__ Kg,
                                                 const rows_t& rows) const {
#pragma unroll
        for (int i = 0; i < CH; ++i)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(Kg + row_offset(row_word(rows, i), koff[i])),
                (PULSECOL_LDS void*)(kslot + (wave * CH + i) * 1024), 16, 0, 0);
    }
    __device__ __forceinline__ void issue_v_tile(byte* __restrict__ vslot, const byte* __restrict__ Vg,
                                                 const rows_t& rows) const {
        if (HAS_V) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(Vg + row_offset(row_word(rows, i), voff[i])),
                    (PULSECOL_LDS void*)(vslot + (wave * CH + i) * 1024), 16, 0, 0);
        }
    }

    // One load of the scheduled half-step in two parts, so that no slot gets more than two
    // instructions on top of its own: the row offset (one VALU instruction) behind the second
    // MFMA of a pair, the load itself behind the first MFMA of the next pair.  The CH loads of a
    // tile share one LDS base in m0 (written with the first address; the VALU instruction behind
    // it also covers the wait state an m0 write needs before its use): load j carries the
    // instruction offset j*1024, which the hardware adds to the LDS address and to the global
    // address alike, so it reads through a base pointer that lies j*1024 bytes lower.
    template <int LDS_OFF, int J>
    __device__ __forceinline__ uint32_t issue_addr(int row, uint32_t piece_off) const {
        uint32_t off;
        if constexpr (J == 0)
            asm volatile("s_add_i32 m0, %1, %2\n\tv_mad_u32_u24 %0, %3, %4, %5"
                         : "=v"(off) : "s"(wave_lds), "n"(LDS_OFF), "v"(row), "s"(row_mul), "v"(piece_off));
        else
            asm volatile("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(off) : "v"(row), "s"(row_mul), "v"(piece_off));
        return off;
    }
    // m0 is written by issue_addr and, in compiler-generated code, only right in front of the
    // compiler's own uses (the prologue's loads): nothing touches it between the loads of a tile
    template <int J>
    __device__ __forceinline__ void issue_load(const byte* g, uint32_t off) const {
        asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(off), "s"(g - J * 1024), "n"(J * 1024) : "memory");
    }

    // ------------------------------------------------------------------ fragment reads
    __device__ __forceinline__ bf16x8 read_k(const byte* __restrict__ kslot, int half, int kk) const {
        return *(const bf16x8*)(kslot + half * HALF_BYTES + kaddr[kk]);
    }
    // V fragment q of a half-step: rows hf*16 .. +15 of the half-tile, d-block db; q = hf*ODB + db
    __device__ __forceinline__ bf16x8 read_v(const byte* __restrict__ vslot, int half, int q) const {
        const int hf = q / ODB, db = q % ODB;
        const byte* p = vslot + half * HALF_BYTES + hf * 16 * ROW_BYTES + vaddr[db];
        const bf16x4 lo = lds_read_tr(p);
        const bf16x4 hi = lds_read_tr(p + 8 * ROW_BYTES);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }

    // ------------------------------------------------------------------ softmax pieces
    // positions of the last tile without an entry of their own (past ns, or a repeat of an
    // earlier position's entry, see load_rows) get weight zero
    __device__ __forceinline__ void mask_tail(int j, f32x16 (&S)[2]) const {
        if (ragged && j >= nhalf - 2) {
            const int tile_start = (j >> 1) * BN;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (!entry_is_new(tile_start + tile_pos((j & 1) * 32 + acc_row(r, lh)))) { S[0][r] = -INFINITY; S[1][r] = -INFINITY; }
        }
    }
    // the same for half `half` of the last tile, right behind the scheduled half-step that formed S
    __device__ __forceinline__ void mask_last_tile(int half, f32x16 (&S)[2]) const {
        if (ragged) {
            mfma_settle(S[0], S[1]);
            mask_tail(nhalf - 2 + half, S);
        }
    }
    // maximum over this lane's 16 values and the 16 of the lane that shares its query column
    __device__ __forceinline__ float half_tile_max(const f32x16& s) const {
        float a0 = fmaxf(fmaxf(s[0], s[1]), s[2]);
        float a1 = fmaxf(fmaxf(s[3], s[4]), s[5]);
        float a2 = fmaxf(fmaxf(s[6], s[7]), s[8]);
        float a3 = fmaxf(fmaxf(s[9], s[10]), s[11]);
        a0 = fmaxf(fmaxf(a0, s[12]), s[13]);
        a1 = fmaxf(fmaxf(a1, s[14]), s[15]);
        return half_max(fmaxf(fmaxf(a0, a1), fmaxf(a2, a3)));
    }
    // P = exp2(S*c2 - mc) in EXP_TICKS small steps that can be spread over MFMA slots: tick i
    // adds value i-2 to the fp32 row sum (packing a bf16 pair after every odd value), forms the
    // scaled, shifted logit of value i and takes exp2 of value i-1.  Value e = qb*16 + r.
    struct ExpPipe { float t[32]; float x[32]; float rs[2]; uint64_t bad; };
    __device__ __forceinline__ void exp_tick(int i, const f32x16 (&S)[2], bf16x8 (&P)[2][2], ExpPipe& ep) {
        // A wave issues in order, one instruction at a time, so every instruction between two
        // MFMAs counts.  Issue order inside a tick: fma (left to the compiler), then one
        // assembler statement with add, pack, exp.  The statement names the fma result as an
        // input so that the fma stays ahead of it: the compiler counts no wait state for an
        // assembler statement and would otherwise pad every pair of dependent statements (tick
        // to tick, MFMA to MFMA on one accumulator) with a no-op.  The hazard that does exist
        // (a transcendental result needs one instruction before its first use) holds by
        // construction: the exp closes its tick, and an fma or an MFMA opens the next.
        const bool has_fma = i < 32, has_val = i >= 2 && i <= 33, has_exp = i >= 1 && i <= 32;
        const int e = has_val ? i - 2 : 0, qb = e >> 4, r = e & 15;
        // value 0 of a query block opens its row sum (no instruction), value 1 is packed with it
        // straight out of the sum's register
        const bool has_add = has_val && r > 0, first_pack = HAS_V && has_val && r == 1;
        const bool has_pack = HAS_V && has_val && (r & 1) && r > 1;
        const int ti = has_fma ? i : 0, te = has_exp ? i - 1 : 0, xp = has_pack ? e - 1 : 0;
        uint32_t w = 0;
        if (has_fma) ep.t[i] = __builtin_fmaf(S[i >> 4][i & 15], c2, -mc[i >> 4]);
        if (has_val && r == 0) ep.rs[qb] = ep.x[e];
        if (first_pack) {
            asm volatile("v_cvt_pk_bf16_f32 %1, %0, %3\n\tv_add_f32 %0, %0, %3\n\tv_exp_f32 %2, %4"
                         : "+v"(ep.rs[qb]), "=&v"(w), "=v"(ep.x[te])
                         : "v"(ep.x[e]), "v"(ep.t[te]), "v"(ep.t[ti]));
        } else if (has_add && has_pack && has_exp) {
            asm volatile("v_add_f32 %0, %0, %3\n\tv_cvt_pk_bf16_f32 %1, %4, %3\n\tv_exp_f32 %2, %5"
                         : "+v"(ep.rs[qb]), "=&v"(w), "=v"(ep.x[te])
                         : "v"(ep.x[e]), "v"(ep.x[xp]), "v"(ep.t[te]), "v"(ep.t[ti]));
        } else if (has_add && has_exp) {
            asm volatile("v_add_f32 %0, %0, %2\n\tv_exp_f32 %1, %3"
                         : "+v"(ep.rs[qb]), "=v"(ep.x[te])
                         : "v"(ep.x[e]), "v"(ep.t[te]), "v"(ep.t[ti]));
        } else if (has_add && has_pack) {
            asm volatile("v_add_f32 %0, %0, %2\n\tv_cvt_pk_bf16_f32 %1, %3, %2"
                         : "+v"(ep.rs[qb]), "=&v"(w)
                         : "v"(ep.x[e]), "v"(ep.x[xp]));
        } else if (has_add) {
            asm volatile("v_add_f32 %0, %0, %1" : "+v"(ep.rs[qb]) : "v"(ep.x[e]));
        } else if (has_exp) {
            asm volatile("v_exp_f32 %0, %1" : "=v"(ep.x[te]) : "v"(ep.t[te]), "v"(ep.t[ti]));
        } else if (has_fma) {
            asm volatile("" : : "v"(ep.t[ti]));
        }
        if (has_pack || first_pack) set_pair(P[qb][r >> 3], (r & 7) >> 1, w);
    }
    __device__ __forceinline__ void exp_begin(ExpPipe& ep) {
        ep.rs[0] = ep.rs[1] = 0.f;
    }
    // Close a half-tile: accept the row sums, or -- if some lane's sum says that its weights
    // outgrew the reference -- fix the reference first.  Every MFMA that adds P(j-1) to the
    // accumulator has been issued.  SCHEDULED half-steps have formed the test one slot before their
    // end (on the bit patterns of the sums, which also catches NaN); the general half-step tests
    // each sum in the NaN-catching floating-point form.
    template <bool SCHEDULED>
    __device__ __forceinline__ void exp_end(ExpPipe& ep, const f32x16 (&S)[2], bf16x8 (&P)[2][2]) {
        if (!SCHEDULED) {
            const float limit = __builtin_amdgcn_exp2f(kTau);
            ep.bad = __ballot(!(ep.rs[0] <= limit) || !(ep.rs[1] <= limit));
        }
        if (__builtin_expect(ep.bad != 0ull, 0)) fix_reference(ep, S, P);
        l_run[0] += ep.rs[0];
        l_run[1] += ep.rs[1];
    }
    // Slow path: true maximum of the half-tile per query, reference moved up by a whole number
    // of log2 units, l and the accumulator scaled by that exact power of two, P recomputed.
    __device__ __forceinline__ void fix_reference(ExpPipe& ep, const f32x16 (&S)[2], bf16x8 (&P)[2][2]) {
        if (HAS_V) mfma_settle_acc(o_acc);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float m2 = half_tile_max(S[qb]) * c2;        // same value in both half-waves
            if (m2 > mc[qb] + 1.0f) {
                const bool first = mc[qb] == -INFINITY;
                const float steps = first ? 0.f : ceilf(m2 - mc[qb]);
                const float alpha = first ? 0.f : fast_exp2(-steps);
                mc[qb] = first ? m2 : mc[qb] + steps;
                l_run[qb] *= alpha;
                if (HAS_V) {
                    // one block at a time, pinned inside this branch: the accumulator passes through
                    // VGPRs, and all of it at once does not fit beside the rest of the loop's registers
#pragma unroll
                    for (int db = 0; db < ODB; ++db) {
                        f32x16 t = o_acc[qb][db];
                        asm volatile("" : "+v"(t));
#pragma unroll
                        for (int r = 0; r < 16; ++r) t[r] *= alpha;
                        o_acc[qb][db] = t;
                        asm volatile("" : "+a"(o_acc[qb][db]));
                    }
                }
                float rs = 0.f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float x0 = fast_exp2(__builtin_fmaf(S[qb][r], c2, -mc[qb]));
                    const float x1 = fast_exp2(__builtin_fmaf(S[qb][r + 1], c2, -mc[qb]));
                    rs += x0;
                    rs += x1;
                    if (HAS_V) {
                        P[qb][r >> 3][r & 7] = (__bf16)x0;
                        P[qb][r >> 3][(r & 7) + 1] = (__bf16)x1;
                    }
                }
                ep.rs[qb] = rs;
            }
        }
    }
    __device__ __forceinline__ void exp_half_tile(const f32x16 (&S)[2], bf16x8 (&P)[2][2]) {
        ExpPipe ep;
        exp_begin(ep);
#pragma unroll
        for (int i = 0; i < EXP_TICKS; ++i) exp_tick(i, S, P, ep);
        exp_end<false>(ep, S, P);
    }

    // ------------------------------------------------------------------ half-steps
    // Plain (unscheduled) matrix steps, used by the general half-step.
    // (All fragment reads go out before the first MFMA: one LDS round trip, not one per fragment.)
    __device__ __forceinline__ void qk_all(const byte* kslot, int half, f32x16 (&S)[2]) const {
        bf16x8 a[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) a[kk] = read_k(kslot, half, kk);
        fence();
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if (kk == 0) { mfma_qk_first(S[0], a[kk], qf[0][kk]); mfma_qk_first(S[1], a[kk], qf[1][kk]); }
            else { mfma_qk(S[0], a[kk], qf[0][kk]); mfma_qk(S[1], a[kk], qf[1][kk]); }
        }
    }
    __device__ __forceinline__ void pv_all(const byte* vslot, int half, const bf16x8 (&P)[2][2]) {
        if constexpr (HAS_V) {
            bf16x8 a[NPV];
#pragma unroll
            for (int q = 0; q < NPV; ++q) a[q] = read_v(vslot, half, q);
            fence();
#pragma unroll
            for (int q = 0; q < NPV; ++q) {
                mfma_pv(o_acc[0][q % ODB], a[q], P[0][q / ODB]);
                mfma_pv(o_acc[1][q % ODB], a[q], P[1][q / ODB]);
            }
        }
    }

    // LDS operations that the read of fragment q of a scheduled half-step issues: one for a K
    // fragment (q < KK, or q >= NP: the next half-step's first K fragments), two for a V fragment.
    // ... that have been issued behind the read of fragment p + WAIT_PAIRS - 1 when pair p starts
    template <bool HAS_NEXT>
    static constexpr int newer_ops(int p) {
        int c = 0;
        for (int i = WAIT_PAIRS; i < AHEAD; ++i) c += frag_ops<HAS_NEXT>(p + i);
        return c;
    }
    template <bool HAS_NEXT>
    static constexpr int frag_ops(int q) { return q < KK ? 1 : (q < NP ? 2 : (HAS_NEXT ? 1 : 0)); }

    // Fast half-step j (1 <= j <= nhalf-4): S_in = S(j), P_in = P(j-1) -> S_out = S(j+1), P_out = P(j).
    // kv / vv are this lane's LDS addresses of its K fragments and V fragments inside slot 0,
    // first half (V: first row group); KOFF / VOFF select slot and half of the K tile of
    // S(j+1) and of the V tile of P(j-1).  kpre holds the first AHEAD K fragments, already
    // requested; with HAS_NEXT it is refilled with requests for the following half-step
    // (offset NKOFF).  ROLE 0 = first half-step of an iteration: besides its own work it loads
    // the row numbers of tile next_tile and issues the direct-to-LDS loads of a K tile (LDS
    // offset KW from the wave's base).  ROLE 1 = second half-step: issues the loads of a V tile
    // (offset VW) and holds the workgroup barrier, see steady_iter.
    template <int KOFF, int VOFF, bool HAS_NEXT, int NKOFF, int ROLE, int KW, int VW>
    __device__ __forceinline__ void fast_step(const uint32_t (&kv)[KK], const uint32_t (&vv)[ODB],
                                              bf16x8 (&kpre)[AHEAD],
                                              int next_tile, const rows_t& krows, const rows_t& vrows,
                                              rows_t& rows_n,
                                              f32x16 (&S_in)[2], f32x16 (&S_out)[2],
                                              bf16x8 (&P_in)[2][2], bf16x8 (&P_out)[2][2]) {
        bf16x8 fr[NP + AHEAD];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) fr[i] = kpre[i];
        ExpPipe ep;
        exp_begin(ep);
        fence();
        fast_pairs<KOFF, VOFF, HAS_NEXT, NKOFF, ROLE, KW, VW>(std::make_integer_sequence<int, NP>{}, kv, vv, fr, ep,
                                                              next_tile, krows, vrows, rows_n, S_in, S_out, P_in, P_out);
        exp_end<true>(ep, S_in, P_out);
        if (HAS_NEXT) {
#pragma unroll
            for (int i = 0; i < AHEAD; ++i) kpre[i] = fr[NP + i];
        }
    }
    template <int KOFF, int VOFF, bool HAS_NEXT, int NKOFF, int ROLE, int KW, int VW, int... Ps>
    __device__ __forceinline__ void fast_pairs(std::integer_sequence<int, Ps...>,
                                               const uint32_t (&kv)[KK], const uint32_t (&vv)[ODB],
                                               bf16x8 (&fr)[NP + AHEAD], ExpPipe& ep,
                                               int next_tile, const rows_t& krows, const rows_t& vrows,
                                               rows_t& rows_n,
                                               f32x16 (&S_in)[2], f32x16 (&S_out)[2],
                                               bf16x8 (&P_in)[2][2], bf16x8 (&P_out)[2][2]) {
        (fast_pair<Ps, KOFF, VOFF, HAS_NEXT, NKOFF, ROLE, KW, VW>(kv, vv, fr, ep, next_tile, krows, vrows, rows_n,
                                                                  S_in, S_out, P_in, P_out), ...);
    }
    // MFMA pair P of a fast half-step: two slots that share one A fragment.
    template <int P, int KOFF, int VOFF, bool HAS_NEXT, int NKOFF, int ROLE, int KW, int VW>
    __device__ __forceinline__ void fast_pair(const uint32_t (&kv)[KK], const uint32_t (&vv)[ODB],
                                              bf16x8 (&fr)[NP + AHEAD], ExpPipe& ep,
                                              int next_tile, const rows_t& krows, const rows_t& vrows,
                                              rows_t& rows_n,
                                              f32x16 (&S_in)[2], f32x16 (&S_out)[2],
                                              bf16x8 (&P_in)[2][2], bf16x8 (&P_out)[2][2]) {
        static_assert(LOAD_STRIDE >= 1 && k_addr_pair(CH - 1) + 1 < NP && v_addr_pair(CH - 1) + 1 < NP, "load schedule fits the half-step");
        // Slot layout: MFMA, then the slot's memory and scalar instructions, then its VALU work.
        // (Measured on gfx950 with one wave per SIMD: the first non-VALU instruction after an
        // MFMA issues for free, the same instruction in front of the MFMA delays it.)
        constexpr int PA = P + AHEAD;       // the fragment requested during this pair
        // The fragments of pairs P .. P+WAIT_PAIRS-1 have landed once only the requests made after
        // them are outstanding; the first pair of each such group waits for all of them.
        constexpr bool WAITS = P % WAIT_PAIRS == 0;
        constexpr int NEWER = newer_ops<HAS_NEXT>(P);
        static_assert(NP % WAIT_PAIRS == 0 && AHEAD >= WAIT_PAIRS, "wait groups tile the half-step");
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int s = 2 * P + qb;
            if constexpr (P < KK) {
                if constexpr (P == 0) {
                    if (qb == 0 && WAITS) mfma_qk_first_after<NEWER>(S_out[qb], fr[P], qf[qb][P]);
                    else mfma_qk_first(S_out[qb], fr[P], qf[qb][P]);
                } else {
                    if (qb == 0 && WAITS) mfma_qk_after<NEWER>(S_out[qb], fr[P], qf[qb][P]);
                    else mfma_qk(S_out[qb], fr[P], qf[qb][P]);
                }
            } else {
                constexpr int q = P - KK;
                if (qb == 0 && WAITS) mfma_pv_after<NEWER>(o_acc[qb][q % ODB], fr[P], P_in[qb][q / ODB]);
                else mfma_pv(o_acc[qb][q % ODB], fr[P], P_in[qb][q / ODB]);
            }
            fence();
            if (qb == 0) {
                if constexpr (ROLE == 1 && HAS_V && P == KK) {
                    // All K reads of this iteration are complete (their fragments have been
                    // consumed).  Everything loaded before this iteration's own loads has landed;
                    // after the barrier the other waves' shares are visible too, and the slots
                    // they free may be refilled.
                    wait_vmcnt_at_most<VM_PER_ISSUE>();
                    __builtin_amdgcn_s_barrier();
                }
                if constexpr (ROLE == 0 && P >= 1) {
                    if constexpr (k_addr_at(P - 1) >= 0) issue_load<k_addr_at(P - 1)>(K, dma_off);
                }
                if constexpr (ROLE == 1 && HAS_V && P >= 1) {
                    if constexpr (v_addr_at(P - 1) >= 0) issue_load<v_addr_at(P - 1)>(V, dma_off);
                }
                if constexpr (PA < KK) {
                    fr[PA] = lds_read_b128_at<KOFF>(kv[PA]);
                } else if constexpr (PA < NP) {
                    constexpr int q = PA - KK, hf = q / ODB, db = q % ODB;
                    set_half(fr[PA], 0, lds_read_tr_at<VOFF + hf * 16 * ROW_BYTES>(vv[db]));
                } else if constexpr (HAS_NEXT) {
                    fr[PA] = lds_read_b128_at<NKOFF>(kv[PA - NP]);
                }
            } else {
                if constexpr (PA >= KK && PA < NP) {
                    constexpr int q = PA - KK, hf = q / ODB, db = q % ODB;
                    set_half(fr[PA], 1, lds_read_tr_at<VOFF + hf * 16 * ROW_BYTES + 8 * ROW_BYTES>(vv[db]));
                }
                if constexpr (ROLE == 0) {
                    if constexpr (P == 0) load_rows_async(next_tile, rows_n);
                    constexpr int j = k_addr_at(P);
                    if constexpr (j >= 0) dma_off = issue_addr<KW, j>(row_word(krows, j), koff[j]);
                }
                if constexpr (ROLE == 1 && HAS_V) {
                    constexpr int j = v_addr_at(P);
                    if constexpr (j >= 0) dma_off = issue_addr<VW, j>(row_word(vrows, j), voff[j]);
                }
            }
            fence();
            // this slot's share of the VALU work
#pragma unroll
            for (int i = exp_ticks_before(s); i < exp_ticks_before(s + 1); ++i) exp_tick(i, S_in, P_out, ep);
            // the row sums are complete one slot early: compare now, branch after the last MFMA
            // (Row sums are sums of exp2 results: non-negative, or NaN / +inf.  On their bit patterns the
            // order of the floats is the order of the integers, NaN lies above everything, and the
            // integer maximum needs no canonicalising copies of its operands.)
            if (s == NS - 2) {
                const uint32_t r0 = __builtin_bit_cast(uint32_t, ep.rs[0]), r1 = __builtin_bit_cast(uint32_t, ep.rs[1]);
                ep.bad = __ballot((r0 > r1 ? r0 : r1) > __builtin_bit_cast(uint32_t, kGrowthLimit));
            }
            fence();
        }
    }
    // General half-step (first step, last tile): same work, plus tail masking; no overlap needed.
    __device__ __forceinline__ void general_step(int j, const byte* kbase, const byte* vbase,
                                                 f32x16 (&S_in)[2], f32x16 (&S_out)[2],
                                                 bf16x8 (&P_in)[2][2], bf16x8 (&P_out)[2][2]) {
        if (j >= 1) pv_all(vbase + (((j - 1) >> 1) % NBUF_V) * TILE_BYTES, (j - 1) & 1, P_in);
        exp_half_tile(S_in, P_out);
        if (j + 1 < nhalf) {
            qk_all(kbase + (((j + 1) >> 1) % NBUF_K) * TILE_BYTES, (j + 1) & 1, S_out);
            mfma_settle(S_out[0], S_out[1]);
            mask_tail(j + 1, S_out);
        }
    }
    // One steady-state iteration u (U4 = u % NBUF): half-steps j = 2u+1 and 2u+2, which read K
    // tile u+1 and V tile u.  `last` marks the iteration whose K tile is the last one of the pattern:
    // its scores get the tail mask.  (It still issues loads, of tiles past the end: load_rows hands
    // those the row numbers of the last tile, and the slots they fill are not read again.)  The first half-step issues the loads of K(u+3), the second one
    // those of V(u+2); the second one also holds the barrier -- placed after its last K read, so
    // that K(u+2), V(u+1) are visible to every wave before anything reads them -- and then
    // requests the first K fragments of the next iteration while its P V MFMAs run.
    template <int U4>
    __device__ __forceinline__ void steady_iter(const uint32_t (&kv)[KK], const uint32_t (&vv)[ODB],
                                                bf16x8 (&kpre)[AHEAD], int next_tile,
                                                const rows_t& krows, const rows_t& vrows, rows_t& rows_n,
                                                f32x16 (&SA)[2], f32x16 (&SB)[2],
                                                bf16x8 (&PA)[2][2], bf16x8 (&PB)[2][2], bool last) {
        static_assert(KK >= AHEAD, "the first fragments of a half-step are K fragments");
        constexpr int KR = (U4 + 1) % NBUF * TILE_BYTES;        // K(u+1)
        constexpr int VR = U4 * TILE_BYTES;                     // V(u)
        constexpr int KN = (U4 + 2) % NBUF * TILE_BYTES;        // K(u+2)
        constexpr int KW = (U4 + 3) % NBUF * TILE_BYTES;        // K(u+3), from the wave's chunk base
        constexpr int VW = (NBUF + (U4 + 2) % NBUF) * TILE_BYTES;   // V(u+2), the V slots follow the K slots
        // odd:  S(j) in SB, P(j-1) in PA -> S(j+1) in SA, P(j) in PB
        fast_step<KR, VR, true, KR + HALF_BYTES, 0, KW, VW>(kv, vv, kpre, next_tile, krows, vrows, rows_n, SB, SA, PA, PB);
        if (last) mask_last_tile(0, SA);
        // even: S(j) in SA, P(j-1) in PB -> S(j+1) in SB, P(j) in PA
        fast_step<KR + HALF_BYTES, VR + HALF_BYTES, HAS_V, KN, 1, KW, VW>(kv, vv, kpre, next_tile, krows, vrows, rows_n,
                                                                         SA, SB, PB, PA);
        if (last) mask_last_tile(1, SB);
        if (!HAS_V) {
            // row pass: no P V stream to cover the barrier; synchronise at the end of the iteration
            wait_vmcnt_at_most<VM_PER_ISSUE>();
            __builtin_amdgcn_s_barrier();
#pragma unroll
            for (int i = 0; i < AHEAD; ++i) kpre[i] = lds_read_b128_at<KN>(kv[i]);
        }
    }
};


// Work distribution.  The grid is a fixed set of workgroups (as many as fit the chip at once)
// that take query blocks from eight queues, one per XCD: queue y holds the query blocks of the
// heads 8*hh + y in order, so that at any time an XCD works on one or two heads whose gathered
// K/V rows fit its L2, and a workgroup takes from the queue of the XCD it runs on (read from the
// hardware's XCC id register, so nothing is assumed about the order in which workgroups are dealt
// to the XCDs).  The XCDs of one chip do not run at the same speed (a few percent apart under this
// load): a workgroup whose queue is empty goes on with the next non-empty one instead of idling
// until the slowest XCD is done.
// Counters: work[y] = (launch stamp << 32) | next item of queue y.  The stamp is a number the host
// gives every launch on a context; a counter that carries another stamp is whatever an earlier
// launch left behind (finished, aborted, or never run) and is restarted by the first workgroup
// that notices.  So a launch depends on no state of the launches before it, and nothing has to be
// cleared between launches.
struct WorkQueues {
    unsigned long long* work;
    uint32_t stamp;
    int bh_total, nqb;
    const int32_t* varlen;      // per batch element: its own sequence length (variable-length batches), or nullptr
    int heads;
    __device__ __forceinline__ int items(int y) const { return y < bh_total ? ((bh_total - y + 7) >> 3) * nqb : 0; }
    // item j of queue q is a query block that lies wholly in the padding of its batch element
    __device__ __forceinline__ bool is_padding(int q, int j) const {
        if (varlen == nullptr) return false;
        const int head_block = j / nqb;
        const int qblk = j - head_block * nqb;
        return qblk * BM >= varlen[(head_block * 8 + q) / heads];
    }
    __device__ __forceinline__ int take(int q) const {
        unsigned long long* const counter = work + q;
        unsigned long long v = __hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        while ((uint32_t)(v >> 32) != stamp) {
            unsigned long long cur = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((uint32_t)(cur >> 32) == stamp) {
                v = __hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                continue;
            }
            // restart the counter at item 1 and keep item 0 (fails if another workgroup was faster, or
            // has just added to the stale value: look again)
            const unsigned long long fresh = ((unsigned long long)stamp << 32) | 1ull;
            if (__hip_atomic_compare_exchange_strong(counter, &cur, fresh, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                return 0;
        }
        return (int)(uint32_t)v;
    }
    // One thread: item j taken from queue q is good, or else the first item that the following
    // queues still have; j = -1 when every queue has been found empty.
    __device__ __forceinline__ void settle(int home, int& q, int& j) const {
        for (;;) {
            while (j >= items(q)) {
                q = (q + 1) & 7;
                if (q == home) { j = -1; return; }
                j = take(q);
            }
            if (!is_padding(q, j)) return;
            j = take(q);            // nothing to do for a block of padding rows: on to the next item
        }
    }
};

// the XCD this wave runs on: bits 3:0 of the XCC id hardware register
__device__ __forceinline__ int xcc_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7; }

template <int D, int MODE>
__global__ void __launch_bounds__(NTHREADS) attn_bf16_kernel(AttnParams p) {
    using W = AttnWave<D, MODE>;
    constexpr int CH = W::CH;
    constexpr int KK = W::KK;
    constexpr int ODB = W::ODB;
    constexpr int TILE_BYTES = W::TILE_BYTES;
    constexpr bool HAS_V = W::HAS_V;

    // ONE shared array for all tile slots: with a single LDS object the alias scopes that the
    // restrict parameters give the direct-to-LDS loads are what the compiler's wait-count
    // insertion sees, and LDS reads of one slot do not wait for loads into another.
    // The Q block is turned around in LDS at the start of a query block: a wave's 64 Q rows are one
    // tile's worth of bytes and go through V slot `wave`, which is not needed yet at that point.
    // (The row pass has no V slots; it loads its Q fragments directly.)
    // One more tile behind them is wave 0's share of the output staging area (the other waves use
    // K slots 1..3): K slot 0 then is free for the next query block's first tile at once.
    __shared__ __attribute__((aligned(1024))) byte lds_all[(NBUF_K + (HAS_V ? NBUF_V + 1 : 0)) * TILE_BYTES];
    byte* const lds_k = lds_all;
    byte* const lds_v = lds_all + (HAS_V ? NBUF_K * TILE_BYTES : 0);

    // Fetch every kernel argument with the first batch of scalar loads: left to itself the compiler
    // loads them where they are first used, one memory round trip after another.
    asm volatile("" : : "s"(p.q), "s"(p.k), "s"(p.v), "s"(p.o), "s"(p.idx), "s"(p.lse), "s"(p.lse_base2),
                         "s"(p.td.sb), "s"(p.td.sh), "s"(p.td.sn), "s"(p.td_kv.sb), "s"(p.td_kv.sh), "s"(p.td_kv.sn),
                         "s"(p.kv_heads), "s"(p.batch), "s"(p.heads), "s"(p.n), "s"(p.ns), "s"(p.groups),
                         "s"(p.group_size), "s"(p.scale), "s"(p.work), "s"(p.work_stamp), "s"(p.varlen), "s"(p.idx_stride));
    const int nqb = (p.n + BM - 1) / BM;
    const WorkQueues queues{p.work, p.work_stamp, p.batch * p.heads, nqb, p.varlen, p.heads};
    __shared__ int32_t lds_item[2];          // the workgroup's next item: queue, index in the queue
    const int home = xcc_id();
    if (threadIdx.x == 0) {
        int q = home, j = queues.take(home);
        queues.settle(home, q, j);
        lds_item[0] = q;
        lds_item[1] = j;
    }
    __syncthreads();
    int cur_q = __builtin_amdgcn_readfirstlane(lds_item[0]), cur_j = __builtin_amdgcn_readfirstlane(lds_item[1]);

    // the geometry that requesting a query block's first loads needs
    W wq;
    wq.lane = threadIdx.x & 63;
    wq.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    wq.ns = p.ns;
    wq.ntiles = (p.ns + BN - 1) / BN;
    wq.lrow = wq.lane / W::PIECES;
    wq.idx = nullptr;
    // Rows and attended columns of a head: the context's, or (variable-length batches) those of the
    // head's batch element: its own length, and of its column sets the leading `kept` entries.
    auto lens_of = [&](int bh, int& rows, int& cols) {
        rows = p.n;
        cols = p.ns;
        if (p.varlen != nullptr) {
            const int b = bh / p.heads;
            rows = p.varlen[b];
            const int kept = p.varlen[p.batch + b];
            cols = W::GATHER ? (kept < p.ns ? kept : p.ns) : rows;
        }
    };
    // item (queue, index) -> head and query block; pointers of a head
    auto decode = [&](int q, int j, int& bh, int& qblk) {
        const int head_block = j / nqb;
        qblk = j - head_block * nqb;
        bh = head_block * 8 + q;
    };
    auto q_of = [&](int bh) {
        const int b = bh / p.heads, h = bh - b * p.heads;
        return (int64_t)b * p.td.sb + (int64_t)h * p.td.sh;
    };
    // the column set of a query block's group (Sec. 3.3: one set per query group)
    auto pattern_of = [&](int bh, int qblk) -> const byte* {
        const int group = p.groups > 1 ? (qblk * BM) / p.group_size : 0;
        return W::GATHER ? (const byte*)(p.idx + ((int64_t)bh * p.groups + group) * p.idx_stride) : nullptr;
    };

    // What a query block needs first, requested ahead of its turn (for the first one: now; for
    // the others: from the epilogue of the block before, once no wave reads the V slots any more):
    // the row numbers of tiles 0..3 and the Q block.  Q is loaded like a K tile -- whole rows
    // straight into LDS, 16 lanes per row, swizzled on the global side -- and read back as
    // B-operand fragments [query lq][d = kk*16 + 8*lh .. +7].  (A direct load of a fragment
    // touches 32 rows x 32 bytes, four instructions per 128-byte line, and the block does not
    // fit the vector cache.)  Each wave stages its own 64 rows.
    typename W::rows_t rows_k, rows_v, rows_n, rows_0, rows_1;
    static_assert(PRO_TILES == 3, "the prologue is written out for three tiles");
    constexpr int Q_LOADS = HAS_V ? TILE_BYTES / 1024 : 0;        // direct-to-LDS loads of a wave's share of Q
    const byte* req_q = nullptr;          // the requested block's head of Q, and its first row for this wave
    int req_q0 = 0, req_n = p.n;          // ... and the rows of that head
    auto request_rows = [&](int q, int j) {
        int bh, qblk;
        decode(q, j, bh, qblk);
        lens_of(bh, req_n, wq.ns);
        wq.ntiles = (wq.ns + BN - 1) / BN;
        const byte* const pattern = pattern_of(bh, qblk);
        wq.load_rows(pattern, 0, rows_0);
        wq.load_rows(pattern, 1, rows_1);
        wq.load_rows(pattern, 2, rows_v);
        wq.load_rows(pattern, 3, rows_k);
        req_q = (const byte*)((const __bf16*)p.q + q_of(bh));
        req_q0 = qblk * BM + wq.wave * 64;
    };
    // The copy itself, loads t0 .. t1-1 of the wave's Q_LOADS: assembly like the gathers of the
    // steady loop (one LDS base in m0 per four loads, told apart by the instruction offset, which
    // the hardware adds on both sides; 24-bit multiply-add for the row offset).  The compiler does
    // not see these loads: the wait in front of the fragment reads is the prologue's own.
    const uint32_t q_row_bytes = (uint32_t)p.td.sn * 2u;
    const uint32_t qstage_lds = __builtin_amdgcn_readfirstlane(lds_address(lds_v) + wq.wave * TILE_BYTES);
    uint32_t q_piece[4];                  // byte offset of this lane's piece inside a Q row, per load of a group
    {
        constexpr int RPC = W::ROWS_PER_CHUNK, PIECES = W::PIECES;
        const int lrow = wq.lane / PIECES, lpiece = wq.lane % PIECES;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) q_piece[jj] = (uint32_t)((lpiece ^ swizzle_k<PIECES>(jj * RPC + lrow)) << 4);
        static_assert((4 * RPC) % PIECES == 0, "the swizzle of a row repeats every four loads");
    }
    auto request_q = [&](auto t0_c, auto t1_c) {
        if constexpr (HAS_V) {
            constexpr int t0 = decltype(t0_c)::value, t1 = decltype(t1_c)::value;
            static_assert(t0 % 4 == 0 && t1 % 4 == 0, "whole groups of four loads");
            constexpr int RPC = W::ROWS_PER_CHUNK;
            const int row0 = req_q0 + wq.lane / W::PIECES;
#pragma unroll
            for (int t = t0; t < t1; ++t) {
                int row = row0 + t * RPC;
                row = row < req_n ? row : req_n - 1;
                uint32_t off;
                if (t % 4 == 0) {
                    asm volatile("s_add_i32 m0, %1, %2\n\tv_mad_u32_u24 %0, %3, %4, %5"
                                 : "=v"(off) : "s"(qstage_lds), "s"((uint32_t)(t * 1024)), "v"(row), "s"(q_row_bytes), "v"(q_piece[0]));
                } else {
                    asm volatile("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(off) : "v"(row), "s"(q_row_bytes), "v"(q_piece[t % 4]));
                }
                switch (t % 4) {
                    case 0: asm volatile("global_load_lds_dwordx4 %0, %1 offset:0" : : "v"(off), "s"(req_q) : "memory"); break;
                    case 1: asm volatile("global_load_lds_dwordx4 %0, %1 offset:1024" : : "v"(off), "s"(req_q - 1024) : "memory"); break;
                    case 2: asm volatile("global_load_lds_dwordx4 %0, %1 offset:2048" : : "v"(off), "s"(req_q - 2048) : "memory"); break;
                    default: asm volatile("global_load_lds_dwordx4 %0, %1 offset:3072" : : "v"(off), "s"(req_q - 3072) : "memory"); break;
                }
            }
        }
    };
    auto request_q_all = [&] { request_q(std::integral_constant<int, 0>{}, std::integral_constant<int, Q_LOADS>{}); };
    if (cur_j >= 0) { request_rows(cur_q, cur_j); request_q_all(); }

  bool k0_on_its_way = false;
  while (cur_j >= 0) {
    int bh, qblk;
    decode(cur_q, cur_j, bh, qblk);
    W w;
    const int tid = threadIdx.x;
    w.lane = tid & 63;
    w.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    w.lq = w.lane & 31;
    w.lh = w.lane >> 5;
    lens_of(bh, w.n, w.ns);
    const int n = w.n;
    w.ntiles = (w.ns + BN - 1) / BN;
    w.nhalf = 2 * w.ntiles;
    w.ragged = (w.ns & (BN - 1)) != 0;
    w.row_bytes = (uint32_t)p.td_kv.sn * 2u;
    w.wave_lds = __builtin_amdgcn_readfirstlane(lds_address(lds_k) + w.wave * CH * 1024);
    w.idx = nullptr;
    w.c2 = p.scale * kLog2e;                 // exp(z*scale) = exp2(z*c2)
    w.init_addresses();
    const int nhalf = w.nhalf;
    byte* const qstage = lds_v + w.wave * TILE_BYTES;      // HAS_V only

    const int b = bh / p.heads, h = bh - b * p.heads;
    const int64_t head_off = q_of(bh);
    // grouped-query layout: query head h reads K/V head h / (heads / kv_heads)
    const int64_t kv_off = (int64_t)b * p.td_kv.sb + (int64_t)(h / (p.heads / p.kv_heads)) * p.td_kv.sh;
    const __bf16* __restrict__ Q = (const __bf16*)p.q + head_off;
    w.K = (const byte*)((const __bf16*)p.k + kv_off);
    w.V = HAS_V ? (const byte*)((const __bf16*)p.v + kv_off) : nullptr;
    w.idx = pattern_of(bh, qblk);
    w.mc[0] = w.mc[1] = -INFINITY;
    w.l_run[0] = w.l_run[1] = 0.f;
    const int q0 = qblk * BM + w.wave * 64;

    // ---- prologue.  The vector memory pipe returns loads in issue order, so each wait names how
    // many of the youngest loads may still be in flight:
    //   (requested ahead: row numbers of tiles 0..3, Q), K(0)  -> everything has landed -> S(0), S(1)
    //   V(0), K(1), V(1), K(2)              -> the last two may be in flight -> first iteration
    //                                       -> its own barrier covers V(1), K(2)
    // (V(2) is loaded by the first iteration itself.)  Afterwards rows_v = tile 2, rows_k = tile 3.
    if constexpr (!HAS_V) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            int row = q0 + qb * 32 + w.lq;
            row = row < n ? row : n - 1;
            const __bf16* src = Q + (int64_t)row * p.td.sn + 8 * w.lh;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) w.qf[qb][kk] = *(const bf16x8*)(src + kk * 16);
        }
    }
    if (!k0_on_its_way) w.issue_k_tile(lds_k, w.K, rows_0);      // else: issued from the epilogue of the block before
    constexpr int LATER_LOADS = CH * (HAS_V ? 4 : 2);     // V(0), K(1), V(1), K(2): issued behind the first barrier
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < ODB; ++db) {
#pragma unroll
            for (int r = 0; r < 16; ++r) w.o_acc[qb][db][r] = 0.f;
            asm volatile("" : "+a"(w.o_acc[qb][db]));
        }
    wait_vmcnt_at_most<0>();
    fence();                        // the compiler does not know that the Q copy wrote what is read next
    if constexpr (HAS_V) {          // all fragment reads, then one wait
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) w.qf[qb][kk] = *(const bf16x8*)(qstage + qb * W::HALF_BYTES + w.kaddr[kk]);
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) asm volatile("" : "+a"(w.qf[qb][kk]));
    __builtin_amdgcn_s_barrier();
    // The next tiles go out now, in the order of need, and arrive while the first half-steps run
    // (issued in front of the first wait they would have held the wave for as long as they queue
    // in the memory pipe).
    w.issue_v_tile(lds_v, w.V, rows_0);
    w.issue_k_tile(lds_k + TILE_BYTES, w.K, rows_1);
    w.issue_v_tile(lds_v + (HAS_V ? TILE_BYTES : 0), w.V, rows_1);
    w.issue_k_tile(lds_k + 2 * TILE_BYTES, w.K, rows_v);

    f32x16 SA[2], SB[2];
    bf16x8 PA[2][2], PB[2][2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int e = 0; e < 8; ++e) { PA[qb][hf][e] = (__bf16)0.f; PB[qb][hf][e] = (__bf16)0.f; }
    w.qk_all(lds_k, 0, SA);
    mfma_settle(SA[0], SA[1]);
    w.mask_tail(0, SA);
    // The first half-tile sets the softmax reference directly (it is the maximum seen so far, so no term
    // can overflow), which keeps the first step off the slow reference-update path.
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) w.mc[qb] = w.half_tile_max(SA[qb]) * w.c2;

    // j = 0: S(0) in SA -> P(0) in PA, S(1) in SB
    w.general_step(0, lds_k, lds_v, SA, SB, PB, PA);

    // ---- steady state: iteration u runs half-steps 2u+1 and 2u+2, u = 0 .. ntiles-2; the last
    // one forms the scores of the last tile.
    const int niter = w.ntiles - 1;
    if (niter > 0) {
        wait_vmcnt_at_most<LATER_LOADS / 2>();            // V(0) and K(1) have landed ...
        __builtin_amdgcn_s_barrier();                     // ... in every wave
        const uint32_t kbase = lds_address(lds_k), vbase = lds_address(lds_v);
        uint32_t kv[KK], vv[ODB];      // fragment addresses inside slot 0; slots and halves are immediates
        constexpr int AHEAD = W::AHEAD;
        bf16x8 kpre[AHEAD];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kv[kk] = kbase + w.kaddr[kk];
#pragma unroll
        for (int db = 0; db < ODB; ++db) vv[db] = vbase + w.vaddr[db];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) kpre[i] = lds_read_b128_at<TILE_BYTES>(kv[i]);     // K tile 1
        // rows_k / rows_v / rows_n rotate by name: after an iteration, v <- k <- n
        int u = 0;
        for (; u + NBUF < niter; u += NBUF) {
            w.template steady_iter<0>(kv, vv, kpre, u + 4, rows_k, rows_v, rows_n, SA, SB, PA, PB, false);
            w.template steady_iter<1>(kv, vv, kpre, u + 5, rows_n, rows_k, rows_v, SA, SB, PA, PB, false);
            w.template steady_iter<2>(kv, vv, kpre, u + 6, rows_v, rows_n, rows_k, SA, SB, PA, PB, false);
            w.template steady_iter<3>(kv, vv, kpre, u + 7, rows_k, rows_v, rows_n, SA, SB, PA, PB, false);
            { const typename W::rows_t t = rows_n; rows_n = rows_v; rows_v = rows_k; rows_k = t; }
        }
        const int rem = niter - u;     // 1 .. NBUF iterations left
        w.template steady_iter<0>(kv, vv, kpre, u + 4, rows_k, rows_v, rows_n, SA, SB, PA, PB, rem == 1);
        if (rem >= 2) w.template steady_iter<1>(kv, vv, kpre, u + 5, rows_n, rows_k, rows_v, SA, SB, PA, PB, rem == 2);
        if (rem >= 3) w.template steady_iter<2>(kv, vv, kpre, u + 6, rows_v, rows_n, rows_k, SA, SB, PA, PB, rem == 3);
        if (rem >= 4) w.template steady_iter<3>(kv, vv, kpre, u + 7, rows_k, rows_v, rows_n, SA, SB, PA, PB, true);
        // The last iteration has requested fragments for a next one that does not exist: their
        // registers must stay reserved until the data has arrived.
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kpre[i]));
    }
    // ---- tail: the last half-step, then the last P V product.
    // The wait names the row-number registers: loads into them that nobody reads any more are
    // still in flight, and the registers must not be handed to other values before they land.
    // It also lets the loads of tiles past the end land before the epilogue reuses the slots.
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(rows_k), "+v"(rows_v), "+v"(rows_n) : : "memory");
    __builtin_amdgcn_s_barrier();
    // The next item is asked for now: late, so that it is not held back for long from workgroups
    // that have nothing left to do, and early enough for the answer to be there when the output
    // tile has been staged (nothing else is in flight in between).
    int early_j = 0;
    if (threadIdx.x == 0) early_j = queues.take(cur_q);
    w.general_step(nhalf - 1, lds_k, lds_v, SB, SA, PA, PB);

    w.pv_all(lds_v + (HAS_V ? (((nhalf - 1) >> 1) % NBUF_V) * TILE_BYTES : 0), (nhalf - 1) & 1, PB);

    // ---- epilogue: O = diag(l)^-1 acc, optional row log-sum-exp; hand-over to the next item.
    // In the accumulator a lane holds one query row in 8-byte runs: stored directly, every
    // instruction would touch 64 different rows.  Each wave turns its 64 x D tile around in
    // its own piece of LDS (16-byte pieces XOR-swizzled by row against bank conflicts) and
    // writes whole rows, 16 bytes per lane.  The staging area is K slots 1..3 and the spare tile:
    // no wave reads K after the barrier above, and the loads that were still writing there have
    // landed.
    float l_tot[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        l_tot[qb] = half_sum(w.l_run[qb]);
        const int row = q0 + qb * 32 + w.lq;
        if (p.lse != nullptr && w.lh == 0 && row < n)
            p.lse[(int64_t)bh * p.n + row] = (w.mc[qb] + fast_log2(l_tot[qb])) * (p.lse_base2 ? 1.0f : kLn2);
    }
    constexpr int OUT_GROUPS = 64 / W::ROWS_PER_CHUNK;
    const int out_lrow = w.lane / W::PIECES, out_lpiece = w.lane % W::PIECES;
    byte* const obase = (byte*)((__bf16*)p.o + head_off) + (int64_t)(q0 + out_lrow) * p.td.sn * 2 + out_lpiece * 16;
    const int64_t group_stride = (int64_t)W::ROWS_PER_CHUNK * p.td.sn * 2;      // bytes between row groups (uniform)

    // The next item.  Behind this barrier every wave has issued its last P V product, so no wave
    // reads the V slots any more and the next block's Q copy may land there; its first loads go
    // out now, spread over the staging of this block's output (the copy comes from memory and
    // holds the wave at every instruction while the memory pipe is full), and ahead of this
    // block's stores.  (The taken index is read in front of every store: its wait would cover
    // them too.)
    const int next_j = __builtin_amdgcn_readfirstlane(early_j);       // meaningful in wave 0 only
    if (threadIdx.x == 0) {
        int q = cur_q, j = next_j;
        queues.settle(home, q, j);
        lds_item[0] = q;
        lds_item[1] = j;
    }
    __syncthreads();
    cur_q = __builtin_amdgcn_readfirstlane(lds_item[0]);
    cur_j = __builtin_amdgcn_readfirstlane(lds_item[1]);
    const bool more = cur_j >= 0;
    if (more) request_rows(cur_q, cur_j);
    if constexpr (HAS_V) {
        constexpr int PIECES = W::PIECES, ROW_BYTES = W::ROW_BYTES, RPC = W::ROWS_PER_CHUNK;
        static_assert(64 * ROW_BYTES <= TILE_BYTES && Q_LOADS % ODB == 0, "a wave's output tile fits one tile slot");
        mfma_settle_acc(w.o_acc);
        byte* const stage = lds_all + (w.wave == 0 ? NBUF_K + NBUF_V : w.wave) * TILE_BYTES;
        const float inv[2] = {1.0f / l_tot[0], 1.0f / l_tot[1]};
        static_assert((Q_LOADS / ODB) % 4 == 0, "whole groups of four loads per d-block");
        const auto stage_db = [&](auto db_c) {
            constexpr int db = decltype(db_c)::value;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const int r = qb * 32 + w.lq;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    bf16x4 o4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(w.o_acc[qb][db][r4 * 4 + e] * inv[qb]);
                    *(bf16x4*)(stage + r * ROW_BYTES + (((db * 4 + r4) ^ (r & (PIECES - 1))) << 4) + 8 * w.lh) = o4;
                }
            }
            fence();
        };
        // piece db of the next block's Q copy
        const auto request_q_piece = [&](auto db_c) {
            constexpr int db = decltype(db_c)::value;
            if (more) request_q(std::integral_constant<int, db * (Q_LOADS / ODB)>{}, std::integral_constant<int, (db + 1) * (Q_LOADS / ODB)>{});
        };
        stage_db(std::integral_constant<int, 0>{});
        // The next block's first K tile goes out as soon as its row numbers are there (they were
        // requested a d-block of staging ago; the compiler's wait for them drains the vector
        // memory pipe, so nothing else is put in flight before it): K slot 0 is not part of the
        // staging area and no wave reads K any more, and the tile lands while the stores queue.
        k0_on_its_way = more;
        if (more) {
            int nbh, nqblk;
            decode(cur_q, cur_j, nbh, nqblk);
            const int nb = nbh / p.heads, nh = nbh - nb * p.heads;
            const int64_t nkv = (int64_t)nb * p.td_kv.sb + (int64_t)(nh / (p.heads / p.kv_heads)) * p.td_kv.sh;
            w.issue_k_tile(lds_k, (const byte*)((const __bf16*)p.k + nkv), rows_0);
        }
        request_q_piece(std::integral_constant<int, 0>{});
        if constexpr (ODB > 1) { stage_db(std::integral_constant<int, 1>{}); request_q_piece(std::integral_constant<int, 1>{}); }
        if constexpr (ODB > 2) {
            stage_db(std::integral_constant<int, 2>{}); request_q_piece(std::integral_constant<int, 2>{});
            stage_db(std::integral_constant<int, 3>{}); request_q_piece(std::integral_constant<int, 3>{});
        }
        // all reads first, then the stores: one LDS round trip instead of one per row group
        u32x4 rows_out[OUT_GROUPS];
#pragma unroll
        for (int t = 0; t < OUT_GROUPS; ++t) {
            const int r = t * RPC + out_lrow;
            rows_out[t] = *(const u32x4*)(stage + r * ROW_BYTES + ((out_lpiece ^ (r & (PIECES - 1))) << 4));
        }
        fence();
#pragma unroll
        for (int t = 0; t < OUT_GROUPS; ++t) {
            const int r = t * RPC + out_lrow;
            if (q0 + r < n) *(u32x4*)(obase + t * group_stride) = rows_out[t];
        }
    }
  }

}

// workgroups that one CU holds at a time (LDS and registers): the row pass fits two
template <int MODE> constexpr int wg_per_cu() { return MODE == kLseOnly ? 2 : 1; }

template <int D, int MODE>
hipError_t launch(const AttnParams& p, hipStream_t s) {
    if (p.work == nullptr) return hipErrorInvalidValue;
    const int64_t items = (int64_t)((p.n + BM - 1) / BM) * p.batch * p.heads;
    const int64_t resident = (int64_t)compute_units() * wg_per_cu<MODE>();
    const int grid = (int)(items < resident ? items : resident);
    hipLaunchKernelGGL((attn_bf16_kernel<D, MODE>), dim3(grid), dim3(NTHREADS), 0, s, p);
    return hipGetLastError();
}

}  // namespace

int compute_units() {
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        cached[dev] = (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : 256;
    }
    return cached[dev];
}

hipError_t launch_attn_bf16(const AttnParams& p, int head_dim, AttnMode mode, hipStream_t s) {
    if (head_dim == 128) {
        if (mode == kSparse) return launch<128, kSparse>(p, s);
        if (mode == kBlock) return launch<128, kBlock>(p, s);
        if (mode == kDense) return launch<128, kDense>(p, s);
        return launch<128, kLseOnly>(p, s);
    }
    if (head_dim == 64) {
        if (mode == kSparse) return launch<64, kSparse>(p, s);
        if (mode == kBlock) return launch<64, kBlock>(p, s);
        if (mode == kDense) return launch<64, kDense>(p, s);
        return launch<64, kLseOnly>(p, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace pulsecol
