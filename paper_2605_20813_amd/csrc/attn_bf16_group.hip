// Column-sparse attention for query groups smaller than the 256-row query block of the main
// bf16 kernel (Sec. 3.3: group-wise sets with G = 32, 64 or 128 queries; Sec. 3.4 and the
// appendix listing "Column-Sparse Attention Forward" for the computation itself).
//
// With one column set per small group nothing is shared between neighbouring query blocks
// any more: every group gathers its own K/V rows, the arithmetic intensity is G flop per
// gathered byte, and the kernel lives on the memory side of the roofline.  So this is the
// plain formulation, not the hand-scheduled one: a workgroup = one query block of
// 32 * QB * NW rows (NW waves, QB blocks of 32 queries per wave), tiles of 32 gathered rows
// that go straight from global memory into one of three LDS slots per operand (direct-to-LDS
// loads, issued two tiles ahead of their use; several workgroups per CU hide the rest of the
// gather latency), online softmax against a lazily raised reference.
// Same MFMA orientation as the main kernel: S^T = K_tile Q^T, O^T = V^T P^T, P in registers.
// Everything here is ordinary compiler-scheduled code: the only hand-placed instructions are
// the waits and barriers that order the direct-to-LDS loads against the LDS reads.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

typedef unsigned char byte;

constexpr int BN = 32;      // gathered rows per tile
constexpr float kGrowthLimit = 256.0f;      // 2^kTau with kTau = 8, as in the main kernel

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

// One tile of K and of V, this wave's share: CH direct-to-LDS loads per operand, each moving
// 64 x 16 bytes into the 1 KB chunk (wave*CH + i) of the slot.  Lane L lands at chunk byte 16*L,
// i.e. tile row chunk*RPC + L/PIECES, LDS piece L%PIECES, and therefore fetches the global piece
// (L%PIECES) ^ swizzle(row) of its row: koff / voff hold that piece's byte offset inside a row.
// (The slot pointers are restrict parameters so that the loads carry alias scopes: the compiler
// then does not make LDS reads of the other slots wait for these loads.)
template <int CH>
__device__ __forceinline__ void issue_tile(byte* __restrict__ kslot, byte* __restrict__ vslot,
                                           const byte* __restrict__ Kg, const byte* __restrict__ Vg,
                                           const int (&rows)[CH], const uint32_t (&koff)[CH],
                                           const uint32_t (&voff)[CH], uint32_t row_bytes, int wave) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        // both factors are below 2^24 and the product below 2^32 (checked on the host)
        const uint32_t off = __umul24((uint32_t)rows[i], row_bytes);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Kg + (off + koff[i])),
                                         (PULSECOL_LDS void*)(kslot + (wave * CH + i) * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Vg + (off + voff[i])),
                                         (PULSECOL_LDS void*)(vslot + (wave * CH + i) * 1024), 16, 0, 0);
    }
}

// NBUF = LDS tile slots per operand: one being read, NBUF-1 on their way (2 or 3).  A third slot
// buys a second tile of lead for the gathers and costs workgroups per CU (LDS); which one wins was
// measured per workgroup size, see launch_by_block.  The 4-wave kernel is held to the register
// budget of three waves per SIMD, so that three workgroups share a CU (it fits without spills).
template <int D, int QB, int NW, int NBUF>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW == 4 ? 3 : 1)))
attn_bf16_group_kernel(AttnParams p) {
    constexpr int BM = 32 * QB * NW;
    constexpr int PIECES = D / 8;                 // 16-byte pieces per row
    constexpr int KK = D / 16;                    // contraction steps of Q K^T
    constexpr int DB = D / 32;                    // 32-wide blocks of the head dimension
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = BN * ROW_BYTES;
    constexpr int RPC = 64 / PIECES;              // tile rows per 1 KB chunk
    constexpr int CH = TILE_BYTES / 1024 / NW;    // chunks per wave, tile and operand
    static_assert(CH >= 1 && CH * NW * 1024 == TILE_BYTES, "the waves' chunks cover the tile exactly");
    static_assert(NBUF == 2 || NBUF == 3, "the loop below is unrolled over the slots");
    constexpr int DIST = NBUF - 1;                // tiles between a load and its use

    // one array per slot: distinct objects, so that reads of one slot are known not to touch another
    // (a slot that no code path names takes no LDS)
    __shared__ __attribute__((aligned(1024))) byte lds_k0[TILE_BYTES], lds_k1[TILE_BYTES], lds_k2[TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) byte lds_v0[TILE_BYTES], lds_v1[TILE_BYTES], lds_v2[TILE_BYTES];

    const int nqb = (p.n + BM - 1) / BM;
    int bh, qblk;
    if (!xcd_tile(blockIdx.x, nqb, p.batch * p.heads, &bh, &qblk)) return;
    const int b = bh / p.heads, h = bh - b * p.heads;
    const int64_t head_off = (int64_t)b * p.td.sb + (int64_t)h * p.td.sh;
    // grouped-query layout: query head h reads K/V head h / (heads / kv_heads)
    const int64_t kv_off = (int64_t)b * p.td_kv.sb + (int64_t)(h / (p.heads / p.kv_heads)) * p.td_kv.sh;
    const __bf16* __restrict__ Q = (const __bf16*)p.q + head_off;
    const byte* __restrict__ K = (const byte*)((const __bf16*)p.k + kv_off);
    const byte* __restrict__ V = (const byte*)((const __bf16*)p.v + kv_off);
    // the column set of this query block's group; group_size is a multiple of BM
    const int group = p.groups > 1 ? (qblk * BM) / p.group_size : 0;
    const int32_t* __restrict__ idx = p.idx + ((int64_t)bh * p.groups + group) * p.ns;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31;       // query column (and K/V row) this lane owns inside a 32-block
    const int lh = lane >> 5;       // which half of the wave
    // variable-length batches: the batch element's own length, and the leading `kept` entries of its sets
    int n = p.n, ns = p.ns;
    if (p.varlen != nullptr) {
        n = p.varlen[b];
        const int kept = p.varlen[p.batch + b];
        ns = kept < ns ? kept : ns;
        if (qblk * BM >= n) return;         // a block of padding rows
    }
    const int ntiles = (ns + BN - 1) / BN;
    const uint32_t row_bytes = (uint32_t)p.td_kv.sn * 2u;

    // ---- Q fragments: B operand, [query lq][d = kk*16 + 8*lh .. +7]
    const int q0 = qblk * BM + wave * (32 * QB);
    bf16x8 qf[QB][KK];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int row = q0 + qb * 32 + lq;
        row = row < n ? row : n - 1;
        const __bf16* src = Q + (int64_t)row * p.td.sn + 8 * lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[qb][kk] = *(const bf16x8*)(src + kk * 16);
    }

    // ---- gather geometry of this lane: chunk i of its wave covers tile row trow[i]
    int trow[CH];
    uint32_t koff[CH], voff[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        trow[i] = (wave * CH + i) * RPC + lane / PIECES;
        koff[i] = (uint32_t)((lane % PIECES) ^ swizzle_k<PIECES>(trow[i])) * 16u;
        voff[i] = (uint32_t)((lane % PIECES) ^ swizzle_v<PIECES>(trow[i])) * 16u;
    }
    // K/V row numbers of tile t for this lane's chunks.  Positions past the end of the pattern
    // (ragged tail, tiles past the last one) take the pattern's last entry: a valid row, whose
    // scores the tail mask removes or whose slot is never read.
    auto load_rows = [&](int t, int (&dst)[CH]) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const uint32_t pos = (uint32_t)(t * BN + trow[i]);          // unsigned: a 32-bit offset from the uniform base
            dst[i] = idx[pos < (uint32_t)ns ? pos : (uint32_t)(ns - 1)];
        }
    };

    // ---- fragment addresses inside a slot: what differs between slots and between the halves of
    // a tile are constants, which the reads carry as instruction offsets
    // K fragment kk: tile row lq, piece 2*kk + lh
    uint32_t kaddr[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kaddr[kk] = (uint32_t)(lq * ROW_BYTES + (((2 * kk + lh) ^ swizzle_k<PIECES>(lq)) << 4));
    // V fragment of d-block db, contraction element e of this lane <-> tile row hf*16 + 8*(e/4) + 4*lh + e%4:
    // the transposing read takes the address of row 4*lh + j16/4 (then +8, and +16 for hf = 1: rows
    // with the same swizzle), 8 bytes at d = db*32 + 16*((lane/16)&1) + 4*(j16%4), j16 = lane%16
    uint32_t vaddr[DB];
    {
        const int j16 = lane & 15;
        const int row0 = 4 * lh + (j16 >> 2);
        const int colpiece = ((lane >> 4) & 1) * 2 + ((j16 & 3) >> 1);   // 16-byte piece inside the 64-byte d-block
        const int inpiece = (j16 & 1) * 8;                               // byte inside the piece
        static_assert(PIECES >= 8, "rows 8 and 16 apart share a swizzle");
#pragma unroll
        for (int db = 0; db < DB; ++db)
            vaddr[db] = (uint32_t)(row0 * ROW_BYTES + inpiece + (((db * 4 + colpiece) ^ swizzle_v<PIECES>(row0)) << 4));
    }

    const float c2 = p.scale * kLog2e;      // exp(z*scale) = exp2(z*c2)
    float ref[QB], l_run[QB];               // l: per-lane partial, sums only this lane's keys
    f32x16 o_acc[QB][DB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        ref[qb] = 0.f;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[qb][db][r] = 0.f;
    }

    // ---- everything a tile contributes, read from its two slots
    auto compute_tile = [&](int t, const byte* __restrict__ kslot, const byte* __restrict__ vslot) {
        // ---- S^T = K_tile Q^T  (32 keys x 32 queries per query block)
        f32x16 s[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[qb][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const bf16x8 a = *(const bf16x8*)(kslot + kaddr[kk]);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) s[qb] = mfma_bf16(a, qf[qb][kk], s[qb]);
        }

        // ---- ragged tail of the last tile: columns past ns get weight zero
        if (t == ntiles - 1 && (ns & (BN - 1))) {
            const int valid = ns - t * BN;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (acc_row(r, lh) >= valid) {
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) s[qb][r] = -INFINITY;
                }
        }

        // ---- online softmax (per lane: one query column per query block) against a reference
        // that moves only when it must: P = exp2(z*c2 - ref) with ref = the maximum of the first
        // tile, raised by whole log2 units once some lane's weights of a tile sum to more than
        // 2^kTau.  Until then nothing is rescaled; l and the accumulator share one reference, so
        // the quotient at the end is the softmax all the same.
        bf16x8 pfrag[QB][2];     // [qb][half of the 32-row tile]
        float rs[QB];
        bool grown = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if (t == 0) {
                float mx = s[qb][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[qb][r]);
                ref[qb] = half_max(mx) * c2;                 // finite: row 0 of a tile is always valid
            }
            rs[qb] = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float e = fast_exp2(__builtin_fmaf(s[qb][r], c2, -ref[qb]));
                rs[qb] += e;
                pfrag[qb][r >> 3][r & 7] = (__bf16)e;
            }
            grown |= !(rs[qb] <= kGrowthLimit);              // also true for NaN
        }
        if (__builtin_expect(__ballot(grown) != 0ull, 0)) {
            // slow path: true maximum of the tile per query, reference up by a whole number of
            // log2 units, l and the accumulator scaled by that exact power of two, P recomputed
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = s[qb][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[qb][r]);
                const float m2 = half_max(mx) * c2;          // same value in both half-waves
                if (m2 > ref[qb] + 1.0f) {
                    const float steps = ceilf(m2 - ref[qb]);
                    const float alpha = fast_exp2(-steps);
                    ref[qb] += steps;
                    l_run[qb] *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o_acc[qb][db][r] *= alpha;
                    rs[qb] = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = fast_exp2(__builtin_fmaf(s[qb][r], c2, -ref[qb]));
                        rs[qb] += e;
                        pfrag[qb][r >> 3][r & 7] = (__bf16)e;
                    }
                }
            }
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) l_run[qb] += rs[qb];

        // ---- O^T += V^T P^T
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x4 lo = lds_read_tr(vslot + vaddr[db] + hf * 16 * ROW_BYTES);
                const bf16x4 hi = lds_read_tr(vslot + vaddr[db] + hf * 16 * ROW_BYTES + 8 * ROW_BYTES);
                const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) o_acc[qb][db] = mfma_bf16(a, pfrag[qb][hf], o_acc[qb][db]);
            }
        }

    };

    // ---- the first DIST tiles go out; the row numbers of tile DIST wait in registers
    int rows_next[CH];
    {
        int rows_0[CH], rows_1[CH];
        load_rows(0, rows_0);
        if constexpr (DIST == 2) load_rows(1, rows_1);
        load_rows(DIST, rows_next);
        issue_tile<CH>(lds_k0, lds_v0, K, V, rows_0, koff, voff, row_bytes, wave);
        if constexpr (DIST == 2) issue_tile<CH>(lds_k1, lds_v1, K, V, rows_1, koff, voff, row_bytes, wave);
    }

    // Step t: tile t has landed in every wave once this wave's loads of the tiles after it are the
    // only ones it still may have in flight (vector memory completes in issue order, and whatever
    // this step issues comes later still) and all waves have said so at the barrier.  The barrier
    // also tells that every wave has finished reading tile t-1, whose slot the loads of tile
    // t+DIST now refill.  Loads are issued for tiles past the end as well (valid rows, slots
    // never read), so the count in flight is the same at every step.
    auto step = [&](int t, const byte* __restrict__ kcur, const byte* __restrict__ vcur,
                    byte* __restrict__ kfill, byte* __restrict__ vfill) {
        wait_vmcnt_at_most<(DIST - 1) * 2 * CH>();
        memory_order_point();
        __builtin_amdgcn_s_barrier();
        memory_order_point();
        // The row numbers of the tile after are requested in front of the loads of tile t+DIST,
        // and kept there: they are then older than those loads, and the next step's wait covers
        // them without waiting for the loads.
        int rows_after[CH];
        load_rows(t + DIST + 1, rows_after);
        memory_order_point();
        issue_tile<CH>(kfill, vfill, K, V, rows_next, koff, voff, row_bytes, wave);
        memory_order_point();
#pragma unroll
        for (int i = 0; i < CH; ++i) rows_next[i] = rows_after[i];
        compute_tile(t, kcur, vcur);
    };
    if constexpr (NBUF == 3) {
        for (int t = 0; t < ntiles; t += 3) {
            step(t, lds_k0, lds_v0, lds_k2, lds_v2);
            if (t + 1 >= ntiles) break;
            step(t + 1, lds_k1, lds_v1, lds_k0, lds_v0);
            if (t + 2 >= ntiles) break;
            step(t + 2, lds_k2, lds_v2, lds_k1, lds_v1);
        }
    } else {
        for (int t = 0; t < ntiles; t += 2) {
            step(t, lds_k0, lds_v0, lds_k1, lds_v1);
            if (t + 1 >= ntiles) break;
            step(t + 1, lds_k1, lds_v1, lds_k0, lds_v0);
        }
    }
    wait_vmcnt_at_most<0>();        // nothing of this workgroup is on its way to LDS when it ends

    // ---- epilogue: O = diag(l)^-1 acc.  The lane number is formed anew here (two instructions),
    // so that no register has to carry the output address across the loop.
    const int lane_out = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int lq_out = lane_out & 31, lh_out = lane_out >> 5;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = half_sum(l_run[qb]);
        const int row = q0 + qb * 32 + lq_out;
        if (row >= n) continue;
        const float inv = 1.0f / l_tot;
        __bf16* dst = (__bf16*)p.o + head_off + (int64_t)row * p.td.sn;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o_acc[qb][db][r4 * 4 + e] * inv);
                *(bf16x4*)(dst + db * 32 + 8 * r4 + 4 * lh_out) = w;
            }
    }
}

template <int D, int QB, int NW, int NBUF>
hipError_t launch(const AttnParams& p, hipStream_t s) {
    constexpr int BM = 32 * QB * NW;
    const int nqb = (p.n + BM - 1) / BM;
    const int bh_pad = (p.batch * p.heads + 7) / 8 * 8;
    hipLaunchKernelGGL((attn_bf16_group_kernel<D, QB, NW, NBUF>), dim3(nqb * bh_pad), dim3(64 * NW), 0, s, p);
    return hipGetLastError();
}

template <int D>
hipError_t launch_by_block(const AttnParams& p, int block_m, hipStream_t s) {
    // One block of 32 queries per wave keeps the register count low enough for several waves per
    // SIMD (two blocks per wave halve the LDS reads per MFMA, and measured slower at every size).
    // Slots, measured at 64K / keep 10%: 128 rows 3 (6.9 ms, against 7.6 with 2), 64 rows 2 (10.8
    // against 12.2), 32 rows 3 (14.7 against 24.4: a one-wave workgroup has nobody to wait with).
    // (Three slots of K with two of V -- 40 KB, a fourth workgroup per CU on paper -- measured
    // 11.3 and 16.9 ms for 64 and 32 rows: worse than either.)
    if (block_m == 128) return launch<D, 1, 4, 3>(p, s);
    if (block_m == 64) return launch<D, 1, 2, 2>(p, s);
    if (block_m == 32) return launch<D, 1, 1, 3>(p, s);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_attn_bf16_group(const AttnParams& p, int head_dim, int block_m, hipStream_t s) {
    if (p.idx == nullptr || p.v == nullptr || p.o == nullptr) return hipErrorInvalidValue;
    if (p.groups > 1 && p.group_size % block_m != 0) return hipErrorInvalidValue;
    if (head_dim == 128) return launch_by_block<128>(p, block_m, s);
    if (head_dim == 64) return launch_by_block<64>(p, block_m, s);
    return hipErrorInvalidValue;
}

}  // namespace pulsecol
