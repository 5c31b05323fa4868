// bf16 attention kernels for gfx950: column-sparse attention (Sec. 3.4 and the appendix
// listing "Column-Sparse Attention Forward"), the dense baseline (Sec. 3.1) and the row
// log-sum-exp pass of the identification step (Sec. 3.3: the softmax matrix P needs the
// row normalisers before column masses can be summed).
//
// One workgroup = 256 query rows (4 waves x 64 rows), one tile = 64 K/V rows, processed as
// two half-tiles of 32.  Q stays in registers as the MFMA B operand for the whole kernel.
// K and V rows are gathered straight into LDS (global_load_lds_dwordx4: 16 lanes cover one
// 256-byte row, the XOR swizzle is applied on the global side) into three tile slots per
// operand, and read back as MFMA A operands (V through the transposing LDS read).  Every
// lane owns one query column of S^T / O^T, so the online-softmax state is two scalars per
// lane and query block.  P is rounded to bf16 only as the MFMA operand; l is summed from the
// fp32 P.  The output accumulator lives in the AGPR half of the register file.
//
// Software pipeline (one wave per SIMD, so overlap has to come from the instruction
// stream): half-step j issues the MFMAs of  S(j+1) = K(j+1) Q^T  and  O += V(j-1) P(j-1)
// while the VALU turns S(j) into P(j).  The three are independent, so the matrix pipe and
// the vector ALU run side by side.  The reference maximum is raised lazily: a half-tile whose
// maximum stays within 2^kTau of the reference keeps it (exact: numerator and denominator
// carry the same factor), so the 128 accumulator registers are rescaled only on rare steps,
// and then by an exact power of two.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int BM = kBlockM_bf16;
constexpr int BN = kBlockN_bf16;
constexpr int NTHREADS = 256;
constexpr int NBUF = 3;            // LDS tile slots per operand
constexpr float kTau = 8.0f;       // log2 of the growth allowed before the reference max is raised

typedef unsigned char byte;

template <int D, int MODE>
struct AttnWave {
    static constexpr int PIECES = D / 8;                 // 16-byte pieces per row
    static constexpr int KK = D / 16;                    // contraction steps of Q K^T
    static constexpr int DB = D / 32;                    // 32-wide blocks of the head dimension
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int TILE_BYTES = BN * ROW_BYTES;
    static constexpr int ROWS_PER_CHUNK = 64 / PIECES;   // one direct-to-LDS load instruction moves 64 x 16 bytes
    static constexpr int CH = BN / ROWS_PER_CHUNK / 4;   // such instructions per wave and tile (per operand)
    static constexpr bool HAS_V = (MODE != kLseOnly);
    static constexpr bool GATHER = (MODE == kSparse);
    static constexpr int ODB = HAS_V ? DB : 1;
    // direct-to-LDS loads per steady-state issue point (the row-number loads are issued before
    // them, so "all but the newest VM_PER_ISSUE" covers every load of earlier iterations)
    static constexpr int VM_PER_ISSUE = CH + (HAS_V ? CH : 0);

    // lane geometry
    int lane, wave, lq, lh;
    // problem
    int n, ns, ntiles, nhalf;
    bool ragged;
    int64_t sn;
    const __bf16* K;
    const __bf16* V;
    const int32_t* idx;
    // registers that live across the whole kernel
    bf16x8 qf[2][KK];
    f32x16 o_acc[2][ODB];
    float c2;
    float mc[2];          // reference maximum in log2 units (raw maximum * c2), equal in both half-waves
    float l_run[2];       // per-lane partial row sum (this lane's keys only)
    float mx_next[2];     // raw maximum of the half-tile whose S is in flight
    int koff[CH], voff[CH];
    int lrow;

    // ------------------------------------------------------------------ gathers
    __device__ __forceinline__ void load_rows(int t, int (&dst)[CH]) const {
        t = t < ntiles ? t : ntiles - 1;          // past the end: repeat the last tile (never read back)
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int pos = t * BN + (wave * CH + i) * ROWS_PER_CHUNK + lrow;
            pos = pos < ns ? pos : ns - 1;        // ragged tail: any valid row; masked later
            dst[i] = GATHER ? idx[pos] : pos;
        }
    }
    // Load instruction i of a wave fills the 1 KB chunk cid = wave*CH + i of a tile slot: lane L
    // lands at chunk byte 16*L, i.e. tile row cid*ROWS_PER_CHUNK + L/PIECES, LDS piece L%PIECES,
    // and therefore fetches the global piece (L%PIECES) ^ swizzle(row) of that row.
    // (Every pointer is a restrict parameter so that the loads carry alias scopes: the compiler
    // then knows that LDS reads of other slots need not wait for these loads.)
    __device__ __forceinline__ void issue_tile(byte* __restrict__ kslot, byte* __restrict__ vslot,
                                               const __bf16* __restrict__ Kg, const __bf16* __restrict__ Vg,
                                               const int (&krows)[CH], const int (&vrows)[CH]) const {
#pragma unroll
        for (int i = 0; i < CH; ++i)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(Kg + (int64_t)krows[i] * sn + koff[i]),
                (PULSECOL_LDS void*)(kslot + (wave * CH + i) * 1024), 16, 0, 0);
        if (HAS_V) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(Vg + (int64_t)vrows[i] * sn + voff[i]),
                    (PULSECOL_LDS void*)(vslot + (wave * CH + i) * 1024), 16, 0, 0);
        }
    }

    // ------------------------------------------------------------------ matrix steps
    // S[qb] = K(half) Q^T for both query blocks; each K fragment read feeds two MFMAs.
    __device__ __forceinline__ void qk(const byte* __restrict__ kslot, int half, f32x16 (&S)[2]) const {
        const int row = half * 32 + lq;
        const byte* rowp = kslot + row * ROW_BYTES;
        const int sw = swizzle_k<PIECES>(row);
#pragma unroll
        for (int r = 0; r < 16; ++r) { S[0][r] = 0.f; S[1][r] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const bf16x8 a = *(const bf16x8*)(rowp + (((2 * kk + lh) ^ sw) << 4));
            S[0] = mfma_bf16(a, qf[0][kk], S[0]);
            S[1] = mfma_bf16(a, qf[1][kk], S[1]);
        }
    }
    // O^T += V(half)^T P^T.  Contraction element e of a lane <-> tile row half*32 + hf*16 + 8*(e/4) + 4*lh + e%4.
    __device__ __forceinline__ void pv(const byte* __restrict__ vslot, int half, const bf16x8 (&P)[2][2]) {
        if (HAS_V) {
            const int j16 = lane & 15;
            const int colpiece = ((lane >> 4) & 1) * 2 + ((j16 & 3) >> 1);   // 16-byte piece inside a 64-byte d-block
            const int inpiece = (j16 & 1) * 8;                               // byte inside the piece
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int row0 = half * 32 + hf * 16 + 4 * lh + (j16 >> 2);
                const int row1 = row0 + 8;
                const byte* r0p = vslot + row0 * ROW_BYTES + inpiece;
                const byte* r1p = vslot + row1 * ROW_BYTES + inpiece;
                const int sw0 = swizzle_v<PIECES>(row0), sw1 = swizzle_v<PIECES>(row1);
#pragma unroll
                for (int db = 0; db < ODB; ++db) {
                    const int piece = db * 4 + colpiece;
                    const bf16x4 lo = lds_read_tr(r0p + ((piece ^ sw0) << 4));
                    const bf16x4 hi = lds_read_tr(r1p + ((piece ^ sw1) << 4));
                    const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    mfma_bf16_agpr(o_acc[0][db], a, P[0][hf]);
                    mfma_bf16_agpr(o_acc[1][db], a, P[1][hf]);
                }
            }
        }
    }

    // ------------------------------------------------------------------ softmax pieces
    // columns of the last tile that lie past ns get weight zero
    __device__ __forceinline__ void mask_tail(int j, f32x16 (&S)[2]) const {
        if (ragged && j >= nhalf - 2) {
            const int valid = ns - (j >> 1) * BN - (j & 1) * 32;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (acc_row(r, lh) >= valid) { S[0][r] = -INFINITY; S[1][r] = -INFINITY; }
        }
    }
    __device__ __forceinline__ void half_tile_max(const f32x16 (&S)[2]) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float a0 = fmaxf(fmaxf(S[qb][0], S[qb][1]), S[qb][2]);
            float a1 = fmaxf(fmaxf(S[qb][3], S[qb][4]), S[qb][5]);
            float a2 = fmaxf(fmaxf(S[qb][6], S[qb][7]), S[qb][8]);
            float a3 = fmaxf(fmaxf(S[qb][9], S[qb][10]), S[qb][11]);
            a0 = fmaxf(fmaxf(a0, S[qb][12]), S[qb][13]);
            a1 = fmaxf(fmaxf(a1, S[qb][14]), S[qb][15]);
            mx_next[qb] = half_max(fmaxf(fmaxf(a0, a1), fmaxf(a2, a3)));
        }
    }
    // P = exp2(S*c2 - mc) against the current reference; sums into l_run
    __device__ __forceinline__ void exp_half_tile(const f32x16 (&S)[2], bf16x8 (&P)[2][2]) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float ref = mc[qb];
            float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float e0 = fast_exp2(__builtin_fmaf(S[qb][r], c2, -ref));
                const float e1 = fast_exp2(__builtin_fmaf(S[qb][r + 1], c2, -ref));
                rs0 += e0;
                rs1 += e1;
                P[qb][r >> 3][r & 7] = (__bf16)e0;
                P[qb][r >> 3][(r & 7) + 1] = (__bf16)e1;
            }
            l_run[qb] += rs0 + rs1;
        }
    }
    // Raise the reference maximum where the incoming half-tile exceeds it by more than 2^kTau.
    // The reference moves by a whole number of log2 units, so the factor applied to l, to the
    // accumulator and to the pending P(j-1) is an exact power of two.
    __device__ __forceinline__ void raise_reference(bf16x8 (&P_pending)[2][2]) {
        const bool need = (mx_next[0] * c2 > mc[0] + kTau) || (mx_next[1] * c2 > mc[1] + kTau);
        if (__builtin_expect(__ballot(need) == 0ull, 1)) return;
        if (HAS_V) mfma_agpr_settle();
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float m2 = mx_next[qb] * c2;
            if (m2 > mc[qb] + kTau) {
                const bool first = mc[qb] == -INFINITY;
                const float steps = first ? 0.f : ceilf(m2 - mc[qb]);
                const float alpha = first ? 0.f : fast_exp2(-steps);
                mc[qb] = first ? m2 : mc[qb] + steps;
                l_run[qb] *= alpha;
                if (HAS_V) {
#pragma unroll
                    for (int db = 0; db < ODB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o_acc[qb][db][r] *= alpha;
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            P_pending[qb][hf][e] = (__bf16)((float)P_pending[qb][hf][e] * alpha);
                }
            }
        }
    }

    // ------------------------------------------------------------------ half-steps
    // Fast half-step j (1 <= j <= nhalf-4): S_in = S(j), P_in = P(j-1) -> S_out = S(j+1), P_out = P(j).
    // qk, exp and pv are independent instruction streams inside one basic block.
    __device__ __forceinline__ void fast_step(const byte* __restrict__ kslot, int khalf,
                                              const byte* __restrict__ vslot, int vhalf,
                                              f32x16 (&S_in)[2], f32x16 (&S_out)[2],
                                              bf16x8 (&P_in)[2][2], bf16x8 (&P_out)[2][2]) {
        raise_reference(P_in);
        qk(kslot, khalf, S_out);
        exp_half_tile(S_in, P_out);
        pv(vslot, vhalf, P_in);
        half_tile_max(S_out);
    }
    // General half-step (first step, last tile): same work, plus tail masking; no overlap needed.
    __device__ __forceinline__ void general_step(int j, const byte* kbase, const byte* vbase,
                                                 f32x16 (&S_in)[2], f32x16 (&S_out)[2],
                                                 bf16x8 (&P_in)[2][2], bf16x8 (&P_out)[2][2]) {
        raise_reference(P_in);
        if (j >= 1) pv(vbase + (((j - 1) >> 1) % NBUF) * TILE_BYTES, (j - 1) & 1, P_in);
        exp_half_tile(S_in, P_out);
        if (j + 1 < nhalf) {
            qk(kbase + (((j + 1) >> 1) % NBUF) * TILE_BYTES, (j + 1) & 1, S_out);
            mask_tail(j + 1, S_out);
            half_tile_max(S_out);
        }
    }
    // One steady-state iteration u: issue K(u+3), V(u+2); half-steps j = 2u+1 and 2u+2, which
    // read K tile u+1 and V tile u.  All four LDS regions are distinct tile slots.
    __device__ __forceinline__ void steady_pair(const byte* __restrict__ kread, const byte* __restrict__ vread,
                                                byte* __restrict__ kwrite, byte* __restrict__ vwrite,
                                                const __bf16* __restrict__ Kg, const __bf16* __restrict__ Vg,
                                                const int (&krows)[CH], const int (&vrows)[CH],
                                                f32x16 (&SA)[2], f32x16 (&SB)[2],
                                                bf16x8 (&PA)[2][2], bf16x8 (&PB)[2][2]) {
        issue_tile(kwrite, vwrite, Kg, Vg, krows, vrows);
        fast_step(kread, 0, vread, 0, SB, SA, PA, PB);   // odd:  S(j) in SB, P(j-1) in PA -> S(j+1) in SA, P(j) in PB
        fast_step(kread, 1, vread, 1, SA, SB, PB, PA);   // even: S(j) in SA, P(j-1) in PB -> S(j+1) in SB, P(j) in PA
    }
};

// s_waitcnt vmcnt(v) with the other counters left alone (gfx9 encoding: vmcnt in [3:0] and [15:14])
template <int v>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (v & 0xF) | ((v & 0x30) << 10));
}

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
    __shared__ __attribute__((aligned(1024))) byte lds_all[(HAS_V ? 2 : 1) * NBUF * TILE_BYTES];
    byte* const lds_k = lds_all;
    byte* const lds_v = lds_all + (HAS_V ? NBUF * TILE_BYTES : 0);

    const int nqb = (p.n + BM - 1) / BM;
    int bh, qblk;
    if (!xcd_tile(blockIdx.x, nqb, p.batch * p.heads, &bh, &qblk)) return;
    const int b = bh / p.heads, h = bh - b * p.heads;
    const int64_t head_off = (int64_t)b * p.td.sb + (int64_t)h * p.td.sh;
    const __bf16* __restrict__ Q = (const __bf16*)p.q + head_off;

    W w;
    const int tid = threadIdx.x;
    w.lane = tid & 63;
    w.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    w.lq = w.lane & 31;
    w.lh = w.lane >> 5;
    w.n = p.n;
    w.ns = p.ns;
    w.ntiles = (p.ns + BN - 1) / BN;
    w.nhalf = 2 * w.ntiles;
    w.ragged = (p.ns & (BN - 1)) != 0;
    w.sn = p.td.sn;
    w.K = (const __bf16*)p.k + head_off;
    w.V = HAS_V ? (const __bf16*)p.v + head_off : nullptr;
    w.idx = W::GATHER ? p.idx + (int64_t)bh * p.ns : nullptr;
    w.c2 = p.scale * kLog2e;                 // exp(z*scale) = exp2(z*c2)
    w.mc[0] = w.mc[1] = -INFINITY;
    w.l_run[0] = w.l_run[1] = 0.f;
    w.lrow = w.lane / W::PIECES;
    {
        const int lslot = w.lane % W::PIECES;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int row = (w.wave * CH + i) * W::ROWS_PER_CHUNK + w.lrow;
            w.koff[i] = (lslot ^ swizzle_k<W::PIECES>(row)) * 8;
            w.voff[i] = (lslot ^ swizzle_v<W::PIECES>(row)) * 8;
        }
    }
    const int n = p.n, nhalf = w.nhalf;

    // ---- Q fragments: B operand, [query lq][d = kk*16 + 8*lh .. +7]
    const int q0 = qblk * BM + w.wave * 64;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        int row = q0 + qb * 32 + w.lq;
        row = row < n ? row : n - 1;
        const __bf16* src = Q + (int64_t)row * p.td.sn + 8 * w.lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) w.qf[qb][kk] = *(const bf16x8*)(src + kk * 16);
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < ODB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) w.o_acc[qb][db][r] = 0.f;

    // ---- prologue: tiles 0..2 of K and V into their slots; then rows_k = tile 3, rows_v = tile 2
    int rows_k[CH], rows_v[CH], rows_n[CH];
#pragma unroll 1
    for (int t = 0; t < NBUF; ++t) {
        w.load_rows(t, rows_k);
        w.issue_tile(lds_k + t * TILE_BYTES, lds_v + (HAS_V ? t * TILE_BYTES : 0), w.K, w.V, rows_k, rows_k);
    }
    w.load_rows(2, rows_v);
    w.load_rows(3, rows_k);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();

    f32x16 SA[2], SB[2];
    bf16x8 PA[2][2], PB[2][2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int e = 0; e < 8; ++e) { PA[qb][hf][e] = (__bf16)0.f; PB[qb][hf][e] = (__bf16)0.f; }
    w.qk(lds_k, 0, SA);
    w.mask_tail(0, SA);
    w.half_tile_max(SA);

    // j = 0: S(0) in SA -> P(0) in PA, S(1) in SB
    w.general_step(0, lds_k, lds_v, SA, SB, PB, PA);

    // ---- steady state: iteration u runs half-steps 2u+1 and 2u+2 (both <= nhalf-4)
    const int npairs = nhalf >= 4 ? (nhalf - 4) / 2 : 0;
    int kr = 1, vr = 0;            // slot of K tile u+1 / of V tile u
    for (int u = 0; u < npairs; ++u) {
        const int kw = vr;                             // K(u+3) -> slot (u+3)%3 == u%3
        const int vw = vr >= 1 ? vr - 1 : vr + 2;      // V(u+2) -> slot (u+2)%3
        w.load_rows(u + 4, rows_n);
        w.steady_pair(lds_k + kr * TILE_BYTES, lds_v + (HAS_V ? vr * TILE_BYTES : 0),
                      lds_k + kw * TILE_BYTES, lds_v + (HAS_V ? vw * TILE_BYTES : 0),
                      w.K, w.V, rows_k, rows_v, SA, SB, PA, PB);
#pragma unroll
        for (int i = 0; i < CH; ++i) { rows_v[i] = rows_k[i]; rows_k[i] = rows_n[i]; }
        kr = kr == 2 ? 0 : kr + 1;
        vr = vr == 2 ? 0 : vr + 1;
        // everything but this iteration's own loads has landed; then all waves swap slots
        wait_vmcnt<W::VM_PER_ISSUE>();
        __builtin_amdgcn_s_barrier();
    }
    // ---- tail: the remaining half-steps (at most three), then the last P V product
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    int j = 2 * npairs + 1;
    if (j < nhalf) {                              // odd
        w.general_step(j, lds_k, lds_v, SB, SA, PA, PB);
        ++j;
        if (j < nhalf) {                          // even, then the last odd one (nhalf is even)
            w.general_step(j, lds_k, lds_v, SA, SB, PB, PA);
            ++j;
            w.general_step(j, lds_k, lds_v, SB, SA, PA, PB);
        }
    }
    w.pv(lds_v + (HAS_V ? (((nhalf - 1) >> 1) % NBUF) * TILE_BYTES : 0), (nhalf - 1) & 1, PB);

    // ---- epilogue: O = diag(l)^-1 acc, optional row log-sum-exp
    if (HAS_V) mfma_agpr_settle();
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float l_tot = half_sum(w.l_run[qb]);
        const int row = q0 + qb * 32 + w.lq;
        if (row >= n) continue;
        if (HAS_V) {
            const float inv = 1.0f / l_tot;
            __bf16* dst = (__bf16*)p.o + head_off + (int64_t)row * p.td.sn;
#pragma unroll
            for (int db = 0; db < ODB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    bf16x4 o4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(w.o_acc[qb][db][r4 * 4 + e] * inv);
                    *(bf16x4*)(dst + db * 32 + 8 * r4 + 4 * w.lh) = o4;
                }
        }
        if (p.lse != nullptr && w.lh == 0)
            p.lse[(int64_t)bh * n + row] = (w.mc[qb] + fast_log2(l_tot)) * (p.lse_base2 ? 1.0f : kLn2);
    }
}

template <int D, int MODE>
hipError_t launch(const AttnParams& p, hipStream_t s) {
    const int nqb = (p.n + BM - 1) / BM;
    const int bh_pad = (p.batch * p.heads + 7) / 8 * 8;
    hipLaunchKernelGGL((attn_bf16_kernel<D, MODE>), dim3(nqb * bh_pad), dim3(NTHREADS), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bf16(const AttnParams& p, int head_dim, AttnMode mode, hipStream_t s) {
    if (head_dim == 128) {
        if (mode == kSparse) return launch<128, kSparse>(p, s);
        if (mode == kDense) return launch<128, kDense>(p, s);
        return launch<128, kLseOnly>(p, s);
    }
    if (head_dim == 64) {
        if (mode == kSparse) return launch<64, kSparse>(p, s);
        if (mode == kDense) return launch<64, kDense>(p, s);
        return launch<64, kLseOnly>(p, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace pulsecol
