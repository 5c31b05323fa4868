// Column-sparse attention for query groups smaller than the 256-row query block of the main
// bf16 kernel (Sec. 3.3: group-wise sets with G = 32, 64 or 128 queries; Sec. 3.4 and the
// appendix listing "Column-Sparse Attention Forward" for the computation itself).
//
// With one column set per small group nothing is shared between neighbouring query blocks
// any more: every group gathers its own K/V rows, the arithmetic intensity is G flop per
// gathered byte, and the kernel lives on the memory side of the roofline.  So this is the
// plain formulation, not the hand-scheduled one: a workgroup = one query block of
// 32 * QB * NW rows (NW waves, QB blocks of 32 queries per wave), tiles of 32 gathered rows
// staged through double-buffered LDS (32 KB per workgroup, several workgroups per CU hide
// the gather latency), classic online softmax with a running row maximum.
// Same MFMA orientation as the main kernel: S^T = K_tile Q^T, O^T = V^T P^T, P in registers.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int BN = 32;      // gathered rows per tile

template <int D, int QB, int NW>
__global__ void __launch_bounds__(64 * NW) attn_bf16_group_kernel(AttnParams p) {
    constexpr int NTHREADS = 64 * NW;
    constexpr int BM = 32 * QB * NW;
    constexpr int PIECES = D / 8;                 // 16-byte pieces per row
    constexpr int KK = D / 16;                    // contraction steps of Q K^T
    constexpr int DB = D / 32;                    // 32-wide blocks of the head dimension
    constexpr int CH = BN * PIECES / NTHREADS;    // 16-byte pieces each thread stages per tile
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = BN * ROW_BYTES;
    static_assert(CH >= 1 && CH * NTHREADS == BN * PIECES, "staging covers the tile exactly");

    __shared__ __attribute__((aligned(16))) unsigned char lds_k[2][TILE_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char lds_v[2][TILE_BYTES];

    const int nqb = (p.n + BM - 1) / BM;
    int bh, qblk;
    if (!xcd_tile(blockIdx.x, nqb, p.batch * p.heads, &bh, &qblk)) return;
    const int b = bh / p.heads, h = bh - b * p.heads;
    const int64_t head_off = (int64_t)b * p.td.sb + (int64_t)h * p.td.sh;
    // grouped-query layout: query head h reads K/V head h / (heads / kv_heads)
    const int64_t kv_off = (int64_t)b * p.td_kv.sb + (int64_t)(h / (p.heads / p.kv_heads)) * p.td_kv.sh;
    const __bf16* __restrict__ Q = (const __bf16*)p.q + head_off;
    const __bf16* __restrict__ K = (const __bf16*)p.k + kv_off;
    const __bf16* __restrict__ V = (const __bf16*)p.v + kv_off;
    // the column set of this query block's group; group_size is a multiple of BM
    const int group = p.groups > 1 ? (qblk * BM) / p.group_size : 0;
    const int32_t* __restrict__ idx = p.idx + ((int64_t)bh * p.groups + group) * p.ns;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lq = lane & 31;       // query column (and K/V row) this lane owns inside a 32-block
    const int lh = lane >> 5;       // which half of the wave
    const int ns = p.ns;
    const int ntiles = (ns + BN - 1) / BN;
    const int n = p.n;

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

    // ---- staging: thread owns pieces c = tid + NTHREADS*j -> (row c / PIECES, piece c % PIECES)
    u32x4 stage_k[CH], stage_v[CH];
    int next_row[CH];               // K/V row numbers of the tile about to be fetched

    auto load_rows = [&](int t) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            int pos = t * BN + (tid + NTHREADS * j) / PIECES;
            pos = pos < ns ? pos : ns - 1;          // ragged tail: any valid row; masked below
            next_row[j] = idx[pos];
        }
    };
    auto fetch = [&]() {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int piece = (tid + NTHREADS * j) % PIECES;
            const int64_t off = (int64_t)next_row[j] * p.td_kv.sn + piece * 8;
            stage_k[j] = *(const u32x4*)(K + off);
            stage_v[j] = *(const u32x4*)(V + off);
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + NTHREADS * j;
            const int row = c / PIECES, piece = c % PIECES;
            *(u32x4*)(lds_k[buf] + row * ROW_BYTES + ((piece ^ swizzle_k<PIECES>(row)) << 4)) = stage_k[j];
            *(u32x4*)(lds_v[buf] + row * ROW_BYTES + ((piece ^ swizzle_v<PIECES>(row)) << 4)) = stage_v[j];
        }
    };

    load_rows(0);
    fetch();
    if (ntiles > 1) load_rows(1);
    commit(0);
    __syncthreads();

    const float c2 = p.scale * kLog2e;      // exp(z*scale) = exp2(z*c2)
    float m_run[QB], l_run[QB];             // l: per-lane partial, sums only this lane's keys
    f32x16 o_acc[QB][DB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[qb][db][r] = 0.f;
    }

    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) {
            fetch();                                  // tile t+1 -> registers (rows loaded one iteration ago)
            if (t + 2 < ntiles) load_rows(t + 2);
        }

        // ---- S^T = K_tile Q^T  (32 keys x 32 queries per query block)
        f32x16 s[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[qb][r] = 0.f;
        {
            const unsigned char* rowp = lds_k[buf] + lq * ROW_BYTES;
            const int sw = swizzle_k<PIECES>(lq);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 a = *(const bf16x8*)(rowp + (((2 * kk + lh) ^ sw) << 4));
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) s[qb] = mfma_bf16(a, qf[qb][kk], s[qb]);
            }
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

        // ---- online softmax (per lane: one query column per query block)
        bf16x8 pfrag[QB][2];     // [qb][half of the 32-row tile]
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mx = s[qb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[qb][r]);
            mx = half_max(mx);                               // finite: row 0 of a tile is always valid
            const float m_new = fmaxf(m_run[qb], mx);
            const float alpha = fast_exp2((m_run[qb] - m_new) * c2);
            const float mc = m_new * c2;
            m_run[qb] = m_new;
            float rs = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float e = fast_exp2(__builtin_fmaf(s[qb][r], c2, -mc));
                rs += e;
                pfrag[qb][r >> 3][r & 7] = (__bf16)e;
            }
            l_run[qb] = l_run[qb] * alpha + rs;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[qb][db][r] *= alpha;
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            // contraction element e of this lane <-> tile row hf*16 + 8*(e/4) + 4*lh + e%4
            const int j16 = lane & 15;
            const int row0 = hf * 16 + 4 * lh + (j16 >> 2);
            const int row1 = row0 + 8;
            const int colpiece = ((lane >> 4) & 1) * 2 + ((j16 & 3) >> 1);   // 16-byte piece inside the 64-byte d-block
            const int inpiece = (j16 & 1) * 8;                               // byte inside the piece
            const unsigned char* r0p = lds_v[buf] + row0 * ROW_BYTES + inpiece;
            const unsigned char* r1p = lds_v[buf] + row1 * ROW_BYTES + inpiece;
            const int sw0 = swizzle_v<PIECES>(row0), sw1 = swizzle_v<PIECES>(row1);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const int piece = db * 4 + colpiece;
                const bf16x4 lo = lds_read_tr(r0p + ((piece ^ sw0) << 4));
                const bf16x4 hi = lds_read_tr(r1p + ((piece ^ sw1) << 4));
                const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) o_acc[qb][db] = mfma_bf16(a, pfrag[qb][hf], o_acc[qb][db]);
            }
        }

        if (t + 1 < ntiles) commit(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: O = diag(l)^-1 acc
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = half_sum(l_run[qb]);
        const int row = q0 + qb * 32 + lq;
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
                *(bf16x4*)(dst + db * 32 + 8 * r4 + 4 * lh) = w;
            }
    }
}

template <int D, int QB, int NW>
hipError_t launch(const AttnParams& p, hipStream_t s) {
    constexpr int BM = 32 * QB * NW;
    const int nqb = (p.n + BM - 1) / BM;
    const int bh_pad = (p.batch * p.heads + 7) / 8 * 8;
    hipLaunchKernelGGL((attn_bf16_group_kernel<D, QB, NW>), dim3(nqb * bh_pad), dim3(64 * NW), 0, s, p);
    return hipGetLastError();
}

template <int D>
hipError_t launch_by_block(const AttnParams& p, int block_m, hipStream_t s) {
    // one block of 32 queries per wave keeps the register count low enough for several waves per SIMD
    if (block_m == 128) return launch<D, 1, 4>(p, s);
    if (block_m == 64) return launch<D, 1, 2>(p, s);
    if (block_m == 32) return launch<D, 1, 1>(p, s);
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
