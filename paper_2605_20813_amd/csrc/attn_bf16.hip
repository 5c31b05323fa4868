// bf16 attention kernels for gfx950: column-sparse attention (Sec. 3.4 and the appendix
// listing "Column-Sparse Attention Forward"), the dense baseline (Sec. 3.1) and the row
// log-sum-exp pass of the identification step (Sec. 3.3: the softmax matrix P needs the
// row normalisers before column masses can be summed).
//
// One workgroup = 256 query rows (4 waves x 64 rows), one tile = 64 K/V rows.  Q stays in
// registers as the MFMA B operand for the whole kernel; K and V tiles are gathered with
// 128-bit loads (16 lanes per 256-byte row), staged through double-buffered LDS and read
// back as MFMA A operands (V through the transposing LDS read).  Every lane owns one query
// column of S^T / O^T, so the online-softmax state (m, l) is two scalars per lane and query
// block.  P is rounded to bf16 only as the MFMA operand; l is summed from the fp32 P.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int BM = kBlockM_bf16;
constexpr int BN = kBlockN_bf16;
constexpr int NTHREADS = 256;

template <int D, int MODE>
__global__ void __launch_bounds__(NTHREADS) attn_bf16_kernel(AttnParams p) {
    constexpr int PIECES = D / 8;                 // 16-byte pieces per row
    constexpr int KK = D / 16;                    // contraction steps of Q K^T
    constexpr int DB = D / 32;                    // 32-wide blocks of the head dimension
    constexpr int CH = BN * PIECES / NTHREADS;    // 16-byte pieces each thread stages per tile
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = BN * ROW_BYTES;
    constexpr bool HAS_V = (MODE != kLseOnly);
    constexpr bool GATHER = (MODE == kSparse);

    __shared__ __attribute__((aligned(16))) unsigned char lds_k[2][TILE_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char lds_v[HAS_V ? 2 : 1][HAS_V ? TILE_BYTES : 16];

    const int nqb = (p.n + BM - 1) / BM;
    int bh, qblk;
    if (!xcd_tile(blockIdx.x, nqb, p.batch * p.heads, &bh, &qblk)) return;
    const int b = bh / p.heads, h = bh - b * p.heads;
    const int64_t head_off = (int64_t)b * p.td.sb + (int64_t)h * p.td.sh;
    const __bf16* __restrict__ Q = (const __bf16*)p.q + head_off;
    const __bf16* __restrict__ K = (const __bf16*)p.k + head_off;
    const __bf16* __restrict__ V = HAS_V ? (const __bf16*)p.v + head_off : nullptr;
    const int32_t* __restrict__ idx = GATHER ? p.idx + (int64_t)bh * p.ns : nullptr;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lq = lane & 31;       // query column (and K/V row) this lane owns inside a 32-block
    const int lh = lane >> 5;       // which half of the wave
    const int ns = p.ns;
    const int ntiles = (ns + BN - 1) / BN;
    const int n = p.n;

    // ---- Q fragments: B operand, [query lq][d = kk*16 + 8*lh .. +7]
    const int q0 = qblk * BM + wave * 64;
    bf16x8 qf[2][KK];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        int row = q0 + qb * 32 + lq;
        row = row < n ? row : n - 1;
        const __bf16* src = Q + (int64_t)row * p.td.sn + 8 * lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[qb][kk] = *(const bf16x8*)(src + kk * 16);
    }

    // ---- staging: thread owns pieces c = tid + 256*j -> (row c / PIECES, piece c % PIECES)
    u32x4 stage_k[CH], stage_v[HAS_V ? CH : 1];
    int next_row[CH];               // K/V row numbers of the tile about to be fetched

    auto load_rows = [&](int t) {   // row numbers of tile t for this thread's pieces
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            int pos = t * BN + (tid + NTHREADS * j) / PIECES;
            pos = pos < ns ? pos : ns - 1;          // ragged tail: any valid row; masked below
            next_row[j] = GATHER ? idx[pos] : pos;
        }
    };
    auto fetch = [&]() {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int piece = (tid + NTHREADS * j) % PIECES;
            const int64_t off = (int64_t)next_row[j] * p.td.sn + piece * 8;
            stage_k[j] = *(const u32x4*)(K + off);
            if (HAS_V) stage_v[j] = *(const u32x4*)(V + off);
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + NTHREADS * j;
            const int row = c / PIECES, piece = c % PIECES;
            *(u32x4*)(lds_k[buf] + row * ROW_BYTES + ((piece ^ swizzle_k<PIECES>(row)) << 4)) = stage_k[j];
            if (HAS_V)
                *(u32x4*)(lds_v[buf] + row * ROW_BYTES + ((piece ^ swizzle_v<PIECES>(row)) << 4)) = stage_v[j];
        }
    };

    load_rows(0);
    fetch();
    if (ntiles > 1) load_rows(1);
    commit(0);
    __syncthreads();

    const float c2 = p.scale * kLog2e;      // exp(z*scale) = exp2(z*c2)
    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};            // per-lane partial: sums only this lane's keys
    f32x16 o_acc[2][HAS_V ? DB : 1];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < (HAS_V ? DB : 1); ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[qb][db][r] = 0.f;

    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) {
            fetch();                                  // tile t+1 -> registers (rows loaded one iteration ago)
            if (t + 2 < ntiles) load_rows(t + 2);
        }

        // ---- S^T = K_tile Q^T
        f32x16 s[2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[qb][kb][r] = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const int row = kb * 32 + lq;
            const unsigned char* rowp = lds_k[buf] + row * ROW_BYTES;
            const int sw = swizzle_k<PIECES>(row);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 a = *(const bf16x8*)(rowp + (((2 * kk + lh) ^ sw) << 4));
                s[0][kb] = mfma_bf16(a, qf[0][kk], s[0][kb]);
                s[1][kb] = mfma_bf16(a, qf[1][kk], s[1][kb]);
            }
        }

        // ---- ragged tail of the last tile: columns past ns get weight zero
        if (t == ntiles - 1 && (ns & (BN - 1))) {
            const int valid = ns - t * BN;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kb * 32 + acc_row(r, lh) >= valid) {
                        s[0][kb][r] = -INFINITY;
                        s[1][kb][r] = -INFINITY;
                    }
        }

        // ---- online softmax (per lane: one query column per query block)
        bf16x8 pfrag[2][2][2];   // [qb][kb][half of the 32-row block]
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float mx = s[qb][0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[qb][kb][r]);
            mx = half_max(mx);                               // finite: row 0 of a tile is always valid
            const float m_new = fmaxf(m_run[qb], mx);
            const float alpha = fast_exp2((m_run[qb] - m_new) * c2);
            const float mc = m_new * c2;
            m_run[qb] = m_new;
            float rs = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = fast_exp2(__builtin_fmaf(s[qb][kb][r], c2, -mc));
                    rs += e;
                    pfrag[qb][kb][r >> 3][r & 7] = (__bf16)e;
                }
            l_run[qb] = l_run[qb] * alpha + rs;
            if (HAS_V) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[qb][db][r] *= alpha;
            }
        }

        // ---- O^T += V^T P^T
        if (HAS_V) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    // contraction element e of this lane <-> tile row kb*32 + hf*16 + 8*(e/4) + 4*lh + e%4
                    const int j16 = lane & 15;
                    const int row0 = kb * 32 + hf * 16 + 4 * lh + (j16 >> 2);
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
                        o_acc[0][db] = mfma_bf16(a, pfrag[0][kb][hf], o_acc[0][db]);
                        o_acc[1][db] = mfma_bf16(a, pfrag[1][kb][hf], o_acc[1][db]);
                    }
                }
        }

        if (t + 1 < ntiles) commit(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: O = diag(l)^-1 acc, optional row log-sum-exp
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float l_tot = half_sum(l_run[qb]);
        const int row = q0 + qb * 32 + lq;
        if (row >= n) continue;
        if (HAS_V) {
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
        if (p.lse != nullptr && lh == 0)
            p.lse[(int64_t)bh * n + row] = (m_run[qb] * c2 + fast_log2(l_tot)) * (p.lse_base2 ? 1.0f : kLn2);
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
