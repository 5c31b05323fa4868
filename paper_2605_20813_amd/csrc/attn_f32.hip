// fp32 attention kernels for gfx950 (the full-precision mode of the library): column-sparse
// attention (Sec. 3.4, appendix listing), dense attention (Sec. 3.1) and the row
// log-sum-exp pass of the identification step (Sec. 3.3).
//
// Same transposed formulation as the bf16 kernels but on the fp32 matrix instruction
// v_mfma_f32_32x32x2_f32 (two contraction indices per step, one per half-wave), so no
// operand is rounded: Q, K, V, P and all accumulators are fp32.  One workgroup = 128 query
// rows (4 waves x 32), one tile = 32 K/V rows staged in padded LDS.
#include "pulsecol_device.h"
#include "pulsecol_kernels.h"

namespace pulsecol {
namespace {

constexpr int BM = kBlockM_f32;
constexpr int BN = kBlockN_f32;
constexpr int NTHREADS = 256;
constexpr int PAD = 4;     // floats of padding per LDS row (keeps 16-byte alignment)

template <int D, int MODE>
__global__ void __launch_bounds__(NTHREADS) attn_f32_kernel(AttnParams p) {
    constexpr int PIECES = D / 4;                 // 16-byte pieces per row
    constexpr int KK = D / 2;                     // contraction steps of Q K^T
    constexpr int DB = D / 32;
    constexpr int CH = BN * PIECES / NTHREADS;
    constexpr int LDW = D + PAD;                  // LDS row stride in floats
    constexpr bool HAS_V = (MODE != kLseOnly);
    constexpr bool GATHER = (MODE == kSparse);

    __shared__ __attribute__((aligned(16))) float lds_k[BN * LDW];
    __shared__ __attribute__((aligned(16))) float lds_v[HAS_V ? BN * LDW : 4];

    const int nqb = (p.n + BM - 1) / BM;
    int bh, qblk;
    if (!xcd_tile(blockIdx.x, nqb, p.batch * p.heads, &bh, &qblk)) return;
    const int b = bh / p.heads, h = bh - b * p.heads;
    const int64_t head_off = (int64_t)b * p.td.sb + (int64_t)h * p.td.sh;
    // grouped-query layout: query head h reads K/V head h / (heads / kv_heads)
    const int64_t kv_off = (int64_t)b * p.td_kv.sb + (int64_t)(h / (p.heads / p.kv_heads)) * p.td_kv.sh;
    const float* __restrict__ Q = (const float*)p.q + head_off;
    const float* __restrict__ K = (const float*)p.k + kv_off;
    const float* __restrict__ V = HAS_V ? (const float*)p.v + kv_off : nullptr;
    // the column set of this query block's group (Sec. 3.3: one set per query group)
    const int group = p.groups > 1 ? (qblk * BM) / p.group_size : 0;
    const int32_t* __restrict__ idx = GATHER ? p.idx + ((int64_t)bh * p.groups + group) * p.ns : nullptr;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, lh = lane >> 5;
    // variable-length batches: the batch element's own length, and the leading `kept` entries of its sets
    int n = p.n, ns = p.ns;
    if (p.varlen != nullptr) {
        n = p.varlen[b];
        const int kept = p.varlen[p.batch + b];
        ns = GATHER ? (kept < ns ? kept : ns) : n;
        if (qblk * BM >= n) return;         // a block of padding rows
    }
    const int ntiles = (ns + BN - 1) / BN;

    // ---- Q fragment: B operand, lane holds Q[query lq][d = 2*kk + lh]
    const int q0 = qblk * BM + wave * 32;
    float qf[KK];
    {
        int row = q0 + lq;
        row = row < n ? row : n - 1;
        const float* src = Q + (int64_t)row * p.td.sn + lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[kk] = src[2 * kk];
    }

    f32x4 stage_k[CH], stage_v[HAS_V ? CH : 1];
    auto fetch = [&](int t) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + NTHREADS * j;
            int pos = t * BN + c / PIECES;
            pos = pos < ns ? pos : ns - 1;
            const int row = GATHER ? idx[pos] : pos;
            const int64_t off = (int64_t)row * p.td_kv.sn + (c % PIECES) * 4;
            stage_k[j] = *(const f32x4*)(K + off);
            if (HAS_V) stage_v[j] = *(const f32x4*)(V + off);
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + NTHREADS * j;
            const int o = (c / PIECES) * LDW + (c % PIECES) * 4;
            *(f32x4*)(lds_k + o) = stage_k[j];
            if (HAS_V) *(f32x4*)(lds_v + o) = stage_v[j];
        }
    };

    const float c2 = p.scale * kLog2e;
    float m_run = -INFINITY, l_run = 0.f;
    f32x16 o_acc[HAS_V ? DB : 1];
#pragma unroll
    for (int db = 0; db < (HAS_V ? DB : 1); ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;

    fetch(0);
    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();              // every wave is done reading the previous tile
        commit();
        __syncthreads();
        if (t + 1 < ntiles) fetch(t + 1);

        // ---- S^T = K_tile Q^T: A operand lane holds K[row lq][d = 2*kk + lh]
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
        const float* krow = lds_k + lq * LDW + lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) s = mfma_f32(krow[2 * kk], qf[kk], s);

        if (t == ntiles - 1 && (ns & (BN - 1))) {
            const int valid = ns - t * BN;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (acc_row(r, lh) >= valid) s[r] = -INFINITY;
        }

        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
        mx = half_max(mx);
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2f((m_run - m_new) * c2);
        const float mc = m_new * c2;
        m_run = m_new;
        float rs = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s[r] = exp2f(__builtin_fmaf(s[r], c2, -mc));
            rs += s[r];
        }
        l_run = l_run * alpha + rs;

        if (HAS_V) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
            // ---- O^T += V^T P^T: step r contracts tile rows acc_row(r, 0) and acc_row(r, 1)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float* vrow = lds_v + acc_row(r, lh) * LDW + lq;
#pragma unroll
                for (int db = 0; db < DB; ++db) o_acc[db] = mfma_f32(vrow[db * 32], s[r], o_acc[db]);
            }
        }
    }

    const float l_tot = half_sum(l_run);
    const int row = q0 + lq;
    if (row < n) {
        if (HAS_V) {
            const float inv = 1.0f / l_tot;
            float* dst = (float*)p.o + head_off + (int64_t)row * p.td.sn;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    f32x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = o_acc[db][r4 * 4 + e] * inv;
                    *(f32x4*)(dst + db * 32 + 8 * r4 + 4 * lh) = w;
                }
        }
        if (p.lse != nullptr && lh == 0)
            p.lse[(int64_t)bh * p.n + row] = (m_run * c2 + log2f(l_tot)) * (p.lse_base2 ? 1.0f : kLn2);
    }
}

template <int D, int MODE>
hipError_t launch(const AttnParams& p, hipStream_t s) {
    const int nqb = (p.n + BM - 1) / BM;
    const int bh_pad = (p.batch * p.heads + 7) / 8 * 8;
    hipLaunchKernelGGL((attn_f32_kernel<D, MODE>), dim3(nqb * bh_pad), dim3(NTHREADS), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_f32(const AttnParams& p, int head_dim, AttnMode mode, hipStream_t s) {
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
