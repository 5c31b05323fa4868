// Host-side launch interface between the C-ABI layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pulsecol {

struct TensorDesc {          // [B, H, n, D] tensor, last dimension contiguous, strides in elements
    int64_t sb, sh, sn;
};

struct AttnParams {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    const int32_t* idx;      // [B*H*groups, idx_stride] (one column set per query group) or nullptr for dense
    int32_t idx_stride;      // entries between the sets of consecutive groups (ns for column sets)
    float* lse;              // optional [B*H, n] row log-sum-exp of the scaled logits
    int32_t lse_base2;       // 0: natural log; 1: log2 units (what the column-mass pass consumes)
    TensorDesc td;           // Q and O: [B, heads, n, D]
    TensorDesc td_kv;        // K and V: [B, kv_heads, n, D]; query head h reads K/V head h / (heads / kv_heads)
    int32_t kv_heads;
    int32_t batch, heads, n, ns;   // ns = columns attended per row (dense: n)
    int32_t groups;          // U query groups per head (1 = the whole head)
    int32_t group_size;      // rows per group, a multiple of the kernel's query block (unused when U = 1)
    float scale;             // logit scale
    // bf16 kernel with 256-row query blocks only: kWorkCounters 64-bit words of device memory through
    // which its workgroups hand out the query blocks, and a stamp that differs from the one of the last
    // launch that used the same words (any contents are fine: counters with another stamp are restarted)
    unsigned long long* work;
    uint32_t work_stamp;
    // variable-length batches: device array [2 * batch] -- per batch element its own sequence length
    // (<= n), then the number of leading entries of its column sets that count (<= ns); nullptr: every
    // element has n rows and ns columns.  Rows and key positions beyond an element's length are padding.
    const int32_t* varlen;
};

constexpr int kWorkCounters = 8;

struct ScoreParams {
    const void* q;
    const void* k;
    const float* lse;        // [B*H, n], log2 units: log2 sum_j exp(z_ij)
    float* scores;           // [B*H*groups, n]
    TensorDesc td;           // Q: [B, heads, n, D]
    TensorDesc td_kv;        // K: [B, kv_heads, n, D]; query head h reads K head h / (heads / kv_heads)
    int32_t kv_heads;
    int32_t batch, heads, n;
    int32_t groups;          // U query groups per head (1 = the whole head)
    int32_t group_size;      // rows per group, a multiple of the kernel's query tile (unused when U = 1)
    float scale;
    const int32_t* varlen;   // as in AttnParams (only the lengths are read); scores beyond them are left untouched
};

struct TopkParams {
    const float* scores;     // [rows, n], consecutive rows `stride` elements apart (a multiple of 4 where n is)
    int32_t* idx;            // [rows, k]
    int32_t rows, n, k;
    int64_t stride;
    // variable-length batches (else nullptr): rows = batch * rows_per_batch; row r belongs to batch
    // element b = r / rows_per_batch and is group u = r % groups of its head; it selects varlen[batch + b]
    // of its first varlen[b] scores and pads the rest of its k entries with -1; rows of groups that lie
    // wholly beyond the element's length are padded altogether
    const int32_t* varlen;
    int32_t batch, rows_per_batch, groups, group_size;
};

// kBlock (bf16 kernel with 256-row query blocks only): idx holds key-BLOCK numbers, one per tile of
// kBlockN_bf16 consecutive keys; ns = kept blocks * kBlockN_bf16
enum AttnMode { kSparse = 0, kDense = 1, kLseOnly = 2, kBlock = 3 };

// Tile geometry of the attention kernels.
constexpr int kBlockM_bf16 = 256;   // query rows per workgroup (4 waves x 64)
constexpr int kBlockN_bf16 = 64;    // gathered columns per tile
constexpr int kBlockM_f32 = 128;    // 4 waves x 32
constexpr int kBlockN_f32 = 32;

// compute units of the current device (cached per device; 256 if the runtime does not say)
int compute_units();

hipError_t launch_attn_bf16(const AttnParams& p, int head_dim, AttnMode mode, hipStream_t s);
// column-sparse attention with query blocks of block_m = 32, 64 or 128 rows (small query groups)
hipError_t launch_attn_bf16_group(const AttnParams& p, int head_dim, int block_m, hipStream_t s);
hipError_t launch_attn_f32(const AttnParams& p, int head_dim, AttnMode mode, hipStream_t s);
hipError_t launch_colmass_bf16(const ScoreParams& p, int head_dim, hipStream_t s);
hipError_t launch_colmass_f32(const ScoreParams& p, int head_dim, hipStream_t s);
hipError_t launch_topk(const TopkParams& p, hipStream_t s);
// Key-block masses for block-sparse selection (Sec. 3.1, block mask): out[r * stride + j] = sum of
// scores[r * stride + j*block .. +block-1], j < n / block, for every score row r (in place is fine: a row's
// sums are written over its own first n / block elements after the whole row has been read)
hipError_t launch_block_sums(const float* scores, float* out, int32_t rows, int32_t n, int64_t stride, int32_t block, hipStream_t s);

// *bad_count (device) = number of wavefront-lanes that saw an entry of idx[0..count) outside [0, n); 0 if none.
// Variable-length batches (varlen != nullptr, per_batch = entries of idx per batch element, k = entries per
// row): of each row only the leading varlen[batch + b] entries are checked, against [0, varlen[b]).
hipError_t launch_index_range_check(const int32_t* idx, int64_t count, int32_t n, int32_t* bad_count,
                                    const int32_t* varlen, int32_t batch, int64_t per_batch, int32_t k, hipStream_t s);

// ---- variable-length batches: the per-batch words the kernels read (device array [2 * batch])
// lens[0..count) -> varlen[first .. first+count) for count <= 64 values carried in the launch itself
struct VarlenChunk { int32_t v[64]; };
hipError_t launch_varlen_store(int32_t* varlen, int32_t first, int32_t count, const VarlenChunk& values, hipStream_t s);
// kept[b] = max(1, floor(keep_ratio * len_b)) (the keep-count rule on the element's own length)
hipError_t launch_varlen_kept_from_ratio(int32_t* varlen, int32_t batch, double keep_ratio, hipStream_t s);
// kept[b] = min(k, len_b)
hipError_t launch_varlen_kept_from_k(int32_t* varlen, int32_t batch, int32_t k, hipStream_t s);
// kept[b] = number of leading non-negative entries of the first column set of batch element b (at most
// min(k, len_b)); per_batch = entries of idx per batch element
hipError_t launch_varlen_kept_from_idx(int32_t* varlen, int32_t batch, const int32_t* idx, int64_t per_batch, int32_t k, hipStream_t s);

}  // namespace pulsecol
