// C-ABI layer of the library: argument validation, scratch ownership, kernel sequencing.
// Host code only; every device-side step lives in the kernel translation units.
#include "../../include/pulsecol.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstdio>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "pulsecol_kernels.h"

struct pulsecol_ctx {
    pulsecol_shape shape;
    int device = 0;
    int groups = 1;                 // U
    float scale = 0.f;
    pulsecol::TensorDesc td{};      // Q, O
    pulsecol::TensorDesc td_kv{};   // K, V
    int kv_heads = 1;
    float* lse = nullptr;           // [B*H, n]   row log-sum-exp, log2 units
    float* scores = nullptr;        // [B*H*U, n]
    int32_t* cached_idx = nullptr;  // [B*H*U, cached_k]
    int32_t cached_k = 0;           // 0 = nothing cached
    int32_t k_max = 0;              // columns per group the cache has room for
    int32_t* bad_count = nullptr;   // one device counter for the validation mode (first word of a small block)
    unsigned long long* work = nullptr;   // work counters of the bf16 attention kernels (same block)
    uint32_t work_stamp = 0;        // stamp of the last launch that used them (every launch takes the next one)
    bool validate = false;          // check column numbers in front of every pulsecol_attn
    int32_t* varlen = nullptr;      // [2 * batch] device words of variable-length batches: lengths, kept counts
    bool varlen_on = false;         // pulsecol_set_seq_lens has given per-element lengths
    int attn_block = 0;             // 0: the cost model picks the one-set-per-head kernel; 256 / 128: the caller has
    std::string last_error;
};

namespace {

thread_local std::string g_last_error;   // failures that have no context to attach to

pulsecol_status fail(pulsecol_ctx* ctx, pulsecol_status st, const std::string& msg) {
    if (ctx) ctx->last_error = msg;
    g_last_error = msg;
    // nothing is printed unless the caller asks for it
    static const bool log = [] { const char* e = std::getenv("PULSECOL_LOG"); return e && e[0] && e[0] != '0'; }();
    if (log) std::fprintf(stderr, "pulsecol: status %d: %s\n", (int)st, msg.c_str());
    return st;
}

pulsecol_status fail_hip(pulsecol_ctx* ctx, hipError_t e, const char* what) {
    return fail(ctx, PULSECOL_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

int elem_align(int dtype) { return dtype == PULSECOL_BF16 ? 8 : 4; }

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// keep_ratio * count with a guard against binary representation error of decimal ratios
int64_t floor_product(double ratio, int64_t count) {
    return (int64_t)std::floor(ratio * (double)count + 1e-9);
}

// K/V strides: explicit, else (multi-head, nothing given) those of Q, else packed [B, kv_heads, n, d]
bool kv_follows_q(const pulsecol_shape* s) {
    return (s->kv_heads == 0 || s->kv_heads == s->heads) && s->kv_stride_b == 0 && s->kv_stride_h == 0 && s->kv_stride_n == 0;
}
int64_t kv_row_stride(const pulsecol_shape* s) {
    if (s->kv_stride_n) return s->kv_stride_n;
    return kv_follows_q(s) && s->stride_n ? s->stride_n : s->head_dim;
}

pulsecol_status check_shape(const pulsecol_shape* s, std::string* why) {
    if (!s) { *why = "shape is NULL"; return PULSECOL_ERR_INVALID_ARG; }
    if (s->batch < 1 || s->heads < 1 || s->seq < 1) { *why = "batch, heads and seq must be >= 1"; return PULSECOL_ERR_INVALID_ARG; }
    if (s->group_size < 0) { *why = "group_size must be >= 0"; return PULSECOL_ERR_INVALID_ARG; }
    if (s->scale < 0.f || !std::isfinite(s->scale)) { *why = "scale must be finite and >= 0"; return PULSECOL_ERR_INVALID_ARG; }
    if (!(s->max_keep_ratio >= 0.0) || !(s->max_keep_ratio <= 1.0)) { *why = "max_keep_ratio must be 0 or in (0, 1]"; return PULSECOL_ERR_INVALID_ARG; }
    if (s->stride_b < 0 || s->stride_h < 0 || s->stride_n < 0) { *why = "strides must be >= 0"; return PULSECOL_ERR_INVALID_ARG; }
    if (s->dtype != PULSECOL_BF16 && s->dtype != PULSECOL_F32) { *why = "dtype must be PULSECOL_BF16 or PULSECOL_F32"; return PULSECOL_ERR_UNSUPPORTED; }
    if (s->head_dim != 64 && s->head_dim != 128) { *why = "head_dim must be 64 or 128"; return PULSECOL_ERR_UNSUPPORTED; }
    if (s->group_size != 0 && s->group_size < s->seq) {
        // a query block of the attention kernels reads ONE column set: groups are whole query blocks
        // (bf16: 256 rows in the main kernel, 128 / 64 / 32 in the small-group kernel; f32: 128)
        const int unit = s->dtype == PULSECOL_BF16 ? 32 : pulsecol::kBlockM_f32;
        if (s->group_size % unit != 0) {
            *why = "group_size must be 0, >= seq, or a multiple of 32 rows (bf16) / 128 rows (f32)";
            return PULSECOL_ERR_UNSUPPORTED;
        }
    }
    if ((int64_t)s->batch * s->heads > (1 << 20)) { *why = "batch*heads too large"; return PULSECOL_ERR_UNSUPPORTED; }
    if (s->stride_n != 0 && s->stride_n < s->head_dim) { *why = "stride_n smaller than head_dim"; return PULSECOL_ERR_INVALID_ARG; }
    if (s->kv_heads < 0 || (s->kv_heads > 0 && (s->kv_heads > s->heads || s->heads % s->kv_heads != 0))) {
        *why = "kv_heads must be 0 or a divisor of heads";
        return PULSECOL_ERR_INVALID_ARG;
    }
    if (s->kv_stride_b < 0 || s->kv_stride_h < 0 || s->kv_stride_n < 0) { *why = "strides must be >= 0"; return PULSECOL_ERR_INVALID_ARG; }
    if (s->kv_stride_n != 0 && s->kv_stride_n < s->head_dim) { *why = "kv_stride_n smaller than head_dim"; return PULSECOL_ERR_INVALID_ARG; }
    {   // the kernels address a head's K/V rows with 32-bit byte offsets
        const int64_t sn = kv_row_stride(s);
        const int64_t esize = s->dtype == PULSECOL_BF16 ? 2 : 4;
        if ((int64_t)s->seq * sn * esize >= ((int64_t)1 << 32)) { *why = "seq * stride_n of K/V exceeds 4 GiB per head"; return PULSECOL_ERR_UNSUPPORTED; }
        if (s->seq >= (1 << 24) || sn * esize >= (1 << 24)) { *why = "seq or the K/V row stride in bytes reaches 2^24"; return PULSECOL_ERR_UNSUPPORTED; }
        // ... and so does the copy of a query block
        const int64_t qn = s->stride_n ? s->stride_n : s->head_dim;
        if ((int64_t)s->seq * qn * esize >= ((int64_t)1 << 32)) { *why = "seq * stride_n of Q exceeds 4 GiB per head"; return PULSECOL_ERR_UNSUPPORTED; }
        if (qn * esize >= (1 << 24)) { *why = "the Q row stride in bytes reaches 2^24"; return PULSECOL_ERR_UNSUPPORTED; }
    }
    const int a = elem_align(s->dtype);
    if (s->stride_b % a || s->stride_h % a || s->stride_n % a || s->kv_stride_b % a || s->kv_stride_h % a || s->kv_stride_n % a) {
        *why = "strides must be multiples of 16 bytes";
        return PULSECOL_ERR_ALIGNMENT;
    }
    return PULSECOL_OK;
}

// the fields of a context that follow from the shape alone (host only)
void derive_from_shape(pulsecol_ctx* c, const pulsecol_shape* shape, int device) {
    c->shape = *shape;
    c->device = device;
    c->groups = (shape->group_size == 0 || shape->group_size >= shape->seq)
                    ? 1 : (shape->seq + shape->group_size - 1) / shape->group_size;
    c->scale = shape->scale > 0.f ? shape->scale : 1.0f / std::sqrt((float)shape->head_dim);
    c->td.sn = shape->stride_n ? shape->stride_n : shape->head_dim;
    c->td.sh = shape->stride_h ? shape->stride_h : (int64_t)shape->seq * c->td.sn;
    c->td.sb = shape->stride_b ? shape->stride_b : (int64_t)shape->heads * c->td.sh;
    c->kv_heads = shape->kv_heads ? shape->kv_heads : shape->heads;
    if (kv_follows_q(shape)) {
        c->td_kv = c->td;
    } else {
        c->td_kv.sn = shape->kv_stride_n ? shape->kv_stride_n : shape->head_dim;
        c->td_kv.sh = shape->kv_stride_h ? shape->kv_stride_h : (int64_t)shape->seq * c->td_kv.sn;
        c->td_kv.sb = shape->kv_stride_b ? shape->kv_stride_b : (int64_t)c->kv_heads * c->td_kv.sh;
    }
}

struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    hipError_t err = hipSuccess;
    explicit DeviceGuard(int dev) {
        err = hipGetDevice(&prev);
        if (err == hipSuccess && prev != dev) {
            err = hipSetDevice(dev);
            switched = (err == hipSuccess);
        }
    }
    ~DeviceGuard() { if (switched) (void)hipSetDevice(prev); }
};

pulsecol::AttnParams attn_params(pulsecol_ctx* c, const void* Q, const void* K, const void* V, void* O,
                                 const int32_t* idx, int32_t ns, float* lse, int lse_base2) {
    pulsecol::AttnParams p{};
    p.q = Q; p.k = K; p.v = V; p.o = O; p.idx = idx; p.lse = lse; p.lse_base2 = lse_base2;
    p.td = c->td; p.td_kv = c->td_kv; p.kv_heads = c->kv_heads;
    p.batch = c->shape.batch; p.heads = c->shape.heads; p.n = c->shape.seq; p.ns = ns; p.idx_stride = ns;
    p.groups = c->groups; p.group_size = c->shape.group_size;
    p.scale = c->scale;
    p.varlen = c->varlen_on ? c->varlen : nullptr;
    p.work = c->work;
    if (++c->work_stamp == 0) c->work_stamp = 1;       // freshly cleared counters carry stamp 0
    p.work_stamp = c->work_stamp;
    return p;
}

// Query rows per workgroup of the column-sparse kernel a call with ns kept columns runs in.  Group-wise
// sets: the largest block that divides the group size.  One set per head: the hand-scheduled kernel
// with 256-row blocks, except for short jobs, where its fixed costs (one workgroup per CU, a long
// start-up per launch and per query block) outweigh its faster steady state and the plain kernel
// with 128-row blocks, three to a CU, finishes first.  The rule is a two-line cost model fitted to
// launches at 4K to 16K context (microseconds; R = 256-row blocks per CU, t = 64-column tiles):
//   scheduled: 33 + R (8.7 + 1.64 t)      plain: 12.6 + R (3.1 + 2.23 t)
int sparse_block_m(const pulsecol_ctx* c, int32_t ns) {
    if (c->shape.dtype != PULSECOL_BF16) return pulsecol::kBlockM_f32;
    if (c->groups == 1) {
        if (c->attn_block != 0) return c->attn_block;
        const double blocks = (double)((c->shape.seq + 255) / 256) * c->shape.batch * c->shape.heads;
        const double R = blocks / (double)pulsecol::compute_units();
        const double t = (double)((ns + 63) / 64);
        const double scheduled = 33.0 + R * (8.7 + 1.64 * t), plain = 12.6 + R * (3.1 + 2.23 * t);
        return plain < scheduled ? 128 : pulsecol::kBlockM_bf16;
    }
    for (int bm : {256, 128, 64}) if (c->shape.group_size % bm == 0) return bm;
    return 32;
}

hipError_t launch_attn(const pulsecol_ctx* c, const pulsecol::AttnParams& p, pulsecol::AttnMode mode, hipStream_t s) {
    if (mode == pulsecol::kSparse && c->shape.dtype == PULSECOL_BF16 && sparse_block_m(c, p.ns) < pulsecol::kBlockM_bf16)
        return pulsecol::launch_attn_bf16_group(p, c->shape.head_dim, sparse_block_m(c, p.ns), s);
    return c->shape.dtype == PULSECOL_BF16 ? pulsecol::launch_attn_bf16(p, c->shape.head_dim, mode, s)
                                           : pulsecol::launch_attn_f32(p, c->shape.head_dim, mode, s);
}

pulsecol_status check_ptrs(pulsecol_ctx* ctx, std::initializer_list<const void*> tensors, const char* who) {
    for (const void* t : tensors) {
        if (!t) return fail(ctx, PULSECOL_ERR_INVALID_ARG, std::string(who) + ": NULL tensor pointer");
        if (misaligned(t)) return fail(ctx, PULSECOL_ERR_ALIGNMENT, std::string(who) + ": tensor pointer not 16-byte aligned");
    }
    return PULSECOL_OK;
}

// column pass of the scoring stage: ctx->lse (log2 units) must hold the row log-sum-exp of Q, K
pulsecol_status run_colmass(pulsecol_ctx* ctx, const void* Q, const void* K, float* out, hipStream_t s) {
    pulsecol::ScoreParams sp{};
    sp.q = Q; sp.k = K; sp.lse = ctx->lse; sp.scores = out; sp.td = ctx->td; sp.td_kv = ctx->td_kv; sp.kv_heads = ctx->kv_heads;
    sp.batch = ctx->shape.batch; sp.heads = ctx->shape.heads; sp.n = ctx->shape.seq; sp.scale = ctx->scale;
    sp.groups = ctx->groups; sp.group_size = ctx->shape.group_size;
    sp.varlen = ctx->varlen_on ? ctx->varlen : nullptr;
    const hipError_t e = ctx->shape.dtype == PULSECOL_BF16 ? pulsecol::launch_colmass_bf16(sp, ctx->shape.head_dim, s)
                                                           : pulsecol::launch_colmass_f32(sp, ctx->shape.head_dim, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "column-mass kernel");
    return PULSECOL_OK;
}

// scores of the current Q, K into `out` (two launches: row pass, column pass)
pulsecol_status run_scores(pulsecol_ctx* ctx, const void* Q, const void* K, float* out, hipStream_t s) {
    pulsecol::AttnParams ap = attn_params(ctx, Q, K, nullptr, nullptr, nullptr, ctx->shape.seq, ctx->lse, 1);
    const hipError_t e = launch_attn(ctx, ap, pulsecol::kLseOnly, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "row log-sum-exp kernel");
    return run_colmass(ctx, Q, K, out, s);
}

// top-k of ctx->scores into idx_out, and into the context's cache
pulsecol_status run_topk(pulsecol_ctx* ctx, const float* scores, int32_t k, int32_t* out, hipStream_t s);

pulsecol_status select_from_scores(pulsecol_ctx* ctx, double keep_ratio, int32_t k, int32_t* idx_out, hipStream_t s, const char* who) {
    if (ctx->varlen_on) {
        // every batch element keeps max(1, floor(keep_ratio * its own length)) columns
        const hipError_t ev = pulsecol::launch_varlen_kept_from_ratio(ctx->varlen, ctx->shape.batch, keep_ratio, s);
        if (ev != hipSuccess) return fail_hip(ctx, ev, (std::string(who) + ": per-element keep counts").c_str());
    }
    pulsecol_status st = run_topk(ctx, ctx->scores, k, idx_out, s);
    if (st != PULSECOL_OK) return st;
    ctx->cached_k = 0;
    const size_t idx_bytes = (size_t)ctx->shape.batch * ctx->shape.heads * ctx->groups * (size_t)k * sizeof(int32_t);
    const hipError_t e = hipMemcpyAsync(ctx->cached_idx, idx_out, idx_bytes, hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return fail_hip(ctx, e, (std::string(who) + ": caching the pattern").c_str());
    ctx->cached_k = k;
    return PULSECOL_OK;
}

pulsecol_status run_topk(pulsecol_ctx* ctx, const float* scores, int32_t k, int32_t* out, hipStream_t s) {
    pulsecol::TopkParams tp{};
    tp.scores = scores; tp.idx = out;
    tp.rows = ctx->shape.batch * ctx->shape.heads * ctx->groups; tp.n = ctx->shape.seq; tp.k = k; tp.stride = ctx->shape.seq;
    tp.varlen = ctx->varlen_on ? ctx->varlen : nullptr;
    tp.batch = ctx->shape.batch; tp.rows_per_batch = ctx->shape.heads * ctx->groups;
    tp.groups = ctx->groups; tp.group_size = ctx->shape.group_size;
    const hipError_t e = pulsecol::launch_topk(tp, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "top-k kernel");
    return PULSECOL_OK;
}

// ---- scratch of the entry point that allocates nothing (pulsecol_select_noalloc)
// A file-scope device array, one copy per GPU, held until the process ends: 256 bytes of work
// counters, then room for kNoallocFloats fp32 words (row log-sum-exp [B*H, n], then scores
// [B*H*U, n]).  The array's name is only a host-side stand-in for the symbol; the address of a
// device's copy comes from hipGetSymbolAddress, asked once per device with that device current.
constexpr size_t kNoallocFloats = (size_t)4 << 20;                 // 16 MiB
constexpr size_t kNoallocCounterBytes = 256;
static __device__ __align__(256) unsigned char scratch[kNoallocCounterBytes + kNoallocFloats * sizeof(float)];

struct NoallocDevice {
    unsigned char* ptr = nullptr;     // this device's copy of `scratch`
    uint32_t stamp = 0;               // stamp of the last launch that used its work counters
};
constexpr int kMaxDevices = 64;
NoallocDevice g_noalloc[kMaxDevices];
std::mutex g_noalloc_mutex;

// the current device's copy of the scratch array (nullptr + *err on failure)
NoallocDevice* noalloc_device(int dev, hipError_t* err) {
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    NoallocDevice* d = &g_noalloc[dev];
    if (d->ptr == nullptr) {
        unsigned char* ptr = nullptr;
        *err = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || ptr == nullptr) {
            if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
            return nullptr;
        }
        d->ptr = ptr;
    }
    return d;
}

// what the block-sparse calls need of a context: the hand-scheduled bf16 kernel (whole 256-row query blocks
// per block mask), whole key blocks, fixed-length batches, and block offsets that the 24-bit multiply holds
pulsecol_status check_block_mode(pulsecol_ctx* ctx, const char* who) {
    const pulsecol_shape& sh = ctx->shape;
    if (sh.dtype != PULSECOL_BF16) return fail(ctx, PULSECOL_ERR_UNSUPPORTED, std::string(who) + ": block-sparse attention is bf16 only");
    if (ctx->groups > 1 && sh.group_size % pulsecol::kBlockM_bf16 != 0)
        return fail(ctx, PULSECOL_ERR_UNSUPPORTED, std::string(who) + ": query blocks of the block mask are multiples of 256 rows (group_size)");
    if (sh.seq % pulsecol::kBlockN_bf16 != 0)
        return fail(ctx, PULSECOL_ERR_UNSUPPORTED, std::string(who) + ": seq must be a multiple of the key block (64)");
    if (ctx->varlen_on) return fail(ctx, PULSECOL_ERR_UNSUPPORTED, std::string(who) + ": not available with per-element sequence lengths");
    if (ctx->td_kv.sn * 2 * pulsecol::kBlockN_bf16 >= (1 << 24))
        return fail(ctx, PULSECOL_ERR_UNSUPPORTED, std::string(who) + ": 64 K/V rows span 2^24 bytes or more");
    return PULSECOL_OK;
}

}  // namespace

extern "C" {

pulsecol_status pulsecol_validate_shape(const pulsecol_shape* shape) {
    std::string why;
    const pulsecol_status st = check_shape(shape, &why);
    return st == PULSECOL_OK ? st : fail(nullptr, st, why);
}

pulsecol_status pulsecol_create(pulsecol_ctx** out, const pulsecol_shape* shape, int device) {
    if (!out) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_create: out is NULL");
    std::string why;
    pulsecol_status st = check_shape(shape, &why);
    if (st != PULSECOL_OK) return fail(nullptr, st, "pulsecol_create: " + why);
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess) return fail_hip(nullptr, e, "pulsecol_create: hipGetDeviceCount");
    if (device < 0 || device >= ndev) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_create: no such device");

    pulsecol_ctx* c = new (std::nothrow) pulsecol_ctx();
    if (!c) return fail(nullptr, PULSECOL_ERR_OOM, "pulsecol_create: host allocation failed");
    derive_from_shape(c, shape, device);

    DeviceGuard guard(device);
    if (guard.err != hipSuccess) { delete c; return fail_hip(nullptr, guard.err, "pulsecol_create: hipSetDevice"); }
    const size_t rows = (size_t)shape->batch * shape->heads;
    const size_t row_bytes = (size_t)shape->seq * sizeof(float);
    hipError_t e1 = hipMalloc((void**)&c->lse, rows * row_bytes);
    hipError_t e2 = e1 == hipSuccess ? hipMalloc((void**)&c->scores, rows * c->groups * row_bytes) : e1;
    c->k_max = shape->max_keep_ratio > 0.0 ? pulsecol_num_keep(shape->seq, shape->max_keep_ratio) : shape->seq;
    hipError_t e3 = e2 == hipSuccess ? hipMalloc((void**)&c->cached_idx, rows * c->groups * (size_t)c->k_max * sizeof(int32_t)) : e2;
    static_assert(64 + pulsecol::kWorkCounters * sizeof(unsigned long long) <= 256, "counter block");
    if (e3 == hipSuccess) e3 = hipMalloc((void**)&c->varlen, 2 * (size_t)shape->batch * sizeof(int32_t));
    if (e3 == hipSuccess) e3 = hipMalloc((void**)&c->bad_count, 256);
    if (e3 == hipSuccess) e3 = hipMemset(c->bad_count, 0, 256);
    if (e3 == hipSuccess) c->work = reinterpret_cast<unsigned long long*>(c->bad_count + 16);
    if (e3 != hipSuccess) {
        if (c->lse) (void)hipFree(c->lse);
        if (c->scores) (void)hipFree(c->scores);
        if (c->cached_idx) (void)hipFree(c->cached_idx);
        if (c->bad_count) (void)hipFree(c->bad_count);
        if (c->varlen) (void)hipFree(c->varlen);
        (void)hipGetLastError();
        delete c;
        return e3 == hipErrorOutOfMemory ? fail(nullptr, PULSECOL_ERR_OOM, "pulsecol_create: scratch allocation failed")
                                         : fail_hip(nullptr, e3, "pulsecol_create: hipMalloc");
    }
    const char* env = std::getenv("PULSECOL_VALIDATE");
    c->validate = env != nullptr && env[0] != '\0' && env[0] != '0';
    *out = c;
    return PULSECOL_OK;
}

pulsecol_status pulsecol_set_validation(pulsecol_ctx* ctx, int on) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_set_validation: ctx is NULL");
    ctx->validate = on != 0;
    return PULSECOL_OK;
}

pulsecol_status pulsecol_set_attn_block(pulsecol_ctx* ctx, int32_t block_m) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_set_attn_block: ctx is NULL");
    if (block_m != 0 && block_m != 128 && block_m != 256)
        return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_set_attn_block: block_m must be 0, 128 or 256");
    ctx->attn_block = block_m;
    return PULSECOL_OK;
}

pulsecol_status pulsecol_set_seq_lens(pulsecol_ctx* ctx, const int32_t* seq_lens, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_set_seq_lens: ctx is NULL");
    if (!seq_lens) { ctx->varlen_on = false; return PULSECOL_OK; }
    const int32_t B = ctx->shape.batch;
    for (int32_t b = 0; b < B; ++b)
        if (seq_lens[b] < 1 || seq_lens[b] > ctx->shape.seq)
            return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_set_seq_lens: need 1 <= seq_lens[b] <= seq");
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_set_seq_lens: hipSetDevice");
    // The lengths travel inside launch arguments, 64 at a time: nothing is read from the caller's array
    // after this call returns, and nothing synchronises.  The kept counts start at the lengths.
    for (int32_t first = 0; first < B; first += 64) {
        pulsecol::VarlenChunk chunk{};
        const int32_t count = B - first < 64 ? B - first : 64;
        for (int32_t i = 0; i < count; ++i) chunk.v[i] = seq_lens[first + i];
        hipError_t e = pulsecol::launch_varlen_store(ctx->varlen, first, count, chunk, (hipStream_t)stream);
        if (e == hipSuccess) e = pulsecol::launch_varlen_store(ctx->varlen, B + first, count, chunk, (hipStream_t)stream);
        if (e != hipSuccess) { ctx->varlen_on = false; return fail_hip(ctx, e, "pulsecol_set_seq_lens: storing the lengths"); }
    }
    ctx->varlen_on = true;
    ctx->cached_k = 0;            // a cached pattern belongs to the lengths it was selected with
    return PULSECOL_OK;
}

pulsecol_status pulsecol_destroy(pulsecol_ctx* ctx) {
    if (!ctx) return PULSECOL_OK;
    DeviceGuard guard(ctx->device);
    (void)hipFree(ctx->lse);
    (void)hipFree(ctx->scores);
    (void)hipFree(ctx->cached_idx);
    (void)hipFree(ctx->bad_count);
    (void)hipFree(ctx->varlen);
    delete ctx;
    return PULSECOL_OK;
}

int32_t pulsecol_num_keep(int32_t seq, double keep_ratio) {
    if (seq < 1 || !(keep_ratio > 0.0) || !(keep_ratio <= 1.0)) return -1;
    const int64_t k = floor_product(keep_ratio, seq);
    return (int32_t)(k < 1 ? 1 : (k > seq ? seq : k));
}

pulsecol_status pulsecol_scores(pulsecol_ctx* ctx, const void* Q, const void* K, float* scores_out, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_scores: ctx is NULL");
    pulsecol_status st = check_ptrs(ctx, {Q, K, scores_out}, "pulsecol_scores");
    if (st != PULSECOL_OK) return st;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_scores: hipSetDevice");
    return run_scores(ctx, Q, K, scores_out, (hipStream_t)stream);
}

pulsecol_status pulsecol_topk(pulsecol_ctx* ctx, const float* scores, int32_t k, int32_t* idx_out, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_topk: ctx is NULL");
    if (!scores || !idx_out) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_topk: NULL pointer");
    if (k < 1 || k > ctx->shape.seq) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_topk: need 1 <= k <= seq");
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_topk: hipSetDevice");
    if (ctx->varlen_on) {
        const hipError_t ev = pulsecol::launch_varlen_kept_from_k(ctx->varlen, ctx->shape.batch, k, (hipStream_t)stream);
        if (ev != hipSuccess) return fail_hip(ctx, ev, "pulsecol_topk: per-element keep counts");
    }
    return run_topk(ctx, scores, k, idx_out, (hipStream_t)stream);
}

pulsecol_status pulsecol_select(pulsecol_ctx* ctx, const void* Q, const void* K, double keep_ratio, int refresh,
                                int32_t* idx_out, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_select: ctx is NULL");
    if (!idx_out) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_select: idx_out is NULL");
    const int32_t k = pulsecol_num_keep(ctx->shape.seq, keep_ratio);
    if (k < 0) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_select: keep_ratio must be in (0, 1]");
    if (k > ctx->k_max) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_select: keep_ratio exceeds the context's max_keep_ratio");
    const size_t idx_bytes = (size_t)ctx->shape.batch * ctx->shape.heads * ctx->groups * (size_t)k * sizeof(int32_t);
    hipStream_t s = (hipStream_t)stream;
    if (!refresh) {
        if (ctx->cached_k == 0) return fail(ctx, PULSECOL_ERR_NO_PATTERN, "pulsecol_select: refresh == 0 but no pattern is cached");
        if (ctx->cached_k != k) return fail(ctx, PULSECOL_ERR_NO_PATTERN, "pulsecol_select: cached pattern has a different k");
        DeviceGuard guard(ctx->device);
        if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_select: hipSetDevice");
        const hipError_t e = hipMemcpyAsync(idx_out, ctx->cached_idx, idx_bytes, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail_hip(ctx, e, "pulsecol_select: copy of the cached pattern");
        return PULSECOL_OK;
    }
    pulsecol_status st = check_ptrs(ctx, {Q, K}, "pulsecol_select");
    if (st != PULSECOL_OK) return st;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_select: hipSetDevice");
    st = run_scores(ctx, Q, K, ctx->scores, s);
    if (st != PULSECOL_OK) return st;
    return select_from_scores(ctx, keep_ratio, k, idx_out, s, "pulsecol_select");
}

pulsecol_status pulsecol_select_noalloc(const pulsecol_shape* shape, const void* Q, const void* K, double keep_ratio,
                                        int32_t* idx_out, void* stream) {
    std::string why;
    pulsecol_status st = check_shape(shape, &why);
    if (st != PULSECOL_OK) return fail(nullptr, st, "pulsecol_select_noalloc: " + why);
    if (!idx_out) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_select_noalloc: idx_out is NULL");
    const int32_t k = pulsecol_num_keep(shape->seq, keep_ratio);
    if (k < 0) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_select_noalloc: keep_ratio must be in (0, 1]");
    st = check_ptrs(nullptr, {Q, K}, "pulsecol_select_noalloc");
    if (st != PULSECOL_OK) return st;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(nullptr, e, "pulsecol_select_noalloc: hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, PULSECOL_ERR_UNSUPPORTED, "pulsecol_select_noalloc: device number out of range");

    pulsecol_ctx c;                                   // host-side bookkeeping only; owns no device memory
    derive_from_shape(&c, shape, dev);
    const size_t rows = (size_t)shape->batch * shape->heads;
    const size_t need = rows * (size_t)shape->seq * (1 + (size_t)c.groups);
    if (need > kNoallocFloats)
        return fail(nullptr, PULSECOL_ERR_UNSUPPORTED,
                    "pulsecol_select_noalloc: batch*heads*seq*(1 + groups) = " + std::to_string(need) +
                    " exceeds the static scratch of " + std::to_string(kNoallocFloats) + " fp32 words");
    NoallocDevice* d = noalloc_device(dev, &e);
    if (!d) return fail_hip(nullptr, e, "pulsecol_select_noalloc: hipGetSymbolAddress");
    c.work = reinterpret_cast<unsigned long long*>(d->ptr);
    c.work_stamp = d->stamp;                          // the launch takes the next stamp: stale counters restart themselves
    c.lse = reinterpret_cast<float*>(d->ptr + kNoallocCounterBytes);
    c.scores = c.lse + rows * (size_t)shape->seq;
    st = run_scores(&c, Q, K, c.scores, (hipStream_t)stream);
    d->stamp = c.work_stamp;
    if (st == PULSECOL_OK) st = run_topk(&c, c.scores, k, idx_out, (hipStream_t)stream);
    if (st != PULSECOL_OK) g_last_error = "pulsecol_select_noalloc: " + c.last_error;
    return st;
}

pulsecol_status pulsecol_refresh_dense(pulsecol_ctx* ctx, const void* Q, const void* K, const void* V,
                                       double keep_ratio, void* O, int32_t* idx_out, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_refresh_dense: ctx is NULL");
    if (!idx_out) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_refresh_dense: idx_out is NULL");
    const int32_t k = pulsecol_num_keep(ctx->shape.seq, keep_ratio);
    if (k < 0) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_refresh_dense: keep_ratio must be in (0, 1]");
    if (k > ctx->k_max) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_refresh_dense: keep_ratio exceeds the context's max_keep_ratio");
    pulsecol_status st = check_ptrs(ctx, {Q, K, V, O}, "pulsecol_refresh_dense");
    if (st != PULSECOL_OK) return st;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_refresh_dense: hipSetDevice");
    hipStream_t s = (hipStream_t)stream;
    // dense attention that leaves the row log-sum-exp (log2 units) where the column pass reads it
    const pulsecol::AttnParams p = attn_params(ctx, Q, K, V, O, nullptr, ctx->shape.seq, ctx->lse, 1);
    const hipError_t e = launch_attn(ctx, p, pulsecol::kDense, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "dense attention kernel");
    st = run_colmass(ctx, Q, K, ctx->scores, s);
    if (st != PULSECOL_OK) return st;
    return select_from_scores(ctx, keep_ratio, k, idx_out, s, "pulsecol_refresh_dense");
}

pulsecol_status pulsecol_attn(pulsecol_ctx* ctx, const void* Q, const void* K, const void* V, const int32_t* idx,
                              int32_t k, void* O, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn: ctx is NULL");
    pulsecol_status st = check_ptrs(ctx, {Q, K, V, O}, "pulsecol_attn");
    if (st != PULSECOL_OK) return st;
    if (!idx) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn: idx is NULL");
    if (k < 1 || k > ctx->shape.seq) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn: need 1 <= k <= seq");
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_attn: hipSetDevice");
    const int64_t per_batch = (int64_t)ctx->shape.heads * ctx->groups * k;
    if (ctx->varlen_on) {
        // how many leading entries of an element's column sets count is read off the sets themselves
        // (their unused tail is -1), so the call depends on no earlier one
        const hipError_t ev = pulsecol::launch_varlen_kept_from_idx(ctx->varlen, ctx->shape.batch, idx, per_batch, k, (hipStream_t)stream);
        if (ev != hipSuccess) return fail_hip(ctx, ev, "pulsecol_attn: per-element keep counts");
    }
    if (ctx->validate) {
        // the one mode that synchronises: the answer has to be known before anything is gathered
        const int64_t count = (int64_t)ctx->shape.batch * per_batch;
        hipError_t ev = pulsecol::launch_index_range_check(idx, count, ctx->shape.seq, ctx->bad_count,
                                                           ctx->varlen_on ? ctx->varlen : nullptr, ctx->shape.batch, per_batch, k,
                                                           (hipStream_t)stream);
        int32_t bad = 0;
        if (ev == hipSuccess) ev = hipMemcpyAsync(&bad, ctx->bad_count, sizeof(bad), hipMemcpyDeviceToHost, (hipStream_t)stream);
        if (ev == hipSuccess) ev = hipStreamSynchronize((hipStream_t)stream);
        if (ev != hipSuccess) return fail_hip(ctx, ev, "pulsecol_attn: index validation");
        if (bad != 0) return fail(ctx, PULSECOL_ERR_BAD_INDEX, "pulsecol_attn: idx holds entries outside [0, seq)");
    }
    const pulsecol::AttnParams p = attn_params(ctx, Q, K, V, O, idx, k, nullptr, 0);
    const hipError_t e = launch_attn(ctx, p, pulsecol::kSparse, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "column-sparse attention kernel");
    return PULSECOL_OK;
}

int32_t pulsecol_num_keep_blocks(int32_t seq, double keep_ratio) {
    if (seq < pulsecol::kBlockN_bf16 || seq % pulsecol::kBlockN_bf16 != 0) return -1;
    return pulsecol_num_keep(seq / pulsecol::kBlockN_bf16, keep_ratio);
}

pulsecol_status pulsecol_select_blocks(pulsecol_ctx* ctx, const void* Q, const void* K, double keep_ratio,
                                       int32_t* block_idx_out, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_select_blocks: ctx is NULL");
    if (!block_idx_out) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_select_blocks: block_idx_out is NULL");
    pulsecol_status st = check_block_mode(ctx, "pulsecol_select_blocks");
    if (st != PULSECOL_OK) return st;
    const int32_t kb = pulsecol_num_keep_blocks(ctx->shape.seq, keep_ratio);
    if (kb < 0) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_select_blocks: keep_ratio must be in (0, 1]");
    st = check_ptrs(ctx, {Q, K}, "pulsecol_select_blocks");
    if (st != PULSECOL_OK) return st;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_select_blocks: hipSetDevice");
    hipStream_t s = (hipStream_t)stream;
    st = run_scores(ctx, Q, K, ctx->scores, s);
    if (st != PULSECOL_OK) return st;
    // block masses over the front of every score row, then the same exact top-k on rows of seq / 64 elements
    const int32_t rows = ctx->shape.batch * ctx->shape.heads * ctx->groups;
    hipError_t e = pulsecol::launch_block_sums(ctx->scores, ctx->scores, rows, ctx->shape.seq, ctx->shape.seq, pulsecol::kBlockN_bf16, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "block-mass kernel");
    pulsecol::TopkParams tp{};
    tp.scores = ctx->scores; tp.idx = block_idx_out; tp.rows = rows;
    tp.n = ctx->shape.seq / pulsecol::kBlockN_bf16; tp.k = kb; tp.stride = ctx->shape.seq;
    e = pulsecol::launch_topk(tp, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "top-k kernel (key blocks)");
    return PULSECOL_OK;
}

pulsecol_status pulsecol_attn_block(pulsecol_ctx* ctx, const void* Q, const void* K, const void* V, const int32_t* block_idx,
                                    int32_t kb, void* O, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn_block: ctx is NULL");
    pulsecol_status st = check_block_mode(ctx, "pulsecol_attn_block");
    if (st != PULSECOL_OK) return st;
    st = check_ptrs(ctx, {Q, K, V, O}, "pulsecol_attn_block");
    if (st != PULSECOL_OK) return st;
    if (!block_idx) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn_block: block_idx is NULL");
    const int32_t nblocks = ctx->shape.seq / pulsecol::kBlockN_bf16;
    if (kb < 1 || kb > nblocks) return fail(ctx, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn_block: need 1 <= kb <= seq / 64");
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_attn_block: hipSetDevice");
    if (ctx->validate) {
        const int64_t count = (int64_t)ctx->shape.batch * ctx->shape.heads * ctx->groups * kb;
        hipError_t ev = pulsecol::launch_index_range_check(block_idx, count, nblocks, ctx->bad_count, nullptr, 0, 0, 0, (hipStream_t)stream);
        int32_t bad = 0;
        if (ev == hipSuccess) ev = hipMemcpyAsync(&bad, ctx->bad_count, sizeof(bad), hipMemcpyDeviceToHost, (hipStream_t)stream);
        if (ev == hipSuccess) ev = hipStreamSynchronize((hipStream_t)stream);
        if (ev != hipSuccess) return fail_hip(ctx, ev, "pulsecol_attn_block: index validation");
        if (bad != 0) return fail(ctx, PULSECOL_ERR_BAD_INDEX, "pulsecol_attn_block: block_idx holds entries outside [0, seq / 64)");
    }
    pulsecol::AttnParams p = attn_params(ctx, Q, K, V, O, block_idx, kb * pulsecol::kBlockN_bf16, nullptr, 0);
    p.idx_stride = kb;
    const hipError_t e = pulsecol::launch_attn_bf16(p, ctx->shape.head_dim, pulsecol::kBlock, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "block-sparse attention kernel");
    return PULSECOL_OK;
}

pulsecol_status pulsecol_attn_dense(pulsecol_ctx* ctx, const void* Q, const void* K, const void* V, void* O,
                                    float* lse_out, void* stream) {
    if (!ctx) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn_dense: ctx is NULL");
    pulsecol_status st = check_ptrs(ctx, {Q, K, V, O}, "pulsecol_attn_dense");
    if (st != PULSECOL_OK) return st;
    DeviceGuard guard(ctx->device);
    if (guard.err != hipSuccess) return fail_hip(ctx, guard.err, "pulsecol_attn_dense: hipSetDevice");
    const pulsecol::AttnParams p = attn_params(ctx, Q, K, V, O, nullptr, ctx->shape.seq, lse_out, 0);
    const hipError_t e = launch_attn(ctx, p, pulsecol::kDense, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "dense attention kernel");
    return PULSECOL_OK;
}

int32_t pulsecol_refresh_schedule(int32_t T, double eta, int32_t R, int32_t* steps_out) {
    if (T < 1 || R < 1 || !(eta > 0.0) || !(eta <= 1.0) || !steps_out) return -1;
    int64_t t_win = floor_product(eta, T);
    if (t_win < 1) t_win = 1;
    if (R == 1) { steps_out[0] = 1; return 1; }
    for (int64_t r = 1; r <= R; ++r) steps_out[r - 1] = (int32_t)(1 + ((r - 1) * (t_win - 1)) / (R - 1));
    return R;
}

int32_t pulsecol_refresh_schedule_power(int32_t T, double eta, int32_t R, int32_t* steps_out) {
    if (T < 1 || R < 1 || !(eta > 0.0) || !(eta <= 1.0) || !steps_out) return -1;
    int64_t t_win = floor_product(eta, T);
    if (t_win < 1) t_win = 1;
    if (R == 1) { steps_out[0] = 1; return 1; }
    const int64_t den = (int64_t)(R - 1) * (R - 1);
    for (int64_t i = 0; i < R; ++i) steps_out[i] = (int32_t)(1 + (i * i * (t_win - 1)) / den);
    return R;
}

int32_t pulsecol_refresh_schedule_random(int32_t T, double eta, int32_t R, const double* uniforms, int32_t* steps_out) {
    if (T < 1 || R < 1 || !(eta > 0.0) || !(eta <= 1.0) || !steps_out) return -1;
    int64_t t_win = floor_product(eta, T);
    if (t_win < 1) t_win = 1;
    const int64_t m = t_win - 1;
    if (R - 1 > m) return -1;
    if (R > 1 && !uniforms) return -1;
    for (int32_t i = 0; i + 1 < R; ++i)
        if (!(uniforms[i] >= 0.0) || !(uniforms[i] < 1.0)) return -1;
    std::vector<int32_t> pool((size_t)m);
    for (int64_t i = 0; i < m; ++i) pool[(size_t)i] = (int32_t)(i + 2);
    for (int64_t i = 0; i + 1 < R; ++i) {
        const int64_t j = i + (int64_t)std::floor(uniforms[i] * (double)(m - i));
        std::swap(pool[(size_t)i], pool[(size_t)j]);
    }
    steps_out[0] = 1;
    for (int32_t i = 0; i + 1 < R; ++i) steps_out[i + 1] = pool[(size_t)i];
    std::sort(steps_out + 1, steps_out + R);
    return R;
}

pulsecol_status pulsecol_attn_tile_shape(const pulsecol_ctx* ctx, int32_t k, int32_t* block_m, int32_t* block_n) {
    if (!ctx || !block_m || !block_n) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn_tile_shape: NULL pointer");
    if (k < 1 || k > ctx->shape.seq) return fail(nullptr, PULSECOL_ERR_INVALID_ARG, "pulsecol_attn_tile_shape: need 1 <= k <= seq");
    const bool bf = ctx->shape.dtype == PULSECOL_BF16;
    *block_m = sparse_block_m(ctx, k);
    *block_n = !bf ? pulsecol::kBlockN_f32 : (*block_m < pulsecol::kBlockM_bf16 ? 32 : pulsecol::kBlockN_bf16);
    return PULSECOL_OK;
}

const char* pulsecol_status_str(pulsecol_status status) {
    switch (status) {
        case PULSECOL_OK: return "ok";
        case PULSECOL_ERR_INVALID_ARG: return "invalid argument";
        case PULSECOL_ERR_UNSUPPORTED: return "unsupported configuration";
        case PULSECOL_ERR_ALIGNMENT: return "misaligned pointer or stride";
        case PULSECOL_ERR_NO_PATTERN: return "no cached pattern";
        case PULSECOL_ERR_OOM: return "out of device memory";
        case PULSECOL_ERR_HIP: return "HIP runtime error";
        case PULSECOL_ERR_BAD_INDEX: return "column number out of range";
    }
    return "unknown status";
}

const char* pulsecol_last_error(const pulsecol_ctx* ctx) {
    return ctx ? ctx->last_error.c_str() : g_last_error.c_str();
}

}  // extern "C"
