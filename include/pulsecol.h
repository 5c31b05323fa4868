/*
 * pulsecol.h -- C ABI of the MI355X (gfx950) PulseCol attention hot path.
 *
 * PulseCol = periodically refreshed column-sparse bidirectional self-attention for
 * diffusion-LLM denoising steps.  The library holds the two kernels of the method and a
 * dense baseline:
 *   - pattern identification (Sec. 3.3 "Group-wise Column-Sparse Pattern Estimation"):
 *     column scores from the softmax mass of the FULL attention matrix, then top-k;
 *   - column-sparse attention (Sec. 3.4 and the appendix listing "Column-Sparse
 *     Attention Forward"): softmax(Q K_S^T / sqrt(d)) V_S over the selected columns only;
 *   - dense attention softmax(Q K^T / sqrt(d)) V (Sec. 3.1), the baseline being beaten.
 *
 * Conventions common to every call
 *   - Q, K, V, O are DEVICE pointers to [batch, heads, seq, head_dim] tensors (K and V:
 *     [batch, kv_heads, seq, head_dim] in the grouped-query layout) whose last
 *     dimension is contiguous; the other three strides are given in ELEMENTS in
 *     pulsecol_shape (0 = packed).  Base pointers must be 16-byte aligned and the strides
 *     multiples of 8 (bf16) or 4 (fp32) elements.  Attention is non-causal; there is no
 *     padding mask.
 *   - Column sets are DEVICE int32 arrays idx[batch, heads, U, k]; U is the number of query
 *     groups per head (U = 1 when group_size == 0: one column set per head).  Entries lie in
 *     [0, seq) and are unique within a row; pulsecol_select emits them ascending.  (With
 *     variable-length batches, see pulsecol_set_seq_lens, the unused tail of a row is -1.)  The
 *     sparse kernel counts a repeated entry twice, as the appendix listing would.  An entry
 *     outside [0, seq) addresses memory outside K and V: a caller that cannot vouch for its
 *     indices turns the validation mode on (pulsecol_set_validation).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on it: they never synchronise and never read device memory on the host
 *     (the validation mode of pulsecol_attn is the one exception).
 *     The caller owns every buffer it passes; the context owns only the scratch it
 *     allocated at creation (row log-sum-exp, column scores, top-k counters, the cached
 *     pattern).  No call allocates or frees device memory except create/destroy.
 *   - Every function returns a pulsecol_status; nothing aborts or throws, and nothing is
 *     printed unless the environment variable PULSECOL_LOG is set (then every failure goes
 *     to stderr as well).  On failure no kernel has been launched.  pulsecol_last_error gives a text for the last failure on a
 *     context.  Two calls on one context must not overlap in time (they share scratch).
 *   - NaN / Inf in the inputs give unspecified values, never a fault.
 */
#ifndef PULSECOL_H
#define PULSECOL_H

#include <stdint.h>

#if defined(__GNUC__)
#define PULSECOL_API __attribute__((visibility("default")))
#else
#define PULSECOL_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pulsecol_ctx pulsecol_ctx;

typedef enum {
    PULSECOL_OK = 0,
    PULSECOL_ERR_INVALID_ARG = 1, /* null pointer, size < 1, ratio outside (0,1], k outside [1,seq] */
    PULSECOL_ERR_UNSUPPORTED = 2, /* head_dim, dtype or group_size the kernels do not cover       */
    PULSECOL_ERR_ALIGNMENT = 3,   /* base pointer or stride not aligned as stated above           */
    PULSECOL_ERR_NO_PATTERN = 4,  /* refresh == 0 with no cached pattern, or with a different k   */
    PULSECOL_ERR_OOM = 5,         /* scratch allocation failed in pulsecol_create                 */
    PULSECOL_ERR_HIP = 6,         /* a HIP runtime call failed; see pulsecol_last_error           */
    PULSECOL_ERR_BAD_INDEX = 7    /* validation mode: idx holds an entry outside [0, seq)         */
} pulsecol_status;

typedef enum { PULSECOL_BF16 = 0, PULSECOL_F32 = 1 } pulsecol_dtype;

/* Problem shape (host struct, copied by pulsecol_create).
 * Sec. 3.1: per step, layer and head, Q, K, V are n x d_h with n = prompt + generation length. */
typedef struct {
    int32_t batch;      /* >= 1 */
    int32_t heads;      /* >= 1: heads of Q and O (K and V: see kv_heads)                         */
    int32_t seq;        /* n >= 1; bf16: n < 2^24                                                */
    int32_t head_dim;   /* d_h: 64 or 128                                                        */
    int32_t dtype;      /* pulsecol_dtype: storage type of Q, K, V, O.  bf16: bf16 MFMA with fp32 */
                        /* accumulation and fp32 softmax; f32: fp32 throughout.                  */
    int32_t group_size; /* queries per group (Sec. 3.3); 0 or >= seq: the whole head is one group
                         * (U = 1).  Otherwise U = ceil(seq / group_size) groups of consecutive
                         * rows; bf16: a multiple of 32 (multiples of 256 run in the main kernel,
                         * smaller ones -- the paper's 32 / 64 / 128 -- in the small-group kernel),
                         * f32: a multiple of 128; else PULSECOL_ERR_UNSUPPORTED                  */
    int64_t stride_b;   /* element strides of batch, head and sequence; 0 = packed.  Multiples of 16 bytes;
                         * bf16: the sequence stride is below 2^24 bytes and one head spans less than
                         * 4 GiB (seq * stride_n), else PULSECOL_ERR_UNSUPPORTED                  */
    int64_t stride_h;
    int64_t stride_n;
    float scale;        /* logit scale; 0 = 1/sqrt(head_dim) (Sec. 3.1, logits equation)         */
    int32_t kv_heads;   /* heads of K and V; 0 = heads (multi-head attention).  Otherwise grouped-
                         * query attention: heads % kv_heads == 0, K and V are [B, kv_heads, n, d]
                         * and query head h reads K/V head h / (heads / kv_heads).  Patterns stay
                         * per query head.                                                        */
    int64_t kv_stride_b; /* element strides of K and V (0 = packed [B, kv_heads, n, d]; with       */
    int64_t kv_stride_h; /* kv_heads == 0 and all three 0: the strides of Q).  Same alignment and  */
    int64_t kv_stride_n; /* size rules as stride_b/h/n                                             */
    double max_keep_ratio; /* the largest keep_ratio pulsecol_select / pulsecol_refresh_dense will be
                         * called with on this context: sizes the cached pattern (Sec. 3.3: the
                         * pattern is stored between refreshes) at pulsecol_num_keep(seq,
                         * max_keep_ratio) columns per group.  0 = 1.0 (room for every column)     */
} pulsecol_shape;

/* Host-only check of a shape against the rules above.  Touches no device. */
PULSECOL_API pulsecol_status pulsecol_validate_shape(const pulsecol_shape* shape);

/* Create a context on HIP device `device`: copies `shape`, allocates the scratch
 * (4*B*H*seq bytes of row statistics, 4*B*H*U*seq bytes of scores, 4*B*H*U*k_max bytes for the
 * cached pattern with k_max = pulsecol_num_keep(seq, max_keep_ratio), 256 bytes of counters).
 * *out is set only on PULSECOL_OK. */
PULSECOL_API pulsecol_status pulsecol_create(pulsecol_ctx** out, const pulsecol_shape* shape, int device);

/* Validation mode (off by default; on at creation if the environment variable
 * PULSECOL_VALIDATE is set to anything but 0): pulsecol_attn first checks on the device that
 * every entry of idx lies in [0, seq), waits for the answer (it synchronises the stream) and
 * returns PULSECOL_ERR_BAD_INDEX without launching the attention kernel if one does not. */
PULSECOL_API pulsecol_status pulsecol_set_validation(pulsecol_ctx* ctx, int on);

/* Which kernel pulsecol_attn runs when the context has one column set per head (bf16): 256 = the
 * hand-scheduled kernel with 256-row query blocks, 128 = the plain kernel with 128-row blocks,
 * 0 (the default) = whichever a small cost model expects to finish first for the call's k (the plain
 * kernel for short jobs, a few query blocks per compute unit; the scheduled one otherwise).  Results
 * agree within the tolerance of the method either way.  Ignored for group-wise sets and fp32. */
PULSECOL_API pulsecol_status pulsecol_set_attn_block(pulsecol_ctx* ctx, int32_t block_m);

/* Variable-length batches: a padded batch whose elements have their own lengths.  seq_lens is a HOST
 * array of `batch` ints, 1 <= seq_lens[b] <= seq, copied by the call (it rides in the arguments of
 * small launches on `stream`: no host-to-device copy, no synchronisation); NULL returns the context
 * to fixed length.  From then on batch element b consists of rows 0 .. seq_lens[b]-1 of its slabs of
 * Q, K, V, O -- Sec. 3.1's n is the element's own length -- and the rest is padding that no call
 * reads or writes:
 *   - scores:  scores_out[b, h, u, j] is written for j < seq_lens[b] and the groups u that hold a real
 *              row (U_b = ceil(seq_lens[b] / group_size)); everything else is left untouched;
 *   - select / refresh_dense / topk: element b keeps k_b = max(1, floor(keep_ratio * seq_lens[b]))
 *              columns (pulsecol_topk: min(k, seq_lens[b])): idx_out[b, h, u, 0..k_b) ascending, then
 *              -1 up to the row length k = pulsecol_num_keep(seq, keep_ratio); rows of groups beyond
 *              U_b are all -1;
 *   - attn:    of idx[b, ...] the leading non-negative entries count (read off the first column set of
 *              the element; every set of an element holds the same number), rows >= seq_lens[b] of O
 *              are not written; attn_dense likewise attends to the element's own keys only.
 * Drops a cached pattern (it belongs to the lengths it was selected with). */
PULSECOL_API pulsecol_status pulsecol_set_seq_lens(pulsecol_ctx* ctx, const int32_t* seq_lens, void* stream);

/* Free the scratch.  The caller must have synchronised the streams it used.  NULL is OK. */
PULSECOL_API pulsecol_status pulsecol_destroy(pulsecol_ctx* ctx);

/* Number of kept columns per query row, k = max(1, floor(keep_ratio * seq)), keep_ratio =
 * 1 - sparsity (Sec. 3.1, sparsity-budget constraint ||S||_0 <= (1 - rho) n^2).  Host only.
 * Returns -1 when seq < 1 or keep_ratio is outside (0, 1]. */
PULSECOL_API int32_t pulsecol_num_keep(int32_t seq, double keep_ratio);

/* Pattern identification pass (Sec. 3.3, score and TopK equations), run at the
 * identification step and at every refresh step.
 *   refresh != 0: compute the column scores of the CURRENT Q, K from the full softmax
 *                 attention matrix, keep the k = pulsecol_num_keep(seq, keep_ratio) highest
 *                 columns of every group (equal scores: lower column index wins), write them
 *                 ascending to idx_out[B, H, U, k] and cache them in the context.
 *                 PULSECOL_ERR_INVALID_ARG if k exceeds what max_keep_ratio left room for.
 *   refresh == 0: Q and K are ignored (may be NULL); the cached pattern is copied to idx_out.
 *                 PULSECOL_ERR_NO_PATTERN if nothing is cached or k differs. */
PULSECOL_API pulsecol_status pulsecol_select(pulsecol_ctx* ctx, const void* Q, const void* K, double keep_ratio,
                                int refresh, int32_t* idx_out, void* stream);

/* The scoring stage alone (Sec. 3.3, score equation):
 * scores_out[b, h, u, j] = (1/|G_u|) sum_{i in G_u} softmax_j(q_i . k_j * scale), fp32 [B, H, U, seq].
 * Row sums of the softmax are accumulated in fp32 in a fixed order: results are
 * bit-identical from run to run. */
PULSECOL_API pulsecol_status pulsecol_scores(pulsecol_ctx* ctx, const void* Q, const void* K, float* scores_out,
                                void* stream);

/* The selection stage alone (Sec. 3.3, TopK equation) on caller-supplied scores
 * [B, H, U, seq] (fp32, non-negative, device): exact top-k of every row, ties to the lower
 * index, output ascending int32 [B, H, U, k].  Does not touch the cached pattern. */
PULSECOL_API pulsecol_status pulsecol_topk(pulsecol_ctx* ctx, const float* scores, int32_t k, int32_t* idx_out,
                              void* stream);

/* Column-sparse attention forward (Sec. 3.4; appendix listing): for every query row i of
 * group u, O_i = softmax over the k logits {q_i . k_j * scale : j in idx[b,h,u,:]} applied to
 * the same rows of V -- equal to the masked form softmax(Z + M(S)) V of Sec. 3.1.  Online
 * softmax over tiles of gathered K/V rows; nothing of size seq x seq or seq x k is written.
 * 1 <= k <= seq.  O has the layout and dtype of Q. */
PULSECOL_API pulsecol_status pulsecol_attn(pulsecol_ctx* ctx, const void* Q, const void* K, const void* V,
                              const int32_t* idx, int32_t k, void* O, void* stream);

/* Block-sparse attention, the formulation the paper contrasts column sparsity with (Sec. 3.1, block-mask
 * equation S(i, j) = G(b(i), b(j))): query blocks are the context's query groups (the whole head, or
 * group_size rows, a multiple of 256), key blocks are 64 consecutive keys.  block_idx[B, H, U, kb] (device,
 * int32) names the key blocks each query block attends to, unique and in [0, seq / 64); the result is
 * softmax(Z + M(S)) V with that mask.  One kernel with the column-sparse one: a tile is a whole key block,
 * fetched as 64 consecutive rows from one block number instead of 64 gathered rows.  bf16 contexts with
 * seq a multiple of 64 and fixed-length batches, else PULSECOL_ERR_UNSUPPORTED. */
PULSECOL_API pulsecol_status pulsecol_attn_block(pulsecol_ctx* ctx, const void* Q, const void* K, const void* V,
                                    const int32_t* block_idx, int32_t kb, void* O, void* stream);

/* Key blocks kept at a ratio: max(1, floor(keep_ratio * seq / 64)) (the same budget rule on blocks); -1 on
 * seq not a multiple of 64 or a ratio outside (0, 1].  Host only. */
PULSECOL_API int32_t pulsecol_num_keep_blocks(int32_t seq, double keep_ratio);

/* Block selection for pulsecol_attn_block, by the same evidence as the column selection: the mass of a
 * key block is the sum of the column scores (Sec. 3.3, score equation) of its 64 keys, and every query
 * block keeps the kb = pulsecol_num_keep_blocks(seq, keep_ratio) heaviest key blocks (equal masses: lower
 * block number wins), written ascending to block_idx_out[B, H, U, kb].  Nothing is cached. */
PULSECOL_API pulsecol_status pulsecol_select_blocks(pulsecol_ctx* ctx, const void* Q, const void* K, double keep_ratio,
                                       int32_t* block_idx_out, void* stream);

/* Dense attention baseline O = softmax(Q K^T * scale) V (Sec. 3.1).  If lse_out is not NULL
 * it receives the row log-sum-exp of the scaled logits, fp32 [B, H, seq]. */
PULSECOL_API pulsecol_status pulsecol_attn_dense(pulsecol_ctx* ctx, const void* Q, const void* K, const void* V,
                                    void* O, float* lse_out, void* stream);

/* pulsecol_select(refresh != 0) for callers that cannot allocate device memory or hold a context
 * that did: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same computation and same idx_out[B, H, U, k] as pulsecol_select on a context of this shape, on
 * the CURRENT device; nothing is cached (there is no context to cache in).  The row statistics,
 * the scores and the work counters live in a static device array of 16 MiB + 256 bytes that each
 * GPU the library runs on holds until the process ends; its address is looked up at the first call
 * on a device.  Limit: batch * heads * seq * (1 + U) <= 4 * 2^20 fp32 words (exactly the 64K-context,
 * 32-head, one-group-per-head shape), else PULSECOL_ERR_UNSUPPORTED with nothing launched.  The call
 * issues no hipMalloc / hipFree / hipMemset, only kernel launches on `stream`.  All calls on one GPU
 * share that GPU's array (it keeps the last call's contents; nothing in it has to start at zero):
 * two calls that overlap in time on one GPU race, whatever their streams.  With no context, the
 * text of a failure is read with pulsecol_last_error(NULL). */
PULSECOL_API pulsecol_status pulsecol_select_noalloc(const pulsecol_shape* shape, const void* Q, const void* K,
                                        double keep_ratio, int32_t* idx_out, void* stream);

/* Refresh step that keeps the dense output (Sec. 3.3: at an identification or refresh step the
 * method "computes full attention" and collects the attention matrix): O = softmax(Q K^T *
 * scale) V as pulsecol_attn_dense, and idx_out / the cached pattern as
 * pulsecol_select(refresh != 0) on the same Q, K.  The row log-sum-exp comes out of the dense
 * pass itself, so the seq x seq logits are formed three times instead of four.  Same argument
 * rules as the two calls it replaces. */
PULSECOL_API pulsecol_status pulsecol_refresh_dense(pulsecol_ctx* ctx, const void* Q, const void* K, const void* V,
                                       double keep_ratio, void* O, int32_t* idx_out, void* stream);

/* Refresh schedule (Sec. 3.3, schedule equation), host only: T_win = max(1, floor(eta*T));
 * R == 1 -> {1}; else tau_r = 1 + floor((r-1)(T_win-1)/(R-1)).  Writes R 1-based steps to
 * steps_out and returns R, or -1 on T < 1, R < 1, eta outside (0, 1] or a NULL pointer. */
PULSECOL_API int32_t pulsecol_refresh_schedule(int32_t T, double eta, int32_t R, int32_t* steps_out);

/* The two alternative placements of the appendix's ablation on the refresh schedule, same
 * window T_win and budget R, host only, 1-based steps, ascending.
 *   power:  normalised positions (i/(R-1))^2, i = 0..R-1: tau_i = 1 + floor(i^2 (T_win-1) / (R-1)^2)
 *           (refreshes concentrated at the beginning of the window; steps may repeat).
 *   random: R distinct steps of the window: step 1 (a pattern must exist before the first
 *           sparse step) and R-1 steps drawn without replacement from 2..T_win by a partial
 *           Fisher-Yates shuffle that consumes uniforms[0..R-2], each in [0, 1): draw i takes
 *           pool position i + floor(uniforms[i] * (T_win-1 - i)).  The caller owns the random
 *           numbers, so a schedule is reproducible from them.
 * Return R, or -1 on the argument errors of pulsecol_refresh_schedule, a uniform outside
 * [0, 1), or (random) a window with fewer than R steps. */
PULSECOL_API int32_t pulsecol_refresh_schedule_power(int32_t T, double eta, int32_t R, int32_t* steps_out);
PULSECOL_API int32_t pulsecol_refresh_schedule_random(int32_t T, double eta, int32_t R, const double* uniforms,
                                         int32_t* steps_out);

/* Launch geometry of the kernel that pulsecol_attn runs on this context with k kept columns (for
 * reports): query rows per workgroup (B_M) and gathered columns per tile (B_N).  Host only. */
PULSECOL_API pulsecol_status pulsecol_attn_tile_shape(const pulsecol_ctx* ctx, int32_t k, int32_t* block_m, int32_t* block_n);

PULSECOL_API const char* pulsecol_status_str(pulsecol_status status);
PULSECOL_API const char* pulsecol_last_error(const pulsecol_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PULSECOL_H */
