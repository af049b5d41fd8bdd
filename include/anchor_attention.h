/*
 * anchor_attention.h -- C ABI of the MI355X (gfx950) AnchorAttention prefill library.
 *
 * The library implements the three stages of AnchorAttention's sparse causal
 * prefill attention (arXiv 2505.23520, Section 3; Algorithms 1-3) as hand-written
 * HIP kernels, one GPU, plus a dense causal flash kernel used as comparator.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  * Every data pointer is caller-owned DEVICE memory; `params` is a HOST struct;
 *    `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *  * The library never allocates, frees or keeps device memory and never
 *    synchronises the stream: calls only enqueue kernels.  The caller keeps all
 *    buffers alive until the stream has run them.  Calls keep no state between
 *    them: concurrent calls from several host threads are safe as long as they
 *    write to different buffers (and workspaces).
 *  * Return value: 0 on success, a negative AA_E* code otherwise.  All argument
 *    checks run on the host before anything is enqueued, so a failing call has
 *    no effect on the device.  anchor_strerror() names a code.
 *  * Tokens are 0-indexed inside their own sequence.  With b_q = block_q,
 *    query block i = r / b_q, group g = i / step, G_g = g*step*b_q,
 *    W_g = max(n_init, G_g - window):
 *        anchor set   A(r) = { j < n_init, j <= r }  u  { W_g <= j <= r }
 *        candidates   C_g  = [ n_init, W_g )
 *    Scores are S(r,j) = softmax_scale * <q_r, k_j> (Eq. 1), theta is in natural
 *    log units.  Query head h reads KV head h / (Hq/Hkv); every query head runs
 *    the whole method on its own.
 *
 * Layouts
 * -------
 *  q, out: element (b, h, r, c) at  b*stride[0] + h*stride[1] + r*stride[2] + c
 *  k, v  : same with KV heads.  The last dimension (d) is contiguous.  Strides
 *  are in ELEMENTS, multiples of 16 bytes; pointers are 16-byte aligned.  bf16:
 *  one head's K (and V) rows must span less than 2 GiB (N * stride[2] * 2 < 2^31).
 *  dtype AA_BF16: 2-byte bfloat16, AA_FP32: 4-byte float.
 *  Packed variable-length batches (cu_seqlens != NULL): sequence b holds tokens
 *  cu_seqlens[b] .. cu_seqlens[b+1]-1 of a packed token axis; stride[0] is
 *  ignored, r is replaced by cu_seqlens[b] + r, N is the longest sequence and
 *  total_tokens = cu_seqlens[B].  A sequence may be empty (cu_seqlens[b] ==
 *  cu_seqlens[b+1]): it owns no rows, blocks or groups.
 *
 *  Per-row arrays (M, L, lse), float:
 *      fixed length: row (b,h,r) at (b*Hq + h)*N + r
 *      packed      : row (b,h,r) at h*total_tokens + cu_seqlens[b] + r
 *  Acc (float, aa_sizes.acc_elems entries):
 *      AA_FP32: d floats per row, rows indexed as above.
 *      AA_BF16 (d = 128, b_q = 128): one slab of 128*128 floats per query block, slab index as
 *      for the per-block arrays below; a slab holds four tiles of 32 rows, tile w = rows
 *      32w..32w+31 of the block, and inside tile w element (row n, column c) sits at float
 *          w*4096 + ((c/32)*4 + (c%32)/8)*256 + (n + 32*((c%8)/4))*4 + c%4
 *      (the register order of the matrix-core accumulators: stage 1 stores and stage 3
 *      reloads a tile with whole 1 KB bursts).  Rows past the end of a sequence are padding.
 *  Per-block arrays (xa_pooled), float, nblk(b) = ceil(len_b / b_q):
 *      fixed length: (b*Hq + h)*nblk + i
 *      packed      : h*blk_cap + (sum_{b'<b} nblk(b')) + i,  blk_cap from anchor_sizes()
 *  Per-group arrays (counts, offsets), ngrp(b) = ceil(len_b / (b_q*step)):
 *      fixed length: t = (b*Hq + h)*ngrp + g
 *      packed      : t = h*grp_cap + (sum_{b'<b} ngrp(b')) + g, grp_cap from anchor_sizes()
 *  Selected columns: group t owns idx[offsets[t] .. offsets[t] + counts[t]),
 *  strictly ascending key positions inside the sequence.  offsets[t] is a
 *  multiple of 64 and the slots up to the next multiple of 64 after a non-empty
 *  list repeat its last entry, so a reader may always fetch whole 64-entry
 *  chunks (an empty list owns no slots).
 */
#ifndef ANCHOR_ATTENTION_H
#define ANCHOR_ATTENTION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { AA_FP32 = 0, AA_BF16 = 1 };
enum { AA_STRIPE = 0, AA_BLOCK = 1 };   /* identification granularity (b_q, 1) or (b_q, b_kv) */
enum { AA_ENGINE_AUTO = 0, AA_ENGINE_128 = 1, AA_ENGINE_256 = 2 };

enum {
    AA_OK = 0,
    AA_EINVAL = -1,       /* null pointer, non-positive size, Hq % Hkv != 0, bad stride ... */
    AA_EUNSUPPORTED = -2, /* a combination the kernels do not implement (aa_params fields)   */
    AA_EWORKSPACE = -3,   /* workspace smaller than anchor_sizes() reports                  */
    AA_EHIP = -4          /* a kernel launch failed; hipGetLastError text via anchor_last_hip_error */
};

typedef struct aa_params {
    int32_t B, Hq, Hkv;       /* batch (sequences), query heads, KV heads (Hq % Hkv == 0;      */
                              /* B * Hq <= 65535)                                              */
    int32_t N;                /* sequence length; longest sequence when cu_seqlens != NULL     */
    int32_t d;                /* head dimension: bf16 -> 128; fp32 -> 32, 64 or 128             */
    int32_t block_q;          /* b_q : bf16 -> 128; fp32 -> 16..128, multiple of 16             */
    int32_t block_kv;         /* b_kv: tile size of the paper's listings; must equal block_q    */
    int32_t n_init;           /* initial tokens always attended (paper: one KV block), >= 0     */
    int32_t window;           /* window reach before the group start, tokens (paper: b_kv), >= 0*/
    int32_t step;             /* query blocks sharing one list (paper: 16), 1..128              */
    float   theta;            /* threshold, nats; +INFINITY selects all, -INFINITY none         */
    float   softmax_scale;    /* 0 -> 1/sqrt(d)                                                 */
    int32_t causal;           /* must be 1                                                      */
    int32_t dtype;            /* AA_FP32 or AA_BF16 (q, k, v, out)                              */
    int32_t use_anchor;       /* 1; 0 = compare against a zero anchor (Table 4, "without")      */
    int32_t granularity;      /* AA_STRIPE (0): one decision per key column, the method's own;    */
                              /* AA_BLOCK (1): one decision per key block (see stripe_select)    */
    int32_t engine;           /* which bf16 tile engine runs stages 1, 3 and dense attention.    */
                              /* AA_ENGINE_AUTO (0): chosen per launch (by length for dense       */
                              /* attention, on the device by the mean list length for stage 3);   */
                              /* AA_ENGINE_128 / AA_ENGINE_256: the engine with 128 / 256 query   */
                              /* rows per work-group (256 needs dense attention or an even step,  */
                              /* falls back to 128 otherwise).  Results agree to rounding.  A     */
                              /* testing / tuning aid, not part of the method; ignored for fp32.  */
    int64_t q_stride[3], k_stride[3], v_stride[3], o_stride[3]; /* batch, head, token; elements */
    const int32_t *cu_seqlens;/* device int32[B+1] or NULL                                      */
    int64_t total_tokens;     /* cu_seqlens[B]; ignored when cu_seqlens == NULL                 */
} aa_params;

/* Element counts of every buffer a caller has to provide (host-side arithmetic only). */
typedef struct aa_sizes {
    int64_t rows;             /* floats in M, L, lse                                            */
    int64_t acc_elems;        /* floats in Acc (fp32: rows * d; bf16: blocks * b_q * d)         */
    int64_t blk_cap;          /* per-head stride of per-block arrays                            */
    int64_t blocks;           /* floats in xa_pooled (= Hq * blk_cap, times B when fixed length)*/
    int64_t grp_cap;          /* per-head stride of per-group arrays                            */
    int64_t groups;           /* entries in counts; offsets has groups + 1                      */
    int64_t idx_capacity_max; /* idx entries that hold any outcome (every candidate selected)   */
    size_t  select_ws_bytes;  /* workspace of stripe_select                                     */
    size_t  prefill_ws_bytes; /* workspace of anchor_attention_prefill                          */
} aa_sizes;

/*
 * Validates params (AA_EINVAL / AA_EUNSUPPORTED) and fills *out.  Host only.  Buffer
 * arithmetic of this library, not an operation of the paper.  idx_capacity_max holds for
 * every split of total_tokens into B sequences of at most N tokens.
 */
int anchor_sizes(const aa_params *params, aa_sizes *out);

/* *bytes_out = aa_sizes.prefill_ws_bytes, the workspace of anchor_attention_prefill.  Host only. */
int anchor_workspace_bytes(const aa_params *params, size_t *bytes_out);

/*
 * Stage 1, pattern-based anchor computation (Sec. 3.1, Eq. 1; Algorithm 1).
 * For every row r:  M = max_{A(r)} S(r,j),  L = sum_{A(r)} exp(S - M),
 * Acc = sum_{A(r)} exp(S - M) v_j  (Acc may be NULL: not written), and per query
 * block the pooled anchor xa_pooled = mean of M over the block's rows (Alg. 2,
 * avgpool of the anchor).
 */
int anchor_compute(const aa_params *params, const void *q, const void *k, const void *v,
                   float *M, float *L, float *Acc, float *xa_pooled, void *stream);

/*
 * Stage 2, difference-aware stripe identification (Sec. 3.2 mask; Algorithm 2;
 * the step rule of Sec. 3.4).  For every group: column j of C_g is selected iff
 * some block i of the group has  xa_pooled_i - scale*<mean of block i's queries, k_j> <= theta.
 * Writes counts[groups], offsets[groups+1] (int64, see Layouts), and the lists.
 * If the lists (with padding) need more than idx_capacity entries, *overflow_flag
 * is set to 1, nothing is written past the capacity, and offsets stay exact
 * (offsets[groups] is the capacity that would have sufficed); the lists are then
 * incomplete and must not be attended.  Otherwise the flag is set to 0.
 * ws: select_ws_bytes of scratch.
 *
 * granularity = AA_BLOCK switches to the block granularity that Sec. 2.1.2 /
 * Table 1 set against stripes: the same difference test, taken once per key block
 * J (block_kv consecutive keys inside C_g) on the block's average key,
 *   xa_pooled_i - scale*<mean of block i's queries, mean of block J's keys> <= theta,
 * and a selected block contributes all its columns to the list (same list format,
 * so stage 3 is unchanged).  Needs n_init and window to be multiples of block_kv
 * (AA_EINVAL otherwise).
 */
int stripe_select(const aa_params *params, const void *q, const void *k, const float *xa_pooled,
                  int32_t *counts, int64_t *offsets, int32_t *idx, int64_t idx_capacity,
                  int32_t *overflow_flag, void *ws, size_t ws_bytes, void *stream);

/*
 * stripe_select for callers that cannot allocate device memory or bring a workspace (code
 * under HIP graph capture, serving loops, harnesses that forbid hipMalloc): same arguments
 * and results as stripe_select, but its scratch is a device array of
 * AA_NOALLOC_SCRATCH_BYTES that is part of the library (one copy per GPU, held until the
 * process ends) and the call allocates nothing.  AA_EWORKSPACE if the parameters need more
 * than that (aa_sizes.select_ws_bytes; the 128k-token, 32-head, step-16 workload needs
 * 48 MiB).  All calls on one GPU share the array: calls that overlap in time on one GPU
 * (different streams or threads) race; calls ordered on one stream do not.  The first call
 * on a GPU looks the array's address up (hipGetSymbolAddress), so make that call outside a
 * graph capture.
 */
#define AA_NOALLOC_SCRATCH_BYTES (64u << 20)
int stripe_select_noalloc(const aa_params *params, const void *q, const void *k,
                          const float *xa_pooled, int32_t *counts, int64_t *offsets, int32_t *idx,
                          int64_t idx_capacity, int32_t *overflow_flag, void *stream);

/*
 * Stage 3, fine-grained sparse attention (Sec. 3.3, Eq. 3-5; Algorithm 3).
 * Continues the online softmax of every row from (M, L, Acc) over the gathered
 * K/V rows of its group's list, out = acc / l.  If M, L and Acc are all NULL the
 * anchor region is computed inside the kernel instead of being read.  lse
 * (nullable) receives log sum_{P(r)} exp S(r,j).
 * counts / offsets / idx are stripe_select's outputs, idx_capacity the entries idx
 * holds.  The kernels never read idx at or beyond idx_capacity: if the lists do not
 * fit (offsets[groups] > idx_capacity, the case stripe_select flags as overflow)
 * the call writes nothing to out and lse.
 */
int sparse_attn(const aa_params *params, const void *q, const void *k, const void *v,
                const float *M, const float *L, const float *Acc,
                const int32_t *counts, const int64_t *offsets, const int32_t *idx,
                int64_t idx_capacity, void *out, float *lse, void *stream);

/*
 * The whole prefill path of Section 3 (Algorithm 1 -> 2 -> 3, with the step rule of
 * Sec. 3.4): anchor_compute, stripe_select and sparse_attn on one stream, intermediates
 * in ws (prefill_ws_bytes, see anchor_workspace_bytes; its index region holds
 * idx_capacity_max entries, so the lists always fit).  stats (nullable, device int64[4])
 * receives { attended (q,k) pairs, total selected list entries, 0, 0 }.
 */
int anchor_attention_prefill(const aa_params *params, const void *q, const void *k, const void *v,
                             void *out, float *lse, int64_t *stats,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * Exact causal softmax attention with the same tile engine.  Not an operation of the
 * paper's method: the same-GPU comparator the speedup is quoted against, and what the
 * method must reproduce at theta = +inf.
 */
int dense_causal_flash(const aa_params *params, const void *q, const void *k, const void *v,
                       void *out, float *lse, void *stream);

const char *anchor_strerror(int code);
/* Text of the last HIP error this thread's calls ran into ("" if none). */
const char *anchor_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ANCHOR_ATTENTION_H */
