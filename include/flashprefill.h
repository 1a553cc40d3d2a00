/*
 * flashprefill.h - C ABI of the MI355X (gfx950) FlashPrefill prefill-attention library.
 *
 * One causal GQA attention layer, computed as the paper's three stages
 * (Appendix B, "Detailed Implementation"):
 *   (i)   fp_block_search    pattern discovery          Sec. 3.1-3.2, Eq. 1-4, Alg. 1
 *   (ii)  fp_threshold       max-based dynamic threshold + index compression
 *                                                        Sec. 3.4, Alg. 2, Appendix A
 *   (iii) fp_sparse_prefill  index-driven block-sparse attention   Sec. 3.5, Alg. 3
 *         fp_dense_prefill   full causal attention, the comparison the paper's
 *                            speedups are quoted against (Experiments, "Baselines")
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the library never
 *     frees or reallocates it.  `cu_seqlens` inside fp_shape is a HOST pointer, read only
 *     during fp_layout / fp_plan_create.
 *   - Q and O are [T, Hq, d], K and V are [Tk, Hkv, d] (d = head_dim), bf16, contiguous, token-major;
 *     T = cu_seqlens[nseq], Tk = cu_seqlens_k[nseq].  Sequence s owns query tokens
 *     cu_seqlens[s] .. cu_seqlens[s+1]-1 and key tokens cu_seqlens_k[s] .. cu_seqlens_k[s+1]-1.
 *     Query head h reads KV head h / (Hq / Hkv).
 *   - Plain prefill: cu_seqlens_k == NULL, keys and queries are the same tokens.  Chunked
 *     prefill (the queries are the last q_len tokens of a sequence whose first kv_len - q_len
 *     keys were produced earlier): query i of the chunk sits at position prefix + i and sees
 *     keys 0 .. prefix + i; prefix = kv_len - q_len must be a multiple of `block`.
 *   - Blocks of `block` tokens (128 in the paper) are aligned to the start of each sequence; a sequence
 *     of kv_len keys has ceil(kv_len / block) key blocks, the last one possibly partial.
 *     Query-block row r = row_offset[s] + I addresses q-block I of sequence s's chunk, which
 *     is block I + prefix / block of the sequence: wherever a comment below says "J <= I",
 *     I is that index within the sequence.  m_total = total rows, n_max = most key blocks
 *     in any one sequence.
 *   - scores: fp32 [Hq, m_total, n_max]; idx: int32 [Hq, m_total, n_max]; cnt: int32
 *     [Hq, m_total]; lse: fp32 [Hq, T].  Head-major so that one row is contiguous (the
 *     paper's Alg. 2 indexes [batch, q-block, k-block, head]).
 *   - Compute calls only enqueue kernels on `hip_stream` (a hipStream_t, NULL = default
 *     stream): they do not allocate, synchronise or touch host memory.  Calls on one plan
 *     must be stream-ordered with respect to each other (they share the plan's workspace).
 *   - Errors are return codes.  Argument checks happen on the host before any launch.
 *     A launch failure is reported as FP_ERR_DEVICE.  NaN/Inf inputs are not checked.
 *   - Device memory: the caller's tensors plus one buffer per plan, either allocated by
 *     fp_plan_create or brought by the caller (fp_workspace_bytes + fp_plan_create_in).
 */
#ifndef FLASHPREFILL_H
#define FLASHPREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FP_OK = 0,
    FP_ERR_INVALID_ARG = 1, /* null pointer, inconsistent shape, bad cu_seqlens            */
    FP_ERR_UNSUPPORTED = 2, /* (head_dim, block) not one of (64|128|256, 128), (128, 64|256); over 4096 blocks/seq; or a */
                            /* KV prefix that is not a multiple of the block                */
    FP_ERR_DEVICE = 3,      /* HIP runtime error (no device, allocation or launch failure) */
    FP_ERR_NOMEM = 4,       /* host allocation failed                                      */
    FP_ERR_WORKSPACE = 5,   /* caller-supplied workspace too small or not 256-byte aligned */
    FP_ERR_STATIC_LIMIT = 6 /* fp_block_search_static: shape beyond the built-in scratch    */
} fp_status;

/* Size of the library's built-in scratch array (one copy per GPU, held until the process ends). */
#define FP_STATIC_SCRATCH_BYTES ((8u << 20) + (128u << 10))

typedef struct {
    int32_t nseq;              /* sequences in the packed batch, >= 1                         */
    const int32_t *cu_seqlens; /* HOST, nseq+1 entries, [0] = 0, strictly increasing          */
    int32_t hq, hkv;           /* query heads, KV heads; hq % hkv == 0                        */
    int32_t head_dim;          /* 64, 128 or 256                                              */
    int32_t block;             /* 128 (Appendix A: uniform block size); 64 and 256 at head_dim 128 */
    float scale;               /* softmax scale tau; <= 0 selects 1/sqrt(head_dim)            */
    const int32_t *cu_seqlens_k; /* HOST, nseq+1 entries, or NULL (= cu_seqlens): key-side      */
                               /* lengths for chunked prefill, kv_len >= q_len per sequence   */
} fp_shape;

typedef struct {
    float alpha;           /* threshold factor (Appendix A: 0.12 / 0.18 / 0.08 per model); <= 0 keeps all */
    int32_t sink_tokens;   /* attention-sink size in tokens (Appendix A: 256); rounded up to blocks      */
    int32_t window_tokens; /* local-window size in tokens (Appendix A: 512); rounded up to blocks,       */
                           /* the window includes the diagonal block                                     */
} fp_params;

/* Opaque: the shape's row tables on the device + the pooled-key workspace.  A plan per shape takes
 * the place of a context object with a fixed workspace: the tables (row records, heavy-first order)
 * depend on cu_seqlens, are built once on the host and are read by every kernel, so they live and
 * die with the shape they describe. */
typedef struct fp_plan fp_plan;

const char *fp_status_string(fp_status s);

/* Host only.  Validates `shape` and reports the row bookkeeping.  Any output pointer may be
 * NULL; row_offset receives nseq+1 entries.  No GPU is touched. */
fp_status fp_layout(const fp_shape *shape, int32_t *m_total, int32_t *n_max, int32_t *row_offset);

/* Bytes of device memory a plan for `shape` needs (row tables + the pooled keys of Alg. 1 stage 1:
 * 2 x (key blocks) x Hkv x head_dim bf16 plus two norms per pooled key); 0 if the shape is invalid or unsupported.  Host only. */
size_t fp_workspace_bytes(const fp_shape *shape);

/* Validates `shape`, selects `device`, allocates one device buffer of fp_workspace_bytes(shape)
 * and fills the plan's tables in it.  Synchronous.  The plan is immutable afterwards and may be
 * used for any number of calls; destroy it with fp_plan_destroy after the work enqueued with it
 * has finished. */
fp_status fp_plan_create(const fp_shape *shape, int device, fp_plan **plan);

/* The same with the device memory brought by the caller: `workspace` is a DEVICE pointer on
 * `device`, 256-byte aligned, of at least fp_workspace_bytes(shape) bytes (FP_ERR_WORKSPACE
 * otherwise, checked before the GPU is touched); it stays the caller's, must outlive the plan and
 * must not be used for anything else meanwhile.  No device allocation happens in this call
 * (the tables are copied in synchronously); workspace == NULL behaves as fp_plan_create. */
fp_status fp_plan_create_in(const fp_shape *shape, int device, void *workspace, size_t workspace_bytes,
                            fp_plan **plan);

/* Frees the plan and, if the library allocated it, its device buffer.  NULL is a no-op. */
void fp_plan_destroy(fp_plan *plan);

/*
 * Stage (i).  Alg. 1: mean-pool each key block (stage 1), for every causal block pair
 * (I, J <= I) reduce the query tile's logits against the pooled key to a max m_IJ and a sum
 * of exponentials S_IJ (stage 2, Eq. 1-2), bring each row to its max and normalise (stage 3,
 * Eq. 3-4):  scores[h, r, J] = S'_IJ / (sum_K S'_IK + eps) for J <= I, and 0 for I < J < N_s, the
 * number of key blocks of the row's own sequence; entries N_s <= J < n_max (a shorter sequence of
 * a packed batch) are not written.  `eps` is an argument, not a field of fp_params: it belongs to
 * Eq. 4, while fp_params holds the hyper-parameters of Alg. 2.
 * The pair-level causal restriction J <= I is the only mask; a partial last block averages its
 * valid keys and leaves out missing queries.
 */
fp_status fp_block_search(fp_plan *plan, const void *Q, const void *K, float eps, float *scores, void *hip_stream);

/*
 * fp_block_search for callers that cannot allocate device memory or hand a workspace over: code
 * under HIP graph capture, tight serving loops that share one scratch area among many plans,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as
 * fp_block_search; the pooled keys of Alg. 1 stage 1 go to a fixed array inside the library
 * (FP_STATIC_SCRATCH_BYTES per GPU) instead of the plan's buffer, so `plan` may be one whose
 * workspace is in use elsewhere.  Limit: (key blocks of the batch) x Hkv x (2 planes x 2 head_dim
 * bytes + 8 B of norms) must fit, i.e. key blocks x Hkv <= 16384 at head_dim 128 (256K tokens at
 * Hkv = 8, 512K at Hkv = 4; half as many at head_dim 256); beyond it the call returns
 * FP_ERR_STATIC_LIMIT and launches nothing.  The call allocates nothing and frees
 * nothing.  All calls on one GPU share that GPU's array: it needs no clearing (every entry a
 * call reads it has written first), but two calls that may overlap in time on one GPU (different
 * streams, or graphs replayed concurrently) race and must be ordered by the caller.
 */
fp_status fp_block_search_static(fp_plan *plan, const void *Q, const void *K, float eps, float *scores,
                                 void *hip_stream);

/*
 * Stage (ii).  Alg. 2: per (head, q-block row): thresh = alpha * max_{J<=I} scores (Sec. 3.4),
 * keep J iff (scores >= thresh or J < sink blocks or 0 <= I-J < window blocks) and J <= I;
 * idx[h, r, 0..cnt[h, r]) holds the kept J in ascending order.  Entries of idx past cnt are
 * not written (the paper pads them with the block count and sorts; the compaction here yields
 * the same prefix without a sort).  `scores` entries with J > I do not affect the result.
 */
fp_status fp_threshold(fp_plan *plan, const float *scores, const fp_params *params, int32_t *idx, int32_t *cnt,
                       void *hip_stream);

/*
 * Stages (i) + (ii) in one pass: the lists fp_threshold would emit from fp_block_search's scores,
 * without the scores ever reaching memory (Alg. 1 stage 3 feeding Alg. 2; the paper's Appendix B
 * keeps the two apart, this entry point is the shortcut its Sec. 3.4 decision rule allows because
 * the rule only looks at one row at a time).  Rows of up to 128 key blocks, ragged q-blocks and
 * alpha <= 0 are computed exactly as the two calls compute them and give identical idx and cnt.
 * Longer rows are scored with half the matrix work (one bf16 plane of the pooled key, which
 * bounds each pair's error), and every pair on which a decision could hinge, that is every pair
 * that may hold the row maximum or whose error interval meets the threshold, is then re-scored
 * exactly; all other pairs are decided with a margin.  The lists are therefore those of exact
 * scores, and can differ from the two-call lists only where a normalised score lies within a few
 * units in the last place of alpha * max (fp32 rounding of the two normalisations).
 * Arguments as in the two calls.
 */
fp_status fp_search_select(fp_plan *plan, const void *Q, const void *K, float eps, const fp_params *params,
                           int32_t *idx, int32_t *cnt, void *hip_stream);

/*
 * Stage (iii).  Alg. 3: for each (head, q-block row) visit only the listed key blocks, online
 * softmax in base 2, causal mask on the diagonal block only; O = acc / l, lse = m + log2 l
 * (base-2 log-sum-exp of tau*log2(e)*q.k over the visited, non-future keys).  `lse` may be
 * NULL.  Lists must be ascending and causal (as fp_threshold emits them); out-of-range entries
 * are clamped into [0, I] rather than dereferenced.  A row with cnt == 0 yields O = 0.
 */
fp_status fp_sparse_prefill(fp_plan *plan, const void *Q, const void *K, const void *V, const int32_t *idx,
                            const int32_t *cnt, void *O, float *lse, void *hip_stream);

/* Full causal attention with the same kernel family (every block J <= I visited). */
fp_status fp_dense_prefill(fp_plan *plan, const void *Q, const void *K, const void *V, void *O, float *lse,
                           void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FLASHPREFILL_H */
