/*
 * dllm_hcsa.h -- C ABI of the Head-Centric Sparse Attention library for AMD MI355X (gfx950).
 *
 * The library implements the attention hot path of a diffusion-LLM denoising step as
 * described in dLLM-Serve, Section 4.5 ("Head-Centric Sparse KV Cache Management") and
 * Section 2.3 ("Two-Phase dLLM Inference Process"):
 *
 *   dllm_hcsa_select           per-head importance scores of every cached position against the
 *                              active block's queries, then a per-head top-k (Section 4.5, Eq. 6
 *                              and the TopK rule stated under it);
 *   dllm_hcsa_attend           bidirectional softmax attention of each sequence's queries over each
 *                              head's own kept rows (Reuse phase, Section 2.3 Eq. 4), with sequences
 *                              flagged dense attending over all their rows in the same call (the
 *                              mixed Refresh + Reuse batch of Section 5.3);
 *   dllm_dense_refresh_attend  dense bidirectional attention, all queries against all keys
 *                              (Refresh phase, Section 2.3 Eq. 3);
 *   dllm_hcsa_pack             gather-copy of each head's kept rows into a dense per-request buffer
 *                              (Section 4.5, the packing done at Refresh time).
 *
 * K and V stay in their dense layout; kept rows are fetched through the index lists at attention time.
 *
 * Conventions that hold for every entry point
 *   Pointers   Members of dllm_batch and the idx / cu_k / seq_mode / o / workspace arguments are
 *              DEVICE pointers owned by the caller.  The dllm_batch struct itself is read on the host.
 *   Layout     Packed variable length, token-major, head_dim contiguous:
 *                q   [total_q , n_q_heads , head_dim]   element strides q_stride_tok , q_stride_head
 *                k,v [total_kv, n_kv_heads, head_dim]   element strides kv_stride_tok, kv_stride_head
 *                o   [total_q , n_q_heads , head_dim]   contiguous, same dtype as q
 *              Sequence b owns query rows cu_q[b]..cu_q[b+1]-1 and KV rows cu_kv[b]..cu_kv[b+1]-1.
 *              Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *              idx is int32 [n_q_heads, total_k]; head h's kept rows of sequence b are
 *              idx[h*total_k + cu_k[b] .. h*total_k + cu_k[b+1]-1], positions LOCAL to the sequence.
 *   Ownership  The library allocates and frees no device memory and keeps no pointer after a call
 *              returns.  Scratch comes from the caller's workspace, sized by the *_workspace query
 *              made with the same arguments; workspace must be 256-byte aligned.
 *   Streams    Work is enqueued on hip_stream (a hipStream_t passed as void*, NULL = default stream).
 *              Calls return without synchronising; nothing is read back to the host, which is why
 *              total_* and max_* are host-side scalars.
 *   Errors     A negative dllm_status is returned and dllm_last_error() describes it.  All argument
 *              checks are made on the host from scalars and pointer nullness; a failed check launches
 *              nothing.  Not checked by the release library (undefined behaviour if violated): cu_*
 *              non-decreasing, starting at 0 and ending at total_*, max_* really bounding the
 *              per-sequence values, 0 <= k_b <= L_b, and idx entries inside [0, L_b).  A library built
 *              with -DDLLM_CHECK_PRECONDITIONS checks all of these on the device before anything
 *              depends on them (see dllm_hcsa_precondition_errors).  NaN inputs are unsupported.
 */
#ifndef DLLM_HCSA_H
#define DLLM_HCSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DLLM_OK = 0,
  DLLM_ERR_INVALID_ARG = -1,  /* null pointer, bad scalar, inconsistent sizes */
  DLLM_ERR_UNSUPPORTED = -2,  /* a valid request this build does not implement */
  DLLM_ERR_WORKSPACE = -3,    /* workspace missing, misaligned or too small */
  DLLM_ERR_DEVICE = -4        /* the HIP runtime refused a launch */
} dllm_status;

typedef enum { DLLM_F32 = 0, DLLM_BF16 = 1 } dllm_dtype;

/* Sequence modes for dllm_hcsa_attend. */
#define DLLM_SEQ_SPARSE 0 /* attend over the rows listed in idx (Reuse) */
#define DLLM_SEQ_DENSE 1  /* attend over every row of the sequence (Refresh) */

typedef struct {
  dllm_dtype dtype;            /* element type of q, k, v and o */
  int32_t batch;               /* number of sequences, >= 1 */
  int32_t n_q_heads;           /* Hq */
  int32_t n_kv_heads;          /* Hkv, divides Hq */
  int32_t head_dim;            /* D: 64 or 128 */
  const void *q, *k, *v;       /* device */
  int64_t q_stride_tok, q_stride_head;   /* in elements; head_dim stride is 1 */
  int64_t kv_stride_tok, kv_stride_head; /* in elements, shared by k and v */
  const int32_t *cu_q;         /* device, [batch+1] */
  const int32_t *cu_kv;        /* device, [batch+1] */
  int32_t total_q, total_kv;   /* cu_q[batch], cu_kv[batch] */
  int32_t max_q, max_kv;       /* upper bounds on per-sequence query count / KV length */
  float softmax_scale;         /* multiplies q.k before the softmax; finite, > 0; 1/sqrt(D) in the paper */
} dllm_batch;

/*
 * Selection (Section 4.5, Eq. 6 with pooling width w, then I^h = TopK(S_h, k)).
 *
 * For every sequence b with k_b = cu_k[b+1]-cu_k[b] > 0, every query head h and every position
 * j < L_b, the score is computed in fp32 in one fixed order so that the kept set is reproducible
 * bit for bit:
 *     qsum[d] = sum over the sequence's query rows (its active block), ascending row, fp32 adds
 *     s[j]    = fma chain over d = 0..D-1 of qsum[d] * K[j, h/G, d], starting from 0
 *     S[j]    = max of s over positions j - pool_w/2 .. j + pool_w/2 clipped to the sequence
 * (the sum over the block ranks positions exactly as the block mean does).  The k_b positions kept
 * are the first k_b under the order "larger S first; equal S: lower position first"; they are
 * written ascending by position into idx_out (layout above).  Sequences with k_b == 0 are skipped.
 *
 * pool_w must be odd and between 1 and 63.  max_k bounds k_b; 1 <= max_k <= max_kv.
 * max_kv may not exceed 32768 (one sequence's scores are ranked by one workgroup, inside one compute unit).
 * Returns DLLM_ERR_WORKSPACE if workspace_bytes < dllm_hcsa_select_workspace(batch, max_k).
 */
size_t dllm_hcsa_select_workspace(const dllm_batch *batch, int32_t max_k);
dllm_status dllm_hcsa_select(const dllm_batch *batch,
                             const int32_t *cu_k, /* device, [batch+1] prefix sums of k_b */
                             int32_t total_k,     /* cu_k[batch] */
                             int32_t max_k,
                             int32_t pool_w,
                             int32_t *idx_out,    /* device, [n_q_heads, total_k] */
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Selection with two options; dllm_hcsa_select is this call with forced_tail = 0 and head_sum = 0.
 *
 * forced_tail = n > 0   Section 2.3 Eq. 4 attends over [K_b; K_cache]: the active block's own keys
 *     and values next to the cache.  With the block stored as the last n positions of every
 *     sequence, those n positions are always kept and never ranked: the k_b - n best of positions
 *     0 .. L_b-n-1 are chosen as above (the pooling window is clipped to these candidates) and the n
 *     block positions close the ascending list.  Requires n <= k_b <= L_b for every sequence with k_b > 0;
 *     n <= max_k is checked on the host, and a sequence that breaks the rest gets no list at all (its
 *     part of idx_out is left as it was; the checked build also reports DLLM_CHECK_FORCED).
 * head_sum = 1          The shared selection of Section 2.4 Eq. 5: the pooled scores are summed over
 *     the query heads (fp32, ascending head, starting from +0), one TopK is taken per sequence under
 *     the same order, and every head's row of idx_out receives that list.
 * Workspace as for dllm_hcsa_select.
 */
dllm_status dllm_hcsa_select_ex(const dllm_batch *batch,
                                const int32_t *cu_k, /* device, [batch+1] */
                                int32_t total_k, int32_t max_k, int32_t pool_w,
                                int32_t forced_tail, int32_t head_sum,
                                int32_t *idx_out,    /* device, [n_q_heads, total_k] */
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Selection runs in one of two forms with identical results.  Two launches: a pass over K writes every
 * fp32 score to the workspace, then one workgroup per list ranks them (any shape).  One launch: one
 * workgroup per (sequence, KV head) walks the head's column of K once, keeps the keys of the head's
 * query heads in registers and ranks them there, so no score travels through HBM; it takes per-head
 * selection (head_sum = 0; any pooling window, with or without a forced block) of lists of up to 8192
 * positions with 1, 2 or 4 query heads per KV head and rows of up to 256 bytes.  By default the
 * library takes the one-launch form when the shape allows it, the (sequence, KV head) pairs fill the
 * compute units in whole rounds or nearly (at least 3/4 of them in a single round, 4/5 of the last of
 * several) and the batch is fairly even (total_kv >= 3/4 * batch * max_kv), where it measures 5 to
 * 30 % faster, and for calls so small (total_kv * n_kv_heads <= 4096) that only launch latency counts.  This call overrides that choice for the whole process (all threads, all later calls);
 * it exists for measurement and for tests that must reach both forms.  Returns the previous setting,
 * or -1 (and changes nothing) for a value that is none of the three.
 */
#define DLLM_SELECT_FORM_AUTO 0
#define DLLM_SELECT_FORM_TWO_LAUNCHES 1
#define DLLM_SELECT_FORM_ONE_LAUNCH 2 /* wherever the shape allows it; other shapes still take two */
int32_t dllm_hcsa_set_select_form(int32_t form);
/*
 * The form a selection call on this batch takes under the current setting: DLLM_SELECT_FORM_ONE_LAUNCH or
 * DLLM_SELECT_FORM_TWO_LAUNCHES; -1 if the batch descriptor is invalid (dllm_last_error says why).  Host
 * only: reads the descriptor, no device memory, launches nothing.  (The compute-unit count is that of the
 * current device, 256 if none can be queried.)
 */
int32_t dllm_hcsa_select_form_of(const dllm_batch *batch, int32_t pool_w, int32_t head_sum);

/*
 * Selection for callers that cannot allocate or hand over device scratch memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result and
 * same argument checks as dllm_hcsa_select_ex, but there is no workspace argument: the fp32 scores
 * (and the row of head sums) live in a buffer of DLLM_SELECT_STATIC_BYTES that is part of the
 * library's device image, one copy per GPU, held until the process ends.  The call allocates and
 * frees nothing (no hipMalloc, no hipFree, no allocating library routine).
 *   Limit     dllm_hcsa_select_workspace(batch, max_k) must not exceed DLLM_SELECT_STATIC_BYTES
 *             (about n_q_heads * total_kv * 4 bytes); larger batches get DLLM_ERR_WORKSPACE and
 *             nothing is launched.
 *   Device    The buffer used is that of the device that is current when the call is made, which
 *             must be the device of hip_stream and of every pointer.  Its address is looked up on
 *             the first call on a device (DLLM_ERR_DEVICE if that fails).
 *   Sharing   Every call on a GPU uses that GPU's one buffer, which keeps the previous call's
 *             contents; the kernels write every score before they read it, so nothing needs
 *             clearing.  Two such calls that overlap in time on one GPU (different streams, or
 *             different host threads on different streams) race and give undefined lists; calls
 *             on one stream are ordered and safe.
 */
#define DLLM_SELECT_STATIC_BYTES (32u << 20)
dllm_status dllm_hcsa_select_static(const dllm_batch *batch,
                                    const int32_t *cu_k, /* device, [batch+1] */
                                    int32_t total_k, int32_t max_k, int32_t pool_w,
                                    int32_t forced_tail, int32_t head_sum,
                                    int32_t *idx_out,    /* device, [n_q_heads, total_k] */
                                    void *hip_stream);

/*
 * Attention over kept rows (Section 2.3 Eq. 4 restricted to each head's kept set; Eq. 3 for
 * sequences flagged dense).  For sequence b, head h, query row i:
 *     O[i,h,:] = sum_t softmax_t(softmax_scale * Q[i,h,:].K[r_t, h/G, :]) * V[r_t, h/G, :]
 * where r_t runs over idx[h, cu_k[b] .. cu_k[b+1]) if seq_mode[b] == DLLM_SEQ_SPARSE and over
 * 0 .. L_b-1 if seq_mode[b] == DLLM_SEQ_DENSE.  No mask, no positional term.  idx need not be
 * sorted and may repeat a row (it then counts twice).  A sequence with nothing to attend to
 * (k_b == 0 sparse, or L_b == 0 dense) gets zeros.  Scores, softmax state and accumulators are
 * fp32; bf16 inputs are multiplied on the matrix cores, fp32 inputs with fp32 arithmetic.
 *
 * seq_mode may be NULL (all sparse).  cu_k may be NULL only if total_k == 0; every sequence not flagged
 * dense then counts as keeping nothing and gets zeros.  idx == NULL with
 * total_k > 0 means the identity lists: sparse sequence b attends over its rows 0 .. k_b-1 in order
 * (k_b from cu_k), which is how a packed cache written by dllm_hcsa_pack is read.
 * max_k bounds k_b over sparse sequences (0 allowed when there are none).
 */
size_t dllm_hcsa_attend_workspace(const dllm_batch *batch, int32_t max_k);
dllm_status dllm_hcsa_attend(const dllm_batch *batch,
                             const int32_t *idx,  /* device, [n_q_heads, total_k] */
                             const int32_t *cu_k, /* device, [batch+1] */
                             int32_t total_k, int32_t max_k,
                             const uint8_t *seq_mode, /* device, [batch] or NULL */
                             void *o,             /* device, [total_q, n_q_heads, head_dim] */
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Pack (Section 4.5, "Decoupling Logical Sparsity from Physical Layout"): copies every head's kept
 * rows, in list order, out of the dense K and V into two buffers of shape
 * [n_q_heads, total_k, head_dim] (same element type), so that a later Reuse step reads them
 * sequentially and needs no index list:
 *     k_packed[h, cu_k[b] + t, :] = K[cu_kv[b] + idx[h, cu_k[b] + t], h / G, :]      (same for V)
 * The packed buffers are themselves a valid K/V operand of this library: describe them in a
 * dllm_batch with n_kv_heads = n_q_heads, kv_stride_tok = head_dim, kv_stride_head =
 * total_k * head_dim, cu_kv = cu_k, total_kv = total_k, max_kv = max_k, and call dllm_hcsa_attend
 * with idx = NULL (see there): that is the paper's Reuse phase over the packed cache.
 * Needs no workspace.  idx, cu_k, k_packed and v_packed are device pointers; k_packed and v_packed
 * must be 16-byte aligned and must not overlap K or V.
 */
dllm_status dllm_hcsa_pack(const dllm_batch *batch,
                           const int32_t *idx,  /* device, [n_q_heads, total_k] */
                           const int32_t *cu_k, /* device, [batch+1] */
                           int32_t total_k, int32_t max_k,
                           void *k_packed,      /* device, [n_q_heads, total_k, head_dim] */
                           void *v_packed,      /* device, [n_q_heads, total_k, head_dim] */
                           void *hip_stream);

/*
 * Dense bidirectional attention of every sequence's queries over all of its keys
 * (Section 2.3 Eq. 3): O = Softmax(softmax_scale * Q K^T) V per (sequence, head), no mask.
 * Same result as dllm_hcsa_attend with every sequence flagged dense.
 */
size_t dllm_dense_refresh_attend_workspace(const dllm_batch *batch);
dllm_status dllm_dense_refresh_attend(const dllm_batch *batch,
                                      void *o, /* device, [total_q, n_q_heads, head_dim] */
                                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Device-side precondition checks (debug aid).  In a library built with -DDLLM_CHECK_PRECONDITIONS
 * every entry point above first verifies, on the device, the conditions the release library leaves to
 * the caller, and sets bits in one error word per GPU; when a bit is set, every kernel of the call, and
 * of later calls, returns without reading or writing anything, so a violating input cannot fault.  This
 * function waits for hip_stream, stores the word in *errors_out (host memory) and clears it.  In the
 * release library nothing is checked: it stores 0 and returns DLLM_ERR_UNSUPPORTED.
 */
#define DLLM_CHECK_CU_Q 1u      /* cu_q: not starting at 0, decreasing, a sequence above max_q, or not ending at total_q */
#define DLLM_CHECK_CU_KV 2u     /* the same for cu_kv, max_kv, total_kv */
#define DLLM_CHECK_CU_K 4u      /* the same for cu_k, max_k, total_k */
#define DLLM_CHECK_K_OVER_L 8u  /* a sparse sequence keeps more rows than it has */
#define DLLM_CHECK_FORCED 16u   /* a sequence with kept rows keeps, or has, fewer than forced_tail rows */
#define DLLM_CHECK_IDX 32u      /* an index outside [0, L_b) in a sparse sequence's list */
dllm_status dllm_hcsa_precondition_errors(void *hip_stream, uint32_t *errors_out /* host */);

/* Text of the calling thread's most recent error ("" if none); static storage, never NULL. */
const char *dllm_last_error(void);

/* Library version as major*10000 + minor*100 + patch. */
int32_t dllm_hcsa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DLLM_HCSA_H */
