/*
 * tree_attn.h -- C ABI of the MI355X (gfx950) decode-attention library.
 *
 * Exact single-token ("decode") attention over a long KV cache, computed the
 * way Tree Attention (arXiv 2408.04093) lays it out: the sequence axis is cut
 * into P chunks, every chunk yields partial softmax statistics (m, l, o), and
 * the partials are merged with the associative max/logsumexp reduction of
 * Section 5.1.  In the paper the chunks live on different GPUs and the merge
 * is three all-reduces (Algorithm 3); here the chunks are workgroups of one
 * GPU and the merge is a kernel.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer unless it says "host".  The
 *     ta_problem struct itself is read on the host.
 *   - The caller owns all buffers.  The library never allocates, frees,
 *     copies to the host or synchronises: work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and the call
 *     returns at once.  Buffers must stay alive until that work has finished.
 *   - Errors are return codes.  All argument checks run on the host before
 *     anything is launched; a failed check launches nothing.
 *   - Scores are s_a = scale * (q . k_a).  scale = 1 is the paper's softmax
 *     (Section 3); the paper has no scale.
 *   - Grouped queries: g = Hq / Hkv, query head h reads KV head h / g (integer
 *     division).  The paper treats heads as independent (Appendix C.1); the
 *     grouping only changes which K/V a head reads.  With bf16 inputs up to 64
 *     heads of a group are processed by the same workgroup so that K/V bytes
 *     are fetched once per group (fp32 inputs: up to 4 heads per pass).
 *   - Keys at positions >= valid_len[b] do not exist and are never read.
 *   - lse is the natural-log logsumexp of the scaled scores over the valid
 *     keys, i.e. the energy F(0) of Observation 1; out is dF/dzeta at 0.
 *     A sequence with no valid key gives out = 0 and lse = -inf (never NaN).
 *   - Partials (Algorithm 3, step 2, kept unnormalised):
 *        m = max_a s_a,  l = sum_a exp(s_a - m),  o = sum_a exp(s_a - m) v_a
 *     over the keys of one chunk, all fp32:  part_m, part_l [B,Hq,P] and
 *     part_o [B,Hq,P,d], contiguous.  The paper's per-device (o, lse) are
 *     o / l and m + log l.  An empty chunk stores (-inf, 0, 0).
 *   - NaN or Inf in q, K or V: behaviour undefined.  Sums are kept in fp32 with
 *     weights of up to 2^8 while a chunk is streamed, so N * max|V| must stay
 *     below ~1e35.
 *   - Several query tokens (Sq > 1; speculative decoding, the tail of a chunked
 *     prefill): the paper's causal energy F_tot = sum_i log sum_{a <= i} exp(..)
 *     (Appendix C.1) restricted to the last Sq positions.  The cache of
 *     sequence b already holds the Sq new tokens' keys and values as its last
 *     Sq valid positions; query token t (0-based) attends to keys
 *     0 .. valid_len[b] - Sq + t.  A token that sees no key gets out = 0,
 *     lse = -inf.  Shapes gain a token axis: q and out [B,Sq,Hq,d],
 *     lse [B,Sq,Hq], partials [B,Sq,Hq,P] and [B,Sq,Hq,P,d]; for
 *     ta_tree_combine pass Sq*Hq as Hq.  All tokens and heads of a KV group
 *     share one pass over K/V as long as Sq * (Hq/Hkv) <= 64; beyond that the
 *     (token, head) pairs of the group, taken token-major, are processed in
 *     slices of 64, each slice reading K/V once (bf16 inputs; fp32 inputs take
 *     the pairs in slices of up to 4).
 */
#ifndef TREE_ATTN_H
#define TREE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TA_OK = 0,
    TA_ERR_NULL = 1,        /* a required pointer is NULL                            */
    TA_ERR_SHAPE = 2,       /* B, Hq, Hkv, d, N, P or a stride is out of range       */
    TA_ERR_DTYPE = 3,       /* unknown ta_dtype                                      */
    TA_ERR_ALIGN = 4,       /* a pointer or a row stride is not 16-byte aligned      */
    TA_ERR_WORKSPACE = 5,   /* workspace smaller than ta_workspace_bytes()           */
    TA_ERR_UNSUPPORTED = 6, /* valid in principle, not built (e.g. d not in {64,128})*/
    TA_ERR_HIP = 7          /* the HIP runtime refused the launch                    */
} ta_status;

typedef enum { TA_BF16 = 0, TA_F32 = 1 } ta_dtype;

/*
 * One decode-attention problem.  Read on the host only.
 *   q   [B,Hq,d]       contiguous  ([B,Sq,Hq,d] when Sq > 1)
 *   K,V [B,Hkv,N,d]    innermost stride 1; the other strides are given in
 *                      ELEMENTS and must keep every row 16-byte aligned
 *                      (stride_n >= d).  A head slice may exceed 4 GiB; what must
 *                      span less than 4 GiB is one CHUNK (row offsets inside a
 *                      chunk are 32-bit): ta_suggest_chunks takes care of it,
 *                      ta_decode_partial refuses a P that is too small, and with
 *                      an explicit chunk table the whole slice must stay below
 *                      4 GiB (TA_ERR_UNSUPPORTED otherwise).
 *   d in {64, 128};  Hq % Hkv == 0 (any group size Hq / Hkv, multi-query included).
 * bf16 inputs: scores and all sums are accumulated in fp32.
 * fp32 inputs: scores and the running max are accumulated in fp64, the
 *              exponentials and sums in fp32.
 */
typedef struct ta_problem {
    int32_t B, Hq, Hkv, d;
    int64_t N;                                   /* key capacity of K and V            */
    int64_t k_stride_b, k_stride_h, k_stride_n;  /* elements                           */
    int64_t v_stride_b, v_stride_h, v_stride_n;  /* elements                           */
    int32_t qkv_dtype;                           /* ta_dtype shared by q, K and V      */
    int32_t out_dtype;                           /* ta_dtype of `out` (ta_decode only) */
    float scale;                                 /* finite; multiplies q . k           */
    const int32_t *valid_len;                    /* device int32 [B], or NULL = N      */
    int32_t Sq;                                  /* query tokens per sequence; 0 or 1 =
                                                    plain decode (see "Several query
                                                    tokens" above)                     */
} ta_problem;

/* Human-readable name of a status code; never NULL; static storage. */
const char *ta_status_string(ta_status s);

/*
 * Chunk count P that ta_decode uses for this problem on the current device.
 * Host-only heuristic: with equal work per chunk, one workgroup per compute
 * unit (P = CUs / (B * Hkv), more rounds only beyond 32768 keys per chunk);
 * with more (batch, kv head) groups than compute units, the fewest chunks per
 * sequence that fill the last round of workgroups, usually 1; for ragged
 * batches beyond the reach of the balanced launch, chunks of a few thousand
 * keys; never shorter than 256 keys.  Returns 0 if the problem is invalid.
 */
int32_t ta_suggest_chunks(const ta_problem *p);

/*
 * Bytes of workspace ta_decode needs when it runs with P chunks:
 * B*Sq*Hq*P*(d+2) floats, rounded up to 256 bytes.  Returns 0 if the problem
 * is invalid or P < 1.
 */
size_t ta_workspace_bytes(const ta_problem *p, int32_t P);

/*
 * Algorithm 3, steps 1-2: split the keys of every sequence into P chunks and
 * reduce each chunk to its partial (m, l, o) for every query head.
 *   chunk_bounds  device int64 [P+1], non-decreasing, shared by every (b, h);
 *                 chunk j holds keys [bounds[j], bounds[j+1]) intersected with
 *                 [0, valid_len[b]).  Values are clamped on the device, so a
 *                 bad table can give wrong chunks but no out-of-range access.
 *                 NULL = P equal chunks of t = ceil(N / P) keys (the paper's
 *                 t = N / p), chunk j = [j t, (j+1) t).
 *   part_m/l/o    outputs, layout above.  Fully overwritten.
 * One launch; every K and V row of a valid chunk is read exactly once.
 */
ta_status ta_decode_partial(const ta_problem *p, const void *q, const void *K, const void *V,
                            int32_t P, const int64_t *chunk_bounds,
                            float *part_m, float *part_l, float *part_o, void *stream);

/*
 * Algorithm 3, steps 3-6 (the arithmetic of the three all-reduces and the
 * final division), as one P-ary reduction per (b, h) -- Appendix B allows any
 * fan-in:
 *     m* = max_j m_j,  w_j = exp(m_j - m*),
 *     l* = sum_j w_j l_j,  o* = sum_j w_j o_j,
 *     out = o* / l*,   lse = m* + log l*.
 * Partials with l_j = 0 are ignored; if all are, out = 0 and lse = -inf.
 *   part_*   inputs, layout above (d in {64,128}, P >= 1)
 *   out      [B,Hq,d] of out_dtype (bf16 is rounded to nearest even)
 *   lse      fp32 [B,Hq]
 */
ta_status ta_tree_combine(int32_t B, int32_t Hq, int32_t d, int32_t P,
                          const float *part_m, const float *part_l, const float *part_o,
                          void *out, int32_t out_dtype, float *lse, void *stream);

/*
 * The whole path: ta_decode_partial with P = ta_suggest_chunks(p) equal
 * chunks into `workspace`, then ta_tree_combine.  When P = 1 (short contexts
 * in a large batch) the single chunk is the result: the streaming kernel
 * normalises and stores out / lse itself and no second kernel is launched.
 * When valid_len is given (a ragged batch, B <= 2048) the chunks are not
 * fixed-size: all valid keys of the batch are cut into equal-cost shares on
 * the device, one per workgroup the GPU holds at a time, whatever the mix of
 * lengths, and the combine merges each row's pieces.  The result is the same attention output;
 * only the (private) workspace layout differs.
 *   workspace        device scratch, 256-byte aligned, at least
 *                    ta_workspace_bytes(p, ta_suggest_chunks(p)) bytes;
 *                    contents undefined before and after.
 *   out [B,Hq,d] (p->out_dtype), lse fp32 [B,Hq].
 */
ta_status ta_decode(const ta_problem *p, const void *q, const void *K, const void *V,
                    void *workspace, size_t workspace_bytes,
                    void *out, float *lse, void *stream);

/*
 * ta_decode for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, checks, kernels and results as
 * ta_decode, but the workspace is a fixed 16 MiB array in device memory that
 * the library's code object brings along (one copy per GPU, held until the
 * process ends); this call allocates and frees nothing.
 *   - A problem whose workspace would exceed 16 MiB
 *     (ta_workspace_bytes(p, ta_suggest_chunks(p)) > 16 << 20) is refused with
 *     TA_ERR_WORKSPACE before anything is launched.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in
 *     time (different streams, different threads) race on it.  Calls on one
 *     stream are ordered and safe; nothing in the array has to be cleared
 *     between calls (every value a kernel reads was written by the same call).
 *   - The array's device address is looked up on the first call on each
 *     device (with the caller's current device); make that first call outside
 *     graph capture.  TA_ERR_HIP if the lookup fails.
 */
ta_status ta_decode_noalloc(const ta_problem *p, const void *q, const void *K, const void *V,
                            void *out, float *lse, void *stream);

/*
 * The energy alone: lse[b,(t,)h] = F(0) = logsumexp_a(scale q.k_a), Algorithm 1
 * (the energy forward pass for one query) with its max and logsumexp
 * reductions fused into one (m, l) reduction.  zeta is zero and never materialised, so V is not
 * an argument and only K is streamed: half the bytes of ta_decode.  Ragged
 * batches take the same equal-cost shares as in ta_decode.
 *   workspace   as for ta_decode (same size and alignment)
 *   lse         fp32 [B,Hq] ([B,Sq,Hq])
 */
ta_status ta_energy(const ta_problem *p, const void *q, const void *K,
                    void *workspace, size_t workspace_bytes, float *lse, void *stream);

/*
 * The paper's two-pass route to the same result as ta_decode: Algorithm 1
 * (ta_energy: lse) followed by Algorithm 2, the gradient with respect to zeta
 * taken by hand:  out = Reduce(sum) over chunks of sum_a exp(s_a - lse) v_a.
 * With lse known no running max and no normaliser are needed and the chunk
 * partials add up plainly.  K is streamed twice (1.5 x the bytes of ta_decode);
 * it exists as an on-GPU cross-check of Observation 1 and for callers that
 * already hold lse.  Arguments as for ta_decode.  A ragged batch takes the
 * equal-cost shares of ta_decode in both passes.
 */
ta_status ta_decode_two_pass(const ta_problem *p, const void *q, const void *K, const void *V,
                             void *workspace, size_t workspace_bytes,
                             void *out, float *lse, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TREE_ATTN_H */
