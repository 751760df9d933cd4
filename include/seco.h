/*
 * seco.h - C ABI of the chunk-wise attention library for AMD MI355X (gfx950).
 *
 * The library implements the attention-layer hot path of Sequential / Sparse
 * Chunk-wise Optimization (SeCO, Alg. 1; SpaCO, Alg. 2 of the paper):
 *
 *   - a sequence is processed in chunks; chunk j's queries see the K/V cache
 *     rows of every earlier chunk plus a causal block over the chunk itself
 *     (Eq. 1 at the attention layer);
 *   - the backward of a chunk returns dQ for that chunk and ADDS its dK/dV
 *     into a persistent fp32 gradient buffer that spans the whole cache (the
 *     ".grad" of the paper's checkpoints m'_i, Alg. 1 second loop);
 *   - SpaCO back-propagates only selected chunks and scales what a call
 *     deposits on earlier selected chunks by the compensation factor k/t
 *     (Sec. 5 "Compensation Factor", Alg. 2).
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers unless a name ends in _host.
 *   - Layout: [batch, head, row, head_dim]; head_dim is contiguous; the three
 *     outer strides are given explicitly, in ELEMENTS.  Every row must start on
 *     a 16-byte boundary (base pointer and strides); a row stride may not exceed 2^22 elements
 *     (SECO_ERR_TOO_LARGE).
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - The caller owns every buffer and the stream.  Entry points validate,
 *     enqueue kernels on `hip_stream` (a hipStream_t, may be NULL for the
 *     default stream) and return without synchronising.  They allocate no
 *     device memory and keep no state between calls (the optional profiler
 *     at the end of this header aside).
 *   - Return value: SECO_OK (0) or a negative seco_status.  On a validation
 *     error nothing is enqueued and no output is touched.
 *   - Results are deterministic: no floating-point atomics are used anywhere;
 *     every gK/gV tile has exactly one owner workgroup per call.
 */
#ifndef SECO_H_
#define SECO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum seco_dtype {
  SECO_F32 = 0,  /* Q,K,V,O,dO,dQ are float; arithmetic in fp32 */
  SECO_BF16 = 1  /* Q,K,V,O,dO,dQ are bfloat16; bf16 matrix-core products, fp32 accumulation/softmax */
} seco_dtype;

typedef enum seco_status {
  SECO_OK = 0,
  SECO_ERR_NULL = -1,        /* a required pointer is NULL */
  SECO_ERR_SHAPE = -2,       /* non-positive size, n_q_heads % n_kv_heads != 0, negative q_start, softmax_scale not finite and > 0 */
  SECO_ERR_HEAD_DIM = -3,    /* head_dim not supported for this dtype (bf16: 128; f32: multiple of 4, <= 256) */
  SECO_ERR_DTYPE = -4,       /* dtype is not a seco_dtype */
  SECO_ERR_ALIGN = -5,       /* pointer or stride breaks the 16-byte row alignment */
  SECO_ERR_WORKSPACE = -6,   /* workspace NULL or smaller than seco_workspace_bytes() */
  SECO_ERR_WEIGHTS = -7,     /* chunk weights: n_chunks/weight_chunk_len do not cover [0, q_start + chunk_len), a weight is not finite, or a dQ weight is negative */
  SECO_ERR_RANGE = -8,       /* row range or selection arguments out of range */
  SECO_ERR_LAUNCH = -9,      /* the HIP runtime refused a launch (hipGetLastError) */
  SECO_ERR_TOO_LARGE = -10   /* a size exceeds what the 32-bit tile indexing supports */
} seco_status;

typedef enum seco_op {
  SECO_OP_FWD = 0,
  SECO_OP_BWD = 1            /* seco_chunk_attn_bwd, spaco_chunk_attn_bwd, spaco_chunk_attn_bwd_sparse_dq,
                                seco_chunk_attn_bwd_gather, spaco_chunk_attn_bwd_gather */
} seco_op;

/* One chunk call.  kv_len = q_start + chunk_len cache rows are visible. */
typedef struct seco_desc {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t chunk_len;      /* C: query rows in this call (the last chunk may be short) */
  int32_t q_start;        /* global position of the chunk's first row (j*C for chunk j) */
  int32_t dtype;          /* seco_dtype */
  float softmax_scale;    /* s > 0, normally 1/sqrt(head_dim) */
  int64_t q_stride[3];    /* Q and dQ  : (batch, head, row) strides in elements */
  int64_t o_stride[3];    /* O and dO  */
  int64_t kv_stride[3];   /* K and V cache (row index = global position); ONE triple: V must be laid out like K */
  int64_t g_stride[3];    /* gK and gV, fp32 (row index = global position); ONE triple: gV laid out like gK */
} seco_desc;

/*
 * Forward of one chunk (Eq. 1; Alg. 1 both loops call it).
 *   S = s * Q K^T over cache rows [0, q_start + chunk_len), row r sees columns c <= q_start + r;
 *   O = softmax_row(S) V;   LSE[r] = ln sum_c exp(S[r,c])  (natural log of the scaled scores).
 * q        in   [B, Hq, C, D]   (q_stride)
 * k_cache  in   [B, Hkv, >= q_start + C, D]   (kv_stride); v_cache alike
 * o        out  [B, Hq, C, D]   (o_stride), overwritten
 * lse      out  fp32 [B, Hq, C] contiguous (no strides are taken for it: a sliced view is not accepted), overwritten
 * ws       optional workspace, 256-byte aligned.  seco_workspace_bytes(desc, SECO_OP_FWD) is non-zero only for
 *          bf16 calls with so few query rows that the row tiles cannot fill the GPU (short chunks, as in the
 *          chunk-size study of Sec. 6.3); given at least that many bytes, the visible cache rows are divided
 *          among several workgroups whose partial results are merged in a fixed order.  With ws NULL or smaller
 *          the call computes the same O and LSE (to rounding) without the division, only slower.
 */
int seco_chunk_attn_fwd(const seco_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                        void* o, float* lse, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Backward of one chunk for SeCO (Alg. 1, "backprop(J_i)" at the attention layer).
 * With P = exp(S - LSE), delta = rowsum(dO * O), dS = P * (dO V^T - delta):
 *   d_q  out  [B, Hq, C, D] (q_stride), overwritten:  dQ = s * dS K          (all visible columns)
 *   gk   i/o  fp32 [B, Hkv, >= q_start + C, D] (g_stride): gK[c] += s * sum_{heads of group} dS^T Q
 *   gv   i/o  same:                                        gV[c] += sum_{heads of group} P^T dO
 * for every visible cache row c.  gk/gv are accumulated into, never overwritten; rows at or
 * beyond q_start + C are not touched.  o, lse are the outputs of seco_chunk_attn_fwd for the
 * same desc; d_o has o's layout.
 * ws: seco_workspace_bytes(desc, SECO_OP_BWD) bytes, 256-byte aligned: one fp32 value per query row (delta; bf16:
 *     two, delta and the log-sum-exp in the form the dK/dV kernel consumes), plus one region shared by the
 *     partial dQ of the short-chunk path described at seco_chunk_attn_fwd and, for bf16 with grouped heads, the
 *     sums of the cache-row tiles whose query heads the dK/dV pass shares out among several workgroups when its
 *     last round of workgroups would be less than half full (at most 32 MiB; merged in head order, so gk/gv
 *     stay bit-reproducible).  SECO_ERR_WORKSPACE if NULL, misaligned or smaller.
 */
int seco_chunk_attn_bwd(const seco_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                        const void* o, const float* lse, const void* d_o,
                        void* d_q, float* gk, float* gv, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Backward of one selected chunk for SpaCO (Alg. 2; appendix listing "grad + base * scaler").
 * Same as seco_chunk_attn_bwd except that the contribution to cache rows of chunk i,
 * i.e. rows [i * weight_chunk_len, (i+1) * weight_chunk_len), is multiplied by
 * chunk_weight_host[i] before it is added:  gK[c] += w[chunk(c)] * dK_c, gV likewise.
 * Column tiles whose weight is exactly 0 are neither computed nor touched.  dQ is exact
 * (all visible columns) whatever the weights.
 *   chunk_weight_host  HOST array of n_chunks floats, read before the call returns
 *   n_chunks * weight_chunk_len must be >= q_start + chunk_len  (and (n_chunks-1)*weight_chunk_len < that)
 * The paper's policy: w = k/t (optionally capped, Sec. 6.4) for earlier selected chunks,
 * 1 for the chunk's own rows, 0 for unselected chunks; see spaco_chunk_weights().
 * With all weights 1 the result is bit-identical to seco_chunk_attn_bwd.
 */
int spaco_chunk_attn_bwd(const seco_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                         const void* o, const float* lse, const void* d_o,
                         void* d_q, float* gk, float* gv,
                         const float* chunk_weight_host, int32_t n_chunks, int32_t weight_chunk_len,
                         void* ws, size_t ws_bytes, void* hip_stream);

/*
 * spaco_chunk_attn_bwd with a dQ that visits only some cache rows as well.  Not in the paper, whose Alg. 2 keeps
 * dQ exact over every earlier cache, so that a selected chunk's backward still grows with the context; the
 * sampling argument of its Sec. 5 (an expected weight of 1 on every term keeps the sum unbiased) applies to the
 * column sum of dQ too, because the term of a cache row needs only that row of K and V and the query row's LSE
 * and delta, both exact here:
 *     dQ = s * sum_i dq_weight_host[i] * sum_{c in chunk i} dS[:, c] K[c, :]
 * with chunk i = rows [i * weight_chunk_len, (i+1) * weight_chunk_len) as for chunk_weight_host.  Rows of chunks
 * with dq weight 0 are not read; all weights 1 give the exact dQ (bit-identical to spaco_chunk_attn_bwd).
 *   dq_weight_host  HOST array of n_chunks finite, non-negative floats, read before the call returns;
 *                   SECO_ERR_WEIGHTS otherwise.  Its non-zero weights may form at most 48 runs of consecutive
 *                   chunks with equal weight (SECO_ERR_TOO_LARGE beyond that).
 * gk/gv, chunk_weight_host and every other argument: as spaco_chunk_attn_bwd.
 * In a model with several attention layers the dQ weights of a chunk's call must be drawn independently per layer
 * for the estimate to stay unbiased (a path that stays inside the chunk meets the same cache rows in every layer).
 */
int spaco_chunk_attn_bwd_sparse_dq(const seco_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                   const void* o, const float* lse, const void* d_o,
                                   void* d_q, float* gk, float* gv,
                                   const float* chunk_weight_host, const float* dq_weight_host,
                                   int32_t n_chunks, int32_t weight_chunk_len,
                                   void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Backward of one chunk in the transposed order (bf16 only).  Alg. 1 lets the backward of chunk j add its dK/dV to
 * the gradient of every earlier checkpoint m'_i; the sum that m'_i.grad holds when chunk i is reached,
 *     gK[rows of chunk i] = sum over chunks j >= i of (dK of chunk j's queries on those rows),
 * can as well be formed when chunk i is reached, because the terms of a later chunk need only its Q, dO, LSE and
 * delta, all known by then.  This call does that for chunk i = desc: it returns dQ of the chunk exactly as
 * seco_chunk_attn_bwd does, and ADDS to rows [q_start, q_start + chunk_len) of gk/gv the contributions of the
 * chunk's own query rows and of the n_later_rows query rows that follow it; no other row of gk/gv is touched.
 * Called for every chunk in descending order with all later rows, the result equals that of seco_chunk_attn_bwd
 * called for every chunk (to rounding: the summation order differs; both orders are fixed, so both are
 * reproducible).  Every call has the same number of cache rows to cover, so its workgroups are equal in length
 * and none re-reads gk/gv rows that another call wrote.
 *   q_rows     in   [B, Hq, chunk_len + n_later_rows, D] (q_stride): queries of sequence rows q_start, q_start+1, ...
 *   d_o_rows   in   the same rows of dO (o_stride)
 *   o, lse     in   forward outputs of the chunk itself ([B, Hq, C, D] with o_stride, [B, Hq, C])
 *   d_q        out  [B, Hq, C, D] (q_stride)
 *   row_stats  i/o  fp32 [2, B, Hq, stat_rows], 16-byte aligned, kept by the caller for the whole backward pass:
 *                   the call writes the entries of its own rows (at positions q_start ..) and reads those of the
 *                   later rows, which the calls of the later chunks wrote.  stat_rows: a multiple of 4 that is
 *                   >= q_start + chunk_len + n_later_rows (SECO_ERR_RANGE otherwise).
 *   ws         as seco_chunk_attn_bwd (same size)
 */
int seco_chunk_attn_bwd_gather(const seco_desc* desc, const void* q_rows, const void* k_cache, const void* v_cache,
                               const void* o, const float* lse, const void* d_o_rows,
                               void* d_q, float* gk, float* gv, float* row_stats, int64_t stat_rows,
                               int32_t n_later_rows, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * seco_chunk_attn_bwd_gather with a weight per chunk of query rows: the SpaCO backward (Alg. 2) in the transposed
 * order.  The rows handed in are divided into chunks of weight_chunk_len rows counted from the call's first row
 * (chunk 0: the call's own rows when weight_chunk_len = chunk_len); the contribution of chunk m's query rows to the
 * call's gK/gV rows is multiplied by row_weight_host[m], and chunks of weight 0 are not read.  With the paper's
 * policy the selected chunk i is called with weight 1 on its own rows, k/t on the later selected chunks and 0 on the
 * others, which gives the gK/gV rows that spaco_chunk_attn_bwd calls for the same selection leave there.
 *   row_weight_host  HOST array of n_row_chunks finite, non-negative floats, read before the call returns
 *   weight_chunk_len a multiple of 64; n_row_chunks * weight_chunk_len >= chunk_len + n_later_rows and
 *                    (n_row_chunks - 1) * weight_chunk_len < that (SECO_ERR_WEIGHTS otherwise); at most 24 runs
 *                    of consecutive chunks with equal non-zero weight (SECO_ERR_TOO_LARGE beyond)
 * dQ is exact, as in spaco_chunk_attn_bwd; every other argument as seco_chunk_attn_bwd_gather.  The row statistics
 * of a later chunk must have been written by that chunk's own call: chunks with non-zero weight are chunks that
 * were called.
 */
int spaco_chunk_attn_bwd_gather(const seco_desc* desc, const void* q_rows, const void* k_cache, const void* v_cache,
                                const void* o, const float* lse, const void* d_o_rows,
                                void* d_q, float* gk, float* gv, float* row_stats, int64_t stat_rows,
                                int32_t n_later_rows, const float* row_weight_host, int32_t n_row_chunks,
                                int32_t weight_chunk_len, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * seco_chunk_attn_bwd without a workspace argument and without any allocation: for callers that cannot allocate
 * device memory (code under HIP graph capture, serving loops, harnesses that forbid it).  The workspace of
 * seco_chunk_attn_bwd is taken from a device array of SECO_STATIC_SCRATCH_BYTES bytes that is part of the library's
 * code object; every GPU the library runs on holds its own copy until the process ends.  Same kernels, same launch
 * plan and therefore bit-identical d_q, gk, gv as seco_chunk_attn_bwd with a caller-supplied workspace.
 *   - SECO_ERR_TOO_LARGE if seco_workspace_bytes(desc, SECO_OP_BWD) exceeds SECO_STATIC_SCRATCH_BYTES (nothing is
 *     enqueued); every other argument and error as seco_chunk_attn_bwd.
 *   - The call uses the current HIP device's copy of the array; its address is looked up on the first call on that
 *     device.  No hipMalloc, hipFree or other allocating call is made, on the device or on the host.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different streams, or
 *     different host threads without ordering) race and give wrong results.  Calls on one stream are safe.
 */
#define SECO_STATIC_SCRATCH_BYTES ((size_t)40 << 20)
int seco_chunk_attn_bwd_noalloc(const seco_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                const void* o, const float* lse, const void* d_o,
                                void* d_q, float* gk, float* gv, void* hip_stream);

/*
 * Zero rows [row_begin, row_end) of the KV gradient buffers (start of a training iteration;
 * the buffers then collect the contributions of Alg. 1's / Alg. 2's second loop).
 * Uses batch, n_kv_heads, head_dim and g_stride of desc.  Either pointer may be NULL (skipped).
 */
int kvgrad_zero(const seco_desc* desc, float* gk, float* gv, int64_t row_begin, int64_t row_end, void* hip_stream);

/*
 * dst[rows] += scale * src[rows] on fp32 KV gradient buffers: the gradient relay of the
 * appendix listing (grad_hook: grad + base * scaler) and of Alg. 2's "(k/t) * m'_i.grad".
 * dst and src both use g_stride.  A NULL dst/src pair is skipped; dst must not alias src.
 */
int kvgrad_accumulate(const seco_desc* desc, float* dst_k, float* dst_v, const float* src_k, const float* src_v,
                      float scale, int64_t row_begin, int64_t row_end, void* hip_stream);

/*
 * Cache append (appendix listing, update_kv_cache): writes the chunk's keys and values into rows
 * [q_start, q_start + chunk_len) of the preallocated caches, after which rows [0, q_start + chunk_len) are what
 * the listing obtains by concatenation.  Uses batch, n_kv_heads, head_dim, dtype, chunk_len, q_start;
 * k_new, v_new: [B, Hkv, C, D] with q_stride; k_cache, v_cache: kv_stride.  Either pair may be NULL (skipped).
 */
int kv_append(const seco_desc* desc, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
              void* hip_stream);

/*
 * Gradient hand-over to a recomputed chunk (appendix listing, copy_grad / grad_hook's "base * scaler"):
 *   d_k_new[b, h, r, :] = (dtype)(scaler * gk[b, h, q_start + r, :]),   d_v_new likewise from gv,
 * product in fp32, rounded to nearest-even for bf16.  gk, gv: fp32 with g_stride; d_k_new, d_v_new: [B, Hkv, C, D]
 * with q_stride, overwritten.  Either pair may be NULL (skipped).  With the in-kernel weights of
 * spaco_chunk_attn_bwd the rows already carry the factor and scaler is 1.
 */
int kvgrad_readout(const seco_desc* desc, const float* gk, const float* gv, void* d_k_new, void* d_v_new,
                   float scaler, void* hip_stream);

/*
 * Rotary position embedding fused into the two calls above and available on its own.  Not part of the paper, whose
 * model code is not shown; the model of its experiments (LLaMA-3) rotates queries and keys before attention, in
 * the "rotate-half" pairing: the pair (x[i], x[i + D/2]), i < D/2, of the row at sequence position p turns by the
 * angle p * rope_base^(-2 i / D).  Angles, sines and cosines are computed in fp64, the result is rounded once
 * (fp64 -> fp32 -> dtype).  head_dim must be a multiple of 8; rope_base must be finite and > 1
 * (SECO_ERR_RANGE otherwise).
 *   kv_append_rope       as kv_append, with the keys rotated for their positions q_start + r on the way into the
 *                        cache (the values are copied); one pass over the data instead of rotate, then copy.
 *   kvgrad_readout_rope  as kvgrad_readout, with the key gradient turned back:
 *                        d_k_new = (dtype) R(-theta)(scaler * gk[rows]); d_v_new as in kvgrad_readout.
 *   rope_rotate          x_out[b, h, r, :] = R(+-theta(pos_start + r)) x_in[b, h, r, :] for [B, n_heads, C, D] tensors
 *                        with q_stride (in) and o_stride (out), e.g. the chunk's queries (inverse = 0) and dQ
 *                        (inverse = 1); uses batch, head_dim, chunk_len, dtype of desc and the given n_heads;
 *                        x_out may be x_in.
 */
int kv_append_rope(const seco_desc* desc, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                   float rope_base, void* hip_stream);
int kvgrad_readout_rope(const seco_desc* desc, const float* gk, const float* gv, void* d_k_new, void* d_v_new,
                        float scaler, float rope_base, void* hip_stream);
int rope_rotate(const seco_desc* desc, int32_t n_heads, const void* x_in, void* x_out, int64_t pos_start,
                float rope_base, int32_t inverse, void* hip_stream);

/*
 * SpaCO chunk selection (Alg. 2, selection step: t different chunks out of k, uniformly), host only.
 * Deterministic in (seed, step): SplitMix64 stream keyed by (seed, step), unbiased bounded
 * draws by rejection, first t steps of a Fisher-Yates shuffle of 0..k-1, result sorted in
 * DESCENDING order (the order in which the chunks have to be back-propagated).
 * out_host: HOST array of t int32.
 */
int spaco_select_chunks(uint64_t seed, uint64_t step, int32_t k, int32_t t, int32_t* out_host);

/*
 * Weight vector of the policy "every chunk back-propagated, each call with its own draw", host only: call j draws
 * m = min(t, j) of its j earlier chunks (spaco_select_chunks with step * 2^20 + j as the step) and weights them
 * j / m, its own rows 1.  Each earlier chunk then has expected weight 1 (unbiased dK/dV for the layer) and dQ is
 * exact, because every chunk is back-propagated: one reading of "a few uniformly sampled earlier chunks plus the
 * current chunk"; Alg. 2 itself draws once per iteration (spaco_select_chunks + spaco_chunk_weights).
 * w_host: HOST array of j+1 floats.
 */
int spaco_percall_weights(uint64_t seed, uint64_t step, int32_t j, int32_t t, float* w_host);

/*
 * Selection by independent inclusion, host only: every chunk 0..k-1 is selected with probability q, independently
 * (the sampling law under which the survival argument of Sec. 5, "Compensation Factor", holds exactly: a chain
 * through p+1 chunks survives with probability q^(p+1); with relay factor 1/q and an overall 1/q the gradient
 * estimate is unbiased).  Same generator and key as spaco_select_chunks; chunk i is selected iff the i-th 64-bit
 * draw is below floor(q * 2^64).  0 < q <= 1.
 * out_host: HOST array of k int32; the selected indices, DESCENDING, are written to its front and their number
 * (possibly 0) to *n_selected_host.
 */
int spaco_select_bernoulli(uint64_t seed, uint64_t step, int32_t k, double q, int32_t* out_host,
                           int32_t* n_selected_host);

/*
 * The compensation factor k/t of Sec. 5, limited to `cap` when cap > 0 (Sec. 6.4 trains with a cap of 2).
 * Returns a negative value on invalid arguments (k < 1, t < 1, t > k).
 */
float spaco_compensation_factor(int32_t k, int32_t t, float cap);

/*
 * Weight vector for the backward call of chunk j under the paper's policy, host only:
 * w[i] = factor for i in selected, i < j;  w[j] = 1;  0 otherwise.
 * factor is k/t (Sec. 5), optionally capped by the caller (Sec. 6.4).
 * selected_host: n_selected chunk indices (any order); w_host: j + 1 floats, overwritten.
 */
int spaco_chunk_weights(const int32_t* selected_host, int32_t n_selected, int32_t j, float factor, float* w_host);

/*
 * Row weights of spaco_chunk_attn_bwd_gather for selected chunk i of k under the paper's policy (Alg. 2 with the
 * factor of Sec. 5), host only: one weight per chunk of query rows from chunk i on,
 *   w[0] = 1 (the chunk's own rows), w[m - i] = factor for a selected chunk m > i, 0 for every other chunk,
 * i.e. the transpose of spaco_chunk_weights: call m of the accumulating order puts `factor` on chunk i exactly
 * when m is selected.  selected_host: n_selected chunk indices (any order); w_host: k - i floats, overwritten.
 */
int spaco_gather_row_weights(const int32_t* selected_host, int32_t n_selected, int32_t i, int32_t k, float factor,
                             float* w_host);

/*
 * Optional per-kernel timing, for benchmarks (not part of the method).  While enabled, every
 * kernel the library launches is bracketed by a pair of HIP events recorded on the launch
 * stream.  seco_profile_read waits for the recorded events, adds up elapsed milliseconds and
 * launch counts per kernel kind (arrays of SECO_PROFILE_KINDS entries, host memory), and
 * forgets them.  This is the only process-wide state the library has; it is not thread-safe.
 */
typedef enum seco_profile_kind {
  SECO_PROFILE_FWD = 0,     /* forward kernel */
  SECO_PROFILE_DELTA = 1,   /* delta = rowsum(dO * O) */
  SECO_PROFILE_DQ = 2,      /* dQ kernel */
  SECO_PROFILE_DKDV = 3,    /* dK/dV kernel with the gK/gV accumulation */
  SECO_PROFILE_KVGRAD = 4,  /* kvgrad_zero / kvgrad_accumulate */
  SECO_PROFILE_MERGE = 5,   /* merge of partial O / dQ on the short-chunk path */
  SECO_PROFILE_KINDS = 6
} seco_profile_kind;
int seco_profile_enable(int on);                    /* all kinds on / off; forgets recorded events */
int seco_profile_enable_kinds(uint32_t kind_mask);  /* bit k set: time kernels of kind k only (events cost a few
                                                       microseconds per launch, so a benchmark brackets only what
                                                       it reports) */
int seco_profile_set_kinds(uint32_t kind_mask);     /* the same mask, but the events recorded so far are kept: lets a
                                                       benchmark bracket only some of its steps */
int seco_profile_read(double* total_ms_host, int64_t* launches_host);

/* Workspace bytes an entry point needs for this desc (0 if none; (size_t)-1 on an invalid desc).  The launch plan,
 * and with it this size, counts workgroups against the number of compute units of the device that is current when
 * the library is first used (256, an MI355X's, when no device can be asked): ask on the device the call will run on. */
size_t seco_workspace_bytes(const seco_desc* desc, int op);

/*
 * How the bf16 kernels would be launched for this desc (host arithmetic only, nothing is launched; for tests and
 * tuning).  n_col_tiles: number of 128-row cache tiles the dK/dV pass of the call covers (rows with non-zero
 * weight, each run of equal weight rounded up to whole tiles).  plan_host receives four values:
 *   [0] workgroups that share the cache rows of one row tile in the forward / dQ pass (1: no division)
 *   [1] row tiles of the forward / dQ pass (work items before that division)
 *   [2] cache tiles per (batch, KV head), counted from the last, that the dK/dV pass shares out by query head
 *   [3] workgroups per such tile (1: none); [2] * [3] * batch * n_kv_heads never exceeds the device's compute units
 * Returns SECO_OK, or the status of an invalid desc; SECO_ERR_DTYPE for fp32 (its kernels have one shape).
 */
int seco_launch_plan(const seco_desc* desc, int32_t n_col_tiles, int32_t* plan_host);

/*
 * What the current HIP device reports, for benchmarks that state the matrix-core peak they compare against
 * (compute units x 4096 bf16 FLOP per clock x clock): number of compute units and maximum engine clock in kHz,
 * written to the two HOST integers.  SECO_ERR_NULL for a NULL pointer, SECO_ERR_LAUNCH if the runtime has no device.
 */
int seco_device_info(int32_t* compute_units_host, int32_t* max_clock_khz_host);

/* Static English description of a status code. */
const char* seco_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SECO_H_ */
