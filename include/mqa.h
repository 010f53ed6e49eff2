/*
 * mqa.h - C ABI of the MI355X (gfx950) multi-query-attention decode library.
 *
 * The library implements one incremental decoding step of multi-query
 * attention (arXiv 1911.02150, Section 3, `MultiquerySelfAttentionIncremental`)
 * and, as the bandwidth comparison, of multi-head attention (Section 2.4,
 * `MultiheadSelfAttentionIncremental`), split into the calls a decode loop
 * makes:  project q and the new K/V row  ->  append the row to the cache  ->
 * attend over the cache  ->  project the heads' outputs.
 *
 * Conventions common to every call
 *  - All pointers are DEVICE pointers unless stated otherwise.  The caller
 *    allocates and frees every buffer (including the workspace and `lens`);
 *    the library never allocates, frees or synchronises.
 *  - `stream` is the caller's hipStream_t (NULL = the default stream).  A call
 *    validates its arguments on the host, enqueues its kernels and returns.
 *  - Tensors are dense, row-major, innermost index last, in the paper's index
 *    order: q [b,h,k], o [b,h,v]; multi-query cache K [b,cap,k], V [b,cap,v];
 *    multi-head cache K [b,h,cap,k], V [b,h,cap,v]; projections P_q [h,d,k],
 *    P_o [h,d,v] (model width before value width), multi-query P_k [d,k],
 *    P_v [d,v], multi-head P_k [h,d,k], P_v [h,d,v].
 *  - x, q, o, y and the projection matrices are float32.  The cache is float32
 *    (MQA_F32) or bfloat16 (MQA_BF16); accumulation is float32.
 *  - `cap` is the cache capacity in positions; `lens[i]` (int32, one per
 *    sequence) is how many positions of sequence i are valid.  The paper's
 *    growing concat (and its padded fixed-shape variant, Section 4.3 footnote)
 *    is replaced by this capacity + length form.  Values of lens outside
 *    [0,cap] are clamped by the kernels.
 *  - Return value: MQA_OK (0) or a positive MQA_ERR_* code.  Arguments are
 *    checked before anything is enqueued, so on MQA_ERR_NULL / _SHAPE / _ALIGN /
 *    _WORKSPACE / _DTYPE the stream is untouched; MQA_ERR_LAUNCH reports a launch
 *    the HIP runtime refused (earlier kernels of the same call may already be in
 *    the stream).  No call aborts or throws.
 *  - Pointers must be 16-byte aligned.
 */
#ifndef MQA_H
#define MQA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MQA_F32 = 0, MQA_BF16 = 1 } mqa_dtype; /* cache element type */

typedef enum {
  MQA_OK = 0,
  MQA_ERR_NULL = 1,       /* a required pointer is NULL                         */
  MQA_ERR_SHAPE = 2,      /* a size is non-positive or not supported            */
  MQA_ERR_ALIGN = 3,      /* a pointer is not 16-byte aligned                   */
  MQA_ERR_WORKSPACE = 4,  /* workspace missing or smaller than required         */
  MQA_ERR_DTYPE = 5,      /* unknown mqa_dtype / mqa_proj_mode                  */
  MQA_ERR_LAUNCH = 6,     /* the HIP runtime refused a launch                   */
  MQA_ERR_SCRATCH_LIMIT = 7 /* mqa_decode_step_noalloc: the call needs more scratch
                               memory than the library's static buffer holds    */
} mqa_status;

typedef enum {
  MQA_PROJ_Q = 0,     /* in [rows,d] . P [h,d,kv] -> out [rows,h,kv]  q = einsum('bd,hdk->bhk')   */
  MQA_PROJ_KV = 1,    /* in [rows,d] . P [d,kv]   -> out [rows,kv]    einsum('bd,dk->bk'); h ignored */
  MQA_PROJ_KV_MH = 2, /* in [rows,d] . P [h,d,kv] -> out [rows,h,kv]  multi-head new rows          */
  MQA_PROJ_O = 3,     /* in [rows,h,kv] . P [h,d,kv] -> out [rows,d]  y = einsum('bhv,hdv->bd')    */
  MQA_PROJ_LINEAR = 4 /* in [rows,d] . P [d,kv]   -> out [rows,kv]    a plain x.W (the decoder stack's
                         feed-forward matrices; not part of the attention path); h ignored      */
} mqa_proj_mode;

/* Optional launch tuning for the decode calls (NULL = library heuristics). */
typedef struct {
  int32_t splits;   /* >0: number of position ranges each sequence is split into */
  int32_t kernel;   /* 0 auto, 1 force the generic kernel, 2 force the MFMA kernel
                       (MQA_ERR_SHAPE if the shape does not qualify)             */
  int32_t flags;    /* MFMA kernel variants, 0 = default (measurement and test switches):
                       bit 0   single bf16 term for q (faster, less accurate)
                       bit 1   single bf16 term for the softmax weights (likewise)
                       bit 2   plain instead of non-temporal cache loads
                       bit 3   more than 32 heads: head groups of 32 as separate
                               workgroups instead of 64 heads per workgroup
                               sharing each tile through LDS
                       bit 4   8 waves per workgroup (up to 32 heads)
                       bit 5   never / bit 6: always schedule the longest
                               sequences first (default: only for large
                               ragged-capable batches)
                       bit 7   two bf16 terms for the weights in the 64-head
                               form too (its default is one, normalised by the
                               sum of the rounded weights)
                       bit 8   2 waves per workgroup for up to 16 heads (default:
                               only for ranges of at most 128 positions in
                               launches of 512 workgroups or more) / bit 9: never
                       bit 10  one workgroup per sequence even where the 64-head
                               form would keep one workgroup per compute unit
                               going over several ranked sequences
                       bit 11  rank by a separate launch even where that kernel
                               would rank up to 1024 sequences itself
                       bit 12  causal rows (prompt pass) in workgroups of 32 rows
                               whose waves split the tiles, instead of 128 rows,
                               32 per wave                                       */
} mqa_tuning;

/*
 * The four projections of the incremental listings (Section 2.4 / Section 3):
 * first line (q), the new K and V rows, and the last line (y).  float32 in and
 * out, float32 accumulation -- except the new K / V rows (MQA_PROJ_KV, _KV_MH
 * and the K / V part of mqa_project_append_qkv), whose products are summed in
 * float64 and rounded once to float32: what is then rounded into a bf16 cache
 * is the correctly rounded projection, whatever the summation order.  `rows`
 * is the number of input rows (b for a decode step, b*m when projecting a whole
 * memory M as in the Section 2.2 one-query listing).  `kv` is k or v.  `out` is
 * overwritten.
 */
int mqa_project_qkvo(mqa_proj_mode mode, const float* in, const float* P, float* out,
                     int rows, int d, int h, int kv, void* stream);

/*
 * The same projections with an epilogue applied to every output element before it is stored,
 * for callers that chain them (a decoder layer's residual stream and feed-forward block):
 * MQA_EPI_STORE as above; MQA_EPI_RELU stores max(x, 0); MQA_EPI_ADD adds x to what `out`
 * already holds (the residual connection around the attention of Section 4.1's layers).
 */
typedef enum { MQA_EPI_STORE = 0, MQA_EPI_RELU = 1, MQA_EPI_ADD = 2 } mqa_proj_epilogue;
int mqa_project_qkvo_ex(mqa_proj_mode mode, const float* in, const float* P, float* out,
                        int rows, int d, int h, int kv, mqa_proj_epilogue epilogue, void* stream);

/*
 * The first three lines of the incremental listings plus the concat, in one launch: q = x . P_q
 * is written to q [b,h,k]; the new rows x . P_k, x . P_v go straight into row lens_in[i] of the
 * caches (rounded as in mqa_append_kv) and lens_out[i] = lens_in[i] + 1.  Same results as
 * mqa_project_qkvo (Q, KV or KV_MH) followed by mqa_append_kv (q up to float32 summation order;
 * the cache rows bit for bit).
 *   x [b,d]; P_q [h,d,k]; h_kv = 1 (multi-query): P_k [d,k], P_v [d,v], K [b,cap,k], V [b,cap,v];
 *   h_kv = h (multi-head): P_k [h,d,k], P_v [h,d,v], K [b,h,cap,k], V [b,h,cap,v].
 *   lens_in and lens_out must be different arrays (the workgroups of the launch read lens_in
 *   while it runs; MQA_ERR_SHAPE if they are the same pointer); a caller alternates two arrays
 *   from step to step.  A sequence at capacity keeps its cache and lens_out[i] = lens_in[i].
 *   d % 8 = 0, k % 16 = 0, v % 16 = 0.
 */
int mqa_project_append_qkv(const float* x, const float* P_q, const float* P_k, const float* P_v,
                           float* q, void* K, void* V, const int32_t* lens_in, int32_t* lens_out,
                           int b, int d, int h, int h_kv, int cap, int k, int v, mqa_dtype dt, void* stream);

/*
 * Encoder-decoder ("memory") attention: the one-query-against-a-memory form of the paper's
 * Section 2.2 listing under the Section 3 rule (K, V, P_k, P_v lose the heads dimension) -- the
 * attention kind that, with the two self-attentions, Section 4.1 converts to multi-query.  The
 * memory M does not change while decoding, so its keys and values are projected once:
 *   mqa_project_memory_kv: K[i,p,:] = M[i,p,:] . P_k, V[i,p,:] = M[i,p,:] . P_v for p < m
 *     (float64 accumulation, rounded once to float32 and then to the cache type, like every new
 *     K / V row), written straight into the caches, and lens[i] = m -- or mem_lens[i] clamped to
 *     [0, m] when mem_lens (device, may be NULL) gives the number of valid memory rows of
 *     sequence i (padded batches).  M [b,m,d]; h_kv = 1: P_k [d,k], P_v [d,v], K [b,cap,k],
 *     V [b,cap,v]; h_kv = h: P_k [h,d,k], P_v [h,d,v], K [b,h,cap,k], V [b,h,cap,v].  m <= cap,
 *     d % 8 = 0, k % 16 = 0, v % 16 = 0.  One launch, no intermediate rows in memory.
 *   mqa_memory_decode_step: every decoding step then attends to that fixed cache: q [b,queries,h,k]
 *     holds the projected queries of the `queries` decoder positions that share memory i at this
 *     step (1 for greedy decoding, the beam width under beam search: all hypotheses of a source
 *     read its memory once), o [b,queries,h,v].  It is mqa_decode_step over queries*h query heads;
 *     same workspace rule with h replaced by queries*h.  The multi-head form with one query per
 *     memory is mha_decode_step over the per-head caches.
 */
int mqa_project_memory_kv(const float* M, const float* P_k, const float* P_v, void* K, void* V,
                          const int32_t* mem_lens, int32_t* lens, int b, int m, int d, int h_kv, int cap,
                          int k, int v, mqa_dtype dt, void* stream);
int mqa_memory_decode_step(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                           int b, int queries, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cache append: the in-place form of the listings' tf.concat.  For every
 * sequence i with lens[i] < cap, writes k_new[i] / v_new[i] (converted to the
 * cache type, round-to-nearest-even for bf16) as position lens[i] and then
 * increments lens[i].  A sequence already at capacity is left untouched.
 * h_kv = 1: multi-query cache, k_new [b,k], v_new [b,v].
 * h_kv = h: multi-head cache,  k_new [b,h,k], v_new [b,h,v].
 * K, V and lens are modified; k_new and v_new are read only.
 */
int mqa_append_kv(void* K, void* V, const float* k_new, const float* v_new, int32_t* lens,
                  int b, int h_kv, int cap, int k, int v, mqa_dtype dt, void* stream);

/*
 * Attention of one multi-query decode step (Section 3 incremental listing,
 * the three lines logits / weights / o):
 *   logits[i,j,p] = scale * sum_c q[i,j,c] K[i,p,c],  p < lens[i]
 *   weights = softmax over p,   o[i,j,:] = sum_p weights[i,j,p] V[i,p,:]
 * Call after mqa_append_kv so that the new token attends to itself.  The paper
 * uses scale = 1 (the 1/sqrt(k) factor is folded into P_q or P_k).
 * lens[i] = 0 gives a zero output row.  K, V, q, lens are read only; o is
 * overwritten; `workspace` (>= mqa_decode_workspace_bytes) holds the partial
 * softmax states of the position ranges and is overwritten.  A call that needs
 * one range per sequence runs without a workspace (NULL, 0); with one, a batch
 * that has several workgroups per compute unit starts its longest sequences
 * first (ragged batches finish sooner; outputs are the same either way).
 * The logits and weights never reach memory.
 */
int mqa_decode_step(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                    int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same step for multi-head attention (Section 2.4 listing): K [b,h,cap,k],
 * V [b,h,cap,v]; head j of sequence i reads only K[i,j], V[i,j].  Same
 * arguments, same workspace rule (use mha_decode_workspace_bytes).
 */
int mha_decode_step(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                    int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Local attention, the variant of the paper's Section 4.1 ("attention to the current position
 * and the previous 31 positions"): as the two calls above, but sequence i attends only to
 * positions [max(0, lens[i] - window), lens[i]).  window > 0 (32 in the paper).  Only the rows
 * inside the window are read.
 */
int mqa_decode_step_window(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                           int b, int h, int cap, int k, int v, mqa_dtype dt, float scale, int window,
                           void* workspace, size_t workspace_bytes, void* stream);
int mha_decode_step_window(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                           int b, int h, int cap, int k, int v, mqa_dtype dt, float scale, int window,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * A whole prompt at once: the multi-query attention of the paper's Section 3 batched listing
 * (`MultiqueryAttentionBatched`) with the causal mask of Section 2.3, fused (logits and weights
 * never reach memory), for n consecutive queries per sequence against the cache.
 *   mqa_append_kv_rows: as mqa_append_kv for n rows per sequence, k_new [b,n,h_kv,k],
 *     v_new [b,n,h_kv,v]; lens[i] += n; a sequence without room for all n rows is left untouched.
 *   mqa_prefill_attention: q [b,n,h,k] (the q projection of the n inputs, rows in that order),
 *     o [b,n,h,v].  Call after the append: query j of sequence i sits at position
 *     lens[i]-n+j and attends to positions 0..lens[i]-n+j.  lens[i] >= n is required (a query
 *     with nothing to attend to yields zeros).  bf16 cache with k = v = 128 only
 *     (MQA_ERR_SHAPE otherwise).  The n*h rows of a sequence share each K/V tile they read.
 */
int mqa_append_kv_rows(void* K, void* V, const float* k_new, const float* v_new, int32_t* lens,
                       int b, int n, int h_kv, int cap, int k, int v, mqa_dtype dt, void* stream);
int mqa_prefill_attention(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                          int b, int n, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                          void* workspace, size_t workspace_bytes, void* stream);
/*
 * The multi-head twin (Section 2.3 listing `MultiheadAttentionBatched` with its causal mask):
 * q [b,h,n,k] and o [b,h,n,v] (head-major, so that the n queries of a head are adjacent rows),
 * K [b,h,cap,k], V [b,h,cap,v]; query j of head t of sequence i attends to positions
 * 0..lens[i]-n+j of K[i,t], V[i,t].  Same restrictions as mqa_prefill_attention.
 */
int mha_prefill_attention(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                          int b, int n, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Beam search (the paper decodes with beam 4 in Section 4.1 and times it in Table 2): the
 * `beam` hypotheses of a source share the memory rows they have in common (the source / prompt)
 * and own only the rows they produced themselves.  The memory of hypothesis (i, e) is
 * K_src[i, :lens_src[i]] followed by K_own[i, e, :lens_own[i*beam+e]] (likewise V); the step is
 * the Section 3 attention over it.  The shared rows are read once per source for all beam*h
 * query rows; the own rows once per hypothesis.
 *   q [b,beam,h,k] device float32; K_src [b,cap_src,k], V_src [b,cap_src,v], lens_src [b];
 *   K_own [b,beam,cap_own,k], V_own [b,beam,cap_own,v], lens_own [b*beam]; o [b,beam,h,v].
 *   A hypothesis with no valid row in either part yields zeros.  Always uses the workspace:
 *   at least mqa_decode_beams_workspace_bytes(...) bytes (0 = unsupported sizes), 16-byte aligned.
 * mqa_beam_reorder_kv: after the search has chosen, for every hypothesis slot r (r = i*beam + e over
 * all sources), the hypothesis parent[r] it continues, slot r of the destination cache receives
 * rows [0, lens_src[parent[r]]) of slot parent[r] of the source cache and its length.  K_* are
 * [n,h_kv,cap,k] (h_kv = 1 for multi-query), V_* [n,h_kv,cap,v], lens_* [n], parent [n] (values
 * outside [0,n) are clamped).  Source and destination must be different buffers (MQA_ERR_SHAPE
 * if a pointer pair is identical; partial overlap is undefined).  Destination rows at and beyond
 * the new length are left as they were.  With multi-query caches this moves 1/h of the bytes
 * the multi-head layout moves.
 */
int mqa_decode_step_beams(const float* q, const void* K_src, const void* V_src, const int32_t* lens_src,
                          const void* K_own, const void* V_own, const int32_t* lens_own, float* o,
                          int b, int beam, int h, int cap_src, int cap_own, int k, int v, mqa_dtype dt,
                          float scale, void* workspace, size_t workspace_bytes, void* stream);
size_t mqa_decode_beams_workspace_bytes(int b, int beam, int h, int cap_src, int cap_own, int k, int v,
                                        mqa_dtype dt);
int mqa_beam_reorder_kv(const void* K_src, const void* V_src, const int32_t* lens_src, const int32_t* parent,
                        void* K_dst, void* V_dst, int32_t* lens_dst,
                        int n, int h_kv, int cap, int k, int v, mqa_dtype dt, void* stream);

/* Same as mqa_decode_step / mha_decode_step with explicit launch tuning (NULL = defaults). */
int mqa_decode_step_ex(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                       int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                       void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning);
int mha_decode_step_ex(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                       int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                       void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning);

/*
 * The two passes of mqa_decode_step as separate calls, for measurement: the
 * first streams K and V and leaves one partial softmax state (running maximum,
 * sum of exponentials, un-normalised weighted sum of V rows) per position
 * range in the workspace (or writes o directly when there is one range); the
 * second merges the ranges: M = max m_i, L = sum l_i e^{m_i-M},
 * o = sum acc_i e^{m_i-M} / L.  Calling them back to back on one stream is
 * identical to mqa_decode_step_ex.
 */
int mqa_decode_partials(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                        int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                        void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning);
int mqa_decode_combine(const int32_t* lens, float* o, int b, int h, int cap, int k, int v, mqa_dtype dt,
                       void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning);

/* Workspace sizes in bytes (host-side arithmetic): an upper bound valid for any tuning ... */
size_t mqa_decode_workspace_bytes(int b, int h, int cap, int v);
size_t mha_decode_workspace_bytes(int b, int h, int cap, int v);
/* ... and exactly what mqa_decode_step / mha_decode_step (library heuristics, no window) use for
 * this shape: the partial states of the ranges they choose plus the length schedule. */
size_t mqa_decode_workspace_bytes_default(int b, int h, int cap, int k, int v, mqa_dtype dt, int multi_head);

/* Number of position ranges the decode calls will use (host-side). multi_head = 0/1. */
int mqa_decode_num_splits(int b, int h, int cap, int k, int v, mqa_dtype dt, int multi_head,
                          const mqa_tuning* tuning);
/* The whole launch plan (host-side): ranges per sequence, positions per range (a multiple of 32)
 * and head groups, for full (window = 0) or local attention.  Any output pointer may be NULL. */
int mqa_decode_plan(int b, int h, int cap, int k, int v, mqa_dtype dt, int multi_head, int window,
                    const mqa_tuning* tuning, int32_t* splits, int32_t* chunk, int32_t* head_groups);

/*
 * mqa_decode_step for callers that cannot allocate or hand over a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the partial softmax
 * states and the length schedule live in a static device buffer of MQA_NOALLOC_SCRATCH_BYTES
 * inside the library (one copy per GPU, held until the process ends).  The call allocates and
 * frees nothing.  Same arguments, kernels and results as mqa_decode_step with the library
 * heuristics.  A shape whose plan needs more than the buffer (see
 * mqa_decode_workspace_bytes_default; the partial states of a default plan stay under 4.3 MB for
 * any shape, the length schedule adds 4 bytes per sequence) returns MQA_ERR_SCRATCH_LIMIT with
 * nothing enqueued.
 * Nothing in the buffer has to start at zero (every slot that is read was written by the same
 * call), so no clearing is done.  All calls on one GPU share the buffer: calls that may overlap
 * in time on one GPU (different streams) race and must be serialised by the caller.
 */
#define MQA_NOALLOC_SCRATCH_BYTES (8u << 20)
int mqa_decode_step_noalloc(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                            int b, int h, int cap, int k, int v, mqa_dtype dt, float scale, void* stream);

/*
 * Measurement helpers: a plain streaming read (every 16-byte word of `src` is
 * loaded once; a checksum per workgroup goes to `sink`, >= 4096 floats) and a
 * plain copy.  They give the box's achievable read / copy bandwidth and a
 * known-size reference for scaling hardware byte counters.  bytes % 16 == 0.
 */
int mqa_stream_read(const void* src, size_t bytes, float* sink, void* stream);
int mqa_stream_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * Glue of the benchmark's decoder-only stack (pre-layernorm residual blocks, ReLU feed-forward,
 * tied token embedding: the model family of Section 4.1), so that a whole decoding loop runs in
 * this library.  Not part of the attention path.  All float32, row-major, device pointers.
 *   layernorm: y[r,:] = (x[r,:] - mean) / sqrt(var + eps), gain 1, bias 0 (biased variance)
 *   embed:     x[r,:] = E[tokens[r],:] + P[positions[r],:], E [vocab,d], P [max_pos,d]; indices outside
 *              the tables are clamped into them
 *   add:       a[i] += b[i];      relu: a[i] = max(a[i], 0)
 *   argmax:    out[r] = index of the largest x[r,:], the lowest index among equals (0 for a row that is
 *              all NaN or all -inf)
 * The feed-forward and the output logits are mqa_project_qkvo calls (LINEAR mode for x.W with
 * W [d,n]; O mode with h = 1 for x.E^T with E [vocab,d]).
 */
int mqa_stack_layernorm(const float* x, float* y, int rows, int d, float eps, void* stream);
int mqa_stack_embed(const int32_t* tokens, const int32_t* positions, const float* E, const float* P, float* x,
                    int rows, int d, int vocab, int max_pos, void* stream);
int mqa_stack_add(float* a, const float* b, size_t n, void* stream);
int mqa_stack_relu(float* a, size_t n, void* stream);
int mqa_stack_argmax(const float* x, int32_t* out, int rows, int n, void* stream);

const char* mqa_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MQA_H */
