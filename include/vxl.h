/*
 * vxl -- chunk-based pre-filling attention and bi-level KV decoding on one MI355X (gfx950).
 *
 * C ABI of libvxl.so.  The operations are those of Video-XL-2's task-aware KV
 * sparsification (paper: Method, "Efficiency Optimization"):
 *
 *   vxl_chunk_prefill      "Chunk-based Pre-filling" and the caption of its figure
 *   vxl_chunk_score_topk   "Bi-level KVs Decoding": relevance score per chunk, selection
 *   vxl_gather_bilevel_kv  "Bi-level KVs Decoding": selective reload + concatenation
 *   vxl_bilevel_decode     "Bi-level KVs Decoding": generation over the mixed KV set
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the layout arrays given to
 *     vxl_layout_create are HOST pointers (copied; the caller may free them afterwards).
 *   - Tensors are dense, row-major, in the storage dtype of the descriptor:
 *       Q, O   [n_q_heads,  n_tokens, head_dim]      K, V [n_kv_heads, n_tokens, head_dim]
 *       Qd, Od [batch, n_q_tokens, n_q_heads, head_dim]
 *       Kmix, Vmix [batch, n_kv_heads, l_cap, head_dim]
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - The four hot calls are asynchronous on `stream` (a hipStream_t; NULL = default stream),
 *     never synchronise and never allocate: scratch comes from the caller's workspace, sized by
 *     vxl_workspace_bytes.  Inputs are never written.  Outputs and workspace must not alias
 *     inputs.  Base pointers must be 16-byte aligned.
 *   - Every call returns a vxl_status.  Argument errors are detected on the host before
 *     anything is launched; a failing HIP call is reported as VXL_ERR_HIP (the text of the
 *     last one is available from vxl_last_error).  The cross-check and measurement hooks of the
 *     library are declared in vxl_debug.h, not here.
 *   - Supported: dtype F32 or BF16; head_dim 64 or 128; n_q_heads a multiple of n_kv_heads;
 *     n_chunks <= VXL_MAX_CHUNKS.  BF16 runs on the matrix cores with fp32 accumulation; F32
 *     runs on the vector ALUs in fp32.
 */
#ifndef VXL_H
#define VXL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VXL_MAX_CHUNKS 4096

typedef enum {
    VXL_OK = 0,
    VXL_ERR_INVALID_ARG = 1,   /* null pointer, inconsistent sizes, malformed layout */
    VXL_ERR_UNSUPPORTED = 2,   /* dtype / head_dim / chunk count outside the supported set */
    VXL_ERR_WORKSPACE = 3,     /* workspace missing or smaller than vxl_workspace_bytes */
    VXL_ERR_HIP = 4,           /* a HIP runtime call failed */
    VXL_ERR_ALLOC = 5          /* host or device memory could not be allocated (handle-creating calls only) */
} vxl_status;

typedef enum { VXL_F32 = 0, VXL_BF16 = 1 } vxl_dtype;

typedef enum {
    VXL_OP_PREFILL = 0,
    VXL_OP_SCORE_TOPK = 1,
    VXL_OP_GATHER = 2,
    VXL_OP_DECODE = 3,
    VXL_OP_SCORE_MASS = 4,
    VXL_OP_DECODE_INPLACE = 5
} vxl_op;

/*
 * Heads, element type and memory layout of the per-layer tensors Q, O (query heads) and K, V (KV
 * heads) over the N tokens of a prompt.  Row (head h, token i) of a tensor starts at element
 * h * stride_head + i * stride_tok and holds head_dim contiguous elements.  All four strides 0
 * (the default) selects the dense head-major layout [heads, N, head_dim]; token-major storage
 * [N, heads, head_dim], as a projection writes it, is stride_head = head_dim, stride_tok =
 * heads * head_dim.  Strides are in elements, each a multiple of 16 bytes' worth (8 for bf16, 4
 * for fp32), stride_tok >= head_dim, and either all four are 0 or all four are set; rows must
 * not overlap (not checked).  O is written in Q's layout.  The mixed KVs, the pooled sparse KVs,
 * the decode queries Qd and every other buffer keep the dense layouts stated at their calls.
 */
typedef struct {
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t dtype;           /* vxl_dtype */
    float softmax_scale;     /* 0 selects 1/sqrt(head_dim); otherwise must be > 0 */
    int32_t reserved;        /* must be 0 */
    int64_t q_stride_head, q_stride_tok;     /* Q and O */
    int64_t kv_stride_head, kv_stride_tok;   /* K and V */
} vxl_attn_desc;

typedef struct vxl_layout vxl_layout;   /* opaque: chunking + kept-token lists of one prompt */
typedef void* vxl_stream;               /* a hipStream_t */

/*
 * Token layout of one prompt ("Chunk-based Pre-filling": the visual token sequence is divided
 * into chunks; the kept tokens of a chunk are the ones later chunks may attend to, in the paper
 * the timestamp tokens.  "Bi-level KVs Decoding": the same chunking indexes the dense and the
 * sparse KVs; here the sparse KVs of a chunk are its kept rows).
 *   n_tokens        N, total tokens; ids 0..n_prefix-1 are the system/text prefix
 *   chunk_bounds    host int32 [n_chunks+1], strictly increasing, [0]==n_prefix, [n_chunks]==N
 *   sparse_offsets  host int32 [n_chunks+1], CSR offsets, [0]==0, non-decreasing
 *   sparse_idx      host int32 [sparse_offsets[n_chunks]], absolute token ids, strictly
 *                   ascending inside a chunk and inside that chunk's bounds (may be NULL when
 *                   no token is kept)
 * The handle owns device copies of these arrays and the pre-filling tile schedule derived from
 * them; creating it allocates device memory and synchronises `stream`.  n_chunks may be 0.
 * Errors: VXL_ERR_INVALID_ARG for any violated condition above, VXL_ERR_UNSUPPORTED for
 * n_chunks > VXL_MAX_CHUNKS, VXL_ERR_ALLOC when the handle or its device memory cannot be
 * allocated, VXL_ERR_HIP for any other failing runtime call.
 */
vxl_status vxl_layout_create(int32_t n_tokens, int32_t n_prefix, int32_t n_chunks,
                             const int32_t* chunk_bounds, const int32_t* sparse_offsets,
                             const int32_t* sparse_idx, vxl_stream stream, vxl_layout** out);
/* The same with the sliding chunk window of "Chunk-based Pre-filling" (the chunk to process is
 * placed by a window that advances by a step smaller than its size, so it overlaps the end of
 * the preceding chunk and sees that part in full detail; the chunks of this interface are the
 * window's steps): the `window` >= 0 tokens right before chunk c, clipped at the end of the
 * prefix, are visible to every token of chunk c as dense rows, in addition to the prefix and
 * the kept tokens of earlier chunks; a kept token inside that range is seen once.
 * window == 0 is vxl_layout_create.  Only vxl_chunk_prefill reads the window; scoring, gather
 * and decode depend on the bounds and the kept lists alone.
 * Errors: as vxl_layout_create; VXL_ERR_INVALID_ARG for window < 0. */
vxl_status vxl_layout_create_windowed(int32_t n_tokens, int32_t n_prefix, int32_t n_chunks,
                                      const int32_t* chunk_bounds, const int32_t* sparse_offsets,
                                      const int32_t* sparse_idx, int32_t window, vxl_stream stream,
                                      vxl_layout** out);
vxl_status vxl_layout_destroy(vxl_layout* layout);

/* Bytes of workspace the given hot call needs (0 on invalid arguments, and for VXL_OP_GATHER,
 * which needs none).  batch, n_q_tokens and l_cap are read by the ops that take them (SCORE_TOPK:
 * batch; SCORE_MASS: batch, n_q_tokens; DECODE: batch, n_q_tokens, l_cap).  The decode call is
 * sized by the capacity of the mixed buffers it will be given, l_cap, and not by the number k of
 * dense chunks, because it takes no layout: l_cap = vxl_mixed_kv_capacity(layout, k) for the
 * caller's k, or anything larger.  layout may be NULL for VXL_OP_DECODE. */
size_t vxl_workspace_bytes(vxl_op op, const vxl_layout* layout, const vxl_attn_desc* desc,
                           int32_t batch, int32_t n_q_tokens, int32_t l_cap);

/* Upper bound of the mixed-KV length when at most k chunks are dense:
 * n_prefix + all kept rows + the k largest (chunk length - kept count).  k is clamped to
 * [0, n_chunks]. */
int32_t vxl_mixed_kv_capacity(const vxl_layout* layout, int32_t k);

/* Number of (query, key) pairs the pre-filling mask allows, in closed form; the effective
 * FLOP count of vxl_chunk_prefill is 4 * head_dim * n_q_heads times this. */
int64_t vxl_prefill_pair_count(const vxl_layout* layout);

/*
 * Chunk-based pre-filling attention ("Chunk-based Pre-filling"; figure caption: the chunk
 * being processed attends to itself, to the historical kept tokens and to the system prompt).
 * For query head h and token i of chunk c:
 *   O[h,i,:] = softmax over j in ([0,P) u kept(0..c-1) u [b_c, i]) of scale*q_i.k_j, times V;
 * prefix tokens attend causally to the prefix.  Internally the kept K/V rows are first
 * compacted (prefix rows, then kept rows in chunk order) so that the history of chunk c is a
 * prefix of one contiguous buffer.
 *   Q, K, V, O   device, layouts above;  LSE device float [n_q_heads, n_tokens] or NULL
 *                (natural-log sum-exp of the scaled logits of each row)
 * Errors: VXL_ERR_INVALID_ARG, VXL_ERR_UNSUPPORTED, VXL_ERR_WORKSPACE, VXL_ERR_HIP.
 */
vxl_status vxl_chunk_prefill(const vxl_layout* layout, const vxl_attn_desc* desc,
                             const void* Q, const void* K, const void* V, void* O, float* LSE,
                             void* workspace, size_t workspace_bytes, vxl_stream stream);

/*
 * Relevance score of every chunk for every query and selection of the dense chunks
 * ("Bi-level KVs Decoding": a relevance score for each video chunk, here by the
 * attention-score mechanism).  score[b,c] = mean over (t, h, j in chunk c) of
 * scale * Qd[b,t,h,:].K[g(h),j,:], computed as scale/Hkv * sum_g mean_q[b,g,:].mean_k[g,c,:].
 * The min(k, n_chunks) best chunks are selected, ties going to the lower chunk id.
 *   Qd          device [batch, n_q_tokens, n_q_heads, head_dim]
 *   K           device dense keys (read only when kbar_ready == 0)
 *   kbar        device float [n_kv_heads, n_chunks, head_dim] per-chunk mean keys: written when
 *               kbar_ready == 0, read as a cache when kbar_ready != 0; NULL uses the workspace
 *   workspace   always needed (it also holds the mean queries), sized by VXL_OP_SCORE_TOPK
 *   topk_idx    device int32 [batch, min(k, n_chunks)], best first (may be NULL if k == 0)
 *   dense_mask  device uint8 [batch, n_chunks], 1 = dense
 *   scores      device float [batch, n_chunks] or NULL
 */
vxl_status vxl_chunk_score_topk(const vxl_layout* layout, const vxl_attn_desc* desc,
                                const void* Qd, int32_t batch, int32_t n_q_tokens,
                                const void* K, int32_t k, float* kbar, int32_t kbar_ready,
                                int32_t* topk_idx, uint8_t* dense_mask, float* scores,
                                void* workspace, size_t workspace_bytes, vxl_stream stream);

/*
 * The same selection with the other reading of the attention-score relevance oracle
 * ("Bi-level KVs Decoding" names the attention score mechanism without a formula): the softmax
 * attention MASS on the chunk,
 *   p[b,t,h,j]  = softmax over all tokens j (prefix and every chunk) of scale * Qd[b,t,h,:].K[g(h),j,:]
 *   score[b,c]  = mean over (t, h) of sum over j in chunk c of p[b,t,h,j]
 * The prefix takes part in the softmax but is not scored.  Unlike the mean-logit score this one
 * is not normalised by the chunk length, and there is no per-chunk summary to cache: every call
 * streams the dense keys once.  Arguments as vxl_chunk_score_topk (K is always read; workspace
 * sized by VXL_OP_SCORE_MASS).  Scores are computed in fp32 with fixed summation orders.
 */
vxl_status vxl_chunk_score_topk_mass(const vxl_layout* layout, const vxl_attn_desc* desc,
                                     const void* Qd, int32_t batch, int32_t n_q_tokens,
                                     const void* K, int32_t k, int32_t* topk_idx,
                                     uint8_t* dense_mask, float* scores, void* workspace,
                                     size_t workspace_bytes, vxl_stream stream);

/*
 * Reload and concatenate ("Bi-level KVs Decoding": dense KVs for the relevant chunks, sparse
 * KVs for the others, concatenated into the mixed KV set).  Row order of the mixed set: the
 * prefix, then the chunks in temporal order, rows ascending inside a chunk.
 *   dense_mask  device uint8 [batch, n_chunks]
 *   Kmix, Vmix  device [batch, n_kv_heads, l_cap, head_dim]; rows >= mix_len[b] are left
 *               untouched
 *   mix_len     device int32 [batch] (written)
 *   src_idx     device int32 [batch, l_cap] source token id of every mixed row, or NULL
 * No workspace.  l_cap must be at least vxl_mixed_kv_capacity(layout, k) for the k that produced
 * the mask.  The mask lives on the device, so the host can only check l_cap >= the capacity for
 * k = 0 (VXL_ERR_INVALID_ARG otherwise); a query whose mask selects more rows than l_cap holds is
 * reported on the device, never truncated: none of its rows is copied and mix_len[b] is set to
 * MINUS the number of rows it needs.  vxl_bilevel_decode treats a length <= 0 as an empty set
 * (O = 0, LSE = -inf), so the chain score -> gather -> decode needs no host check in between and
 * a caller finds the overflow in mix_len whenever it next looks.
 */
vxl_status vxl_gather_bilevel_kv(const vxl_layout* layout, const vxl_attn_desc* desc,
                                 const void* K, const void* V, const uint8_t* dense_mask,
                                 int32_t batch, void* Kmix, void* Vmix, int32_t l_cap,
                                 int32_t* mix_len, int32_t* src_idx, vxl_stream stream);

/*
 * Pooled sparse KVs ("Bi-level KVs Decoding": the dense KVs are chunked and a pooling operation on
 * every chunk yields its sparse KVs; the paper gives neither window nor stride).  Chunk c, which
 * the layout represents by s_c = sparse_offsets[c+1] - sparse_offsets[c] sparse rows, is cut into
 * s_c consecutive groups, group m = rows [floor(m*len_c/s_c), floor((m+1)*len_c/s_c)) of the
 * chunk, and pooled row sparse_offsets[c] + m is the arithmetic mean of the group's rows (K and V
 * alike; fp32 sums in row order, rounded once to the storage dtype).  The kept-token ids of the
 * layout are not read, only their counts.
 *   K, V      device dense [n_kv_heads, n_tokens, head_dim]
 *   Ksp, Vsp  device [n_kv_heads, S_total, head_dim] (written), S_total = sparse_offsets[n_chunks]
 * No workspace.  Errors: VXL_ERR_INVALID_ARG (null / misaligned / aliasing buffers),
 * VXL_ERR_UNSUPPORTED, VXL_ERR_HIP.
 */
vxl_status vxl_pool_sparse_kv(const vxl_layout* layout, const vxl_attn_desc* desc, const void* K,
                              const void* V, void* Ksp, void* Vsp, vxl_stream stream);

/*
 * vxl_gather_bilevel_kv with pooled sparse KVs: a chunk that is not dense contributes its pooled
 * rows Ksp/Vsp[:, sparse_offsets[c] .. sparse_offsets[c+1]) instead of its kept rows.  Lengths,
 * order and capacity are those of vxl_gather_bilevel_kv; src_idx (if given) holds the token id of
 * a dense row and -1 - (pooled row index) of a pooled row.
 */
vxl_status vxl_gather_bilevel_kv_pooled(const vxl_layout* layout, const vxl_attn_desc* desc,
                                        const void* K, const void* V, const void* Ksp,
                                        const void* Vsp, const uint8_t* dense_mask, int32_t batch,
                                        void* Kmix, void* Vmix, int32_t l_cap, int32_t* mix_len,
                                        int32_t* src_idx, vxl_stream stream);

/*
 * GQA decode attention over the mixed KV set ("Bi-level KVs Decoding"): every query token
 * attends to rows 0..mix_len[b]-1 of its mixed set; no mask among the query tokens.  Split-KV
 * partial results are merged by log-sum-exp in a fixed order (deterministic).
 *   Qd, O    device [batch, n_q_tokens, n_q_heads, head_dim];  LSE device float
 *            [batch, n_q_tokens, n_q_heads] or NULL
 *   mix_len  device int32 [batch]; entries above l_cap are read as l_cap, entries <= 0 (an empty
 *            set, or the overflow report of vxl_gather_bilevel_kv) give O = 0 and LSE = -inf
 */
vxl_status vxl_bilevel_decode(const vxl_attn_desc* desc, const void* Qd, int32_t batch,
                              int32_t n_q_tokens, const void* Kmix, const void* Vmix,
                              int32_t l_cap, const int32_t* mix_len, void* O, float* LSE,
                              void* workspace, size_t workspace_bytes, vxl_stream stream);

/*
 * Gather-free decode ("Bi-level KVs Decoding": generation attends to the dense KVs of the relevant
 * chunks and the sparse KVs of the others): the result of vxl_gather_bilevel_kv[_pooled] followed
 * by vxl_bilevel_decode, without building the mixed buffers.  A first pass writes only the row map
 * of every query (4 bytes per mixed row) and the lengths; the split-KV kernels then read the dense
 * rows from K / V and the sparse rows from Ksp / Vsp in place, through that map.  It saves the
 * gather's write and the re-read of 2 * n_kv_heads * mix_len * head_dim elements per query, and the
 * mixed buffers themselves.
 *   K, V        device dense keys / values of the layer (layout of the descriptor)
 *   Ksp, Vsp    device [n_kv_heads, S_total, head_dim] sparse rows in chunk order -- the pooled rows of
 *               vxl_pool_sparse_kv, or the kept rows compacted (consecutive sparse chunks are then
 *               contiguous, which is the fast case); both NULL: the kept rows are read where they
 *               lie in K / V, through the kept-token ids of the layout
 *   dense_mask  device uint8 [batch, n_chunks]
 *   l_cap       capacity of the row map per query, at least vxl_mixed_kv_capacity(layout, k) for the
 *               k that produced the mask; a query that needs more is reported as in
 *               vxl_gather_bilevel_kv (length = -(rows needed), O = 0, LSE = -inf)
 *   map_ready   0: build the row map and the lengths first (one more launch, a few microseconds);
 *               != 0: reuse those an earlier call with the same layout, mask, l_cap, batch and
 *               sparse source left in this workspace (and in mix_len, if given) -- the later
 *               tokens of a query, whose selection does not change.  n_q_tokens may differ from
 *               that call's (the question in one call, then one token per call) if the workspace
 *               is large enough for both.  A workspace that holds no such map must not be passed
 *               with map_ready != 0: its entries are used as row addresses unchecked.
 *   O, LSE      as vxl_bilevel_decode
 *   mix_len     device int32 [batch] (the mixed lengths: written when map_ready == 0, read
 *               otherwise) or NULL (they are then kept in the workspace)
 *   workspace   sized by vxl_workspace_bytes(VXL_OP_DECODE_INPLACE, layout, desc, batch, n_q_tokens, l_cap)
 * The set of rows a query attends to is exactly that of the gathered path; the summation order
 * differs, so results agree with it within the tolerance of the path, not bit for bit.
 * Errors: VXL_ERR_INVALID_ARG, VXL_ERR_UNSUPPORTED, VXL_ERR_WORKSPACE, VXL_ERR_HIP.
 */
vxl_status vxl_bilevel_decode_inplace(const vxl_layout* layout, const vxl_attn_desc* desc, const void* Qd,
                                      int32_t batch, int32_t n_q_tokens, const void* K, const void* V,
                                      const void* Ksp, const void* Vsp, const uint8_t* dense_mask,
                                      int32_t l_cap, int32_t map_ready, void* O, float* LSE,
                                      int32_t* mix_len, void* workspace, size_t workspace_bytes,
                                      vxl_stream stream);

/*
 * vxl_bilevel_decode for callers that cannot allocate device memory or carry a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-for-bit the same results as vxl_bilevel_decode, without the workspace pair:
 * the split-KV partial results go to an array of VXL_STATIC_SCRATCH_BYTES bytes that the library
 * holds in device memory (one per GPU it runs on, from the first call on that GPU until the
 * process ends).  The call allocates nothing and frees nothing; its first call on a device looks
 * up the array's address and sets kernel attributes.
 *   - A call whose partial results need more than VXL_STATIC_SCRATCH_BYTES (what
 *     vxl_workspace_bytes(VXL_OP_DECODE, ...) reports for the same arguments) is rejected with
 *     VXL_ERR_WORKSPACE before anything is launched; vxl_last_error says how much it needed.
 *   - Every call on a GPU shares that GPU's array: calls that may overlap (different streams,
 *     different threads) race on it; order them on one stream or use vxl_bilevel_decode with
 *     separate workspaces.  Nothing in the array has to start at zero (each call writes every
 *     value it later reads), so it is not cleared between calls.
 * Other errors as vxl_bilevel_decode.
 */
#define VXL_STATIC_SCRATCH_BYTES (32u << 20)
vxl_status vxl_bilevel_decode_static(const vxl_attn_desc* desc, const void* Qd, int32_t batch,
                                     int32_t n_q_tokens, const void* Kmix, const void* Vmix,
                                     int32_t l_cap, const int32_t* mix_len, void* O, float* LSE,
                                     vxl_stream stream);

/*
 * Offline (host-memory) bi-level KV store of one layer ("Bi-level KVs Decoding": both the dense
 * and the sparse KVs are stored in an offline memory and selectively reloaded for a query).
 * The store owns pinned host copies of the dense K/V [n_kv_heads, n_tokens, head_dim] and of the
 * sparse K/V [n_kv_heads, S_total, head_dim] (kept rows in chunk order, or the pooled rows of
 * vxl_pool_sparse_kv).
 *   vxl_kv_store_create   allocates the pinned memory (hipHostMalloc; synchronous, not a hot call)
 *   vxl_kv_store_offload  device -> host copies of K, V (read in the layout of the descriptor given
 *                         at creation; the host copy is dense) and Ksp, Vsp (sparse; may be NULL
 *                         when the layout keeps no rows), asynchronous on `stream`; the store may
 *                         be reloaded from once these copies have completed
 *   vxl_kv_store_reload   builds the mixed KV set of `batch` queries in DEVICE memory straight
 *                         from the host store, with the row order and lengths of
 *                         vxl_gather_bilevel_kv: one strided host -> device copy per run of rows
 *                         that are consecutive in one source, asynchronous on `stream`
 *       dense_mask     HOST uint8 [batch, n_chunks] (the caller has brought the selection back)
 *       Kmix, Vmix     device [batch, n_kv_heads, l_cap, head_dim]; rows >= length untouched
 *       mix_len_host   host int32 [batch] written before the call returns, or NULL
 *       mix_len        device int32 [batch] written by a one-block kernel on `stream` that carries
 *                      the lengths as launch arguments, or NULL (batch <= 256); reloads of one
 *                      store may be issued back to back, on one stream or on several
 *   Errors: VXL_ERR_INVALID_ARG (null pointers; a query whose mixed length exceeds l_cap --
 *   nothing is copied then), VXL_ERR_UNSUPPORTED, VXL_ERR_ALLOC (create), VXL_ERR_HIP.
 * The reload moves 2 * n_kv_heads * mix_len * head_dim * elem bytes per query over the host link;
 * on a side stream it overlaps the decode of another query.
 */
typedef struct vxl_kv_store vxl_kv_store;
vxl_status vxl_kv_store_create(const vxl_layout* layout, const vxl_attn_desc* desc, vxl_kv_store** out);
vxl_status vxl_kv_store_destroy(vxl_kv_store* store);
size_t vxl_kv_store_host_bytes(const vxl_kv_store* store);
vxl_status vxl_kv_store_offload(vxl_kv_store* store, const void* K, const void* V, const void* Ksp,
                                const void* Vsp, vxl_stream stream);
vxl_status vxl_kv_store_reload(vxl_kv_store* store, const uint8_t* dense_mask, int32_t batch,
                               void* Kmix, void* Vmix, int32_t l_cap, int32_t* mix_len_host,
                               int32_t* mix_len, vxl_stream stream);

const char* vxl_status_string(vxl_status s);
const char* vxl_last_error(void);   /* text of the last failing HIP call on this thread */
int vxl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VXL_H */
