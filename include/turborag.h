/*
 * turborag.h - C ABI of the MI355X (gfx950) TurboRAG online-prefill library.
 *
 * The library implements the data-parallel hot path of TurboRAG (arXiv 2410.07590):
 *   Sec. 3.4 step 5  contextual KV-cache formation  -> tr_plan, tr_kv_assemble[_batched], tr_kv_append[_batched],
 *                                                       tr_kv_assemble_append, tr_kv_assemble_raw
 *   Sec. 3.4 step 6  KV-cache prefill of the query   -> tr_prefill_attn[_batched], tr_prefill_attn_gather
 *   Sec. 3.4 step 7  one new token per request        -> tr_decode_attn
 *   Sec. 3.4 step 2  offline document prefill (attention part, independent attention of Sec. 3.2)
 *                                                     -> tr_chunk_prefill_attn
 *   Sec. 3.3         documents and query in one pass with the masks and position ids of inference
 *                                                     -> tr_sequence_plan, tr_sequence_prefill_attn
 *   Eq. 1            projections around the attention for the query tokens -> tr_linear
 *
 * Conventions (all entry points):
 *   - Tensors are token-major, contiguous: [rows, heads, head_dim], element type `tr_shape.dtype`
 *     (TR_BF16: bfloat16 bit patterns; TR_F32: IEEE float).  Tensor pointers are DEVICE pointers owned by
 *     the caller; the library never frees them and keeps none past the call, except that a tr_store
 *     records (does not copy) the two store base pointers.
 *   - Small index arrays marked "host" are HOST pointers, consumed before the call returns.
 *     Arrays marked "device" are device pointers read by the kernels.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All GPU work is enqueued on
 *     it; no call synchronises.  Arguments are validated on the host before anything is enqueued; on error
 *     nothing has been enqueued.
 *   - Every function returns a tr_status (0 = TR_OK, negative = error).  tr_last_error() returns a
 *     thread-local message for the last error on the calling thread.  Nothing throws, aborts or prints.
 *   - Results are deterministic: same inputs, same bits (no atomics in any reduction).  How a launch is cut into
 *     workgroups depends only on the shapes and lengths passed in; the library reads no environment variable
 *     (tr_set_tuning is the one, explicit, way to override the launch policy).
 *   - RoPE follows Eq. 3: pair m of a head is turned by pos * theta_m, theta_m = rope_base^(-2m/head_dim).
 *     TR_ROPE_INTERLEAVED: pair m = channels (2m, 2m+1), the layout Eq. 3 prints.  TR_ROPE_HALF: pair m =
 *     channels (m, m + head_dim/2), the layout in which the released weights of the models of Sec. 4 keep
 *     their heads.  Queries, stored keys and new keys of one shape all use that shape's layout.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - Supported shapes: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads; row counts below 2^31.
 */
#ifndef TURBORAG_H
#define TURBORAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TR_OK = 0,
    TR_ERR_INVALID_ARG = -1,  /* null pointer, negative count, inconsistent lengths */
    TR_ERR_BAD_CHUNK_ID = -2, /* chunk id outside [0, n_chunks) of the store */
    TR_ERR_BAD_PLAN = -3,     /* offsets are not the prefix sum of the chunk lengths, or exceed capacity */
    TR_ERR_SHAPE = -4,        /* unsupported head_dim / head counts / dtype */
    TR_ERR_UNSUPPORTED = -5,  /* valid request the library does not implement */
    TR_ERR_HIP = -6,          /* a HIP runtime call failed (message holds hipGetErrorString) */
    TR_ERR_WORKSPACE = -7,    /* workspace missing, misaligned or too small */
    TR_ERR_NO_MEMORY = -8     /* host memory for the call's bookkeeping could not be allocated */
} tr_status;

typedef enum { TR_POS_COMPOSITE = 0, TR_POS_REORDERED = 1 } tr_pos_mode; /* Sec. 3.2 */
typedef enum { TR_F32 = 0, TR_BF16 = 1 } tr_dtype;
typedef enum { TR_ROPE_INTERLEAVED = 0, TR_ROPE_HALF = 1 } tr_rope_layout;

typedef struct tr_shape {
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t dtype;       /* tr_dtype */
    double rope_base;    /* 10000 in the paper's Eq. 3; a parameter here */
    int32_t rope_layout; /* tr_rope_layout */
    int32_t reserved;    /* must be 0 */
} tr_shape;

typedef struct tr_store tr_store; /* opaque: the per-chunk KV database of Sec. 3.4 step 2, device resident */

/* Message for the last error returned on this thread ("" if none).  Never NULL. */
const char* tr_last_error(void);

/* ---- the chunk KV store ---------------------------------------------------------------------------------
 * k_store, v_store: device [store_rows, n_kv_heads, head_dim].  Keys are stored ALREADY ROTATED at their
 * chunk-local positions 0..len-1 (what the offline prefill of Sec. 3.4 step 2 writes; see
 * tr_chunk_prefill_attn's k_rot_out).  chunk_row_start: host [n_chunks+1], non-decreasing, chunk c owns rows
 * [chunk_row_start[c], chunk_row_start[c+1]) (empty chunks allowed).  The table is copied; the two device
 * pointers are recorded, not copied, and must outlive the store.  No GPU work.
 * Errors: TR_ERR_INVALID_ARG (also an unknown rope layout), TR_ERR_SHAPE. */
int tr_store_create(const tr_shape* shape, const void* k_store, const void* v_store,
                    const int64_t* chunk_row_start, int32_t n_chunks, tr_store** out);
int tr_store_destroy(tr_store* store);

/* ---- gather plan and position ids (Sec. 3.2) ----------------------------------------------------------------
 * Host only.  For the retrieved ids in order: offsets[i] = total length of the chunks before i,
 * offsets[n] = n_doc.  pos_ids (optional, may be NULL): the RoPE position id of every assembled document
 * row - composite: the chunk-local index t; reordered: offsets[i] + t.  pos_capacity = entries available in
 * pos_ids.  Errors: TR_ERR_BAD_CHUNK_ID; TR_ERR_BAD_PLAN if n_doc > pos_capacity (pos_ids non-NULL) or
 * n_doc >= 2^31. */
int tr_plan(const tr_store* store, const int32_t* chunk_ids /*host [n]*/, int32_t n, int32_t pos_mode,
            int64_t* offsets /*host out [n+1]*/, int32_t* pos_ids /*host out [n_doc] or NULL*/,
            int64_t pos_capacity);

/* ---- contextual KV-cache formation (Sec. 3.4 step 5; Sec. 3.2) --------------------------------------------
 * out_k/out_v: device [out_capacity_rows, n_kv_heads, head_dim].  Rows [offsets[i], offsets[i+1]) receive
 * chunk chunk_ids[i]:  out_v <- V (copy, both modes);
 *   composite:  out_k <- K' (copy: keys keep their chunk-local positions);
 *   reordered:  out_k <- R(offsets[i]) K' (Eq. 3 rotation by the chunk's offset, so the key stored at local
 *               position t ends at global position offsets[i]+t; computed in fp64, rounded once).
 * offsets: host [n_chunks+1]; must equal the plan tr_plan returns (exclusive prefix sum of the chunk
 * lengths), else TR_ERR_BAD_PLAN; offsets[n_chunks] must be <= out_capacity_rows.  Duplicated ids are legal.
 * n_chunks == 0 is a no-op.  One pass: every byte is read once and written once. */
int tr_kv_assemble(const tr_store* store, const int32_t* chunk_ids /*host*/, const int64_t* offsets /*host*/,
                   int32_t n_chunks, int32_t pos_mode, void* out_k, void* out_v, int64_t out_capacity_rows,
                   void* stream);

/* The same formation from a store whose k rows are UN-rotated keys (Sec. 3.2: keeping K of Eq. 1 and applying
 * the position encoding after concatenation; the store handle is created the same way and simply holds raw
 * keys).  Rows [offsets[i], offsets[i+1]) receive chunk chunk_ids[i]: out_v <- V (copy); out_k <- R(p) K with the
 * position id p = t (composite) or offsets[i] + t (reordered) of row t of the chunk, in fp64, rounded once - one
 * rounding where the pre-rotated store has two.  Arguments, plan check and errors as for tr_kv_assemble. */
int tr_kv_assemble_raw(const tr_store* store, const int32_t* chunk_ids /*host*/, const int64_t* offsets /*host*/,
                       int32_t n_chunks, int32_t pos_mode, void* out_k, void* out_v, int64_t out_capacity_rows,
                       void* stream);

/* Batched form: request r retrieves chunk_ids[cu_chunks[r] .. cu_chunks[r+1]) and owns cache rows
 * [cache_row_start[r], cache_row_start[r+1]) of out_k/out_v; its documents fill the first n_doc_r rows of
 * that range (the plan is computed here), with pos_modes[r] per request.  All index arrays are host arrays.
 * TR_ERR_BAD_PLAN when a request's documents do not fit its row range or the ranges exceed the capacity. */
int tr_kv_assemble_batched(const tr_store* store, const int32_t* chunk_ids, const int32_t* cu_chunks /*[n_req+1]*/,
                           const int32_t* pos_modes /*[n_req]*/, const int64_t* cache_row_start /*[n_req+1]*/,
                           int32_t n_req, void* out_k, void* out_v, int64_t out_capacity_rows, void* stream);

/* Query tokens' own K/V into the cache (the cache holds K' and V of every token, text after Eq. 4):
 * cache_k[dst_row+i] <- R(q_pos[i]) k_new[i] (fp64, rounded once), cache_v[dst_row+i] <- v_new[i].
 * k_new/v_new: device [n_q, n_kv_heads, head_dim] raw; q_pos: device int32 [n_q] position ids. */
int tr_kv_append(const tr_shape* shape, const void* k_new, const void* v_new, const int32_t* q_pos /*device*/,
                 int32_t n_q, void* cache_k, void* cache_v, int64_t dst_row, int64_t cache_capacity_rows,
                 void* stream);

/* Assemble and append of ONE request in a single launch (Sec. 3.4 step 5 followed by the query tokens' own rows):
 * exactly tr_kv_assemble(store, chunk_ids, offsets, n_chunks, pos_mode, out_k, out_v, ...) followed by
 * tr_kv_append(shape, k_new, v_new, q_pos, n_q, out_k, out_v, dst_row = offsets[n_chunks], ...), same results bit
 * for bit, one kernel instead of two.  out_capacity_rows must hold n_doc + n_q rows.  Same errors as those two. */
int tr_kv_assemble_append(const tr_store* store, const int32_t* chunk_ids /*host*/, const int64_t* offsets /*host*/,
                          int32_t n_chunks, int32_t pos_mode, const void* k_new, const void* v_new,
                          const int32_t* q_pos /*device*/, int32_t n_q, void* out_k, void* out_v,
                          int64_t out_capacity_rows, void* stream);

/* Batched form: tokens packed [cu_q[n_req], ...]; request r's n_q_r tokens go to the LAST n_q_r rows of its
 * cache range [cache_row_start[r], cache_row_start[r+1]). */
int tr_kv_append_batched(const tr_shape* shape, const void* k_new, const void* v_new, const int32_t* q_pos /*device*/,
                         const int32_t* cu_q /*host [n_req+1]*/, const int64_t* cache_row_start /*host [n_req+1]*/,
                         int32_t n_req, void* cache_k, void* cache_v, int64_t cache_capacity_rows, void* stream);

/* ---- KV-cache prefill of the query (Sec. 3.4 step 6; Eq. 2, Eq. 4) ---------------------------------------
 * q: device [n_q, n_q_heads, head_dim] RAW queries; they are rotated in the kernel at q_pos (Eq. 3; the ids
 * differ from the cache row index under composite positions, which is why both q_pos and kv_len are
 * arguments).  k, v: device [kv_len, n_kv_heads, head_dim], the assembled cache whose last n_q rows are the
 * query tokens themselves.  Query token i attends cache rows j <= kv_len - n_q + i (all documents, causal
 * among the query tokens); scores are scaled by 1/sqrt(head_dim); masked keys get zero weight.
 * out: device [n_q, n_q_heads, head_dim].  TR_BF16: bf16 MFMA with fp32 accumulation and fp32 softmax;
 * TR_F32: fp32 throughout.
 * workspace: device scratch of at least tr_prefill_attn_workspace_size() bytes, 256-byte aligned, used for
 * split-KV partial results; its contents are undefined afterwards.  n_q == 0 is a no-op.
 * Errors: TR_ERR_INVALID_ARG (kv_len < n_q, null pointers), TR_ERR_SHAPE, TR_ERR_WORKSPACE. */
size_t tr_prefill_attn_workspace_size(const tr_shape* shape, int32_t n_q, int64_t kv_len);
int tr_prefill_attn(const tr_shape* shape, const void* q, const void* k, const void* v,
                    const int32_t* q_pos /*device*/, int32_t n_q, int64_t kv_len, void* out,
                    void* workspace, size_t workspace_bytes, void* stream);

/* The same call for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  tr_prefill_attn's split-KV partial results go to a file-scope device array of
 * tr_prefill_attn_static_scratch_bytes() = 32 MiB inside the library instead of a caller's workspace (each GPU the
 * library runs on holds that array until the process ends); the call performs no hipMalloc / hipFree and uses no
 * allocating library routine.  Arguments, results (bit for bit) and errors as for tr_prefill_attn, plus
 * TR_ERR_WORKSPACE when the shape needs more scratch than the array holds (then nothing is enqueued; use
 * tr_prefill_attn).  Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race on it; calls on one stream are ordered and safe.  Nothing in the array has to be cleared between
 * calls: each call writes every partial row it reads. */
size_t tr_prefill_attn_static_scratch_bytes(void);
int tr_prefill_attn_static(const tr_shape* shape, const void* q, const void* k, const void* v,
                           const int32_t* q_pos /*device*/, int32_t n_q, int64_t kv_len, void* out, void* stream);

/* Batched form (one launch for many requests): q/out packed over requests by cu_q; request r's cache is rows
 * [cache_row_start[r], cache_row_start[r+1]) of k/v (kv_len_r = the range length, its last n_q_r rows are
 * the request's query tokens); q_pos packed like q.  Index arrays are host arrays. */
size_t tr_prefill_attn_batched_workspace_size(const tr_shape* shape, const int32_t* cu_q,
                                              const int64_t* cache_row_start, int32_t n_req);
int tr_prefill_attn_batched(const tr_shape* shape, const void* q, const void* k, const void* v,
                            const int32_t* q_pos /*device*/, const int32_t* cu_q /*host*/,
                            const int64_t* cache_row_start /*host*/, int32_t n_req, void* out,
                            void* workspace, size_t workspace_bytes, void* stream);

/* ---- the same prefill without waiting for the assembled document rows (Sec. 3.2, Sec. 3.4 steps 5-6) ---------
 * Attention of the n_q query tokens over the request's retrieved chunks, read where they lie in the store, and
 * over the query tokens' own rows, read from cache rows [n_doc, n_doc + n_q) of cache_k / cache_v (write them
 * first with tr_kv_append, dst_row = n_doc = offsets[n_chunks]; the document rows of the cache are NOT read, so
 * tr_kv_assemble may run at the same time on another stream).  Under TR_POS_REORDERED the stored keys sit at
 * chunk-local positions; instead of turning each key by its chunk's offset the kernel turns the query by minus
 * the offset, once per chunk, which gives the same scores (relative-position property of Eq. 3).  Result: what
 * tr_prefill_attn computes on the assembled cache, up to the rounding of the re-rotated keys to the storage
 * type, which this path skips.  chunk_ids, offsets, pos_mode as for tr_kv_assemble.  TR_BF16 only
 * (TR_ERR_UNSUPPORTED otherwise, and for more than 95 non-empty chunks in a request). */
size_t tr_prefill_attn_gather_workspace_size(const tr_store* store, const int32_t* chunk_ids /*host*/,
                                             const int64_t* offsets /*host*/, int32_t n_chunks, int32_t pos_mode, int32_t n_q);
int tr_prefill_attn_gather(const tr_store* store, const int32_t* chunk_ids /*host*/, const int64_t* offsets /*host*/,
                           int32_t n_chunks, int32_t pos_mode, const void* q, const void* cache_k, const void* cache_v,
                           const int32_t* q_pos /*device*/, int32_t n_q, int64_t cache_capacity_rows, void* out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ---- decode step over the assembled cache (Sec. 3.4 step 7: answer generation reuses the cache) -----------
 * One new token per request, for a batch of requests: q, out: device [n_req, n_q_heads, head_dim]; q_pos:
 * device [n_req]; request r's cache is rows [cache_row_start[r], cache_row_start[r+1]) of k/v (host array),
 * and its LAST row is the new token itself (append it first with tr_kv_append[_batched]); the token attends
 * every row of its range.  Same arithmetic as tr_prefill_attn with n_q = 1; the kernel behind it lets the
 * waves of a workgroup split the keys instead of the rows, because the g rows of a KV head cannot fill a
 * workgroup.  An empty range is an error (TR_ERR_INVALID_ARG).  Workspace as for tr_prefill_attn. */
size_t tr_decode_attn_workspace_size(const tr_shape* shape, const int64_t* cache_row_start /*host*/, int32_t n_req);
int tr_decode_attn(const tr_shape* shape, const void* q, const void* k, const void* v, const int32_t* q_pos /*device*/,
                   const int64_t* cache_row_start /*host [n_req+1]*/, int32_t n_req, void* out,
                   void* workspace, size_t workspace_bytes, void* stream);

/* ---- offline document prefill, attention part (Sec. 3.4 step 2; independent attention, Sec. 3.2) ----------
 * Chunks packed on one token axis: q device [total_tokens, n_q_heads, d], k, v device
 * [total_tokens, n_kv_heads, d], all RAW; cu_chunk_lens: DEVICE int32 [n_chunks+1], cu[0] = 0,
 * cu[n_chunks] = total_tokens, chunk c owns rows [cu[c], cu[c+1]).  Token t of chunk c attends rows
 * cu[c] .. t of its own chunk only (block-diagonal causal mask); q and k are rotated at the chunk-local
 * position t - cu[c] (Eq. 3).  out: device [total_tokens, n_q_heads, d].
 * k_rot_out: device [total_tokens, n_kv_heads, d], REQUIRED: receives K' = R(t - cu[c]) k (fp64, rounded
 * once) - the keys the store keeps; it may alias k (in-place).  The attention reads K' from it.
 * max_chunk_len: an upper bound on the chunk lengths (sizes the position table).
 * workspace: at least tr_chunk_prefill_attn_workspace_size() bytes, 256-byte aligned. */
size_t tr_chunk_prefill_attn_workspace_size(const tr_shape* shape, int64_t total_tokens, int32_t max_chunk_len);
int tr_chunk_prefill_attn(const tr_shape* shape, const void* q, const void* k, const void* v,
                          const int32_t* cu_chunk_lens /*device*/, int32_t n_chunks, int64_t total_tokens,
                          int32_t max_chunk_len, void* out, void* k_rot_out,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ---- one pass over a packed sequence [chunk_1 .. chunk_k, tail] (Sec. 3.3: fine-tuning runs with the attention
 * mask and position ids of inference; also a whole prefill, documents and query, in one call) ---------------------
 * tr_sequence_plan (host): token t of chunk c gets seg_start = first row of c and pos = t - start (composite) or t
 * (reordered) (Sec. 3.2); the n_tail query/answer tokens get seg_start = 0 and pos = tail_start + i, where
 * tail_start < 0 selects the default (the longest chunk's length under composite positions, n_doc under reordered).
 * seg_start, pos: host int32 arrays of `capacity` entries; TR_ERR_BAD_PLAN if the sequence is longer.
 * tr_sequence_prefill_attn: q [T, n_q_heads, d], k, v [T, n_kv_heads, d] raw, seg_start, pos device int32 [T]
 * (0 <= seg_start[t] <= t; values outside are clamped).  k_rot_out <- R(pos[t]) k[t] (fp64, one rounding; required,
 * may alias k); token t attends rows seg_start[t] .. t of k_rot_out / v with the query rotated at pos[t];
 * out [T, n_q_heads, d].  With seg_start = chunk starts and chunk-local pos this is tr_chunk_prefill_attn.
 * seg_start_host: NULL, or a HOST copy of seg_start (what tr_sequence_plan wrote), read before the call returns and
 * used only to balance the launch: tokens whose key range is long against the chip's fair share (query tokens behind
 * many documents) have it cut into pieces that run as separate workgroups and are merged afterwards.  The result does
 * not depend on it beyond rounding; if it differs from the device array only speed is lost.  workspace: at least
 * tr_sequence_prefill_attn_workspace_size() bytes (0 without the host copy, for fp32, and when nothing is cut),
 * 256-byte aligned, else TR_ERR_WORKSPACE. */
int tr_sequence_plan(const int32_t* chunk_lens /*host*/, int32_t n_chunks, int32_t n_tail, int32_t pos_mode, int32_t tail_start,
                     int32_t* seg_start /*host out*/, int32_t* pos /*host out*/, int64_t capacity);
size_t tr_sequence_prefill_attn_workspace_size(const tr_shape* shape, const int32_t* seg_start_host /*host, may be NULL*/,
                                               int64_t total_tokens);
int tr_sequence_prefill_attn(const tr_shape* shape, const void* q, const void* k, const void* v,
                             const int32_t* seg_start /*device*/, const int32_t* pos /*device*/,
                             const int32_t* seg_start_host /*host, may be NULL*/, int64_t total_tokens,
                             void* out, void* k_rot_out, void* workspace, size_t workspace_bytes, void* stream);

/* ---- projections around the attention for the query tokens (Eq. 1: Q, K, V = X W; the output projection is the
 * same product) ---------------------------------------------------------------------------------------------------------
 * For j < n_out (1 .. 4 weights that share x, e.g. query, key and value in one launch):
 *   y[j][m, n] = sum_k x[m, k] w[j][n, k],
 * x device [M, K]; w[j] device [n_features[j], K] (the layout of a linear layer's weight: out_features x in_features);
 * y[j] device [M, n_features[j]]; all bf16, fp32 accumulation, one rounding of the result.  w, y: HOST arrays of
 * n_out device pointers, n_features: host array, all consumed before the call returns.
 * M <= 128 (the weights are streamed from HBM exactly once, which is what bounds a product with so few rows; more
 * rows: TR_ERR_UNSUPPORTED - that is a library GEMM's work); every n_features[j] a multiple of 32 and K a multiple
 * of 16 (else TR_ERR_SHAPE); x and w[j] 16-byte aligned.  M == 0 is a no-op.  workspace:
 * tr_linear_workspace_size() bytes (fp32 partial sums of the slices of k that run in different workgroups; 0 when
 * there is one slice), 256-byte aligned, else TR_ERR_WORKSPACE. */
size_t tr_linear_workspace_size(int32_t M, int32_t n_out, const int32_t* n_features /*host*/, int32_t K);
int tr_linear(const void* x, int32_t M, int32_t K, int32_t n_out, const void* const* w /*host*/, void* const* y /*host*/,
              const int32_t* n_features /*host*/, void* workspace, size_t workspace_bytes, void* stream);

/* ---- launch-policy override for tests and sweeps -------------------------------------------------------------------------
 * Sets a process-wide override of one value of the launch policy; value 0 restores the default.  Names: "wg_rows"
 * (packed rows per attention workgroup: 32, 128, 256), "target_items", "min_split_keys", "asm_span", "bd_piece_tiles",
 * "bd_slots", "lin_split", "lin_msplit".  Results never depend on these beyond the rounding of a different
 * summation order; a *_workspace_size() query and the call it sizes must see the same overrides.  Not meant for
 * concurrent use with running calls.  Errors: TR_ERR_INVALID_ARG (unknown name, negative value). */
int tr_set_tuning(const char* name, int32_t value);

/* Measurement aid, not a step of the method: the rate at which this chip issues the matrix instruction of the
 * attention kernels (v_mfma_f32_32x32x16_bf16, operands read from LDS, 8 waves on each of the 256 compute units, no
 * softmax, no global memory traffic).  A caller times the launch with events on `stream` and divides *flops (host,
 * out: multiply-adds x 2 of the launch) by the duration: that is the ceiling the MFMA-bound rows of a roofline are
 * really up against, next to the published peak.  random_operands != 0 fills the operands with bf16 values of random
 * sign and mantissa (magnitude 0.5..4), the kind of data attention feeds the instruction; 0 uses a few constants,
 * which draw less power and clock higher.  sink: device, at least tr_probe_mfma_loop_sink_bytes() bytes, overwritten.
 * iters: loop trips of 8 instructions per wave, 1 .. 2^24.  Errors: TR_ERR_INVALID_ARG, TR_ERR_HIP. */
size_t tr_probe_mfma_loop_sink_bytes(void);
int tr_probe_mfma_loop(int32_t iters, int32_t random_operands, float* sink, size_t sink_bytes, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TURBORAG_H */
