// Host side of the C ABI: argument validation, gather plans, launch geometry.  No kernels here.
#include "tr_internal.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <functional>
#include <mutex>
#include <new>

// ---- errors ---------------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

int tr_fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}
void tr_clear_error() { g_err[0] = 0; }

extern "C" const char* tr_last_error(void) { return g_err; }

// ---- launch-policy overrides ----------------------------------------------------------------------------------------
static std::atomic<int> g_knob[TR_KNOB_COUNT];
static const char* const KNOB_NAMES[TR_KNOB_COUNT] = {"wg_rows", "target_items", "min_split_keys", "asm_span",
                                                      "bd_piece_tiles", "bd_slots", "lin_split", "lin_msplit"};

int tr_knob(int which, int dflt)
{
    const int v = g_knob[which].load(std::memory_order_relaxed);
    return v != 0 ? v : dflt;
}

extern "C" int tr_set_tuning(const char* name, int32_t value)
{
    tr_clear_error();
    if (!name) return tr_fail(TR_ERR_INVALID_ARG, "tr_set_tuning: name is NULL");
    if (value < 0) return tr_fail(TR_ERR_INVALID_ARG, "tr_set_tuning: value %d is negative", value);
    for (int i = 0; i < TR_KNOB_COUNT; ++i)
        if (strcmp(name, KNOB_NAMES[i]) == 0) {
            g_knob[i].store(value, std::memory_order_relaxed);
            return TR_OK;
        }
    return tr_fail(TR_ERR_INVALID_ARG, "tr_set_tuning: unknown name '%s'", name);
}

extern "C" int tr_probe_mfma_loop(int32_t iters, int32_t random_operands, float* sink, size_t sink_bytes, double* flops, void* stream)
{
    tr_clear_error();
    if (!sink || !flops) return tr_fail(TR_ERR_INVALID_ARG, "tr_probe_mfma_loop: sink or flops is NULL");
    if (iters < 1 || iters > (1 << 24)) return tr_fail(TR_ERR_INVALID_ARG, "tr_probe_mfma_loop: iters %d outside [1, 2^24]", iters);
    if (sink_bytes < tr_probe_mfma_loop_sink_bytes())
        return tr_fail(TR_ERR_INVALID_ARG, "tr_probe_mfma_loop: sink holds %zu bytes, %zu needed", sink_bytes, tr_probe_mfma_loop_sink_bytes());
    if (tr_launch_mfma_loop_probe(iters, random_operands != 0, sink, (hipStream_t)stream, flops) != 0)
        return tr_fail(TR_ERR_HIP, "tr_probe_mfma_loop: launch failed: %s", hipGetErrorString(hipGetLastError()));
    return TR_OK;
}

extern "C" size_t tr_probe_mfma_loop_sink_bytes(void) { return (size_t)TrChip::CUS * 512 * sizeof(float); }

// No C++ exception may cross the C boundary: the entry points run inside these.
template <class F> static int tr_guard_int(F&& f)
{
    try {
        return f();
    } catch (const std::bad_alloc&) {
        return tr_fail(TR_ERR_NO_MEMORY, "out of host memory");
    } catch (...) {
        return tr_fail(TR_ERR_INVALID_ARG, "unexpected C++ exception");
    }
}
template <class F> static size_t tr_guard_size(F&& f)
{
    try {
        return f();
    } catch (...) {
        return 0;
    }
}

int tr_check_shape(const tr_shape* s)
{
    if (!s) return tr_fail(TR_ERR_INVALID_ARG, "shape is NULL");
    if (s->dtype != TR_F32 && s->dtype != TR_BF16) return tr_fail(TR_ERR_SHAPE, "dtype %d is not TR_F32/TR_BF16", s->dtype);
    if (s->head_dim != 64 && s->head_dim != 128) return tr_fail(TR_ERR_SHAPE, "head_dim %d: only 64 and 128 are supported", s->head_dim);
    if (s->n_kv_heads < 1 || s->n_q_heads < 1 || s->n_q_heads % s->n_kv_heads != 0)
        return tr_fail(TR_ERR_SHAPE, "n_q_heads %d must be a positive multiple of n_kv_heads %d", s->n_q_heads, s->n_kv_heads);
    if (s->n_q_heads / s->n_kv_heads > 128) return tr_fail(TR_ERR_SHAPE, "group size above 128");
    if (!(s->rope_base > 1.0) || !isfinite(s->rope_base)) return tr_fail(TR_ERR_SHAPE, "rope_base must be finite and > 1");
    if (s->rope_layout != TR_ROPE_INTERLEAVED && s->rope_layout != TR_ROPE_HALF) return tr_fail(TR_ERR_INVALID_ARG, "rope_layout %d", s->rope_layout);
    if (s->reserved != 0) return tr_fail(TR_ERR_INVALID_ARG, "reserved must be 0");
    return TR_OK;
}

void tr_fill_theta(const tr_shape* s, double* theta)
{
    for (int m = 0; m < 64; ++m) theta[m] = 0.0;
    for (int m = 0; m < s->head_dim / 2; ++m) theta[m] = pow(s->rope_base, -2.0 * (double)m / (double)s->head_dim);
}

static const int64_t ROW_LIMIT = ((int64_t)1 << 31) - 1;

// ---- store ----------------------------------------------------------------------------------------------------
extern "C" int tr_store_create(const tr_shape* shape, const void* k_store, const void* v_store,
                               const int64_t* chunk_row_start, int32_t n_chunks, tr_store** out)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    if (!out) return tr_fail(TR_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    int rc = tr_check_shape(shape);
    if (rc) return rc;
    if (n_chunks < 0 || !chunk_row_start) return tr_fail(TR_ERR_INVALID_ARG, "chunk_row_start NULL or n_chunks < 0");
    if (chunk_row_start[0] < 0) return tr_fail(TR_ERR_INVALID_ARG, "chunk_row_start[0] < 0");
    for (int c = 0; c < n_chunks; ++c)
        if (chunk_row_start[c + 1] < chunk_row_start[c]) return tr_fail(TR_ERR_INVALID_ARG, "chunk_row_start decreases at chunk %d", c);
    if (chunk_row_start[n_chunks] > ROW_LIMIT) return tr_fail(TR_ERR_UNSUPPORTED, "store has 2^31 rows or more");
    if (chunk_row_start[n_chunks] > 0 && (!k_store || !v_store)) return tr_fail(TR_ERR_INVALID_ARG, "store pointer is NULL");
    tr_store* st = new (std::nothrow) tr_store;
    if (!st) return tr_fail(TR_ERR_NO_MEMORY, "out of host memory");
    st->shape = *shape;
    st->k = k_store;
    st->v = v_store;
    st->row_start.assign(chunk_row_start, chunk_row_start + n_chunks + 1);
    *out = st;
    return TR_OK;
    });
}

extern "C" int tr_store_destroy(tr_store* store)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    delete store;
    return TR_OK;
    });
}

// ---- plan (Sec. 3.2) --------------------------------------------------------------------------------------------
extern "C" int tr_plan(const tr_store* store, const int32_t* chunk_ids, int32_t n, int32_t pos_mode,
                       int64_t* offsets, int32_t* pos_ids, int64_t pos_capacity)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    if (!store || !offsets || n < 0 || (n > 0 && !chunk_ids)) return tr_fail(TR_ERR_INVALID_ARG, "tr_plan: NULL argument or n < 0");
    if (pos_mode != TR_POS_COMPOSITE && pos_mode != TR_POS_REORDERED) return tr_fail(TR_ERR_INVALID_ARG, "pos_mode %d", pos_mode);
    const int n_store = (int)store->row_start.size() - 1;
    int64_t off = 0;
    for (int i = 0; i < n; ++i) {
        const int32_t c = chunk_ids[i];
        if (c < 0 || c >= n_store) return tr_fail(TR_ERR_BAD_CHUNK_ID, "chunk_ids[%d] = %d outside [0, %d)", i, c, n_store);
        offsets[i] = off;
        off += store->row_start[c + 1] - store->row_start[c];
    }
    offsets[n] = off;
    if (off > ROW_LIMIT) return tr_fail(TR_ERR_BAD_PLAN, "assembled context has 2^31 rows or more");
    if (pos_ids) {
        if (off > pos_capacity) return tr_fail(TR_ERR_BAD_PLAN, "pos_ids holds %lld entries, plan needs %lld", (long long)pos_capacity, (long long)off);
        for (int i = 0; i < n; ++i) {
            const int64_t len = offsets[i + 1] - offsets[i];
            const int64_t first = (pos_mode == TR_POS_REORDERED) ? offsets[i] : 0;
            for (int64_t t = 0; t < len; ++t) pos_ids[offsets[i] + t] = (int32_t)(first + t);
        }
    }
    return TR_OK;
    });
}

// ---- KV-cache formation ---------------------------------------------------------------------------------------------
namespace {

struct CopyRun { int64_t src_row, dst_row, n_rows, delta; };

// tail (optional): query tokens appended by extra blocks of the last launch
int launch_runs(const tr_store* store, const std::vector<CopyRun>& runs, void* out_k, void* out_v, hipStream_t stream,
                const TrAppendTail* tail = nullptr)
{
    const tr_shape* sh = &store->shape;
    const int eb = tr_elem_bytes(sh);
    const int row_units = sh->n_kv_heads * sh->head_dim * eb / 16;
    int64_t total_units = 0;
    for (const CopyRun& r : runs) total_units += r.n_rows * row_units;
    if (total_units == 0) return TR_OK;
    // span: units of K (and V) per block.  512 units (8 KB of K and 8 KB of V: two loads of each per lane, all issued
    // before anything else) measured best wherever the rows come from HBM and not from a warm cache: 52 against 57 us
    // with spans of 2048 at configuration 4, 69 against 72 us for configuration 3's batch; longer spans only pay
    // when the same buffers are replayed out of the last-level cache.  Small launches take 256 so that every CU gets
    // a block.
    int64_t span = total_units >= 512 * (int64_t)TrChip::CUS ? 512 : 256;
    if (const int forced = tr_knob(TR_KNOB_ASM_SPAN, 0); forced >= 256) span = (forced / 256) * 256;

    TrAssembleArgs a;
    memset(&a, 0, sizeof a);
    a.k_src = store->k;
    a.v_src = store->v;
    a.k_dst = out_k;
    a.v_dst = out_v;
    a.row_units = row_units;
    a.head_units = sh->head_dim * eb / 16;
    a.span_units = (int32_t)span;
    a.half_dim = sh->head_dim / 2;
    a.rope_half = tr_rope_half(sh);
    tr_fill_theta(sh, a.theta);
    size_t i = 0;
    while (i < runs.size()) {
        int n = 0, blocks = 0;
        while (i < runs.size() && n < TR_MAX_COPY_DESC) {
            const CopyRun& r = runs[i++];
            if (r.n_rows == 0) continue;
            TrCopyDesc& d = a.desc[n++];
            d.src_row = (int32_t)r.src_row;
            d.dst_row = (int32_t)r.dst_row;
            d.n_rows = (int32_t)r.n_rows;
            d.delta = (int32_t)r.delta;
            d.blk_start = blocks;
            blocks += (int)((r.n_rows * row_units + span - 1) / span);
        }
        a.n_desc = n;
        if (n == 0) continue;
        if (tail && i == runs.size()) { // last launch carries the append
            a.app = *tail;
            a.app.first_block = blocks;
            blocks += (int)(((int64_t)tail->n_q * (sh->head_dim / 2) + 255) / 256);
        }
        int rc = tr_launch_assemble(a, sh->dtype, blocks, stream);
        if (rc) return rc;
    }
    return TR_OK;
}

} // namespace

namespace {
// Checks one request's plan against the store and lists its chunk runs.
int request_runs(const char* who, const tr_store* store, const int32_t* chunk_ids, const int64_t* offsets, int32_t n_chunks,
                 int32_t pos_mode, const void* out_k, const void* out_v, int64_t out_capacity_rows, std::vector<CopyRun>* runs)
{
    if (!store || n_chunks < 0) return tr_fail(TR_ERR_INVALID_ARG, "%s: store NULL or n_chunks < 0", who);
    if (pos_mode != TR_POS_COMPOSITE && pos_mode != TR_POS_REORDERED) return tr_fail(TR_ERR_INVALID_ARG, "pos_mode %d", pos_mode);
    if (n_chunks == 0) return TR_OK;
    if (!chunk_ids || !offsets) return tr_fail(TR_ERR_INVALID_ARG, "chunk_ids or offsets is NULL");
    if (out_capacity_rows < 0 || out_capacity_rows > ROW_LIMIT) return tr_fail(TR_ERR_INVALID_ARG, "out_capacity_rows out of range");
    const int n_store = (int)store->row_start.size() - 1;
    runs->reserve(n_chunks);
    int64_t off = 0;
    for (int i = 0; i < n_chunks; ++i) {
        const int32_t c = chunk_ids[i];
        if (c < 0 || c >= n_store) return tr_fail(TR_ERR_BAD_CHUNK_ID, "chunk_ids[%d] = %d outside [0, %d)", i, c, n_store);
        if (offsets[i] != off) return tr_fail(TR_ERR_BAD_PLAN, "offsets[%d] = %lld, the prefix sum of the chunk lengths is %lld", i, (long long)offsets[i], (long long)off);
        const int64_t len = store->row_start[c + 1] - store->row_start[c];
        runs->push_back({store->row_start[c], off, len, pos_mode == TR_POS_REORDERED ? off : 0});
        off += len;
    }
    if (offsets[n_chunks] != off) return tr_fail(TR_ERR_BAD_PLAN, "offsets[%d] = %lld, expected n_doc = %lld", n_chunks, (long long)offsets[n_chunks], (long long)off);
    if (off > out_capacity_rows) return tr_fail(TR_ERR_BAD_PLAN, "plan needs %lld rows, the cache holds %lld", (long long)off, (long long)out_capacity_rows);
    if (off > 0 && (!out_k || !out_v)) return tr_fail(TR_ERR_INVALID_ARG, "out_k or out_v is NULL");
    return TR_OK;
}
} // namespace

extern "C" int tr_kv_assemble(const tr_store* store, const int32_t* chunk_ids, const int64_t* offsets, int32_t n_chunks,
                              int32_t pos_mode, void* out_k, void* out_v, int64_t out_capacity_rows, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    std::vector<CopyRun> runs;
    const int rc = request_runs("tr_kv_assemble", store, chunk_ids, offsets, n_chunks, pos_mode, out_k, out_v, out_capacity_rows, &runs);
    if (rc) return rc;
    return launch_runs(store, runs, out_k, out_v, (hipStream_t)stream);
    });
}

extern "C" int tr_kv_assemble_batched(const tr_store* store, const int32_t* chunk_ids, const int32_t* cu_chunks,
                                      const int32_t* pos_modes, const int64_t* cache_row_start, int32_t n_req,
                                      void* out_k, void* out_v, int64_t out_capacity_rows, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    if (!store || n_req < 0) return tr_fail(TR_ERR_INVALID_ARG, "tr_kv_assemble_batched: store NULL or n_req < 0");
    if (n_req == 0) return TR_OK;
    if (!cu_chunks || !pos_modes || !cache_row_start) return tr_fail(TR_ERR_INVALID_ARG, "index array is NULL");
    if (out_capacity_rows < 0 || out_capacity_rows > ROW_LIMIT) return tr_fail(TR_ERR_INVALID_ARG, "out_capacity_rows out of range");
    if (cu_chunks[0] != 0 || cache_row_start[0] < 0) return tr_fail(TR_ERR_INVALID_ARG, "cu_chunks[0] must be 0 and cache_row_start[0] >= 0");
    const int n_store = (int)store->row_start.size() - 1;
    std::vector<CopyRun> runs;
    int64_t total = 0;
    for (int r = 0; r < n_req; ++r) {
        if (cu_chunks[r + 1] < cu_chunks[r]) return tr_fail(TR_ERR_INVALID_ARG, "cu_chunks decreases at request %d", r);
        if (cache_row_start[r + 1] < cache_row_start[r]) return tr_fail(TR_ERR_BAD_PLAN, "cache_row_start decreases at request %d", r);
        if (pos_modes[r] != TR_POS_COMPOSITE && pos_modes[r] != TR_POS_REORDERED) return tr_fail(TR_ERR_INVALID_ARG, "pos_modes[%d] = %d", r, pos_modes[r]);
        if (cu_chunks[r + 1] > cu_chunks[r] && !chunk_ids) return tr_fail(TR_ERR_INVALID_ARG, "chunk_ids is NULL");
        int64_t off = 0;
        for (int i = cu_chunks[r]; i < cu_chunks[r + 1]; ++i) {
            const int32_t c = chunk_ids[i];
            if (c < 0 || c >= n_store) return tr_fail(TR_ERR_BAD_CHUNK_ID, "chunk_ids[%d] = %d outside [0, %d)", i, c, n_store);
            const int64_t len = store->row_start[c + 1] - store->row_start[c];
            runs.push_back({store->row_start[c], cache_row_start[r] + off, len, pos_modes[r] == TR_POS_REORDERED ? off : 0});
            off += len;
        }
        if (off > cache_row_start[r + 1] - cache_row_start[r])
            return tr_fail(TR_ERR_BAD_PLAN, "request %d: documents need %lld rows, its cache range has %lld", r, (long long)off,
                           (long long)(cache_row_start[r + 1] - cache_row_start[r]));
        total += off;
    }
    if (cache_row_start[n_req] > out_capacity_rows) return tr_fail(TR_ERR_BAD_PLAN, "cache ranges end at row %lld, the cache holds %lld", (long long)cache_row_start[n_req], (long long)out_capacity_rows);
    if (total > 0 && (!out_k || !out_v)) return tr_fail(TR_ERR_INVALID_ARG, "out_k or out_v is NULL");
    return launch_runs(store, runs, out_k, out_v, (hipStream_t)stream);
    });
}

// ---- query append ---------------------------------------------------------------------------------------------------
namespace {
int launch_append(const tr_shape* shape, const void* k_new, const void* v_new, const int32_t* q_pos,
                  const std::vector<TrAppendDesc>& descs, void* cache_k, void* cache_v, hipStream_t stream)
{
    TrAppendArgs a;
    memset(&a, 0, sizeof a);
    a.k_new = k_new;
    a.v_new = v_new;
    a.q_pos = q_pos;
    a.cache_k = cache_k;
    a.cache_v = cache_v;
    a.n_kv_heads = shape->n_kv_heads;
    a.head_dim = shape->head_dim;
    a.rope_half = tr_rope_half(shape);
    tr_fill_theta(shape, a.theta);
    size_t i = 0;
    while (i < descs.size()) {
        int n = 0, tokens = 0;
        while (i < descs.size() && n < TR_MAX_APPEND_DESC) {
            if (descs[i].n_q > 0) { a.desc[n++] = descs[i]; tokens += descs[i].n_q; }
            ++i;
        }
        a.n_desc = n;
        a.total_tokens = tokens;
        if (n == 0) continue;
        int rc = tr_launch_append(a, shape->dtype, stream);
        if (rc) return rc;
    }
    return TR_OK;
}
} // namespace

extern "C" int tr_kv_append(const tr_shape* shape, const void* k_new, const void* v_new, const int32_t* q_pos, int32_t n_q,
                            void* cache_k, void* cache_v, int64_t dst_row, int64_t cache_capacity_rows, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    int rc = tr_check_shape(shape);
    if (rc) return rc;
    if (n_q < 0 || dst_row < 0) return tr_fail(TR_ERR_INVALID_ARG, "n_q or dst_row negative");
    if (n_q == 0) return TR_OK;
    if (!k_new || !v_new || !q_pos || !cache_k || !cache_v) return tr_fail(TR_ERR_INVALID_ARG, "tr_kv_append: NULL pointer");
    if (cache_capacity_rows > ROW_LIMIT || dst_row + n_q > cache_capacity_rows)
        return tr_fail(TR_ERR_BAD_PLAN, "rows [%lld, %lld) do not fit a cache of %lld rows", (long long)dst_row, (long long)(dst_row + n_q), (long long)cache_capacity_rows);
    std::vector<TrAppendDesc> d(1);
    d[0].q_row0 = 0;
    d[0].n_q = n_q;
    d[0].dst_row0 = (int32_t)dst_row;
    return launch_append(shape, k_new, v_new, q_pos, d, cache_k, cache_v, (hipStream_t)stream);
    });
}

// assemble + append of one request in a single launch
extern "C" int tr_kv_assemble_append(const tr_store* store, const int32_t* chunk_ids, const int64_t* offsets, int32_t n_chunks,
                                     int32_t pos_mode, const void* k_new, const void* v_new, const int32_t* q_pos, int32_t n_q,
                                     void* out_k, void* out_v, int64_t out_capacity_rows, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    if (!store) return tr_fail(TR_ERR_INVALID_ARG, "tr_kv_assemble_append: store is NULL");
    if (n_q < 0 || n_chunks < 0) return tr_fail(TR_ERR_INVALID_ARG, "negative count");
    if (n_chunks > 0 && !offsets) return tr_fail(TR_ERR_INVALID_ARG, "offsets is NULL");
    const int64_t n_doc_claimed = n_chunks > 0 ? offsets[n_chunks] : 0;
    // no documents or no query tokens: nothing to fuse
    if (n_q == 0) return tr_kv_assemble(store, chunk_ids, offsets, n_chunks, pos_mode, out_k, out_v, out_capacity_rows, stream);
    if (!k_new || !v_new || !q_pos || !out_k || !out_v) return tr_fail(TR_ERR_INVALID_ARG, "tr_kv_assemble_append: NULL pointer");
    if (n_chunks == 0 || n_doc_claimed == 0) { // validated by tr_kv_assemble below
        int rc = tr_kv_assemble(store, chunk_ids, offsets, n_chunks, pos_mode, out_k, out_v, out_capacity_rows, stream);
        if (rc) return rc;
        return tr_kv_append(&store->shape, k_new, v_new, q_pos, n_q, out_k, out_v, 0, out_capacity_rows, stream);
    }
    if (pos_mode != TR_POS_COMPOSITE && pos_mode != TR_POS_REORDERED) return tr_fail(TR_ERR_INVALID_ARG, "pos_mode %d", pos_mode);
    if (!chunk_ids) return tr_fail(TR_ERR_INVALID_ARG, "chunk_ids is NULL");
    if (out_capacity_rows < 0 || out_capacity_rows > ROW_LIMIT) return tr_fail(TR_ERR_INVALID_ARG, "out_capacity_rows out of range");
    const int n_store = (int)store->row_start.size() - 1;
    std::vector<CopyRun> runs;
    runs.reserve(n_chunks);
    int64_t off = 0;
    for (int i = 0; i < n_chunks; ++i) {
        const int32_t c = chunk_ids[i];
        if (c < 0 || c >= n_store) return tr_fail(TR_ERR_BAD_CHUNK_ID, "chunk_ids[%d] = %d outside [0, %d)", i, c, n_store);
        if (offsets[i] != off) return tr_fail(TR_ERR_BAD_PLAN, "offsets[%d] = %lld, the prefix sum of the chunk lengths is %lld", i, (long long)offsets[i], (long long)off);
        const int64_t len = store->row_start[c + 1] - store->row_start[c];
        if (len > 0) runs.push_back({store->row_start[c], off, len, pos_mode == TR_POS_REORDERED ? off : 0}); // the last run carries the tail
        off += len;
    }
    if (offsets[n_chunks] != off) return tr_fail(TR_ERR_BAD_PLAN, "offsets[%d] = %lld, expected n_doc = %lld", n_chunks, (long long)offsets[n_chunks], (long long)off);
    if (off + n_q > out_capacity_rows) return tr_fail(TR_ERR_BAD_PLAN, "plan needs %lld rows, the cache holds %lld", (long long)(off + n_q), (long long)out_capacity_rows);
    TrAppendTail tail;
    tail.k_new = k_new;
    tail.v_new = v_new;
    tail.q_pos = q_pos;
    tail.n_q = n_q;
    tail.dst_row0 = (int32_t)off;
    tail.first_block = 0;
    tail.n_kv_heads = store->shape.n_kv_heads;
    return launch_runs(store, runs, out_k, out_v, (hipStream_t)stream, &tail);
    });
}

extern "C" int tr_kv_append_batched(const tr_shape* shape, const void* k_new, const void* v_new, const int32_t* q_pos,
                                    const int32_t* cu_q, const int64_t* cache_row_start, int32_t n_req, void* cache_k,
                                    void* cache_v, int64_t cache_capacity_rows, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    int rc = tr_check_shape(shape);
    if (rc) return rc;
    if (n_req < 0) return tr_fail(TR_ERR_INVALID_ARG, "n_req < 0");
    if (n_req == 0) return TR_OK;
    if (!cu_q || !cache_row_start) return tr_fail(TR_ERR_INVALID_ARG, "index array is NULL");
    if (cu_q[0] != 0) return tr_fail(TR_ERR_INVALID_ARG, "cu_q[0] must be 0");
    if (cache_capacity_rows > ROW_LIMIT || cache_row_start[n_req] > cache_capacity_rows || cache_row_start[0] < 0)
        return tr_fail(TR_ERR_BAD_PLAN, "cache ranges exceed the capacity");
    std::vector<TrAppendDesc> d;
    for (int r = 0; r < n_req; ++r) {
        const int n_q = cu_q[r + 1] - cu_q[r];
        const int64_t len = cache_row_start[r + 1] - cache_row_start[r];
        if (n_q < 0 || len < 0) return tr_fail(TR_ERR_INVALID_ARG, "cu_q or cache_row_start decreases at request %d", r);
        if (n_q > len) return tr_fail(TR_ERR_BAD_PLAN, "request %d: %d query tokens, cache range of %lld rows", r, n_q, (long long)len);
        TrAppendDesc e;
        e.pos0 = 0;
        e.q_row0 = cu_q[r];
        e.n_q = n_q;
        e.dst_row0 = (int32_t)(cache_row_start[r + 1] - n_q);
        d.push_back(e);
    }
    if (cu_q[n_req] > 0 && (!k_new || !v_new || !q_pos || !cache_k || !cache_v)) return tr_fail(TR_ERR_INVALID_ARG, "tr_kv_append_batched: NULL pointer");
    return launch_append(shape, k_new, v_new, q_pos, d, cache_k, cache_v, (hipStream_t)stream);
    });
}

// ---- KV-cache formation from a store of UN-rotated keys (Sec. 3.2: keep K of Eq. 1, rotate after concatenation) ------
extern "C" int tr_kv_assemble_raw(const tr_store* store, const int32_t* chunk_ids, const int64_t* offsets, int32_t n_chunks,
                                  int32_t pos_mode, void* out_k, void* out_v, int64_t out_capacity_rows, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    std::vector<CopyRun> runs;
    const int rc = request_runs("tr_kv_assemble_raw", store, chunk_ids, offsets, n_chunks, pos_mode, out_k, out_v, out_capacity_rows, &runs);
    if (rc) return rc;
    // every row is a token whose key is turned once, at its position id (the run's first id plus the row's index):
    // the arithmetic of the query append, one thread per (row, channel pair)
    std::vector<TrAppendDesc> d;
    d.reserve(runs.size());
    for (const CopyRun& r : runs) {
        TrAppendDesc e;
        e.q_row0 = (int32_t)r.src_row;
        e.n_q = (int32_t)r.n_rows;
        e.dst_row0 = (int32_t)r.dst_row;
        e.pos0 = (int32_t)r.delta;
        d.push_back(e);
    }
    return launch_append(&store->shape, store->k, store->v, nullptr, d, out_k, out_v, (hipStream_t)stream);
    });
}

// ---- query prefill attention ------------------------------------------------------------------------------------------
namespace {

struct ReqGeom { int32_t q_row0, n_q; int64_t kv_row0, kv_len; };

constexpr int KEY_TILE = 64;
constexpr int TARGET_ITEMS = TrChip::CUS;   // workgroups to aim for when splitting keys: one per CU (more splits cost more partial traffic than they gain)
constexpr int MIN_SPLIT_KEYS = 256;
#ifndef TR_MAX_SPLIT
#define TR_MAX_SPLIT 64
#endif
constexpr int MAX_SPLIT = TR_MAX_SPLIT;  // the combine kernel holds two splits per lane of a half-wave

// Packed rows per workgroup: 256 (8 waves, deep LDS ring) when one KV head has enough rows to fill such tiles,
// else 128 (4 waves).  The wg_rows override of tr_set_tuning wins.
int pick_wg_rows(const tr_shape* sh, int64_t max_rows_per_kv_head)
{
    const int forced = tr_knob(TR_KNOB_WG_ROWS, 0);
    const int g = sh->n_q_heads / sh->n_kv_heads;
    if (forced == 128 || forced == 256 || (forced == 32 && g <= 32)) return forced;
    if (max_rows_per_kv_head <= 32) return 32; // decode and other very short queries: waves split keys, not rows
    return max_rows_per_kv_head >= 512 ? 256 : 128;
}

// How a request's keys are cut: n_split pieces of split_len keys (a multiple of the key tile).
struct SplitPlan { int n_split; int64_t split_len; };

SplitPlan cut_keys(int64_t kv_len, int want, int min_split_keys, int key_tile)
{
    int n_split = want;
    const int64_t max_split = (kv_len + min_split_keys - 1) / min_split_keys;
    if (n_split > max_split) n_split = (int)max_split;
    if (n_split > MAX_SPLIT) n_split = MAX_SPLIT;
    if (n_split < 1) n_split = 1;
    int64_t split_len = (kv_len + n_split - 1) / n_split;
    split_len = ((split_len + key_tile - 1) / key_tile) * key_tile;
    n_split = (int)((kv_len + split_len - 1) / split_len);
    return {n_split, split_len};
}

// Finishing time, in key-tile steps, of a launch whose items (in launch order) walk item_tiles[i] key tiles each.
// Blocks are dealt round-robin to the XCDs and the kernels map each XCD to one contiguous range of items, so
// every XCD works through its own range on its own slots; a workgroup costs FIXED steps besides its tiles.
double launch_makespan(const std::vector<int>& item_tiles, int slots_per_xcd)
{
    const double FIXED = TrChip::WORKGROUP_FIXED_STEPS;
    const size_t X = TrChip::XCDS;
    const size_t n = item_tiles.size(), q = n / X, r = n % X;
    double worst = 0.0;
    std::vector<double> slot;
    for (size_t x = 0; x < X; ++x) {
        const size_t lo = x * q + std::min(x, r), hi = lo + q + (x < r ? 1 : 0);
        slot.assign((size_t)slots_per_xcd, 0.0);
        for (size_t i = lo; i < hi; ++i) { // the next block goes to the slot that frees first
            std::pop_heap(slot.begin(), slot.end(), std::greater<double>());
            slot.back() += FIXED + item_tiles[i];
            std::push_heap(slot.begin(), slot.end(), std::greater<double>());
        }
        for (double t : slot) worst = std::max(worst, t);
    }
    return worst;
}

// The key cuts the launch search chose for the last few batch shapes (host memory only; any thread).
struct CutCacheEntry {
    std::vector<int64_t> key;
    std::vector<SplitPlan> cut;
};
constexpr int CUT_CACHE_ENTRIES = 8;
std::mutex g_cut_mu;
CutCacheEntry g_cut_cache[CUT_CACHE_ENTRIES];
unsigned g_cut_next = 0;

bool cut_cache_lookup(const std::vector<int64_t>& key, std::vector<SplitPlan>* cut)
{
    std::lock_guard<std::mutex> lock(g_cut_mu);
    for (const CutCacheEntry& e : g_cut_cache)
        if (e.key == key) {
            *cut = e.cut;
            return true;
        }
    return false;
}

void cut_cache_store(const std::vector<int64_t>& key, const std::vector<SplitPlan>& cut)
{
    std::lock_guard<std::mutex> lock(g_cut_mu);
    CutCacheEntry& e = g_cut_cache[g_cut_next++ % CUT_CACHE_ENTRIES];
    e.key = key;
    e.cut = cut;
}

// Fills the per-request descriptors of one launch (requests [r0, r1)); returns the partial rows it needs.
int64_t plan_prefix(const tr_shape* sh, const std::vector<ReqGeom>& reqs, size_t r0, size_t r1, TrPrefixArgs* a,
                    bool* any_split, int* total_tokens, int* wg_rows_out)
{
    const int g = sh->n_q_heads / sh->n_kv_heads;
    int64_t max_rows = 0;
    for (size_t r = r0; r < r1; ++r) max_rows = std::max<int64_t>(max_rows, (int64_t)reqs[r].n_q * g);
    const int wg_rows = pick_wg_rows(sh, max_rows);
    const int tpt = wg_rows / g;
    const int target = tr_knob(TR_KNOB_TARGET_ITEMS, TARGET_ITEMS);
    const int min_split_keys = std::max(KEY_TILE, tr_knob(TR_KNOB_MIN_SPLIT_KEYS, MIN_SPLIT_KEYS));
    int64_t base_items = 0;
    for (size_t r = r0; r < r1; ++r) base_items += (int64_t)((reqs[r].n_q + tpt - 1) / tpt) * sh->n_kv_heads;
    int want_split = 1;
    if (sh->dtype == TR_BF16 && base_items > 0 && base_items < target) want_split = (int)((target + base_items - 1) / base_items);
    if (want_split > MAX_SPLIT) want_split = MAX_SPLIT;
    const int key_tile = wg_rows == 32 ? 2 * KEY_TILE : KEY_TILE; // the short-query kernel walks 128 keys a step
    std::vector<SplitPlan> cut(r1 - r0);
    for (size_t r = r0; r < r1; ++r) cut[r - r0] = cut_keys(reqs[r].kv_len, want_split, min_split_keys, key_tile);
    // A batch of requests of different lengths: one split count for all leaves workgroups of very different lengths,
    // and how the launch then packs onto the chip swings by tens of percent with the count.  Instead every request is
    // cut into pieces of about one common length, and that length is chosen by playing the launch through
    // (launch_makespan) for a range of candidates, with the traffic of the partial results priced in.
    if (want_split > 1 && r1 - r0 > 1 && wg_rows != 32 && tr_knob(TR_KNOB_TARGET_ITEMS, 0) == 0) {
        // The search costs tens of microseconds of host time and a call runs it twice (workspace check, then the
        // launch), after the caller's own workspace query: its result is kept for the last few batch shapes.  The
        // key is everything the search reads: head counts, tile geometry, the split floor, and (n_q, kv_len) of every
        // request in order.
        std::vector<int64_t> key;
        key.reserve(8 + 2 * (r1 - r0));
        for (int64_t x : {(int64_t)sh->n_q_heads, (int64_t)sh->n_kv_heads, (int64_t)sh->head_dim, (int64_t)wg_rows, (int64_t)min_split_keys,
                          (int64_t)key_tile})
            key.push_back(x);
        for (size_t r = r0; r < r1; ++r) {
            key.push_back(reqs[r].n_q);
            key.push_back(reqs[r].kv_len);
        }
        if (!cut_cache_lookup(key, &cut)) {
        double walked = 0.0; // keys walked by all row tiles of all KV heads
        for (size_t r = r0; r < r1; ++r) walked += (double)((reqs[r].n_q + tpt - 1) / tpt) * sh->n_kv_heads * (double)reqs[r].kv_len;
        const int slots_per_xcd = (wg_rows == 256 ? TrChip::SLOTS_256 : TrChip::SLOTS_128) / TrChip::XCDS;
        const double STEP_US = TrChip::KEY_TILE_STEP_US, PARTIAL_BYTES_PER_US = TrChip::PARTIAL_BYTES_PER_US;
        double best = 1e300;
        std::vector<SplitPlan> cand(r1 - r0);
        std::vector<int> item_tiles;
        for (int c = 0; c < 24; ++c) {
            const double n_items = (double)TrChip::XCDS * slots_per_xcd * 0.75 * pow(4.0 / 0.75, c / 23.0); // 0.75x .. 4x the resident workgroups
            const double keys_per_item = walked / n_items;
            item_tiles.clear();
            double partial_bytes = 0.0;
            for (size_t r = r0; r < r1; ++r) {
                const ReqGeom& q = reqs[r];
                if (q.n_q == 0) continue;
                const SplitPlan sp = cut_keys(q.kv_len, (int)((double)q.kv_len / keys_per_item + 0.5), min_split_keys, key_tile);
                cand[r - r0] = sp;
                const int n_tiles = (q.n_q + tpt - 1) / tpt;
                const int64_t n_doc = q.kv_len - q.n_q;
                for (int kvh = 0; kvh < sh->n_kv_heads; ++kvh)
                    for (int sp_i = 0; sp_i < sp.n_split; ++sp_i)
                        for (int tile = 0; tile < n_tiles; ++tile) { // the kernel's item order
                            const int64_t sb = (int64_t)sp_i * sp.split_len;
                            const int64_t last_tok = std::min<int64_t>((int64_t)(tile + 1) * tpt, q.n_q) - 1;
                            const int64_t se = std::min<int64_t>(std::min<int64_t>(sb + sp.split_len, q.kv_len), n_doc + last_tok + 1);
                            item_tiles.push_back(se > sb ? (int)((se - sb + key_tile - 1) / key_tile) : 0);
                        }
                if (sp.n_split > 1) partial_bytes += (double)sp.n_split * q.n_q * sh->n_q_heads * (sh->head_dim * 2 + 8);
            }
            const double cost = launch_makespan(item_tiles, slots_per_xcd) * STEP_US + 2.0 * partial_bytes / PARTIAL_BYTES_PER_US;
            if (cost < best) { best = cost; cut = cand; }
        }
        cut_cache_store(key, cut);
        }
    }
    int items = 0, n = 0, toks = 0;
    int64_t ws_rows = 0;
    bool any = false;
    for (size_t r = r0; r < r1; ++r) {
        const ReqGeom& q = reqs[r];
        if (q.n_q == 0) continue;
        const int n_split = cut[r - r0].n_split;
        const int64_t split_len = cut[r - r0].split_len;
        if (a) {
            TrSeqDesc& d = a->seq[n];
            d.q_row0 = q.q_row0;
            d.n_q = q.n_q;
            d.kv_row0 = (int32_t)q.kv_row0;
            d.kv_len = (int32_t)q.kv_len;
            d.item0 = items;
            d.n_tiles = (q.n_q + tpt - 1) / tpt;
            d.n_split = n_split;
            d.split_len = (int32_t)split_len;
            d.ws_row0 = (int32_t)ws_rows;
            d.pad_ = 0;
        }
        ++n;
        items += ((q.n_q + tpt - 1) / tpt) * sh->n_kv_heads * n_split;
        toks += q.n_q;
        if (n_split > 1) {
            any = true;
            ws_rows += (int64_t)n_split * q.n_q * sh->n_q_heads;
        }
    }
    if (a) { a->n_seq = n; a->n_items = items; a->tok_per_tile = tpt; }
    if (any_split) *any_split = any;
    if (total_tokens) *total_tokens = toks;
    if (wg_rows_out) *wg_rows_out = wg_rows;
    return ws_rows;
}

size_t prefix_ws_bytes(const tr_shape* sh, const std::vector<ReqGeom>& reqs)
{
    size_t need = 0;
    for (size_t r0 = 0; r0 < reqs.size(); r0 += TR_MAX_SEQ) {
        size_t r1 = r0 + TR_MAX_SEQ < reqs.size() ? r0 + TR_MAX_SEQ : reqs.size();
        int64_t rows = plan_prefix(sh, reqs, r0, r1, nullptr, nullptr, nullptr, nullptr);
        size_t b = tr_align256((size_t)rows * sh->head_dim * 2) + tr_align256((size_t)rows * 8);
        if (b > need) need = b;
    }
    return need;
}

int run_prefix(const tr_shape* sh, const void* q, const void* k, const void* v, const int32_t* q_pos,
               const std::vector<ReqGeom>& reqs, void* out, void* ws, size_t ws_bytes, hipStream_t stream)
{
    const size_t need = prefix_ws_bytes(sh, reqs);
    if (need > 0) {
        if (!ws) return tr_fail(TR_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
        if (((uintptr_t)ws & 255) != 0) return tr_fail(TR_ERR_WORKSPACE, "workspace is not 256-byte aligned");
        if (ws_bytes < need) return tr_fail(TR_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", ws_bytes, need);
    }
    TrPrefixArgs a;
    memset(&a, 0, sizeof a);
    a.q = q; a.k = k; a.v = v; a.q_pos = q_pos; a.out = out;
    a.n_q_heads = sh->n_q_heads;
    a.n_kv_heads = sh->n_kv_heads;
    a.group = sh->n_q_heads / sh->n_kv_heads;
    a.scale = (float)(1.0 / sqrt((double)sh->head_dim));
    a.scale_log2e = (float)(1.4426950408889634074 / sqrt((double)sh->head_dim));
    a.rope_half = tr_rope_half(sh);
    tr_fill_theta(sh, a.theta);
    for (int m = 0; m < 64; ++m) a.theta_rev[m] = a.theta[m] / 6.283185307179586476925;
    for (size_t r0 = 0; r0 < reqs.size(); r0 += TR_MAX_SEQ) {
        size_t r1 = r0 + TR_MAX_SEQ < reqs.size() ? r0 + TR_MAX_SEQ : reqs.size();
        bool any_split = false;
        int toks = 0, wg_rows = 128;
        int64_t rows = plan_prefix(sh, reqs, r0, r1, &a, &any_split, &toks, &wg_rows);
        a.ws_o = (_Float16*)ws;
        a.ws_ml = (float*)((char*)ws + tr_align256((size_t)rows * sh->head_dim * 2));
        if (a.n_seq == 0) continue;
        int rc = sh->dtype == TR_F32 ? tr_launch_prefix_attn_f32(a, sh->head_dim, toks * sh->n_q_heads, stream)
                                     : tr_launch_prefix_attn(a, sh->head_dim, wg_rows, any_split, toks * sh->n_q_heads, stream);
        if (rc) return rc;
    }
    return TR_OK;
}

int batched_geom(const int32_t* cu_q, const int64_t* cache_row_start, int32_t n_req, std::vector<ReqGeom>* reqs)
{
    if (n_req < 0) return tr_fail(TR_ERR_INVALID_ARG, "n_req < 0");
    if (n_req > 0 && (!cu_q || !cache_row_start)) return tr_fail(TR_ERR_INVALID_ARG, "index array is NULL");
    if (n_req > 0 && (cu_q[0] != 0 || cache_row_start[0] < 0)) return tr_fail(TR_ERR_INVALID_ARG, "cu_q[0] must be 0 and cache_row_start[0] >= 0");
    for (int r = 0; r < n_req; ++r) {
        const int n_q = cu_q[r + 1] - cu_q[r];
        const int64_t len = cache_row_start[r + 1] - cache_row_start[r];
        if (n_q < 0 || len < 0) return tr_fail(TR_ERR_INVALID_ARG, "cu_q or cache_row_start decreases at request %d", r);
        if (len < n_q) return tr_fail(TR_ERR_INVALID_ARG, "request %d: kv_len %lld < n_q %d", r, (long long)len, n_q);
        if (cache_row_start[r + 1] > ROW_LIMIT) return tr_fail(TR_ERR_UNSUPPORTED, "cache has 2^31 rows or more");
        reqs->push_back({cu_q[r], n_q, cache_row_start[r], len});
    }
    return TR_OK;
}

} // namespace

extern "C" size_t tr_prefill_attn_workspace_size(const tr_shape* shape, int32_t n_q, int64_t kv_len)
{
    return tr_guard_size([&]() -> size_t {
    if (tr_check_shape(shape) || n_q <= 0 || kv_len < n_q || kv_len > ROW_LIMIT) return 0;
    std::vector<ReqGeom> reqs{{0, n_q, 0, kv_len}};
    return prefix_ws_bytes(shape, reqs);
    });
}

extern "C" int tr_prefill_attn(const tr_shape* shape, const void* q, const void* k, const void* v, const int32_t* q_pos,
                               int32_t n_q, int64_t kv_len, void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    int rc = tr_check_shape(shape);
    if (rc) return rc;
    if (n_q < 0) return tr_fail(TR_ERR_INVALID_ARG, "n_q < 0");
    if (kv_len < n_q) return tr_fail(TR_ERR_INVALID_ARG, "kv_len %lld < n_q %d: the cache must hold the query tokens", (long long)kv_len, n_q);
    if (kv_len > ROW_LIMIT) return tr_fail(TR_ERR_UNSUPPORTED, "kv_len of 2^31 or more");
    if (n_q == 0) return TR_OK;
    if (!q || !k || !v || !q_pos || !out) return tr_fail(TR_ERR_INVALID_ARG, "tr_prefill_attn: NULL pointer");
    std::vector<ReqGeom> reqs{{0, n_q, 0, kv_len}};
    return run_prefix(shape, q, k, v, q_pos, reqs, out, workspace, workspace_bytes, (hipStream_t)stream);
    });
}

// ---- the same prefill for callers that cannot allocate device memory -------------------------------------------------
// The split-KV partial results live in a file-scope device array instead of a caller's workspace.  The array's name is a
// host-side stand-in in host code; its device address is looked up once per device with hipGetSymbolAddress (each GPU
// holds its own copy) and that pointer is what the kernels get.  Nothing in it has to start at zero: every partial row
// the merge reads was written by the attention kernel of the same call.
#define TR_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
#define TR_MAX_DEVICES 64
static __device__ __align__(256) unsigned char tr_static_scratch[TR_STATIC_SCRATCH_BYTES];
static std::atomic<void*> g_static_scratch[TR_MAX_DEVICES];

static int static_scratch_ptr(void** out)
{
    int dev = 0;
    TR_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= TR_MAX_DEVICES) return tr_fail(TR_ERR_UNSUPPORTED, "device ordinal %d: at most %d devices", dev, TR_MAX_DEVICES);
    void* p = g_static_scratch[dev].load(std::memory_order_acquire);
    if (!p) {
        TR_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(tr_static_scratch)));
        if (!p || ((uintptr_t)p & 255) != 0) return tr_fail(TR_ERR_HIP, "the static scratch array has no usable device address");
        g_static_scratch[dev].store(p, std::memory_order_release); // a race stores the same address twice
    }
    *out = p;
    return TR_OK;
}

extern "C" size_t tr_prefill_attn_static_scratch_bytes(void) { return TR_STATIC_SCRATCH_BYTES; }

extern "C" int tr_prefill_attn_static(const tr_shape* shape, const void* q, const void* k, const void* v, const int32_t* q_pos,
                                      int32_t n_q, int64_t kv_len, void* out, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    int rc = tr_check_shape(shape);
    if (rc) return rc;
    if (n_q < 0) return tr_fail(TR_ERR_INVALID_ARG, "n_q < 0");
    if (kv_len < n_q) return tr_fail(TR_ERR_INVALID_ARG, "kv_len %lld < n_q %d: the cache must hold the query tokens", (long long)kv_len, n_q);
    if (kv_len > ROW_LIMIT) return tr_fail(TR_ERR_UNSUPPORTED, "kv_len of 2^31 or more");
    if (n_q == 0) return TR_OK;
    if (!q || !k || !v || !q_pos || !out) return tr_fail(TR_ERR_INVALID_ARG, "tr_prefill_attn_static: NULL pointer");
    std::vector<ReqGeom> reqs{{0, n_q, 0, kv_len}};
    const size_t need = prefix_ws_bytes(shape, reqs);
    if (need > TR_STATIC_SCRATCH_BYTES)
        return tr_fail(TR_ERR_WORKSPACE, "tr_prefill_attn_static: this shape needs %zu bytes of split-KV scratch, the static array holds %zu; "
                       "use tr_prefill_attn with a workspace", need, (size_t)TR_STATIC_SCRATCH_BYTES);
    void* scratch = nullptr;
    if (need > 0 && (rc = static_scratch_ptr(&scratch))) return rc;
    return run_prefix(shape, q, k, v, q_pos, reqs, out, scratch, need > 0 ? TR_STATIC_SCRATCH_BYTES : 0, (hipStream_t)stream);
    });
}

extern "C" size_t tr_prefill_attn_batched_workspace_size(const tr_shape* shape, const int32_t* cu_q,
                                                         const int64_t* cache_row_start, int32_t n_req)
{
    return tr_guard_size([&]() -> size_t {
    std::vector<ReqGeom> reqs;
    if (tr_check_shape(shape) || batched_geom(cu_q, cache_row_start, n_req, &reqs)) return 0;
    return prefix_ws_bytes(shape, reqs);
    });
}

extern "C" int tr_prefill_attn_batched(const tr_shape* shape, const void* q, const void* k, const void* v,
                                       const int32_t* q_pos, const int32_t* cu_q, const int64_t* cache_row_start,
                                       int32_t n_req, void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    int rc = tr_check_shape(shape);
    if (rc) return rc;
    std::vector<ReqGeom> reqs;
    rc = batched_geom(cu_q, cache_row_start, n_req, &reqs);
    if (rc) return rc;
    if (n_req == 0 || cu_q[n_req] == 0) return TR_OK;
    if (!q || !k || !v || !q_pos || !out) return tr_fail(TR_ERR_INVALID_ARG, "tr_prefill_attn_batched: NULL pointer");
    return run_prefix(shape, q, k, v, q_pos, reqs, out, workspace, workspace_bytes, (hipStream_t)stream);
    });
}

// ---- query prefill that gathers the chunks itself (no assembled document rows needed) ---------------------------
namespace {

struct GatherPlan {
    std::vector<TrGatherSeg> segs; // document segments, then the query-token segment
    int64_t n_doc = 0;
    int n_tiles = 0;
    int row_tiles = 0;
    int n_split = 1;
    int tiles_per_split = 0;
    int tok_per_tile = 0;
};

int plan_gather(const tr_store* store, const int32_t* chunk_ids, const int64_t* offsets, int32_t n_chunks, int32_t pos_mode,
                int32_t n_q, GatherPlan* p)
{
    const tr_shape* sh = &store->shape;
    if (pos_mode != TR_POS_COMPOSITE && pos_mode != TR_POS_REORDERED) return tr_fail(TR_ERR_INVALID_ARG, "pos_mode %d", pos_mode);
    if (n_chunks > 0 && (!chunk_ids || !offsets)) return tr_fail(TR_ERR_INVALID_ARG, "chunk_ids or offsets is NULL");
    const int n_store = (int)store->row_start.size() - 1;
    int64_t off = 0;
    int tiles = 0;
    for (int i = 0; i < n_chunks; ++i) {
        const int32_t c = chunk_ids[i];
        if (c < 0 || c >= n_store) return tr_fail(TR_ERR_BAD_CHUNK_ID, "chunk_ids[%d] = %d outside [0, %d)", i, c, n_store);
        if (offsets[i] != off) return tr_fail(TR_ERR_BAD_PLAN, "offsets[%d] = %lld, the prefix sum of the chunk lengths is %lld", i, (long long)offsets[i], (long long)off);
        const int64_t len = store->row_start[c + 1] - store->row_start[c];
        if (len > 0) {
            TrGatherSeg e;
            e.src_row = (int32_t)store->row_start[c];
            e.n_rows = (int32_t)len;
            e.delta = pos_mode == TR_POS_REORDERED ? (int32_t)off : 0;
            e.tile0 = tiles;
            e.cache_row = (int32_t)off;
            p->segs.push_back(e);
            tiles += (int)((len + KEY_TILE - 1) / KEY_TILE);
        }
        off += len;
    }
    if (n_chunks > 0 && offsets[n_chunks] != off) return tr_fail(TR_ERR_BAD_PLAN, "offsets[%d] = %lld, expected n_doc = %lld", n_chunks, (long long)offsets[n_chunks], (long long)off);
    if (off + n_q > ROW_LIMIT) return tr_fail(TR_ERR_UNSUPPORTED, "2^31 rows or more");
    if ((int)p->segs.size() + 1 > TR_MAX_GATHER_SEG)
        return tr_fail(TR_ERR_UNSUPPORTED, "%d non-empty chunks in one request, at most %d", (int)p->segs.size(), TR_MAX_GATHER_SEG - 1);
    TrGatherSeg t;
    t.src_row = (int32_t)off; // the query tokens sit behind the documents in the request's cache
    t.n_rows = n_q;
    t.delta = 0;
    t.tile0 = tiles;
    t.cache_row = (int32_t)off;
    p->segs.push_back(t);
    tiles += (n_q + KEY_TILE - 1) / KEY_TILE;
    p->n_doc = off;
    p->n_tiles = tiles;
    const int g = sh->n_q_heads / sh->n_kv_heads;
    p->tok_per_tile = 128 / g;
    p->row_tiles = (n_q + p->tok_per_tile - 1) / p->tok_per_tile;
    const int base_items = p->row_tiles * sh->n_kv_heads;
    if (base_items == 0) return TR_OK; // no query tokens: nothing will be launched
    int want = base_items < TARGET_ITEMS ? (TARGET_ITEMS + base_items - 1) / base_items : 1;
    if (want > MAX_SPLIT) want = MAX_SPLIT;
    const int max_split = std::max(1, tiles / (MIN_SPLIT_KEYS / KEY_TILE));
    if (want > max_split) want = max_split;
    p->tiles_per_split = (tiles + want - 1) / want;
    p->n_split = (tiles + p->tiles_per_split - 1) / p->tiles_per_split;
    return TR_OK;
}

size_t gather_ws_bytes(const tr_shape* sh, const GatherPlan& p, int32_t n_q)
{
    if (p.n_split <= 1) return 0;
    const size_t rows = (size_t)p.n_split * n_q * sh->n_q_heads;
    return tr_align256(rows * sh->head_dim * 2) + tr_align256(rows * 8);
}

} // namespace

extern "C" size_t tr_prefill_attn_gather_workspace_size(const tr_store* store, const int32_t* chunk_ids, const int64_t* offsets,
                                                        int32_t n_chunks, int32_t pos_mode, int32_t n_q)
{
    return tr_guard_size([&]() -> size_t {
    if (!store || n_chunks < 0 || n_q <= 0) return 0;
    GatherPlan p;
    if (plan_gather(store, chunk_ids, offsets, n_chunks, pos_mode, n_q, &p)) return 0;
    return gather_ws_bytes(&store->shape, p, n_q);
    });
}

extern "C" int tr_prefill_attn_gather(const tr_store* store, const int32_t* chunk_ids, const int64_t* offsets, int32_t n_chunks,
                                      int32_t pos_mode, const void* q, const void* cache_k, const void* cache_v,
                                      const int32_t* q_pos, int32_t n_q, int64_t cache_capacity_rows, void* out,
                                      void* workspace, size_t workspace_bytes, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    if (!store) return tr_fail(TR_ERR_INVALID_ARG, "tr_prefill_attn_gather: store is NULL");
    if (n_chunks < 0 || n_q < 0) return tr_fail(TR_ERR_INVALID_ARG, "negative count");
    const tr_shape* sh = &store->shape;
    if (sh->dtype != TR_BF16) return tr_fail(TR_ERR_UNSUPPORTED, "tr_prefill_attn_gather is implemented for TR_BF16 only");
    GatherPlan p;
    int rc = plan_gather(store, chunk_ids, offsets, n_chunks, pos_mode, n_q, &p);
    if (rc) return rc;
    if (n_q == 0) return TR_OK;
    if (!q || !cache_k || !cache_v || !q_pos || !out) return tr_fail(TR_ERR_INVALID_ARG, "tr_prefill_attn_gather: NULL pointer");
    if (p.n_doc + n_q > cache_capacity_rows) return tr_fail(TR_ERR_BAD_PLAN, "the cache holds %lld rows, the query tokens end at row %lld", (long long)cache_capacity_rows, (long long)(p.n_doc + n_q));
    const size_t need = gather_ws_bytes(sh, p, n_q);
    if (need > 0) {
        if (!workspace) return tr_fail(TR_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
        if (((uintptr_t)workspace & 255) != 0) return tr_fail(TR_ERR_WORKSPACE, "workspace is not 256-byte aligned");
        if (workspace_bytes < need) return tr_fail(TR_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
    }
    TrGatherArgs a;
    memset(&a, 0, sizeof a);
    a.q = q;
    a.k_store = store->k;
    a.v_store = store->v;
    a.k_cache = cache_k;
    a.v_cache = cache_v;
    a.q_pos = q_pos;
    a.out = out;
    const size_t rows = (size_t)p.n_split * n_q * sh->n_q_heads;
    a.ws_o = (_Float16*)workspace;
    a.ws_ml = need ? (float*)((char*)workspace + tr_align256(rows * sh->head_dim * 2)) : nullptr;
    a.n_q = n_q;
    a.n_doc = (int32_t)p.n_doc;
    a.n_seg = (int32_t)p.segs.size();
    a.n_tiles_total = p.n_tiles;
    a.n_split = p.n_split;
    a.tiles_per_split = p.tiles_per_split;
    a.row_tiles = p.row_tiles;
    a.n_items = p.row_tiles * sh->n_kv_heads * p.n_split;
    a.n_q_heads = sh->n_q_heads;
    a.n_kv_heads = sh->n_kv_heads;
    a.group = sh->n_q_heads / sh->n_kv_heads;
    a.tok_per_tile = p.tok_per_tile;
    a.scale_log2e = (float)(1.4426950408889634074 / sqrt((double)sh->head_dim));
    a.rope_half = tr_rope_half(sh);
    double theta[64];
    tr_fill_theta(sh, theta);
    for (int m = 0; m < 64; ++m) a.theta_rev[m] = theta[m] / 6.283185307179586476925;
    for (size_t i = 0; i < p.segs.size(); ++i) a.seg[i] = p.segs[i];
    // the merge kernel reads the same partial layout as for tr_prefill_attn
    TrPrefixArgs ca;
    memset(&ca, 0, sizeof ca);
    ca.out = out;
    ca.ws_o = a.ws_o;
    ca.ws_ml = a.ws_ml;
    ca.n_seq = 1;
    ca.n_q_heads = sh->n_q_heads;
    ca.n_kv_heads = sh->n_kv_heads;
    ca.group = a.group;
    ca.seq[0].q_row0 = 0;
    ca.seq[0].n_q = n_q;
    ca.seq[0].n_split = p.n_split;
    ca.seq[0].ws_row0 = 0;
    return tr_launch_gather_attn(a, ca, sh->head_dim, (hipStream_t)stream);
    });
}

// ---- one pass over a packed sequence with per-token visible ranges and position ids -----------------------------
extern "C" int tr_sequence_plan(const int32_t* chunk_lens, int32_t n_chunks, int32_t n_tail, int32_t pos_mode, int32_t tail_start,
                                int32_t* seg_start, int32_t* pos, int64_t capacity)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    if (n_chunks < 0 || n_tail < 0) return tr_fail(TR_ERR_INVALID_ARG, "negative count");
    if (pos_mode != TR_POS_COMPOSITE && pos_mode != TR_POS_REORDERED) return tr_fail(TR_ERR_INVALID_ARG, "pos_mode %d", pos_mode);
    if (n_chunks > 0 && !chunk_lens) return tr_fail(TR_ERR_INVALID_ARG, "chunk_lens is NULL");
    int64_t n_doc = 0, longest = 0;
    for (int c = 0; c < n_chunks; ++c) {
        if (chunk_lens[c] < 0) return tr_fail(TR_ERR_INVALID_ARG, "chunk_lens[%d] < 0", c);
        n_doc += chunk_lens[c];
        longest = std::max<int64_t>(longest, chunk_lens[c]);
    }
    const int64_t total = n_doc + n_tail;
    if (total > ROW_LIMIT) return tr_fail(TR_ERR_UNSUPPORTED, "2^31 tokens or more");
    if (total > capacity) return tr_fail(TR_ERR_BAD_PLAN, "the sequence has %lld tokens, the arrays hold %lld", (long long)total, (long long)capacity);
    if (total > 0 && (!seg_start || !pos)) return tr_fail(TR_ERR_INVALID_ARG, "seg_start or pos is NULL");
    int64_t off = 0;
    for (int c = 0; c < n_chunks; ++c) {
        for (int64_t t = 0; t < chunk_lens[c]; ++t) {
            seg_start[off + t] = (int32_t)off;
            pos[off + t] = (int32_t)(pos_mode == TR_POS_REORDERED ? off + t : t);
        }
        off += chunk_lens[c];
    }
    const int64_t start = tail_start >= 0 ? tail_start : (pos_mode == TR_POS_REORDERED ? n_doc : longest);
    for (int64_t i = 0; i < n_tail; ++i) {
        seg_start[n_doc + i] = 0;
        pos[n_doc + i] = (int32_t)(start + i);
    }
    return TR_OK;
    });
}

namespace {

constexpr int BD_SLOTS = TrChip::SLOTS_128; // 128-row workgroups resident at once: two per CU
constexpr int BD_MIN_PIECE_TILES = 16;

// Work list of the block-diagonal kernel.  Without a host copy of the starts every row tile is one item per KV head.
// With it, row tiles whose key walk is long against the chip's fair share (a query behind many documents walks all of
// them while document tokens walk one chunk) are cut into pieces, which run as separate workgroups and are merged by
// the combine kernel.  Fills a->seg, a->n_seg, a->items_per_head and, when comb != NULL, the merge's descriptors.
// Returns the partial rows needed, or -1 with the error set.
int64_t plan_blockdiag(const tr_shape* sh, const int32_t* start_host, int64_t T, int tpt, TrBlockDiagArgs* a, TrPrefixArgs* comb,
                       int* comb_rows)
{
    const int64_t n_tiles = (T + tpt - 1) / tpt;
    std::vector<int32_t> ns((size_t)n_tiles, 1), span;
    if (start_host && sh->dtype == TR_BF16) {
        span.resize((size_t)n_tiles);
        double walked = 0.0; // key tiles walked by all row tiles of one KV head
        for (int64_t tile = 0; tile < n_tiles; ++tile) {
            const int64_t t0 = tile * tpt, t1 = std::min<int64_t>(t0 + tpt, T);
            int64_t lo = t0;
            for (int64_t t = t0; t < t1; ++t) lo = std::min<int64_t>(lo, std::min<int64_t>(std::max<int64_t>(start_host[t], 0), t));
            span[(size_t)tile] = (int32_t)(t1 - lo);
            walked += (double)((t1 - lo + KEY_TILE - 1) / KEY_TILE);
        }
        const int slots = std::max(1, tr_knob(TR_KNOB_BD_SLOTS, BD_SLOTS));
        const double fair = walked * sh->n_kv_heads / slots; // key tiles per resident workgroup
        int piece = (int)(fair / 3.0);
        if (piece < BD_MIN_PIECE_TILES) piece = BD_MIN_PIECE_TILES;
        piece = tr_knob(TR_KNOB_BD_PIECE_TILES, piece);
        if (piece < 1) piece = 1;
        for (int64_t tile = 0; tile < n_tiles; ++tile) {
            const int st = (span[(size_t)tile] + KEY_TILE - 1) / KEY_TILE;
            if (st > 2 * piece) ns[(size_t)tile] = std::min(32, (st + piece - 1) / piece);
        }
        // runs of equal split count, at most TR_MAX_BD_SEG of them: else one run from the first to the last split tile
        int runs = 1;
        for (int64_t tile = 1; tile < n_tiles; ++tile) runs += ns[(size_t)tile] != ns[(size_t)tile - 1];
        if (runs > TR_MAX_BD_SEG) {
            int64_t first = -1, last = -1;
            int32_t most = 1;
            for (int64_t tile = 0; tile < n_tiles; ++tile)
                if (ns[(size_t)tile] > 1) { if (first < 0) first = tile; last = tile; most = std::max(most, ns[(size_t)tile]); }
            for (int64_t tile = first; tile <= last; ++tile) ns[(size_t)tile] = most;
        }
    }
    int n_seg = 0;
    int64_t items = 0, ws_rows = 0;
    for (int64_t hi = n_tiles - 1; hi >= 0;) {
        int64_t lo = hi;
        while (lo > 0 && ns[(size_t)lo - 1] == ns[(size_t)hi]) --lo;
        TrBdSeg& g = a->seg[n_seg++];
        g.tile_hi = (int32_t)hi;
        g.n_tiles = (int32_t)(hi - lo + 1);
        g.n_split = ns[(size_t)hi];
        g.item0 = (int32_t)items;
        g.tok0 = (int32_t)(lo * tpt);
        g.n_tok = (int32_t)(std::min<int64_t>((hi + 1) * tpt, T) - lo * tpt);
        g.split_len = 0;
        g.ws_row0 = 0;
        if (g.n_split > 1) {
            int32_t longest = 0;
            for (int64_t tile = lo; tile <= hi; ++tile) longest = std::max(longest, span[(size_t)tile]);
            const int64_t len = (longest + g.n_split - 1) / g.n_split;
            g.split_len = (int32_t)(((len + KEY_TILE - 1) / KEY_TILE) * KEY_TILE);
            g.ws_row0 = (int32_t)ws_rows;
            ws_rows += (int64_t)g.n_split * g.n_tok * sh->n_q_heads;
        }
        items += (int64_t)g.n_tiles * g.n_split;
        hi = lo - 1;
    }
    if (items * sh->n_kv_heads > ROW_LIMIT || ws_rows > ROW_LIMIT) {
        tr_fail(TR_ERR_UNSUPPORTED, "the sequence needs 2^31 work items or partial rows, or more");
        return -1;
    }
    a->n_seg = n_seg;
    a->items_per_head = (int32_t)items;
    if (comb) {
        // the merge walks the tokens from the first split segment to the last; segments are in descending token order
        memset(comb, 0, sizeof *comb);
        int first = -1, last = -1;
        for (int i = 0; i < n_seg; ++i)
            if (a->seg[i].n_split > 1) { if (first < 0) first = i; last = i; }
        *comb_rows = 0;
        if (first >= 0) {
            int n = 0;
            int64_t toks = 0;
            for (int i = last; i >= first; --i) { // ascending tokens
                const TrBdSeg& g = a->seg[i];
                TrSeqDesc& d = comb->seq[n++];
                d.q_row0 = g.tok0;
                d.n_q = g.n_tok;
                d.n_split = g.n_split;
                d.ws_row0 = g.ws_row0;
                toks += g.n_tok;
            }
            comb->n_seq = n;
            comb->n_q_heads = sh->n_q_heads;
            comb->n_kv_heads = sh->n_kv_heads;
            comb->group = sh->n_q_heads / sh->n_kv_heads;
            *comb_rows = (int)(toks * sh->n_q_heads);
        }
    }
    return ws_rows;
}

size_t blockdiag_ws_bytes(const tr_shape* sh, int64_t ws_rows)
{
    return ws_rows > 0 ? tr_align256((size_t)ws_rows * sh->head_dim * 2) + tr_align256((size_t)ws_rows * 8) : 0;
}

int sequence_tok_per_tile(const tr_shape* sh, int* wg_rows)
{
    *wg_rows = tr_knob(TR_KNOB_WG_ROWS, 0) == 256 ? 256 : 128;
    return *wg_rows / (sh->n_q_heads / sh->n_kv_heads);
}

} // namespace

extern "C" size_t tr_sequence_prefill_attn_workspace_size(const tr_shape* shape, const int32_t* seg_start_host, int64_t total_tokens)
{
    return tr_guard_size([&]() -> size_t {
    if (tr_check_shape(shape) || total_tokens <= 0 || total_tokens > ROW_LIMIT || !seg_start_host) return 0;
    int wg_rows;
    const int tpt = sequence_tok_per_tile(shape, &wg_rows);
    TrBlockDiagArgs a;
    const int64_t rows = plan_blockdiag(shape, seg_start_host, total_tokens, tpt, &a, nullptr, nullptr);
    return rows > 0 ? blockdiag_ws_bytes(shape, rows) : 0;
    });
}

extern "C" int tr_sequence_prefill_attn(const tr_shape* shape, const void* q, const void* k, const void* v, const int32_t* seg_start,
                                        const int32_t* pos, const int32_t* seg_start_host, int64_t total_tokens, void* out,
                                        void* k_rot_out, void* workspace, size_t workspace_bytes, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    int rc = tr_check_shape(shape);
    if (rc) return rc;
    if (total_tokens < 0) return tr_fail(TR_ERR_INVALID_ARG, "total_tokens < 0");
    if (total_tokens > ROW_LIMIT) return tr_fail(TR_ERR_UNSUPPORTED, "2^31 tokens or more");
    if (total_tokens == 0) return TR_OK;
    if (!q || !k || !v || !seg_start || !pos || !out) return tr_fail(TR_ERR_INVALID_ARG, "tr_sequence_prefill_attn: NULL pointer");
    if (!k_rot_out) return tr_fail(TR_ERR_INVALID_ARG, "k_rot_out is required (it may alias k)");
    hipStream_t s = (hipStream_t)stream;
    TrBlockDiagArgs a;
    memset(&a, 0, sizeof a);
    TrPrefixArgs comb;
    int comb_rows = 0, wg_rows;
    a.tok_per_tile = sequence_tok_per_tile(shape, &wg_rows);
    const int64_t ws_rows = plan_blockdiag(shape, seg_start_host, total_tokens, a.tok_per_tile, &a, &comb, &comb_rows);
    if (ws_rows < 0) return TR_ERR_UNSUPPORTED;
    const size_t need = blockdiag_ws_bytes(shape, ws_rows);
    if (need > 0) {
        if (!workspace) return tr_fail(TR_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
        if (((uintptr_t)workspace & 255) != 0) return tr_fail(TR_ERR_WORKSPACE, "workspace is not 256-byte aligned");
        if (workspace_bytes < need) return tr_fail(TR_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
        a.ws_o = (_Float16*)workspace;
        a.ws_ml = (float*)((char*)workspace + tr_align256((size_t)ws_rows * shape->head_dim * 2));
        comb.ws_o = a.ws_o;
        comb.ws_ml = a.ws_ml;
        comb.out = out;
    }
    // keys rotated at their position ids, fp64, one rounding (the arithmetic of the query append), values untouched
    std::vector<TrAppendDesc> d(1);
    d[0].q_row0 = 0;
    d[0].n_q = (int32_t)total_tokens;
    d[0].dst_row0 = 0;
    rc = launch_append(shape, k, nullptr, pos, d, k_rot_out, nullptr, s);
    if (rc) return rc;
    tr_fill_theta(shape, a.theta);
    for (int m = 0; m < 64; ++m) a.theta_rev[m] = a.theta[m] / 6.283185307179586476925;
    a.q = q;
    a.k = k_rot_out;
    a.v = v;
    a.tok_start = seg_start;
    a.pos = pos;
    a.out = out;
    a.total_tokens = (int32_t)total_tokens;
    a.n_q_heads = shape->n_q_heads;
    a.n_kv_heads = shape->n_kv_heads;
    a.group = shape->n_q_heads / shape->n_kv_heads;
    a.rope_half = tr_rope_half(shape);
    a.n_tiles = (int32_t)((total_tokens + a.tok_per_tile - 1) / a.tok_per_tile);
    a.scale = (float)(1.0 / sqrt((double)shape->head_dim));
    a.scale_log2e = (float)(1.4426950408889634074 / sqrt((double)shape->head_dim));
    if (shape->dtype == TR_F32) return tr_launch_blockdiag_attn_f32(a, shape->head_dim, s);
    return tr_launch_blockdiag_attn(a, comb_rows > 0 ? &comb : nullptr, comb_rows, shape->head_dim, wg_rows, s);
    });
}

// ---- projections around the attention (Eq. 1) for the query tokens ------------------------------------------------------
namespace {
constexpr int LINEAR_MAX_ROWS = 128;
// returns the status and, through n_total, the summed feature count
int check_linear(int32_t M, int32_t n_out, const int32_t* n_features, int32_t K, int64_t* n_total)
{
    if (M < 0 || K <= 0) return tr_fail(TR_ERR_INVALID_ARG, "tr_linear: M %d, K %d", M, K);
    if (n_out < 1 || n_out > TR_LINEAR_MAX_OUT) return tr_fail(TR_ERR_INVALID_ARG, "tr_linear: %d outputs, 1 .. %d supported", n_out, TR_LINEAR_MAX_OUT);
    if (!n_features) return tr_fail(TR_ERR_INVALID_ARG, "tr_linear: n_features is NULL");
    int64_t N = 0;
    for (int j = 0; j < n_out; ++j) {
        if (n_features[j] <= 0) return tr_fail(TR_ERR_INVALID_ARG, "tr_linear: n_features[%d] = %d", j, n_features[j]);
        if (n_features[j] % 32 != 0) return tr_fail(TR_ERR_SHAPE, "tr_linear: n_features[%d] = %d is not a multiple of 32", j, n_features[j]);
        N += n_features[j];
    }
    if (K % 16 != 0) return tr_fail(TR_ERR_SHAPE, "tr_linear: K (%d) must be a multiple of 16", K);
    if (N > (1 << 24)) return tr_fail(TR_ERR_UNSUPPORTED, "tr_linear: %lld output features", (long long)N);
    if (M > LINEAR_MAX_ROWS) return tr_fail(TR_ERR_UNSUPPORTED, "tr_linear streams the weights once for at most %d rows of x (got %d); larger products are a library GEMM's work", LINEAR_MAX_ROWS, M);
    *n_total = N;
    return TR_OK;
}
size_t linear_ws_bytes(int32_t M, int64_t N, int32_t K)
{
    const int n_split = tr_linear_splits(M, (int32_t)N, K);
    return n_split > 1 ? tr_align256((size_t)n_split * M * N * 4) : 0;
}
} // namespace

extern "C" size_t tr_linear_workspace_size(int32_t M, int32_t n_out, const int32_t* n_features, int32_t K)
{
    return tr_guard_size([&]() -> size_t {
    int64_t N = 0;
    if (check_linear(M, n_out, n_features, K, &N) || M == 0) return 0;
    return linear_ws_bytes(M, N, K);
    });
}

extern "C" int tr_linear(const void* x, int32_t M, int32_t K, int32_t n_out, const void* const* w, void* const* y,
                         const int32_t* n_features, void* workspace, size_t workspace_bytes, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    int64_t N = 0;
    const int rc = check_linear(M, n_out, n_features, K, &N);
    if (rc) return rc;
    if (M == 0) return TR_OK;
    if (!x || !w || !y) return tr_fail(TR_ERR_INVALID_ARG, "tr_linear: NULL pointer");
    if (((uintptr_t)x & 15) != 0) return tr_fail(TR_ERR_INVALID_ARG, "tr_linear: x must be 16-byte aligned");
    for (int j = 0; j < n_out; ++j) {
        if (!w[j] || !y[j]) return tr_fail(TR_ERR_INVALID_ARG, "tr_linear: w[%d] or y[%d] is NULL", j, j);
        if (((uintptr_t)w[j] & 15) != 0 || ((uintptr_t)y[j] & 7) != 0) return tr_fail(TR_ERR_INVALID_ARG, "tr_linear: w[%d] must be 16-byte aligned, y[%d] 8-byte aligned", j, j);
    }
    const size_t need = linear_ws_bytes(M, N, K);
    if (need > 0) {
        if (!workspace) return tr_fail(TR_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
        if (((uintptr_t)workspace & 255) != 0) return tr_fail(TR_ERR_WORKSPACE, "workspace is not 256-byte aligned");
        if (workspace_bytes < need) return tr_fail(TR_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
    }
    return tr_launch_linear(x, n_out, w, y, n_features, need > 0 ? workspace : nullptr, M, K, (hipStream_t)stream);
    });
}

// ---- decode step: one query token per request ---------------------------------------------------------------------
namespace {
int decode_cu(int32_t n_req, std::vector<int32_t>* cu)
{
    if (n_req < 0) return tr_fail(TR_ERR_INVALID_ARG, "n_req < 0");
    cu->resize((size_t)n_req + 1);
    for (int32_t r = 0; r <= n_req; ++r) (*cu)[r] = r;
    return TR_OK;
}
} // namespace

extern "C" size_t tr_decode_attn_workspace_size(const tr_shape* shape, const int64_t* cache_row_start, int32_t n_req)
{
    return tr_guard_size([&]() -> size_t {
    std::vector<int32_t> cu;
    if (decode_cu(n_req, &cu)) return 0;
    return tr_prefill_attn_batched_workspace_size(shape, cu.data(), cache_row_start, n_req);
    });
}

extern "C" int tr_decode_attn(const tr_shape* shape, const void* q, const void* k, const void* v, const int32_t* q_pos,
                              const int64_t* cache_row_start, int32_t n_req, void* out, void* workspace,
                              size_t workspace_bytes, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    std::vector<int32_t> cu;
    int rc = decode_cu(n_req, &cu);
    if (rc) return rc;
    return tr_prefill_attn_batched(shape, q, k, v, q_pos, cu.data(), cache_row_start, n_req, out, workspace, workspace_bytes, stream);
    });
}

// ---- offline chunk prefill --------------------------------------------------------------------------------------------
extern "C" size_t tr_chunk_prefill_attn_workspace_size(const tr_shape* shape, int64_t total_tokens, int32_t max_chunk_len)
{
    return tr_guard_size([&]() -> size_t {
    if (tr_check_shape(shape) || total_tokens <= 0 || max_chunk_len <= 0) return 0;
    return tr_align256((size_t)max_chunk_len * (shape->head_dim / 2) * 16) + tr_align256((size_t)total_tokens * 4);
    });
}

extern "C" int tr_chunk_prefill_attn(const tr_shape* shape, const void* q, const void* k, const void* v,
                                     const int32_t* cu_chunk_lens, int32_t n_chunks, int64_t total_tokens,
                                     int32_t max_chunk_len, void* out, void* k_rot_out, void* workspace,
                                     size_t workspace_bytes, void* stream)
{
    return tr_guard_int([&]() -> int {
    tr_clear_error();
    int rc = tr_check_shape(shape);
    if (rc) return rc;
    if (n_chunks < 0 || total_tokens < 0 || max_chunk_len < 0) return tr_fail(TR_ERR_INVALID_ARG, "negative count");
    if (total_tokens > ROW_LIMIT) return tr_fail(TR_ERR_UNSUPPORTED, "2^31 tokens or more");
    if (total_tokens == 0 || n_chunks == 0) return TR_OK;
    if (max_chunk_len == 0 || max_chunk_len > total_tokens) return tr_fail(TR_ERR_INVALID_ARG, "max_chunk_len %d must be in [1, total_tokens]", max_chunk_len);
    if (!q || !k || !v || !cu_chunk_lens || !out) return tr_fail(TR_ERR_INVALID_ARG, "tr_chunk_prefill_attn: NULL pointer");
    if (!k_rot_out) return tr_fail(TR_ERR_INVALID_ARG, "k_rot_out is required (it may alias k)");
    const size_t need = tr_chunk_prefill_attn_workspace_size(shape, total_tokens, max_chunk_len);
    if (!workspace) return tr_fail(TR_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
    if (((uintptr_t)workspace & 255) != 0) return tr_fail(TR_ERR_WORKSPACE, "workspace is not 256-byte aligned");
    if (workspace_bytes < need) return tr_fail(TR_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
    hipStream_t s = (hipStream_t)stream;
    double* table = (double*)workspace;
    int32_t* tok_start = (int32_t*)((char*)workspace + tr_align256((size_t)max_chunk_len * (shape->head_dim / 2) * 16));

    TrBlockDiagArgs a;
    memset(&a, 0, sizeof a);
    tr_fill_theta(shape, a.theta);
    for (int m = 0; m < 64; ++m) a.theta_rev[m] = a.theta[m] / 6.283185307179586476925;
    rc = tr_launch_rope_table(table, max_chunk_len, shape->head_dim / 2, a.theta, s);
    if (rc) return rc;
    rc = tr_launch_rope_rows(k, k_rot_out, cu_chunk_lens, n_chunks, max_chunk_len, tok_start, table, max_chunk_len, total_tokens, shape, s);
    if (rc) return rc;
    a.q = q;
    a.k = k_rot_out;
    a.v = v;
    a.tok_start = tok_start;
    a.out = out;
    a.total_tokens = (int32_t)total_tokens;
    a.n_q_heads = shape->n_q_heads;
    a.n_kv_heads = shape->n_kv_heads;
    a.group = shape->n_q_heads / shape->n_kv_heads;
    a.rope_half = tr_rope_half(shape);
    // chunks are short (a row tile walks a few key tiles only), so two independent 4-wave workgroups per CU, which
    // overlap one's prologue and epilogue with the other's tile loop, beat one 8-wave workgroup
    const int forced_rows = tr_knob(TR_KNOB_WG_ROWS, 0);
    const int wg_rows = forced_rows == 256 ? 256 : 128;
    a.tok_per_tile = wg_rows / a.group;
    a.n_tiles = (int32_t)((total_tokens + a.tok_per_tile - 1) / a.tok_per_tile);
    a.scale = (float)(1.0 / sqrt((double)shape->head_dim));
    a.scale_log2e = (float)(1.4426950408889634074 / sqrt((double)shape->head_dim));
    if (plan_blockdiag(shape, nullptr, total_tokens, a.tok_per_tile, &a, nullptr, nullptr) < 0) return TR_ERR_UNSUPPORTED;
    if (shape->dtype == TR_F32) return tr_launch_blockdiag_attn_f32(a, shape->head_dim, s);
    return tr_launch_blockdiag_attn(a, nullptr, 0, shape->head_dim, wg_rows, s);
    });
}
