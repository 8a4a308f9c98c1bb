// Internal declarations shared by the translation units of libturborag_hip.so.
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <stddef.h>
#include <vector>

#include "../../include/turborag.h"

// ---- error plumbing -------------------------------------------------------------------------------------
int tr_fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void tr_clear_error();
#define TR_HIP(expr)                                                                           \
    do {                                                                                       \
        hipError_t e__ = (expr);                                                               \
        if (e__ != hipSuccess) return tr_fail(TR_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

// A kernel that needs more dynamic LDS than the default limit has the limit raised once per device: the attribute
// belongs to the function on the device that is current, so a process that uses a second device must set it there
// too.  `done` holds one bit per device ordinal (mod 64) and is safe to race on: the worst case sets it twice.
static inline int tr_raise_lds_limit(const void* kernel, int bytes, std::atomic<uint64_t>* done)
{
    int dev = 0;
    TR_HIP(hipGetDevice(&dev));
    const uint64_t bit = 1ull << (dev & 63);
    if (!(done->load(std::memory_order_acquire) & bit)) {
        TR_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
        done->fetch_or(bit, std::memory_order_release);
    }
    return TR_OK;
}

int tr_check_shape(const tr_shape* s);
static inline int tr_elem_bytes(const tr_shape* s) { return s->dtype == TR_F32 ? 4 : 2; }
static inline size_t tr_align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct tr_store {
    tr_shape shape;
    const void* k;
    const void* v;
    std::vector<int64_t> row_start; // n_chunks + 1
};

// ---- launch-policy overrides (tr_set_tuning) --------------------------------------------------------------------
// The library reads no environment variable.  Tests and sweeps override a policy value through tr_set_tuning();
// tr_knob() returns the override, or dflt when none is set (0 = not set).
enum TrKnob {
    TR_KNOB_WG_ROWS,        // packed rows per attention workgroup: 32, 128 or 256
    TR_KNOB_TARGET_ITEMS,   // workgroups a single request's key split aims for
    TR_KNOB_MIN_SPLIT_KEYS, // shortest key split
    TR_KNOB_ASM_SPAN,       // 16-byte units of K (and V) per assemble workgroup
    TR_KNOB_BD_PIECE_TILES, // key tiles per piece when the one-pass kernel cuts a long key range
    TR_KNOB_BD_SLOTS,       // resident workgroups the one-pass planner balances for
    TR_KNOB_LIN_SPLIT,      // slices of k in tr_linear
    TR_KNOB_LIN_MSPLIT,     // 1: never split the rows of x over two workgroups
    TR_KNOB_COUNT
};
int tr_knob(int which, int dflt);

// ---- the chip the launch planners are written for (MI355X, gfx950) ------------------------------------------------
// One table instead of constants scattered over the planners.  The *_US and *_PER_US figures are measured on that
// part and only steer how work is cut; no result depends on them.
struct TrChip {
    static constexpr int XCDS = 8;                 // accelerator dies; blocks are dealt to them round-robin
    static constexpr int CUS = 256;                // compute units, 32 per XCD
    static constexpr int SLOTS_128 = 512;          // resident 128-row attention workgroups (two per CU)
    static constexpr int SLOTS_256 = 256;          // resident 256-row attention workgroups (one per CU)
    static constexpr double KEY_TILE_STEP_US = 2.0;        // one 64-key step of a resident attention workgroup
    static constexpr double WORKGROUP_FIXED_STEPS = 3.0;   // prologue + epilogue of a workgroup, in such steps
    static constexpr double PARTIAL_BYTES_PER_US = 2.0e6;  // split partials, written and read back: ~4 TB/s for both
};

// theta_m = base^(-2m/d) in double (text after Eq. 3)
void tr_fill_theta(const tr_shape* s, double* theta /*[64]*/);

// ---- kernel argument blocks (passed by value; each stays below 4 KB of kernarg) ------------------------------

// One contiguous run of rows to move: src rows [src_row, src_row+n_rows) -> dst rows [dst_row, ...),
// keys additionally turned by delta positions (0: plain copy).
struct TrCopyDesc {
    int32_t src_row;
    int32_t dst_row;
    int32_t n_rows;
    int32_t delta;
    int32_t blk_start; // first block of the grid that works on this run
};
#define TR_MAX_COPY_DESC 168 // what the 4 KB argument block holds
// optional tail of an assemble launch: one request's query tokens appended by the blocks from first_block on
struct TrAppendTail {
    const void* k_new;
    const void* v_new;
    const int32_t* q_pos;
    int32_t n_q; // 0: no tail
    int32_t dst_row0;
    int32_t first_block;
    int32_t n_kv_heads;
};
struct TrAssembleArgs {
    const void* k_src;
    const void* v_src;
    void* k_dst;
    void* v_dst;
    int32_t n_desc;
    int32_t row_units;  // 16-byte units per row (n_kv_heads * head_dim * elem / 16)
    int32_t head_units; // 16-byte units per head
    int32_t span_units; // units of K (and of V) one block moves; multiple of 256
    int32_t half_dim;   // head_dim / 2
    int32_t rope_half;  // 1: pairs are (m, m + d/2) instead of (2m, 2m+1)
    double theta[64];
    TrAppendTail app;
    TrCopyDesc desc[TR_MAX_COPY_DESC];
};

// append: request r's tokens [q_row0, q_row0+n_q) go to cache rows [dst_row0, dst_row0+n_q)
struct TrAppendDesc {
    int32_t q_row0;
    int32_t n_q;
    int32_t dst_row0;
    int32_t pos0; // position id of the first token when the launch carries no q_pos array (raw-store assembly)
};
#define TR_MAX_APPEND_DESC 128
struct TrAppendArgs {
    const void* k_new;
    const void* v_new;
    const int32_t* q_pos;
    void* cache_k;
    void* cache_v;
    int32_t n_desc;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t total_tokens; // tokens covered by this launch (sum of n_q)
    int32_t rope_half;
    int32_t pad_;
    double theta[64];
    TrAppendDesc desc[TR_MAX_APPEND_DESC];
};

// prefix attention: one request
struct TrSeqDesc {
    int32_t q_row0;    // first packed query token of the request (row of q / out / q_pos)
    int32_t n_q;
    int32_t kv_row0;   // first cache row of the request
    int32_t kv_len;
    int32_t item0;     // first work item of the request in this launch
    int32_t n_tiles;   // row tiles
    int32_t n_split;   // KV splits (>= 1)
    int32_t split_len; // keys per split, multiple of the key tile
    int32_t ws_row0;   // first partial row of the request in the workspace
    int32_t pad_;
};
#define TR_MAX_SEQ 64
struct TrPrefixArgs {
    const void* q;
    const void* k;
    const void* v;
    const int32_t* q_pos;
    void* out;
    _Float16* ws_o; // [partial rows][head_dim] partial outputs, each normalised by its own denominator
    float* ws_ml; // [partial rows][2] reference maximum (log2 domain) and softmax denominator
    int32_t n_seq;
    int32_t n_items;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t group;
    int32_t tok_per_tile;
    float scale_log2e; // log2(e) / sqrt(head_dim)
    float scale;       // 1 / sqrt(head_dim)
    int32_t rope_half;
    int32_t pad_;
    double theta_rev[64]; // theta_m / (2 pi): position * theta_rev = angle in revolutions
    double theta[64];
    TrSeqDesc seq[TR_MAX_SEQ];
};

// gather attention: the keys of one request, read where they lie.  A segment is one retrieved chunk in the store
// (rows src_row .. +n_rows, keys stored at chunk-local positions, delta = the chunk's offset under reordered
// positions, else 0), or, last, the request's own query tokens in its cache (delta 0).
struct TrGatherSeg {
    int32_t src_row;
    int32_t n_rows;
    int32_t delta;
    int32_t tile0;     // first 64-key tile of the segment in the request's tile list
    int32_t cache_row; // cache row its first key would have after assembly
};
#define TR_MAX_GATHER_SEG 96
struct TrGatherArgs {
    const void* q;
    const void* k_store;
    const void* v_store;
    const void* k_cache;
    const void* v_cache;
    const int32_t* q_pos;
    void* out;
    _Float16* ws_o;
    float* ws_ml;
    int32_t n_q;
    int32_t n_doc;
    int32_t n_seg;           // segments, the query-token segment included (it is the last)
    int32_t n_tiles_total;
    int32_t n_split;
    int32_t tiles_per_split;
    int32_t row_tiles;
    int32_t n_items;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t group;
    int32_t tok_per_tile;
    float scale_log2e;
    int32_t rope_half;
    double theta_rev[64];
    TrGatherSeg seg[TR_MAX_GATHER_SEG];
};

// A run of consecutive row tiles of the block-diagonal kernel that share one split count.  Items of a KV head are
// numbered segment by segment, tiles in DESCENDING order inside a segment, the splits of a tile next to each other.
struct TrBdSeg {
    int32_t tile_hi;   // last (highest) row tile of the segment: the first one issued
    int32_t n_tiles;
    int32_t n_split;   // pieces the key walk of each tile is cut into (>= 1)
    int32_t split_len; // keys per piece, a multiple of 64; the last piece runs to the end of the walk
    int32_t item0;     // first item of the segment inside a KV head's item list
    int32_t ws_row0;   // first partial row of the segment (n_split > 1)
    int32_t tok0;      // first token of the segment
    int32_t n_tok;     // tokens in the segment
};
#define TR_MAX_BD_SEG 64
struct TrBlockDiagArgs {
    const void* q;
    const void* k; // rotated keys K'
    const void* v;
    const int32_t* tok_start; // [T] first row each token may attend (the start of its chunk)
    const int32_t* pos;       // [T] RoPE position ids, or NULL: position = t - tok_start[t]
    void* out;
    int32_t total_tokens;
    int32_t n_tiles;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t group;
    int32_t tok_per_tile;
    float scale_log2e;
    float scale;
    int32_t rope_half;
    int32_t n_seg;
    int32_t items_per_head;
    int32_t pad_;
    _Float16* ws_o; // partial outputs and statistics of split tiles, laid out as in TrPrefixArgs
    float* ws_ml;
    double theta_rev[64];
    double theta[64];
    TrBdSeg seg[TR_MAX_BD_SEG];
};

static_assert(sizeof(TrAssembleArgs) <= 4096 && sizeof(TrAppendArgs) <= 4096 && sizeof(TrPrefixArgs) <= 4096 &&
                  sizeof(TrGatherArgs) <= 4096 && sizeof(TrBlockDiagArgs) <= 4096,
              "kernel argument blocks must fit the 4 KB kernarg segment");

// ---- launchers implemented in the .hip files --------------------------------------------------------------
int tr_launch_assemble(const TrAssembleArgs& a, int dtype, int n_blocks, hipStream_t s);
int tr_launch_append(const TrAppendArgs& a, int dtype, hipStream_t s);
int tr_launch_prefix_attn(const TrPrefixArgs& a, int head_dim, int wg_rows, bool any_split, int total_rows, hipStream_t s);
int tr_launch_prefix_attn_f32(const TrPrefixArgs& a, int head_dim, int total_rows, hipStream_t s);
int tr_launch_rope_table(double* table, int n_pos, int half_dim, const double* theta, hipStream_t s);
int tr_launch_rope_rows(const void* k, void* k_rot, const int32_t* cu, int n_chunks, int max_chunk_len, int32_t* tok_start,
                        const double* table, int table_rows, int64_t total_tokens, const tr_shape* shape, hipStream_t s);
static inline int tr_rope_half(const tr_shape* s) { return s->rope_layout == TR_ROPE_HALF ? 1 : 0; }
// combine: NULL, or the arguments of the merge over the split tiles' tokens (combine_rows = tokens x query heads)
int tr_launch_blockdiag_attn(const TrBlockDiagArgs& a, const TrPrefixArgs* combine, int combine_rows, int head_dim, int wg_rows,
                             hipStream_t s);
int tr_launch_gather_attn(const TrGatherArgs& a, const TrPrefixArgs& combine_args, int head_dim, hipStream_t s);
int tr_launch_blockdiag_attn_f32(const TrBlockDiagArgs& a, int head_dim, hipStream_t s);
// y_j = x w_j^T for at most 128 rows of x and up to TR_LINEAR_MAX_OUT weights that share x; N = sum of the feature
// counts; partial: fp32 [tr_linear_splits(M, N, K), M, N] when that count exceeds 1
#define TR_LINEAR_MAX_OUT 4
int tr_linear_splits(int32_t M, int32_t N, int32_t K);
// sink: 256 * 512 floats.  *flops receives the multiply-add count x 2 of the launch.
int tr_launch_mfma_loop_probe(int iters, int random_operands, float* sink, hipStream_t s, double* flops);
int tr_launch_linear(const void* x, int32_t n_out, const void* const* w, void* const* y, const int32_t* n_features, void* partial,
                     int32_t M, int32_t K, hipStream_t s);
