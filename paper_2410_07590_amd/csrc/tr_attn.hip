// bf16 MFMA attention kernels for gfx950: query prefill over an assembled cache (Sec. 3.4 step 6) and the
// offline block-diagonal chunk prefill (Sec. 3.4 step 2, independent attention of Sec. 3.2).
//
// Work decomposition.  A "packed row" is one (query token, query head of a GQA group) pair: the g query heads
// that share a KV head are stacked along the MFMA M dimension, so one K/V tile fetched from HBM serves all of
// them.  A workgroup of NW wavefronts owns 32*NW packed rows of one KV head; each wavefront owns 32 rows and
// walks the visible keys in tiles of 64.
//
// Transposed products.  S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16: A = K rows / V^T rows
// from LDS, B = rotated queries / P^T from registers.  Each lane then owns ONE query column, so the softmax
// statistics are per-lane scalars, and the S^T accumulator layout already is the B-operand layout of the
// second product, up to a permutation of the 16 keys inside a k-step that the V^T reads apply as well.
// V^T operands come from row-major V tiles through the transposing LDS read (ds_read_b64_tr_b16).
//
// Data movement.  K/V tiles go global -> LDS directly (global_load_lds_dwordx4, no staging registers) into a
// ring of NS stages; rows are stored unpadded and XOR-swizzled per 16-byte chunk so that the MFMA operand
// reads are bank-conflict free.  One s_barrier per tile; s_waitcnt vmcnt counts are managed by hand because
// the loads are asynchronous with respect to the wave that issued them.
//
// Softmax works in the log2 domain with a lazily updated reference maximum: the accumulators are rescaled
// only when the running maximum grew by more than 2^8, which is exact (softmax is invariant to the reference)
// and keeps P <= 256.
#include "tr_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

constexpr int KT = 64;               // keys per tile
constexpr float RESCALE_SLACK = 8.f; // log2 units a tile maximum may exceed the reference before a rescale
constexpr int K_PREFETCH = 2;        // k-steps the K operand reads run ahead of the score products
constexpr float REREF_BELOW = -32.f; // a row's first visible tile re-references when its maximum is below this

template <int D> struct Geo {
    static constexpr int CPR = D / 8;            // 16-byte chunks per row of one head
    static constexpr int RPI = 64 / CPR;         // rows moved by one wave-wide 1 KB load
    static constexpr int NI = KT / RPI;          // such loads per K (or V) tile
    static constexpr int TILE_BYTES = KT * D * 2;
    static constexpr int STAGE_BYTES = 2 * TILE_BYTES; // K tile then V tile
    static constexpr int GPR = CPR / 4;          // 64-byte groups per row
    // K: chunk c of row r sits at chunk c ^ kswz(r): 16 consecutive rows of one logical chunk cover all banks
    __device__ static __forceinline__ int kswz(int r) { return (r / (16 / CPR)) & (CPR - 1); }
    // V: 64-byte group q of row r sits at group q ^ vswz(r): 4 consecutive rows of one group cover all banks
    __device__ static __forceinline__ int vswz(int r) { return (r / (4 / GPR)) & (GPR - 1); }
};

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
template <int N> __device__ __forceinline__ void wait_vm() { __builtin_amdgcn_s_waitcnt(vmcnt_imm(N)); }

struct RowCtx {
    bool valid;
    int orow;    // q_tok * n_q_heads + head: row of q / out in units of head vectors
    int key_lo;  // first visible cache row
    int key_hi;  // last visible cache row
};

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ int xcd_remap(int bid, int n)
{
    // Blocks are dealt round-robin to the 8 XCDs; give each XCD one contiguous range of items so that
    // items sharing K/V tiles meet in the same L2.
    const int x = bid & 7, idx = bid >> 3;
    const int q = n >> 3, r = n & 7;
    return x * q + (x < r ? x : r) + idx;
}

// Maximum and sum over the two lanes c and c + 32, which hold the two key halves of one query column, through the
// cross-half swap of the vector unit.  These exchanges sit on the critical path of every tile: an LDS permute would put
// an LDS round trip there, and its wait would also wait for every operand read in flight.
// permlane32_swap(u, u): result[0] = lanes 0..31 of u in both halves, result[1] = lanes 32..63 of u in both halves.
__device__ __forceinline__ float column_max(float x)
{
    const uint32_t u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float column_sum(float x)
{
    const uint32_t u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Maximum / minimum of an int over the wave, as a uniform value.  Four cross-lane steps inside each row of 16 lanes on
// the vector unit's data-parallel path (pairs, quads, the mirrored half-row, the mirrored row: max and min do not care
// which lanes meet, only that all do), then the four rows' results through scalar registers.  Every lane of the wave must
// be active.  (A butterfly of six LDS permutes does the same with six dependent LDS round trips; a workgroup of the
// offline kernel needs four such reductions before its first tile load can go out.)
template <bool MAX> __device__ __forceinline__ int wave_reduce_i(int v)
{
    auto op = [](int a, int b) { return MAX ? max(a, b) : min(a, b); };
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xf, 0xf, false));  // quad_perm [1,0,3,2]
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xf, 0xf, false));  // quad_perm [2,3,0,1]
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xf, 0xf, false)); // row_half_mirror
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xf, 0xf, false)); // row_mirror
    const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
    const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
    return op(op(r0, r1), op(r2, r3));
}
__device__ __forceinline__ int wave_max_i(int v) { return wave_reduce_i<true>(v); }
__device__ __forceinline__ int wave_min_i(int v) { return wave_reduce_i<false>(v); }

// ---- rotated queries (Eq. 3 at the token's position id) -------------------------------------------------------
// Lane (c = lane & 31, h = lane >> 5) ends up holding Q'[row c][16 ks + 8 h .. +7] for ks < D/16, scaled by
// log2(e)/sqrt(d) before its single rounding to bf16.  Angles are reduced in fp64 to [-1/2, 1/2] revolutions and
// then go through v_sin/v_cos, which take revolutions.

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int ROT_SLOTS = 8; // token slots per rotation pass; covers a wave's 32 packed rows when the GQA group is >= 4

// Issue the loads of this lane's raw fragments; rows that do not exist read row 0 and are zeroed later.
template <int D>
__device__ __forceinline__ void load_q_raw(const __bf16* __restrict__ q, const RowCtx& rc, int h, u32x4 (&raw)[D / 16])
{
    const __bf16* qrow = q + (int64_t)(rc.valid ? rc.orow : 0) * D + 8 * h;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) raw[ks] = *(const u32x4*)(qrow + 16 * ks);
}

// cn, sn: cosine and sine of the pair's angle, already multiplied by the score scale.  Rows that do not exist are
// rotated like any other (they hold row 0's values and are never stored).
__device__ __forceinline__ void rot_pair(uint32_t w, float cn, float sn, bf16x8& f, int p)
{
    const float xa = bf_lo(w), xb = bf_hi(w);
    f[2 * p] = (__bf16)(xa * cn - xb * sn);
    f[2 * p + 1] = (__bf16)(xb * cn + xa * sn);
}

// The g query heads of a token share its angles, so a wave's 32 rows need at most ROT_SLOTS x D/2 distinct
// (cos, sin) pairs instead of 32 x D/2: the wave computes them once into a private LDS table, lane -> pair index,
// one token slot (two for D = 64) per step.  pos_lane: position id of slot (lane & 7).
// Table layout: slot j, pair m at byte j * 4 D + (((m >> 1) ^ 2 j) * 16) + (m & 1) * 8.
template <int D>
__device__ __forceinline__ void build_rot_table(LDS_AS char* tab, double th /* theta_rev[lane % (D/2)] */, int lane, int pos_lane,
                                                float sl2e /* log2(e) / sqrt(d): folded into the table */)
{
    constexpr int PAIRS = D / 2, LPS = 64 / PAIRS;
    const int m = lane % PAIRS;
#pragma unroll
    for (int pass = 0; pass < ROT_SLOTS / LPS; ++pass) {
        const int j = pass * LPS + lane / PAIRS;
        double rev = (double)__shfl(pos_lane, j) * th;
        rev -= rint(rev);
        const float x = (float)rev;
        f32x2 cs;
        cs[0] = __builtin_amdgcn_cosf(x) * sl2e;
        cs[1] = __builtin_amdgcn_sinf(x) * sl2e;
        *(LDS_AS f32x2*)(tab + j * (4 * D) + (((m >> 1) ^ (2 * j)) * 16) + (m & 1) * 8) = cs;
    }
}

template <int D>
__device__ __forceinline__ void rotate_q_shared(const u32x4 (&raw)[D / 16], LDS_AS const char* tab, int slot, int h,
                                                bf16x8 (&qf)[D / 16])
{
    LDS_AS const char* row = tab + slot * (4 * D);
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        // pairs 8 ks + 4 h .. +3 = 16-byte chunks 2 u, 2 u + 1 with u = 2 ks + h
        const int ch = (2 * (2 * ks + h)) ^ (2 * slot);
        const f32x4 cs0 = *(LDS_AS const f32x4*)(row + ch * 16);
        const f32x4 cs1 = *(LDS_AS const f32x4*)(row + ch * 16 + 16);
        bf16x8 f;
        rot_pair(raw[ks][0], cs0[0], cs0[1], f, 0);
        rot_pair(raw[ks][1], cs0[2], cs0[3], f, 1);
        rot_pair(raw[ks][2], cs1[0], cs1[1], f, 2);
        rot_pair(raw[ks][3], cs1[2], cs1[3], f, 3);
        qf[ks] = f;
    }
}

// Half-split layout: channel c < D/2 pairs with c + D/2, i.e. fragment ks (channels 16 ks + 8 h .. +7) pairs element by
// element with fragment ks + D/32, and the pair index of element e is 16 ks + 8 h + e.  row: the token slot's table
// row, sw: twice the slot (the swizzle of its 16-byte chunks).
template <int D>
__device__ __forceinline__ void rot_frag_half(const u32x4& lo, const u32x4& hi, LDS_AS const char* row, int ks, int h, int sw,
                                              bf16x8& flo, bf16x8& fhi)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) { // two pairs (one 16-byte table chunk) at a time
        const int ch = (8 * ks + 4 * h + q) ^ sw;
        const f32x4 cs = *(LDS_AS const f32x4*)(row + ch * 16);
        const float la = bf_lo(lo[q]), lb = bf_hi(lo[q]);
        const float ha = bf_lo(hi[q]), hb = bf_hi(hi[q]);
        flo[2 * q] = (__bf16)(la * cs[0] - ha * cs[1]);
        fhi[2 * q] = (__bf16)(ha * cs[0] + la * cs[1]);
        flo[2 * q + 1] = (__bf16)(lb * cs[2] - hb * cs[3]);
        fhi[2 * q + 1] = (__bf16)(hb * cs[2] + lb * cs[3]);
    }
}

template <int D>
__device__ __forceinline__ void rotate_q_shared_half(const u32x4 (&raw)[D / 16], LDS_AS const char* tab, int slot, int h,
                                                     bf16x8 (&qf)[D / 16])
{
    LDS_AS const char* row = tab + slot * (4 * D);
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) rot_frag_half<D>(raw[ks], raw[ks + D / 32], row, ks, h, 2 * slot, qf[ks], qf[ks + D / 32]);
}

// Rotated, scaled queries of a wave from their raw fragments.  slot: which of the wave's tokens this lane's row
// belongs to (0 .. n_slots-1, n_slots wave-uniform); pos_of_slot(s): position id of the wave's token slot s (any
// value for slots past the wave's last token).  Tokens go through the table ROT_SLOTS at a time: one pass when the
// GQA group is >= 4, up to four for smaller groups.
template <int D, bool HALF, class PosFn>
__device__ __forceinline__ void rotate_queries(const u32x4 (&raw)[D / 16], LDS_AS char* tab, double th, int lane, int h, int slot,
                                               int n_slots, float sl2e, PosFn pos_of_slot, bf16x8 (&qf)[D / 16])
{
    n_slots = __builtin_amdgcn_readfirstlane(n_slots);
    for (int p0 = 0; p0 < n_slots; p0 += ROT_SLOTS) {
        build_rot_table<D>(tab, th, lane, pos_of_slot(p0 + (lane & (ROT_SLOTS - 1))), sl2e);
        const bool mine = (slot >= p0) && (slot < p0 + ROT_SLOTS);
        bf16x8 f[D / 16];
        if (HALF) rotate_q_shared_half<D>(raw, tab, mine ? slot - p0 : 0, h, f);
        else rotate_q_shared<D>(raw, tab, mine ? slot - p0 : 0, h, f);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            if (mine || p0 == 0) qf[ks] = f[ks]; // the first pass initialises every lane's fragments
        __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0): the table is read before the next pass (or a tile load) overwrites it
    }
}

// Per-wave state of the tile loop.
template <int D> struct Acc {
    f32x16 o[D / 32]; // O^T: element e of block db is channel 32 db + 8 (e >> 2) + 4 h + (e & 3) of query column c
    float mref;       // reference maximum, log2 domain (score * log2(e)/sqrt(d))
    float l;          // this half-wave's share of the softmax denominator
};

// Issue this wave's share of the direct global->LDS loads of tile [kt, kt+KROWS) into one stage (K rows, then V rows).
// AUX is the cache policy of the loads: 0 where other workgroups read the same tile soon (the row tiles of a long
// query), DMA_STREAM (non-temporal) where every key is read exactly once (decode: 114 -> 100 us for 64 x 4096 rows;
// the same hint on the long-query kernels, whose row tiles share keys through L2, cost 5-8 %).
constexpr int DMA_STREAM = 2;
template <int D, int NW, int KROWS = KT, int AUX = 0>
__device__ __forceinline__ void issue_tile(const __bf16* __restrict__ k, const __bf16* __restrict__ v, int64_t row_elems,
                                           int head_off, int kt, int key_clamp, LDS_AS char* stage, int wave, int lane)
{
    using G = Geo<D>;
    constexpr int NI = KROWS / G::RPI;
    static_assert(NI % NW == 0, "tile loads must divide evenly over the waves");
    const int r_in = lane / G::CPR, pc = lane % G::CPR;
#pragma unroll
    for (int ii = 0; ii < NI / NW; ++ii) {
        const int i = wave + NW * ii;
        const int row = i * G::RPI + r_in;
        int key = kt + row;
        key = key > key_clamp ? key_clamp : key;
        const int ck = pc ^ G::kswz(row);
        const int cv = 4 * ((pc >> 2) ^ G::vswz(row)) + (pc & 3);
        const int64_t base = (int64_t)key * row_elems + head_off;
        __builtin_amdgcn_global_load_lds((const GLB_AS void*)(k + base + ck * 8), (LDS_AS void*)(stage + i * 1024), 16, 0, AUX);
        __builtin_amdgcn_global_load_lds((const GLB_AS void*)(v + base + cv * 8),
                                         (LDS_AS void*)(stage + KROWS * D * 2 + i * 1024), 16, 0, AUX);
    }
}

// One tile of 32 KB keys in two phases.  Phase A: S^T = K Q^T and the online softmax, leaving P^T packed as bf16 B
// operands.  Phase B: O^T += V^T P^T.  krows / vrows point at the tile's first K / V row in LDS, kt is its first key.
struct NoHook {
    __device__ __forceinline__ void operator()(int) const {}
};

// between(ks) runs after the products of k-step ks have been issued: the tile loop puts its loads of a later tile
// there, so that their issue falls into the shadow of the matrix instructions instead of in front of them.
template <int D, int KB, class Between = NoHook>
__device__ __forceinline__ void scores_softmax(LDS_AS const char* krows, const bf16x8 (&qf)[D / 16], const RowCtx& rc, int kt,
                                               bool need_mask, const int (&koff)[D / 16], int h, Acc<D>& acc, bf16x8 (&bpk)[KB][2],
                                               Between between = Between())
{
    // scores relative to the row reference, in the log2 domain (the queries carry log2(e)/sqrt(d)): the
    // accumulators start at -mref, so P = exp2(S) needs no further arithmetic
    f32x16 s[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[kb][e] = -acc.mref;
    // operand reads run K_PREFETCH k-steps ahead of the products that use them (the compiler, left alone, reads one
    // step ahead and waits out the full LDS latency before every pair of products)
    constexpr int PD = K_PREFETCH, STEPS = D / 16;
    bf16x8 a[PD][KB];
#pragma unroll
    for (int ks = 0; ks < PD; ++ks)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) a[ks][kb] = *(LDS_AS const bf16x8*)(krows + koff[ks] + kb * 32 * D * 2);
#pragma unroll
    for (int ks = 0; ks < STEPS; ++ks) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks % PD][kb], qf[ks], s[kb], 0, 0, 0);
        if (ks + PD < STEPS) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) a[ks % PD][kb] = *(LDS_AS const bf16x8*)(krows + koff[ks + PD] + kb * 32 * D * 2);
        }
        between(ks);
        __builtin_amdgcn_sched_barrier(0);
    }
    // accumulator element e of block kb is key kt + 32 kb + 8 (e >> 2) + 4 h + (e & 3), query column c
    if (need_mask) { // workgroup-uniform: only tiles that straddle a mask edge
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = kt + 32 * kb + 8 * (e >> 2) + 4 * h + (e & 3);
                if (key < rc.key_lo || key > rc.key_hi) s[kb][e] = -INFINITY;
            }
    }
    float part[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY}; // four short chains instead of one long one
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) part[e & 3] = fmaxf(part[e & 3], s[kb][e]);
    float mx = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    mx = column_max(mx); // both half-waves hold keys of the same query column
    // lazy reference update (exact: any reference gives the same softmax).  `first`: nothing accumulated yet and the
    // tile sits far below the reference - move the reference down so that exp2 does not underflow.  Lanes c and c + 32
    // hold the two key halves of ONE query column and share its reference, so the decision is taken on the column's
    // denominator: a row whose first visible keys all fell into one half must not move the other half's reference alone.
    const float l_col = column_sum(acc.l);
    const bool first = (l_col == 0.0f) && (mx < REREF_BELOW) && (mx > -INFINITY);
    const bool grow = (mx > RESCALE_SLACK) || first;
    if (__any(grow)) { // rare
        const float delta = grow ? mx : 0.0f;
        const float alpha = first ? 1.0f : __builtin_amdgcn_exp2f(-delta); // first: accumulators are still zero
        acc.mref += delta;
        acc.l *= alpha;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc.o[db][e] *= alpha;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) s[kb][e] -= delta;
    }
    // P = exp2(S), packed to bf16 B-operands; the denominator sums the rounded weights the product uses
    {
        bf16x2 ones;
        ones[0] = (__bf16)1.0f;
        ones[1] = (__bf16)1.0f;
        float l = acc.l;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                bf16x2 pr;
                pr[0] = (__bf16)__builtin_amdgcn_exp2f(s[kb][2 * i]);
                pr[1] = (__bf16)__builtin_amdgcn_exp2f(s[kb][2 * i + 1]);
                bpk[kb][i / 4][2 * (i % 4)] = pr[0];
                bpk[kb][i / 4][2 * (i % 4) + 1] = pr[1];
                l = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l, false);
            }
        acc.l = l;
    }
}

// O^T += V^T P^T.  k-slot j of k-step (kb, t) is key 32 kb + 16 t + 8 (j >> 2) + 4 h + (j & 3).
template <int D, int KB>
__device__ __forceinline__ void weighted_values(LDS_AS const char* vrows, const bf16x8 (&bpk)[KB][2], const int (&voff)[D / 32],
                                                Acc<D>& acc)
{
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const bf16x8 bp = bpk[kb][t];
            const int rbase = (32 * kb + 16 * t) * D * 2;
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                LDS_AS const char* p0 = vrows + rbase + voff[db];
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(p0 + 8 * D * 2));
                const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                acc.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), bp, acc.o[db], 0, 0, 0);
            }
        }
}

// The rows of K/V one workgroup walks: tiles of 64 keys from kt_begin, n_tiles of them; key_clamp is the last row
// that may be loaded (rows past it are never visible and read that row instead).
struct Walk {
    int kt_begin;
    int n_tiles;
    int key_clamp;
    int head_off;
    int64_t row_elems;
};

__device__ __forceinline__ Walk make_walk(int kt_begin, int kt_end, int key_clamp, int n_kv_heads, int kvh, int d)
{
    Walk w;
    w.kt_begin = kt_begin;
    w.n_tiles = kt_end > kt_begin ? (kt_end - kt_begin + KT - 1) / KT : 0;
    w.key_clamp = key_clamp;
    w.head_off = kvh * d;
    w.row_elems = (int64_t)n_kv_heads * d;
    return w;
}

// Tiles 0 .. NS-2 in flight.  Stage NS-1 stays free until the tile loop's first iteration has passed its barrier.
template <int D, int NW, int NS, int AUX = 0>
__device__ __forceinline__ void issue_prologue(const __bf16* __restrict__ k, const __bf16* __restrict__ v, const Walk& w,
                                               LDS_AS char* smem, int wave, int lane)
{
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (p < w.n_tiles)
            issue_tile<D, NW, KT, AUX>(k, v, w.row_elems, w.head_off, w.kt_begin + p * KT, w.key_clamp, smem + p * Geo<D>::STAGE_BYTES, wave, lane);
}

// This wave's loads of one whole tile whose 64 rows all exist (no clamping): the lane's byte offsets inside the tile
// were computed once (dk, dv), the tile's first row is a uniform base, so a load costs no vector arithmetic.
// load pair ii of this wave: 1 KB of the K tile and 1 KB of the V tile
template <int D, int NW, int AUX>
__device__ __forceinline__ void issue_pair_at(const char* __restrict__ ktile, const char* __restrict__ vtile, uint32_t dk, uint32_t dv,
                                              uint32_t lds_wave, int stage_off, int ii)
{
    const uint32_t dst = lds_wave + (uint32_t)(stage_off + NW * ii * 1024);
    __builtin_amdgcn_global_load_lds((const GLB_AS void*)(ktile + dk), (LDS_AS void*)(uintptr_t)dst, 16, 0, AUX);
    __builtin_amdgcn_global_load_lds((const GLB_AS void*)(vtile + dv), (LDS_AS void*)(uintptr_t)(dst + Geo<D>::TILE_BYTES), 16, 0, AUX);
}

template <int D, int NW, int AUX>
__device__ __forceinline__ void issue_tile_at(const char* __restrict__ ktile, const char* __restrict__ vtile,
                                              const uint32_t (&dk)[Geo<D>::NI / NW], const uint32_t (&dv)[Geo<D>::NI / NW],
                                              uint32_t lds_wave /* LDS address of this wave's first 1 KB slot in stage 0 (uniform) */,
                                              int stage_off /* constant */)
{
    using G = Geo<D>;
#pragma unroll
    for (int ii = 0; ii < G::NI / NW; ++ii) issue_pair_at<D, NW, AUX>(ktile, vtile, dk[ii], dv[ii], lds_wave, stage_off, ii);
}

// The tile loop shared by both kernels (issue_prologue has run).  Tile [kt, kt+64) needs per-element masking iff
// kt+63 > mask_hi_min or kt < mask_lo_max.  The loop is unrolled over the ring so that the stage of every LDS
// access is a constant of the instruction: the operand reads then need no address arithmetic at all (the lane's
// offsets inside a stage are loop constants, the stage goes into the instruction's offset field, whose 16 bits
// reach two 32 KB stages: a four-stage ring keeps a second set of offsets for stages 2 and 3).
template <int D, int NW, int NS, int AUX = 0>
__device__ __forceinline__ void attn_tiles(const __bf16* __restrict__ k, const __bf16* __restrict__ v, const Walk& w,
                                           const RowCtx& rc, const bf16x8 (&qf)[D / 16], int mask_hi_min, int mask_lo_max,
                                           LDS_AS char* smem, Acc<D>& acc)
{
    using G = Geo<D>;
    constexpr int IPW = 2 * G::NI / NW; // loads each wave issues per tile
    static_assert(G::NI % NW == 0, "tile loads must divide evenly over the waves");
    static_assert(NS == 2 || NS == 4, "the ring has two or four stages");
    constexpr int BANKS = NS / 2;        // sets of lane offsets: one per 64 KB of ring
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, colhalf = (lane >> 4) & 1;

    const int wave_hi_max = wave_max_i(rc.valid ? rc.key_hi : INT32_MIN);
    const int wave_lo_min = wave_min_i(rc.valid ? rc.key_lo : INT32_MAX);

    // LDS addresses of this lane's operands in stage 2b (bank b serves stages 2b and 2b + 1): whole addresses, the
    // ring's base included, so that what an access adds is a constant that fits its offset field
    const int lds0 = (int)(uintptr_t)smem;
    const uint32_t lds_wave = (uint32_t)__builtin_amdgcn_readfirstlane(lds0 + wave * 1024);
    int koff[BANKS][D / 16];
    int voff[BANKS][D / 32];
#pragma unroll
    for (int b = 0; b < BANKS; ++b) {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) koff[b][ks] = lds0 + b * 2 * G::STAGE_BYTES + c * D * 2 + (((2 * ks + h) ^ G::kswz(c)) * 16);
        const int r = 4 * h + (i16 >> 2); // row inside an 8-row k-slot block; rows 8 apart share the swizzle
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
            voff[b][db] = lds0 + b * 2 * G::STAGE_BYTES + r * D * 2 + (4 * (db ^ G::vswz(r)) + 2 * colhalf + ((i16 & 3) >> 1)) * 16 + (i16 & 1) * 8;
    }
    // byte offsets of this wave's tile loads from the tile's first row
    uint32_t dk[G::NI / NW], dv[G::NI / NW];
    {
        const int r_in = lane / G::CPR, pc = lane % G::CPR;
        const uint32_t row_bytes = (uint32_t)w.row_elems * 2u;
#pragma unroll
        for (int ii = 0; ii < G::NI / NW; ++ii) {
            const int row = (wave + NW * ii) * G::RPI + r_in;
            const int ck = pc ^ G::kswz(row);
            const int cv = 4 * ((pc >> 2) ^ G::vswz(row)) + (pc & 3);
            dk[ii] = (uint32_t)row * row_bytes + (uint32_t)(w.head_off + ck * 8) * 2u;
            dv[ii] = (uint32_t)row * row_bytes + (uint32_t)(w.head_off + cv * 8) * 2u;
        }
    }
    const int64_t row_bytes64 = w.row_elems * 2;

    const int n_tiles = w.n_tiles;
    bf16x8 bpk[2][2];
    // Interior tiles first, a ring-full at a time, in a loop with nothing to decide: every row of the workgroup sees
    // every key of the tile (no mask, every wave that has rows computes), the tile requested behind each barrier
    // exists and has all its rows (the plain loads), so the wait counts are constants.  A long document prefix is almost all interior; the general loop below takes over wherever this stops.
    // Only the eight-wave kernel has it (2 % at the long-query configuration): in the four-wave kernels it would have to
    // give up the loads issued between the score products (with them the compiler spills), and measured 2 % slower.
    int t0 = 0;
    if (NW == 8) {
        // tiles [0, t_b) lie wholly below the first row's causal edge; the lower edge must not cut into the walk at all
        const int t_b = mask_lo_max <= w.kt_begin ? (mask_hi_min - (KT - 1) - w.kt_begin >= 0 ? (mask_hi_min - (KT - 1) - w.kt_begin) / KT + 1 : 0) : 0;
        const bool wave_has_rows = wave_hi_max != INT32_MIN;
        // a group of NS tiles from t0: all interior (t0 + NS <= t_b), all requested tiles t0 + NS - 1 .. t0 + 2 NS - 2 exist
        // and are not the walk's last tile, the only one that may lack rows (t0 + 2 NS <= n_tiles)
        for (; t0 + NS <= t_b && t0 + 2 * NS <= n_tiles; t0 += NS) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                wait_vm<(NS - 2) * IPW>();
                __builtin_amdgcn_s_barrier();
                const int dst_off = ((s + NS - 1) % NS) * G::STAGE_BYTES;
                const int ktn = w.kt_begin + (t0 + s + NS - 1) * KT;
                const char* ktile = (const char*)k + (int64_t)ktn * row_bytes64;
                const char* vtile = (const char*)v + (int64_t)ktn * row_bytes64;
                LDS_AS const char* stage = (LDS_AS const char*)(uintptr_t)((s % 2) * G::STAGE_BYTES);
                issue_tile_at<D, NW, AUX>(ktile, vtile, dk, dv, lds_wave, dst_off);
                if (wave_has_rows) {
                    scores_softmax<D, 2>(stage, qf, rc, 0, false, koff[s / 2], h, acc, bpk);
                    weighted_values<D, 2>(stage + G::TILE_BYTES, bpk, voff[s / 2], acc);
                }
            }
        }
    }
    for (; t0 < n_tiles; t0 += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int t = t0 + s;
            if (t >= n_tiles) break;
            const int kt = w.kt_begin + t * KT;
            // tile t has landed once at most the loads of the tiles issued after it are outstanding
            const int later = min(NS - 2, n_tiles - 1 - t);
            if (NS >= 4 && later >= 2) wait_vm<2 * IPW>();
            else if (NS >= 3 && later >= 1) wait_vm<IPW>();
            else wait_vm<0>();
            __builtin_amdgcn_s_barrier(); // every wave's share of tile t is in LDS; everyone is done with tile t-1
            const bool active = (kt <= wave_hi_max) && (kt + KT - 1 >= wave_lo_min); // wave-uniform
            const int ktn = kt + (NS - 1) * KT;
            const int dst_off = ((s + NS - 1) % NS) * G::STAGE_BYTES; // a constant once the loop is unrolled
            const bool more = t + NS - 1 < n_tiles;
            const bool whole = ktn + KT - 1 <= w.key_clamp;
            const char* ktile = (const char*)k + (int64_t)ktn * row_bytes64;
            const char* vtile = (const char*)v + (int64_t)ktn * row_bytes64;
            // the loads of tile t + NS - 1: a wave that computes this tile issues them between its first score products
            // (below); a wave that skips the tile, or a tile with clamped rows, issues them here
            // (measured: the four-wave kernels, whose waves issue twice as many loads per tile, gain 2-5 %; the
            // eight-wave kernel loses the 2 % the unrolled ring gave it, so it keeps its loads in front)
            const bool defer = (NW == 4) && more && whole && active;
            if (more && !defer) {
                if (whole) issue_tile_at<D, NW, AUX>(ktile, vtile, dk, dv, lds_wave, dst_off);
                else issue_tile<D, NW, KT, AUX>(k, v, w.row_elems, w.head_off, ktn, w.key_clamp, smem + dst_off, wave, lane);
            }
            if (active) {
                // stages 2b and 2b + 1 are addressed from bank b's offsets; the rest is a constant of the instruction
                LDS_AS const char* stage = (LDS_AS const char*)(uintptr_t)((s % 2) * G::STAGE_BYTES);
                const bool need_mask = (kt + KT - 1 > mask_hi_min) || (kt < mask_lo_max);
                scores_softmax<D, 2>(stage, qf, rc, kt, need_mask, koff[s / 2], h, acc, bpk, [&](int ks) {
                    if (ks < G::NI / NW && defer) issue_pair_at<D, NW, AUX>(ktile, vtile, dk[ks], dv[ks], lds_wave, dst_off, ks);
                });
                weighted_values<D, 2>(stage + G::TILE_BYTES, bpk, voff[s / 2], acc);
            }
        }
    }
}

// The ordinary loads of a workgroup's start, issued as one batch before anything waits: the position id of the lane's
// token slot and whatever indices the caller needs (issued by the caller, first), theta, then the raw query rows.
// Loads return in order, so the small ones in front are back after one L2 round trip while the query rows are
// still on their way from HBM.
template <int D> struct QLoads {
    double th;          // theta_rev[lane % (D/2)]
    u32x4 raw[D / 16];  // this lane's raw query fragments
};

// PINNED: theta is kept in front of the query rows and the batch is closed with a scheduling fence.  That pays where
// the query rows come from HBM (the offline and one-pass kernels: every row is new); where they sit in L2 (a request's
// few query tokens, read by every key split) the compiler's own order measured 2 % faster.
template <int D, bool PINNED>
__device__ __forceinline__ void issue_q_loads(const __bf16* __restrict__ q, const double* theta_rev, const RowCtx& rc, QLoads<D>& ql)
{
    const int lane = threadIdx.x & 63, h = lane >> 5;
    ql.th = theta_rev[lane % (D / 2)];
    if (PINNED) __builtin_amdgcn_sched_barrier(0);
    load_q_raw<D>(q, rc, h, ql.raw);
    if (PINNED) __builtin_amdgcn_sched_barrier(0);
}

// The first K/V tiles, then the rotation: the tile loads fly while the angles are computed.  theta is waited for
// before the tile loads go out (with it pos_lane, the position id of token slot (lane & 7) of this wave, which the
// caller loaded in front of it): a vector-memory result that is first touched after the tile loads would wait for
// the tiles as well.  The query rows are touched after the angle table is built; pos_of_slot serves the later passes
// of small GQA groups.  The rotation table sits in stage NS-1, which no tile load targets
// before the first barrier of the tile loop.
template <int D, int NW, int NS, bool HALF, int AUX = 0, class PosFn>
__device__ __forceinline__ void prologue(const __bf16* __restrict__ k, const __bf16* __restrict__ v, const Walk& w, QLoads<D>& ql,
                                         int pos_lane, int slot, int n_slots, PosFn pos_of_slot, float sl2e, LDS_AS char* smem,
                                         bf16x8 (&qf)[D / 16])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5;
    asm volatile("" : "+v"(ql.th));
    __builtin_amdgcn_sched_barrier(0);
    issue_prologue<D, NW, NS, AUX>(k, v, w, smem, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    LDS_AS char* tab = smem + (NS - 1) * Geo<D>::STAGE_BYTES + wave * (ROT_SLOTS * 4 * D);
    rotate_queries<D, HALF>(ql.raw, tab, ql.th, lane, h, slot, n_slots, sl2e,
                            [&](int s) { return s < ROT_SLOTS ? pos_lane : pos_of_slot(s); }, qf);
}

// Write the wave's 32 x D accumulator as rows: stage O^T through LDS (64 channels at a time) so that every
// global store instruction writes whole contiguous row segments.
//   PARTIAL = false: out[orow][:] = bf16(O / l)          PARTIAL = true: ws_o[prow][:] = fp16(O / l)
// A partial is normalised by its own denominator, so it is a convex combination of V rows and fp16 (11 bits,
// 8 times finer than the bf16 result) holds it; the merge weighs it with l again.
template <int D, bool PARTIAL>
__device__ __forceinline__ void store_rows(const Acc<D>& acc, float l_tot, bool valid, int64_t dst_row, void* dst,
                                           LDS_AS char* wave_buf, int lane)
{
    constexpr int STRIDE = 64 * 4 + 16; // bytes per staged row: 64 floats + pad
    const int c = lane & 31, h = lane >> 5;
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    const int r_in = lane >> 4, c4 = lane & 15;
#pragma unroll
    for (int half = 0; half < D / 64; ++half) {
#pragma unroll
        for (int dbl = 0; dbl < 2; ++dbl)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int db = 2 * half + dbl;
                f32x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = acc.o[db][4 * q4 + e] * inv;
                *(LDS_AS f32x4*)(wave_buf + c * STRIDE + (32 * dbl + 8 * q4 + 4 * h) * 4) = x;
            }
        // 4 rows per instruction: lane -> (row 4 rr + lane / 16, channels 4 (lane % 16) .. +3 of this half)
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const int row = 4 * rr + r_in;
            const f32x4 x = *(LDS_AS const f32x4*)(wave_buf + row * STRIDE + c4 * 16);
            const int64_t drow = __shfl(dst_row, row);       // row's owner lane is lane `row` (c == row, h == 0)
            const int ok = __shfl((int)valid, row);
            if (ok) {
                if (PARTIAL) {
                    f16x4 y;
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[e] = (_Float16)x[e];
                    // written once and read once, by the merge kernel: a streaming store (0.7 us less at 6 MB of partials)
                    __builtin_nontemporal_store(y, (f16x4*)((_Float16*)dst + drow * D + 64 * half + 4 * c4));
                } else {
                    bf16x4 y;
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[e] = (__bf16)x[e];
                    *(bf16x4*)((__bf16*)dst + drow * D + 64 * half + 4 * c4) = y;
                }
            }
        }
    }
}

// ---- step 6: query prefill over the assembled cache -------------------------------------------------------------
// AUX: cache policy of the K/V tile loads; DMA_STREAM when no request of the launch has more than one row tile, so
// that every key is read by exactly one workgroup (a few query tokens over a long context: 24.0 -> 22.5 us for
// 16 tokens over 12288 rows, Qwen2-7B heads).
template <int D, int NW, int NS, bool HALF, int AUX>
__global__ __launch_bounds__(64 * NW, 2) void prefix_attn_kernel(const TrPrefixArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
    LDS_AS char* smem = (LDS_AS char*)smem_raw;
    const int item = xcd_remap(blockIdx.x, a.n_items);
    int lo = 0, hi = a.n_seq - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (a.seq[mid].item0 <= item) lo = mid; else hi = mid - 1;
    }
    const TrSeqDesc sd = a.seq[lo];
    const int local = item - sd.item0;
    const int tile = local % sd.n_tiles;
    const int rest = local / sd.n_tiles;
    const int split = rest % sd.n_split;
    const int kvh = rest / sd.n_split;
    const int g = a.group, tpt = a.tok_per_tile;
    const int n_doc = sd.kv_len - sd.n_q;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int rl = 32 * wave + c;
    const int tok_local = tile * tpt + rl / g;
    RowCtx rc;
    rc.valid = (rl < tpt * g) && (tok_local < sd.n_q);
    rc.orow = (sd.q_row0 + tok_local) * a.n_q_heads + kvh * g + rl % g;
    rc.key_lo = sd.kv_row0;
    rc.key_hi = sd.kv_row0 + n_doc + tok_local;
    // position ids per token slot of the wave
    const int wave_tok0 = tile * tpt + (32 * wave) / g;
    const int slot = min(rl / g - (32 * wave) / g, 31);
    const int n_slots = (32 * wave + 31) / g - (32 * wave) / g + 1;
    auto pos_of_slot = [&](int s) { return a.q_pos[sd.q_row0 + min(wave_tok0 + s, sd.n_q - 1)]; };
    const int pos_lane = pos_of_slot(lane & (ROT_SLOTS - 1));
    QLoads<D> ql;
    issue_q_loads<D, false>((const __bf16*)a.q, a.theta_rev, rc, ql);

    const int first_tok = tile * tpt;
    const int last_tok = min(first_tok + tpt, sd.n_q) - 1;
    const int sb = sd.kv_row0 + split * sd.split_len;
    const int se = min(sb + sd.split_len, sd.kv_row0 + sd.kv_len);
    const Walk w = make_walk(sb, min(se, sd.kv_row0 + n_doc + last_tok + 1), sd.kv_row0 + sd.kv_len - 1, a.n_kv_heads, kvh, D);

    bf16x8 qf[D / 16];
    prologue<D, NW, NS, HALF, AUX>((const __bf16*)a.k, (const __bf16*)a.v, w, ql, pos_lane, slot, n_slots, pos_of_slot, a.scale_log2e, smem, qf);

    Acc<D> acc;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc.o[db][e] = 0.0f;
    acc.mref = 0.0f;
    acc.l = 0.0f;

    attn_tiles<D, NW, NS, AUX>((const __bf16*)a.k, (const __bf16*)a.v, w, rc, qf, sd.kv_row0 + n_doc + first_tok, sd.kv_row0, smem, acc);

    const float l_tot = acc.l + __shfl_xor(acc.l, 32);
    __builtin_amdgcn_s_barrier(); // all waves are done with the K/V stages; reuse them as store staging
    LDS_AS char* wave_buf = smem + wave * (32 * (64 * 4 + 16));
    if (sd.n_split == 1) {
        store_rows<D, false>(acc, l_tot, rc.valid, (int64_t)rc.orow, a.out, wave_buf, lane);
    } else {
        const int rows_s = sd.n_q * g;
        const int64_t prow = (int64_t)sd.ws_row0 + (int64_t)(split * a.n_kv_heads + kvh) * rows_s + tok_local * g + rl % g;
        store_rows<D, true>(acc, l_tot, rc.valid, prow, a.ws_o, wave_buf, lane);
        // a split in which the row saw no key reports m = -inf so that the merge ignores it
        if (rc.valid && h == 0) *(float2*)(a.ws_ml + prow * 2) = make_float2(l_tot > 0.0f ? acc.mref : -INFINITY, l_tot);
    }
}

// ---- step 6 without a materialised cache: attention that gathers the chunks itself --------------------------------
// The document keys are read straight from the store, where they are rotated at chunk-local positions.  Under
// reordered positions the score needs R(off + t) k; since <R(p) q, R(off + t) k> = <R(p - off) q, R(t) k> (the
// relative-position property behind Eq. 3), the kernel turns the QUERY by -off once per chunk instead of turning
// every key.  The request's own query tokens are read from the cache rows that tr_kv_append wrote.  The walk is a
// list of 64-key tiles, chunk by chunk; the last tile of a chunk may be partial (its missing keys are masked).
constexpr int GATHER_NW = 4, GATHER_NS = 2;
template <int D> constexpr int gather_lds_bytes() { return GATHER_NS * Geo<D>::STAGE_BYTES + GATHER_NW * ROT_SLOTS * 4 * D; }

template <int D, bool HALF>
__global__ __launch_bounds__(64 * GATHER_NW, 2) void gather_attn_kernel(const TrGatherArgs a)
{
    using G = Geo<D>;
    constexpr int NW = GATHER_NW, NS = GATHER_NS;
    extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
    LDS_AS char* smem = (LDS_AS char*)smem_raw;
    const int item = xcd_remap(blockIdx.x, a.n_items);
    const int tile = item % a.row_tiles;
    const int rest = item / a.row_tiles;
    const int split = rest % a.n_split;
    const int kvh = rest / a.n_split;
    const int g = a.group, tpt = a.tok_per_tile;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, colhalf = (lane >> 4) & 1;
    const int rl = 32 * wave + c;
    const int tok_local = tile * tpt + rl / g;
    RowCtx rc;
    rc.valid = (rl < tpt * g) && (tok_local < a.n_q);
    rc.orow = tok_local * a.n_q_heads + kvh * g + rl % g;
    rc.key_lo = 0;
    rc.key_hi = a.n_doc + tok_local;
    const int wave_tok0 = tile * tpt + (32 * wave) / g;
    const int slot = min(rl / g - (32 * wave) / g, 31);
    const int n_slots = (32 * wave + 31) / g - (32 * wave) / g + 1;
    const int first_tok = tile * tpt;
    const int last_tok = min(first_tok + tpt, a.n_q) - 1;

    // this workgroup's tiles: a contiguous range of the request's tile list, cut at the causal end of its rows
    const int tail = a.n_seg - 1;
    const int g0 = split * a.tiles_per_split;
    int g1 = min(g0 + a.tiles_per_split, a.n_tiles_total);
    g1 = min(g1, a.seg[tail].tile0 + last_tok / KT + 1);
    const int n_tiles = g1 > g0 ? g1 - g0 : 0;
    int s_issue = 0;
    while (s_issue + 1 < a.n_seg && a.seg[s_issue + 1].tile0 <= g0) ++s_issue;
    int s_comp = s_issue;

    const int64_t row_elems = (int64_t)a.n_kv_heads * D;
    const int head_off = kvh * D;
    auto issue = [&](int gt, int sg, LDS_AS char* stage) {
        const TrGatherSeg e = a.seg[sg];
        const int first = e.src_row + (gt - e.tile0) * KT;
        const bool from_cache = sg == tail;
        issue_tile<D, NW>((const __bf16*)(from_cache ? a.k_cache : a.k_store), (const __bf16*)(from_cache ? a.v_cache : a.v_store),
                          row_elems, head_off, first, e.src_row + e.n_rows - 1, stage, wave, lane);
    };

    if (n_tiles > 0) issue(g0, s_issue, smem);
    // The queries are rotated at the top of the tile loop whenever the chunk (hence the offset) changes, the first
    // tile included.  The raw rows are fetched again each time rather than held in 32 registers through the loop:
    // the change is rare (once per chunk) and the rows are in L2.
    LDS_AS char* tab = smem + NS * G::STAGE_BYTES + wave * (ROT_SLOTS * 4 * D); // private to the wave, outside the ring
    bf16x8 qf[D / 16];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qf[ks] = bf16x8{};
    int cur_delta = INT32_MIN;

    Acc<D> acc;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc.o[db][e] = 0.0f;
    acc.mref = 0.0f;
    acc.l = 0.0f;

    const int wave_hi_max = wave_max_i(rc.valid ? rc.key_hi : INT32_MIN);
    const int mask_hi_min = a.n_doc + first_tok;
    int koff[D / 16];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) koff[ks] = c * D * 2 + (((2 * ks + h) ^ G::kswz(c)) * 16);
    int voff[D / 32];
    {
        const int r = 4 * h + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
            voff[db] = r * D * 2 + (4 * (db ^ G::vswz(r)) + 2 * colhalf + ((i16 & 3) >> 1)) * 16 + (i16 & 1) * 8;
    }

    bf16x8 bpk[2][2];
    for (int t = 0; t < n_tiles; ++t) {
        const int gt = g0 + t;
        while (s_comp + 1 < a.n_seg && a.seg[s_comp + 1].tile0 <= gt) ++s_comp;
        const TrGatherSeg e = a.seg[s_comp];
        if (e.delta != cur_delta) { // a new chunk: the queries turn to its offset
            cur_delta = e.delta;
            const double th = a.theta_rev[lane % (D / 2)];
            const __bf16* qrow = (const __bf16*)a.q + (int64_t)(rc.valid ? rc.orow : 0) * D + 8 * h;
            const int ns = __builtin_amdgcn_readfirstlane(n_slots);
            for (int p0 = 0; p0 < ns; p0 += ROT_SLOTS) { // one pass when the GQA group is >= 4
                build_rot_table<D>(tab, th, lane, a.q_pos[min(wave_tok0 + p0 + (lane & (ROT_SLOTS - 1)), a.n_q - 1)] - cur_delta, a.scale_log2e);
                const bool mine = (slot >= p0) && (slot < p0 + ROT_SLOTS);
                LDS_AS const char* row = tab + (mine ? slot - p0 : 0) * (4 * D);
                const int sw = 2 * (mine ? slot - p0 : 0);
                // the raw fragments come in two parts so that they never hold more than 16 registers
                if (HALF) {
#pragma unroll
                    for (int part = 0; part < 2; ++part) {
                        u32x4 qlo[D / 64], qhi[D / 64];
#pragma unroll
                        for (int i = 0; i < D / 64; ++i) {
                            qlo[i] = *(const u32x4*)(qrow + 16 * (part * (D / 64) + i));
                            qhi[i] = *(const u32x4*)(qrow + 16 * (part * (D / 64) + i + D / 32));
                        }
#pragma unroll
                        for (int i = 0; i < D / 64; ++i) {
                            const int ks = part * (D / 64) + i;
                            bf16x8 flo, fhi;
                            rot_frag_half<D>(qlo[i], qhi[i], row, ks, h, sw, flo, fhi);
                            if (mine || p0 == 0) { qf[ks] = flo; qf[ks + D / 32] = fhi; }
                        }
                    }
                } else {
#pragma unroll
                    for (int part = 0; part < 2; ++part) {
                        u32x4 raw[D / 32];
#pragma unroll
                        for (int i = 0; i < D / 32; ++i) raw[i] = *(const u32x4*)(qrow + 16 * (part * (D / 32) + i));
#pragma unroll
                        for (int i = 0; i < D / 32; ++i) {
                            const int ks = part * (D / 32) + i;
                            const int ch = (2 * (2 * ks + h)) ^ sw;
                            const f32x4 cs0 = *(LDS_AS const f32x4*)(row + ch * 16);
                            const f32x4 cs1 = *(LDS_AS const f32x4*)(row + ch * 16 + 16);
                            bf16x8 f;
                            rot_pair(raw[i][0], cs0[0], cs0[1], f, 0);
                            rot_pair(raw[i][1], cs0[2], cs0[3], f, 1);
                            rot_pair(raw[i][2], cs1[0], cs1[1], f, 2);
                            rot_pair(raw[i][3], cs1[2], cs1[3], f, 3);
                            if (mine || p0 == 0) qf[ks] = f;
                        }
                    }
                }
                __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0): the table is read before the next pass rewrites it
            }
        }
        wait_vm<0>(); // two stages: tile t is the only load in flight here
        __builtin_amdgcn_s_barrier();
        if (t + 1 < n_tiles) {
            while (s_issue + 1 < a.n_seg && a.seg[s_issue + 1].tile0 <= gt + 1) ++s_issue;
            issue(gt + 1, s_issue, smem + ((t + 1) % NS) * G::STAGE_BYTES);
        }
        const int j = gt - e.tile0;
        const int kt = e.cache_row + j * KT;                      // cache row the tile's first key stands for
        const int last_valid = e.cache_row + min(e.n_rows, (j + 1) * KT) - 1;
        if (kt <= wave_hi_max) {
            LDS_AS const char* stage = smem + (t % NS) * G::STAGE_BYTES;
            RowCtx rct = rc;
            rct.key_hi = min(rc.key_hi, last_valid);
            const bool need_mask = (kt + KT - 1 > mask_hi_min) || (last_valid < kt + KT - 1);
            scores_softmax<D, 2>(stage, qf, rct, kt, need_mask, koff, h, acc, bpk);
            weighted_values<D, 2>(stage + G::TILE_BYTES, bpk, voff, acc);
        }
    }

    const float l_tot = acc.l + __shfl_xor(acc.l, 32);
    __builtin_amdgcn_s_barrier(); // all waves are done with the K/V stages; reuse them as store staging
    LDS_AS char* wave_buf = smem + wave * (32 * (64 * 4 + 16));
    if (a.n_split == 1) {
        store_rows<D, false>(acc, l_tot, rc.valid, (int64_t)rc.orow, a.out, wave_buf, lane);
    } else {
        const int rows_s = a.n_q * g;
        const int64_t prow = (int64_t)(split * a.n_kv_heads + kvh) * rows_s + tok_local * g + rl % g;
        store_rows<D, true>(acc, l_tot, rc.valid, prow, a.ws_o, wave_buf, lane);
        if (rc.valid && h == 0) *(float2*)(a.ws_ml + prow * 2) = make_float2(l_tot > 0.0f ? acc.mref : -INFINITY, l_tot);
    }
}

// ---- step 6 / step 7 for very short queries (decode: one new token per request) --------------------------------
// When the packed rows of a (request, KV head) fit one 32-row MFMA block, giving each wave its own rows would
// leave three of four waves idle.  Here all four waves hold the SAME rows and split the keys instead: a tile is
// 128 keys, wave w owns keys [32 w, 32 w + 32) of it, and the four partial results are merged through LDS at
// the end.  The kernel then streams K/V at four times the rate of one wave, which is what a memory-bound
// decode step needs.
constexpr int SHORT_NW = 4, SHORT_NS = 2, SHORT_KT = 32 * SHORT_NW;

template <int D> constexpr int short_stage_bytes() { return 2 * SHORT_KT * D * 2; }
template <int D> constexpr int short_merge_row_bytes() { return D * 4 + 16; }

template <int D, bool HALF>
__global__ __launch_bounds__(64 * SHORT_NW, 1) void short_attn_kernel(const TrPrefixArgs a)
{
    using G = Geo<D>;
    constexpr int NW = SHORT_NW, NS = SHORT_NS;
    constexpr int STAGE = short_stage_bytes<D>();
    extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
    LDS_AS char* smem = (LDS_AS char*)smem_raw;
    const int item = xcd_remap(blockIdx.x, a.n_items);
    int lo = 0, hi = a.n_seq - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (a.seq[mid].item0 <= item) lo = mid; else hi = mid - 1;
    }
    const TrSeqDesc sd = a.seq[lo];
    const int local = item - sd.item0;
    const int tile = local % sd.n_tiles;
    const int rest = local / sd.n_tiles;
    const int split = rest % sd.n_split;
    const int kvh = rest / sd.n_split;
    const int g = a.group, tpt = a.tok_per_tile;
    const int n_doc = sd.kv_len - sd.n_q;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, colhalf = (lane >> 4) & 1;
    const int tok_local = tile * tpt + c / g;
    RowCtx rc;
    rc.valid = (c < tpt * g) && (tok_local < sd.n_q);
    rc.orow = (sd.q_row0 + tok_local) * a.n_q_heads + kvh * g + c % g;
    rc.key_lo = sd.kv_row0;
    rc.key_hi = sd.kv_row0 + n_doc + tok_local;
    const int slot = min(c / g, 31);
    const int n_slots = 31 / g + 1;
    auto pos_of_slot = [&](int s) { return a.q_pos[sd.q_row0 + min(tile * tpt + s, sd.n_q - 1)]; };
    const int pos_lane = pos_of_slot(lane & (ROT_SLOTS - 1));

    const int first_tok = tile * tpt;
    const int last_tok = min(first_tok + tpt, sd.n_q) - 1;
    const int sb = sd.kv_row0 + split * sd.split_len;
    const int se = min(sb + sd.split_len, sd.kv_row0 + sd.kv_len);
    const int kt_begin = sb;
    const int kt_end = min(se, sd.kv_row0 + n_doc + last_tok + 1);
    const int n_tiles = kt_end > kt_begin ? (kt_end - kt_begin + SHORT_KT - 1) / SHORT_KT : 0;
    const int key_clamp = sd.kv_row0 + sd.kv_len - 1;
    const int64_t row_elems = (int64_t)a.n_kv_heads * D;
    const int head_off = kvh * D;
    const __bf16* kp = (const __bf16*)a.k;
    const __bf16* vp = (const __bf16*)a.v;

    // prologue: ordinary loads, then tile 0, then the rotation (every wave rotates the same rows)
    double th = a.theta_rev[lane % (D / 2)];
    u32x4 raw[D / 16];
    load_q_raw<D>((const __bf16*)a.q, rc, h, raw);
    asm volatile("" : "+v"(th));
    __builtin_amdgcn_sched_barrier(0);
    if (n_tiles > 0) issue_tile<D, NW, SHORT_KT, DMA_STREAM>(kp, vp, row_elems, head_off, kt_begin, key_clamp, smem, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 qf[D / 16];
    {
        LDS_AS char* tab = smem + STAGE + wave * (ROT_SLOTS * 4 * D); // stage 1 is free until the first barrier
        rotate_queries<D, HALF>(raw, tab, th, lane, h, slot, n_slots, a.scale_log2e,
                                [&](int s) { return s < ROT_SLOTS ? pos_lane : pos_of_slot(s); }, qf);
    }

    Acc<D> acc;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc.o[db][e] = 0.0f;
    acc.mref = 0.0f;
    acc.l = 0.0f;

    const int wave_hi_max = wave_max_i(rc.valid ? rc.key_hi : INT32_MIN);
    const int mask_hi_min = sd.kv_row0 + n_doc + first_tok;
    int koff[D / 16];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) koff[ks] = (32 * wave + c) * D * 2 + (((2 * ks + h) ^ G::kswz(c)) * 16);
    int voff[D / 32];
    {
        const int r = 4 * h + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
            voff[db] = (32 * wave + r) * D * 2 + (4 * (db ^ G::vswz(r)) + 2 * colhalf + ((i16 & 3) >> 1)) * 16 + (i16 & 1) * 8;
    }

    bf16x8 bpk[1][2];
    for (int t = 0; t < n_tiles; ++t) {
        const int kt = kt_begin + t * SHORT_KT;
        wait_vm<0>(); // two stages: tile t is the only load in flight here
        __builtin_amdgcn_s_barrier(); // tile t is in LDS; everyone is done with tile t-1
        if (t + 1 < n_tiles)
            issue_tile<D, NW, SHORT_KT, DMA_STREAM>(kp, vp, row_elems, head_off, kt + SHORT_KT, key_clamp, smem + ((t + 1) % NS) * STAGE, wave, lane);
        const int ktw = kt + 32 * wave; // this wave's 32 keys
        if (ktw <= wave_hi_max && ktw < kt_end) {
            LDS_AS const char* stage = smem + (t % NS) * STAGE;
            const bool need_mask = ktw + 31 > mask_hi_min;
            scores_softmax<D, 1>(stage, qf, rc, ktw, need_mask, koff, h, acc, bpk);
            weighted_values<D, 1>(stage + SHORT_KT * D * 2, bpk, voff, acc);
        }
    }

    // merge the four key slices: every wave parks (m, l) and its unnormalised O in LDS
    constexpr int ROWB = short_merge_row_bytes<D>();
    const float l_tot = acc.l + __shfl_xor(acc.l, 32);
    __builtin_amdgcn_s_barrier(); // all waves are done with the K/V stages
    LDS_AS char* obuf = smem + wave * (32 * ROWB);
    LDS_AS float* mlbuf = (LDS_AS float*)(smem + NW * 32 * ROWB);
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            f32x4 x;
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = acc.o[db][4 * q4 + e];
            *(LDS_AS f32x4*)(obuf + c * ROWB + (32 * db + 8 * q4 + 4 * h) * 4) = x;
        }
    if (h == 0) {
        mlbuf[(wave * 32 + c) * 2] = l_tot > 0.0f ? acc.mref : -INFINITY;
        mlbuf[(wave * 32 + c) * 2 + 1] = l_tot;
    }
    __syncthreads();
    // thread -> (row r, D/8 consecutive channels)
    constexpr int CPT = D / 8;
    const int r = tid >> 3, j = tid & 7;
    float mw[NW], lw[NW], M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        mw[w] = mlbuf[(w * 32 + r) * 2];
        lw[w] = mlbuf[(w * 32 + r) * 2 + 1];
        M = fmaxf(M, mw[w]);
    }
    float L = 0.0f, ww[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        ww[w] = (mw[w] == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mw[w] - M);
        L += ww[w] * lw[w];
    }
    float o[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) o[e] = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int e4 = 0; e4 < CPT / 4; ++e4) {
            const f32x4 x = *(LDS_AS const f32x4*)(smem + w * (32 * ROWB) + r * ROWB + (CPT * j + 4 * e4) * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[4 * e4 + e] += ww[w] * x[e];
        }
    const int r_tok = tile * tpt + r / g;
    const bool r_valid = (r < tpt * g) && (r_tok < sd.n_q);
    if (!r_valid) return;
    const float inv = L > 0.0f ? 1.0f / L : 0.0f;
    if (sd.n_split == 1) {
        __bf16* op = (__bf16*)a.out + ((int64_t)(sd.q_row0 + r_tok) * a.n_q_heads + kvh * g + r % g) * D + CPT * j;
#pragma unroll
        for (int e4 = 0; e4 < CPT / 4; ++e4) {
            bf16x4 y;
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] = (__bf16)(o[4 * e4 + e] * inv);
            *(bf16x4*)(op + 4 * e4) = y;
        }
    } else {
        const int rows_s = sd.n_q * g;
        const int64_t prow = (int64_t)sd.ws_row0 + (int64_t)(split * a.n_kv_heads + kvh) * rows_s + r_tok * g + r % g;
        _Float16* op = a.ws_o + prow * D + CPT * j;
#pragma unroll
        for (int e4 = 0; e4 < CPT / 4; ++e4) {
            f16x4 y;
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] = (_Float16)(o[4 * e4 + e] * inv);
            *(f16x4*)(op + 4 * e4) = y;
        }
        if (j == 0) *(float2*)(a.ws_ml + prow * 2) = make_float2(L > 0.0f ? M : -INFINITY, L);
    }
}

// Merge the split-KV partial results: out = sum_s w_s l_s P_s / sum_s w_s l_s with w_s = 2^(m_s - max_s m_s) and
// P_s = O_s / l_s the normalised partial of split s.
// 32 lanes per output row (4 channels each); lane i of the row also owns split i's statistics.
// WIDE: some request of the launch has more than 32 key splits, so a lane of the row's half-wave holds two of them
// (splits i and i + 32); the narrow form keeps one and is what every launch with at most 32 splits runs.
template <int D, bool WIDE>
__global__ __launch_bounds__(256) void combine_kernel(const TrPrefixArgs a, int total_rows)
{
    static_assert(D == 128 || D == 64, "");
    constexpr int LPR = 32;                     // lanes per row
    constexpr int CPLN = D / LPR;               // channels per lane: 4 or 2
    const int lane_r = threadIdx.x & 31;
    const int64_t R = (int64_t)blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
    if (R >= total_rows) return;
    const int tq = a.seq[0].q_row0 + (int)(R / a.n_q_heads);
    const int hq = (int)(R % a.n_q_heads);
    int lo = 0, hi = a.n_seq - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (a.seq[mid].q_row0 <= tq) lo = mid; else hi = mid - 1;
    }
    const TrSeqDesc sd = a.seq[lo];
    if (sd.n_split == 1) return;
    const int g = a.group;
    const int kvh = hq / g;
    const int64_t rows_s = (int64_t)sd.n_q * g;
    const int64_t prow0 = (int64_t)sd.ws_row0 + kvh * rows_s + (tq - sd.q_row0) * g + hq % g;
    const int64_t pstride = (int64_t)a.n_kv_heads * rows_s; // partial rows between consecutive splits
    // statistics: lane i of the row's half-wave loads split i (and split i + 32 in the wide form)
    constexpr int NK = WIDE ? 2 : 1;
    float m_i[2] = {-INFINITY, -INFINITY}, l_i[2] = {0.0f, 0.0f};
#pragma unroll
    for (int k = 0; k < NK; ++k)
        if (lane_r + 32 * k < sd.n_split) {
            const float2 ml = *(const float2*)(a.ws_ml + (prow0 + (lane_r + 32 * k) * pstride) * 2);
            m_i[k] = ml.x;
            l_i[k] = ml.y;
        }
    float M = fmaxf(m_i[0], m_i[1]);
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    float w_i[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) w_i[k] = (k >= NK || m_i[k] == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m_i[k] - M) * l_i[k];
    float L = w_i[0] + w_i[1];
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) L += __shfl_xor(L, o);
    float acc[CPLN];
#pragma unroll
    for (int e = 0; e < CPLN; ++e) acc[e] = 0.0f;
    const _Float16* base = a.ws_o + prow0 * D + CPLN * lane_r;
    const int row_lane0 = threadIdx.x & 32; // first lane of this row's half-wave
    // eight splits per round so that eight loads are in flight (the loop count is a run-time value)
    constexpr int PER_ROUND = 8;
    for (int sp0 = 0; sp0 < sd.n_split; sp0 += PER_ROUND) {
        f32x4 x[PER_ROUND];
        float w[PER_ROUND];
        const float w_src = (!WIDE || sp0 < 32) ? w_i[0] : w_i[1]; // a round never straddles 32
#pragma unroll
        for (int u = 0; u < PER_ROUND; ++u) {
            const int sp = sp0 + u;
            const bool ok = sp < sd.n_split;
            const _Float16* p = base + (int64_t)(ok ? sp : 0) * pstride * D;
            if (CPLN == 4) {
                const f16x4 t = *(const f16x4*)p;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[u][e] = (float)t[e];
            } else {
                const f16x2 t = *(const f16x2*)p;
                x[u][0] = (float)t[0]; x[u][1] = (float)t[1]; x[u][2] = 0.0f; x[u][3] = 0.0f;
            }
            const float ws = __shfl(w_src, row_lane0 + (sp & 31));
            w[u] = ok ? ws : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < PER_ROUND; ++u)
#pragma unroll
            for (int e = 0; e < CPLN; ++e) acc[e] += w[u] * x[u][e];
    }
    const float inv = 1.0f / L;
    __bf16* op = (__bf16*)a.out + ((int64_t)tq * a.n_q_heads + hq) * D + CPLN * lane_r;
    if (CPLN == 4) {
        bf16x4 y;
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (__bf16)(acc[e] * inv);
        *(bf16x4*)op = y;
    } else {
        op[0] = (__bf16)(acc[0] * inv);
        op[1] = (__bf16)(acc[1] * inv);
    }
}

// ---- step 2 (offline): block-diagonal causal attention over packed chunks --------------------------------------
// First row of the chunk that owns token t.  Clamped into [0, t] so that a cu_chunk_lens array that does not cover
// every token can only give wrong numbers, never an access outside the tensors.
__device__ __forceinline__ int chunk_start(const int32_t* tok_start, int t) { return min(max(tok_start[t], 0), t); }

template <int D, int NW, int NS, bool HALF>
__global__ __launch_bounds__(64 * NW, 2) void blockdiag_attn_kernel(const TrBlockDiagArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
    LDS_AS char* smem = (LDS_AS char*)smem_raw;
    const int item = xcd_remap(blockIdx.x, a.items_per_head * a.n_kv_heads);
    const int kvh = item / a.items_per_head;
    const int j = item % a.items_per_head;
    int slo = 0, shi = a.n_seg - 1;
    while (slo < shi) {
        const int mid = (slo + shi + 1) >> 1;
        if (a.seg[mid].item0 <= j) slo = mid; else shi = mid - 1;
    }
    const TrBdSeg sg = a.seg[slo];
    // last row tiles first: under a causal mask they walk the most keys (a query behind the documents walks all of
    // them), so they must not be the ones that start last
    const int tile = sg.tile_hi - (j - sg.item0) / sg.n_split;
    const int split = (j - sg.item0) % sg.n_split;
    const int g = a.group, tpt = a.tok_per_tile;
    const int T = a.total_tokens;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31;
    const int rl = 32 * wave + c;
    const int t = tile * tpt + rl / g;
    RowCtx rc;
    rc.valid = (rl < tpt * g) && (t < T);
    rc.orow = t * a.n_q_heads + kvh * g + rl % g;
    rc.key_hi = t;
    const int wave_t0 = tile * tpt + (32 * wave) / g;
    const int slot = min(rl / g - (32 * wave) / g, 31);
    const int n_slots = (32 * wave + 31) / g - (32 * wave) / g + 1;
    const int t_first = tile * tpt;
    const int t_last = min(t_first + tpt, T) - 1;
    // One batch of loads, nothing waited for in between: this row's chunk start, the position id (or chunk start) of
    // the lane's token slot, the chunk start of the tile's token `lane` (tokens 64 and up of a tile, which only small
    // GQA groups have, follow below), then theta and the raw query rows.  Indices are clamped instead of branched on.
    const int ts_lane = min(wave_t0 + (lane & (ROT_SLOTS - 1)), T - 1);
    const int start_row_raw = a.tok_start[min(t, T - 1)];
    const int slot_raw = a.pos ? a.pos[ts_lane] : a.tok_start[ts_lane];
    const int start_tile_raw = a.tok_start[min(t_first + lane, t_last)];
    __builtin_amdgcn_sched_barrier(0);
    QLoads<D> ql;
    issue_q_loads<D, true>((const __bf16*)a.q, a.theta_rev, rc, ql);

    rc.key_lo = rc.valid ? min(max(start_row_raw, 0), t) : 0;
    // position id of each token slot of this wave: given, or chunk-local
    auto pos_of_slot = [&](int s) {
        const int ts = min(wave_t0 + s, T - 1);
        return a.pos ? a.pos[ts] : ts - chunk_start(a.tok_start, ts);
    };
    const int pos_lane = a.pos ? slot_raw : ts_lane - min(max(slot_raw, 0), ts_lane);

    // first row any token of the tile attends, and the largest such start (tiles below it need the lower mask);
    // the starts need not be monotone: a query token behind the documents starts at row 0 again
    int lo_first = INT32_MAX, lo_last = 0;
    if (t_first + lane <= t_last) lo_first = lo_last = min(max(start_tile_raw, 0), t_first + lane);
    for (int tt = t_first + 64 + lane; tt <= t_last; tt += 64) {
        const int st = chunk_start(a.tok_start, tt);
        lo_first = min(lo_first, st);
        lo_last = max(lo_last, st);
    }
    lo_first = wave_min_i(lo_first);
    lo_last = wave_max_i(lo_last);
    // this item's piece of the walk [lo_first, t_last]: pieces of split_len keys, the last one open-ended
    int kb = lo_first, ke = t_last + 1;
    if (sg.n_split > 1) {
        const int64_t kb64 = (int64_t)lo_first + (int64_t)split * sg.split_len;
        kb = (int)(kb64 < ke ? kb64 : ke);
        if (split + 1 < sg.n_split && (int64_t)kb + sg.split_len < ke) ke = kb + sg.split_len;
    }
    const Walk w = make_walk(kb, ke, T - 1, a.n_kv_heads, kvh, D);

    bf16x8 qf[D / 16];
    prologue<D, NW, NS, HALF>((const __bf16*)a.k, (const __bf16*)a.v, w, ql, pos_lane, slot, n_slots, pos_of_slot, a.scale_log2e, smem, qf);

    Acc<D> acc;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc.o[db][e] = 0.0f;
    acc.mref = 0.0f;
    acc.l = 0.0f;

    attn_tiles<D, NW, NS>((const __bf16*)a.k, (const __bf16*)a.v, w, rc, qf, t_first, lo_last, smem, acc);

    const float l_tot = acc.l + __shfl_xor(acc.l, 32);
    __builtin_amdgcn_s_barrier();
    LDS_AS char* wave_buf = smem + wave * (32 * (64 * 4 + 16));
    if (sg.n_split == 1) {
        store_rows<D, false>(acc, l_tot, rc.valid, (int64_t)rc.orow, a.out, wave_buf, lane);
    } else { // the layout the merge kernel reads: [split][KV head][token of the segment x group]
        const int64_t rows_s = (int64_t)sg.n_tok * g;
        const int64_t prow = (int64_t)sg.ws_row0 + ((int64_t)split * a.n_kv_heads + kvh) * rows_s + (int64_t)(t - sg.tok0) * g + rl % g;
        store_rows<D, true>(acc, l_tot, rc.valid, prow, a.ws_o, wave_buf, lane);
        if (rc.valid && lane < 32) *(float2*)(a.ws_ml + prow * 2) = make_float2(l_tot > 0.0f ? acc.mref : -INFINITY, l_tot);
    }
}

template <int D, int NW, int NS> constexpr int smem_bytes()
{
    constexpr int stages = NS * Geo<D>::STAGE_BYTES;
    constexpr int staging = NW * 32 * (64 * 4 + 16);
    return stages > staging ? stages : staging;
}

template <int D, int NW, int NS, bool HALF, int AUX = 0>
int launch_prefix(const TrPrefixArgs& a, hipStream_t s)
{
    auto kern = prefix_attn_kernel<D, NW, NS, HALF, AUX>;
    constexpr int lds = smem_bytes<D, NW, NS>();
    static std::atomic<uint64_t> configured{0};
    if (int rc = tr_raise_lds_limit((const void*)kern, lds, &configured)) return rc;
    hipLaunchKernelGGL(kern, dim3(a.n_items), dim3(64 * NW), lds, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

template <int D, bool HALF>
int launch_short(const TrPrefixArgs& a, hipStream_t s)
{
    auto kern = short_attn_kernel<D, HALF>;
    constexpr int ring = SHORT_NS * short_stage_bytes<D>();
    constexpr int merge = SHORT_NW * 32 * short_merge_row_bytes<D>() + SHORT_NW * 32 * 8;
    constexpr int lds = ring > merge ? ring : merge;
    static std::atomic<uint64_t> configured{0};
    if (int rc = tr_raise_lds_limit((const void*)kern, lds, &configured)) return rc;
    hipLaunchKernelGGL(kern, dim3(a.n_items), dim3(64 * SHORT_NW), lds, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

template <int D, bool HALF>
int launch_gather(const TrGatherArgs& a, hipStream_t s)
{
    auto kern = gather_attn_kernel<D, HALF>;
    constexpr int staging = GATHER_NW * 32 * (64 * 4 + 16);
    constexpr int lds = gather_lds_bytes<D>() > staging ? gather_lds_bytes<D>() : staging;
    static std::atomic<uint64_t> configured{0};
    if (int rc = tr_raise_lds_limit((const void*)kern, lds, &configured)) return rc;
    hipLaunchKernelGGL(kern, dim3(a.n_items), dim3(64 * GATHER_NW), lds, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

template <int D, int NW, int NS, bool HALF>
int launch_blockdiag(const TrBlockDiagArgs& a, hipStream_t s)
{
    auto kern = blockdiag_attn_kernel<D, NW, NS, HALF>;
    constexpr int lds = smem_bytes<D, NW, NS>();
    static std::atomic<uint64_t> configured{0};
    if (int rc = tr_raise_lds_limit((const void*)kern, lds, &configured)) return rc;
    hipLaunchKernelGGL(kern, dim3(a.items_per_head * a.n_kv_heads), dim3(64 * NW), lds, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

template <bool HALF>
int prefix_dispatch(const TrPrefixArgs& a, int head_dim, int wg_rows, hipStream_t s)
{
    if (wg_rows == 32) return head_dim == 128 ? launch_short<128, HALF>(a, s) : launch_short<64, HALF>(a, s);
    if (wg_rows == 128) {
        bool one_tile = true; // every request fits one row tile: its keys are read once
        for (int i = 0; i < a.n_seq; ++i) one_tile = one_tile && a.seq[i].n_tiles == 1;
        if (one_tile)
            return head_dim == 128 ? launch_prefix<128, 4, 2, HALF, DMA_STREAM>(a, s) : launch_prefix<64, 4, 2, HALF, DMA_STREAM>(a, s);
    }
    if (head_dim == 128) return wg_rows == 256 ? launch_prefix<128, 8, 4, HALF>(a, s) : launch_prefix<128, 4, 2, HALF>(a, s);
    return wg_rows == 256 ? launch_prefix<64, 8, 4, HALF>(a, s) : launch_prefix<64, 4, 2, HALF>(a, s);
}

template <bool HALF>
int blockdiag_dispatch(const TrBlockDiagArgs& a, int head_dim, int wg_rows, hipStream_t s)
{
    if (head_dim == 128) return wg_rows == 256 ? launch_blockdiag<128, 8, 4, HALF>(a, s) : launch_blockdiag<128, 4, 2, HALF>(a, s);
    return wg_rows == 256 ? launch_blockdiag<64, 8, 4, HALF>(a, s) : launch_blockdiag<64, 4, 2, HALF>(a, s);
}

} // namespace

// the merge kernel for a launch whose largest split count is max_split
static int launch_combine(const TrPrefixArgs& a, int head_dim, int blocks, int total_rows, hipStream_t s)
{
    int max_split = 1;
    for (int i = 0; i < a.n_seq; ++i) max_split = a.seq[i].n_split > max_split ? a.seq[i].n_split : max_split;
    if (max_split > 32) {
        if (head_dim == 128) hipLaunchKernelGGL((combine_kernel<128, true>), dim3(blocks), dim3(256), 0, s, a, total_rows);
        else hipLaunchKernelGGL((combine_kernel<64, true>), dim3(blocks), dim3(256), 0, s, a, total_rows);
    } else {
        if (head_dim == 128) hipLaunchKernelGGL((combine_kernel<128, false>), dim3(blocks), dim3(256), 0, s, a, total_rows);
        else hipLaunchKernelGGL((combine_kernel<64, false>), dim3(blocks), dim3(256), 0, s, a, total_rows);
    }
    TR_HIP(hipGetLastError());
    return TR_OK;
}

// wg_rows: 128 (4 waves, 2-stage ring, two workgroups per CU), 256 (8 waves, 4-stage ring, one per CU) or 32 (the
// short-query kernel: 4 waves share 32 rows and split the keys)
int tr_launch_prefix_attn(const TrPrefixArgs& a, int head_dim, int wg_rows, bool any_split, int total_rows, hipStream_t s)
{
    if (a.n_items <= 0) return TR_OK;
    const int rc = a.rope_half ? prefix_dispatch<true>(a, head_dim, wg_rows, s) : prefix_dispatch<false>(a, head_dim, wg_rows, s);
    if (rc) return rc;
    if (any_split) {
        const int rows_per_block = 256 / 32;
        const int blocks = (total_rows + rows_per_block - 1) / rows_per_block;
        if (int rc2 = launch_combine(a, head_dim, blocks, total_rows, s)) return rc2;
    }
    return TR_OK;
}

int tr_launch_gather_attn(const TrGatherArgs& a, const TrPrefixArgs& combine_args, int head_dim, hipStream_t s)
{
    if (a.n_items <= 0) return TR_OK;
    int rc;
    if (a.rope_half) rc = head_dim == 128 ? launch_gather<128, true>(a, s) : launch_gather<64, true>(a, s);
    else rc = head_dim == 128 ? launch_gather<128, false>(a, s) : launch_gather<64, false>(a, s);
    if (rc) return rc;
    if (a.n_split > 1) {
        const int total_rows = a.n_q * a.n_q_heads;
        const int blocks = (total_rows + 7) / 8;
        if (int rc2 = launch_combine(combine_args, head_dim, blocks, total_rows, s)) return rc2;
    }
    return TR_OK;
}

int tr_launch_blockdiag_attn(const TrBlockDiagArgs& a, const TrPrefixArgs* combine, int combine_rows, int head_dim, int wg_rows,
                             hipStream_t s)
{
    if (a.total_tokens <= 0) return TR_OK;
    const int rc = a.rope_half ? blockdiag_dispatch<true>(a, head_dim, wg_rows, s) : blockdiag_dispatch<false>(a, head_dim, wg_rows, s);
    if (rc) return rc;
    if (combine && combine_rows > 0) {
        const int blocks = (combine_rows + 7) / 8;
        if (int rc2 = launch_combine(*combine, head_dim, blocks, combine_rows, s)) return rc2;
    }
    return TR_OK;
}
