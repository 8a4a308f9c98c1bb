// Bandwidth-bound kernels: KV-cache formation (gather + per-chunk RoPE re-rotation), query append,
// and the offline key rotation.  All key rotations are computed in fp64 and rounded once to the
// storage type, so the rotated keys are reproducible to the last bit against an fp64 definition.
#include "tr_internal.h"
#include <type_traits>

namespace {

// ---- storage helpers ------------------------------------------------------------------------------------

__device__ __forceinline__ double bf16_bits_to_double(uint32_t b16)
{
    return (double)__uint_as_float(b16 << 16);
}

// double -> bf16 with a single rounding (nearest, ties to even), done on the bit pattern: the 45 mantissa bits
// below bf16's seven are folded to "above / at / below half" with integer arithmetic (the low word only matters as
// a sticky bit), and a carry out of the mantissa lands in the exponent as it should.  Values outside bf16's normal
// range (zero, subnormal, overflow, NaN) take the conversion route: truncate to fp32, sticky bit, round.
__device__ __forceinline__ uint32_t double_to_bf16_bits_slow(double y)
{
    float f = __double2float_rz(y);
    uint32_t u = __float_as_uint(f);
    u |= ((double)f != y) ? 1u : 0u;
    if (y != y) return 0x7fc0u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t double_to_bf16_bits(double y)
{
    const uint64_t b = (uint64_t)__double_as_longlong(y);
    uint32_t hi = (uint32_t)(b >> 32);
    hi |= ((uint32_t)b != 0u) ? 1u : 0u;          // sticky: bit 0 is among the 13 bits rounded away
    hi += 0xfffu + ((hi >> 13) & 1u);             // nearest, ties to even, at bit 13
    const uint32_t t = hi >> 13;                  // sign | 11-bit exponent | 7-bit mantissa
    const uint32_t e = ((t >> 7) & 0x7ffu) - 896u; // exponent rebased from 1023 to 127
    if (e - 1u < 254u) return ((t >> 18) << 15) | (e << 7) | (t & 0x7fu);
    return double_to_bf16_bits_slow(y);
}

// y = R(angle) x on one pair, unfused multiplies and adds (the order Eq. 3 is written in)
__device__ __forceinline__ void rotate_pair(double xa, double xb, double c, double s, double& ya, double& yb)
{
    ya = __dsub_rn(__dmul_rn(xa, c), __dmul_rn(xb, s));
    yb = __dadd_rn(__dmul_rn(xb, c), __dmul_rn(xa, s));
}

template <int DTYPE> struct Unit; // one 16-byte unit of a row

template <> struct Unit<TR_BF16> {
    static constexpr int PAIRS = 4;
    __device__ static __forceinline__ uint4 rotate(uint4 x, const double* c, const double* s)
    {
        uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            double xa = bf16_bits_to_double(w[p] & 0xffffu), xb = bf16_bits_to_double(w[p] >> 16);
            double ya, yb;
            rotate_pair(xa, xb, c[p], s[p], ya, yb);
            w[p] = double_to_bf16_bits(ya) | (double_to_bf16_bits(yb) << 16);
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// Half-split layout: channel c < d/2 pairs with c + d/2, so a unit of the low half pairs element by element with
// the unit d/2 channels further on.  me / partner: the two units, low: whether `me` is the low half; c, s: the
// (cos, sin) of the ELEMS pair indices the unit covers.  y_lo = x_lo c - x_hi s, y_hi = x_hi c + x_lo s.
template <int DTYPE> struct UnitHalf;
template <> struct UnitHalf<TR_BF16> {
    static constexpr int ELEMS = 8;
    __device__ static __forceinline__ uint4 rotate(uint4 me, uint4 partner, bool low, const double* c, const double* s)
    {
        uint32_t a[4] = {me.x, me.y, me.z, me.w}, b[4] = {partner.x, partner.y, partner.z, partner.w};
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            uint32_t r[2];
#pragma unroll
            for (int hw = 0; hw < 2; ++hw) {
                const double xm = bf16_bits_to_double(hw ? a[p] >> 16 : a[p] & 0xffffu);
                const double xp = bf16_bits_to_double(hw ? b[p] >> 16 : b[p] & 0xffffu);
                const double t0 = __dmul_rn(xm, c[2 * p + hw]), t1 = __dmul_rn(xp, s[2 * p + hw]);
                r[hw] = double_to_bf16_bits(low ? __dsub_rn(t0, t1) : __dadd_rn(t0, t1));
            }
            a[p] = r[0] | (r[1] << 16);
        }
        return make_uint4(a[0], a[1], a[2], a[3]);
    }
};
template <> struct UnitHalf<TR_F32> {
    static constexpr int ELEMS = 4;
    __device__ static __forceinline__ uint4 rotate(uint4 me, uint4 partner, bool low, const double* c, const double* s)
    {
        uint32_t a[4] = {me.x, me.y, me.z, me.w}, b[4] = {partner.x, partner.y, partner.z, partner.w};
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const double t0 = __dmul_rn((double)__uint_as_float(a[p]), c[p]), t1 = __dmul_rn((double)__uint_as_float(b[p]), s[p]);
            a[p] = __float_as_uint(__double2float_rn(low ? __dsub_rn(t0, t1) : __dadd_rn(t0, t1)));
        }
        return make_uint4(a[0], a[1], a[2], a[3]);
    }
};
__device__ __forceinline__ uint4 shfl_xor_u4(uint4 x, int mask)
{
    return make_uint4(__shfl_xor(x.x, mask), __shfl_xor(x.y, mask), __shfl_xor(x.z, mask), __shfl_xor(x.w, mask));
}

template <> struct Unit<TR_F32> {
    static constexpr int PAIRS = 2;
    __device__ static __forceinline__ uint4 rotate(uint4 x, const double* c, const double* s)
    {
        uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            double xa = (double)__uint_as_float(w[2 * p]), xb = (double)__uint_as_float(w[2 * p + 1]);
            double ya, yb;
            rotate_pair(xa, xb, c[p], s[p], ya, yb);
            w[2 * p] = __float_as_uint(__double2float_rn(ya));
            w[2 * p + 1] = __float_as_uint(__double2float_rn(yb));
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// streaming (read-once) 16-byte load
__device__ __forceinline__ uint4 ld_stream(const uint4* p)
{
    const u32x4 r = __builtin_nontemporal_load((const u32x4*)p);
    return make_uint4(r[0], r[1], r[2], r[3]);
}

constexpr int APPEND_MAX_HEADS = 16; // KV heads held in registers at once; more go round the loop again

// The same for the half-split layout: the pair is (channel m, channel m + d/2) of every head.
template <int DTYPE>
__device__ __forceinline__ void append_pair_half(const void* k_new, const void* v_new, int pos, void* cache_k,
                                                 void* cache_v, int n_kv_heads, int half, double theta_m, int64_t src_row,
                                                 int64_t dst_row, int m)
{
    typedef typename std::conditional<DTYPE == TR_BF16, uint16_t, float>::type Elem;
    const int d = 2 * half;
    const Elem* ks = (const Elem*)k_new + src_row * n_kv_heads * d + m;
    const Elem* vs = (const Elem*)v_new + src_row * n_kv_heads * d + m;
    Elem* kd = (Elem*)cache_k + dst_row * n_kv_heads * d + m;
    Elem* vd = (Elem*)cache_v + dst_row * n_kv_heads * d + m;
    const double angle = (double)pos * theta_m;
    double sn = 0.0, cn = 1.0;
    for (int h0 = 0; h0 < n_kv_heads; h0 += APPEND_MAX_HEADS) {
        Elem ka[APPEND_MAX_HEADS], kb[APPEND_MAX_HEADS], va[APPEND_MAX_HEADS], vb[APPEND_MAX_HEADS];
#pragma unroll
        for (int j = 0; j < APPEND_MAX_HEADS; ++j)
            if (h0 + j < n_kv_heads) {
                ka[j] = ks[(h0 + j) * d];
                kb[j] = ks[(h0 + j) * d + half];
                if (v_new) { va[j] = vs[(h0 + j) * d]; vb[j] = vs[(h0 + j) * d + half]; }
            }
        if (h0 == 0) sincos(angle, &sn, &cn);
#pragma unroll
        for (int j = 0; j < APPEND_MAX_HEADS; ++j)
            if (h0 + j < n_kv_heads) {
                double xa, xb, ya, yb;
                if constexpr (DTYPE == TR_BF16) {
                    xa = bf16_bits_to_double(ka[j]);
                    xb = bf16_bits_to_double(kb[j]);
                } else {
                    xa = (double)ka[j];
                    xb = (double)kb[j];
                }
                rotate_pair(xa, xb, cn, sn, ya, yb);
                if constexpr (DTYPE == TR_BF16) {
                    kd[(h0 + j) * d] = (uint16_t)double_to_bf16_bits(ya);
                    kd[(h0 + j) * d + half] = (uint16_t)double_to_bf16_bits(yb);
                } else {
                    kd[(h0 + j) * d] = __double2float_rn(ya);
                    kd[(h0 + j) * d + half] = __double2float_rn(yb);
                }
                if (v_new) { vd[(h0 + j) * d] = va[j]; vd[(h0 + j) * d + half] = vb[j]; }
            }
    }
}

// ---- one (token, pair m) of the query append: K' rotated at q_pos, V copied, for every KV head ----------------
// The angle is shared by all KV heads of the token (the fp64 sincos is by far the longest thing a thread does, so
// it is done once per thread), and the loads go out before it.
template <int DTYPE, bool HALF>
__device__ __forceinline__ void append_pair(const void* k_new, const void* v_new, int pos, void* cache_k,
                                            void* cache_v, int n_kv_heads, int half, double theta_m, int64_t src_row,
                                            int64_t dst_row, int m)
{
    if constexpr (HALF) {
        append_pair_half<DTYPE>(k_new, v_new, pos, cache_k, cache_v, n_kv_heads, half, theta_m, src_row, dst_row, m);
        return;
    }
    typedef typename std::conditional<DTYPE == TR_BF16, uint32_t, float2>::type Pair; // one (even, odd) channel pair
    const Pair* ks = (const Pair*)k_new + src_row * n_kv_heads * half + m;
    const Pair* vs = (const Pair*)v_new + src_row * n_kv_heads * half + m;
    Pair* kd = (Pair*)cache_k + dst_row * n_kv_heads * half + m;
    Pair* vd = (Pair*)cache_v + dst_row * n_kv_heads * half + m;
    const double angle = (double)pos * theta_m;
    double sn = 0.0, cn = 1.0;
    for (int h0 = 0; h0 < n_kv_heads; h0 += APPEND_MAX_HEADS) {
        Pair kx[APPEND_MAX_HEADS], vx[APPEND_MAX_HEADS];
#pragma unroll
        for (int j = 0; j < APPEND_MAX_HEADS; ++j)
            if (h0 + j < n_kv_heads) {
                kx[j] = ks[(h0 + j) * half];
                if (v_new) vx[j] = vs[(h0 + j) * half];
            }
        if (h0 == 0) sincos(angle, &sn, &cn);
#pragma unroll
        for (int j = 0; j < APPEND_MAX_HEADS; ++j)
            if (h0 + j < n_kv_heads) {
                double xa, xb, ya, yb;
                if constexpr (DTYPE == TR_BF16) {
                    xa = bf16_bits_to_double(kx[j] & 0xffffu);
                    xb = bf16_bits_to_double(kx[j] >> 16);
                } else {
                    xa = (double)kx[j].x;
                    xb = (double)kx[j].y;
                }
                rotate_pair(xa, xb, cn, sn, ya, yb);
                if constexpr (DTYPE == TR_BF16) kd[(h0 + j) * half] = double_to_bf16_bits(ya) | (double_to_bf16_bits(yb) << 16);
                else kd[(h0 + j) * half] = make_float2(__double2float_rn(ya), __double2float_rn(yb));
                if (v_new) vd[(h0 + j) * half] = vx[j]; // v_new == NULL: keys only
            }
    }
}

// ---- KV-cache formation: Sec. 3.4 step 5 with the reordered-position rotation of Sec. 3.2 -------------------
// A run of rows is contiguous in the store and in the cache, so a block moves a flat span of 16-byte
// units.  A thread's unit index modulo the units-per-head never changes while it strides by 256, hence
// the (cos, sin) of "its" pairs for this chunk's offset are loop constants.
constexpr int ASM_UNROLL = 4;

__device__ __forceinline__ void st_stream(uint4* p, uint4 x) { *p = x; }

template <int DTYPE, bool HALF>
__global__ __launch_bounds__(256) void assemble_kernel(const TrAssembleArgs a)
{
    __shared__ double cs[64][2];
    const int b = blockIdx.x;
    if (a.app.n_q > 0 && b >= a.app.first_block) {
        // tail blocks: the request's own query tokens, one thread per (token, pair)
        const int gid = (b - a.app.first_block) * 256 + (int)threadIdx.x;
        const int tok = gid / a.half_dim, m = gid % a.half_dim;
        if (tok < a.app.n_q)
            append_pair<DTYPE, HALF>(a.app.k_new, a.app.v_new, a.app.q_pos[tok], a.k_dst, a.v_dst, a.app.n_kv_heads, a.half_dim,
                                     a.theta[m], tok, (int64_t)a.app.dst_row0 + tok, m);
        return;
    }
    int lo = 0, hi = a.n_desc - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (a.desc[mid].blk_start <= b) lo = mid; else hi = mid - 1;
    }
    const TrCopyDesc d = a.desc[lo];
    const int64_t run_units = (int64_t)d.n_rows * a.row_units;
    const int64_t u0 = (int64_t)(b - d.blk_start) * a.span_units;
    int64_t u1 = u0 + a.span_units;
    if (u1 > run_units) u1 = run_units;
    const int tid = threadIdx.x;

    const uint4* ks = (const uint4*)a.k_src + (int64_t)d.src_row * a.row_units;
    const uint4* vs = (const uint4*)a.v_src + (int64_t)d.src_row * a.row_units;
    uint4* kd = (uint4*)a.k_dst + (int64_t)d.dst_row * a.row_units;
    uint4* vd = (uint4*)a.v_dst + (int64_t)d.dst_row * a.row_units;

    // the first round of loads goes out before the angle work, which needs no data
    uint4 kx[ASM_UNROLL], vx[ASM_UNROLL];
    int64_t u = u0 + tid;
#pragma unroll
    for (int i = 0; i < ASM_UNROLL; ++i) {
        const int64_t uu = u + 256 * i;
        if (uu < u1) { kx[i] = ld_stream(ks + uu); vx[i] = ld_stream(vs + uu); }
    }

    constexpr int P = Unit<DTYPE>::PAIRS, E = UnitHalf<DTYPE>::ELEMS;
    double c[HALF ? E : P], s[HALF ? E : P];
    const bool rot = d.delta != 0;
    const int hu = (int)((u0 + tid) % a.head_units); // unit inside its head: the same for every unit this thread moves
    const int hmask = a.head_units >> 1;             // lane distance to the unit d/2 channels away
    const bool low = hu < hmask;
    if (rot) {
        if (tid < a.half_dim) {
            double sn, cn;
            sincos((double)d.delta * a.theta[tid], &sn, &cn);
            cs[tid][0] = cn;
            cs[tid][1] = sn;
        }
        __syncthreads();
        if constexpr (HALF) {
            const int m0 = (low ? hu : hu - hmask) * E;
#pragma unroll
            for (int p = 0; p < E; ++p) { c[p] = cs[m0 + p][0]; s[p] = cs[m0 + p][1]; }
        } else {
            const int m0 = hu * P;
#pragma unroll
            for (int p = 0; p < P; ++p) { c[p] = cs[m0 + p][0]; s[p] = cs[m0 + p][1]; }
        }
    }

    while (u < u1) {
#pragma unroll
        for (int i = 0; i < ASM_UNROLL; ++i) {
            const int64_t uu = u + 256 * i;
            // the 16-byte units of one head sit in neighbouring lanes and runs are whole rows, so a lane and the lane
            // that holds its partner unit are always in this branch together
            if (uu < u1) {
                uint4 y = kx[i];
                if (rot) {
                    if constexpr (HALF) y = UnitHalf<DTYPE>::rotate(kx[i], shfl_xor_u4(kx[i], hmask), low, c, s);
                    else y = Unit<DTYPE>::rotate(kx[i], c, s);
                }
                st_stream(kd + uu, y);
                st_stream(vd + uu, vx[i]);
            }
        }
        u += 256 * ASM_UNROLL;
#pragma unroll
        for (int i = 0; i < ASM_UNROLL; ++i) {
            const int64_t uu = u + 256 * i;
            if (uu < u1) { kx[i] = ld_stream(ks + uu); vx[i] = ld_stream(vs + uu); }
        }
    }
}

// ---- query append: cache rows of the query tokens (K' rotated at q_pos, V copied) -------------------------
template <int DTYPE, bool HALF>
__global__ __launch_bounds__(256) void append_kernel(const TrAppendArgs a)
{
    const int half = a.head_dim >> 1;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int tok = (int)(gid / half), m = (int)(gid % half);
    if (tok >= a.total_tokens) return;
    // request that owns packed token `tok` of this launch
    int r = 0, base = 0;
    while (r + 1 < a.n_desc && tok >= base + a.desc[r].n_q) { base += a.desc[r].n_q; ++r; }
    const int i = tok - base;
    // position id: the caller's, or (raw-store assembly) the run's first position plus the row's index in the run
    const int pos = a.q_pos ? a.q_pos[a.desc[r].q_row0 + i] : a.desc[r].pos0 + i;
    append_pair<DTYPE, HALF>(a.k_new, a.v_new, pos, a.cache_k, a.cache_v, a.n_kv_heads, half, a.theta[m],
                             (int64_t)a.desc[r].q_row0 + i, (int64_t)a.desc[r].dst_row0 + i, m);
}

// The same rows for launches of many tokens (a store of un-rotated keys assembled at the final position ids, the key
// rotation of the one-pass sequence call): a thread owns one 16-byte unit of a token, computes the (cos, sin) of the
// pairs that unit takes part in once, and walks the KV heads with 16-byte accesses, where the kernel above moves one
// pair (4 bytes) per thread and head.  Same arithmetic, so the same bits.
constexpr int APPEND_UNITS_HEADS = 8; // KV heads in flight per thread
template <int DTYPE, bool HALF>
__global__ __launch_bounds__(256) void append_units_kernel(const TrAppendArgs a)
{
    constexpr int P = Unit<DTYPE>::PAIRS, E = UnitHalf<DTYPE>::ELEMS;
    constexpr int N_CS = HALF ? E : P; // pairs this thread's unit takes part in
    const int head_units = a.head_dim * (DTYPE == TR_BF16 ? 2 : 4) / 16; // a power of two, at most 32: a token's units share a wave
    const int hmask = head_units >> 1;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int tok = (int)(gid / head_units), unit = (int)(gid % head_units);
    if (tok >= a.total_tokens) return; // whole tokens leave together, so the partner lane of the half-split layout stays
    int r = 0, base = 0;
    while (r + 1 < a.n_desc && tok >= base + a.desc[r].n_q) { base += a.desc[r].n_q; ++r; }
    const int i = tok - base;
    const int pos = a.q_pos ? a.q_pos[a.desc[r].q_row0 + i] : a.desc[r].pos0 + i;
    const int64_t row_units = (int64_t)a.n_kv_heads * head_units;
    const uint4* ks = (const uint4*)a.k_new + ((int64_t)a.desc[r].q_row0 + i) * row_units + unit;
    const uint4* vs = (const uint4*)a.v_new + ((int64_t)a.desc[r].q_row0 + i) * row_units + unit;
    uint4* kd = (uint4*)a.cache_k + ((int64_t)a.desc[r].dst_row0 + i) * row_units + unit;
    uint4* vd = (uint4*)a.cache_v + ((int64_t)a.desc[r].dst_row0 + i) * row_units + unit;
    const bool low = unit < hmask;
    const int m0 = HALF ? (low ? unit : unit - hmask) * E : unit * P;
    double c[N_CS], s[N_CS];
    for (int h0 = 0; h0 < a.n_kv_heads; h0 += APPEND_UNITS_HEADS) {
        uint4 kx[APPEND_UNITS_HEADS], vx[APPEND_UNITS_HEADS];
#pragma unroll
        for (int j = 0; j < APPEND_UNITS_HEADS; ++j)
            if (h0 + j < a.n_kv_heads) {
                kx[j] = ld_stream(ks + (h0 + j) * head_units);
                if (a.v_new) vx[j] = ld_stream(vs + (h0 + j) * head_units);
            }
        if (h0 == 0) { // the loads are on their way while the angles are computed
#pragma unroll
            for (int p = 0; p < N_CS; ++p) sincos((double)pos * a.theta[m0 + p], &s[p], &c[p]);
        }
#pragma unroll
        for (int j = 0; j < APPEND_UNITS_HEADS; ++j)
            if (h0 + j < a.n_kv_heads) {
                uint4 y;
                if constexpr (HALF) y = UnitHalf<DTYPE>::rotate(kx[j], shfl_xor_u4(kx[j], hmask), low, c, s);
                else y = Unit<DTYPE>::rotate(kx[j], c, s);
                kd[(h0 + j) * head_units] = y;
                if (a.v_new) vd[(h0 + j) * head_units] = vx[j]; // v_new == NULL: keys only
            }
    }
}

// ---- offline key rotation (Sec. 3.4 step 2): K' = R(t - cu[c]) k -------------------------------------------
// table[pos][m] = (cos, sin)(pos * theta_m) in fp64, positions 0 .. n_pos-1
struct ThetaArg { double v[64]; };
__global__ __launch_bounds__(256) void rope_table_kernel(double2* table, int n_pos, int half_dim, const ThetaArg theta_arg)
{
    const double* theta = theta_arg.v;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= (int64_t)n_pos * half_dim) return;
    const int pos = (int)(gid / half_dim), m = (int)(gid % half_dim);
    double sn, cn;
    sincos((double)pos * theta[m], &sn, &cn);
    table[gid] = make_double2(cn, sn);
}

// Grid (row blocks, chunks); a thread owns one 16-byte unit position inside a head for one token and walks the
// KV heads, so the (cos, sin) it fetched from the table serve every head.  Row blocks stride over the chunk, so
// every token of [cu[c], cu[c+1]) is covered whatever the chunk's length.  Also records, per token, the first
// row of its chunk.
constexpr int ROPE_ROWS_HEADS = 8; // KV heads in flight per thread

template <int DTYPE, bool HALF>
__global__ __launch_bounds__(256) void rope_rows_kernel(const uint4* k, uint4* k_rot, const int32_t* cu, int32_t* tok_start,
                                                        const double2* table, int table_rows, int64_t total_tokens,
                                                        int n_kv_heads, int head_units, int half_dim)
{
    constexpr int P = Unit<DTYPE>::PAIRS, E = UnitHalf<DTYPE>::ELEMS;
    const int hmask = head_units >> 1;
    const int chunk = blockIdx.y;
    int start = cu[chunk], end = cu[chunk + 1];
    if (start < 0) start = 0;
    if (end > total_tokens) end = (int)total_tokens;
    const int tpb = 256 / head_units; // tokens per block
    const int unit = threadIdx.x % head_units;
    const int row_units = n_kv_heads * head_units;
    for (int t = start + blockIdx.x * tpb + threadIdx.x / head_units; t < end; t += gridDim.x * tpb) {
        if (unit == 0) tok_start[t] = start;
        int pos = t - start;
        if (pos > table_rows - 1) pos = table_rows - 1; // caller promised max_chunk_len; never read past the table
        const uint4* src = k + (int64_t)t * row_units + unit;
        uint4* dst = k_rot + (int64_t)t * row_units + unit;
        for (int h0 = 0; h0 < n_kv_heads; h0 += ROPE_ROWS_HEADS) {
            uint4 x[ROPE_ROWS_HEADS];
#pragma unroll
            for (int j = 0; j < ROPE_ROWS_HEADS; ++j)
                if (h0 + j < n_kv_heads) x[j] = ld_stream(src + (h0 + j) * head_units);
            constexpr int N_CS = HALF ? E : P; // pairs this thread's unit takes part in
            double c[N_CS], s[N_CS];
            const bool low = unit < hmask;
            const int m0 = HALF ? (low ? unit : unit - hmask) * E : unit * P;
#pragma unroll
            for (int p = 0; p < N_CS; ++p) {
                const double2 e = table[(int64_t)pos * half_dim + m0 + p];
                c[p] = e.x;
                s[p] = e.y;
            }
            // a token's units sit in neighbouring lanes (head_units of them, a power of two), so the partner lane of the
            // half-split layout is in this iteration too
#pragma unroll
            for (int j = 0; j < ROPE_ROWS_HEADS; ++j)
                if (h0 + j < n_kv_heads) {
                    uint4 y = x[j];
                    if constexpr (HALF) y = UnitHalf<DTYPE>::rotate(x[j], shfl_xor_u4(x[j], hmask), low, c, s);
                    else if (pos != 0) y = Unit<DTYPE>::rotate(x[j], c, s);
                    dst[(h0 + j) * head_units] = y;
                }
        }
    }
}

} // namespace

int tr_launch_assemble(const TrAssembleArgs& a, int dtype, int n_blocks, hipStream_t s)
{
    if (n_blocks <= 0) return TR_OK;
    auto kern = dtype == TR_BF16 ? (a.rope_half ? assemble_kernel<TR_BF16, true> : assemble_kernel<TR_BF16, false>)
                                 : (a.rope_half ? assemble_kernel<TR_F32, true> : assemble_kernel<TR_F32, false>);
    hipLaunchKernelGGL(kern, dim3(n_blocks), dim3(256), 0, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

int tr_launch_append(const TrAppendArgs& a, int dtype, hipStream_t s)
{
    // many tokens: the form with 16-byte accesses (57 -> 51 us for 32768 rows of 8 heads); a request's few query tokens:
    // one thread per pair, whose single angle is the shortest path to the first store
    const int head_units = a.head_dim * (dtype == TR_BF16 ? 2 : 4) / 16;
    if ((int64_t)a.total_tokens * head_units >= 65536) {
        const int64_t n = (int64_t)a.total_tokens * head_units;
        auto kern = dtype == TR_BF16 ? (a.rope_half ? append_units_kernel<TR_BF16, true> : append_units_kernel<TR_BF16, false>)
                                     : (a.rope_half ? append_units_kernel<TR_F32, true> : append_units_kernel<TR_F32, false>);
        hipLaunchKernelGGL(kern, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
        TR_HIP(hipGetLastError());
        return TR_OK;
    }
    int64_t threads = (int64_t)a.total_tokens * (a.head_dim / 2);
    if (threads <= 0) return TR_OK;
    int blocks = (int)((threads + 255) / 256);
    auto kern = dtype == TR_BF16 ? (a.rope_half ? append_kernel<TR_BF16, true> : append_kernel<TR_BF16, false>)
                                 : (a.rope_half ? append_kernel<TR_F32, true> : append_kernel<TR_F32, false>);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), 0, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

int tr_launch_rope_table(double* table, int n_pos, int half_dim, const double* theta, hipStream_t s)
{
    int64_t threads = (int64_t)n_pos * half_dim;
    if (threads <= 0) return TR_OK;
    ThetaArg th;
    for (int m = 0; m < 64; ++m) th.v[m] = theta[m];
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                       (double2*)table, n_pos, half_dim, th);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

int tr_launch_rope_rows(const void* k, void* k_rot, const int32_t* cu, int n_chunks, int max_chunk_len, int32_t* tok_start,
                        const double* table, int table_rows, int64_t total_tokens, const tr_shape* shape, hipStream_t s)
{
    const int eb = tr_elem_bytes(shape);
    const int head_units = shape->head_dim * eb / 16;
    if (total_tokens <= 0 || n_chunks <= 0) return TR_OK;
    const int tpb = 256 / head_units;
    int row_blocks = (max_chunk_len + tpb - 1) / tpb;
    if (row_blocks < 1) row_blocks = 1;
    if (row_blocks > 1024) row_blocks = 1024;
    // grid.y carries the chunk index: at most 65535 chunks per launch
    for (int c0 = 0; c0 < n_chunks; c0 += 65535) {
        const int nc = n_chunks - c0 < 65535 ? n_chunks - c0 : 65535;
        dim3 grid((unsigned)row_blocks, (unsigned)nc);
        const bool half = tr_rope_half(shape) != 0;
        auto kern = shape->dtype == TR_BF16 ? (half ? rope_rows_kernel<TR_BF16, true> : rope_rows_kernel<TR_BF16, false>)
                                            : (half ? rope_rows_kernel<TR_F32, true> : rope_rows_kernel<TR_F32, false>);
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, s, (const uint4*)k, (uint4*)k_rot, cu + c0, tok_start, (const double2*)table,
                           table_rows, total_tokens, shape->n_kv_heads, head_units, shape->head_dim / 2);
        TR_HIP(hipGetLastError());
    }
    return TR_OK;
}
