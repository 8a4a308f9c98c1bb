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

// ---- one (token, pair m) of the query append: K' rotated at q_pos, V copied, for every KV head ----------------
// The angle is shared by all KV heads of the token (the fp64 sincos is by far the longest thing a thread does, so
// it is done once per thread), and the loads go out before it.
constexpr int APPEND_MAX_HEADS = 16; // KV heads held in registers at once; more go round the loop again

template <int DTYPE>
__device__ __forceinline__ void append_pair(const void* k_new, const void* v_new, const int32_t* q_pos, void* cache_k,
                                            void* cache_v, int n_kv_heads, int half, double theta_m, int64_t src_row,
                                            int64_t dst_row, int m)
{
    typedef typename std::conditional<DTYPE == TR_BF16, uint32_t, float2>::type Pair; // one (even, odd) channel pair
    const Pair* ks = (const Pair*)k_new + src_row * n_kv_heads * half + m;
    const Pair* vs = (const Pair*)v_new + src_row * n_kv_heads * half + m;
    Pair* kd = (Pair*)cache_k + dst_row * n_kv_heads * half + m;
    Pair* vd = (Pair*)cache_v + dst_row * n_kv_heads * half + m;
    const double angle = (double)q_pos[src_row] * theta_m;
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

__device__ __forceinline__ void st_stream(uint4* p, uint4 x)
{
#ifdef TR_ASM_NT_STORE
    u32x4 r;
    r[0] = x.x; r[1] = x.y; r[2] = x.z; r[3] = x.w;
    __builtin_nontemporal_store(r, (u32x4*)p);
#else
    *p = x;
#endif
}

template <int DTYPE>
__global__ __launch_bounds__(256) void assemble_kernel(const TrAssembleArgs a)
{
    __shared__ double cs[64][2];
    const int b = blockIdx.x;
    if (a.app.n_q > 0 && b >= a.app.first_block) {
        // tail blocks: the request's own query tokens, one thread per (token, pair)
        const int gid = (b - a.app.first_block) * 256 + (int)threadIdx.x;
        const int tok = gid / a.half_dim, m = gid % a.half_dim;
        if (tok < a.app.n_q)
            append_pair<DTYPE>(a.app.k_new, a.app.v_new, a.app.q_pos, a.k_dst, a.v_dst, a.app.n_kv_heads, a.half_dim, a.theta[m],
                               tok, (int64_t)a.app.dst_row0 + tok, m);
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

    constexpr int P = Unit<DTYPE>::PAIRS;
    double c[P], s[P];
    const bool rot = d.delta != 0;
    if (rot) {
        if (tid < a.half_dim) {
            double sn, cn;
            sincos((double)d.delta * a.theta[tid], &sn, &cn);
            cs[tid][0] = cn;
            cs[tid][1] = sn;
        }
        __syncthreads();
        const int m0 = (int)((u0 + tid) % a.head_units) * P;
#pragma unroll
        for (int p = 0; p < P; ++p) { c[p] = cs[m0 + p][0]; s[p] = cs[m0 + p][1]; }
    }

    while (u < u1) {
#pragma unroll
        for (int i = 0; i < ASM_UNROLL; ++i) {
            const int64_t uu = u + 256 * i;
            if (uu < u1) {
                st_stream(kd + uu, rot ? Unit<DTYPE>::rotate(kx[i], c, s) : kx[i]);
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
template <int DTYPE>
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
    append_pair<DTYPE>(a.k_new, a.v_new, a.q_pos, a.cache_k, a.cache_v, a.n_kv_heads, half, a.theta[m],
                       (int64_t)a.desc[r].q_row0 + i, (int64_t)a.desc[r].dst_row0 + i, m);
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

template <int DTYPE>
__global__ __launch_bounds__(256) void rope_rows_kernel(const uint4* k, uint4* k_rot, const int32_t* cu, int32_t* tok_start,
                                                        const double2* table, int table_rows, int64_t total_tokens,
                                                        int n_kv_heads, int head_units, int half_dim)
{
    constexpr int P = Unit<DTYPE>::PAIRS;
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
            double c[P], s[P];
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const double2 e = table[(int64_t)pos * half_dim + unit * P + p];
                c[p] = e.x;
                s[p] = e.y;
            }
#pragma unroll
            for (int j = 0; j < ROPE_ROWS_HEADS; ++j)
                if (h0 + j < n_kv_heads) dst[(h0 + j) * head_units] = (pos == 0) ? x[j] : Unit<DTYPE>::rotate(x[j], c, s);
        }
    }
}

} // namespace

int tr_launch_assemble(const TrAssembleArgs& a, int dtype, int n_blocks, hipStream_t s)
{
    if (n_blocks <= 0) return TR_OK;
    if (dtype == TR_BF16) hipLaunchKernelGGL(assemble_kernel<TR_BF16>, dim3(n_blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(assemble_kernel<TR_F32>, dim3(n_blocks), dim3(256), 0, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

int tr_launch_append(const TrAppendArgs& a, int dtype, hipStream_t s)
{
    int64_t threads = (int64_t)a.total_tokens * (a.head_dim / 2);
    if (threads <= 0) return TR_OK;
    int blocks = (int)((threads + 255) / 256);
    if (dtype == TR_BF16) hipLaunchKernelGGL(append_kernel<TR_BF16>, dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(append_kernel<TR_F32>, dim3(blocks), dim3(256), 0, s, a);
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
        if (shape->dtype == TR_BF16)
            hipLaunchKernelGGL(rope_rows_kernel<TR_BF16>, grid, dim3(256), 0, s, (const uint4*)k, (uint4*)k_rot, cu + c0, tok_start,
                               (const double2*)table, table_rows, total_tokens, shape->n_kv_heads, head_units, shape->head_dim / 2);
        else
            hipLaunchKernelGGL(rope_rows_kernel<TR_F32>, grid, dim3(256), 0, s, (const uint4*)k, (uint4*)k_rot, cu + c0, tok_start,
                               (const double2*)table, table_rows, total_tokens, shape->n_kv_heads, head_units, shape->head_dim / 2);
        TR_HIP(hipGetLastError());
    }
    return TR_OK;
}
