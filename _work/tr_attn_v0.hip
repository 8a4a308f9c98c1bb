// Attention kernels for gfx950.
//
// bf16 path (MFMA): one workgroup = 4 wavefronts = 128 "packed rows"; a packed row is one (query token,
// query head of the group) pair, so the g query heads that share a KV head sit in the same MFMA tile and
// every K/V tile fetched from HBM serves all of them.  Each wavefront owns 32 packed rows.
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K tile rows (from LDS), B = rotated queries (registers)
//   O^T = V^T P^T same instruction, A = V^T (transposing LDS reads), B = P^T (registers, straight from S^T)
// Working on the transposed problem leaves each lane with one query column: the softmax statistics are
// per-lane scalars, and the S^T accumulator layout is already the B-operand layout of the second product
// (up to a permutation of the 16 keys inside a k-step, which the V^T reads apply too).
//
// fp32 path: plain FMA arithmetic, one wavefront per (token, head); for the small fp32 configuration only.
#include "tr_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int KT = 64;        // keys per tile

template <int D> struct alignas(16) Smem {
    static constexpr int KS = D + 8;  // K row stride (elements): 16 B pad -> conflict-free 16 B row reads
    static constexpr int VS = D + 32; // V row stride: 64 B pad -> 4 consecutive rows x 64 B hit distinct banks
    __bf16 k[KT][KS];
    __bf16 v[KT][VS];
};

struct RowCtx {
    bool valid;
    int q_tok;   // row of q / out
    int head;    // query head
    int key_lo;  // first visible cache row
    int key_hi;  // last visible cache row
    double pos;  // RoPE position id of the query token
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

__device__ __forceinline__ int wave_max32(int v)
{
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) v = max(v, __shfl_xor(v, o));
    v = max(v, __shfl_xor(v, 32));
    return __builtin_amdgcn_readfirstlane(v);
}
__device__ __forceinline__ int wave_min32(int v)
{
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) v = min(v, __shfl_xor(v, o));
    v = min(v, __shfl_xor(v, 32));
    return __builtin_amdgcn_readfirstlane(v);
}

// Rotated query fragments: lane (c = lane & 31, h = lane >> 5) holds Q'[row c][16 ks + 8 h .. +7].
template <int D>
__device__ __forceinline__ void load_q_frags(const __bf16* __restrict__ q, int n_q_heads, const RowCtx& rc,
                                             const double* theta_rev, int h, bf16x8 (&qf)[D / 16])
{
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        bf16x8 f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (__bf16)0.0f;
        if (rc.valid) {
            const int d0 = 16 * ks + 8 * h;
            const uint4 raw = *(const uint4*)(q + ((int64_t)rc.q_tok * n_q_heads + rc.head) * D + d0);
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const double t0 = theta_rev[8 * ks + p], t1 = theta_rev[8 * ks + 4 + p];
                double rev = rc.pos * (h ? t1 : t0);
                rev -= rint(rev);
                const float x = (float)rev;
                const float sn = __builtin_amdgcn_sinf(x), cn = __builtin_amdgcn_cosf(x);
                const float xa = bf_lo(w[p]), xb = bf_hi(w[p]);
                f[2 * p] = (__bf16)(xa * cn - xb * sn);
                f[2 * p + 1] = (__bf16)(xb * cn + xa * sn);
            }
        }
        qf[ks] = f;
    }
}

// The tile loop shared by the prefix and the block-diagonal kernels.
// kt_begin..kt_end: cache rows this workgroup walks (workgroup-uniform); key_clamp: last row that may be
// loaded; a tile [kt, kt+KT) needs per-element masking iff kt+KT-1 > mask_hi_min or kt < mask_lo_max.
template <int D>
__device__ __forceinline__ void attn_tiles(const __bf16* __restrict__ k, const __bf16* __restrict__ v, int n_kv_heads,
                                           int kvh, const RowCtx& rc, const bf16x8 (&qf)[D / 16], int kt_begin,
                                           int kt_end, int key_clamp, int mask_hi_min, int mask_lo_max,
                                           float sl2e, Smem<D>& sm, f32x16 (&o)[D / 32], float& m_run, float& l_run)
{
    constexpr int UPR = D / 8;              // 16-byte units per K row of one head
    constexpr int LOADS = KT * UPR / 256;   // units per thread per tile
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int c = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, colhalf = (lane >> 4) & 1;

    const int wave_hi_max = wave_max32(rc.valid ? rc.key_hi : INT32_MIN);
    const int wave_lo_min = wave_min32(rc.valid ? rc.key_lo : INT32_MAX);

    u32x4 kreg[LOADS], vreg[LOADS];
    auto issue_loads = [&](int kt) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx / UPR, u = idx % UPR;
            int key = kt + row;
            key = key > key_clamp ? key_clamp : key;
            const int64_t off = ((int64_t)key * n_kv_heads + kvh) * D + u * 8;
            kreg[i] = *(const u32x4*)(k + off);
            vreg[i] = *(const u32x4*)(v + off);
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx / UPR, u = idx % UPR;
            *(u32x4*)&sm.k[row][u * 8] = kreg[i];
            *(u32x4*)&sm.v[row][u * 8] = vreg[i];
        }
    };

    if (kt_begin < kt_end) issue_loads(kt_begin);
    for (int kt = kt_begin; kt < kt_end; kt += KT) {
        __syncthreads(); // every wave is done reading the previous tile
        store_lds();
        __syncthreads();
        if (kt + KT < kt_end) issue_loads(kt + KT); // in flight while this tile is computed

        const bool active = (kt <= wave_hi_max) && (kt + KT - 1 >= wave_lo_min); // wave-uniform
        if (!active) continue;

        // ---- S^T = K Q^T : two 32-key blocks
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) s[kb][e] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            const bf16x8 a0 = *(const bf16x8*)&sm.k[c][16 * ks + 8 * h];
            const bf16x8 a1 = *(const bf16x8*)&sm.k[32 + c][16 * ks + 8 * h];
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[ks], s[0], 0, 0, 0);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[ks], s[1], 0, 0, 0);
        }
        // accumulator element e of block kb is key kt + 32 kb + 8 (e >> 2) + 4 h + (e & 3), query column c
        const bool need_mask = (kt + KT - 1 > mask_hi_min) || (kt < mask_lo_max);
        if (need_mask) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = kt + 32 * kb + 8 * (e >> 2) + 4 * h + (e & 3);
                    if (key < rc.key_lo || key > rc.key_hi) s[kb][e] = -INFINITY;
                }
        }
        // ---- online softmax; the two half-waves hold the two key halves of the same query column
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[kb][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * sl2e);
        const float mb = m_use * sl2e;
        float lsum = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][e], sl2e, -mb));
                s[kb][e] = p;
                lsum += p;
            }
        l_run = l_run * alpha + lsum;
        m_run = m_new;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                bf16x8 bp;
#pragma unroll
                for (int e = 0; e < 8; ++e) bp[e] = (__bf16)s[kb][8 * t + e];
                // k-slot j of this k-step is key 32 kb + 16 t + 8 (j >> 2) + 4 h + (j & 3)
                const int krow = 32 * kb + 16 * t + 4 * h + (i16 >> 2);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const __bf16* p0 = &sm.v[krow][32 * db + 16 * colhalf + 4 * (i16 & 3)];
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3)))*)(p0));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3)))*)(p0 + 8 * Smem<D>::VS));
                    const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), bp, o[db], 0, 0, 0);
                }
            }
    }
}

// ---- step 6: query prefill over the assembled cache -------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 2) void prefix_attn_kernel(const TrPrefixArgs a)
{
    __shared__ Smem<D> sm;
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
    rc.q_tok = sd.q_row0 + tok_local;
    rc.head = kvh * g + rl % g;
    rc.key_lo = sd.kv_row0;
    rc.key_hi = sd.kv_row0 + n_doc + tok_local;
    rc.pos = rc.valid ? (double)a.q_pos[rc.q_tok] : 0.0;

    const int first_tok = tile * tpt;
    const int last_tok = min(first_tok + tpt, sd.n_q) - 1;
    const int sb = sd.kv_row0 + split * sd.split_len;
    const int se = min(sb + sd.split_len, sd.kv_row0 + sd.kv_len);
    const int kt_begin = sb;
    const int kt_end = min(se, sd.kv_row0 + n_doc + last_tok + 1);

    bf16x8 qf[D / 16];
    load_q_frags<D>((const __bf16*)a.q, a.n_q_heads, rc, a.theta_rev, h, qf);

    f32x16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    attn_tiles<D>((const __bf16*)a.k, (const __bf16*)a.v, a.n_kv_heads, kvh, rc, qf, kt_begin, kt_end,
                  sd.kv_row0 + sd.kv_len - 1, sd.kv_row0 + n_doc + first_tok, sd.kv_row0, a.scale_log2e, sm, o,
                  m_run, l_run);

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!rc.valid) return;
    // accumulator element e of block db is channel 32 db + 8 (e >> 2) + 4 h + (e & 3)
    if (sd.n_split == 1) {
        const float inv = 1.0f / l_tot;
        __bf16* op = (__bf16*)a.out + ((int64_t)rc.q_tok * a.n_q_heads + rc.head) * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = (__bf16)(o[db][4 * q4 + e] * inv);
                *(bf16x4*)(op + 32 * db + 8 * q4 + 4 * h) = r;
            }
    } else {
        const int rows_s = sd.n_q * g;
        const int64_t prow = (int64_t)sd.ws_row0 + (int64_t)(split * a.n_kv_heads + kvh) * rows_s + tok_local * g + rl % g;
        float* wp = a.ws_o + prow * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *(float4*)(wp + 32 * db + 8 * q4 + 4 * h) =
                    make_float4(o[db][4 * q4], o[db][4 * q4 + 1], o[db][4 * q4 + 2], o[db][4 * q4 + 3]);
        if (h == 0) *(float2*)(a.ws_ml + prow * 2) = make_float2(m_run, l_tot);
    }
}

// Merge the split-KV partial results: out = sum_s w_s O_s / sum_s w_s l_s, w_s = 2^((m_s - max m) * sl2e)
template <int D>
__global__ __launch_bounds__(256) void combine_kernel(const TrPrefixArgs a, int total_rows)
{
    constexpr int TPR = D / 4; // threads per output row, 4 channels each
    const int64_t R = (int64_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    const int d4 = threadIdx.x % TPR;
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
    const int rows_s = sd.n_q * g;
    const int r = (tq - sd.q_row0) * g + hq % g;
    float M = -INFINITY;
    for (int sp = 0; sp < sd.n_split; ++sp) {
        const int64_t prow = (int64_t)sd.ws_row0 + (int64_t)(sp * a.n_kv_heads + kvh) * rows_s + r;
        M = fmaxf(M, a.ws_ml[prow * 2]);
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float L = 0.0f;
    for (int sp = 0; sp < sd.n_split; ++sp) {
        const int64_t prow = (int64_t)sd.ws_row0 + (int64_t)(sp * a.n_kv_heads + kvh) * rows_s + r;
        const float2 ml = *(const float2*)(a.ws_ml + prow * 2);
        const float w = __builtin_amdgcn_exp2f((ml.x - M) * a.scale_log2e);
        const float4 x = *(const float4*)(a.ws_o + prow * D + 4 * d4);
        acc.x += w * x.x; acc.y += w * x.y; acc.z += w * x.z; acc.w += w * x.w;
        L += w * ml.y;
    }
    const float inv = 1.0f / L;
    bf16x4 rr;
    rr[0] = (__bf16)(acc.x * inv); rr[1] = (__bf16)(acc.y * inv); rr[2] = (__bf16)(acc.z * inv); rr[3] = (__bf16)(acc.w * inv);
    *(bf16x4*)((__bf16*)a.out + ((int64_t)tq * a.n_q_heads + hq) * D + 4 * d4) = rr;
}

// ---- step 2 (offline): block-diagonal causal attention over packed chunks --------------------------------------
template <int D>
__global__ __launch_bounds__(256, 2) void blockdiag_attn_kernel(const TrBlockDiagArgs a)
{
    __shared__ Smem<D> sm;
    const int n_items = a.n_tiles * a.n_kv_heads;
    const int item = xcd_remap(blockIdx.x, n_items);
    const int tile = item % a.n_tiles;
    const int kvh = item / a.n_tiles;
    const int g = a.group, tpt = a.tok_per_tile;
    const int T = a.total_tokens;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int rl = 32 * wave + c;
    const int t = tile * tpt + rl / g;
    RowCtx rc;
    rc.valid = (rl < tpt * g) && (t < T);
    rc.q_tok = t;
    rc.head = kvh * g + rl % g;
    rc.key_lo = rc.valid ? a.tok_start[t] : 0;
    rc.key_hi = t;
    rc.pos = (double)(t - rc.key_lo);

    const int t_first = tile * tpt;
    const int t_last = min(t_first + tpt, T) - 1;
    const int lo_first = a.tok_start[t_first];
    const int lo_last = a.tok_start[t_last];

    bf16x8 qf[D / 16];
    load_q_frags<D>((const __bf16*)a.q, a.n_q_heads, rc, a.theta_rev, h, qf);

    f32x16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    attn_tiles<D>((const __bf16*)a.k, (const __bf16*)a.v, a.n_kv_heads, kvh, rc, qf, lo_first, t_last + 1, T - 1,
                  t_first, lo_last, a.scale_log2e, sm, o, m_run, l_run);

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!rc.valid) return;
    const float inv = 1.0f / l_tot;
    __bf16* op = (__bf16*)a.out + ((int64_t)rc.q_tok * a.n_q_heads + rc.head) * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 r;
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = (__bf16)(o[db][4 * q4 + e] * inv);
            *(bf16x4*)(op + 32 * db + 8 * q4 + 4 * h) = r;
        }
}

// ---- fp32 path ----------------------------------------------------------------------------------------------
// One wavefront per (query token, query head).  Keys are walked in blocks of 256: scores with lane <-> key,
// then the weighted sum with lane <-> channel.  Queries are rotated in fp64.
struct F32Row {
    const float* q;   // raw query vector
    float* out;
    int key_lo, key_hi, kvh;
    double pos;
};

template <int D>
__device__ __forceinline__ void attn_f32_row(const F32Row& r, const float* __restrict__ k, const float* __restrict__ v,
                                             int n_kv_heads, const double* theta, float scale)
{
    __shared__ float qs[D];
    __shared__ float ps[256];
    const int lane = threadIdx.x;
    for (int m = lane; m < D / 2; m += 64) {
        double sn, cn;
        sincos(r.pos * theta[m], &sn, &cn);
        const double xa = (double)r.q[2 * m], xb = (double)r.q[2 * m + 1];
        qs[2 * m] = (float)(xa * cn - xb * sn);
        qs[2 * m + 1] = (float)(xb * cn + xa * sn);
    }
    __syncthreads();
    constexpr int CPL = D / 64; // channels per lane
    float o[CPL];
#pragma unroll
    for (int e = 0; e < CPL; ++e) o[e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    for (int kb = r.key_lo; kb <= r.key_hi; kb += 256) {
        float s[4];
        float bmax = -INFINITY;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int j = kb + 64 * t + lane;
            s[t] = -INFINITY;
            if (j <= r.key_hi) {
                const float4* kp = (const float4*)(k + ((int64_t)j * n_kv_heads + r.kvh) * D);
                float acc = 0.0f;
#pragma unroll 4
                for (int e = 0; e < D / 4; ++e) {
                    const float4 x = kp[e];
                    acc = fmaf(qs[4 * e], x.x, acc);
                    acc = fmaf(qs[4 * e + 1], x.y, acc);
                    acc = fmaf(qs[4 * e + 2], x.z, acc);
                    acc = fmaf(qs[4 * e + 3], x.w, acc);
                }
                s[t] = acc * scale;
            }
            bmax = fmaxf(bmax, s[t]);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) bmax = fmaxf(bmax, __shfl_xor(bmax, off));
        const float m_new = fmaxf(m_run, bmax); // the block holds at least one visible key, so it is finite
        const float alpha = expf(m_run - m_new);
        float lsum = 0.0f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float p = expf(s[t] - m_new);
            ps[64 * t + lane] = p;
            lsum += p;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) lsum += __shfl_xor(lsum, off);
        l_run = l_run * alpha + lsum;
        m_run = m_new;
#pragma unroll
        for (int e = 0; e < CPL; ++e) o[e] *= alpha;
        __syncthreads();
        const int nk = min(256, r.key_hi - kb + 1);
        for (int jj = 0; jj < nk; ++jj) {
            const float p = ps[jj];
            const float* vp = v + ((int64_t)(kb + jj) * n_kv_heads + r.kvh) * D;
#pragma unroll
            for (int e = 0; e < CPL; ++e) o[e] = fmaf(p, vp[lane + 64 * e], o[e]);
        }
        __syncthreads();
    }
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int e = 0; e < CPL; ++e) r.out[lane + 64 * e] = o[e] * inv;
}

template <int D>
__global__ __launch_bounds__(64) void prefix_attn_f32_kernel(const TrPrefixArgs a)
{
    // block = (packed token of this launch, query head)
    const int tq = a.seq[0].q_row0 + blockIdx.x / a.n_q_heads;
    const int hq = blockIdx.x % a.n_q_heads;
    int lo = 0, hi = a.n_seq - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (a.seq[mid].q_row0 <= tq) lo = mid; else hi = mid - 1;
    }
    const TrSeqDesc sd = a.seq[lo];
    const int i = tq - sd.q_row0;
    F32Row r;
    r.q = (const float*)a.q + ((int64_t)tq * a.n_q_heads + hq) * D;
    r.out = (float*)a.out + ((int64_t)tq * a.n_q_heads + hq) * D;
    r.key_lo = sd.kv_row0;
    r.key_hi = sd.kv_row0 + (sd.kv_len - sd.n_q) + i;
    r.kvh = hq / a.group;
    r.pos = (double)a.q_pos[tq];
    attn_f32_row<D>(r, (const float*)a.k, (const float*)a.v, a.n_kv_heads, a.theta, a.scale);
}

template <int D>
__global__ __launch_bounds__(64) void blockdiag_attn_f32_kernel(const TrBlockDiagArgs a)
{
    const int t = blockIdx.x / a.n_q_heads;
    const int hq = blockIdx.x % a.n_q_heads;
    F32Row r;
    r.q = (const float*)a.q + ((int64_t)t * a.n_q_heads + hq) * D;
    r.out = (float*)a.out + ((int64_t)t * a.n_q_heads + hq) * D;
    r.key_lo = a.tok_start[t];
    r.key_hi = t;
    r.kvh = hq / a.group;
    r.pos = (double)(t - r.key_lo);
    attn_f32_row<D>(r, (const float*)a.k, (const float*)a.v, a.n_kv_heads, a.theta, a.scale);
}

} // namespace

int tr_launch_prefix_attn(const TrPrefixArgs& a, int dtype, int head_dim, bool any_split, int total_rows, hipStream_t s)
{
    if (dtype == TR_F32) {
        if (total_rows <= 0) return TR_OK;
        if (head_dim == 128) hipLaunchKernelGGL(prefix_attn_f32_kernel<128>, dim3(total_rows), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(prefix_attn_f32_kernel<64>, dim3(total_rows), dim3(64), 0, s, a);
        TR_HIP(hipGetLastError());
        return TR_OK;
    }
    if (a.n_items <= 0) return TR_OK;
    if (head_dim == 128) hipLaunchKernelGGL(prefix_attn_kernel<128>, dim3(a.n_items), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(prefix_attn_kernel<64>, dim3(a.n_items), dim3(256), 0, s, a);
    TR_HIP(hipGetLastError());
    if (any_split) {
        const int rows_per_block = 256 / (head_dim / 4);
        const int blocks = (total_rows + rows_per_block - 1) / rows_per_block;
        if (head_dim == 128) hipLaunchKernelGGL(combine_kernel<128>, dim3(blocks), dim3(256), 0, s, a, total_rows);
        else hipLaunchKernelGGL(combine_kernel<64>, dim3(blocks), dim3(256), 0, s, a, total_rows);
        TR_HIP(hipGetLastError());
    }
    return TR_OK;
}

int tr_launch_blockdiag_attn(const TrBlockDiagArgs& a, int dtype, int head_dim, hipStream_t s)
{
    if (a.total_tokens <= 0) return TR_OK;
    if (dtype == TR_F32) {
        const int blocks = a.total_tokens * a.n_q_heads;
        if (head_dim == 128) hipLaunchKernelGGL(blockdiag_attn_f32_kernel<128>, dim3(blocks), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(blockdiag_attn_f32_kernel<64>, dim3(blocks), dim3(64), 0, s, a);
    } else {
        const int blocks = a.n_tiles * a.n_kv_heads;
        if (head_dim == 128) hipLaunchKernelGGL(blockdiag_attn_kernel<128>, dim3(blocks), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(blockdiag_attn_kernel<64>, dim3(blocks), dim3(256), 0, s, a);
    }
    TR_HIP(hipGetLastError());
    return TR_OK;
}
