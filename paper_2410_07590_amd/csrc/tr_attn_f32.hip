// fp32 attention path: plain FMA arithmetic, one wavefront per (query token, query head).
// Used for fp32 storage (the tiny fp32 configuration); accuracy first, speed irrelevant.
#include "tr_internal.h"

namespace {

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
                                             int n_kv_heads, const double* theta, float scale, int rope_half)
{
    __shared__ float qs[D];
    __shared__ float ps[256];
    const int lane = threadIdx.x;
    for (int m = lane; m < D / 2; m += 64) {
        double sn, cn;
        sincos(r.pos * theta[m], &sn, &cn);
        const int ia = rope_half ? m : 2 * m, ib = rope_half ? m + D / 2 : 2 * m + 1; // the pair's two channels
        const double xa = (double)r.q[ia], xb = (double)r.q[ib];
        qs[ia] = (float)(xa * cn - xb * sn);
        qs[ib] = (float)(xb * cn + xa * sn);
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
    attn_f32_row<D>(r, (const float*)a.k, (const float*)a.v, a.n_kv_heads, a.theta, a.scale, a.rope_half);
}

template <int D>
__global__ __launch_bounds__(64) void blockdiag_attn_f32_kernel(const TrBlockDiagArgs a)
{
    const int t = blockIdx.x / a.n_q_heads;
    const int hq = blockIdx.x % a.n_q_heads;
    F32Row r;
    r.q = (const float*)a.q + ((int64_t)t * a.n_q_heads + hq) * D;
    r.out = (float*)a.out + ((int64_t)t * a.n_q_heads + hq) * D;
    r.key_lo = min(max(a.tok_start[t], 0), t);
    r.key_hi = t;
    r.kvh = hq / a.group;
    r.pos = a.pos ? (double)a.pos[t] : (double)(t - r.key_lo);
    attn_f32_row<D>(r, (const float*)a.k, (const float*)a.v, a.n_kv_heads, a.theta, a.scale, a.rope_half);
}

} // namespace

int tr_launch_prefix_attn_f32(const TrPrefixArgs& a, int head_dim, int total_rows, hipStream_t s)
{
    if (total_rows <= 0) return TR_OK;
    if (head_dim == 128) hipLaunchKernelGGL(prefix_attn_f32_kernel<128>, dim3(total_rows), dim3(64), 0, s, a);
    else hipLaunchKernelGGL(prefix_attn_f32_kernel<64>, dim3(total_rows), dim3(64), 0, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

int tr_launch_blockdiag_attn_f32(const TrBlockDiagArgs& a, int head_dim, hipStream_t s)
{
    if (a.total_tokens <= 0) return TR_OK;
    const int blocks = a.total_tokens * a.n_q_heads;
    if (head_dim == 128) hipLaunchKernelGGL(blockdiag_attn_f32_kernel<128>, dim3(blocks), dim3(64), 0, s, a);
    else hipLaunchKernelGGL(blockdiag_attn_f32_kernel<64>, dim3(blocks), dim3(64), 0, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}
