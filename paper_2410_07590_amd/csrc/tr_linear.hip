// Projections around the attention (Eq. 1: Q, K, V = X W; the output projection is the same product) for the
// query tokens of a request: y[m, n] = sum_k x[m, k] w[n, k] with at most 128 rows of x.  With so few rows the
// product is bound by streaming the weights once from HBM, so the kernel is organised around that stream.
//   * A workgroup owns 128 output features (four waves x 32 rows of w, each row contiguous along k) and a slice of k.
//   * k is walked in chunks of 128 values.  Every wave fetches its 32 x 256-byte piece of w with direct global -> LDS
//     loads that read whole 256-byte runs (16-byte pieces XOR-swizzled by the row on the source side) and reads it
//     back in the matrix instruction's operand layout; reading w straight in operand layout would touch 32 rows x
//     32 bytes per instruction, which the memory system serves at a fraction of its rate.
//   * The chunk of x (all rows x 256 bytes) is fetched once per workgroup the same way and shared by the four waves:
//     x is re-read once per 128 features, not once per 32.
//   * v_mfma_f32_32x32x16_bf16 with w rows as the A operand and x rows as the B operand makes the arithmetic free,
//     provided its operand reads are batched ahead of it: read-wait-multiply per step left the products of a chunk
//     as one chain of LDS latencies, which showed as soon as x had more than 32 rows.
//   * Up to three chunks per workgroup are in flight in a ring of LDS slots while the current one is multiplied.
// Slices of k that live in different workgroups write fp32 partial sums that a second small kernel adds in a fixed
// order: no atomics, same inputs, same bits.
#include "tr_internal.h"

#include <stdlib.h>
#include <string.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Up to TR_LINEAR_MAX_OUT weights share x in one launch (query, key and value): output j owns the 32-feature tiles
// [tile0[j], tile0[j+1]) and the columns [32 tile0[j], 32 tile0[j+1]) of the partial sums.
struct TrLinearArgs {
    const __bf16* x;                    // [M, K]
    const __bf16* w[TR_LINEAR_MAX_OUT]; // [N_j, K]
    __bf16* y[TR_LINEAR_MAX_OUT];       // [M, N_j]
    float* partial;                     // [n_split, M, N] when n_split > 1, N = sum of the N_j
    int32_t tile0[TR_LINEAR_MAX_OUT + 1];
    int32_t n_out;
    int32_t M, N, K;
    int32_t n_split;
    int32_t m_split;                    // 1, or 2: rows [0, 64) and [64, M) of x go to two workgroups of the same XCD
};

constexpr int LIN_CK = 128;           // values of k per chunk: 256 bytes of every row
constexpr int LIN_PPR = LIN_CK / 8;   // 16-byte pieces per row of a chunk: 16
constexpr int LIN_ROW = LIN_CK * 2;   // bytes per parked row
constexpr int LIN_MAX_SPLIT = 16;     // k-slices across workgroups, at most

#define LDS_AS __attribute__((address_space(3)))

__device__ __forceinline__ int lin_piece_off(int row, int piece) { return row * LIN_ROW + ((piece ^ (row & (LIN_PPR - 1))) * 16); }

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
constexpr int lin_vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
template <int N> __device__ __forceinline__ void lin_wait_vm() { __builtin_amdgcn_s_waitcnt(lin_vmcnt_imm(N)); }

template <int MT> constexpr int lin_slot_bytes() { return (4 + MT) * 32 * LIN_ROW; }    // four waves' w pieces, then x
// Chunks in flight per workgroup.  A small weight (the attention projections) is over within a few round trips, so
// one workgroup per CU requests its whole slice at once (DEEP: three chunks, two from 96 rows of x on, <= 144 KB of
// LDS).  A large weight (an MLP's) streams better with one chunk per workgroup and three workgroups per CU.
template <int MT, bool DEEP> constexpr int lin_slots() { return !DEEP ? 1 : (MT <= 2 ? 3 : 2); }
constexpr int64_t LIN_LARGE_WEIGHT_BYTES = 64ll << 20;

// MT: 32-row blocks of x (ceil(M / 32), 1..4)
template <int MT, bool DEEP>
__global__ __launch_bounds__(256) void linear_kernel(const TrLinearArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) char lds_raw[];
    LDS_AS char* lds = (LDS_AS char*)lds_raw;
    constexpr int NSLOT = lin_slots<MT, DEEP>(), SLOT = lin_slot_bytes<MT>();
    constexpr int IPC = 8 + 2 * MT; // load instructions per wave and chunk: its 8 KB of w, its quarter of x
    const int groups = (a.N / 32 + 3) / 4;                      // workgroups along the features
    // With two row halves, blocks b and b + 8 (same XCD, dispatched together) take the two halves of one
    // (features, k-slice) item, so that the second read of its weights is served by that XCD's L2.
    int item = blockIdx.x, m0 = 0;
    if (a.m_split == 2) {
        item = ((blockIdx.x >> 4) << 3) | (blockIdx.x & 7);
        m0 = ((blockIdx.x >> 3) & 1) * (32 * MT);
        if (item >= groups * a.n_split) return;                 // padding of the grid to a multiple of 16 (whole workgroup)
    }
    const int M = min(a.M - m0, 32 * MT);                       // rows of x this workgroup multiplies
    const __bf16* xrows = a.x + (int64_t)m0 * a.K;
    const int group = item % groups, split = item / groups;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int tile = min(4 * group + wave, a.N / 32 - 1);       // a wave past the last tile redoes it and stores nothing
    const bool tile_mine = 4 * group + wave < a.N / 32;
    int j = 0; // the output this tile belongs to
    while (j + 1 < a.n_out && tile >= a.tile0[j + 1]) ++j;
    const int ltile = tile - a.tile0[j];
    const int Nj = 32 * (a.tile0[j + 1] - a.tile0[j]);
    // chunks of this workgroup: a contiguous range; the last chunk of a row may be short
    const int total_chunks = (a.K + LIN_CK - 1) / LIN_CK;
    const int c0 = (int)((int64_t)total_chunks * split / a.n_split), c1 = (int)((int64_t)total_chunks * (split + 1) / a.n_split);
    const int n_chunks = c1 - c0;

    // Direct global -> LDS loads: instruction i of a wave fills 1 KB, lane l the 16-byte piece 64 i + l of the
    // destination, i.e. row (64 i + l) / 16, parked piece (64 i + l) % 16; it therefore fetches the logical piece
    // parked there (the XOR swizzle is applied on the source side).  Four rows x 256 contiguous bytes per instruction.
    const int lrow = lane / LIN_PPR, ppiece = lane % LIN_PPR;
    const int last_piece = a.K / 8 - 1; // pieces past the end of a row are read from its last piece and never used
    const __bf16* wbase = a.w[j] + (int64_t)(ltile * 32) * a.K;
    auto issue_chunk = [&](int c, LDS_AS char* slot) {
        LDS_AS char* wdst = slot + wave * (32 * LIN_ROW);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = 4 * i + lrow;
            const int piece = min(c * LIN_PPR + (ppiece ^ (row & (LIN_PPR - 1))), last_piece);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(wbase + (int64_t)row * a.K + 8 * piece),
                                             (LDS_AS void*)(wdst + i * 1024), 16, 0, 0);
        }
        LDS_AS char* xdst = slot + 4 * 32 * LIN_ROW;
#pragma unroll
        for (int i = 0; i < 2 * MT; ++i) {
            const int row = 4 * (wave * 2 * MT + i) + lrow; // this wave's quarter of the 32 MT rows
            const int piece = min(c * LIN_PPR + (ppiece ^ (row & (LIN_PPR - 1))), last_piece);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xrows + (int64_t)min(row, M - 1) * a.K + 8 * piece),
                                             (LDS_AS void*)(xdst + (wave * 2 * MT + i) * 1024), 16, 0, 0);
        }
    };

    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mt][e] = 0.0f;

#pragma unroll
    for (int p = 0; p < NSLOT; ++p)
        if (p < n_chunks) issue_chunk(c0 + p, lds + p * SLOT);
    for (int t = 0; t < n_chunks; ++t) {
        // chunk t has landed once only the loads of the chunks issued after it are outstanding
        const int later = min(NSLOT - 1, n_chunks - 1 - t);
        if (later >= 2) lin_wait_vm<2 * IPC>();
        else if (later == 1) lin_wait_vm<IPC>();
        else lin_wait_vm<0>();
        __builtin_amdgcn_s_barrier(); // every wave's part of chunk t (its share of x included) is in LDS
        LDS_AS const char* slot = lds + (t % NSLOT) * SLOT;
        LDS_AS const char* wb = slot + wave * (32 * LIN_ROW);
        LDS_AS const char* xb0 = slot + 4 * 32 * LIN_ROW;
        const int steps = min(LIN_CK, a.K - (c0 + t) * LIN_CK) / 16;
        auto step = [&](int s) {
            const bf16x8 wa = *(LDS_AS const bf16x8*)(wb + lin_piece_off(r, 2 * s + h));
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16x8 xb = *(LDS_AS const bf16x8*)(xb0 + lin_piece_off(32 * mt + r, 2 * s + h));
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, xb, acc[mt], 0, 0, 0);
            }
        };
        if (steps == LIN_CK / 16) { // a whole chunk: the operands of SB steps are read before their products start
            constexpr int SB = 2; // deeper batches measured the same and cost registers
#pragma unroll
            for (int s0 = 0; s0 < LIN_CK / 16; s0 += SB) {
                bf16x8 wa[SB], xb[MT][SB];
#pragma unroll
                for (int s = 0; s < SB; ++s) {
                    wa[s] = *(LDS_AS const bf16x8*)(wb + lin_piece_off(r, 2 * (s0 + s) + h));
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) xb[mt][s] = *(LDS_AS const bf16x8*)(xb0 + lin_piece_off(32 * mt + r, 2 * (s0 + s) + h));
                }
                __builtin_amdgcn_sched_barrier(0); // keep the reads above: the scheduler would sink each to its use
#pragma unroll
                for (int s = 0; s < SB; ++s)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[s], xb[mt][s], acc[mt], 0, 0, 0);
            }
        } else {                    // the short last chunk of a row (workgroup-uniform)
#pragma unroll
            for (int s = 0; s < LIN_CK / 16; ++s)
                if (s < steps) step(s);
        }
        if (t + NSLOT < n_chunks) {
            __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0): this wave's operand reads of the slot are done
            __builtin_amdgcn_s_barrier();        // ... and everyone else's: the slot can be refilled
            issue_chunk(c0 + t + NSLOT, lds + (t % NSLOT) * SLOT);
        }
    }
    if (!tile_mine) return;

    // element e of acc[mt] is y_j[32 mt + r][32 ltile + 8 (e >> 2) + 4 h + (e & 3)]
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (32 * mt + r >= M) continue;
        const int m = m0 + 32 * mt + r;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int n = 32 * tile + 8 * q4 + 4 * h; // column among all outputs
            if (a.n_split == 1) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[mt][4 * q4 + e];
                *(bf16x4*)(a.y[j] + (int64_t)m * Nj + (n - 32 * a.tile0[j])) = o;
            } else {
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = acc[mt][4 * q4 + e];
                *(f32x4*)(a.partial + ((int64_t)split * a.M + m) * a.N + n) = o;
            }
        }
    }
}

// y = bf16(sum over the k-slices, in slice order); four outputs per thread
__global__ __launch_bounds__(256) void linear_combine_kernel(const TrLinearArgs a)
{
    const int64_t total4 = (int64_t)a.M * a.N / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total4) return;
    const int m = (int)(4 * i / a.N), n = (int)(4 * i % a.N);
    int j = 0;
    while (j + 1 < a.n_out && n >= 32 * a.tile0[j + 1]) ++j;
    // every slice's load is issued before the first sum needs one: the latencies overlap instead of adding up
    f32x4 t[LIN_MAX_SPLIT];
#pragma unroll
    for (int sp = 0; sp < LIN_MAX_SPLIT; ++sp)
        if (sp < a.n_split) t[sp] = *(const f32x4*)(a.partial + (int64_t)sp * a.M * a.N + 4 * i);
    f32x4 s = t[0];
#pragma unroll
    for (int sp = 1; sp < LIN_MAX_SPLIT; ++sp)
        if (sp < a.n_split) {
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] += t[sp][e];
        }
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (__bf16)s[e];
    *(bf16x4*)(a.y[j] + (int64_t)m * (32 * (a.tile0[j + 1] - a.tile0[j])) + (n - 32 * a.tile0[j])) = o;
}

} // namespace

// k-slices across workgroups.  Small weights: one workgroup per CU, about 200 of them measured best (more slices
// cost more partial traffic and shorter streams than the last CUs gain).  Large weights: about 450 workgroups, up
// to three per CU.  At least two 128-value chunks of k in each.

static bool lin_large(int32_t N, int32_t K) { return (int64_t)N * K * 2 >= LIN_LARGE_WEIGHT_BYTES; }
// More than 96 rows of x against a small weight: two workgroups per item, one per 64 rows, each with the ring of
// three chunks that 64 rows leave room for (128 rows x 4608 x 3584: 20.7 -> 18.9 us; at 65..96 rows and for large
// weights one workgroup per item measured faster).  tr_set_tuning("lin_msplit", 1) keeps one.
static int lin_m_split(int32_t M, int32_t N, int32_t K)
{
    if (tr_knob(TR_KNOB_LIN_MSPLIT, 0) == 1) return 1;
    return (M > 96 && !lin_large(N, K)) ? 2 : 1;
}

int tr_linear_splits(int32_t M, int32_t N, int32_t K)
{
    const int groups = (N / 32 + 3) / 4 * lin_m_split(M, N, K), chunks = (K + LIN_CK - 1) / LIN_CK;
    int n_split = ((lin_large(N, K) ? 450 : 200) + groups / 2) / groups;
    if (n_split > chunks / 2) n_split = chunks / 2;
    if (n_split > LIN_MAX_SPLIT) n_split = LIN_MAX_SPLIT;
    if (const int forced = tr_knob(TR_KNOB_LIN_SPLIT, 0); forced >= 1 && forced <= chunks && forced <= LIN_MAX_SPLIT) n_split = forced;
    if (n_split < 1) n_split = 1;
    return n_split;
}

template <int MT, bool DEEP>
static int launch_linear_mt(const TrLinearArgs& a, hipStream_t s)
{
    auto kern = linear_kernel<MT, DEEP>;
    constexpr int lds = lin_slots<MT, DEEP>() * lin_slot_bytes<MT>();
    static std::atomic<uint64_t> configured{0};
    if (int rc = tr_raise_lds_limit((const void*)kern, lds, &configured)) return rc;
    const int items = (a.N / 32 + 3) / 4 * a.n_split;
    const int blocks = a.m_split == 2 ? 16 * ((items + 7) / 8) : items;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), lds, s, a);
    TR_HIP(hipGetLastError());
    return TR_OK;
}

int tr_launch_linear(const void* x, int32_t n_out, const void* const* w, void* const* y, const int32_t* n_features, void* partial,
                     int32_t M, int32_t K, hipStream_t s)
{
    TrLinearArgs a;
    memset(&a, 0, sizeof a);
    a.x = (const __bf16*)x;
    a.n_out = n_out;
    int32_t N = 0;
    for (int j = 0; j < n_out; ++j) {
        a.w[j] = (const __bf16*)w[j];
        a.y[j] = (__bf16*)y[j];
        a.tile0[j] = N / 32;
        N += n_features[j];
    }
    a.tile0[n_out] = N / 32;
    a.partial = (float*)partial;
    a.M = M;
    a.N = N;
    a.K = K;
    a.n_split = tr_linear_splits(M, N, K);
    a.m_split = lin_m_split(M, N, K);
    int rc;
    const bool deep = !lin_large(N, K);
    switch (a.m_split == 2 ? 2 : (M + 31) / 32) {
    case 1: rc = deep ? launch_linear_mt<1, true>(a, s) : launch_linear_mt<1, false>(a, s); break;
    case 2: rc = deep ? launch_linear_mt<2, true>(a, s) : launch_linear_mt<2, false>(a, s); break;
    case 3: rc = deep ? launch_linear_mt<3, true>(a, s) : launch_linear_mt<3, false>(a, s); break;
    default: rc = deep ? launch_linear_mt<4, true>(a, s) : launch_linear_mt<4, false>(a, s); break;
    }
    if (rc) return rc;
    if (a.n_split > 1) {
        const int64_t total4 = (int64_t)M * N / 4;
        hipLaunchKernelGGL(linear_combine_kernel, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s, a);
        TR_HIP(hipGetLastError());
    }
    return TR_OK;
}
