// Issue-rate ceiling of the attention loop's matrix instruction on this chip, measured rather than quoted.
//
// The kernel is the inner loop of the attention kernels with everything but the matrix work taken out: 8 waves per
// compute unit, one workgroup per compute unit, v_mfma_f32_32x32x16_bf16 with the A operand read from LDS through the
// same swizzled 16-byte reads the key tiles use, four independent accumulators per wave.  With `random_operands` the
// LDS holds bf16 values of random sign and mantissa with magnitudes in [0.5, 4), the kind of data attention feeds the
// instruction; without it the operands are a few constants.  The two rates differ because the chip's clock follows
// its power draw, and the data decide how much the multiplier array toggles.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tr_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define TR_LDS __attribute__((address_space(3)))

namespace {

constexpr int PROBE_THREADS = 512;
constexpr int PROBE_LDS = 65536;
constexpr int PROBE_UNROLL = 8;

__device__ inline uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// sign and 7 mantissa bits random, exponent 126..128
__device__ inline uint32_t random_bf16(uint32_t r)
{
    return (r & 0x8000u) | ((126u + (r >> 16) % 3u) << 7) | (r & 0x7fu);
}

__global__ __launch_bounds__(PROBE_THREADS, 1) void mfma_loop_probe_kernel(float* sink, int iters, int random_operands)
{
    extern __shared__ __attribute__((aligned(1024))) char probe_lds[];
    for (int i = threadIdx.x; i < PROBE_LDS / 4; i += PROBE_THREADS) {
        const uint32_t r = mix32(i * 2654435761u + blockIdx.x * 40503u + 1u);
        ((uint32_t*)probe_lds)[i] = random_operands ? (random_bf16(r) | (random_bf16(mix32(r)) << 16)) : (0x3c003c00u + (i & 7));
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    TR_LDS const char* lb = (TR_LDS const char*)probe_lds;
    int koff[PROBE_UNROLL];
#pragma unroll
    for (int ks = 0; ks < PROBE_UNROLL; ++ks) koff[ks] = c * 256 + (((2 * ks + h) ^ (c & 15)) * 16);
    bf16x8 b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t r = mix32(threadIdx.x * 131u + e * 71u + blockIdx.x * 17u);
        b[e] = random_operands ? (__bf16)(((int)(r % 257u) - 128) * 0.011f) : (__bf16)(0.001f * (lane + e));
    }
    f32x16 acc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
    bf16x8 a_next[2] = {b, b};
    for (int it = 0; it < iters; ++it) {
        const int shift = (it & 3) * 8192 + (it & 1) * 32768;
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u) {
            const bf16x8 a = a_next[u & 1];
            a_next[u & 1] = *(TR_LDS const bf16x8*)(lb + koff[u] + shift);
            acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[u & 3], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[a][e];
    sink[blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

}  // namespace

int tr_launch_mfma_loop_probe(int iters, int random_operands, float* sink, hipStream_t stream, double* flops)
{
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)mfma_loop_probe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, PROBE_LDS) != hipSuccess) return -1;
        configured = true;
    }
    const int groups = TrChip::CUS;
    hipLaunchKernelGGL(mfma_loop_probe_kernel, dim3(groups), dim3(PROBE_THREADS), PROBE_LDS, stream, sink, iters, random_operands);
    // one v_mfma_f32_32x32x16_bf16 is 32 x 32 x 16 multiply-adds
    *flops = (double)groups * (PROBE_THREADS / 64) * (double)iters * PROBE_UNROLL * (2.0 * 32 * 32 * 16);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
