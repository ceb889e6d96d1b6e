// Measurement aid, not part of the operator: a stream of nothing but the 2:4-sparse INT8 matrix
// instruction the lookup of Eq. 4 runs on (arXiv 2302.03213, Eq. 4 as a one-hot contraction), one wave
// per SIMD on every SIMD of the chip.  What it answers: how fast the matrix pipes go on a given kind of
// operand data - the clock the chip holds depends on how many operand bits toggle - which is the floor
// of any kernel built on that instruction and the yardstick bench.py quotes beside the nominal peak.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "lutnn_kernels.h"

namespace lutnn {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));

// acc += A (2:4 sparse) x B; the accumulator is tied to the accumulation registers so that sixteen
// of them (256 registers) fit beside the operands.  Nothing here reads an accumulator before the loop
// has ended, so the wait states the compiler cannot insert for an instruction it does not see are
// not needed.  The host pass only parses this function.
__device__ __forceinline__ void smfmac(v16i& acc, const v4i& a, const v8i& b, int pos) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("v_smfmac_i32_32x32x64_i8 %0, %1, %2, %3" : "+a"(acc) : "v"(a), "v"(b), "v"(pos));
#endif
}

// OPERANDS 0: the same small constants in every instruction; 1: B = eight register sets of random
// 32-bit words (full-range INT8 values), A = random one-hot slices with random positions, as the
// lookup feeds them; 2: as 1 with B values of three bits.
template <int OPERANDS>
__global__ __launch_bounds__(256) void smfmac_stream_kernel(int32_t* __restrict__ sink, int iterations) {
    uint32_t seed = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    auto rnd = [&]() {
        seed = seed * 1664525u + 1013904223u;
        return seed;
    };
    v8i b[8];
    v4i a[4];
    int pos[4];
    for (int k = 0; k < 8; ++k)
        for (int r = 0; r < 8; ++r) {
            uint32_t v = OPERANDS == 0 ? 0x01020304u : rnd();
            if (OPERANDS == 2) v &= 0x07070707u;
            b[k][r] = (int)v;
        }
    for (int k = 0; k < 4; ++k) {
        for (int r = 0; r < 4; ++r) a[k][r] = 0;
        const uint32_t g0 = OPERANDS == 0 ? 0u : rnd() >> 30, g1 = OPERANDS == 0 ? 0u : rnd() >> 30;
        a[k][g0 >> 1] |= 1 << (16 * (g0 & 1));
        a[k][2 + (g1 >> 1)] |= 1 << (16 * (g1 & 1));
        pos[k] = OPERANDS == 0 ? 0x1b1b1b1b : (int)((rnd() >> 30) * 0x1111u | (rnd() >> 30) * 0x11110000u);
    }
    v16i acc[16];
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) smfmac(acc[i], a[i & 3], b[(i * 5 + (i >> 2)) & 7], pos[i & 3]);
    }
    asm volatile("s_nop 15\n\ts_nop 15");  // the last results, before vector instructions read them
    int sum = 0;
    for (int i = 0; i < 16; ++i) sum += acc[i][0] + acc[i][7];
    sink[blockIdx.x * 256 + threadIdx.x] = sum;
}

}  // namespace

hipError_t launch_probe_smfmac_stream(int operands, int iterations, int32_t* sink, hipStream_t s) {
    const dim3 grid((unsigned)compute_units()), block(256);
    if (operands == 0)
        hipLaunchKernelGGL(smfmac_stream_kernel<0>, grid, block, 0, s, sink, iterations);
    else if (operands == 1)
        hipLaunchKernelGGL(smfmac_stream_kernel<1>, grid, block, 0, s, sink, iterations);
    else
        hipLaunchKernelGGL(smfmac_stream_kernel<2>, grid, block, 0, s, sink, iterations);
    return hipGetLastError();
}

}  // namespace lutnn
