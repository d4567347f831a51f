// Measurement aid: what the matrix units sustain when nothing else runs.
//
// A register-resident copy of the large tile's inner loop: 256 workgroups of eight waves (two per SIMD),
// every wave a window of 4 x 2 MFMA 32x32 tiles, four reduction sub-steps per step with fragments of their
// own, so that the operands change from one MFMA to the next exactly as they do in igemm_kernel -- but no
// LDS, no global traffic, no barriers.  Its rate on the benchmark's kind of operands is the ceiling any
// kernel on this chip can approach: the clock of a busy matrix pipe is set by power management and falls
// with the switching activity of the operands (constant operands run at the nominal clock, uniformly
// random ones well below it), and "keeping the matrix units busy" (the paper's criterion, Section VI-B)
// can only be judged against that.  Every wave also reports the shader clock it saw (core cycle counter
// against the 100 MHz real-time counter).
#include "unit_internal.h"

namespace unit {

static __device__ __forceinline__ unsigned mix(unsigned x)
{
    x ^= x >> 16;  x *= 0x7feb352dU;  x ^= x >> 15;  x *= 0x846ca68bU;  x ^= x >> 16;
    return x;
}

template <int DT>
__global__ void __launch_bounds__(512, 1)
mfma_ceiling_kernel(int steps, int random_operands, unsigned long long *out)
{
    typedef Mma<DT, 32> M;
    const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
    v4i a[4][4], b[4][2];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            const unsigned h = mix(threadIdx.x * 977u + blockIdx.x * 131071u + s * 7919u + i * 104729u + 1u);
            v4i v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // bytes uniform over the whole range; 2-byte types: random sign and mantissa, exponent of 1.0
                unsigned r = random_operands ? mix(h + e) : 0x01010101u;
                if (DT == DT_F16) r = random_operands ? ((r & 0x83ff83ffu) | 0x3c003c00u) : 0x3c003c00u;
                if (DT == DT_BF16) r = random_operands ? ((r & 0x807f807fu) | 0x3f803f80u) : 0x3f803f80u;
                v[e] = (int)r;
            }
            if (i < 4) a[s][i] = v; else b[s][i - 4] = v;
        }
    typename M::acc_t acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
    for (int it = 0; it < steps; ++it) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) M::run(acc[i][j], a[s][i], b[s][j]);
    }
    typename M::elem_t sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) sum += acc[i][j][e];
    const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
    if ((threadIdx.x & 63) == 0) {
        unsigned long long *o = out + ((size_t)blockIdx.x * 8 + threadIdx.x / 64) * 4;
        o[0] = c1 - c0;  o[1] = r1 - r0;  o[2] = r0;  o[3] = r1 + (sum == (typename M::elem_t)12345 ? 1 : 0);
    }
}

// out: UNIT_MEASURE_WORKGROUPS * 8 waves * 4 values (core cycles, real-time ticks, start tick, end tick)
hipError_t launch_mfma_ceiling(int dtype, int steps, int random_operands, void *out, hipStream_t st)
{
    unsigned long long *o = static_cast<unsigned long long *>(out);
    const dim3 grid(256), block(512);
    switch (dtype) {
    case 0: hipLaunchKernelGGL(mfma_ceiling_kernel<DT_I8>, grid, block, 0, st, steps, random_operands, o); break;
    case 1: hipLaunchKernelGGL(mfma_ceiling_kernel<DT_F16>, grid, block, 0, st, steps, random_operands, o); break;
    case 2: hipLaunchKernelGGL(mfma_ceiling_kernel<DT_BF16>, grid, block, 0, st, steps, random_operands, o); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace unit
