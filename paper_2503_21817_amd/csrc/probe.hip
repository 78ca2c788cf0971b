// Measurement aid: what the matrix cores of this chip sustain with NO operand traffic at all.
// Every wavefront keeps its A and B fragments in registers and issues independent
// v_mfma_f32_16x16x32_bf16 back to back, in the form and operand order of a compute phase of the
// GEMM core (how often an operand register set changes between consecutive MFMAs matters for the
// power drawn); operands are either one constant or pseudo-random
// bf16 values (the power drawn by the multipliers, and with it the clock the chip can hold,
// depends on the data).  The result is the ceiling the GEMM kernels are compared with next to
// the published peak.  It also reports the shader clock it ran at (cycle counter against the
// 100 MHz wall counter).
#include "kernels.hpp"

namespace skipffn {

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_MI = 8, PROBE_NI = 4;   // the MFMA tiles of a wave of the GEMM core: 32 per iteration, 16384 FLOP each

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(PROBE_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void mfma_probe_kernel(int iters, int random_operands,
                                                                   float* __restrict__ out,
                                                                   long long* __restrict__ clocks) {
    const uint32_t gid = blockIdx.x * PROBE_THREADS + threadIdx.x;
    // operand registers as a wave of the GEMM core holds them during a compute phase: 8 fragments of
    // one operand, 4 of the other, every pair multiplied once per iteration in the same order
    bf16x8 a[PROBE_MI], b[PROBE_NI];
#pragma unroll
    for (int f = 0; f < PROBE_MI + PROBE_NI; ++f) {
        u32x4 r;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (random_operands) {
                // sign, exponent within [2^-4, 2^0), random mantissa: about N(0, 1)-like spread
                auto val = [](uint32_t r) { return ((r & 1u) << 15) | ((0x7bu + ((r >> 1) & 3u)) << 7) | ((r >> 8) & 127u); };
                const uint32_t h0 = probe_hash(gid * 64u + f * 4u + k);
                r[k] = val(h0) | (val(h0 >> 16) << 16);
            } else {
                r[k] = 0x3f803f80u;     // 1.0, 1.0
            }
        }
        if (f < PROBE_MI) a[f] = __builtin_bit_cast(bf16x8, r);
        else b[f - PROBE_MI] = __builtin_bit_cast(bf16x8, r);
    }
    f32x4 acc[PROBE_MI][PROBE_NI];
#pragma unroll
    for (int i = 0; i < PROBE_MI; ++i)
#pragma unroll
        for (int j = 0; j < PROBE_NI; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;
    const long long w0 = wall_clock64(), c0 = clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_MI; ++i)
#pragma unroll
            for (int jj = 0; jj < PROBE_NI; ++jj) {
                const int j = (i & 1) ? PROBE_NI - 1 - jj : jj;      // boustrophedon, as in the GEMM core
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
            }
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < PROBE_MI; ++i)
#pragma unroll
        for (int j = 0; j < PROBE_NI; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += acc[i][j][r];
    out[gid] = s;
    if (threadIdx.x == 0) {
        clocks[2 * blockIdx.x] = c1 - c0;
        clocks[2 * blockIdx.x + 1] = w1 - w0;
    }
}

hipError_t launch_mfma_probe(int blocks, int iters, int random_operands, float* out, long long* clocks,
                             hipStream_t s) {
    if (blocks <= 0 || iters <= 0) return hipSuccess;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)blocks), dim3(PROBE_THREADS), 0, s, iters,
                       random_operands, out, clocks);
    return hipGetLastError();
}

}  // namespace skipffn
