// Measurement aid, no part of the method: the rate the gfx950 matrix cores sustain on the instructions the score
// and matching kernels are built on, with everything else taken away.  Every wave keeps 8 A fragments and 16 B
// fragments in registers and issues blocks of 64 x 32 x 128 multiply-adds: 16 MFMAs of 32x32x16 in two accumulator
// chains (the matching kernel's inner block), or 32 MFMAs of 16x16x32 on eight accumulators (the score kernels') -
// the inner blocks without LDS, memory or epilogue.  With constant operands the chip runs
// close to its nominal clock; with operands that change from one instruction to the next, as real keys and
// queries do, it sustains less: that second figure, not the datasheet peak, is what the MFMA-bound kernels of
// this library can approach, and bench.py prints it beside their rooflines.
#include "common.h"

namespace lookm {

typedef __attribute__((ext_vector_type(8))) __bf16 pbf16x8;
typedef __attribute__((ext_vector_type(16))) float pf32x16;
typedef __attribute__((ext_vector_type(4))) float pf32x4;

__device__ __forceinline__ uint32_t probe_hash(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// a pair of bf16 values: random sign and mantissa, magnitude in [0.25, 4) - or the constant 1.0
__device__ __forceinline__ uint32_t probe_word(uint32_t key, int random)
{
    if (!random) return 0x3f803f80u;
    const uint32_t r = probe_hash(key);
    const uint32_t lo = (r & 0x807fu) | ((125u + ((r >> 8) & 3u)) << 7);
    const uint32_t hi = ((r >> 16) & 0x807fu) | ((125u + ((r >> 28) & 3u)) << 7);
    return lo | (hi << 16);
}

template <int SHAPE>   // 32: v_mfma_f32_32x32x16_bf16, 16: v_mfma_f32_16x16x32_bf16
__global__ void __launch_bounds__(256, 3)
k_probe_mfma(int iters, int random, float* __restrict__ sink)
{
    const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
    pbf16x8 a[8], b[2][8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        uint4 w;
        w.x = probe_word(gid * 96u + ks * 4u + 0u, random); w.y = probe_word(gid * 96u + ks * 4u + 1u, random);
        w.z = probe_word(gid * 96u + ks * 4u + 2u, random); w.w = probe_word(gid * 96u + ks * 4u + 3u, random);
        a[ks] = __builtin_bit_cast(pbf16x8, w);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const uint32_t base = gid * 96u + 32u + (cb * 8u + ks) * 4u;
            w.x = probe_word(base, random); w.y = probe_word(base + 1u, random);
            w.z = probe_word(base + 2u, random); w.w = probe_word(base + 3u, random);
            b[cb][ks] = __builtin_bit_cast(pbf16x8, w);
        }
    }
    float s = 0.f;
    if (SHAPE == 32) {
        pf32x16 X = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        pf32x16 Y = X;
#pragma unroll 1
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                X = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], b[0][ks], X, 0, 0, 0);
                Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], b[1][ks], Y, 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) s += X[r] + Y[r];
    } else {
        // the same registers as two streamed row groups x four steps (a) and four stationary groups x four steps (b)
        pf32x4 T[2][4];
#pragma unroll
        for (int j = 0; j < 8; ++j) T[j >> 2][j & 3] = pf32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int cg = 0; cg < 4; ++cg)
#pragma unroll
                    for (int rg = 0; rg < 2; ++rg)
                        T[rg][cg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rg * 4 + ks], b[cg >> 1][(cg & 1) * 4 + ks],
                                                                           T[rg][cg], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) s += T[j >> 2][j & 3][0] + T[j >> 2][j & 3][1] + T[j >> 2][j & 3][2] + T[j >> 2][j & 3][3];
    }
    sink[gid] = s;
}

}  // namespace lookm

extern "C" int lookm_probe_mfma(int random_operands, int waves_per_simd, int iters, int reps, float* tflops_host,
                                void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!tflops_host || !workspace) return LOOKM_ERR_INVALID_ARG;
    if (waves_per_simd < 1 || waves_per_simd > 3 || iters < 1 || iters > (1 << 20) || reps < 1 || reps > 1000 ||
        random_operands < 0 || random_operands > 2)
        return LOOKM_ERR_INVALID_ARG;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return LOOKM_ERR_DEVICE;
    const unsigned grid = (unsigned)prop.multiProcessorCount * (unsigned)waves_per_simd;
    if (workspace_bytes < (size_t)grid * 256 * sizeof(float)) return LOOKM_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return LOOKM_ERR_DEVICE;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return LOOKM_ERR_DEVICE; }
    // the first half of the launches brings the chip into its steady state; the second half is timed as one interval
    const int warm = reps / 2, timed = reps - warm;
    int rc = LOOKM_OK;
    for (int r = 0; r < reps; ++r) {
        if (r == warm) (void)hipEventRecord(e0, st);
        if (random_operands == 2)
            hipLaunchKernelGGL(lookm::k_probe_mfma<16>, dim3(grid), dim3(256), 0, st, iters, 1, (float*)workspace);
        else
            hipLaunchKernelGGL(lookm::k_probe_mfma<32>, dim3(grid), dim3(256), 0, st, iters, random_operands,
                               (float*)workspace);
    }
    (void)hipEventRecord(e1, st);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) rc = LOOKM_ERR_DEVICE;
    float ms = 0.f;
    if (rc == LOOKM_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = LOOKM_ERR_DEVICE;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != LOOKM_OK) return rc;
    const double flop = (double)grid * 4.0 * (double)iters * 16.0 * 32768.0 * (double)timed;
    *tflops_host = (ms > 0.f) ? (float)(flop / ((double)ms * 1e-3) / 1e12) : 0.f;
    return LOOKM_OK;
}
