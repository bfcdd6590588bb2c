// Nearest conserved key by cosine similarity (Section 3.3, Eq. 9) on the gfx950 matrix cores:
// bf16 keys, head_dim 128.  Same machine as the score passes: a workgroup keeps the MFMA B-operand
// fragments of 256 evicted keys (gathered through the evicted index list) in registers and streams
// the conserved keys (gathered through the kept index list) past them in 64-row LDS tiles as the
// A operand.  A lane's 16 accumulator values are 16 conserved slots against ONE evicted key, so the
// running argmax is in-lane; the lane pair (lane, lane^32) is merged once after the loop.
// The similarity matrix never exists in memory.  Ties go to the lower slot (= lower position).
#include "common.h"

namespace lookm {

typedef __attribute__((ext_vector_type(8))) __bf16 nbf16x8;
typedef __attribute__((ext_vector_type(16))) float nf32x16;

constexpr int ND = 128, NBS = 256, NBX = 64, NXSTRIDE = 136;

__global__ void __launch_bounds__(256, 2)
k_nearest_mfma(const bf16_t* __restrict__ k, const float* __restrict__ rnorm, const int32_t* __restrict__ kept,
               const int32_t* __restrict__ evicted, int H, int L, int B, int Le, int32_t* __restrict__ assign,
               float* __restrict__ sim)
{
    __shared__ __attribute__((aligned(16))) bf16_t xs[2][NBX * NXSTRIDE];
    __shared__ __attribute__((aligned(16))) float xr[2][NBX];

    const int h = blockIdx.x % H, tile = blockIdx.x / H;
    k += (size_t)h * L * ND;
    rnorm += (size_t)h * L;
    kept += (size_t)h * B;
    evicted += (size_t)h * Le;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, n = lane & 31;
    const int w0 = tile * NBS + wave * 64;   // first evicted-list index of this wave

    nbf16x8 sf[2][8];
    for (int cb = 0; cb < 2; ++cb) {
        const int e = w0 + cb * 32 + n;
        const bf16_t* row = (e < Le) ? k + (size_t)evicted[e] * ND : nullptr;
        for (int ks = 0; ks < 8; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row) v = *reinterpret_cast<const uint4*>(row + ks * 16 + half * 8);
            sf[cb][ks] = __builtin_bit_cast(nbf16x8, v);
        }
    }

    const int n_it = (B + NBX - 1) / NBX;
    const int ld_row = tid >> 4, ld_chunk = tid & 15;
    uint4 stage[4];
    float stage_r = 0.f;
    auto load_tile = [&](int x0) {
        for (int i = 0; i < 4; ++i) {
            const int slot = x0 + ld_row + 16 * i;
            stage[i] = make_uint4(0, 0, 0, 0);
            if (slot < B) stage[i] = *reinterpret_cast<const uint4*>(k + (size_t)kept[slot] * ND + ld_chunk * 8);
        }
        if (tid < NBX) stage_r = (x0 + tid < B) ? rnorm[kept[x0 + tid]] : 0.f;
    };
    auto store_tile = [&](int buf) {
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<uint4*>(&xs[buf][(ld_row + 16 * i) * NXSTRIDE + ld_chunk * 8]) = stage[i];
        if (tid < NBX) xr[buf][tid] = stage_r;
    };

    float bv[2] = {-INFINITY, -INFINITY};
    int bs[2] = {0x7fffffff, 0x7fffffff};

    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int it = 0; it < n_it; ++it) {
        const int buf = it & 1, x0 = it * NBX;
        if (it + 1 < n_it) load_tile(x0 + NBX);
        const bool tail = x0 + NBX > B;
        for (int rb = 0; rb < 2; ++rb) {
            nbf16x8 a[8];
            const bf16_t* ap = &xs[buf][(rb * 32 + n) * NXSTRIDE + half * 8];
            for (int ks = 0; ks < 8; ++ks) a[ks] = __builtin_bit_cast(nbf16x8, *reinterpret_cast<const uint4*>(ap + ks * 16));
            float rn[16];
            for (int g = 0; g < 4; ++g) {
                const float4 v = *reinterpret_cast<const float4*>(&xr[buf][rb * 32 + 8 * g + 4 * half]);
                rn[4 * g + 0] = v.x; rn[4 * g + 1] = v.y; rn[4 * g + 2] = v.z; rn[4 * g + 3] = v.w;
            }
            const int xb = x0 + rb * 32 + 4 * half;   // slot of element r: xb + 8*(r/4) + r%4 (ascending in r)
            for (int cb = 0; cb < 2; ++cb) {
                nf32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                for (int ks = 0; ks < 8; ++ks)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], sf[cb][ks], acc, 0, 0, 0);
                for (int r = 0; r < 16; ++r) {
                    const int slot = xb + 8 * (r >> 2) + (r & 3);
                    float v = acc[r] * rn[r];
                    if (tail && slot >= B) v = -INFINITY;
                    if (v > bv[cb]) { bv[cb] = v; bs[cb] = slot; }
                }
            }
        }
        if (it + 1 < n_it) store_tile(buf ^ 1);
        __syncthreads();
    }

    for (int cb = 0; cb < 2; ++cb) {
        const float ov = __shfl_xor(bv[cb], 32);
        const int os = __shfl_xor(bs[cb], 32);
        float v = bv[cb];
        int s = bs[cb];
        if (ov > v || (ov == v && os < s)) { v = ov; s = os; }
        const int e = w0 + cb * 32 + n;
        if (half == 0 && e < Le) {
            assign[(size_t)h * Le + e] = s;
            sim[(size_t)h * Le + e] = v * rnorm[evicted[e]];
        }
    }
}

}  // namespace lookm

namespace lookm_host {

int launch_nearest_mfma(const void* k, const int32_t* kept, const int32_t* evicted, int H, int L, int budget,
                        const float* rnorm, int32_t* assign, float* sim, hipStream_t st)
{
    const int Le = L - budget;
    const int tiles = (Le + lookm::NBS - 1) / lookm::NBS;
    hipLaunchKernelGGL(lookm::k_nearest_mfma, dim3((unsigned)(tiles * H)), dim3(256), 0, st, (const lookm::bf16_t*)k,
                       rnorm, kept, evicted, H, L, budget, Le, assign, sim);
    mark(LOOKM_K_NEAREST);
    return hip_ok(hipGetLastError());
}

}  // namespace lookm_host
