// Accumulated attention scores (Section 3.2, Eq. 4) on the gfx950 matrix cores: bf16, head_dim 128.
//
// Both passes are the same machine with the roles of Q and K swapped.  A workgroup (4 waves)
// owns 256 "stationary" rows - query rows in pass 1, key rows in pass 2 - whose MFMA B-operand
// fragments stay in registers (64 rows x 128 dims per wave = 64 VGPRs), and streams the other
// tensor past them in 64-row tiles through double-buffered LDS as the A operand.  With
// v_mfma_f32_32x32x16_bf16 a lane's 16 accumulator values then belong to ONE stationary row and
// 16 streamed rows, so both reductions of the method are in-lane:
//   pass 1: running (max, sum) of 2^(c q.k) over the keys of a query row   -> lse2[i]
//   pass 2: running sum of 2^(c q.k - lse2[i]) over the query rows of a key -> A_s[j]
// The two lanes that share a stationary row (lane, lane^32) are combined once, after the loop.
// Nothing is atomically accumulated; every sum has a fixed order, so results are bitwise
// repeatable.  c = log2(e)/sqrt(d) folds the softmax scale into the exp2 argument.
#include "common.h"

namespace lookm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int SD = 128;        // head dim
constexpr int BS = 256;        // stationary rows per workgroup
constexpr int BX = 64;         // streamed rows per iteration
constexpr int XSTRIDE = 136;   // LDS row stride in bf16 (272 B): 16-byte reads of 8 consecutive rows hit all banks once

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int PASS>
__global__ void __launch_bounds__(256, 2)
k_score_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, int H, int L, float scale2,
             float* __restrict__ lse2, float* __restrict__ scores)
{
    __shared__ __attribute__((aligned(16))) bf16_t xs[2][BX * XSTRIDE];
    __shared__ __attribute__((aligned(16))) float xl[2][BX];

    const int h = blockIdx.x % H;      // heads interleave across consecutive workgroups (and so across XCDs)
    const int t = blockIdx.x / H;
    const int nS = (L + BS - 1) / BS;
    const int tile = (PASS == 1) ? (nS - 1 - t) : t;   // longest strips first
    const int s0 = tile * BS;
    const bf16_t* S = ((PASS == 1) ? q : k) + (size_t)h * L * SD;   // stationary tensor
    const bf16_t* X = ((PASS == 1) ? k : q) + (size_t)h * L * SD;   // streamed tensor
    const float* lse_h = lse2 + (size_t)h * L;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, n = lane & 31;
    const int w0 = s0 + wave * 64;

    // stationary fragments: lane holds row (w0 + cb*32 + n), dims ks*16 + half*8 .. +7
    bf16x8 sf[2][8];
    for (int cb = 0; cb < 2; ++cb) {
        const int row = w0 + cb * 32 + n;
        for (int ks = 0; ks < 8; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row < L) v = *reinterpret_cast<const uint4*>(S + (size_t)row * SD + ks * 16 + half * 8);
            sf[cb][ks] = as_bf16x8(v);
        }
    }

    const int x_begin = (PASS == 1) ? 0 : s0;
    const int x_end = (PASS == 1) ? min(L, s0 + BS) : L;
    const int n_it = (x_end - x_begin + BX - 1) / BX;

    // staging: thread loads 4 chunks of 16 B: rows (tid/16) + 16*i, chunk tid%16
    const int ld_row = tid >> 4, ld_chunk = tid & 15;
    uint4 stage[4];
    float stage_l = 0.f;
    auto load_tile = [&](int x0) {
        for (int i = 0; i < 4; ++i) {
            const int row = x0 + ld_row + 16 * i;
            stage[i] = make_uint4(0, 0, 0, 0);
            if (row < L) stage[i] = *reinterpret_cast<const uint4*>(X + (size_t)row * SD + ld_chunk * 8);
        }
        if (PASS == 2 && tid < BX) stage_l = (x0 + tid < L) ? lse_h[x0 + tid] : INFINITY;
    };
    auto store_tile = [&](int buf) {
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<uint4*>(&xs[buf][(ld_row + 16 * i) * XSTRIDE + ld_chunk * 8]) = stage[i];
        if (PASS == 2 && tid < BX) xl[buf][tid] = stage_l;
    };

    float m[2] = {-1e30f, -1e30f}, l[2] = {0.f, 0.f};   // pass 1 state per stationary row of this lane
    float run[2] = {0.f, 0.f}, run_hi[2] = {0.f, 0.f};  // pass 2 state (two-level running sum)

    load_tile(x_begin);
    store_tile(0);
    __syncthreads();

    for (int it = 0; it < n_it; ++it) {
        const int buf = it & 1;
        const int x0 = x_begin + it * BX;
        if (it + 1 < n_it) load_tile(x0 + BX);

        // wave-uniform tile classification against the causal boundary (query index >= key index)
        const bool skip = (PASS == 1) ? (x0 > w0 + 63) : (x0 + BX - 1 < w0);
        const bool need_mask = (PASS == 1) ? (x0 + BX - 1 > w0) : (x0 < w0 + 63);
        if (!skip) {
            for (int rb = 0; rb < 2; ++rb) {
                bf16x8 a[8];
                const bf16_t* ap = &xs[buf][(rb * 32 + n) * XSTRIDE + half * 8];
                for (int ks = 0; ks < 8; ++ks) a[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(ap + ks * 16));
                float lrow[16];
                if (PASS == 2) {
                    for (int g = 0; g < 4; ++g) {
                        const float4 v = *reinterpret_cast<const float4*>(&xl[buf][rb * 32 + 8 * g + 4 * half]);
                        lrow[4 * g + 0] = v.x; lrow[4 * g + 1] = v.y; lrow[4 * g + 2] = v.z; lrow[4 * g + 3] = v.w;
                    }
                }
                for (int cb = 0; cb < 2; ++cb) {
                    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    for (int ks = 0; ks < 8; ++ks)
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], sf[cb][ks], acc, 0, 0, 0);
                    const int s = w0 + cb * 32 + n;                    // stationary index of this lane
                    const int xb = x0 + rb * 32 + 4 * half;            // streamed index of element r: xb + 8*(r/4) + r%4
                    if (PASS == 1) {
                        float v[16];
                        for (int r = 0; r < 16; ++r) v[r] = acc[r] * scale2;
                        if (need_mask)
                            for (int r = 0; r < 16; ++r)
                                if (xb + 8 * (r >> 2) + (r & 3) > s) v[r] = -INFINITY;
                        float bm = v[0];
                        for (int r = 1; r < 16; ++r) bm = fmaxf(bm, v[r]);
                        const float mn = fmaxf(m[cb], bm);
                        float sum = 0.f;
                        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(v[r] - mn);
                        l[cb] = l[cb] * __builtin_amdgcn_exp2f(m[cb] - mn) + sum;
                        m[cb] = mn;
                    } else {
                        float p[16];
                        for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(fmaf(acc[r], scale2, -lrow[r]));
                        if (need_mask)
                            for (int r = 0; r < 16; ++r)
                                if (xb + 8 * (r >> 2) + (r & 3) < s) p[r] = 0.f;
                        float sum = 0.f;
                        for (int r = 0; r < 16; ++r) sum += p[r];
                        run[cb] += sum;
                    }
                }
            }
            if (PASS == 2 && (it & 31) == 31) {
                for (int cb = 0; cb < 2; ++cb) { run_hi[cb] += run[cb]; run[cb] = 0.f; }
            }
        }
        if (it + 1 < n_it) store_tile(buf ^ 1);
        __syncthreads();
    }

    for (int cb = 0; cb < 2; ++cb) {
        const int s = w0 + cb * 32 + n;
        if (PASS == 1) {
            const float mo = __shfl_xor(m[cb], 32), lo = __shfl_xor(l[cb], 32);
            const float M = fmaxf(m[cb], mo);
            // lower half first, so both lanes of a pair form the same sum
            const float la = half ? lo : l[cb], ma = half ? mo : m[cb];
            const float lb = half ? l[cb] : lo, mb = half ? m[cb] : mo;
            const float Ls = la * __builtin_amdgcn_exp2f(ma - M) + lb * __builtin_amdgcn_exp2f(mb - M);
            if (half == 0 && s < L) lse2[(size_t)h * L + s] = M + log2f(Ls);
        } else {
            const float tot = run_hi[cb] + run[cb];
            const float other = __shfl_xor(tot, 32);
            if (half == 0 && s < L) scores[(size_t)h * L + s] = tot + other;
        }
    }
}

}  // namespace lookm

namespace lookm_host {

int launch_scores_mfma(const void* q, const void* k, int H, int L, int d, float* lse, float* scores, hipStream_t st)
{
    if (d != lookm::SD) return LOOKM_ERR_UNSUPPORTED;
    const int nS = (L + lookm::BS - 1) / lookm::BS;
    const float scale2 = lookm::kLog2e / sqrtf((float)d);
    dim3 grid((unsigned)(nS * H)), block(256);
    hipLaunchKernelGGL(lookm::k_score_mfma<1>, grid, block, 0, st, (const lookm::bf16_t*)q, (const lookm::bf16_t*)k, H,
                       L, scale2, lse, scores);
    mark(LOOKM_K_SCORE_LSE);
    hipLaunchKernelGGL(lookm::k_score_mfma<2>, grid, block, 0, st, (const lookm::bf16_t*)q, (const lookm::bf16_t*)k, H,
                       L, scale2, lse, scores);
    mark(LOOKM_K_SCORE_COLSUM);
    return hip_ok(hipGetLastError());
}

}  // namespace lookm_host
