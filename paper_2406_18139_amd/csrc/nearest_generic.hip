// Many-to-one nearest-neighbour matching (Section 3.3, Eq. 9): for every evicted key the conserved
// key with the highest cosine similarity, on the ORIGINAL keys.  Portable fp32-FMA kernels for any
// supported dtype / head_dim; bf16 with head_dim 128 takes the matrix-core kernel in nearest_mfma.hip.
//
// The L^e x L^c similarity matrix is never stored: a workgroup owns 64 evicted rows (gathered through
// the evicted index list), walks the conserved rows in 64-wide tiles, and keeps a running
// (best value, best slot) per row.  cos(i, j) = (k_i . k_j) * rnorm_i * rnorm_j with rnorm = 1/||k||
// (0 for a zero key, which gives cosine 0 against everything).  Ties go to the lower slot.
#include "common.h"

namespace lookm {

constexpr int NT_TS = 64;

// rnorm[h, j] = 1 / ||k[h, j, :]||, or 0 when the norm vanishes.  One 8-lane group per row.  The squares are summed
// in binary64 (for bf16 keys every square and, in practice, every partial sum is exact), so that the result is the
// correctly rounded inverse norm up to one final rounding: the matching on the matrix cores budgets half a unit in
// the last place for this factor.
template <typename T>
__global__ void __launch_bounds__(256) k_rnorm(const T* __restrict__ k, size_t rows, int d, float* __restrict__ rnorm)
{
    const size_t row = (size_t)blockIdx.x * 32 + (threadIdx.x >> 3);
    const int sub = threadIdx.x & 7;
    double s = 0.0;
    if (row < rows) {
        for (int c0 = sub * 8; c0 < d; c0 += 64) {
            float v[8];
            load8(k + row * d + c0, v);
            for (int i = 0; i < 8; ++i) s = fma((double)v[i], (double)v[i], s);
        }
    }
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    s += __shfl_xor(s, 4);
    if (row < rows && sub == 0) rnorm[row] = inverse_norm(s);
}

// stage 64 gathered rows of x into LDS as xt[c][r]; list entries past n read as zero rows
template <typename T>
__device__ __forceinline__ void stage_gather(const T* __restrict__ x, const int32_t* __restrict__ idx, int i0, int n,
                                             int d, float* xt)
{
    const int chunks = NT_TS * (d / 8);
    for (int ch = threadIdx.x; ch < chunks; ch += blockDim.x) {
        const int r = ch % NT_TS, c0 = (ch / NT_TS) * 8;
        float v[8];
        if (i0 + r < n) load8(x + (size_t)idx[i0 + r] * d + c0, v);
        else
            for (int i = 0; i < 8; ++i) v[i] = 0.f;
        for (int i = 0; i < 8; ++i) xt[(c0 + i) * NT_TS + r] = v[i];
    }
}

template <typename T>
__global__ void __launch_bounds__(256)
k_nearest_generic(const T* __restrict__ k, const float* __restrict__ rnorm, const int32_t* __restrict__ kept,
                  const int32_t* __restrict__ evicted, int L, int d, int B, int Le, int32_t* __restrict__ assign,
                  float* __restrict__ sim)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* et = smem;                          // evicted tile  [d][64]
    float* ct = smem + (size_t)d * NT_TS;      // conserved tile [d][64]
    __shared__ float c_rn[NT_TS];
    const int h = blockIdx.y, e0 = blockIdx.x * NT_TS;
    k += (size_t)h * L * d;
    rnorm += (size_t)h * L;
    kept += (size_t)h * B;
    evicted += (size_t)h * Le;
    const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;

    stage_gather(k, evicted, e0, Le, d, et);
    float bv[4];
    int bs[4];
    for (int r = 0; r < 4; ++r) { bv[r] = -INFINITY; bs[r] = 0x7fffffff; }
    for (int r0 = 0; r0 < B; r0 += NT_TS) {
        __syncthreads();
        stage_gather(k, kept, r0, B, d, ct);
        if (threadIdx.x < NT_TS) c_rn[threadIdx.x] = (r0 + threadIdx.x < B) ? rnorm[kept[r0 + threadIdx.x]] : 0.f;
        __syncthreads();
        float acc[4][4];
        for (int r = 0; r < 4; ++r)
            for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
        for (int c = 0; c < d; ++c) {
            const float4 a = *reinterpret_cast<const float4*>(et + c * NT_TS + ty * 4);
            const float4 b = *reinterpret_cast<const float4*>(ct + c * NT_TS + tx * 4);
            const float av[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
            for (int r = 0; r < 4; ++r)
                for (int cc = 0; cc < 4; ++cc) acc[r][cc] = fmaf(av[r], bw[cc], acc[r][cc]);
        }
        for (int cc = 0; cc < 4; ++cc) {             // ascending slot inside the thread
            const int slot = r0 + tx * 4 + cc;
            if (slot >= B) break;
            const float rn = c_rn[tx * 4 + cc];
            for (int r = 0; r < 4; ++r) {
                const float v = acc[r][cc] * rn;
                if (v > bv[r]) { bv[r] = v; bs[r] = slot; }
            }
        }
    }
    __syncthreads();
    float* pv = smem;                                   // [64][16]
    int* ps = reinterpret_cast<int*>(smem + NT_TS * 16);  // [64][16]
    for (int r = 0; r < 4; ++r) {
        pv[(ty * 4 + r) * 16 + tx] = bv[r];
        ps[(ty * 4 + r) * 16 + tx] = bs[r];
    }
    __syncthreads();
    if (threadIdx.x < NT_TS && e0 + threadIdx.x < Le) {
        float v = -INFINITY;
        int s = 0x7fffffff;
        for (int t = 0; t < 16; ++t) {
            const float tv = pv[threadIdx.x * 16 + t];
            const int tsl = ps[threadIdx.x * 16 + t];
            if (tv > v || (tv == v && tsl < s)) { v = tv; s = tsl; }
        }
        const int e = e0 + threadIdx.x;
        assign[(size_t)h * Le + e] = s;
        sim[(size_t)h * Le + e] = v * rnorm[evicted[e]];
    }
}

}  // namespace lookm

namespace lookm_host {

int launch_nearest_mfma(const void* k, const int32_t* kept, const int32_t* evicted, int H, int L, int budget,
                        const float* rnorm, int32_t* assign, float* sim, void* scratch, hipStream_t st);
size_t nearest_mfma_scratch_bytes(int H, int L, int B);

template <typename T>
static int launch_nearest_t(const T* k, const int32_t* kept, const int32_t* evicted, int H, int L, int d, int budget,
                            float* rnorm, bool rnorm_ready, int32_t* assign, float* sim, void* scratch, hipStream_t st,
                            bool mfma)
{
    const int Le = L - budget;
    if (Le == 0) return LOOKM_OK;
    const LaunchCheck check;
    const size_t rows = (size_t)H * L;
    if (!rnorm_ready)
        hipLaunchKernelGGL(lookm::k_rnorm<T>, dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, st, k, rows, d, rnorm);
    mark(LOOKM_K_RNORM);
    if (mfma) return launch_nearest_mfma(k, kept, evicted, H, L, budget, rnorm, assign, sim, scratch, st);
    size_t lds = (size_t)2 * d * lookm::NT_TS * sizeof(float);
    if (lds < 8192) lds = 8192;
    dim3 grid((Le + lookm::NT_TS - 1) / lookm::NT_TS, H);
    hipLaunchKernelGGL(lookm::k_nearest_generic<T>, grid, dim3(256), lds, st, k, rnorm, kept, evicted, L, d, budget,
                       Le, assign, sim);
    mark(LOOKM_K_NEAREST);
    return check.status();
}

int set_attributes_nearest_generic()
{
    const bool ok = hipFuncSetAttribute((const void*)lookm::k_nearest_generic<float>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024) == hipSuccess &&
                    hipFuncSetAttribute((const void*)lookm::k_nearest_generic<lookm::bf16_t>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024) == hipSuccess;
    return ok ? LOOKM_OK : LOOKM_ERR_DEVICE;
}

size_t nearest_scratch_bytes(int H, int L, int d, lookm_dtype dt, int budget)
{
    return (dt == LOOKM_BF16 && d == 128) ? nearest_mfma_scratch_bytes(H, L, budget) : 0;
}

int launch_nearest(const void* k, const int32_t* kept, const int32_t* evicted, int H, int L, int d, lookm_dtype dt,
                   int budget, float* rnorm, bool rnorm_ready, int32_t* assign, float* sim, void* scratch,
                   hipStream_t st)
{
    if (dt == LOOKM_BF16)
        return launch_nearest_t((const lookm::bf16_t*)k, kept, evicted, H, L, d, budget, rnorm, rnorm_ready, assign,
                                sim, scratch, st, d == 128);
    return launch_nearest_t((const float*)k, kept, evicted, H, L, d, budget, rnorm, rnorm_ready, assign, sim, scratch,
                            st, false);
}

}  // namespace lookm_host
