// Accumulated attention scores (Section 3.2, Eq. 4) - portable fp32-FMA kernels for any supported
// dtype / head_dim.  bf16 inputs with head_dim 128 take the matrix-core kernels in score_mfma.hip.
//
// Two passes over the causal half of Q K^T, neither of which stores it:
//   pass 1 (row tiles):    lse2[i] = log2 sum_{j<=i} 2^(c * q_i.k_j),  c = log2(e)/sqrt(d)
//   pass 2 (column tiles): A_s[j]  = sum_{i>=j} 2^(c * q_i.k_j - lse2[i])
// A workgroup owns a 64-row (pass 1) or 64-column (pass 2) strip and walks the other axis in
// 64-wide tiles staged through LDS in [d][64] layout; a thread owns a 4x4 block of each tile.
// Reductions run in a fixed order, so results are bitwise repeatable.
#include "common.h"

namespace lookm {

constexpr int TS = 64;  // tile side

// stage rows [row0, row0+64) of x ([L, d]) into LDS as xt[c][r]; rows >= L read as zero
template <typename T>
__device__ __forceinline__ void stage_tile(const T* __restrict__ x, int row0, int L, int d, float* xt)
{
    const int chunks = TS * (d / 8);
    for (int ch = threadIdx.x; ch < chunks; ch += blockDim.x) {
        const int r = ch % TS, c0 = (ch / TS) * 8;
        float v[8];
        if (row0 + r < L) load8(x + (size_t)(row0 + r) * d + c0, v);
        else
            for (int i = 0; i < 8; ++i) v[i] = 0.f;
        for (int i = 0; i < 8; ++i) xt[(c0 + i) * TS + r] = v[i];
    }
}

__device__ __forceinline__ void tile_dot(const float* qt, const float* kt, int d, int ty, int tx, float (&acc)[4][4])
{
    for (int r = 0; r < 4; ++r)
        for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
    for (int c = 0; c < d; ++c) {
        const float4 a = *reinterpret_cast<const float4*>(qt + c * TS + ty * 4);
        const float4 b = *reinterpret_cast<const float4*>(kt + c * TS + tx * 4);
        const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
        for (int r = 0; r < 4; ++r)
            for (int cc = 0; cc < 4; ++cc) acc[r][cc] = fmaf(av[r], bv[cc], acc[r][cc]);
    }
}

template <typename T>
__global__ void __launch_bounds__(256) k_score_lse_generic(const T* __restrict__ q, const T* __restrict__ k, int group,
                                                           int L, int R0, int d, float scale2,
                                                           float* __restrict__ lse2)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* qt = smem;
    float* kt = smem + (size_t)d * TS;
    const int nb = (L + TS - 1) / TS;
    const int ib = nb - 1 - (int)blockIdx.x;  // longest strips first
    if ((ib + 1) * TS <= R0) return;          // no query row of this strip counts (observation window)
    const int h = blockIdx.y;                 // query head; `group` consecutive query heads read key head h / group
    q += (size_t)h * L * d;
    k += (size_t)(h / group) * L * d;
    const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;

    stage_tile(q, ib * TS, L, d, qt);
    float m[4], l[4];
    for (int r = 0; r < 4; ++r) { m[r] = -INFINITY; l[r] = 0.f; }
    for (int jb = 0; jb <= ib; ++jb) {
        __syncthreads();
        stage_tile(k, jb * TS, L, d, kt);
        __syncthreads();
        float acc[4][4];
        tile_dot(qt, kt, d, ty, tx, acc);
        for (int r = 0; r < 4; ++r) {
            const int row = ib * TS + ty * 4 + r;
            float tmax = -INFINITY;
            for (int c = 0; c < 4; ++c) {
                const int col = jb * TS + tx * 4 + c;
                acc[r][c] = (col <= row) ? acc[r][c] * scale2 : -INFINITY;
                tmax = fmaxf(tmax, acc[r][c]);
            }
            if (tmax == -INFINITY) continue;
            const float mn = fmaxf(m[r], tmax);
            float s = l[r] * exp2f(m[r] - mn);  // m = -inf gives 0
            for (int c = 0; c < 4; ++c) s += exp2f(acc[r][c] - mn);
            m[r] = mn;
            l[r] = s;
        }
    }
    // combine the 16 column-owners of each row, in thread order
    __syncthreads();
    float* pm = smem;             // [64][16]
    float* pl = smem + TS * 16;   // [64][16]
    for (int r = 0; r < 4; ++r) {
        pm[(ty * 4 + r) * 16 + tx] = m[r];
        pl[(ty * 4 + r) * 16 + tx] = l[r];
    }
    __syncthreads();
    if (threadIdx.x < TS) {
        const int row = ib * TS + threadIdx.x;
        if (row < L) {
            float M = -INFINITY;
            for (int t = 0; t < 16; ++t) M = fmaxf(M, pm[threadIdx.x * 16 + t]);
            float S = 0.f;
            for (int t = 0; t < 16; ++t) {
                const float mt = pm[threadIdx.x * 16 + t];
                if (mt != -INFINITY) S += pl[threadIdx.x * 16 + t] * exp2f(mt - M);
            }
            lse2[(size_t)h * L + row] = M + log2f(S);
        }
    }
}

template <typename T>
__global__ void __launch_bounds__(256) k_score_colsum_generic(const T* __restrict__ q, const T* __restrict__ k, int group,
                                                              int L, int R0, int d, float scale2,
                                                              const float* __restrict__ lse2,
                                                              float lse_scale, float* __restrict__ scores)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* qt = smem;
    float* kt = smem + (size_t)d * TS;
    const int nb = (L + TS - 1) / TS;
    const int jb = blockIdx.x;  // column strip 0 is the longest
    const int h = blockIdx.y;                 // key head: the column sums of its `group` query heads are added up
    q += (size_t)h * group * L * d;
    k += (size_t)h * L * d;
    lse2 += (size_t)h * group * L;
    const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;

    stage_tile(k, jb * TS, L, d, kt);
    float colsum[4] = {0.f, 0.f, 0.f, 0.f};
    for (int m = 0; m < group; ++m, q += (size_t)L * d, lse2 += L)
    for (int ib = max(jb, R0 / TS); ib < nb; ++ib) {   // query rows before R0 do not count
        __syncthreads();
        stage_tile(q, ib * TS, L, d, qt);
        __syncthreads();
        float acc[4][4];
        tile_dot(qt, kt, d, ty, tx, acc);
        for (int r = 0; r < 4; ++r) {
            const int row = ib * TS + ty * 4 + r;
            if (row >= L || row < R0) continue;
            const float lr = lse2[row] * lse_scale;   // base-2 log-sum-exp of the row
            for (int c = 0; c < 4; ++c) {
                const int col = jb * TS + tx * 4 + c;
                if (col <= row) colsum[c] += exp2f(fmaf(acc[r][c], scale2, -lr));
            }
        }
    }
    __syncthreads();
    float* part = smem;  // [16][64]
    for (int c = 0; c < 4; ++c) part[ty * TS + tx * 4 + c] = colsum[c];
    __syncthreads();
    if (threadIdx.x < TS) {
        const int col = jb * TS + threadIdx.x;
        if (col < L) {
            float s = 0.f;
            for (int t = 0; t < 16; ++t) s += part[t * TS + threadIdx.x];
            scores[(size_t)h * L + col] = s;
        }
    }
}

}  // namespace lookm

namespace lookm_host {

int launch_scores_mfma(const void* q, const void* k, int H, int kv_heads, int L, int d, int R0, float* lse,
                       const float* lse_in, float* scores, float* rnorm, float* scratch, const uint8_t* mask, int M,
                       int32_t* lists, hipStream_t st);
size_t scores_mfma_scratch_floats(int H, int L);

template <typename T>
static int launch_scores_generic(const T* q, const T* k, int H, int kv_heads, int L, int d, int R0, float* lse,
                                 const float* lse_in, float* scores, hipStream_t st)
{
    const int group = H / kv_heads;
    const int nb = (L + lookm::TS - 1) / lookm::TS;
    size_t lds = (size_t)2 * d * lookm::TS * sizeof(float);
    if (lds < 8192) lds = 8192;   // the final cross-thread combine reuses the tile buffers
    const float scale2 = lookm::kLog2e / sqrtf((float)d);
    dim3 grid(nb, H), block(256);
    const LaunchCheck check;
    if (!lse_in) {
        hipLaunchKernelGGL(lookm::k_score_lse_generic<T>, grid, block, lds, st, q, k, group, L, R0, d, scale2, lse);
        mark(LOOKM_K_SCORE_LSE);
    }
    // a caller-supplied row log-sum-exp is natural-log: one factor log2(e) brings it to the kernels' base
    hipLaunchKernelGGL(lookm::k_score_colsum_generic<T>, dim3(nb, kv_heads), block, lds, st, q, k, group, L, R0, d, scale2,
                       lse_in ? lse_in : lse, lse_in ? lookm::kLog2e : 1.0f, scores);
    mark(LOOKM_K_SCORE_COLSUM);
    return check.status();
}

template <typename T> static bool score_generic_attributes()
{
    return hipFuncSetAttribute((const void*)lookm::k_score_lse_generic<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               160 * 1024) == hipSuccess &&
           hipFuncSetAttribute((const void*)lookm::k_score_colsum_generic<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               160 * 1024) == hipSuccess;
}

int set_attributes_score_generic()
{
    return (score_generic_attributes<float>() && score_generic_attributes<lookm::bf16_t>()) ? LOOKM_OK : LOOKM_ERR_DEVICE;
}

size_t scores_scratch_floats(int H, int L, int d, lookm_dtype dt)
{
    return (dt == LOOKM_BF16 && d == 128) ? scores_mfma_scratch_floats(H, L) : 0;
}

int launch_scores(const void* q, const void* k, int H, int kv_heads, int L, int d, lookm_dtype dt, int first_row,
                  float* lse, const float* lse_in, float* scores, float* rnorm, float* scratch, const uint8_t* mask, int M,
                  int32_t* lists, hipStream_t st)
{
    const int R0 = first_row;
    if (dt == LOOKM_BF16) {
        if (scores_write_rnorm(d, dt))
            return launch_scores_mfma(q, k, H, kv_heads, L, d, R0, lse, lse_in, scores, rnorm, scratch, mask, M, lists, st);
        return launch_scores_generic((const lookm::bf16_t*)q, (const lookm::bf16_t*)k, H, kv_heads, L, d, R0, lse, lse_in,
                                     scores, st);
    }
    return launch_scores_generic((const float*)q, (const float*)k, H, kv_heads, L, d, R0, lse, lse_in, scores, st);
}

}  // namespace lookm_host
