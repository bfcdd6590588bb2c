// Attention of one new token over a cache (Section 3.1, Eq. 3): out = Softmax(q K^T / sqrt(d)) V, per head,
// over the first S rows of a [H, rows, d] cache - the step that the compressed cache of Eq. 6-7 exists for.
// Bound by HBM: every key row and every value row in use is read exactly once.
//
// The cache rows of a head are cut into `nsplit` contiguous pieces, one workgroup each (a piece is one step of
// the loop below unless the cache is very long), so that a few heads fill the chip and a workgroup pays the
// memory latency once.  Inside a workgroup G = d/8 (rounded up to a power of two) lanes share a row, 16 bytes
// per lane; a lane group takes every NG-th row of the piece, four rows (four key loads and four value loads in
// flight per lane) at a time, and keeps a running (max, sum, weighted value) in base 2 with the softmax scale
// folded in.  The groups of a workgroup, and then the pieces of a head, are merged in a fixed order, so the
// result is bitwise repeatable.
#include "common.h"

#include <mutex>

namespace lookm {

constexpr int DC_THREADS = 256;
constexpr int DC_ROWS = 4;          // rows per lane group and step
constexpr int DC_MAX_SPLIT = 256;
constexpr int DC_MERGE_THREADS = 1024;

// sum over the G lanes of a group (G a power of two <= 32, groups aligned to G lanes)
__device__ __forceinline__ float group_sum(float x, int G)
{
    for (int off = 1; off < G; off <<= 1) x += __shfl_xor(x, off);
    return x;
}

// part: per (head, piece): [0] running max (base-2 logits), [1] sum of weights, [2 .. 2+d) weighted value sum
template <typename T>
__global__ void __launch_bounds__(DC_THREADS)
k_decode_partial(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, int rows, int S, int d,
                 int G, int nsplit, float scale2, float* __restrict__ part)
{
    extern __shared__ float sm[];   // [NG] max, [NG] sum, [NG][G*8] values
    const int h = blockIdx.y, piece = blockIdx.x, tid = threadIdx.x;
    const int NG = DC_THREADS / G, grp = tid / G, c0 = (tid % G) * 8;
    const bool live = c0 < d;       // lanes past the head dim (d not a power of two times 8) carry zeros
    const int per = (S + nsplit - 1) / nsplit;
    const int r_begin = piece * per, r_end = min(S, r_begin + per);
    k += (size_t)h * rows * d;
    v += (size_t)h * rows * d;

    float qv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (live) load8(q + (size_t)h * d + c0, qv);
    float m = -INFINITY, l = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r0 = r_begin + grp * DC_ROWS; r0 < r_end; r0 += NG * DC_ROWS) {
        float kr[DC_ROWS][8], vr[DC_ROWS][8];
#pragma unroll
        for (int j = 0; j < DC_ROWS; ++j) {
            const int r = min(r0 + j, r_end - 1);        // a short last step re-reads the last row with weight 0
            if (live) {
                load8(k + (size_t)r * d + c0, kr[j]);
                load8(v + (size_t)r * d + c0, vr[j]);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) { kr[j][i] = 0.f; vr[j][i] = 0.f; }
            }
        }
        float s[DC_ROWS];
#pragma unroll
        for (int j = 0; j < DC_ROWS; ++j) {
            float dot = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) dot = fmaf(qv[i], kr[j][i], dot);
            s[j] = (r0 + j < r_end) ? group_sum(dot, G) * scale2 : -INFINITY;
        }
        float mn = m;
#pragma unroll
        for (int j = 0; j < DC_ROWS; ++j) mn = fmaxf(mn, s[j]);
        const float keep = __builtin_amdgcn_exp2f(m - mn);   // m = -inf on the first step: 0, and o, l are 0 anyway
        l *= keep;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] *= keep;
#pragma unroll
        for (int j = 0; j < DC_ROWS; ++j) {
            const float p = __builtin_amdgcn_exp2f(s[j] - mn);
            l += p;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = fmaf(p, vr[j][i], o[i]);
        }
        m = mn;
    }

    // merge the lane groups of the workgroup, group 0 first
    float* gm = sm;
    float* gl = sm + NG;
    float* go = sm + 2 * NG;
    const int W8 = G * 8;
    if (tid % G == 0) { gm[grp] = m; gl[grp] = l; }
#pragma unroll
    for (int i = 0; i < 8; ++i) go[grp * W8 + c0 + i] = o[i];
    __syncthreads();
    float* out = part + ((size_t)h * nsplit + piece) * (d + 2);
    float M = -INFINITY;
    for (int g = 0; g < NG; ++g) M = fmaxf(M, gm[g]);
    __syncthreads();
    if (tid < NG) {                                      // every group's weight, once
        const float wg = (gm[tid] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(gm[tid] - M);
        gm[tid] = wg;
        gl[tid] *= wg;
    }
    __syncthreads();
    if (tid < d) {
        float acc = 0.f;
        for (int g = 0; g < NG; ++g) acc = fmaf(go[g * W8 + tid], gm[g], acc);
        out[2 + tid] = acc;
    }
    if (tid == 0) {
        float acc = 0.f;
        for (int g = 0; g < NG; ++g) acc += gl[g];
        out[0] = M;
        out[1] = acc;
    }
}

// Merges the pieces of a head and normalises: one workgroup per head.  The pieces' maxima and sums go through
// LDS (every piece's weight 2^(max - M) is computed once); thread (slice, c) then sums dim c over the pieces
// slice, slice + NSL, ... with independent loads, and the slices are added in order.
template <typename T>
__global__ void __launch_bounds__(DC_MERGE_THREADS)
k_decode_merge(const float* __restrict__ part, int d, int dpad, int nsplit, T* __restrict__ out)
{
    __shared__ float wgt[DC_MAX_SPLIT], sums[DC_MAX_SPLIT];
    __shared__ float red[DC_MERGE_THREADS];
    const int h = blockIdx.x, tid = threadIdx.x;
    const float* p = part + (size_t)h * nsplit * (d + 2);
    if (tid < nsplit) {
        wgt[tid] = p[(size_t)tid * (d + 2)];
        sums[tid] = p[(size_t)tid * (d + 2) + 1];
    }
    __syncthreads();
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, wgt[s]);        // LDS broadcast reads
    __syncthreads();
    if (tid < nsplit) wgt[tid] = (wgt[tid] == -INFINITY) ? 0.f : exp2f(wgt[tid] - M);   // an empty piece: weight 0
    __syncthreads();
    float den = 0.f;
    for (int s = 0; s < nsplit; ++s) den = fmaf(sums[s], wgt[s], den);
    const int NSL = DC_MERGE_THREADS / dpad, slice = tid / dpad, c = tid % dpad;
    float num = 0.f;
    if (c < d) {
        int s = slice;
        for (; s + 3 * NSL < nsplit; s += 4 * NSL) {
            const float a0 = p[(size_t)s * (d + 2) + 2 + c], a1 = p[(size_t)(s + NSL) * (d + 2) + 2 + c];
            const float a2 = p[(size_t)(s + 2 * NSL) * (d + 2) + 2 + c], a3 = p[(size_t)(s + 3 * NSL) * (d + 2) + 2 + c];
            num = fmaf(a0, wgt[s], num);
            num = fmaf(a1, wgt[s + NSL], num);
            num = fmaf(a2, wgt[s + 2 * NSL], num);
            num = fmaf(a3, wgt[s + 3 * NSL], num);
        }
        for (; s < nsplit; s += NSL) num = fmaf(p[(size_t)s * (d + 2) + 2 + c], wgt[s], num);
    }
    red[tid] = num;
    __syncthreads();
    if (slice == 0 && c < d) {
        float tot = 0.f;
        for (int sl = 0; sl < NSL; ++sl) tot += red[sl * dpad + c];
        elem<T>::store(out + (size_t)h * d + c, tot / den);
    }
}

}  // namespace lookm

namespace lookm_host {

// pieces per head: one step of the partial kernel covers 256 / G * DC_ROWS rows; a piece is one or two such steps
// (two when that still leaves four workgroups per compute unit), so that a workgroup pays the memory latency
// once or twice and its closing merge is spread over more rows
static int decode_pieces(int H, int S, int G)
{
    const int step = lookm::DC_THREADS / G * lookm::DC_ROWS;
    int n = (S + step - 1) / step;
    if ((long)H * (n / 2) >= 1024) n = (n + 1) / 2;
    if (n > lookm::DC_MAX_SPLIT) n = lookm::DC_MAX_SPLIT;
    return n < 1 ? 1 : n;
}

size_t decode_scratch_bytes(int H, int d) { return (size_t)H * lookm::DC_MAX_SPLIT * (d + 2) * sizeof(float); }

// bytes of partial results one call really writes and reads (at most decode_scratch_bytes)
size_t decode_partial_bytes(int H, int S, int d)
{
    int G = 1;
    while (G * 8 < d) G <<= 1;
    return (size_t)H * decode_pieces(H, S, G) * (d + 2) * sizeof(float);
}

template <typename T>
static int launch_decode_t(const T* q, const T* k, const T* v, int H, int rows, int S, int d, T* out, float* part,
                           hipStream_t st)
{
    const LaunchCheck check;
    int G = 1;
    while (G * 8 < d) G <<= 1;
    const int NG = lookm::DC_THREADS / G, nsplit = decode_pieces(H, S, G);
    int dpad = 8;
    while (dpad < d) dpad <<= 1;
    const size_t lds = (size_t)(2 * NG + NG * G * 8) * sizeof(float);
    const float scale2 = lookm::kLog2e / sqrtf((float)d);
    hipLaunchKernelGGL(lookm::k_decode_partial<T>, dim3(nsplit, H), dim3(lookm::DC_THREADS), lds, st, q, k, v, rows, S, d,
                       G, nsplit, scale2, part);
    hipLaunchKernelGGL(lookm::k_decode_merge<T>, dim3(H), dim3(lookm::DC_MERGE_THREADS), 0, st, part, d, dpad, nsplit,
                       out);
    return check.status();
}

int launch_decode(const void* q, const void* k, const void* v, int H, int rows, int S, int d, lookm_dtype dt, void* out,
                  float* part, hipStream_t st)
{
    if (dt == LOOKM_BF16)
        return launch_decode_t((const lookm::bf16_t*)q, (const lookm::bf16_t*)k, (const lookm::bf16_t*)v, H, rows, S, d,
                               (lookm::bf16_t*)out, part, st);
    return launch_decode_t((const float*)q, (const float*)k, (const float*)v, H, rows, S, d, (float*)out, part, st);
}

// ---- scratch for callers that may not allocate ---------------------------------------------------------------
// lookm_decode_attention_noalloc keeps the partial results of its two kernels in this array instead of a
// caller's workspace.  Every GPU the library runs on holds its own copy, at its own address, until the process
// ends.  In host code the array's name is only a stand-in for the symbol: the device address is asked for once per
// device (with that device current) and kept; kernels get that pointer as their argument, exactly as they get the
// caller's workspace in lookm_decode_attention.  Nothing in the array has to start at zero: the first kernel writes
// every partial the second one reads.
static __device__ __align__(256) unsigned char scratch[LOOKM_DECODE_NOALLOC_SCRATCH_BYTES];

static std::mutex g_scratch_mutex;
static float* g_scratch_ptr[64];     // per device; null until resolved

int decode_static_scratch_setup()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LOOKM_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] != nullptr) return LOOKM_OK;
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return LOOKM_ERR_DEVICE;
    g_scratch_ptr[dev] = static_cast<float*>(ptr);
    return LOOKM_OK;
}

// the current device's copy of the array, or null when decode_static_scratch_setup has not succeeded on it
float* decode_static_scratch()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    return g_scratch_ptr[dev];
}

}  // namespace lookm_host
