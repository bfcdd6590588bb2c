// KV-pair merging and compaction (Section 3.3, Eq. 10-12; layout of Eq. 6-7).
//
// k_bucket groups the evicted tokens of a head by the conserved slot they were matched to (the
// paper's one-to-many similarity sets k_sim), as a stable counting sort so that every set lists its
// members' positions (with their matching cosines) in ascending position.  k_merge then GATHERS: one lane group per conserved slot reads its
// own row and its members' rows and writes one compact output row - no scatter, no float atomics,
// fixed summation order, coalesced 16-byte accesses along the head dimension.  Keys and values use
// the same sets and (for weighted merging) the same cosine weights.
#include "common.h"

namespace lookm {

constexpr int BK_THREADS = 1024;

// lanes of the wave whose (valid) key equals this lane's key
__device__ __forceinline__ uint64_t match_key(int key, bool valid, int nbits)
{
    uint64_t peers = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (key >> b) & 1;
        const uint64_t m = __ballot(bit && valid);
        peers &= bit ? m : ~m;
    }
    return peers;
}

// One workgroup per head.  cnt is [W][B] in LDS: wave w < W owns a contiguous segment of the evicted
// list; counts per (wave, slot) are turned into start offsets in slot-major, wave-minor order, which
// makes the fill stable across waves; inside a wave, 64-entry chunks are taken in order and lanes
// with equal slots are ranked by lane.
__global__ void __launch_bounds__(BK_THREADS)
k_bucket(const int32_t* __restrict__ assign, const int32_t* __restrict__ evicted, const float* __restrict__ sim,
         int Le, int B, int W, int nbits, int32_t* __restrict__ offsets, int32_t* __restrict__ member_pos,
         float* __restrict__ member_w)
{
    extern __shared__ int cnt[];   // [W][B]
    __shared__ int wsum[BK_THREADS / 64];
    const int h = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    assign += (size_t)h * Le;
    evicted += (size_t)h * Le;
    sim += (size_t)h * Le;
    offsets += (size_t)h * (B + 1);
    member_pos += (size_t)h * Le;
    member_w += (size_t)h * Le;

    for (int i = tid; i < W * B; i += BK_THREADS) cnt[i] = 0;
    __syncthreads();
    const int seg = (((Le + W - 1) / W) + 63) / 64 * 64;
    const int seg_lo = wave * seg, seg_hi = min(Le, seg_lo + seg);
    if (wave < W)
        for (int e = seg_lo + lane; e < seg_hi; e += 64) {
            const int a = min(max(assign[e], 0), B - 1);
            atomicAdd(&cnt[wave * B + a], 1);
        }
    __syncthreads();

    const int per = (B + BK_THREADS - 1) / BK_THREADS;
    const int a0 = min(B, tid * per), a1 = min(B, a0 + per);
    int local = 0;
    for (int a = a0; a < a1; ++a)
        for (int w = 0; w < W; ++w) local += cnt[w * B + a];
    int incl = local;
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int run = incl - local;
    for (int w = 0; w < wave; ++w) run += wsum[w];
    for (int a = a0; a < a1; ++a) {
        offsets[a] = run;
        for (int w = 0; w < W; ++w) {
            const int c = cnt[w * B + a];
            cnt[w * B + a] = run;
            run += c;
        }
    }
    if (tid == 0) offsets[B] = Le;
    __syncthreads();

    if (wave < W)
        for (int c0 = seg_lo; c0 < seg_hi; c0 += 64) {
            const int e = c0 + lane;
            const bool valid = e < seg_hi;
            const int a = valid ? min(max(assign[e], 0), B - 1) : 0;
            const uint64_t peers = match_key(a, valid, nbits);
            int base = 0;
            if (valid) {
                base = cnt[wave * B + a];
                const int dst = base + mask_rank(peers);
                member_pos[dst] = evicted[e];      // the set lists positions (ascending) and their cosines
                member_w[dst] = sim[e];
            }
            __builtin_amdgcn_wave_barrier();
            if (valid && (peers >> lane) == 1ull) cnt[wave * B + a] = base + __popcll(peers);   // highest peer updates
            __builtin_amdgcn_wave_barrier();
        }
}

// G lanes per conserved slot, each lane 8 consecutive head dims.  A slot's members are fetched four at a
// time (positions and weights are plain sequential reads, the four row loads are independent), so the
// gather keeps several loads in flight per lane group instead of one dependent chain per member.
template <typename T>
__global__ void __launch_bounds__(256)
k_merge(const T* __restrict__ k, const T* __restrict__ v, const int32_t* __restrict__ kept,
        const int32_t* __restrict__ offsets, const int32_t* __restrict__ member_pos,
        const float* __restrict__ member_w, int L, int d, int B, int Le, int mode, int G, T* __restrict__ k_out,
        T* __restrict__ v_out)
{
    const int h = blockIdx.y;
    const int slot = blockIdx.x * (256 / G) + (int)threadIdx.x / G;
    const int c0 = ((int)threadIdx.x % G) * 8;
    if (slot >= B || c0 >= d) return;
    const T* x = (blockIdx.z ? v : k) + (size_t)h * L * d + c0;
    T* out = (blockIdx.z ? v_out : k_out) + ((size_t)h * B + slot) * d + c0;
    kept += (size_t)h * B;

    float xc[8];
    load8(x + (size_t)kept[slot] * d, xc);
    if (mode != LOOKM_MERGE_NONE) {
        member_pos += (size_t)h * Le;
        member_w += (size_t)h * Le;
        offsets += (size_t)h * (B + 1);
        const int o0 = offsets[slot], o1 = offsets[slot + 1];
        const int n = o1 - o0;                       // L_sim: size of this slot's similarity set
        if (n > 0) {
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            const bool weighted = (mode == LOOKM_MERGE_WEIGHTED);
            int t = o0;
            for (; t + 4 <= o1; t += 4) {            // ascending position
                int p[4];
                float w[4], xe[4][8];
#pragma unroll
                for (int j = 0; j < 4; ++j) { p[j] = member_pos[t + j]; w[j] = weighted ? member_w[t + j] : 1.0f; }
#pragma unroll
                for (int j = 0; j < 4; ++j) load8(x + (size_t)p[j] * d, xe[j]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[i] = weighted ? fmaf(xe[j][i], w[j], acc[i]) : acc[i] + xe[j][i];
            }
            for (; t < o1; ++t) {
                float xe[8];
                const float w = weighted ? member_w[t] : 1.0f;
                load8(x + (size_t)member_pos[t] * d, xe);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = weighted ? fmaf(xe[i], w, acc[i]) : acc[i] + xe[i];
            }
            const float inv = 1.0f / (float)(n + 1);
            if (mode == LOOKM_MERGE_PIVOTAL)         // Eq. 11: (x_c + 1/2 sum (x_e + x_c)) / (n + 1)
#pragma unroll
                for (int i = 0; i < 8; ++i) xc[i] = (xc[i] + 0.5f * fmaf((float)n, xc[i], acc[i])) * inv;
            else                                     // Eq. 10 / Eq. 12: (x_c + sum w_e x_e) / (n + 1)
#pragma unroll
                for (int i = 0; i < 8; ++i) xc[i] = (xc[i] + acc[i]) * inv;
        }
    }
    store8(out, xc);
}

}  // namespace lookm

namespace lookm_host {

// number of waves of k_bucket that get their own counter row, given ~150 KB of LDS
static int bucket_waves(int B)
{
    int w = (150 * 1024) / (4 * B);
    return w > 16 ? 16 : (w < 1 ? 1 : w);
}

template <typename T>
static void launch_merge_t(const T* k, const T* v, const int32_t* kept, const int32_t* offsets,
                           const int32_t* member_pos, const float* member_w, int H, int L, int d, int B, int mode,
                           T* k_out, T* v_out, hipStream_t st)
{
    int G = 1;
    while (G * 8 < d) G <<= 1;
    const int spb = 256 / G;
    dim3 grid((B + spb - 1) / spb, H, 2);
    hipLaunchKernelGGL(lookm::k_merge<T>, grid, dim3(256), 0, st, k, v, kept, offsets, member_pos, member_w, L, d, B,
                       L - B, mode, G, k_out, v_out);
}

int launch_merge(const void* k, const void* v, const int32_t* kept, const int32_t* evicted, const int32_t* assign,
                 const float* sim, int H, int L, int d, lookm_dtype dt, int budget, int mode, int32_t* offsets,
                 int32_t* member_pos, float* member_w, void* k_out, void* v_out, hipStream_t st)
{
    const int B = budget, Le = L - B;
    if (B == 0) return LOOKM_OK;
    if (Le == 0) mode = LOOKM_MERGE_NONE;
    if (mode != LOOKM_MERGE_NONE) {
        const int W = bucket_waves(B);
        int nbits = 1;
        while ((1 << nbits) < B) ++nbits;
        static bool attr_done = false;
        if (!attr_done) {
            if (hipFuncSetAttribute((const void*)lookm::k_bucket, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    152 * 1024) != hipSuccess)
                return LOOKM_ERR_DEVICE;
            attr_done = true;
        }
        hipLaunchKernelGGL(lookm::k_bucket, dim3(H), dim3(lookm::BK_THREADS), (size_t)W * B * sizeof(int), st, assign,
                           evicted, sim, Le, B, W, nbits, offsets, member_pos, member_w);
        mark(LOOKM_K_BUCKET);
    }
    if (dt == LOOKM_BF16)
        launch_merge_t((const lookm::bf16_t*)k, (const lookm::bf16_t*)v, kept, offsets, member_pos, member_w, H, L, d,
                       B, mode, (lookm::bf16_t*)k_out, (lookm::bf16_t*)v_out, st);
    else
        launch_merge_t((const float*)k, (const float*)v, kept, offsets, member_pos, member_w, H, L, d, B, mode,
                       (float*)k_out, (float*)v_out, st);
    mark(LOOKM_K_MERGE);
    return hip_ok(hipGetLastError());
}

}  // namespace lookm_host
