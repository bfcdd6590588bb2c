// Text-prior selection (Section 3.2, Eq. 5-8): one workgroup per head.
//
// Protected positions (text tokens, and the last M positions of any modality) are always
// conserved; the remaining budget k_img = B - |protected| goes to the image positions outside the
// window with the highest accumulated score.  Eq. 5's "add max(A_s) to text scores" only serves to
// rank every text token above every image token, so it is realised as a class, not as a float add.
// The k_img-th largest score is found by an MSB-first radix select over the monotone integer image
// of the float bits (4 passes of 8 bits, LDS histograms); equal scores are resolved towards the
// lower position by an ordered prefix count.  Kept and evicted index lists come out ascending.
#include "common.h"

namespace lookm {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;

// order-preserving map float -> uint32 (larger float <=> larger key); -0 is folded onto +0
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t b = __float_as_uint(s);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// exclusive prefix count of a predicate over the workgroup, in thread order; total returned via ref.
// Uses two barriers; `wtot` is a 16-entry LDS array reserved for this helper.
__device__ __forceinline__ int block_prefix_count(bool pred, int* wtot, int& total)
{
    const uint64_t b = __ballot(pred);
    const int wave = threadIdx.x >> 6;
    if (lane_id() == 0) wtot[wave] = __popcll(b);
    __syncthreads();
    int before = 0, tot = 0;
    for (int w = 0; w < SEL_WAVES; ++w) {
        const int c = wtot[w];
        before += (w < wave) ? c : 0;
        tot += c;
    }
    __syncthreads();
    total = tot;
    return before + mask_rank(b);
}

__global__ void __launch_bounds__(SEL_THREADS)
k_select(const float* __restrict__ scores, const uint8_t* __restrict__ mask, int L, int B, int M,
         int32_t* __restrict__ kept, int32_t* __restrict__ evicted, int32_t* __restrict__ status)
{
    __shared__ int hist[256];
    __shared__ int wtot[SEL_WAVES];
    __shared__ int sh_bin, sh_k;

    const int h = blockIdx.x, tid = threadIdx.x;
    scores += (size_t)h * L;
    kept += (size_t)h * B;
    evicted += (size_t)h * (L - B);
    const int head_len = L - M;   // positions [0, head_len) are outside the recent window

    // |T u R|
    int nprot = 0;
    for (int c0 = 0; c0 < L; c0 += SEL_THREADS) {
        const int j = c0 + tid;
        int tot;
        block_prefix_count(j < L && (mask[j] == 0 || j >= head_len), wtot, tot);
        nprot += tot;
    }
    const int k_img = B - nprot;
    if (k_img < 0) {
        // text + window do not fit: report, and leave in-range (meaningless) index lists behind
        if (tid == 0) *status = LOOKM_ERR_BUDGET_BELOW_PROTECTED;
        for (int r = tid; r < B; r += SEL_THREADS) kept[r] = r;
        for (int e = tid; e < L - B; e += SEL_THREADS) evicted[e] = B + e;
        return;
    }
    if (tid == 0 && h == 0) *status = LOOKM_OK;
    const int n_evictable = L - nprot;
    const bool keep_all = (k_img == n_evictable), keep_none = (k_img == 0);

    // radix select: key of the k_img-th largest evictable score, and how many equal keys to take
    uint32_t thr = 0;
    int need_eq = 0;
    if (!keep_all && !keep_none) {
        uint32_t prefix = 0;
        int kk = k_img;
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int j = tid; j < head_len; j += SEL_THREADS) {
                if (mask[j] == 0) continue;
                const uint32_t key = score_key(scores[j]);
                if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
            }
            __syncthreads();
            if (tid < 64) {
                // wave 0: lane i owns bins 255-4i .. 252-4i (descending); find the bin where the
                // running count from the top first reaches kk
                int c[4], sum = 0;
                for (int i = 0; i < 4; ++i) { c[i] = hist[255 - 4 * tid - i]; sum += c[i]; }
                int incl = sum;
                for (int off = 1; off < 64; off <<= 1) {
                    const int v = __shfl_up(incl, off);
                    if (tid >= off) incl += v;
                }
                int cum = incl - sum;   // count in bins above this lane's bins
                for (int i = 0; i < 4; ++i) {
                    if (cum < kk && cum + c[i] >= kk) { sh_bin = 255 - 4 * tid - i; sh_k = kk - cum; }
                    cum += c[i];
                }
            }
            __syncthreads();
            prefix = (prefix << 8) | (uint32_t)sh_bin;
            kk = sh_k;
            __syncthreads();
        }
        thr = prefix;
        need_eq = kk;
    }

    // ordered compaction
    int kept_base = 0, ev_base = 0, eq_base = 0;
    for (int c0 = 0; c0 < L; c0 += SEL_THREADS) {
        const int j = c0 + tid;
        const bool valid = j < L;
        bool prot = false, evictable = false;
        uint32_t key = 0;
        if (valid) {
            prot = (mask[j] == 0) || (j >= head_len);
            evictable = !prot;
            if (evictable) key = score_key(scores[j]);
        }
        bool keep = prot;
        if (evictable) {
            if (keep_all) keep = true;
            else if (!keep_none) keep = key > thr;
        }
        const bool is_eq = evictable && !keep_all && !keep_none && key == thr;
        int eq_tot;
        const int eq_rank = eq_base + block_prefix_count(is_eq, wtot, eq_tot);
        eq_base += eq_tot;
        if (is_eq && eq_rank < need_eq) keep = true;
        int keep_tot;
        const int kp = block_prefix_count(keep, wtot, keep_tot);
        if (valid) {
            if (keep) kept[kept_base + kp] = j;
            else evicted[ev_base + (tid - kp)] = j;
        }
        kept_base += keep_tot;
        ev_base += min(SEL_THREADS, L - c0) - keep_tot;
    }
}

}  // namespace lookm

namespace lookm_host {

int launch_select(const float* scores, const uint8_t* mask, int H, int L, int budget, int M, int32_t* kept,
                  int32_t* evicted, int32_t* status, hipStream_t st)
{
    hipLaunchKernelGGL(lookm::k_select, dim3(H), dim3(lookm::SEL_THREADS), 0, st, scores, mask, L, budget, M, kept,
                       evicted, status);
    mark(LOOKM_K_SELECT);
    return hip_ok(hipGetLastError());
}

}  // namespace lookm_host
