// Text-prior selection (Section 3.2, Eq. 5-8): one workgroup per head.
//
// Protected positions (text tokens, and the last M positions of any modality) are always
// conserved; the remaining budget k_img = B - |protected| goes to the image positions outside the
// window with the highest accumulated score.  Eq. 5's "add max(A_s) to text scores" only serves to
// rank every text token above every image token, so it is realised as a class, not as a float add.
// The k_img-th largest score is found by an MSB-first radix select over the monotone integer image
// of the float bits (digits of 12, 12 and 8 bits, LDS histograms); equal scores are resolved towards the
// lower position by an ordered prefix count.  Kept and evicted index lists come out ascending.
// Supports L <= 32 * 1024 (32 positions per thread).
#include "common.h"

namespace lookm {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_BINS = 4096;    // 12-bit digits
constexpr int SEL_CAND = 4096;    // capacity of the LDS candidate list

// order-preserving map float -> uint32 (larger float <=> larger key); -0 is folded onto +0
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t b = __float_as_uint(s);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// exclusive prefix sum over the workgroup's 16 waves of one wave-uniform int, and the total.  Two barriers;
// `wtot` is a 16-entry LDS array reserved for this helper.
__device__ __forceinline__ int wave_scan_excl(int wave_value, int* wtot, int& total)
{
    const int wave = threadIdx.x >> 6;
    if (lane_id() == 0) wtot[wave] = wave_value;
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) {
        const int c = wtot[w];
        before += (w < wave) ? c : 0;
        tot += c;
    }
    __syncthreads();
    total = tot;
    return before;
}

// rnorm[r] = 1 / ||x[r, :]|| (0 for a zero row) over all rows, by workgroup b of nb: one 8-lane group per row,
// rows of a wave adjacent in memory.  NCH = ceil(d / 64) 16-byte pieces per lane and row; a group keeps UNR
// rows (eight or so loads per lane) in flight, all issued before the first use.
template <typename T, int NCH>
__device__ __forceinline__ void rnorm_stream(const T* __restrict__ x, size_t rows, int d, int b, int nb,
                                             float* __restrict__ rnorm)
{
    constexpr int UNR = (NCH == 1) ? 8 : (NCH == 2) ? 4 : 2;
    const int sub = threadIdx.x & 7;
    const size_t stride = (size_t)nb * (SEL_THREADS / 8);
    for (size_t r0 = (size_t)b * (SEL_THREADS / 8) + (threadIdx.x >> 3); r0 < rows; r0 += UNR * stride) {
        float v[UNR][NCH][8];
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int t = 0; t < NCH; ++t) {
                const size_t r = r0 + u * stride;
                const int c0 = sub * 8 + t * 64;
                if (r < rows && c0 < d) load8(x + r * d + c0, v[u][t]);
                else
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[u][t][i] = 0.f;
            }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            float acc = 0.f;
#pragma unroll
            for (int t = 0; t < NCH; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc = fmaf(v[u][t][i], v[u][t][i], acc);
            acc += __shfl_xor(acc, 1);
            acc += __shfl_xor(acc, 2);
            acc += __shfl_xor(acc, 4);
            const size_t r = r0 + u * stride;
            if (r < rows && sub == 0) rnorm[r] = (acc > 0.f) ? 1.0f / sqrtf(acc) : 0.f;
        }
    }
}

template <typename T>
__device__ __forceinline__ void rnorm_blocks(const T* __restrict__ x, size_t rows, int d, int b, int nb,
                                             float* __restrict__ rnorm)
{
    switch ((d + 63) / 64) {
        case 1: rnorm_stream<T, 1>(x, rows, d, b, nb, rnorm); break;
        case 2: rnorm_stream<T, 2>(x, rows, d, b, nb, rnorm); break;
        case 3: rnorm_stream<T, 3>(x, rows, d, b, nb, rnorm); break;
        default: rnorm_stream<T, 4>(x, rows, d, b, nb, rnorm); break;
    }
}

// Wave w owns the contiguous segment [w*64*IPT, (w+1)*64*IPT) of positions; inside it lane l holds
// positions seg + i*64 + l, i < IPT, so global reads and writes are coalesced.  Keys and classes are
// read once and stay in registers for the radix passes and the compaction; ordered counts are ballots
// inside the wave plus one 16-entry scan across waves.
//
// Workgroups past the first H do unrelated work that only needs the keys: the inverse row norms for the cosine
// matching (Eq. 9).  The selection occupies one compute unit per head and is bound by latency, so the norms -
// a plain streaming read of K - run beside it on the rest of the chip instead of in a launch of their own.
template <int IPT>
__global__ void __launch_bounds__(SEL_THREADS)
k_select(const float* __restrict__ scores, const uint8_t* __restrict__ mask, int H, int L, int B, int M,
         int32_t* __restrict__ kept, int32_t* __restrict__ evicted, int32_t* __restrict__ status,
         const void* __restrict__ k_rows, int d, int k_is_bf16, float* __restrict__ rnorm)
{
    if ((int)blockIdx.x >= H) {
        const size_t rows = (size_t)H * L;
        const int b = (int)blockIdx.x - H, nb = (int)gridDim.x - H;
        if (k_is_bf16) rnorm_blocks(static_cast<const bf16_t*>(k_rows), rows, d, b, nb, rnorm);
        else rnorm_blocks(static_cast<const float*>(k_rows), rows, d, b, nb, rnorm);
        return;
    }
    __shared__ int hist[SEL_BINS];
    __shared__ uint32_t cand[SEL_CAND];     // keys that share the threshold's top 12 bits
    __shared__ int wtot[SEL_WAVES];
    __shared__ uint32_t wmin[SEL_WAVES], wmax[SEL_WAVES];
    __shared__ int sh_bin, sh_k, sh_ncand;

    const int h = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    scores += (size_t)h * L;
    kept += (size_t)h * B;
    evicted += (size_t)h * (L - B);
    const int head_len = L - M;   // positions [0, head_len) are outside the recent window
    const int seg = wave * 64 * IPT;

    // every load is issued before the first use, so the whole read costs one memory latency
    uint32_t key[IPT];
    uint8_t img[IPT];
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int j = seg + i * 64 + lane;
        const int jc = min(j, L - 1);   // unconditional loads of a clamped index: nothing waits on a branch
        key[i] = __float_as_uint(scores[jc]);
        img[i] = mask[jc];
    }
    uint32_t prot_m = 0, evic_m = 0;   // bit i: position seg + i*64 + lane is protected / evictable
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    int nprot_wave = 0;
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int j = seg + i * 64 + lane;
        bool prot = false;
        if (j < L) {
            prot = (img[i] == 0 || j >= head_len);
            if (prot) prot_m |= 1u << i;
            else {
                evic_m |= 1u << i;
                key[i] = score_key(__uint_as_float(key[i]));
                kmin = min(kmin, key[i]);
                kmax = max(kmax, key[i]);
            }
        }
        nprot_wave += __popcll(__ballot(prot));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
    }
    if (lane == 0) { wmin[wave] = kmin; wmax[wave] = kmax; }

    int nprot;   // |T u R|
    wave_scan_excl(nprot_wave, wtot, nprot);
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) { kmin = min(kmin, wmin[w]); kmax = max(kmax, wmax[w]); }
    // Scores of a head crowd into a few binades, so the raw top bits would send most keys to a handful of
    // histogram bins (LDS atomics on one address serialise).  Keys are re-based to the head's own range
    // [kmin, kmax] and shifted up to use all 32 bits: order and equality are unchanged, the digits spread.
    {
        const uint32_t range = (kmax >= kmin) ? kmax - kmin : 0u;
        const int lz = range ? __clz(range) : 0;
#pragma unroll
        for (int i = 0; i < IPT; ++i) key[i] = (key[i] - kmin) << lz;   // only evictable entries are used below
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

    // Radix select, MSB first in digits of 12, 12 and 8 bits: key of the k_img-th largest evictable score
    // and how many keys equal to it to take.  After the first digit the few surviving keys are copied to
    // an LDS list, so the later digits cost one pass over that list instead of one over all positions
    // (if more than SEL_CAND keys share their top 12 bits, the later digits re-read the registers).
    uint32_t thr = 0;
    int need_eq = 0;
    if (!keep_all && !keep_none) {
        int kk = k_img;
        // finds the bin (counting from the top) where the running count first reaches kk; every thread
        // owns SEL_BINS / SEL_THREADS consecutive bins in descending order
        auto find_bin = [&](int nbins) {
            const int per = (nbins + SEL_THREADS - 1) / SEL_THREADS;   // 4 or 1
            int c[4] = {0, 0, 0, 0}, sum = 0;
            for (int i = 0; i < per; ++i) {
                const int bin = nbins - 1 - (tid * per + i);
                c[i] = (bin >= 0) ? hist[bin] : 0;
                sum += c[i];
            }
            int incl = sum;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int v = __shfl_up(incl, off);
                if (lane >= off) incl += v;
            }
            int tot;
            int cum = wave_scan_excl(__shfl(incl, 63), wtot, tot) + incl - sum;   // count in bins above mine
            for (int i = 0; i < per; ++i) {
                if (cum < kk && cum + c[i] >= kk) { sh_bin = nbins - 1 - (tid * per + i); sh_k = kk - cum; }
                cum += c[i];
            }
            __syncthreads();
            kk = sh_k;
            return (uint32_t)sh_bin;
        };

        for (int i = tid; i < SEL_BINS; i += SEL_THREADS) hist[i] = 0;
        if (tid == 0) sh_ncand = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < IPT; ++i)
            if ((evic_m >> i) & 1u) atomicAdd(&hist[key[i] >> 20], 1);
        __syncthreads();
        const uint32_t d0 = find_bin(SEL_BINS);
        const int n_cand = hist[d0];
        const bool listed = n_cand <= SEL_CAND;
        __syncthreads();
        for (int i = tid; i < SEL_BINS; i += SEL_THREADS) hist[i] = 0;
        if (listed) {
#pragma unroll
            for (int i = 0; i < IPT; ++i)
                if (((evic_m >> i) & 1u) && (key[i] >> 20) == d0) cand[atomicAdd(&sh_ncand, 1)] = key[i];
        }
        __syncthreads();
        if (listed) {
            for (int c = tid; c < n_cand; c += SEL_THREADS) atomicAdd(&hist[(cand[c] >> 8) & 0xfffu], 1);
        } else {
#pragma unroll
            for (int i = 0; i < IPT; ++i)
                if (((evic_m >> i) & 1u) && (key[i] >> 20) == d0) atomicAdd(&hist[(key[i] >> 8) & 0xfffu], 1);
        }
        __syncthreads();
        const uint32_t d1 = find_bin(SEL_BINS);
        const uint32_t top24 = (d0 << 12) | d1;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        if (listed) {
            for (int c = tid; c < n_cand; c += SEL_THREADS)
                if ((cand[c] >> 8) == top24) atomicAdd(&hist[cand[c] & 0xffu], 1);
        } else {
#pragma unroll
            for (int i = 0; i < IPT; ++i)
                if (((evic_m >> i) & 1u) && (key[i] >> 8) == top24) atomicAdd(&hist[key[i] & 0xffu], 1);
        }
        __syncthreads();
        const uint32_t d2 = find_bin(256);
        thr = (top24 << 8) | d2;
        need_eq = kk;
    }

    // ordered compaction.  First the equal keys: those at the lowest positions fill what is left.
    uint32_t keep_m = prot_m, eq_m = 0;
    int eq_wave = 0;
    if (keep_all) keep_m |= evic_m;
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        bool eq = false;
        if (!keep_all && !keep_none && ((evic_m >> i) & 1u)) {
            if (key[i] > thr) keep_m |= 1u << i;
            else if (key[i] == thr) { eq = true; eq_m |= 1u << i; }
        }
        eq_wave += __popcll(__ballot(eq));
    }
    int eq_tot;
    int eq_run = wave_scan_excl(eq_wave, wtot, eq_tot);   // equal keys in lower waves
    int keep_wave = 0;
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const bool eq = (eq_m >> i) & 1u;
        const uint64_t eb = __ballot(eq);
        if (eq && eq_run + mask_rank(eb) < need_eq) keep_m |= 1u << i;
        eq_run += __popcll(eb);
        keep_wave += __popcll(__ballot((keep_m >> i) & 1u));
    }
    int keep_tot;
    int kp = wave_scan_excl(keep_wave, wtot, keep_tot);   // kept positions in lower waves
    int ep = min(seg, L) - kp;                             // evicted positions in lower waves
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int j = seg + i * 64 + lane;
        const bool valid = j < L, keep = (keep_m >> i) & 1u;
        const uint64_t kb = __ballot(valid && keep), vb = __ballot(valid);
        if (valid) {
            const int r = mask_rank(kb);
            if (keep) kept[kp + r] = j;
            else evicted[ep + lane - r] = j;               // valid lanes are a prefix of the wave
        }
        kp += __popcll(kb);
        ep += __popcll(vb) - __popcll(kb);
    }
}

}  // namespace lookm

namespace lookm_host {

int launch_select(const float* scores, const uint8_t* mask, int H, int L, int budget, int M, int32_t* kept,
                  int32_t* evicted, int32_t* status, const void* k_rows, int d, lookm_dtype dt, float* rnorm,
                  hipStream_t st)
{
    const int per_thread = (L + lookm::SEL_THREADS - 1) / lookm::SEL_THREADS;
    const bool norms = k_rows != nullptr && rnorm != nullptr;
    // the norm workgroups stream over all rows in a grid-stride loop: one per compute unit the selection leaves free
    const size_t rows_per_block = lookm::SEL_THREADS / 8;
    const size_t want = ((size_t)H * L + rows_per_block - 1) / rows_per_block;
    const size_t free_cus = H < 192 ? 256 - H : 64;
    const unsigned extra = norms ? (unsigned)(want < free_cus ? want : free_cus) : 0u;
    dim3 grid((unsigned)H + extra), block(lookm::SEL_THREADS);
    const int bf = (dt == LOOKM_BF16) ? 1 : 0;
#define LOOKM_LAUNCH_SELECT(IPT)                                                                                  \
    hipLaunchKernelGGL(lookm::k_select<IPT>, grid, block, 0, st, scores, mask, H, L, budget, M, kept, evicted, status, \
                       k_rows, d, bf, rnorm)
    if (per_thread <= 4) LOOKM_LAUNCH_SELECT(4);
    else if (per_thread <= 8) LOOKM_LAUNCH_SELECT(8);
    else if (per_thread <= 16) LOOKM_LAUNCH_SELECT(16);
    else if (per_thread <= 32) LOOKM_LAUNCH_SELECT(32);
    else return LOOKM_ERR_UNSUPPORTED;
#undef LOOKM_LAUNCH_SELECT
    mark(LOOKM_K_SELECT);
    return hip_ok(hipGetLastError());
}

}  // namespace lookm_host
