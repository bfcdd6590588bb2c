// Text-prior selection (Section 3.2, Eq. 5-8): one workgroup per head.
//
// Protected positions (text tokens, and the last M positions of any modality) are always
// conserved; the remaining budget k_img = B - |protected| goes to the image positions outside the
// window with the highest accumulated score.  Eq. 5's "add max(A_s) to text scores" only serves to
// rank every text token above every image token, so it is realised as a class, not as a float add.
// The k_img-th largest score is found by an MSB-first radix select over the monotone integer image
// of the float bits, re-based to the head's own range (a 12-bit LDS histogram; the few keys that share
// the threshold's digit are then ranked against each other directly, or, if they are many, by two more
// digits of 12 and 8 bits); equal scores are resolved towards the lower position by an ordered prefix
// count.  Kept and evicted index lists come out ascending.
// Supports L <= 32 * 1024 (32 positions per thread).
#include "common.h"

namespace lookm {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_BINS = 4096;    // 12-bit digits
constexpr int SEL_CAND = 4096;    // capacity of the LDS candidate list
constexpr int SEL_FAST = 128;     // up to this many candidates are ranked all against all

// order-preserving map float -> uint32 (larger float <=> larger key); -0 is folded onto +0
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t b = __float_as_uint(s);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// exclusive prefix sum over the workgroup's 16 waves of one wave-uniform int, and the total.  One barrier;
// `wtot` is a 16-entry LDS array that nothing else touches (every scan of the kernel has its own).
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
    total = tot;
    return before;
}

// Wave w owns the contiguous segment [w*64*IPT, (w+1)*64*IPT) of positions; inside it lane l holds
// positions seg + i*64 + l, i < IPT, so global reads and writes are coalesced.  Keys and classes are
// read once and stay in registers for the radix passes and the compaction; ordered counts are ballots
// inside the wave plus one 16-entry scan across waves.
template <int IPT>
__global__ void __launch_bounds__(SEL_THREADS)
k_select(const float* __restrict__ scores, const uint8_t* __restrict__ mask, int L, int B, int M, int rule,
         int32_t* __restrict__ kept, int32_t* __restrict__ evicted, int32_t* __restrict__ status)
{
    __shared__ int hist[SEL_BINS];
    __shared__ uint32_t cand[SEL_CAND];     // keys that share the threshold's top 12 bits
    __shared__ int wtot[8][SEL_WAVES];      // one row per workgroup-wide scan
    __shared__ uint32_t wmin[SEL_WAVES], wmax[SEL_WAVES], wtmin[SEL_WAVES], wtmax[SEL_WAVES];
    __shared__ int sh_bin, sh_k, sh_ncand;
    __shared__ uint32_t sh_thr;

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
        const int jc = min(seg + i * 64 + lane, L - 1);   // unconditional loads of a clamped index: nothing waits on a branch
        key[i] = __float_as_uint(scores[jc]);
        img[i] = mask[jc];
    }
    for (int i = tid; i < SEL_BINS; i += SEL_THREADS) hist[i] = 0;
    if (tid == 0) sh_ncand = 0;

    // bit i of each mask: position seg + i*64 + lane is in the recent window / a text token before it / an image
    // token before it
    uint32_t win_m = 0, text_m = 0, img_m = 0;
    uint32_t kmin = 0xffffffffu, kmax = 0u;       // over the image tokens before the window
    uint32_t tmin = 0xffffffffu, tmax = 0u;       // over the text tokens before the window (literal rule only)
    int ntext_wave = 0;
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int j = seg + i * 64 + lane;
        bool text = false;
        if (j < L) {
            key[i] = score_key(__uint_as_float(key[i]));
            if (j >= head_len) win_m |= 1u << i;
            else if (img[i] == 0) {
                text = true;
                text_m |= 1u << i;
                if (rule == LOOKM_SELECT_LITERAL) { tmin = min(tmin, key[i]); tmax = max(tmax, key[i]); }
            } else {
                img_m |= 1u << i;
                kmin = min(kmin, key[i]);
                kmax = max(kmax, key[i]);
            }
        }
        ntext_wave += __popcll(__ballot(text));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
    }
    if (rule == LOOKM_SELECT_LITERAL) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            tmin = min(tmin, (uint32_t)__shfl_xor((int)tmin, off));
            tmax = max(tmax, (uint32_t)__shfl_xor((int)tmax, off));
        }
    }
    if (lane == 0) { wmin[wave] = kmin; wmax[wave] = kmax; wtmin[wave] = tmin; wtmax[wave] = tmax; }

    int ntext;   // text tokens before the window; |T u R| = ntext + M
    wave_scan_excl(ntext_wave, wtot[0], ntext);
    const int nprot = ntext + M;
    // Eq. 8 has N = B - M places before the window.  If they hold every text token, text and window are sure and
    // the image tokens compete for the rest; if not, the default rule reports an error, while the literal rule
    // lets the (boosted, hence always higher-ranked) text tokens compete for the N places and conserves no image.
    const bool text_competes = (B < nprot) && (rule == LOOKM_SELECT_LITERAL);
    if (B < nprot && !text_competes) {
        // text + window do not fit: report, and leave in-range (meaningless) index lists behind
        if (tid == 0) *status = LOOKM_ERR_BUDGET_BELOW_PROTECTED;
        for (int r = tid; r < B; r += SEL_THREADS) kept[r] = r;
        for (int e = tid; e < L - B; e += SEL_THREADS) evicted[e] = B + e;
        return;
    }
    if (tid == 0 && h == 0) *status = LOOKM_OK;
    const uint32_t prot_m = text_competes ? win_m : (win_m | text_m);   // conserved whatever the scores
    const uint32_t evic_m = text_competes ? text_m : img_m;             // compete by score
    const int k_img = text_competes ? B - M : B - nprot;                // places they compete for
    const int n_evictable = text_competes ? ntext : L - nprot;
    kmin = 0xffffffffu;
    kmax = 0u;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) {
        kmin = min(kmin, text_competes ? wtmin[w] : wmin[w]);
        kmax = max(kmax, text_competes ? wtmax[w] : wmax[w]);
    }
    // Scores of a head crowd into a few binades, so the raw top bits would send most keys to a handful of
    // histogram bins.  Keys are re-based to the competing tokens' own range [kmin, kmax] and shifted up to use
    // all 32 bits: order and equality are unchanged, the first digit spreads over the bins, and few keys are
    // left to tell apart after it.
    {
        const uint32_t range = (kmax >= kmin) ? kmax - kmin : 0u;
        const int lz = range ? __clz(range) : 0;
#pragma unroll
        for (int i = 0; i < IPT; ++i) key[i] = (key[i] - kmin) << lz;   // only competing entries are used below
    }
    const bool keep_all = (k_img == n_evictable), keep_none = (k_img == 0);

    // key of the k_img-th largest evictable score, and how many keys equal to it to take
    uint32_t thr = 0;
    int need_eq = 0;
    if (!keep_all && !keep_none) {
        int kk = k_img;
        int scan_row = 1;
        // finds the bin (counting from the top) where the running count first reaches kk; every thread
        // owns SEL_BINS / SEL_THREADS consecutive bins in descending order.  Two barriers.
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
            int cum = wave_scan_excl(__shfl(incl, 63), wtot[scan_row++], tot) + incl - sum;   // count in bins above mine
            for (int i = 0; i < per; ++i) {
                if (cum < kk && cum + c[i] >= kk) { sh_bin = nbins - 1 - (tid * per + i); sh_k = kk - cum; }
                cum += c[i];
            }
            __syncthreads();
            kk = sh_k;
            return (uint32_t)sh_bin;
        };

#pragma unroll
        for (int i = 0; i < IPT; ++i)
            if ((evic_m >> i) & 1u) atomicAdd(&hist[key[i] >> 20], 1);   // hist was cleared before the first barrier
        __syncthreads();
        const uint32_t d0 = find_bin(SEL_BINS);
        const int n_cand = hist[d0];
        const bool listed = n_cand <= SEL_CAND;
        if (listed) {
#pragma unroll
            for (int i = 0; i < IPT; ++i)
                if (((evic_m >> i) & 1u) && (key[i] >> 20) == d0) cand[atomicAdd(&sh_ncand, 1)] = key[i];
        }
        __syncthreads();
        if (n_cand <= SEL_FAST) {
            // few candidates: each is compared with all the others (the list is read as LDS broadcasts)
            if (tid < n_cand) {
                const uint32_t mine = cand[tid];
                int above = 0, same = 0;
                for (int c = 0; c < n_cand; ++c) {
                    const uint32_t x = cand[c];
                    above += (x > mine) ? 1 : 0;
                    same += (x == mine) ? 1 : 0;
                }
                if (above < kk && kk <= above + same) { sh_thr = mine; sh_k = kk - above; }
            }
            __syncthreads();
            thr = sh_thr;
            need_eq = sh_k;
        } else {
            // many keys share the first digit: two more digits of 12 and 8 bits, over the LDS list, or over the
            // registers when even the list is too small
            for (int i = tid; i < SEL_BINS; i += SEL_THREADS) hist[i] = 0;
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
    }

    // ordered compaction.  Keys above the threshold and protected positions are conserved; of the keys equal
    // to it, those at the lowest positions fill what is left.  One scan carries both counts.
    uint32_t keep_m = prot_m, eq_m = 0;
    int sure_wave = 0, eq_wave = 0;
    if (keep_all) keep_m |= evic_m;
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        bool eq = false;
        if (!keep_all && !keep_none && ((evic_m >> i) & 1u)) {
            if (key[i] > thr) keep_m |= 1u << i;
            else if (key[i] == thr) { eq = true; eq_m |= 1u << i; }
        }
        eq_wave += __popcll(__ballot(eq));
        sure_wave += __popcll(__ballot((keep_m >> i) & 1u));
    }
    if (lane == 0) { wtot[6][wave] = sure_wave; wtot[7][wave] = eq_wave; }
    __syncthreads();
    int sure_before = 0, eq_run = 0;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) {
        sure_before += (w < wave) ? wtot[6][w] : 0;
        eq_run += (w < wave) ? wtot[7][w] : 0;
    }
    int kp = sure_before + min(eq_run, need_eq);           // conserved positions in lower waves
    int ep = min(seg, L) - kp;                              // evicted positions in lower waves
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const bool eq = (eq_m >> i) & 1u;
        const uint64_t eb = __ballot(eq);
        if (eq && eq_run + mask_rank(eb) < need_eq) keep_m |= 1u << i;
        eq_run += __popcll(eb);
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

int launch_select(const float* scores, const uint8_t* mask, int H, int L, int budget, int M, int rule, int32_t* kept,
                  int32_t* evicted, int32_t* status, hipStream_t st)
{
    const LaunchCheck check;
    const int per_thread = (L + lookm::SEL_THREADS - 1) / lookm::SEL_THREADS;
    dim3 grid(H), block(lookm::SEL_THREADS);
    if (per_thread <= 4)
        hipLaunchKernelGGL(lookm::k_select<4>, grid, block, 0, st, scores, mask, L, budget, M, rule, kept, evicted, status);
    else if (per_thread <= 8)
        hipLaunchKernelGGL(lookm::k_select<8>, grid, block, 0, st, scores, mask, L, budget, M, rule, kept, evicted, status);
    else if (per_thread <= 16)
        hipLaunchKernelGGL(lookm::k_select<16>, grid, block, 0, st, scores, mask, L, budget, M, rule, kept, evicted, status);
    else if (per_thread <= 32)
        hipLaunchKernelGGL(lookm::k_select<32>, grid, block, 0, st, scores, mask, L, budget, M, rule, kept, evicted, status);
    else
        return LOOKM_ERR_UNSUPPORTED;
    mark(LOOKM_K_SELECT);
    return check.status();
}

}  // namespace lookm_host
