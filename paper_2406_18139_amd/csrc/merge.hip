// KV-pair merging and compaction (Section 3.3, Eq. 10-12; layout of Eq. 6-7).
//
// k_bucket groups the evicted tokens of a head by the conserved slot they were matched to (the
// paper's one-to-many similarity sets k_sim), as a stable counting sort so that every set lists its
// members' positions (with their matching cosines) in ascending position.  k_merge then GATHERS: one
// lane group per conserved slot reads its own row and its members' rows and writes one compact output
// row - no scatter, no float atomics, fixed summation order, coalesced 16-byte accesses along the head
// dimension.  Keys and values use the same sets and (for weighted merging) the same cosine weights.
#include "common.h"

namespace lookm {

constexpr int BK_THREADS = 1024;
constexpr int BK_WAVES = BK_THREADS / 64;
constexpr int BK_MAX_SEG = 1024;   // slots per workgroup: 16 counter rows of this many ints, and the entry lists, fit in LDS

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

// One workgroup per (head, segment of S consecutive conserved slots); the segments of a head run on
// different compute units.  Every workgroup reads the head's whole assignment list once - each thread its IPT
// entries, all loads in flight together - counts the entries matched to slots below its segment (that is
// where its part of the member lists starts) and sorts the entries matched to its own slots: wave w owns
// entries [w*64*IPT, (w+1)*64*IPT), lane l holds entries seg + i*64 + l.  The wave first compacts its own
// entries into an LDS list, in order, so that the ranking below runs over full 64-lane rows of entries that
// matter rather than over rows where most lanes belong to other segments.  Counts per (wave, slot) are turned
// into start offsets in slot-major, wave-minor order, which makes the fill stable across waves; inside a wave
// the list is taken 64 entries at a time and lanes with equal slots are ranked by lane.
//
// It also writes the segment's part of the merge plan: its slots ordered by the size of their similarity
// set, largest first, one int4 {slot, first member, set size n, position of the conserved token} per entry.
// k_merge hands consecutive plan entries to the lane groups of a wave, so groups that run in lockstep have
// sets of (nearly) equal size, and the longest sets start first.  Sizes are classed as min(n, 63); the order
// inside a class is arbitrary (it only decides which lane group handles which slot, not any result).
template <int IPT>
__global__ void __launch_bounds__(BK_THREADS)
k_bucket(const int32_t* __restrict__ assign, const int32_t* __restrict__ evicted, const float* __restrict__ sim,
         const int32_t* __restrict__ kept, int Le, int B, int S, int nbits, int4* __restrict__ plan,
         int32_t* __restrict__ member_pos, float* __restrict__ member_w)
{
    extern __shared__ int lds[];   // cnt [BK_WAVES][ns] ints, then own [BK_WAVES][64 * IPT] 16-bit entry numbers
    __shared__ int wsum[BK_WAVES], wbelow[BK_WAVES];
    __shared__ int cls[64];
    const int h = blockIdx.y, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int lo = blockIdx.x * S, ns = min(B, lo + S) - lo;   // this workgroup's slots [lo, lo + ns)
    if (ns <= 0) return;
    int* cnt = lds;
    unsigned short* own = reinterpret_cast<unsigned short*>(lds + BK_WAVES * ns) + wave * (64 * IPT);   // this wave's
    assign += (size_t)h * Le;
    evicted += (size_t)h * Le;
    sim += (size_t)h * Le;
    kept += (size_t)h * B + lo;
    plan += (size_t)h * B + lo;
    member_pos += (size_t)h * Le;
    member_w += (size_t)h * Le;

    const int seg = wave * 64 * IPT;
    int a[IPT];
#pragma unroll
    for (int i = 0; i < IPT; ++i) a[i] = assign[min(seg + i * 64 + lane, Le - 1)];   // clamped: masked below
    for (int i = tid; i < BK_WAVES * ns; i += BK_THREADS) cnt[i] = 0;
    if (tid < 64) cls[tid] = 0;
    __syncthreads();
    int below_wave = 0, n_own = 0;
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int e = seg + i * 64 + lane;
        int s = -1;
        if (e < Le) s = min(max(a[i], 0), B - 1) - lo;
        below_wave += __popcll(__ballot(e < Le && s < 0));
        const bool mine = s >= 0 && s < ns;
        const uint64_t mb = __ballot(mine);
        if (mine) {
            atomicAdd(&cnt[wave * ns + s], 1);
            own[n_own + mask_rank(mb)] = (unsigned short)(i * 64 + lane);
        }
        n_own += __popcll(mb);
    }
    // the wave's first two rows of own entries: their slot, position and cosine are fetched now and arrive while
    // the offsets and the plan are being worked out
    int pre_key[2], pre_pos[2];
    float pre_w[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const bool valid = u * 64 + lane < n_own;
        const int e = min(seg + (valid ? (int)own[u * 64 + lane] : 0), Le - 1);
        pre_key[u] = assign[e];
        pre_pos[u] = evicted[e];
        pre_w[u] = sim[e];
    }
    if (lane == 0) wbelow[wave] = below_wave;
    __syncthreads();

    const int per = (ns + BK_THREADS - 1) / BK_THREADS;
    const int a0 = min(ns, tid * per), a1 = min(ns, a0 + per);
    int local = 0;
    for (int s = a0; s < a1; ++s)
#pragma unroll
        for (int w = 0; w < BK_WAVES; ++w) local += cnt[w * ns + s];
    int incl = local;
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int run = incl - local, total = 0;
#pragma unroll
    for (int w = 0; w < BK_WAVES; ++w) {
        run += wbelow[w] + ((w < wave) ? wsum[w] : 0);   // members of lower segments, then of lower slots
        total += wbelow[w] + wsum[w];
    }
    for (int s = a0; s < a1; ++s)
#pragma unroll
        for (int w = 0; w < BK_WAVES; ++w) {
            const int c = cnt[w * ns + s];
            cnt[w * ns + s] = run;
            run += c;
        }
    __syncthreads();

    // the merge plan of this segment; row 0 of cnt holds every slot's first member, `total` ends the last set
    for (int j = 0; j < per; ++j) {
        const int s = tid * per + j;
        const bool valid = s < ns;
        const int n = valid ? ((s + 1 < ns) ? cnt[s + 1] : total) - cnt[s] : 0;
        const int c = 63 - min(n, 63);
        const uint64_t peers = match_key(c, valid, 6);
        if (valid && mask_rank(peers) == 0) atomicAdd(&cls[c], __popcll(peers));
    }
    __syncthreads();
    if (wave == 0) {
        const int v = cls[lane];
        int in2 = v;
        for (int off = 1; off < 64; off <<= 1) {
            const int u = __shfl_up(in2, off);
            if (lane >= off) in2 += u;
        }
        cls[lane] = in2 - v;
    }
    __syncthreads();
    for (int j = 0; j < per; ++j) {
        const int s = tid * per + j;
        const bool valid = s < ns;
        const int s0 = valid ? cnt[s] : 0;
        const int n = valid ? ((s + 1 < ns) ? cnt[s + 1] : total) - s0 : 0;
        const int c = 63 - min(n, 63);
        const uint64_t peers = match_key(c, valid, 6);
        const int leader = valid ? __ffsll((unsigned long long)peers) - 1 : lane;
        int base = 0;
        if (valid && lane == leader) base = atomicAdd(&cls[c], __popcll(peers));
        base = __shfl(base, leader);
        if (valid) plan[base + mask_rank(peers)] = make_int4(lo + s, s0, n, kept[s]);
    }
    __syncthreads();

    // one 64-entry row of the wave's list: rank lanes with equal slots, store, advance the slots' offsets
    auto place = [&](bool valid, int raw_slot, int pos, float sw) {
        const int key = valid ? min(max(raw_slot, 0), B - 1) - lo : 0;
        const uint64_t peers = match_key(key, valid, nbits);
        int base = 0;
        if (valid) {
            base = cnt[wave * ns + key];
            const int dst = base + mask_rank(peers);
            member_pos[dst] = pos;           // the set lists positions (ascending) and their cosines
            member_w[dst] = sw;
        }
        __builtin_amdgcn_wave_barrier();
        if (valid && (peers >> lane) == 1ull) cnt[wave * ns + key] = base + __popcll(peers);   // highest peer updates
        __builtin_amdgcn_wave_barrier();
    };
    if (n_own > 0) place(lane < n_own, pre_key[0], pre_pos[0], pre_w[0]);
    if (n_own > 64) place(64 + lane < n_own, pre_key[1], pre_pos[1], pre_w[1]);
    // further rows (a segment that most of the wave's entries belong to - few slots hold most members): each row's
    // slot, position and cosine are fetched while the row before it is being placed
    if (n_own > 128) {
        auto fetch_row = [&](int c0, int& key, int& pos, float& sw) {
            const bool valid = c0 + lane < n_own;
            const int e = min(seg + (valid ? (int)own[c0 + lane] : 0), Le - 1);
            key = assign[e];
            pos = evicted[e];
            sw = sim[e];
        };
        int key, pos;
        float sw;
        fetch_row(128, key, pos, sw);
        for (int c0 = 128; c0 < n_own; c0 += 64) {
            const int ck = key, cp = pos;
            const float cw = sw;
            if (c0 + 64 < n_own) fetch_row(c0 + 64, key, pos, sw);
            place(c0 + lane < n_own, ck, cp, cw);
        }
    }
}

// G lanes per conserved slot, each lane 8 consecutive head dims of the key row and of the value row (both use
// the same set, the same weights and the same index reads).  The head's merge plan is NS segments of S entries,
// each ordered by set size; consecutive workgroups take the next 256/G entries of consecutive segments, so the
// big sets of every segment are started early.  A slot's members are fetched NB at a time (positions and
// weights are plain sequential reads, the 2*NB row loads are independent), so the gather keeps many loads in
// flight per lane group instead of one dependent chain per member.  A short last batch repeats the set's last
// member with weight zero.
template <typename T, int NT, int NB>   // NT = 2: one lane group does the key row and the value row; 1: blockIdx.z picks
__global__ void __launch_bounds__(256)
k_merge(const T* __restrict__ k, const T* __restrict__ v, const int32_t* __restrict__ kept,
        const int4* __restrict__ plan, const int32_t* __restrict__ member_pos,
        const float* __restrict__ member_w, int L, int d, int B, int Le, int mode, int G, int S, int NS,
        T* __restrict__ k_out, T* __restrict__ v_out)
{
    // heads vary fastest over the grid: the workgroups with the largest sets of every head are dispatched first
    const int h = blockIdx.x;
    const int g = (int)blockIdx.y % NS, in_seg = ((int)blockIdx.y / NS) * (256 / G) + (int)threadIdx.x / G;
    const int idx = g * S + in_seg;
    const int c0 = ((int)threadIdx.x % G) * 8;
    if (in_seg >= S || idx >= B || c0 >= d) return;
    int slot = idx, o0 = 0, n = 0, pos;
    if (mode != LOOKM_MERGE_NONE) {
        const int4 pl = plan[(size_t)h * B + idx];
        slot = pl.x;
        o0 = pl.y;
        n = pl.z;                                    // L_sim: size of this slot's similarity set
        pos = pl.w;
    } else {
        pos = kept[(size_t)h * B + slot];
    }
    const T* x[NT];
    T* out[NT];
    const size_t in_off = (size_t)h * L * d + c0, out_off = ((size_t)h * B + slot) * d + c0;
    if (NT == 2) {
        x[0] = k + in_off;
        x[NT - 1] = v + in_off;
        out[0] = k_out + out_off;
        out[NT - 1] = v_out + out_off;
    } else {
        x[0] = (blockIdx.z ? v : k) + in_off;
        out[0] = (blockIdx.z ? v_out : k_out) + out_off;
    }

    float xc[NT][8];
#pragma unroll
    for (int s = 0; s < NT; ++s) load8(x[s] + (size_t)pos * d, xc[s]);
    if (n > 0) {
        member_pos += (size_t)h * Le;
        member_w += (size_t)h * Le;
        float acc[NT][8];
#pragma unroll
        for (int s = 0; s < NT; ++s)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[s][i] = 0.f;
        const bool weighted = (mode == LOOKM_MERGE_WEIGHTED);
        const int o1 = o0 + n;
        // positions and weights of a batch are fetched one batch ahead, so that a long set costs one memory round
        // trip per batch (the rows) instead of two dependent ones (positions, then rows)
        int p[NB];
        float w[NB];
        auto fetch_members = [&](int t) {
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int tt = min(t + j, o1 - 1);
                p[j] = member_pos[tt];
                w[j] = (t + j < o1) ? (weighted ? member_w[tt] : 1.0f) : 0.0f;
            }
        };
        fetch_members(o0);
        for (int t = o0; t < o1; t += NB) {          // ascending position
            float xe[NT][NB][8];
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int s = 0; s < NT; ++s) load8(x[s] + (size_t)p[j] * d, xe[s][j]);
            float wc[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j) wc[j] = w[j];
            if (t + NB < o1) fetch_members(t + NB);  // in flight together with this batch's rows
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int s = 0; s < NT; ++s)
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[s][i] = fmaf(xe[s][j][i], wc[j], acc[s][i]);
        }
        const float inv = 1.0f / (float)(n + 1);
#pragma unroll
        for (int s = 0; s < NT; ++s) {
            if (mode == LOOKM_MERGE_PIVOTAL)         // Eq. 11: (x_c + 1/2 sum (x_e + x_c)) / (n + 1)
#pragma unroll
                for (int i = 0; i < 8; ++i) xc[s][i] = (xc[s][i] + 0.5f * fmaf((float)n, xc[s][i], acc[s][i])) * inv;
            else                                     // Eq. 10 / Eq. 12: (x_c + sum w_e x_e) / (n + 1)
#pragma unroll
                for (int i = 0; i < 8; ++i) xc[s][i] = (xc[s][i] + acc[s][i]) * inv;
        }
    }
#pragma unroll
    for (int s = 0; s < NT; ++s) store8(out[s], xc[s]);
}

}  // namespace lookm

namespace lookm_host {

#ifndef LOOKM_MERGE_NT
#define LOOKM_MERGE_NT 2
#endif
#ifndef LOOKM_MERGE_NB
#define LOOKM_MERGE_NB 8
#endif

// Segments per head: enough workgroups to cover the chip's 256 compute units, and no more than
// BK_MAX_SEG slots in one segment.
static void bucket_segments(int H, int B, int& S, int& NS)
{
    int ns = (256 + H - 1) / H;
    if (ns > 16) ns = 16;
    const int need = (B + lookm::BK_MAX_SEG - 1) / lookm::BK_MAX_SEG;
    if (ns < need) ns = need;
    if (ns > B) ns = B;
    S = (B + ns - 1) / ns;
    NS = (B + S - 1) / S;
}

template <typename T>
static void launch_merge_t(const T* k, const T* v, const int32_t* kept, const int4* plan,
                           const int32_t* member_pos, const float* member_w, int H, int L, int d, int B, int mode,
                           int S, int NS, T* k_out, T* v_out, hipStream_t st)
{
    int G = 1;
    while (G * 8 < d) G <<= 1;
    const int spb = 256 / G;
    constexpr int NT = LOOKM_MERGE_NT, NB = LOOKM_MERGE_NB;
    dim3 grid(H, NS * ((S + spb - 1) / spb), 3 - NT);
    hipLaunchKernelGGL((lookm::k_merge<T, NT, NB>), grid, dim3(256), 0, st, k, v, kept, plan, member_pos, member_w, L, d, B,
                       L - B, mode, G, S, NS, k_out, v_out);
}

template <int IPT>
static int launch_bucket(const int32_t* assign, const int32_t* evicted, const float* sim, const int32_t* kept,
                         int H, int Le, int B, int S, int NS, int4* plan, int32_t* member_pos, float* member_w,
                         hipStream_t st)
{
    const size_t lds = (size_t)lookm::BK_WAVES * (S * sizeof(int) + 64 * IPT * sizeof(unsigned short));
    int nbits = 1;
    while ((1 << nbits) < S) ++nbits;
    hipLaunchKernelGGL(lookm::k_bucket<IPT>, dim3(NS, H), dim3(lookm::BK_THREADS), lds, st, assign, evicted, sim, kept,
                       Le, B, S, nbits, plan, member_pos, member_w);
    return LOOKM_OK;
}

int launch_merge(const void* k, const void* v, const int32_t* kept, const int32_t* evicted, const int32_t* assign,
                 const float* sim, int H, int L, int d, lookm_dtype dt, int budget, int mode, int32_t* plan_words,
                 int32_t* member_pos, float* member_w, void* k_out, void* v_out, hipStream_t st)
{
    const int B = budget, Le = L - B;
    if (B == 0) return LOOKM_OK;
    const LaunchCheck check;
    if (Le == 0) mode = LOOKM_MERGE_NONE;
    int4* plan = reinterpret_cast<int4*>(plan_words);
    int S, NS;
    bucket_segments(H, B, S, NS);
    if (mode != LOOKM_MERGE_NONE) {
        const int per_thread = (Le + lookm::BK_THREADS - 1) / lookm::BK_THREADS;
        int rc;
        if (per_thread <= 4)
            rc = launch_bucket<4>(assign, evicted, sim, kept, H, Le, B, S, NS, plan, member_pos, member_w, st);
        else if (per_thread <= 8)
            rc = launch_bucket<8>(assign, evicted, sim, kept, H, Le, B, S, NS, plan, member_pos, member_w, st);
        else if (per_thread <= 16)
            rc = launch_bucket<16>(assign, evicted, sim, kept, H, Le, B, S, NS, plan, member_pos, member_w, st);
        else if (per_thread <= 32)
            rc = launch_bucket<32>(assign, evicted, sim, kept, H, Le, B, S, NS, plan, member_pos, member_w, st);
        else
            return LOOKM_ERR_UNSUPPORTED;
        if (rc != LOOKM_OK) return rc;
        mark(LOOKM_K_BUCKET);
    }
    if (dt == LOOKM_BF16)
        launch_merge_t((const lookm::bf16_t*)k, (const lookm::bf16_t*)v, kept, plan, member_pos, member_w, H, L, d,
                       B, mode, S, NS, (lookm::bf16_t*)k_out, (lookm::bf16_t*)v_out, st);
    else
        launch_merge_t((const float*)k, (const float*)v, kept, plan, member_pos, member_w, H, L, d, B, mode, S, NS,
                       (float*)k_out, (float*)v_out, st);
    mark(LOOKM_K_MERGE);
    return check.status();
}

template <int IPT> static bool bucket_attribute()
{
    return hipFuncSetAttribute((const void*)lookm::k_bucket<IPT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               lookm::BK_WAVES * (lookm::BK_MAX_SEG * 4 + 64 * IPT * 2)) == hipSuccess;
}

int set_attributes_merge()
{
    return (bucket_attribute<4>() && bucket_attribute<8>() && bucket_attribute<16>() && bucket_attribute<32>())
               ? LOOKM_OK : LOOKM_ERR_DEVICE;
}

}  // namespace lookm_host
