// Accumulated attention scores (Section 3.2, Eq. 4) on the gfx950 matrix cores: bf16, head_dim 128.
//
// Both passes are the same machine with the roles of Q and K swapped.  A workgroup (4 waves)
// owns 256 "stationary" rows - query rows in pass 1, key rows in pass 2 - whose MFMA B-operand
// fragments stay in registers (64 rows x 128 dims per wave = 64 VGPRs), and streams the other
// tensor past them in 64-row tiles through double-buffered LDS as the A operand.  The MFMA is
// v_mfma_f32_16x16x32_bf16: a 32-row block of the streamed tensor against the wave's 64 stationary rows is
// eight 16x16 tiles (two groups of 16 streamed rows x four groups of 16 stationary rows), and of every tile a
// lane (c = lane % 16, q = lane / 16) holds the streamed rows 4q .. 4q+3 against stationary row c.  A lane's
// 32 accumulator values of a block thus belong to FOUR stationary rows, eight streamed rows each, and both
// reductions of the method stay in-lane:
//   pass 1: running (max, sum) of 2^(c q.k) over the keys of a query row   -> lse2[i]
//   pass 2: running sum of 2^(c q.k - lse2[i]) over the query rows of a key -> A_s[j]
// The four lanes that share a stationary row (equal c) are combined once, after the loop.  (The 32x32x16 form
// of the instruction, with which a lane holds 16 streamed rows of two stationary rows, does the same work in
// the same registers, but this chip sustains 13 % less of it under this load, measured with random operands;
// with the epilogues the two score passes together are 6 % faster this way.)
// Nothing is atomically accumulated; every sum has a fixed order, so results are bitwise
// repeatable.  c = log2(e)/sqrt(d) folds the softmax scale into the exp2 argument.
#include "common.h"

#include <algorithm>
#include <type_traits>

namespace lookm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int SD = 128;        // head dim
constexpr int BS = 256;        // stationary rows per workgroup
constexpr int BX = 64;         // streamed rows per iteration
static_assert(BX == 64, "the lse staging of pass 2 is done by wave 0, one row per lane");
constexpr int XROW = 128;       // LDS row = 256 B, unpadded; the 16-byte chunk c of row r sits at chunk c ^ (r & 7),
                               // so 16-byte reads of 8 consecutive rows at the same c hit all 32 banks once

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Epilogues of a finished block: acc[rg][cg], rg = which 16 of the block's 32 streamed rows, cg = which 16 of the
// wave's 64 stationary rows.  Entry i of acc[rg][cg] is streamed row xq + 16*rg + i (xq = block start + 4q) against
// this lane's stationary row of group cg, whose position is sP[cg].
//   PASS 2: running sums of 2^(c*(s - b_i)) over the query rows of the lane's four keys, b_i = lse2_i / c; the
//           accumulators arrive with -b_i already in them (the MFMA chain starts from it instead of from zero),
//           so no per-row value has to be held in registers here.
template <bool MASK>
__device__ __forceinline__ void colsum_block_epilogue(const f32x4 (&acc)[2][4], float scale2, int xq, const int (&sP)[4],
                                                      float (&run)[4])
{
#pragma unroll
    for (int cg = 0; cg < 4; ++cg) {
        float sum;   // (started from its first term: 0 + x is an addition the compiler may not drop)
#pragma unroll
        for (int rg = 0; rg < 2; ++rg)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float p = __builtin_amdgcn_exp2f(acc[rg][cg][i] * scale2);
                if (MASK && (xq + 16 * rg + i < sP[cg])) p = 0.f;   // query before the key
                sum = (rg == 0 && i == 0) ? p : sum + p;
            }
        run[cg] += sum;
    }
}

// Pass 1, a finished block (32 streamed keys against the lane's four query rows).
// The reference of a running sum is refreshed lazily: a block is first summed against the row's current reference m;
// only if a sum overflows (the first block of a row, where m is still "minus infinity", or a logit more than 64
// binades above the reference) is the block maximum taken and the running sum rescaled.  The result is the same up
// to rounding - a float sum keeps its relative precision at any magnitude below 2^64 - and the common case saves
// the maximum over the block.  One wave-uniform test covers the whole block (a branch on a vector result drains the
// wave's vector pipeline); the refresh is valid for a row that did not overflow as well.
__device__ __forceinline__ void lse_refresh(const f32x4& lo, const f32x4& hi, float scale2, float& m, float& l)
{
    const float bm = fmaxf(fmaxf(fmaxf(fmaxf(lo[0], lo[1]), lo[2]), fmaxf(fmaxf(lo[3], hi[0]), hi[1])), fmaxf(hi[2], hi[3]));
    const float mn = fmaxf(m, bm * scale2);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) sum += __builtin_amdgcn_exp2f(fmaf(lo[i], scale2, -mn));
#pragma unroll
    for (int i = 0; i < 4; ++i) sum += __builtin_amdgcn_exp2f(fmaf(hi[i], scale2, -mn));
    l = fmaf(l, __builtin_amdgcn_exp2f(m - mn), sum);
    m = mn;
}

template <bool MASK>
__device__ __forceinline__ void lse_block_epilogue(f32x4 (&acc)[2][4], float scale2, int xq, const int (&sP)[4],
                                                   float (&m)[4], float (&l)[4])
{
    if (MASK) {
#pragma unroll
        for (int cg = 0; cg < 4; ++cg)
#pragma unroll
            for (int rg = 0; rg < 2; ++rg)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (xq + 16 * rg + i > sP[cg]) acc[rg][cg][i] = -INFINITY;   // key after the query
    }
    float sum[4];
#pragma unroll
    for (int cg = 0; cg < 4; ++cg) {
#pragma unroll
        for (int rg = 0; rg < 2; ++rg)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = __builtin_amdgcn_exp2f(fmaf(acc[rg][cg][i], scale2, -m[cg]));
                sum[cg] = (rg == 0 && i == 0) ? p : sum[cg] + p;   // (0 + x is an addition the compiler may not drop)
            }
    }
    const bool over = !(sum[0] <= 1.8e19f) || !(sum[1] <= 1.8e19f) || !(sum[2] <= 1.8e19f) || !(sum[3] <= 1.8e19f);
    if (__builtin_expect(__any(over), 0)) {     // also true for NaN; wave-uniform
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) lse_refresh(acc[0][cg], acc[1][cg], scale2, m[cg], l[cg]);
    } else {
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) l[cg] += sum[cg];
    }
}

// ---- work decomposition -------------------------------------------------------------------------------
// A strip is 256 stationary rows; its streamed range (keys 0..strip end in pass 1, query rows strip
// start..L in pass 2) is 4..L/64 tiles long.  The streamed axis is cut at multiples of CT = C*64 rows
// into chunks, one workgroup per (strip, chunk), so that no workgroup is much longer than the average
// (the longest strip alone would otherwise set the kernel's duration).  Chunk boundaries are the same
// for every strip, and work is enumerated chunk-major, so the workgroups resident on an XCD at one
// time stream the SAME rows of the same head and share them in that XCD's L2.  Each workgroup writes a
// partial result per stationary row; a small second kernel folds a strip's chunks together in order.
//
// With an observation window only the query rows R0 .. L-1 count (R0 = 0: all rows, Eq. 4 as printed): pass 1
// then needs only the strips that hold such rows, and pass 2 streams a strip's query rows from max(strip start,
// R0) on, so the chunks below R0 are empty for every strip.
__host__ __device__ inline int first_chunk(int pass, int t, int CT, int R0)
{
    return (pass == 1) ? 0 : max(t * BS, R0) / CT;
}
__host__ __device__ inline int strip_chunks(int pass, int t, int L, int CT, int R0)
{
    if (pass == 1) return ((t + 1) * BS > R0) ? (min(L, (t + 1) * BS) + CT - 1) / CT : 0;
    return (L + CT - 1) / CT - max(t * BS, R0) / CT;
}

// The matrix pipe and the vector ALU of a SIMD overlap ACROSS waves far better than within one (measured), so a
// wave's arithmetic stays in two phases - MFMA chains, then the epilogue - and the kernel is sized for three
// resident waves per SIMD; what a wave does overlap with its own arithmetic is memory latency (LDS fragment
// fetches one block ahead, tile loads one tile ahead).
//   PASS 1 writes part_a = running max, part_b = running sum (base-2 domain) per (chunk, stationary row).
//   PASS 2 writes part_a = partial column sum per (chunk, stationary row).  Its stationary rows are keys: when
//   `rnorm` is given, the workgroup of a strip's first chunk also writes rnorm[h, j] = 1 / ||k_j|| (0 for a
//   zero key) for the matching of Eq. 9, from the registers it holds anyway - the keys are not read again for it.
// ---- scores for the competing keys only -------------------------------------------------------------------
// Selection ranks only the image tokens before the recent window (Eq. 5-8: text tokens and the window are
// conserved whatever their score).  When the caller does not ask for the scores themselves, pass 2 therefore
// runs over those keys alone: its strips are 256 consecutive entries of the ascending list of competing positions
// instead of 256 consecutive positions, and everything else - chunk boundaries, the tiles a key's column sum runs
// over, the order of every addition - is unchanged, so the scores of the competing keys come out bit for bit as
// on the dense path.  The lists are built from the modality mask by one extra workgroup of pass 1 (or by a small
// kernel of its own when pass 1 is skipped):
//   lists[0] = number of competing keys, lists[1] = number of protected keys,
//   lists[LIST_HEAD .. +L) competing positions ascending, lists[LIST_HEAD + L .. +L) protected positions ascending.
constexpr int LIST_HEAD = 64;

__device__ __forceinline__ void build_key_lists(const uint8_t* __restrict__ mask, int L, int M, int32_t* __restrict__ lists,
                                                int* scan /* LDS, 256 ints */)
{
    // Thread t owns the positions [t * per, t * per + per), per <= LOOKM_MAX_L / 256 = 128.  Their mask bytes are
    // fetched sixteen at a time, all sixteen loads in flight together (one at a time, a 12 K-token mask cost this
    // workgroup fifty memory latencies twice over), and kept as 128 flag bits for the second sweep.
    static_assert(LOOKM_MAX_L <= 256 * 128, "a thread's range must fit its 128 flag bits");
    const int tid = threadIdx.x, per = (L + 255) / 256, lo = min(L, tid * per), hi = min(L, lo + per);
    uint64_t flags[2] = {0ull, 0ull};
    int nc = 0;
#pragma unroll
    for (int j0 = 0; j0 < 128; j0 += 16) {
        if (j0 < per) {                                  // uniform
            uint8_t b[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) b[u] = mask[min(lo + j0 + u, L - 1)];
            uint32_t w = 0;
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int j = lo + j0 + u;
                w |= (j < hi && b[u] != 0 && j < L - M) ? (1u << u) : 0u;
            }
            flags[j0 >> 6] |= (uint64_t)w << (j0 & 63);
            nc += __popc(w);
        }
    }
    scan[tid] = nc;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {          // inclusive scan of the competing counts
        const int v = (tid >= off) ? scan[tid - off] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    int c_at = scan[tid] - nc, p_at = lo - c_at;       // competing / protected keys before this thread's range
    if (tid == 255) { lists[0] = scan[255]; lists[1] = L - scan[255]; }
    for (int j = lo; j < hi; ++j) {
        const int r = j - lo;
        const bool competing = (((r < 64) ? flags[0] : flags[1]) >> (r & 63)) & 1ull;
        if (competing) lists[LIST_HEAD + c_at++] = j;
        else lists[LIST_HEAD + L + p_at++] = j;
    }
}

__global__ void __launch_bounds__(256) k_score_lists(const uint8_t* __restrict__ mask, int L, int M, int32_t* __restrict__ lists)
{
    __shared__ int scan[256];
    build_key_lists(mask, L, M, lists, scan);
}

template <int PASS, bool SPARSE>
__global__ void __launch_bounds__(256, 3)
k_score_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, int H, int group, int L, int R0, float scale2,
             int C, int U, const float* __restrict__ lse2, float lse_scale, float* __restrict__ part_a,
             float* __restrict__ part_b, float* __restrict__ rnorm, const uint8_t* __restrict__ modality, int M,
             int32_t* __restrict__ lists)
{
    // Two tiles as separate arrays, with the buffer of a tile known at compile time (the tile loop is unrolled by
    // two): the compiler then sees that a fragment read of one array cannot alias the loads in flight to the
    // other.  With one array indexed by a run-time buffer number it waits for every outstanding load before a
    // tile's first LDS read, which serialises the prefetch with the MFMA block of the same wave.
    __shared__ __attribute__((aligned(16))) bf16_t xs0[BX * XROW];
    __shared__ __attribute__((aligned(16))) bf16_t xs1[BX * XROW];
    __shared__ __attribute__((aligned(16))) float xl0[BX];   // pass 2: -lse2[i] of the streamed query rows
    __shared__ __attribute__((aligned(16))) float xl1[BX];
    __shared__ int spos[SPARSE ? 4 * 256 : 1];   // sparse pass 2: positions of every lane's four stationary rows

    // pass 1 with a mask: the launch has one workgroup more, which builds the key lists for pass 2
    if (PASS == 1 && modality != nullptr && blockIdx.x == gridDim.x - 1) {
        build_key_lists(modality, L, M, lists, reinterpret_cast<int*>(xs0));
        return;
    }
    // pass 2 with lists: stationary rows are entries of the list of competing positions
    static_assert(PASS == 2 || !SPARSE, "only pass 2 has a sparse form");
    constexpr bool sparse = SPARSE;
    const int NC = sparse ? lists[0] : L;                 // stationary rows in all
    const int32_t* clist = lists + LIST_HEAD;

    // Consecutive workgroup ids go to consecutive XCDs.  With 8 or more heads, XCD x works through heads
    // x, x+8, ... one at a time, so its L2 holds one head's current chunk; with fewer heads each head
    // gets 8/H XCDs that share its units round-robin.
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    int h, e;
    if (H >= 8) {
        h = (j / U) * 8 + xcd;
        e = j % U;
    } else {
        const int xph = 8 / H;            // XCDs per head
        h = xcd / xph;
        e = j * xph + xcd % xph;
    }
    if (h >= H || e >= U) return;
    const int nS = (L + BS - 1) / BS, CT = C * BX;
    int g = (PASS == 1) ? 0 : R0 / CT, tile = 0;
    for (;; ++g) {      // chunk-major enumeration: all strips that touch chunk g, then chunk g+1, ...
        const int t_first = (PASS == 1) ? max((g * CT) / BS, R0 / BS) : 0;
        const int cnt = (PASS == 1) ? nS - t_first : min(nS, ((g + 1) * CT + BS - 1) / BS);
        if (e < cnt) { tile = t_first + e; break; }
        e -= cnt;
    }
    const int s0 = tile * BS;
    const int n_chunks_total = (L + CT - 1) / CT;
    // slot of this (chunk, strip) in the partial arrays [h][chunk][strip][256]; pass 1 under an observation window
    // only has the strips from the window's first one on, and indexes them from there
    const int t_base = (PASS == 1) ? R0 / BS : 0, nSp = nS - t_base;
    const int u = g * nSp + (tile - t_base);
    // h runs over the query heads; with grouped query heads, `group` consecutive ones read key head h / group
    const bf16_t* qh = q + (size_t)h * L * SD;
    const bf16_t* kh = k + (size_t)(h / group) * L * SD;
    const bf16_t* S = (PASS == 1) ? qh : kh;   // stationary tensor
    const bf16_t* X = (PASS == 1) ? kh : qh;   // streamed tensor
    const float* lse_h = lse2 + (size_t)h * L;

    // the wave number is uniform across a wave: taken through a scalar register, everything derived from it (the
    // wave's first row, loop bounds, LDS addresses) stays in scalar registers and scalar branches
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, q4 = lane >> 4,
              c16 = lane & 15;   // this lane: column c16 of every 16x16 tile, rows 4*q4 .. 4*q4+3
    const int w0 = s0 + wave * 64;

    // The strip's first row decides where its streamed range starts (sparse: a list entry).
    const int p_strip = !sparse ? s0 : (s0 < NC) ? __builtin_amdgcn_readfirstlane(clist[min(s0, L - 1)]) : 0;
    const int strip_begin = (PASS == 1) ? 0 : (p_strip / BX) * BX;
    const int strip_end = (PASS == 1) ? min(L, s0 + BS) : L;
    const int x_begin = max(max(strip_begin, g * CT), (PASS == 2) ? (R0 / BX) * BX : 0);   // tile-aligned
    const int x_end = min(strip_end, (g + 1) * CT);
    // (sparse) no such strip of competing keys, or the chunk ends before the strip's first key: such a unit runs no
    // tile and writes partials that nothing reads (an early exit here costs the kernel its register budget)
    const bool idle = sparse && (s0 >= NC || x_end <= x_begin);

    // Positions of this lane's four stationary rows (row 16*cg + c16 of the wave, cg = 0..3) and of the wave's first
    // and last row: row numbers themselves on the dense path, list entries on the sparse one (rows past the end of the
    // list: a position past the prompt, which no query row reaches).
    int p_wave_lo = w0, p_wave_hi = w0 + 63;
    if (sparse) {
        // wave-uniform values: kept in scalar registers
        p_wave_lo = (w0 < NC) ? __builtin_amdgcn_readfirstlane(clist[min(w0, NC - 1)]) : 0x3fffffff;
        p_wave_hi = (w0 < NC) ? __builtin_amdgcn_readfirstlane(clist[min(w0 + 63, NC - 1)]) : 0x3fffffff;
    }
    // the position of stationary row cg of this lane (sparse: from LDS, see below)
    auto stationary_pos = [&](int cg) { return sparse ? spos[cg * 256 + tid] : w0 + 16 * cg + c16; };

    // stationary fragments: of row 16*cg + c16, the dims 32*ks + 8*q4 .. +7 (the B operand of MFMA step ks)
    bf16x8 sf[4][4];
#pragma unroll
    for (int cg = 0; cg < 4; ++cg) {
        int row = w0 + 16 * cg + c16;
        if (sparse) {
            row = (row < NC) ? clist[row] : 0x3fffffff;
            // the per-lane positions are only needed again where a tile touches the diagonal (and for the norms):
            // parked in LDS meanwhile (each lane reads back what it wrote itself, so no barrier is involved)
            spos[cg * 256 + tid] = row;
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row < L) v = *reinterpret_cast<const uint4*>(S + (size_t)row * SD + ks * 32 + q4 * 8);
            sf[cg][ks] = as_bf16x8(v);
        }
    }

    const int n_it = idle ? 0 : (x_end - x_begin + BX - 1) / BX;

    // Staging goes from global memory straight into LDS (global_load_lds_dwordx4): the 64 lanes of a wave
    // fill 1 KB = 4 consecutive LDS rows, lane l landing at chunk l%16 of row l/16, so the swizzle is applied
    // on the global side: the lane fetches chunk (l%16) ^ (row & 7) of its row.  Rows past the end re-read the
    // last row (their contribution is masked out or weighted by 2^-inf).  No staging registers, no LDS stores.
    constexpr int NLD = BX / 16;   // 1 KB pieces per wave and tile
    const int ld_sub = lane >> 4, ld_pos = lane & 15;
    float stage_l = 0.f;
    // byte offset of this lane's 16 bytes inside a tile: row (wave*4 + ld_sub) of the first 1 KB piece, swizzled chunk
    // (the 16 rows between two pieces do not change row & 7)
    // (pass 1 works it out again for every tile - six instructions - instead of holding it: with its registers all
    // taken the compiler otherwise parks it in scratch memory and waits for the reload at the top of every tile)
    auto lane_offset = [&]() {
        int t = lane;
        if (PASS == 1) {   // the lane number afresh (two instructions), so that no register has to hold it meanwhile
            t = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
            asm volatile("" : "+v"(t));
        }
        const int sub = t >> 4, pos = t & 15;
        return (uint32_t)((wave * 4 + sub) * (SD * 2) + ((pos ^ ((wave * 4 + sub) & 7)) * 16));
    };
    const char* Xb = reinterpret_cast<const char*>(X);
    auto load_tile = [&](int x0, bf16_t* xsb) {
        const uint32_t lane_off = lane_offset();
        if (x0 + BX <= L) {          // scalar test: a whole tile inside the tensor needs no clamping
            const uint32_t o = (uint32_t)x0 * (SD * 2) + lane_off;
#pragma unroll
            for (int i = 0; i < NLD; ++i)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(Xb + (o + (uint32_t)i * 16 * SD * 2)),
                    (__attribute__((address_space(3))) void*)&xsb[(i * 4 + wave) * 4 * XROW], 16, 0, 0);
        } else {                     // the tensor's last tile: rows past the end re-read the last row
            const int lane_row = (int)(lane_off >> 8), lane_chunk = (int)(lane_off & 255);   // SD * 2 = 256 bytes per row
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const uint32_t o = (uint32_t)min(x0 + i * 16 + lane_row, L - 1) * (SD * 2) + lane_chunk;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xb + o),
                                                 (__attribute__((address_space(3))) void*)&xsb[(i * 4 + wave) * 4 * XROW],
                                                 16, 0, 0);
            }
        }
        // Pass 2 also needs lse2 of the tile's rows: wave 0 (threads 0 .. BX-1, a scalar test) loads one value per
        // lane here, unconditionally (rows outside the tensor read its last row), and store_tile puts it into LDS at
        // the end of the previous tile.  Nothing may touch the loaded value before that: a use right after the load
        // would make the wave wait for everything it has just issued, the tile's rows included - hence the empty asm
        // in store_tile, which keeps the compiler from moving the arithmetic up here.
        if (PASS == 2 && wave == 0) stage_l = lse_h[min(x0 + tid, L - 1)];
    };
    // x0: first row of the tile that was loaded.  Value stored: -lse2_i / c (the start of the MFMA chains of pass 2);
    // rows outside [R0, L) get -inf and contribute nothing.
    auto store_tile = [&](float* xlb, int x0) {
        if (PASS == 2 && wave == 0) {
            float v = stage_l;
            asm volatile("" : "+v"(v));
            xlb[tid] = (x0 + tid < L && x0 + tid >= R0) ? -v * lse_scale : -INFINITY;
        }
    };

    float m[4] = {-1e30f, -1e30f, -1e30f, -1e30f}, l[4] = {0.f, 0.f, 0.f, 0.f};   // pass 1 state per stationary row of this lane
    float run[4] = {0.f, 0.f, 0.f, 0.f};                                            // pass 2 state

    load_tile(x_begin, xs0);
    store_tile(xl0, x_begin);
    if (PASS == 2 && rnorm != nullptr && g == max(strip_begin, (R0 / BX) * BX) / CT && h % group == 0) {
        // A key row's 128 dims sit in the four lanes of equal c16: lane q4 holds the 8-dim groups q4, 4 + q4, 8 + q4
        // and 12 + q4.  The sum of squares is taken in the order of the stand-alone norm kernel (k_rnorm: eight
        // partial sums, number p over the groups p and p + 8, then a pairwise tree), so both give the same bits
        // and the stage call lookm_nearest reproduces the matching of the whole path exactly.
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) {
            double part[2];   // partial sums number q4 and 4 + q4, in binary64 as in k_rnorm
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                double ss = 0.0;
#pragma unroll
                for (int rep = 0; rep < 2; ++rep) {      // group 4*j + q4 (step j), then group 8 + 4*j + q4 (step j + 2)
                    const uint4 v = __builtin_bit_cast(uint4, sf[cg][j + 2 * rep]);
                    const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float lo = __uint_as_float(w4[i] << 16), hi = __uint_as_float(w4[i] & 0xffff0000u);
                        ss = fma((double)lo, (double)lo, ss);
                        ss = fma((double)hi, (double)hi, ss);
                    }
                }
                part[j] = ss;
            }
            // (p0 + p1) + (p2 + p3) and (p4 + p5) + (p6 + p7), then their sum
            double lo4 = part[0] + __shfl_xor(part[0], 16), hi4 = part[1] + __shfl_xor(part[1], 16);
            lo4 += __shfl_xor(lo4, 32);
            hi4 += __shfl_xor(hi4, 32);
            const double ss = lo4 + hi4;
            const int row = stationary_pos(cg);
            if (q4 == 0 && row < L) rnorm[(size_t)(h / group) * L + row] = inverse_norm(ss);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the direct-to-LDS loads have landed
    __syncthreads();

    // element offsets of this lane's first two fragments inside its LDS row (swizzled chunks 4*ks + q4); the
    // chunks of steps 2 and 3 lie 8 chunks after those of steps 0 and 1
    int frag_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) frag_off[ks] = ((4 * ks + q4) ^ (c16 & 7)) * 8;

    // Which tiles need the mask (wave-uniform, so the choice is a scalar branch):
    //   pass 1, keys stream upwards: tiles with x0 + BX - 1 <= w0 hold only keys at or before every query row of
    //   this wave, the tiles after them touch the diagonal;
    //   pass 2, query rows stream upwards from the diagonal: tiles with x0 >= w0 + 63 need no mask.
    int plain_from, plain_to;
    if (PASS == 1) {
        const int n_plain = (w0 - x_begin + 1) / BX;        // largest count with x_begin + BX*count - 1 <= w0
        plain_from = 0;
        plain_to = max(0, min(n_plain, n_it));
    } else {
        const int n_masked = (min(p_wave_hi, L) - x_begin + BX - 1) / BX;
        plain_from = max(0, min(n_masked, n_it));
        plain_to = n_it;
    }
    // fragments of one block of 32 streamed rows (the A operands of its 32 MFMAs: row 16*rg + c16 of the block,
    // dims 32*ks + 8*q4 .. +7), fetched one block ahead
    bf16x8 a[2][4];
    auto fetch_group = [&](const bf16_t* tile_rows, int rb, int rg) {
        const bf16_t* ap = &tile_rows[(rb * 32 + 16 * rg + c16) * XROW];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            a[rg][ks] = as_bf16x8(*reinterpret_cast<const uint4*>(ap + frag_off[ks]));
            a[rg][ks + 2] = as_bf16x8(*reinterpret_cast<const uint4*>(ap + frag_off[ks] + 64));
        }
    };
    auto fetch = [&](const bf16_t* tile_rows, int rb) {
        fetch_group(tile_rows, rb, 0);
        fetch_group(tile_rows, rb, 1);
    };
    // pass 1 (its epilogue keeps twice the state of pass 2's and needs registers to work in): the fragments of the
    // first two MFMA steps before the epilogue, those of the last two - needed after sixteen MFMAs - after it
    auto fetch_early = [&](const bf16_t* tile_rows, int rb) {
#pragma unroll
        for (int rg = 0; rg < 2; ++rg) {
            const bf16_t* ap = &tile_rows[(rb * 32 + 16 * rg + c16) * XROW];
            a[rg][0] = as_bf16x8(*reinterpret_cast<const uint4*>(ap + frag_off[0]));
            a[rg][1] = as_bf16x8(*reinterpret_cast<const uint4*>(ap + frag_off[1]));
        }
    };
    auto fetch_late = [&](const bf16_t* tile_rows, int rb) {
#pragma unroll
        for (int rg = 0; rg < 2; ++rg) {
            const bf16_t* ap = &tile_rows[(rb * 32 + 16 * rg + c16) * XROW];
            a[rg][2] = as_bf16x8(*reinterpret_cast<const uint4*>(ap + frag_off[0] + 64));
            a[rg][3] = as_bf16x8(*reinterpret_cast<const uint4*>(ap + frag_off[1] + 64));
        }
    };
    if (n_it > 0) fetch(xs0, 0);

    // One tile, with its LDS buffer known at compile time.  Tiles that touch the diagonal evaluate the causal
    // condition per element in their epilogues; tiles known to lie entirely inside the causal region run the same
    // epilogue minus the comparisons.  The choice is wave-uniform and made by a scalar branch around the epilogue
    // only, so that there is one tile body per buffer (with a body per mask variant the fragments carried from one
    // tile to the next would have to meet in the same registers on four paths, and the kernel no longer fits).
    auto tile_step = [&](auto buf_tag, int it) {
        constexpr int BUF = decltype(buf_tag)::value;
        bf16_t* cur = BUF ? xs1 : xs0;
        bf16_t* nxt = BUF ? xs0 : xs1;
        float* cur_l = BUF ? xl1 : xl0;
        float* nxt_l = BUF ? xl0 : xl1;
        const int x0 = x_begin + it * BX;
        if (it + 1 < n_it) load_tile(x0 + BX, nxt);
        // wave-uniform: a tile that lies entirely outside the causal region is not computed at all
        const bool mask = !(it >= plain_from && it < plain_to);
        const bool skip = mask && ((PASS == 1) ? (x0 > w0 + 63) : (x0 + BX - 1 < p_wave_lo));

        // End of the tile's LDS reads: wait for the next tile's loads, meet the other waves, and fetch the next
        // tile's first fragments - before the epilogue of this tile's second block, which hides their latency.
        // (pass 1 fetches only the first row group here and the second after the epilogue: see below)
        auto finish_tile = [&](bool all_fragments) {
            if (it + 1 < n_it) store_tile(nxt_l, x0 + BX);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the next tile's direct-to-LDS loads have landed
            __syncthreads();
            // unconditional: after the last tile this reads an old tile and the values are never used
            if (all_fragments) fetch(nxt, 0);
            else fetch_early(nxt, 0);
        };
        if (!skip) {
            // Two blocks of 32 streamed rows; the fragments of block 0 are in `a` already (fetched by the previous
            // tile, or before the loop).  A block's fragments are dead once its MFMAs have been issued, so the next
            // block's are fetched into the same registers right away and their LDS latency passes under the
            // epilogue.  The scheduling barriers keep the compiler from undoing the order, and from holding more
            // than one block's values at a time: the kernel has to stay within 168 VGPRs.
            f32x4 acc[2][4];
            // the MFMA chains of a block start from zero in pass 1 and from -lse2_i / c of the lane's streamed rows
            // (two 16-byte LDS reads; every chain's first MFMA takes them as its C operand) in pass 2
            auto multiply = [&](int rb) {
                if (PASS == 1) {
                    // step by step over all eight tiles, so that a tile's next MFMA is eight instructions away; the
                    // fragments of the last step were asked for after the previous epilogue and land meanwhile
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};   // an inline constant of the instruction, no registers
#pragma unroll
                    for (int cg = 0; cg < 4; ++cg)
#pragma unroll
                        for (int rg = 0; rg < 2; ++rg)
                            acc[rg][cg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rg][0], sf[cg][0], zero, 0, 0, 0);
#pragma unroll
                    for (int ks = 1; ks < 4; ++ks)
#pragma unroll
                        for (int cg = 0; cg < 4; ++cg)
#pragma unroll
                            for (int rg = 0; rg < 2; ++rg)
                                acc[rg][cg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rg][ks], sf[cg][ks], acc[rg][cg], 0, 0, 0);
                } else {
#pragma unroll
                    for (int rg = 0; rg < 2; ++rg) {
                        const float4 v = *reinterpret_cast<const float4*>(&cur_l[rb * 32 + 16 * rg + 4 * q4]);
                        const f32x4 init = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int cg = 0; cg < 4; ++cg)
                            acc[rg][cg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rg][0], sf[cg][0], init, 0, 0, 0);
                    }
#pragma unroll
                    for (int ks = 1; ks < 4; ++ks)
#pragma unroll
                        for (int cg = 0; cg < 4; ++cg)
#pragma unroll
                            for (int rg = 0; rg < 2; ++rg)
                                acc[rg][cg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rg][ks], sf[cg][ks], acc[rg][cg], 0, 0, 0);
                }
            };
            auto epilogue = [&](int rb) {
                const int xq = x0 + rb * 32 + 4 * q4;   // streamed index of entry i of acc[rg][.]: xq + 16*rg + i
                if (mask) {      // a scalar branch; both sides leave the prefetched fragments alone
                    const int sP[4] = {stationary_pos(0), stationary_pos(1), stationary_pos(2), stationary_pos(3)};
                    if (PASS == 1) lse_block_epilogue<true>(acc, scale2, xq, sP, m, l);
                    else colsum_block_epilogue<true>(acc, scale2, xq, sP, run);
                } else {
                    const int sP[4] = {0, 0, 0, 0};
                    if (PASS == 1) lse_block_epilogue<false>(acc, scale2, xq, sP, m, l);
                    else colsum_block_epilogue<false>(acc, scale2, xq, sP, run);
                }
            };
            // The two blocks as a loop: unrolled, neither pass fits into 168 VGPRs.  Pass 1, whose epilogue keeps
            // twice the state of pass 2's, holds only HALF of the next block's fragments (row group 0) during the
            // epilogue and asks for the other half after it.
            if (PASS == 1) {
                multiply(0);
                __builtin_amdgcn_sched_barrier(0);
                fetch_early(cur, 1);
                __builtin_amdgcn_sched_barrier(0);
                epilogue(0);
                __builtin_amdgcn_sched_barrier(0);
                fetch_late(cur, 1);
                __builtin_amdgcn_sched_barrier(0);
                multiply(1);
                __builtin_amdgcn_sched_barrier(0);
                finish_tile(false);
                __builtin_amdgcn_sched_barrier(0);
                epilogue(1);
                __builtin_amdgcn_sched_barrier(0);
                fetch_late(nxt, 0);
                __builtin_amdgcn_sched_barrier(0);
            } else {
#pragma unroll 1
                for (int rb = 0; rb < BX / 32; ++rb) {
                    multiply(rb);
                    __builtin_amdgcn_sched_barrier(0);
                    if (rb == 0) fetch(cur, 1);
                    else finish_tile(true);
                    __builtin_amdgcn_sched_barrier(0);
                    epilogue(rb);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
            finish_tile(true);
        }
    };
    for (int it = 0; it < n_it; it += 2) {
        tile_step(std::integral_constant<int, 0>{}, it);
        if (it + 1 < n_it) tile_step(std::integral_constant<int, 1>{}, it + 1);
    }

    // fold the four lanes (equal c16) that share a stationary row - the pairs (q4, q4 ^ 1) first, lower lane first,
    // then the two pairs - and write the chunk's partial for rows 0..255 of the strip
    float* pa = part_a + ((size_t)h * n_chunks_total * nSp + u) * BS;
    float* pb = part_b + ((size_t)h * n_chunks_total * nSp + u) * BS;
#pragma unroll
    for (int cg = 0; cg < 4; ++cg) {
        const int r = wave * 64 + cg * 16 + c16;
        if (PASS == 1) {
            float mm = m[cg], ll = l[cg];
#pragma unroll
            for (int step = 16; step <= 32; step <<= 1) {
                const bool upper = (lane & step) != 0;
                const float mo = __shfl_xor(mm, step), lo = __shfl_xor(ll, step);
                const float M = fmaxf(mm, mo);
                const float la = upper ? lo : ll, ma = upper ? mo : mm;   // the lower lane's values first
                const float lb = upper ? ll : lo, mb = upper ? mm : mo;
                ll = la * __builtin_amdgcn_exp2f(ma - M) + lb * __builtin_amdgcn_exp2f(mb - M);
                mm = M;
            }
            if (q4 == 0) { pa[r] = mm; pb[r] = ll; }
        } else {
            float v = run[cg];
#pragma unroll
            for (int step = 16; step <= 32; step <<= 1) {
                const float other = __shfl_xor(v, step);
                v = (lane & step) ? other + v : v + other;
            }
            if (q4 == 0) pa[r] = v;
        }
    }
}

// Folds the chunks of every strip, in chunk order: pass 1 -> lse2[h, i] = log2 sum_j 2^(c q_i.k_j) per query
// head; pass 2 -> scores[h, j] = A_s[j] per key head, the partials of its `group` query heads added in head
// order (group = 1: one query head per key head).  One thread per (head, row).  With key lists (pass 2 over the
// competing keys only) row r of strip t is the list's entry t * 256 + r and its score goes to that key's
// position; the workgroups nS .. 2 nS - 1 of the grid then write the inverse norms of the PROTECTED keys, which
// pass 2 no longer holds (summed in the order of the stand-alone norm kernel, so all three give the same bits).
template <int PASS>
__global__ void __launch_bounds__(256)
k_score_combine(int group, int L, int R0, int C, const float* __restrict__ part_a, const float* __restrict__ part_b,
                float* __restrict__ out, const int32_t* __restrict__ lists, const bf16_t* __restrict__ k,
                float* __restrict__ rnorm, int nS)
{
    const int h = blockIdx.y, r = threadIdx.x;
    int tile = blockIdx.x;
    if (PASS == 2 && lists != nullptr && tile >= nS) {
        // inverse norms of the protected keys: eight lanes per key, lane p summing the dims 8p .. 8p+7 and
        // 64+8p .. 64+8p+7 in order, then a pairwise tree over the lanes - the order of the stand-alone norm kernel
        if (rnorm == nullptr) return;
        const int NP = lists[1], sub = r & 7;
        for (int idx = (tile - nS) * 32 + (r >> 3); idx < NP; idx += 32 * nS) {     // uniform per group of eight lanes
            const int pos = lists[LIST_HEAD + L + idx];
            const bf16_t* row = k + ((size_t)h * L + pos) * SD;
            double ss = 0.0;
#pragma unroll
            for (int rep = 0; rep < 2; ++rep) {
                float v[8];
                load8(row + sub * 8 + rep * 64, v);
#pragma unroll
                for (int i = 0; i < 8; ++i) ss = fma((double)v[i], (double)v[i], ss);
            }
            ss += __shfl_xor(ss, 1);
            ss += __shfl_xor(ss, 2);
            ss += __shfl_xor(ss, 4);
            if (sub == 0) rnorm[(size_t)h * L + pos] = inverse_norm(ss);
        }
        return;
    }
    const bool sparse = PASS == 2 && lists != nullptr;
    int row = tile * BS + r;
    if (row >= (sparse ? lists[0] : L)) return;
    const int CT = C * BX, G = (L + CT - 1) / CT;
    int g0 = first_chunk(PASS, tile, CT, R0), nc = strip_chunks(PASS, tile, L, CT, R0);
    if (sparse) {
        g0 = max((lists[LIST_HEAD + tile * BS] / BX) * BX, (R0 / BX) * BX) / CT;    // as in k_score_mfma
        nc = G - g0;
        row = lists[LIST_HEAD + row];
    }
    if (nc == 0) return;     // pass 1 under a window: a strip with no row that counts (its values are never read)
    const int t_base = (PASS == 1) ? R0 / BS : 0, nSp = nS - t_base;   // as in k_score_mfma
    const size_t stride = (size_t)nSp * BS;     // from one chunk of a strip to the next
    const int h_first = (PASS == 1) ? h : h * group;      // first query head whose partials are read
    const float* pa = part_a + (((size_t)h_first * G + g0) * nSp + (tile - t_base)) * BS + r;
    const float* pb = part_b + (((size_t)h_first * G + g0) * nSp + (tile - t_base)) * BS + r;
    if (PASS == 1) {
        float M = -1e30f;
#pragma unroll 8   // the loads do not depend on each other: eight in flight
        for (int c = 0; c < nc; ++c) M = fmaxf(M, pa[c * stride]);
        float Ls = 0.f;
#pragma unroll 8
        for (int c = 0; c < nc; ++c) Ls = fmaf(pb[c * stride], exp2f(pa[c * stride] - M), Ls);
        out[(size_t)h * L + row] = M + log2f(Ls);
    } else {
        float sum = 0.f;
        for (int m = 0; m < group; ++m)
            for (int c = 0; c < nc; ++c) sum += pa[((size_t)m * G + c) * stride];
        out[(size_t)h * L + row] = sum;
    }
}

}  // namespace lookm

namespace lookm_host {

// tiles per chunk: aim at ~8 workgroups per resident slot (256 CUs x 3), at least 8 tiles per chunk
static int chunk_tiles(int H, int L)
{
    long total = 0;
    const int nS = (L + lookm::BS - 1) / lookm::BS;
    for (int t = 0; t < nS; ++t) total += (L - t * lookm::BS + lookm::BX - 1) / lookm::BX;
#ifndef LOOKM_UNITS_TARGET
#define LOOKM_UNITS_TARGET 6144
#endif
    long c = (total * H + LOOKM_UNITS_TARGET - 1) / LOOKM_UNITS_TARGET;
    return (int)(c < 8 ? 8 : (c > 256 ? 256 : c));
}

static int total_chunks(int pass, int L, int C, int R0)
{
    const int nS = (L + lookm::BS - 1) / lookm::BS;
    int u = 0;
    for (int t = 0; t < nS; ++t) u += lookm::strip_chunks(pass, t, L, C * lookm::BX, R0);
    return u;
}

// workgroups of one score pass: 8 XCD lanes x (units per lane), see the mapping at the top of k_score_mfma
static unsigned score_grid(int H, int U)
{
    if (H >= 8) return 8u * (unsigned)((H + 7) / 8) * (unsigned)U;
    const int xph = 8 / H;
    return 8u * (unsigned)((U + xph - 1) / xph);
}

// floats of scratch for the chunk partials: two arrays [H][chunks][strips][256]
size_t scores_mfma_scratch_floats(int H, int L)
{
    const int C = chunk_tiles(H, L), CT = C * lookm::BX;
    const int nS = (L + lookm::BS - 1) / lookm::BS, G = (L + CT - 1) / CT;
    return (size_t)2 * H * G * nS * lookm::BS;
}

// mask / M / lists: when given (the caller does not want the scores of the protected keys), pass 2 runs over the
// competing keys only; lists: device, 2 * L + LIST_HEAD ints
int launch_scores_mfma(const void* q, const void* k, int H, int kv_heads, int L, int d, int R0, float* lse,
                       const float* lse_in, float* scores, float* rnorm, float* scratch, const uint8_t* mask, int M,
                       int32_t* lists, hipStream_t st)
{
    if (d != lookm::SD) return LOOKM_ERR_UNSUPPORTED;
    const LaunchCheck check;
    const int group = H / kv_heads;
    const int nS = (L + lookm::BS - 1) / lookm::BS;
    const int C = chunk_tiles(H, L);
    const int G = (L + C * lookm::BX - 1) / (C * lookm::BX);
    // Pass 2 keeps the full problem's chunk length also under a window (its partial arrays keep their layout).
    // Pass 1 under a window runs only the last strips, each over all keys: shorter chunks give the chip enough
    // workgroups, as far as the partial arrays (sized for the full problem) hold them.
    int C1 = C;
    if (R0 > 0) {
        const int nS1 = nS - R0 / lookm::BS;
        const long want = (long)nS1 * ((L + lookm::BX - 1) / lookm::BX) * H / 2048;   // tiles per chunk for ~2048 units
        C1 = (int)std::min<long>(C, std::max<long>(4, want));
        while (C1 < C && (long)((L + C1 * lookm::BX - 1) / (C1 * lookm::BX)) * nS1 > (long)G * nS) ++C1;
    }
    const int U1 = total_chunks(1, L, C1, R0), U2 = total_chunks(2, L, C, R0);
    float* part_a = scratch;
    float* part_b = scratch + (size_t)H * G * nS * lookm::BS;
    const float scale2 = lookm::kLog2e / sqrtf((float)d);
    const lookm::bf16_t* qq = (const lookm::bf16_t*)q;
    const lookm::bf16_t* kk = (const lookm::bf16_t*)k;
    const bool sparse = mask != nullptr && lists != nullptr;
    if (!lse_in) {
        // with a mask the launch has one workgroup more: it builds the key lists while the others compute
        hipLaunchKernelGGL((lookm::k_score_mfma<1, false>), dim3(score_grid(H, U1) + (sparse ? 1u : 0u)), dim3(256), 0, st, qq, kk, H,
                           group, L, R0, scale2, C1, U1, lse, 1.0f, part_a, part_b, (float*)nullptr,
                           sparse ? mask : (const uint8_t*)nullptr, M, lists);
        mark(LOOKM_K_SCORE_LSE);
        hipLaunchKernelGGL(lookm::k_score_combine<1>, dim3(nS, H), dim3(256), 0, st, 1, L, R0, C1, part_a, part_b, lse,
                           (const int32_t*)nullptr, (const lookm::bf16_t*)nullptr, (float*)nullptr, nS);
        mark(LOOKM_K_SCORE_LSE_FOLD);
    } else if (sparse) {
        hipLaunchKernelGGL(lookm::k_score_lists, dim3(1), dim3(256), 0, st, mask, L, M, lists);
    }
    // a caller-supplied row log-sum-exp is natural-log: one factor log2(e) brings it to the kernels' base
    if (sparse)
        hipLaunchKernelGGL((lookm::k_score_mfma<2, true>), dim3(score_grid(H, U2)), dim3(256), 0, st, qq, kk, H, group, L,
                           R0, scale2, C, U2, lse_in ? lse_in : lse, (lse_in ? lookm::kLog2e : 1.0f) / scale2, part_a,
                           part_b, rnorm, (const uint8_t*)nullptr, M, lists);
    else
        hipLaunchKernelGGL((lookm::k_score_mfma<2, false>), dim3(score_grid(H, U2)), dim3(256), 0, st, qq, kk, H, group, L,
                           R0, scale2, C, U2, lse_in ? lse_in : lse, (lse_in ? lookm::kLog2e : 1.0f) / scale2, part_a,
                           part_b, rnorm, (const uint8_t*)nullptr, M, (int32_t*)nullptr);
    mark(LOOKM_K_SCORE_COLSUM);
    hipLaunchKernelGGL(lookm::k_score_combine<2>, dim3(sparse ? 2 * nS : nS, kv_heads), dim3(256), 0, st, group, L, R0, C,
                       part_a, part_b, scores, sparse ? (const int32_t*)lists : (const int32_t*)nullptr, kk, rnorm, nS);
    mark(LOOKM_K_SCORE_COLSUM_FOLD);
    return check.status();
}

}  // namespace lookm_host
