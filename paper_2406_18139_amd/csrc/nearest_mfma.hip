// Nearest conserved key by cosine similarity (Section 3.3, Eq. 9) on the gfx950 matrix cores:
// bf16 keys, head_dim 128.  Same machine as the score passes: a workgroup keeps the MFMA B-operand
// fragments of 256 evicted keys (gathered through the evicted index list) in registers and streams
// conserved keys (gathered through the kept index list) past them in 64-row LDS tiles as the A operand.
// A lane's 16 accumulator values are 16 conserved slots against ONE evicted key, so the running argmax
// is in-lane; the lane pair (lane, lane^32) is merged once after the loop.  The similarity matrix never
// exists in memory.
//
// Argmax without per-element compare/select chains: y = (k_e.k_c)/||k_c|| = cos * ||k_e|| orders the conserved
// keys of one evicted key like the cosine does, and the float bits of a positive y order like signed integers
// (every positive y beats every negative one; a row whose best y is not positive is decided by the exact pass
// below).  The low 4 mantissa bits of each entry are replaced by 15 - r (r = entry number inside the 32x32 block),
// and one tree of v_max3 / v_med3 per block yields the block's largest key - value and place at once - and its
// second largest.  Candidates are therefore compared at 20 mantissa bits (one unit = 16 ulp, at most 1.9e-6
// relative); equal keys still resolve to the lower slot exactly.  Across blocks, chunks and the lane pair the
// order is (truncated value descending, slot ascending), and the runner-up's key is carried along.
//
// Exact decisions.  The matrix-core value of y differs from the true one by a few ulp (fp32 accumulation of exact
// products, one inverse norm, one product; more, relative to y, the smaller the cosine: see near_units), so the true
// maximum can only be a key whose truncated value lies within a band of a few units below the best one - the
// band of the evicted key, which widens as its best cosine gets smaller.  Besides the best key, a lane
// therefore keeps (i) the largest runner-up INSIDE a 32x32 block it has seen and (ii) per block class (block
// number modulo the number of classes: 32, 16 or 8) a count of the blocks whose best value came within the band
// of its running best (all cleared whenever the best jumps by more than that, so that at the end the counters
// cover every block that can still hold a contender; counts rather than bits, because two such blocks may fall
// into one class).  k_nearest_fold takes the matrix-core choice where the winner's block is the only one counted
// and its runner-up inside the block is farther away; every other evicted key (one in six hundred at the headline
// shape) is decided again exactly: the slots of every block of the classes counted are evaluated in binary64 with
// a fixed arithmetic contract - sequential sums over k = 0..d-1 of products that are exact in binary64, binary64
// square roots, one product, one division, first maximum in slot order - which is a definition, not an
// approximation, so any implementation of the same contract takes the same decision.
//
// The conserved axis is cut into chunks (one workgroup per (evicted strip, chunk)) chosen so that the
// number of workgroups fills the resident slots evenly; enumeration is chunk-major and XCD-affine as in
// the score passes.
#include "common.h"

#include <algorithm>
#include <type_traits>

namespace lookm {

typedef __attribute__((ext_vector_type(8))) __bf16 nbf16x8;
typedef __attribute__((ext_vector_type(16))) float nf32x16;

constexpr int ND = 128, NBS = 256, NBX = 64, NXROW = 128;   // LDS rows are unpadded, chunks swizzled
static_assert(NBX == 64, "the norms of a tile are staged by wave 0, one row per lane");

// How far below the best truncated value a runner-up may lie and still has to be decided exactly: the band, in
// units of 16 ulp.  The error budget behind it, with u = 2^-24: y = fl(fl(k_e.k_c) * rnorm_c) = exact * (1 + delta);
// the matrix-core dot product is eight fp32 accumulations of partial sums bounded by sum |a_k b_k| <= |k_e||k_c|,
// so it is off by at most 8u / cos relative to the dot (measured over two million pairs: 4.1u / cos); the inverse
// norm, summed in binary64, by 2u; the product by u.  Two values that the kernels tell apart WITHOUT the exact pass
// have keys at least band + 1 units apart and therefore differ by more than 16 band ulp >= 16 band u relative,
// which must cover both errors: 2 (8u / cos + 3u) <= 16 band u, i.e. band >= 1 / cos + 0.375 - two units for the
// similar keys the method is about, more where a key has no similar conserved key.  `cos` may be any lower bound
// of the evicted key's best cosine: a wider band only sends more keys through the exact pass.  Below COS_MIN
// (band above NEAR_UNITS_MAX) every slot goes through it.
constexpr int NEAR_UNITS_MAX = 14;         // the runner-up distance in a partial saturates at 15
constexpr float COS_MIN = 0.08f;           // 1 / 0.08 + 1.376 < NEAR_UNITS_MAX + 1
__device__ __forceinline__ int near_units(float cos_lower_bound)
{
    // floor(x + 1) >= ceil(x); the factor covers the reciprocal's and the inverse norm's rounding; a NaN or a
    // value that is not positive fails the comparison
    const int nu = (int)(__frcp_rn(cos_lower_bound) * 1.0001f + 1.376f);
    return (cos_lower_bound > COS_MIN) ? min(nu, NEAR_UNITS_MAX) : NEAR_UNITS_MAX;
}

// partial result of one (evicted strip, chunk), the lane pair that shares an evicted key already merged:
//   key   (truncated value of the best conserved key) << 4 | how many units the best runner-up inside a block of the
//         winning lane lies below it (15 = fifteen or more)
//   slot  the best key's slot
//   marks per lane of the pair (first: slots 0-3 of every eight, second: slots 4-7) a word of 32 / w counters of
//         w bits: counter b = how many of the blocks b, b + 32 / w, ... of the chunk can hold a key within
//         the band (near_units) of the chunk's best value (a COUNT, so that two such blocks of one class are still seen
//         as two); zero for a lane whose own best value is farther away than that.  w = 1, 2 or 4 is the
//         narrowest width whose counters can count all blocks of a class (near_counter_bits): a chunk of up to
//         32 blocks has a class per block.
struct __attribute__((aligned(16))) NearestPartial {
    int32_t key;
    int32_t slot;
    uint32_t marks[2];
};
constexpr int NEAR_MAX_BLOCKS = 120;       // per chunk: eight 4-bit counters count 15 blocks each
constexpr int NEAR_MAX_CHUNKS = 9;         // LOOKM_MAX_L / 64 tiles in chunks of at most 60 tiles (120 blocks)

// counter width for a chunk of nb blocks: 32 classes of 1 bit, 16 of 2 bits (up to 3 blocks each) or 8 of 4 bits
__host__ __device__ inline int near_counter_bits(int nb) { return nb <= 32 ? 1 : nb <= 48 ? 2 : 4; }

// sum of the counters of a mark word
__device__ __forceinline__ int near_count(uint32_t m, int bits)
{
    if (bits == 1) return __popc(m);
    if (bits == 2) m = (m & 0x33333333u) + ((m >> 2) & 0x33333333u);    // pairs of counters: at most 6 per nibble
    return (int)((((m & 0x0f0f0f0fu) + ((m >> 4) & 0x0f0f0f0fu)) * 0x01010101u) >> 24);
}

__device__ __forceinline__ int imax3(int a, int b, int c) { return max(max(a, b), c); }
__device__ __forceinline__ int imed3(int a, int b, int c) { return max(min(a, b), min(max(a, b), c)); }

// largest and second largest of 16 distinct keys in 20 three-input operations: five triples give their maximum
// and their median; the largest key is the maximum of the maxima, and the runner-up is either the median of the
// triple (or of the group of maxima) that holds the largest key, or the best of the rest - all of which are below
// the largest key, so their maximum is the runner-up whichever group won.
__device__ __forceinline__ void top2_of_16(const int (&u)[16], int& first, int& second)
{
    const int m0 = imax3(u[0], u[1], u[2]), d0 = imed3(u[0], u[1], u[2]);
    const int m1 = imax3(u[3], u[4], u[5]), d1 = imed3(u[3], u[4], u[5]);
    const int m2 = imax3(u[6], u[7], u[8]), d2 = imed3(u[6], u[7], u[8]);
    const int m3 = imax3(u[9], u[10], u[11]), d3 = imed3(u[9], u[10], u[11]);
    const int m4 = imax3(u[12], u[13], u[14]), d4 = imed3(u[12], u[13], u[14]);
    const int a1 = imax3(m0, m1, m2), a2 = imed3(m0, m1, m2);
    const int b1 = imax3(m3, m4, u[15]), b2 = imed3(m3, m4, u[15]);
    first = max(a1, b1);
    second = max(imax3(d0, d1, d2), imax3(d3, d4, imax3(min(a1, b1), a2, b2)));
}

__global__ void __launch_bounds__(256, 3)
k_nearest_mfma(const bf16_t* __restrict__ k, const float* __restrict__ rnorm, const int32_t* __restrict__ kept,
               const int32_t* __restrict__ evicted, int H, int L, int B, int Le, int n_strips, int n_chunks, int CT,
               int cbits, NearestPartial* __restrict__ part)
{
    // Two tiles as separate arrays, and a tile loop unrolled by two with the buffer known at compile time: the
    // compiler then sees that a fragment read of one array cannot alias the loads in flight to the other and
    // does not wait for them (with one array indexed by a run-time buffer number it waits for every outstanding
    // load before the first LDS read of a tile, which serialises the prefetch with the MFMA block of the same wave).
    __shared__ __attribute__((aligned(16))) bf16_t xs0[NBX * NXROW];
    __shared__ __attribute__((aligned(16))) bf16_t xs1[NBX * NXROW];
    __shared__ __attribute__((aligned(16))) float xr0[NBX];
    __shared__ __attribute__((aligned(16))) float xr1[NBX];

    // XCD-affine enumeration (see k_score_mfma): units of a head are chunk-major
    const int U = n_strips * n_chunks;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    int h, e;
    if (H >= 8) {
        h = (j / U) * 8 + xcd;
        e = j % U;
    } else {
        const int xph = 8 / H;
        h = xcd / xph;
        e = j * xph + xcd % xph;
    }
    if (h >= H || e >= U) return;
    const int chunk = e / n_strips, strip = e % n_strips;

    k += (size_t)h * L * ND;
    rnorm += (size_t)h * L;
    kept += (size_t)h * B;
    evicted += (size_t)h * Le;
    // the wave number goes through a scalar register, so that what derives from it stays scalar
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, half = lane >> 5,
              n = lane & 31;
    const int w0 = strip * NBS + wave * 64;   // first evicted-list index of this wave

    // Evicted keys of this lane: positions first (list entries past the end of the list repeat its last entry; their
    // results land in partial slots that nothing reads), so that every load below is unconditional and the
    // prologue is two round trips to memory - positions, then rows - instead of one per branch.
    const int ev0 = min(w0 + n, Le - 1), ev1 = min(w0 + 32 + n, Le - 1);
    const int pos0 = evicted[ev0], pos1 = evicted[ev1];
    const float rn_e[2] = {rnorm[pos0], rnorm[pos1]};   // for the bands: cosine = y / |k_e|
    const int x_begin = chunk * CT, x_end = min(B, x_begin + CT);
    const int n_it = (x_end - x_begin + NBX - 1) / NBX;
    const int ld_row = tid >> 4, ld_chunk = tid & 15;
    // Conserved rows go from global memory straight into LDS (global_load_lds_dwordx4, as in the score passes): the
    // 64 lanes of a wave fill 1 KB = 4 consecutive LDS rows, lane l landing at chunk l%16 of row l/16, and fetch
    // chunk (l%16) ^ (row & 7) of their row, so that the fragment reads below are conflict-free without padding.
    // The gather is two dependent loads (position, then row); the positions are fetched one tile ahead of the rows
    // so that neither wait is exposed.  Slots past the end of the conserved list are staged as copies of the last
    // conserved key: they tie with it and lose on the slot rule.  (Index registers are plain scalars: an array
    // captured by a helper ended up in scratch memory.)
    float stage_r = 0.f;
    int ix0, ix1, ix2, ix3, ridx = 0;
#define LOOKM_LOAD_INDEX(x0)                                   \
    do {                                                       \
        ix0 = kept[min((x0) + ld_row, B - 1)];                 \
        ix1 = kept[min((x0) + ld_row + 16, B - 1)];            \
        ix2 = kept[min((x0) + ld_row + 32, B - 1)];            \
        ix3 = kept[min((x0) + ld_row + 48, B - 1)];            \
        if (wave == 0) ridx = kept[min((x0) + tid, B - 1)];    \
    } while (0)
    // a uniform base plus a 32-bit byte offset per lane (a position is below 2^15, a row 256 bytes); the 16 rows
    // between two pieces do not change row & 7, so the swizzled chunk is the same for all four
    const char* kb = reinterpret_cast<const char*>(k);
    const uint32_t chunk_off = (uint32_t)((ld_chunk ^ (ld_row & 7)) * 16);
#define LOOKM_ROW_TO_LDS(o, j, buf)                                                                               \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kb + (o)),                   \
                                     (__attribute__((address_space(3))) void*)&(buf)[((j)*4 + wave) * 4 * NXROW], 16,   \
                                     0, 0)
    // All four offsets are formed before the first load to LDS is issued (the empty asm keeps them together): once a
    // load to LDS is in flight next to ordinary loads the compiler waits for everything outstanding, which in the
    // prologue would be the 16 row loads of the stationary keys.
#define LOOKM_LOAD_TILE(buf)                                                                  \
    do {                                                                                      \
        const uint32_t o0 = (uint32_t)ix0 * (ND * 2) + chunk_off, o1 = (uint32_t)ix1 * (ND * 2) + chunk_off, \
                       o2 = (uint32_t)ix2 * (ND * 2) + chunk_off, o3 = (uint32_t)ix3 * (ND * 2) + chunk_off; \
        asm volatile("" ::"v"(o0), "v"(o1), "v"(o2), "v"(o3), "v"(ridx));                     \
        LOOKM_ROW_TO_LDS(o0, 0, buf);                                                         \
        LOOKM_ROW_TO_LDS(o1, 1, buf);                                                         \
        LOOKM_ROW_TO_LDS(o2, 2, buf);                                                         \
        LOOKM_ROW_TO_LDS(o3, 3, buf);                                                         \
        if (wave == 0) stage_r = rnorm[ridx];                                                 \
    } while (0)
    // x0: first slot of the tile that was loaded; slots past the end of the conserved list get inverse norm 0, so
    // their y is zero and they lose to every positive value (a row with no positive value is decided exactly)
#define LOOKM_STORE_TILE(rbuf, x0)                                       \
    do {                                                                 \
        if (wave == 0) (rbuf)[tid] = ((x0) + tid < B) ? stage_r : 0.f;   \
    } while (0)

    // element offsets of this lane's first four fragments inside its LDS row (swizzled chunks); scalars, not an array
    const int fo0 = ((0 + half) ^ (n & 7)) * 8, fo1 = ((2 + half) ^ (n & 7)) * 8, fo2 = ((4 + half) ^ (n & 7)) * 8,
              fo3 = ((6 + half) ^ (n & 7)) * 8;

    // per stationary row of this lane; the initial state is below every key and decodes to slot 0
    constexpr int KEY_MIN = (int)0x80000000;
    // the band of each of this lane's two evicted keys, in keys (whose low 4 bits are tags): from the running best
    // value, so it starts at its widest and narrows as better keys appear (a band wider than needed is harmless)
    int near_key[2] = {(NEAR_UNITS_MAX << 4) + 15, (NEAR_UNITS_MAX << 4) + 15};
    int bkey[2] = {KEY_MIN | 15, KEY_MIN | 15};   // best key (low 4 bits: 15 - entry number)
    int bsec[2] = {KEY_MIN, KEY_MIN};             // largest runner-up inside one block
    int bxb[2] = {0, 0};                          // slot of entry 0 of the block the best key came from
    uint32_t bnear[2] = {0u, 0u};                 // per block class, how many blocks can still hold a contender
    const int cls_mask = 32 / cbits - 1;          // classes are block numbers modulo their count

    LOOKM_LOAD_INDEX(x_begin);           // in flight together with the evicted positions

    nbf16x8 sf[2][8];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int pos = cb ? pos1 : pos0;
        const bf16_t* row = k + (size_t)pos * ND;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            sf[cb][ks] = __builtin_bit_cast(nbf16x8, *reinterpret_cast<const uint4*>(row + ks * 16 + half * 8));
    }
    LOOKM_LOAD_TILE(xs0);
    LOOKM_LOAD_INDEX(x_begin + NBX);     // clamped, so always in range
    LOOKM_STORE_TILE(xr0, x_begin);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the direct-to-LDS loads have landed
    __syncthreads();

    auto tile_step = [&](auto buf_tag, int it) {
        constexpr int BUF = decltype(buf_tag)::value;
        bf16_t* cur = BUF ? xs1 : xs0;
        bf16_t* nxt = BUF ? xs0 : xs1;
        float* cur_r = BUF ? xr1 : xr0;
        float* nxt_r = BUF ? xr0 : xr1;
        const int x0 = x_begin + it * NBX;
        if (it + 1 < n_it) {
            LOOKM_LOAD_TILE(nxt);                // rows of tile it+1 (positions fetched one iteration ago)
            LOOKM_LOAD_INDEX(x0 + 2 * NBX);      // positions of tile it+2
        }
        // The bands follow the running best values: after the first tile, where the best moves most, then every
        // fourth tile (the lower edge of the best key's truncation interval is a lower bound of y).
        if (it == 1 || (it > 0 && (it & 3) == 0)) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
                near_key[cb] = (near_units(__uint_as_float((uint32_t)bkey[cb] & 0xfffffff0u) * rn_e[cb]) << 4) + 15;
        }
#pragma unroll 1
        for (int rb = 0; rb < 2; ++rb) {
            nbf16x8 a[8];
            const bf16_t* ap = &cur[(rb * 32 + n) * NXROW];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {   // chunk (2*(ks+4) + half) ^ (n & 7) lies 8 chunks after that of ks
                const int fo = (ks == 0) ? fo0 : (ks == 1) ? fo1 : (ks == 2) ? fo2 : fo3;
                a[ks] = __builtin_bit_cast(nbf16x8, *reinterpret_cast<const uint4*>(ap + fo));
                a[ks + 4] = __builtin_bit_cast(nbf16x8, *reinterpret_cast<const uint4*>(ap + fo + 64));
            }
            nf32x16 acc[2];
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[0][r] = 0.f; acc[1][r] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], sf[0][ks], acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], sf[1][ks], acc[1], 0, 0, 0);
            }
            const int xb = x0 + rb * 32 + 4 * half;   // slot of entry r: xb + 8*(r/4) + r%4
            const uint32_t blk_one = 1u << (cbits * ((2 * it + rb) & cls_mask));   // one in this block's counter
            const float* rp = &cur_r[rb * 32 + 4 * half];
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                int u[16];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 rv = *reinterpret_cast<const float4*>(rp + 8 * g);
                    const float rn[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int r = 4 * g + i;
                        // y = (k_e.k_c) * rnorm_c (a zero evicted key gives 0 everywhere: decided exactly, slot 0)
                        const float y = acc[cb][r] * rn[i];
                        u[r] = (int)((__float_as_uint(y) & 0xfffffff0u) | (uint32_t)(15 - r));
                    }
                }
                int bm, bs2;
                top2_of_16(u, bm, bs2);
                const bool better = (bm >> 4) > (bkey[cb] >> 4);   // strict: an equal value in a later block loses
                // a jump by more than the band leaves every earlier block out of reach; a block within the band of
                // the running best (from either side) stays a candidate
                const int ahead = __builtin_elementwise_sub_sat(bm, bkey[cb]);   // saturating: the first block's lead is huge
                bnear[cb] = (ahead > near_key[cb]) ? 0u : bnear[cb];
                bnear[cb] += (ahead >= -near_key[cb]) ? blk_one : 0u;   // cannot overflow: see near_counter_bits
                bsec[cb] = max(bsec[cb], bs2);
                bkey[cb] = better ? bm : bkey[cb];
                bxb[cb] = better ? xb : bxb[cb];
            }
        }
        if (it + 1 < n_it) LOOKM_STORE_TILE(nxt_r, x0 + NBX);
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): the next tile's direct-to-LDS loads have landed
        __syncthreads();
    };
    for (int it = 0; it < n_it; it += 2) {
        tile_step(std::integral_constant<int, 0>{}, it);
        if (it + 1 < n_it) tile_step(std::integral_constant<int, 1>{}, it + 1);
    }
#undef LOOKM_ROW_TO_LDS
#undef LOOKM_LOAD_INDEX
#undef LOOKM_LOAD_TILE
#undef LOOKM_STORE_TILE

    NearestPartial* out = part + (((size_t)h * n_chunks + chunk) * n_strips + strip) * NBS;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int r = 15 - (bkey[cb] & 15);
        int slot = bxb[cb] + 8 * (r >> 2) + (r & 3);
        int hi = bkey[cb] >> 4, sec = bsec[cb] >> 4;
        uint32_t mine = bnear[cb];
        const int ohi = __shfl_xor(hi, 32), oslot = __shfl_xor(slot, 32), osec = __shfl_xor(sec, 32);
        uint32_t theirs = (uint32_t)__shfl_xor((int)mine, 32);
        const bool other = ohi > hi || (ohi == hi && oslot < slot);
        // the losing lane's blocks only matter if its best value is within the band of the winner's
        const int band = max(near_key[cb], __shfl_xor(near_key[cb], 32)) >> 4;   // the wider of the pair's bands
        if (other) mine = (hi >= ohi - band) ? mine : 0u;
        else theirs = (ohi >= hi - band) ? theirs : 0u;
        if (other) { hi = ohi; slot = oslot; sec = osec; }
        if (half == 0) {
            NearestPartial p;
            p.key = (int)(((uint32_t)hi << 4) | (uint32_t)min(hi - sec, 15));   // sec <= hi
            p.slot = slot;
            p.marks[0] = mine;
            p.marks[1] = theirs;
            out[wave * 64 + cb * 32 + n] = p;
        }
    }
}

// cosine of two keys under the exact contract: sequential binary64 sums over k = 0..127 (every product of two
// bf16 values is exact in binary64, so a fused multiply-add gives the same bits as multiply-then-add), binary64
// square roots (correctly rounded), one product, one division; 0 when either norm vanishes.  Both rows come from
// global memory an eighth at a time, the next eighth in flight while one is summed (a loop, not unrolled
// further: this runs on a handful of threads per call).
__device__ __forceinline__ double cosine_exact(const bf16_t* __restrict__ a, const bf16_t* __restrict__ b)
{
    double na = 0.0, nb = 0.0, ab = 0.0;
    uint4 an[2], bn[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        an[j] = *reinterpret_cast<const uint4*>(a + 8 * j);
        bn[j] = *reinterpret_cast<const uint4*>(b + 8 * j);
    }
    // a row is two cache lines: the second ones are asked for now, so that only one memory latency is paid per row
    uint4 a_mid = *reinterpret_cast<const uint4*>(a + 64), b_mid = *reinterpret_cast<const uint4*>(b + 64);
#pragma unroll 1
    for (int q = 0; q < 8; ++q) {
        uint4 ac[2], bc[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) { ac[j] = an[j]; bc[j] = bn[j]; }
        if (q < 7) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                an[j] = *reinterpret_cast<const uint4*>(a + 16 * (q + 1) + 8 * j);
                bn[j] = *reinterpret_cast<const uint4*>(b + 16 * (q + 1) + 8 * j);
            }
            if (q == 3) { an[0] = a_mid; bn[0] = b_mid; }      // element 64: already here
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t aw[4] = {ac[j].x, ac[j].y, ac[j].z, ac[j].w}, bw[4] = {bc[j].x, bc[j].y, bc[j].z, bc[j].w};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const double xa = (double)__uint_as_float((i & 1) ? (aw[i >> 1] & 0xffff0000u) : (aw[i >> 1] << 16));
                const double yb = (double)__uint_as_float((i & 1) ? (bw[i >> 1] & 0xffff0000u) : (bw[i >> 1] << 16));
                na = fma(xa, xa, na);
                nb = fma(yb, yb, nb);
                ab = fma(xa, yb, ab);
            }
            // the three sums advance together (left alone, the compiler finishes one sum before it starts the next
            // and keeps every widened value alive in between, which spills)
            asm volatile("" : "+v"(na), "+v"(nb), "+v"(ab));
        }
    }
    if (na == 0.0 || nb == 0.0) return 0.0;
    return ab / (sqrt(na) * sqrt(nb));
}

constexpr int NF_THREADS = 256;
constexpr int NF_ITEMS = 768;     // (evicted key, candidate slot) pairs evaluated exactly per round of a workgroup
constexpr int NF_GROUPS = NF_ITEMS / 16;
constexpr int NF_LDS_CHUNKS = 4;  // chunks whose block masks the fold keeps in LDS (further chunks are read again)

// Folds the chunks of every evicted key (value descending, slot ascending): one thread per evicted key.  Where
// the winner's block is the only marked block of all chunks whose best value is within the key's band of the
// overall best, and the winner's lane saw no runner-up inside a block within that distance, the matrix-core choice
// stands: assign[h, e] = its slot, sim[h, e] = the cosine decoded from the centre of the key's truncation interval
// (|error| < 1.2e-6).  The other keys of the workgroup are decided exactly, together: their threads list the slots
// of the marked blocks as (key, slot) items in LDS, every thread of the workgroup evaluates items with
// cosine_exact and folds the result into its key's maximum (LDS atomics: the largest cosine, then the lowest slot
// that reaches it = the first maximum in slot order).  A key
// whose best value is not positive (integer order of the bits is not float order there), or whose best cosine is
// below COS_MIN, takes every slot.
// (few registers and little LDS on purpose: all workgroups of the headline shape are resident at once, so the
// kernel takes as long as its slowest workgroup, not twice that)
template <int cbits>   // counter width of the mark words (near_counter_bits of the chunk length)
__global__ void __launch_bounds__(NF_THREADS, 6)
k_nearest_fold(const bf16_t* __restrict__ k, const float* __restrict__ rnorm, const int32_t* __restrict__ kept,
               const int32_t* __restrict__ evicted, int L, int B, int Le, int n_strips, int n_chunks, int CT,
               const NearestPartial* __restrict__ part, int32_t* __restrict__ assign, float* __restrict__ sim)
{
    // items come in groups of 16 (the slots one lane holds of a 32x32 block, or 16 consecutive slots)
    __shared__ int grp_pos_e[NF_GROUPS];      // position of the group's evicted key, or -1 for an empty entry
    __shared__ int grp_first[NF_GROUPS];      // first slot (below 2^15) | owner thread << 16 | consecutive slots << 24
    __shared__ int grp_limit[NF_GROUPS];      // slots from here on do not exist
    __shared__ unsigned long long item_s[NF_ITEMS];    // the item's cosine, as an integer of the same order
    __shared__ unsigned long long best_s[NF_THREADS];  // per owner thread: the largest such integer ...
    __shared__ int best_r[NF_THREADS];                 // ... and the lowest slot that reaches it
    __shared__ uint2 near_m[NF_LDS_CHUNKS][NF_THREADS];      // block counters per key and chunk (both lanes'); 0: chunk out of reach
    __shared__ int n_groups;
    const int h = blockIdx.y, tid = threadIdx.x;
    k += (size_t)h * L * ND;
    rnorm += (size_t)h * L;
    kept += (size_t)h * B;
    evicted += (size_t)h * Le;
    assign += (size_t)h * Le;
    sim += (size_t)h * Le;
    const int ev = blockIdx.x * NF_THREADS + tid;

    bool pending = false;                     // this thread's key still needs the exact decision
    bool all_slots = false;                   // ... over every slot: its best value is too small to trust any order
    int pos_e = 0, bk = 0, band = NEAR_UNITS_MAX;
    const NearestPartial* mine = part;        // this key's partial of chunk 0; chunk c is n_strips * NBS entries further
    if (ev < Le) {
        pos_e = evicted[ev];
        mine = part + ((size_t)h * n_chunks * n_strips + ev / NBS) * NBS + ev % NBS;
        int key[NEAR_MAX_CHUNKS], bs = 0x7fffffff, bd = 15, marks[NEAR_MAX_CHUNKS];
        bk = (int)0x80000000;
#pragma unroll
        for (int c = 0; c < NEAR_MAX_CHUNKS; ++c) {
            key[c] = (int)0x80000000;
            marks[c] = 0;
            if (c < n_chunks) {
                const NearestPartial p = mine[(size_t)c * n_strips * NBS];
                key[c] = p.key >> 4;
                marks[c] = near_count(p.marks[0], cbits) + near_count(p.marks[1], cbits);
                if (c < NF_LDS_CHUNKS) near_m[c][tid] = make_uint2(p.marks[0], p.marks[1]);
                if (key[c] > bk || (key[c] == bk && p.slot < bs)) { bk = key[c]; bs = p.slot; bd = p.key & 15; }
            }
        }
        // this key's band, from the lower edge of its best key's truncation interval
        const float rn_e = rnorm[pos_e], cos_low = __uint_as_float((uint32_t)bk << 4) * rn_e;
        band = near_units(cos_low);
        int marked = 0;
#pragma unroll
        for (int c = 0; c < NEAR_MAX_CHUNKS; ++c) {
            const bool reach = key[c] >= bk - band;                // chunks within reach only
            marked += reach ? marks[c] : 0;
            if (c < NF_LDS_CHUNKS && c < n_chunks && !reach) near_m[c][tid] = make_uint2(0u, 0u);
        }
        // the best value is zero or negative (the integer order of the bits is not the order of the values there),
        // or the best cosine is so small that the rounding errors of the dot products, which grow like 1 / cos in
        // units of the value, may exceed the band: every slot is a candidate then
        const float y = __uint_as_float(((uint32_t)bk << 4) | 8u);         // (k_e.k_c) * rnorm_c, centre of the interval
        const float cos_best = y * rn_e;
        all_slots = bk <= 0 || !(cos_low > COS_MIN);
        pending = all_slots || bd <= band || marked > 1;
        if (!pending) {
            assign[ev] = min(max(bs, 0), B - 1);
            sim[ev] = cos_best;
        }
    }
    if (!__syncthreads_or(pending)) return;

    // The block counters of chunk c for this thread's key (zero when the chunk is out of reach).
    auto chunk_marks = [&](int c, uint32_t (&m)[2]) {
        if (c < NF_LDS_CHUNKS) {
            const uint2 both = near_m[c][tid];
            m[0] = both.x;
            m[1] = both.y;
        } else {                                                       // more chunks than LDS holds: read again
            const NearestPartial p = mine[(size_t)c * n_strips * NBS];
            const bool reach = (p.key >> 4) >= bk - band;
            m[0] = reach ? p.marks[0] : 0u;
            m[1] = reach ? p.marks[1] : 0u;
        }
    };
    // Walks through the candidate slots of this thread's key in groups of 16: the slots this lane half holds of
    // every marked block of every chunk within reach (first slot f: f + 8 * (g / 4) + g % 4, g = 0..15), or runs of
    // 16 consecutive slots over the whole list when the best value is not positive.  A non-zero counter b stands
    // for the blocks b, b + n_cls, ... of the chunk, all of which are visited.  visit(first, limit, consecutive).
    constexpr int n_cls = 32 / cbits, cls_shift = cbits >> 1;  // counter number = bit number >> cls_shift
    constexpr uint32_t field = (1u << cbits) - 1u;
    auto for_each_group = [&](auto&& visit) {
        if (all_slots) {
            for (int s = 0; s < B; s += 16) visit(s, B, 1);
            return;
        }
        for (int c = 0; c < n_chunks; ++c) {
            uint32_t m[2];
            chunk_marks(c, m);
            const int lo = c * CT, hi = min(B, lo + CT);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                for (uint32_t rest = m[half]; rest != 0u;) {
                    const int cls = (__ffs((int)rest) - 1) >> cls_shift;
                    rest &= ~(field << (cbits * cls));
                    for (int b = cls; lo + 32 * b < hi; b += n_cls) visit(lo + 32 * b + 4 * half, hi, 0);
                }
            }
        }
    };
    auto group_slot = [](int first, int consecutive, int g) {
        return consecutive ? first + g : first + 8 * (g >> 2) + (g & 3);
    };
    int cnt = 0;                                  // groups of this thread's key
    if (pending) {
        if (all_slots) cnt = (B + 15) / 16;
        else
            for (int c = 0; c < n_chunks; ++c) {
                uint32_t m[2];
                chunk_marks(c, m);
                const int nb = (min(B, (c + 1) * CT) - c * CT + 31) / 32;      // blocks of this chunk
#pragma unroll
                for (int half = 0; half < 2; ++half)
                    for (uint32_t rest = m[half]; rest != 0u;) {
                        const int cls = (__ffs((int)rest) - 1) >> cls_shift;
                        rest &= ~(field << (cbits * cls));
                        cnt += (cls < nb) ? (nb - cls + n_cls - 1) / n_cls : 0;
                    }
            }
    }
    // binary64 values as unsigned integers of the same order (x < y <=> key(x) < key(y); no cosine is -0.0: the sums
    // start at +0.0), so that the maximum over a key's items is one LDS atomic per item
    auto ordered = [](double x) -> unsigned long long {
        const unsigned long long b = (unsigned long long)__double_as_longlong(x);
        return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
    };
    auto unordered = [](unsigned long long u) -> double {
        return __longlong_as_double((long long)((u >> 63) ? (u & 0x7fffffffffffffffull) : ~u));
    };
    while (true) {
        if (tid < NF_GROUPS) grp_pos_e[tid] = -1;
        best_s[tid] = 0ull;                   // below the image of every number
        best_r[tid] = 0x7fffffff;
        if (tid == 0) n_groups = 0;
        __syncthreads();
        // keys whose groups fit into this round's list write them (whoever reserves first always fits if its count
        // is at most the capacity; the order of the reservations decides no result): a few LDS stores per key -
        // the slots of a group and their conserved positions are worked out by the threads that evaluate them
        int base = -1;
        if (pending && cnt <= NF_GROUPS) {
            base = atomicAdd(&n_groups, cnt);
            if (base + cnt > NF_GROUPS) base = -1;
        }
        if (base >= 0) {
            int at = base;
            for_each_group([&](int first, int limit, int consecutive) {
                grp_pos_e[at] = pos_e;
                grp_first[at] = first | (tid << 16) | (consecutive << 24);
                grp_limit[at] = limit;
                ++at;
            });
        }
        __syncthreads();
        const int n = 16 * min(n_groups, NF_GROUPS);
        for (int i = tid; i < n; i += NF_THREADS) {
            const int e = i >> 4, pe = grp_pos_e[e], packed = grp_first[e];
            const int slot = group_slot(packed & 0xffff, packed >> 24, i & 15);
            const bool valid = pe >= 0 && slot < grp_limit[e];
            unsigned long long c = 0ull;      // an item that does not exist is below every cosine
            if (valid) {
                c = ordered(cosine_exact(k + (size_t)pe * ND, k + (size_t)kept[slot] * ND));
                atomicMax(&best_s[(packed >> 16) & 0xff], c);
            }
            item_s[i] = c;
        }
        __syncthreads();
        for (int i = tid; i < n; i += NF_THREADS) {       // first maximum in slot order: the lowest slot that reaches it
            const unsigned long long c = item_s[i];
            if (c != 0ull) {
                const int packed = grp_first[i >> 4], owner = (packed >> 16) & 0xff;
                if (c == best_s[owner]) atomicMin(&best_r[owner], group_slot(packed & 0xffff, packed >> 24, i & 15));
            }
        }
        __syncthreads();
        if (base >= 0) {
            assign[ev] = (best_r[tid] == 0x7fffffff) ? 0 : best_r[tid];
            sim[ev] = (best_r[tid] == 0x7fffffff) ? 0.f : (float)unordered(best_s[tid]);
            pending = false;
        } else if (pending && cnt > NF_GROUPS) {
            // more candidates than a round holds (many keys of equal direction): this thread walks through them alone
            double top_s = 0.0;
            int top_r = 0x7fffffff;
            for_each_group([&](int first, int limit, int consecutive) {
                for (int g = 0; g < 16; ++g) {
                    const int sl = group_slot(first, consecutive, g);
                    if (sl >= limit) continue;
                    const double c = cosine_exact(k + (size_t)pos_e * ND, k + (size_t)kept[sl] * ND);
                    if (top_r == 0x7fffffff || c > top_s || (c == top_s && sl < top_r)) { top_s = c; top_r = sl; }
                }
            });
            assign[ev] = (top_r == 0x7fffffff) ? 0 : top_r;
            sim[ev] = (float)top_s;
            pending = false;
        }
        if (!__syncthreads_or(pending)) break;
    }
}

}  // namespace lookm

namespace lookm_host {

// chunks of the conserved axis: the count (at most 8, at least 4 tiles each) whose workgroup total fills
// the resident slots (256 CUs x 3) most evenly - more if a chunk would otherwise hold more blocks of one class
// than a mark counter can count
static int nearest_chunks(int H, int Le, int B)
{
    const int strips = (Le + lookm::NBS - 1) / lookm::NBS, tiles = (B + lookm::NBX - 1) / lookm::NBX;
    int best = 1;
    double best_eff = 0.0;
    for (int c = 1; c <= 8 && (c == 1 || tiles / c >= 4); ++c) {
        const long units = (long)strips * c * H;
        const double eff = (double)units / (double)(((units + 767) / 768) * 768);
        if (eff > best_eff + 0.02) { best_eff = eff; best = c; }
    }
    // A chunk of at most 32 blocks has a mark class per block, so the exact pass looks at contenders only, not at
    // whole classes of blocks: worth more chunks if they fill the machine as evenly.
    auto blocks = [&](int c) { return 2 * ((tiles + c - 1) / c); };   // two blocks per tile
    if (blocks(best) > 32)
        for (int c = best + 1; c <= 8 && tiles / c >= 4; ++c) {
            const long units = (long)strips * c * H;
            const double eff = (double)units / (double)(((units + 767) / 768) * 768);
            if (blocks(c) <= 32 && eff >= best_eff - 0.02) { best = c; break; }
        }
    while (blocks(best) > lookm::NEAR_MAX_BLOCKS) ++best;
    return best;
}

size_t nearest_mfma_scratch_bytes(int H, int L, int B)
{
    const int Le = L - B;
    if (Le <= 0 || B <= 0) return 0;
    const int strips = (Le + lookm::NBS - 1) / lookm::NBS;
    return (size_t)H * nearest_chunks(H, Le, B) * strips * lookm::NBS * sizeof(lookm::NearestPartial);
}

int launch_nearest_mfma(const void* k, const int32_t* kept, const int32_t* evicted, int H, int L, int budget,
                        const float* rnorm, int32_t* assign, float* sim, void* scratch, hipStream_t st)
{
    const LaunchCheck check;
    const int B = budget, Le = L - B;
    const int strips = (Le + lookm::NBS - 1) / lookm::NBS, tiles = (B + lookm::NBX - 1) / lookm::NBX;
    const int nc = nearest_chunks(H, Le, B);
    const int CT = ((tiles + nc - 1) / nc) * lookm::NBX;        // conserved slots per chunk
    const int n_chunks = (B + CT - 1) / CT;
    if (n_chunks > lookm::NEAR_MAX_CHUNKS) return LOOKM_ERR_UNSUPPORTED;   // cannot happen for L <= LOOKM_MAX_L
    const int U = strips * n_chunks;
    const int cbits = lookm::near_counter_bits(CT / 32);        // blocks of a full chunk
    unsigned grid;
    if (H >= 8) grid = 8u * (unsigned)((H + 7) / 8) * (unsigned)U;
    else { const int xph = 8 / H; grid = 8u * (unsigned)((U + xph - 1) / xph); }
    lookm::NearestPartial* part = (lookm::NearestPartial*)scratch;
    const lookm::bf16_t* kk = (const lookm::bf16_t*)k;
    hipLaunchKernelGGL(lookm::k_nearest_mfma, dim3(grid), dim3(256), 0, st, kk, rnorm, kept, evicted, H, L, B, Le, strips,
                       n_chunks, CT, cbits, part);
    mark(LOOKM_K_NEAREST);
    const dim3 fold_grid((Le + lookm::NF_THREADS - 1) / lookm::NF_THREADS, H);
#define LOOKM_FOLD(W)                                                                                                  \
    hipLaunchKernelGGL(lookm::k_nearest_fold<W>, fold_grid, dim3(lookm::NF_THREADS), 0, st, kk, rnorm, kept, evicted, \
                       L, B, Le, strips, n_chunks, CT, part, assign, sim)
    if (cbits == 1) LOOKM_FOLD(1);
    else if (cbits == 2) LOOKM_FOLD(2);
    else LOOKM_FOLD(4);
#undef LOOKM_FOLD
    mark(LOOKM_K_NEAREST_FOLD);
    return check.status();
}

}  // namespace lookm_host
