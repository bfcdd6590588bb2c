// Shared device-side helpers for the LOOK-M kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lookm.h"

namespace lookm {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round-to-nearest-even fp32 -> bf16; NaN stays a quiet NaN
__device__ __forceinline__ bf16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct elem;
template <> struct elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16_rne(v); }
};

// 8 consecutive elements -> 8 floats (one 16-byte load for bf16, two for fp32); p 16-byte aligned
__device__ __forceinline__ void load8(const float* p, float (&o)[8])
{
    float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float (&o)[8])
{
    uint4 a = *reinterpret_cast<const uint4*>(p);
    o[0] = __uint_as_float(a.x << 16); o[1] = __uint_as_float(a.x & 0xffff0000u);
    o[2] = __uint_as_float(a.y << 16); o[3] = __uint_as_float(a.y & 0xffff0000u);
    o[4] = __uint_as_float(a.z << 16); o[5] = __uint_as_float(a.z & 0xffff0000u);
    o[6] = __uint_as_float(a.w << 16); o[7] = __uint_as_float(a.w & 0xffff0000u);
}
// 1 / sqrt(sum of squares), 0 for a zero key: binary64 square root and division, one rounding to fp32 at the end
__device__ __forceinline__ float inverse_norm(double sum_of_squares)
{
    return (sum_of_squares > 0.0) ? (float)(1.0 / sqrt(sum_of_squares)) : 0.f;
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8])
{
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8])
{
    uint4 a;
    a.x = (uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16);
    a.y = (uint32_t)f32_to_bf16_rne(v[2]) | ((uint32_t)f32_to_bf16_rne(v[3]) << 16);
    a.z = (uint32_t)f32_to_bf16_rne(v[4]) | ((uint32_t)f32_to_bf16_rne(v[5]) << 16);
    a.w = (uint32_t)f32_to_bf16_rne(v[6]) | ((uint32_t)f32_to_bf16_rne(v[7]) << 16);
    *reinterpret_cast<uint4*>(p) = a;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// number of set bits of a 64-bit wave mask below this lane
__device__ __forceinline__ int mask_rank(uint64_t m)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

constexpr float kLog2e = 1.4426950408889634f;

}  // namespace lookm

// host-side launch plumbing shared by the stage launchers (api.hip owns validation)
namespace lookm_host {

// lse_in: optional caller-supplied natural-log row log-sum-exp [H, L]; when given, pass 1 is skipped
// rnorm: optional [H, L]; the matrix-core path (see scores_write_rnorm) fills it with 1/||k row|| on the way
// first_row: only the query rows first_row .. L-1 are summed (0 = all rows, Eq. 4 as printed)
// H query heads in groups of H / kv_heads that read one key head each (kv_heads = H: plain multi-head attention);
// lse, lse_in: [H, L]; scores, rnorm: [kv_heads, L]
// mask, M, lists (all or none): the caller only needs the scores of the keys that compete in the selection (image
// tokens before the recent window); the matrix-core path then skips the other keys in pass 2 and leaves their
// entries of `scores` unwritten (the portable path computes every score regardless).  lists: device scratch of
// score_list_ints(L) ints.
int launch_scores(const void* q, const void* k, int H, int kv_heads, int L, int d, lookm_dtype dt, int first_row,
                  float* lse, const float* lse_in, float* scores, float* rnorm, float* scratch, const uint8_t* mask, int M,
                  int32_t* lists, hipStream_t st);
inline size_t score_list_ints(int L) { return (size_t)2 * L + 64; }
inline bool scores_write_rnorm(int d, lookm_dtype dt) { return dt == LOOKM_BF16 && d == 128; }
size_t scores_scratch_floats(int H, int L, int d, lookm_dtype dt);
int launch_select(const float* scores, const uint8_t* mask, int H, int L, int budget, int M, int rule, int32_t* kept,
                  int32_t* evicted, int32_t* status, hipStream_t st);
// rnorm_ready: rnorm already holds the inverse key norms (written by launch_scores)
int launch_nearest(const void* k, const int32_t* kept, const int32_t* evicted, int H, int L, int d, lookm_dtype dt,
                   int budget, float* rnorm, bool rnorm_ready, int32_t* assign, float* sim, void* scratch,
                   hipStream_t st);
size_t nearest_scratch_bytes(int H, int L, int d, lookm_dtype dt, int budget);
int launch_merge(const void* k, const void* v, const int32_t* kept, const int32_t* evicted, const int32_t* assign,
                 const float* sim, int H, int L, int d, lookm_dtype dt, int budget, int mode, int32_t* plan_words,
                 int32_t* member_pos, float* member_w, void* k_out, void* v_out, hipStream_t st);

int launch_decode(const void* q, const void* k, const void* v, int H, int rows, int S, int d, lookm_dtype dt, void* out,
                  float* part, hipStream_t st);
size_t decode_scratch_bytes(int H, int d);
size_t decode_partial_bytes(int H, int S, int d);
int decode_static_scratch_setup();     // once per device: resolves the device address of the static scratch array
float* decode_static_scratch();        // that address for the current device (null before the set-up)

inline int hip_ok(hipError_t e) { return e == hipSuccess ? LOOKM_OK : LOOKM_ERR_DEVICE; }

// A launcher's verdict on its own launches: an error that is pending on this host thread after them and was not
// pending before.  Nothing is cleared, so an error that an unrelated earlier call left behind is neither taken
// for a failed launch nor hidden from the caller.
struct LaunchCheck {
    hipError_t before;
    LaunchCheck() : before(hipPeekAtLastError()) {}
    int status() const
    {
        const hipError_t after = hipPeekAtLastError();
        return (after == hipSuccess || after == before) ? LOOKM_OK : LOOKM_ERR_DEVICE;
    }
};

// Kernels that need more dynamic LDS than the default limit get the attribute set for EVERY template instance,
// once per device, by ensure_device_ready() (api.hip) - never lazily per instance, so that a shape met for the
// first time inside a stream capture finds its kernel ready.  Each returns LOOKM_OK or LOOKM_ERR_DEVICE.
int set_attributes_score_generic();
int set_attributes_nearest_generic();
int set_attributes_merge();
int ensure_device_ready();

// Per-kernel timing for lookm_compress_profile: when a timer is installed, every launcher records an
// event after each kernel it enqueues (ids follow the LOOKM_K_* order of the header).
struct KernelTimer {
    hipEvent_t ev[LOOKM_N_KERNELS + 1];
    hipStream_t st;
};
extern thread_local KernelTimer* g_timer;
inline void mark(int kernel_id)
{
    if (g_timer) (void)hipEventRecord(g_timer->ev[kernel_id + 1], g_timer->st);
}

}  // namespace lookm_host
