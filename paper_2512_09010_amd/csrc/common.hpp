// Device-side helpers shared by the gfx950 kernels of libluvc: storage-type access, wave64
// reductions, error plumbing.  Nothing here is shared with the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/luvc.h"

namespace luvc {

constexpr int kWave = 64;

// ------------------------------------------------------------------ host-side error text
void set_error(const char* fmt, ...);
// true when a workspace of `have` bytes at ws serves a need of `need` bytes (NULL is fine for a need of 0); sets the error text otherwise
bool workspace_ok(const void* ws, size_t have, size_t need);
luvc_status check_launch(const char* what);

// ------------------------------------------------------------------ optional timing of the library's launches
// While a caller has installed a list of events (luvc_profile_start), every launch goes out with a
// start and a stop event attached to the dispatch itself, so their difference is the kernel's own
// run time on the device.  prof_take() hands out the next pair (or returns false).
bool prof_take(const char* kernel, hipEvent_t* start, hipEvent_t* stop);

#define LUVC_LAUNCH(NAME, KERNEL, GRID, BLOCK, LDS, ST, ...)                                              \
    do {                                                                                                  \
        hipEvent_t e0_, e1_;                                                                              \
        if (::luvc::prof_take(NAME, &e0_, &e1_))                                                          \
            hipExtLaunchKernelGGL(KERNEL, GRID, BLOCK, LDS, ST, e0_, e1_, 0, __VA_ARGS__);                \
        else                                                                                              \
            hipLaunchKernelGGL(KERNEL, GRID, BLOCK, LDS, ST, __VA_ARGS__);                                \
    } while (0)

static inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------ storage types
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even fp32 -> bf16 (NaN kept quiet)
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// fp64 -> bf16 with a single nearest-even rounding, branch-free.  Adding and subtracting
// C = sign(v) * 2^(e + 45), e = exponent of v clamped at the smallest normal bf16 exponent, makes the
// fp64 adder round v to a multiple of 2^(e - 7): 8 significant bits for normal results, the fixed
// quantum 2^-133 for subnormal ones.  The rounded value is exact in fp32; its upper half is the bf16.
__device__ __forceinline__ uint16_t f64_to_bf16(double v)
{
    const uint32_t hi = (uint32_t)__double2hiint(v);
    uint32_t ef = hi & 0x7ff00000u;
    ef = ef < (897u << 20) ? (897u << 20) : ef;
    const double C = __hiloint2double((int)((hi & 0x80000000u) | (ef + (45u << 20))), 0);
    const double r = (v + C) - C;
    return (uint16_t)(__float_as_uint((float)r) >> 16);
}

template <typename T> struct io_traits;
template <> struct io_traits<float> {
    static constexpr int kVec = 4;                        // elements per 16-byte access
    using vec_t = float4;
    __device__ static __forceinline__ float load(const float* p) { return *p; }
    __device__ static __forceinline__ void store(float* p, double v) { *p = (float)v; }
    __device__ static __forceinline__ void unpack(const vec_t& v, float* o) { o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w; }
};
template <> struct io_traits<bf16_t> {
    static constexpr int kVec = 8;
    using vec_t = uint4;
    __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(p->bits); }
    __device__ static __forceinline__ void store(bf16_t* p, double v) { p->bits = f64_to_bf16(v); }
    __device__ static __forceinline__ void unpack(const vec_t& v, float* o)
    {
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
        o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
        o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
    }
};

// ------------------------------------------------------------------ XCD-aware workgroup order
// Workgroups are dealt to the 8 XCDs round-robin by linear id, and each XCD has its own L2.  This
// maps linear id g of G workgroups to a work item such that every XCD walks one contiguous range
// of work items in order: neighbouring items (which share halo tokens or cache lines) then meet in
// the same L2 at about the same time.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned g, unsigned G)
{
    constexpr unsigned kXcd = 8;
    const unsigned k = g % kXcd, i = g / kXcd, q = G / kXcd, r = G % kXcd;
    return k * q + (k < r ? k : r) + i;
}

// ------------------------------------------------------------------ wave64 reductions (all lanes get the result)
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
    // DPP adds inside each row of 16 lanes, two row broadcasts, then the total (held by lane 63) read back as a
    // wave-uniform value: no trip through the LDS crossbar, one fixed order
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));   // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));   // row_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x142, 0xa, 0xf, false));   // row_bcast:15 -> rows 1, 3
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x143, 0xc, 0xf, false));   // row_bcast:31 -> rows 2, 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

}  // namespace luvc
