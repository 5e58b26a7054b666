// Channel fetches shared by the wide-matching kernels of OIM (paper Section 3.2, Algorithm 1): eight consecutive
// channels of a token as raw words, widened to fp64 where they are used.
#pragma once
#include "common.hpp"

namespace luvc {

namespace {

typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((__vector_size__(16)));

// 8 consecutive elements of a token: fetched as raw words (so that several fetches can be in flight before the
// first is used), widened to fp64 afterwards; zeros past the end of the token or for a token that is not there
template <typename T, bool VECTOR> struct chan8;
template <bool VECTOR> struct chan8<bf16_t, VECTOR> {
    struct raw_t { u32x4 q; };
    // r spans the whole image (one descriptor for the wavefront); tok_off = byte offset of the token in it
    __device__ static __forceinline__ raw_t fetch(__amdgpu_buffer_rsrc_t r, uint32_t tok_off, const bf16_t* tok, int D, int d0, bool present)
    {
        raw_t o;
        if (VECTOR) {        // rows are multiples of 16 bytes: a piece lies inside the token or past its end, never across
            o.q = __builtin_amdgcn_raw_buffer_load_b128(r, (present && d0 < D) ? tok_off + (uint32_t)d0 * 2u : 0x80000000u, 0, 0);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = (present && d0 + 2 * i < D) ? tok[d0 + 2 * i].bits : 0u;
                const uint32_t hi = (present && d0 + 2 * i + 1 < D) ? tok[d0 + 2 * i + 1].bits : 0u;
                o.q[i] = lo | (hi << 16);
            }
        }
        return o;
    }
    // 16-byte aligned rows reached through a pointer of the lane's own (a token behind an index)
    __device__ static __forceinline__ raw_t fetch_ptr(const bf16_t* tok, int D, int d0, bool present)
    {
        raw_t o;
        o.q = u32x4{0u, 0u, 0u, 0u};
        if (present && d0 < D) o.q = *reinterpret_cast<const u32x4*>(tok + d0);
        return o;
    }
    __device__ static __forceinline__ void widen(const raw_t& w, double (&o)[8])
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = (double)__uint_as_float(w.q[i] << 16);
            o[2 * i + 1] = (double)__uint_as_float(w.q[i] & 0xffff0000u);
        }
    }
};
template <bool VECTOR> struct chan8<float, VECTOR> {
    struct raw_t { u32x4 q0, q1; };
    __device__ static __forceinline__ raw_t fetch(__amdgpu_buffer_rsrc_t r, uint32_t tok_off, const float* tok, int D, int d0, bool present)
    {
        raw_t o;
        if (VECTOR) {
            o.q0 = __builtin_amdgcn_raw_buffer_load_b128(r, (present && d0 < D) ? tok_off + (uint32_t)d0 * 4u : 0x80000000u, 0, 0);
            o.q1 = __builtin_amdgcn_raw_buffer_load_b128(r, (present && d0 + 4 < D) ? tok_off + (uint32_t)d0 * 4u + 16u : 0x80000000u, 0, 0);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                o.q0[i] = (present && d0 + i < D) ? __float_as_uint(tok[d0 + i]) : 0u;
                o.q1[i] = (present && d0 + 4 + i < D) ? __float_as_uint(tok[d0 + 4 + i]) : 0u;
            }
        }
        return o;
    }
    __device__ static __forceinline__ raw_t fetch_ptr(const float* tok, int D, int d0, bool present)
    {
        raw_t o;
        o.q0 = u32x4{0u, 0u, 0u, 0u};
        o.q1 = u32x4{0u, 0u, 0u, 0u};
        if (present && d0 < D) o.q0 = *reinterpret_cast<const u32x4*>(tok + d0);
        if (present && d0 + 4 < D) o.q1 = *reinterpret_cast<const u32x4*>(tok + d0 + 4);
        return o;
    }
    __device__ static __forceinline__ void widen(const raw_t& w, double (&o)[8])
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[i] = (double)__uint_as_float(w.q0[i]); o[4 + i] = (double)__uint_as_float(w.q1[i]); }
    }
};

}  // namespace

}  // namespace luvc
