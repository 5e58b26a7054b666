// Token-in-registers helpers shared by the fused OIM kernels (paper Section 3.2): a token is held
// as NCH 16-byte chunks per lane; similarity sums are screened in fp32 and, where a decision is
// too close for fp32, repeated in fp64.
#pragma once
#include "common.hpp"

namespace luvc {

namespace {

struct Scal { double na, nb, dab, dbc; };     // |a|^2, |b|^2, a.b, b.c of one slot (na, nb become 1/|a|, 1/|b| before the exchange)

template <typename T, int NCH>
struct Tok {
    typename io_traits<T>::vec_t v[NCH];
};

typedef unsigned int u32x4 __attribute__((__vector_size__(16)));

// One token = one buffer resource: lanes past the end of the token read zeros from the hardware
// bounds check, so the 16-byte loads need no branch and all of them can be in flight together.
template <typename T, int NCH>
__device__ __forceinline__ void load_tok(Tok<T, NCH>& t, const T* p, int D, int lane, bool present = true)
{
    using tr = io_traits<T>;
    constexpr int V = tr::kVec;
    // a token that is not there (past the end of the line) is a zero-length buffer: every lane reads zeros
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(p), 0, present ? D * (int)sizeof(T) : 0, 0x00020000);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const u32x4 r = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (i * 64 + lane) * V * (int)sizeof(T), 0, 0);
        typename tr::vec_t v;
        __builtin_memcpy(&v, &r, 16);
        t.v[i] = v;
    }
}

// element e (compile-time) of a 16-byte chunk as fp32
template <typename T> __device__ __forceinline__ float elem(const typename io_traits<T>::vec_t& v, int e);
template <> __device__ __forceinline__ float elem<float>(const float4& v, int e)
{
    return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
}
template <> __device__ __forceinline__ float elem<bf16_t>(const uint4& v, int e)
{
    const uint32_t wd = (e >> 1) == 0 ? v.x : (e >> 1) == 1 ? v.y : (e >> 1) == 2 ? v.z : v.w;
    return __uint_as_float((e & 1) ? (wd & 0xffff0000u) : (wd << 16));
}

// Similarity sweep of one wavefront.  Always: |a|^2, |b|^2, a.b, b.c.  With HALO: also |c|^2, |h|^2 and
// h.a (LEFT: h is the token before a) or c.h (h is the token after c).
template <typename T, int NCH, bool HALO, bool LEFT>
__device__ __forceinline__ void sweep(const Tok<T, NCH>& A, const Tok<T, NCH>& B, const Tok<T, NCH>& C, const Tok<T, NCH>& Hx,
                                      Scal& me, double& ncc, double& nhh, double& dh)
{
    constexpr int V = io_traits<T>::kVec;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const double a = (double)elem<T>(A.v[i], e), b = (double)elem<T>(B.v[i], e), c = (double)elem<T>(C.v[i], e);
            me.na = fma(a, a, me.na);
            me.nb = fma(b, b, me.nb);
            me.dab = fma(a, b, me.dab);
            me.dbc = fma(b, c, me.dbc);
            if (HALO) {
                const double h = (double)elem<T>(Hx.v[i], e);
                ncc = fma(c, c, ncc);
                nhh = fma(h, h, nhh);
                dh = LEFT ? fma(h, a, dh) : fma(c, h, dh);
            }
        }
    }
}

// ---- fp32 screening
struct ScalF { float ia, ib, dab, dbc; };      // 1/|a|, 1/|b|, a.b, b.c of one slot

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// acc += <x, y> over one 16-byte chunk in fp32
template <typename T> __device__ __forceinline__ float dot_chunk32(float acc, const typename io_traits<T>::vec_t& x, const typename io_traits<T>::vec_t& y);
template <> __device__ __forceinline__ float dot_chunk32<bf16_t>(float acc, const uint4& x, const uint4& y)
{
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        bf16x2_t a, b;
        __builtin_memcpy(&a, &xs[k], 4);
        __builtin_memcpy(&b, &ys[k], 4);
        acc = __builtin_amdgcn_fdot2_f32_bf16(a, b, acc, false);
    }
    return acc;
}
template <> __device__ __forceinline__ float dot_chunk32<float>(float acc, const float4& x, const float4& y)
{
    acc = fmaf(x.x, y.x, acc); acc = fmaf(x.y, y.y, acc); acc = fmaf(x.z, y.z, acc); acc = fmaf(x.w, y.w, acc);
    return acc;
}

template <typename T, int NCH, bool HALO, bool LEFT>
__device__ __forceinline__ void sweep32(const Tok<T, NCH>& A, const Tok<T, NCH>& B, const Tok<T, NCH>& C, const Tok<T, NCH>& Hx,
                                        float& na, float& nb, float& dab, float& dbc, float& ncc, float& nhh, float& dh)
{
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        na = dot_chunk32<T>(na, A.v[i], A.v[i]);
        nb = dot_chunk32<T>(nb, B.v[i], B.v[i]);
        dab = dot_chunk32<T>(dab, A.v[i], B.v[i]);
        dbc = dot_chunk32<T>(dbc, B.v[i], C.v[i]);
        if (HALO) {
            ncc = dot_chunk32<T>(ncc, C.v[i], C.v[i]);
            nhh = dot_chunk32<T>(nhh, Hx.v[i], Hx.v[i]);
            dh = LEFT ? dot_chunk32<T>(dh, Hx.v[i], A.v[i]) : dot_chunk32<T>(dh, C.v[i], Hx.v[i]);
        }
    }
}

// wave64 sum in a fixed order: DPP adds inside each row of 16 lanes, then the four rows
__device__ __forceinline__ float wave_sum32(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));   // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));   // row_mirror
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

// 1 / |x| for the screening - or NaN, which makes the screening abstain (the fp64 values decide), when the squared
// norm lies outside [2^-60, 2^100]: inside that window the fp32 sums neither lose terms to underflow (the packed bf16
// dot product flushes products below 2^-126: 2^-54 of such a norm at most) nor overflow, which is what the error
// bound behind tau assumes.  Zero and near-zero tokens (cosine defined through the 1e-12 clamp) go to fp64 as well.
__device__ __forceinline__ float inv_norm32(float n2)
{
    return (n2 >= 8.6736174e-19f && n2 <= 1.2676506e30f) ? 1.0f / sqrtf(n2) : __builtin_nanf("");
}

// Screening verdict for one source: +1 = left for certain, -1 = right for certain, 0 = too close to call
__device__ __forceinline__ int screen_source(bool has_left, bool has_right, float inv_src,
                                             float dot_l, float inv_l, float dot_r, float inv_r, float tau)
{
    if (!has_left) return -1;
    if (!has_right) return 1;
    const float sl = (dot_l * inv_src) * inv_l;
    const float sr = (dot_r * inv_src) * inv_r;
    const float d = sl - sr;
    if (d > tau) return 1;
    if (d < -tau) return -1;
    return 0;                                   // includes NaN
}

// Hides a token's registers from value numbering: the merge phase re-widens the packed data instead
// of keeping the fp64 copies of the similarity phase alive across the barrier (which spills).
template <typename T, int NCH>
__device__ __forceinline__ void forget(Tok<T, NCH>& t)
{
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        uint32_t* q = reinterpret_cast<uint32_t*>(&t.v[i]);
        asm volatile("" : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3]));
    }
}

// 1 / max(|x|, 1e-12) from the squared norm
__device__ __forceinline__ double inv_norm(double n2)
{
    const double n = sqrt(n2);
    return 1.0 / (n < 1e-12 ? 1e-12 : n);
}

// Does a source go to its LEFT destination?  Cosines are formed as (dot * 1/|src|) * 1/|dst| - the
// same expression, on the same bits, in both wavefronts that look at a source; tie -> left.
__device__ __forceinline__ bool source_goes_left(bool has_left, bool has_right, double inv_src,
                                                 double dot_l, double inv_l, double dot_r, double inv_r)
{
    if (!has_left) return false;
    if (!has_right) return true;
    const double sl = (dot_l * inv_src) * inv_l;
    const double sr = (dot_r * inv_src) * inv_r;
    return !(sr > sl);
}

}  // namespace

}  // namespace luvc
