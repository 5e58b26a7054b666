// Pieces shared by the kernels that fuse two halving passes of OIM (paper Section 3.2, Algorithm 1) into one launch:
// a token held in registers as 16-byte pieces per lane plus a short tail piece, wave-wide sums in fp32 and fp64,
// the decision expressions, the size-weighted merge with one rounding, and the cut of long lines into runs.
#pragma once
#include "common.hpp"
#include "oim.hpp"

namespace luvc {

namespace {

typedef unsigned int u32x4 __attribute__((__vector_size__(16)));
typedef unsigned int u32x2 __attribute__((__vector_size__(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

struct PairGeom {
    int L1, L2;      // line length of the first pass, of the second pass
    int nd1, nd2;    // L1 / 2, L2 / 2: destinations (= output slots) per line
    int sA, sB;      // input grid: tokens between neighbours along the first / second axis
    int oA, oB;      // output grid: slots between neighbours along the first / second axis
    int n_in, n_out; // tokens per image before / after the pair
    int D;
    int segs, seg_out;   // the nd2 second-pass outputs of a line are cut into `segs` runs of `seg_out`
};

// ------------------------------------------------------------------ a token in registers
template <int NQ, int TW>
struct Tok {
    static constexpr int N = 4 * NQ + TW;     // 32-bit words per lane
    uint32_t w[N];
};

template <typename T> struct words;            // storage elements per 32-bit word
template <> struct words<bf16_t> { static constexpr int per = 2; };
template <> struct words<float> { static constexpr int per = 1; };

template <int NQ, int TW>
__device__ __forceinline__ void zero_tok(Tok<NQ, TW>& t)
{
#pragma unroll
    for (int i = 0; i < Tok<NQ, TW>::N; ++i) t.w[i] = 0u;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t token_rsrc(const void* p, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

// cache policy of token loads (buffer aux bits): default, because the neighbouring workgroups read the same tokens
// again from L2 (the non-temporal hint was measured slower: 36.3 against 34.9 us on 8 x 64 x 64 x 1280 bf16)
constexpr int kLoadAux = 0;
// a token that is not there (past the end of the line) is a zero-length buffer: every lane reads zeros
template <int NQ, int TW>
__device__ __forceinline__ void load_tok(Tok<NQ, TW>& t, const void* p, int bytes, int lane, bool present = true)
{
    const __amdgpu_buffer_rsrc_t rsrc = token_rsrc(p, present ? bytes : 0);
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const u32x4 r = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (q * 64 + lane) * 16, 0, kLoadAux);
        t.w[4 * q] = r[0]; t.w[4 * q + 1] = r[1]; t.w[4 * q + 2] = r[2]; t.w[4 * q + 3] = r[3];
    }
    if (TW == 1) t.w[4 * NQ] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, NQ * 1024 + lane * 4, 0, kLoadAux);
    if (TW == 2) {
        const u32x2 r = __builtin_amdgcn_raw_buffer_load_b64(rsrc, NQ * 1024 + lane * 8, 0, kLoadAux);
        t.w[4 * NQ] = r[0]; t.w[4 * NQ + 1] = r[1];
    }
}

// output tokens are not read again by this kernel: non-temporal stores (2) leave less dirty data in L2 for the end of
// the kernel (measured: 36.2 -> 34.9 us, and a shorter gap to the next launch)
constexpr int kStoreAux = 2;
template <int NQ, int TW>
__device__ __forceinline__ void store_tok(void* p, int bytes, const Tok<NQ, TW>& t, int lane)
{
    const __amdgpu_buffer_rsrc_t rsrc = token_rsrc(p, bytes);
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        u32x4 r;
        r[0] = t.w[4 * q]; r[1] = t.w[4 * q + 1]; r[2] = t.w[4 * q + 2]; r[3] = t.w[4 * q + 3];
        __builtin_amdgcn_raw_buffer_store_b128(r, rsrc, (q * 64 + lane) * 16, 0, kStoreAux);
    }
    if (TW == 1) __builtin_amdgcn_raw_buffer_store_b32(t.w[4 * NQ], rsrc, NQ * 1024 + lane * 4, 0, kStoreAux);
    if (TW == 2) {
        u32x2 r;
        r[0] = t.w[4 * NQ]; r[1] = t.w[4 * NQ + 1];
        __builtin_amdgcn_raw_buffer_store_b64(r, rsrc, NQ * 1024 + lane * 8, 0, kStoreAux);
    }
}

// ------------------------------------------------------------------ sums
// wave64 sum without the LDS crossbar: DPP adds inside each row of 16 lanes, two row broadcasts,
// and the total (held by lane 63) read back as a wave-uniform value.  One fixed order everywhere.
__device__ __forceinline__ float wave_total32(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));   // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));   // row_mirror
    // every lane of a row now holds the row's sum; lane 15 of row r is added into row r+1, then
    // lane 31 into rows 2 and 3: lane 63 ends with all four
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x142, 0xa, 0xf, false));   // row_bcast:15 -> rows 1, 3
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x143, 0xc, 0xf, false));   // row_bcast:31 -> rows 2, 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

template <typename T> __device__ __forceinline__ float dot_word(float acc, uint32_t x, uint32_t y);
template <> __device__ __forceinline__ float dot_word<bf16_t>(float acc, uint32_t x, uint32_t y)
{
    bf16x2_t a, b;
    __builtin_memcpy(&a, &x, 4);
    __builtin_memcpy(&b, &y, 4);
    return __builtin_amdgcn_fdot2_f32_bf16(a, b, acc, false);
}
template <> __device__ __forceinline__ float dot_word<float>(float acc, uint32_t x, uint32_t y)
{
    return fmaf(__uint_as_float(x), __uint_as_float(y), acc);
}

// Eight wave64 sums at once.  Three exchange steps inside a quad / half row keep, in every lane, only
// the partial sum of value (lane & 7): each step halves the number of registers instead of adding every
// value in every lane.  Then one add across the half rows, one across the two halves of the wave
// and one across neighbouring rows (lane-swap instructions), and lane i holds the total of value i.
// Six additions per term, like the one-value sum above.
__device__ __forceinline__ float dpp_get(float v, const int sel)
{
    const int x = __float_as_int(v);
    switch (sel) {
        case 0: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, true));    // quad_perm [1,0,3,2]: lane ^ 1
        case 1: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, true));    // quad_perm [2,3,0,1]: lane ^ 2
        case 2: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x141, 0xf, 0xf, true));   // row_half_mirror: lane ^ 7
        case 3: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x1B, 0xf, 0xf, true));    // quad_perm [3,2,1,0]: lane ^ 3
        default: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x128, 0xf, 0xf, true));  // row_ror:8: lane ^ 8
    }
}

__device__ __forceinline__ void wave_total32x8(float (&v)[8], int lane)
{
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
    float p[4], q[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float keep = b0 ? v[2 * i + 1] : v[2 * i], send = b0 ? v[2 * i] : v[2 * i + 1];
        p[i] = keep + dpp_get(send, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const float keep = b1 ? p[2 * i + 1] : p[2 * i], send = b1 ? p[2 * i] : p[2 * i + 1];
        q[i] = keep + dpp_get(send, 1);
    }
    const float keep = b2 ? q[1] : q[0], send = b2 ? q[0] : q[1];
    float r = keep + dpp_get(dpp_get(send, 2), 3);                  // (lane ^ 7) ^ 3 = lane ^ 4
    r += dpp_get(r, 4);
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(r), __float_as_uint(r), false, false);
    r = __uint_as_float(h[0]) + __uint_as_float(h[1]);
    const auto g = __builtin_amdgcn_permlane16_swap(__float_as_uint(r), __float_as_uint(r), false, false);
    r = __uint_as_float(g[0]) + __uint_as_float(g[1]);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(r), i));
}

// this lane's part of <x, y>
template <typename T, int NQ, int TW>
__device__ __forceinline__ float dot32_lane(const Tok<NQ, TW>& x, const Tok<NQ, TW>& y)
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < Tok<NQ, TW>::N; ++i) acc = dot_word<T>(acc, x.w[i], y.w[i]);
    return acc;
}

// screening sum <x, y> in fp32 (wave-uniform result)
template <typename T, int NQ, int TW>
__device__ __forceinline__ float dot32(const Tok<NQ, TW>& x, const Tok<NQ, TW>& y)
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < Tok<NQ, TW>::N; ++i) acc = dot_word<T>(acc, x.w[i], y.w[i]);
    return wave_total32(acc);
}

// element e of a word, widened
template <typename T> __device__ __forceinline__ double elem64(uint32_t w, int e);
template <> __device__ __forceinline__ double elem64<bf16_t>(uint32_t w, int e)
{
    return (double)__uint_as_float(e ? (w & 0xffff0000u) : (w << 16));
}
template <> __device__ __forceinline__ double elem64<float>(uint32_t w, int) { return (double)__uint_as_float(w); }

// wave64 sum of fp64 values, same DPP pattern as wave_total32 applied to both halves of the value
__device__ __forceinline__ double dpp_move64(double v, const int ctrl_sel)
{
    const int lo = __double2loint(v), hi = __double2hiint(v);
    int xl, xh;
    switch (ctrl_sel) {
        case 0: xl = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xf, 0xf, false); xh = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xf, 0xf, false); break;
        case 1: xl = __builtin_amdgcn_update_dpp(0, lo, 0x4E, 0xf, 0xf, false); xh = __builtin_amdgcn_update_dpp(0, hi, 0x4E, 0xf, 0xf, false); break;
        case 2: xl = __builtin_amdgcn_update_dpp(0, lo, 0x141, 0xf, 0xf, false); xh = __builtin_amdgcn_update_dpp(0, hi, 0x141, 0xf, 0xf, false); break;
        case 3: xl = __builtin_amdgcn_update_dpp(0, lo, 0x140, 0xf, 0xf, false); xh = __builtin_amdgcn_update_dpp(0, hi, 0x140, 0xf, 0xf, false); break;
        case 4: xl = __builtin_amdgcn_update_dpp(0, lo, 0x142, 0xa, 0xf, false); xh = __builtin_amdgcn_update_dpp(0, hi, 0x142, 0xa, 0xf, false); break;
        default: xl = __builtin_amdgcn_update_dpp(0, lo, 0x143, 0xc, 0xf, false); xh = __builtin_amdgcn_update_dpp(0, hi, 0x143, 0xc, 0xf, false); break;
    }
    return __hiloint2double(xh, xl);
}

__device__ __forceinline__ double wave_total64(double v)
{
    v += dpp_move64(v, 0);
    v += dpp_move64(v, 1);
    v += dpp_move64(v, 2);
    v += dpp_move64(v, 3);
    v += dpp_move64(v, 4);       // rows the broadcast does not reach add the zero of the disabled lanes
    v += dpp_move64(v, 5);
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63), __builtin_amdgcn_readlane(__double2loint(v), 63));
}

// Hides a token's registers from value numbering, so that the rarely taken fp64 code widens the
// packed words where it uses them instead of keeping fp64 copies of whole tokens alive.
template <int NQ, int TW>
__device__ __forceinline__ void forget(Tok<NQ, TW>& t)
{
#pragma unroll
    for (int i = 0; i < Tok<NQ, TW>::N; ++i) asm volatile("" : "+v"(t.w[i]));
}

// <x, y> in fp64.  The words are widened one at a time (scheduling fences keep the widened copies
// from piling up in registers: this code runs for a fraction of a percent of the decisions).
template <typename T, int NQ, int TW>
__device__ __forceinline__ double dot64(Tok<NQ, TW>& x, Tok<NQ, TW>& y)
{
    forget(x);
    forget(y);
    double acc = 0.0;
#pragma unroll
    for (int i = 0; i < Tok<NQ, TW>::N; ++i) {
#pragma unroll
        for (int e = 0; e < words<T>::per; ++e) acc = fma(elem64<T>(x.w[i], e), elem64<T>(y.w[i], e), acc);
        __builtin_amdgcn_sched_barrier(0);
    }
    return wave_total64(acc);
}

template <typename T, int NQ, int TW>
__device__ __forceinline__ double norm64(Tok<NQ, TW>& x) { return dot64<T>(x, x); }

// fp64 squared norms n[p] = <P_p, P_p> and neighbour products d[p] = <P_p, P_p+1> of five tokens that
// follow each other on a line
template <typename T, int NQ, int TW>
__device__ __forceinline__ void chain_sums64(Tok<NQ, TW>& P0, Tok<NQ, TW>& P1, Tok<NQ, TW>& P2, Tok<NQ, TW>& P3, Tok<NQ, TW>& P4,
                                             double (&n)[5], double (&d)[4])
{
    n[0] = norm64<T>(P0); n[1] = norm64<T>(P1); n[2] = norm64<T>(P2); n[3] = norm64<T>(P3); n[4] = norm64<T>(P4);
    d[0] = dot64<T>(P0, P1); d[1] = dot64<T>(P1, P2); d[2] = dot64<T>(P2, P3); d[3] = dot64<T>(P3, P4);
}

// 1 / |x| from the squared norm, screening precision (hardware reciprocal square root) - or NaN, which makes the
// screening abstain (the fp64 values decide), when the squared norm lies outside [2^-60, 2^100]: the error bound of
// the screening counts relative roundings only, and those are all there is inside that window (terms that the
// packed bf16 dot product flushes to zero are below 2^-126 each, 2^-54 of such a norm at most; nothing overflows).
// Zero and near-zero tokens, for which the cosine is defined through the 1e-12 clamp, go to fp64 the same way.
__device__ __forceinline__ float inv_norm32(float n2)
{
    return (n2 >= 8.6736174e-19f && n2 <= 1.2676506e30f) ? __builtin_amdgcn_rsqf(n2) : __builtin_nanf("");
}

__device__ __forceinline__ double inv_norm64(double n2)
{
    const double n = sqrt(n2);
    return 1.0 / (n < 1e-12 ? 1e-12 : n);
}

// Screening verdict for one source between its lower-position ("left") and higher-position
// ("right") destination: +1 = left for certain, -1 = right for certain, 0 = too close to call.
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

// The fp64 decision: cosines formed as (dot * 1/|src|) * 1/|dst|, the same expression on the same
// bits wherever a source is looked at; tie -> left (the lower position).
__device__ __forceinline__ bool source_goes_left(bool has_left, bool has_right, double inv_src,
                                                 double dot_l, double inv_l, double dot_r, double inv_r)
{
    if (!has_left) return false;
    if (!has_right) return true;
    const double sl = (dot_l * inv_src) * inv_l;
    const double sr = (dot_r * inv_src) * inv_r;
    return !(sr > sl);
}

// ------------------------------------------------------------------ merge
template <typename T> __device__ __forceinline__ uint32_t pack_word(double q0, double q1);
// fp64 -> bf16 with one nearest-even rounding: Veltkamp's splitting with the constant 2^45 + 1 leaves
// the 8 leading bits of q, rounded to nearest even (the product and the two differences each round
// once, and their errors cancel exactly); that value is exact in fp32, whose upper half is the bf16.
// The hardware conversion takes it from there, which only matters below the smallest normal bf16
// (2^-126), where it rounds the 8-bit value once more onto the subnormal grid.
template <> __device__ __forceinline__ uint32_t pack_word<bf16_t>(double q0, double q1)
{
    // The three operations must each round on their own: fused into c * q + (q - g) the product would stay exact and
    // nothing would be rounded to 8 bits here (the fp32 conversion below would then round a second time).
#pragma clang fp contract(off)
    const double c = 35184372088833.0;            // 2^45 + 1
    const double g0 = c * q0, g1 = c * q1;
    f32x2_t v;
    v[0] = (float)(g0 + (q0 - g0));
    v[1] = (float)(g1 + (q1 - g1));
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    uint32_t u;
    __builtin_memcpy(&u, &r, 4);
    return u;
}
template <> __device__ __forceinline__ uint32_t pack_word<float>(double q0, double) { return __float_as_uint((float)q0); }

// Size-weighted mean of destination b and the sources folded into it, fp64, terms in position
// order b, a, c (an absent source has size 0 and adds an exact zero), rounded once to the storage
// type.  The quotient is formed with the reciprocal and one residual correction: exact whenever
// acc / S is representable, which covers every rounding boundary of the storage types.
template <typename T, int NQ, int TW>
__device__ __forceinline__ void merge64(Tok<NQ, TW>& out, const Tok<NQ, TW>& B, const Tok<NQ, TW>& A, const Tok<NQ, TW>& C,
                                        double dsb, double dsa, double dsc, double dS, double rS)
{
#pragma unroll
    for (int i = 0; i < Tok<NQ, TW>::N; ++i) {
        double q[2] = {0.0, 0.0};
#pragma unroll
        for (int e = 0; e < words<T>::per; ++e) {
            double acc = dsb * elem64<T>(B.w[i], e);
            acc = fma(dsa, elem64<T>(A.w[i], e), acc);
            acc = fma(dsc, elem64<T>(C.w[i], e), acc);
            double v = acc * rS;
            v = fma(fma(-v, dS, acc), rS, v);
            q[e] = v;
        }
        out.w[i] = pack_word<T>(q[0], q[1]);
    }
}

// (b + x) / 2 for bf16 storage in fp32 (see the head of this file for why this is exact)
template <int NQ, int TW>
__device__ __forceinline__ void average_bf16(Tok<NQ, TW>& out, const Tok<NQ, TW>& B, const Tok<NQ, TW>& X)
{
#pragma unroll
    for (int i = 0; i < Tok<NQ, TW>::N; ++i) {
        const float b0 = __uint_as_float(B.w[i] << 16), b1 = __uint_as_float(B.w[i] & 0xffff0000u);
        const float x0 = __uint_as_float(X.w[i] << 16), x1 = __uint_as_float(X.w[i] & 0xffff0000u);
        f32x2_t v;
        v[0] = fmaf(b0, 0.5f, x0 * 0.5f);
        v[1] = fmaf(b1, 0.5f, x1 * 0.5f);
        const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
        __builtin_memcpy(&out.w[i], &r, 4);
    }
}

// Destination b with sizes sb absorbs a (size sa, 0 = not absorbed) and c (size sc, 0 = not absorbed).
template <typename T, int NQ, int TW>
__device__ __forceinline__ void merge_tok(Tok<NQ, TW>& out, const Tok<NQ, TW>& B, const Tok<NQ, TW>& A, const Tok<NQ, TW>& C,
                                          int sb, int sa, int sc)
{
    if (words<T>::per == 2 && ((sc == 0 && sa == sb) || (sa == 0 && sc == sb))) {
        if (sc == 0) average_bf16(out, B, A);
        else average_bf16(out, B, C);
        return;
    }
    const int S = sb + sa + sc;
    merge64<T>(out, B, A, C, (double)sb, (double)sa, (double)sc, (double)S, 1.0 / (double)S);
}


struct PairPlan { int segs, seg_out, waves; };

// Cut the nd2 outputs of a line so that a workgroup needs at most `nw` wavefronts: its own rows,
// two rows below (one more wavefront at most) and the single-row wavefront above.
PairPlan plan_pair(int L2, int nw, int64_t lines)
{
    const int nd2 = L2 / 2;
    PairPlan p;
    // A grid with fewer line positions than the chip has CUs would leave most of it idle with one workgroup
    // per position: cut the lines into runs of 8 outputs then (measured on 2 x 112 x 112, 56 x 56 and
    // 28 x 28 grids: 64 us for the three calls against 78; runs of 2, 6 or 14 gain less).
    const int forced = (lines < 256 && nd2 > 8) ? 8 : 0;
    if ((L2 + 3) / 4 <= nw && forced <= 0) {
        p.segs = 1;
        p.seg_out = nd2;
        p.waves = (L2 + 3) / 4;
        return p;
    }
    int cap = 2 * (nw - 1) - 1;                    // (2 * seg_out + 2 + 3) / 4 + 1 <= nw
    if (cap & 1) --cap;                            // even: workgroups start on a multiple of four rows
    if (cap < 2) cap = 2;
    if (forced > 0 && forced < cap) cap = forced + (forced & 1);
    p.segs = (nd2 + cap - 1) / cap;
    p.seg_out = (nd2 + p.segs - 1) / p.segs;
    if (p.seg_out & 1) ++p.seg_out;
    p.segs = (nd2 + p.seg_out - 1) / p.seg_out;
    p.waves = p.segs == 1 ? (L2 + 3) / 4 : (2 * p.seg_out + 2 + 3) / 4 + 1;
    if (p.waves > nw) p.waves = nw;
    return p;
}

}  // namespace

}  // namespace luvc
