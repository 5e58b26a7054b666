// OIM (paper Section 3.2, Algorithm 1) - one launch for a PAIR of halving passes on orthogonal
// axes (row merge then column merge, or the other way round): H x W -> H/2 x W/2 without the
// intermediate grid ever leaving the chip.
//
// Work split.  A workgroup owns one line position j of the first pass (output column j for a
// row-then-column pair) and a run of output slots of the second pass.  Each wavefront owns four
// consecutive lines of the first pass: for each of them it loads destination b = 2j+1, its two
// sources a = 2j, c = 2j+2 and the two destinations beyond them (l = 2j-1, r = 2j+3, needed only
// to decide where a and c go), forms the first-pass token, rounds it to the storage type - the
// second pass must read what a separate launch would have read from memory - and keeps it packed
// in registers.  The four intermediate tokens of a wavefront are two destinations of the second
// pass with the sources between them; the one token a wavefront needs from its neighbour (the
// first token of the next wavefront) goes through LDS, as do the norms and neighbour dot
// products every wavefront needs from the tokens around its own.  A workgroup that owns only
// part of a long line recomputes the three intermediate tokens just outside its run.
//
// A token in registers is NQ 16-byte pieces per lane plus a 4- or 8-byte tail piece, so that a
// token of 1280 bf16 values costs 10 registers per lane, not 12; buffer resources bound every
// piece, so lanes past the end of a token read zeros and write nothing.
//
// Decisions are fp64 decisions reached in two steps, as in the single-pass kernel: a screening
// sweep in fp32 with a rigorous error bound, and a repeat in fp64 of whatever is closer than the
// bound.  In the first pass the repeat is local to a wavefront; in the second pass it is taken by
// the whole workgroup, because the sums of a decision live in two wavefronts.  A source shared by
// two workgroups is decided from the same bits by the same expressions in both.
//
// The merge is the size-weighted mean evaluated in fp64 in position order and rounded once.  One
// case needs no fp64: bf16 storage, one absorbed source, equal sizes.  Then the mean is (b + x) / 2
// and the fp32 sum, halved and rounded to bf16 by the hardware conversion, is the correctly rounded
// result: either the sum is exact in fp32 (exponents at most 15 apart), or the smaller term is below
// 2^-15 of the larger, whose half lies on the bf16 grid at least 2^-10 (relative) away from every
// rounding boundary - too far for the smaller term or the fp32 rounding to matter.
#include <cstdlib>

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

}  // namespace

template <typename T, int NQ, int TW, int NW>
__global__ void __launch_bounds__(NW * 64)
oim_halve_pair(const T* __restrict__ x, const int32_t* __restrict__ sizes_in, PairGeom g,
               const int32_t* __restrict__ kept_prev, T* __restrict__ x_out, int32_t* __restrict__ sizes_out,
               int32_t* __restrict__ pair_map, int32_t* __restrict__ kept_out)
{
    using TokT = Tok<NQ, TW>;
    constexpr int N = TokT::N;
    constexpr int kRows = 4 * NW + 8;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint32_t* lds_tok = reinterpret_cast<uint32_t*>(lds_raw);     // [live waves][N][64]: first token of each wave
    __shared__ float inv32[kRows], dt32[kRows];                   // 1/|T[r]|, <T[r], T[r+1]> of the intermediate tokens
    __shared__ double inv64[kRows], dt64[kRows];
    __shared__ int szl[kRows];
    __shared__ int redo;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int j = item % g.nd1;
    const int seg = (item / g.nd1) % g.segs;
    const int b = item / (g.nd1 * g.segs);
    const int u0 = seg * g.seg_out;
    const int nseg = min(g.seg_out, g.nd2 - u0);                  // second-pass outputs of this workgroup
    const int row_base = 2 * u0;
    const int row_lo = u0 > 0 ? row_base - 1 : row_base;          // one intermediate row above the run decides its first source
    const int row_end = min(g.L2 - 1, row_base + 2 * nseg + 1);   // two below decide its last source (or close an odd line)
    const int nwm = (row_end - row_base + 1 + 3) >> 2;            // wavefronts with rows of the run
    const bool is_main = w < nwm;
    const bool is_halo = u0 > 0 && w == nwm;                      // holds row_base - 1 as ITS LAST row
    const bool active = is_main || is_halo;
    const int r0 = is_halo ? row_base - 4 : row_base + 4 * w;
    const int rr0 = r0 - row_base + 1;                            // LDS index of row r0 (negative only for the halo wave's unused rows)
    // Error bound of the screening, in units of u = 2^-24.  A sum takes at most E = R + 6 roundings of
    // relative size u on partial sums bounded by the sum of the magnitudes of its terms (R per lane: two
    // per packed bf16 product pair, one per fp32 product; six reduction steps); against |a||b| that is E u
    // on a dot product and E u on each squared norm, i.e. (E + 4) u on the two reciprocal norms together
    // (hardware reciprocal square root: 1 ulp each), plus two products: 2 E + 6 per cosine, 4 E + 13 on
    // the difference of two.  tau is 1.5 times that.  Each step of the packed bf16 dot product is taken as one or two
    // roundings to nearest of the exact value (tests/test_gpu_oim.py pins the instruction's sums against fp64);
    // underflow and overflow are kept out by inv_norm32().
    constexpr int kE = N * (words<T>::per == 2 ? 2 : 1) + 6;
    const float tau = (float)(6 * kE + 20) * 5.9604645e-8f;
    const int tok_bytes = g.D * (int)sizeof(T);
    if (threadIdx.x == 0) redo = 0;

    // ------------------------------------------------------------------ first pass: four intermediate tokens
    const int pa = 2 * j, pb = pa + 1, pc = pa + 2;
    const bool has_l = j > 0, has_c = pc < g.L1, has_r = pc + 1 < g.L1;
    const int64_t img_in = (int64_t)b * g.n_in;
    TokT T0, T1, T2, T3;
    zero_tok(T0); zero_tok(T1); zero_tok(T2); zero_tok(T3);
    int s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    unsigned took_a = 0, took_c = 0;                              // bit k: row k absorbed its a / its c
    // the four rows unrolled: the compiler renames T0..T3 instead of moving 10 registers per token and row
    // (measured: 35.3 -> 34.2 us on 8 x 64 x 64 x 1280 bf16)
#pragma unroll 4
    for (int k = 0; k < 4; ++k) {
        const int r = r0 + k;
        TokT Tn;
        int sn = 0;
        if (active && r >= row_lo && r <= row_end) {
            const int64_t t0 = img_in + (int64_t)r * g.sB;        // token of position 0 on this line
            const int64_t ta = t0 + (int64_t)pa * g.sA, tb = t0 + (int64_t)pb * g.sA, tc = t0 + (int64_t)pc * g.sA;
            TokT A, Bt, C, Lt, Rt;
            load_tok(A, x + ta * g.D, tok_bytes, lane);
            load_tok(Bt, x + tb * g.D, tok_bytes, lane);
            load_tok(C, x + (has_c ? tc : tb) * g.D, tok_bytes, lane, has_c);
            load_tok(Lt, x + (has_l ? ta - g.sA : tb) * g.D, tok_bytes, lane, has_l);
            load_tok(Rt, x + (has_r ? tc + g.sA : tb) * g.D, tok_bytes, lane, has_r);
            const int sb = sizes_in ? sizes_in[tb] : 1;
            const int sa_in = sizes_in ? sizes_in[ta] : 1;
            const int sc_in = (sizes_in && has_c) ? sizes_in[tc] : 1;
            // screening: every sum is formed lower position first, so the sum two workgroups share has the same bits
            // (tokens that are not there were loaded as zeros: their sums are zero and never looked at)
            float sm[8] = {dot32_lane<T>(A, A), dot32_lane<T>(Bt, Bt), dot32_lane<T>(A, Bt), dot32_lane<T>(Lt, A),
                           dot32_lane<T>(Lt, Lt), dot32_lane<T>(C, C), dot32_lane<T>(Bt, C), dot32_lane<T>(C, Rt)};
            wave_total32x8(sm, lane);
            const float ia = inv_norm32(sm[0]), ib = inv_norm32(sm[1]), dab = sm[2];
            int va = -1, vc = -1;
            if (has_l) va = screen_source(true, true, ia, sm[3], inv_norm32(sm[4]), dab, ib, tau);
            if (has_c) {
                vc = 1;
                if (has_r) vc = screen_source(true, true, inv_norm32(sm[5]), sm[6], ib, sm[7], inv_norm32(dot32<T>(Rt, Rt)), tau);
            }
            bool a_left = va > 0, c_left = vc > 0;
            if (va == 0 || vc == 0) {                             // too close for fp32: the fp64 cosines decide
                double n[5], d[4];
                chain_sums64<T>(Lt, A, Bt, C, Rt, n, d);
                const double jb = inv_norm64(n[2]);
                if (va == 0) a_left = source_goes_left(true, true, inv_norm64(n[1]), d[0], inv_norm64(n[0]), d[1], jb);
                if (vc == 0) c_left = source_goes_left(true, true, inv_norm64(n[3]), d[2], jb, d[3], inv_norm64(n[4]));
            }
            const bool take_a = !a_left, take_c = has_c && c_left;
            const int sa = take_a ? sa_in : 0, sc = take_c ? sc_in : 0;
            sn = sb + sa + sc;
            if (take_a) took_a |= 1u << k;
            if (take_c) took_c |= 1u << k;
            if (!take_a && !take_c) Tn = Bt;
            else merge_tok<T>(Tn, Bt, A, C, sb, sa, sc);
        } else {
            zero_tok(Tn);
        }
        T0 = T1; T1 = T2; T2 = T3; T3 = Tn;
        s0 = s1; s1 = s2; s2 = s3; s3 = sn;
    }

    // ------------------------------------------------------------------ second pass: exchange
    if (is_main) {
#pragma unroll
        for (int i = 0; i < N; ++i) lds_tok[(w * N + i) * 64 + lane] = T0.w[i];
    }
    __syncthreads();
    TokT Tx;                                                      // the token after T3: first token of the next wavefront
    const bool has_x = active && r0 + 4 <= row_end;
    if (has_x) {
        const int nxt = is_halo ? 0 : w + 1;
#pragma unroll
        for (int i = 0; i < N; ++i) Tx.w[i] = lds_tok[(nxt * N + i) * 64 + lane];
    } else {
        zero_tok(Tx);
    }
    if (active) {
        float sm[8] = {dot32_lane<T>(T0, T0), dot32_lane<T>(T1, T1), dot32_lane<T>(T2, T2), dot32_lane<T>(T3, T3),
                       dot32_lane<T>(T0, T1), dot32_lane<T>(T1, T2), dot32_lane<T>(T2, T3), dot32_lane<T>(T3, Tx)};
        wave_total32x8(sm, lane);
        const float n0 = sm[0], n1 = sm[1], n2 = sm[2], n3 = sm[3], d0 = sm[4], d1 = sm[5], d2 = sm[6], d3 = sm[7];
        if (lane < 4) {
            const int k = lane, r = r0 + k;
            if (r >= row_lo && r <= row_end) {
                inv32[rr0 + k] = inv_norm32(k == 0 ? n0 : k == 1 ? n1 : k == 2 ? n2 : n3);
                dt32[rr0 + k] = k == 0 ? d0 : k == 1 ? d1 : k == 2 ? d2 : d3;
                szl[rr0 + k] = k == 0 ? s0 : k == 1 ? s1 : k == 2 ? s2 : s3;
            }
        }
    }
    __syncthreads();
    // a source at intermediate row r (LDS index q) goes UP (to the lower position) unless the row below is strictly more similar
    auto verdict32 = [&](int r, int q) -> int {
        const bool has_up = r >= 1, has_dn = r + 1 < g.L2;
        const int qm = q > 0 ? q - 1 : 0;
        return screen_source(has_up, has_dn, inv32[q], dt32[qm], inv32[qm], dt32[q], inv32[q + 1], tau);
    };
    auto decide64 = [&](int r, int q) -> bool {
        const bool has_up = r >= 1, has_dn = r + 1 < g.L2;
        const int qm = q > 0 ? q - 1 : 0;
        return source_goes_left(has_up, has_dn, inv64[q], dt64[qm], inv64[qm], dt64[q], inv64[q + 1]);
    };
    const bool e2 = r0 + 2 <= row_end, e4 = r0 + 4 <= row_end;
    int v0 = -1, v2 = -1, v4 = -1;
    if (is_main) {
        v0 = verdict32(r0, rr0);
        if (e2) v2 = verdict32(r0 + 2, rr0 + 2);
        if (e4) v4 = verdict32(r0 + 4, rr0 + 4);
        if ((v0 == 0 || v2 == 0 || v4 == 0) && lane == 0) redo = 1;
    }
    __syncthreads();
    bool up0 = v0 > 0, up2 = v2 > 0, up4 = v4 > 0;
    if (redo) {                                                   // uniform over the workgroup
        if (active) {
            double n[5], d[4];
            chain_sums64<T>(T0, T1, T2, T3, Tx, n, d);
            if (lane < 4) {
                const int k = lane, r = r0 + k;
                if (r >= row_lo && r <= row_end) {
                    inv64[rr0 + k] = inv_norm64(k == 0 ? n[0] : k == 1 ? n[1] : k == 2 ? n[2] : n[3]);
                    dt64[rr0 + k] = k == 0 ? d[0] : k == 1 ? d[1] : k == 2 ? d[2] : d[3];
                }
            }
        }
        __syncthreads();
        if (is_main) {
            up0 = decide64(r0, rr0);
            up2 = e2 && decide64(r0 + 2, rr0 + 2);
            up4 = e4 && decide64(r0 + 4, rr0 + 4);
        }
    }
    if (!is_main) return;

    // ------------------------------------------------------------------ second pass: merge, write, maps
    const int own_end = row_base + 2 * nseg;                      // rows below it belong to the next run ...
    const bool tail = (g.L2 & 1) && own_end == g.L2 - 1;          // ... except the last source of an odd line
    const int64_t img_out = (int64_t)b * g.n_out;
    const int uo = r0 >> 1;                                       // output slot (second axis) of destination r0 + 1
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        const int dest = r0 + 1 + 2 * o;
        if (dest >= own_end) break;
        const bool take_a = o == 0 ? !up0 : !up2;                 // the source above comes down
        const bool take_c = o == 0 ? (e2 && up2) : (e4 && up4);   // the source below goes up
        const TokT& Bt = o == 0 ? T1 : T3;
        const TokT& A = o == 0 ? T0 : T2;
        const TokT& C = o == 0 ? T2 : Tx;
        const int sb = o == 0 ? s1 : s3;
        const int sa = take_a ? (o == 0 ? s0 : s2) : 0;
        const int sc = take_c ? (o == 0 ? s2 : szl[rr0 + 4]) : 0;
        const int slot = (uo + o) * g.oB + j * g.oA;
        T* op = x_out + (img_out + slot) * g.D;
        if (lane == 0) {
            sizes_out[img_out + slot] = sb + sa + sc;
            if (kept_out) {
                const int p_in = dest * g.sB + pb * g.sA;
                kept_out[img_out + slot] = kept_prev ? kept_prev[img_in + p_in] : p_in;
            }
        }
        if (!take_a && !take_c) {
            store_tok(op, tok_bytes, Bt, lane);
        } else {
            TokT R;
            merge_tok<T>(R, Bt, A, C, sb, sa, sc);
            store_tok(op, tok_bytes, R, lane);
        }
    }
    if (pair_map && lane < 4) {
        const int k = lane, r = r0 + k;
        if (r <= row_end && (r < own_end || (tail && r == own_end))) {
            // intermediate row r lands in output slot: odd rows are destinations; an even row goes up or down
            int u;
            if (r & 1) u = r >> 1;
            else u = (k == 0 ? up0 : up2) ? (r >> 1) - 1 : (r >> 1);
            const int slot = u * g.oB + j * g.oA;
            const int64_t t0 = img_in + (int64_t)r * g.sB;
            pair_map[t0 + (int64_t)pb * g.sA] = slot;
            if ((took_a >> k) & 1u) pair_map[t0 + (int64_t)pa * g.sA] = slot;
            if ((took_c >> k) & 1u) pair_map[t0 + (int64_t)pc * g.sA] = slot;
        }
    }
}

// ------------------------------------------------------------------ host side
namespace {

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

template <typename T, int NQ, int TW>
luvc_status launch_pair(const T* x, const int32_t* sizes_in, int B, int H, int W, int D, int first_axis,
                        const int32_t* kept_prev, T* x_out, int32_t* sizes_out, int32_t* pair_map, int32_t* kept_out,
                        hipStream_t st)
{
    constexpr int N = 4 * NQ + TW;
    constexpr int NW = N <= 10 ? 16 : 8;           // 16 wavefronts leave 128 registers per lane, 8 leave 256
    PairGeom g;
    g.L1 = first_axis ? W : H;
    g.L2 = first_axis ? H : W;
    g.nd1 = g.L1 / 2;
    g.nd2 = g.L2 / 2;
    g.sA = first_axis ? 1 : W;
    g.sB = first_axis ? W : 1;
    const int Wo = W / 2;
    g.oA = first_axis ? 1 : Wo;
    g.oB = first_axis ? Wo : 1;
    g.n_in = H * W;
    g.n_out = (H / 2) * Wo;
    g.D = D;
    const PairPlan p = plan_pair(g.L2, NW, (int64_t)B * g.nd1);
    g.segs = p.segs;
    g.seg_out = p.seg_out;
    const size_t lds = (size_t)p.waves * N * 64 * 4;           // at most 16 * 10 * 256 = 40 KiB
    LUVC_LAUNCH("oim_halve_pair", (oim_halve_pair<T, NQ, TW, NW>), dim3((unsigned)((int64_t)B * g.segs * g.nd1)), dim3(64 * p.waves), lds, st,
                       x, sizes_in, g, kept_prev, x_out, sizes_out, pair_map, kept_out);
    return check_launch("oim halving pair");
}

template <typename T>
luvc_status dispatch_pair(const T* x, const int32_t* sizes_in, int B, int H, int W, int D, int first_axis,
                          const int32_t* kept_prev, T* x_out, int32_t* sizes_out, int32_t* pair_map, int32_t* kept_out,
                          hipStream_t st)
{
    // 16-byte pieces per lane, then a 4- or 8-byte tail piece if that covers what is left
    const int bytes = D * (int)sizeof(T);
    int nq = bytes / 1024, tw = 0;
    const int rem = bytes % 1024;
    if (rem > 512) ++nq;
    else if (rem > 256) tw = 2;
    else if (rem > 0) tw = 1;
#define LUVC_PAIR(Q, W_) if (nq == Q && tw == W_) return launch_pair<T, Q, W_>(x, sizes_in, B, H, W, D, first_axis, kept_prev, x_out, sizes_out, pair_map, kept_out, st)
    LUVC_PAIR(0, 1); LUVC_PAIR(0, 2);
    LUVC_PAIR(1, 0); LUVC_PAIR(1, 1); LUVC_PAIR(1, 2);
    LUVC_PAIR(2, 0); LUVC_PAIR(2, 1); LUVC_PAIR(2, 2);
    LUVC_PAIR(3, 0); LUVC_PAIR(3, 1); LUVC_PAIR(3, 2);
    LUVC_PAIR(4, 0);
#undef LUVC_PAIR
    set_error("oim pair: unsupported D");
    return LUVC_ERR_UNSUPPORTED;
}

}  // namespace

bool oim_pair_supported(int H, int W, int D, luvc_dtype dt, int axis0, int m0, int axis1, int m1, bool vec)
{
    if (!vec || axis0 == axis1) return false;
    const int len0 = axis0 ? W : H, len1 = axis1 ? W : H;           // the second pass runs on the untouched axis
    if (len0 < 2 || len1 < 2 || m0 != (len0 + 1) / 2 || m1 != (len1 + 1) / 2) return false;
    return (int64_t)D * (dt == LUVC_F32 ? 4 : 2) <= 4096;
}

luvc_status oim_pair_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int first_axis,
                          void* x_out, int32_t* sizes_out, int32_t* pair_map, const int32_t* kept_prev, int32_t* kept_out,
                          hipStream_t st)
{
    if (dt == LUVC_F32)
        return dispatch_pair<float>((const float*)x, sizes_in, B, H, W, D, first_axis, kept_prev, (float*)x_out, sizes_out,
                                    pair_map, kept_out, st);
    return dispatch_pair<bf16_t>((const bf16_t*)x, sizes_in, B, H, W, D, first_axis, kept_prev, (bf16_t*)x_out, sizes_out,
                                 pair_map, kept_out, st);
}

}  // namespace luvc
