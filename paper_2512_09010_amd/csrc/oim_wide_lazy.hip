// OIM (paper Section 3.2, Algorithm 1) with candidates beyond the adjacent destinations, for schedules that take few
// tokens out of a line per pass (the paper's appendix runs a merge number of 2): one launch per pass, and the
// tokens are moved once, at the end of the call.
//
// Between the passes a grid is not a tensor of tokens but a tensor of ROW IDS: id < n0 names a token of the call's
// input, id >= n0 a row of the "overlay", the buffer that receives every token a merge produces.  A pass reads the
// ids of its grid, fetches the tokens behind them, and writes the ids of the next grid (compacted: survivors move
// up on their line), the sizes, the anchors and the pass map; only the merged destinations - at most m per line -
// are written as tokens, into overlay rows of their own.  After the last pass oim_wide_gather copies the rows behind
// the final ids to the output.  A pass that rewrote its whole grid would move 97 % of the tokens unchanged when two
// of 64 leave a line.
//
// oim_wide_line, one workgroup per line (lines of at most 128 tokens).  The decisions are the fp64 decisions of the
// method, reached in two steps:
//   1. SCREENING.  The source x destination dot products of the line on the matrix cores in the storage precision
//      (v_mfma_f32_32x32x16_bf16, or four v_mfma_f32_32x32x2_f32 for fp32 tokens): a 32 x 32 tile at a time, the four
//      wavefronts split the channels, every token byte is fetched once per tile.  The squared norms are summed in fp64
//      on the way.  A screened cosine is taken to be within eps = (D + 2) 2^-22 of the fp64 cosine: the products of
//      bf16 values are exact in fp32, and D accumulation steps of at most 2^-23 each (relative to the sum of the
//      magnitudes of the products, which is at most the product of the norms) plus the rounding of fp32 products
//      stay below half of that; tests/test_gpu_oim_wide.py pins the contraction against fp64 on adversarial rows.
//   2. EXACT.  A source whose best screened cosine is within 2 eps of the m-th best of the line may be among the m
//      best of the line, nobody else can; for each such source, the destinations within 2 eps of its best screened
//      cosine may be its best destination, no other can.  Their dot products are repeated in fp64 (a wavefront per
//      pair), and the rules of the method - higher cosine wins, ties go to the lower position - are applied to the
//      fp64 values.  With a merge number of 2 that is a handful of pairs per line instead of 1024.
//   3. Survivor layout by ballot counts; ids / sizes / anchors / maps of the next grid.
//   4. Size-weighted mean of every destination that absorbs sources (destination first, then the sources in
//      ascending position, fp64, one rounding), a wavefront per destination.
#include "common.hpp"
#include "oim.hpp"
#include "oim_wide_tok.hpp"

namespace luvc {

namespace {

struct LazyGeom {
    int n0;         // tokens per image of the call's input grid: ids below it are rows of x
    int h, w;       // grid before this pass
    int D, axis, m, radius;
    int cap;        // overlay rows per image over the whole call
    int ov_base;    // first overlay row of this pass
    int per_line;   // overlay rows a line of this pass may write: min(m, destinations of the line)
};

// floats between the rows of the screened matrix: the smallest value of at least n_dst that is 4 mod 32
__host__ __device__ inline int lazy_row_stride(int n_dst) { return n_dst <= 4 ? 4 : 32 * ((n_dst - 4 + 31) / 32) + 4; }

template <typename T>
__device__ __forceinline__ const T* row_of(const T* x, const T* ov, int64_t b, int id, const LazyGeom& g, int D)
{
    return id < g.n0 ? x + (b * g.n0 + id) * D : ov + (b * g.cap + (id - g.n0)) * D;
}

}  // namespace

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// What a lane feeds to the matrix cores per step of the screening contraction: 16 bytes of a token.  Lane l belongs
// to row l % 32 of the tile (a source for the A side, a destination for the B side) and to half l / 32 of the
// step's channels.
template <typename T> struct screen;
template <> struct screen<bf16_t> {
    static constexpr int KS = 16, KL = 8;      // channels per step, per lane
    __device__ static __forceinline__ f32x16 mac(f32x16 acc, const u32x4& a, const u32x4& c)
    {
        bf16x8_t va, vc;
        __builtin_memcpy(&va, &a, 16);
        __builtin_memcpy(&vc, &c, 16);
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, vc, acc, 0, 0, 0);
    }
    __device__ static __forceinline__ double sq(const u32x4& a, double acc)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const double lo = (double)__uint_as_float(a[i] << 16), hi = (double)__uint_as_float(a[i] & 0xffff0000u);
            acc = fma(lo, lo, acc);
            acc = fma(hi, hi, acc);
        }
        return acc;
    }
    __device__ static __forceinline__ double dot(const u32x4& a, const u32x4& c, double acc)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc = fma((double)__uint_as_float(a[i] << 16), (double)__uint_as_float(c[i] << 16), acc);
            acc = fma((double)__uint_as_float(a[i] & 0xffff0000u), (double)__uint_as_float(c[i] & 0xffff0000u), acc);
        }
        return acc;
    }
};
template <> struct screen<float> {
    static constexpr int KS = 8, KL = 4;
    // instruction e contracts channels {e, 4 + e} of the step: the same pairing on both sides
    __device__ static __forceinline__ f32x16 mac(f32x16 acc, const u32x4& a, const u32x4& c)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]), __uint_as_float(c[e]), acc, 0, 0, 0);
        return acc;
    }
    __device__ static __forceinline__ double sq(const u32x4& a, double acc)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) { const double v = (double)__uint_as_float(a[i]); acc = fma(v, v, acc); }
        return acc;
    }
    __device__ static __forceinline__ double dot(const u32x4& a, const u32x4& c, double acc)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = fma((double)__uint_as_float(a[i]), (double)__uint_as_float(c[i]), acc);
        return acc;
    }
};

// 16 bytes of a token at channel d, zeros past its end or for a token that is not there (rows are multiples of 16 bytes)
template <typename T>
__device__ __forceinline__ u32x4 piece(const T* tok, int D, int d, bool present)
{
    u32x4 v = {0u, 0u, 0u, 0u};
    if (present && d < D) v = *reinterpret_cast<const u32x4*>(tok + d);
    return v;
}

// wave64 sum of fp64 values without the LDS crossbar: DPP adds inside each row of 16 lanes on both halves of the value,
// two row broadcasts, the total read back from lane 63
template <int CTRL, int ROWS>
__device__ __forceinline__ double dpp_mov64(double v)
{
    return __hiloint2double(__builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROWS, 0xf, false),
                            __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROWS, 0xf, false));
}
__device__ __forceinline__ double wave_total64(double v)
{
    v += dpp_mov64<0xB1, 0xf>(v);        // quad_perm [1,0,3,2]
    v += dpp_mov64<0x4E, 0xf>(v);        // quad_perm [2,3,0,1]
    v += dpp_mov64<0x141, 0xf>(v);       // row_half_mirror
    v += dpp_mov64<0x140, 0xf>(v);       // row_mirror
    v += dpp_mov64<0x142, 0xa>(v);       // row_bcast:15 -> rows 1, 3 (the other rows add the zero of the disabled lanes)
    v += dpp_mov64<0x143, 0xc>(v);       // row_bcast:31 -> rows 2, 3
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63), __builtin_amdgcn_readlane(__double2loint(v), 63));
}

// <a1, c1> and <a2, c2> in fp64 by one wavefront, all fetches of both in flight together
template <typename T>
__device__ __forceinline__ void dot64_wave2(const T* a1, const T* c1, const T* a2, const T* c2, int D, int lane, double& d1, double& d2)
{
    constexpr int V = 16 / (int)sizeof(T);
    double acc1 = 0.0, acc2 = 0.0;
    for (int d0 = 0; d0 < D; d0 += 64 * V * 4) {
        u32x4 ra1[4], rc1[4], ra2[4], rc2[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int d = d0 + (u * 64 + lane) * V;
            ra1[u] = piece(a1, D, d, true);
            rc1[u] = piece(c1, D, d, true);
            ra2[u] = piece(a2, D, d, true);
            rc2[u] = piece(c2, D, d, true);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc1 = screen<T>::dot(ra1[u], rc1[u], acc1);
            acc2 = screen<T>::dot(ra2[u], rc2[u], acc2);
        }
    }
    d1 = wave_total64(acc1);
    d2 = wave_total64(acc2);
}

__device__ __forceinline__ float quad_max(float v)
{
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true)));    // lane ^ 1
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true)));    // lane ^ 2
    return v;
}

}  // namespace

// the screening tile of one wavefront over all channels (a test hook: tests pin the contraction's error against fp64).
// a, c: [32, D] rows; out[i * 32 + j] = <a_i, c_j>.
template <typename T>
__global__ void __launch_bounds__(64)
selftest_screen_tile(const T* __restrict__ a, const T* __restrict__ c, int D, float* __restrict__ out)
{
    using sc = screen<T>;
    const int lane = threadIdx.x, r = lane & 31, kh = lane >> 5;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int d = 0; d < D; d += sc::KS)         // the same trip count in every lane: the matrix instructions want the whole wavefront
        acc = sc::mac(acc, piece(a + (int64_t)r * D, D, d + kh * sc::KL, true), piece(c + (int64_t)r * D, D, d + kh * sc::KL, true));
#pragma unroll
    for (int v = 0; v < 16; ++v) out[(8 * (v >> 2) + 4 * kh + (v & 3)) * 32 + r] = acc[v];
}

constexpr int kLazyLoads = 8;                    // steps of the screening contraction fetched before the first is used
template <typename T>
__global__ void __launch_bounds__(256)
oim_wide_line(const T* __restrict__ x, T* ov, const T* __restrict__ xk /* metric [.., Dk] the decisions are taken on, or null: x */,
              T* ovk /* its overlay */, int Dk, const int32_t* __restrict__ idx_in /* null: identity */,
              const int32_t* __restrict__ sizes_in /* null: ones */, const int32_t* __restrict__ kept_in /* null: identity */,
              LazyGeom g, int32_t* __restrict__ idx_out, int32_t* __restrict__ sizes_out, int32_t* __restrict__ kept_out /* or null */,
              int32_t* __restrict__ pass_map /* or null */)
{
    using sc = screen<T>;
    using tr = io_traits<T>;
    constexpr int V = tr::kVec;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int len = g.axis ? g.w : g.h, nlines = g.axis ? g.h : g.w;
    const int n_src = (len + 1) / 2, n_dst = len / 2;
    const int Wo = g.axis ? g.w - g.m : g.w, Ho = g.axis ? g.h : g.h - g.m;
    double* pn = reinterpret_cast<double*>(smem_raw);    // [4][len] squared norms, the part of each wavefront
    double* nrm = pn + 4 * len;                          // [len] max(norm, 1e-12)
    float* P = reinterpret_cast<float*>(nrm + len);      // [4][32 * 32] a tile, the part of each wavefront; later the list of pairs
    // [n_src][sd] screened dot products, then cosines; later [pairs] fp64 cosines.  Rows are sd = 4 mod 32 floats apart, so
    // that the four lanes per source of the cosine step fall into different banks
    float* S = P + 4 * 1024;
    const int sd = lazy_row_stride(n_dst);
    float* b32 = S + n_src * max(2 * n_dst, sd);         // [n_src] best screened cosine
    float* inv32 = b32 + n_src;                          // [len] 1 / nrm
    int* rid = reinterpret_cast<int*>(inv32 + len);      // [len] row id of the token at position p
    int* sz = rid + len;                                 // [len] its size
    int* snew = sz + len;                                // [len] its size after the pass (survivors)
    int* addsz = snew + len;                             // [len] sizes of the sources a destination takes in
    int* best = addsz + len;                             // [n_src] position of the best destination, -1: not looked at
    int* pstart = best + n_src;                          // [n_src] first pair of the source in the list
    int* pcount = pstart + n_src;                        // [n_src] its number of pairs
    int* slot_of = pcount + n_src;                       // [len]
    int* dlist = slot_of + len;                          // [len] destinations that absorb sources, ascending
    int* tot = dlist + len;                              // [4] counts handed between the wavefronts
    int* npairs = tot + 4;                               // [1]
    float* thr = reinterpret_cast<float*>(npairs + 1);   // [1] m-th best screened cosine of the line
    unsigned char* merged = reinterpret_cast<unsigned char*>(thr + 1);   // [len]
    unsigned char* absorb = merged + len;                // [len]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x / nlines;
    const int line = blockIdx.x % nlines;
    const int64_t img = b * g.h * g.w, img_out = b * Ho * Wo;
    auto in_flat = [&](int p) -> int { return g.axis ? line * g.w + p : p * g.w + line; };
    auto out_flat = [&](int q) -> int { return g.axis ? line * Wo + q : q * Wo + line; };
    // eps: bound of |screened cosine - fp64 cosine| (head of this file); both selections use 2 eps
    // the tensor the decisions are taken on
    const T* dx = xk ? xk : x;
    const T* dov = xk ? ovk : ov;
    const int dD = xk ? Dk : g.D;
    const float tau = 2.f * (float)(dD + 2) * 2.3841858e-7f;

    for (int p = tid; p < len; p += blockDim.x) {
        const int f = in_flat(p);
        rid[p] = idx_in ? idx_in[img + f] : f;
        sz[p] = sizes_in ? sizes_in[img + f] : 1;
        merged[p] = 0;
    }
    if (tid == 0) {
        *thr = -INFINITY;                                // stays there only if the cosines do not order (NaN): then every source is looked at
        *npairs = 0;
    }
    __syncthreads();

    // ------------------------------------------------------------------ 1. screening: dot products and squared norms
    // Result layout of the 32 x 32 instructions: lane l, register v holds row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32.
    {
        const int tiles_s = (n_src + 31) / 32, tiles_d = (n_dst + 31) / 32;
        const int r = lane & 31, kh = lane >> 5;
        for (int t = 0; t < tiles_s * tiles_d; ++t) {
            const int ts = t / tiles_d, td = t % tiles_d;
            const int js = ts * 32 + r, jd = td * 32 + r;
            const bool has_s = js < n_src, has_d = jd < n_dst;
            const T* tok_s = row_of<T>(dx, dov, b, has_s ? rid[2 * js] : rid[0], g, dD);
            const T* tok_d = row_of<T>(dx, dov, b, has_d ? rid[2 * jd + 1] : rid[0], g, dD);
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            double na = 0.0, nc = 0.0;
            // wavefront w takes steps w, w + 4, ... of KS channels, a lane its half of each; the trip count is the same in
            // every lane (the matrix instructions want the whole wavefront), pieces past the end of the token are zeros
            for (int d0 = wave * sc::KS; d0 < dD; d0 += 4 * sc::KS * kLazyLoads) {
                u32x4 ra[kLazyLoads], rc[kLazyLoads];
#pragma unroll
                for (int u = 0; u < kLazyLoads; ++u) {
                    ra[u] = piece(tok_s, dD, d0 + 4 * sc::KS * u + kh * sc::KL, has_s);
                    rc[u] = piece(tok_d, dD, d0 + 4 * sc::KS * u + kh * sc::KL, has_d);
                }
#pragma unroll
                for (int u = 0; u < kLazyLoads; ++u) {
                    acc = sc::mac(acc, ra[u], rc[u]);
                    if (td == 0) na = sc::sq(ra[u], na);
                    if (ts == 0) nc = sc::sq(rc[u], nc);
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) P[wave * 1024 + (8 * (v >> 2) + 4 * kh + (v & 3)) * 32 + r] = acc[v];
            na += __shfl_xor(na, 32, kWave);                              // the two channel halves of a step
            nc += __shfl_xor(nc, 32, kWave);
            if (kh == 0) {
                if (td == 0 && has_s) pn[wave * len + 2 * js] = na;
                if (ts == 0 && has_d) pn[wave * len + 2 * jd + 1] = nc;
            }
            __syncthreads();
            for (int e = tid; e < 1024; e += 256) {
                const int row = ts * 32 + (e >> 5), col = td * 32 + (e & 31);
                if (row < n_src && col < n_dst) S[row * sd + col] = ((P[e] + P[1024 + e]) + P[2048 + e]) + P[3072 + e];
            }
            __syncthreads();
        }
    }
    for (int p = tid; p < len; p += blockDim.x) {
        double v = 1.0;                                  // a line of one token has no products and no decisions
        if (n_dst > 0) v = sqrt(((pn[p] + pn[len + p]) + pn[2 * len + p]) + pn[3 * len + p]);
        v = v < 1e-12 ? 1e-12 : v;
        nrm[p] = v;
        inv32[p] = (float)(1.0 / v);
        addsz[p] = 0;
        absorb[p] = 0;
    }
    __syncthreads();
    // screened cosines (fp32 from here: four more roundings, inside the "+ 2" of eps) and the best of each source:
    // four lanes per source
    {
        const int j = tid >> 2, part = tid & 3;
        float mx = -INFINITY;
        if (j < n_src) {
            const int a = 2 * j;
            const float ia = inv32[a];
            for (int k = part; k < n_dst; k += 4) {
                const int c = 2 * k + 1;
                const int dist = c > a ? c - a : a - c;
                float s = -INFINITY;                     // outside the radius: never a candidate
                if (g.radius <= 0 || dist <= 2 * g.radius - 1) s = (S[j * sd + k] * ia) * inv32[c];
                S[j * sd + k] = s;
                mx = fmaxf(mx, s);
            }
        }
        mx = quad_max(mx);
        if (j < n_src && part == 0) b32[j] = mx;
    }
    __syncthreads();
    // the m-th best of them: the value v with fewer than m values above it and at least m values not below it
    // (wavefront 0, a source per lane, the values passed around in registers)
    if (wave == 0 && g.m > 0 && g.m < n_src) {
        const float v = lane < n_src ? b32[lane] : -INFINITY;
        int gt = 0, ge = 0;
        for (int i = 0; i < n_src; ++i) {
            const float t = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), i));
            gt += t > v ? 1 : 0;
            ge += t >= v ? 1 : 0;
        }
        if (lane < n_src && gt < g.m && g.m <= ge) *thr = v;
    }
    __syncthreads();

    // ------------------------------------------------------------------ 2. exact: fp64 cosines where the screening cannot tell
    // the (source, destination) pairs to repeat: a wavefront scans every fourth source, its lanes one destination each
    int* pairs = reinterpret_cast<int*>(P);              // the tile buffer is free: up to n_src * n_dst <= 4096 pairs
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int j = wave; j < n_src; j += 4) {
        const float bj = b32[j];
        const bool contender = g.m > 0 && bj > -INFINITY && (g.m == n_src || bj >= *thr - tau);
        int start = 0, cnt = 0;
        if (contender) {                                 // wave-uniform
            const unsigned long long cand = __ballot(lane < n_dst && S[j * sd + lane] >= bj - tau);
            cnt = __popcll(cand);
            if (lane == 0) start = atomicAdd(npairs, cnt);
            start = __builtin_amdgcn_readfirstlane(start);
            if ((cand >> lane) & 1ull) pairs[start + __popcll(cand & below)] = (j << 8) | lane;   // ascending destination
        }
        if (lane == 0) { pstart[j] = start; pcount[j] = cnt; }
    }
    __syncthreads();
    // their fp64 cosines, a wavefront per pair, two pairs in flight; S is dead from here and the values take its place
    double* E = reinterpret_cast<double*>(S);
    {
        const int np = *npairs;
        for (int i = wave; i < np; i += 8) {
            const bool two = i + 4 < np;
            const int pr1 = pairs[i], pr2 = pairs[two ? i + 4 : i];
            const int a1 = 2 * (pr1 >> 8), c1 = 2 * (pr1 & 255) + 1, a2 = 2 * (pr2 >> 8), c2 = 2 * (pr2 & 255) + 1;
            double d1, d2;
            dot64_wave2<T>(row_of<T>(dx, dov, b, rid[a1], g, dD), row_of<T>(dx, dov, b, rid[c1], g, dD), row_of<T>(dx, dov, b, rid[a2], g, dD),
                           row_of<T>(dx, dov, b, rid[c2], g, dD), dD, lane, d1, d2);
            if (lane == 0) {
                E[i] = d1 / (nrm[a1] * nrm[c1]);
                if (two) E[i + 4] = d2 / (nrm[a2] * nrm[c2]);
            }
        }
    }
    __syncthreads();
    // best destination of every source looked at (higher cosine wins, equal cosines keep the lower position), then the m
    // best sources (higher cosine, equal cosines: lower position): wavefront 0, a source per lane; the sources not looked
    // at are below all of these
    if (wave == 0) {
        const int j = lane;
        double bs = -INFINITY;
        int bc = -1;
        if (j < n_src) {
            const int st = pstart[j], cn = pcount[j];
            for (int i = 0; i < cn; ++i) {
                const double s = E[st + i];
                const int c = 2 * (pairs[st + i] & 255) + 1;
                if (bc < 0 || s > bs || (s == bs && c < bc)) { bs = s; bc = c; }
            }
            best[j] = bc;
        }
        bool mg = false;
        if (g.m == n_src) {
            mg = bc >= 0;
        } else if (g.m > 0) {
            unsigned long long looked = __ballot(bc >= 0);
            int rank = 0;
            while (looked) {                             // wave-uniform
                const int i = (int)__builtin_ctzll(looked);
                looked &= looked - 1;
                const double t = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(bs), i), __builtin_amdgcn_readlane(__double2loint(bs), i));
                rank += (t > bs || (t == bs && i < j)) ? 1 : 0;
            }
            mg = bc >= 0 && rank < g.m;
        }
        if (mg) {
            merged[2 * j] = 1;
            atomicAdd(&addsz[bc], sz[2 * j]);
            absorb[bc] = 1;
        }
    }
    __syncthreads();

    // ------------------------------------------------------------------ 3. layout of the next grid
    // thread p looks at position p (len <= 128: wavefronts 0 and 1); counts before a position by ballot
    {
        const int p = tid;
        const bool alive = p < len && !merged[p];
        const bool absorbs = alive && absorb[p];         // a destination that takes in sources (destinations are never merged)
        const int Sz = p < len ? sz[p] + addsz[p] : 0;
        const unsigned long long bal_a = __ballot(alive), bal_d = __ballot(absorbs);
        int q = __popcll(bal_a & below), k = __popcll(bal_d & below);
        if (wave == 0 && lane == 0) { tot[0] = __popcll(bal_a); tot[1] = __popcll(bal_d); }
        if (wave == 1 && lane == 0) tot[2] = __popcll(bal_d);
        __syncthreads();
        if (wave == 1) { q += tot[0]; k += tot[1]; }
        if (alive) {
            const int of = out_flat(q), f = in_flat(p);
            slot_of[p] = of;
            snew[p] = Sz;
            if (absorbs) dlist[k] = p;
            idx_out[img_out + of] = absorbs ? g.n0 + g.ov_base + line * g.per_line + k : rid[p];
            sizes_out[img_out + of] = Sz;
            if (kept_out) kept_out[img_out + of] = kept_in ? kept_in[img + f] : f;
            if (pass_map) pass_map[img + f] = of;
        }
    }
    __syncthreads();
    if (pass_map)
        for (int j = tid; j < n_src; j += blockDim.x)
            if (merged[2 * j]) pass_map[img + in_flat(2 * j)] = slot_of[best[j]];    // a merged source lands in its destination's slot

    // ------------------------------------------------------------------ 4. the merged destinations
    // the destination's pieces and those of the first two sources are in flight together
    // (features, and the metric too when the decisions were taken on one: it follows its own decisions)
    const int n_abs = tot[1] + tot[2];
    for (int kk = wave; kk < (xk ? 2 : 1) * n_abs; kk += 4) {
        const bool on_metric = kk >= n_abs;
        const int k = on_metric ? kk - n_abs : kk;
        const T* mx = on_metric ? xk : x;
        T* mov = on_metric ? ovk : ov;
        const int mD = on_metric ? Dk : g.D;
        const int c = dlist[k];
        const T* xp = row_of<T>(mx, mov, b, rid[c], g, mD);
        T* o = mov + (b * g.cap + g.ov_base + line * g.per_line + k) * mD;
        const double sp = (double)sz[c], dS = (double)snew[c];
        const unsigned long long hits = __ballot(lane < n_src && merged[2 * lane] && best[lane] == c);   // n_src <= 64
        for (int d0 = 0; d0 < mD; d0 += 64 * V * 4) {
            double acc[4][V];
            {
                u32x4 rp[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) rp[u] = piece(xp, mD, d0 + (u * 64 + lane) * V, true);
                unsigned long long h = hits;
                bool first = true;
                do {
                    const int j1 = h ? (int)__builtin_ctzll(h) : -1;
                    h &= h - 1;
                    const int j2 = h ? (int)__builtin_ctzll(h) : -1;
                    h &= h - 1;
                    const T* x1 = row_of<T>(mx, mov, b, rid[j1 >= 0 ? 2 * j1 : 0], g, mD);
                    const T* x2 = row_of<T>(mx, mov, b, rid[j2 >= 0 ? 2 * j2 : 0], g, mD);
                    u32x4 r1[4], r2[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        r1[u] = piece(x1, mD, d0 + (u * 64 + lane) * V, j1 >= 0);
                        r2[u] = piece(x2, mD, d0 + (u * 64 + lane) * V, j2 >= 0);
                    }
                    const double s1 = j1 >= 0 ? (double)sz[2 * j1] : 0.0, s2 = j2 >= 0 ? (double)sz[2 * j2] : 0.0;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        float f[V];
                        if (first) {
                            tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(&rp[u]), f);
#pragma unroll
                            for (int i = 0; i < V; ++i) acc[u][i] = sp * (double)f[i];
                        }
                        if (j1 >= 0) {
                            tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(&r1[u]), f);
#pragma unroll
                            for (int i = 0; i < V; ++i) acc[u][i] += s1 * (double)f[i];
                        }
                        if (j2 >= 0) {
                            tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(&r2[u]), f);
#pragma unroll
                            for (int i = 0; i < V; ++i) acc[u][i] += s2 * (double)f[i];
                        }
                    }
                    first = false;
                } while (h);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int d = d0 + (u * 64 + lane) * V;
                if (d >= mD) continue;
                T r[V];
#pragma unroll
                for (int i = 0; i < V; ++i) tr::store(&r[i], acc[u][i] / dS);
                *reinterpret_cast<typename tr::vec_t*>(o + d) = *reinterpret_cast<const typename tr::vec_t*>(r);
            }
        }
    }
}

// ------------------------------------------------------------------ the rows behind the final ids
typedef unsigned int lazy_u32x4 __attribute__((__vector_size__(16)));
__device__ __forceinline__ const unsigned char* lazy_row(const unsigned char* x, const unsigned char* ov, const int32_t* idx, int64_t row,
                                                         int n0, int cap, int n_out_per, int row_bytes)
{
    const int64_t b = row / n_out_per;
    int id = idx[row];
    id = id < 0 ? 0 : (id >= n0 + cap ? n0 + cap - 1 : id);            // ids come from oim_wide_line; stay in bounds regardless
    return id < n0 ? x + (b * n0 + id) * (int64_t)row_bytes : ov + (b * cap + (id - n0)) * (int64_t)row_bytes;
}

// one wavefront per row
__global__ void __launch_bounds__(256)
oim_wide_gather(const unsigned char* __restrict__ x, const unsigned char* __restrict__ ov, const int32_t* __restrict__ idx,
                int n0, int cap, int n_out_per, int row_bytes, int64_t n_rows, unsigned char* __restrict__ x_out)
{
    const int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const unsigned char* in = lazy_row(x, ov, idx, row, n0, cap, n_out_per, row_bytes);
    unsigned char* o = x_out + row * (int64_t)row_bytes;
    // eight 16-byte pieces per lane in flight before the first store; the descriptors bound every piece
    const __amdgpu_buffer_rsrc_t ri = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(in), 0, row_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(o, 0, row_bytes, 0x00020000);
    for (int base = 0; base < row_bytes; base += 8 * 1024) {
        lazy_u32x4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = __builtin_amdgcn_raw_buffer_load_b128(ri, base + k * 1024 + lane * 16, 0, 0);
#pragma unroll
        for (int k = 0; k < 8; ++k) __builtin_amdgcn_raw_buffer_store_b128(v[k], ro, base + k * 1024 + lane * 16, 0, 2);
    }
}

// short rows (at most 512 bytes, e.g. the keys of one attention head): LPR = 16 or 32 lanes per row, several rows per
// wavefront, so that a launch has a quarter or half of the wavefronts - each is three memory round trips long whatever it moves
template <int LPR>
__global__ void __launch_bounds__(256)
oim_wide_gather_short(const unsigned char* __restrict__ x, const unsigned char* __restrict__ ov, const int32_t* __restrict__ idx,
                      int n0, int cap, int n_out_per, int row_bytes, int64_t n_rows, unsigned char* __restrict__ x_out)
{
    constexpr int RPW = 64 / LPR;
    const int lane = threadIdx.x & 63, sub = lane % LPR;
    const int64_t row = (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6) * RPW + lane / LPR;
    if (row >= n_rows) return;
    const unsigned char* in = lazy_row(x, ov, idx, row, n0, cap, n_out_per, row_bytes);
    unsigned char* o = x_out + row * (int64_t)row_bytes;
    const int off = sub * 16;
    if (off < row_bytes) *reinterpret_cast<lazy_u32x4*>(o + off) = *reinterpret_cast<const lazy_u32x4*>(in + off);
}

// ------------------------------------------------------------------ host side
int oim_wide_lazy_rows(int h, int w, int axis, int m)
{
    const int len = axis ? w : h, nlines = axis ? h : w, n_dst = len / 2;
    return nlines * (m < n_dst ? m : n_dst);
}

template <typename T>
static luvc_status run_lazy_pass(const T* x, T* ov, const T* xk, T* ovk, int Dk, const int32_t* idx_in, const int32_t* sizes_in, const int32_t* kept_in,
                                 int B, int n0, int h, int w, int D, int axis, int m, int radius, int cap, int ov_base,
                                 int32_t* idx_out, int32_t* sizes_out, int32_t* kept_out, int32_t* pass_map, hipStream_t st)
{
    const int len = axis ? w : h, nlines = axis ? h : w, n_src = (len + 1) / 2, n_dst = len / 2;
    if (len > kLazyMaxLen) { set_error("wide matching (one launch per pass): line of %d tokens", len); return LUVC_ERR_UNSUPPORTED; }
    LazyGeom g;
    g.n0 = n0; g.h = h; g.w = w; g.D = D; g.axis = axis; g.m = m; g.radius = radius; g.cap = cap; g.ov_base = ov_base;
    g.per_line = m < n_dst ? m : n_dst;
    const int sd = lazy_row_stride(n_dst);
    const size_t lds = sizeof(double) * ((size_t)5 * len) + sizeof(float) * ((size_t)n_src * (2 * n_dst > sd ? 2 * n_dst : sd) + 4096 + n_src + len) +
                       sizeof(int) * ((size_t)6 * len + 3 * n_src + 6) + (size_t)2 * len + 16;
    LUVC_LAUNCH("oim_wide_line", (oim_wide_line<T>), dim3((unsigned)(B * nlines)), dim3(256), lds, st, x, ov, xk, ovk, Dk, idx_in, sizes_in, kept_in, g,
                idx_out, sizes_out, kept_out, pass_map);
    return check_launch("oim pass (wide matching, one launch)");
}

luvc_status oim_wide_lazy_pass(const void* x, void* ov, const void* metric, void* ov_metric, int Dm, const int32_t* idx_in, const int32_t* sizes_in, const int32_t* kept_in,
                               int B, int n0, int h, int w, int D, luvc_dtype dt, int axis, int m, int radius, int cap, int ov_base,
                               int32_t* idx_out, int32_t* sizes_out, int32_t* kept_out, int32_t* pass_map, hipStream_t st)
{
    if (dt == LUVC_F32)
        return run_lazy_pass<float>((const float*)x, (float*)ov, (const float*)metric, (float*)ov_metric, Dm, idx_in, sizes_in, kept_in, B, n0, h, w, D, axis, m, radius, cap, ov_base,
                                    idx_out, sizes_out, kept_out, pass_map, st);
    return run_lazy_pass<bf16_t>((const bf16_t*)x, (bf16_t*)ov, (const bf16_t*)metric, (bf16_t*)ov_metric, Dm, idx_in, sizes_in, kept_in, B, n0, h, w, D, axis, m, radius, cap, ov_base,
                                 idx_out, sizes_out, kept_out, pass_map, st);
}

luvc_status oim_wide_lazy_gather(const void* x, const void* ov, const int32_t* idx, int B, int n0, int cap, int n_out_per, int D,
                                 luvc_dtype dt, void* x_out, hipStream_t st)
{
    const int64_t rows = (int64_t)B * n_out_per;
    const int row_bytes = D * (dt == LUVC_F32 ? 4 : 2);
    if (row_bytes <= 512) {
        const int rpw = row_bytes <= 256 ? 4 : 2;
        const unsigned grid = (unsigned)(((rows + rpw - 1) / rpw * 64 + 255) / 256);
        if (rpw == 4) LUVC_LAUNCH("oim_wide_gather", (oim_wide_gather_short<16>), dim3(grid), dim3(256), 0, st, (const unsigned char*)x, (const unsigned char*)ov, idx,
                                  n0, cap, n_out_per, row_bytes, rows, (unsigned char*)x_out);
        else          LUVC_LAUNCH("oim_wide_gather", (oim_wide_gather_short<32>), dim3(grid), dim3(256), 0, st, (const unsigned char*)x, (const unsigned char*)ov, idx,
                                  n0, cap, n_out_per, row_bytes, rows, (unsigned char*)x_out);
        return check_launch("oim wide matching, output rows");
    }
    const unsigned grid = (unsigned)((rows * 64 + 255) / 256);
    LUVC_LAUNCH("oim_wide_gather", oim_wide_gather, dim3(grid), dim3(256), 0, st, (const unsigned char*)x, (const unsigned char*)ov, idx,
                n0, cap, n_out_per, row_bytes, rows, (unsigned char*)x_out);
    return check_launch("oim wide matching, output rows");
}

}  // namespace luvc

extern "C" luvc_status luvc_selftest_screen_tile(const void* a, const void* c, int D, luvc_dtype dtype, float* out, void* hip_stream)
{
    using namespace luvc;
    const int es = dtype == LUVC_F32 ? 4 : 2;
    if ((dtype != LUVC_F32 && dtype != LUVC_BF16) || !a || !c || !out || D < 1 || (D * es) % 16 != 0 ||
        ((uintptr_t)a | (uintptr_t)c) % 16 || (uintptr_t)out % 4) {
        set_error("luvc_selftest_screen_tile: unknown dtype, null or misaligned pointer, or rows that are not multiples of 16 bytes");
        return LUVC_ERR_INVALID_ARG;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    if (dtype == LUVC_F32) LUVC_LAUNCH("selftest_screen_tile", (selftest_screen_tile<float>), dim3(1), dim3(64), 0, st, (const float*)a, (const float*)c, D, out);
    else                   LUVC_LAUNCH("selftest_screen_tile", (selftest_screen_tile<bf16_t>), dim3(1), dim3(64), 0, st, (const bf16_t*)a, (const bf16_t*)c, D, out);
    return check_launch("selftest screen tile");
}
