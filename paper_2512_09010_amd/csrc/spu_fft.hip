// SPU score (paper Section 3.3, Eq. 4-8): fast path for N = N1 * N2 with N1 = 16 * Q, Q in {16, 15, 9},
// and 2*sigma + 1 <= N1 (N = 1024, 2048, 720, 144 ... of the benchmark workloads).
//
// Two real channels (d, d+1) are packed as one complex signal z = x_d + i x_{d+1}.  The mask of
// Eq. 5 is real and symmetric in k, so the filter is a real linear operator and Re / Im of the
// filtered z are the two filtered channels: no unpacking is ever needed.
//
// Transform decomposition along the token index, n = N2 * n1 + n2 (n1 < N1, n2 < N2):
//   Eq. 4 on the pass band:  F[k] = sum_{n2} W_N^{k n2} Y_{n2}[k mod N1],  |k| <= sigma,
//                            Y_{n2} = N1-point DFT of the stride-N2 subsequence n2;
//   Eq. 6:                   F[k] *= M[|k|] / N;
//   Eq. 7:                   z'[N2 n1 + n2] = N1-point inverse DFT over k1 of F[k] W_N^{-k n2};
//   Eq. 8:                   |z'|^2 summed over the channel pairs of the tile.
// Each N1-point transform is 16 x Q (n1 = Q j + t, k1 = ka + 16 kb): a radix-16 butterfly over j held
// in registers, the twiddle W_N1^{t ka}, one exchange through LDS, and a Q-point transform over t
// (radix-16 again, or 3 x 5 by the prime-factor map, or 3 x 3).  A workgroup owns 16 channel pairs
// (32 channels, 64-byte row segments for bf16); thread (c, t) = (pair, residue): Q of the 16 residue
// threads hold 16 points each for the radix-16 side, all 16 hold Q points each for the other side.
// The pass-band accumulators F stay in registers across the N2 subsequences, so x is read exactly
// once and nothing but N floats per tile is written.
//
// Thinned inverse.  The energy of a token over the channels of a tile, e[n] = sum_d x'[n,d]^2, is a trigonometric
// polynomial of degree <= 2 sigma in n, so its values at the tokens n = dec * m (dec divides N2, N / dec >
// 4 sigma) fix all N of them.  The inverse therefore runs on every dec-th subsequence first; the workgroup fills
// in the tokens between with a Kaiser-windowed sinc (fp64 taps and sums; cut-off half the coarse rate, stop band
// 140 dB down: design error 1e-7 of the energies around the token) and checks, token by token, that the value it
// got is not small against the absolute sum  a[n] = sum |tap| e[m]  it came from: e^[n] >= a[n] / 8.  The fp32
// transform leaves an absolute error of about eps x_rms on every filtered value, whatever its size, hence
// 2 sqrt(e[m]) eps x_rms on an energy; a filled-in energy collects sum |tap| times that, and the score, its square
// root, (sum |tap| sqrt(e[m])) / sqrt(e[n]) times the error the full inverse would leave on it.  The check keeps the
// energies around a filled-in token within about three times its own (the taps sum to about 2.5 in absolute value),
// so that factor stays below five: a tile that passes hands over scores whose error is a few 1e-7 of the sample's
// largest score at worst, next to the 1e-7 of the full inverse.  The design error of the kernel is of another
// kind: what the window cuts off the sinc only cancels for a band-limited sequence as a whole, so the error is
// about 2e-7 of the LARGEST energy anywhere near, not of the token's own - a filled-in token must therefore also
// reach 1/32 of the tile's largest coarse energy (then the design error is below 7e-6 of its energy, 3.2e-6 of its
// score).  The sum over tiles inherits both bounds.  A tile with a token that fails either test (a token whose
// filtered channels all but vanish where others' do not) runs the remaining subsequences and hands over what
// Eq. 7-8 say, as if dec were 1.
#include <type_traits>

#include "common.hpp"
#include "spu.hpp"
#include "spu_tiles.hpp"

namespace luvc {

namespace {

struct cf { float x, y; };
__device__ __forceinline__ cf operator+(cf a, cf b) { return {a.x + b.x, a.y + b.y}; }
__device__ __forceinline__ cf operator-(cf a, cf b) { return {a.x - b.x, a.y - b.y}; }
__device__ __forceinline__ cf cmul(cf a, cf w) { return {fmaf(a.x, w.x, -a.y * w.y), fmaf(a.x, w.y, a.y * w.x)}; }
__device__ __forceinline__ cf cmulc(cf a, cf w) { return {fmaf(a.x, w.x, a.y * w.y), fmaf(a.y, w.x, -a.x * w.y)}; }   // a * conj(w)

// radix-4 butterfly, INV = false: e^{-i...}; true: e^{+i...}
template <bool INV>
__device__ __forceinline__ void bf4(cf& a0, cf& a1, cf& a2, cf& a3)
{
    const cf t0 = a0 + a2, t1 = a0 - a2, t2 = a1 + a3, d = a1 - a3;
    const cf t3 = INV ? cf{-d.y, d.x} : cf{d.y, -d.x};          // d * (+i) or d * (-i)
    a0 = t0 + t2; a1 = t1 + t3; a2 = t0 - t2; a3 = t1 - t3;
}

// 16-point DFT in registers: X[k] = sum_j v[j] e^{-+ 2 pi i jk/16}; natural order in, natural order out
template <bool INV>
__device__ __forceinline__ void fft16(cf (&v)[16])
{
    constexpr float c1 = 0.9238795325112867f, s1 = 0.3826834323650898f, r = 0.7071067811865476f;
#pragma unroll
    for (int i = 0; i < 4; ++i) bf4<INV>(v[i], v[i + 4], v[i + 8], v[i + 12]);
    // v[i + 4q] now holds the q-th output of column i; twiddle by W16^{i q}
    const cf w1{c1, -s1}, w2{r, -r}, w3{s1, -c1}, w6{-r, -r}, w9{-c1, s1};
    auto tw = [](cf a, cf w) { return INV ? cmulc(a, w) : cmul(a, w); };
    v[1 + 4] = tw(v[1 + 4], w1);  v[1 + 8] = tw(v[1 + 8], w2);  v[1 + 12] = tw(v[1 + 12], w3);
    v[2 + 4] = tw(v[2 + 4], w2);
    v[2 + 8] = INV ? cf{-v[2 + 8].y, v[2 + 8].x} : cf{v[2 + 8].y, -v[2 + 8].x};     // W16^4 = -i
    v[2 + 12] = tw(v[2 + 12], w6);
    v[3 + 4] = tw(v[3 + 4], w3);  v[3 + 8] = tw(v[3 + 8], w6);  v[3 + 12] = tw(v[3 + 12], w9);
#pragma unroll
    for (int q = 0; q < 4; ++q) bf4<INV>(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    // v[4q + p] holds X[q + 4p]: transpose the 4x4 index back to natural order
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int p = q + 1; p < 4; ++p) { const cf s = v[4 * q + p]; v[4 * q + p] = v[4 * p + q]; v[4 * p + q] = s; }
}

// 3-point DFT (INV: conjugate twiddles)
template <bool INV>
__device__ __forceinline__ void dft3(cf& a, cf& b, cf& c)
{
    constexpr float s3 = 0.8660254037844386f;
    const cf t = b + c, m{a.x - 0.5f * t.x, a.y - 0.5f * t.y};
    const cf d{(b.x - c.x) * s3, (b.y - c.y) * s3};
    const cf r = INV ? cf{-d.y, d.x} : cf{d.y, -d.x};          // d * (+i) or d * (-i)
    a = a + t; b = m + r; c = m - r;
}

// 5-point DFT
template <bool INV>
__device__ __forceinline__ void dft5(cf& x0, cf& x1, cf& x2, cf& x3, cf& x4)
{
    constexpr float c1 = 0.30901699437494745f, c2 = -0.8090169943749475f, s1 = 0.9510565162951535f, s2 = 0.5877852522924731f;
    const cf t1 = x1 + x4, t2 = x2 + x3, t3 = x1 - x4, t4 = x2 - x3;
    const cf m1{fmaf(c2, t2.x, fmaf(c1, t1.x, x0.x)), fmaf(c2, t2.y, fmaf(c1, t1.y, x0.y))};
    const cf m2{fmaf(c1, t2.x, fmaf(c2, t1.x, x0.x)), fmaf(c1, t2.y, fmaf(c2, t1.y, x0.y))};
    const cf u1{fmaf(s2, t4.x, s1 * t3.x), fmaf(s2, t4.y, s1 * t3.y)};
    const cf u2{fmaf(-s1, t4.x, s2 * t3.x), fmaf(-s1, t4.y, s2 * t3.y)};
    const cf r1 = INV ? cf{-u1.y, u1.x} : cf{u1.y, -u1.x};
    const cf r2 = INV ? cf{-u2.y, u2.x} : cf{u2.y, -u2.x};
    x0 = x0 + t1 + t2;
    x1 = m1 + r1; x4 = m1 - r1;
    x2 = m2 + r2; x3 = m2 - r2;
}

// Q-point DFT in registers, natural order in and out
template <int Q, bool INV> struct dftq;
template <bool INV> struct dftq<16, INV> {
    __device__ static __forceinline__ void run(cf (&v)[16]) { fft16<INV>(v); }
};
template <bool INV> struct dftq<15, INV> {
    // prime-factor map (no twiddles): n = (5 n1 + 3 n2) mod 15, k = (10 k1 + 6 k2) mod 15
    __device__ static __forceinline__ void run(cf (&v)[15])
    {
        cf u[3][5];
#pragma unroll
        for (int n2 = 0; n2 < 5; ++n2) {
            cf a = v[(3 * n2) % 15], b = v[(5 + 3 * n2) % 15], c = v[(10 + 3 * n2) % 15];
            dft3<INV>(a, b, c);
            u[0][n2] = a; u[1][n2] = b; u[2][n2] = c;
        }
#pragma unroll
        for (int k1 = 0; k1 < 3; ++k1) {
            dft5<INV>(u[k1][0], u[k1][1], u[k1][2], u[k1][3], u[k1][4]);
#pragma unroll
            for (int k2 = 0; k2 < 5; ++k2) v[(10 * k1 + 6 * k2) % 15] = u[k1][k2];
        }
    }
};
template <bool INV> struct dftq<9, INV> {
    // 3 x 3: n = 3 n1 + n2, k = k1 + 3 k2, twiddle W_9^{n2 k1}
    __device__ static __forceinline__ void run(cf (&v)[9])
    {
        constexpr float c1 = 0.766044443118978f, s1 = 0.6427876096865393f;      // W_9^1
        constexpr float c2 = 0.17364817766693036f, s2 = 0.984807753012208f;     // W_9^2
        constexpr float c4 = -0.9396926207859084f, s4 = 0.3420201433256687f;    // W_9^4
        cf u[3][3];
#pragma unroll
        for (int n2 = 0; n2 < 3; ++n2) {
            cf a = v[n2], b = v[3 + n2], c = v[6 + n2];
            dft3<INV>(a, b, c);
            u[0][n2] = a; u[1][n2] = b; u[2][n2] = c;
        }
        auto tw = [](cf a, cf w) { return INV ? cmulc(a, w) : cmul(a, w); };
        u[1][1] = tw(u[1][1], cf{c1, -s1}); u[1][2] = tw(u[1][2], cf{c2, -s2});
        u[2][1] = tw(u[2][1], cf{c2, -s2}); u[2][2] = tw(u[2][2], cf{c4, -s4});
#pragma unroll
        for (int k1 = 0; k1 < 3; ++k1) {
            dft3<INV>(u[k1][0], u[k1][1], u[k1][2]);
#pragma unroll
            for (int k2 = 0; k2 < 3; ++k2) v[k1 + 3 * k2] = u[k1][k2];
        }
    }
};

typedef unsigned int u32x2 __attribute__((__vector_size__(8)));

// One channel pair of one token.  Rows are addressed through a buffer resource that spans the whole
// sample; a lane whose pair lies past D is given an offset beyond the resource and reads zeros, so
// the loads need no branch.
template <typename T> struct pair_io;
template <> struct pair_io<bf16_t> {
    using raw_t = uint32_t;
    __device__ static __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, uint32_t off, bool second, bool aligned)
    {
        if (aligned) return __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0);
        const uint32_t lo = __builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0);
        const uint32_t hi = second ? (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, off + 2, 0, 0) : 0u;
        return (lo & 0xffffu) | (hi << 16);
    }
    __device__ static __forceinline__ cf widen(raw_t r) { return {__uint_as_float(r << 16), __uint_as_float(r & 0xffff0000u)}; }
};
template <> struct pair_io<float> {
    using raw_t = u32x2;
    __device__ static __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, uint32_t off, bool second, bool aligned)
    {
        if (aligned) return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
        raw_t v;
        v[0] = __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0);
        v[1] = second ? __builtin_amdgcn_raw_buffer_load_b32(r, off + 4, 0, 0) : 0u;
        return v;
    }
    __device__ static __forceinline__ cf widen(raw_t r) { return {__uint_as_float(r[0]), __uint_as_float(r[1])}; }
};

constexpr int kPairs = 16;                       // channel pairs per workgroup
constexpr int kRowPad = 16 * kPairs + kPairs;    // float2 per exchange row: 16 x 16 pairs + one pad group

// largest value over the 16 lanes of a DPP row, in every lane of the row
__device__ __forceinline__ float row16_max(float v)
{
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false)));
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false)));
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false)));
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false)));
    return v;
}

// sum over the 16 lanes of a DPP row; every lane of the row ends up with the total, fixed order
__device__ __forceinline__ float row16_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));   // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));   // row_mirror
    return v;
}

// ---- interpolation kernel of the thinned inverse
// Kaiser window: I0 by its power series in z = x^2 / 4 (all terms positive; 40 terms cover x <= 16 to fp64 accuracy)
constexpr int kI0Terms = 40;
struct I0Coef {
    double c[kI0Terms];
    constexpr I0Coef() : c()
    {
        double f = 1.0;
        for (int k = 0; k < kI0Terms; ++k) {
            if (k) f /= (double)k * (double)k;
            c[k] = f;                            // 1 / (k!)^2
        }
    }
};
__device__ __forceinline__ double bessel_i0(double x)
{
    constexpr I0Coef K{};
    const double z = 0.25 * x * x;
    double s = K.c[kI0Terms - 1];
#pragma unroll
    for (int k = kI0Terms - 2; k >= 0; --k) s = fma(s, z, K.c[k]);
    return s;
}
constexpr double kKaiserAtten = 140.0;                           // dB
constexpr double kKaiserBeta = 0.1102 * (kKaiserAtten - 8.7);    // 14.5
constexpr double kPi = 3.14159265358979323846;
constexpr double kCondition = 1.0 / 8.0;                         // a tile is filled in only if e^[n] >= kCondition * a[n] ...
constexpr double kFloorShare = 1.0 / 32.0;                       // ... and e^[n] >= kFloorShare * (largest coarse energy of the tile), for all n
constexpr int kMaxTaps = 256;                                    // (dec - 1) * 2 H, doubles in LDS

// Half-width (in coarse samples) of the kernel for Ns samples of a polynomial of degree <= 2 sigma: the transition
// band runs from 2 sigma / Ns to 1 - 2 sigma / Ns cycles per coarse sample.  <= 0: Ns is too small.
double interp_half_width(int Ns, int sigma)
{
    const double df = 1.0 - 4.0 * (double)sigma / (double)Ns;
    if (df <= 0.0) return -1.0;
    return 0.5 * ((kKaiserAtten - 8.0) / (2.285 * 2.0 * kPi * df) + 1.0);
}
// taps on each side of a token: ceil(hw), rounded up to a multiple of 4
int interp_taps_half(double hw) { const int h = (int)hw + ((double)(int)hw < hw ? 1 : 0); return (h + 3) / 4 * 4; }

// taps[(s - 1) * 2 H + i] = h(s / dec - (i - H + 1)), s = 1 .. dec - 1, i < 2 H;  h(u) = sinc(u) kaiser(u / hw)
__device__ __forceinline__ void interp_build_taps(double* taps, int dec, int H, double hw)
{
    const int e = threadIdx.x;
    if (e >= (dec - 1) * 2 * H) return;
    const int s = e / (2 * H) + 1, i = e - (s - 1) * 2 * H, m = i - H + 1;
    const double frac = (double)s / (double)dec, u = frac - (double)m, q = u / hw;
    double h = 0.0;
    if (q > -1.0 && q < 1.0) {
        const double sn = (m & 1) ? -sinpi(frac) : sinpi(frac);        // sin(pi u)
        h = sn / (kPi * u) * bessel_i0(kKaiserBeta * sqrt(1.0 - q * q)) / bessel_i0(kKaiserBeta);
    }
    taps[e] = h;
}

}  // namespace

template <typename T, int Q, bool POW2, bool ALIGNED, bool THIN>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((Q == 9 || (Q == 15 && sizeof(T) == 2)) ? 3 : 2)))
spu_fft16q(const T* __restrict__ x, int N, int D, int64_t row_stride, int sigma, int use_hamming,
           int dec_arg /* THIN: the inverse starts with the subsequences n2 = 0, dec, 2 dec, ... */, int taps_h, double taps_hw,
           float* __restrict__ partial /* [B, n_tiles, N] */, float* __restrict__ gpartial /* [B, n_groups, N] */,
           const TileSync sy, float* __restrict__ scores /* [B, N] */)
{
    using pio = pair_io<T>;
    constexpr int N1 = 16 * Q;
    const int dec = THIN ? dec_arg : 1;
    extern __shared__ float2 smem[];
    float2* xbuf = smem;                         // [16][kRowPad]  exchange between the two passes
    float2* tw = smem + 16 * kRowPad;            // [N]    (cos, sin)(2 pi i / N)
    float2* tw1 = tw + N;                        // [N1]   (cos, sin)(2 pi i / N1)
    float* eperm = reinterpret_cast<float*>(tw1 + N1);      // [N2][Q t][16 j] energies of this tile
    float* gm = eperm + N;                       // [sigma + 1]  M[f] / N  (Eq. 5 with the 1/N of Eq. 7)
    double* taps = reinterpret_cast<double*>(smem + 16 * kRowPad + N + N1) + (N + sigma + 1 + 1) / 2;    // [(dec - 1) 2 H]
    __shared__ int is_last, ill;                 // ill: some token of the tile cannot be interpolated
    __shared__ float emax_w[4];                  // largest coarse energy of the tile, per wavefront
    const int tid = threadIdx.x, c = tid & 15, t = tid >> 4;
    // neighbouring channel tiles share 128-byte lines of every token row: keep them on one XCD
    const int n_tiles = gridDim.x;
    const unsigned item = xcd_contiguous(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y);
    const int tile = item % n_tiles, b = item / n_tiles;
    const int N2 = N / N1;

    const int d0 = tile * 32 + 2 * c;
    const bool rdx = Q == 16 || t < Q;           // this thread takes part in the radix-16 side
    const bool live = d0 < D && rdx, second = d0 + 1 < D;
    const uint32_t es = (uint32_t)sizeof(T);
    const uint32_t row_bytes = (uint32_t)row_stride * es;
    // resource over sample b (N rows); lanes without a channel pair point past its end
    const uint64_t span = (uint64_t)(N - 1) * row_bytes + (uint64_t)D * es;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(x) + (int64_t)b * N * row_stride, 0, (int)(span > 0x7fffffffull ? 0x7fffffffull : span), 0x00020000);
    const uint32_t lane_off = live ? (uint32_t)d0 * es : 0x80000000u;

    // this thread's output bins of every N1-point transform: k1 = t + 16 kb (t doubles as ka)
    int kpos[Q], ph[Q];
    cf F[Q];
#pragma unroll
    for (int kb = 0; kb < Q; ++kb) {
        const int k1 = t + 16 * kb;
        kpos[kb] = 8 * (k1 <= sigma ? k1 : N - N1 + k1);  // k mod N (bins outside the band are masked later), as a byte offset into tw
        ph[kb] = 0;                                        // (k * n2) mod N, likewise
        F[kb] = {0.f, 0.f};
    }
    // W_N^{+-k n2} for bin kb of this thread: a power-of-two N takes the product modulo N directly, any other N
    // keeps a running sum.  The thinned inverse visits n2 = dec i2: its exponent k dec i2 mod N is dec times
    // (k i2 mod N / dec), a running sum modulo N / dec of k reduced modulo N / dec (kpos is reduced in place once
    // the forward transform is done).
    const int ph_mod = 8 * N / dec;
    auto tw_k = [&](int kb, int n2, auto inv) {
        int off;
        if (POW2) off = (int)__umul24((unsigned)kpos[kb], (unsigned)n2) & (8 * N - 1);
        else if constexpr (decltype(inv)::value) {
            off = (int)__umul24((unsigned)ph[kb], (unsigned)dec);
            ph[kb] += kpos[kb];
            if (ph[kb] >= ph_mod) ph[kb] -= ph_mod;
        }
        else {
            off = ph[kb];
            ph[kb] += kpos[kb];
            if (ph[kb] >= 8 * N) ph[kb] -= 8 * N;
        }
        return *reinterpret_cast<const float2*>(reinterpret_cast<const char*>(tw) + off);
    };
    // the same for any n2, from scratch (the subsequences the thinned inverse left out, if they are needed after all)
    auto tw_any = [&](int kb, int n2) {
        const int k1 = t + 16 * kb;
        const unsigned k8 = 8u * (unsigned)(k1 <= sigma ? k1 : N - N1 + k1);
        const unsigned off = POW2 ? (__umul24(k8, (unsigned)n2) & (unsigned)(8 * N - 1)) : (k8 * (unsigned)n2) % (unsigned)(8 * N);
        return *reinterpret_cast<const float2*>(reinterpret_cast<const char*>(tw) + off);
    };

    typename pio::raw_t raw[16];
    auto load_sub = [&](int n2) {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            raw[j] = pio::load(rsrc, lane_off + (uint32_t)(N2 * (Q * j + t) + n2) * row_bytes, second, ALIGNED);
    };
    load_sub(0);
    // Tables, built while the first loads are in flight.  One octant of the circle is evaluated in fp64
    // and rounded once; the other seven follow by symmetry (8 divides N).
    {
        const int n8 = N >> 3, n4 = N >> 2, nh = N >> 1, n34 = nh + n4;
        for (int i = tid; i <= n8; i += 256) {
            double sd, cd;
            sincospi(2.0 * (double)i / (double)N, &sd, &cd);
            const float cs = (float)cd, sn = (float)sd;
            tw[i] = make_float2(cs, sn);
            tw[n4 - i] = make_float2(sn, cs);
            tw[n4 + i] = make_float2(-sn, cs);
            tw[nh - i] = make_float2(-cs, sn);
            tw[nh + i] = make_float2(-cs, -sn);
            tw[n34 - i] = make_float2(-sn, -cs);
            tw[n34 + i] = make_float2(sn, -cs);
            if (i) tw[N - i] = make_float2(cs, -sn);
        }
        // the window weights on the upper half of the workgroup: for N <= 1024 the octant above keeps the lower one busy
        if (tid >= 128 && tid - 128 <= sigma) {
            const int f = tid - 128;
            double w = 1.0;
            if (use_hamming) w = 0.54 + 0.46 * cospi(2.0 * (double)f / (double)(N - 1));
            gm[f] = (float)(w / (double)N);
        }
        if (THIN) interp_build_taps(taps, dec, taps_h, taps_hw);
        if (tid == 0) ill = 0;
    }
    __syncthreads();
    // W_N1^{t i}, i < 16: the twiddles between the two passes of every N1-point transform, both directions
    constexpr bool kHoist = Q == 16;
    cf w1[16];
    if (kHoist) {
        int e1 = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float2 w = tw[e1 * N2];
            w1[i] = {w.x, w.y};
            e1 += t;
            if (e1 >= N1) e1 -= N1;
        }
    }
    else {
        if (tid < N1) tw1[tid] = tw[tid * N2];
        __syncthreads();
    }
    // without the register copy: walk the N1 table, i = 0, 1, 2, ... in order (o1 = t i mod N1)
    int o1 = 0;
    auto tw1_next = [&](int i) {
        if (kHoist) return w1[i];
        const float2 w = tw1[o1];
        o1 += t;
        if (o1 >= N1) o1 -= N1;
        return cf{w.x, w.y};
    };

    // ------------------------------------------------------------------ forward (Eq. 4 on the pass band)
    // The subsequence n2 = 0 carries the twiddle W_N^0 = 1: its pass is a copy of the loop body without the
    // pass-band multiplications (the same holds for the inverse below).
    auto forward = [&](int n2, auto first) {
        cf v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = pio::widen(raw[j]);
        if (n2 + 1 < N2) load_sub(n2 + 1);       // next subsequence in flight while this one is transformed
        if (rdx) {
            fft16<false>(v);                     // over j -> ka
            o1 = 0;
#pragma unroll
            for (int ka = 0; ka < 16; ++ka) {
                const cf r = cmulc(v[ka], tw1_next(ka));         // * W_N1^{t ka}
                xbuf[ka * kRowPad + t * kPairs + c] = make_float2(r.x, r.y);
            }
        }
        __syncthreads();
        cf u[Q];
#pragma unroll
        for (int s = 0; s < Q; ++s) { const float2 q = xbuf[t * kRowPad + s * kPairs + c]; u[s] = {q.x, q.y}; }
        __syncthreads();
        dftq<Q, false>::run(u);                  // over the residue -> kb ; u[kb] = Y[t + 16 kb]
#pragma unroll
        for (int kb = 0; kb < Q; ++kb) {
            if constexpr (decltype(first)::value) {
                F[kb] = u[kb];
                ph[kb] = kpos[kb];               // (k * 1) mod N for the next subsequence
            }
            else {
                const float2 w = tw_k(kb, n2, std::false_type{});
                F[kb] = F[kb] + cmulc(u[kb], cf{w.x, w.y});    // * W_N^{k n2}
            }
        }
    };
    forward(0, std::true_type{});
    for (int n2 = 1; n2 < N2; ++n2) forward(n2, std::false_type{});
    const tile_tag_t seen = tiles_look<4>(sy, b, tile, n_tiles);     // no loads follow: nothing waits behind this one
    // ------------------------------------------------------------------ mask (Eq. 5-6) with the 1/N of Eq. 7
#pragma unroll
    for (int kb = 0; kb < Q; ++kb) {
        const int k1 = t + 16 * kb;
        const bool lo = k1 <= sigma, hi = k1 >= N1 - sigma;
        const float g = (lo || hi) ? gm[lo ? k1 : N1 - k1] : 0.f;
        F[kb] = {F[kb].x * g, F[kb].y * g};
        ph[kb] = 0;
        if (THIN && !POW2)
            while (kpos[kb] >= ph_mod) kpos[kb] -= ph_mod;         // at most dec - 1 rounds
    }
    // ------------------------------------------------------------------ inverse (Eq. 7) and energy (Eq. 8)
    // (`rest`: one of the subsequences the thinned pass left out - its twiddles are worked out from scratch)
    auto inverse = [&](int n2, auto first, bool rest) {
        cf u[Q];
        if constexpr (decltype(first)::value) {
#pragma unroll
            for (int kb = 0; kb < Q; ++kb) {
                u[kb] = F[kb];
                ph[kb] = kpos[kb];               // phase of the next subsequence of the thinned pass
            }
        }
        else if (rest) {
#pragma unroll
            for (int kb = 0; kb < Q; ++kb) {
                const float2 w = tw_any(kb, n2);
                u[kb] = cmul(F[kb], cf{w.x, w.y});
            }
        }
        else {
#pragma unroll
            for (int kb = 0; kb < Q; ++kb) {
                const float2 w = tw_k(kb, n2, std::true_type{});
                u[kb] = cmul(F[kb], cf{w.x, w.y});   // F[k] W_N^{-k n2}
            }
        }
        dftq<Q, true>::run(u);                   // over kb -> residue s
        o1 = 0;
#pragma unroll
        for (int s = 0; s < Q; ++s) {
            const cf r = cmul(u[s], tw1_next(s));               // * W_N1^{-s ka}
            xbuf[s * kRowPad + t * kPairs + c] = make_float2(r.x, r.y);
        }
        __syncthreads();
        if (rdx) {
            cf v[16];
#pragma unroll
            for (int ka = 0; ka < 16; ++ka) { const float2 q = xbuf[t * kRowPad + ka * kPairs + c]; v[ka] = {q.x, q.y}; }
            fft16<true>(v);                      // over ka -> j ; v[j] = z'[N2 (Q j + t) + n2]
            float e[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) e[j] = row16_sum(fmaf(v[j].x, v[j].x, v[j].y * v[j].y));   // over the 16 pairs
            if (c == 0) {
                float4* dst = reinterpret_cast<float4*>(eperm + (n2 * Q + t) * 16);
#pragma unroll
                for (int q = 0; q < 4; ++q) dst[q] = make_float4(e[4 * q], e[4 * q + 1], e[4 * q + 2], e[4 * q + 3]);
            }
        }
        __syncthreads();
    };
    // ------------------------------------------------------------------ thinned inverse: fill in, check
    // (the exchange buffer is free between two subsequences: it holds the coarse energies in token order, with
    // the taps_h - 1 before and the taps_h + 1 after them repeated at either end, and all N energies once filled in)
    const int N2c = N2 / dec, Ns = N / dec;
    float* ec = reinterpret_cast<float*>(xbuf);                   // [Ns + 2 taps_h + 2]: ec[i] = e[dec ((i - taps_h + 1) mod Ns)]
    float* efull = ec + Ns + 2 * taps_h + 2;                      // [N]
    auto fill_in = [&]() {
        const int H = taps_h;
        float big = 0.f;
        for (int i = tid; i < Ns + 2 * H + 2; i += 256) {
            int m = i - H + 1;                   // 2 H <= Ns: one wrap at most
            m = m < 0 ? m + Ns : (m >= Ns ? m - Ns : m);
            const int i2 = POW2 ? (m & (N2c - 1)) : m % N2c, q = (m - i2) / N2c;       // token dec m = N2 q + dec i2
            const int tq = Q == 16 ? (q & 15) : q % Q, j = Q == 16 ? (q >> 4) : q / Q;
            const float v = eperm[(i2 * dec * Q + tq) * 16 + j];
            ec[i] = v;
            big = fmaxf(big, v);
        }
        auto rl = [](float v, int l) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l)); };
        big = row16_max(big);
        big = fmaxf(fmaxf(rl(big, 0), rl(big, 16)),
                    fmaxf(rl(big, 32), rl(big, 48)));
        if ((tid & 63) == 0) emax_w[tid >> 6] = big;
        __syncthreads();
        const double emax_share = kFloorShare * (double)fmaxf(fmaxf(emax_w[0], emax_w[1]), fmaxf(emax_w[2], emax_w[3]));
        // The tap of phase s at index i (coarse token p - H + 1 + i) is h(s / dec - (i - H + 1)) with h even, so the
        // taps of phase dec - s are those of phase s in reverse; and h takes the sign of sinc: with H even, a tap is
        // positive at odd i in the lower half of the window and at even i in the upper half, negative (or zero)
        // elsewhere.  A pair (k, 2 H - 1 - k) therefore has one sign - negative for even k, positive for odd k - and
        // the sums over even and over odd k are the negative and the positive part of e^[n]: their difference is a[n].
        // A thread takes two neighbouring coarse tokens A = pp, B = pp + 1, whose windows differ by one entry: the
        // loop is bound by what it reads from LDS: the energies stay fp32 there and are widened in registers (kept as
        // doubles in LDS, the same loop was measured 5 % of the kernel slower); taps are broadcast reads.
        bool bad = false;
        auto emit = [&](float* dst, double pos, double neg) {
            const double v = pos + neg;
            bad |= v < kCondition * (pos - neg) || v < emax_share;
            *dst = (float)v;
        };
        for (int pp = 2 * tid; pp < Ns; pp += 512) {
            const float* w = ec + pp;            // w[i]: e at coarse token pp - H + 1 + i; A reads w[i], B reads w[i + 1]
            float* out = efull + dec * pp;
            out[0] = w[H - 1];
            out[dec] = w[H];
            for (int s = 1; 2 * s <= dec; ++s) {
                const double* tp = taps + (s - 1) * 2 * H;
                if (2 * s == dec) {              // its own mirror image: the window folds
                    double nA = 0.0, pA = 0.0, nB = 0.0, pB = 0.0;
#pragma unroll 2
                    for (int k = 0; k < H; k += 2) {
                        const double t0 = tp[k], t1 = tp[k + 1];
                        const double a0 = (double)w[k], a1 = (double)w[k + 1], a2 = (double)w[k + 2];
                        const double b0 = (double)w[2 * H - k], b1 = (double)w[2 * H - 1 - k], b2 = (double)w[2 * H - 2 - k];
                        nA = fma(t0, a0 + b1, nA);
                        pA = fma(t1, a1 + b2, pA);
                        nB = fma(t0, a1 + b0, nB);
                        pB = fma(t1, a2 + b1, pB);
                    }
                    emit(out + s, pA, nA);
                    emit(out + dec + s, pB, nB);
                }
                else {                           // phases s and dec - s share the taps
                    double nAs = 0.0, pAs = 0.0, nAd = 0.0, pAd = 0.0, nBs = 0.0, pBs = 0.0, nBd = 0.0, pBd = 0.0;
#pragma unroll 2
                    for (int k = 0; k < H; k += 2) {
                        const double t0 = tp[k], u0 = tp[2 * H - 1 - k], t1 = tp[k + 1], u1 = tp[2 * H - 2 - k];
                        const double a0 = (double)w[k], a1 = (double)w[k + 1], a2 = (double)w[k + 2];
                        const double b0 = (double)w[2 * H - k], b1 = (double)w[2 * H - 1 - k], b2 = (double)w[2 * H - 2 - k];
                        nAs = fma(t0, a0, fma(u0, b1, nAs));
                        nAd = fma(t0, b1, fma(u0, a0, nAd));
                        pAs = fma(t1, a1, fma(u1, b2, pAs));
                        pAd = fma(t1, b2, fma(u1, a1, pAd));
                        nBs = fma(t0, a1, fma(u0, b0, nBs));
                        nBd = fma(t0, b0, fma(u0, a1, nBd));
                        pBs = fma(t1, a2, fma(u1, b1, pBs));
                        pBd = fma(t1, b1, fma(u1, a2, pBd));
                    }
                    emit(out + s, pAs, nAs);
                    emit(out + dec - s, pAd, nAd);
                    emit(out + dec + s, pBs, nBs);
                    emit(out + 2 * dec - s, pBd, nBd);
                }
            }
        }
        if (bad) ill = 1;
        __syncthreads();
    };
    inverse(0, std::true_type{}, false);
    tiles_claim<4>(sy, b, tile, n_tiles, seen);
    bool thin = THIN;                            // the energies are known at the tokens n = dec m only
    for (int it = 1; it < N2; ++it) {
        if (THIN && it == N2c) {                 // the thinned pass is complete
            fill_in();
            if (!ill) break;
            thin = false;                        // some token cannot be trusted: the remaining subsequences after all
        }
        const bool rest = THIN && it >= N2c;
        int n2 = it * dec;
        if (rest) { const int r = it - N2c; n2 = r + r / (dec - 1) + 1; }       // the r-th n2 that dec does not divide
        inverse(n2, std::false_type{}, rest);
    }
    float* pout = partial + ((int64_t)b * n_tiles + tile) * N;
    if (THIN && thin) {
        for (int n = tid; n < N; n += 256) tile_store(pout + n, efull[n]);
    }
    else {
        for (int n = tid; n < N; n += 256) {     // n = N2 (Q j + t') + n2
            const int n2 = POW2 ? (n & (N2 - 1)) : n % N2;
            const int q = (n - n2) / N2;
            const int tq = Q == 16 ? (q & 15) : q % Q, j = Q == 16 ? (q >> 4) : q / Q;
            tile_store(pout + n, eperm[(n2 * Q + tq) * 16 + j]);
        }
    }
    // ------------------------------------------------------------------ Eq. 8 across the channel tiles
    tiles_to_scores<256, 4>(partial, gpartial, sy, scores, b, tile, n_tiles, N, &is_last);
}

static size_t fft_lds_bytes(int N, int Q, int sigma, int n_taps)
{
    return sizeof(float2) * (size_t)(16 * kRowPad + N + 16 * Q) + sizeof(float) * (size_t)((N + sigma + 1 + 1) / 2 * 2) + sizeof(double) * (size_t)n_taps;
}

// the residue-side length Q of the 16 x Q transform that serves (N, sigma); 0 if none does
static int fft_pick_q(int N, int sigma)
{
    if (N > 4096) return 0;
    for (int Q : {16, 15, 9}) {
        const int N1 = 16 * Q;
        if (N % N1 == 0 && 2 * sigma + 1 <= N1) return Q;
    }
    return 0;
}

bool spu_fft_supported(int N, int sigma) { return fft_pick_q(N, sigma) != 0; }

// How far the inverse is thinned out: the divisor dec of N2 that saves the most, counting a subsequence of the
// inverse at its ~630 vector instructions per wavefront and a tap of the fill-in at 6 (two LDS reads, four fp64
// operations) per coarse token and phase; 1 if nothing saves a fifth of the inverse or fits.
struct ThinPlan { int dec, taps_h; double taps_hw; };
static ThinPlan fft_thin_plan(int N, int Q, int sigma)
{
    ThinPlan best{1, 0, 0.0};
    const int N2 = N / (16 * Q);
    double best_gain = 0.2 * 630.0 * N2;
    for (int dec = 2; dec <= N2; ++dec) {
        if (N2 % dec) continue;
        const int Ns = N / dec;
        const double hw = interp_half_width(Ns, sigma);
        if (hw <= 0.0) continue;
        const int H = interp_taps_half(hw);
        if (2 * H > Ns || (dec - 1) * 2 * H > kMaxTaps) continue;
        if (sizeof(float) * (size_t)(Ns + 2 * H + 2 + N) > sizeof(float2) * (size_t)(16 * kRowPad)) continue;
        const double gain = 630.0 * (N2 - N2 / dec) - 6.0 * (dec - 1) * 2 * H * ((Ns + 255) / 256);
        if (gain > best_gain) { best_gain = gain; best = ThinPlan{dec, H, hw}; }
    }
    return best;
}

luvc_status spu_score_fft(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dt, int sigma, int use_hamming,
                          float* partial, float* gpartial, const TileSync& sy, int n_tiles, float* scores, hipStream_t st)
{
    const int Q = fft_pick_q(N, sigma);
    const ThinPlan tp = fft_thin_plan(N, Q, sigma);
    const int dec = tp.dec, taps_h = tp.taps_h;
    const double taps_hw = tp.taps_hw;
    const size_t lds = fft_lds_bytes(N, Q, sigma, (dec - 1) * 2 * taps_h);
    const bool pow2 = (N & (N - 1)) == 0;
    // channel pairs are fetched with one access when every pair is naturally aligned
    const size_t es = dt == LUVC_F32 ? 4 : 2;
    const bool aligned = (row_stride % 2 == 0) && ((uintptr_t)x % (2 * es) == 0) && (D % 2 == 0);
    if (n_tiles > 65535) { set_error("D=%d exceeds the supported width of the fft path", D); return LUVC_ERR_UNSUPPORTED; }
    const dim3 grid((unsigned)n_tiles, (unsigned)B);
#define LUVC_FFT_H(TT, QQ, P2, AL, TH) LUVC_LAUNCH("spu_fft16q", (spu_fft16q<TT, QQ, P2, AL, TH>), grid, dim3(256), lds, st, (const TT*)x, N, D, row_stride, sigma, use_hamming, dec, taps_h, taps_hw, partial, gpartial, sy, scores)
#define LUVC_FFT(TT, QQ, P2, AL) do { if (dec > 1) LUVC_FFT_H(TT, QQ, P2, AL, true); else LUVC_FFT_H(TT, QQ, P2, AL, false); } while (0)
#define LUVC_FFT_A(TT, QQ, P2) do { if (aligned) LUVC_FFT(TT, QQ, P2, true); else LUVC_FFT(TT, QQ, P2, false); } while (0)
#define LUVC_FFT_T(TT) do { if (Q == 16) { if (pow2) LUVC_FFT_A(TT, 16, true); else LUVC_FFT_A(TT, 16, false); } \
                            else if (Q == 15) LUVC_FFT_A(TT, 15, false); else LUVC_FFT_A(TT, 9, false); } while (0)
    if (dt == LUVC_F32) LUVC_FFT_T(float); else LUVC_FFT_T(bf16_t);
#undef LUVC_FFT_T
#undef LUVC_FFT_A
#undef LUVC_FFT
#undef LUVC_FFT_H
    return check_launch("spu score (fft)");
}

}  // namespace luvc
