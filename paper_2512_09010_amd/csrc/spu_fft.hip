// SPU score (paper Section 3.3, Eq. 4-8): fast path for N = 256 * N2, 2*sigma + 1 <= 256.
//
// Two real channels (d, d+1) are packed as one complex signal z = x_d + i x_{d+1}.  The mask of
// Eq. 5 is real and symmetric in k, so the filter is a real linear operator and Re / Im of the
// filtered z are the two filtered channels: no unpacking is ever needed.
//
// Transform decomposition along the token index, n = N2 * n1 + n2 (n1 < 256, n2 < N2):
//   Eq. 4 on the pass band:  F[k] = sum_{n2} W_N^{k n2} Y_{n2}[k mod 256],  |k| <= sigma,
//                            Y_{n2} = 256-point DFT of the stride-N2 subsequence n2;
//   Eq. 6:                   F[k] *= M[|k|] / N;
//   Eq. 7:                   z'[N2 n1 + n2] = 256-point inverse DFT over k1 of F[k] W_N^{-k n2};
//   Eq. 8:                   |z'|^2 summed over the channel pairs of the tile.
// Each 256-point transform is 16 x 16: a radix-16 butterfly held in registers, one exchange through
// LDS, a second radix-16.  A workgroup owns 16 channel pairs (32 channels, 64-byte row segments for
// bf16); thread (c, t) = (pair, residue).  The pass-band accumulators F stay in registers across the
// N2 subsequences, so x is read exactly once and nothing but N floats per tile is written.
#include "common.hpp"
#include "spu.hpp"

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

// sum over the 16 lanes of a DPP row; every lane of the row ends up with the total, fixed order
__device__ __forceinline__ float row16_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));   // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));   // row_mirror
    return v;
}

}  // namespace

template <typename T, bool POW2, bool ALIGNED>
__global__ void __launch_bounds__(256)
spu_fft256(const T* __restrict__ x, int N, int D, int64_t row_stride, int sigma,
           const float2* __restrict__ tw_g, const float* __restrict__ gm /* M[f]/N */,
           float* __restrict__ partial /* [B, n_tiles, N] */)
{
    using pio = pair_io<T>;
    extern __shared__ float2 smem[];
    float2* xbuf = smem;                         // [16][kRowPad]  exchange between the two radix-16 passes
    float2* tw = smem + 16 * kRowPad;            // [N]    (cos, sin)(2 pi i / N)
    float2* tw256 = tw + N;                      // [256]  (cos, sin)(2 pi i / 256)
    float* eperm = reinterpret_cast<float*>(tw256 + 256);   // [N2][16 t][16 j] energies of this tile
    const int tid = threadIdx.x, c = tid & 15, t = tid >> 4;
    // neighbouring channel tiles share 128-byte lines of every token row: keep them on one XCD
    const int n_tiles = gridDim.x;
    const unsigned item = xcd_contiguous(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y);
    const int tile = item % n_tiles, b = item / n_tiles;
    const int N2 = N >> 8;
    for (int i = tid; i < N; i += 256) tw[i] = tw_g[i];
    tw256[tid] = tw_g[tid * N2];

    const int d0 = tile * 32 + 2 * c;
    const bool live = d0 < D, second = d0 + 1 < D;
    const uint32_t es = (uint32_t)sizeof(T);
    const uint32_t row_bytes = (uint32_t)row_stride * es;
    // resource over sample b (N rows); lanes without a channel pair point past its end
    const uint64_t span = (uint64_t)(N - 1) * row_bytes + (uint64_t)D * es;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(x) + (int64_t)b * N * row_stride, 0, (int)(span > 0x7fffffffull ? 0x7fffffffull : span), 0x00020000);
    const uint32_t lane_off = live ? (uint32_t)d0 * es : 0x80000000u;

    // this thread's output bins of every 256-point transform: k1 = t + 16 kb (t doubles as ka)
    int kpos[16], ph[16];
    cf F[16];
#pragma unroll
    for (int kb = 0; kb < 16; ++kb) {
        const int k1 = t + 16 * kb;
        kpos[kb] = k1 <= sigma ? k1 : N - 256 + k1;       // k mod N (bins outside the band are masked later)
        ph[kb] = 0;                                        // (k * n2) mod N
        F[kb] = {0.f, 0.f};
    }
    auto advance = [&](int kb) {
        ph[kb] += kpos[kb];
        if (POW2) ph[kb] &= N - 1;
        else if (ph[kb] >= N) ph[kb] -= N;
    };

    typename pio::raw_t raw[16];
    auto load_sub = [&](int n2) {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            raw[j] = pio::load(rsrc, lane_off + (uint32_t)(N2 * (16 * j + t) + n2) * row_bytes, second, ALIGNED);
    };
    load_sub(0);
    __syncthreads();                             // twiddle tables ready

    // ------------------------------------------------------------------ forward (Eq. 4 on the pass band)
    for (int n2 = 0; n2 < N2; ++n2) {
        cf v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = pio::widen(raw[j]);
        if (n2 + 1 < N2) load_sub(n2 + 1);       // next subsequence in flight while this one is transformed
        fft16<false>(v);                         // over j -> ka
        int e256 = 0;
#pragma unroll
        for (int ka = 0; ka < 16; ++ka) {
            const float2 w = tw256[e256];
            e256 = (e256 + t) & 255;
            const cf r = cmulc(v[ka], cf{w.x, w.y});       // * W_256^{t ka}
            xbuf[ka * kRowPad + t * kPairs + c] = make_float2(r.x, r.y);
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 16; ++s) { const float2 q = xbuf[t * kRowPad + s * kPairs + c]; v[s] = {q.x, q.y}; }
        __syncthreads();
        fft16<false>(v);                         // over the residue -> kb ; v[kb] = Y[t + 16 kb]
#pragma unroll
        for (int kb = 0; kb < 16; ++kb) {
            const float2 w = tw[ph[kb]];
            F[kb] = F[kb] + cmulc(v[kb], cf{w.x, w.y});    // * W_N^{k n2}
            advance(kb);
        }
    }
    // ------------------------------------------------------------------ mask (Eq. 5-6) with the 1/N of Eq. 7
#pragma unroll
    for (int kb = 0; kb < 16; ++kb) {
        const int k1 = t + 16 * kb;
        const bool lo = k1 <= sigma, hi = k1 >= 256 - sigma;
        const float g = (lo || hi) ? gm[lo ? k1 : 256 - k1] : 0.f;
        F[kb] = {F[kb].x * g, F[kb].y * g};
        ph[kb] = 0;
    }
    // ------------------------------------------------------------------ inverse (Eq. 7) and energy (Eq. 8)
    for (int n2 = 0; n2 < N2; ++n2) {
        cf v[16];
#pragma unroll
        for (int kb = 0; kb < 16; ++kb) {
            const float2 w = tw[ph[kb]];
            v[kb] = cmul(F[kb], cf{w.x, w.y});   // F[k] W_N^{-k n2}
            advance(kb);
        }
        fft16<true>(v);                          // over kb -> residue s
        int e256 = 0;
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const float2 w = tw256[e256];
            e256 = (e256 + t) & 255;
            const cf r = cmul(v[s], cf{w.x, w.y});
            xbuf[s * kRowPad + t * kPairs + c] = make_float2(r.x, r.y);
        }
        __syncthreads();
#pragma unroll
        for (int ka = 0; ka < 16; ++ka) { const float2 q = xbuf[t * kRowPad + ka * kPairs + c]; v[ka] = {q.x, q.y}; }
        __syncthreads();
        fft16<true>(v);                          // over ka -> j ; v[j] = z'[N2 (16 j + t) + n2]
        float e[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) e[j] = row16_sum(fmaf(v[j].x, v[j].x, v[j].y * v[j].y));   // over the 16 pairs
        if (c == 0) {
            float4* dst = reinterpret_cast<float4*>(eperm + (n2 * 16 + t) * 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) dst[q] = make_float4(e[4 * q], e[4 * q + 1], e[4 * q + 2], e[4 * q + 3]);
        }
    }
    __syncthreads();
    float* pout = partial + ((int64_t)b * n_tiles + tile) * N;
    for (int n = tid; n < N; n += 256) {         // n = N2 (16 j + t') + n2
        const int n2 = POW2 ? (n & (N2 - 1)) : n % N2;
        const int q = (n - n2) / N2;
        pout[n] = eperm[(n2 * 16 + (q & 15)) * 16 + (q >> 4)];
    }
}

static size_t fft_lds_bytes(int N) { return sizeof(float2) * (size_t)(16 * kRowPad + N + 256) + sizeof(float) * (size_t)N; }

bool spu_fft_supported(int N, int sigma)
{
    return N >= 256 && N % 256 == 0 && N <= 4096 && 2 * sigma + 1 <= 256;
}

luvc_status spu_score_fft(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dt, int sigma,
                          const float2* tw, const float* gm, float* partial, int n_tiles, hipStream_t st)
{
    const dim3 grid((unsigned)n_tiles, (unsigned)B);
    const size_t lds = fft_lds_bytes(N);
    const bool pow2 = (N & (N - 1)) == 0;
    // channel pairs are fetched with one access when every pair is naturally aligned
    const size_t pair_bytes = dt == LUVC_F32 ? 8 : 4;
    const bool aligned = (row_stride % 2 == 0) && ((uintptr_t)x % pair_bytes == 0) && (D % 2 == 0);
#define LUVC_FFT(TT, P2, AL) LUVC_LAUNCH("spu_fft256", (spu_fft256<TT, P2, AL>), grid, dim3(256), lds, st, (const TT*)x, N, D, row_stride, sigma, tw, gm, partial)
#define LUVC_FFT_T(TT) do { if (pow2) { if (aligned) LUVC_FFT(TT, true, true); else LUVC_FFT(TT, true, false); } \
                            else { if (aligned) LUVC_FFT(TT, false, true); else LUVC_FFT(TT, false, false); } } while (0)
    if (dt == LUVC_F32) LUVC_FFT_T(float); else LUVC_FFT_T(bf16_t);
#undef LUVC_FFT_T
#undef LUVC_FFT
    return check_launch("spu score (fft)");
}

}  // namespace luvc
