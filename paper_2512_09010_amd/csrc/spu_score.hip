// SPU score (paper Section 3.3, Eq. 4-8): direct pass-band DFT path, valid for any N.
//
// The mask of Eq. 5 is real and symmetric in k, so for a real signal x[n] the filtered signal is
//     x'[n] = sum_{k=0..sigma} g_k ( C_k cos(2 pi k n / N) + S_k sin(2 pi k n / N) ),
//     C_k = sum_n x[n] cos(2 pi k n / N),  S_k = sum_n x[n] sin(2 pi k n / N),
//     g_0 = M[0]/N,  g_k = 2 M[k]/N  (g_k = M[k]/N when 2k = N, the self-mirrored bin),
// i.e. Eq. 4 evaluated on the pass-band bins only (all other bins are multiplied by zero in Eq. 6)
// and Eq. 7 with the +k / -k terms paired.  Lanes of a wavefront are channels, so twiddles are
// wave-uniform and come through the scalar path; token rows are read coalesced.
//
//   spu_tables      twiddles (fp64 sincospi rounded to fp32) and the weights g_k
//   spu_fwd_dense   C_k, S_k for a tile of 64 channels and a group of bins
//   spu_inv_dense   x'[n] for a tile of 64 channels and a chunk of tokens, squared and summed over the tile
//   spu_finish      fixed-order sum over channel tiles, square root (Eq. 8)
//   spu_dense_fused all of the above in one launch, for samples whose tables and pass-band spectrum of a
//                   64-channel tile fit in LDS (small N and sigma, where the launches themselves dominate)
#include <atomic>
#include <chrono>
#include <cstdlib>
#include <random>
#include <type_traits>

#include "common.hpp"
#include "spu.hpp"
#include "spu_tiles.hpp"

namespace luvc {

__global__ void __launch_bounds__(256)
spu_tables(int N, int sigma, int use_hamming, float2* __restrict__ tw, float* __restrict__ gk, float* __restrict__ gm)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) {
        double s, c;
        sincospi(2.0 * (double)i / (double)N, &s, &c);
        tw[i] = make_float2((float)c, (float)s);
    }
    if (i <= sigma) {
        double w = 1.0;
        if (use_hamming && N > 1) w = 0.54 + 0.46 * cospi(2.0 * (double)i / (double)(N - 1));
        const double pair = (i == 0 || 2 * i == N) ? 1.0 : 2.0;
        gk[i] = (float)(pair * w / (double)N);     // +k and -k paired (real-signal form)
        gm[i] = (float)(w / (double)N);            // per bin (complex form)
    }
}

constexpr int kKPW = 8;    // bins per wavefront in the forward kernel
constexpr int kNB = 8;     // tokens per register block in the inverse kernel
constexpr int kNChunk = 128;  // tokens per workgroup in the inverse kernel (4 waves x 4 blocks x kNB)

template <typename T>
__global__ void __launch_bounds__(256)
spu_fwd_dense(const T* __restrict__ x, int N, int D, int64_t row_stride, int sigma,
              const float2* __restrict__ tw, float* __restrict__ Fc, float* __restrict__ Fs)
{
    using tr = io_traits<T>;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int d = blockIdx.x * 64 + lane;
    const int b = blockIdx.z;
    const int k0 = (blockIdx.y * 4 + wave) * kKPW;
    if (k0 > sigma) return;
    const bool live = d < D;
    const T* xb = x + (int64_t)b * N * row_stride + (live ? d : 0);
    float ac[kKPW], as[kKPW];
    int idx[kKPW], kstep[kKPW];
#pragma unroll
    for (int j = 0; j < kKPW; ++j) { ac[j] = 0.f; as[j] = 0.f; idx[j] = 0; kstep[j] = (k0 + j <= sigma) ? k0 + j : 0; }
    for (int n = 0; n < N; ++n) {
        const float xv = live ? tr::load(xb + (int64_t)n * row_stride) : 0.f;
#pragma unroll
        for (int j = 0; j < kKPW; ++j) {
            const float2 t = tw[idx[j]];
            ac[j] = fmaf(xv, t.x, ac[j]);
            as[j] = fmaf(xv, t.y, as[j]);
            idx[j] += kstep[j];                    // (k * n) mod N, kept incrementally (k <= sigma < N)
            if (idx[j] >= N) idx[j] -= N;
        }
    }
    if (!live) return;
#pragma unroll
    for (int j = 0; j < kKPW; ++j) {
        const int k = k0 + j;
        if (k <= sigma) {
            Fc[((int64_t)b * (sigma + 1) + k) * D + d] = ac[j];
            Fs[((int64_t)b * (sigma + 1) + k) * D + d] = as[j];
        }
    }
}

__global__ void __launch_bounds__(256)
spu_inv_dense(const float* __restrict__ Fc, const float* __restrict__ Fs, int N, int D, int sigma,
              const float2* __restrict__ tw, const float* __restrict__ gk,
              float* __restrict__ partial /* [B, n_tiles, N] */)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tile = blockIdx.x, n_tiles = gridDim.x;
    const int d = tile * 64 + lane;
    const int b = blockIdx.z;
    const bool live = d < D;
    const float* fc = Fc + (int64_t)b * (sigma + 1) * D + (live ? d : 0);
    const float* fs = Fs + (int64_t)b * (sigma + 1) * D + (live ? d : 0);
    for (int blk = 0; blk < kNChunk / (4 * kNB); ++blk) {
        const int n0 = blockIdx.y * kNChunk + (blk * 4 + wave) * kNB;
        if (n0 >= N) break;
        float acc[kNB];
        int idx[kNB], stepn[kNB];
#pragma unroll
        for (int j = 0; j < kNB; ++j) { acc[j] = 0.f; idx[j] = 0; stepn[j] = (n0 + j) % N; }
        for (int k = 0; k <= sigma; ++k) {
            const float g = gk[k];
            const float c = live ? g * fc[(int64_t)k * D] : 0.f;
            const float s = live ? g * fs[(int64_t)k * D] : 0.f;
#pragma unroll
            for (int j = 0; j < kNB; ++j) {
                const float2 t = tw[idx[j]];
                acc[j] = fmaf(c, t.x, acc[j]);
                acc[j] = fmaf(s, t.y, acc[j]);
                idx[j] += stepn[j];                // (k * n) mod N
                if (idx[j] >= N) idx[j] -= N;
            }
        }
#pragma unroll
        for (int j = 0; j < kNB; ++j) {
            const float e = wave_sum(acc[j] * acc[j]);
            if (lane == 0 && n0 + j < N) partial[((int64_t)b * n_tiles + tile) * N + n0 + j] = e;
        }
    }
}

// Eq. 8: fixed-order sum of the per-tile energies, then the square root.  A workgroup owns 64
// consecutive tokens; its 8 waves split the channel tiles, partial sums meet in LDS in wave order.
constexpr int kFinParts = 8;
__global__ void __launch_bounds__(64 * kFinParts)
spu_finish(const float* __restrict__ partial, int N, int n_tiles, int64_t total, float* __restrict__ scores)
{
    __shared__ double part_sum[kFinParts][64];
    const int lane = threadIdx.x & 63, part = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + lane;
    double e = 0.0;
    if (i < total) {
        const int64_t b = i / N;
        const int n = (int)(i - b * N);
        for (int t = part; t < n_tiles; t += kFinParts) e += (double)partial[(b * n_tiles + t) * N + n];
    }
    part_sum[part][lane] = e;
    __syncthreads();
    if (part == 0 && i < total) {
        double tot = 0.0;
#pragma unroll
        for (int p = 0; p < kFinParts; ++p) tot += part_sum[p][lane];
        scores[i] = (float)sqrt(tot);
    }
}

// ------------------------------------------------------------------ one launch for small samples
// Workgroup (tile, b): 64 channels (lanes) x 16 wavefronts.  Tokens are taken in mirrored pairs (p, N - p), which
// share their cosines and have opposite sines (half the products both ways, half the table).  The twiddles of every
// (pair, bin) sit in an LDS table T[p][k] = (cos, sin)(2 pi k p / N), p <= N/2, k < KP (the pass band padded to a
// multiple of kDfBins), so that a pair's kDfBins twiddles are three 16-byte reads and no index arithmetic is left
// in the loops.  Forward: the wavefronts split the pairs (p = wave, wave + 16, ...), each accumulates kDfBins bins
// at a time, the 16 partial sums of a bin meet in LDS (wavefront w + 8 folded into w, then wavefront order) as
// F = g_k (C_k, S_k).  Inverse: the wavefronts split the pairs again, kDfTok pairs per register block; energies
// summed over the lanes; tiles summed by the hand-over of spu_tiles.hpp.
constexpr int kDfWaves = 16, kDfBins = 6, kDfTok = 4, kDfChunk = 16;

static int dense_fused_kp(int sigma) { return (sigma + 1 + kDfBins - 1) / kDfBins * kDfBins; }

static size_t dense_fused_lds(int N, int sigma)
{
    const size_t kp = (size_t)dense_fused_kp(sigma);
    const size_t red = sizeof(float) * (size_t)(kDfWaves / 2) * kDfBins * 128;     // also holds the N-entry table while T is built
    return sizeof(float2) * (size_t)(N / 2 + 1) * kp + sizeof(float) * (kp * 128 + kp) + (red > sizeof(float2) * (size_t)N ? red : sizeof(float2) * (size_t)N);
}

// LDS a workgroup of the one-launch kernel may take (of the 160 KB of a compute unit; above 64 KB one workgroup
// per compute unit is resident)
static size_t dense_fused_cap() { return (size_t)144 * 1024; }

template <typename T>
__global__ void __launch_bounds__(64 * kDfWaves)
spu_dense_fused(const T* __restrict__ x, int N, int D, int64_t row_stride, int sigma, int use_hamming,
                float* __restrict__ partial, float* __restrict__ gpartial, const TileSync sy,
                float* __restrict__ scores)
{
    using tr = io_traits<T>;
    extern __shared__ __align__(16) float2 dsm[];
    const int KP = (sigma + 1 + kDfBins - 1) / kDfBins * kDfBins;
    const int P = N / 2 + 1;                                        // token pairs (p, N - p); p = 0 and p = N/2 stand alone
    float2* Tt = dsm;                                               // [P][KP]  (cos, sin)(2 pi k p / N)
    float* F = reinterpret_cast<float*>(Tt + (size_t)P * KP);       // [KP][2][64]  g_k C_k, g_k S_k (zero beyond sigma)
    float* gk = F + (size_t)KP * 128;                               // [KP]
    float* red = gk + KP;                                           // [8][kDfBins][2][64]
    float2* tw = reinterpret_cast<float2*>(red);                    // [N]  (cos, sin)(2 pi i / N): only until T is built
    __shared__ int flag;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile = blockIdx.x, n_tiles = gridDim.x, b = blockIdx.y;
    const int d = tile * 64 + lane;
    const bool live = d < D;
    const T* xb = x + (int64_t)b * N * row_stride + (live ? d : 0);

    // Tokens p and N - p see the same cosines and opposite sines: with u = x[p] + x[N-p], v = x[p] - x[N-p] a bin takes
    // C += u cos, S += v sin (half the products), and the inverse gives x'[p] = A + B, x'[N-p] = A - B from
    // A = sum F_c cos, B = sum F_s sin.  A token that stands alone (p = 0, p = N/2) has sin = 0 exactly and a partner
    // value of zero.
    // A sample of at most 16 x kDfChunk pairs gives every wavefront a single batch: it is fetched once, here, ahead of
    // the table arithmetic, and serves all groups of bins.  Longer samples fetch batch by batch, per group.
    const bool one_batch = P <= kDfWaves * kDfChunk;
    // (slots = pairs a wavefront takes per batch: half a batch when the whole sample fits in that)
    auto fetch = [&](int pb, float (&xu)[kDfChunk], float (&xv)[kDfChunk], auto slots) {
        constexpr int CH = decltype(slots)::value;
        float xa[CH], xm[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int p = pb + kDfWaves * i, q = (p < P && p > 0) ? N - p : 0;     // always valid addresses: no branch around the loads
            xa[i] = tr::load(xb + (int64_t)(p < P ? p : 0) * row_stride);
            xm[i] = tr::load(xb + (int64_t)q * row_stride);
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int p = pb + kDfWaves * i;
            const bool there = live && p < P, paired = there && p > 0 && 2 * p != N;
            const float a = there ? xa[i] : 0.f, m = paired ? xm[i] : 0.f;
            xu[i] = a + m;
            xv[i] = a - m;
        }
    };
    using full_t = std::integral_constant<int, kDfChunk>;
    using half_t = std::integral_constant<int, kDfChunk / 2>;
    using quarter_t = std::integral_constant<int, kDfChunk / 4>;
    const bool half_batch = P <= kDfWaves * (kDfChunk / 2), quarter_batch = P <= kDfWaves * (kDfChunk / 4);
    float u0[kDfChunk], v0[kDfChunk];
    if (quarter_batch) fetch(wave, u0, v0, quarter_t{});
    else if (half_batch) fetch(wave, u0, v0, half_t{});
    else if (one_batch) fetch(wave, u0, v0, full_t{});

    for (int i = tid; i < N; i += 64 * kDfWaves) {
        double sd, cd;
        sincospi(2.0 * (double)i / (double)N, &sd, &cd);
        tw[i] = make_float2((float)cd, (float)sd);
    }
    for (int k = tid; k < KP; k += 64 * kDfWaves) {
        double w = 1.0;
        if (use_hamming && N > 1) w = 0.54 + 0.46 * cospi(2.0 * (double)k / (double)(N - 1));
        const double pair = (k == 0 || 2 * k == N) ? 1.0 : 2.0;       // +k and -k paired (real-signal form)
        gk[k] = k <= sigma ? (float)(pair * w / (double)N) : 0.f;
    }
    __syncthreads();
    for (int e = tid; e < P * KP; e += 64 * kDfWaves) {
        const uint32_t n = (uint32_t)e / (uint32_t)KP, k = (uint32_t)e - n * (uint32_t)KP;
        Tt[e] = tw[(k * n) % (uint32_t)N];                            // k n < 2^24
    }
    __syncthreads();                                                  // tw (inside red) is free from here on

    // ---- forward (Eq. 4 on the pass band), mask (Eq. 5-6) with the 1/N of Eq. 7
    for (int k0 = 0; k0 < KP; k0 += kDfBins) {
        float ac[kDfBins], as[kDfBins];
#pragma unroll
        for (int j = 0; j < kDfBins; ++j) { ac[j] = 0.f; as[j] = 0.f; }
        auto accumulate = [&](int pb, const float (&xu)[kDfChunk], const float (&xv)[kDfChunk], auto slots) {
#pragma unroll
            for (int i = 0; i < decltype(slots)::value; ++i) {
                // no branch in this loop (a pair past the end adds zeros): the loads stay together, ahead of all uses
                const int p = pb + kDfWaves * i;
                const float4* tn = reinterpret_cast<const float4*>(Tt + (size_t)(p < P ? p : 0) * KP + k0);
#pragma unroll
                for (int j = 0; j < kDfBins / 2; ++j) {
                    const float4 t = tn[j];                           // bins k0 + 2j, k0 + 2j + 1
                    ac[2 * j] = fmaf(xu[i], t.x, ac[2 * j]);
                    as[2 * j] = fmaf(xv[i], t.y, as[2 * j]);
                    ac[2 * j + 1] = fmaf(xu[i], t.z, ac[2 * j + 1]);
                    as[2 * j + 1] = fmaf(xv[i], t.w, as[2 * j + 1]);
                }
            }
        };
        if (quarter_batch) accumulate(wave, u0, v0, quarter_t{});
        else if (half_batch) accumulate(wave, u0, v0, half_t{});
        else if (one_batch) accumulate(wave, u0, v0, full_t{});
        else
            for (int pb = wave; pb < P; pb += kDfWaves * kDfChunk) {  // this wavefront's pairs, 2 kDfChunk loads in flight at a time
                float xu[kDfChunk], xv[kDfChunk];
                fetch(pb, xu, xv, full_t{});
                accumulate(pb, xu, xv, full_t{});
            }
        // the 16 partial sums of a bin meet in two steps, so that the exchange buffer holds 8 wavefronts' worth:
        // wavefront w + 8 hands its sums to wavefront w, then the 8 pair sums are added in wavefront order
        const int slot = wave & (kDfWaves / 2 - 1);
        if (wave >= kDfWaves / 2) {
#pragma unroll
            for (int j = 0; j < kDfBins; ++j) {
                red[((slot * kDfBins + j) * 2 + 0) * 64 + lane] = ac[j];
                red[((slot * kDfBins + j) * 2 + 1) * 64 + lane] = as[j];
            }
        }
        __syncthreads();
        if (wave < kDfWaves / 2) {                                     // reads and rewrites its own slot only
#pragma unroll
            for (int j = 0; j < kDfBins; ++j) {
                float* rc = red + ((slot * kDfBins + j) * 2 + 0) * 64 + lane;
                float* rs = red + ((slot * kDfBins + j) * 2 + 1) * 64 + lane;
                *rc = ac[j] + *rc;
                *rs = as[j] + *rs;
            }
        }
        __syncthreads();
        for (int i = tid; i < kDfBins * 128; i += 64 * kDfWaves) {     // i = (j, cos/sin, lane)
            const int k = k0 + (i >> 7);
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < kDfWaves / 2; ++w) sum += red[w * kDfBins * 128 + i];
            F[k * 128 + (i & 127)] = gk[k] * sum;                      // bins past sigma carry weight zero
        }
        __syncthreads();
    }

    // ---- inverse (Eq. 7, +k and -k paired) and energy over the tile's channels (Eq. 8)
    float* pout = partial + ((int64_t)b * n_tiles + tile) * N;
    const tile_tag_t seen = tiles_look<1>(sy, b, tile, n_tiles);      // no loads follow: nothing waits behind this one
    for (int pb = wave; pb < P; pb += kDfWaves * kDfTok) {
        float accA[kDfTok], accB[kDfTok];
#pragma unroll
        for (int j = 0; j < kDfTok; ++j) { accA[j] = 0.f; accB[j] = 0.f; }
        for (int k0 = 0; k0 < KP; k0 += kDfBins) {
            float fc[kDfBins], fs[kDfBins];
#pragma unroll
            for (int q = 0; q < kDfBins; ++q) { fc[q] = F[(k0 + q) * 128 + lane]; fs[q] = F[(k0 + q) * 128 + 64 + lane]; }
#pragma unroll
            for (int j = 0; j < kDfTok; ++j) {
                const int p = pb + kDfWaves * j;
                const float4* tn = reinterpret_cast<const float4*>(Tt + (size_t)(p < P ? p : 0) * KP + k0);
#pragma unroll
                for (int q = 0; q < kDfBins / 2; ++q) {
                    const float4 t = tn[q];
                    accA[j] = fmaf(fc[2 * q], t.x, accA[j]);
                    accB[j] = fmaf(fs[2 * q], t.y, accB[j]);
                    accA[j] = fmaf(fc[2 * q + 1], t.z, accA[j]);
                    accB[j] = fmaf(fs[2 * q + 1], t.w, accB[j]);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < kDfTok; ++j) {
            const int p = pb + kDfWaves * j;
            const float xp = accA[j] + accB[j], xq = accA[j] - accB[j];            // x'[p], x'[N - p]
            const float ep = wave_sum(xp * xp), eq = wave_sum(xq * xq);
            if (lane == 0 && p < P) {
                tile_store(pout + p, ep);
                if (p > 0 && 2 * p != N) tile_store(pout + (N - p), eq);
            }
        }
        if (pb == wave) tiles_claim<1>(sy, b, tile, n_tiles, seen);    // by the end of the loop the swap has long been served
    }
    tiles_to_scores<64 * kDfWaves, 1>(partial, gpartial, sy, scores, b, tile, n_tiles, N, &flag);
}

// Tags of the arrival words (spu_tiles.hpp): one per launch, from a process-wide sequence that starts at a random
// 48-bit value, so that whatever a workspace held before cannot pass for a word of this launch.  Never zero.
tile_tag_t spu_next_tag()
{
    static std::atomic<unsigned long long> next{[] {
        unsigned long long r = 0;
        try {
            std::random_device rd;
            r = ((unsigned long long)rd() << 32) ^ (unsigned long long)rd();
        } catch (...) {                                    // no entropy source: the clock and an address will have to do
            r = (unsigned long long)(uintptr_t)&r;
        }
        const unsigned long long t = (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count();
        return r ^ (t * 0x9E3779B97F4A7C15ull);
    }()};
    for (;;) {
        const tile_tag_t tag = next.fetch_add(1, std::memory_order_relaxed) & 0xffffffffffffull;
        if (tag) return tag;
    }
}

// ------------------------------------------------------------------ host side
SpuLayout spu_layout(int B, int N, int D, int sigma)
{
    SpuLayout L;
    L.fast = spu_fft_supported(N, sigma);
    L.n_tiles = L.fast ? (D + 31) / 32 : (D + 63) / 64;
    const size_t spec = L.fast ? 0 : (size_t)B * (sigma + 1) * D;   // pass-band spectra of the direct path
    size_t off = 0;
    // the fast path builds its tables in LDS
    L.tw = off;      off += L.fast ? 0 : align_up(sizeof(float2) * (size_t)N);
    L.gk = off;      off += L.fast ? 0 : align_up(sizeof(float) * (size_t)(sigma + 1));
    L.gm = off;      off += L.fast ? 0 : align_up(sizeof(float) * (size_t)(sigma + 1));
    L.Fc = off;      off += align_up(sizeof(float) * spec);
    L.Fs = off;      off += align_up(sizeof(float) * spec);
    L.partial = off; off += align_up(sizeof(float) * (size_t)B * L.n_tiles * N);
    L.gpartial = off; off += align_up(sizeof(float) * (size_t)B * spu_tile_groups(L.n_tiles) * N);
    L.arrive = off;  off += align_up(sizeof(tile_tag_t) * (size_t)B * (spu_tile_groups(L.n_tiles) + 1));
    L.bytes = off;
    return L;
}

luvc_status spu_score_dense(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dt, int sigma,
                            int use_hamming, float* scores, void* workspace, hipStream_t st)
{
    const SpuLayout L = spu_layout(B, N, D, sigma);
    char* ws = (char*)workspace;
    float2* tw = (float2*)(ws + L.tw);
    float* gk = (float*)(ws + L.gk);
    float* gm = (float*)(ws + L.gm);
    float* Fc = (float*)(ws + L.Fc);
    float* Fs = (float*)(ws + L.Fs);
    float* partial = (float*)(ws + L.partial);
    float* gpartial = (float*)(ws + L.gpartial);
    if (L.n_tiles > 65535) { set_error("D=%d exceeds the supported width", D); return LUVC_ERR_UNSUPPORTED; }
    TileSync sy;
    sy.arrive = (tile_tag_t*)(ws + L.arrive);
    sy.tag = spu_next_tag();
    if (L.fast) return spu_score_fft(x, B, N, D, row_stride, dt, sigma, use_hamming, partial, gpartial, sy, L.n_tiles, scores, st);
    if (dense_fused_lds(N, sigma) <= dense_fused_cap()) {
        const dim3 grid((unsigned)L.n_tiles, (unsigned)B);
        if (dt == LUVC_F32)
            LUVC_LAUNCH("spu_dense_fused", (spu_dense_fused<float>), grid, dim3(64 * kDfWaves), dense_fused_lds(N, sigma), st,
                        (const float*)x, N, D, row_stride, sigma, use_hamming, partial, gpartial, sy, scores);
        else
            LUVC_LAUNCH("spu_dense_fused", (spu_dense_fused<bf16_t>), grid, dim3(64 * kDfWaves), dense_fused_lds(N, sigma), st,
                        (const bf16_t*)x, N, D, row_stride, sigma, use_hamming, partial, gpartial, sy, scores);
        return check_launch("spu score (dense, one launch)");
    }
    LUVC_LAUNCH("spu_tables", spu_tables, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, N, sigma, use_hamming, tw, gk, gm);
    const int64_t total = (int64_t)B * N;
    const dim3 gf((unsigned)L.n_tiles, (unsigned)((sigma + 1 + 4 * kKPW - 1) / (4 * kKPW)), (unsigned)B);
    if (dt == LUVC_F32)
        LUVC_LAUNCH("spu_fwd_dense", (spu_fwd_dense<float>), gf, dim3(256), 0, st, (const float*)x, N, D, row_stride, sigma, tw, Fc, Fs);
    else
        LUVC_LAUNCH("spu_fwd_dense", (spu_fwd_dense<bf16_t>), gf, dim3(256), 0, st, (const bf16_t*)x, N, D, row_stride, sigma, tw, Fc, Fs);
    const dim3 gi((unsigned)L.n_tiles, (unsigned)((N + kNChunk - 1) / kNChunk), (unsigned)B);
    LUVC_LAUNCH("spu_inv_dense", spu_inv_dense, gi, dim3(256), 0, st, Fc, Fs, N, D, sigma, tw, gk, partial);
    LUVC_LAUNCH("spu_finish", spu_finish, dim3((unsigned)((total + 63) / 64)), dim3(64 * kFinParts), 0, st, partial, N, L.n_tiles, total, scores);
    return check_launch("spu score");
}

}  // namespace luvc
