// SPU prune (paper Algorithm 2, last two steps): order-preserving top-k keep and gather.
//
//   spu_select   one workgroup per sample.  Scores are mapped to unsigned keys whose integer order
//                is the float order; a most-significant-digit radix select (4 passes of 8 bits,
//                histogram in LDS) finds the key T of the n_keep-th largest score and how many
//                tokens with key == T still belong to the keep set; a stable block-wide compaction
//                then emits, in ascending index order, every token with key > T and the first of
//                those with key == T (equal scores: the lower index wins).
//   spu_gather   one wavefront per kept token copies the ORIGINAL row.
#include "common.hpp"
#include "spu.hpp"

namespace luvc {

__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0;                      // -0 and +0 compare equal
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// inclusive prefix sum over the 64 lanes without the LDS crossbar: shifts inside each row of 16 lanes, then the
// last lane of rows 0 / 2 into rows 1 / 3, then lane 31 into the upper half (lanes without a source add zero)
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);     // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);     // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);     // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);     // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);     // row_bcast:15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);     // row_bcast:31 -> rows 2, 3
    return v;
}

// largest value of the wavefront in every lane's hands: DPP row steps, then the four row results through readlane
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    auto mx = [](uint32_t a, int b) { return a > (uint32_t)b ? a : (uint32_t)b; };
    v = mx(v, __builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xf, 0xf, false));     // quad_perm [1,0,3,2]
    v = mx(v, __builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xf, 0xf, false));     // quad_perm [2,3,0,1]
    v = mx(v, __builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xf, 0xf, false));    // row_half_mirror
    v = mx(v, __builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xf, 0xf, false));    // row_mirror
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16),
                   r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    const uint32_t a = r0 > r1 ? r0 : r1, c = r2 > r3 ? r2 : r3;
    return a > c ? a : c;
}

constexpr int kSelThreads = 1024;

// inclusive block scan of one int per thread; returns the inclusive prefix, *total gets the block sum
__device__ __forceinline__ int block_scan_incl(int v, int* wave_tot /*[16]*/, int* total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = (int)wave_scan_incl((uint32_t)v);
    __syncthreads();                                   // wave_tot may still be read from a previous scan
    if (lane == 63) wave_tot[wave] = s;
    __syncthreads();
    int base = 0, tot = 0;
    const int nw = blockDim.x >> 6;
    for (int w = 0; w < nw; ++w) {
        const int t = wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    *total = tot;
    return s + base;
}

constexpr int kSelMaxRegKeys = 8;                     // keys cached in registers per thread (N <= 8 * 1024)

__global__ void __launch_bounds__(kSelThreads)
spu_select(const float* __restrict__ scores, int N, int n_keep, int32_t* __restrict__ kept_idx,
           const int32_t* __restrict__ origin_in /* [B,N] or null: identity */, int32_t* __restrict__ origin_out /* [B,n_keep] or null */)
{
    __shared__ int hist[256];
    __shared__ int wave_tot[16];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_remaining;
    const int b = blockIdx.x, tid = threadIdx.x;
    const float* s = scores + (int64_t)b * N;
    int32_t* out = kept_idx + (int64_t)b * n_keep;

    // keys of tokens tid, tid + 1024, ... stay in registers when the sample is small enough
    const bool cached = N <= kSelMaxRegKeys * kSelThreads;
    uint32_t key[kSelMaxRegKeys];
#pragma unroll
    for (int i = 0; i < kSelMaxRegKeys; ++i) {
        const int n = tid + i * kSelThreads;
        key[i] = (cached && n < N) ? score_key(s[n]) : 0u;
    }

    uint32_t prefix = 0, mask = 0;
    int remaining = n_keep;                            // still to pick among keys matching the prefix
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        if (cached) {
#pragma unroll
            for (int i = 0; i < kSelMaxRegKeys; ++i)
                if (tid + i * kSelThreads < N && (key[i] & mask) == prefix) atomicAdd(&hist[(key[i] >> shift) & 255u], 1);
        } else {
            for (int n = tid; n < N; n += kSelThreads) {
                const uint32_t k = score_key(s[n]);
                if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
            }
        }
        __syncthreads();
        // digit d is the one where (tokens with a larger digit) < remaining <= (those plus hist[d]);
        // thread i looks at digit 255 - i so that an inclusive scan counts "this digit and larger"
        int h = 0, incl = 0, tot;
        if (tid < 256) h = hist[255 - tid];
        incl = block_scan_incl(tid < 256 ? h : 0, wave_tot, &tot);
        if (tid < 256 && incl - h < remaining && remaining <= incl) {
            sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
            sh_remaining = remaining - (incl - h);
        }
        __syncthreads();
        prefix = sh_prefix;
        remaining = sh_remaining;
        mask |= 255u << shift;
    }
    const uint32_t T = prefix;                         // key of the n_keep-th largest score
    const int take_eq = remaining;                     // tokens with key == T that are kept (lowest indices)

    int eq_before = 0, sel_before = 0;
    for (int n0 = 0, i = 0; n0 < N; n0 += kSelThreads, ++i) {
        const int n = n0 + tid;
        uint32_t k = 0;
        bool eq = false, gt = false;
        if (n < N) {
            k = score_key(s[n]);                       // L1/L2-resident re-read; keeps the loop free of dynamic register indexing
            eq = (k == T);
            gt = (k > T);
        }
        int tot_eq, tot_sel;
        const int eq_incl = block_scan_incl(eq ? 1 : 0, wave_tot, &tot_eq);
        const bool sel = gt || (eq && (eq_before + eq_incl - 1) < take_eq);
        const int sel_incl = block_scan_incl(sel ? 1 : 0, wave_tot, &tot_sel);
        if (sel) {
            const int q = sel_before + sel_incl - 1;
            if (q < n_keep) {
                out[q] = n;
                if (origin_out) origin_out[(int64_t)b * n_keep + q] = origin_in ? origin_in[(int64_t)b * N + n] : n;
            }
        }
        eq_before += tot_eq;
        sel_before += tot_sel;
    }
}

template <int BYTES>   // 16: vector rows, 4 / 2: element rows
__global__ void __launch_bounds__(256)
spu_gather(const unsigned char* __restrict__ x, const int32_t* __restrict__ kept_idx, int N, int n_keep,
           int64_t row_bytes_in, int64_t row_bytes_out, int64_t n_rows, unsigned char* __restrict__ x_out)
{
    const int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const int64_t b = row / n_keep;
    int src = kept_idx[row];
    src = src < 0 ? 0 : (src >= N ? N - 1 : src);      // indices come from spu_select; stay in bounds regardless
    const unsigned char* in = x + (b * N + src) * row_bytes_in;
    unsigned char* o = x_out + row * row_bytes_out;
    if (BYTES == 16) {
        for (int64_t i = (int64_t)lane * 16; i < row_bytes_out; i += 64 * 16)
            *reinterpret_cast<uint4*>(o + i) = *reinterpret_cast<const uint4*>(in + i);
    } else if (BYTES == 4) {
        for (int64_t i = (int64_t)lane * 4; i < row_bytes_out; i += 64 * 4)
            *reinterpret_cast<uint32_t*>(o + i) = *reinterpret_cast<const uint32_t*>(in + i);
    } else {
        for (int64_t i = (int64_t)lane * 2; i < row_bytes_out; i += 64 * 2)
            *reinterpret_cast<uint16_t*>(o + i) = *reinterpret_cast<const uint16_t*>(in + i);
    }
}

// ------------------------------------------------------------------ select + gather in one launch (N <= 4096)
// Workgroup (g, b) of 256 threads repeats the selection of sample b on its own (the scores of a sample
// are a few KB, and the groups run side by side), keeps the list of kept tokens in LDS, and then copies
// its share of the kept rows: row q goes to wavefront q mod (4 G) of the sample.  Group 0 also writes
// kept_idx.  Compared with a selection launch followed by a gather launch this saves a dispatch and the
// wait between the two, which is most of the time at these sizes.
// cache policy of the row copies (buffer aux bits): the copied rows are not read again by this kernel, so the stores
// carry the non-temporal hint (2) and leave less dirty data in L2 for the end of the kernel (measured: -0.3 us)
constexpr int kPruneLoadAux = 0, kPruneStoreAux = 2;
typedef unsigned int prune_u32x4 __attribute__((__vector_size__(16)));
constexpr int kFusedMaxN = 4096, kFusedThreads = 256, kFusedKeys = kFusedMaxN / kFusedThreads;

template <int BYTES>
__global__ void __launch_bounds__(kFusedThreads)
spu_prune_fused(const unsigned char* __restrict__ x, const float* __restrict__ scores, int N, int n_keep,
                int64_t row_bytes_in, int64_t row_bytes_out, int32_t* __restrict__ kept_idx, unsigned char* __restrict__ x_out,
                const int32_t* __restrict__ origin_in /* [B,N] or null: identity */, int32_t* __restrict__ origin_out /* [B,n_keep] or null */)
{
    __shared__ int32_t kept[kFusedMaxN];
    __shared__ int hist[4][256];                       // one histogram per digit pass: none has to be cleared in between
    __shared__ uint32_t wave_tot[4], wave_hi[4], wave_lo[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x, G = gridDim.x, b = blockIdx.y;
    const float* s = scores + (int64_t)b * N;
    // thread tid owns the K consecutive tokens tid * K .. tid * K + K - 1 and reads them straight from memory
    // (a wavefront covers 64 K consecutive scores; a few KB per sample, served by the caches)
    const int K = (N + kFusedThreads - 1) / kFusedThreads, n0 = tid * K;
    uint32_t key[kFusedKeys];
#pragma unroll
    for (int i = 0; i < kFusedKeys; ++i) key[i] = (i < K && n0 + i < N) ? score_key(s[n0 + i]) : 0u;
    hist[0][tid] = 0; hist[1][tid] = 0; hist[2][tid] = 0; hist[3][tid] = 0;
    // Largest and smallest key of the sample: the bits above the highest one in which they differ are common to all
    // keys and need no digit pass (scores of one sample share sign and most of the exponent, so the first of four
    // 8-bit passes would pile every key onto one or two counters - same-address LDS atomics, one after the other).
    uint32_t hi = 0u, lo = 0xffffffffu;
#pragma unroll
    for (int i = 0; i < kFusedKeys; ++i)
        if (i < K && n0 + i < N) { hi = key[i] > hi ? key[i] : hi; lo = key[i] < lo ? key[i] : lo; }
    hi = wave_max_u32(hi);
    lo = ~wave_max_u32(~lo);
    if (lane == 0) { wave_hi[wave] = hi; wave_lo[wave] = lo; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 4; ++w) { hi = wave_hi[w] > hi ? wave_hi[w] : hi; lo = wave_lo[w] < lo ? wave_lo[w] : lo; }
    const int nb = 32 - __clz((int)(hi ^ lo));         // the keys differ in their low nb bits only (0: all equal)

    // MSD radix select on those bits, 8 at a time (the last pass takes what is left).  Every wavefront scans the
    // histogram of a pass on its own - same counters, same result - so a pass costs one barrier and nothing is
    // handed from wavefront to wavefront.
    uint32_t prefix = nb >= 32 ? 0u : (hi >> nb) << nb, mask = nb >= 32 ? 0u : ~((1u << nb) - 1u);
    int remaining = n_keep;                            // still to pick among keys matching the prefix
    for (int top = nb, pass = 0; top > 0; top -= 8, ++pass) {
        const int shift = top > 8 ? top - 8 : 0, width = top - shift;
        const uint32_t dmask = (1u << width) - 1u;
        int* h_pass = hist[pass];
#pragma unroll
        for (int i = 0; i < kFusedKeys; ++i)
            if (i < K && n0 + i < N && (key[i] & mask) == prefix) atomicAdd(&h_pass[(key[i] >> shift) & dmask], 1);
        __syncthreads();
        // lane l looks at digits 255 - 4 l .. 252 - 4 l, largest first
        int h[4], sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { h[j] = h_pass[255 - 4 * lane - j]; sum += h[j]; }
        const int incl = (int)wave_scan_incl((uint32_t)sum);
        int above = incl - sum;                        // tokens with a larger digit
        int digit = 0, left = 0;
        bool found = false;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (above < remaining && remaining <= above + h[j]) { digit = 255 - 4 * lane - j; left = remaining - above; found = true; }
            above += h[j];
        }
        const unsigned long long who = __ballot(found);
        if (who) {                                     // one lane at most (none only when nothing is kept)
            const int src = (int)__builtin_ctzll(who);
            digit = __builtin_amdgcn_readlane(digit, src);
            remaining = __builtin_amdgcn_readlane(left, src);
        }
        prefix |= (uint32_t)digit << shift;
        mask |= dmask << shift;
    }
    const uint32_t T = prefix;                         // key of the n_keep-th largest score
    const int take_eq = remaining;                     // tokens with key == T that are kept (lowest indices)

    // one scan for both counts: tokens above T in the low half, tokens equal to T in the high half
    uint32_t cnt = 0;
#pragma unroll
    for (int i = 0; i < kFusedKeys; ++i)
        if (i < K && n0 + i < N) cnt += (key[i] > T ? 1u : 0u) + (key[i] == T ? 0x10000u : 0u);
    const uint32_t incl = wave_scan_incl(cnt);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = incl - cnt;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    int eq_rank = (int)(before >> 16);
    int pos = (int)(before & 0xffffu) + (eq_rank < take_eq ? eq_rank : take_eq);
#pragma unroll
    for (int i = 0; i < kFusedKeys; ++i) {
        if (i < K && n0 + i < N) {
            const bool eq = key[i] == T;
            if (key[i] > T || (eq && eq_rank < take_eq)) {
                if (pos < n_keep) kept[pos] = n0 + i;
                ++pos;
            }
            eq_rank += eq ? 1 : 0;
        }
    }
    __syncthreads();
    if (g == 0) {
        for (int q = tid; q < n_keep; q += kFusedThreads) kept_idx[(int64_t)b * n_keep + q] = kept[q];
        // position of every kept token before the first stage of a cascade
        if (origin_out)
            for (int q = tid; q < n_keep; q += kFusedThreads)
                origin_out[(int64_t)b * n_keep + q] = origin_in ? origin_in[(int64_t)b * N + kept[q]] : kept[q];
    }
    if (!x_out) return;
    for (int q = g * 4 + wave; q < n_keep; q += G * 4) {
        int src = kept[q];
        src = src < 0 ? 0 : (src >= N ? N - 1 : src);  // in bounds whatever the scores held
        const unsigned char* in = x + ((int64_t)b * N + src) * row_bytes_in;
        unsigned char* o = x_out + ((int64_t)b * n_keep + q) * row_bytes_out;
        if (BYTES == 16) {
            // eight 16-byte pieces per lane in flight before the first store (bounds by the buffer descriptors: pieces
            // past the end of the row read zeros and write nothing), so a row costs one trip to memory, not seven
            const int rb = (int)(row_bytes_out > 0x7fffffff ? 0x7fffffff : row_bytes_out);
            const __amdgpu_buffer_rsrc_t ri = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(in), 0, rb, 0x00020000);
            const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(o, 0, rb, 0x00020000);
            for (int base = 0; base < rb; base += 8 * 1024) {
                prune_u32x4 v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = __builtin_amdgcn_raw_buffer_load_b128(ri, base + k * 1024 + lane * 16, 0, kPruneLoadAux);
#pragma unroll
                for (int k = 0; k < 8; ++k) __builtin_amdgcn_raw_buffer_store_b128(v[k], ro, base + k * 1024 + lane * 16, 0, kPruneStoreAux);
            }
        } else if (BYTES == 4) {
            for (int64_t i = (int64_t)lane * 4; i < row_bytes_out; i += 64 * 4)
                *reinterpret_cast<uint32_t*>(o + i) = *reinterpret_cast<const uint32_t*>(in + i);
        } else {
            for (int64_t i = (int64_t)lane * 2; i < row_bytes_out; i += 64 * 2)
                *reinterpret_cast<uint16_t*>(o + i) = *reinterpret_cast<const uint16_t*>(in + i);
        }
    }
}

luvc_status spu_prune_run(const void* x, const float* scores, int B, int N, int D, int64_t row_stride, luvc_dtype dt,
                          int n_keep, int32_t* kept_idx, void* x_out, const int32_t* origin_in, int32_t* origin_out, hipStream_t st)
{
    const int es = dt == LUVC_F32 ? 4 : 2;
    const int64_t rin = row_stride * es, rout = (int64_t)D * es, rows = (int64_t)B * n_keep;
    const bool v16 = x_out && rin % 16 == 0 && rout % 16 == 0 && ((uintptr_t)x % 16 == 0) && ((uintptr_t)x_out % 16 == 0);
    if (N <= kFusedMaxN && B <= 65535) {
        int G = x_out ? (n_keep + 3) / 4 : 1;          // one kept row per wavefront, up to 256 groups per sample
        G = G > 256 ? 256 : G;
        const dim3 grid((unsigned)G, (unsigned)B);
        if (v16 || !x_out)
            LUVC_LAUNCH("spu_prune_fused", (spu_prune_fused<16>), grid, dim3(kFusedThreads), 0, st, (const unsigned char*)x, scores, N, n_keep, rin, rout, kept_idx, (unsigned char*)x_out, origin_in, origin_out);
        else if (es == 4)
            LUVC_LAUNCH("spu_prune_fused", (spu_prune_fused<4>), grid, dim3(kFusedThreads), 0, st, (const unsigned char*)x, scores, N, n_keep, rin, rout, kept_idx, (unsigned char*)x_out, origin_in, origin_out);
        else
            LUVC_LAUNCH("spu_prune_fused", (spu_prune_fused<2>), grid, dim3(kFusedThreads), 0, st, (const unsigned char*)x, scores, N, n_keep, rin, rout, kept_idx, (unsigned char*)x_out, origin_in, origin_out);
        return check_launch("spu prune");
    }
    LUVC_LAUNCH("spu_select", spu_select, dim3((unsigned)B), dim3(kSelThreads), 0, st, scores, N, n_keep, kept_idx, origin_in, origin_out);
    if (x_out) {
        const unsigned g = (unsigned)((rows * 64 + 255) / 256);
        if (v16)
            LUVC_LAUNCH("spu_gather", (spu_gather<16>), dim3(g), dim3(256), 0, st, (const unsigned char*)x, kept_idx, N, n_keep, rin, rout, rows, (unsigned char*)x_out);
        else if (es == 4)
            LUVC_LAUNCH("spu_gather", (spu_gather<4>), dim3(g), dim3(256), 0, st, (const unsigned char*)x, kept_idx, N, n_keep, rin, rout, rows, (unsigned char*)x_out);
        else
            LUVC_LAUNCH("spu_gather", (spu_gather<2>), dim3(g), dim3(256), 0, st, (const unsigned char*)x, kept_idx, N, n_keep, rin, rout, rows, (unsigned char*)x_out);
    }
    return check_launch("spu prune");
}

}  // namespace luvc
