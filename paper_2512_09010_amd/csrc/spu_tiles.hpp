// Eq. 8 of the paper (Section 3.3) across workgroups: every workgroup of an SPU score kernel owns one
// channel tile of one sample and has the tile's energies  sum_d x'[n,d]^2  (n < N) in LDS; the score
// needs the sum over all tiles of the sample.  This header holds the hand-over that lets the same
// launch finish the job, in two levels that both add in index order (so the result does not depend
// on which workgroup does the adding): the workgroup that completes a group of kTileGroup tiles last
// adds those tiles; the one that completes the last group of the sample adds the groups and takes
// the square root.
//
// Tile energies and group sums travel as device-scope (write-through) stores and are read back with
// device-scope loads: the workgroups of a sample run on several XCDs, whose L2s are not kept coherent
// with each other inside a launch, and a full release / acquire fence (an L2 write-back and invalidate
// per workgroup) costs more than the whole transform.  Before a workgroup bumps a counter, each of its
// wavefronts has waited for its own stores to complete and all of them have met at a barrier.
//
// Arrival words: 1 + n_groups 64-bit words per sample (the sample's, then one per group) in the caller's
// workspace, whose contents are arbitrary when a call starts.  The upper 48 bits of a word name the launch (a
// non-zero tag the host draws from a process-wide sequence with a random start and passes as a kernel argument),
// the lower 16 count arrivals.  Every workgroup looks, some time before it arrives, at the words that may be
// bumped after its own arrival and before any other workgroup's claim, and, where the tag is missing, tries one
// compare-and-swap from what it saw to (tag, 0).  If that fails the word has changed since the look, and the only
// thing that changes a word without the tag during this launch is another workgroup's successful swap: either way
// the word carries the tag before this workgroup - or any other - bumps it, since a workgroup bumps only after
// its own attempt.  The workgroup that completes a count stores zero (no tag), so that a captured launch replayed
// with the same tag starts over the same way.  Nothing has to be set up before a launch and nothing is shared
// between launches: any number of calls may be in flight, each on a workspace of its own.
// (An arrival is an atomic add: a compare-and-swap loop in its place makes the workgroups of a group, which end
// together, retry one after the other, a trip to memory each - measured at +17 us per launch.  Atomics on one
// address are served one at a time, a microsecond apart, and a wavefront's later loads return behind them:
// look and claim sit where no loads follow - after the forward transform.)
#pragma once
#include "common.hpp"

namespace luvc {

constexpr int kTileGroup = 16;                   // channel tiles whose energies are added in one go

__device__ __forceinline__ void tile_store(float* p, float v)
{
    __hip_atomic_store(reinterpret_cast<unsigned int*>(p), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// W consecutive floats (W = 4: one 16-byte access, needs 16-byte alignment) with device scope
template <int W> struct tile_vec { float v[W]; };
typedef unsigned int tile_u32x4 __attribute__((__vector_size__(16)));
constexpr int kAuxSc1 = 16;                      // cache-policy bit of the buffer instructions: device scope

template <int W>
__device__ __forceinline__ tile_vec<W> tile_load(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    tile_vec<W> o;
    if (W == 4) {
        const tile_u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kAuxSc1);
        o.v[0] = __uint_as_float(q[0]); o.v[1 % W] = __uint_as_float(q[1]); o.v[2 % W] = __uint_as_float(q[2]); o.v[3 % W] = __uint_as_float(q[3]);
    } else {
        o.v[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, kAuxSc1));
    }
    return o;
}
template <int W>
__device__ __forceinline__ void tile_store(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, const tile_vec<W>& o)
{
    if (W == 4) {
        tile_u32x4 q;
        q[0] = __float_as_uint(o.v[0]); q[1] = __float_as_uint(o.v[1 % W]); q[2] = __float_as_uint(o.v[2 % W]); q[3] = __float_as_uint(o.v[3 % W]);
        __builtin_amdgcn_raw_buffer_store_b128(q, r, byte_off, 0, kAuxSc1);
    } else {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o.v[0]), r, byte_off, 0, kAuxSc1);
    }
}

// out[n] = sum over `count` rows (row stride N floats) of in[row][n], added in row order in fp64; FIN: square root.
// Up to TRIP rows per trip, all loads of a trip in flight together (a short trip re-reads its last row).
template <int THREADS, int W, bool FIN, int TRIP = kTileGroup>
__device__ __forceinline__ void tile_rows_sum(const float* in, int count, int N, float* out)
{
    const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(in), 0, count * N * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(out, 0, N * 4, 0x00020000);
    for (int i = threadIdx.x * W; i < N; i += THREADS * W) {
        double e[W];
#pragma unroll
        for (int c = 0; c < W; ++c) e[c] = 0.0;
        for (int r0 = 0; r0 < count; r0 += TRIP) {
            const int left = count - r0;
            tile_vec<W> p[TRIP];
#pragma unroll
            for (int r = 0; r < TRIP; ++r)
                p[r] = tile_load<W>(rin, (uint32_t)(((r0 + (r < left ? r : left - 1)) * N + i) * 4));
#pragma unroll
            for (int r = 0; r < TRIP; ++r)
#pragma unroll
                for (int c = 0; c < W; ++c) e[c] += r < left ? (double)p[r].v[c] : 0.0;
        }
        tile_vec<W> o;
#pragma unroll
        for (int c = 0; c < W; ++c) o.v[c] = FIN ? (float)sqrt(e[c]) : (float)e[c];
        if (FIN) {
#pragma unroll
            for (int c = 0; c < W; ++c) out[i + c] = o.v[c];       // scores: ordinary stores, no alignment assumed
        } else {
            tile_store<W>(rout, (uint32_t)(i * 4), o);
        }
    }
}

// ------------------------------------------------------------------ arrival words
typedef unsigned long long tile_tag_t;

struct TileSync {
    tile_tag_t* arrive;          // [B][1 + n_groups] arrival words inside the workspace
    tile_tag_t tag;              // 48 bits, non-zero
};

constexpr int kTileGroupOneLevelMax = 64;        // W = 1: up to this many tiles are added in one level
inline __host__ __device__ int spu_tile_groups(int n_tiles) { return (n_tiles + kTileGroup - 1) / kTileGroup; }
template <int W>
__device__ __forceinline__ bool tiles_two_level(int n_tiles)
{
    // scalar accesses (W = 1) leave room for 64 loads in flight per thread
    return spu_tile_groups(n_tiles) > 1 && !(W == 1 && n_tiles <= kTileGroupOneLevelMax);
}

__device__ __forceinline__ tile_tag_t tag_load(const tile_tag_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void tag_store(tile_tag_t* p, tile_tag_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// The words the workgroup of (sample b, tile) claims: lane 0 of every workgroup handles the word it will bump
// itself (its group's, or the sample's where there is no group level); lane 1 of the first workgroup of every
// group handles the sample's word, which the workgroup that completes the group bumps - after every workgroup of
// the group has arrived, the first one with its claim behind it.
template <int W>
__device__ __forceinline__ tile_tag_t* tiles_word(const TileSync& sy, int b, int tile, int n_tiles)
{
    const int n_groups = spu_tile_groups(n_tiles);
    tile_tag_t* w = sy.arrive + (int64_t)b * (n_groups + 1);
    const bool two_level = tiles_two_level<W>(n_tiles);
    if (threadIdx.x == 0) return two_level ? w + 1 + tile / kTileGroup : w;
    if (threadIdx.x == 1 && two_level && tile % kTileGroup == 0) return w;
    return nullptr;
}
template <int W>
__device__ __forceinline__ tile_tag_t tiles_look(const TileSync& sy, int b, int tile, int n_tiles)
{
    const tile_tag_t* w = tiles_word<W>(sy, b, tile, n_tiles);
    return w ? tag_load(w) : 0;
}
template <int W>
__device__ __forceinline__ void tiles_claim(const TileSync& sy, int b, int tile, int n_tiles, tile_tag_t seen)
{
    tile_tag_t* w = tiles_word<W>(sy, b, tile, n_tiles);
    if (w && (seen >> 16) != sy.tag) {
        tile_tag_t expect = seen;
        (void)__hip_atomic_compare_exchange_strong(w, &expect, sy.tag << 16, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// One thread: bump the word, true if this was arrival number `total` (the word then goes back to "no tag").
__device__ __forceinline__ bool tiles_arrive(tile_tag_t* w, int total)
{
    const tile_tag_t old = __hip_atomic_fetch_add(w, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = (int)(old & 0xffffu) == total - 1;
    if (last) tag_store(w, 0ull);
    return last;
}

// Called by all THREADS threads of the workgroup of (sample b, tile) after they have written the tile's
// energies to partial[(b * n_tiles + tile) * N + n] with tile_store().  `flag` is a __shared__ word.
// W = 4 needs N % 4 == 0 (and the 256-byte alignment the workspace has anyway).  A sample of at most
// kTileGroup tiles has no group level: its last workgroup adds the tiles directly.
template <int THREADS, int W>
__device__ __forceinline__ void tiles_to_scores(float* __restrict__ partial /* [B, n_tiles, N] */,
                                                float* __restrict__ gpartial /* [B, n_groups, N] */,
                                                const TileSync sy,
                                                float* __restrict__ scores /* [B, N] */,
                                                int b, int tile, int n_tiles, int N, int* flag)
{
    const int tid = threadIdx.x;
    const int n_groups = spu_tile_groups(n_tiles);
    tile_tag_t* cnt = sy.arrive + (int64_t)b * (n_groups + 1);
    const bool two_level = tiles_two_level<W>(n_tiles);
    if (two_level) {
        const int grp = tile / kTileGroup, t_first = grp * kTileGroup;
        const int t_cnt = n_tiles - t_first < kTileGroup ? n_tiles - t_first : kTileGroup;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's stores have been performed
        __syncthreads();
        if (tid == 0) *flag = tiles_arrive(cnt + 1 + grp, t_cnt);
        __syncthreads();
        if (!*flag) return;
        tile_rows_sum<THREADS, W, false>(partial + ((int64_t)b * n_tiles + t_first) * N, t_cnt, N,
                                         gpartial + ((int64_t)b * n_groups + grp) * N);
    }
    const int last_cnt = two_level ? n_groups : n_tiles;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                             // also: every thread has read the flag
    if (tid == 0) *flag = tiles_arrive(cnt, last_cnt);
    __syncthreads();
    if (!*flag) return;
    if (two_level)
        tile_rows_sum<THREADS, W, true>(gpartial + (int64_t)b * n_groups * N, last_cnt, N, scores + (int64_t)b * N);
    else
        tile_rows_sum<THREADS, W, true, (W == 1 ? kTileGroupOneLevelMax : kTileGroup)>(partial + (int64_t)b * n_tiles * N, last_cnt, N, scores + (int64_t)b * N);
}

// Host side: 48-bit non-zero tag of the next launch (process-wide sequence, random start)
tile_tag_t spu_next_tag();

}  // namespace luvc
