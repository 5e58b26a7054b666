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
// Counters: 1 + n_groups per sample, zero before the launch; the workgroup that finds a counter complete
// wraps it back to zero (atomic increment with wrap), so they are zero again afterwards.
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

// Called by all THREADS threads of the workgroup of (sample b, tile) after they have written the tile's
// energies to partial[(b * n_tiles + tile) * N + n] with tile_store().  `flag` is a __shared__ word.
// W = 4 needs N % 4 == 0 (and the 256-byte alignment the workspace has anyway).  A sample of at most
// kTileGroup tiles has no group level: its last workgroup adds the tiles directly.
template <int THREADS, int W>
__device__ __forceinline__ void tiles_to_scores(float* __restrict__ partial /* [B, n_tiles, N] */,
                                                float* __restrict__ gpartial /* [B, n_groups, N] */,
                                                unsigned int* __restrict__ done /* [B][1 + n_groups] */,
                                                float* __restrict__ scores /* [B, N] */,
                                                int b, int tile, int n_tiles, int N, int* flag)
{
    const int tid = threadIdx.x;
    const int n_groups = (n_tiles + kTileGroup - 1) / kTileGroup;
    unsigned int* cnt = done + (int64_t)b * (n_groups + 1);
    // scalar accesses (W = 1) leave room for 64 loads in flight per thread: up to 64 tiles are added in one level
    const bool two_level = n_groups > 1 && !(W == 1 && n_tiles <= 64);
    if (two_level) {
        const int grp = tile / kTileGroup, t_first = grp * kTileGroup;
        const int t_cnt = n_tiles - t_first < kTileGroup ? n_tiles - t_first : kTileGroup;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's stores have been performed
        __syncthreads();
        if (tid == 0) *flag = atomicInc(cnt + 1 + grp, (unsigned)t_cnt - 1u) == (unsigned)t_cnt - 1u;
        __syncthreads();
        if (!*flag) return;
        tile_rows_sum<THREADS, W, false>(partial + ((int64_t)b * n_tiles + t_first) * N, t_cnt, N,
                                         gpartial + ((int64_t)b * n_groups + grp) * N);
    }
    const int last_cnt = two_level ? n_groups : n_tiles;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                             // also: every thread has read the flag
    if (tid == 0) *flag = atomicInc(cnt, (unsigned)last_cnt - 1u) == (unsigned)last_cnt - 1u;
    __syncthreads();
    if (!*flag) return;
    if (two_level)
        tile_rows_sum<THREADS, W, true>(gpartial + (int64_t)b * n_groups * N, last_cnt, N, scores + (int64_t)b * N);
    else
        tile_rows_sum<THREADS, W, true, (W == 1 ? 64 : kTileGroup)>(partial + (int64_t)b * n_tiles * N, last_cnt, N, scores + (int64_t)b * N);
}

// Host side: counters for one launch over `samples` samples with `n_tiles` tiles each (device pointer into
// a static array; nullptr with an error set if the launch needs more than a slot holds).
constexpr int kSlotCounters = 16384;
unsigned int* spu_take_counters();
inline int spu_tile_groups(int n_tiles) { return (n_tiles + kTileGroup - 1) / kTileGroup; }

}  // namespace luvc
