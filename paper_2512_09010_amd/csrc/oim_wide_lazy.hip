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
// oim_wide_line, one workgroup per line (lines of at most 128 tokens):
//   1. the source x destination dot products of the line in fp64 on the matrix cores (v_mfma_f64_16x16x4_f64), a
//      wavefront per 16 x 16 tile, results and squared norms to LDS;
//   2. cosines, best destination per source (tie -> lower position), the m best sources (tie -> lower position);
//   3. survivor layout by ballot counts, ids / sizes / anchors / maps of the next grid;
//   4. size-weighted mean of every destination that absorbs sources (destination first, then the sources in
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

template <typename T>
__device__ __forceinline__ const T* row_of(const T* x, const T* ov, int64_t b, int id, const LazyGeom& g)
{
    return id < g.n0 ? x + (b * g.n0 + id) * g.D : ov + (b * g.cap + (id - g.n0)) * g.D;
}

}  // namespace

constexpr int kLazySteps = 4;                    // 32-channel blocks fetched before the first is used
template <typename T>
__global__ void __launch_bounds__(256)
oim_wide_line(const T* __restrict__ x, T* ov, const int32_t* __restrict__ idx_in /* null: identity */,
              const int32_t* __restrict__ sizes_in /* null: ones */, const int32_t* __restrict__ kept_in /* null: identity */,
              LazyGeom g, int32_t* __restrict__ idx_out, int32_t* __restrict__ sizes_out, int32_t* __restrict__ kept_out /* or null */,
              int32_t* __restrict__ pass_map /* or null */)
{
    using ch = chan8<T, true>;
    using tr = io_traits<T>;
    constexpr int V = tr::kVec;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int len = g.axis ? g.w : g.h, nlines = g.axis ? g.h : g.w;
    const int n_src = (len + 1) / 2, n_dst = len / 2;
    const int Wo = g.axis ? g.w - g.m : g.w, Ho = g.axis ? g.h : g.h - g.m;
    double* G = reinterpret_cast<double*>(smem_raw);     // [n_src][n_dst]
    double* nrm = G + n_src * n_dst;                     // [len] squared norms, then max(norm, 1e-12)
    double* score = nrm + len;                           // [n_src]
    int* rid = reinterpret_cast<int*>(score + n_src);    // [len] row id of the token at position p
    int* sz = rid + len;                                 // [len] its size
    int* snew = sz + len;                                // [len] its size after the pass (survivors)
    int* best = snew + len;                              // [n_src]
    int* slot_of = best + n_src;                         // [len]
    int* ovk = slot_of + len;                            // [len] destination that absorbs sources: which overlay row of the line, else -1
    int* dlist = ovk + len;                              // [n_dst] those destinations, ascending
    int* tot = dlist + len;                              // [4] counts handed between the wavefronts
    unsigned char* merged = reinterpret_cast<unsigned char*>(tot + 4);   // [len]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x / nlines;
    const int line = blockIdx.x % nlines;
    const int64_t img = b * g.h * g.w, img_out = b * Ho * Wo;
    auto in_flat = [&](int p) -> int { return g.axis ? line * g.w + p : p * g.w + line; };
    auto out_flat = [&](int q) -> int { return g.axis ? line * Wo + q : q * Wo + line; };

    for (int p = tid; p < len; p += blockDim.x) {
        const int f = in_flat(p);
        rid[p] = idx_in ? idx_in[img + f] : f;
        sz[p] = sizes_in ? sizes_in[img + f] : 1;
        merged[p] = 0;
        ovk[p] = -1;
        nrm[p] = 1.0;                                    // a line of one token has no products and no decisions
    }
    __syncthreads();

    // ------------------------------------------------------------------ 1. dot products, sources x destinations
    // Lane l of a wavefront feeds source i = l % 16 and destination i of its tile, channels 8 (l / 16) .. + 7 of every
    // block of 32: matrix instruction e of a block contracts channels {e, 8 + e, 16 + e, 24 + e}.  Result layout:
    // lane l, register r holds row 4 r + l / 16 (source), column l % 16.  The squared norms fall out on the way.
    {
        const int tiles_s = (n_src + 15) / 16, tiles_d = (n_dst + 15) / 16;
        const int i = lane & 15, q4 = lane >> 4;
        for (int t = wave; t < tiles_s * tiles_d; t += 4) {
            const int ts = t / tiles_d, td = t % tiles_d;
            const int js = ts * 16 + i, jd = td * 16 + i;
            const bool has_s = js < n_src, has_d = jd < n_dst;
            const T* tok_s = row_of<T>(x, ov, b, has_s ? rid[2 * js] : rid[0], g);
            const T* tok_d = row_of<T>(x, ov, b, has_d ? rid[2 * jd + 1] : rid[0], g);
            f64x4 acc = {0.0, 0.0, 0.0, 0.0};
            double na = 0.0, nc = 0.0;
            for (int d0 = 0; d0 < g.D; d0 += 32 * kLazySteps) {
                typename ch::raw_t ra[kLazySteps], rc[kLazySteps];
#pragma unroll
                for (int u = 0; u < kLazySteps; ++u) {                    // past the end of the token: zeros
                    ra[u] = ch::fetch_ptr(tok_s, g.D, d0 + 32 * u + 8 * q4, has_s);
                    rc[u] = ch::fetch_ptr(tok_d, g.D, d0 + 32 * u + 8 * q4, has_d);
                }
#pragma unroll
                for (int u = 0; u < kLazySteps; ++u) {
                    double a[8], c[8];
                    ch::widen(ra[u], a);
                    ch::widen(rc[u], c);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[e], c[e], acc, 0, 0, 0);
                        na = fma(a[e], a[e], na);
                        nc = fma(c[e], c[e], nc);
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = ts * 16 + 4 * r + q4, col = td * 16 + i;
                if (row < n_src && col < n_dst) G[row * n_dst + col] = acc[r];
            }
            na += __shfl_xor(na, 16, kWave); na += __shfl_xor(na, 32, kWave);     // the four channel quarters of token i
            nc += __shfl_xor(nc, 16, kWave); nc += __shfl_xor(nc, 32, kWave);
            if (q4 == 0) {
                if (td == 0 && has_s) nrm[2 * js] = na;
                if (ts == 0 && has_d) nrm[2 * jd + 1] = nc;
            }
        }
    }
    __syncthreads();
    if (n_dst > 0)
        for (int p = tid; p < len; p += blockDim.x) {
            const double v = sqrt(nrm[p]);
            nrm[p] = v < 1e-12 ? 1e-12 : v;
        }
    __syncthreads();

    // ------------------------------------------------------------------ 2. decisions
    // one wavefront per source, lanes over the destinations; a lane walks its candidates in ascending position,
    // the lanes are then combined with the same rule: higher cosine wins, equal cosines keep the lower position
    for (int j = wave; j < n_src; j += 4) {
        const int a = 2 * j;
        double bs = -INFINITY;
        int bc = -1;
        for (int k = lane; k < n_dst; k += 64) {
            const int c = 2 * k + 1;
            const int dist = c > a ? c - a : a - c;
            if (g.radius > 0 && dist > 2 * g.radius - 1) continue;
            const double s = G[j * n_dst + k] / (nrm[a] * nrm[c]);
            if (bc < 0 || s > bs) { bs = s; bc = c; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double os = __shfl_xor(bs, o, kWave);
            const int oc = __shfl_xor(bc, o, kWave);
            if (oc >= 0 && (bc < 0 || os > bs || (os == bs && oc < bc))) { bs = os; bc = oc; }
        }
        if (lane == 0) { best[j] = bc; score[j] = bs; }
    }
    __syncthreads();
    if (g.m == n_src) {
        for (int j = tid; j < n_src; j += blockDim.x) merged[2 * j] = best[j] >= 0 ? 1 : 0;
    } else if (g.m > 0) {
        // rank of source j = number of sources that beat it (higher score, or equal score and lower position)
        for (int j = tid; j < n_src; j += blockDim.x) {
            const double s = score[j];
            int rank = 0;
            for (int i = 0; i < n_src; ++i) {
                const double t = score[i];
                rank += (t > s || (t == s && i < j)) ? 1 : 0;
            }
            if (rank < g.m && best[j] >= 0) merged[2 * j] = 1;
        }
    }
    __syncthreads();

    // ------------------------------------------------------------------ 3. layout of the next grid
    // thread p looks at position p (len <= 128: wavefronts 0 and 1); counts before a position by ballot
    {
        const int p = tid;
        const bool alive = p < len && !merged[p];
        int S = p < len ? sz[p] : 0;
        bool absorbs = false;
        if (alive && (p & 1)) {
            for (int j = 0; j < n_src; ++j)
                if (merged[2 * j] && best[j] == p) { S += sz[2 * j]; absorbs = true; }
        }
        const unsigned long long below = (1ull << lane) - 1ull;
        const unsigned long long bal_a = __ballot(alive), bal_d = __ballot(absorbs);
        int q = __popcll(bal_a & below), k = __popcll(bal_d & below);
        if (wave == 0 && lane == 0) { tot[0] = __popcll(bal_a); tot[1] = __popcll(bal_d); }
        if (wave == 1 && lane == 0) tot[2] = __popcll(bal_d);
        __syncthreads();
        if (wave == 1) { q += tot[0]; k += tot[1]; }
        if (alive) {
            const int of = out_flat(q), f = in_flat(p);
            slot_of[p] = of;
            snew[p] = S;
            if (absorbs) { ovk[p] = k; dlist[k] = p; }
            idx_out[img_out + of] = absorbs ? g.n0 + g.ov_base + line * g.per_line + k : rid[p];
            sizes_out[img_out + of] = S;
            if (kept_out) kept_out[img_out + of] = kept_in ? kept_in[img + f] : f;
            if (pass_map) pass_map[img + f] = of;
        }
    }
    __syncthreads();
    if (pass_map)
        for (int j = tid; j < n_src; j += blockDim.x)
            if (merged[2 * j]) pass_map[img + in_flat(2 * j)] = slot_of[best[j]];    // a merged source lands in its destination's slot

    // ------------------------------------------------------------------ 4. the merged destinations
    const int n_abs = tot[1] + tot[2];
    for (int k = wave; k < n_abs; k += 4) {
        const int c = dlist[k];
        const T* xp = row_of<T>(x, ov, b, rid[c], g);
        T* o = ov + (b * g.cap + g.ov_base + line * g.per_line + k) * g.D;
        const double sp = (double)sz[c], dS = (double)snew[c];
        for (int d0 = 0; d0 < g.D; d0 += 64 * V) {
            const int d = d0 + lane * V;
            const bool in = d < g.D;
            double acc[V];
            float f[V];
#pragma unroll
            for (int i = 0; i < V; ++i) f[i] = 0.f;
            if (in) tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(xp + d), f);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = sp * (double)f[i];
            for (int j = 0; j < n_src; ++j) {
                if (!merged[2 * j] || best[j] != c) continue;                // wave-uniform
                const double sa = (double)sz[2 * j];
                const T* xa = row_of<T>(x, ov, b, rid[2 * j], g);
#pragma unroll
                for (int i = 0; i < V; ++i) f[i] = 0.f;
                if (in) tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(xa + d), f);
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] += sa * (double)f[i];
            }
            if (!in) continue;
            T r[V];
#pragma unroll
            for (int i = 0; i < V; ++i) tr::store(&r[i], acc[i] / dS);
            *reinterpret_cast<typename tr::vec_t*>(o + d) = *reinterpret_cast<const typename tr::vec_t*>(r);
        }
    }
}

// ------------------------------------------------------------------ the rows behind the final ids
typedef unsigned int lazy_u32x4 __attribute__((__vector_size__(16)));
__global__ void __launch_bounds__(256)
oim_wide_gather(const unsigned char* __restrict__ x, const unsigned char* __restrict__ ov, const int32_t* __restrict__ idx,
                int n0, int cap, int n_out_per, int row_bytes, int64_t n_rows, unsigned char* __restrict__ x_out)
{
    const int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const int64_t b = row / n_out_per;
    int id = idx[row];
    id = id < 0 ? 0 : (id >= n0 + cap ? n0 + cap - 1 : id);            // ids come from oim_wide_line; stay in bounds regardless
    const unsigned char* in = id < n0 ? x + (b * n0 + id) * (int64_t)row_bytes : ov + (b * cap + (id - n0)) * (int64_t)row_bytes;
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

// ------------------------------------------------------------------ host side
int oim_wide_lazy_rows(int h, int w, int axis, int m)
{
    const int len = axis ? w : h, nlines = axis ? h : w, n_dst = len / 2;
    return nlines * (m < n_dst ? m : n_dst);
}

template <typename T>
static luvc_status run_lazy_pass(const T* x, T* ov, const int32_t* idx_in, const int32_t* sizes_in, const int32_t* kept_in,
                                 int B, int n0, int h, int w, int D, int axis, int m, int radius, int cap, int ov_base,
                                 int32_t* idx_out, int32_t* sizes_out, int32_t* kept_out, int32_t* pass_map, hipStream_t st)
{
    const int len = axis ? w : h, nlines = axis ? h : w, n_src = (len + 1) / 2, n_dst = len / 2;
    if (len > kLazyMaxLen) { set_error("wide matching (one launch per pass): line of %d tokens", len); return LUVC_ERR_UNSUPPORTED; }
    LazyGeom g;
    g.n0 = n0; g.h = h; g.w = w; g.D = D; g.axis = axis; g.m = m; g.radius = radius; g.cap = cap; g.ov_base = ov_base;
    g.per_line = m < n_dst ? m : n_dst;
    const size_t lds = sizeof(double) * ((size_t)n_src * n_dst + len + n_src) + sizeof(int) * ((size_t)7 * len + n_src + 4) + (size_t)len + 16;
    LUVC_LAUNCH("oim_wide_line", (oim_wide_line<T>), dim3((unsigned)(B * nlines)), dim3(256), lds, st, x, ov, idx_in, sizes_in, kept_in, g,
                idx_out, sizes_out, kept_out, pass_map);
    return check_launch("oim pass (wide matching, one launch)");
}

luvc_status oim_wide_lazy_pass(const void* x, void* ov, const int32_t* idx_in, const int32_t* sizes_in, const int32_t* kept_in,
                               int B, int n0, int h, int w, int D, luvc_dtype dt, int axis, int m, int radius, int cap, int ov_base,
                               int32_t* idx_out, int32_t* sizes_out, int32_t* kept_out, int32_t* pass_map, hipStream_t st)
{
    if (dt == LUVC_F32)
        return run_lazy_pass<float>((const float*)x, (float*)ov, idx_in, sizes_in, kept_in, B, n0, h, w, D, axis, m, radius, cap, ov_base,
                                    idx_out, sizes_out, kept_out, pass_map, st);
    return run_lazy_pass<bf16_t>((const bf16_t*)x, (bf16_t*)ov, idx_in, sizes_in, kept_in, B, n0, h, w, D, axis, m, radius, cap, ov_base,
                                 idx_out, sizes_out, kept_out, pass_map, st);
}

luvc_status oim_wide_lazy_gather(const void* x, const void* ov, const int32_t* idx, int B, int n0, int cap, int n_out_per, int D,
                                 luvc_dtype dt, void* x_out, hipStream_t st)
{
    const int64_t rows = (int64_t)B * n_out_per;
    const int row_bytes = D * (dt == LUVC_F32 ? 4 : 2);
    const unsigned grid = (unsigned)((rows * 64 + 255) / 256);
    LUVC_LAUNCH("oim_wide_gather", oim_wide_gather, dim3(grid), dim3(256), 0, st, (const unsigned char*)x, (const unsigned char*)ov, idx,
                n0, cap, n_out_per, row_bytes, rows, (unsigned char*)x_out);
    return check_launch("oim wide matching, output rows");
}

}  // namespace luvc
