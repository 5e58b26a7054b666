// OIM (paper Section 3.2, Algorithm 1) with candidates beyond the adjacent destinations: every source
// (even position) of a line is compared with every destination (odd position) of the line, or with
// those within a radius.  This is the bipartite matching behind the paper's similarity cost
// O(n_v^1.5 k) (Section 3.1) and the one its appendix runs with a merge number of 2; a destination can
// absorb several sources.
//
// One pass = three launches:
//   oim_line_gram  the source x destination dot products of every line, fp64, as a dense contraction
//                  over the channels on the matrix cores (v_mfma_f64_16x16x4_f64): a wavefront owns a
//                  16 x 16 tile of one line's matrix and walks the channels 32 at a time; the squared
//                  norms of the tokens fall out on the way;
//   oim_decide_wide one workgroup per line: cosines, best destination per source (tie -> lower
//                  position), the m best sources (tie -> lower position), survivor layout, maps;
//   oim_merge_wide one wavefront per surviving token: copy, or size-weighted mean of the destination
//                  and all sources folded into it (ascending position, fp64, one rounding).
#include "common.hpp"
#include "oim.hpp"
#include "oim_wide_tok.hpp"

namespace luvc {

// ------------------------------------------------------------------ dot products of a line: sources x destinations
// Lane l of a wavefront feeds source i = l % 16 and destination i of its tile, channels 8 (l / 16) .. + 7 of
// every block of 32: matrix instruction e of a block contracts channels {e, 8 + e, 16 + e, 24 + e}.
// Result layout of the instruction: lane l, register r holds row 4 r + l / 16 (source), column l % 16.
// The squared norms fall out on the way (every lane sees all channels of its two tokens, a quarter each):
// the tiles of the first column of a line write those of the sources, the first row those of the destinations.
constexpr int kGramSteps = 4;                    // 32-channel blocks fetched before the first is used
template <typename T, bool VECTOR>
__global__ void __launch_bounds__(256)
oim_line_gram(const T* __restrict__ x, double* __restrict__ G /* [B*nlines, n_src, n_dst] */, double* __restrict__ n2 /* [B,H*W] */,
              int H, int W, int D, int axis, int64_t n_tiles, int tiles_s, int tiles_d)
{
    using ch = chan8<T, VECTOR>;
    const int lane = threadIdx.x & 63;
    const uint32_t tile = __builtin_amdgcn_readfirstlane(blockIdx.x * 4u + (threadIdx.x >> 6));   // fewer than 2^31 tiles (host check)
    if (tile >= (uint32_t)n_tiles) return;
    const int len = axis ? W : H, nlines = axis ? H : W;
    const int n_src = (len + 1) / 2, n_dst = len / 2;
    const int td = (int)(tile % (uint32_t)tiles_d), ts = (int)((tile / (uint32_t)tiles_d) % (uint32_t)tiles_s);
    const int64_t bl = tile / ((uint32_t)tiles_d * (uint32_t)tiles_s);  // b * nlines + line
    const int line = (int)((uint32_t)bl % (uint32_t)nlines);
    const int64_t b = (uint32_t)bl / (uint32_t)nlines;
    const int i = lane & 15, g = lane >> 4;
    const int js = ts * 16 + i, jd = td * 16 + i;                         // source / destination index on the line
    const bool has_s = js < n_src, has_d = jd < n_dst;
    const int ps = 2 * js, pd = 2 * jd + 1;                               // their positions
    auto flat = [&](int p) -> int64_t { return axis ? (int64_t)line * W + p : (int64_t)p * W + line; };
    const int64_t t_s = b * H * W + (has_s ? flat(ps) : 0), t_d = b * H * W + (has_d ? flat(pd) : 0);
    const T* tok_s = x + t_s * D;
    const T* tok_d = x + t_d * D;
    // one descriptor over the image for the whole wavefront (a descriptor per token would have to be walked lane by lane)
    const __amdgpu_buffer_rsrc_t rimg = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(x) + b * H * W * D, 0, (int)((int64_t)H * W * D * (int64_t)sizeof(T)), 0x00020000);
    const uint32_t off_s = (uint32_t)((has_s ? flat(ps) : 0) * D * (int64_t)sizeof(T));
    const uint32_t off_d = (uint32_t)((has_d ? flat(pd) : 0) * D * (int64_t)sizeof(T));
    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
    double na = 0.0, nc = 0.0;
    for (int d0 = 0; d0 < D; d0 += 32 * kGramSteps) {
        typename ch::raw_t ra[kGramSteps], rc[kGramSteps];
#pragma unroll
        for (int u = 0; u < kGramSteps; ++u) {                            // past the end of the token: zeros
            ra[u] = ch::fetch(rimg, off_s, tok_s, D, d0 + 32 * u + 8 * g, has_s);
            rc[u] = ch::fetch(rimg, off_d, tok_d, D, d0 + 32 * u + 8 * g, has_d);
        }
#pragma unroll
        for (int u = 0; u < kGramSteps; ++u) {
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
    double* Gl = G + bl * n_src * n_dst;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = ts * 16 + 4 * r + g, col = td * 16 + i;
        if (row < n_src && col < n_dst) Gl[(int64_t)row * n_dst + col] = acc[r];
    }
    na += __shfl_xor(na, 16, kWave); na += __shfl_xor(na, 32, kWave);     // the four channel quarters of token i
    nc += __shfl_xor(nc, 16, kWave); nc += __shfl_xor(nc, 32, kWave);
    if (g == 0) {
        if (td == 0 && has_s) n2[t_s] = na;
        if (ts == 0 && has_d) n2[t_d] = nc;
    }
}

// ------------------------------------------------------------------ per-line decisions and layout
// Dynamic LDS: double score[n_src]; double nrm[len]; int best[n_src]; int slot_of[len]; int scan[blockDim + 1]; uint8 merged[len].
__global__ void __launch_bounds__(256)
oim_decide_wide(const double* __restrict__ n2, const double* __restrict__ G,
                int H, int W, int axis, int m, int radius,
                int32_t* __restrict__ pass_map,   // [B,H*W]   input flat -> output flat slot
                int32_t* __restrict__ anchor,     // [B,Ho*Wo] output slot -> input flat index
                int32_t* __restrict__ src_dest)   // [B*nlines, n_src] position of the destination a merged source goes to, else -1
{
    extern __shared__ unsigned char smem_raw[];
    const int len = axis ? W : H, nlines = axis ? H : W;
    const int n_src = (len + 1) / 2, n_dst = len / 2;
    const int Wo = axis ? W - m : W, Ho = axis ? H : H - m;
    double* score = reinterpret_cast<double*>(smem_raw);
    double* nrm = score + n_src;
    int* best = reinterpret_cast<int*>(nrm + len);
    int* slot_of = best + n_src;
    int* scan = slot_of + len;
    unsigned char* merged = reinterpret_cast<unsigned char*>(scan + blockDim.x + 1);

    const int b = blockIdx.x / nlines, line = blockIdx.x % nlines;
    const int64_t img = (int64_t)b * H * W;
    const int tid = threadIdx.x;
    auto in_flat = [&](int p) -> int { return axis ? line * W + p : p * W + line; };
    auto out_flat = [&](int q) -> int { return axis ? line * Wo + q : q * Wo + line; };
    const double* Gl = G + (int64_t)blockIdx.x * n_src * n_dst;

    for (int p = tid; p < len; p += blockDim.x) {
        const double v = n_dst > 0 ? sqrt(n2[img + in_flat(p)]) : 1.0;   // a line of one token has no norms (and no decisions)
        nrm[p] = v < 1e-12 ? 1e-12 : v;
        merged[p] = 0;
    }
    __syncthreads();
    // one wavefront per source, lanes over the destinations; a lane walks its candidates in ascending position,
    // the lanes are then combined with the same rule: higher cosine wins, equal cosines keep the lower position
    {
        const int lane = tid & 63, wv = tid >> 6, nwv = blockDim.x >> 6;
        for (int j = wv; j < n_src; j += nwv) {
            const int a = 2 * j;
            double bs = -INFINITY;
            int bc = -1;
            for (int k = lane; k < n_dst; k += 64) {
                const int c = 2 * k + 1;
                const int dist = c > a ? c - a : a - c;
                if (radius > 0 && dist > 2 * radius - 1) continue;
                const double s = Gl[(int64_t)j * n_dst + k] / (nrm[a] * nrm[c]);
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
    }
    __syncthreads();
    if (m == n_src) {
        for (int j = tid; j < n_src; j += blockDim.x) merged[2 * j] = best[j] >= 0 ? 1 : 0;
    } else if (m > 0) {
        // rank of source j = number of sources that beat it (higher score, or equal score and lower position)
        for (int j = tid; j < n_src; j += blockDim.x) {
            const double s = score[j];
            int rank = 0;
            for (int i = 0; i < n_src; ++i) {
                const double t = score[i];
                rank += (t > s || (t == s && i < j)) ? 1 : 0;
            }
            if (rank < m && best[j] >= 0) merged[2 * j] = 1;
        }
    }
    __syncthreads();
    // survivors before position p: exclusive scan of (1 - merged) in contiguous per-thread chunks
    const int chunk = (len + blockDim.x - 1) / blockDim.x;
    const int p0 = min(tid * chunk, len), p1 = min(p0 + chunk, len);
    int local = 0;
    for (int p = p0; p < p1; ++p) local += merged[p] ? 0 : 1;
    scan[tid] = local;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int t = 0; t < (int)blockDim.x; ++t) { const int v = scan[t]; scan[t] = run; run += v; }
    }
    __syncthreads();
    int q = scan[tid];
    for (int p = p0; p < p1; ++p) {
        if (merged[p]) continue;
        const int of = out_flat(q);
        slot_of[p] = of;
        anchor[(int64_t)b * Ho * Wo + of] = in_flat(p);
        pass_map[img + in_flat(p)] = of;
        ++q;
    }
    __syncthreads();
    for (int j = tid; j < n_src; j += blockDim.x) {
        const bool mg = merged[2 * j] != 0;
        src_dest[(int64_t)blockIdx.x * n_src + j] = mg ? best[j] : -1;
        if (mg) pass_map[img + in_flat(2 * j)] = slot_of[best[j]];    // a merged source lands in its destination's slot
    }
}

// ------------------------------------------------------------------ weighted merge + compaction
template <typename T, bool VECTOR>
__global__ void __launch_bounds__(256)
oim_merge_wide(const T* __restrict__ x, const int32_t* __restrict__ sizes_in,
               const int32_t* __restrict__ anchor, const int32_t* __restrict__ src_dest,
               const int32_t* __restrict__ kept_prev,      // [B, n_in_per] anchors of the previous passes, or NULL (identity)
               int64_t n_out_tok, int H, int W, int Ho, int Wo, int D, int axis,
               T* __restrict__ x_out, int32_t* __restrict__ sizes_out, int32_t* __restrict__ kept_out)
{
    using tr = io_traits<T>;
    constexpr int V = tr::kVec;
    const int64_t slot = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (slot >= n_out_tok) return;
    const int n_in_per = H * W, n_out_per = Ho * Wo;
    const int64_t b = slot / n_out_per;
    const int p_flat = anchor[slot];
    const int len = axis ? W : H, nlines = axis ? H : W, n_src = (len + 1) / 2;
    const int line = axis ? p_flat / W : p_flat % W, pos = axis ? p_flat % W : p_flat / W;
    const int64_t step = axis ? 1 : W;
    const int64_t t_line0 = b * n_in_per + (axis ? (int64_t)line * W : line);      // token of position 0 on the line
    const int64_t tp = b * n_in_per + p_flat;
    const int32_t* sd = src_dest + (b * nlines + line) * n_src;
    const int sp = sizes_in ? sizes_in[tp] : 1;
    // sources folded into this token (only a destination can have any): their sizes first
    int S = sp;
    bool any = false;
    if (pos & 1) {
        for (int j0 = 0; j0 < n_src; j0 += 64) {
            const int j = j0 + lane;
            const bool hit = j < n_src && sd[j] == pos;
            int sa = hit ? (sizes_in ? sizes_in[t_line0 + (int64_t)(2 * j) * step] : 1) : 0;
            sa = (int)wave_sum((double)sa);                      // exact: sizes sums stay below 2^31
            S += sa;
            any = any || sa > 0;
        }
    }
    const T* xp = x + tp * D;
    T* o = x_out + slot * D;
    if (lane == 0) {
        sizes_out[slot] = S;
        if (kept_out) kept_out[slot] = kept_prev ? kept_prev[b * n_in_per + p_flat] : p_flat;
    }
    if (!any) {                                              // untouched token: bit copy
        if (VECTOR) {
            for (int d = lane * V; d < D; d += 64 * V)
                *reinterpret_cast<typename tr::vec_t*>(o + d) = *reinterpret_cast<const typename tr::vec_t*>(xp + d);
        } else {
            for (int d = lane; d < D; d += 64) o[d] = xp[d];
        }
        return;
    }
    const double dS = (double)S;
    // channels in blocks of 64 * V (VECTOR) or 64: acc = s_p x_p, then every folded source in ascending position
    const int blk = VECTOR ? 64 * V : 64;
    for (int d0 = 0; d0 < D; d0 += blk) {
        double acc[V];
        const int d = d0 + (VECTOR ? lane * V : lane);
        const bool in = d < D;
        if (VECTOR) {
            float f[V];
#pragma unroll
            for (int i = 0; i < V; ++i) f[i] = 0.f;
            if (in) tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(xp + d), f);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = (double)sp * (double)f[i];
        } else {
            acc[0] = in ? (double)sp * (double)tr::load(xp + d) : 0.0;
        }
        for (int j0 = 0; j0 < n_src; j0 += 64) {
            const int j = j0 + lane;
            unsigned long long hits = __ballot(j < n_src && sd[j] == pos);
            while (hits) {
                const int jj = j0 + (int)__builtin_ctzll(hits);
                hits &= hits - 1;
                const int64_t ta = t_line0 + (int64_t)(2 * jj) * step;
                const double sa = (double)(sizes_in ? sizes_in[ta] : 1);
                const T* xa = x + ta * D;
                if (VECTOR) {
                    float f[V];
#pragma unroll
                    for (int i = 0; i < V; ++i) f[i] = 0.f;
                    if (in) tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(xa + d), f);
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[i] += sa * (double)f[i];
                } else if (in) {
                    acc[0] += sa * (double)tr::load(xa + d);
                }
            }
        }
        if (!in) continue;
        if (VECTOR) {
            T r[V];
#pragma unroll
            for (int i = 0; i < V; ++i) tr::store(&r[i], acc[i] / dS);
            *reinterpret_cast<typename tr::vec_t*>(o + d) = *reinterpret_cast<const typename tr::vec_t*>(r);
        } else {
            tr::store(o + d, acc[0] / dS);
        }
    }
}

// ------------------------------------------------------------------ host side
size_t oim_wide_gram_bytes(int B, int H, int W, int axis)
{
    const int len = axis ? W : H, nlines = axis ? H : W;
    return sizeof(double) * (size_t)B * nlines * ((len + 1) / 2) * (len / 2);
}

size_t oim_wide_srcdest_bytes(int B, int H, int W, int axis)
{
    const int len = axis ? W : H, nlines = axis ? H : W;
    return sizeof(int32_t) * (size_t)B * nlines * ((len + 1) / 2);
}

template <typename T>
static luvc_status run_wide_decide(const T* metric, int B, int H, int W, int Dm, int axis, int m, int radius, bool vec,
                                   int32_t* pass_map, const OimScratch& ws, double* G, int32_t* src_dest, hipStream_t st)
{
    const int len = axis ? W : H, nlines = axis ? H : W, n_src = (len + 1) / 2, n_dst = len / 2;
    if (n_dst > 0) {
        const int tiles_s = (n_src + 15) / 16, tiles_d = (n_dst + 15) / 16;
        const int64_t n_tiles = (int64_t)B * nlines * tiles_s * tiles_d;
        if (n_tiles >= ((int64_t)1 << 31)) { set_error("wide matching: too many 16 x 16 tiles in one pass"); return LUVC_ERR_UNSUPPORTED; }
        const unsigned g1 = (unsigned)((n_tiles + 3) / 4);
        if (vec) LUVC_LAUNCH("oim_line_gram", (oim_line_gram<T, true>), dim3(g1), dim3(256), 0, st, metric, G, ws.n2, H, W, Dm, axis, n_tiles, tiles_s, tiles_d);
        else     LUVC_LAUNCH("oim_line_gram", (oim_line_gram<T, false>), dim3(g1), dim3(256), 0, st, metric, G, ws.n2, H, W, Dm, axis, n_tiles, tiles_s, tiles_d);
    }
    const size_t lds = sizeof(double) * (size_t)(n_src + len) + sizeof(int) * (size_t)(n_src + len + 256 + 1) + (size_t)len + 16;
    LUVC_LAUNCH("oim_decide_wide", oim_decide_wide, dim3((unsigned)(B * nlines)), dim3(256), lds, st, ws.n2, G, H, W, axis, m, radius,
                pass_map, ws.anchor, src_dest);
    return check_launch("oim pass (wide matching, decisions)");
}

template <typename T>
static luvc_status run_wide_apply(const T* x, const int32_t* sizes_in, int B, int H, int W, int D, int axis, int m, bool vec,
                                  T* x_out, int32_t* sizes_out, const int32_t* kept_prev, int32_t* kept_out,
                                  const OimScratch& ws, const int32_t* src_dest, hipStream_t st)
{
    const int Ho = axis ? H : H - m, Wo = axis ? W - m : W;
    const int64_t n_out = (int64_t)B * Ho * Wo;
    const unsigned g3 = (unsigned)((n_out * 64 + 255) / 256);
    if (vec) LUVC_LAUNCH("oim_merge_wide", (oim_merge_wide<T, true>), dim3(g3), dim3(256), 0, st, x, sizes_in, ws.anchor, src_dest, kept_prev,
                         n_out, H, W, Ho, Wo, D, axis, x_out, sizes_out, kept_out);
    else     LUVC_LAUNCH("oim_merge_wide", (oim_merge_wide<T, false>), dim3(g3), dim3(256), 0, st, x, sizes_in, ws.anchor, src_dest, kept_prev,
                         n_out, H, W, Ho, Wo, D, axis, x_out, sizes_out, kept_out);
    return check_launch("oim pass (wide matching, merge)");
}

luvc_status oim_wide_decide(const void* metric, int B, int H, int W, int Dm, luvc_dtype dt, int axis, int m, int radius, bool vec,
                            int32_t* pass_map, const OimScratch& ws, double* G, int32_t* src_dest, hipStream_t st)
{
    if (dt == LUVC_F32) return run_wide_decide<float>((const float*)metric, B, H, W, Dm, axis, m, radius, vec, pass_map, ws, G, src_dest, st);
    return run_wide_decide<bf16_t>((const bf16_t*)metric, B, H, W, Dm, axis, m, radius, vec, pass_map, ws, G, src_dest, st);
}

luvc_status oim_wide_apply(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int axis, int m, bool vec,
                           void* x_out, int32_t* sizes_out, const int32_t* kept_prev, int32_t* kept_out,
                           const OimScratch& ws, const int32_t* src_dest, hipStream_t st)
{
    if (dt == LUVC_F32)
        return run_wide_apply<float>((const float*)x, sizes_in, B, H, W, D, axis, m, vec, (float*)x_out, sizes_out, kept_prev, kept_out, ws, src_dest, st);
    return run_wide_apply<bf16_t>((const bf16_t*)x, sizes_in, B, H, W, D, axis, m, vec, (bf16_t*)x_out, sizes_out, kept_prev, kept_out, ws, src_dest, st);
}

luvc_status oim_wide_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt,
                          int axis, int m, int radius, bool vec, void* x_out, int32_t* sizes_out, int32_t* pass_map,
                          const int32_t* kept_prev, int32_t* kept_out,
                          const OimScratch& ws, double* G, int32_t* src_dest, hipStream_t st)
{
    const luvc_status rc = oim_wide_decide(x, B, H, W, D, dt, axis, m, radius, vec, pass_map, ws, G, src_dest, st);
    if (rc != LUVC_OK) return rc;
    return oim_wide_apply(x, sizes_in, B, H, W, D, dt, axis, m, vec, x_out, sizes_out, kept_prev, kept_out, ws, src_dest, st);
}

}  // namespace luvc
