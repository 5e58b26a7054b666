// OIM - Orthogonal Iterative Merger (paper Section 3.2, Algorithm 1): general path.
//
// One pass along one grid axis runs as three kernels:
//   oim_pairdot   one wavefront per token: squared norm and dot product with the next token
//                 on its line, accumulated in fp64 (the decisions below must not depend on
//                 summation order more than fp64 rounding);
//   oim_decide    one workgroup per line: cosine of every source (even position) with its two
//                 adjacent destinations (odd positions), pick, rank the sources of the line,
//                 mark the m best as merged, and lay out the survivors in position order;
//   oim_merge     one wavefront per surviving token: size-weighted mean of the destination
//                 and the sources folded into it, rounded once to the storage type.
// Launchers for fused fast paths live in oim_fast.hip; both share the layout produced here.
#include "common.hpp"
#include "oim.hpp"

namespace luvc {

// ------------------------------------------------------------------ kernel 1: norms and neighbour dots
template <typename T, bool VECTOR>
__global__ void __launch_bounds__(256)
oim_pairdot(const T* __restrict__ x, double* __restrict__ n2, double* __restrict__ dn,
            int64_t n_tok, int H, int W, int D, int axis)
{
    using tr = io_traits<T>;
    const int64_t tok = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (tok >= n_tok) return;
    const int w = (int)(tok % W), h = (int)((tok / W) % H);
    const bool has_next = axis ? (w + 1 < W) : (h + 1 < H);
    const T* a = x + tok * D;
    const T* c = a + (has_next ? (axis ? (int64_t)D : (int64_t)W * D) : 0);
    double sn = 0.0, sd = 0.0;
    if (VECTOR) {
        constexpr int V = tr::kVec;
        for (int d = lane * V; d < D; d += 64 * V) {
            float fa[V], fc[V];
            tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(a + d), fa);
            tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(c + d), fc);
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const double da = (double)fa[i];
                sn = fma(da, da, sn);
                sd = fma(da, (double)fc[i], sd);
            }
        }
    } else {
        for (int d = lane; d < D; d += 64) {
            const double da = (double)tr::load(a + d);
            sn = fma(da, da, sn);
            sd = fma(da, (double)tr::load(c + d), sd);
        }
    }
    sn = wave_sum(sn);
    sd = wave_sum(sd);
    if (lane == 0) {
        n2[tok] = sn;
        dn[tok] = has_next ? sd : 0.0;
    }
}

// ------------------------------------------------------------------ kernel 2: per-line decisions and layout
// Dynamic LDS: double score[n_src]; int best[n_src]; uint8 merged[len]; int scan[blockDim].
__global__ void __launch_bounds__(256)
oim_decide(const double* __restrict__ n2, const double* __restrict__ dn,
           int H, int W, int axis, int m,
           int32_t* __restrict__ pass_map,   // [B,H*W]   input flat -> output flat slot
           int32_t* __restrict__ anchor,     // [B,Ho*Wo] output slot -> input flat index
           int32_t* __restrict__ absorb)     // [B,Ho*Wo] bit0: takes the source before it, bit1: the one after
{
    extern __shared__ unsigned char smem_raw[];
    const int len = axis ? W : H, nlines = axis ? H : W;
    const int n_src = (len + 1) / 2;
    const int Wo = axis ? W - m : W, Ho = axis ? H : H - m;
    double* score = reinterpret_cast<double*>(smem_raw);
    int* best = reinterpret_cast<int*>(score + n_src);
    int* scan = best + n_src;
    unsigned char* merged = reinterpret_cast<unsigned char*>(scan + blockDim.x + 1);

    const int b = blockIdx.x / nlines, line = blockIdx.x % nlines;
    const int64_t img = (int64_t)b * H * W;
    const int tid = threadIdx.x;
    auto in_flat = [&](int p) -> int { return axis ? line * W + p : p * W + line; };
    auto out_flat = [&](int q) -> int { return axis ? line * Wo + q : q * Wo + line; };
    const double eps = 1e-12;

    for (int j = tid; j < n_src; j += blockDim.x) {
        const int a = 2 * j;
        double na = sqrt(n2[img + in_flat(a)]);
        na = na < eps ? eps : na;
        double sl = 0.0, sr = 0.0;
        const bool hl = a >= 1, hr = a + 1 < len;
        if (hl) {
            double nb = sqrt(n2[img + in_flat(a - 1)]);
            nb = nb < eps ? eps : nb;
            sl = dn[img + in_flat(a - 1)] / (na * nb);
        }
        if (hr) {
            double nb = sqrt(n2[img + in_flat(a + 1)]);
            nb = nb < eps ? eps : nb;
            sr = dn[img + in_flat(a)] / (na * nb);
        }
        const bool left = hl && (!hr || !(sr > sl));      // tie -> lower position
        best[j] = (hl || hr) ? (left ? a - 1 : a + 1) : -1;
        score[j] = left ? sl : sr;
    }
    for (int p = tid; p < len; p += blockDim.x) merged[p] = 0;
    __syncthreads();
    if (m == n_src) {
        for (int j = tid; j < n_src; j += blockDim.x) merged[2 * j] = 1;
    } else if (m > 0) {
        // rank of source j = number of sources that beat it (higher score, or equal score and lower position)
        for (int j = tid; j < n_src; j += blockDim.x) {
            const double s = score[j];
            int rank = 0;
            for (int i = 0; i < n_src; ++i) {
                const double t = score[i];
                rank += (t > s || (t == s && i < j)) ? 1 : 0;
            }
            if (rank < m) merged[2 * j] = 1;
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
        int fl = 0;
        if (p & 1) {
            if (merged[p - 1] && best[(p - 1) / 2] == p) fl |= 1;
            if (p + 1 < len && merged[p + 1] && best[(p + 1) / 2] == p) fl |= 2;
        }
        anchor[(int64_t)b * Ho * Wo + of] = in_flat(p);
        absorb[(int64_t)b * Ho * Wo + of] = fl;
        pass_map[img + in_flat(p)] = of;
        // sources folded into p land in the same slot
        if (fl & 1) pass_map[img + in_flat(p - 1)] = of;
        if (fl & 2) pass_map[img + in_flat(p + 1)] = of;
        ++q;
    }
}

// ------------------------------------------------------------------ kernel 3: weighted merge + compaction
template <typename T, bool VECTOR>
__global__ void __launch_bounds__(256)
oim_merge(const T* __restrict__ x, const int32_t* __restrict__ sizes_in,
          const int32_t* __restrict__ anchor, const int32_t* __restrict__ absorb,
          const int32_t* __restrict__ kept_prev,      // [B, n_in_per] anchors of the previous passes, or NULL (identity)
          int64_t n_out_tok, int n_in_per, int n_out_per, int W, int D, int axis,
          T* __restrict__ x_out, int32_t* __restrict__ sizes_out, int32_t* __restrict__ kept_out)
{
    using tr = io_traits<T>;
    const int64_t slot = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (slot >= n_out_tok) return;
    const int64_t b = slot / n_out_per;
    const int p = anchor[slot], fl = absorb[slot];
    const int64_t step = axis ? 1 : W;
    const int64_t tp = b * n_in_per + p;
    const int64_t ta = tp - step, tc = tp + step;        // only dereferenced when flagged
    const int sp = sizes_in ? sizes_in[tp] : 1;
    const int sa = (fl & 1) ? (sizes_in ? sizes_in[ta] : 1) : 0;
    const int sc = (fl & 2) ? (sizes_in ? sizes_in[tc] : 1) : 0;
    const int S = sp + sa + sc;
    const T* xp = x + tp * D;
    const T* xa = x + ((fl & 1) ? ta : tp) * D;
    const T* xc = x + ((fl & 2) ? tc : tp) * D;
    T* o = x_out + slot * D;
    if (lane == 0) {
        sizes_out[slot] = S;
        if (kept_out) kept_out[slot] = kept_prev ? kept_prev[b * n_in_per + p] : p;
    }
    if (fl == 0) {                                       // untouched token: bit copy
        if (VECTOR) {
            constexpr int V = tr::kVec;
            for (int d = lane * V; d < D; d += 64 * V)
                *reinterpret_cast<typename tr::vec_t*>(o + d) = *reinterpret_cast<const typename tr::vec_t*>(xp + d);
        } else {
            for (int d = lane; d < D; d += 64) o[d] = xp[d];
        }
        return;
    }
    const double dsp = sp, dsa = sa, dsc = sc, dS = S;
    if (VECTOR) {
        constexpr int V = tr::kVec;
        for (int d = lane * V; d < D; d += 64 * V) {
            float fp[V], fa[V], fc[V];
            tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(xp + d), fp);
            tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(xa + d), fa);
            tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(xc + d), fc);
            T r[V];
#pragma unroll
            for (int i = 0; i < V; ++i) {
                double acc = dsp * (double)fp[i];
                if (fl & 1) acc += dsa * (double)fa[i];
                if (fl & 2) acc += dsc * (double)fc[i];
                tr::store(&r[i], acc / dS);
            }
            *reinterpret_cast<typename tr::vec_t*>(o + d) = *reinterpret_cast<const typename tr::vec_t*>(r);
        }
    } else {
        for (int d = lane; d < D; d += 64) {
            double acc = dsp * (double)tr::load(xp + d);
            if (fl & 1) acc += dsa * (double)tr::load(xa + d);
            if (fl & 2) acc += dsc * (double)tr::load(xc + d);
            tr::store(o + d, acc / dS);
        }
    }
}

// ------------------------------------------------------------------ map composition over the passes of a call
struct PassMaps {
    const int32_t* map[kMaxPasses];
    int32_t n_in[kMaxPasses];
    int n;
};

__global__ void __launch_bounds__(256)
oim_compose_merged(PassMaps pm, int64_t total, int n_first, int32_t* __restrict__ merged_out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int64_t b = i / n_first;
    int t = (int)(i - b * n_first);
    for (int k = 0; k < pm.n; ++k) t = pm.map[k][b * pm.n_in[k] + t];
    merged_out[i] = t;
}

// ------------------------------------------------------------------ host side
luvc_status oim_norms(const void* x, int B, int H, int W, int D, luvc_dtype dt, int axis, bool vec,
                      const OimScratch& ws, hipStream_t st);

// A pass in two stages, so that the decisions can be taken on one tensor (the metric) and applied to another.
luvc_status oim_general_decide(const void* metric, int B, int H, int W, int Dm, luvc_dtype dt, int axis, int m, bool vec,
                               int32_t* pass_map, const OimScratch& ws, hipStream_t st)
{
    const int len = axis ? W : H, nlines = axis ? H : W, n_src = (len + 1) / 2;
    const luvc_status rc = oim_norms(metric, B, H, W, Dm, dt, axis, vec, ws, st);
    if (rc != LUVC_OK) return rc;
    const size_t lds = sizeof(double) * n_src + sizeof(int) * n_src + sizeof(int) * (256 + 1) + (size_t)len + 16;
    LUVC_LAUNCH("oim_decide", oim_decide, dim3((unsigned)(B * nlines)), dim3(256), lds, st, ws.n2, ws.dn, H, W, axis, m,
                       pass_map, ws.anchor, ws.absorb);
    return check_launch("oim pass (decisions)");
}

template <typename T>
static luvc_status run_apply(const T* x, const int32_t* sizes_in, int B, int H, int W, int D, int axis, int m,
                             bool vec, T* x_out, int32_t* sizes_out, const int32_t* kept_prev, int32_t* kept_out,
                             const OimScratch& ws, hipStream_t st)
{
    const int Ho = axis ? H : H - m, Wo = axis ? W - m : W;
    const int64_t n_out = (int64_t)B * Ho * Wo;
    const unsigned g3 = (unsigned)((n_out * 64 + 255) / 256);
    if (vec) LUVC_LAUNCH("oim_merge", (oim_merge<T, true>), dim3(g3), dim3(256), 0, st, x, sizes_in, ws.anchor, ws.absorb, kept_prev,
                                n_out, H * W, Ho * Wo, W, D, axis, x_out, sizes_out, kept_out);
    else     LUVC_LAUNCH("oim_merge", (oim_merge<T, false>), dim3(g3), dim3(256), 0, st, x, sizes_in, ws.anchor, ws.absorb, kept_prev,
                                n_out, H * W, Ho * Wo, W, D, axis, x_out, sizes_out, kept_out);
    return check_launch("oim pass (merge)");
}

luvc_status oim_general_apply(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int axis, int m,
                              bool vec, void* x_out, int32_t* sizes_out, const int32_t* kept_prev, int32_t* kept_out,
                              const OimScratch& ws, hipStream_t st)
{
    if (dt == LUVC_F32)
        return run_apply<float>((const float*)x, sizes_in, B, H, W, D, axis, m, vec, (float*)x_out, sizes_out, kept_prev, kept_out, ws, st);
    return run_apply<bf16_t>((const bf16_t*)x, sizes_in, B, H, W, D, axis, m, vec, (bf16_t*)x_out, sizes_out, kept_prev, kept_out, ws, st);
}

luvc_status oim_norms(const void* x, int B, int H, int W, int D, luvc_dtype dt, int axis, bool vec,
                      const OimScratch& ws, hipStream_t st)
{
    const int64_t n_tok = (int64_t)B * H * W;
    const unsigned g1 = (unsigned)((n_tok * 64 + 255) / 256);
    if (dt == LUVC_F32) {
        if (vec) LUVC_LAUNCH("oim_pairdot", (oim_pairdot<float, true>), dim3(g1), dim3(256), 0, st, (const float*)x, ws.n2, ws.dn, n_tok, H, W, D, axis);
        else     LUVC_LAUNCH("oim_pairdot", (oim_pairdot<float, false>), dim3(g1), dim3(256), 0, st, (const float*)x, ws.n2, ws.dn, n_tok, H, W, D, axis);
    } else {
        if (vec) LUVC_LAUNCH("oim_pairdot", (oim_pairdot<bf16_t, true>), dim3(g1), dim3(256), 0, st, (const bf16_t*)x, ws.n2, ws.dn, n_tok, H, W, D, axis);
        else     LUVC_LAUNCH("oim_pairdot", (oim_pairdot<bf16_t, false>), dim3(g1), dim3(256), 0, st, (const bf16_t*)x, ws.n2, ws.dn, n_tok, H, W, D, axis);
    }
    return check_launch("oim norms");
}

luvc_status oim_general_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt,
                             int axis, int m, bool vec, void* x_out, int32_t* sizes_out, int32_t* pass_map,
                             const int32_t* kept_prev, int32_t* kept_out,
                             const OimScratch& ws, hipStream_t st)
{
    const luvc_status rc = oim_general_decide(x, B, H, W, D, dt, axis, m, vec, pass_map, ws, st);
    if (rc != LUVC_OK) return rc;
    return oim_general_apply(x, sizes_in, B, H, W, D, dt, axis, m, vec, x_out, sizes_out, kept_prev, kept_out, ws, st);
}

luvc_status oim_compose(const int32_t* const* maps, const int32_t* n_in, int n, int B, int n_first,
                        int32_t* merged_out, hipStream_t st)
{
    PassMaps pm;
    pm.n = n;
    for (int i = 0; i < n; ++i) { pm.map[i] = maps[i]; pm.n_in[i] = n_in[i]; }
    const int64_t total = (int64_t)B * n_first;
    LUVC_LAUNCH("oim_compose_merged", oim_compose_merged, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, pm, total, n_first,
                       merged_out);
    return check_launch("oim compose");
}

}  // namespace luvc
