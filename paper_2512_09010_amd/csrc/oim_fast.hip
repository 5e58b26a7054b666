// OIM (paper Section 3.2) - fused single-launch pass for the schedules that merge EVERY source
// of a line (m = ceil(len/2), the halving used by the benchmark configurations).
//
// With every source merged the survivors are exactly the destinations (odd positions), so output
// slot j of a line is destination 2j+1 and no per-line ranking is needed.  One wavefront produces
// one output token: it keeps source a = 2j, destination b = 2j+1 and the next source c = 2j+2 in
// registers (each token is read once per use, 16 bytes per lane per access), accumulates the
// squared norms and the two neighbour dot products, trades those four scalars with the
// neighbouring wavefronts of its workgroup through LDS, decides where a and c go, and writes the
// size-weighted mean.  The waves at the two ends of a workgroup's run of slots evaluate the one
// or two halo tokens they need themselves, with the same routine, so the decision about a source
// is bit-identical in both wavefronts that look at it.
//
// Decisions are fp64 decisions, reached in two steps.  A screening sweep forms the cosines in fp32
// (packed bf16 dot instructions) with a rigorous error bound tau; a source whose two cosines differ
// by more than tau goes where the fp32 values say - the fp64 values cannot say otherwise.  If any
// decision of the workgroup is closer than tau (or an exact tie), every wavefront of the workgroup
// repeats the sweep in fp64 and the fp64 cosines decide.  The verdict "closer than tau" is a
// function of the screening values of that source alone, which are the same bits in every
// wavefront and workgroup that looks at it, so neighbours always agree on a shared source.
#include <cstdlib>

#include "common.hpp"
#include "oim.hpp"
#include "oim_tok.hpp"

namespace luvc {


template <typename T, int NCH>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(NCH <= 3 ? 4 : 2)))
oim_halve(const T* __restrict__ x, const int32_t* __restrict__ sizes_in, int H, int W, int D, int axis,
          int tiles_per_line, int slots_per_tile,
          const int32_t* __restrict__ kept_prev, T* __restrict__ x_out, int32_t* __restrict__ sizes_out,
          int32_t* __restrict__ pass_map, int32_t* __restrict__ kept_out)
{
    using tr = io_traits<T>;
    constexpr int V = tr::kVec;
    __shared__ Scal sc[8];
    __shared__ double halo[5];                    // left: 1/|l|, l.a0 ; right: 1/|c|, 1/|r|, c.r
    __shared__ ScalF scf[8];                      // the same exchange for the fp32 screening sweep
    __shared__ float halof[6];                    // ... plus [5]: right-hand source could not be screened
    __shared__ int redo;                          // some decision of this workgroup is too close for fp32

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int len = axis ? W : H, nlines = axis ? H : W;
    const int nd = len >> 1;                      // destinations = output slots per line
    const int Wo = axis ? nd : W;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);   // tiles of a line stay on one XCD
    const int tile = item % tiles_per_line;
    const int line = (item / tiles_per_line) % nlines;
    const int b = item / (tiles_per_line * nlines);
    const int j0 = tile * slots_per_tile;
    const int nslot = min(slots_per_tile, nd - j0);        // live waves of this workgroup
    const int j = j0 + w;
    const bool live = w < nslot;
    const int64_t step = axis ? 1 : W;                     // tokens between neighbours on the line
    const int64_t img = (int64_t)b * H * W;
    const int64_t line0 = img + (axis ? (int64_t)line * W : line);    // token index of position 0
    auto tok_ptr = [&](int pos) { return x + (line0 + pos * step) * D; };

    Tok<T, NCH> A, Bt, C, Hx;
    const int pa = 2 * j, pb = 2 * j + 1, pc = 2 * j + 2;
    const bool has_c = live && pc < len;
    // the end waves of the workgroup also need one token beyond its run of slots
    const bool need_l = live && (w == 0) && pa >= 1;
    const bool need_r = live && (w == nslot - 1) && has_c;  // c's own right neighbour, if any, decides with us
    const bool has_r = need_r && pc + 1 < len;
    // error bound of a screening cosine: (NCH*V + 8) roundings of at most 2^-23 each on the dot product,
    // the same on each norm, doubled for safety; two cosines are compared
    const float tau = 16.0f * (float)(NCH * V + 8) * 5.9604645e-8f;
    if (threadIdx.x == 0) redo = 0;
    if (live) {
        load_tok<T, NCH>(A, tok_ptr(pa), D, lane);
        load_tok<T, NCH>(Bt, tok_ptr(pb), D, lane);
        load_tok<T, NCH>(C, tok_ptr(has_c ? pc : pb), D, lane, has_c);
        load_tok<T, NCH>(Hx, tok_ptr(need_l ? pa - 1 : (has_r ? pc + 1 : pb)), D, lane, need_l || has_r);
        float na = 0.f, nb = 0.f, dab = 0.f, dbc = 0.f, ncc = 0.f, nhh = 0.f, dh = 0.f;
        if (need_l) sweep32<T, NCH, true, true>(A, Bt, C, Hx, na, nb, dab, dbc, ncc, nhh, dh);
        else if (need_r) sweep32<T, NCH, true, false>(A, Bt, C, Hx, na, nb, dab, dbc, ncc, nhh, dh);
        else sweep32<T, NCH, false, false>(A, Bt, C, Hx, na, nb, dab, dbc, ncc, nhh, dh);
        ScalF f;
        f.ia = inv_norm32(wave_sum32(na)); f.ib = inv_norm32(wave_sum32(nb));
        f.dab = wave_sum32(dab); f.dbc = wave_sum32(dbc);
        if (lane == 0) scf[w] = f;
        if (need_l) {
            const float il = inv_norm32(wave_sum32(nhh)), dl = wave_sum32(dh);
            if (lane == 0) { halof[0] = il; halof[1] = dl; }
        }
        if (need_r) {
            const float ic = inv_norm32(wave_sum32(ncc));
            // a one-wave workgroup holds its left halo in Hx: its right-hand source is then sent to the fp64 sweep
            const bool unknown = need_l && has_r;
            const float ir = (has_r && !unknown) ? inv_norm32(wave_sum32(nhh)) : 0.f;
            const float dcr = (has_r && !unknown) ? wave_sum32(dh) : 0.f;
            if (lane == 0) { halof[2] = ic; halof[3] = ir; halof[4] = dcr; halof[5] = unknown ? 1.f : 0.f; }
        }
    }
    __syncthreads();
    int va = -1, vc = 0;                          // screening verdicts for a and c (see screen_source)
    if (live) {
        const ScalF me = scf[w];
        float l_ib = 0.f, l_dbc = 0.f;
        if (pa >= 1) {
            if (w > 0) { l_ib = scf[w - 1].ib; l_dbc = scf[w - 1].dbc; }
            else { l_ib = halof[0]; l_dbc = halof[1]; }
        }
        va = screen_source(pa >= 1, true, me.ia, l_dbc, l_ib, me.dab, me.ib, tau);
        if (has_c) {
            if (w + 1 < nslot) vc = screen_source(true, pc + 1 < len, scf[w + 1].ia, me.dbc, me.ib, scf[w + 1].dab, scf[w + 1].ib, tau);
            else vc = halof[5] != 0.f ? 0 : screen_source(true, pc + 1 < len, halof[2], me.dbc, me.ib, halof[4], halof[3], tau);
        } else {
            vc = -1;
        }
        if ((va == 0 || vc == 0) && lane == 0) redo = 1;
    }
    __syncthreads();
    bool a_left = va > 0, c_left = vc > 0;
    if (redo) {                                   // uniform over the workgroup: every wave repeats the sweep in fp64
        Scal me{0, 0, 0, 0};
        if (live) {
            double nl = 0.0, dl = 0.0, nc = 0.0, nr = 0.0, dcr = 0.0;
            // every accumulator sees its terms in the same (chunk, element) order in whichever wavefront
            // evaluates it, so a dot product shared by two wavefronts has the same bits in both
            if (need_l) {
                sweep<T, NCH, true, true>(A, Bt, C, Hx, me, nc, nl, dl);
                if (has_r) {                                    // single-wave workgroup: the other end as well
                    load_tok<T, NCH>(Hx, tok_ptr(pc + 1), D, lane);
                    double unused = 0.0;
                    Scal tmp{0, 0, 0, 0};
                    sweep<T, NCH, true, false>(A, Bt, C, Hx, tmp, unused, nr, dcr);
                }
            } else if (need_r) {
                sweep<T, NCH, true, false>(A, Bt, C, Hx, me, nc, nr, dcr);
            } else {
                double u0 = 0.0, u1 = 0.0, u2 = 0.0;
                sweep<T, NCH, false, false>(A, Bt, C, Hx, me, u0, u1, u2);
            }
            me.na = inv_norm(wave_sum(me.na)); me.nb = inv_norm(wave_sum(me.nb)); me.dab = wave_sum(me.dab);
            if (has_c) me.dbc = wave_sum(me.dbc);
            if (need_l) {
                nl = inv_norm(wave_sum(nl)); dl = wave_sum(dl);
                if (lane == 0) { halo[0] = nl; halo[1] = dl; }
            }
            if (need_r) {
                nc = inv_norm(wave_sum(nc));
                if (has_r) { nr = inv_norm(wave_sum(nr)); dcr = wave_sum(dcr); }
                if (lane == 0) { halo[2] = nc; halo[3] = nr; halo[4] = dcr; }
            }
            if (lane == 0) sc[w] = me;
        }
        __syncthreads();
        if (live) {
            // ---- source a = 2j: right (into b) unless its left destination 2j-1 is at least as similar
            double l_nb = 0.0, l_dbc = 0.0;               // 1/|2j-1| and <2j-1, 2j>
            if (pa >= 1) {
                if (w > 0) { l_nb = sc[w - 1].nb; l_dbc = sc[w - 1].dbc; }
                else { l_nb = halo[0]; l_dbc = halo[1]; }
            }
            a_left = source_goes_left(pa >= 1, true, me.na, l_dbc, l_nb, me.dab, me.nb);
            // ---- source c = 2j+2: left (into b) unless its right destination 2j+3 is strictly more similar
            c_left = false;
            if (has_c) {
                double nc, nr, dcr;
                if (w + 1 < nslot) { nc = sc[w + 1].na; nr = sc[w + 1].nb; dcr = sc[w + 1].dab; }
                else { nc = halo[2]; nr = halo[3]; dcr = halo[4]; }
                c_left = source_goes_left(true, pc + 1 < len, nc, me.dbc, me.nb, dcr, nr);
            }
        }
    }
    if (!live) return;
    forget<T, NCH>(A);
    forget<T, NCH>(Bt);
    forget<T, NCH>(C);
    const bool take_a = !a_left, take_c = c_left;

    const int64_t ta = line0 + pa * step, tb = line0 + pb * step, tc = line0 + pc * step;
    const int sb = sizes_in ? sizes_in[tb] : 1;
    const int sa = take_a ? (sizes_in ? sizes_in[ta] : 1) : 0;
    const int scz = take_c ? (sizes_in ? sizes_in[tc] : 1) : 0;
    const int S = sb + sa + scz;
    const int64_t n_out_per = (int64_t)(axis ? H : nd) * Wo;
    const int out_in_img = axis ? line * Wo + j : j * Wo + line;
    const int64_t slot = b * n_out_per + out_in_img;
    if (lane == 0) {
        sizes_out[slot] = S;
        const int p_in = (int)(tb - img);
        if (kept_out) kept_out[slot] = kept_prev ? kept_prev[img + p_in] : p_in;
        // a lands here or in the previous slot of the line; the last source of an odd line has no
        // slot of its own and always folds into the last destination
        const int prev_slot = axis ? out_in_img - 1 : out_in_img - Wo;
        pass_map[tb] = out_in_img;
        pass_map[ta] = take_a ? out_in_img : prev_slot;
        if (has_c && pc + 1 >= len) pass_map[tc] = out_in_img;
    }
    T* o = x_out + slot * D;
    if (!take_a && !take_c) {                     // nothing absorbed: bit copy
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int d = (i * 64 + lane) * V;
            if (d < D) *reinterpret_cast<typename tr::vec_t*>(o + d) = Bt.v[i];
        }
        return;
    }
    // size-weighted mean in fp64, terms in position order b, a, c (sizes of absent terms are 0).  The
    // quotient is formed with the reciprocal and one residual correction: exact whenever acc / S is
    // representable, which covers every rounding boundary of the storage types.
    const double dsb = sb, dsa = sa, dsc = scz, dS = S, rS = 1.0 / dS;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int d = (i * 64 + lane) * V;
        T r[V];
#pragma unroll
        for (int e = 0; e < V; ++e) {
            double acc = dsb * (double)elem<T>(Bt.v[i], e);
            acc = fma(dsa, (double)elem<T>(A.v[i], e), acc);
            acc = fma(dsc, (double)elem<T>(C.v[i], e), acc);
            double q = acc * rS;
            q = fma(fma(-q, dS, acc), rS, q);
            tr::store(&r[e], q);
        }
        if (d < D) *reinterpret_cast<typename tr::vec_t*>(o + d) = *reinterpret_cast<const typename tr::vec_t*>(r);
    }
}

template <typename T, int NCH>
static void launch_halve(const T* x, const int32_t* sizes_in, int B, int H, int W, int D, int axis,
                         const int32_t* kept_prev, T* x_out, int32_t* sizes_out, int32_t* pass_map, int32_t* kept_out,
                         hipStream_t st)
{
    const int len = axis ? W : H, nlines = axis ? H : W, nd = len / 2;
    constexpr int cap = 4;
    const int spt = nd < cap ? nd : cap;                   // wavefronts (= output slots) per workgroup
    const int tiles = (nd + spt - 1) / spt;
    LUVC_LAUNCH("oim_halve", (oim_halve<T, NCH>), dim3((unsigned)((int64_t)B * nlines * tiles)), dim3(64 * spt), 0, st,
                       x, sizes_in, H, W, D, axis, tiles, spt, kept_prev, x_out, sizes_out, pass_map, kept_out);
}

template <typename T>
static bool dispatch_halve(const T* x, const int32_t* sizes_in, int B, int H, int W, int D, int axis,
                           const int32_t* kept_prev, T* x_out, int32_t* sizes_out, int32_t* pass_map, int32_t* kept_out,
                           hipStream_t st)
{
    const int per_wave = 64 * io_traits<T>::kVec;
    const int nch = (D + per_wave - 1) / per_wave;
#define LUVC_HALVE(N) launch_halve<T, N>(x, sizes_in, B, H, W, D, axis, kept_prev, x_out, sizes_out, pass_map, kept_out, st); return true
    switch (nch) {
        case 1: LUVC_HALVE(1);
        case 2: LUVC_HALVE(2);
        case 3: LUVC_HALVE(3);
        case 4: LUVC_HALVE(4);
        case 5: LUVC_HALVE(5);
        case 6: LUVC_HALVE(6);
        case 7: LUVC_HALVE(7);
        case 8: LUVC_HALVE(8);
        default: return false;
    }
#undef LUVC_HALVE
}

bool oim_halve_supported(int H, int W, int D, luvc_dtype dt, int axis, int m, bool vec)
{
    const int len = axis ? W : H;
    const int per_wave = 64 * (dt == LUVC_F32 ? 4 : 8);
    return vec && len >= 2 && m == (len + 1) / 2 && (D + per_wave - 1) / per_wave <= 8;
}

luvc_status oim_halve_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int axis,
                           void* x_out, int32_t* sizes_out, int32_t* pass_map, const int32_t* kept_prev, int32_t* kept_out,
                           hipStream_t st)
{
    bool ok;
    if (dt == LUVC_F32)
        ok = dispatch_halve<float>((const float*)x, sizes_in, B, H, W, D, axis, kept_prev, (float*)x_out, sizes_out, pass_map, kept_out, st);
    else
        ok = dispatch_halve<bf16_t>((const bf16_t*)x, sizes_in, B, H, W, D, axis, kept_prev, (bf16_t*)x_out, sizes_out, pass_map, kept_out, st);
    if (!ok) { set_error("oim_halve_pass: unsupported D"); return LUVC_ERR_UNSUPPORTED; }
    return check_launch("oim halving pass");
}

}  // namespace luvc

// ------------------------------------------------------------------ self-test aid
namespace luvc {
__global__ void __launch_bounds__(256)
selftest_fdot2(const uint32_t* __restrict__ x, const uint32_t* __restrict__ y, int rows, int nwords, float* __restrict__ out)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    float acc = 0.f;
    for (int i = 0; i < nwords; ++i) {
        bf16x2_t a, b;
        const uint32_t xa = x[(int64_t)r * nwords + i], yb = y[(int64_t)r * nwords + i];
        __builtin_memcpy(&a, &xa, 4);
        __builtin_memcpy(&b, &yb, 4);
        acc = __builtin_amdgcn_fdot2_f32_bf16(a, b, acc, false);
    }
    out[r] = acc;
}
}  // namespace luvc

extern "C" luvc_status luvc_selftest_fdot2(const void* x, const void* y, int rows, int words, float* out, void* hip_stream)
{
    using namespace luvc;
    if (!x || !y || !out || rows < 1 || words < 1 || ((uintptr_t)x | (uintptr_t)y | (uintptr_t)out) % 4) {
        set_error("luvc_selftest_fdot2: null or misaligned pointer, or rows / words < 1");
        return LUVC_ERR_INVALID_ARG;
    }
    LUVC_LAUNCH("selftest_fdot2", selftest_fdot2, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, (hipStream_t)hip_stream,
                (const uint32_t*)x, (const uint32_t*)y, rows, words, out);
    return check_launch("selftest fdot2");
}
