// OIM (paper Section 3.2, Algorithm 1) - one launch for a PAIR of halving passes on orthogonal
// axes (row merge then column merge, or the other way round): H x W -> H/2 x W/2 without the
// intermediate grid ever leaving the chip.
//
// Work split.  A workgroup owns one line position j of the first pass (output column j for a
// row-then-column pair) and a run of output slots of the second pass.  Each wavefront owns four
// consecutive lines of the first pass: for each of them it loads destination b = 2j+1, its two
// sources a = 2j, c = 2j+2 and the two destinations beyond them (l = 2j-1, r = 2j+3, needed only
// to decide where a and c go), forms the first-pass token, rounds it to the storage type - the
// second pass must read what a separate launch would have read from memory - and keeps it packed
// in registers.  The four intermediate tokens of a wavefront are two destinations of the second
// pass with the sources between them; the one token a wavefront needs from its neighbour (the
// first token of the next wavefront) goes through LDS, as do the norms and neighbour dot
// products every wavefront needs from the tokens around its own.  A workgroup that owns only
// part of a long line recomputes the three intermediate tokens just outside its run.
//
// A token in registers is NQ 16-byte pieces per lane plus a 4- or 8-byte tail piece, so that a
// token of 1280 bf16 values costs 10 registers per lane, not 12; buffer resources bound every
// piece, so lanes past the end of a token read zeros and write nothing.
//
// Decisions are fp64 decisions reached in two steps, as in the single-pass kernel: a screening
// sweep in fp32 with a rigorous error bound, and a repeat in fp64 of whatever is closer than the
// bound.  In the first pass the repeat is local to a wavefront; in the second pass it is taken by
// the whole workgroup, because the sums of a decision live in two wavefronts.  A source shared by
// two workgroups is decided from the same bits by the same expressions in both.
//
// The merge is the size-weighted mean evaluated in fp64 in position order and rounded once.  One
// case needs no fp64: bf16 storage, one absorbed source, equal sizes.  Then the mean is (b + x) / 2
// and the fp32 sum, halved and rounded to bf16 by the hardware conversion, is the correctly rounded
// result: either the sum is exact in fp32 (exponents at most 15 apart), or the smaller term is below
// 2^-15 of the larger, whose half lies on the bf16 grid at least 2^-10 (relative) away from every
// rounding boundary - too far for the smaller term or the fp32 rounding to matter.
#include <cstdlib>

#include "oim_pair_tok.hpp"

namespace luvc {

// Tokens of at most 8 words per lane (1 KB in bf16) are compiled for six wavefronts per SIMD (80 registers, a few spilled
// in the fp64 repeat): on batches of small grids a workgroup is 6 wavefronts, and four workgroups per compute unit instead
// of three put 80 x 24 x 24 grids (960 workgroups) on the chip in one round - measured 36.8 -> 33.9 us.  The same
// hint on wider tokens (96 instead of 103 registers) measured slower on every workload and is not given.
template <typename T, int NQ, int TW, int NW>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu((4 * NQ + TW <= 8 && NW == 16) ? 6 : 1)))
oim_halve_pair(const T* __restrict__ x, const int32_t* __restrict__ sizes_in, PairGeom g,
               const int32_t* __restrict__ kept_prev, T* __restrict__ x_out, int32_t* __restrict__ sizes_out,
               int32_t* __restrict__ pair_map, int32_t* __restrict__ kept_out)
{
    using TokT = Tok<NQ, TW>;
    constexpr int N = TokT::N;
    constexpr int kRows = 4 * NW + 8;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint32_t* lds_tok = reinterpret_cast<uint32_t*>(lds_raw);     // [live waves][N][64]: first token of each wave
    __shared__ float inv32[kRows], dt32[kRows];                   // 1/|T[r]|, <T[r], T[r+1]> of the intermediate tokens
    __shared__ double inv64[kRows], dt64[kRows];
    __shared__ int szl[kRows];
    __shared__ int redo;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int j = item % g.nd1;
    const int seg = (item / g.nd1) % g.segs;
    const int b = item / (g.nd1 * g.segs);
    const int u0 = seg * g.seg_out;
    const int nseg = min(g.seg_out, g.nd2 - u0);                  // second-pass outputs of this workgroup
    const int row_base = 2 * u0;
    const int row_lo = u0 > 0 ? row_base - 1 : row_base;          // one intermediate row above the run decides its first source
    const int row_end = min(g.L2 - 1, row_base + 2 * nseg + 1);   // two below decide its last source (or close an odd line)
    const int nwm = (row_end - row_base + 1 + 3) >> 2;            // wavefronts with rows of the run
    const bool is_main = w < nwm;
    const bool is_halo = u0 > 0 && w == nwm;                      // holds row_base - 1 as ITS LAST row
    const bool active = is_main || is_halo;
    const int r0 = is_halo ? row_base - 4 : row_base + 4 * w;
    const int rr0 = r0 - row_base + 1;                            // LDS index of row r0 (negative only for the halo wave's unused rows)
    // Error bound of the screening, in units of u = 2^-24.  A sum takes at most E = R + 6 roundings of
    // relative size u on partial sums bounded by the sum of the magnitudes of its terms (R per lane: two
    // per packed bf16 product pair, one per fp32 product; six reduction steps); against |a||b| that is E u
    // on a dot product and E u on each squared norm, i.e. (E + 4) u on the two reciprocal norms together
    // (hardware reciprocal square root: 1 ulp each), plus two products: 2 E + 6 per cosine, 4 E + 13 on
    // the difference of two.  tau is 1.5 times that.  Each step of the packed bf16 dot product is taken as one or two
    // roundings to nearest of the exact value (tests/test_gpu_oim.py pins the instruction's sums against fp64);
    // underflow and overflow are kept out by inv_norm32().
    constexpr int kE = N * (words<T>::per == 2 ? 2 : 1) + 6;
    const float tau = (float)(6 * kE + 20) * 5.9604645e-8f;
    const int tok_bytes = g.D * (int)sizeof(T);
    if (threadIdx.x == 0) redo = 0;

    // ------------------------------------------------------------------ first pass: four intermediate tokens
    const int pa = 2 * j, pb = pa + 1, pc = pa + 2;
    const bool has_l = j > 0, has_c = pc < g.L1, has_r = pc + 1 < g.L1;
    const int64_t img_in = (int64_t)b * g.n_in;
    TokT T0, T1, T2, T3;
    zero_tok(T0); zero_tok(T1); zero_tok(T2); zero_tok(T3);
    int s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    unsigned took_a = 0, took_c = 0;                              // bit k: row k absorbed its a / its c
    // the four rows unrolled: the compiler renames T0..T3 instead of moving 10 registers per token and row
    // (measured: 35.3 -> 34.2 us on 8 x 64 x 64 x 1280 bf16)
#pragma unroll 4
    for (int k = 0; k < 4; ++k) {
        const int r = r0 + k;
        TokT Tn;
        int sn = 0;
        if (active && r >= row_lo && r <= row_end) {
            const int64_t t0 = img_in + (int64_t)r * g.sB;        // token of position 0 on this line
            const int64_t ta = t0 + (int64_t)pa * g.sA, tb = t0 + (int64_t)pb * g.sA, tc = t0 + (int64_t)pc * g.sA;
            TokT A, Bt, C, Lt, Rt;
            load_tok(A, x + ta * g.D, tok_bytes, lane);
            load_tok(Bt, x + tb * g.D, tok_bytes, lane);
            load_tok(C, x + (has_c ? tc : tb) * g.D, tok_bytes, lane, has_c);
            load_tok(Lt, x + (has_l ? ta - g.sA : tb) * g.D, tok_bytes, lane, has_l);
            load_tok(Rt, x + (has_r ? tc + g.sA : tb) * g.D, tok_bytes, lane, has_r);
            const int sb = sizes_in ? sizes_in[tb] : 1;
            const int sa_in = sizes_in ? sizes_in[ta] : 1;
            const int sc_in = (sizes_in && has_c) ? sizes_in[tc] : 1;
            // screening: every sum is formed lower position first, so the sum two workgroups share has the same bits
            // (tokens that are not there were loaded as zeros: their sums are zero and never looked at)
            float sm[8] = {dot32_lane<T>(A, A), dot32_lane<T>(Bt, Bt), dot32_lane<T>(A, Bt), dot32_lane<T>(Lt, A),
                           dot32_lane<T>(Lt, Lt), dot32_lane<T>(C, C), dot32_lane<T>(Bt, C), dot32_lane<T>(C, Rt)};
            wave_total32x8(sm, lane);
            const float ia = inv_norm32(sm[0]), ib = inv_norm32(sm[1]), dab = sm[2];
            int va = -1, vc = -1;
            if (has_l) va = screen_source(true, true, ia, sm[3], inv_norm32(sm[4]), dab, ib, tau);
            if (has_c) {
                vc = 1;
                if (has_r) vc = screen_source(true, true, inv_norm32(sm[5]), sm[6], ib, sm[7], inv_norm32(dot32<T>(Rt, Rt)), tau);
            }
            bool a_left = va > 0, c_left = vc > 0;
            if (va == 0 || vc == 0) {                             // too close for fp32: the fp64 cosines decide
                double n[5], d[4];
                chain_sums64<T>(Lt, A, Bt, C, Rt, n, d);
                const double jb = inv_norm64(n[2]);
                if (va == 0) a_left = source_goes_left(true, true, inv_norm64(n[1]), d[0], inv_norm64(n[0]), d[1], jb);
                if (vc == 0) c_left = source_goes_left(true, true, inv_norm64(n[3]), d[2], jb, d[3], inv_norm64(n[4]));
            }
            const bool take_a = !a_left, take_c = has_c && c_left;
            const int sa = take_a ? sa_in : 0, sc = take_c ? sc_in : 0;
            sn = sb + sa + sc;
            if (take_a) took_a |= 1u << k;
            if (take_c) took_c |= 1u << k;
            if (!take_a && !take_c) Tn = Bt;
            else merge_tok<T>(Tn, Bt, A, C, sb, sa, sc);
        } else {
            zero_tok(Tn);
        }
        T0 = T1; T1 = T2; T2 = T3; T3 = Tn;
        s0 = s1; s1 = s2; s2 = s3; s3 = sn;
    }

    // ------------------------------------------------------------------ second pass: exchange
    if (is_main) {
#pragma unroll
        for (int i = 0; i < N; ++i) lds_tok[(w * N + i) * 64 + lane] = T0.w[i];
    }
    __syncthreads();
    TokT Tx;                                                      // the token after T3: first token of the next wavefront
    const bool has_x = active && r0 + 4 <= row_end;
    if (has_x) {
        const int nxt = is_halo ? 0 : w + 1;
#pragma unroll
        for (int i = 0; i < N; ++i) Tx.w[i] = lds_tok[(nxt * N + i) * 64 + lane];
    } else {
        zero_tok(Tx);
    }
    if (active) {
        float sm[8] = {dot32_lane<T>(T0, T0), dot32_lane<T>(T1, T1), dot32_lane<T>(T2, T2), dot32_lane<T>(T3, T3),
                       dot32_lane<T>(T0, T1), dot32_lane<T>(T1, T2), dot32_lane<T>(T2, T3), dot32_lane<T>(T3, Tx)};
        wave_total32x8(sm, lane);
        const float n0 = sm[0], n1 = sm[1], n2 = sm[2], n3 = sm[3], d0 = sm[4], d1 = sm[5], d2 = sm[6], d3 = sm[7];
        if (lane < 4) {
            const int k = lane, r = r0 + k;
            if (r >= row_lo && r <= row_end) {
                inv32[rr0 + k] = inv_norm32(k == 0 ? n0 : k == 1 ? n1 : k == 2 ? n2 : n3);
                dt32[rr0 + k] = k == 0 ? d0 : k == 1 ? d1 : k == 2 ? d2 : d3;
                szl[rr0 + k] = k == 0 ? s0 : k == 1 ? s1 : k == 2 ? s2 : s3;
            }
        }
    }
    __syncthreads();
    // a source at intermediate row r (LDS index q) goes UP (to the lower position) unless the row below is strictly more similar
    auto verdict32 = [&](int r, int q) -> int {
        const bool has_up = r >= 1, has_dn = r + 1 < g.L2;
        const int qm = q > 0 ? q - 1 : 0;
        return screen_source(has_up, has_dn, inv32[q], dt32[qm], inv32[qm], dt32[q], inv32[q + 1], tau);
    };
    auto decide64 = [&](int r, int q) -> bool {
        const bool has_up = r >= 1, has_dn = r + 1 < g.L2;
        const int qm = q > 0 ? q - 1 : 0;
        return source_goes_left(has_up, has_dn, inv64[q], dt64[qm], inv64[qm], dt64[q], inv64[q + 1]);
    };
    const bool e2 = r0 + 2 <= row_end, e4 = r0 + 4 <= row_end;
    int v0 = -1, v2 = -1, v4 = -1;
    if (is_main) {
        v0 = verdict32(r0, rr0);
        if (e2) v2 = verdict32(r0 + 2, rr0 + 2);
        if (e4) v4 = verdict32(r0 + 4, rr0 + 4);
        if ((v0 == 0 || v2 == 0 || v4 == 0) && lane == 0) redo = 1;
    }
    __syncthreads();
    bool up0 = v0 > 0, up2 = v2 > 0, up4 = v4 > 0;
    if (redo) {                                                   // uniform over the workgroup
        if (active) {
            double n[5], d[4];
            chain_sums64<T>(T0, T1, T2, T3, Tx, n, d);
            if (lane < 4) {
                const int k = lane, r = r0 + k;
                if (r >= row_lo && r <= row_end) {
                    inv64[rr0 + k] = inv_norm64(k == 0 ? n[0] : k == 1 ? n[1] : k == 2 ? n[2] : n[3]);
                    dt64[rr0 + k] = k == 0 ? d[0] : k == 1 ? d[1] : k == 2 ? d[2] : d[3];
                }
            }
        }
        __syncthreads();
        if (is_main) {
            up0 = decide64(r0, rr0);
            up2 = e2 && decide64(r0 + 2, rr0 + 2);
            up4 = e4 && decide64(r0 + 4, rr0 + 4);
        }
    }
    if (!is_main) return;

    // ------------------------------------------------------------------ second pass: merge, write, maps
    const int own_end = row_base + 2 * nseg;                      // rows below it belong to the next run ...
    const bool tail = (g.L2 & 1) && own_end == g.L2 - 1;          // ... except the last source of an odd line
    const int64_t img_out = (int64_t)b * g.n_out;
    const int uo = r0 >> 1;                                       // output slot (second axis) of destination r0 + 1
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        const int dest = r0 + 1 + 2 * o;
        if (dest >= own_end) break;
        const bool take_a = o == 0 ? !up0 : !up2;                 // the source above comes down
        const bool take_c = o == 0 ? (e2 && up2) : (e4 && up4);   // the source below goes up
        const TokT& Bt = o == 0 ? T1 : T3;
        const TokT& A = o == 0 ? T0 : T2;
        const TokT& C = o == 0 ? T2 : Tx;
        const int sb = o == 0 ? s1 : s3;
        const int sa = take_a ? (o == 0 ? s0 : s2) : 0;
        const int sc = take_c ? (o == 0 ? s2 : szl[rr0 + 4]) : 0;
        const int slot = (uo + o) * g.oB + j * g.oA;
        T* op = x_out + (img_out + slot) * g.D;
        if (lane == 0) {
            sizes_out[img_out + slot] = sb + sa + sc;
            if (kept_out) {
                const int p_in = dest * g.sB + pb * g.sA;
                kept_out[img_out + slot] = kept_prev ? kept_prev[img_in + p_in] : p_in;
            }
        }
        if (!take_a && !take_c) {
            store_tok(op, tok_bytes, Bt, lane);
        } else {
            TokT R;
            merge_tok<T>(R, Bt, A, C, sb, sa, sc);
            store_tok(op, tok_bytes, R, lane);
        }
    }
    if (pair_map && lane < 4) {
        const int k = lane, r = r0 + k;
        if (r <= row_end && (r < own_end || (tail && r == own_end))) {
            // intermediate row r lands in output slot: odd rows are destinations; an even row goes up or down
            int u;
            if (r & 1) u = r >> 1;
            else u = (k == 0 ? up0 : up2) ? (r >> 1) - 1 : (r >> 1);
            const int slot = u * g.oB + j * g.oA;
            const int64_t t0 = img_in + (int64_t)r * g.sB;
            pair_map[t0 + (int64_t)pb * g.sA] = slot;
            if ((took_a >> k) & 1u) pair_map[t0 + (int64_t)pa * g.sA] = slot;
            if ((took_c >> k) & 1u) pair_map[t0 + (int64_t)pc * g.sA] = slot;
        }
    }
}

// ------------------------------------------------------------------ host side
namespace {

template <typename T, int NQ, int TW>
luvc_status launch_pair(const T* x, const int32_t* sizes_in, int B, int H, int W, int D, int first_axis,
                        const int32_t* kept_prev, T* x_out, int32_t* sizes_out, int32_t* pair_map, int32_t* kept_out,
                        hipStream_t st)
{
    constexpr int N = 4 * NQ + TW;
    constexpr int NW = N <= 10 ? 16 : 8;           // 16 wavefronts leave 128 registers per lane, 8 leave 256
    PairGeom g;
    g.L1 = first_axis ? W : H;
    g.L2 = first_axis ? H : W;
    g.nd1 = g.L1 / 2;
    g.nd2 = g.L2 / 2;
    g.sA = first_axis ? 1 : W;
    g.sB = first_axis ? W : 1;
    const int Wo = W / 2;
    g.oA = first_axis ? 1 : Wo;
    g.oB = first_axis ? Wo : 1;
    g.n_in = H * W;
    g.n_out = (H / 2) * Wo;
    g.D = D;
    const PairPlan p = plan_pair(g.L2, NW, (int64_t)B * g.nd1);
    g.segs = p.segs;
    g.seg_out = p.seg_out;
    const size_t lds = (size_t)p.waves * N * 64 * 4;           // at most 16 * 10 * 256 = 40 KiB
    LUVC_LAUNCH("oim_halve_pair", (oim_halve_pair<T, NQ, TW, NW>), dim3((unsigned)((int64_t)B * g.segs * g.nd1)), dim3(64 * p.waves), lds, st,
                       x, sizes_in, g, kept_prev, x_out, sizes_out, pair_map, kept_out);
    return check_launch("oim halving pair");
}

template <typename T>
luvc_status dispatch_pair(const T* x, const int32_t* sizes_in, int B, int H, int W, int D, int first_axis,
                          const int32_t* kept_prev, T* x_out, int32_t* sizes_out, int32_t* pair_map, int32_t* kept_out,
                          hipStream_t st)
{
    // 16-byte pieces per lane, then a 4- or 8-byte tail piece if that covers what is left
    const int bytes = D * (int)sizeof(T);
    int nq = bytes / 1024, tw = 0;
    const int rem = bytes % 1024;
    if (rem > 512) ++nq;
    else if (rem > 256) tw = 2;
    else if (rem > 0) tw = 1;
#define LUVC_PAIR(Q, W_) if (nq == Q && tw == W_) return launch_pair<T, Q, W_>(x, sizes_in, B, H, W, D, first_axis, kept_prev, x_out, sizes_out, pair_map, kept_out, st)
    LUVC_PAIR(0, 1); LUVC_PAIR(0, 2);
    LUVC_PAIR(1, 0); LUVC_PAIR(1, 1); LUVC_PAIR(1, 2);
    LUVC_PAIR(2, 0); LUVC_PAIR(2, 1); LUVC_PAIR(2, 2);
    LUVC_PAIR(3, 0); LUVC_PAIR(3, 1); LUVC_PAIR(3, 2);
    LUVC_PAIR(4, 0);
#undef LUVC_PAIR
    set_error("oim pair: unsupported D");
    return LUVC_ERR_UNSUPPORTED;
}

}  // namespace

bool oim_pair_supported(int H, int W, int D, luvc_dtype dt, int axis0, int m0, int axis1, int m1, bool vec)
{
    if (!vec || axis0 == axis1) return false;
    const int len0 = axis0 ? W : H, len1 = axis1 ? W : H;           // the second pass runs on the untouched axis
    if (len0 < 2 || len1 < 2 || m0 != (len0 + 1) / 2 || m1 != (len1 + 1) / 2) return false;
    return (int64_t)D * (dt == LUVC_F32 ? 4 : 2) <= 4096;
}

luvc_status oim_pair_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int first_axis,
                          void* x_out, int32_t* sizes_out, int32_t* pair_map, const int32_t* kept_prev, int32_t* kept_out,
                          hipStream_t st)
{
    if (dt == LUVC_F32)
        return dispatch_pair<float>((const float*)x, sizes_in, B, H, W, D, first_axis, kept_prev, (float*)x_out, sizes_out,
                                    pair_map, kept_out, st);
    return dispatch_pair<bf16_t>((const bf16_t*)x, sizes_in, B, H, W, D, first_axis, kept_prev, (bf16_t*)x_out, sizes_out,
                                 pair_map, kept_out, st);
}

}  // namespace luvc
