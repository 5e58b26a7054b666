// OIM decided on a separate metric tensor (paper Section 3.1, complexity paragraph: similarity in "the dimension
// of keys"; Section 3.2, Algorithm 1) - one launch for a PAIR of halving passes on orthogonal axes.
//
// Same work split as oim_halve_pair: a workgroup owns one line position j of the first pass and a run of output
// slots of the second pass, a wavefront owns four consecutive lines of the first pass, the intermediate grid stays
// in registers and LDS.  What differs: every token comes as two rows, its features (D values, merged and written)
// and its metric (Dm values: the decisions are taken on it, and it is merged and written the same way, because the
// second pass decides on the merged metric).  The metric of a token is at most 1 KB, a few registers per lane, so
// all similarity sums are formed in fp64 straight away - there is no fp32 screening - and the features of tokens
// that are only looked at for a decision (the two destinations beyond the sources of the first pass, the rows just
// outside a workgroup's run) are never loaded.
#include "oim_pair_tok.hpp"

namespace luvc {

namespace {

// ------------------------------------------------------------------ fp64 sums over the wavefront, eight at a time
__device__ __forceinline__ double dpp_get64(double v, const int sel)
{
    const float lo = dpp_get(__int_as_float(__double2loint(v)), sel), hi = dpp_get(__int_as_float(__double2hiint(v)), sel);
    return __hiloint2double(__float_as_int(hi), __float_as_int(lo));
}

// v + (v of the lane 32 away), then 16 away: lane-swap instructions on both halves of the value
__device__ __forceinline__ double add_far_lanes64(double r)
{
    const uint32_t lo = (uint32_t)__double2loint(r), hi = (uint32_t)__double2hiint(r);
    const auto l32 = __builtin_amdgcn_permlane32_swap(lo, lo, false, false), h32 = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    r = __hiloint2double((int)h32[0], (int)l32[0]) + __hiloint2double((int)h32[1], (int)l32[1]);
    const uint32_t lo2 = (uint32_t)__double2loint(r), hi2 = (uint32_t)__double2hiint(r);
    const auto l16 = __builtin_amdgcn_permlane16_swap(lo2, lo2, false, false), h16 = __builtin_amdgcn_permlane16_swap(hi2, hi2, false, false);
    return __hiloint2double((int)h16[0], (int)l16[0]) + __hiloint2double((int)h16[1], (int)l16[1]);
}

// Eight wave64 sums at once, the scheme of wave_total32x8: three exchange steps (lanes 1, 2, 4 apart) after which a
// lane keeps only the partial sum of value (lane & 7), then lanes 8, 32 and 16 apart.  Every step adds the partial sums
// of two lane groups, so all eight values - and wave_total64b below - are summed over the same tree: a sum has the
// same bits in whichever of these places it is formed, which two workgroups that look at one source rely on.
__device__ __forceinline__ void wave_total64x8(double (&v)[8], int lane)
{
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
    double p[4], q[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const double keep = b0 ? v[2 * i + 1] : v[2 * i], send = b0 ? v[2 * i] : v[2 * i + 1];
        p[i] = keep + dpp_get64(send, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const double keep = b1 ? p[2 * i + 1] : p[2 * i], send = b1 ? p[2 * i] : p[2 * i + 1];
        q[i] = keep + dpp_get64(send, 1);
    }
    const double keep = b2 ? q[1] : q[0], send = b2 ? q[0] : q[1];
    double r = keep + dpp_get64(dpp_get64(send, 2), 3);             // (lane ^ 7) ^ 3 = lane ^ 4
    r += dpp_get64(r, 4);
    r = add_far_lanes64(r);
#pragma unroll
    for (int i = 0; i < 8; ++i)
        v[i] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(r), i), __builtin_amdgcn_readlane(__double2loint(r), i));
}

// one sum over the same tree
__device__ __forceinline__ double wave_total64b(double v)
{
    v += dpp_get64(v, 0);
    v += dpp_get64(v, 1);
    v += dpp_get64(dpp_get64(v, 2), 3);
    v += dpp_get64(v, 4);
    v = add_far_lanes64(v);
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 0), __builtin_amdgcn_readlane(__double2loint(v), 0));
}

// fp64 squared norms n[p] = <P_p, P_p> and neighbour products d[p] = <P_p, P_p+1> of five metric rows that follow
// each other on a line; n[4], the ninth sum, only with FIVE
template <typename T, bool FIVE, int MQ, int MW>
__device__ __forceinline__ void metric_sums64(const Tok<MQ, MW>& P0, const Tok<MQ, MW>& P1, const Tok<MQ, MW>& P2, const Tok<MQ, MW>& P3,
                                              const Tok<MQ, MW>& P4, double (&n)[5], double (&d)[4], int lane)
{
    double s[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0}, t = 0.0;
#pragma unroll
    for (int i = 0; i < Tok<MQ, MW>::N; ++i) {
#pragma unroll
        for (int e = 0; e < words<T>::per; ++e) {
            const double p0 = elem64<T>(P0.w[i], e), p1 = elem64<T>(P1.w[i], e), p2 = elem64<T>(P2.w[i], e), p3 = elem64<T>(P3.w[i], e),
                         p4 = elem64<T>(P4.w[i], e);
            s[0] = fma(p0, p0, s[0]); s[1] = fma(p1, p1, s[1]); s[2] = fma(p2, p2, s[2]); s[3] = fma(p3, p3, s[3]);
            s[4] = fma(p0, p1, s[4]); s[5] = fma(p1, p2, s[5]); s[6] = fma(p2, p3, s[6]); s[7] = fma(p3, p4, s[7]);
            if (FIVE) t = fma(p4, p4, t);
        }
    }
    wave_total64x8(s, lane);
    n[0] = s[0]; n[1] = s[1]; n[2] = s[2]; n[3] = s[3];
    d[0] = s[4]; d[1] = s[5]; d[2] = s[6]; d[3] = s[7];
    n[4] = FIVE ? wave_total64b(t) : 0.0;
}

}  // namespace

template <typename T, int NQ, int TW, int MQ, int MW, int NW>
__global__ void __launch_bounds__(NW * 64)
oim_halve_pair_keyed(const T* __restrict__ x, const T* __restrict__ metric, const int32_t* __restrict__ sizes_in, PairGeom g, int Dm,
                     const int32_t* __restrict__ kept_prev, T* __restrict__ x_out, T* __restrict__ metric_out,
                     int32_t* __restrict__ sizes_out, int32_t* __restrict__ pair_map, int32_t* __restrict__ kept_out)
{
    using TokX = Tok<NQ, TW>;
    using TokM = Tok<MQ, MW>;
    constexpr int NX = TokX::N, NM = TokM::N, NL = NX + NM;
    constexpr int kRows = 4 * NW + 8;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint32_t* lds_tok = reinterpret_cast<uint32_t*>(lds_raw);     // [live waves][NX + NM][64]: first token of each wave, features then metric
    __shared__ double inv64[kRows], dt64[kRows];                  // 1/|M[r]|, <M[r], M[r+1]> of the intermediate metric rows
    __shared__ int szl[kRows];

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
    const int own_end = row_base + 2 * nseg;                      // last row whose features can end up in an output of this run
    const int nwm = (row_end - row_base + 1 + 3) >> 2;            // wavefronts with rows of the run
    const bool is_main = w < nwm;
    const bool is_halo = u0 > 0 && w == nwm;                      // holds row_base - 1 as ITS LAST row
    const bool active = is_main || is_halo;
    const int r0 = is_halo ? row_base - 4 : row_base + 4 * w;
    const int rr0 = r0 - row_base + 1;                            // LDS index of row r0 (negative only for the halo wave's unused rows)
    const int x_bytes = g.D * (int)sizeof(T), m_bytes = Dm * (int)sizeof(T);

    // ------------------------------------------------------------------ first pass: four intermediate tokens
    const int pa = 2 * j, pb = pa + 1, pc = pa + 2;
    const bool has_l = j > 0, has_c = pc < g.L1, has_r = pc + 1 < g.L1;
    const int64_t img_in = (int64_t)b * g.n_in;
    TokX T0, T1, T2, T3;
    TokM M0, M1, M2, M3;
    zero_tok(T0); zero_tok(T1); zero_tok(T2); zero_tok(T3);
    zero_tok(M0); zero_tok(M1); zero_tok(M2); zero_tok(M3);
    int s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    unsigned took_a = 0, took_c = 0;                              // bit k: row k absorbed its a / its c
#pragma unroll 4
    for (int k = 0; k < 4; ++k) {
        const int r = r0 + k;
        TokX Tn;
        TokM Mn;
        int sn = 0;
        zero_tok(Tn);
        zero_tok(Mn);
        if (active && r >= row_lo && r <= row_end) {
            const int64_t t0 = img_in + (int64_t)r * g.sB;        // token of position 0 on this line
            const int64_t ta = t0 + (int64_t)pa * g.sA, tb = t0 + (int64_t)pb * g.sA, tc = t0 + (int64_t)pc * g.sA;
            const bool need_x = is_main && r <= own_end;          // wave-uniform
            TokX A, Bt, C;
            if (need_x) {
                load_tok(A, x + ta * g.D, x_bytes, lane);
                load_tok(Bt, x + tb * g.D, x_bytes, lane);
                load_tok(C, x + (has_c ? tc : tb) * g.D, x_bytes, lane, has_c);
            }
            TokM Ma, Mb, Mc, Ml, Mr;
            load_tok(Ma, metric + ta * Dm, m_bytes, lane);
            load_tok(Mb, metric + tb * Dm, m_bytes, lane);
            load_tok(Mc, metric + (has_c ? tc : tb) * Dm, m_bytes, lane, has_c);
            load_tok(Ml, metric + (has_l ? ta - g.sA : tb) * Dm, m_bytes, lane, has_l);
            load_tok(Mr, metric + (has_r ? tc + g.sA : tb) * Dm, m_bytes, lane, has_r);
            const int sb = sizes_in ? sizes_in[tb] : 1;
            const int sa_in = sizes_in ? sizes_in[ta] : 1;
            const int sc_in = (sizes_in && has_c) ? sizes_in[tc] : 1;
            // every sum is formed lower position first, so the sum two workgroups share has the same bits
            // (tokens that are not there were loaded as zeros: their sums are zero and never looked at)
            double n[5], d[4];
            metric_sums64<T, true>(Ml, Ma, Mb, Mc, Mr, n, d, lane);
            const double jb = inv_norm64(n[2]);
            const bool a_left = has_l && source_goes_left(true, true, inv_norm64(n[1]), d[0], inv_norm64(n[0]), d[1], jb);
            const bool c_left = has_c && (!has_r || source_goes_left(true, true, inv_norm64(n[3]), d[2], jb, d[3], inv_norm64(n[4])));
            const bool take_a = !a_left, take_c = c_left;
            const int sa = take_a ? sa_in : 0, sc = take_c ? sc_in : 0;
            sn = sb + sa + sc;
            if (take_a) took_a |= 1u << k;
            if (take_c) took_c |= 1u << k;
            if (!take_a && !take_c) {
                Mn = Mb;
                if (need_x) Tn = Bt;
            } else {
                merge_tok<T>(Mn, Mb, Ma, Mc, sb, sa, sc);
                if (need_x) merge_tok<T>(Tn, Bt, A, C, sb, sa, sc);
            }
        }
        T0 = T1; T1 = T2; T2 = T3; T3 = Tn;
        M0 = M1; M1 = M2; M2 = M3; M3 = Mn;
        s0 = s1; s1 = s2; s2 = s3; s3 = sn;
    }

    // ------------------------------------------------------------------ second pass: exchange
    if (is_main) {
#pragma unroll
        for (int i = 0; i < NX; ++i) lds_tok[(w * NL + i) * 64 + lane] = T0.w[i];
#pragma unroll
        for (int i = 0; i < NM; ++i) lds_tok[(w * NL + NX + i) * 64 + lane] = M0.w[i];
    }
    __syncthreads();
    TokX Tx;                                                      // the token after T3: first token of the next wavefront
    TokM Mx;
    zero_tok(Tx);
    zero_tok(Mx);
    if (active && r0 + 4 <= row_end) {
        const int nxt = is_halo ? 0 : w + 1;
#pragma unroll
        for (int i = 0; i < NX; ++i) Tx.w[i] = lds_tok[(nxt * NL + i) * 64 + lane];
#pragma unroll
        for (int i = 0; i < NM; ++i) Mx.w[i] = lds_tok[(nxt * NL + NX + i) * 64 + lane];
    }
    if (active) {
        double n[5], d[4];
        metric_sums64<T, false>(M0, M1, M2, M3, Mx, n, d, lane);
        if (lane < 4) {
            const int k = lane, r = r0 + k;
            if (r >= row_lo && r <= row_end) {
                inv64[rr0 + k] = inv_norm64(k == 0 ? n[0] : k == 1 ? n[1] : k == 2 ? n[2] : n[3]);
                dt64[rr0 + k] = k == 0 ? d[0] : k == 1 ? d[1] : k == 2 ? d[2] : d[3];
                szl[rr0 + k] = k == 0 ? s0 : k == 1 ? s1 : k == 2 ? s2 : s3;
            }
        }
    }
    __syncthreads();
    if (!is_main) return;
    // a source at intermediate row r (LDS index q) goes UP (to the lower position) unless the row below is strictly more similar
    auto decide64 = [&](int r, int q) -> bool {
        const bool has_up = r >= 1, has_dn = r + 1 < g.L2;
        const int qm = q > 0 ? q - 1 : 0;
        return source_goes_left(has_up, has_dn, inv64[q], dt64[qm], inv64[qm], dt64[q], inv64[q + 1]);
    };
    const bool e2 = r0 + 2 <= row_end, e4 = r0 + 4 <= row_end;
    const bool up0 = decide64(r0, rr0);
    const bool up2 = e2 && decide64(r0 + 2, rr0 + 2);
    const bool up4 = e4 && decide64(r0 + 4, rr0 + 4);

    // ------------------------------------------------------------------ second pass: merge, write, maps
    const bool tail = (g.L2 & 1) && own_end == g.L2 - 1;          // the last source of an odd line belongs to this run
    const int64_t img_out = (int64_t)b * g.n_out;
    const int uo = r0 >> 1;                                       // output slot (second axis) of destination r0 + 1
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        const int dest = r0 + 1 + 2 * o;
        if (dest >= own_end) break;
        const bool take_a = o == 0 ? !up0 : !up2;                 // the source above comes down
        const bool take_c = o == 0 ? (e2 && up2) : (e4 && up4);   // the source below goes up
        const TokX& Bt = o == 0 ? T1 : T3;
        const TokX& A = o == 0 ? T0 : T2;
        const TokX& C = o == 0 ? T2 : Tx;
        const TokM& Mb = o == 0 ? M1 : M3;
        const TokM& Ma = o == 0 ? M0 : M2;
        const TokM& Mc = o == 0 ? M2 : Mx;
        const int sb = o == 0 ? s1 : s3;
        const int sa = take_a ? (o == 0 ? s0 : s2) : 0;
        const int sc = take_c ? (o == 0 ? s2 : szl[rr0 + 4]) : 0;
        const int slot = (uo + o) * g.oB + j * g.oA;
        T* op = x_out + (img_out + slot) * g.D;
        T* om = metric_out ? metric_out + (img_out + slot) * Dm : nullptr;
        if (lane == 0) {
            sizes_out[img_out + slot] = sb + sa + sc;
            if (kept_out) {
                const int p_in = dest * g.sB + pb * g.sA;
                kept_out[img_out + slot] = kept_prev ? kept_prev[img_in + p_in] : p_in;
            }
        }
        if (!take_a && !take_c) {
            store_tok(op, x_bytes, Bt, lane);
            if (om) store_tok(om, m_bytes, Mb, lane);
        } else {
            TokX R;
            merge_tok<T>(R, Bt, A, C, sb, sa, sc);
            store_tok(op, x_bytes, R, lane);
            if (om) {
                TokM Rm;
                merge_tok<T>(Rm, Mb, Ma, Mc, sb, sa, sc);
                store_tok(om, m_bytes, Rm, lane);
            }
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

// 16-byte pieces per lane, then a 4- or 8-byte tail piece if that covers what is left
void token_form(int bytes, int* nq, int* tw)
{
    *nq = bytes / 1024;
    *tw = 0;
    const int rem = bytes % 1024;
    if (rem > 512) ++*nq;
    else if (rem > 256) *tw = 2;
    else if (rem > 0) *tw = 1;
}

template <typename T, int NQ, int TW, int MQ, int MW>
luvc_status launch_keyed(const T* x, const T* metric, const int32_t* sizes_in, int B, int H, int W, int D, int Dm, int first_axis,
                         const int32_t* kept_prev, T* x_out, T* metric_out, int32_t* sizes_out, int32_t* pair_map, int32_t* kept_out,
                         hipStream_t st)
{
    constexpr int N = 4 * NQ + TW, NM = 4 * MQ + MW, NL = N + NM;
    // 16 wavefronts leave 128 registers per lane, 8 leave 256; a metric word costs more of them than a feature word
    // (nine metric tokens are live while the sums of a row are formed, widened to fp64 piece by piece)
    constexpr int NW = (N <= 10 && N + 6 * NM <= 20) ? 16 : 8;
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
    const size_t lds = (size_t)p.waves * NL * 64 * 4;          // at most 16 * 14 * 256 = 56 KiB
    LUVC_LAUNCH("oim_halve_pair_keyed", (oim_halve_pair_keyed<T, NQ, TW, MQ, MW, NW>), dim3((unsigned)((int64_t)B * g.segs * g.nd1)),
                dim3(64 * p.waves), lds, st, x, metric, sizes_in, g, Dm, kept_prev, x_out, metric_out, sizes_out, pair_map, kept_out);
    return check_launch("oim keyed halving pair");
}

template <typename T, int NQ, int TW>
luvc_status dispatch_metric(const T* x, const T* metric, const int32_t* sizes_in, int B, int H, int W, int D, int Dm, int first_axis,
                            const int32_t* kept_prev, T* x_out, T* metric_out, int32_t* sizes_out, int32_t* pair_map, int32_t* kept_out,
                            hipStream_t st)
{
    int mq, mw;
    token_form(Dm * (int)sizeof(T), &mq, &mw);
#define LUVC_KEYED(Q, W_) if (mq == Q && mw == W_) return launch_keyed<T, NQ, TW, Q, W_>(x, metric, sizes_in, B, H, W, D, Dm, first_axis, kept_prev, x_out, metric_out, sizes_out, pair_map, kept_out, st)
    LUVC_KEYED(0, 1); LUVC_KEYED(0, 2); LUVC_KEYED(1, 0);
#undef LUVC_KEYED
    set_error("oim keyed pair: unsupported Dm");
    return LUVC_ERR_UNSUPPORTED;
}

template <typename T>
luvc_status dispatch_keyed(const T* x, const T* metric, const int32_t* sizes_in, int B, int H, int W, int D, int Dm, int first_axis,
                           const int32_t* kept_prev, T* x_out, T* metric_out, int32_t* sizes_out, int32_t* pair_map, int32_t* kept_out,
                           hipStream_t st)
{
    int nq, tw;
    token_form(D * (int)sizeof(T), &nq, &tw);
#define LUVC_KEYED(Q, W_) if (nq == Q && tw == W_) return dispatch_metric<T, Q, W_>(x, metric, sizes_in, B, H, W, D, Dm, first_axis, kept_prev, x_out, metric_out, sizes_out, pair_map, kept_out, st)
    LUVC_KEYED(0, 1); LUVC_KEYED(0, 2);
    LUVC_KEYED(1, 0); LUVC_KEYED(1, 1); LUVC_KEYED(1, 2);
    LUVC_KEYED(2, 0); LUVC_KEYED(2, 1); LUVC_KEYED(2, 2);
    LUVC_KEYED(3, 0); LUVC_KEYED(3, 1); LUVC_KEYED(3, 2);
    LUVC_KEYED(4, 0);
#undef LUVC_KEYED
    set_error("oim keyed pair: unsupported D");
    return LUVC_ERR_UNSUPPORTED;
}

}  // namespace

bool oim_pair_keyed_supported(int H, int W, int D, int Dm, luvc_dtype dt, int axis0, int m0, int axis1, int m1, bool vec_x, bool vec_m)
{
    if (!vec_m || (int64_t)Dm * (dt == LUVC_F32 ? 4 : 2) > 1024) return false;
    return oim_pair_supported(H, W, D, dt, axis0, m0, axis1, m1, vec_x);
}

luvc_status oim_pair_keyed_pass(const void* x, const void* metric, const int32_t* sizes_in, int B, int H, int W, int D, int Dm,
                                luvc_dtype dt, int first_axis, void* x_out, void* metric_out, int32_t* sizes_out, int32_t* pair_map,
                                const int32_t* kept_prev, int32_t* kept_out, hipStream_t st)
{
    if (dt == LUVC_F32)
        return dispatch_keyed<float>((const float*)x, (const float*)metric, sizes_in, B, H, W, D, Dm, first_axis, kept_prev,
                                     (float*)x_out, (float*)metric_out, sizes_out, pair_map, kept_out, st);
    return dispatch_keyed<bf16_t>((const bf16_t*)x, (const bf16_t*)metric, sizes_in, B, H, W, D, Dm, first_axis, kept_prev,
                                  (bf16_t*)x_out, (bf16_t*)metric_out, sizes_out, pair_map, kept_out, st);
}

}  // namespace luvc
