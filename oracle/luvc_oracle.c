/*
 * CPU ORACLE for LUVC's token-compression hot path (OIM + SPU).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the
 * smoke check and the benchmark's "cpu_baseline" leg may call it.  It shares
 * no code, header, table or constant with the HIP library and never calls it.
 *
 * Style: plain, slow, fp64 everywhere, no blocking / fusion / reordering
 * beyond what the method states, so every loop can be checked against the
 * paper by eye.  OpenMP pragmas only spread independent images / samples over
 * host threads; they never change the arithmetic of one image or sample.
 *
 * What follows the paper and where:
 *   OIM  - Section 3.2 (row merge H x W -> H x (W-m), then column merge
 *          -> (H-m) x (W-m); "similarity calculations and binary matching"),
 *          Algorithm 1 (size vector s = number of merged tokens), appendix
 *          "Iterative Strategy and Pseudocode of OIM" (alternating axes).
 *   SPU  - Section 3.3: Eq. 4 (DFT along the token index), Eq. 5-6 (Hamming
 *          weighted low-pass mask), Eq. 7 (inverse DFT with 1/N), Eq. 8
 *          (per-token L2 energy), Algorithm 2 (top-k indices, gather of the
 *          ORIGINAL tokens).
 *
 * Readings taken where the paper is silent or garbled (listed in full in the
 * design notes of the repository):
 *   - inside a line, even positions are merge sources and odd positions are
 *     destinations (bipartite matching restricted to a line); a source's
 *     candidates are the destinations within distance 2R-1 (R=1: the two
 *     adjacent tokens); similarity = cosine of the token features with norms
 *     clamped at 1e-12; ties go to the lower position;
 *   - merging = size-weighted mean, sizes add;
 *   - the mask of Eq. 5 is the symmetric Hamming window centred on DC over the
 *     folded frequency f(k)=min(k,N-k):  w(f)=0.54+0.46 cos(2 pi f/(N-1)),
 *     pass-band f(k) <= sigma (two sided so that the filtered signal is real);
 *   - kept indices are returned in ascending order, ties -> lower index.
 *
 *   - Section 3.1 counts the similarity cost in "the dimension of keys": the
 *     keyed call takes its decisions on a separate metric tensor and applies
 *     the merge to the tokens (oracle_oim_merge_keyed); Eq. 3's value
 *     enhancement V + log(s) is oracle_value_enhance.
 *
 * Pinned by tests/test_oracle_*.py (brute-force matcher, hand cases, mass
 * conservation, numpy.fft, constant / low-band signals, Parseval, stable sort).
 * Unpinned parameters (not functions): the cut-off sigma and the cascade keep
 * schedule have no value in the paper - "parity unpinned" for those choices.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_EPS_NORM 1e-12

/* ---------------------------------------------------------------- rounding */

/* Round a double to the storage type of a pass output.
 * mode 0: keep fp64; 1: nearest fp32; 2: nearest-even bfloat16.            */
static double round_to_io(double v, int mode)
{
    if (mode == 0) return v;
    float f = (float)v;                /* IEEE round-to-nearest-even */
    if (mode == 1) return (double)f;
    /* bfloat16 = top 16 bits of the fp32 pattern.  Rounding the fp64 value to
     * fp32 first and then to bf16 could round twice; do it in one step by
     * finding the two bf16 neighbours of v and picking the nearer (even on a
     * tie).                                                                 */
    if (!isfinite(v) || v == 0.0) return (double)f;
    uint32_t bits;
    float fa = (float)fabs(v);
    /* truncate fa toward zero to a bf16 value <= |v| */
    memcpy(&bits, &fa, 4);
    if ((double)fa > fabs(v)) bits -= 1;          /* fa was rounded up: step below |v| */
    uint32_t lo_bits = bits & 0xFFFF0000u;
    uint32_t hi_bits = lo_bits + 0x00010000u;
    float lo, hi;
    memcpy(&lo, &lo_bits, 4);
    memcpy(&hi, &hi_bits, 4);
    double a = fabs(v), dl = a - (double)lo, dh = (double)hi - a, r;
    if (dl < dh) r = lo;
    else if (dh < dl) r = hi;
    else r = ((lo_bits >> 16) & 1u) ? hi : lo;    /* tie: even mantissa */
    return v < 0 ? -r : r;
}

/* --------------------------------------------------------------------- OIM */

static double dot_d(const double *a, const double *b, int D)
{
    double s = 0.0;
    for (int d = 0; d < D; ++d) s += a[d] * b[d];
    return s;
}

/* cosine similarity with clamped norms */
static double cosine(const double *a, const double *b, int D)
{
    double na = sqrt(dot_d(a, a, D)), nb = sqrt(dot_d(b, b, D));
    if (na < ORACLE_EPS_NORM) na = ORACLE_EPS_NORM;
    if (nb < ORACLE_EPS_NORM) nb = ORACLE_EPS_NORM;
    return dot_d(a, b, D) / (na * nb);
}

/*
 * One OIM pass along one axis of a batch of grids.
 *
 *   x         [B,H,W,D] fp64 (bf16 / fp32 inputs are widened by the caller)
 *   sizes_in  [B,H,W] or NULL (= all ones)
 *   axis      1: lines are rows, W -> W-m;  0: lines are columns, H -> H-m
 *   m         sources merged per line, 0 <= m <= ceil(len/2), len-m >= 1
 *   R         candidate radius: destinations b with |b-a| <= 2R-1; R <= 0
 *             means the whole line
 *   round_mode  storage type the pass output is rounded to (see round_to_io)
 *   x_out     [B,H',W',D]; sizes_out [B,H',W']
 *   merged_map [B,H*W]  input flat index -> output flat slot
 *   kept_map   [B,H'*W'] output slot -> input flat index of the survivor
 *              (for a merged group: its destination)
 *   margin    in/out: lowered to the smallest gap seen between a winning and
 *             a losing alternative of any decision (best-candidate choice and
 *             the m-th / (m+1)-th source score of a line); may be NULL
 * returns 0, or -1 on invalid arguments.
 */
int oracle_oim_pass(const double *x, const int64_t *sizes_in,
                    int B, int H, int W, int D, int axis, int m, int R,
                    int round_mode,
                    double *x_out, int64_t *sizes_out,
                    int32_t *merged_map, int32_t *kept_map, double *margin)
{
    if (B < 0 || H < 1 || W < 1 || D < 1 || (axis != 0 && axis != 1)) return -1;
    const int len = axis ? W : H;          /* tokens on a line            */
    const int nlines = axis ? H : W;       /* lines per image             */
    const int n_src = (len + 1) / 2;       /* even positions 0,2,4,...    */
    if (m < 0 || m > n_src || len - m < 1) return -1;
    const int Ho = axis ? H : H - m, Wo = axis ? W - m : W;
    double global_margin = margin ? *margin : INFINITY;

#pragma omp parallel for schedule(dynamic) reduction(min : global_margin)
    for (int64_t job = 0; job < (int64_t)B * nlines; ++job) {
        const int b = (int)(job / nlines), line = (int)(job % nlines);
        /* flat index (inside the image) of position p on this line */
#define IN_FLAT(p)  (axis ? (int64_t)line * W + (p) : (int64_t)(p) * W + line)
#define OUT_FLAT(q) (axis ? (int64_t)line * Wo + (q) : (int64_t)(q) * Wo + line)
        const double *img = x + (int64_t)b * H * W * D;
        const int64_t *simg = sizes_in ? sizes_in + (int64_t)b * H * W : NULL;

        int *best = (int *)malloc(sizeof(int) * (size_t)len);      /* per source position */
        double *score = (double *)malloc(sizeof(double) * (size_t)len);
        char *merged = (char *)calloc((size_t)len, 1);
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);

        /* similarity + matching: every source picks its most similar candidate */
        for (int a = 0; a < len; a += 2) {
            best[a] = -1;
            score[a] = -INFINITY;
            double runner = -INFINITY;
            for (int c = 1; c < len; c += 2) {                      /* ascending: tie -> lower c */
                int dist = c > a ? c - a : a - c;
                if (R > 0 && dist > 2 * R - 1) continue;
                double s = cosine(img + IN_FLAT(a) * D, img + IN_FLAT(c) * D, D);
                if (s > score[a]) { runner = score[a]; score[a] = s; best[a] = c; }
                else if (s > runner) runner = s;
            }
            if (best[a] >= 0 && runner > -INFINITY && score[a] - runner < global_margin)
                global_margin = score[a] - runner;
        }
        /* the m sources with the highest score are merged (tie -> lower position);
         * a source without any candidate (len == 1) can never be merged          */
        for (int pick = 0; pick < m; ++pick) {
            int arg = -1;
            for (int a = 0; a < len; a += 2)
                if (!merged[a] && best[a] >= 0 && (arg < 0 || score[a] > score[arg])) arg = a;
            if (arg < 0) break;        /* cannot happen for validated m: every source of a line with len >= 2 has a candidate */
            merged[arg] = 1;
        }
        if (m > 0 && m < n_src) {          /* gap between last merged and best unmerged */
            double lo_in = INFINITY, hi_out = -INFINITY;
            for (int a = 0; a < len; a += 2) {
                if (merged[a]) { if (score[a] < lo_in) lo_in = score[a]; }
                else if (best[a] >= 0 && score[a] > hi_out) hi_out = score[a];
            }
            if (lo_in - hi_out < global_margin) global_margin = lo_in - hi_out;
        }
        /* survivors in increasing position order */
        int q = 0;
        for (int p = 0; p < len; ++p) {
            if (merged[p]) continue;
            const int64_t s_p = simg ? simg[IN_FLAT(p)] : 1;
            int64_t S = s_p;
            for (int d = 0; d < D; ++d) acc[d] = (double)s_p * img[IN_FLAT(p) * D + d];
            if (p & 1) {                    /* destination: absorb the sources matched to it */
                for (int a = 0; a < len; a += 2) {
                    if (!merged[a] || best[a] != p) continue;
                    const int64_t s_a = simg ? simg[IN_FLAT(a)] : 1;
                    S += s_a;
                    for (int d = 0; d < D; ++d) acc[d] += (double)s_a * img[IN_FLAT(a) * D + d];
                }
            }
            double *o = x_out + ((int64_t)b * Ho * Wo + OUT_FLAT(q)) * D;
            if (S == s_p)                   /* nothing absorbed: the token passes through untouched */
                for (int d = 0; d < D; ++d) o[d] = round_to_io(img[IN_FLAT(p) * D + d], round_mode);
            else
                for (int d = 0; d < D; ++d) o[d] = round_to_io(acc[d] / (double)S, round_mode);
            sizes_out[(int64_t)b * Ho * Wo + OUT_FLAT(q)] = S;
            if (kept_map) kept_map[(int64_t)b * Ho * Wo + OUT_FLAT(q)] = (int32_t)IN_FLAT(p);
            if (merged_map) merged_map[(int64_t)b * H * W + IN_FLAT(p)] = (int32_t)OUT_FLAT(q);
            ++q;
        }
        /* merged sources land in the slot of their destination */
        if (merged_map)
            for (int a = 0; a < len; a += 2)
                if (merged[a])
                    merged_map[(int64_t)b * H * W + IN_FLAT(a)] =
                        merged_map[(int64_t)b * H * W + IN_FLAT(best[a])];
        free(best); free(score); free(merged); free(acc);
#undef IN_FLAT
#undef OUT_FLAT
    }
    if (margin) *margin = global_margin;
    return 0;
}

/*
 * A whole OIM call: passes[] = (axis, m) pairs applied in order; every pass
 * materialises its output in the I/O type before the next one reads it; the
 * two maps are composed so that they refer to the call's input grid.
 * x_out / sizes_out / kept_map are sized for the final grid, merged_map for
 * the input grid.  Returns 0 or -1.
 */
int oracle_oim_merge(const double *x, const int64_t *sizes_in,
                     int B, int H, int W, int D,
                     const int32_t *pass_axis, const int32_t *pass_m, int n_passes,
                     int R, int round_mode,
                     double *x_out, int64_t *sizes_out,
                     int32_t *merged_map, int32_t *kept_map, double *margin)
{
    if (n_passes < 0) return -1;
    const int64_t n_in = (int64_t)H * W;
    int h = H, w = W;
    double *cur = (double *)malloc(sizeof(double) * (size_t)(B * n_in * D + 1));
    int64_t *cur_s = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B * n_in + 1));
    int32_t *tot_merged = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_in + 1));
    int32_t *tot_kept = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_in + 1));
    memcpy(cur, x, sizeof(double) * (size_t)(B * n_in * D));
    for (int64_t i = 0; i < B * n_in; ++i) cur_s[i] = sizes_in ? sizes_in[i] : 1;
    for (int b = 0; b < B; ++b)
        for (int64_t p = 0; p < n_in; ++p) tot_merged[b * n_in + p] = tot_kept[b * n_in + p] = (int32_t)p;
    int rc = 0;
    for (int i = 0; i < n_passes && rc == 0; ++i) {
        const int axis = pass_axis[i], m = pass_m[i];
        const int ho = axis ? h : h - m, wo = axis ? w - m : w;
        if ((axis != 0 && axis != 1) || ho < 1 || wo < 1) { rc = -1; break; }
        const int64_t n_cur = (int64_t)h * w, n_new = (int64_t)ho * wo;
        double *nx = (double *)malloc(sizeof(double) * (size_t)(B * n_new * D + 1));
        int64_t *ns = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B * n_new + 1));
        int32_t *mm = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_cur + 1));
        int32_t *km = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_new + 1));
        rc = oracle_oim_pass(cur, cur_s, B, h, w, D, axis, m, R, round_mode, nx, ns, mm, km, margin);
        if (rc == 0) {
            /* input token p sat in slot t of the current grid; it moves on with t */
            for (int b = 0; b < B; ++b)
                for (int64_t p = 0; p < n_in; ++p)
                    tot_merged[b * n_in + p] = mm[b * n_cur + tot_merged[b * n_in + p]];
            int32_t *nk = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_in + 1));
            for (int b = 0; b < B; ++b)
                for (int64_t q = 0; q < n_new; ++q)
                    nk[b * n_in + q] = tot_kept[b * n_in + km[b * n_new + q]];
            free(tot_kept);
            tot_kept = nk;
        }
        free(cur); free(cur_s); free(mm); free(km);
        cur = nx; cur_s = ns; h = ho; w = wo;
    }
    if (rc == 0) {
        const int64_t n_out = (int64_t)h * w;
        memcpy(x_out, cur, sizeof(double) * (size_t)(B * n_out * D));
        memcpy(sizes_out, cur_s, sizeof(int64_t) * (size_t)(B * n_out));
        if (merged_map) memcpy(merged_map, tot_merged, sizeof(int32_t) * (size_t)(B * n_in));
        if (kept_map)
            for (int b = 0; b < B; ++b)
                memcpy(kept_map + b * n_out, tot_kept + b * n_in, sizeof(int32_t) * (size_t)n_out);
    }
    free(cur); free(cur_s); free(tot_merged); free(tot_kept);
    return rc;
}

/* ------------------------------------------------ OIM with a separate metric */

/*
 * The merge of one pass applied to a second tensor: the groups are those of
 * `merged_map` / `kept_map` of a pass that was decided on another tensor
 * (Section 3.1 counts the similarity cost in k, "the dimension of keys": the
 * similarity is taken on the keys, the merge is applied to the tokens).
 * Each output slot q receives the size-weighted mean of its group: the
 * anchor kept_map[q] first, then the other members in ascending flat index
 * (= ascending position on the line), exactly the order of oracle_oim_pass.
 *   y        [B,H,W,Dy];  y_out [B,Ho*Wo,Dy]
 */
int oracle_oim_apply(const double *y, const int64_t *sizes_in, int B, int H, int W, int Dy,
                     int n_out, const int32_t *merged_map, const int32_t *kept_map,
                     int round_mode, double *y_out)
{
    if (B < 0 || H < 1 || W < 1 || Dy < 1 || n_out < 1) return -1;
    const int64_t n_in = (int64_t)H * W;
    double *acc = (double *)malloc(sizeof(double) * (size_t)Dy);
    for (int b = 0; b < B; ++b) {
        for (int q = 0; q < n_out; ++q) {
            const int64_t p = kept_map[(int64_t)b * n_out + q];
            const int64_t s_p = sizes_in ? sizes_in[b * n_in + p] : 1;
            int64_t S = s_p;
            for (int d = 0; d < Dy; ++d) acc[d] = (double)s_p * y[(b * n_in + p) * Dy + d];
            for (int64_t a = 0; a < n_in; ++a) {
                if (a == p || merged_map[b * n_in + a] != q) continue;
                const int64_t s_a = sizes_in ? sizes_in[b * n_in + a] : 1;
                S += s_a;
                for (int d = 0; d < Dy; ++d) acc[d] += (double)s_a * y[(b * n_in + a) * Dy + d];
            }
            double *o = y_out + ((int64_t)b * n_out + q) * Dy;
            if (S == s_p)
                for (int d = 0; d < Dy; ++d) o[d] = round_to_io(y[(b * n_in + p) * Dy + d], round_mode);
            else
                for (int d = 0; d < Dy; ++d) o[d] = round_to_io(acc[d] / (double)S, round_mode);
        }
    }
    free(acc);
    return 0;
}

/*
 * A whole OIM call whose decisions are taken on `metric` [B,H,W,Dm] (the
 * keys) while `x` [B,H,W,D] follows: every pass is decided by
 * oracle_oim_pass on the current metric, its merge is applied to x with
 * oracle_oim_apply, both tensors are rounded to the I/O type after every
 * pass, maps are composed as in oracle_oim_merge.  metric_out may be NULL.
 */
int oracle_oim_merge_keyed(const double *x, const double *metric, const int64_t *sizes_in,
                           int B, int H, int W, int D, int Dm,
                           const int32_t *pass_axis, const int32_t *pass_m, int n_passes,
                           int R, int round_mode,
                           double *x_out, double *metric_out, int64_t *sizes_out,
                           int32_t *merged_map, int32_t *kept_map, double *margin)
{
    if (n_passes < 0) return -1;
    const int64_t n_in = (int64_t)H * W;
    int h = H, w = W;
    double *cx = (double *)malloc(sizeof(double) * (size_t)(B * n_in * D + 1));
    double *ck = (double *)malloc(sizeof(double) * (size_t)(B * n_in * Dm + 1));
    int64_t *cs = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B * n_in + 1));
    int32_t *tot_merged = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_in + 1));
    int32_t *tot_kept = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_in + 1));
    memcpy(cx, x, sizeof(double) * (size_t)(B * n_in * D));
    memcpy(ck, metric, sizeof(double) * (size_t)(B * n_in * Dm));
    for (int64_t i = 0; i < B * n_in; ++i) cs[i] = sizes_in ? sizes_in[i] : 1;
    for (int b = 0; b < B; ++b)
        for (int64_t p = 0; p < n_in; ++p) tot_merged[b * n_in + p] = tot_kept[b * n_in + p] = (int32_t)p;
    int rc = 0;
    for (int i = 0; i < n_passes && rc == 0; ++i) {
        const int axis = pass_axis[i], m = pass_m[i];
        const int ho = axis ? h : h - m, wo = axis ? w - m : w;
        if ((axis != 0 && axis != 1) || ho < 1 || wo < 1) { rc = -1; break; }
        const int64_t n_cur = (int64_t)h * w, n_new = (int64_t)ho * wo;
        double *nk_ = (double *)malloc(sizeof(double) * (size_t)(B * n_new * Dm + 1));
        double *nx = (double *)malloc(sizeof(double) * (size_t)(B * n_new * D + 1));
        int64_t *ns = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B * n_new + 1));
        int32_t *mm = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_cur + 1));
        int32_t *km = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_new + 1));
        rc = oracle_oim_pass(ck, cs, B, h, w, Dm, axis, m, R, round_mode, nk_, ns, mm, km, margin);
        if (rc == 0) rc = oracle_oim_apply(cx, cs, B, h, w, D, (int)n_new, mm, km, round_mode, nx);
        if (rc == 0) {
            for (int b = 0; b < B; ++b)
                for (int64_t p = 0; p < n_in; ++p)
                    tot_merged[b * n_in + p] = mm[b * n_cur + tot_merged[b * n_in + p]];
            int32_t *nk = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B * n_in + 1));
            for (int b = 0; b < B; ++b)
                for (int64_t q = 0; q < n_new; ++q)
                    nk[b * n_in + q] = tot_kept[b * n_in + km[b * n_new + q]];
            free(tot_kept);
            tot_kept = nk;
        }
        free(cx); free(ck); free(cs); free(mm); free(km);
        cx = nx; ck = nk_; cs = ns; h = ho; w = wo;
    }
    if (rc == 0) {
        const int64_t n_out = (int64_t)h * w;
        memcpy(x_out, cx, sizeof(double) * (size_t)(B * n_out * D));
        if (metric_out) memcpy(metric_out, ck, sizeof(double) * (size_t)(B * n_out * Dm));
        memcpy(sizes_out, cs, sizeof(int64_t) * (size_t)(B * n_out));
        if (merged_map) memcpy(merged_map, tot_merged, sizeof(int32_t) * (size_t)(B * n_in));
        if (kept_map)
            for (int b = 0; b < B; ++b)
                memcpy(kept_map + b * n_out, tot_kept + b * n_in, sizeof(int32_t) * (size_t)n_out);
    }
    free(cx); free(ck); free(cs); free(tot_merged); free(tot_kept);
    return rc;
}

/* ------------------------------------------------------- value enhancement */

/*
 * Eq. 3 (Section 3.2): the values that enter attention are V + log(s), s =
 * number of tokens merged into each token, added to every channel of the
 * token's row.   v [rows, D], s [rows] -> out [rows, D], rounded to the I/O type.
 */
int oracle_value_enhance(const double *v, const int64_t *s, int64_t rows, int D, int round_mode, double *out)
{
    if (rows < 0 || D < 1) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        if (s[r] < 1) return -1;
        const double ls = log((double)s[r]);
        for (int d = 0; d < D; ++d) out[r * D + d] = round_to_io(v[r * D + d] + ls, round_mode);
    }
    return 0;
}

/* --------------------------------------------------------------------- SPU */

/* Low-pass mask of Eq. 5 on bin k of an N-point spectrum. */
double oracle_spu_mask(int k, int N, int sigma, int use_hamming)
{
    const int f = k < N - k ? k : N - k;        /* folded frequency */
    if (f > sigma) return 0.0;
    if (!use_hamming || N == 1) return 1.0;
    return 0.54 + 0.46 * cos(2.0 * M_PI * (double)f / (double)(N - 1));
}

/* e^{sign * i 2 pi k n / N}; the product k*n is reduced mod N first so the
 * argument handed to cos/sin stays in [0, 2 pi).                            */
static void unit_root(int64_t k, int64_t n, int N, int sign, double *re, double *im)
{
    const int64_t r = (k * n) % N;
    const double th = 2.0 * M_PI * (double)r / (double)N;
    *re = cos(th);
    *im = sign * sin(th);
}

/*
 * Spectral score of every token: Eq. 4 (plain O(N^2) DFT along the token
 * index, one channel at a time), Eq. 5-6 (mask), Eq. 7 (inverse with 1/N),
 * Eq. 8 (L2 norm over channels).  Bins whose mask is zero are skipped - they
 * are multiplied by zero anyway.
 *   x [B,N,D] fp64;  scores [B,N];  filtered [B,N,D] or NULL (the real part
 *   of the inverse transform);  max_imag: largest |imaginary part| met in the
 *   inverse (a self-check: must vanish up to rounding), may be NULL.
 */
int oracle_spu_score(const double *x, int B, int N, int D, int sigma, int use_hamming,
                     double *scores, double *filtered, double *max_imag)
{
    if (B < 0 || N < 1 || D < 1 || sigma < 0 || sigma > N / 2) return -1;
    double worst_imag = 0.0;
#pragma omp parallel for schedule(dynamic) reduction(max : worst_imag)
    for (int b = 0; b < B; ++b) {
        const double *xb = x + (int64_t)b * N * D;
        double *Fr = (double *)calloc((size_t)N * D, sizeof(double));
        double *Fi = (double *)calloc((size_t)N * D, sizeof(double));
        /* Eq. 4 then Eq. 6 */
        for (int k = 0; k < N; ++k) {
            const double Mk = oracle_spu_mask(k, N, sigma, use_hamming);
            if (Mk == 0.0) continue;
            for (int n = 0; n < N; ++n) {
                double c, s;
                unit_root(k, n, N, -1, &c, &s);
                for (int d = 0; d < D; ++d) {
                    Fr[(int64_t)k * D + d] += xb[(int64_t)n * D + d] * c;
                    Fi[(int64_t)k * D + d] += xb[(int64_t)n * D + d] * s;
                }
            }
            for (int d = 0; d < D; ++d) { Fr[(int64_t)k * D + d] *= Mk; Fi[(int64_t)k * D + d] *= Mk; }
        }
        /* Eq. 7 and Eq. 8 */
        double *re = (double *)malloc(sizeof(double) * (size_t)D);
        double *im = (double *)malloc(sizeof(double) * (size_t)D);
        for (int n = 0; n < N; ++n) {
            memset(re, 0, sizeof(double) * (size_t)D);
            memset(im, 0, sizeof(double) * (size_t)D);
            for (int k = 0; k < N; ++k) {
                if (oracle_spu_mask(k, N, sigma, use_hamming) == 0.0) continue;
                double c, s;
                unit_root(k, n, N, +1, &c, &s);
                for (int d = 0; d < D; ++d) {
                    const double fr = Fr[(int64_t)k * D + d], fi = Fi[(int64_t)k * D + d];
                    re[d] += fr * c - fi * s;
                    im[d] += fr * s + fi * c;
                }
            }
            double e = 0.0;
            for (int d = 0; d < D; ++d) {
                const double v = re[d] / (double)N, w = fabs(im[d] / (double)N);
                if (filtered) filtered[((int64_t)b * N + n) * D + d] = v;
                if (w > worst_imag) worst_imag = w;
                e += v * v;
            }
            scores[(int64_t)b * N + n] = sqrt(e);
        }
        free(Fr); free(Fi); free(re); free(im);
    }
    if (max_imag) *max_imag = worst_imag;
    return 0;
}

/*
 * Order-preserving top-k keep (Algorithm 2, last two steps): the n_keep
 * largest scores, equal scores won by the lower index; indices returned in
 * ascending order; rows of the ORIGINAL x gathered when x / x_out are given.
 *   margin: in/out, lowered to the smallest relative gap between the last
 *   kept and the best dropped score of a sample; may be NULL.
 */
int oracle_spu_prune(const double *scores, const double *x, int B, int N, int D, int n_keep,
                     int32_t *kept_idx, double *x_out, double *margin)
{
    if (B < 0 || N < 1 || n_keep < 1 || n_keep > N) return -1;
    double worst = margin ? *margin : INFINITY;
    for (int b = 0; b < B; ++b) {
        const double *s = scores + (int64_t)b * N;
        char *taken = (char *)calloc((size_t)N, 1);
        double last = INFINITY;
        for (int pick = 0; pick < n_keep; ++pick) {       /* selection by repeated arg-max */
            int arg = -1;
            for (int n = 0; n < N; ++n)                   /* ascending scan + strict '>' : tie -> lower n */
                if (!taken[n] && (arg < 0 || s[n] > s[arg])) arg = n;
            taken[arg] = 1;
            last = s[arg];
        }
        if (n_keep < N) {
            double next = -INFINITY;
            for (int n = 0; n < N; ++n) if (!taken[n] && s[n] > next) next = s[n];
            const double scale = fabs(last) > 0 ? fabs(last) : 1.0;
            if ((last - next) / scale < worst) worst = (last - next) / scale;
        }
        int q = 0;
        for (int n = 0; n < N; ++n) {
            if (!taken[n]) continue;
            kept_idx[(int64_t)b * n_keep + q] = n;
            if (x && x_out)
                memcpy(x_out + ((int64_t)b * n_keep + q) * D, x + ((int64_t)b * N + n) * D,
                       sizeof(double) * (size_t)D);
            ++q;
        }
        free(taken);
    }
    if (margin) *margin = worst;
    return 0;
}

/* floor(ratio*N + 0.5) clamped to [1, N] */
int oracle_keep_count(int N, double keep_ratio)
{
    int k = (int)floor(keep_ratio * (double)N + 0.5);
    if (k < 1) k = 1;
    if (k > N) k = N;
    return k;
}
