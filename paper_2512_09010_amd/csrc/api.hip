// C ABI of libluvc (declared in include/luvc.h): argument validation, workspace carving and
// dispatch to the gfx950 kernels.  Every check happens before the first launch, so a failing
// call enqueues nothing.
#include <cstdarg>
#include <cstdio>
#include <cmath>

#include "common.hpp"
#include "oim.hpp"
#include "spu.hpp"

namespace luvc {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

luvc_status check_launch(const char* what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: %s", what, hipGetErrorString(e));
        return LUVC_ERR_HIP;
    }
    return LUVC_OK;
}

// ---- timing aid: events handed over by the caller, two per launch
static thread_local hipEvent_t* g_prof_ev = nullptr;
static thread_local int g_prof_cap = 0, g_prof_n = 0;
constexpr int kProfMax = 8192;
static thread_local const char* g_prof_name[kProfMax];

bool prof_take(const char* kernel, hipEvent_t* start, hipEvent_t* stop)
{
    if (!g_prof_ev || g_prof_n >= g_prof_cap || g_prof_n >= kProfMax) return false;
    const int slot = g_prof_n++;
    g_prof_name[slot] = kernel;
    *start = g_prof_ev[2 * slot];
    *stop = g_prof_ev[2 * slot + 1];
    return true;
}

static bool dtype_ok(luvc_dtype dt) { return dt == LUVC_F32 || dt == LUVC_BF16; }
static size_t esize(luvc_dtype dt) { return dt == LUVC_F32 ? 4 : 2; }

// Shapes along a schedule; returns false (with an error message) on an invalid one.
struct OimPlan {
    int n;
    int h[kMaxPasses + 1], w[kMaxPasses + 1];     // grid before pass i (and after the last one)
};

static bool walk_schedule(int B, int H, int W, int D, const luvc_oim_pass* passes, int n_passes, OimPlan* pl)
{
    if (B < 1 || H < 1 || W < 1 || D < 1) { set_error("B, H, W, D must be positive (got %d,%d,%d,%d)", B, H, W, D); return false; }
    if ((int64_t)B * H * W >= ((int64_t)1 << 31)) { set_error("B*H*W must stay below 2^31"); return false; }
    if (!passes || n_passes < 1 || n_passes > kMaxPasses) { set_error("need 1..%d passes", kMaxPasses); return false; }
    pl->n = n_passes;
    pl->h[0] = H;
    pl->w[0] = W;
    for (int i = 0; i < n_passes; ++i) {
        const int axis = passes[i].axis, m = passes[i].m;
        if (axis != 0 && axis != 1) { set_error("pass %d: axis must be 0 (H) or 1 (W)", i); return false; }
        const int len = axis ? pl->w[i] : pl->h[i];
        if (len > kMaxLineLen) { set_error("pass %d: line length %d exceeds %d", i, len, kMaxLineLen); return false; }
        if (m < 0 || m > (len + 1) / 2 || len - m < 1) {
            set_error("pass %d: m=%d is outside 0..ceil(%d/2) or leaves no token", i, m, len);
            return false;
        }
        pl->h[i + 1] = axis ? pl->h[i] : pl->h[i] - m;
        pl->w[i + 1] = axis ? pl->w[i] - m : pl->w[i];
    }
    return true;
}

struct OimLayout {
    size_t xbuf[2], sbuf[2], kbuf[2], maps[kMaxPasses], n2, dn, anchor, absorb, gram, srcdest, lazy_idx[2], lazy_ov, bytes;
    int lazy_cap;      // overlay rows per image (wide matching with one launch per pass)
};

static OimLayout oim_layout(int B, int D, luvc_dtype dt, const OimPlan& pl, const luvc_oim_pass* passes = nullptr, int radius = 1)
{
    OimLayout L{};
    size_t off = 0;
    // ping-pong buffers for the outputs of all launches but the last.  Launch s (one pass, or two passes fused) writes
    // buffer s & 1; which passes fuse is decided later, so both buffers hold the largest intermediate grid
    size_t tok[2] = {0, 0};
    for (int i = 0; i + 1 < pl.n; ++i) {
        const size_t t = (size_t)B * pl.h[i + 1] * pl.w[i + 1];
        if (t > tok[0]) tok[0] = tok[1] = t;
    }
    for (int j = 0; j < 2; ++j) {
        L.xbuf[j] = off; off += align_up(tok[j] * D * esize(dt));
        L.sbuf[j] = off; off += align_up(tok[j] * sizeof(int32_t));
        L.kbuf[j] = off; off += align_up(tok[j] * sizeof(int32_t));
    }
    size_t max_in = 0, max_out = 0;
    for (int i = 0; i < pl.n; ++i) {
        const size_t tin = (size_t)B * pl.h[i] * pl.w[i], tout = (size_t)B * pl.h[i + 1] * pl.w[i + 1];
        L.maps[i] = off; off += align_up(tin * sizeof(int32_t));
        if (tin > max_in) max_in = tin;
        if (tout > max_out) max_out = tout;
    }
    L.n2 = off;     off += align_up(max_in * sizeof(double));
    L.dn = off;     off += align_up(max_in * sizeof(double));
    L.anchor = off; off += align_up(max_out * sizeof(int32_t));
    L.absorb = off; off += align_up(max_out * sizeof(int32_t));
    // wide matching: the largest source x destination matrix set and merge list of any pass
    size_t gram = 0, srcdest = 0;
    if (radius != 1 && passes)
        for (int i = 0; i < pl.n; ++i) {
            const size_t gb = oim_wide_gram_bytes(B, pl.h[i], pl.w[i], passes[i].axis), sb = oim_wide_srcdest_bytes(B, pl.h[i], pl.w[i], passes[i].axis);
            if (gb > gram) gram = gb;
            if (sb > srcdest) srcdest = sb;
        }
    L.gram = off;    off += align_up(gram);
    L.srcdest = off; off += align_up(srcdest);
    // wide matching with one launch per pass: two grids of row ids and the rows of the merged destinations
    // (whether a call can run that way depends on the alignment of its buffers, so the space is always there)
    int64_t cap = 0;
    if (radius != 1 && passes)
        for (int i = 0; i < pl.n; ++i) cap += oim_wide_lazy_rows(pl.h[i], pl.w[i], passes[i].axis, passes[i].m);
    L.lazy_cap = (int)cap;
    for (int j = 0; j < 2; ++j) {
        L.lazy_idx[j] = off;
        off += (radius != 1 && passes) ? align_up((size_t)B * pl.h[0] * pl.w[0] * sizeof(int32_t)) : 0;
    }
    L.lazy_ov = off; off += align_up((size_t)B * (size_t)cap * D * esize(dt));
    L.bytes = off;
    return L;
}

bool workspace_ok(const void* ws, size_t have, size_t need)
{
    if (need == 0) return true;
    if (!ws) { set_error("workspace is NULL but %zu bytes are needed", need); return false; }
    if ((uintptr_t)ws % 256 != 0) { set_error("workspace must be 256-byte aligned"); return false; }
    if (have < need) { set_error("workspace holds %zu bytes, %zu are needed", have, need); return false; }
    return true;
}

}  // namespace luvc

using namespace luvc;

extern "C" {

const char* luvc_version(void) { return "libluvc 0.1 (gfx950)"; }

const char* luvc_last_error(void) { return g_err; }

luvc_status luvc_profile_start(void** hip_events, int n_events)
{
    if (!hip_events || n_events < 2 || (n_events & 1)) { set_error("luvc_profile_start needs an even number of events"); return LUVC_ERR_INVALID_ARG; }
    g_prof_ev = reinterpret_cast<hipEvent_t*>(hip_events);
    g_prof_cap = n_events / 2;
    g_prof_n = 0;
    return LUVC_OK;
}

int luvc_profile_stop(void)
{
    const int n = g_prof_n;
    g_prof_ev = nullptr;
    g_prof_cap = 0;
    return n;
}

const char* luvc_profile_kernel(int i) { return (i >= 0 && i < g_prof_n) ? g_prof_name[i] : ""; }

luvc_status luvc_oim_plan(int H, int W, int64_t target_tokens, luvc_oim_pass* passes, int max_passes, int* n_passes)
{
    if (!passes || !n_passes || max_passes < 1) { set_error("passes / n_passes must be given"); return LUVC_ERR_INVALID_ARG; }
    if (H < 1 || W < 1 || target_tokens < 1 || target_tokens > (int64_t)H * W) {
        set_error("target_tokens must lie in 1..H*W");
        return LUVC_ERR_INVALID_ARG;
    }
    int h = H, w = W, n = 0, axis = 1;
    while ((int64_t)h * w > target_tokens) {
        if (n >= max_passes) { set_error("schedule needs more than %d passes", max_passes); return LUVC_ERR_INVALID_ARG; }
        int len = axis ? w : h;
        const int other = axis ? h : w;
        if (len == 1) {                      // nothing left on this axis: try the other one
            axis ^= 1;
            len = axis ? w : h;
            if (len == 1) break;
            continue;
        }
        int m = (len + 1) / 2;
        if ((int64_t)(len - m) * other < target_tokens) {
            // the exact m on this axis, if the other side divides the target
            if (target_tokens % other != 0) { set_error("target %lld is not reachable from %dx%d", (long long)target_tokens, h, w); return LUVC_ERR_INVALID_ARG; }
            m = len - (int)(target_tokens / other);
        }
        passes[n].axis = axis;
        passes[n].m = m;
        ++n;
        if (axis) w -= m; else h -= m;
        axis ^= 1;
    }
    if ((int64_t)h * w != target_tokens) { set_error("target %lld is not reachable", (long long)target_tokens); return LUVC_ERR_INVALID_ARG; }
    *n_passes = n;
    return LUVC_OK;
}

size_t luvc_oim_workspace_bytes(int B, int H, int W, int D, luvc_dtype dtype, const luvc_oim_pass* passes, int n_passes)
{
    OimPlan pl;
    if (!dtype_ok(dtype) || !walk_schedule(B, H, W, D, passes, n_passes, &pl)) return 0;
    return oim_layout(B, D, dtype, pl).bytes;
}

static luvc_status oim_merge_impl(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dtype,
                                  const luvc_oim_pass* passes, int n_passes, int radius, int64_t target_tokens,
                                  void* x_out, int32_t* sizes_out, int32_t* merged_map, int32_t* kept_map,
                                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!dtype_ok(dtype)) { set_error("unknown dtype %d", (int)dtype); return LUVC_ERR_INVALID_ARG; }
    if (!x || !x_out || !sizes_out) { set_error("x, x_out and sizes_out must not be NULL"); return LUVC_ERR_INVALID_ARG; }
    OimPlan pl;
    if (!walk_schedule(B, H, W, D, passes, n_passes, &pl)) return LUVC_ERR_INVALID_ARG;
    const int Ho = pl.h[pl.n], Wo = pl.w[pl.n];
    if (target_tokens != 0 && target_tokens != (int64_t)Ho * Wo) {
        set_error("schedule ends at %dx%d = %lld tokens, target is %lld", Ho, Wo, (long long)Ho * Wo, (long long)target_tokens);
        return LUVC_ERR_INVALID_ARG;
    }
    if (radius < 0) { set_error("radius must be 0 (whole line) or positive"); return LUVC_ERR_INVALID_ARG; }
    if (radius != 1)
        for (int i = 0; i < pl.n; ++i)
            if ((passes[i].axis ? pl.w[i] : pl.h[i]) > kMaxWideLineLen) {
                set_error("pass %d: wide matching supports lines of at most %d tokens", i, kMaxWideLineLen);
                return LUVC_ERR_UNSUPPORTED;
            }
    if (radius != 1 && (int64_t)H * W * D * (int64_t)esize(dtype) >= ((int64_t)1 << 31)) {
        set_error("wide matching supports grids of less than 2 GiB per image");
        return LUVC_ERR_UNSUPPORTED;
    }
    const OimLayout L = oim_layout(B, D, dtype, pl, passes, radius);
    if (!workspace_ok(workspace, workspace_bytes, L.bytes)) return LUVC_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const size_t es = esize(dtype);
    // 16-byte accesses need aligned rows in every buffer the kernels touch
    const bool vec = ((size_t)D * es) % 16 == 0 && (uintptr_t)x % 16 == 0 && (uintptr_t)x_out % 16 == 0;

    bool lazy = radius != 1 && vec && (int64_t)H * W + L.lazy_cap < ((int64_t)1 << 31);
    for (int i = 0; i < pl.n; ++i)
        if ((passes[i].axis ? pl.w[i] : pl.h[i]) > kLazyMaxLen) lazy = false;
    if (lazy) {
        // one launch per pass on grids of row ids, the tokens move once at the end
        const int32_t *cur_i = nullptr, *cur_sz = sizes_in, *cur_kp = nullptr;
        const int32_t* lmaps[kMaxPasses];
        int32_t ln_in[kMaxPasses];
        int ov_base = 0;
        for (int i = 0; i < pl.n; ++i) {
            const bool last = i + 1 == pl.n;
            int32_t* oi = (int32_t*)(ws + L.lazy_idx[i & 1]);
            int32_t* os = last ? sizes_out : (int32_t*)(ws + L.sbuf[i & 1]);
            int32_t* ok = last ? kept_map : (int32_t*)(ws + L.kbuf[i & 1]);
            int32_t* pm = merged_map ? ((pl.n == 1) ? merged_map : (int32_t*)(ws + L.maps[i])) : nullptr;
            lmaps[i] = pm;
            ln_in[i] = pl.h[i] * pl.w[i];
            const luvc_status rc = oim_wide_lazy_pass(x, ws + L.lazy_ov, nullptr, nullptr, 0, cur_i, cur_sz, cur_kp, B, H * W, pl.h[i], pl.w[i], D, dtype,
                                                      passes[i].axis, passes[i].m, radius, L.lazy_cap, ov_base, oi, os, ok, pm, st);
            if (rc != LUVC_OK) return rc;
            ov_base += oim_wide_lazy_rows(pl.h[i], pl.w[i], passes[i].axis, passes[i].m);
            cur_i = oi;
            cur_sz = os;
            cur_kp = ok;
        }
        const luvc_status rc = oim_wide_lazy_gather(x, ws + L.lazy_ov, cur_i, B, H * W, L.lazy_cap, Ho * Wo, D, dtype, x_out, st);
        if (rc != LUVC_OK) return rc;
        if (merged_map && pl.n > 1) return oim_compose(lmaps, ln_in, pl.n, B, H * W, merged_map, st);
        return LUVC_OK;
    }

    OimScratch sc;
    sc.n2 = (double*)(ws + L.n2);
    sc.dn = (double*)(ws + L.dn);
    sc.anchor = (int32_t*)(ws + L.anchor);
    sc.absorb = (int32_t*)(ws + L.absorb);

    const void* cur_x = x;
    const int32_t* cur_s = sizes_in;
    const int32_t* cur_k = nullptr;
    // launches of the call: a pair of halving passes on different axes runs as one launch
    struct Step { int first, count; };
    Step steps[kMaxPasses];
    int n_steps = 0;
    for (int i = 0; i < pl.n;) {
        const bool pair = radius == 1 && i + 1 < pl.n && oim_pair_supported(pl.h[i], pl.w[i], D, dtype, passes[i].axis, passes[i].m,
                                                             passes[i + 1].axis, passes[i + 1].m, vec);
        steps[n_steps++] = Step{i, pair ? 2 : 1};
        i += pair ? 2 : 1;
    }
    const int32_t* maps[kMaxPasses];
    int32_t n_in[kMaxPasses];
    for (int s = 0; s < n_steps; ++s) {
        const int i = steps[s].first, e = i + steps[s].count - 1;          // passes i..e
        const bool last = e + 1 == pl.n;
        // by launch, not by pass: a fused pair after a single pass would otherwise read and write the same buffer
        void* ox = last ? x_out : (void*)(ws + L.xbuf[s & 1]);
        int32_t* os = last ? sizes_out : (int32_t*)(ws + L.sbuf[s & 1]);
        int32_t* ok = last ? kept_map : (int32_t*)(ws + L.kbuf[s & 1]);
        // a call that is a single launch writes its map straight to the caller
        int32_t* pm = (n_steps == 1 && merged_map) ? merged_map : (int32_t*)(ws + L.maps[i]);
        maps[s] = pm;
        n_in[s] = pl.h[i] * pl.w[i];
        luvc_status rc;
        if (radius != 1)
            rc = oim_wide_pass(cur_x, cur_s, B, pl.h[i], pl.w[i], D, dtype, passes[i].axis, passes[i].m, radius, vec,
                               ox, os, pm, cur_k, ok, sc, (double*)(ws + L.gram), (int32_t*)(ws + L.srcdest), st);
        else if (steps[s].count == 2)
            rc = oim_pair_pass(cur_x, cur_s, B, pl.h[i], pl.w[i], D, dtype, passes[i].axis, ox, os, pm, cur_k, ok, st);
        else if (oim_halve_supported(pl.h[i], pl.w[i], D, dtype, passes[i].axis, passes[i].m, vec))
            rc = oim_halve_pass(cur_x, cur_s, B, pl.h[i], pl.w[i], D, dtype, passes[i].axis, ox, os, pm, cur_k, ok, st);
        else
            rc = oim_general_pass(cur_x, cur_s, B, pl.h[i], pl.w[i], D, dtype, passes[i].axis, passes[i].m, vec,
                                  ox, os, pm, cur_k, ok, sc, st);
        if (rc != LUVC_OK) return rc;
        cur_x = ox;
        cur_s = os;
        cur_k = ok;
    }
    if (merged_map && n_steps > 1) return oim_compose(maps, n_in, n_steps, B, H * W, merged_map, st);
    return LUVC_OK;
}

luvc_status luvc_oim_merge(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dtype,
                           const luvc_oim_pass* passes, int n_passes, int64_t target_tokens,
                           void* x_out, int32_t* sizes_out, int32_t* merged_map, int32_t* kept_map,
                           void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return oim_merge_impl(x, sizes_in, B, H, W, D, dtype, passes, n_passes, 1, target_tokens, x_out, sizes_out, merged_map, kept_map,
                          workspace, workspace_bytes, hip_stream);
}

size_t luvc_oim_wide_workspace_bytes(int B, int H, int W, int D, luvc_dtype dtype, const luvc_oim_pass* passes, int n_passes, int radius)
{
    OimPlan pl;
    if (!dtype_ok(dtype) || radius < 0 || !walk_schedule(B, H, W, D, passes, n_passes, &pl)) return 0;
    return oim_layout(B, D, dtype, pl, passes, radius).bytes;
}

luvc_status luvc_oim_merge_wide(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dtype,
                                const luvc_oim_pass* passes, int n_passes, int radius, int64_t target_tokens,
                                void* x_out, int32_t* sizes_out, int32_t* merged_map, int32_t* kept_map,
                                void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return oim_merge_impl(x, sizes_in, B, H, W, D, dtype, passes, n_passes, radius, target_tokens, x_out, sizes_out, merged_map, kept_map,
                          workspace, workspace_bytes, hip_stream);
}

// ---- OIM decided on a separate metric tensor: a pair of halving passes is one launch (oim_pair_keyed.hip), any other pass
// runs its decisions and its two merges (features, metric) as separate stages on the general kernels
struct KeyedLayout {
    OimLayout base;
    size_t mbuf[2], mov, bytes;     // ping-pong buffers of the merged metric between passes; overlay of the metric (one launch per pass)
};

static KeyedLayout keyed_layout(int B, int D, int Dm, luvc_dtype dt, const OimPlan& pl, const luvc_oim_pass* passes, int radius)
{
    KeyedLayout K;
    // the wide-matching scratch is sized by oim_layout when radius != 1; a radius of 1 needs none
    K.base = oim_layout(B, D, dt, pl, passes, radius);
    size_t off = K.base.bytes;
    size_t tok[2] = {0, 0};
    // launch s (one pass, or two passes fused) writes buffer s & 1; which passes fuse depends on the alignment of the
    // caller's buffers, so both hold the largest grid any pass writes (the last one too: metric_out may be NULL)
    for (int i = 0; i < pl.n; ++i) {
        const size_t t = (size_t)B * pl.h[i + 1] * pl.w[i + 1];
        if (t > tok[0]) tok[0] = tok[1] = t;
    }
    for (int j = 0; j < 2; ++j) { K.mbuf[j] = off; off += align_up(tok[j] * Dm * esize(dt)); }
    K.mov = off; off += align_up((size_t)B * (size_t)K.base.lazy_cap * Dm * esize(dt));
    K.bytes = off;
    return K;
}

static bool keyed_args_ok(int radius, int Dm)
{
    if (radius < 0) { set_error("radius must be 0 (whole line) or positive"); return false; }
    if (Dm < 1) { set_error("Dm must be positive (got %d)", Dm); return false; }
    return true;
}

size_t luvc_oim_keyed_workspace_bytes(int B, int H, int W, int D, int Dm, luvc_dtype dtype, const luvc_oim_pass* passes, int n_passes, int radius)
{
    OimPlan pl;
    if (!dtype_ok(dtype) || radius < 0 || Dm < 1 || !walk_schedule(B, H, W, D, passes, n_passes, &pl)) return 0;
    return keyed_layout(B, D, Dm, dtype, pl, passes, radius).bytes;
}

luvc_status luvc_oim_merge_keyed(const void* x, const void* metric, const int32_t* sizes_in,
                                 int B, int H, int W, int D, int Dm, luvc_dtype dtype,
                                 const luvc_oim_pass* passes, int n_passes, int radius, int64_t target_tokens,
                                 void* x_out, void* metric_out, int32_t* sizes_out, int32_t* merged_map, int32_t* kept_map,
                                 void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!dtype_ok(dtype)) { set_error("unknown dtype %d", (int)dtype); return LUVC_ERR_INVALID_ARG; }
    if (!x || !metric || !x_out || !sizes_out) { set_error("x, metric, x_out and sizes_out must not be NULL"); return LUVC_ERR_INVALID_ARG; }
    if (!keyed_args_ok(radius, Dm)) return LUVC_ERR_INVALID_ARG;
    OimPlan pl;
    if (!walk_schedule(B, H, W, D, passes, n_passes, &pl)) return LUVC_ERR_INVALID_ARG;
    const int Ho = pl.h[pl.n], Wo = pl.w[pl.n];
    if (target_tokens != 0 && target_tokens != (int64_t)Ho * Wo) {
        set_error("schedule ends at %dx%d = %lld tokens, target is %lld", Ho, Wo, (long long)Ho * Wo, (long long)target_tokens);
        return LUVC_ERR_INVALID_ARG;
    }
    if (radius != 1) {
        for (int i = 0; i < pl.n; ++i)
            if ((passes[i].axis ? pl.w[i] : pl.h[i]) > kMaxWideLineLen) {
                set_error("pass %d: wide matching supports lines of at most %d tokens", i, kMaxWideLineLen);
                return LUVC_ERR_UNSUPPORTED;
            }
        if ((int64_t)H * W * Dm * (int64_t)esize(dtype) >= ((int64_t)1 << 31)) {
            set_error("wide matching supports grids of less than 2 GiB per image");
            return LUVC_ERR_UNSUPPORTED;
        }
    }
    const KeyedLayout K = keyed_layout(B, D, Dm, dtype, pl, passes, radius);
    const OimLayout& L = K.base;
    if (!workspace_ok(workspace, workspace_bytes, K.bytes)) return LUVC_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const size_t es = esize(dtype);
    const bool vec_x = ((size_t)D * es) % 16 == 0 && (uintptr_t)x % 16 == 0 && (uintptr_t)x_out % 16 == 0;
    const bool vec_m = ((size_t)Dm * es) % 16 == 0 && (uintptr_t)metric % 16 == 0 && (!metric_out || (uintptr_t)metric_out % 16 == 0);
    OimScratch sc;
    sc.n2 = (double*)(ws + L.n2);
    sc.dn = (double*)(ws + L.dn);
    sc.anchor = (int32_t*)(ws + L.anchor);
    sc.absorb = (int32_t*)(ws + L.absorb);
    double* G = (double*)(ws + L.gram);
    int32_t* src_dest = (int32_t*)(ws + L.srcdest);

    bool lazy = radius != 1 && vec_x && vec_m && (int64_t)H * W + L.lazy_cap < ((int64_t)1 << 31);
    for (int i = 0; i < pl.n; ++i)
        if ((passes[i].axis ? pl.w[i] : pl.h[i]) > kLazyMaxLen) lazy = false;
    if (lazy) {
        // wide matching on the metric, one launch per pass on grids of row ids; tokens and metric move once at the end
        const int32_t *cur_i = nullptr, *cur_sz = sizes_in, *cur_kp = nullptr;
        const int32_t* lmaps[kMaxPasses];
        int32_t ln_in[kMaxPasses];
        int ov_base = 0;
        for (int i = 0; i < pl.n; ++i) {
            const bool last = i + 1 == pl.n;
            int32_t* oi = (int32_t*)(ws + L.lazy_idx[i & 1]);
            int32_t* os = last ? sizes_out : (int32_t*)(ws + L.sbuf[i & 1]);
            int32_t* ok = last ? kept_map : (int32_t*)(ws + L.kbuf[i & 1]);
            int32_t* pm = merged_map ? ((pl.n == 1) ? merged_map : (int32_t*)(ws + L.maps[i])) : nullptr;
            lmaps[i] = pm;
            ln_in[i] = pl.h[i] * pl.w[i];
            const luvc_status rc = oim_wide_lazy_pass(x, ws + L.lazy_ov, metric, ws + K.mov, Dm, cur_i, cur_sz, cur_kp, B, H * W, pl.h[i], pl.w[i],
                                                      D, dtype, passes[i].axis, passes[i].m, radius, L.lazy_cap, ov_base, oi, os, ok, pm, st);
            if (rc != LUVC_OK) return rc;
            ov_base += oim_wide_lazy_rows(pl.h[i], pl.w[i], passes[i].axis, passes[i].m);
            cur_i = oi;
            cur_sz = os;
            cur_kp = ok;
        }
        luvc_status rc = oim_wide_lazy_gather(x, ws + L.lazy_ov, cur_i, B, H * W, L.lazy_cap, Ho * Wo, D, dtype, x_out, st);
        if (rc != LUVC_OK) return rc;
        if (metric_out) {
            rc = oim_wide_lazy_gather(metric, ws + K.mov, cur_i, B, H * W, L.lazy_cap, Ho * Wo, Dm, dtype, metric_out, st);
            if (rc != LUVC_OK) return rc;
        }
        if (merged_map && pl.n > 1) return oim_compose(lmaps, ln_in, pl.n, B, H * W, merged_map, st);
        return LUVC_OK;
    }

    const void *cur_x = x, *cur_m = metric;
    const int32_t* cur_s = sizes_in;
    const int32_t* cur_k = nullptr;
    // launches of the call: a pair of halving passes on different axes with adjacent matching runs as one launch
    struct Step { int first, count; };
    Step steps[kMaxPasses];
    int n_steps = 0;
    for (int i = 0; i < pl.n;) {
        const bool pair = radius == 1 && i + 1 < pl.n &&
                          oim_pair_keyed_supported(pl.h[i], pl.w[i], D, Dm, dtype, passes[i].axis, passes[i].m, passes[i + 1].axis, passes[i + 1].m, vec_x, vec_m);
        steps[n_steps++] = Step{i, pair ? 2 : 1};
        i += pair ? 2 : 1;
    }
    const int32_t* maps[kMaxPasses];
    int32_t n_in[kMaxPasses];
    for (int s = 0; s < n_steps; ++s) {
        const int i = steps[s].first, e = i + steps[s].count - 1;          // passes i..e
        const bool last = e + 1 == pl.n;
        const int h = pl.h[i], w = pl.w[i], axis = passes[i].axis, m = passes[i].m;
        void* ox = last ? x_out : (void*)(ws + L.xbuf[s & 1]);
        void* om = (last && metric_out) ? metric_out : (void*)(ws + K.mbuf[s & 1]);
        int32_t* os = last ? sizes_out : (int32_t*)(ws + L.sbuf[s & 1]);
        int32_t* ok = last ? kept_map : (int32_t*)(ws + L.kbuf[s & 1]);
        int32_t* pm = (n_steps == 1 && merged_map) ? merged_map : (int32_t*)(ws + L.maps[i]);
        maps[s] = pm;
        n_in[s] = h * w;
        luvc_status rc;
        if (steps[s].count == 2) {
            rc = oim_pair_keyed_pass(cur_x, cur_m, cur_s, B, h, w, D, Dm, dtype, axis, ox, (last && !metric_out) ? nullptr : om, os, pm, cur_k, ok, st);
            if (rc != LUVC_OK) return rc;
        } else {
            if (radius == 1) rc = oim_general_decide(cur_m, B, h, w, Dm, dtype, axis, m, vec_m, pm, sc, st);
            else             rc = oim_wide_decide(cur_m, B, h, w, Dm, dtype, axis, m, radius, vec_m, pm, sc, G, src_dest, st);
            if (rc != LUVC_OK) return rc;
            if (radius == 1) rc = oim_general_apply(cur_x, cur_s, B, h, w, D, dtype, axis, m, vec_x, ox, os, cur_k, ok, sc, st);
            else             rc = oim_wide_apply(cur_x, cur_s, B, h, w, D, dtype, axis, m, vec_x, ox, os, cur_k, ok, sc, src_dest, st);
            if (rc != LUVC_OK) return rc;
            if (!last || metric_out) {               // the metric follows its own decisions (sizes and anchors are written again, same values)
                if (radius == 1) rc = oim_general_apply(cur_m, cur_s, B, h, w, Dm, dtype, axis, m, vec_m, om, os, nullptr, nullptr, sc, st);
                else             rc = oim_wide_apply(cur_m, cur_s, B, h, w, Dm, dtype, axis, m, vec_m, om, os, nullptr, nullptr, sc, src_dest, st);
                if (rc != LUVC_OK) return rc;
            }
        }
        cur_x = ox;
        cur_m = om;
        cur_s = os;
        cur_k = ok;
    }
    if (merged_map && n_steps > 1) return oim_compose(maps, n_in, n_steps, B, H * W, merged_map, st);
    return LUVC_OK;
}

luvc_status luvc_value_enhance(const void* v, const int32_t* sizes, int64_t rows, int D, int64_t v_stride, luvc_dtype dtype,
                               void* out, int64_t out_stride, void* hip_stream)
{
    if (!dtype_ok(dtype)) { set_error("unknown dtype %d", (int)dtype); return LUVC_ERR_INVALID_ARG; }
    if (!v || !sizes || !out) { set_error("v, sizes and out must not be NULL"); return LUVC_ERR_INVALID_ARG; }
    if (rows < 1 || D < 1) { set_error("rows and D must be positive"); return LUVC_ERR_INVALID_ARG; }
    if (v_stride < D || out_stride < D) { set_error("row strides must be at least D=%d", D); return LUVC_ERR_INVALID_ARG; }
    if (rows > ((int64_t)1 << 40)) { set_error("too many rows"); return LUVC_ERR_UNSUPPORTED; }
    return value_enhance_run(v, sizes, rows, D, v_stride, out_stride, dtype, out, (hipStream_t)hip_stream);
}

size_t luvc_spu_workspace_bytes(int B, int N, int D, luvc_dtype dtype, int sigma)
{
    if (!dtype_ok(dtype) || B < 1 || N < 1 || D < 1 || sigma < 0 || sigma > N / 2 || N > kSpuMaxN) return 0;
    return spu_layout(B, N, D, sigma).bytes;
}

luvc_status luvc_spu_score(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dtype, int sigma,
                           int use_hamming, float* scores, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!dtype_ok(dtype)) { set_error("unknown dtype %d", (int)dtype); return LUVC_ERR_INVALID_ARG; }
    if (!x || !scores) { set_error("x and scores must not be NULL"); return LUVC_ERR_INVALID_ARG; }
    if (B < 1 || N < 1 || D < 1) { set_error("B, N, D must be positive (got %d,%d,%d)", B, N, D); return LUVC_ERR_INVALID_ARG; }
    if (row_stride < D) { set_error("row_stride %lld is smaller than D=%d", (long long)row_stride, D); return LUVC_ERR_INVALID_ARG; }
    if (sigma < 0 || sigma > N / 2) { set_error("sigma=%d must lie in 0..N/2=%d", sigma, N / 2); return LUVC_ERR_INVALID_ARG; }
    if (N > kSpuMaxN) { set_error("N=%d exceeds the supported %d tokens per sample", N, kSpuMaxN); return LUVC_ERR_UNSUPPORTED; }
    if (B > 65535) { set_error("B=%d exceeds 65535 samples per call", B); return LUVC_ERR_UNSUPPORTED; }
    const size_t need = spu_layout(B, N, D, sigma).bytes;
    if (!workspace_ok(workspace, workspace_bytes, need)) return LUVC_ERR_WORKSPACE;
    return spu_score_dense(x, B, N, D, row_stride, dtype, sigma, use_hamming ? 1 : 0, scores, workspace, (hipStream_t)hip_stream);
}

int luvc_keep_count(int N, double keep_ratio)
{
    if (N < 1) return 0;
    double v = std::floor(keep_ratio * (double)N + 0.5);
    if (!(v >= 1.0)) v = 1.0;
    if (v > (double)N) v = (double)N;
    return (int)v;
}

luvc_status luvc_spu_prune(const void* x, const float* scores, int B, int N, int D, int64_t row_stride, luvc_dtype dtype,
                           int n_keep, int32_t* kept_idx, void* x_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    (void)workspace;
    (void)workspace_bytes;
    if (!dtype_ok(dtype)) { set_error("unknown dtype %d", (int)dtype); return LUVC_ERR_INVALID_ARG; }
    if (!scores || !kept_idx) { set_error("scores and kept_idx must not be NULL"); return LUVC_ERR_INVALID_ARG; }
    if (x_out && !x) { set_error("x_out given without x"); return LUVC_ERR_INVALID_ARG; }
    if (B < 1 || N < 1 || D < 1) { set_error("B, N, D must be positive (got %d,%d,%d)", B, N, D); return LUVC_ERR_INVALID_ARG; }
    if (row_stride < D) { set_error("row_stride %lld is smaller than D=%d", (long long)row_stride, D); return LUVC_ERR_INVALID_ARG; }
    if (n_keep < 1 || n_keep > N) { set_error("n_keep=%d must lie in 1..N=%d", n_keep, N); return LUVC_ERR_INVALID_ARG; }
    if ((int64_t)B * N >= ((int64_t)1 << 31)) { set_error("B*N must stay below 2^31"); return LUVC_ERR_UNSUPPORTED; }
    return spu_prune_run(x, scores, B, N, D, row_stride, dtype, n_keep, kept_idx, x_out, nullptr, nullptr, (hipStream_t)hip_stream);
}

int luvc_spu_cascade_keeps(int N0, double keep_ratio, int n_stages, int eliminate, int* keeps)
{
    if (N0 < 1 || n_stages < 1 || !keeps || !(keep_ratio > 0.0) || keep_ratio > 1.0) return 0;
    int n = N0;
    for (int i = 0; i < n_stages; ++i) {
        n = (eliminate && i == n_stages - 1) ? 0 : luvc_keep_count(n, keep_ratio);
        keeps[i] = n;
    }
    return n_stages;
}

luvc_status luvc_spu_stage(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dtype, int sigma, int use_hamming,
                           int n_keep, const int32_t* origin_in, float* scores, int32_t* kept_idx, int32_t* origin_out, void* x_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (n_keep < 0 || n_keep > N) { set_error("n_keep=%d must lie in 0..N=%d", n_keep, N); return LUVC_ERR_INVALID_ARG; }
    if (n_keep > 0 && (!kept_idx || !origin_out)) { set_error("kept_idx and origin_out must not be NULL"); return LUVC_ERR_INVALID_ARG; }
    if (n_keep == 0) {                                 // the eliminating stage: nothing survives, nothing is computed or written
        if (B < 1 || N < 1 || D < 1) { set_error("B, N, D must be positive (got %d,%d,%d)", B, N, D); return LUVC_ERR_INVALID_ARG; }
        return LUVC_OK;
    }
    const luvc_status rc = luvc_spu_score(x, B, N, D, row_stride, dtype, sigma, use_hamming, scores, workspace, workspace_bytes, hip_stream);
    if (rc != LUVC_OK) return rc;
    if ((int64_t)B * N >= ((int64_t)1 << 31)) { set_error("B*N must stay below 2^31"); return LUVC_ERR_UNSUPPORTED; }
    return spu_prune_run(x, scores, B, N, D, row_stride, dtype, n_keep, kept_idx, x_out, origin_in, origin_out, (hipStream_t)hip_stream);
}

}  // extern "C"
