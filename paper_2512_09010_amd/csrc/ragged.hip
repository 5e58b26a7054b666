// Ragged batches (appendix "Iterative Strategy and Pseudocode of OIM": with any-resolution inputs every image has
// its own grid and its own number of merges): images / samples of different shapes packed back to back.  Host code
// only: consecutive items of equal shape and schedule form a run, and every run is one batched call of the entry
// points in api.hip, on slices of the packed buffers.  Every item is validated before the first launch.
#include <vector>

#include "common.hpp"
#include "oim.hpp"
#include "spu.hpp"

namespace luvc {

namespace {

struct OimRun {
    int count;                   // consecutive images of this shape and schedule
    int H, W;
    const luvc_oim_pass* passes;
    int n_passes;
    int64_t tok_in, tok_out;     // packed token offsets of the first image
};

bool same_schedule(const luvc_oim_pass* a, int na, const luvc_oim_pass* b, int nb)
{
    if (na != nb) return false;
    for (int i = 0; i < na; ++i)
        if (a[i].axis != b[i].axis || a[i].m != b[i].m) return false;
    return true;
}

// Splits the images into runs; false (with an error message) when an argument is unusable.
bool oim_runs(int n_images, const int32_t* H, const int32_t* W, const luvc_oim_pass* passes, const int32_t* n_passes,
              std::vector<OimRun>* runs)
{
    if (n_images < 1 || !H || !W || !passes || !n_passes) { set_error("n_images, H, W, passes and n_passes must be given"); return false; }
    int64_t tin = 0, tout = 0;
    const luvc_oim_pass* p = passes;
    for (int i = 0; i < n_images; ++i) {
        if (H[i] < 1 || W[i] < 1) { set_error("image %d: H and W must be positive (got %d,%d)", i, H[i], W[i]); return false; }
        if (n_passes[i] < 1 || n_passes[i] > kMaxPasses) { set_error("image %d: need 1..%d passes", i, kMaxPasses); return false; }
        int h = H[i], w = W[i];
        for (int k = 0; k < n_passes[i]; ++k) {
            const int axis = p[k].axis, m = p[k].m;
            if (axis != 0 && axis != 1) { set_error("image %d pass %d: axis must be 0 (H) or 1 (W)", i, k); return false; }
            const int len = axis ? w : h;
            if (m < 0 || m > (len + 1) / 2 || len - m < 1) { set_error("image %d pass %d: m=%d does not fit a line of %d", i, k, m, len); return false; }
            if (axis) w -= m; else h -= m;
        }
        const bool extend = !runs->empty() && runs->back().H == H[i] && runs->back().W == W[i] &&
                            same_schedule(runs->back().passes, runs->back().n_passes, p, n_passes[i]);
        if (extend) ++runs->back().count;
        else runs->push_back(OimRun{1, H[i], W[i], p, n_passes[i], tin, tout});
        tin += (int64_t)H[i] * W[i];
        tout += (int64_t)h * w;
        if (tin >= ((int64_t)1 << 31)) { set_error("the packed batch must stay below 2^31 tokens"); return false; }
        p += n_passes[i];
    }
    return true;
}

struct SpuRun {
    int count, N, sigma, keep;   // consecutive samples with these parameters
    int64_t tok_in, tok_out;
};

bool spu_runs(int n_samples, const int32_t* N, const int32_t* sigma, const int32_t* n_keep, std::vector<SpuRun>* runs)
{
    if (n_samples < 1 || !N || !sigma) { set_error("n_samples, N and sigma must be given"); return false; }
    int64_t tin = 0, tout = 0;
    for (int i = 0; i < n_samples; ++i) {
        const int keep = n_keep ? n_keep[i] : 0;
        if (N[i] < 1 || N[i] > kSpuMaxN) { set_error("sample %d: N=%d must lie in 1..%d", i, N[i], kSpuMaxN); return false; }
        if (sigma[i] < 0 || sigma[i] > N[i] / 2) { set_error("sample %d: sigma=%d must lie in 0..N/2=%d", i, sigma[i], N[i] / 2); return false; }
        if (keep < 0 || keep > N[i]) { set_error("sample %d: n_keep=%d must lie in 0..N=%d", i, keep, N[i]); return false; }
        const bool extend = !runs->empty() && runs->back().N == N[i] && runs->back().sigma == sigma[i] && runs->back().keep == keep &&
                            runs->back().count < 65535;
        if (extend) ++runs->back().count;
        else runs->push_back(SpuRun{1, N[i], sigma[i], keep, tin, tout});
        tin += N[i];
        tout += keep;
        if (tin >= ((int64_t)1 << 31)) { set_error("the packed batch must stay below 2^31 tokens"); return false; }
    }
    return true;
}

size_t esz(luvc_dtype dt) { return dt == LUVC_F32 ? 4 : 2; }

}  // namespace

}  // namespace luvc

using namespace luvc;

extern "C" {

luvc_status luvc_oim_plan_anyres(int H, int W, int64_t max_tokens, luvc_oim_pass* passes, int max_passes, int* n_passes)
{
    if (!passes || !n_passes || max_passes < 1) { set_error("passes / n_passes must be given"); return LUVC_ERR_INVALID_ARG; }
    if (H < 1 || W < 1 || max_tokens < 1) { set_error("H, W and max_tokens must be positive"); return LUVC_ERR_INVALID_ARG; }
    int h = H, w = W, n = 0;
    while ((int64_t)h * w > max_tokens) {
        if (n >= max_passes) { set_error("schedule needs more than %d passes", max_passes); return LUVC_ERR_INVALID_ARG; }
        const int axis = w >= h ? 1 : 0;                 // the longer side; a square grid starts with the row merge
        const int len = axis ? w : h;                    // > 1 here: h * w > max_tokens >= 1
        passes[n].axis = axis;
        passes[n].m = (len + 1) / 2;
        ++n;
        if (axis) w = len / 2; else h = len / 2;
    }
    if (n == 0) {                                        // nothing to merge: the pass that leaves every line as it is
        passes[0].axis = 1;
        passes[0].m = 0;
        n = 1;
    }
    *n_passes = n;
    return LUVC_OK;
}

size_t luvc_oim_ragged_workspace_bytes(int n_images, const int32_t* H, const int32_t* W, int D, luvc_dtype dtype,
                                       const luvc_oim_pass* passes, const int32_t* n_passes)
{
    std::vector<OimRun> runs;
    if (D < 1 || !oim_runs(n_images, H, W, passes, n_passes, &runs)) return 0;
    size_t need = 0;
    for (const OimRun& r : runs) {
        const size_t b = luvc_oim_workspace_bytes(r.count, r.H, r.W, D, dtype, r.passes, r.n_passes);
        if (b == 0) return 0;
        need = b > need ? b : need;
    }
    return need;
}

luvc_status luvc_oim_merge_ragged(const void* x, const int32_t* sizes_in, int n_images, const int32_t* H, const int32_t* W,
                                  int D, luvc_dtype dtype, const luvc_oim_pass* passes, const int32_t* n_passes,
                                  void* x_out, int32_t* sizes_out, int32_t* merged_map, int32_t* kept_map,
                                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (dtype != LUVC_F32 && dtype != LUVC_BF16) { set_error("unknown dtype %d", (int)dtype); return LUVC_ERR_INVALID_ARG; }
    if (!x || !x_out || !sizes_out) { set_error("x, x_out and sizes_out must not be NULL"); return LUVC_ERR_INVALID_ARG; }
    if (D < 1) { set_error("D must be positive (got %d)", D); return LUVC_ERR_INVALID_ARG; }
    std::vector<OimRun> runs;
    if (!oim_runs(n_images, H, W, passes, n_passes, &runs)) return LUVC_ERR_INVALID_ARG;
    // all runs are checked (shape limits, workspace) before the first one is launched
    for (const OimRun& r : runs) {
        const size_t b = luvc_oim_workspace_bytes(r.count, r.H, r.W, D, dtype, r.passes, r.n_passes);
        if (b == 0) return LUVC_ERR_INVALID_ARG;         // message set by the query
        if (!workspace_ok(workspace, workspace_bytes, b)) return LUVC_ERR_WORKSPACE;
    }
    const size_t row = (size_t)D * esz(dtype);
    for (const OimRun& r : runs) {
        const luvc_status rc = luvc_oim_merge(
            (const char*)x + (size_t)r.tok_in * row, sizes_in ? sizes_in + r.tok_in : nullptr, r.count, r.H, r.W, D, dtype,
            r.passes, r.n_passes, 0, (char*)x_out + (size_t)r.tok_out * row, sizes_out + r.tok_out,
            merged_map ? merged_map + r.tok_in : nullptr, kept_map ? kept_map + r.tok_out : nullptr,
            workspace, workspace_bytes, hip_stream);
        if (rc != LUVC_OK) return rc;
    }
    return LUVC_OK;
}

size_t luvc_spu_ragged_workspace_bytes(int n_samples, const int32_t* N, int D, luvc_dtype dtype, const int32_t* sigma)
{
    std::vector<SpuRun> runs;
    if (D < 1 || !spu_runs(n_samples, N, sigma, nullptr, &runs)) return 0;
    size_t need = 0;
    for (const SpuRun& r : runs) {
        const size_t b = luvc_spu_workspace_bytes(r.count, r.N, D, dtype, r.sigma);
        if (b == 0) return 0;
        need = b > need ? b : need;
    }
    return need;
}

luvc_status luvc_spu_stage_ragged(const void* x, int n_samples, const int32_t* N, int D, int64_t row_stride, luvc_dtype dtype,
                                  const int32_t* sigma, int use_hamming, const int32_t* n_keep, const int32_t* origin_in,
                                  float* scores, int32_t* kept_idx, int32_t* origin_out, void* x_out,
                                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (dtype != LUVC_F32 && dtype != LUVC_BF16) { set_error("unknown dtype %d", (int)dtype); return LUVC_ERR_INVALID_ARG; }
    if (!x || !scores) { set_error("x and scores must not be NULL"); return LUVC_ERR_INVALID_ARG; }
    if (D < 1 || row_stride < D) { set_error("need D >= 1 and row_stride >= D (got %d, %lld)", D, (long long)row_stride); return LUVC_ERR_INVALID_ARG; }
    if (n_keep && (!kept_idx || !origin_out)) { set_error("kept_idx and origin_out must be given with n_keep"); return LUVC_ERR_INVALID_ARG; }
    std::vector<SpuRun> runs;
    if (!spu_runs(n_samples, N, sigma, n_keep, &runs)) return LUVC_ERR_INVALID_ARG;
    for (const SpuRun& r : runs) {
        const size_t b = luvc_spu_workspace_bytes(r.count, r.N, D, dtype, r.sigma);
        if (b == 0) { set_error("run of %d samples with N=%d, sigma=%d is not supported", r.count, r.N, r.sigma); return LUVC_ERR_INVALID_ARG; }
        if (!workspace_ok(workspace, workspace_bytes, b)) return LUVC_ERR_WORKSPACE;
    }
    const size_t es = esz(dtype);
    for (const SpuRun& r : runs) {
        const char* xr = (const char*)x + (size_t)r.tok_in * (size_t)row_stride * es;
        luvc_status rc;
        if (!n_keep || r.keep == 0)                      // scores only (a sample that is eliminated still gets its scores)
            rc = luvc_spu_score(xr, r.count, r.N, D, row_stride, dtype, r.sigma, use_hamming, scores + r.tok_in,
                                workspace, workspace_bytes, hip_stream);
        else
            rc = luvc_spu_stage(xr, r.count, r.N, D, row_stride, dtype, r.sigma, use_hamming, r.keep,
                                origin_in ? origin_in + r.tok_in : nullptr, scores + r.tok_in, kept_idx + r.tok_out,
                                origin_out + r.tok_out, x_out ? (char*)x_out + (size_t)r.tok_out * D * es : nullptr,
                                workspace, workspace_bytes, hip_stream);
        if (rc != LUVC_OK) return rc;
    }
    return LUVC_OK;
}

}  // extern "C"
