// Internal interface between the C-ABI layer and the OIM kernels.
#pragma once
#include "common.hpp"

namespace luvc {

constexpr int kMaxPasses = 16;      // passes per luvc_oim_merge call
constexpr int kMaxLineLen = 8192;   // tokens on one line (bounded by the decision kernel's LDS use)

// Scratch of one pass, carved from the caller's workspace.
struct OimScratch {
    double* n2;        // [B*H*W] squared norms
    double* dn;        // [B*H*W] dot product with the next token on the line
    int32_t* anchor;   // [B*Ho*Wo]
    int32_t* absorb;   // [B*Ho*Wo]
};

luvc_status oim_general_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt,
                             int axis, int m, bool vec, void* x_out, int32_t* sizes_out, int32_t* pass_map,
                             const int32_t* kept_prev, int32_t* kept_out,
                             const OimScratch& ws, hipStream_t st);

// Squared norms of all tokens into ws.n2 (ws.dn receives the dot products with the next token on the line).
luvc_status oim_norms(const void* x, int B, int H, int W, int D, luvc_dtype dt, int axis, bool vec,
                      const OimScratch& ws, hipStream_t st);

// Pass with candidates beyond the adjacent destinations (oim_wide.hip): radius 0 = every destination of the
// line, radius R >= 1 = destinations within 2R - 1 positions.  G and src_dest are scratch of the sizes below.
constexpr int kMaxWideLineLen = 2048;
size_t oim_wide_gram_bytes(int B, int H, int W, int axis);
size_t oim_wide_srcdest_bytes(int B, int H, int W, int axis);
luvc_status oim_wide_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt,
                          int axis, int m, int radius, bool vec, void* x_out, int32_t* sizes_out, int32_t* pass_map,
                          const int32_t* kept_prev, int32_t* kept_out,
                          const OimScratch& ws, double* G, int32_t* src_dest, hipStream_t st);

// Wide matching with one launch per pass and the tokens moved once, at the end (oim_wide_lazy.hip): grids between the
// passes are tensors of row ids (below n0: a token of x; from n0: a row of the overlay `ov`, which receives the merged
// destinations).  Lines of at most kLazyMaxLen tokens, 16-byte aligned rows.
constexpr int kLazyMaxLen = 128;
int oim_wide_lazy_rows(int h, int w, int axis, int m);      // overlay rows per image that a pass may write
// metric / ov_metric / Dm: the tensor the decisions are taken on and its overlay (merged like x), or NULL / NULL / 0: x itself
luvc_status oim_wide_lazy_pass(const void* x, void* ov, const void* metric, void* ov_metric, int Dm, const int32_t* idx_in, const int32_t* sizes_in, const int32_t* kept_in,
                               int B, int n0, int h, int w, int D, luvc_dtype dt, int axis, int m, int radius, int cap, int ov_base,
                               int32_t* idx_out, int32_t* sizes_out, int32_t* kept_out, int32_t* pass_map, hipStream_t st);
luvc_status oim_wide_lazy_gather(const void* x, const void* ov, const int32_t* idx, int B, int n0, int cap, int n_out_per, int D,
                                 luvc_dtype dt, void* x_out, hipStream_t st);

// The two stages of a pass on their own: decisions on one tensor (`metric`), merge applied to another.
luvc_status oim_general_decide(const void* metric, int B, int H, int W, int Dm, luvc_dtype dt, int axis, int m, bool vec,
                               int32_t* pass_map, const OimScratch& ws, hipStream_t st);
luvc_status oim_general_apply(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int axis, int m,
                              bool vec, void* x_out, int32_t* sizes_out, const int32_t* kept_prev, int32_t* kept_out,
                              const OimScratch& ws, hipStream_t st);
luvc_status oim_wide_decide(const void* metric, int B, int H, int W, int Dm, luvc_dtype dt, int axis, int m, int radius, bool vec,
                            int32_t* pass_map, const OimScratch& ws, double* G, int32_t* src_dest, hipStream_t st);
luvc_status oim_wide_apply(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int axis, int m, bool vec,
                           void* x_out, int32_t* sizes_out, const int32_t* kept_prev, int32_t* kept_out,
                           const OimScratch& ws, const int32_t* src_dest, hipStream_t st);

// Eq. 3 of the paper: out = v + log(s) on every channel of a row (value.hip)
luvc_status value_enhance_run(const void* v, const int32_t* sizes, int64_t rows, int D, int64_t v_stride, int64_t out_stride,
                              luvc_dtype dt, void* out, hipStream_t st);

// Fused pass for m = ceil(len/2) (oim_fast.hip); `vec` = rows are 16-byte aligned.
bool oim_halve_supported(int H, int W, int D, luvc_dtype dt, int axis, int m, bool vec);
luvc_status oim_halve_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int axis,
                           void* x_out, int32_t* sizes_out, int32_t* pass_map, const int32_t* kept_prev, int32_t* kept_out,
                           hipStream_t st);

// One launch for two consecutive halving passes on different axes (oim_pair.hip); pair_map sends an
// input flat index of the first pass to an output slot of the second.
bool oim_pair_supported(int H, int W, int D, luvc_dtype dt, int axis0, int m0, int axis1, int m1, bool vec);
luvc_status oim_pair_pass(const void* x, const int32_t* sizes_in, int B, int H, int W, int D, luvc_dtype dt, int first_axis,
                          void* x_out, int32_t* sizes_out, int32_t* pair_map, const int32_t* kept_prev, int32_t* kept_out,
                          hipStream_t st);

// The same pair of passes decided on a metric tensor of Dm values per token (oim_pair_keyed.hip): features and
// metric are merged alike; metric_out may be NULL when the merged metric is not wanted.
bool oim_pair_keyed_supported(int H, int W, int D, int Dm, luvc_dtype dt, int axis0, int m0, int axis1, int m1, bool vec_x, bool vec_m);
luvc_status oim_pair_keyed_pass(const void* x, const void* metric, const int32_t* sizes_in, int B, int H, int W, int D, int Dm,
                                luvc_dtype dt, int first_axis, void* x_out, void* metric_out, int32_t* sizes_out, int32_t* pair_map,
                                const int32_t* kept_prev, int32_t* kept_out, hipStream_t st);

luvc_status oim_compose(const int32_t* const* maps, const int32_t* n_in, int n, int B, int n_first,
                        int32_t* merged_out, hipStream_t st);

}  // namespace luvc
