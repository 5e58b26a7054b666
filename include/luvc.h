/*
 * luvc.h - C ABI of the MI355X (gfx950) implementation of LUVC's training-free
 * visual-token compression hot path:
 *
 *   OIM  Orthogonal Iterative Merger   (paper Section 3.2, Algorithm 1)
 *   SPU  Spectrum Pruning Unit         (paper Section 3.3, Eq. 4-8, Algorithm 2)
 *
 * General conventions
 *   - "device" pointers are HIP device memory of the GPU that is current on the
 *     calling thread; "host" pointers are ordinary process memory.
 *   - The caller owns every buffer.  The library allocates no device memory; all
 *     scratch lives in the caller's `workspace` (sized by the *_workspace_bytes
 *     query for the same arguments, 256-byte aligned).
 *   - Inputs are never modified.  Input, output and workspace buffers must not
 *     overlap.
 *   - All work is enqueued asynchronously on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream).  No call synchronises with the host or
 *     copies device data to the host.
 *   - Arguments are validated on the host before anything is enqueued; a call that
 *     returns a status other than LUVC_OK has enqueued nothing.  luvc_last_error()
 *     then describes the problem.
 *   - Tensors are dense, row-major, innermost dimension D contiguous.  Flat token
 *     index inside one grid: p = h * W + w.
 *   - Non-finite input values give unspecified output VALUES, but every access
 *     stays in bounds and index outputs stay well formed.
 */
#ifndef LUVC_H
#define LUVC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LUVC_OK = 0,
    LUVC_ERR_INVALID_ARG = 1,  /* NULL pointer, non-positive size, inconsistent schedule ...   */
    LUVC_ERR_UNSUPPORTED = 2,  /* valid request outside what the kernels implement              */
    LUVC_ERR_WORKSPACE = 3,    /* workspace missing, misaligned or smaller than the query says  */
    LUVC_ERR_HIP = 4           /* a HIP launch failed; luvc_last_error() carries hipGetErrorString */
} luvc_status;

typedef enum {
    LUVC_F32 = 0,   /* IEEE binary32                                    */
    LUVC_BF16 = 1   /* bfloat16 (upper half of binary32), 2 bytes/value */
} luvc_dtype;

/* One merge pass of OIM (Section 3.2): along axis 1 every row of W tokens becomes W-m
 * tokens ("row merge", H x W -> H x (W-m)); along axis 0 every column of H tokens becomes
 * H-m ("column merge").  m = number of tokens merged per line, 0 <= m <= ceil(len/2) and
 * len-m >= 1.  The paper's setting is m = 2 (appendix "Iterative Strategy and Pseudocode of
 * OIM"); m = ceil(len/2) halves the axis. */
typedef struct {
    int32_t axis; /* 1 = along W, 0 = along H */
    int32_t m;
} luvc_oim_pass;

/* Version / build information: static string, never NULL. */
const char* luvc_version(void);

/* Text of the last error raised on the calling thread ("" if none).  Static storage. */
const char* luvc_last_error(void);

/*
 * Merge schedule for a target token count (Section 3.2 order: row merge first, then
 * column merge, alternating as in Algorithm 1's consecutive layers).  Starting from H x W,
 * passes alternate W, H, W, ...; a pass halves its axis (m = ceil(len/2)) while the halved
 * grid still holds at least target_tokens tokens; otherwise it takes the one m that lands
 * exactly on target_tokens, and the schedule ends.
 *   passes      host, capacity max_passes
 *   n_passes    host, receives the number of passes written
 * Returns LUVC_OK, or LUVC_ERR_INVALID_ARG when the target cannot be hit exactly or
 * max_passes is too small.
 */
luvc_status luvc_oim_plan(int H, int W, int64_t target_tokens,
                          luvc_oim_pass* passes, int max_passes, int* n_passes);

/* Bytes of workspace luvc_oim_merge needs for these arguments (0 on invalid arguments). */
size_t luvc_oim_workspace_bytes(int B, int H, int W, int D, luvc_dtype dtype,
                                const luvc_oim_pass* passes, int n_passes);

/*
 * OIM: iterative merging of similar, spatially adjacent tokens along alternating grid axes
 * while keeping the 2-D layout (Section 3.2; size vector s of Algorithm 1).
 *
 * One pass, on every line independently: tokens at even positions are merge sources, tokens
 * at odd positions destinations.  Each source picks the more similar (cosine of the features,
 * norms clamped at 1e-12, evaluated in fp64; tie -> lower position) of its adjacent
 * destinations; the m sources with the highest similarity (tie -> lower position) are folded
 * into their pick by size-weighted mean, sizes add; survivors keep their order.  The output
 * of a pass is rounded once to `dtype` before the next pass reads it.
 *
 *   x           device [B,H,W,D] dtype
 *   sizes_in    device [B,H,W] int32 >= 1, or NULL (every token counts 1)
 *   passes      host [n_passes], applied in order; n_passes >= 1
 *   target_tokens  0 = no check; otherwise must equal H' * W' of the schedule
 *   x_out       device [B,H',W',D] dtype
 *   sizes_out   device [B,H',W'] int32
 *   merged_map  device [B,H*W] int32: input flat index -> output flat slot, or NULL
 *   kept_map    device [B,H'*W'] int32: output slot -> input flat index of the token that
 *               anchors it (the destination of a merged group), or NULL
 * Limits: B*H*W < 2^31, sizes sums < 2^31.
 */
luvc_status luvc_oim_merge(const void* x, const int32_t* sizes_in,
                           int B, int H, int W, int D, luvc_dtype dtype,
                           const luvc_oim_pass* passes, int n_passes, int64_t target_tokens,
                           void* x_out, int32_t* sizes_out, int32_t* merged_map, int32_t* kept_map,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * OIM with a wider candidate set (the bipartite matching behind the similarity cost O(n_v^1.5 k)
 * of Section 3.1; the appendix "Iterative Strategy and Pseudocode of OIM" runs it with a merge
 * number of 2): as luvc_oim_merge, except that a source at position a of a line considers every
 * destination b of the line with |b - a| <= 2 * radius - 1, or every destination of the line when
 * radius = 0; a destination can then absorb several sources (size-weighted mean over all of them,
 * added in ascending position).  radius = 1 is luvc_oim_merge itself.
 * The decisions are fp64 decisions.  Lines of at most 128 tokens with 16-byte aligned rows (x, x_out and D * element
 * size multiples of 16) are screened on the matrix cores in the storage precision and only the pairs the screening cannot
 * tell are repeated in fp64; between the passes of such a call the grids are kept as row indices and the tokens are
 * moved once, at the end.  Longer lines or unaligned rows: every dot product in fp64 on the matrix cores, every pass
 * written out.  The results are the same either way.
 * Limits: lines of at most 2048 tokens and images of less than 2 GiB when radius != 1.
 * Workspace: luvc_oim_wide_workspace_bytes for the same arguments.
 */
size_t luvc_oim_wide_workspace_bytes(int B, int H, int W, int D, luvc_dtype dtype,
                                     const luvc_oim_pass* passes, int n_passes, int radius);
luvc_status luvc_oim_merge_wide(const void* x, const int32_t* sizes_in,
                                int B, int H, int W, int D, luvc_dtype dtype,
                                const luvc_oim_pass* passes, int n_passes, int radius, int64_t target_tokens,
                                void* x_out, int32_t* sizes_out, int32_t* merged_map, int32_t* kept_map,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * OIM whose decisions are taken on a separate tensor (Section 3.1 counts the similarity cost in k, "the
 * dimension of keys": similarity on the attention keys, merge applied to the tokens): as
 * luvc_oim_merge_wide, except that the cosines are those of `metric` while x is merged along; the metric
 * is merged the same way, so that the next pass (or the next layer) can go on with it.
 *   metric      device [B,H,W,Dm] dtype
 *   metric_out  device [B,H',W',Dm] dtype, or NULL
 *   radius      1 = adjacent destinations, R > 1 = within 2R-1 positions, 0 = the whole line
 * A pair of halving passes on different axes with adjacent matching (radius 1), keys of at most 1 KB per token and
 * 16-byte aligned rows of x, metric and the outputs runs as one launch; wide matching (radius != 1) on lines of at most
 * 128 tokens with aligned rows runs one launch per pass like luvc_oim_merge_wide; anything else runs decisions and
 * merges (tokens, metric) as separate launches.  The results are the same either way.
 */
size_t luvc_oim_keyed_workspace_bytes(int B, int H, int W, int D, int Dm, luvc_dtype dtype,
                                      const luvc_oim_pass* passes, int n_passes, int radius);
luvc_status luvc_oim_merge_keyed(const void* x, const void* metric, const int32_t* sizes_in,
                                 int B, int H, int W, int D, int Dm, luvc_dtype dtype,
                                 const luvc_oim_pass* passes, int n_passes, int radius, int64_t target_tokens,
                                 void* x_out, void* metric_out, int32_t* sizes_out,
                                 int32_t* merged_map, int32_t* kept_map,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Value enhancement (Section 3.2, Eq. 3): O = A (V + log s) - this call forms V + log(s), s = number of
 * tokens merged into each token (the size vector of Algorithm 1), added to every channel of the token's row.
 *   v        device [rows,*] dtype, row r starts at v + r * v_stride (elements), v_stride >= D
 *   sizes    device [rows] int32 >= 1 (values below 1 are read as 1)
 *   out      device [rows,*] dtype with out_stride >= D; may be v itself (in place) when the strides agree
 * The sum is formed in fp64 and rounded once to dtype.  Needs no workspace.
 */
luvc_status luvc_value_enhance(const void* v, const int32_t* sizes, int64_t rows, int D, int64_t v_stride,
                               luvc_dtype dtype, void* out, int64_t out_stride, void* hip_stream);

/* Bytes of workspace luvc_spu_score needs (0 on invalid arguments). */
size_t luvc_spu_workspace_bytes(int B, int N, int D, luvc_dtype dtype, int sigma);

/*
 * SPU score (Section 3.3): per sample and channel, DFT along the token index n (Eq. 4),
 * multiplication by the low-pass mask M[k] (Eq. 5-6), inverse DFT with 1/N (Eq. 7), then the
 * L2 norm over the D channels of each filtered token (Eq. 8).
 *
 * Mask: with the folded frequency f(k) = min(k, N-k), M[k] = w(f) for f <= sigma and 0 above;
 * w(f) = 0.54 + 0.46 cos(2 pi f / (N-1)) (Hamming window centred on DC; w = 1 when N = 1) if
 * use_hamming, else w = 1 (the "wo HW" ablation of the paper's core-component table).
 *
 *   x           device [B,N,*] dtype, token n of sample b starts at x + (b*N + n)*row_stride
 *   row_stride  elements between consecutive tokens, >= D
 *   sigma       cut-off, 0 <= sigma <= N/2
 *   scores      device [B,N] fp32
 * Arithmetic is fp32 (bf16 is a storage type only).  The sum over channels is taken in a fixed order:
 * the same input gives the same bits on every call.
 * Accuracy: within 1e-5 relative of Eq. 4-8 evaluated exactly, plus 1e-6 of the sample's largest score for tokens
 * whose filtered energy all but vanishes.  For lengths N = 16 Q N2 (Q = 16, 15, 9) with 2 sigma + 1 <= 16 Q and
 * N / dec > 4 sigma for a divisor dec of N2, Eq. 7 is evaluated on every dec-th token and the energies between are
 * filled in from the band limit 2 sigma of the energy sequence, 32 channels at a time, wherever two conditioning
 * tests show that this stays inside the same bounds; elsewhere Eq. 7 is evaluated on every token.
 * Concurrency: calls may overlap on different streams, or with replays of a captured graph, as long as each call
 * in flight has its own workspace.  The workspace may hold anything when the call starts (the completion counters
 * the single-launch kernels keep in it recognise stale contents), and nothing in it is needed afterwards.
 */
luvc_status luvc_spu_score(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dtype,
                           int sigma, int use_hamming, float* scores,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * luvc_spu_score for callers that cannot allocate device memory and so have no workspace to pass: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same arithmetic and
 * the same bits in `scores` as luvc_spu_score; the scratch lives in a static device array of
 * LUVC_SPU_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends).  The call
 * allocates and frees no device memory and calls no library routine that does.
 *   x, B, N, D, row_stride, dtype, sigma, use_hamming, scores, hip_stream   as for luvc_spu_score
 * Returns LUVC_ERR_WORKSPACE (nothing enqueued) when luvc_spu_workspace_bytes(B, N, D, dtype, sigma) exceeds
 * LUVC_SPU_STATIC_SCRATCH_BYTES; the message carries both figures.
 * Every call on a GPU uses that GPU's one array: two calls that overlap in time on one GPU (different streams, or a
 * captured graph replayed while another call runs) race on it and give wrong scores.  Calls on one stream, one
 * after the other, are fine, whatever their sizes.
 */
#define LUVC_SPU_STATIC_SCRATCH_BYTES (8u << 20)
luvc_status luvc_spu_score_static(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dtype,
                                  int sigma, int use_hamming, float* scores, void* hip_stream);

/* Number of tokens to keep for a keep ratio: floor(ratio*N + 0.5) clamped to [1, N]. */
int luvc_keep_count(int N, double keep_ratio);

/*
 * SPU prune (Algorithm 2, last two steps): keep the n_keep tokens with the largest score
 * (equal scores: the lower index wins) and return them in their original order, gathering
 * the ORIGINAL (unfiltered) tokens.
 *
 *   x           device [B,N,*] dtype with row_stride as above; may be NULL iff x_out is NULL
 *   scores      device [B,N] fp32
 *   n_keep      1..N
 *   kept_idx    device [B,n_keep] int32, strictly ascending within a sample
 *   x_out       device [B,n_keep,D] dtype (dense), or NULL for indices only
 * Needs no workspace today; the arguments are kept so callers are ready for one
 * (pass NULL / 0).
 */
luvc_status luvc_spu_prune(const void* x, const float* scores, int B, int N, int D, int64_t row_stride,
                           luvc_dtype dtype, int n_keep, int32_t* kept_idx, void* x_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Keep counts of an SPU cascade (Section 3.3, last paragraph; appendix on the SPU parameters l_0, l_delta): SPU is
 * applied at LLM layers l_0, l_0 + l_delta, ... and removes the visual tokens step by step, all of them at the end.
 * The paper gives no per-stage counts; this helper applies one keep ratio stage after stage:
 *   keeps[i] = luvc_keep_count(keeps[i-1], keep_ratio), keeps[-1] = N0; with eliminate != 0 the last stage keeps 0.
 *   keeps     host [n_stages] int, written
 * Returns n_stages, or 0 on invalid arguments (N0 < 1, n_stages < 1, keep_ratio outside (0, 1], keeps NULL).
 * Host arithmetic only.
 */
int luvc_spu_cascade_keeps(int N0, double keep_ratio, int n_stages, int eliminate, int* keeps);

/*
 * One stage of the SPU cascade (Algorithm 2 applied to the tokens that are still alive): luvc_spu_score followed by
 * luvc_spu_prune on the same x, plus the bookkeeping a cascade needs - where every surviving token sat before the
 * first stage.
 *
 *   x, B, N, D, row_stride, dtype, sigma, use_hamming, scores, workspace   as for luvc_spu_score
 *                 (workspace of luvc_spu_workspace_bytes(B, N, D, dtype, sigma) bytes)
 *   n_keep        0..N tokens kept per sample.  0 is the eliminating stage: the call checks B, N, D, launches
 *                 nothing and writes nothing
 *   origin_in     device [B,N] int32: position of token n before the first stage, or NULL for the first stage
 *                 (identity).  Values are copied, never used as addresses
 *   kept_idx      device [B,n_keep] int32, ascending positions within this stage's x
 *   origin_out    device [B,n_keep] int32 = origin_in[b, kept_idx[b, q]] (kept_idx itself when origin_in is NULL);
 *                 feed it to the next stage as origin_in
 *   x_out         device [B,n_keep,D] dtype (dense): the ORIGINAL rows of the kept tokens, or NULL
 * Same arithmetic, tie rule, determinism and limits as the two calls it is made of.
 */
luvc_status luvc_spu_stage(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dtype,
                           int sigma, int use_hamming, int n_keep, const int32_t* origin_in,
                           float* scores, int32_t* kept_idx, int32_t* origin_out, void* x_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Ragged batches (appendix "Iterative Strategy and Pseudocode of OIM": with any-resolution inputs the merges along
 * the two axes follow the aspect ratio of each image; a batch then holds grids of different shapes).  The items of a
 * ragged call are packed back to back, item after item, without padding; shapes, schedules and counts are HOST
 * arrays.  Consecutive items of equal shape and schedule are served by one batched launch sequence, so sort the
 * batch by shape where the order is free.  Results are those of the batched entry points item by item.  Every item is
 * checked before the first launch.
 */

/*
 * Merge schedule that follows the aspect ratio: every pass halves the longer side of the grid (m = ceil(len/2); a
 * square grid starts with the row merge of Section 3.2) until H' * W' <= max_tokens.  The paper states that the
 * number of merges per axis is "adjusted based on the aspect ratio" and prints no rule: this one is this library's.
 *   passes / n_passes   host, as for luvc_oim_plan; a grid that is within max_tokens already gets the single pass
 *                       (axis 1, m 0), which copies it, so that n_passes >= 1 always
 */
luvc_status luvc_oim_plan_anyres(int H, int W, int64_t max_tokens,
                                 luvc_oim_pass* passes, int max_passes, int* n_passes);

/*
 * luvc_oim_merge on n_images grids of their own shape H[i] x W[i] and their own schedule.
 *   H, W        host [n_images]
 *   passes      host: the schedules of all images, image after image; n_passes host [n_images], each >= 1
 *   x           device: image i is a dense [H[i],W[i],D] block at token offset sum_{j<i} H[j]*W[j]
 *   sizes_in    device, packed like x (one int32 per token), or NULL
 *   x_out, sizes_out   device, packed by the output grids H'[i] x W'[i] the schedules end at
 *   merged_map  device, packed like x: input flat index -> output slot WITHIN the image, or NULL
 *   kept_map    device, packed like x_out: output slot -> input flat index WITHIN the image, or NULL
 *   workspace   luvc_oim_ragged_workspace_bytes for the same arguments (the largest need of any run)
 * Limits: those of luvc_oim_merge per run; fewer than 2^31 tokens in the batch.
 */
size_t luvc_oim_ragged_workspace_bytes(int n_images, const int32_t* H, const int32_t* W, int D, luvc_dtype dtype,
                                       const luvc_oim_pass* passes, const int32_t* n_passes);
luvc_status luvc_oim_merge_ragged(const void* x, const int32_t* sizes_in,
                                  int n_images, const int32_t* H, const int32_t* W, int D, luvc_dtype dtype,
                                  const luvc_oim_pass* passes, const int32_t* n_passes,
                                  void* x_out, int32_t* sizes_out, int32_t* merged_map, int32_t* kept_map,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * luvc_spu_stage on n_samples sequences of their own length.
 *   N, sigma    host [n_samples]: tokens and cut-off of every sample (0 <= sigma[i] <= N[i]/2)
 *   n_keep      host [n_samples], each 0..N[i]; NULL = scores only (kept_idx, origin_out, x_out are not touched)
 *   x           device: sample i is [N[i],*] with row_stride, at token offset sum_{j<i} N[j]
 *   origin_in   device, packed like x (one int32 per token), or NULL (identity within each sample)
 *   scores      device fp32, packed like x; written for every sample, also for one that keeps nothing
 *   kept_idx, origin_out   device int32, packed by n_keep; kept_idx counts from the start of its sample
 *   x_out       device [sum n_keep, D] dtype, or NULL
 *   workspace   luvc_spu_ragged_workspace_bytes for the same N, D, dtype, sigma
 */
size_t luvc_spu_ragged_workspace_bytes(int n_samples, const int32_t* N, int D, luvc_dtype dtype, const int32_t* sigma);
luvc_status luvc_spu_stage_ragged(const void* x, int n_samples, const int32_t* N, int D, int64_t row_stride,
                                  luvc_dtype dtype, const int32_t* sigma, int use_hamming, const int32_t* n_keep,
                                  const int32_t* origin_in, float* scores, int32_t* kept_idx, int32_t* origin_out,
                                  void* x_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Timing aid for benchmarks (not a step of the paper's method; for callers that want the duration of
 * each kernel the library launches, measured on the launch stream itself).
 *
 *   hip_events  host array of n_events hipEvent_t handles created by the caller with timing enabled
 *               (n_events even, >= 2); the caller keeps ownership and must keep them alive until
 *               luvc_profile_stop()
 * From luvc_profile_start() until luvc_profile_stop(), on the calling thread, every kernel launched by
 * a luvc_* call carries events[2i] as its start and events[2i+1] as its stop event (attached to the dispatch
 * itself, so hipEventElapsedTime of the pair is the kernel's run time on the device), i = 0, 1, ... in
 * launch order; launches beyond n_events / 2 (or 8192) are not recorded.
 * luvc_profile_stop() ends the recording and returns the number of launches recorded;
 * luvc_profile_kernel(i) names the kernel of launch i of the last recording (static string).
 * Timed launches are dispatched one by one: do not leave it on in production.
 */
luvc_status luvc_profile_start(void** hip_events, int n_events);
int luvc_profile_stop(void);
const char* luvc_profile_kernel(int i);

/*
 * Self-test aid (not a step of the paper's method): the fp32 sums the OIM screening forms with the packed bf16 dot
 * product instruction, exposed so that a test can hold them against exact sums - the error bound the screening relies
 * on (Section 3.2 decisions are fp64 decisions; fp32 only screens them) counts one rounding per product pair and one
 * per accumulation.
 *   x, y      device [rows, 2 * words] bf16: row r holds `words` pairs of elements
 *   out       device [rows] fp32: out[r] = the instruction applied to the pairs of row r in order, starting from 0
 */
luvc_status luvc_selftest_fdot2(const void* x, const void* y, int rows, int words, float* out, void* hip_stream);

/*
 * Self-test aid (not a step of the paper's method): the 32 x 32 tile of dot products that the wide matching of
 * luvc_oim_merge_wide forms on the matrix cores in the storage precision to screen its fp64 decisions (Section 3.2,
 * Algorithm 1; the decisions themselves are taken on fp64 cosines), exposed so that a test can hold it against exact
 * sums: the screening assumes |out - exact| <= D 2^-23 times the sum of the magnitudes of the products.
 *   a, c      device [32, D] rows of `dtype`, 16-byte aligned, D * element size a multiple of 16
 *   out       device [32 * 32] fp32: out[i * 32 + j] = <a_i, c_j>
 */
luvc_status luvc_selftest_screen_tile(const void* a, const void* c, int D, luvc_dtype dtype, float* out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LUVC_H */
