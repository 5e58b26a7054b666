// Internal interface between the C-ABI layer and the SPU kernels.
#pragma once
#include "common.hpp"

namespace luvc {

constexpr int kSpuMaxN = 32768;     // tokens per sample (twiddle index arithmetic stays in int32)

// Offsets (bytes) of the score kernels' scratch inside the caller's workspace.
struct SpuLayout {
    size_t tw, gk, gm, Fc, Fs, partial, gpartial, arrive, bytes;
    int n_tiles;
    bool fast;      // transform-decomposition FFT path instead of the direct pass-band DFT
};
SpuLayout spu_layout(int B, int N, int D, int sigma);

luvc_status spu_score_dense(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dt, int sigma,
                            int use_hamming, float* scores, void* workspace, hipStream_t st);

// Fast path (spu_fft.hip): N = 16 * Q * N2 with Q in {16, 15, 9}, 2 * sigma + 1 <= 16 * Q, N <= 4096.
bool spu_fft_supported(int N, int sigma);
struct TileSync;
luvc_status spu_score_fft(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dt, int sigma, int use_hamming,
                          float* partial, float* gpartial, const TileSync& sy, int n_tiles, float* scores, hipStream_t st);

luvc_status spu_prune_run(const void* x, const float* scores, int B, int N, int D, int64_t row_stride, luvc_dtype dt,
                          int n_keep, int32_t* kept_idx, void* x_out, const int32_t* origin_in, int32_t* origin_out, hipStream_t st);

}  // namespace luvc
