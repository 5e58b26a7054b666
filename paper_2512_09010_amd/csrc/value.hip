// Value enhancement (paper Section 3.2, Eq. 3): the values that enter attention are V + log(s), where s is
// the number of tokens merged into each token; the logarithm is added to every channel of the token's row.
//
// One wavefront owns kRows consecutive rows: the first kRows lanes take the fp64 logarithms of their rows'
// sizes (one pass through the log code for all of them), every row is then streamed with 16-byte accesses,
// the sum formed in fp64 and rounded once to the storage type.  Bound: HBM, 2 * rows * D * e bytes.
#include "common.hpp"
#include "oim.hpp"

namespace luvc {

constexpr int kVeRows = 8;

template <typename T, bool VECTOR>
__global__ void __launch_bounds__(256)
value_enhance(const T* __restrict__ v, const int32_t* __restrict__ sizes, int64_t rows, int D, int64_t v_stride, int64_t out_stride,
              T* __restrict__ out)
{
    using tr = io_traits<T>;
    constexpr int V = tr::kVec;
    const int lane = threadIdx.x & 63;
    const int64_t row0 = (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6) * kVeRows;
    if (row0 >= rows) return;
    const int64_t mine = row0 + (lane < kVeRows ? lane : 0);
    const int s_mine = mine < rows ? sizes[mine] : 1;
    const double ls_mine = log((double)(s_mine < 1 ? 1 : s_mine));
    for (int r = 0; r < kVeRows; ++r) {
        const int64_t row = row0 + r;
        if (row >= rows) break;
        const double ls = __shfl(ls_mine, r, kWave);
        const T* in = v + row * v_stride;
        T* o = out + row * out_stride;
        if (VECTOR) {
            for (int d = lane * V; d < D; d += 64 * V) {
                float f[V];
                tr::unpack(*reinterpret_cast<const typename tr::vec_t*>(in + d), f);
                T q[V];
#pragma unroll
                for (int i = 0; i < V; ++i) tr::store(&q[i], (double)f[i] + ls);
                *reinterpret_cast<typename tr::vec_t*>(o + d) = *reinterpret_cast<const typename tr::vec_t*>(q);
            }
        } else {
            for (int d = lane; d < D; d += 64) tr::store(o + d, (double)tr::load(in + d) + ls);
        }
    }
}

luvc_status value_enhance_run(const void* v, const int32_t* sizes, int64_t rows, int D, int64_t v_stride, int64_t out_stride,
                              luvc_dtype dt, void* out, hipStream_t st)
{
    const size_t es = dt == LUVC_F32 ? 4 : 2;
    const bool vec = ((size_t)D * es) % 16 == 0 && ((size_t)v_stride * es) % 16 == 0 && ((size_t)out_stride * es) % 16 == 0 &&
                     (uintptr_t)v % 16 == 0 && (uintptr_t)out % 16 == 0;
    const int64_t waves = (rows + kVeRows - 1) / kVeRows;
    const unsigned g = (unsigned)((waves * 64 + 255) / 256);
#define LUVC_VE(TT, VV) LUVC_LAUNCH("value_enhance", (value_enhance<TT, VV>), dim3(g), dim3(256), 0, st, (const TT*)v, sizes, rows, D, v_stride, out_stride, (TT*)out)
    if (dt == LUVC_F32) { if (vec) LUVC_VE(float, true); else LUVC_VE(float, false); }
    else                { if (vec) LUVC_VE(bf16_t, true); else LUVC_VE(bf16_t, false); }
#undef LUVC_VE
    return check_launch("value enhancement");
}

}  // namespace luvc
