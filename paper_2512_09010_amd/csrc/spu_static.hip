// luvc_spu_score_static: the SPU score (paper Section 3.3, Eq. 4-8) for callers that cannot hand over a
// workspace because they cannot allocate one - code under HIP graph capture, tight serving loops, harnesses
// that forbid hipMalloc.  Same kernels as luvc_spu_score; the scratch they need (tile energies, group sums,
// arrival words, and for the three-launch path the tables and pass-band spectra) sits in a static
// device array of this library instead of the caller's workspace.
#include <atomic>

#include "common.hpp"
#include "spu.hpp"

namespace luvc {
namespace {

constexpr size_t kStaticScratchBytes = LUVC_SPU_STATIC_SCRATCH_BYTES;

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress: the address kernels can use is looked up below, once per device.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// device address of `scratch` on the current device (nullptr with the error text set)
void* static_scratch()
{
    constexpr int kMaxDev = 64;
    static std::atomic<void*> base_of[kMaxDev];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) {
        (void)hipGetLastError();
        set_error("luvc_spu_score_static: no current device");
        return nullptr;
    }
    void* base = base_of[dev].load(std::memory_order_acquire);
    if (!base) {
        const hipError_t e = hipGetSymbolAddress(&base, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !base) {
            (void)hipGetLastError();
            set_error("luvc_spu_score_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
            return nullptr;
        }
        base_of[dev].store(base, std::memory_order_release);
    }
    return base;
}

}  // namespace
}  // namespace luvc

extern "C" luvc_status luvc_spu_score_static(const void* x, int B, int N, int D, int64_t row_stride, luvc_dtype dtype,
                                             int sigma, int use_hamming, float* scores, void* hip_stream)
{
    using namespace luvc;
    const size_t need = luvc_spu_workspace_bytes(B, N, D, dtype, sigma);
    // invalid arguments (need == 0): the checks of luvc_spu_score name the problem; no workspace is looked at before they fail
    if (need == 0) return luvc_spu_score(x, B, N, D, row_stride, dtype, sigma, use_hamming, scores, nullptr, 0, hip_stream);
    if (need > kStaticScratchBytes) {
        set_error("luvc_spu_score_static: B=%d N=%d D=%d sigma=%d needs %zu bytes of scratch, the static buffer holds %zu; "
                  "use luvc_spu_score with a workspace", B, N, D, sigma, need, kStaticScratchBytes);
        return LUVC_ERR_WORKSPACE;
    }
    void* ws = static_scratch();
    if (!ws) return LUVC_ERR_HIP;
    // nothing in the scratch has to start at zero: tile energies and group sums are written before they are read, and
    // the arrival words recognise what an earlier call left behind by its tag
    return luvc_spu_score(x, B, N, D, row_stride, dtype, sigma, use_hamming, scores, ws, kStaticScratchBytes, hip_stream);
}
