// Packed prefill attention, bf16 MFMA, head dimension 128 (Sec. 3.1): the launch.  The kernel's
// device code is in prefill_body.hip.h.
#include "prefill_body.hip.h"

namespace pk {
namespace {

__global__ __launch_bounds__(256, 2) void prefill_bf16_dma_kernel(PrefillArgs a) {
    __shared__ __align__(1024) unsigned char lds[5 * TILE_BYTES];
    prefill_tile_body(a, static_cast<int>(blockIdx.x), lds);
}

}  // namespace

int launch_prefill_bf16_pipe(const PrefillArgs& a, void* stream) {
    const int r = a.Hq / a.Hkv;
    int64_t grid;
    if (a.xcd_swizzle) {
        const int64_t pairs = static_cast<int64_t>(a.n_tiles) * a.Hkv;
        grid = (pairs + 7) / 8 * 8 * r;
    } else {
        grid = static_cast<int64_t>(a.n_tiles) * a.Hq;
    }
    if (grid == 0) return 0;
    hipLaunchKernelGGL(prefill_bf16_dma_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace pk
