// Packed prefill attention, bf16 MFMA, head dimensions 128 and 64 (Sec. 3.1): the launches.  The
// kernels' device code is in prefill_body.hip.h, included once per head dimension.
#define PK_D 128
#define PK_DNS d128
#include "prefill_body.hip.h"
#undef PK_D
#undef PK_DNS
#define PK_D 64
#define PK_DNS d64
#include "prefill_body.hip.h"
#undef PK_D
#undef PK_DNS

namespace pk {
namespace {

__global__ __launch_bounds__(256, 2) void prefill_bf16_dma_kernel(PrefillArgs a) {
    __shared__ __align__(1024) unsigned char lds[5 * d128::TILE_BYTES];
    d128::prefill_tile_body(a, static_cast<int>(blockIdx.x), lds);
}

__global__ __launch_bounds__(256, 2) void prefill_bf16_dma64_kernel(PrefillArgs a) {
    __shared__ __align__(1024) unsigned char lds[5 * d64::TILE_BYTES];
    d64::prefill_tile_body(a, static_cast<int>(blockIdx.x), lds);
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
    if (a.d == 128)
        hipLaunchKernelGGL(prefill_bf16_dma_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), a);
    else if (a.d == 64)
        hipLaunchKernelGGL(prefill_bf16_dma64_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), a);
    else
        return static_cast<int>(hipErrorInvalidValue);
    return static_cast<int>(hipGetLastError());
}

}  // namespace pk
