// Fused mixed step (Sec. 3, overview: prefill and decode requests of one continuous-batching step
// share the packed execution): the packed prefill tiles and the packed decode work items of one
// step in ONE launch.  Prefill is bound by the matrix pipe, decode by HBM; side by side on a
// compute unit they use what the other leaves idle.  The two kernels launched one after the other
// cannot do that, and launched on two streams they hardly overlap: the prefill workgroups take
// every register and LDS slot first.  Here the roles are dealt by workgroup number instead: while
// decode work remains, runs of prefill workgroups alternate with runs of decode workgroups (four
// waves, one (work item, KV head) pair each), so that each compute unit tends to hold one prefill
// and one decode workgroup; the prefill workgroups keep their numbers modulo 8, i.e. their XCD, so
// the heads of a KV head still share an L2.  The LSE merge of the decode partials is a
// second, short launch.
#include "decode_body.hip.h"
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

// Workgroups are handed to the compute units of an XCD one per unit before any unit gets its second:
// a run of kRun = 8 XCDs x 32 units prefill workgroups followed by as many decode workgroups gives
// every unit one of each (as long as both kinds last).
constexpr int kRun = 256;

// one kernel per head dimension (NS: the namespace of the prefill body, D: the head dimension)
#define PK_MIXED_STEP_KERNEL(NAME, NS, D)                                                            \
    __global__ __launch_bounds__(256, 2) void NAME(PrefillArgs pa, DecodeArgs da, int n_prefill_blocks, \
                                                   int n_decode_blocks) {                            \
        __shared__ __align__(1024) unsigned char lds[5 * NS::TILE_BYTES];                             \
        const int x = static_cast<int>(blockIdx.x);                                                  \
        const int decode_groups = (n_decode_blocks + kRun - 1) / kRun;                               \
        int prefill_block;                                                                           \
        if (x / (2 * kRun) < decode_groups) {                                                        \
            const int grp = x / (2 * kRun), pos = x % (2 * kRun);                                    \
            if (pos >= kRun) { /* a decode workgroup: four (work item, KV head) pairs */              \
                const int unit = ((grp * kRun + pos - kRun) * 4) + static_cast<int>(threadIdx.x >> 6); \
                const int item = unit / da.Hkv, kvh = unit % da.Hkv;                                 \
                if (item >= da.n_items) return;                                                      \
                if (item < da.n_wide) decode_body<D, 2, 2>(da, item, kvh);                           \
                else decode_body<D, 1, 1>(da, item, kvh);                                            \
                return;                                                                              \
            }                                                                                        \
            prefill_block = grp * kRun + pos;                                                        \
        } else {                                                                                     \
            prefill_block = x - decode_groups * kRun;                                                \
        }                                                                                            \
        if (prefill_block >= n_prefill_blocks) return;                                               \
        NS::prefill_tile_body(pa, prefill_block, lds);                                               \
    }
PK_MIXED_STEP_KERNEL(mixed_step_kernel, d128, 128)
PK_MIXED_STEP_KERNEL(mixed_step64_kernel, d64, 64)
#undef PK_MIXED_STEP_KERNEL

}  // namespace

// bf16, d = 128 or 64.  Returns a hipError_t as int.
int launch_mixed_step_bf16(const PrefillArgs& pa, const DecodeArgs& da, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int r = pa.Hq / pa.Hkv;
    const int64_t pairs = static_cast<int64_t>(pa.n_tiles) * pa.Hkv;
    const int64_t n_prefill = (pairs + 7) / 8 * 8 * r;                      // as in the prefill launch (XCD map)
    const int64_t units = static_cast<int64_t>(da.n_items) * da.Hkv;
    const int64_t n_decode = (units + 3) / 4;
    const int64_t decode_groups = (n_decode + kRun - 1) / kRun;
    // prefill workgroups beyond the interleaved stretch follow it; if there are fewer prefill than
    // decode groups the stretch is padded with workgroups that exit at once
    const int64_t grid = decode_groups * 2 * kRun + (n_prefill > decode_groups * kRun ? n_prefill - decode_groups * kRun : 0);
    if (grid > 0x7FFFFFFF) return static_cast<int>(hipErrorInvalidValue);
    if (pa.d != da.d || (pa.d != 128 && pa.d != 64)) return static_cast<int>(hipErrorInvalidValue);
    if (grid > 0) {
        if (pa.d == 128)
            hipLaunchKernelGGL(mixed_step_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0, st, pa, da,
                               static_cast<int>(n_prefill), static_cast<int>(n_decode));
        else
            hipLaunchKernelGGL(mixed_step64_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0, st, pa, da,
                               static_cast<int>(n_prefill), static_cast<int>(n_decode));
    }
    const int e = static_cast<int>(hipGetLastError());
    if (e != 0) return e;
    return launch_decode_merge_bf16(da, stream);
}

}  // namespace pk
