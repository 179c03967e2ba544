// Packed decode attention (Sec. 3.2): one query row per request over the
// group-contiguous buffer, split-KV partials and a log-sum-exp merge.
//
// A work item is a run of buffer tokens [tok_begin, tok_end) of one segment
// (a shared prefix or a private suffix) together with the requests whose
// queries attend to it: one request for a suffix, all members of the
// (sub-)family for a prefix -- the prefix is streamed from HBM once and used
// for every member's rows.  One wave handles (work item, KV head): the query
// rows of up to 32/r requests x r heads sit on the N side of 16x16x32 bf16
// MFMAs, the buffer tiles are already in MFMA operand order, so every load is
// a fully coalesced 16-byte-per-lane read straight into the operand
// registers (no LDS).  HBM-bound: 4*D bytes per token and KV head.
#include <mutex>

#include "../../include/packinfer.h"
#include "common.hip.h"
#include "decode_body.hip.h"
#include "kernels.h"

namespace pk {
namespace {

// Work items with at most 16 query rows: one column tile, tile loads double buffered.
template <int D>
__global__ __launch_bounds__(64) void decode_bf16_kernel(DecodeArgs a) {
    decode_body<D, 1, 1>(a, blockIdx.x, blockIdx.y);
}

// Batches with shared prefixes: the first n_wide work items carry 17..32 query rows (two column
// tiles).  Both kinds run in ONE launch so that the short prefix pass and the suffix pass fill
// the chip together; occupancy, not register prefetch, hides the load latency here.
template <int D>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void decode_bf16_mixed_kernel(DecodeArgs a) {
    if (static_cast<int>(blockIdx.x) < a.n_wide) decode_body<D, 2, 2>(a, blockIdx.x, blockIdx.y);
    else decode_body<D, 1, 2>(a, blockIdx.x, blockIdx.y);
}

// out[i, h, :] = sum_j exp(lse_j - lse) o_j over the request's partial slots (consecutive).
// Workgroup = (request, head), WAVES waves; wave w takes slots w, w + WAVES, ... four at a time
// (all loads of a batch are issued before the first use), every lane owns D/64 columns; with
// more than one wave the partial sums meet in LDS.  One wave is enough when no request has more
// than a handful of partial results (short launches then end sooner).  Requests with a single
// work item were written by the decode kernel and are skipped.
template <int D, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void decode_merge_kernel(DecodeArgs a) {
    constexpr int CPL = D / 64;                    // columns per lane
    __shared__ float red_acc[WAVES][D];
    __shared__ float red_tot[WAVES];
    const int i = blockIdx.x, h = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p0 = a.req_part_start[i], p1 = a.req_part_start[i + 1];
    if (p1 <= p0) return;
    const float* lse_base = a.part_lse + h;
    float mx = -INFINITY;
    for (int p = p0 + lane; p < p1; p += 64) mx = fmaxf(mx, lse_base[static_cast<int64_t>(p) * a.Hq]);
    mx = wave_max(mx);
    float acc[CPL], tot = 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;
    for (int p = p0 + wave; p < p1; p += 4 * WAVES) {
        float lse[4], v[4][CPL];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = p + WAVES * u;
            lse[u] = q < p1 ? lse_base[static_cast<int64_t>(q) * a.Hq] : -INFINITY;
#pragma unroll
            for (int c = 0; c < CPL; ++c)
                v[u][c] = q < p1 ? a.part_o[(static_cast<int64_t>(q) * a.Hq + h) * D + lane * CPL + c] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = (lse[u] == -INFINITY) ? 0.f : expf(lse[u] - mx);
            tot += w;
#pragma unroll
            for (int c = 0; c < CPL; ++c) acc[c] = fmaf(w, v[u][c], acc[c]);
        }
    }
    if constexpr (WAVES > 1) {
#pragma unroll
        for (int c = 0; c < CPL; ++c) red_acc[wave][lane * CPL + c] = acc[c];
        if (lane == 0) red_tot[wave] = tot;
        __syncthreads();
        if (wave != 0) return;
        tot = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) tot += red_tot[w];
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            acc[c] = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) acc[c] += red_acc[w][lane * CPL + c];
        }
    }
    const float inv = tot > 0.f ? 1.f / tot : 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int col = lane * CPL + c;
        const int64_t dst = (static_cast<int64_t>(i) * a.Hq + h) * D + col;
        if (a.out_f32) static_cast<float*>(a.out)[dst] = acc[c] * inv;
        else static_cast<uint16_t*>(a.out)[dst] = float_to_bf16_bits(acc[c] * inv);
    }
}

template <int D>
void launch_merge(const DecodeArgs& a, hipStream_t st) {
    if (a.n > 0 && a.max_parts > 0) {
        const dim3 mgrid(static_cast<unsigned>(a.n), static_cast<unsigned>(a.Hq));
        if (a.max_parts <= 8) hipLaunchKernelGGL((decode_merge_kernel<D, 1>), mgrid, dim3(64), 0, st, a);
        else hipLaunchKernelGGL((decode_merge_kernel<D, 4>), mgrid, dim3(256), 0, st, a);
    }
}

template <int D>
int launch_d(const DecodeArgs& a, hipStream_t st) {
    if (a.n_items > 0) {
        dim3 grid(static_cast<unsigned>(a.n_items), static_cast<unsigned>(a.Hkv));
        if (a.n_wide > 0) hipLaunchKernelGGL(decode_bf16_mixed_kernel<D>, grid, dim3(64), 0, st, a);
        else hipLaunchKernelGGL(decode_bf16_kernel<D>, grid, dim3(64), 0, st, a);
    }
    launch_merge<D>(a, st);
    return static_cast<int>(hipGetLastError());
}

}  // namespace

// Scratch of pk_packed_decode_attn_static (plan tables + split-KV partials) for callers that
// cannot allocate.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address differs per GPU and is looked up once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[PK_STATIC_SCRATCH_BYTES];

int static_scratch_address(void** ptr) {
    constexpr int kMaxDevices = 64;
    static std::mutex mutex;
    static void* address[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return static_cast<int>(e);
    if (dev < 0 || dev >= kMaxDevices) return static_cast<int>(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(mutex);
    if (!address[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return static_cast<int>(e);
        if (!p) return static_cast<int>(hipErrorInvalidSymbol);
        address[dev] = p;
    }
    *ptr = address[dev];
    return 0;
}

int launch_decode_merge_bf16(const DecodeArgs& a, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.d == 128) launch_merge<128>(a, st);
    else if (a.d == 64) launch_merge<64>(a, st);
    else return static_cast<int>(hipErrorInvalidValue);
    return static_cast<int>(hipGetLastError());
}

int launch_decode_bf16(const DecodeArgs& a, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.d == 128) return launch_d<128>(a, st);
    if (a.d == 64) return launch_d<64>(a, st);
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace pk
