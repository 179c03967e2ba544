// kv_reorganize, bf16: gathers valid tokens from the paged pool into the
// group-contiguous buffer (Alg. 1 Part 2; Sec. 3.2 consolidation), writing the
// tile layout that the decode kernel streams (see packinfer.h).
//
// One workgroup moves one tile: 32 buffer tokens of one KV head (K and V).
// Rows are read from the pages with 16-byte loads (a token's head row is 2*D
// contiguous bytes), staged in LDS, and written out as whole contiguous tiles,
// so both the HBM reads and the HBM writes are coalesced; the shuffle into
// MFMA operand order happens in LDS.  HBM-bound: 2 * D * 2 bytes read and the
// same written per token and head.
#include "common.hip.h"
#include "kernels.h"

namespace pk {
namespace {

template <int D>
__global__ __launch_bounds__(256) void reorg_bf16_kernel(ReorgArgs a) {
    constexpr int CH = D / 8;                     // 16-byte chunks per token row
    constexpr int KP = D * 2 + 16;                // LDS pitch of K rows (bytes)
    constexpr int VP = D * 2 + 8;                 // LDS pitch of V rows (bytes)
    __shared__ __align__(16) unsigned char k_s[32 * KP];
    __shared__ __align__(16) unsigned char v_s[32 * VP + 16];
    __shared__ int64_t src_s[32];                 // source token slot per buffer token, -1 = hole

    const int blk = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    if (tid < 32) {
        const int64_t tok = static_cast<int64_t>(blk) * 32 + tid;
        int s = a.blk_first[blk];
        while (s < a.n_seg && static_cast<int64_t>(a.seg[4 * s]) + a.seg[4 * s + 1] <= tok) ++s;
        int64_t src = -1;
        if (s < a.n_seg && a.seg[4 * s] <= tok) {
            const int req = a.seg[4 * s + 2];
            const int64_t pos = a.seg[4 * s + 3] + (tok - a.seg[4 * s]);
            int64_t page = a.block_table[static_cast<int64_t>(req) * a.max_blocks + pos / a.page_size];
            page = page < 0 ? 0 : (page >= a.num_blocks ? a.num_blocks - 1 : page);
            src = page * a.page_size + pos % a.page_size;
        }
        src_s[tid] = src;
    }
    __syncthreads();
    // (a tile without any valid token is written as zeros too: tokens appended later into the
    // headroom share tiles with such slots, and a masked key must not meet stale bits in V)
    const u32x4* kp = static_cast<const u32x4*>(a.k_pages);
    const u32x4* vp = static_cast<const u32x4*>(a.v_pages);
    for (int x = tid; x < 32 * CH; x += 256) {
        const int tok = x / CH, c = x % CH;
        const int64_t src = src_s[tok];
        u32x4 kv = {0u, 0u, 0u, 0u}, vv = kv;
        if (src >= 0) {                           // pages are read once: keep them out of the caches
            const int64_t off = (src * a.Hkv + h) * CH + c;
            kv = __builtin_nontemporal_load(kp + off);
            vv = __builtin_nontemporal_load(vp + off);
        }
        *reinterpret_cast<u32x4*>(k_s + tok * KP + c * 16) = kv;
        uint2* vd = reinterpret_cast<uint2*>(v_s + tok * VP + c * 16);
        vd[0] = make_uint2(vv[0], vv[1]);
        vd[1] = make_uint2(vv[2], vv[3]);
    }
    __syncthreads();

    const int64_t n_tiles = a.buf_tokens / 32;
    u32x4* tile = static_cast<u32x4*>(a.kv_buf) +
                  (static_cast<int64_t>(h) * n_tiles + blk) * (2 * 32 * CH);
    // K part: chunk (u, s, l)[j] = K[16u + l%16][32s + 8(l/16) + j]
    for (int o = tid; o < 32 * CH; o += 256) {
        const int l = o & 63, s = (o >> 6) % (D / 32), u = o / (64 * (D / 32));
        const int tok = 16 * u + (l & 15), c = 4 * s + (l >> 4);
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(k_s + tok * KP + c * 16), tile + o);
    }
    // V part: chunk (t, l)[j] = V[kappa(l/16, j)][16t + l%16]
    for (int o = tid; o < 32 * CH; o += 256) {
        const int l = o & 63, t = o >> 6;
        const int g = l >> 4, col = 16 * t + (l & 15);
        uint16_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int tok = j < 4 ? 4 * g + j : 16 + 4 * g + (j - 4);
            e[j] = *reinterpret_cast<const uint16_t*>(v_s + tok * VP + col * 2);
        }
        u32x4 w;
        w[0] = e[0] | (static_cast<uint32_t>(e[1]) << 16);
        w[1] = e[2] | (static_cast<uint32_t>(e[3]) << 16);
        w[2] = e[4] | (static_cast<uint32_t>(e[5]) << 16);
        w[3] = e[6] | (static_cast<uint32_t>(e[7]) << 16);
        __builtin_nontemporal_store(w, tile + 32 * CH + o);
    }
}

// The token that decode step `step` produced goes into the headroom behind its request's suffix
// (Sec. 3.2, M(Q_i) = L_Q + delta), in the tile layout above.  One workgroup per (request, KV
// head), one thread per column; a K row is D/8 whole 16-byte chunks, a V row is D single elements.
template <int D>
__global__ __launch_bounds__(D) void append_bf16_kernel(AppendArgs a) {
    constexpr int CH = D / 8;
    const int i = blockIdx.x, h = blockIdx.y, c = threadIdx.x;
    const int32_t* seg = a.req_seg + 4 * i;
    const int64_t tok = static_cast<int64_t>(seg[2]) + seg[3] + a.step;
    const int64_t tile = tok / 32;
    const int tt = static_cast<int>(tok % 32);
    const int64_t n_tiles = a.buf_tokens / 32;
    uint16_t* base = static_cast<uint16_t*>(a.kv_buf) + (static_cast<int64_t>(h) * n_tiles + tile) * (2 * 32 * CH) * 8;
    const int64_t src = (static_cast<int64_t>(i) * a.Hkv + h) * D + c;
    // K: chunk (u, s, l)[j] = K[16u + l%16][32s + 8(l/16) + j]
    {
        const int u = tt >> 4, s = c >> 5, gq = (c & 31) >> 3, j = c & 7, l = 16 * gq + (tt & 15);
        base[((u * (D / 32) + s) * 64 + l) * 8 + j] = static_cast<const uint16_t*>(a.k_new)[src];
    }
    // V: chunk (t, l)[j] = V[kappa(l/16, j)][16t + l%16], kappa(g, j) = 4g + j (j < 4), 16 + 4g + (j - 4)
    {
        const int g = tt < 16 ? tt >> 2 : (tt - 16) >> 2, j = tt < 16 ? tt & 3 : 4 + ((tt - 16) & 3);
        const int t = c >> 4, l = 16 * g + (c & 15);
        base[(32 * CH + t * 64 + l) * 8 + j] = static_cast<const uint16_t*>(a.v_new)[src];
    }
}

}  // namespace

int launch_append_bf16(const AppendArgs& a, void* stream) {
    if (a.n == 0) return 0;
    dim3 grid(static_cast<unsigned>(a.n), static_cast<unsigned>(a.Hkv));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.d == 128) hipLaunchKernelGGL(append_bf16_kernel<128>, grid, dim3(128), 0, st, a);
    else if (a.d == 64) hipLaunchKernelGGL(append_bf16_kernel<64>, grid, dim3(64), 0, st, a);
    else return static_cast<int>(hipErrorInvalidValue);
    return static_cast<int>(hipGetLastError());
}

int launch_reorg_bf16(const ReorgArgs& a, void* stream) {
    const int64_t n_tiles = a.buf_tokens / 32;
    if (n_tiles == 0) return 0;
    dim3 grid(static_cast<unsigned>(n_tiles), static_cast<unsigned>(a.Hkv));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.d == 128) hipLaunchKernelGGL(reorg_bf16_kernel<128>, grid, dim3(256), 0, st, a);
    else if (a.d == 64) hipLaunchKernelGGL(reorg_bf16_kernel<64>, grid, dim3(256), 0, st, a);
    else return static_cast<int>(hipErrorInvalidValue);
    return static_cast<int>(hipGetLastError());
}

}  // namespace pk
