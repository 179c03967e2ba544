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
#include "common.hip.h"
#include "kernels.h"

namespace pk {
namespace {

template <int D, int NT>
__global__ __launch_bounds__(64) void decode_bf16_kernel(DecodeArgs a) {
    constexpr int KS = D / 32;                 // K steps per 16-key sub-tile
    constexpr int VT = D / 16;                 // V column blocks
    constexpr int TILE_U4 = 2 * 32 * (D / 8);  // uint4 per tile (K part + V part)
    const int lane = threadIdx.x, n = lane & 15, g = lane >> 4;
    const int kvh = blockIdx.y;
    const int r = a.Hq / a.Hkv;
    const int32_t* it = a.items + 8 * static_cast<int64_t>(blockIdx.x);
    const int tok_begin = it[0], tok_end = it[1], mem_first = it[2], n_mem = it[3], part_base = it[4];

    // query operand (B side): lane (n, g) holds Q[row n][32s + 8g .. +8]
    bf16x8 qf[NT][KS];
    int req_of[NT], hq_of[NT];
#pragma unroll
    for (int c = 0; c < NT; ++c) {
        const int mi = (c * 16 + n) / r;
        const bool ok = mi < n_mem;
        req_of[c] = ok ? a.members[mem_first + mi] : -1;
        hq_of[c] = kvh * r + (c * 16 + n) % r;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (ok) raw = *reinterpret_cast<const uint4*>(
                static_cast<const uint16_t*>(a.q) +
                (static_cast<int64_t>(req_of[c]) * a.Hq + hq_of[c]) * D + 32 * s + 8 * g);
            qf[c][s] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    floatx4 o[NT][VT];
    float m[NT], l[NT];
#pragma unroll
    for (int c = 0; c < NT; ++c) {
        m[c] = -INFINITY; l[c] = 0.f;
#pragma unroll
        for (int t = 0; t < VT; ++t) o[c][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    const int64_t n_tiles = a.buf_tokens / 32;
    const uint4* base = static_cast<const uint4*>(a.kv_buf) + static_cast<int64_t>(kvh) * n_tiles * TILE_U4;
    const int b0 = tok_begin / 32, b1 = (tok_end + 31) / 32;
    const float sl2 = a.scale * kLog2e;

    for (int b = b0; b < b1; ++b) {
        const uint4* tile = base + static_cast<int64_t>(b) * TILE_U4;
        uint4 kraw[2][KS], vraw[VT];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int s = 0; s < KS; ++s) kraw[u][s] = tile[(u * KS + s) * 64 + lane];
#pragma unroll
        for (int t = 0; t < VT; ++t) vraw[t] = tile[2 * KS * 64 + t * 64 + lane];

        const bool edge = (b * 32 < tok_begin) || (b * 32 + 32 > tok_end);
#pragma unroll
        for (int c = 0; c < NT; ++c) {
            floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[0][s]), qf[c][s], s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[1][s]), qf[c][s], s1, 0, 0, 0);
            }
            // lane (n, g) now holds scores of row n against keys 32b + 16u + 4g + j
            float x[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) { x[j] = s0[j] * sl2; x[4 + j] = s1[j] * sl2; }
            if (edge) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int key = b * 32 + (j < 4 ? 4 * g + j : 16 + 4 * g + (j - 4));
                    if (key < tok_begin || key >= tok_end) x[j] = -INFINITY;
                }
            }
            float mx = x[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) mx = fmaxf(mx, x[j]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m[c], mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = exp2f(m[c] - m_use);      // 0 on the first tile
            float p[8], ps = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) { p[j] = exp2f(x[j] - m_use); ps += p[j]; }
            l[c] = l[c] * alpha + ps;
            m[c] = m_new;
            uint4 pw;
            pw.x = pack_bf16x2(p[0], p[1]); pw.y = pack_bf16x2(p[2], p[3]);
            pw.z = pack_bf16x2(p[4], p[5]); pw.w = pack_bf16x2(p[6], p[7]);
            const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
            for (int t = 0; t < VT; ++t) {
                floatx4 acc = o[c][t];
                acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
                o[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vraw[t]), pf, acc, 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int c = 0; c < NT; ++c) {
        float lt = l[c];
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        if (req_of[c] < 0) continue;
        const int slot = part_base + (c * 16 + n) / r;
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        float* po = a.part_o + (static_cast<int64_t>(slot) * a.Hq + hq_of[c]) * D;
#pragma unroll
        for (int t = 0; t < VT; ++t) {
            float4 w = make_float4(o[c][t][0] * inv, o[c][t][1] * inv, o[c][t][2] * inv, o[c][t][3] * inv);
            *reinterpret_cast<float4*>(po + 16 * t + 4 * g) = w;
        }
        if (g == 0)
            a.part_lse[static_cast<int64_t>(slot) * a.Hq + hq_of[c]] =
                lt > 0.f ? (m[c] + log2f(lt)) * kLn2 : -INFINITY;
    }
}

// out[i, h, :] = sum_j exp(lse_j - lse) o_j over the request's partial slots.
template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(DecodeArgs a) {
    const int i = blockIdx.x, h = blockIdx.y, c = threadIdx.x;
    const int p0 = a.req_part_start[i], p1 = a.req_part_start[i + 1];
    float mx = -INFINITY;
    for (int p = p0; p < p1; ++p)
        mx = fmaxf(mx, a.part_lse[static_cast<int64_t>(a.req_parts[p]) * a.Hq + h]);
    float acc = 0.f, tot = 0.f;
    for (int p = p0; p < p1; ++p) {
        const int64_t slot = a.req_parts[p];
        const float lse = a.part_lse[slot * a.Hq + h];
        const float w = (lse == -INFINITY) ? 0.f : expf(lse - mx);
        tot += w;
        acc = fmaf(w, a.part_o[(slot * a.Hq + h) * D + c], acc);
    }
    const float o = tot > 0.f ? acc / tot : 0.f;
    const int64_t dst = (static_cast<int64_t>(i) * a.Hq + h) * D + c;
    if (a.out_f32) static_cast<float*>(a.out)[dst] = o;
    else static_cast<uint16_t*>(a.out)[dst] = float_to_bf16_bits(o);
}

template <int D>
int launch_d(const DecodeArgs& a, hipStream_t st) {
    if (a.n_wide > 0) {                        // items with 17..32 query rows: two column tiles
        dim3 grid(static_cast<unsigned>(a.n_wide), static_cast<unsigned>(a.Hkv));
        hipLaunchKernelGGL((decode_bf16_kernel<D, 2>), grid, dim3(64), 0, st, a);
    }
    if (a.n_items > a.n_wide) {
        DecodeArgs b = a;
        b.items = a.items + 8 * static_cast<int64_t>(a.n_wide);
        dim3 grid(static_cast<unsigned>(a.n_items - a.n_wide), static_cast<unsigned>(a.Hkv));
        hipLaunchKernelGGL((decode_bf16_kernel<D, 1>), grid, dim3(64), 0, st, b);
    }
    if (a.n > 0)
        hipLaunchKernelGGL(decode_merge_kernel<D>, dim3(static_cast<unsigned>(a.n), static_cast<unsigned>(a.Hq)),
                           dim3(D), 0, st, a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace

int launch_decode_bf16(const DecodeArgs& a, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.d == 128) return launch_d<128>(a, st);
    if (a.d == 64) return launch_d<64>(a, st);
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace pk
