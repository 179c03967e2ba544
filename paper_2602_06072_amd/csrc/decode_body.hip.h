// Device code of the packed decode work item (Sec. 3.2), shared by the decode kernels and by the
// fused mixed-step kernel: one wave handles (work item, KV head).
#pragma once
#include "common.hip.h"
#include "kernels.h"

namespace pk {
namespace {

// PREFETCH: 0 = one tile at a time; 1 = two register sets (the loads of tile b+1 are in flight while
// tile b is processed); 2 = one register set, rolling: the K part of tile b+1 is requested as soon as
// the scores of tile b are done and its V part as soon as P.V of tile b is done, so that each half of
// the next tile is in flight under the other half's arithmetic without a second set of registers
// (for work items with two column tiles of query rows, which have no registers to spare).
template <int D, int NT, int PREFETCH>
__device__ __forceinline__ void decode_body(const DecodeArgs& a, const int item, const int kvh) {
    constexpr int KS = D / 32;                 // K steps per 16-key sub-tile
    constexpr int VT = D / 16;                 // V column blocks
    constexpr int NK = 2 * KS;                 // 16-byte chunks per lane of a tile's K part
    constexpr int TILE_U4 = 2 * 32 * (D / 8);  // 16-byte chunks per tile (K part + V part)
    const int lane = threadIdx.x & 63, n = lane & 15, g = lane >> 4;   // (one wave per work item and KV head)
    const int r = a.Hq / a.Hkv;
    const int32_t* it = a.items + 8 * static_cast<int64_t>(item);
    // the last item of a suffix also covers the tokens appended since the plan was made
    const int tok_begin = it[0], tok_end = it[1] + (it[4] ? a.grown : 0), mem_first = it[2], n_mem = it[3];
    const int64_t n_tiles = a.buf_tokens / 32;
    const u32x4* base = static_cast<const u32x4*>(a.kv_buf) + static_cast<int64_t>(kvh) * n_tiles * TILE_U4 + lane;
    const int b0 = tok_begin / 32, b1 = (tok_end + 31) / 32;

    // Two register sets: the loads of tile b+1 are in flight while tile b is processed.  The
    // first tile is requested before anything else so that it overlaps the query set-up.
    u32x4 ka[NK], va[VT], kb_[NK], vb_[VT];
#define PK_LOAD_TILE(KR, VR, B)                                                      \
    {                                                                                \
        const u32x4* tile_ = base + static_cast<int64_t>(B) * TILE_U4;               \
        _Pragma("unroll") for (int i = 0; i < NK; ++i) KR[i] = __builtin_nontemporal_load(tile_ + i * 64);        \
        _Pragma("unroll") for (int i = 0; i < VT; ++i) VR[i] = __builtin_nontemporal_load(tile_ + (NK + i) * 64); \
    }
    PK_LOAD_TILE(ka, va, b0);

    // query operand (B side): lane (n, g) holds Q[row n][32s + 8g .. +8]
    bf16x8 qf[NT][KS];
    int req_of[NT], hq_of[NT], slot_of[NT];
#pragma unroll
    for (int c = 0; c < NT; ++c) {
        const int mi = (c * 16 + n) / r;
        const bool ok = mi < n_mem;
        req_of[c] = ok ? a.members[mem_first + mi] : -1;
        slot_of[c] = ok ? a.member_slot[mem_first + mi] : -1;
        hq_of[c] = kvh * r + (c * 16 + n) % r;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (ok) raw = *reinterpret_cast<const u32x4*>(
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
    const float sl2 = a.scale * kLog2e;

    // scores and probabilities of tile b for column tile c: leaves P (bf16, B operand) and the
    // factor alpha for what has been accumulated so far
    auto scores = [&](const u32x4 (&kraw)[NK], int b, int c, bf16x8& pf, float& alpha) {
        const bool edge = (b * 32 < tok_begin) || (b * 32 + 32 > tok_end);
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[s]), qf[c][s], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[KS + s]), qf[c][s], s1, 0, 0, 0);
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
        alpha = __builtin_amdgcn_exp2f(m[c] - m_use);      // 0 on the first tile
        float ps = 0.f;
        uint32_t pw[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            floatx2 pp;
            pp[0] = __builtin_amdgcn_exp2f(x[2 * j] - m_use);
            pp[1] = __builtin_amdgcn_exp2f(x[2 * j + 1] - m_use);
            ps += pp[0] + pp[1];
            pw[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, bf16x2));
        }
        l[c] = l[c] * alpha + ps;
        m[c] = m_new;
        pf = __builtin_bit_cast(bf16x8, u32x4{pw[0], pw[1], pw[2], pw[3]});
    };
    auto pv = [&](const u32x4 (&vraw)[VT], int c, const bf16x8& pf, float alpha) {
#pragma unroll
        for (int t = 0; t < VT; ++t) {
            floatx4 acc = o[c][t];
            acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
            o[c][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vraw[t]), pf, acc, 0, 0, 0);
        }
    };
    auto process = [&](const u32x4 (&kraw)[NK], const u32x4 (&vraw)[VT], int b) {
#pragma unroll
        for (int c = 0; c < NT; ++c) {
            bf16x8 pf;
            float alpha;
            scores(kraw, b, c, pf, alpha);
            pv(vraw, c, pf, alpha);
        }
    };

    if (PREFETCH == 2) {
        for (int b = b0; b < b1; ++b) {
            bf16x8 pf[NT];
            float alpha[NT];
#pragma unroll
            for (int c = 0; c < NT; ++c) scores(ka, b, c, pf[c], alpha[c]);
            if (b + 1 < b1) {                       // K registers are free: the next tile's K part
                const u32x4* tile_ = base + static_cast<int64_t>(b + 1) * TILE_U4;
#pragma unroll
                for (int i = 0; i < NK; ++i) ka[i] = __builtin_nontemporal_load(tile_ + i * 64);
            }
#pragma unroll
            for (int c = 0; c < NT; ++c) pv(va, c, pf[c], alpha[c]);
            if (b + 1 < b1) {                       // V registers are free: the next tile's V part
                const u32x4* tile_ = base + static_cast<int64_t>(b + 1) * TILE_U4;
#pragma unroll
                for (int i = 0; i < VT; ++i) va[i] = __builtin_nontemporal_load(tile_ + (NK + i) * 64);
            }
        }
    } else if (PREFETCH == 1) {
        for (int b = b0; b < b1; b += 2) {
            if (b + 1 < b1) PK_LOAD_TILE(kb_, vb_, b + 1);
            process(ka, va, b);
            if (b + 1 < b1) {
                if (b + 2 < b1) PK_LOAD_TILE(ka, va, b + 2);
                process(kb_, vb_, b + 1);
            }
        }
    } else {
        for (int b = b0; b < b1; ++b) {
            if (b > b0) PK_LOAD_TILE(ka, va, b);
            process(ka, va, b);
        }
    }
#undef PK_LOAD_TILE

#pragma unroll
    for (int c = 0; c < NT; ++c) {
        float lt = l[c];
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        if (req_of[c] < 0) continue;
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        if (slot_of[c] < 0) {
            // the only work item of this request: write the final output
            const int64_t dst = (static_cast<int64_t>(req_of[c]) * a.Hq + hq_of[c]) * D;
#pragma unroll
            for (int t = 0; t < VT; ++t) {
                const float x0 = o[c][t][0] * inv, x1 = o[c][t][1] * inv, x2 = o[c][t][2] * inv, x3 = o[c][t][3] * inv;
                if (a.out_f32)
                    *reinterpret_cast<float4*>(static_cast<float*>(a.out) + dst + 16 * t + 4 * g) = make_float4(x0, x1, x2, x3);
                else
                    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + dst + 16 * t + 4 * g) =
                        make_uint2(pack_bf16x2(x0, x1), pack_bf16x2(x2, x3));
            }
            continue;
        }
        const int slot = slot_of[c];
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

}  // namespace
}  // namespace pk
