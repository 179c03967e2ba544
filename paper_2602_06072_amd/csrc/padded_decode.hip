// In-run comparison for decode (Sec. 2.2, Sec. 3.2): per-request execution over
// the PAGED pool, the way request-aligned kernels run it.  Grid = (request,
// KV head, split) with the SAME number of splits for every request, sized by
// the longest one (waves of short requests exit at once); K/V are fetched
// through the block table page by page; a shared prefix is read again by every
// member of its family.  Same mathematics, MFMA scheme and load discipline as
// the packed decode kernel -- 16-byte loads, the tile after next in flight in a
// second register set while the current one is processed -- so that what is
// left between the two is the method: paged rows instead of operand-order
// tiles (K rows go straight from the pages into the A operand, one token row
// per lane; V rows have to be transposed on the way, through LDS), uniform
// splits, no prefix sharing.
#include "common.hip.h"
#include "kernels.h"

namespace pk {
namespace {

typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;

template <int D>
__global__ __launch_bounds__(64) void padded_decode_kernel(PagedDecodeArgs a) {
    constexpr int KS = D / 32, VT = D / 16, CH = D / 8;
    constexpr int VX = 32 * CH / 64;                // 16-byte chunks of a tile's V rows per lane
    constexpr int VP = D * 2 + 64;                  // LDS pitch of V rows: 4-row transpose reads hit distinct banks
    __shared__ __align__(16) unsigned char v_s[2][32 * VP];
    const int lane = threadIdx.x, n = lane & 15, g = lane >> 4;
    const int i = blockIdx.x, kvh = blockIdx.y, sp = blockIdx.z;
    const int r = a.Hq / a.Hkv;
    const int len = a.kv_start[i + 1] - a.kv_start[i];
    const int tok_begin = sp * a.split_tokens;
    const int tok_end = min(len, tok_begin + a.split_tokens);
    const int64_t slot = static_cast<int64_t>(i) * a.n_splits + sp;
    if (tok_begin >= tok_end) {                     // padded grid slot: nothing to do
        if (lane < r) a.part_lse[slot * a.Hq + kvh * r + lane] = -INFINITY;
        return;
    }
    const int32_t* bt = a.block_table + static_cast<int64_t>(i) * a.max_blocks;
    const u32x4* kp = static_cast<const u32x4*>(a.k_pages);
    const u32x4* vp = static_cast<const u32x4*>(a.v_pages);

    auto token_row = [&](int tok) -> int64_t {      // row of a logical token in the pool (clamped)
        const int tc = tok < len ? tok : len - 1;
        int64_t page = bt[tc / a.page_size];
        page = page < 0 ? 0 : (page >= a.num_blocks ? a.num_blocks - 1 : page);
        return page * a.page_size + tc % a.page_size;
    };
    // Raw loads of the tile that starts at token t0.  K operand of sub-tile u: lane (n, g) reads 16
    // bytes of token t0 + 16u + n; V: the 32 rows as coalesced 16-byte chunks.
    u32x4 ka[2][KS], va[VX], kb[2][KS], vb[VX];
#define PK_LOAD_TILE(KR, VR, T0)                                                             \
    {                                                                                        \
        _Pragma("unroll") for (int u = 0; u < 2; ++u) {                                      \
            const int64_t row_ = token_row((T0) + 16 * u + n);                               \
            _Pragma("unroll") for (int s = 0; s < KS; ++s)                                   \
                KR[u][s] = __builtin_nontemporal_load(kp + (row_ * a.Hkv + kvh) * CH + 4 * s + g); \
        }                                                                                    \
        _Pragma("unroll") for (int x = 0; x < VX; ++x) {                                     \
            const int idx_ = lane + 64 * x;                                                  \
            const int64_t row_ = token_row((T0) + idx_ / CH);                                \
            VR[x] = __builtin_nontemporal_load(vp + (row_ * a.Hkv + kvh) * CH + idx_ % CH);  \
        }                                                                                    \
    }
    PK_LOAD_TILE(ka, va, tok_begin);
    if (tok_begin + 32 < tok_end) PK_LOAD_TILE(kb, vb, tok_begin + 32);

    // query operand: lane (n, g) holds Q[head n][32s + 8g .. +8] for n < r
    bf16x8 qf[KS];
    const int hq = kvh * r + n;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (n < r) raw = *reinterpret_cast<const u32x4*>(
            static_cast<const uint16_t*>(a.q) + (static_cast<int64_t>(i) * a.Hq + hq) * D + 32 * s + 8 * g);
        qf[s] = __builtin_bit_cast(bf16x8, raw);
    }
    floatx4 o[VT];
#pragma unroll
    for (int t = 0; t < VT; ++t) o[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;
    const float sl2 = a.scale * kLog2e;

    // One tile: scores from the K registers, the V registers into the LDS buffer, then (both sets of
    // registers free again) the loads of the tile after next, softmax, and P.V from the transposed reads.
    auto process = [&](u32x4 (&kraw)[2][KS], u32x4 (&vraw)[VX], unsigned char* vbuf, int t0, bool prefetch) {
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[0][s]), qf[s], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[1][s]), qf[s], s1, 0, 0, 0);
        }
#pragma unroll
        for (int x = 0; x < VX; ++x) {
            const int idx = lane + 64 * x;
            *reinterpret_cast<u32x4*>(vbuf + (idx / CH) * VP + (idx % CH) * 16) = vraw[x];
        }
        if (prefetch) PK_LOAD_TILE(kraw, vraw, t0 + 64);
        float x[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) { x[j] = s0[j] * sl2; x[4 + j] = s1[j] * sl2; }
        if (t0 + 32 > tok_end) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int key = t0 + (j < 4 ? 4 * g + j : 16 + 4 * g + (j - 4));
                if (key >= tok_end) x[j] = -INFINITY;
            }
        }
        float mx = x[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) mx = fmaxf(mx, x[j]);
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);
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
        l = l * alpha + ps;
        m = m_new;
        const bf16x8 pf = __builtin_bit_cast(bf16x8, u32x4{pw[0], pw[1], pw[2], pw[3]});
        __syncthreads();                            // one wave: the LDS writes above are visible
        // V^T operand of column block t: lane (n, g) needs V[keys 4g..4g+3 and 16+4g..][16t + n]
#pragma unroll
        for (int t = 0; t < VT; ++t) {
            const unsigned char* p0 = vbuf + (4 * g + (n >> 2)) * VP + (16 * t + 4 * (n & 3)) * 2;
            const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
            const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0 + 16 * VP));
            const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
            floatx4 acc = o[t];
            acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
            o[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, acc, 0, 0, 0);
        }
    };
    for (int t0 = tok_begin; t0 < tok_end; t0 += 64) {
        process(ka, va, v_s[0], t0, t0 + 64 < tok_end);
        if (t0 + 32 < tok_end) process(kb, vb, v_s[1], t0 + 32, t0 + 96 < tok_end);
    }
#undef PK_LOAD_TILE
    float lt = l;
    lt += __shfl_xor(lt, 16, 64);
    lt += __shfl_xor(lt, 32, 64);
    if (n >= r) return;
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    float* po = a.part_o + (slot * a.Hq + hq) * D;
#pragma unroll
    for (int t = 0; t < VT; ++t)
        *reinterpret_cast<float4*>(po + 16 * t + 4 * g) =
            make_float4(o[t][0] * inv, o[t][1] * inv, o[t][2] * inv, o[t][3] * inv);
    if (g == 0) a.part_lse[slot * a.Hq + hq] = lt > 0.f ? (m + log2f(lt)) * kLn2 : -INFINITY;
}

// out[i, h, :] = LSE-weighted sum over the n_splits slots of request i.
template <int D>
__global__ __launch_bounds__(D) void padded_merge_kernel(PagedDecodeArgs a) {
    const int i = blockIdx.x, h = blockIdx.y, c = threadIdx.x;
    const int64_t s0 = static_cast<int64_t>(i) * a.n_splits;
    float mx = -INFINITY;
    for (int s = 0; s < a.n_splits; ++s) mx = fmaxf(mx, a.part_lse[(s0 + s) * a.Hq + h]);
    float acc = 0.f, tot = 0.f;
    for (int s = 0; s < a.n_splits; ++s) {
        const float lse = a.part_lse[(s0 + s) * a.Hq + h];
        if (lse == -INFINITY) continue;
        const float w = expf(lse - mx);
        tot += w;
        acc = fmaf(w, a.part_o[((s0 + s) * a.Hq + h) * D + c], acc);
    }
    const float o = tot > 0.f ? acc / tot : 0.f;
    const int64_t dst = (static_cast<int64_t>(i) * a.Hq + h) * D + c;
    if (a.out_f32) static_cast<float*>(a.out)[dst] = o;
    else static_cast<uint16_t*>(a.out)[dst] = float_to_bf16_bits(o);
}

template <int D>
int launch_pd(const PagedDecodeArgs& a, hipStream_t st) {
    dim3 grid(static_cast<unsigned>(a.n), static_cast<unsigned>(a.Hkv), static_cast<unsigned>(a.n_splits));
    hipLaunchKernelGGL(padded_decode_kernel<D>, grid, dim3(64), 0, st, a);
    hipLaunchKernelGGL(padded_merge_kernel<D>, dim3(static_cast<unsigned>(a.n), static_cast<unsigned>(a.Hq)),
                       dim3(D), 0, st, a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace

int launch_padded_decode_bf16(const PagedDecodeArgs& a, void* stream) {
    if (a.n == 0) return 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.d == 128) return launch_pd<128>(a, st);
    if (a.d == 64) return launch_pd<64>(a, st);
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace pk
