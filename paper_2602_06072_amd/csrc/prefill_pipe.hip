// Packed prefill attention, bf16 MFMA, head dimension 128: software-pipelined
// kernel (Sec. 3.1).  Same tables, same arithmetic and same operand scheme as
// prefill.hip (S^T = K.Q^T, O^T += V^T.P^T with v_mfma_f32_32x32x16_bf16, one
// wave per 32 query rows, key tiles of 64), but
//   * K/V tiles go HBM/L2 -> LDS directly (buffer_load ... lds, 16 bytes per
//     lane, no staging registers, hardware bounds check); rows are unpadded
//     and the 16-byte chunks of a row are XOR-swizzled -- the swizzle is
//     applied on the global side of the copy, so that both the K row reads
//     (ds_read_b128) and the V transpose reads (ds_read_b64_tr_b16) are free
//     of bank conflicts;
//   * the loop is pipelined over key tiles: iteration j issues the score
//     MFMAs of tile j+1, the PV MFMAs of tile j-1 and the softmax of tile j,
//     which are independent, hand-interleaved so that the matrix pipe runs
//     under the exponentials.  K is therefore staged two tiles ahead of the
//     softmax and V zero tiles ahead; each has two LDS stages and there is
//     one barrier per tile.
#include <cstdlib>
#include <type_traits>

#include "common.hip.h"
#include "kernels.h"

namespace pk {
namespace {

constexpr int BM = 128, BN = 64, D = 128;
constexpr int ROWB = D * 2;                        // bytes per K/V row in LDS (unpadded)
constexpr int TILE_BYTES = BN * ROWB;              // 16 KiB
constexpr int KS = D / 16, DB = D / 32;

typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// chunk position p of row `row` holds logical chunk p ^ swz(row)
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

struct LaneOffsets {
    int k[KS];          // K operand read: row n, logical chunk 2 st + hlf (add 32 kb rows)
    int v1[DB];         // V transpose read of column block b, rows +0..3 (add (32 kb + 16 t) rows); the read
                        // of rows +8..11 is at (v1 ^ 32) + 8 rows: its swizzle differs in one bit
    int g[4];           // global byte offsets of this lane's four copy instructions
};

// S^T = K . Q^T for one tile of 64 keys: s[kb] holds keys 32kb..32kb+31.
__device__ __forceinline__ void qk_tile(floatx16 (&s)[2], const bf16x8 (&qf)[KS],
                                        const unsigned char* ks, const LaneOffsets& lo) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[kb][e] = 0.f;
#pragma unroll
    for (int st = 0; st < KS; ++st)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks + lo.k[st] + kb * 32 * ROWB);
            s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[kb], 0, 0, 0);
        }
}

__device__ __forceinline__ bf16x8 v_operand(const unsigned char* vs, const LaneOffsets& lo, int kb, int t, int b) {
    const unsigned char* p = vs + (32 * kb + 16 * t) * ROWB;
    const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p + lo.v1[b]));
    const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p + 8 * ROWB + (lo.v1[b] ^ 32)));
    return __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
}

// O^T += V^T . P^T; MFMA (kb, t) contracts keys 32kb + 16t + {4hlf..+3} and {8+4hlf..+3}.
__device__ __forceinline__ void pv_tile(floatx16 (&o)[DB], const bf16x8 (&pf)[2][2],
                                        const unsigned char* vs, const LaneOffsets& lo) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int b = 0; b < DB; ++b)
                o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(vs, lo, kb, t, b), pf[kb][t], o[b], 0, 0, 0);
}

// -inf for the keys of a tile that a query row may not see (outside [lo, hi_t)).
__device__ __forceinline__ void mask_tile(floatx16 (&s)[2], int lo, int hi_t, int k_start, int hlf) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int key = k_start + 32 * kb + 8 * (e >> 2) + 4 * hlf + (e & 3);
            if (key < lo || key >= hi_t) s[kb][e] = -INFINITY;
            // ties the masked value to this place, so that the selects stay behind the caller's branch
            asm volatile("" : "+v"(s[kb][e]));
        }
}

// Online softmax of one score tile with lazy rescaling (see prefill.hip for the argument).
template <bool MASK>
__device__ __forceinline__ float softmax_tile(floatx16 (&s)[2], bf16x8 (&pf)[2][2], float& m, float& l,
                                              float sl2, float lazy, int lo, int hi_t, int k_start,
                                              int hlf, bool* rescale) {
    if (MASK) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = k_start + 32 * kb + 8 * (e >> 2) + 4 * hlf + (e & 3);
                if (key < lo || key >= hi_t) s[kb][e] = -INFINITY;
            }
    }
    float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(fmaxf(mx, s[0][e]), s[1][e]);
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    const bool raise = __builtin_amdgcn_ballot_w64(mx > m + lazy || m == -INFINITY) != 0;
    *rescale = raise;
    const float m_new = raise ? fmaxf(m, mx) : m;
    const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f((m - m_ref) * sl2);   // m = -inf -> 0; unchanged m -> 1
    m = m_new;
    const float msl = m_ref * sl2;
    float l0 = l * alpha, l1 = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            uint32_t w[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                floatx2 pp;
                pp[0] = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * t + 2 * x], sl2, -msl));
                pp[1] = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * t + 2 * x + 1], sl2, -msl));
                const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
                if (x & 1) l1 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l1, false);
                else l0 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l0, false);
                w[x] = __builtin_bit_cast(uint32_t, pb);
            }
            pf[kb][t] = __builtin_bit_cast(bf16x8, u32x4{w[0], w[1], w[2], w[3]});
        }
    l = l0 + l1;
    return alpha;
}

// One steady-state iteration, hand-interleaved: each of the 16 score MFMAs of tile j+1 and of
// the 16 PV MFMAs of tile j-1 is followed by a slice of the softmax of tile j (row maximum,
// decision, then one exp/convert/sum slice per MFMA); LDS operand reads run PF MFMAs ahead.
__device__ __forceinline__ float steady_step(floatx16 (&s_next)[2], floatx16 (&s_cur)[2], floatx16 (&o)[DB],
                                             bf16x8 (&p)[2][2], const bf16x8 (&qf)[KS],
                                             const unsigned char* ks, const unsigned char* vs,
                                             const LaneOffsets& lo, float& m, float& l, float sl2,
                                             float lazy, bool* rescale) {
    constexpr int PF = 8;
    auto kread = [&](int i) -> bf16x8 {            // MFMA i of the score phase: st = i / 2, kb = i % 2
        return *reinterpret_cast<const bf16x8*>(ks + lo.k[i >> 1] + (i & 1) * 32 * ROWB);
    };
    auto vread = [&](int i) -> bf16x8 {            // MFMA i of the PV phase: (kb, t) = (i/8, (i/4)%2), b = i % 4
        return v_operand(vs, lo, i >> 3, (i >> 2) & 1, i & 3);
    };
    float mx0 = -INFINITY, mx1 = -INFINITY, alpha = 1.f, msl = 0.f, l0 = 0.f, l1 = 0.f;
    uint32_t pw[16];
    auto slice = [&](int c) {
        if (c < 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                mx0 = fmaxf(mx0, s_cur[0][4 * c + e]);
                mx1 = fmaxf(mx1, s_cur[1][4 * c + e]);
            }
        } else if (c == 4) {
            float mx = fmaxf(mx0, mx1);
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
            mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            const bool raise = __builtin_amdgcn_ballot_w64(mx > m + lazy || m == -INFINITY) != 0;
            *rescale = raise;
            const float m_new = raise ? fmaxf(m, mx) : m;
            const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
            alpha = __builtin_amdgcn_exp2f((m - m_ref) * sl2);
            m = m_new;
            msl = m_ref * sl2;
            l0 = l * alpha;
        } else if (c < 21) {
            const int x = c - 5, kb = x >> 3, e = 2 * (x & 7);
            floatx2 pp;
            pp[0] = __builtin_amdgcn_exp2f(fmaf(s_cur[kb][e], sl2, -msl));
            pp[1] = __builtin_amdgcn_exp2f(fmaf(s_cur[kb][e + 1], sl2, -msl));
            const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
            if (x & 1) l1 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l1, false);
            else l0 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l0, false);
            pw[x] = __builtin_bit_cast(uint32_t, pb);
        }
    };

    // PV of tile j-1 first: its P operands die as the new probabilities are produced
    bf16x8 vf[PF + 1];
#pragma unroll
    for (int i = 0; i < PF; ++i) vf[i] = vread(i);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (i + PF < 16) vf[(i + PF) % (PF + 1)] = vread(i + PF);
        o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % (PF + 1)], p[i >> 3][(i >> 2) & 1], o[i & 3], 0, 0, 0);
        slice(i);
    }
    const floatx16 zero = {};
    bf16x8 kf[PF + 1];
#pragma unroll
    for (int i = 0; i < PF; ++i) kf[i] = kread(i);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (i + PF < 16) kf[(i + PF) % (PF + 1)] = kread(i + PF);
        s_next[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % (PF + 1)], qf[i >> 1], i < 2 ? zero : s_next[i & 1], 0, 0, 0);
        slice(16 + i);
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
            p[kb][t] = __builtin_bit_cast(bf16x8, u32x4{pw[8 * kb + 4 * t], pw[8 * kb + 4 * t + 1],
                                                       pw[8 * kb + 4 * t + 2], pw[8 * kb + 4 * t + 3]});
    l = l0 + l1;
    return alpha;
}

// What a workgroup works on, and this lane's share of it.
struct WorkUnit {
    int head, kvh, n_kv, wave, lane, n, hlf;
    int qrow, lo, hi;                  // this lane's query row (-1: padding) and its key range [lo, hi)
    const int32_t* kvt;                // key-tile list of the query tile: (first key row, info) pairs
    int64_t row_bytes;                 // bytes between consecutive K/V rows in global memory
};

// Decodes the workgroup id, loads the row metadata and the Q operand, derives the lane offsets.
// Returns false for grid padding and for query tiles without key tiles.
__device__ __forceinline__ bool setup(const PrefillArgs& a, WorkUnit& u, LaneOffsets& off, bf16x8 (&qf)[KS]) {
    const int r = a.Hq / a.Hkv;
    int tile;
    if (a.xcd_swizzle) {               // see prefill.hip: the r heads of a KV head stay on one XCD
        const int x = blockIdx.x, c = x & 7, y = x >> 3, j = y % r, slot = y / r;
        const int64_t p = static_cast<int64_t>(slot) * 8 + c;
        if (p >= static_cast<int64_t>(a.n_tiles) * a.Hkv) return false;
        tile = static_cast<int>(p / a.Hkv); u.kvh = static_cast<int>(p % a.Hkv); u.head = u.kvh * r + j;
    } else {
        tile = blockIdx.x / a.Hq; u.head = blockIdx.x % a.Hq; u.kvh = u.head / r;
    }
    const int32_t* desc = a.tiles + 4 * static_cast<int64_t>(tile);
    u.n_kv = desc[1];
    if (u.n_kv == 0) return false;
    u.kvt = a.kvtiles + 2 * static_cast<int64_t>(desc[0]);
    const int tid = threadIdx.x;
    u.lane = tid & 63; u.n = u.lane & 31; u.hlf = u.lane >> 5;
    u.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rr = tile * BM + u.wave * 32 + u.n;
    u.qrow = a.row_q[rr]; u.lo = a.row_lo[rr]; u.hi = a.row_hi[rr];
    u.row_bytes = static_cast<int64_t>(a.Hkv) * ROWB;

    const int fl = swz(u.n);
#pragma unroll
    for (int st = 0; st < KS; ++st) off.k[st] = u.n * ROWB + (((2 * st + u.hlf) ^ fl) << 4);
    const int i16 = u.lane & 15, gl = (u.lane >> 4) & 1, r4 = i16 >> 2;
    const int f1 = (r4 << 2) | u.hlf;  // rows +8: (hlf + 2) & 3 = hlf ^ 2, i.e. chunk ^ 2, byte offset ^ 32
    const int rowl = 4 * u.hlf + r4, byte = (i16 & 1) * 8;
#pragma unroll
    for (int b = 0; b < DB; ++b) {
        const int c = 4 * b + 2 * gl + ((i16 & 3) >> 1);
        off.v1[b] = rowl * ROWB + ((c ^ f1) << 4) + byte;
    }
    const int r_in = u.lane >> 4, pos = u.lane & 15;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = 16 * u.wave + 4 * q + r_in;
        off.g[q] = static_cast<int>(row * u.row_bytes + u.kvh * ROWB + ((pos ^ swz(row)) << 4));
    }
    // Q operand: lane (n, hlf) holds Q[row n][16s + 8hlf .. +8]
    const uint16_t* qp = static_cast<const uint16_t*>(a.q) +
                         (static_cast<int64_t>(u.qrow < 0 ? 0 : u.qrow) * a.Hq + u.head) * D + 8 * u.hlf;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (u.qrow >= 0) raw = *reinterpret_cast<const u32x4*>(qp + 16 * s);
        qf[s] = __builtin_bit_cast(bf16x8, raw);
    }
    return true;
}

// o / l to global memory; lane (n, hlf) owns columns 32b + 8q + 4hlf .. +3 of its query row.
__device__ __forceinline__ void store_output(const PrefillArgs& a, const WorkUnit& u, const floatx16 (&o)[DB], float l) {
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l), __float_as_uint(l), false, false);
        l = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    if (u.qrow < 0) return;
    const float inv = l > 0.f ? 1.f / l : 0.f;
    const int64_t obase = (static_cast<int64_t>(u.qrow) * a.Hq + u.head) * D;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int col = 32 * b + 8 * q4 + 4 * u.hlf;
            const float x0 = o[b][4 * q4] * inv, x1 = o[b][4 * q4 + 1] * inv;
            const float x2 = o[b][4 * q4 + 2] * inv, x3 = o[b][4 * q4 + 3] * inv;
            if (a.out_f32) {
                *reinterpret_cast<float4*>(static_cast<float*>(a.out) + obase + col) = make_float4(x0, x1, x2, x3);
            } else {
                *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + obase + col) =
                    make_uint2(pack_bf16x2(x0, x1), pack_bf16x2(x2, x3));
            }
        }
}

// copies the tile that starts at key row KSTART of `src` (a.k or a.v) into the LDS stage DST:
// four 1-KiB wave instructions per wave, each lane fetching the chunk that belongs at its
// (swizzled) LDS position; rows past the end of the array arrive as zeros
#define PK_COPY_TILE(SRC, KSTART, DST)                                                       \
    {                                                                                        \
        const int64_t ks_ = (KSTART);                                                        \
        const int64_t left_ = (a.total_kv_rows - ks_) * u.row_bytes;                         \
        const __amdgpu_buffer_rsrc_t rs_ = __builtin_amdgcn_make_buffer_rsrc(                \
            const_cast<char*>(static_cast<const char*>(SRC)) + ks_ * u.row_bytes, 0,         \
            static_cast<int>(left_ > 0x7FFFFFFFll ? 0x7FFFFFFFll : left_), 0x00020000);      \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                        \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(                                        \
                rs_, (lds_void_ptr)((DST) + u.wave * 4096 + q * 1024), 16, off.g[q], 0, 0, 0); \
    }
#define PK_WAIT_ALL_COPIES() __builtin_amdgcn_s_waitcnt(0x0F70)      /* vmcnt(0) */
#define PK_CODE(INFO) (((INFO) >> (8 + 2 * u.wave)) & 3)          /* 0 skip, 1 masked, 2 unmasked */

// ---------------------------------------------------------------------------------------------
// Kernel A (default): two workgroups per CU (80 KiB of LDS each): three stages for K, two for V.
// Iteration j requests K(j+2) and V(j+1) first, then runs QK(j) and the softmax, waits for the
// copies of the PREVIOUS iteration (so every copy has one and a half to two iterations to land),
// meets the other waves (barrier A: V(j) is complete), runs PV(j), and meets them again (barrier
// B: the stages that the next iteration overwrites are no longer read).
__global__ __launch_bounds__(256, 2) void prefill_bf16_dma_kernel(PrefillArgs a) {
    __shared__ __align__(1024) unsigned char lds[5 * TILE_BYTES];   // K stages 0..2, V stages 3..4
    WorkUnit u;
    LaneOffsets off;
    bf16x8 qf[KS];
    if (!setup(a, u, off, qf)) return;
    const int n_kv = u.n_kv;
    const __attribute__((address_space(4))) int32_t* kvt_c =
        (const __attribute__((address_space(4))) int32_t*)(u.kvt);
    auto entry = [&](int j, int& ks, int& info) {   // scalar loads; indices past the end are clamped
        const int jj = j < n_kv ? j : n_kv - 1;
        ks = kvt_c[2 * jj]; info = kvt_c[2 * jj + 1];
    };

    floatx16 o[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[b][e] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float sl2 = a.scale * kLog2e;
    const float lazy = 8.0f / sl2;

    // window of tile-list entries: e0 = tile j, e1 = tile j+1, e2 = tile j+2 (e3 is fetched for the next turn)
    int e0s, e0i, e1s, e1i, e2s, e2i;
    entry(0, e0s, e0i); entry(1, e1s, e1i); entry(2, e2s, e2i);
    // prologue: K(0), K(1), V(0) (copies of tiles past the end are clamped duplicates into free stages)
    PK_COPY_TILE(a.k, e0s, lds);
    PK_COPY_TILE(a.k, e1s, lds + TILE_BYTES);
    PK_COPY_TILE(a.v, e0s, lds + 3 * TILE_BYTES);
    PK_WAIT_ALL_COPIES();
    __syncthreads();

    int k_cur = 0, k_fill = 2 * TILE_BYTES;         // byte offsets of the K stage read now / filled now
    int v_cur = 3 * TILE_BYTES, v_fill = 4 * TILE_BYTES;
    for (int j = 0; j < n_kv; ++j) {
        PK_COPY_TILE(a.k, e2s, lds + k_fill);
        PK_COPY_TILE(a.v, e1s, lds + v_fill);
        int e3s, e3i;
        entry(j + 3, e3s, e3i);
        const int code = PK_CODE(e0i);
        const int k_start = e0s;
        const int hi_t = min(u.hi, k_start + (e0i & 0xFF));   // keys past the tile's valid count are foreign
        floatx16 s[2];
        bf16x8 p[2][2];
        float alpha = 1.f;
        bool rescale = false;
        if (code != 0) {
            qk_tile(s, qf, lds + k_cur, off);
            if (code == 1) {                          // diagonal or ragged tile: mask in place (unmasked tiles skip it)
                mask_tile(s, u.lo, hi_t, k_start, u.hlf);
            }
            alpha = softmax_tile<false>(s, p, m, l, sl2, lazy, u.lo, hi_t, k_start, u.hlf, &rescale);
        }
        // Barrier A is taken with this iteration's eight copies still in flight (the compiler's
        // own barrier would wait for all of them): everything requested earlier has landed.
        asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
        if (code != 0) {
            if (rescale) {                            // rare: the stored maximum was raised
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[b][e] *= alpha;
            }
            pv_tile(o, p, lds + v_cur, off);
        }
        e0s = e1s; e0i = e1i; e1s = e2s; e1i = e2i; e2s = e3s; e2i = e3i;
        k_cur = k_cur == 2 * TILE_BYTES ? 0 : k_cur + TILE_BYTES;
        k_fill = k_fill == 2 * TILE_BYTES ? 0 : k_fill + TILE_BYTES;
        const int tmp = v_cur; v_cur = v_fill; v_fill = tmp;
        // barrier B: the stages overwritten by the next iteration's copies are no longer read
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
    PK_WAIT_ALL_COPIES();                          // nothing may still be writing LDS when the block ends
    store_output(a, u, o, l);
}

// ---------------------------------------------------------------------------------------------
// Kernel B (experimental, PK_PREFILL_PIPE=1): one workgroup per CU, four LDS stages per operand,
// software-pipelined tile loop (see the head of this file).
__global__ __launch_bounds__(256, 1) void prefill_bf16_pipe_kernel(PrefillArgs a) {
    // four stages each for K and V (128 KiB: one workgroup per CU); separate arrays so that the
    // copy into one stage is known not to alias the reads of another
    __shared__ __align__(1024) unsigned char k_lds0[TILE_BYTES];
    __shared__ __align__(1024) unsigned char k_lds1[TILE_BYTES];
    __shared__ __align__(1024) unsigned char k_lds2[TILE_BYTES];
    __shared__ __align__(1024) unsigned char k_lds3[TILE_BYTES];
    __shared__ __align__(1024) unsigned char v_lds0[TILE_BYTES];
    __shared__ __align__(1024) unsigned char v_lds1[TILE_BYTES];
    __shared__ __align__(1024) unsigned char v_lds2[TILE_BYTES];
    __shared__ __align__(1024) unsigned char v_lds3[TILE_BYTES];

    WorkUnit u;
    LaneOffsets off;
    bf16x8 qf[KS];
    if (!setup(a, u, off, qf)) return;
    const int n_kv = u.n_kv, hlf = u.hlf, lo = u.lo, hi = u.hi;
    const int32_t* kvt = u.kvt;

    floatx16 o[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[b][e] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float sl2 = a.scale * kLog2e;
    const float lazy = 8.0f / sl2;

    // Entries (first key row, info) of the tile list are needed as scalars (copy descriptors,
    // wave codes).  They are read through the constant address space (scalar loads, which do not
    // share a counter with the tile copies) one iteration ahead of their use, and kept in a window:
    // es[x], ei[x] describe tile j + x.
    const __attribute__((address_space(4))) int32_t* kvt_c =
        (const __attribute__((address_space(4))) int32_t*)(kvt);
    auto entry = [&](int j, int& ks, int& info) {
        const int jj = j < n_kv ? j : n_kv - 1;
        ks = kvt_c[2 * jj]; info = kvt_c[2 * jj + 1];
    };
    int es[6], ei[6];
#pragma unroll
    for (int x = 0; x < 6; ++x) entry(x, es[x], ei[x]);

    // ---- prologue: K(0..3), V(0), V(1) into LDS, scores of tile 0 -------------
    // (tile indices past the end are clamped: such copies land in stages nobody reads)
    PK_COPY_TILE(a.k, es[0], k_lds0);
    PK_COPY_TILE(a.k, es[1], k_lds1);
    PK_COPY_TILE(a.k, es[2], k_lds2);
    PK_COPY_TILE(a.k, es[3], k_lds3);
    PK_COPY_TILE(a.v, es[0], v_lds0);
    PK_COPY_TILE(a.v, es[1], v_lds1);
    PK_WAIT_ALL_COPIES();
    __syncthreads();
    floatx16 s_a[2], s_b[2];
    bf16x8 p_prev[2][2];
    int c_prev = 0, c_cur = PK_CODE(ei[0]);
    if (c_cur) qk_tile(s_a, qf, k_lds0, off);
    __syncthreads();                               // stage 0 of K is free again

    // Iteration j: s_c holds the scores of tile j, s_n receives those of tile j+1.
    // In LDS: K(j+1) in k_next, V(j-1) in v_prev.  Copied now: K(j+4) -> k_free (held K(j)),
    // V(j+2) -> v_free (held V(j-2)).  At the end K(j+2) and V(j) must have landed: they were
    // requested two iterations ago, so the 16 copy instructions of this and of the previous
    // iteration may remain in flight.
    auto iteration = [&](int j, floatx16 (&s_c)[2], floatx16 (&s_n)[2], unsigned char* k_next,
                         unsigned char* k_free, unsigned char* v_prev, unsigned char* v_free) {
        PK_COPY_TILE(a.k, es[4], k_free);
        PK_COPY_TILE(a.v, es[2], v_free);
        int ns, ni;
        entry(j + 6, ns, ni);
        const int c_next = (j + 1 < n_kv) ? PK_CODE(ei[1]) : 0;
        const int k_start = es[0];
        const int hi_t = min(hi, k_start + (ei[0] & 0xFF));   // keys past the tile's valid count are foreign
        bool rescale = false;
        float alpha = 1.f;
        if (c_next != 0 && c_prev != 0 && c_cur == 2) {
            alpha = steady_step(s_n, s_c, o, p_prev, qf, k_next, v_prev, off, m, l, sl2, lazy, &rescale);
        } else {
            if (c_next != 0) qk_tile(s_n, qf, k_next, off);
            if (c_prev != 0) pv_tile(o, p_prev, v_prev, off);
            if (c_cur == 2) alpha = softmax_tile<false>(s_c, p_prev, m, l, sl2, lazy, lo, hi_t, k_start, hlf, &rescale);
            else if (c_cur == 1) alpha = softmax_tile<true>(s_c, p_prev, m, l, sl2, lazy, lo, hi_t, k_start, hlf, &rescale);
        }
        if (rescale) {                              // rare after the first tiles (wave-uniform)
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[b][e] *= alpha;
        }
        c_prev = c_cur;                             // p_prev now holds the probabilities of tile j
        c_cur = c_next;
#pragma unroll
        for (int x = 0; x < 5; ++x) { es[x] = es[x + 1]; ei[x] = ei[x + 1]; }
        es[5] = ns; ei[5] = ni;
        // Barrier with copies still in flight: the compiler's own barrier would first wait for
        // every outstanding memory operation, so the wait and the barrier are spelled out.  All
        // copies are bounds-checked buffer loads; this wave's LDS reads of the stages that are
        // overwritten next were consumed by MFMAs above.
        asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");
    };
    for (int j = 0; j < n_kv; j += 4) {
        iteration(j, s_a, s_b, k_lds1, k_lds0, v_lds3, v_lds2);
        if (j + 1 < n_kv) iteration(j + 1, s_b, s_a, k_lds2, k_lds1, v_lds0, v_lds3);
        if (j + 2 < n_kv) iteration(j + 2, s_a, s_b, k_lds3, k_lds2, v_lds1, v_lds0);
        if (j + 3 < n_kv) iteration(j + 3, s_b, s_a, k_lds0, k_lds3, v_lds2, v_lds1);
    }
    PK_WAIT_ALL_COPIES();                          // nothing may still be writing LDS when the block ends
    // drain: PV of the last tile
    if (c_prev != 0) {
        const int last = (n_kv - 1) & 3;
        pv_tile(o, p_prev, last == 0 ? v_lds0 : last == 1 ? v_lds1 : last == 2 ? v_lds2 : v_lds3, off);
    }
    store_output(a, u, o, l);
}

#undef PK_COPY_TILE
#undef PK_WAIT_ALL_COPIES
#undef PK_CODE

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
    static const bool pipelined = [] { const char* e = getenv("PK_PREFILL_PIPE"); return e && e[0] == '1'; }();
    if (pipelined)
        hipLaunchKernelGGL(prefill_bf16_pipe_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), a);
    else
        hipLaunchKernelGGL(prefill_bf16_dma_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace pk
