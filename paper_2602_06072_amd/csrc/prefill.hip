// Packed prefill attention, bf16 MFMA (Sec. 3.1): causal attention over the
// packed query-key regions of each group with a per-request block-diagonal
// mask and online softmax.  The same kernel runs the padded per-request
// schedule of the in-run comparison; only the tables differ.
//
// Workgroup = (query tile of 128 packed rows, query head), 4 waves x 32 rows.
// Per key tile of 64 keys a wave computes
//     S^T (keys x queries) = K . Q^T      A = K rows from LDS, B = Q in registers
//     O^T (d x queries)   += V^T . P^T    A = V^T by LDS transpose reads, B = P
// with v_mfma_f32_32x32x16_bf16.  Working on the transposed problem keeps each
// query's scores inside one lane (plus its partner lane^32), so the softmax
// row reductions are in-register, and P^T leaves the first MFMA already in the
// operand layout of the second.
//
// The loop is software-pipelined over key tiles: in iteration j a wave issues
// the score MFMAs of tile j+1, the PV MFMAs of tile j-1 and the softmax of
// tile j.  The three are independent, so the matrix pipe works while the
// vector ALU does the exponentials.  K tiles are therefore staged two tiles
// ahead and V tiles zero tiles ahead of the softmax (both double buffered in
// LDS, one barrier per tile).  MFMA-bound: 4*D flops per (query, key) pair.
#include "common.hip.h"
#include "kernels.h"

namespace pk {
namespace {

constexpr int BM = 128, BN = 64;

template <int D> struct Smem {
    static constexpr int KP = D * 2 + 16;          // K row pitch (bytes): conflict-free 16-byte row reads
    static constexpr int VP = D * 2 + 64;          // V row pitch (bytes): transpose reads of 8 rows hit 8 x 16 banks
    static constexpr int K_BYTES = BN * KP;
    static constexpr int V_BYTES = BN * VP;
    static constexpr int TOTAL = 2 * K_BYTES + 2 * V_BYTES;
};

typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;

// S^T = K . Q^T for one tile of 64 keys: s[kb] holds keys 32kb..32kb+31.
// Lane (n, hlf), register e: key 32kb + 8(e/4) + 4hlf + e%4, query row n.
template <int D>
__device__ __forceinline__ void qk_tile(floatx16 (&s)[2], const bf16x8 (&qf)[D / 16],
                                        const unsigned char* ks, int n, int hlf) {
    using SM = Smem<D>;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[kb][e] = 0.f;
#pragma unroll
    for (int st = 0; st < D / 16; ++st)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks + (32 * kb + n) * SM::KP + 16 * hlf + 32 * st);
            s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[kb], 0, 0, 0);
        }
}

// O^T += V^T . P^T.  MFMA (kb, t) contracts keys 32kb + 16t + {4hlf..4hlf+3} and
// {8+4hlf..8+4hlf+3}; the transpose read hands lane i of a 16-lane group column i of a
// 4-row x 16-column patch of V.
template <int D>
__device__ __forceinline__ void pv_tile(floatx16 (&o)[D / 32], const bf16x8 (&pf)[2][2],
                                        const unsigned char* vs, int lane) {
    using SM = Smem<D>;
    const int i16 = lane & 15, gl = (lane >> 4) & 1, hlf = lane >> 5;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int key0 = 32 * kb + 16 * t + 4 * hlf + (i16 >> 2);
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
                const int col = 32 * b + 16 * gl + 4 * (i16 & 3);
                const unsigned char* p0 = vs + key0 * SM::VP + col * 2;
                const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
                const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0 + 8 * SM::VP));
                const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][t], o[b], 0, 0, 0);
            }
        }
}

// Online softmax of one score tile.  m is the stored row maximum of the RAW scores; it is only
// raised when some row's maximum grew by more than `lazy` (= 8 / sl2), so until then
// p = exp2((s - m) sl2) <= 2^8, harmless in fp32/bf16, and o / l is unchanged because both use the
// same m.  Returns the factor by which the caller must scale the output accumulators (1 unless
// the maximum was raised; *rescale is the wave-uniform "was raised" flag).
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
                // the row sum uses the rounded probabilities, like the PV product does
                if (x & 1) l1 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l1, false);
                else l0 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l0, false);
                w[x] = __builtin_bit_cast(uint32_t, pb);
            }
            pf[kb][t] = __builtin_bit_cast(bf16x8, u32x4{w[0], w[1], w[2], w[3]});
        }
    l = l0 + l1;
    return alpha;
}

// One steady-state iteration, hand-interleaved: the 16 score MFMAs of tile j+1 and the 16 PV
// MFMAs of tile j-1 are each followed by a slice of the softmax of tile j (row maximum first,
// then one exp/convert/sum slice per MFMA), with the LDS operand reads running three MFMAs
// ahead.  Same arithmetic as qk_tile + pv_tile + softmax_tile<false>.
template <int D>
__device__ __forceinline__ float steady_step(floatx16 (&s_next)[2], floatx16 (&s_cur)[2], floatx16 (&o)[D / 32],
                                             bf16x8 (&p)[2][2], const bf16x8 (&qf)[D / 16],
                                             const unsigned char* ks, const unsigned char* vs,
                                             float& m, float& l, float sl2, float lazy, int lane, bool* rescale) {
    using SM = Smem<D>;
    static_assert(D == 128, "the slice plan below is written for 16 + 16 MFMAs");
    constexpr int PF = 3;                          // operand reads run this many MFMAs ahead
    const int n = lane & 31, hlf = lane >> 5, i16 = lane & 15, gl = (lane >> 4) & 1;
    const unsigned char* kbase = ks + n * SM::KP + 16 * hlf;
    const unsigned char* vbase = vs + (4 * hlf + (i16 >> 2)) * SM::VP + (16 * gl + 4 * (i16 & 3)) * 2;
    // MFMA i of the score phase: k-step st = i / 2, key block kb = i % 2
    auto kread = [&](int i) -> bf16x8 {
        return *reinterpret_cast<const bf16x8*>(kbase + (32 * (i & 1)) * SM::KP + 32 * (i >> 1));
    };
    // MFMA i of the PV phase: (kb, t) = (i / 8, (i / 4) % 2), column block b = i % 4
    auto vread = [&](int i) -> bf16x8 {
        const unsigned char* p0 = vbase + (32 * (i >> 3) + 16 * ((i >> 2) & 1)) * SM::VP + (32 * (i & 3)) * 2;
        const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
        const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0 + 8 * SM::VP));
        return __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    bf16x8 p_old[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int t = 0; t < 2; ++t) p_old[kb][t] = p[kb][t];

    float mx0 = -INFINITY, mx1 = -INFINITY, alpha = 1.f, msl = 0.f, l0 = 0.f, l1 = 0.f;
    uint32_t pw[16];
    // softmax slices: 0..3 row maximum (8 scores each), 4 decision, 5..20 one bf16 pair each
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

#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s_next[kb][e] = 0.f;
    bf16x8 kf[PF + 1];
#pragma unroll
    for (int i = 0; i < PF; ++i) kf[i] = kread(i);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (i + PF < 16) kf[(i + PF) % (PF + 1)] = kread(i + PF);
        s_next[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % (PF + 1)], qf[i >> 1], s_next[i & 1], 0, 0, 0);
        slice(i);
    }
    bf16x8 vf[PF + 1];
#pragma unroll
    for (int i = 0; i < PF; ++i) vf[i] = vread(i);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (i + PF < 16) vf[(i + PF) % (PF + 1)] = vread(i + PF);
        o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % (PF + 1)], p_old[i >> 3][(i >> 2) & 1], o[i & 3], 0, 0, 0);
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

template <int D>
__global__ __launch_bounds__(256, 1) void prefill_bf16_kernel(PrefillArgs a) {
    using SM = Smem<D>;
    constexpr int KS = D / 16;                     // MFMA k-steps over the head dimension
    constexpr int DB = D / 32;                     // 32-column blocks of the output
    constexpr int CH = D / 8;                      // 16-byte chunks per row
    constexpr int LD = BN * CH / 256;              // chunks per thread per tile (K and V each)
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* const kbuf = smem;                        // 2 x K_BYTES
    unsigned char* const vbuf = smem + 2 * SM::K_BYTES;      // 2 x V_BYTES

    // ---- work unit ---------------------------------------------------------
    const int r = a.Hq / a.Hkv;
    int tile, head, kvh;
    if (a.xcd_swizzle) {
        // consecutive workgroup ids go round-robin over the 8 XCDs: keep the r heads of one
        // (tile, KV head) pair on one XCD and adjacent in time so K/V tiles hit in its L2
        const int x = blockIdx.x, c = x & 7, y = x >> 3, j = y % r, slot = y / r;
        const int64_t p = static_cast<int64_t>(slot) * 8 + c;
        if (p >= static_cast<int64_t>(a.n_tiles) * a.Hkv) return;
        tile = static_cast<int>(p / a.Hkv); kvh = static_cast<int>(p % a.Hkv); head = kvh * r + j;
    } else {
        tile = blockIdx.x / a.Hq; head = blockIdx.x % a.Hq; kvh = head / r;
    }
    const int32_t* desc = a.tiles + 4 * static_cast<int64_t>(tile);
    const int kv_first = desc[0], n_kv = desc[1];
    if (n_kv == 0) return;
    const int32_t* kvt = a.kvtiles + 2 * static_cast<int64_t>(kv_first);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, hlf = lane >> 5;
    const int rr = tile * BM + wave * 32 + n;
    const int qrow = a.row_q[rr], lo = a.row_lo[rr], hi = a.row_hi[rr];

    // ---- Q operand: lane (n, hlf) holds Q[row n][16s + 8hlf .. +8] ----------
    bf16x8 qf[KS];
    {
        const uint16_t* qp = static_cast<const uint16_t*>(a.q) +
                             (static_cast<int64_t>(qrow < 0 ? 0 : qrow) * a.Hq + head) * D + 8 * hlf;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (qrow >= 0) raw = *reinterpret_cast<const u32x4*>(qp + 16 * s);
            qf[s] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    floatx16 o[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[b][e] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float sl2 = a.scale * kLog2e;
    const float lazy = 8.0f / sl2;

    // ---- tile loader (global -> registers -> LDS) ----------------------------
    // Buffer loads: the tile's first row goes into the (scalar) resource base, each thread keeps
    // constant byte offsets, and rows past the end of the array read as zero in hardware.
    const int ld_row = tid / CH, ld_c = tid % CH;  // this thread's first chunk; the next ones 256/CH rows on
    const int64_t row_bytes = static_cast<int64_t>(a.Hkv) * D * 2;
    int ld_off[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i)
        ld_off[i] = static_cast<int>((ld_row + i * (256 / CH)) * row_bytes + kvh * D * 2 + ld_c * 16);
    u32x4 kreg[2][LD], vreg[2][LD];                // two register sets: loads run two tiles ahead
#define PK_GLOAD(REG, SRC, J)                                                                \
    {                                                                                        \
        const int64_t ks_ = kvt[2 * (J)];                                                    \
        const int64_t left_ = (a.total_kv_rows - ks_) * row_bytes;                           \
        const __amdgpu_buffer_rsrc_t rs_ = __builtin_amdgcn_make_buffer_rsrc(                \
            const_cast<char*>(static_cast<const char*>(SRC)) + ks_ * row_bytes, 0,           \
            static_cast<int>(left_ > 0x7FFFFFFFll ? 0x7FFFFFFFll : left_), 0x00020000);      \
        _Pragma("unroll") for (int i = 0; i < LD; ++i)                                       \
            REG[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_, ld_off[i], 0, 0);            \
    }
#define PK_SSTORE(REG, BASE, PITCH)                                                          \
    {                                                                                        \
        _Pragma("unroll") for (int i = 0; i < LD; ++i) {                                     \
            const int row = ld_row + i * (256 / CH);                                         \
            *reinterpret_cast<u32x4*>((BASE) + row * (PITCH) + ld_c * 16) = REG[i];          \
        }                                                                                    \
    }
#define PK_CODE(J) ((kvt[2 * (J) + 1] >> (8 + 2 * wave)) & 3)   /* 0 skip, 1 masked, 2 unmasked */

    // ---- prologue: K(0), K(1) into LDS, scores of tile 0, loads of K(2), V(0) in flight ----
    PK_GLOAD(kreg[0], a.k, 0);
    if (n_kv > 1) PK_GLOAD(kreg[1], a.k, 1);
    PK_SSTORE(kreg[0], kbuf, SM::KP);
    if (n_kv > 1) PK_SSTORE(kreg[1], kbuf + SM::K_BYTES, SM::KP);
    __syncthreads();
    if (n_kv > 2) PK_GLOAD(kreg[1], a.k, 2);
    PK_GLOAD(vreg[1], a.v, 0);
    floatx16 s_cur[2], s_next[2];
    bf16x8 p_prev[2][2];
    int c_prev = 0, c_cur = PK_CODE(0);
    if (c_cur) qk_tile<D>(s_cur, qf, kbuf, n, hlf);

    // One iteration; s_c holds the scores of tile j, s_n receives those of tile j+1; register
    // set `ld` receives K(j+3) and V(j+1), set `st` (loaded one iteration ago) goes to LDS.  The
    // loop is unrolled by two with the roles swapped, so nothing is copied.
    auto iteration = [&](int j, floatx16 (&s_c)[2], floatx16 (&s_n)[2], u32x4 (&k_ld)[LD], u32x4 (&v_ld)[LD],
                         u32x4 (&k_st)[LD], u32x4 (&v_st)[LD]) {
        // in LDS now: K(j+1) in kbuf[(j+1)&1], V(j-1) in vbuf[(j-1)&1]
        if (j + 3 < n_kv) PK_GLOAD(k_ld, a.k, j + 3);
        if (j + 1 < n_kv) PK_GLOAD(v_ld, a.v, j + 1);
        const int c_next = (j + 1 < n_kv) ? PK_CODE(j + 1) : 0;
        const unsigned char* k_next = kbuf + ((j + 1) & 1) * SM::K_BYTES;
        const unsigned char* v_prev = vbuf + ((j - 1) & 1) * SM::V_BYTES;
        const int k_start = kvt[2 * j];
        const int hi_t = min(hi, k_start + (kvt[2 * j + 1] & 0xFF));   // keys past the tile's valid count are foreign
        bool rescale = false;
        float alpha = 1.f;
        if (c_next != 0 && c_prev != 0 && c_cur == 2) {
            // steady state: three independent streams, interleaved by hand
            if constexpr (D == 128) {
                alpha = steady_step<D>(s_n, s_c, o, p_prev, qf, k_next, v_prev, m, l, sl2, lazy, lane, &rescale);
            } else {
                qk_tile<D>(s_n, qf, k_next, n, hlf);
                pv_tile<D>(o, p_prev, v_prev, lane);
                alpha = softmax_tile<false>(s_c, p_prev, m, l, sl2, lazy, lo, hi_t, k_start, hlf, &rescale);
            }
        } else {
            if (c_next != 0) qk_tile<D>(s_n, qf, k_next, n, hlf);
            if (c_prev != 0) pv_tile<D>(o, p_prev, v_prev, lane);
            if (c_cur == 2) alpha = softmax_tile<false>(s_c, p_prev, m, l, sl2, lazy, lo, hi_t, k_start, hlf, &rescale);
            else if (c_cur == 1) alpha = softmax_tile<true>(s_c, p_prev, m, l, sl2, lazy, lo, hi_t, k_start, hlf, &rescale);
        }
        if (rescale) {                              // rare after the first tiles (wave-uniform)
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[b][e] *= alpha;
        }
        // p_prev now holds the probabilities of tile j (if c_cur != 0)
        c_prev = c_cur;
        c_cur = c_next;
        if (j + 2 < n_kv) PK_SSTORE(k_st, kbuf + (j & 1) * SM::K_BYTES, SM::KP);
        PK_SSTORE(v_st, vbuf + (j & 1) * SM::V_BYTES, SM::VP);
        __syncthreads();
    };
    for (int j = 0; j < n_kv; j += 2) {
        iteration(j, s_cur, s_next, kreg[0], vreg[0], kreg[1], vreg[1]);
        if (j + 1 < n_kv) iteration(j + 1, s_next, s_cur, kreg[1], vreg[1], kreg[0], vreg[0]);
    }
    // drain: PV of the last tile
    if (c_prev != 0) pv_tile<D>(o, p_prev, vbuf + ((n_kv - 1) & 1) * SM::V_BYTES, lane);
#undef PK_GLOAD
#undef PK_SSTORE
#undef PK_CODE

    // ---- epilogue ----------------------------------------------------------
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l), __float_as_uint(l), false, false);
        l = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    if (qrow < 0) return;
    const float inv = l > 0.f ? 1.f / l : 0.f;
    const int64_t obase = (static_cast<int64_t>(qrow) * a.Hq + head) * D;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int col = 32 * b + 8 * q4 + 4 * hlf;
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

template <int D>
int launch_p(const PrefillArgs& a, hipStream_t st) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_bf16_kernel<D>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Smem<D>::TOTAL);
        if (e != hipSuccess) return static_cast<int>(e);
        attr_set = true;
    }
    const int r = a.Hq / a.Hkv;
    int64_t grid;
    if (a.xcd_swizzle) {
        const int64_t pairs = static_cast<int64_t>(a.n_tiles) * a.Hkv;
        grid = (pairs + 7) / 8 * 8 * r;
    } else {
        grid = static_cast<int64_t>(a.n_tiles) * a.Hq;
    }
    if (grid == 0) return 0;
    hipLaunchKernelGGL(prefill_bf16_kernel<D>, dim3(static_cast<unsigned>(grid)), dim3(256), Smem<D>::TOTAL, st, a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace

int launch_prefill_bf16(const PrefillArgs& a, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.d == 128) return launch_p<128>(a, st);
    if (a.d == 64) return launch_p<64>(a, st);
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace pk
