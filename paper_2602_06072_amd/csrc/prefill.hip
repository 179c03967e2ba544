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
// operand layout of the second.  K/V tiles are staged through LDS (double
// buffered, one barrier per tile); global loads of tile j+1 are issued before
// the math of tile j.  MFMA-bound: 4*D flops per (query, key) pair.
// This register-staged kernel is the second pipeline (pk_plan_tune, PK_TUNE_PREFILL_PIPELINE = 1);
// by default both head dimensions run the direct-to-LDS kernels of prefill_pipe.hip (same tables,
// same tile shape, same arithmetic).

#include <mutex>

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
    static constexpr int STAGE = K_BYTES + V_BYTES;
    static constexpr int TOTAL = 2 * STAGE;
};

typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;

template <int D>
__global__ __launch_bounds__(256, 2) void prefill_bf16_kernel(PrefillArgs a) {
    using SM = Smem<D>;
    constexpr int KS = D / 16;                     // MFMA k-steps over the head dimension
    constexpr int DB = D / 32;                     // 32-column blocks of the output
    constexpr int CH = D / 8;                      // 16-byte chunks per row
    constexpr int LD = BN * CH / 256;              // chunks per thread per tile (K and V each)
    extern __shared__ __align__(16) unsigned char smem[];

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
    const int32_t* desc = a.tiles + 16 * static_cast<int64_t>(tile);     // (16 words per descriptor; this kernel uses the first 8)
    const int kv_first = desc[0], n_kv = desc[1];
    if (n_kv == 0) return;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, hlf = lane >> 5;
    int qrow, lo, hi;
    prefill_tile_row(a, tile, desc[4], desc[5], desc[6], desc[7], wave * 32 + n, qrow, lo, hi);

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
    // m: running row maximum of the RAW scores (it may lag behind the true maximum by up to
    // kLazy / sl2, see below); l: this lane's share of sum_j exp2((s_j - m) * sl2)
    float m = -INFINITY, l = 0.f;
    const float sl2 = a.scale * kLog2e;
    const float lazy = 8.0f / sl2;                 // rescale only when the maximum grows by > 2^8

    // ---- tile loader (global -> registers -> LDS) ----------------------------
    // Buffer loads: the tile's first row goes into the (scalar) resource base, each thread keeps
    // constant byte offsets, and rows past the end of the array read as zero in hardware.
    const int ld_row = tid / CH, ld_c = tid % CH;  // this thread's first chunk; the next ones 256/CH rows on
    const int64_t row_bytes = static_cast<int64_t>(a.Hkv) * D * 2;
    int ld_off[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i)
        ld_off[i] = static_cast<int>((ld_row + i * (256 / CH)) * row_bytes + kvh * D * 2 + ld_c * 16);
    u32x4 kreg[LD], vreg[LD];
#define PK_GLOAD(KSTART)                                                                     \
    {                                                                                        \
        const int64_t ks_ = (KSTART);                                                        \
        const int64_t left_ = (a.total_kv_rows - ks_) * row_bytes;                           \
        const int nrec_ = static_cast<int>(left_ > 0x7FFFFFFFll ? 0x7FFFFFFFll : left_);     \
        const __amdgpu_buffer_rsrc_t rk_ = __builtin_amdgcn_make_buffer_rsrc(                \
            const_cast<char*>(static_cast<const char*>(a.k)) + ks_ * row_bytes, 0, nrec_, 0x00020000); \
        const __amdgpu_buffer_rsrc_t rv_ = __builtin_amdgcn_make_buffer_rsrc(                \
            const_cast<char*>(static_cast<const char*>(a.v)) + ks_ * row_bytes, 0, nrec_, 0x00020000); \
        _Pragma("unroll") for (int i = 0; i < LD; ++i) {                                     \
            kreg[i] = __builtin_amdgcn_raw_buffer_load_b128(rk_, ld_off[i], 0, 0);           \
            vreg[i] = __builtin_amdgcn_raw_buffer_load_b128(rv_, ld_off[i], 0, 0);           \
        }                                                                                    \
    }
#define PK_SSTORE(SIDX)                                                                      \
    {                                                                                        \
        unsigned char* ks_ = smem + (SIDX) * SM::STAGE;                                      \
        unsigned char* vs_ = ks_ + SM::K_BYTES;                                              \
        _Pragma("unroll") for (int i = 0; i < LD; ++i) {                                     \
            const int row = ld_row + i * (256 / CH);                                         \
            *reinterpret_cast<u32x4*>(ks_ + row * SM::KP + ld_c * 16) = kreg[i];             \
            *reinterpret_cast<u32x4*>(vs_ + row * SM::VP + ld_c * 16) = vreg[i];             \
        }                                                                                    \
    }

    // Entries (first key row, info) of the tile list are needed as scalars.  Loads issued after a
    // barrier are not scalarised by the compiler and their latency would sit in every iteration,
    // so they run through a window: e0 / e1 hold tiles j, j+1 and the entry of j+2 is in flight.
    const int32_t* kvt = a.kvtiles + 2 * static_cast<int64_t>(kv_first);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto entry_load = [&](int j) -> int2 {
        return *reinterpret_cast<const int2*>(kvt + 2 * (j < n_kv ? j : n_kv - 1));
    };
    int e0s, e0i, e1s, e1i;
    {
        const int2 x0 = entry_load(0), x1 = entry_load(1);
        e0s = __builtin_amdgcn_readfirstlane(x0.x); e0i = __builtin_amdgcn_readfirstlane(x0.y);
        e1s = __builtin_amdgcn_readfirstlane(x1.x); e1i = __builtin_amdgcn_readfirstlane(x1.y);
    }
    PK_GLOAD(e0s);
    PK_SSTORE(0);
    __syncthreads();

    const int i16 = lane & 15, gl = (lane >> 4) & 1;
    for (int j = 0; j < n_kv; ++j) {
        const int stage = j & 1;
        if (j + 1 < n_kv) PK_GLOAD(e1s);
        const int2 e2 = entry_load(j + 2);
        const int32_t k_start = e0s, info = e0i;
        const int code = (info >> (8 + 2 * wave_u)) & 3;     // 0 skip, 1 masked, 2 unmasked
        if (code != 0) {
            const unsigned char* ks = smem + stage * SM::STAGE;
            const unsigned char* vs = ks + SM::K_BYTES;
            // ---- S^T = K . Q^T: two blocks of 32 keys -----------------------
            // All operand reads of a phase are issued before its first MFMA (sched_barrier keeps the
            // scheduler from sinking them back next to their uses): the LDS latency is paid once
            // per phase instead of once per MFMA.
            floatx16 s[2];
            {
                bf16x8 kf[2][KS];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int st = 0; st < KS; ++st)
                        kf[kb][st] = *reinterpret_cast<const bf16x8*>(ks + (32 * kb + n) * SM::KP + 16 * hlf + 32 * st);
                __builtin_amdgcn_sched_barrier(0);
                const floatx16 zero = {};
#pragma unroll
                for (int st = 0; st < KS; ++st)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
                        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][st], qf[st], st == 0 ? zero : s[kb], 0, 0, 0);
            }
            // lane (n, hlf), register e of block kb: key k_start + 32kb + 8(e/4) + 4hlf + e%4
            if (code == 1) {
                // keys past the tile's valid count belong to whatever follows in memory
                const int hi_t = min(hi, k_start + (info & 0xFF));
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
            // Lazy rescaling: the stored maximum is only raised when some row's maximum grew by
            // more than `lazy`; until then p = exp2((s - m) sl2) <= 2^8, harmless in fp32/bf16,
            // and the final o / l is unchanged because o and l use the same m.
            if (__builtin_amdgcn_ballot_w64(mx > m + lazy) != 0 || __builtin_amdgcn_ballot_w64(m == -INFINITY) != 0) {
                const float m_new = fmaxf(m, mx);
                const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f((m - m_ref) * sl2);   // m = -inf -> 0
                m = m_new;
                l *= alpha;
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[b][e] *= alpha;
            }
            const float msl = ((m == -INFINITY) ? 0.f : m) * sl2;
            bf16x8 pf[2][2];
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
                        l = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l, false);
                        w[x] = __builtin_bit_cast(uint32_t, pb);
                    }
                    pf[kb][t] = __builtin_bit_cast(bf16x8, u32x4{w[0], w[1], w[2], w[3]});
                }
            // ---- O^T += V^T . P^T --------------------------------------------
            // MFMA (kb, t) contracts keys 32kb + 16t + {4hlf..4hlf+3} and {8+4hlf..8+4hlf+3}; the
            // transpose read hands lane i of a 16-lane group column i of a 4-row x 16-column patch.
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                bf16x8 vf[2][DB];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int key0 = 32 * kb + 16 * t + 4 * hlf + (i16 >> 2);
#pragma unroll
                    for (int b = 0; b < DB; ++b) {
                        const int col = 32 * b + 16 * gl + 4 * (i16 & 3);
                        const unsigned char* p0 = vs + key0 * SM::VP + col * 2;
                        const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
                        const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0 + 8 * SM::VP));
                        vf[t][b] = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int b = 0; b < DB; ++b)
                        o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][b], pf[kb][t], o[b], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        e0s = e1s; e0i = e1i;
        e1s = __builtin_amdgcn_readfirstlane(e2.x); e1i = __builtin_amdgcn_readfirstlane(e2.y);
        if (j + 1 < n_kv) PK_SSTORE(stage ^ 1);
        __syncthreads();
    }
#undef PK_GLOAD
#undef PK_SSTORE

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
    static std::mutex attr_mutex;                   // plans may be used from several host threads
    static bool attr_set = false;
    std::lock_guard<std::mutex> attr_lock(attr_mutex);
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

int launch_prefill_bf16_pipe(const PrefillArgs& a, void* stream);

int launch_prefill_bf16(const PrefillArgs& a, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.pipeline == 0) return launch_prefill_bf16_pipe(a, stream);   // direct-to-LDS kernels (prefill_pipe.hip)
    if (a.d == 128) return launch_p<128>(a, st);                       // the register-staged kernel of this file
    if (a.d == 64) return launch_p<64>(a, st);
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace pk
