// Packed prefill attention, bf16 MFMA, head dimension PK_D = 128 or 64 (Sec. 3.1).  Same tables, same
// arithmetic and same operand scheme as prefill.hip (S^T = K.Q^T, O^T += V^T.P^T with
// v_mfma_f32_32x32x16_bf16, one wave per 32 query rows, key tiles of 64), but
//   * K/V tiles go HBM/L2 -> LDS directly (buffer_load ... lds, 16 bytes per lane, no staging
//     registers, hardware bounds check); rows are unpadded and the 16-byte chunks of a row are
//     XOR-swizzled -- the swizzle is applied on the global side of the copy, so that both the K
//     row reads (ds_read_b128) and the V transpose reads (ds_read_b64_tr_b16) are free of bank
//     conflicts;
//   * a key tile is processed as two halves of 32 keys whose softmax steps are interleaved,
//     slice by slice, with the MFMAs of the neighbouring phase, and the LDS operand reads run
//     four MFMAs ahead in a ring of registers: matrix pipe, vector ALU and LDS overlap inside
//     one wave, with no state crossing tiles except the accumulators;
//   * copies are requested one tile ahead for V and two for K; one barrier per tile.

// Device code only: included by prefill_pipe.hip (the prefill launch) and by mixed_step.hip (the
// fused prefill + decode launch).  The includer defines PK_D (the head dimension) and PK_DNS (the
// namespace this instance goes into) first; the file may be included once per head dimension.
// With PK_D = 64 a row is 128 bytes, a tile 8 KiB (two 1-KiB copy instructions per wave) and a
// half tile four MFMAs instead of eight, each followed by two softmax slices instead of one.
#include <cstdint>

#include "common.hip.h"
#include "kernels.h"

#if !defined(PK_D) || !defined(PK_DNS) || (PK_D != 128 && PK_D != 64)
#error "define PK_D (128 or 64) and PK_DNS before including prefill_body.hip.h"
#endif

namespace pk {
namespace {
namespace PK_DNS {

constexpr int BM = 128, BN = 64, D = PK_D;
constexpr int ROWB = D * 2;                        // bytes per K/V row in LDS (unpadded)
constexpr int TILE_BYTES = BN * ROWB;              // 16 KiB (8 KiB for D = 64)
constexpr int KS = D / 16, DB = D / 32;
constexpr int PIECES = TILE_BYTES / 4096;          // 1-KiB copy instructions per wave and tile
constexpr int WAVE_PART = TILE_BYTES / 4;          // bytes of a stage that one wave fills

typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// chunk position p of row `row` holds logical chunk p ^ swz(row)
#if PK_D == 128
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
#else
// 128-byte rows: two rows share a line of the 64 banks, so rows of the same parity need eight
// different values (K row reads of 16 consecutive rows), and rows r and r + 2 must differ in
// bit 2 (the transpose reads take 64 bytes from each of four consecutive rows)
__device__ __forceinline__ int swz(int row) { const int x = (row >> 1) & 7; return ((x & 1) << 2) | (x >> 1); }
#endif

struct LaneOffsets {
    int k[KS];          // K operand read: row n, logical chunk 2 st + hlf (add 32 kb rows)
    int v1[DB];         // V transpose read of column block b, rows +0..3 (add (32 kb + 16 t) rows); the read
                        // of rows +8..11 is at (v1 ^ 32) + 8 rows: its swizzle differs in one bit
#if PK_D == 64
    int v2[DB];         // (128-byte rows: the read of rows +8..11 has an offset of its own)
#endif
    int g[PIECES];      // global byte offsets of this lane's copy instructions
};

__device__ __forceinline__ bf16x8 v_operand(const unsigned char* vs, const LaneOffsets& lo, int kb, int t, int b) {
    const unsigned char* p = vs + (32 * kb + 16 * t) * ROWB;
    const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p + lo.v1[b]));
#if PK_D == 128
    const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p + 8 * ROWB + (lo.v1[b] ^ 32)));
#else
    const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p + lo.v2[b]));
#endif
    return __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
}

// What a workgroup works on, and this lane's share of it.
struct WorkUnit {
    int head, kvh, n_kv, n_lead, n_active, wave, lane, n, hlf;   // this wave computes key tiles [n_lead, n_active)
    int ks0, ks1;                      // first key rows of the tile's first two key tiles
    int qrow, lo, hi;                  // this lane's query row (-1: padding) and its key range [lo, hi)
    const int32_t* kvt;                // key-tile list of the query tile: (first key row, info) pairs
    int64_t row_bytes;                 // bytes between consecutive K/V rows in global memory
    uint32_t row_bytes32, total_rows32;  // the same, and the number of K/V rows, as 32-bit scalars
};

// Decodes the workgroup id, loads the row metadata and the Q operand, derives the lane offsets.
// Returns false for grid padding and for query tiles without key tiles.
__device__ __forceinline__ bool setup(const PrefillArgs& a, const int block, WorkUnit& u, LaneOffsets& off, bf16x8 (&qf)[KS]) {
    const int r = a.Hq / a.Hkv;
    int tile;
    if (a.xcd_swizzle) {               // see prefill.hip: the r heads of a KV head stay on one XCD
        const int x = block, c = x & 7, y = x >> 3, j = y % r, slot = y / r;
        const int64_t p = static_cast<int64_t>(slot) * 8 + c;
        if (p >= static_cast<int64_t>(a.n_tiles) * a.Hkv) return false;
        tile = static_cast<int>(p / a.Hkv); u.kvh = static_cast<int>(p % a.Hkv); u.head = u.kvh * r + j;
    } else {
        tile = block / a.Hq; u.head = block % a.Hq; u.kvh = u.head / r;
    }
    // everything about the tile in one 64-byte scalar load, including the first key rows of its first
    // key tiles: the first K/V copies do not wait for the key-tile list
    typedef int32_t i32x16 __attribute__((ext_vector_type(16)));
    const i32x16 desc = *(const __attribute__((address_space(4))) i32x16*)(a.tiles + 16 * static_cast<int64_t>(tile));
    u.n_kv = desc[1];
    if (u.n_kv == 0) return false;
    u.kvt = a.kvtiles + 2 * static_cast<int64_t>(desc[0]);
    u.ks0 = desc[8]; u.ks1 = desc[9];
    const int tid = threadIdx.x;
    u.lane = tid & 63; u.n = u.lane & 31; u.hlf = u.lane >> 5;
    u.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    u.n_active = u.n_kv - ((desc[3] >> (8 * u.wave)) & 0xFF);
    u.n_lead = min((desc[2] >> (8 * u.wave)) & 0xFF, u.n_active);
    prefill_tile_row(a, tile, desc[4], desc[5], desc[6], desc[7], u.wave * 32 + u.n, u.qrow, u.lo, u.hi);
    u.row_bytes = static_cast<int64_t>(a.Hkv) * ROWB;
    u.row_bytes32 = static_cast<uint32_t>(a.Hkv) * ROWB;
    u.total_rows32 = static_cast<uint32_t>(a.total_kv_rows);

    const int fl = swz(u.n);
#pragma unroll
    for (int st = 0; st < KS; ++st) off.k[st] = u.n * ROWB + (((2 * st + u.hlf) ^ fl) << 4);
    const int i16 = u.lane & 15, gl = (u.lane >> 4) & 1, r4 = i16 >> 2;
    const int rowl = 4 * u.hlf + r4, byte = (i16 & 1) * 8;
#if PK_D == 128
    const int f1 = (r4 << 2) | u.hlf;  // rows +8: (hlf + 2) & 3 = hlf ^ 2, i.e. chunk ^ 2, byte offset ^ 32
#pragma unroll
    for (int b = 0; b < DB; ++b) {
        const int c = 4 * b + 2 * gl + ((i16 & 3) >> 1);
        off.v1[b] = rowl * ROWB + ((c ^ f1) << 4) + byte;
    }
    const int r_in = u.lane >> 4, pos = u.lane & 15;   // a copy instruction takes 4 rows of 16 chunks
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = 16 * u.wave + 4 * q + r_in;
        off.g[q] = static_cast<int>(row * u.row_bytes + u.kvh * ROWB + ((pos ^ swz(row)) << 4));
    }
#else
#pragma unroll
    for (int b = 0; b < DB; ++b) {
        const int c = 4 * b + 2 * gl + ((i16 & 3) >> 1);
        off.v1[b] = rowl * ROWB + ((c ^ swz(rowl)) << 4) + byte;
        off.v2[b] = (rowl + 8) * ROWB + ((c ^ swz(rowl + 8)) << 4) + byte;
    }
    const int r_in = u.lane >> 3, pos = u.lane & 7;    // a copy instruction takes 8 rows of 8 chunks
#pragma unroll
    for (int q = 0; q < PIECES; ++q) {
        const int row = 16 * u.wave + 8 * q + r_in;
        off.g[q] = static_cast<int>(row * u.row_bytes + u.kvh * ROWB + ((pos ^ swz(row)) << 4));
    }
#endif
    // Q operand: lane (n, hlf) holds Q[row n][16s + 8hlf .. +8], as it is in memory: the MFMAs
    // deliver raw scores, exact products of the bf16 inputs summed in fp32.  Only requested here;
    // the first K/V copies follow at once, so that the two round trips to memory overlap.
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

// bf16 output through LDS, so that every row leaves as whole 16-byte pieces (four rows of 256
// bytes, or eight of 128, per store instruction) instead of 8-byte pieces of 32 different rows.
// The wave uses two pieces of LDS of 16 rows each that belong to it alone (rows 0..15 in qa, rows
// 16..31 in qb); the 16-byte chunks of a row are XOR-swizzled with the row number, which keeps
// both sides off bank conflicts.
__device__ __forceinline__ void store_output_bf16(const PrefillArgs& a, const WorkUnit& u, const floatx16 (&o)[DB],
                                                  float l, unsigned char* qa, unsigned char* qb) {
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l), __float_as_uint(l), false, false);
        l = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    constexpr int CPR = D / 8, RPI = 64 / CPR;     // 16-byte chunks per row; rows per store instruction
    const float inv = l > 0.f ? 1.f / l : 0.f;
    const int rr = u.n & 15;
    unsigned char* wrow = (u.n < 16 ? qa : qb) + rr * ROWB + 8 * u.hlf;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {       // columns 32b + 8q4 + 4hlf .. +3: chunk 4b + q4, half hlf
            const float x0 = o[b][4 * q4] * inv, x1 = o[b][4 * q4 + 1] * inv;
            const float x2 = o[b][4 * q4 + 2] * inv, x3 = o[b][4 * q4 + 3] * inv;
            *reinterpret_cast<uint2*>(wrow + (((4 * b + q4) ^ (rr & (CPR - 1))) << 4)) =
                make_uint2(pack_bf16x2(x0, x1), pack_bf16x2(x2, x3));
        }
    const int chunk = u.lane & (CPR - 1);
#pragma unroll
    for (int k = 0; k < 32 / RPI; ++k) {
        const int row = RPI * k + u.lane / CPR, r2 = row & 15;
        const u32x4 v = *reinterpret_cast<const u32x4*>((row < 16 ? qa : qb) + r2 * ROWB + ((chunk ^ (r2 & (CPR - 1))) << 4));
        const int qrow = __shfl(u.qrow, row, 64);
        if (qrow >= 0)
            *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(a.out) +
                                      (static_cast<int64_t>(qrow) * a.Hq + u.head) * D + 8 * chunk) = v;
    }
}

// Copies of K/V tiles into LDS stages.  A tile is 16 instructions of 1 KiB (four per wave; eight and
// two for D = 64), each
// lane fetching the 16-byte chunk that belongs at its (swizzled) LDS position; rows past the end
// of the array arrive as zeros (the descriptor's size is what is left of the array; a tile past
// the end of the key-tile list gets size 0: zeros, no memory traffic).  The copy is issued from
// inline assembly on purpose: the compiler makes every later LDS read wait for all copies it
// knows of, also those into another stage, which would serialise the pipeline.  The waits are
// explicit instead (vmcnt before the barrier that publishes a stage).  Descriptor and LDS address
// are built from wave-uniform values on the scalar ALU; the compiler does not look into the
// assembly for hazards, so the statement carries its own wait states: one is what a scalar write
// of M0 needs, five would cover a descriptor word written by a vector instruction.
__device__ __forceinline__ void lds_copy_16(const u32x4& rsrc, uint32_t lds_addr, int voffset) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory");                       // M0 has no other user in this file
}
// descriptor of the tile that starts at key row KSTART of SRC (a.k or a.v); ENABLED = false: empty
#define PK_TILE_DESC(RS, SRC, KSTART, ENABLED)                                               \
    u32x4 RS;                                                                                \
    {                                                                                        \
        const uint32_t ks_ = static_cast<uint32_t>(KSTART);       /* row counts fit 31 bits */ \
        const uint64_t base_ = reinterpret_cast<uint64_t>(SRC) + static_cast<uint64_t>(ks_) * u.row_bytes32; \
        const uint64_t left_ = static_cast<uint64_t>(u.total_rows32 - ks_) * u.row_bytes32;  \
        RS[0] = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(base_));               \
        RS[1] = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(base_ >> 32) & 0xFFFFu);  /* stride 0: raw buffer */ \
        RS[2] = __builtin_amdgcn_readfirstlane((ENABLED) ? static_cast<uint32_t>(left_ > 0x7FFFFFFFull ? 0x7FFFFFFFull : left_) : 0u); \
        RS[3] = 0x00020000u;                                                                 \
    }
// this wave's piece Q (0..3) of a tile into the stage at byte offset DST
#define PK_COPY_PIECE(RS, DST, Q) lds_copy_16(RS, lds_wave + (DST) + (Q) * 1024, off.g[Q])
#define PK_COPY_TILE(SRC, KSTART, DST, ENABLED)                                              \
    {                                                                                        \
        PK_TILE_DESC(rs_, SRC, KSTART, ENABLED)                                              \
        _Pragma("unroll") for (int q = 0; q < PIECES; ++q) PK_COPY_PIECE(rs_, DST, q);       \
    }
#define PK_WAIT_ALL_COPIES() __builtin_amdgcn_s_waitcnt(0x0F70)      /* vmcnt(0) */
#define PK_CODE(INFO) (((INFO) >> (8 + 2 * u.wave)) & 3)          /* 0 skip, 1 masked, 2 unmasked */

// ---------------------------------------------------------------------------------------------
// Kernel A (default).  Two workgroups per CU (80 KiB of LDS each: three stages for K, two for V).
// A key tile is handled as two halves of 32 keys, each with its own online-softmax step, so that
// within one wave the matrix pipe and the vector ALU overlap without state that crosses tiles:
//   phase 1   S0 = K(half 0) Q^T      with the requests for V(j+1), K(j+2)   (8 MFMAs + 8 copies)
//   phase 2   S1 = K(half 1) Q^T      with the softmax of S0       (8 MFMAs + vector work)
//   phase 3   O += V(half 0)^T P0^T   with the softmax of S1       (8 MFMAs + vector work)
//   phase 4   O += V(half 1)^T P1^T                                (8 MFMAs)
//   barrier   this wave's copies have landed; every wave is done with the tile
// The LDS operand reads run four MFMAs ahead, in a ring of four operand registers that carries over
// the tile boundary (the first operands of tile j + 1 are read during the last MFMAs of tile j).
// Softmax state of a query row.  The MFMAs work on Q and K as they are in memory, so a raw score is
// the exact sum of bf16 products in fp32; one fused multiply-add per score turns it into an exponent
// of two relative to the row's reference: x = sc * s - m_ref, sc = scale * log2 e.  (Folding sc
// into Q instead would save that instruction but costs another rounding of Q to bf16: 2^-9
// relative per element, which for scores of a few units' spread is an error of 0.03 .. 0.04 in
// the output, measured.)
//   m_ref   reference that the exponentials are taken against, in the exp2 domain; it only has to
//           stay within 2^13 of the running maximum, so it moves rarely ("lazy" rescaling);
//   m_set   the row has seen a key (m_ref means something);  l  this lane's share of the row sum.
// Fast path of a half tile (16 scores per lane): p = exp2(x), pairs rounded to bf16, row sums of
// the rounded pairs by dot2, no maximum.  The increment of the sum tells whether the reference is
// still good: if any lane's increment exceeds 2^13 (or a row has no reference yet) the whole wave
// redoes the half tile on the slow path below, which finds the maximum, moves the reference and
// rescales what has been accumulated.  Scores that are still in the making (the other half tile's)
// are raw and meet the new reference when their turn comes.
struct HalfSoftmax {
    float l0, l1;
    uint32_t pw[8];
};
constexpr float kIncLimit = 8192.f;                // 2^13
constexpr float kRaiseBy = 8.f;                    // a set reference is only raised by more than this

// max without the canonicalising self-maximum that fmaxf() costs per operand (scores are never NaN;
// -inf is ordinary here).  Not volatile: the compiler schedules these like any arithmetic.
__device__ __forceinline__ float max3f(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float max2f(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Slice C (0..7) of the fast path: pair C of the half tile, in two stages, so that the conversion
// never waits for its exponentials: stage A (fma, exp) right behind MFMA C, stage B (round, sum,
// pack) behind MFMA C + 1 (1.4 % on the whole kernel; a third stage between fma and exp: nothing).
// The row sum takes the ROUNDED pair, the same numbers that go into P.V: a probability is taken
// against a reference that may lie far from the row maximum, so even a dominant one is not a round
// number, and its rounding error (2^-9 relative) has to cancel between numerator and denominator.
// (Measured: with the unrounded values in the sum a row that one key dominates is off by 1.4e-2,
// with the rounded ones by 5e-3, like a kernel that takes exp against the maximum.)
template <int C>
__device__ __forceinline__ floatx2 slice_a(const floatx16& s, const float sc, const float m_ref) {
    floatx2 pp;
    pp[0] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * C], sc, -m_ref));
    pp[1] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * C + 1], sc, -m_ref));
    return pp;
}
template <int C>
__device__ __forceinline__ void slice_b(const floatx2 pp, HalfSoftmax& h) {
    const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
    if constexpr (C & 1) h.l1 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, h.l1, false);
    else h.l0 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, h.l0, false);
    h.pw[C] = __builtin_bit_cast(uint32_t, pb);
}

// Slow path of a half tile (wave-uniform, rare): s holds the scores relative to the current
// reference.  First the scalars: the row maximum (both lanes of a row agree through the swap),
// the shift `delta` of the reference for the rows that need one, the factor alpha for what has
// been accumulated so far.  The caller then shifts the scores, recomputes the probabilities and
// rescales, each in a branch of its own that holds nothing but updates in place: written as one
// block, the paths join with the 64 accumulators in fresh registers, more than the kernel has.
__device__ __forceinline__ void softmax_slow_scalars(const floatx16& s, float& m_ref, bool& m_set,
                                                     float& delta, float& alpha) {
    float mx = max3f(max3f(max3f(max2f(s[0], s[1]), s[2], s[3]), s[4], s[5]), s[6], s[7]);
    mx = max3f(max3f(max3f(max3f(mx, s[8], s[9]), s[10], s[11]), s[12], s[13]), s[14], s[15]);
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
    mx = max2f(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    const bool seen = mx > -INFINITY;              // the row has a visible key in this half tile
    delta = (seen && (!m_set || mx > kRaiseBy)) ? mx : 0.f;
    alpha = m_set ? __builtin_amdgcn_exp2f(-delta) : 1.f;   // nothing accumulated before the first key
    m_set = m_set || seen;
    m_ref += delta;
}
__device__ __forceinline__ void softmax_redo(floatx16& s, HalfSoftmax& h, float delta) {
    h.l0 = 0.f; h.l1 = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        floatx2 pp;
        pp[0] = __builtin_amdgcn_exp2f(s[2 * q] - delta);
        pp[1] = __builtin_amdgcn_exp2f(s[2 * q + 1] - delta);
        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
        if (q & 1) h.l1 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, h.l1, false);
        else h.l0 = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, h.l0, false);
        h.pw[q] = __builtin_bit_cast(uint32_t, pb);
    }
}
#define PK_SOFTMAX_CHECK(S, H)                                                                 \
    {                                                                                          \
        const bool slow = __builtin_amdgcn_ballot_w64((H.l0 + H.l1) > kIncLimit || !m_set) != 0; \
        float delta = 0.f, alpha = 1.f;                                                        \
        /* the empty asm statements keep the compiler from computing the rare branches always */ \
        if (slow) {                                                                            \
            asm volatile("");                                                                  \
            /* exponents of two relative to the present reference */                           \
            _Pragma("unroll") for (int e = 0; e < 16; ++e) S[e] = __builtin_fmaf(S[e], sc, -m_ref); \
            softmax_slow_scalars(S, m_ref, m_set, delta, alpha);                               \
        }                                                                                      \
        if (slow) { asm volatile(""); softmax_redo(S, H, delta); }                             \
        l = l * alpha + (H.l0 + H.l1);                                                         \
        if (slow) {                                                                            \
            _Pragma("unroll") for (int b = 0; b < DB; ++b)                                     \
                _Pragma("unroll") for (int e = 0; e < 16; ++e) o[b][e] *= alpha;               \
        }                                                                                      \
    }

// The compiler is free to move the (side-effect free) softmax arithmetic and the MFMAs of a phase
// apart again.  Two empty volatile asm statements per slice tie them together: the first makes the
// slice's inputs depend on the point after MFMA i, the second makes the operand of MFMA i+1 depend
// on the point after the slice's results.
template <int C>
__device__ __forceinline__ void pin_slice_inputs(floatx16& acc, floatx16& s) {
    // (not after the first MFMA of a chain: tying its fresh result to the statement makes the
    // compiler copy the sixteen start values into it instead of naming them as the C operand)
    if constexpr (C == 0) asm volatile("" : "+v"(s));
    else asm volatile("" : "+v"(acc), "+v"(s));
}
template <int C>
__device__ __forceinline__ void pin_slice_outputs(bf16x8& next_operand, HalfSoftmax& h) {
    asm volatile("" : "+v"(next_operand), "+v"(h.pw[C]), "+v"(h.l0), "+v"(h.l1));
}

// -inf for the keys of half `half` of a tile that a query row may not see (outside [lo, hi_t)):
// one unsigned comparison per score, (key - lo) < (hi_t - lo).
__device__ __forceinline__ void mask_half(floatx16& s, int half, int lo, int hi_t, int k_start, int hlf) {
    const uint32_t span = static_cast<uint32_t>(max(hi_t - lo, 0));
    const uint32_t base = static_cast<uint32_t>(k_start + 4 * hlf + 32 * half - lo);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        if (base + static_cast<uint32_t>(8 * (e >> 2) + (e & 3)) >= span) s[e] = -INFINITY;
        asm volatile("" : "+v"(s[e]));   // ties the selects to this place, behind the caller's branch
    }
}

// operand x (0..7) of a half tile: K rows of contraction step x; V^T block (t, b) = (x / 4, x % 4)
__device__ __forceinline__ bf16x8 k_operand(const unsigned char* ks, const LaneOffsets& lo, int half, int x) {
    return *reinterpret_cast<const bf16x8*>(ks + lo.k[x] + half * 32 * ROWB);
}
__device__ __forceinline__ bf16x8 v_operand_x(const unsigned char* vs, const LaneOffsets& lo, int half, int x) {
    return v_operand(vs, lo, half, x / DB, x % DB);
}
// Operand stream of a tile (KS operands per half tile; shown for D = 128): 0..7 K(half 0), 8..15
// K(half 1), 16..23 V(half 0), 24..31 V(half 1), 32..35 the first K operands of the next tile.
// MFMA k takes ring[k % 4] and then refills that slot with operand k + 4, so that every LDS read
// has four MFMAs (and their vector slices) to land.
template <int K>
__device__ __forceinline__ bf16x8 stream_operand(const unsigned char* k_cur, const unsigned char* v_cur,
                                                 const unsigned char* k_next, const LaneOffsets& off) {
    if constexpr (K < 2 * KS) return k_operand(k_cur, off, K / KS, K % KS);
    else if constexpr (K < 4 * KS) return v_operand_x(v_cur, off, (K - 2 * KS) / KS, K % KS);
    else return k_operand(k_next, off, 0, K - 4 * KS);
}
#define PK_REFILL(K0) ring[i & 3] = stream_operand<(K0) + i + 4>(lds + k_cur, lds + v_cur, lds + k_next, off)
#define PK_SLICE(C, S, H, ACC, BODY)                                                          \
    {                                                                                          \
        constexpr int i = C;                                                                   \
        BODY;                                                                                  \
        pin_slice_inputs<C>(ACC, S);                                                           \
        if constexpr (C > 0) slice_b<(C > 0 ? C - 1 : 0)>(pend, H);                            \
        pend = slice_a<C>(S, sc, m_ref);                                                       \
        asm volatile("" : "+v"(pend));                                                         \
        pin_slice_outputs<(C > 0 ? C - 1 : 0)>(ring[(C + 1) & 3], H);                          \
    }
#if PK_D == 128
// eight MFMAs (BODY, with accumulator ACC) interleaved with the softmax of the scores S
#define PK_SLICES(S, H, ACC, BODY)                                                             \
    {                                                                                          \
    floatx2 pend;                                                                              \
    PK_SLICE(0, S, H, ACC, BODY) PK_SLICE(1, S, H, ACC, BODY) PK_SLICE(2, S, H, ACC, BODY)       \
    PK_SLICE(3, S, H, ACC, BODY) PK_SLICE(4, S, H, ACC, BODY) PK_SLICE(5, S, H, ACC, BODY)       \
    PK_SLICE(6, S, H, ACC, BODY) PK_SLICE(7, S, H, ACC, BODY)                                    \
    slice_b<7>(pend, H);                                                                       \
    }

#define PK_EIGHT(BODY)                                                                         \
    {                                                                                          \
        { constexpr int i = 0; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 1; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 2; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 3; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 4; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 5; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 6; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 7; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
    }
#else
// D = 64: four MFMAs per half tile, each followed by two of the eight softmax slices
#define PK_SLICE2(I, S, H, ACC, BODY)                                                          \
    {                                                                                          \
        constexpr int i = I;                                                                   \
        BODY;                                                                                  \
        pin_slice_inputs<I>(ACC, S);                                                           \
        if constexpr ((I) > 0) {                                                               \
            slice_b<((I) > 0 ? 2 * (I) - 2 : 0)>(pend, H);                                     \
            slice_b<((I) > 0 ? 2 * (I) - 1 : 1)>(pend2, H);                                    \
        }                                                                                      \
        pend = slice_a<2 * (I)>(S, sc, m_ref);                                                 \
        pend2 = slice_a<2 * (I) + 1>(S, sc, m_ref);                                            \
        asm volatile("" : "+v"(pend), "+v"(pend2));                                            \
        pin_slice_outputs<((I) > 0 ? 2 * (I) - 2 : 0)>(ring[((I) + 1) & 3], H);                \
        pin_slice_outputs<((I) > 0 ? 2 * (I) - 1 : 1)>(ring[((I) + 1) & 3], H);                \
    }
#define PK_SLICES(S, H, ACC, BODY)                                                             \
    {                                                                                          \
    floatx2 pend, pend2;                                                                       \
    PK_SLICE2(0, S, H, ACC, BODY) PK_SLICE2(1, S, H, ACC, BODY) PK_SLICE2(2, S, H, ACC, BODY)    \
    PK_SLICE2(3, S, H, ACC, BODY)                                                              \
    slice_b<6>(pend, H);                                                                       \
    slice_b<7>(pend2, H);                                                                      \
    }

#define PK_EIGHT(BODY)                                                                         \
    {                                                                                          \
        { constexpr int i = 0; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 1; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 2; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
        { constexpr int i = 3; BODY; __builtin_amdgcn_sched_barrier(0); }                      \
    }
#endif

// `block`: the workgroup's number in the prefill launch order; `lds`: 5 * TILE_BYTES, 1 KiB aligned
// (K stages 0..2, V stages 3..4).
__device__ __forceinline__ void prefill_tile_body(const PrefillArgs& a, const int block, unsigned char* lds) {
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void_ptr)lds));
    WorkUnit u;
    LaneOffsets off;
    bf16x8 qf[KS];
    if (!setup(a, block, u, off, qf)) return;
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
    // rows without a query count as "set" so that they never ask for the slow path
    float m_ref = 0.f, l = 0.f;
    bool m_set = u.qrow < 0;
    const floatx16 zero16 = {};
    const float sc = a.scale * kLog2e;             // raw score -> exponent of two (the API admits only finite scale > 0)

    // this wave's quarter of a stage, as a scalar
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds_base + u.wave * WAVE_PART);
    // window of tile-list entries: e0 = tile j, e1 = tile j+1, e2 = tile j+2 (e3 is fetched for the next turn)
    int e0s, e0i, e1s, e1i, e2s, e2i;
    entry(0, e0s, e0i); entry(1, e1s, e1i); entry(2, e2s, e2i);
    // prologue: K(0), K(1), V(0), from the key rows in the descriptor (the entries above arrive meanwhile)
    PK_COPY_TILE(a.k, u.ks0, 0, true);
    PK_COPY_TILE(a.k, u.ks1, TILE_BYTES, 1 < n_kv);
    PK_COPY_TILE(a.v, u.ks0, 3 * TILE_BYTES, true);
    PK_WAIT_ALL_COPIES();
    __syncthreads();

    bf16x8 ring[4];                                 // LDS operands of the next four MFMAs
#pragma unroll
    for (int x = 0; x < 4; ++x) ring[x] = k_operand(lds, off, 0, x);
    int k_cur = 0, k_next = TILE_BYTES, k_fill = 2 * TILE_BYTES;   // K stage read now / next / filled now
    int v_cur = 3 * TILE_BYTES, v_fill = 4 * TILE_BYTES;
    // Tile j: while S0 is computed, V(j+1) and K(j+2) are requested into the stages of V(j-1) and
    // K(j-1), one 1-KiB piece behind each of the eight MFMAs, where their issue costs nothing.  The
    // barrier at the END of the tile (after this wave's copies have landed: only they matter, the
    // compiler's own barrier would also wait for the LDS reads) says that every wave is done with
    // tile j and that V(j+1) and K(j+2) are complete; K(j+1), whose first operands are read during
    // the last MFMAs of tile j, was published a tile earlier.
#define PK_TILE_BEGIN()                                                                       \
    PK_TILE_DESC(rs_k, a.k, e2s, j + 2 < n_kv)                                                 \
    PK_TILE_DESC(rs_v, a.v, e1s, j + 1 < n_kv)
#define PK_COPY_STEP(I)                                                                       \
    if constexpr ((I) < PIECES) PK_COPY_PIECE(rs_k, k_fill, (I));                              \
    else PK_COPY_PIECE(rs_v, v_fill, (I) - PIECES);
    // (the next list entry is fetched right before the barrier: scalar loads and LDS reads share a
    // counter and return out of order, so the first wait after the fetch drains the operand ring;
    // here the ring has the whole barrier to land anyway)
#define PK_TILE_END()                                                                         \
    int e3s, e3i;                                                                              \
    entry(j + 3, e3s, e3i);                                                                    \
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");                              \
    e0s = e1s; e0i = e1i; e1s = e2s; e1i = e2i; e2s = e3s; e2i = e3i;                          \
    { const int kc = k_cur; k_cur = k_next; k_next = k_fill; k_fill = kc; }                    \
    { const int vc = v_cur; v_cur = v_fill; v_fill = vc; }

    int j = 0;
    // leading tiles that this wave skips: it only takes part in the copies and in the barriers,
    // then picks up its first operands from the stage that is current by then
    for (; j < u.n_lead; ++j) {
        PK_TILE_BEGIN();
#pragma unroll
        for (int q = 0; q < PIECES; ++q) { PK_COPY_PIECE(rs_k, k_fill, q); PK_COPY_PIECE(rs_v, v_fill, q); }
        PK_TILE_END();
    }
    if (u.n_lead > 0) {
#pragma unroll
        for (int x = 0; x < 4; ++x) ring[x] = k_operand(lds + k_cur, off, 0, x);
    }
    for (; j < u.n_active; ++j) {
        // a tile that this wave could skip inside its active range is computed as a masked one
        const bool masked = PK_CODE(e0i) != 2;
        const int k_start = e0s;
        const int hi_t = min(u.hi, k_start + (e0i & 0xFF));   // keys past the tile's valid count are foreign
        PK_TILE_BEGIN();
        floatx16 s0, s1;
        PK_EIGHT(s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i & 3], qf[i], i == 0 ? zero16 : s0, 0, 0, 0);
                 PK_REFILL(0); PK_COPY_STEP(i));
        HalfSoftmax h0, h1;
        h0.l0 = 0.f; h0.l1 = 0.f; h1.l0 = 0.f; h1.l1 = 0.f;
        if (masked) mask_half(s0, 0, u.lo, hi_t, k_start, u.hlf);    // unmasked tiles skip the compares
        PK_SLICES(s0, h0, s1, s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i & 3], qf[i], i == 0 ? zero16 : s1, 0, 0, 0);
                  PK_REFILL(KS));
        PK_SOFTMAX_CHECK(s0, h0)
        bf16x8 p0[2], p1[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
            p0[t] = __builtin_bit_cast(bf16x8, u32x4{h0.pw[4 * t], h0.pw[4 * t + 1], h0.pw[4 * t + 2], h0.pw[4 * t + 3]});
        if (masked) mask_half(s1, 1, u.lo, hi_t, k_start, u.hlf);
        PK_SLICES(s1, h1, o[i % DB], o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i & 3], p0[i / DB], o[i % DB], 0, 0, 0);
                  PK_REFILL(2 * KS));
        PK_SOFTMAX_CHECK(s1, h1)
#pragma unroll
        for (int t = 0; t < 2; ++t)
            p1[t] = __builtin_bit_cast(bf16x8, u32x4{h1.pw[4 * t], h1.pw[4 * t + 1], h1.pw[4 * t + 2], h1.pw[4 * t + 3]});
        // phase 4; its last refills are the first operands of the next tile
        PK_EIGHT(o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i & 3], p1[i / DB], o[i % DB], 0, 0, 0);
                 PK_REFILL(3 * KS));
        PK_TILE_END();
    }
    // trailing tiles that this wave skips: it only takes part in the copies and in the barriers
    for (; j < n_kv; ++j) {
        PK_TILE_BEGIN();
#pragma unroll
        for (int q = 0; q < PIECES; ++q) { PK_COPY_PIECE(rs_k, k_fill, q); PK_COPY_PIECE(rs_v, v_fill, q); }
        PK_TILE_END();
    }
    // After the last barrier nobody reads or fills the two stages that would have taken tiles
    // n_kv and n_kv + 1 (after the final rotation: k_next and v_cur), and a wave's copies only
    // ever touch its own quarter of a stage: those two quarters stage this wave's output.
    PK_WAIT_ALL_COPIES();                          // (none is outstanding here; kept as a guard)
    if (a.out_f32) store_output(a, u, o, l);
    else store_output_bf16(a, u, o, l, lds + k_next + u.wave * WAVE_PART, lds + v_cur + u.wave * WAVE_PART);
}

#undef PK_COPY_TILE
#undef PK_TILE_DESC
#undef PK_COPY_PIECE
#undef PK_COPY_STEP
#undef PK_SOFTMAX_CHECK
#undef PK_TILE_BEGIN
#undef PK_TILE_END
#undef PK_SLICE
#undef PK_SLICE2
#undef PK_SLICES
#undef PK_EIGHT
#undef PK_REFILL
#undef PK_WAIT_ALL_COPIES
#undef PK_CODE

}  // namespace PK_DNS
}  // namespace
}  // namespace pk
