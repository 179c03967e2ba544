// Host-callable launchers of the gfx950 kernels.  Every launcher enqueues on
// `stream` and returns the hipError_t of the launch as int (0 = success).
// All pointers are device pointers.
#pragma once
#include <cstdint>

namespace pk {

struct ReorgArgs {
    const void* k_pages; const void* v_pages;       // [num_blocks][page][Hkv][d]
    const int32_t* block_table; int32_t max_blocks; int32_t page_size; int64_t num_blocks;
    const int32_t* seg; int32_t n_seg;              // [n_seg][4]
    const int32_t* blk_first;                       // [n_tiles]
    void* kv_buf; int64_t buf_tokens; int Hkv; int d;
};
int launch_reorg_bf16(const ReorgArgs& a, void* stream);
int launch_reorg_f32(const ReorgArgs& a, void* stream);

struct AppendArgs {
    const void* k_new; const void* v_new;           // [n][Hkv][d]
    void* kv_buf; const int32_t* req_seg;           // [n][4]: prefix_off, L_P, suffix_off, L_Q (absolute tokens)
    int64_t buf_tokens; int32_t n; int32_t step; int Hkv; int d;
};
int launch_append_bf16(const AppendArgs& a, void* stream);
int launch_append_f32(const AppendArgs& a, void* stream);

struct DecodeArgs {
    const void* q; const void* kv_buf; void* out;
    const int32_t* items; int32_t n_items; int32_t n_wide;   // the first n_wide items have > 16 query rows
    const int32_t* members; const int32_t* member_slot;
    const int32_t* req_part_start;
    const int32_t* req_seg;
    const int32_t* chain_start; const int32_t* chain;   // per request: (offset, tokens) of its shared segments
    float* part_o; float* part_lse;
    int64_t buf_tokens; int32_t n; int Hq; int Hkv; int d; float scale; int out_f32;
    int32_t grown;                                  // tokens appended to every suffix since the plan was made
    int32_t max_parts;                              // most partial results of one request
};
int launch_decode_bf16(const DecodeArgs& a, void* stream);
int launch_decode_merge_bf16(const DecodeArgs& a, void* stream);   // the LSE merge alone
// Device address of the library's fixed scratch array on the current device (looked up once per
// device); returns a hipError_t as int.
int static_scratch_address(void** ptr);
int launch_decode_f32(const DecodeArgs& a, void* stream);

struct PrefillArgs {
    const void* q; const void* k; const void* v; void* out;
    const int32_t* tiles; int32_t n_tiles;
    const int32_t* run_first; const int32_t* runs;   // rows of a tile beyond its first run of consecutive rows
    const int32_t* kvtiles;
    const int32_t* q_start; const int32_t* kv_start; int32_t n;
    int64_t total_q_rows; int64_t total_kv_rows;
    int Hq; int Hkv; int d; float scale; int out_f32;
    int xcd_swizzle;                                // 1: place the heads of a KV head on one XCD
    int pipeline;                                   // 0: K/V tiles copied straight into LDS; 1: staged through registers
};
#if defined(__HIPCC__)
// Row `local` (0..127) of query tile `tile`: its Q row (-1: padding) and its key range [lo, hi).
// d4..d7 are words 4..7 of the tile's descriptor (rows | runs << 16; Q row, lo, hi of tile row 0).
// A run is a stretch of consecutive rows of one request: inside it the Q row and hi advance by one
// per row.  Tiles of one run (nearly all) need nothing but the descriptor.
__device__ __forceinline__ void prefill_tile_row(const PrefillArgs& a, int tile, int d4, int d5, int d6, int d7,
                                                 int local, int& qrow, int& lo, int& hi) {
    const int n_rows = d4 & 0xFFFF, n_runs = d4 >> 16;
    int begin = 0, q0 = d5, l0 = d6, h0 = d7;
    if (n_runs > 1) {                               // uniform: a packed tile that holds several requests
        const int32_t* rp = a.runs + 4 * static_cast<int64_t>(a.run_first[tile]);
        for (int r = 1; r < n_runs; ++r, rp += 4) {
            const int rb = rp[0];
            if (local >= rb) { begin = rb; q0 = rp[1]; l0 = rp[2]; h0 = rp[3]; }
        }
    }
    const bool valid = local < n_rows;
    qrow = valid ? q0 + (local - begin) : -1;
    lo = valid ? l0 : 0;
    hi = valid ? h0 + (local - begin) : 0;
}
#endif
int launch_prefill_bf16(const PrefillArgs& a, void* stream);
int launch_prefill_f32(const PrefillArgs& a, void* stream);
// prefill tiles and decode work items of one step in one launch (bf16, d = 128), then the LSE merge
int launch_mixed_step_bf16(const PrefillArgs& pa, const DecodeArgs& da, void* stream);

struct PagedDecodeArgs {
    const void* q; const void* k_pages; const void* v_pages; void* out;
    const int32_t* block_table; int32_t max_blocks; int32_t page_size; int64_t num_blocks;
    const int32_t* kv_start;                        // [n+1] cumulative kv_lens
    float* part_o; float* part_lse;
    int32_t n; int32_t n_splits; int32_t split_tokens;
    int Hq; int Hkv; int d; float scale; int out_f32;
};
int launch_padded_decode_bf16(const PagedDecodeArgs& a, void* stream);

}  // namespace pk
