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
};
int launch_decode_bf16(const DecodeArgs& a, void* stream);
int launch_decode_f32(const DecodeArgs& a, void* stream);

struct PrefillArgs {
    const void* q; const void* k; const void* v; void* out;
    const int32_t* tiles; int32_t n_tiles;
    const int32_t* row_q; const int32_t* row_lo; const int32_t* row_hi;
    const int32_t* kvtiles;
    const int32_t* q_start; const int32_t* kv_start; int32_t n;
    int64_t total_q_rows; int64_t total_kv_rows;
    int Hq; int Hkv; int d; float scale; int out_f32;
    int xcd_swizzle;                                // 1: place the heads of a KV head on one XCD
};
int launch_prefill_bf16(const PrefillArgs& a, void* stream);
int launch_prefill_f32(const PrefillArgs& a, void* stream);

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
