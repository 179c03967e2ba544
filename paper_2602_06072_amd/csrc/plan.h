// Internal structures of the packing plan and of its device tables.
// Host-side only; the device kernels see the tables as plain int32 arrays.
#pragma once
#include <cstddef>
#include <cstdint>
#include <exception>
#include <new>
#include <string>
#include <vector>

#include "../../include/packinfer.h"

namespace pk {

// ---- tile shapes shared by the schedule builder and the kernels -----------
constexpr int kPrefillBM = 128;     // query rows per workgroup tile (4 waves x 32)
constexpr int kPrefillBN = 64;      // keys per K/V tile
constexpr int kDecodeBlock = PK_KV_BLOCK;   // tokens per buffer tile
constexpr int kDecodeMaxRows = 32;  // query rows (members x heads-per-KV-head) per work item
constexpr int kTileDescWords = 16;  // int32 words per query-tile descriptor of the prefill schedules (one 64-byte scalar load)

struct Member {                     // O_g[i] of Alg. 1 Part 2, offsets relative to the group base
    int32_t req, prefix_off, lp, suffix_off, lq;   // prefix_off / lp: the innermost shared segment (suffix_off / 0: none)
    int32_t node = -1;              // index of that segment in Group::nodes
    int32_t shared = 0;             // tokens of the request that lie in shared segments (its suffix starts there)
};

struct Node {                       // a shared segment of the group's prefix forest (Sec. 3.2, Eq. 5)
    int32_t id = 0;                 // the caller's node number (tree plans) or a running number
    int32_t off = 0, len = 0;       // where it lies in the group buffer
    int32_t parent = -1;            // index in Group::nodes; parents come first
    int32_t start = 0;              // logical token position of its first token inside a request
    std::vector<int32_t> reqs;      // the requests below it, ascending
};

struct Group {
    int64_t load = 0;               // L(S_g): unique KV tokens
    int64_t buf_tokens = 0;         // M(S_g) incl. headroom
    int64_t buf_base = 0;           // token offset of B_g inside the buffer
    std::vector<Member> members;    // layout order
    std::vector<Node> nodes;        // layout order (a one-level family is one node)
};

// One array inside the workspace.
struct TableRef {
    size_t offset = 0;              // bytes from the workspace base
    size_t count = 0;               // int32 elements
};

// Host image of everything that is copied to the device for one head shape.
struct DeviceTables {
    int Hq = 0, Hkv = 0, d = 0, dtype = -1;
    std::vector<int32_t> host;      // concatenated tables (each 64-int aligned)
    // common
    TableRef q_start, kv_start;     // [n+1] caller-order cumulative rows
    // re-layout
    TableRef reorg_seg;             // [nseg][4] dst0, ntok, req, src0 (sorted by dst0)
    TableRef reorg_blk_first;       // [NB] first segment that may overlap tile b
    int32_t n_reorg_seg = 0;
    // decode
    TableRef dec_items;             // [n_items][8]
    TableRef dec_members;           // request ids of the work items' rows
    TableRef dec_member_slot;       // partial slot of each (item, member), -1: the item writes the output
    TableRef dec_req_part_start;    // [n+1] first slot of each request (slots of a request are consecutive)
    TableRef dec_req_seg;           // [n][4] absolute prefix_off, L_P, suffix_off, L_Q (innermost shared segment)
    TableRef dec_chain_start;       // [n+1] first entry of each request in dec_chain
    TableRef dec_chain;             // (absolute offset, tokens) of a request's shared segments, outermost first
    int32_t n_dec_items = 0, n_dec_wide = 0, n_dec_parts = 0, dec_split_tokens = 0;
    int32_t dec_max_parts = 0;      // most partial results of one request
    int32_t pad_split_tokens = 0, pad_n_splits = 0;   // padded decode comparison: uniform splits
    // prefill (packed and padded schedules share one format)
    struct PrefillSched {
        TableRef tiles;             // [n_tiles][8] kv_first, n_kv, leading / trailing skipped key tiles per wave (4 x 8 bits each),
                                    // rows | runs << 16, then Q row, lo, hi of tile row 0 (the first run)
        TableRef run_first;         // [n_tiles] first entry of the tile's further runs
        TableRef runs;              // (first tile row, its Q row, lo, its hi) of the runs after a tile's first
        TableRef kvtiles;           // [n_kv_total][2] k_start, n | wavemask<<8 | full<<16
        int32_t n_tiles = 0;
        int64_t issued_pairs = 0;
    } packed, padded;
    // padded prefill schedule: built on first use, uploaded behind the partial results
    std::vector<int32_t> host_padded;
    bool padded_built = false, padded_uploaded = false;
    size_t padded_offset = 0;
    // partial results (floats) live after the tables
    size_t tables_bytes = 0;
    size_t partial_offset = 0;      // bytes
    size_t partial_bytes = 0;
    size_t total_bytes = 0;
    size_t decode_only_bytes = 0;   // tables + the packed decode partials alone (what the static scratch must hold)
};

}  // namespace pk

struct pk_plan {
    int32_t n = 0;
    int64_t token_budget = 0;
    int32_t headroom = 0;
    bool decode_only = false;       // every q_len == 1
    bool tree = false;              // made by pk_pack_plan_tree (nested shared segments)
    std::vector<int32_t> kv_lens, q_lens, prefix_lens;   // prefix_lens: 0 if no family
    std::vector<pk::Group> groups;
    int64_t buf_tokens = 0;         // whole buffer, multiple of PK_KV_BLOCK
    int64_t unique_tokens = 0;
    int64_t unmasked_pairs = 0;
    std::vector<int32_t> words;     // canonical serialisation
    int32_t tune_decode_split = 0;  // pk_plan_tune: 0 = chosen by the schedule builder
    int32_t tune_prefill_pipeline = 0;   // 1: the register-staged prefill kernel (pk_plan_tune)
    // binding state: a cache of what was last built / uploaded for this plan, also filled by the
    // size query on a const plan (calls on one plan are serialised by the caller)
    mutable pk::DeviceTables tables;
    mutable void* bound_ws = nullptr;
    mutable size_t bound_bytes = 0;
    uint64_t bound_stamp = 0;       // stamp of the bind that wrote bound_ws (0: none)
};

namespace pk {

void set_error(const std::string& msg);

// Exception barrier of the C ABI: nothing may unwind through an extern "C" entry point.  Host
// containers can throw (std::bad_alloc, std::length_error); the entry point then reports an
// error code and a message like any other failure.
template <class R, class F>
R guarded(R on_alloc, R on_other, const char* who, F&& body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        try { set_error(std::string(who) + ": out of host memory"); } catch (...) {}
        return on_alloc;
    } catch (const std::exception& e) {
        try { set_error(std::string(who) + ": " + e.what()); } catch (...) {}
        return on_other;
    } catch (...) {
        try { set_error(std::string(who) + ": unknown failure"); } catch (...) {}
        return on_other;
    }
}

// schedule.cpp
void build_tables(const pk_plan& plan, int Hq, int Hkv, int d, int dtype, int num_cus, DeviceTables& out);
void build_prefill_padded(const pk_plan& plan, DeviceTables& t);
size_t kv_buf_bytes(const pk_plan& plan, int Hkv, int d, int dtype);

}  // namespace pk
