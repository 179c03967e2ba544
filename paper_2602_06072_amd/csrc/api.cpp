// C ABI: argument validation, binding of plan tables to a workspace, launches.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <initializer_list>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "kernels.h"
#include "plan.h"

using namespace pk;

namespace {

int fail(int code, const std::string& msg) {
    set_error(msg);
    return code;
}

int hip_fail(const char* where, int err) {
    return fail(PK_EHIP, std::string(where) + ": " + hipGetErrorString(static_cast<hipError_t>(err)));
}

// the kernels move 16 bytes per lane: every tensor pointer must be 16-byte aligned
bool aligned16(std::initializer_list<const void*> ptrs) {
    for (const void* p : ptrs)
        if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return false;
    return true;
}

bool shape_ok(int Hq, int Hkv, int d, int dtype, std::string& why) {
    if (Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0) { why = "need Hq, Hkv, d > 0 and Hq % Hkv == 0"; return false; }
    if (dtype != PK_BF16 && dtype != PK_F32) { why = "dtype must be PK_BF16 or PK_F32"; return false; }
    return true;
}

// Pinned host staging for the table copies.  A copy from pageable memory blocks the host until the
// stream has drained; from pinned memory it is asynchronous, so the planning of the next batch
// overlaps the kernels of the current one.  Buffers are recycled once the event recorded behind
// their copy has completed; the pool only grows while every buffer is still in flight.
struct Staging {
    void* ptr = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool used = false;                              // an event has been recorded for it
    bool busy = false;                              // handed out and not yet released by copy_tables
};
std::mutex g_staging_mutex;
std::vector<Staging> g_staging;

// may_allocate = false: only a buffer that already exists is handed out
Staging* staging_acquire(size_t bytes, bool may_allocate) {
    std::lock_guard<std::mutex> lock(g_staging_mutex);
    for (Staging& s : g_staging)
        if (!s.busy && s.cap >= bytes && (!s.used || hipEventQuery(s.done) == hipSuccess)) { s.busy = true; return &s; }
    if (!may_allocate || g_staging.size() >= 64) return nullptr;     // fall back to a pageable copy
    Staging s;
    s.cap = (bytes + (1u << 20) - 1) >> 20 << 20;
    if (hipHostMalloc(&s.ptr, s.cap, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    if (hipEventCreateWithFlags(&s.done, hipEventDisableTiming) != hipSuccess) {
        (void)hipGetLastError(); (void)hipHostFree(s.ptr); return nullptr;
    }
    s.busy = true;
    g_staging.reserve(64);                          // pointers into the vector stay valid
    g_staging.push_back(s);
    return &g_staging.back();
}

// recorded: the event behind the copy has been recorded (otherwise the buffer is free at once)
void staging_release(Staging* s, bool recorded) {
    std::lock_guard<std::mutex> lock(g_staging_mutex);
    s->used = recorded;
    s->busy = false;
}

int copy_tables(void* dst, const void* src, size_t bytes, void* stream, bool may_allocate = true) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    Staging* s = staging_acquire(bytes, may_allocate);
    if (!s) return static_cast<int>(hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, st));
    std::memcpy(s->ptr, src, bytes);
    hipError_t e = hipMemcpyAsync(dst, s->ptr, bytes, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) {
        // the copy may or may not have been queued: keep the buffer out of circulation until the stream drains
        (void)hipStreamSynchronize(st);
        staging_release(s, false);
        return static_cast<int>(e);
    }
    e = hipEventRecord(s->done, st);
    if (e != hipSuccess) (void)hipStreamSynchronize(st);    // no event to wait for: drain instead
    staging_release(s, e == hipSuccess);
    return static_cast<int>(e);
}

// Which bind wrote a workspace last.  A plan only skips the upload of its tables when it was the
// last one to bind that workspace: two plans that take turns on one workspace through the compute
// calls each find the other's stamp and upload again.  (What the caller does to the bytes of a
// workspace behind the library's back cannot be seen here; pk_plan_bind always uploads.)
std::mutex g_owner_mutex;
std::unordered_map<const void*, uint64_t> g_owner;   // workspace -> stamp of its last bind
uint64_t g_next_stamp = 1;

bool owns_workspace(const pk_plan* plan, const void* workspace) {
    std::lock_guard<std::mutex> lock(g_owner_mutex);
    auto it = g_owner.find(workspace);
    return it != g_owner.end() && it->second == plan->bound_stamp;
}

uint64_t claim_workspace(const void* workspace) {
    std::lock_guard<std::mutex> lock(g_owner_mutex);
    if (g_owner.size() > 4096) g_owner.clear();     // forgetting an owner only costs it an upload
    return g_owner[workspace] = g_next_stamp++;
}

// Compute units of the current device (the decode schedule sizes its work items to fill them);
// 256 when there is no device to ask (table sizes can be queried on a host without one).
int device_cus() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    return cus;
}

// Makes sure the plan's device tables for this shape live in `workspace`.
// fixed_scratch: `workspace` is the library's own fixed array (pk_packed_decode_attn_static): it
// only has to hold the tables and the packed decode partials, and nothing may be allocated.
int ensure_bound(pk_plan* plan, int Hq, int Hkv, int d, int dtype, void* workspace,
                 size_t workspace_bytes, void* stream, bool fixed_scratch = false) {
    DeviceTables& t = plan->tables;
    const bool same_shape = t.Hq == Hq && t.Hkv == Hkv && t.d == d && t.dtype == dtype;
    if (same_shape && plan->bound_ws == workspace && plan->bound_bytes == workspace_bytes &&
        owns_workspace(plan, workspace)) return PK_OK;
    if (!workspace) return fail(PK_EINVAL, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return fail(PK_EINVAL, "workspace must be 256-byte aligned");
    if (!same_shape) build_tables(*plan, Hq, Hkv, d, dtype, device_cus(), t);
    if (fixed_scratch) {
        if (workspace_bytes < t.decode_only_bytes)
            return fail(PK_EUNSUPPORTED, "pk_packed_decode_attn_static: the plan needs " + std::to_string(t.decode_only_bytes) +
                        " bytes of tables and partial results, the fixed scratch holds " + std::to_string(workspace_bytes) +
                        " (PK_STATIC_SCRATCH_BYTES); use pk_packed_decode_attn with a workspace");
    } else if (workspace_bytes < t.total_bytes) {
        return fail(PK_EINVAL, "workspace smaller than pk_workspace_bytes");
    }
    if (t.tables_bytes) {
        const int e = copy_tables(workspace, t.host.data(), t.tables_bytes, stream, !fixed_scratch);
        if (e != 0) return hip_fail("pk_plan_bind (copy of tables)", e);
    }
    plan->bound_ws = workspace;
    plan->bound_bytes = workspace_bytes;
    plan->bound_stamp = claim_workspace(workspace);
    t.padded_uploaded = false;
    return PK_OK;
}

// The padded comparison schedule is built and copied on its first use only.
int ensure_padded(pk_plan* plan, void* stream) {
    DeviceTables& t = plan->tables;
    if (!t.padded_built) build_prefill_padded(*plan, t);
    if (t.padded_uploaded) return PK_OK;
    if (t.padded_offset + t.host_padded.size() * sizeof(int32_t) > plan->bound_bytes)
        return fail(PK_EINVAL, "workspace smaller than pk_workspace_bytes");
    if (!t.host_padded.empty()) {
        const int e = copy_tables(static_cast<char*>(plan->bound_ws) + t.padded_offset, t.host_padded.data(),
                                  t.host_padded.size() * sizeof(int32_t), stream);
        if (e != 0) return hip_fail("copy of the padded schedule", e);
    }
    t.padded_uploaded = true;
    return PK_OK;
}

const int32_t* tab(const pk_plan* plan, const TableRef& r, size_t base = 0) {
    return reinterpret_cast<const int32_t*>(static_cast<const char*>(plan->bound_ws) + base + r.offset);
}

}  // namespace

extern "C" size_t pk_kv_buf_bytes(const pk_plan* plan, int Hkv, int d, int dtype) {
    return pk::guarded<size_t>(size_t{0}, size_t{0}, "pk_kv_buf_bytes", [&]() -> size_t {
        if (!plan || Hkv <= 0 || d <= 0) return 0;
        return kv_buf_bytes(*plan, Hkv, d, dtype);
    });
}

extern "C" size_t pk_workspace_bytes(const pk_plan* plan, int Hq, int Hkv, int d, int dtype) {
    return pk::guarded<size_t>(size_t{0}, size_t{0}, "pk_workspace_bytes", [&]() -> size_t {
        std::string why;
        if (!plan || !shape_ok(Hq, Hkv, d, dtype, why)) return 0;
        const DeviceTables& t = plan->tables;
        if (t.Hq == Hq && t.Hkv == Hkv && t.d == d && t.dtype == dtype) return t.total_bytes;
        // the tables are a cache inside the plan (mutable): the bind that follows reuses them
        build_tables(*plan, Hq, Hkv, d, dtype, device_cus(), plan->tables);
        plan->bound_ws = nullptr;
        return plan->tables.total_bytes;
    });
}

extern "C" int pk_plan_bind(pk_plan* plan, int Hq, int Hkv, int d, int dtype,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_plan_bind", [&]() -> int {
        std::string why;
        if (!plan) return fail(PK_EINVAL, "pk_plan_bind: plan is NULL");
        if (!shape_ok(Hq, Hkv, d, dtype, why)) return fail(PK_EINVAL, "pk_plan_bind: " + why);
        plan->bound_ws = nullptr;                      // force the copy
        return ensure_bound(plan, Hq, Hkv, d, dtype, workspace, workspace_bytes, stream);
    });
}

extern "C" int pk_kv_reorganize(pk_plan* plan, const void* k_pages, const void* v_pages,
                                const int32_t* block_table, int32_t max_blocks_per_req,
                                int32_t page_size, int64_t num_blocks, int Hkv, int d, int dtype,
                                void* kv_buf, void* workspace, size_t workspace_bytes, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_kv_reorganize", [&]() -> int {
        std::string why;
        if (!plan) return fail(PK_EINVAL, "pk_kv_reorganize: plan is NULL");
        if (plan->n == 0) return PK_OK;
        if (!k_pages || !v_pages || !block_table || !kv_buf) return fail(PK_EINVAL, "pk_kv_reorganize: NULL pointer");
        if (!aligned16({k_pages, v_pages, kv_buf})) return fail(PK_EINVAL, "pk_kv_reorganize: tensors must be 16-byte aligned");
        if (page_size <= 0 || num_blocks <= 0) return fail(PK_EINVAL, "pk_kv_reorganize: page_size and num_blocks must be positive");
        int Hq = plan->tables.Hkv == Hkv && plan->tables.d == d && plan->tables.dtype == dtype ? plan->tables.Hq : Hkv;
        if (!shape_ok(Hq, Hkv, d, dtype, why)) return fail(PK_EINVAL, "pk_kv_reorganize: " + why);
        if (dtype == PK_BF16 && d != 64 && d != 128) return fail(PK_EUNSUPPORTED, "pk_kv_reorganize: bf16 path needs d in {64,128}");
        int32_t max_len = 0;
        for (int32_t L : plan->kv_lens) max_len = L > max_len ? L : max_len;
        if (static_cast<int64_t>(max_blocks_per_req) * page_size < max_len)
            return fail(PK_EINVAL, "pk_kv_reorganize: max_blocks_per_req too small for the longest request");
        int rc = ensure_bound(plan, Hq, Hkv, d, dtype, workspace, workspace_bytes, stream);
        if (rc != PK_OK) return rc;
        const DeviceTables& t = plan->tables;
        ReorgArgs a{};
        a.k_pages = k_pages; a.v_pages = v_pages; a.block_table = block_table;
        a.max_blocks = max_blocks_per_req; a.page_size = page_size; a.num_blocks = num_blocks;
        a.seg = tab(plan, t.reorg_seg); a.n_seg = t.n_reorg_seg; a.blk_first = tab(plan, t.reorg_blk_first);
        a.kv_buf = kv_buf; a.buf_tokens = plan->buf_tokens; a.Hkv = Hkv; a.d = d;
        const int e = dtype == PK_BF16 ? launch_reorg_bf16(a, stream) : launch_reorg_f32(a, stream);
        return e ? hip_fail("pk_kv_reorganize", e) : PK_OK;
    });
}

// args_out != nullptr: validate, bind and fill the kernel arguments, but launch nothing (the fused step)
static int prefill_common(pk_plan* plan, const void* q, const void* k, const void* v, void* out,
                          float scale, int Hq, int Hkv, int d, int dtype, int out_dtype,
                          void* workspace, size_t workspace_bytes, void* stream, bool padded,
                          PrefillArgs* args_out = nullptr, const char* who_override = nullptr) {
    const char* who = who_override ? who_override : padded ? "pk_padded_prefill_attn" : "pk_packed_prefill_attn";
    std::string why;
    if (!plan) return fail(PK_EINVAL, std::string(who) + ": plan is NULL");
    if (plan->n == 0) return PK_OK;
    if (!q || !k || !v || !out) return fail(PK_EINVAL, std::string(who) + ": NULL pointer");
    if (!aligned16({q, k, v, out})) return fail(PK_EINVAL, std::string(who) + ": tensors must be 16-byte aligned");
    if (!shape_ok(Hq, Hkv, d, dtype, why)) return fail(PK_EINVAL, std::string(who) + ": " + why);
    if (out_dtype != PK_BF16 && out_dtype != PK_F32) return fail(PK_EINVAL, std::string(who) + ": bad out_dtype");
    if (!(scale > 0.f) || !std::isfinite(scale)) return fail(PK_EINVAL, std::string(who) + ": scale must be finite and positive");
    if (dtype == PK_BF16 && d != 64 && d != 128) return fail(PK_EUNSUPPORTED, std::string(who) + ": bf16 path needs d in {64,128}");
    if (dtype == PK_F32 && d > 256) return fail(PK_EUNSUPPORTED, std::string(who) + ": fp32 path needs d <= 256");
    int rc = ensure_bound(plan, Hq, Hkv, d, dtype, workspace, workspace_bytes, stream);
    if (rc != PK_OK) return rc;
    if (padded && dtype == PK_BF16) {
        rc = ensure_padded(plan, stream);
        if (rc != PK_OK) return rc;
    }
    const DeviceTables& t = plan->tables;
    const DeviceTables::PrefillSched& s = padded ? t.padded : t.packed;
    const size_t base = padded ? t.padded_offset : 0;
    PrefillArgs a{};
    a.q = q; a.k = k; a.v = v; a.out = out;
    a.tiles = tab(plan, s.tiles, base); a.n_tiles = s.n_tiles;
    a.run_first = tab(plan, s.run_first, base); a.runs = tab(plan, s.runs, base);
    a.kvtiles = tab(plan, s.kvtiles, base);
    a.q_start = tab(plan, t.q_start); a.kv_start = tab(plan, t.kv_start); a.n = plan->n;
    int64_t tq = 0, tkv = 0;
    for (int32_t i = 0; i < plan->n; ++i) { tq += plan->q_lens[i]; tkv += plan->kv_lens[i]; }
    if (tkv > INT32_MAX) return fail(PK_EUNSUPPORTED, std::string(who) + ": more than 2^31 KV rows");
    a.total_q_rows = tq; a.total_kv_rows = tkv;
    a.Hq = Hq; a.Hkv = Hkv; a.d = d; a.scale = scale; a.out_f32 = out_dtype == PK_F32;
    a.xcd_swizzle = 1;             // both schedules: the r heads of a KV head share an XCD (and its L2)
    a.pipeline = plan->tune_prefill_pipeline;
    if (args_out) { *args_out = a; return PK_OK; }
    const int e = dtype == PK_BF16 ? launch_prefill_bf16(a, stream) : launch_prefill_f32(a, stream);
    return e ? hip_fail(who, e) : PK_OK;
}

extern "C" int pk_packed_prefill_attn(pk_plan* plan, const void* q, const void* k, const void* v,
                                      void* out, float scale, int Hq, int Hkv, int d,
                                      int dtype, int out_dtype,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_packed_prefill_attn", [&]() -> int {
        return prefill_common(plan, q, k, v, out, scale, Hq, Hkv, d, dtype, out_dtype, workspace, workspace_bytes, stream, false);
    });
}

extern "C" int pk_padded_prefill_attn(pk_plan* plan, const void* q, const void* k, const void* v,
                                      void* out, float scale, int Hq, int Hkv, int d,
                                      int dtype, int out_dtype,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_padded_prefill_attn", [&]() -> int {
        return prefill_common(plan, q, k, v, out, scale, Hq, Hkv, d, dtype, out_dtype, workspace, workspace_bytes, stream, true);
    });
}

namespace {

int decode_common(const char* who, pk_plan* plan, const void* q, const void* kv_buf,
                  void* out, float scale, int32_t grown, int Hq, int Hkv, int d,
                  int dtype, int out_dtype,
                  void* workspace, size_t workspace_bytes, void* stream, bool fixed_scratch = false,
                  DecodeArgs* args_out = nullptr) {
    const std::string w(who);
    std::string why;
    if (!plan) return fail(PK_EINVAL, w + ": plan is NULL");
    if (plan->n == 0) return PK_OK;
    if (!plan->decode_only) return fail(PK_EINVAL, w + ": the plan must have q_len == 1 for every request");
    if (!q || !kv_buf || !out) return fail(PK_EINVAL, w + ": NULL pointer");
    if (!aligned16({q, kv_buf, out})) return fail(PK_EINVAL, w + ": tensors must be 16-byte aligned");
    if (grown < 0 || grown > plan->headroom)
        return fail(PK_EINVAL, w + ": grown must be in [0, headroom] (regroup when the headroom is used up)");
    if (!shape_ok(Hq, Hkv, d, dtype, why)) return fail(PK_EINVAL, w + ": " + why);
    if (out_dtype != PK_BF16 && out_dtype != PK_F32) return fail(PK_EINVAL, w + ": bad out_dtype");
    if (!(scale > 0.f) || !std::isfinite(scale)) return fail(PK_EINVAL, w + ": scale must be finite and positive");
    if (dtype == PK_BF16 && (d != 64 && d != 128)) return fail(PK_EUNSUPPORTED, w + ": bf16 path needs d in {64,128}");
    if (dtype == PK_BF16 && Hq / Hkv > 32) return fail(PK_EUNSUPPORTED, w + ": bf16 path needs Hq/Hkv <= 32");
    if (dtype == PK_F32 && d > 256) return fail(PK_EUNSUPPORTED, w + ": fp32 path needs d <= 256");
    if (fixed_scratch) {                            // after the argument checks: the look-up touches the device
        const int e = static_scratch_address(&workspace);
        if (e != 0) return hip_fail("pk_packed_decode_attn_static (address of the fixed scratch)", e);
        workspace_bytes = PK_STATIC_SCRATCH_BYTES;
    }
    int rc = ensure_bound(plan, Hq, Hkv, d, dtype, workspace, workspace_bytes, stream, fixed_scratch);
    if (rc != PK_OK) return rc;
    const DeviceTables& t = plan->tables;
    DecodeArgs a{};
    a.q = q; a.kv_buf = kv_buf; a.out = out;
    a.items = tab(plan, t.dec_items); a.n_items = t.n_dec_items; a.n_wide = t.n_dec_wide;
    a.members = tab(plan, t.dec_members); a.member_slot = tab(plan, t.dec_member_slot);
    a.req_part_start = tab(plan, t.dec_req_part_start);
    a.req_seg = tab(plan, t.dec_req_seg);
    a.chain_start = tab(plan, t.dec_chain_start); a.chain = tab(plan, t.dec_chain);
    a.part_o = reinterpret_cast<float*>(static_cast<char*>(workspace) + t.partial_offset);
    a.part_lse = a.part_o + static_cast<size_t>(t.n_dec_parts) * Hq * d;
    a.buf_tokens = plan->buf_tokens; a.n = plan->n;
    a.Hq = Hq; a.Hkv = Hkv; a.d = d; a.scale = scale; a.out_f32 = out_dtype == PK_F32;
    a.grown = grown;
    a.max_parts = t.dec_max_parts;
    if (args_out) { *args_out = a; return PK_OK; }
    const int e = dtype == PK_BF16 ? launch_decode_bf16(a, stream) : launch_decode_f32(a, stream);
    return e ? hip_fail(who, e) : PK_OK;
}

}  // namespace

extern "C" int pk_packed_decode_attn(pk_plan* plan, const void* q, const void* kv_buf,
                                     void* out, float scale, int Hq, int Hkv, int d,
                                     int dtype, int out_dtype,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_packed_decode_attn", [&]() -> int {
        return decode_common("pk_packed_decode_attn", plan, q, kv_buf, out, scale, 0, Hq, Hkv, d, dtype, out_dtype,
                             workspace, workspace_bytes, stream);
    });
}

extern "C" int pk_packed_decode_attn_static(pk_plan* plan, const void* q, const void* kv_buf,
                                            void* out, float scale, int Hq, int Hkv, int d,
                                            int dtype, int out_dtype, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_packed_decode_attn_static", [&]() -> int {
        return decode_common("pk_packed_decode_attn_static", plan, q, kv_buf, out, scale, 0, Hq, Hkv, d, dtype, out_dtype,
                             nullptr, 0, stream, true);
    });
}

extern "C" int pk_packed_mixed_step(pk_plan* prefill_plan, const void* q, const void* k, const void* v, void* out,
                                    void* prefill_workspace, size_t prefill_workspace_bytes,
                                    pk_plan* decode_plan, const void* decode_q, const void* kv_buf, void* decode_out,
                                    void* decode_workspace, size_t decode_workspace_bytes,
                                    float scale, int Hq, int Hkv, int d, int dtype, int out_dtype, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_packed_mixed_step", [&]() -> int {
        const char* who = "pk_packed_mixed_step";
        if (!prefill_plan || !decode_plan) return fail(PK_EINVAL, "pk_packed_mixed_step: plan is NULL");
        if (dtype != PK_BF16 || (d != 128 && d != 64))
            return fail(PK_EUNSUPPORTED, "pk_packed_mixed_step: the fused launch is built for bf16 and d in {64,128} "
                                         "(call pk_packed_prefill_attn and pk_packed_decode_attn otherwise)");
        if (prefill_workspace && prefill_workspace == decode_workspace)
            return fail(PK_EINVAL, "pk_packed_mixed_step: the two plans need a workspace each");
        // either half may be empty: the other call does the whole step then
        if (prefill_plan->n == 0)
            return decode_common(who, decode_plan, decode_q, kv_buf, decode_out, scale, 0, Hq, Hkv, d, dtype, out_dtype,
                                 decode_workspace, decode_workspace_bytes, stream);
        if (decode_plan->n == 0)
            return prefill_common(prefill_plan, q, k, v, out, scale, Hq, Hkv, d, dtype, out_dtype, prefill_workspace,
                                  prefill_workspace_bytes, stream, false, nullptr, who);
        PrefillArgs pa{};
        DecodeArgs da{};
        int rc = prefill_common(prefill_plan, q, k, v, out, scale, Hq, Hkv, d, dtype, out_dtype, prefill_workspace,
                                prefill_workspace_bytes, stream, false, &pa, who);
        if (rc != PK_OK) return rc;
        rc = decode_common(who, decode_plan, decode_q, kv_buf, decode_out, scale, 0, Hq, Hkv, d, dtype, out_dtype,
                           decode_workspace, decode_workspace_bytes, stream, false, &da);
        if (rc != PK_OK) return rc;
        const int e = launch_mixed_step_bf16(pa, da, stream);
        return e ? hip_fail(who, e) : PK_OK;
    });
}

extern "C" int pk_packed_decode_attn_grown(pk_plan* plan, const void* q, const void* kv_buf,
                                           void* out, float scale, int32_t grown, int Hq, int Hkv, int d,
                                           int dtype, int out_dtype,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_packed_decode_attn_grown", [&]() -> int {
        return decode_common("pk_packed_decode_attn_grown", plan, q, kv_buf, out, scale, grown, Hq, Hkv, d, dtype,
                             out_dtype, workspace, workspace_bytes, stream);
    });
}

extern "C" int pk_kv_append(pk_plan* plan, const void* k_new, const void* v_new, void* kv_buf,
                            int32_t step, int Hkv, int d, int dtype,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_kv_append", [&]() -> int {
        std::string why;
        if (!plan) return fail(PK_EINVAL, "pk_kv_append: plan is NULL");
        if (plan->n == 0) return PK_OK;
        if (!plan->decode_only) return fail(PK_EINVAL, "pk_kv_append: the plan must have q_len == 1 for every request");
        if (!k_new || !v_new || !kv_buf) return fail(PK_EINVAL, "pk_kv_append: NULL pointer");
        if (!aligned16({k_new, v_new, kv_buf})) return fail(PK_EINVAL, "pk_kv_append: tensors must be 16-byte aligned");
        if (step < 0 || step >= plan->headroom)
            return fail(PK_EINVAL, "pk_kv_append: step must be in [0, headroom): no slot left, regroup");
        int Hq = plan->tables.Hkv == Hkv && plan->tables.d == d && plan->tables.dtype == dtype ? plan->tables.Hq : Hkv;
        if (!shape_ok(Hq, Hkv, d, dtype, why)) return fail(PK_EINVAL, "pk_kv_append: " + why);
        if (dtype == PK_BF16 && d != 64 && d != 128) return fail(PK_EUNSUPPORTED, "pk_kv_append: bf16 path needs d in {64,128}");
        int rc = ensure_bound(plan, Hq, Hkv, d, dtype, workspace, workspace_bytes, stream);
        if (rc != PK_OK) return rc;
        const DeviceTables& t = plan->tables;
        AppendArgs a{};
        a.k_new = k_new; a.v_new = v_new; a.kv_buf = kv_buf;
        a.req_seg = tab(plan, t.dec_req_seg);
        a.buf_tokens = plan->buf_tokens; a.n = plan->n; a.step = step; a.Hkv = Hkv; a.d = d;
        const int e = dtype == PK_BF16 ? launch_append_bf16(a, stream) : launch_append_f32(a, stream);
        return e ? hip_fail("pk_kv_append", e) : PK_OK;
    });
}

extern "C" int pk_regroup_due(const pk_plan* plan, int32_t steps, int32_t* flags, int64_t* drift) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_regroup_due", [&]() -> int {
        if (!plan || !flags) return fail(PK_EINVAL, "pk_regroup_due: NULL pointer");
        if (steps < 0) return fail(PK_EINVAL, "pk_regroup_due: steps must be non-negative");
        // [0]: all groups; [1]: without the groups opened for an item longer than C
        int64_t lo[2] = {0, 0}, hi[2] = {0, 0};
        bool first[2] = {true, true};
        for (const Group& g : plan->groups) {
            const int64_t load = g.load + static_cast<int64_t>(steps) * static_cast<int64_t>(g.members.size());
            for (int k = 0; k < 2; ++k) {
                if (k == 1 && g.load > plan->token_budget) continue;
                if (first[k] || load < lo[k]) lo[k] = load;
                if (first[k] || load > hi[k]) hi[k] = load;
                first[k] = false;
            }
        }
        const int64_t dl = first[0] ? 0 : hi[0] - lo[0], dl_in = first[1] ? 0 : hi[1] - lo[1];
        int32_t f = 0;
        if (2 * static_cast<int64_t>(steps) * dl >= plan->token_budget) f |= PK_REGROUP_DRIFT;
        if (steps >= plan->headroom) f |= PK_REGROUP_HEADROOM;
        if (2 * static_cast<int64_t>(steps) * dl_in >= plan->token_budget) f |= PK_REGROUP_DRIFT_WITHIN_BUDGET;
        *flags = f;
        if (drift) *drift = dl;
        return PK_OK;
    });
}

extern "C" int pk_padded_decode_attn(pk_plan* plan, const void* q,
                                     const void* k_pages, const void* v_pages,
                                     const int32_t* block_table, int32_t max_blocks_per_req,
                                     int32_t page_size, int64_t num_blocks,
                                     void* out, float scale, int Hq, int Hkv, int d,
                                     int dtype, int out_dtype,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_padded_decode_attn", [&]() -> int {
        std::string why;
        if (!plan) return fail(PK_EINVAL, "pk_padded_decode_attn: plan is NULL");
        if (plan->n == 0) return PK_OK;
        if (!plan->decode_only) return fail(PK_EINVAL, "pk_padded_decode_attn: the plan must have q_len == 1 for every request");
        if (!q || !k_pages || !v_pages || !block_table || !out) return fail(PK_EINVAL, "pk_padded_decode_attn: NULL pointer");
        if (!aligned16({q, k_pages, v_pages, out})) return fail(PK_EINVAL, "pk_padded_decode_attn: tensors must be 16-byte aligned");
        if (page_size <= 0 || num_blocks <= 0) return fail(PK_EINVAL, "pk_padded_decode_attn: page_size and num_blocks must be positive");
        if (!shape_ok(Hq, Hkv, d, dtype, why)) return fail(PK_EINVAL, "pk_padded_decode_attn: " + why);
        if (out_dtype != PK_BF16 && out_dtype != PK_F32) return fail(PK_EINVAL, "pk_padded_decode_attn: bad out_dtype");
        if (!(scale > 0.f) || !std::isfinite(scale)) return fail(PK_EINVAL, "pk_padded_decode_attn: scale must be finite and positive");
        if (dtype != PK_BF16) return fail(PK_EUNSUPPORTED, "pk_padded_decode_attn: bf16 only");
        if (d != 64 && d != 128) return fail(PK_EUNSUPPORTED, "pk_padded_decode_attn: needs d in {64,128}");
        if (Hq / Hkv > 16) return fail(PK_EUNSUPPORTED, "pk_padded_decode_attn: needs Hq/Hkv <= 16");
        int32_t max_len = 0;
        for (int32_t L : plan->kv_lens) max_len = L > max_len ? L : max_len;
        if (static_cast<int64_t>(max_blocks_per_req) * page_size < max_len)
            return fail(PK_EINVAL, "pk_padded_decode_attn: max_blocks_per_req too small for the longest request");
        int rc = ensure_bound(plan, Hq, Hkv, d, dtype, workspace, workspace_bytes, stream);
        if (rc != PK_OK) return rc;
        const DeviceTables& t = plan->tables;
        PagedDecodeArgs a{};
        a.q = q; a.k_pages = k_pages; a.v_pages = v_pages; a.out = out;
        a.block_table = block_table; a.max_blocks = max_blocks_per_req; a.page_size = page_size; a.num_blocks = num_blocks;
        a.kv_start = tab(plan, t.kv_start);
        a.n = plan->n; a.n_splits = t.pad_n_splits; a.split_tokens = t.pad_split_tokens;
        a.part_o = reinterpret_cast<float*>(static_cast<char*>(workspace) + t.partial_offset);
        a.part_lse = a.part_o + static_cast<size_t>(plan->n) * t.pad_n_splits * Hq * d;
        a.Hq = Hq; a.Hkv = Hkv; a.d = d; a.scale = scale; a.out_f32 = out_dtype == PK_F32;
        const int e = launch_padded_decode_bf16(a, stream);
        return e ? hip_fail("pk_padded_decode_attn", e) : PK_OK;
    });
}

extern "C" int pk_plan_tune(pk_plan* plan, int knob, int64_t value) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_plan_tune", [&]() -> int {
        if (!plan) return fail(PK_EINVAL, "pk_plan_tune: plan is NULL");
        if (knob == PK_TUNE_PREFILL_PIPELINE) {
            if (value != 0 && value != 1) return fail(PK_EINVAL, "pk_plan_tune: prefill pipeline must be 0 (direct to LDS) or 1 (staged through registers)");
            plan->tune_prefill_pipeline = static_cast<int32_t>(value);
            return PK_OK;                              // (read at every prefill call; the tables do not depend on it)
        }
        if (knob != PK_TUNE_DECODE_SPLIT) return fail(PK_EINVAL, "pk_plan_tune: unknown knob");
        if (value < 0 || value > (1 << 20)) return fail(PK_EINVAL, "pk_plan_tune: decode split must be in [0, 2^20] tokens");
        plan->tune_decode_split = static_cast<int32_t>(value);
        plan->tables = DeviceTables();                 // the next size query or bind builds the tables again
        plan->bound_ws = nullptr;
        return PK_OK;
    });
}

extern "C" int64_t pk_plan_stat(const pk_plan* plan, int what) {
    return pk::guarded<int64_t>(int64_t{0}, int64_t{0}, "pk_plan_stat", [&]() -> int64_t {
        if (!plan) return 0;
        switch (what) {
            case 0: return plan->unmasked_pairs;
            case 1: return plan->tables.packed.issued_pairs;
            case 2:
                if (!plan->tables.padded_built && plan->tables.dtype >= 0)
                    build_prefill_padded(*plan, plan->tables);
                return plan->tables.padded.issued_pairs;
            case 3: return plan->tables.n_dec_items;
            case 4: return plan->tables.n_dec_parts;
            case 5: return plan->tables.dec_split_tokens;
            case 6: return plan->tables.packed.n_tiles;
            case 7:
                if (!plan->tables.padded_built && plan->tables.dtype >= 0)
                    build_prefill_padded(*plan, plan->tables);
                return plan->tables.padded.n_tiles;
            default: return 0;
        }
    });
}
