// Test infrastructure: drives the host side of the library (planner, prefix tree, device-table
// builder, argument validation) under AddressSanitizer / UndefinedBehaviorSanitizer.  Reads cases
// from a text file written by the test (inputs + the words the CPU oracle expects), calls the C ABI
// and compares.  Built with g++, no device code: the kernel launchers are stubs that are never
// reached (every call here stops at validation or is host only).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <fstream>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "../../include/packinfer.h"
#include "../../paper_2602_06072_amd/csrc/kernels.h"

namespace pk {   // launch stubs: nothing in this driver gets as far as a launch
int launch_reorg_bf16(const ReorgArgs&, void*) { std::abort(); }
int launch_reorg_f32(const ReorgArgs&, void*) { std::abort(); }
int launch_append_bf16(const AppendArgs&, void*) { std::abort(); }
int launch_append_f32(const AppendArgs&, void*) { std::abort(); }
int launch_decode_bf16(const DecodeArgs&, void*) { std::abort(); }
int launch_decode_f32(const DecodeArgs&, void*) { std::abort(); }
int launch_decode_merge_bf16(const DecodeArgs&, void*) { std::abort(); }
int static_scratch_address(void**) { return 1; }
int launch_prefill_bf16(const PrefillArgs&, void*) { std::abort(); }
int launch_prefill_f32(const PrefillArgs&, void*) { std::abort(); }
int launch_mixed_step_bf16(const PrefillArgs&, const DecodeArgs&, void*) { std::abort(); }
int launch_padded_decode_bf16(const PagedDecodeArgs&, void*) { std::abort(); }
}  // namespace pk

static std::vector<int32_t> read_vec(std::istringstream& in) {
    long n; in >> n;
    std::vector<int32_t> v(static_cast<size_t>(n < 0 ? 0 : n));
    for (auto& x : v) in >> x;
    return v;
}
static int failures = 0;
#define CHECK(COND, WHAT) do { if (!(COND)) { ++failures; std::fprintf(stderr, "line %ld: %s\n", lineno, WHAT); } } while (0)

int main(int argc, char** argv) {
    if (argc < 2) return 2;
    std::ifstream f(argv[1]);
    std::string line;
    long lineno = 0, cases = 0;
    while (std::getline(f, line)) {
        ++lineno;
        std::istringstream in(line);
        std::string kind; in >> kind;
        if (kind == "plan") {                  // plan C hr has_q has_pfx kv q pid plen expect_rc words
            long long C; int hr, has_q, has_pfx; in >> C >> hr >> has_q >> has_pfx;
            auto kv = read_vec(in), q = read_vec(in), pid = read_vec(in), plen = read_vec(in);
            int expect_rc; in >> expect_rc;
            auto want = read_vec(in);
            pk_plan* plan = nullptr;
            const int rc = pk_pack_plan(kv.data(), has_q ? q.data() : nullptr, has_pfx ? pid.data() : nullptr,
                                        has_pfx ? plen.data() : nullptr, static_cast<int32_t>(kv.size()), C, hr, &plan);
            CHECK(rc == expect_rc, "pk_pack_plan return code");
            if (rc == PK_OK) {
                std::vector<int32_t> got(static_cast<size_t>(pk_plan_serialized_words(plan)));
                CHECK(pk_plan_serialize(plan, got.data(), static_cast<int64_t>(got.size())) == static_cast<int64_t>(got.size()), "serialize");
                CHECK(got == want, "plan words differ from the oracle's");
                CHECK(pk_plan_serialize(plan, got.data(), static_cast<int64_t>(got.size()) - 1) == PK_EINVAL || got.empty(), "short buffer");
                // device tables for a prefill shape, a decode shape and the fp32 layout
                for (int d : {64, 128}) {
                    const size_t ws = pk_workspace_bytes(plan, 8, 2, d, PK_BF16);
                    CHECK(ws % 256 == 0, "workspace size");
                    CHECK(pk_plan_stat(plan, 1) >= pk_plan_stat(plan, 0), "issued >= unmasked pairs");
                    CHECK(pk_plan_stat(plan, 2) >= pk_plan_stat(plan, 0), "padded issued >= unmasked pairs");
                    (void)pk_plan_stat(plan, 3); (void)pk_plan_stat(plan, 4); (void)pk_plan_stat(plan, 5);
                    (void)pk_plan_stat(plan, 6); (void)pk_plan_stat(plan, 7);
                    CHECK(pk_kv_buf_bytes(plan, 2, d, PK_BF16) == static_cast<size_t>(pk_plan_buf_tokens(plan)) * 2 * d * 4, "kv_buf bytes");
                }
                (void)pk_workspace_bytes(plan, 32, 1, 128, PK_BF16);
                (void)pk_workspace_bytes(plan, 3, 1, 96, PK_F32);
                CHECK(pk_plan_tune(plan, PK_TUNE_DECODE_SPLIT, 64) == PK_OK, "tune");
                (void)pk_workspace_bytes(plan, 8, 2, 128, PK_BF16);
                int32_t flags = 0; int64_t drift = 0;
                CHECK(pk_regroup_due(plan, 3, &flags, &drift) == PK_OK, "regroup_due");
                // compute entry points stop at validation (NULL tensors): no launch, no device
                CHECK(pk_packed_prefill_attn(plan, nullptr, nullptr, nullptr, nullptr, 1.f, 8, 2, 128, PK_BF16, PK_F32, nullptr, 0, nullptr) == PK_EINVAL || kv.empty(), "prefill validation");
                CHECK(pk_packed_decode_attn(plan, nullptr, nullptr, nullptr, 1.f, 8, 2, 128, PK_BF16, PK_F32, nullptr, 0, nullptr) == PK_EINVAL || kv.empty(), "decode validation");
                CHECK(pk_packed_mixed_step(plan, nullptr, nullptr, nullptr, nullptr, nullptr, 0, plan, nullptr, nullptr, nullptr, nullptr, 0,
                                           1.f, 8, 2, 128, PK_BF16, PK_F32, nullptr) != PK_OK || kv.empty(), "mixed step validation");
                pk_plan_destroy(plan);
            }
            ++cases;
        } else if (kind == "tree") {           // tree min_prefix C hr lens tokens | parent len req_node saved words
            int mp, hr; long long C; in >> mp >> C >> hr;
            auto lens = read_vec(in), toks = read_vec(in), par_w = read_vec(in), len_w = read_vec(in), rn_w = read_vec(in);
            long long saved_w; in >> saved_w;
            auto want = read_vec(in);
            const int32_t n = static_cast<int32_t>(lens.size());
            std::vector<int32_t> par(static_cast<size_t>(n) + 1), nl(static_cast<size_t>(n) + 1), rn(static_cast<size_t>(n) + 1);
            int32_t nn = 0; int64_t saved = 0;
            CHECK(pk_trie_tree(toks.data(), lens.data(), n, mp, par.data(), nl.data(), &nn, rn.data(), &saved) == PK_OK, "pk_trie_tree");
            par.resize(static_cast<size_t>(nn)); nl.resize(static_cast<size_t>(nn)); rn.resize(static_cast<size_t>(n));
            CHECK(par == par_w && nl == len_w && rn == rn_w && saved == saved_w, "prefix tree differs from the oracle's");
            std::vector<int32_t> ids(static_cast<size_t>(n) + 1), pl(static_cast<size_t>(n) + 1);
            CHECK(pk_trie_partition(toks.data(), lens.data(), n, mp, ids.data(), pl.data(), &saved) == PK_OK, "pk_trie_partition");
            pk_plan* plan = nullptr;
            std::vector<int32_t> ones(static_cast<size_t>(n), 1);
            CHECK(pk_pack_plan_tree(lens.data(), ones.data(), n, par.data(), nl.data(), nn, rn.data(), C, hr, &plan) == PK_OK, "pk_pack_plan_tree");
            if (plan) {
                std::vector<int32_t> got(static_cast<size_t>(pk_plan_serialized_words(plan)));
                (void)pk_plan_serialize(plan, got.data(), static_cast<int64_t>(got.size()));
                CHECK(got == want, "tree plan words differ from the oracle's");
                (void)pk_workspace_bytes(plan, 8, 2, 128, PK_BF16);
                (void)pk_workspace_bytes(plan, 8, 2, 64, PK_F32);
                pk_plan_destroy(plan);
            }
            ++cases;
        }
    }
    // NULL handling
    long dummy = 0; (void)dummy;
    if (pk_pack_plan(nullptr, nullptr, nullptr, nullptr, 0, 8, 0, nullptr) != PK_EINVAL) ++failures;
    if (pk_plan_num_groups(nullptr) != 0 || pk_plan_tune(nullptr, 0, 0) != PK_EINVAL) ++failures;
    pk_plan_destroy(nullptr);
    std::printf("%ld cases, %d failures\n", cases, failures);
    return failures ? 1 : 0;
}
