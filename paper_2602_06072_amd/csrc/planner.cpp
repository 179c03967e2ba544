// Packing planner: Alg. 1 Part 1 (greedy length-balanced grouping under the
// token term of the feasibility test, Eq. 2) and the bookkeeping of Part 2
// (prefix-first layout, offset tables O_g).  Host only, integers only,
// deterministic: the same inputs always give the same serialised words.
#include <algorithm>
#include <map>
#include <memory>
#include <new>
#include <numeric>
#include <queue>
#include <utility>

#include "plan.h"

namespace pk {

static thread_local std::string g_error;
void set_error(const std::string& msg) { g_error = msg; }

namespace {

struct TNode {                      // shared segment of an item's prefix tree, in pre-order
    int32_t id, len, parent;        // parent: index in Item::nodes or -1
    std::vector<int32_t> direct;    // requests that continue right after this segment, ascending
};

struct Item {                       // atomic unit of assignment: a request, a (sub-)family or a prefix tree
    int64_t length;                 // unique tokens: shared segments once + the suffixes (Sec. 3.2, Eq. 5)
    int32_t first;                  // lowest member index (tie-break)
    std::vector<TNode> nodes;       // empty: a single request
    int32_t single;                 // that request
};

inline void push64(std::vector<int32_t>& w, int64_t x) {
    w.push_back(static_cast<int32_t>(static_cast<uint32_t>(x & 0xFFFFFFFFll)));
    w.push_back(static_cast<int32_t>(static_cast<uint32_t>((x >> 32) & 0xFFFFFFFFll)));
}

int fail(const char* msg) {
    set_error(msg);
    return PK_EINVAL;
}

}  // namespace
}  // namespace pk

using namespace pk;

namespace {

// Common part of the two planners: Part 1 (greedy least-loaded assignment of the items) and the
// layout bookkeeping of Part 2 (parent segment first, then the suffixes of the requests attached
// to it, then its child segments), then the canonical words.
int finish_plan(std::unique_ptr<pk_plan> plan, std::vector<Item>& items, const int32_t* kv_lens, pk_plan** out) {
    const int64_t C = plan->token_budget;
    const int32_t headroom = plan->headroom;
    int64_t l_total = 0;
    for (const Item& it : items) l_total += it.length;
    // G <- ceil(L_total / C).  Groups beyond the number of items would stay empty (every item that
    // fits takes the lowest-numbered empty group, an item longer than C opens its own) and empty
    // groups are dropped, so the count is capped there: a tiny C cannot make the tables huge.
    const int64_t G0 = std::min<int64_t>((l_total + C - 1) / C, static_cast<int64_t>(items.size()));
    std::vector<int64_t> loads(static_cast<size_t>(G0), 0);
    std::vector<std::vector<int32_t>> assigned(static_cast<size_t>(G0));   // item indices
    std::vector<int32_t> order(items.size());
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (items[a].length != items[b].length) return items[a].length > items[b].length;
        return items[a].first < items[b].first;
    });
    // arg min over the group loads (lowest index on ties) through a heap of (load, index): only the
    // chosen group's load changes, so a request costs O(log G) instead of a scan of all groups
    using Slot = std::pair<int64_t, size_t>;
    std::priority_queue<Slot, std::vector<Slot>, std::greater<Slot>> least;
    for (size_t g = 0; g < loads.size(); ++g) least.push({0, g});
    for (int32_t idx : order) {
        const Item& it = items[idx];
        if (!least.empty() && least.top().first + it.length <= C) {
            const size_t g = least.top().second;
            least.pop();
            loads[g] += it.length;
            assigned[g].push_back(idx);
            least.push({loads[g], g});
        } else {                                                  // else-branch: open a new group
            loads.push_back(it.length);
            assigned.push_back({idx});
            least.push({it.length, loads.size() - 1});
        }
    }

    int64_t base = 0;
    for (size_t g = 0; g < loads.size(); ++g) {
        if (assigned[g].empty()) continue;
        Group grp;
        grp.load = loads[g];
        int64_t delta = 0;
        for (int32_t idx : assigned[g]) {
            const Item& it = items[idx];
            if (it.nodes.empty()) {
                Member m{it.single, static_cast<int32_t>(delta), 0, static_cast<int32_t>(delta), kv_lens[it.single]};
                grp.members.push_back(m);
                delta += kv_lens[it.single] + headroom;
                continue;
            }
            const size_t n0 = grp.nodes.size();
            for (const TNode& tn : it.nodes) {                    // pre-order = parent first
                Node nd;
                nd.id = tn.id; nd.off = static_cast<int32_t>(delta); nd.len = tn.len;
                nd.parent = tn.parent < 0 ? -1 : static_cast<int32_t>(n0) + tn.parent;
                nd.start = nd.parent < 0 ? 0 : grp.nodes[static_cast<size_t>(nd.parent)].start +
                                                   grp.nodes[static_cast<size_t>(nd.parent)].len;
                delta += tn.len;
                const int32_t self = static_cast<int32_t>(grp.nodes.size());
                const int32_t shared = nd.start + nd.len;
                grp.nodes.push_back(nd);
                for (int32_t i : tn.direct) {
                    Member m{i, nd.off, nd.len, static_cast<int32_t>(delta), kv_lens[i] - shared};
                    m.node = self; m.shared = shared;
                    grp.members.push_back(m);
                    delta += m.lq + headroom;
                    for (int32_t k = self; k >= 0; k = grp.nodes[static_cast<size_t>(k)].parent)
                        grp.nodes[static_cast<size_t>(k)].reqs.push_back(i);
                }
            }
            for (size_t k = n0; k < grp.nodes.size(); ++k) std::sort(grp.nodes[k].reqs.begin(), grp.nodes[k].reqs.end());
        }
        if (delta > INT32_MAX) { return fail("pk_pack_plan: group buffer exceeds 2^31 tokens"); }
        grp.buf_tokens = delta;
        grp.buf_base = base;
        base = (base + delta + PK_GROUP_ALIGN - 1) / PK_GROUP_ALIGN * PK_GROUP_ALIGN;
        plan->unique_tokens += grp.load;
        plan->groups.push_back(std::move(grp));
    }
    plan->buf_tokens = base;
    if (base > INT32_MAX) { return fail("pk_pack_plan: buffer exceeds 2^31 tokens"); }

    // ---- canonical serialisation ---------------------------------------------
    std::vector<int32_t>& w = plan->words;
    w.push_back(0x504B504C);
    w.push_back(plan->tree ? 2 : 1);
    w.push_back(plan->n);
    w.push_back(static_cast<int32_t>(plan->groups.size()));
    push64(w, C);
    w.push_back(headroom);
    w.push_back(PK_GROUP_ALIGN);
    push64(w, plan->buf_tokens);
    for (const Group& grp : plan->groups) {
        push64(w, grp.load);
        push64(w, grp.buf_tokens);
        push64(w, grp.buf_base);
        if (plan->tree) {
            w.push_back(static_cast<int32_t>(grp.nodes.size()));
            w.push_back(static_cast<int32_t>(grp.members.size()));
            for (const Node& nd : grp.nodes) {
                w.push_back(nd.id); w.push_back(nd.off); w.push_back(nd.len); w.push_back(nd.parent);
            }
            for (const Member& m : grp.members) {
                w.push_back(m.req); w.push_back(m.node); w.push_back(m.suffix_off); w.push_back(m.lq);
            }
        } else {
            w.push_back(static_cast<int32_t>(grp.members.size()));
            for (const Member& m : grp.members) {
                w.push_back(m.req); w.push_back(m.prefix_off); w.push_back(m.lp);
                w.push_back(m.suffix_off); w.push_back(m.lq);
            }
        }
    }
    *out = plan.release();
    return PK_OK;
}

std::unique_ptr<pk_plan> new_plan(const int32_t* kv_lens, const int32_t* q_lens, int32_t n, int64_t token_budget, int32_t headroom) {
    std::unique_ptr<pk_plan> plan(new pk_plan());
    plan->n = n;
    plan->token_budget = token_budget;
    plan->headroom = headroom;
    plan->kv_lens.assign(kv_lens, kv_lens + n);
    if (q_lens) plan->q_lens.assign(q_lens, q_lens + n); else plan->q_lens = plan->kv_lens;
    plan->prefix_lens.assign(n, 0);
    plan->decode_only = n > 0;
    for (int32_t i = 0; i < n; ++i) {
        if (plan->q_lens[i] != 1) plan->decode_only = false;
        const int64_t lq = plan->q_lens[i], ctx = plan->kv_lens[i] - lq;
        plan->unmasked_pairs += lq * ctx + lq * (lq + 1) / 2;
    }
    return plan;
}

}  // namespace

extern "C" int pk_pack_plan(const int32_t* kv_lens, const int32_t* q_lens,
                            const int32_t* prefix_ids, const int32_t* prefix_lens,
                            int32_t n, int64_t token_budget, int32_t headroom, pk_plan** out) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_pack_plan", [&]() -> int {
        if (!out) return fail("pk_pack_plan: out is NULL");
        *out = nullptr;
        if (n < 0) return fail("pk_pack_plan: n < 0");
        if (n > 0 && !kv_lens) return fail("pk_pack_plan: kv_lens is NULL");
        if (token_budget <= 0) return fail("pk_pack_plan: token_budget must be positive");
        if (headroom < 0) return fail("pk_pack_plan: headroom must be non-negative");
        if ((prefix_ids == nullptr) != (prefix_lens == nullptr))
            return fail("pk_pack_plan: prefix_ids and prefix_lens must be given together");

        std::map<int32_t, int32_t> fam_len;
        for (int32_t i = 0; i < n; ++i) {
            if (kv_lens[i] <= 0) return fail("pk_pack_plan: kv_len must be positive");
            if (q_lens && (q_lens[i] <= 0 || q_lens[i] > kv_lens[i]))
                return fail("pk_pack_plan: q_len must be in [1, kv_len]");
            if (prefix_ids) {
                const int32_t pl = prefix_lens[i];
                if (pl < 0 || pl > kv_lens[i]) return fail("pk_pack_plan: prefix_len must be in [0, kv_len]");
                if (prefix_ids[i] >= 0 && pl > 0) {
                    auto it = fam_len.emplace(prefix_ids[i], pl).first;
                    if (it->second != pl) return fail("pk_pack_plan: prefix_len differs inside a family");
                }
            }
        }
        std::unique_ptr<pk_plan> plan = new_plan(kv_lens, q_lens, n, token_budget, headroom);

        // ---- items: requests, and families cut into the fewest consecutive sub-families that fit ----
        const int64_t C = token_budget;
        std::vector<Item> items;
        std::map<int32_t, std::vector<int32_t>> families;   // ordered by id; order is irrelevant after the sort
        for (int32_t i = 0; i < n; ++i) {
            const bool in_family = prefix_ids && prefix_ids[i] >= 0 && prefix_lens[i] > 0;
            if (in_family) {
                families[prefix_ids[i]].push_back(i);
                plan->prefix_lens[i] = prefix_lens[i];
            } else {
                items.push_back(Item{kv_lens[i], i, {}, i});
            }
        }
        int32_t running = 0;
        for (auto& kv : families) {
            const std::vector<int32_t>& mem = kv.second;
            const int32_t lp = prefix_lens[mem[0]];
            Item cur{lp, mem[0], {TNode{running++, lp, -1, {}}}, -1};
            for (int32_t i : mem) {
                const int64_t lq = kv_lens[i] - lp;
                if (!cur.nodes[0].direct.empty() && cur.length + lq > C) {
                    items.push_back(cur);
                    cur = Item{lp, i, {TNode{running++, lp, -1, {}}}, -1};
                }
                if (cur.nodes[0].direct.empty()) cur.first = i;
                cur.nodes[0].direct.push_back(i);
                cur.length += lq;
            }
            items.push_back(cur);
        }
        return finish_plan(std::move(plan), items, kv_lens, out);
    });
}

extern "C" int pk_pack_plan_tree(const int32_t* kv_lens, const int32_t* q_lens, int32_t n,
                                 const int32_t* node_parent, const int32_t* node_len, int32_t n_nodes,
                                 const int32_t* req_node, int64_t token_budget, int32_t headroom,
                                 pk_plan** out) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_pack_plan_tree", [&]() -> int {
        if (!out) return fail("pk_pack_plan_tree: out is NULL");
        *out = nullptr;
        if (n < 0 || n_nodes < 0) return fail("pk_pack_plan_tree: negative count");
        if (n > 0 && (!kv_lens || !req_node)) return fail("pk_pack_plan_tree: NULL pointer");
        if (n_nodes > 0 && (!node_parent || !node_len)) return fail("pk_pack_plan_tree: NULL pointer");
        if (token_budget <= 0) return fail("pk_pack_plan_tree: token_budget must be positive");
        if (headroom < 0) return fail("pk_pack_plan_tree: headroom must be non-negative");
        std::vector<int64_t> depth(static_cast<size_t>(n_nodes), 0);
        for (int32_t k = 0; k < n_nodes; ++k) {
            if (node_len[k] <= 0) return fail("pk_pack_plan_tree: node_len must be positive");
            if (node_parent[k] < -1 || node_parent[k] >= k) return fail("pk_pack_plan_tree: node_parent[k] must be in [-1, k)");
            depth[k] = node_len[k] + (node_parent[k] >= 0 ? depth[node_parent[k]] : 0);
        }
        std::vector<std::vector<int32_t>> direct(static_cast<size_t>(n_nodes)), kids(static_cast<size_t>(n_nodes));
        std::vector<int32_t> below(static_cast<size_t>(n_nodes), 0);
        for (int32_t i = 0; i < n; ++i) {
            if (kv_lens[i] <= 0) return fail("pk_pack_plan_tree: kv_len must be positive");
            if (q_lens && (q_lens[i] <= 0 || q_lens[i] > kv_lens[i])) return fail("pk_pack_plan_tree: q_len must be in [1, kv_len]");
            const int32_t k = req_node[i];
            if (k < -1 || k >= n_nodes) return fail("pk_pack_plan_tree: req_node out of range");
            if (k >= 0 && depth[k] > kv_lens[i]) return fail("pk_pack_plan_tree: a request is shorter than the segments above it");
            if (k >= 0) direct[k].push_back(i);
            for (int32_t j = k; j >= 0; j = node_parent[j]) ++below[j];
        }
        for (int32_t k = 0; k < n_nodes; ++k) {
            if (below[k] == 0) return fail("pk_pack_plan_tree: a node without requests below it");
            if (node_parent[k] >= 0) kids[node_parent[k]].push_back(k);
        }
        std::unique_ptr<pk_plan> plan = new_plan(kv_lens, q_lens, n, token_budget, headroom);
        plan->tree = true;
        for (int32_t i = 0; i < n; ++i) plan->prefix_lens[i] = req_node[i] >= 0 ? static_cast<int32_t>(depth[req_node[i]]) : 0;

        std::vector<Item> items;
        for (int32_t i = 0; i < n; ++i)
            if (req_node[i] < 0) items.push_back(Item{kv_lens[i], i, {}, i});
        for (int32_t root = 0; root < n_nodes; ++root) {
            if (node_parent[root] >= 0) continue;
            Item it{0, INT32_MAX, {}, -1};
            // pre-order walk with an explicit stack (children in ascending node number)
            std::vector<std::pair<int32_t, int32_t>> stack{{root, -1}};
            while (!stack.empty()) {
                const int32_t k = stack.back().first, par = stack.back().second;
                stack.pop_back();
                const int32_t self = static_cast<int32_t>(it.nodes.size());
                it.nodes.push_back(TNode{k, node_len[k], par, direct[k]});
                it.length += node_len[k];
                for (int32_t i : direct[k]) { it.length += kv_lens[i] - depth[k]; it.first = std::min(it.first, i); }
                for (auto c = kids[k].rbegin(); c != kids[k].rend(); ++c) stack.push_back({*c, self});
            }
            items.push_back(std::move(it));
        }
        return finish_plan(std::move(plan), items, kv_lens, out);
    });
}

extern "C" void pk_plan_destroy(pk_plan* plan) { delete plan; }

extern "C" int32_t pk_plan_num_requests(const pk_plan* plan) { return plan ? plan->n : 0; }
extern "C" int32_t pk_plan_num_groups(const pk_plan* plan) {
    return plan ? static_cast<int32_t>(plan->groups.size()) : 0;
}
extern "C" int64_t pk_plan_buf_tokens(const pk_plan* plan) { return plan ? plan->buf_tokens : 0; }
extern "C" int64_t pk_plan_unique_tokens(const pk_plan* plan) { return plan ? plan->unique_tokens : 0; }

extern "C" int64_t pk_plan_serialized_words(const pk_plan* plan) {
    return plan ? static_cast<int64_t>(plan->words.size()) : 0;
}

extern "C" int64_t pk_plan_serialize(const pk_plan* plan, int32_t* out, int64_t cap) {
    return pk::guarded<int64_t>(int64_t{PK_ENOMEM}, int64_t{PK_EINVAL}, "pk_plan_serialize", [&]() -> int64_t {
        if (!plan || !out) return fail("pk_plan_serialize: NULL argument");
        const int64_t nw = static_cast<int64_t>(plan->words.size());
        if (cap < nw) return fail("pk_plan_serialize: capacity too small");
        std::copy(plan->words.begin(), plan->words.end(), out);
        return nw;
    });
}

extern "C" const char* pk_last_error(void) { return pk::g_error.c_str(); }
