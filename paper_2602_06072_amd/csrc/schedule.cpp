// Device tables of a plan: the re-layout segment list, the split-KV decode
// work items and the prefill tile schedules (packed and padded).  Host only.
//
// Packed prefill (Sec. 3.1, execution domain = union of valid query-key
// regions): query tiles are cut from the packed token stream of each group
// and may span requests; a tile lists only the key tiles that hold at least
// one unmasked pair for it, and each key tile says per wave (32 query rows)
// whether that wave skips it, computes it with the mask, or computes it
// without any mask.
#include <algorithm>
#include <numeric>

#include "plan.h"

namespace pk {

namespace {

struct Builder {
    std::vector<int32_t>& host;
    explicit Builder(std::vector<int32_t>& h) : host(h) {}
    TableRef add(const std::vector<int32_t>& v) {
        TableRef r;
        host.resize((host.size() + 63) / 64 * 64, 0);
        r.offset = host.size() * sizeof(int32_t);
        r.count = v.size();
        host.insert(host.end(), v.begin(), v.end());
        return r;
    }
};

// ---- re-layout -------------------------------------------------------------
void build_reorg(const pk_plan& plan, Builder& b, DeviceTables& t) {
    struct Seg { int64_t dst0; int32_t ntok, req, src0; };
    std::vector<Seg> segs;
    for (const Group& g : plan.groups) {
        for (const Node& nd : g.nodes)                            // a shared segment once, via its lowest request
            segs.push_back({g.buf_base + nd.off, nd.len, nd.reqs[0], nd.start});
        for (const Member& m : g.members)
            if (m.lq > 0) segs.push_back({g.buf_base + m.suffix_off, m.lq, m.req, m.shared});
    }
    std::sort(segs.begin(), segs.end(), [](const Seg& x, const Seg& y) { return x.dst0 < y.dst0; });
    std::vector<int32_t> flat;
    flat.reserve(segs.size() * 4);
    for (const Seg& s : segs) {
        flat.push_back(static_cast<int32_t>(s.dst0)); flat.push_back(s.ntok);
        flat.push_back(s.req); flat.push_back(s.src0);
    }
    const int64_t nb = plan.buf_tokens / kDecodeBlock;
    std::vector<int32_t> first(static_cast<size_t>(nb), 0);
    size_t cur = 0;
    for (int64_t blk = 0; blk < nb; ++blk) {
        const int64_t t0 = blk * kDecodeBlock;
        while (cur < segs.size() && segs[cur].dst0 + segs[cur].ntok <= t0) ++cur;
        first[static_cast<size_t>(blk)] = static_cast<int32_t>(cur);
    }
    t.n_reorg_seg = static_cast<int32_t>(segs.size());
    t.reorg_seg = b.add(flat);
    t.reorg_blk_first = b.add(first);
}

// ---- decode ----------------------------------------------------------------
void build_decode(const pk_plan& plan, int Hq, int Hkv, int num_cus, Builder& b, DeviceTables& t) {
    const int r = Hq / Hkv;
    const int max_members = std::max(1, kDecodeMaxRows / r);
    // split length: about 1500 waves (work items x KV heads) keep enough loads in flight to fill
    // the memory system (each has 64 KiB outstanding); beyond that, longer items mean fewer
    // partial results to write and merge
    int64_t split = (plan.unique_tokens * Hkv / 1536 + kDecodeBlock - 1) / kDecodeBlock * kDecodeBlock;
    split = std::min<int64_t>(std::max<int64_t>(split, 128), 2048);
    {
        // All waves of the launch should be resident at once (a second, partly filled round of
        // waves is a tail as long as a whole item): 16 waves per CU fit, 8 of the kernel that
        // also handles 32-row items.  Short suffixes cost an item each whatever the split, so the
        // items are counted for the candidate and the split is raised until they fit.
        bool wide = false;
        for (const Group& g : plan.groups)
            for (const Node& nd : g.nodes) wide = wide || static_cast<int>(std::min<size_t>(nd.reqs.size(), max_members)) * r > 16;
        const int64_t capacity = static_cast<int64_t>(wide ? 8 : 16) * num_cus * 9 / 10;
        auto pieces_of = [&](int64_t len, int64_t sp) { return len <= 0 ? int64_t{0} : ((len + kDecodeBlock - 1) / kDecodeBlock * kDecodeBlock + sp - 1) / sp; };
        auto count_items = [&](int64_t sp) {
            int64_t c = 0;
            for (const Group& g : plan.groups) {
                for (const Node& nd : g.nodes)
                    c += pieces_of(nd.len, sp) * static_cast<int64_t>((nd.reqs.size() + max_members - 1) / max_members);
                for (const Member& m : g.members) c += std::max<int64_t>(pieces_of(m.lq, sp), plan.headroom > 0 ? 1 : 0);
            }
            return c;
        };
        while (split < 2048 && count_items(split) * Hkv > capacity)
            split = std::min<int64_t>(2048, (split * 5 / 4 + kDecodeBlock - 1) / kDecodeBlock * kDecodeBlock);
    }
    if (plan.tune_decode_split > 0) split = plan.tune_decode_split;     // pk_plan_tune (profiling sweeps)
    split = (split + kDecodeBlock - 1) / kDecodeBlock * kDecodeBlock;
    t.dec_split_tokens = static_cast<int32_t>(split);

    struct Item { int64_t a, e; std::vector<int32_t> reqs; bool grows = false; };
    std::vector<Item> items;
    // suffix: the segment is a request's private suffix; its last item is marked so that the
    // kernel extends it by the tokens appended into the headroom since the plan was made (an
    // empty suffix with headroom still gets an item for them)
    auto add_segment = [&](int64_t a, int64_t e, const std::vector<int32_t>& reqs, bool suffix) {
        if (e <= a) {
            if (suffix && plan.headroom > 0) { items.push_back({a, a, reqs}); items.back().grows = true; }
            return;
        }
        // the fewest pieces of at most `split` tokens, all of (nearly) the same length: a full-length
        // piece next to a short remainder would set the pace of the launch for little work
        const int64_t a_blk = a / kDecodeBlock * kDecodeBlock;
        const int64_t blocks = (e - a_blk + kDecodeBlock - 1) / kDecodeBlock;
        const int64_t pieces = (blocks * kDecodeBlock + split - 1) / split;
        const int64_t piece = (blocks + pieces - 1) / pieces * kDecodeBlock;
        for (size_t m0 = 0; m0 < reqs.size(); m0 += max_members) {
            std::vector<int32_t> chunk(reqs.begin() + m0,
                                       reqs.begin() + std::min(reqs.size(), m0 + max_members));
            for (int64_t p0 = a_blk; p0 < e; p0 += piece) {
                items.push_back({std::max(a, p0), std::min(e, p0 + piece), chunk});
                items.back().grows = suffix && p0 + piece >= e;
            }
        }
    };
    std::vector<int32_t> req_seg(static_cast<size_t>(plan.n) * 4, 0);
    std::vector<std::vector<int32_t>> chain_of(static_cast<size_t>(plan.n));
    for (const Group& g : plan.groups) {
        // work items in layout order: a shared segment attends for every request below it
        struct Piece { int32_t off; int32_t node, member; };
        std::vector<Piece> pieces;
        for (size_t k = 0; k < g.nodes.size(); ++k) pieces.push_back({g.nodes[k].off, static_cast<int32_t>(k), -1});
        for (size_t k = 0; k < g.members.size(); ++k) pieces.push_back({g.members[k].suffix_off, -1, static_cast<int32_t>(k)});
        std::stable_sort(pieces.begin(), pieces.end(), [](const Piece& x, const Piece& y) { return x.off < y.off; });
        for (const Piece& pc : pieces) {
            if (pc.node >= 0) {
                const Node& nd = g.nodes[static_cast<size_t>(pc.node)];
                add_segment(g.buf_base + nd.off, g.buf_base + nd.off + nd.len, nd.reqs, false);
                continue;
            }
            const Member& mm = g.members[static_cast<size_t>(pc.member)];
            add_segment(g.buf_base + mm.suffix_off, g.buf_base + mm.suffix_off + mm.lq, {mm.req}, true);
            int32_t* rs = &req_seg[static_cast<size_t>(mm.req) * 4];
            rs[0] = static_cast<int32_t>(g.buf_base + mm.prefix_off); rs[1] = mm.lp;
            rs[2] = static_cast<int32_t>(g.buf_base + mm.suffix_off); rs[3] = mm.lq;
            std::vector<int32_t>& ch = chain_of[static_cast<size_t>(mm.req)];
            for (int32_t k = mm.node; k >= 0; k = g.nodes[static_cast<size_t>(k)].parent) {
                ch.push_back(g.nodes[static_cast<size_t>(k)].len);            // reversed below: innermost first here
                ch.push_back(static_cast<int32_t>(g.buf_base + g.nodes[static_cast<size_t>(k)].off));
            }
            std::reverse(ch.begin(), ch.end());                   // (offset, tokens) pairs, outermost first
        }
    }
    std::vector<int32_t> chain_start(static_cast<size_t>(plan.n) + 1, 0), chain;
    for (int32_t i = 0; i < plan.n; ++i) {
        chain.insert(chain.end(), chain_of[static_cast<size_t>(i)].begin(), chain_of[static_cast<size_t>(i)].end());
        chain_start[static_cast<size_t>(i) + 1] = static_cast<int32_t>(chain.size() / 2);
    }
    // items with more than 16 query rows first (they run the two-column-tile kernel), then
    // the others; inside each class the longest first (stable: deterministic)
    auto wide = [&](const Item& it) { return static_cast<int>(it.reqs.size()) * r > 16; };
    std::vector<int32_t> order(items.size());
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
        if (wide(items[x]) != wide(items[y])) return wide(items[x]);
        return items[x].e - items[x].a > items[y].e - items[y].a;
    });
    t.n_dec_wide = 0;
    for (const Item& it : items) t.n_dec_wide += wide(it) ? 1 : 0;
    // Partial slots: the slots of one request are consecutive (the merge streams them without
    // indirection); a request covered by a single work item gets no slot: that item writes the
    // final output itself (slot -1).
    std::vector<int32_t> n_items_of(static_cast<size_t>(plan.n), 0), start(static_cast<size_t>(plan.n) + 1, 0);
    for (const Item& it : items)
        for (int32_t rq : it.reqs) ++n_items_of[static_cast<size_t>(rq)];
    int32_t n_parts = 0;
    for (int32_t i = 0; i < plan.n; ++i) {
        start[static_cast<size_t>(i)] = n_parts;
        if (n_items_of[static_cast<size_t>(i)] > 1) n_parts += n_items_of[static_cast<size_t>(i)];
    }
    start[static_cast<size_t>(plan.n)] = n_parts;
    std::vector<int32_t> next_slot(start.begin(), start.end() - 1);
    std::vector<int32_t> flat, members, member_slot;
    for (int32_t idx : order) {
        const Item& it = items[idx];
        flat.push_back(static_cast<int32_t>(it.a));
        flat.push_back(static_cast<int32_t>(it.e));
        flat.push_back(static_cast<int32_t>(members.size()));
        flat.push_back(static_cast<int32_t>(it.reqs.size()));
        flat.push_back(it.grows ? 1 : 0); flat.push_back(0); flat.push_back(0); flat.push_back(0);
        for (int32_t rq : it.reqs) {
            members.push_back(rq);
            member_slot.push_back(n_items_of[static_cast<size_t>(rq)] > 1 ? next_slot[static_cast<size_t>(rq)]++ : -1);
        }
    }
    t.n_dec_items = static_cast<int32_t>(items.size());
    t.n_dec_parts = n_parts;
    t.dec_max_parts = 0;
    for (int32_t c : n_items_of) t.dec_max_parts = std::max(t.dec_max_parts, c > 1 ? c : 0);
    t.dec_items = b.add(flat);
    t.dec_members = b.add(members);
    t.dec_member_slot = b.add(member_slot);
    t.dec_req_part_start = b.add(start);
    t.dec_req_seg = b.add(req_seg);
    t.dec_chain_start = b.add(chain_start);
    t.dec_chain = b.add(chain);
}

// ---- prefill ---------------------------------------------------------------
struct QRow { int32_t req, t; };       // packed row -> (request, query position)

// Flat arrays of a schedule under construction (tiles in construction order).
struct SchedBuild {
    std::vector<int32_t> runs;                    // (first tile row, its Q row, lo, its hi) of every run of rows of one request
    std::vector<int32_t> run_first, n_runs;       // per tile
    std::vector<int32_t> kv;                      // (k_start, info) pairs of all tiles
    std::vector<int32_t> kv_first, n_kv, n_rows;  // per tile
    std::vector<int64_t> weight;                  // active (wave, key tile) pairs per tile
    int64_t issued = 0;
};

// Appends one query tile (rows[0..nrows)) and its key-tile list.  all_waves: the padded
// schedule never lets a wave skip.
void add_tile(const pk_plan& plan, const std::vector<int64_t>& q_start,
              const std::vector<int64_t>& kv_start, const QRow* rows, int nrows,
              bool all_waves, SchedBuild& sb) {
    constexpr int BM = kPrefillBM, BN = kPrefillBN, WR = 32, NW = BM / WR;
    sb.run_first.push_back(static_cast<int32_t>(sb.runs.size() / 4));
    const size_t kv0 = sb.kv.size();
    int64_t weight = 0;
    int i = 0;
    while (i < nrows) {                            // runs of rows of the same request
        const int32_t rq = rows[i].req;
        int j = i + 1;
        while (j < nrows && rows[j].req == rq) ++j;
        const int64_t ks0 = kv_start[rq];
        const int64_t ctx = plan.kv_lens[rq] - plan.q_lens[rq];
        const int64_t kend = ks0 + ctx + rows[j - 1].t + 1;              // hi of the run's last row
        // row x of the run is Q row q_start + t + (x - i) and sees the keys [ks0, ks0 + ctx + t + 1 + (x - i))
        sb.runs.push_back(i);
        sb.runs.push_back(static_cast<int32_t>(q_start[rq] + rows[i].t));
        sb.runs.push_back(static_cast<int32_t>(ks0));
        sb.runs.push_back(static_cast<int32_t>(ks0 + ctx + rows[i].t + 1));
        // per wave: its rows inside the run, and whether it holds rows of no other request
        int wa[NW], wb[NW];
        bool pure[NW];
        for (int w = 0; w < NW; ++w) {
            wa[w] = std::max(i, w * WR);
            wb[w] = std::min(j, (w + 1) * WR);
            pure[w] = i <= w * WR && std::min(nrows, (w + 1) * WR) <= j;
        }
        for (int64_t ks = ks0; ks < kend; ks += BN) {
            const int64_t ke = std::min(kend, ks + BN);
            int32_t flags = 0;
            for (int w = 0; w < NW; ++w) {
                int code = 0;
                if (wa[w] < wb[w] && ks < ks0 + ctx + rows[wb[w] - 1].t + 1) {
                    const bool below = ke <= ks0 + ctx + rows[wa[w]].t + 1;
                    code = (pure[w] && below && ke - ks == BN) ? 2 : 1;
                } else if (all_waves) {
                    code = 1;
                }
                weight += code != 0;
                flags |= code << (2 * w);
            }
            if (flags == 0) continue;
            sb.kv.push_back(static_cast<int32_t>(ks));
            sb.kv.push_back(static_cast<int32_t>(ke - ks) | (flags << 8));
        }
        i = j;
    }
    sb.issued += weight * WR * BN;
    sb.kv_first.push_back(static_cast<int32_t>(kv0 / 2));
    sb.n_kv.push_back(static_cast<int32_t>((sb.kv.size() - kv0) / 2));
    sb.n_rows.push_back(nrows);
    sb.n_runs.push_back(static_cast<int32_t>(sb.runs.size() / 4) - sb.run_first.back());
    sb.weight.push_back(weight);
}

void add_idle_tile(SchedBuild& sb) {               // padded grid slot of a request without that many tiles
    sb.run_first.push_back(static_cast<int32_t>(sb.runs.size() / 4));
    sb.n_runs.push_back(0);
    sb.kv_first.push_back(static_cast<int32_t>(sb.kv.size() / 2));
    sb.n_kv.push_back(0); sb.n_rows.push_back(0); sb.weight.push_back(0);
}

// Writes the tiles in the given order (key-tile lists are re-based accordingly).
void emit_sched(const SchedBuild& sb, const std::vector<int32_t>& order, Builder& b,
                DeviceTables::PrefillSched& s) {
    std::vector<int32_t> desc, more_first, more, kv;
    desc.reserve(order.size() * kTileDescWords);
    more_first.reserve(order.size());
    kv.reserve(sb.kv.size());
    for (int32_t idx : order) {
        desc.push_back(static_cast<int32_t>(kv.size() / 2));
        desc.push_back(sb.n_kv[idx]);
        // per wave (8 bits each, saturating): how many key tiles at the START and at the END of the
        // list the wave skips (a packed query tile that straddles requests lists the key tiles of all
        // of them; the rows of one wave mostly belong to one)
        int32_t leading = 0, trailing = 0;
        for (int w = 0; w < 4; ++w) {
            auto code = [&](int32_t e) {
                return (sb.kv[2 * (static_cast<size_t>(sb.kv_first[idx]) + e) + 1] >> (8 + 2 * w)) & 3;
            };
            int32_t lead = 0, trail = 0;
            while (lead < sb.n_kv[idx] && lead < 255 && code(lead) == 0) ++lead;
            while (trail < sb.n_kv[idx] - lead && trail < 255 && code(sb.n_kv[idx] - 1 - trail) == 0) ++trail;
            leading |= lead << (8 * w);
            trailing |= trail << (8 * w);
        }
        desc.push_back(leading);
        desc.push_back(trailing);
        // The rows of a tile are runs of consecutive rows of one request each; most tiles are one
        // run, which sits in the descriptor itself (its Q row, lo, hi of tile row 0): the kernel
        // needs no second look-up before it can fetch its Q operand.  Further runs go to a list.
        const int32_t nr = sb.n_runs[idx];
        const int32_t* run = sb.runs.data() + 4 * static_cast<size_t>(sb.run_first[idx]);
        desc.push_back(sb.n_rows[idx] | (nr << 16));
        for (int x = 1; x < 4; ++x) desc.push_back(nr > 0 ? run[x] : 0);
        // words 8..10: the first key rows of the tile's first three key tiles (the last one repeated
        // if there are fewer), so that the kernel can request its first K/V tiles without waiting for
        // a look-up in the key-tile list; the rest pads the descriptor to 64 bytes
        for (int e = 0; e < 3; ++e) {
            const int32_t ee = sb.n_kv[idx] > 0 ? std::min(e, sb.n_kv[idx] - 1) : 0;
            desc.push_back(sb.n_kv[idx] > 0 ? sb.kv[2 * (static_cast<size_t>(sb.kv_first[idx]) + ee)] : 0);
        }
        for (int x = 11; x < kTileDescWords; ++x) desc.push_back(0);
        more_first.push_back(static_cast<int32_t>(more.size() / 4));
        if (nr > 1) more.insert(more.end(), run + 4, run + 4 * static_cast<size_t>(nr));
        kv.insert(kv.end(), sb.kv.begin() + 2 * sb.kv_first[idx], sb.kv.begin() + 2 * (sb.kv_first[idx] + sb.n_kv[idx]));
    }
    s.n_tiles = static_cast<int32_t>(order.size());
    s.issued_pairs = sb.issued;
    s.tiles = b.add(desc);
    s.run_first = b.add(more_first); s.runs = b.add(more);
    s.kvtiles = b.add(kv);
}

// packed: tiles over each group's packed row stream, heaviest tile first
void build_prefill_packed(const pk_plan& plan, const std::vector<int64_t>& q_start,
                          const std::vector<int64_t>& kv_start, int Hq, int num_cus, Builder& b, DeviceTables& t) {
    constexpr int BM = kPrefillBM;
    // A batch so small that even one tile per request piece leaves workgroup slots empty (two per
    // compute unit) gains nothing from sharing tiles between requests: a shared tile walks the key
    // tiles of both requests one after the other, which only lengthens the longest workgroup.
    int64_t aligned_tiles = 0;
    for (int32_t i = 0; i < plan.n; ++i) aligned_tiles += (plan.q_lens[i] + BM - 1) / BM;
    const bool may_share = aligned_tiles * Hq > 2 * static_cast<int64_t>(num_cus);
    SchedBuild sb;
    std::vector<QRow> rows;
    std::vector<int32_t> tile_req;                 // request of a tile's first row
    rows.reserve(BM);
    for (const Group& g : plan.groups) {
        rows.clear();
        for (const Member& m : g.members) {
            // A request that does not fit into what is left of the current tile shares it only if
            // that saves the request a tile of its own (its head then rides along with few key
            // tiles); otherwise the tile is closed and the request starts on a fresh one: a shared
            // tile walks the key tiles of both requests one after the other and runs them masked.
            const int32_t lq = plan.q_lens[m.req];
            const int32_t room = BM - static_cast<int32_t>(rows.size());
            if (!rows.empty() && (lq > room || !may_share)) {
                const int32_t last = lq % BM == 0 ? BM : lq % BM;   // rows of its last tile when it starts fresh
                if (room < last || !may_share) {
                    tile_req.push_back(rows[0].req);
                    add_tile(plan, q_start, kv_start, rows.data(), static_cast<int>(rows.size()), false, sb);
                    rows.clear();
                }
            }
            for (int32_t x = 0; x < plan.q_lens[m.req]; ++x) {
                rows.push_back({m.req, x});
                if (rows.size() == BM) {
                    tile_req.push_back(rows[0].req);
                    add_tile(plan, q_start, kv_start, rows.data(), BM, false, sb);
                    rows.clear();
                }
            }
        }
        if (!rows.empty()) {
            tile_req.push_back(rows[0].req);
            add_tile(plan, q_start, kv_start, rows.data(), static_cast<int>(rows.size()), false, sb);
        }
    }
    std::vector<int32_t> order(sb.n_kv.size());
    std::iota(order.begin(), order.end(), 0);
    // Launch order: request by request (the request whose heaviest tile is heaviest first), and
    // inside a request the heaviest tile first.  Workgroups that run at the same time on one XCD
    // then stream the same K/V rows, which keeps them in that XCD's L2; the many short tiles at
    // the end of the list even out the tail.
    std::vector<int64_t> req_weight(static_cast<size_t>(plan.n), 0);
    for (size_t x = 0; x < tile_req.size(); ++x)
        req_weight[static_cast<size_t>(tile_req[x])] = std::max(req_weight[static_cast<size_t>(tile_req[x])], sb.weight[x]);
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
        const int32_t rx = tile_req[static_cast<size_t>(x)], ry = tile_req[static_cast<size_t>(y)];
        if (rx != ry) {
            if (req_weight[static_cast<size_t>(rx)] != req_weight[static_cast<size_t>(ry)])
                return req_weight[static_cast<size_t>(rx)] > req_weight[static_cast<size_t>(ry)];
            return rx < ry;
        }
        return sb.weight[x] > sb.weight[y];
    });
    emit_sched(sb, order, b, t.packed);
}

}  // namespace

// padded: request-aligned grid (request, tile) sized by the longest request, natural order.
// Built on first use into its own host image (uploaded behind the partial results).
void build_prefill_padded(const pk_plan& plan, DeviceTables& t) {
    constexpr int BM = kPrefillBM;
    std::vector<int64_t> q_start(static_cast<size_t>(plan.n) + 1, 0), kv_start(static_cast<size_t>(plan.n) + 1, 0);
    for (int32_t i = 0; i < plan.n; ++i) {
        q_start[i + 1] = q_start[i] + plan.q_lens[i];
        kv_start[i + 1] = kv_start[i] + plan.kv_lens[i];
    }
    int32_t max_tiles = 0;
    for (int32_t i = 0; i < plan.n; ++i) max_tiles = std::max(max_tiles, (plan.q_lens[i] + BM - 1) / BM);
    SchedBuild sb;
    std::vector<QRow> rows;
    for (int32_t i = 0; i < plan.n; ++i) {
        for (int32_t tt = 0; tt < max_tiles; ++tt) {
            rows.clear();
            for (int32_t x = tt * BM; x < std::min(plan.q_lens[i], (tt + 1) * BM); ++x) rows.push_back({i, x});
            if (rows.empty()) add_idle_tile(sb);
            else add_tile(plan, q_start, kv_start, rows.data(), static_cast<int>(rows.size()), true, sb);
        }
    }
    std::vector<int32_t> order(sb.n_kv.size());
    std::iota(order.begin(), order.end(), 0);
    t.host_padded.clear();
    Builder b(t.host_padded);
    emit_sched(sb, order, b, t.padded);
    t.host_padded.resize((t.host_padded.size() + 63) / 64 * 64, 0);
    t.padded_built = true;
}

namespace {

// Upper bound (bytes) of the padded schedule's tables, without building them.
size_t padded_bound_bytes(const pk_plan& plan) {
    constexpr int64_t BM = kPrefillBM, BN = kPrefillBN;
    int64_t max_tiles = 0, kv_entries = 0;
    for (int32_t i = 0; i < plan.n; ++i) max_tiles = std::max<int64_t>(max_tiles, (plan.q_lens[i] + BM - 1) / BM);
    for (int32_t i = 0; i < plan.n; ++i) {
        const int64_t ctx = plan.kv_lens[i] - plan.q_lens[i];
        for (int64_t tt = 0; tt * BM < plan.q_lens[i]; ++tt)
            kv_entries += (ctx + std::min<int64_t>(plan.q_lens[i], (tt + 1) * BM) + BN - 1) / BN;
    }
    const int64_t tiles = max_tiles * plan.n;
    const int64_t ints = tiles * kTileDescWords + tiles + 2 * kv_entries + 6 * 64;   // a padded tile is one run: the run list is empty
    return static_cast<size_t>((ints + 63) / 64 * 64) * sizeof(int32_t);
}

}  // namespace

size_t kv_buf_bytes(const pk_plan& plan, int Hkv, int d, int dtype) {
    const size_t elem = dtype == PK_F32 ? 4 : 2;
    return static_cast<size_t>(plan.buf_tokens) * Hkv * d * 2 * elem;
}

void build_tables(const pk_plan& plan, int Hq, int Hkv, int d, int dtype, int num_cus, DeviceTables& t) {
    t = DeviceTables();
    t.Hq = Hq; t.Hkv = Hkv; t.d = d; t.dtype = dtype;
    Builder b(t.host);
    std::vector<int64_t> q_start(static_cast<size_t>(plan.n) + 1, 0), kv_start(static_cast<size_t>(plan.n) + 1, 0);
    for (int32_t i = 0; i < plan.n; ++i) {
        q_start[i + 1] = q_start[i] + plan.q_lens[i];
        kv_start[i + 1] = kv_start[i] + plan.kv_lens[i];
    }
    t.q_start = b.add(std::vector<int32_t>(q_start.begin(), q_start.end()));
    t.kv_start = b.add(std::vector<int32_t>(kv_start.begin(), kv_start.end()));
    build_reorg(plan, b, t);
    if (plan.decode_only) build_decode(plan, Hq, Hkv, num_cus, b, t);
    build_prefill_packed(plan, q_start, kv_start, Hq, num_cus, b, t);
    t.host.resize((t.host.size() + 63) / 64 * 64, 0);
    t.tables_bytes = t.host.size() * sizeof(int32_t);
    t.partial_offset = t.tables_bytes;
    t.partial_bytes = static_cast<size_t>(t.n_dec_parts) * Hq * (static_cast<size_t>(d) + 1) * sizeof(float);
    t.decode_only_bytes = t.partial_offset + t.partial_bytes;
    if (plan.decode_only) {
        // the padded comparison kernel keeps (request, split) partials in the same region: the
        // same number of splits for every request, sized by the longest -- at most 64, each a
        // multiple of 32 tokens and at least 512 tokens long (enough waves to fill the chip from the
        // long requests alone; more splits only add empty grid slots and partial results)
        int32_t max_len = 0;
        for (int32_t L : plan.kv_lens) max_len = std::max(max_len, L);
        int32_t split = std::max(512, ((max_len + 63) / 64 + 31) / 32 * 32);
        t.pad_split_tokens = split;
        t.pad_n_splits = (max_len + split - 1) / split;
        const size_t pad_bytes = static_cast<size_t>(plan.n) * t.pad_n_splits * Hq * (static_cast<size_t>(d) + 1) * sizeof(float);
        t.partial_bytes = std::max(t.partial_bytes, pad_bytes);
    }
    t.padded_offset = (t.partial_offset + t.partial_bytes + 255) / 256 * 256;
    t.total_bytes = (t.padded_offset + padded_bound_bytes(plan) + 255) / 256 * 256;
}

}  // namespace pk
