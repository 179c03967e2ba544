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
#include <cstdlib>
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

int env_int(const char* name, int dflt) {
    const char* s = std::getenv(name);
    if (!s || !*s) return dflt;
    const int v = std::atoi(s);
    return v > 0 ? v : dflt;
}

// ---- re-layout -------------------------------------------------------------
void build_reorg(const pk_plan& plan, Builder& b, DeviceTables& t) {
    struct Seg { int64_t dst0; int32_t ntok, req, src0; };
    std::vector<Seg> segs;
    for (const Group& g : plan.groups) {
        int32_t last_poff = -1;
        for (const Member& m : g.members) {
            if (m.lp > 0 && m.prefix_off != last_poff) {          // prefix once, via its first member
                segs.push_back({g.buf_base + m.prefix_off, m.lp, m.req, 0});
                last_poff = m.prefix_off;
            }
            if (m.lq > 0) segs.push_back({g.buf_base + m.suffix_off, m.lq, m.req, m.lp});
        }
    }
    // segments are produced in increasing dst0 already (layout order)
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
void build_decode(const pk_plan& plan, int Hq, int Hkv, Builder& b, DeviceTables& t) {
    const int r = Hq / Hkv;
    const int max_members = std::max(1, kDecodeMaxRows / r);
    // split length: enough work items to fill the chip, long enough to amortise the partials
    int64_t split = (plan.unique_tokens * Hkv / 16384 + kDecodeBlock - 1) / kDecodeBlock * kDecodeBlock;
    split = std::min<int64_t>(std::max<int64_t>(split, 128), 2048);
    split = env_int("PK_DECODE_SPLIT", static_cast<int>(split));
    split = (split + kDecodeBlock - 1) / kDecodeBlock * kDecodeBlock;
    t.dec_split_tokens = static_cast<int32_t>(split);

    struct Item { int64_t a, e; std::vector<int32_t> reqs; };
    std::vector<Item> items;
    auto add_segment = [&](int64_t a, int64_t e, const std::vector<int32_t>& reqs) {
        if (e <= a) return;
        const int64_t a_blk = a / kDecodeBlock * kDecodeBlock;
        for (size_t m0 = 0; m0 < reqs.size(); m0 += max_members) {
            std::vector<int32_t> chunk(reqs.begin() + m0,
                                       reqs.begin() + std::min(reqs.size(), m0 + max_members));
            for (int64_t p0 = a_blk; p0 < e; p0 += split)
                items.push_back({std::max(a, p0), std::min(e, p0 + split), chunk});
        }
    };
    std::vector<int32_t> req_seg(static_cast<size_t>(plan.n) * 4, 0);
    for (const Group& g : plan.groups) {
        size_t i = 0;
        while (i < g.members.size()) {
            const Member& m = g.members[i];
            size_t j = i + 1;
            if (m.lp > 0) {
                while (j < g.members.size() && g.members[j].lp > 0 &&
                       g.members[j].prefix_off == m.prefix_off) ++j;
                std::vector<int32_t> fam;
                for (size_t k = i; k < j; ++k) fam.push_back(g.members[k].req);
                add_segment(g.buf_base + m.prefix_off, g.buf_base + m.prefix_off + m.lp, fam);
            }
            for (size_t k = i; k < j; ++k) {
                const Member& mm = g.members[k];
                add_segment(g.buf_base + mm.suffix_off, g.buf_base + mm.suffix_off + mm.lq, {mm.req});
                int32_t* rs = &req_seg[static_cast<size_t>(mm.req) * 4];
                rs[0] = static_cast<int32_t>(g.buf_base + mm.prefix_off); rs[1] = mm.lp;
                rs[2] = static_cast<int32_t>(g.buf_base + mm.suffix_off); rs[3] = mm.lq;
            }
            i = j;
        }
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
    std::vector<int32_t> flat, members;
    std::vector<std::vector<int32_t>> parts_of(static_cast<size_t>(plan.n));
    int32_t n_parts = 0;
    for (int32_t idx : order) {
        const Item& it = items[idx];
        flat.push_back(static_cast<int32_t>(it.a));
        flat.push_back(static_cast<int32_t>(it.e));
        flat.push_back(static_cast<int32_t>(members.size()));
        flat.push_back(static_cast<int32_t>(it.reqs.size()));
        flat.push_back(n_parts);
        flat.push_back(0); flat.push_back(0); flat.push_back(0);
        for (int32_t rq : it.reqs) {
            members.push_back(rq);
            parts_of[static_cast<size_t>(rq)].push_back(n_parts++);
        }
    }
    std::vector<int32_t> start(static_cast<size_t>(plan.n) + 1, 0), parts;
    for (int32_t i = 0; i < plan.n; ++i) {
        start[static_cast<size_t>(i)] = static_cast<int32_t>(parts.size());
        parts.insert(parts.end(), parts_of[static_cast<size_t>(i)].begin(), parts_of[static_cast<size_t>(i)].end());
    }
    start[static_cast<size_t>(plan.n)] = static_cast<int32_t>(parts.size());
    t.n_dec_items = static_cast<int32_t>(items.size());
    t.n_dec_parts = n_parts;
    t.dec_items = b.add(flat);
    t.dec_members = b.add(members);
    t.dec_req_part_start = b.add(start);
    t.dec_req_parts = b.add(parts);
    t.dec_req_seg = b.add(req_seg);
}

// ---- prefill ---------------------------------------------------------------
struct QRow { int32_t req, t; };       // packed row -> (request, query position); req < 0: padding

struct TileOut {
    std::vector<int32_t> row_q, row_lo, row_hi;   // BM entries
    std::vector<int32_t> kv;                      // pairs
    int64_t weight = 0;
    int32_t n_rows = 0;
};

// Builds the key-tile list of one query tile.  all_waves: the padded schedule
// never lets a wave skip.
TileOut make_tile(const pk_plan& plan, const std::vector<int64_t>& q_start,
                  const std::vector<int64_t>& kv_start, const std::vector<QRow>& rows,
                  bool all_waves, int64_t* issued) {
    constexpr int BM = kPrefillBM, BN = kPrefillBN, WR = 32, NW = BM / WR;
    TileOut o;
    o.row_q.assign(BM, -1); o.row_lo.assign(BM, 0); o.row_hi.assign(BM, 0);
    o.n_rows = static_cast<int32_t>(rows.size());
    for (size_t i = 0; i < rows.size(); ++i) {
        const int32_t rq = rows[i].req;
        if (rq < 0) continue;
        const int64_t ctx = plan.kv_lens[rq] - plan.q_lens[rq];
        o.row_q[i] = static_cast<int32_t>(q_start[rq] + rows[i].t);
        o.row_lo[i] = static_cast<int32_t>(kv_start[rq]);
        o.row_hi[i] = static_cast<int32_t>(kv_start[rq] + ctx + rows[i].t + 1);
    }
    // runs of rows of the same request
    size_t i = 0;
    while (i < rows.size()) {
        const int32_t rq = rows[i].req;
        size_t j = i + 1;
        while (j < rows.size() && rows[j].req == rq) ++j;
        if (rq >= 0) {
            const int64_t ks0 = kv_start[rq];
            const int64_t ctx = plan.kv_lens[rq] - plan.q_lens[rq];
            const int64_t kend = ks0 + ctx + rows[j - 1].t + 1;          // hi of the run's last row
            for (int64_t ks = ks0; ks < kend; ks += BN) {
                const int64_t ke = std::min(kend, ks + BN);
                int32_t flags = 0;
                for (int w = 0; w < NW; ++w) {
                    // rows of this wave that belong to the run
                    const size_t wa = std::max<size_t>(i, static_cast<size_t>(w) * WR);
                    const size_t wb = std::min<size_t>(j, static_cast<size_t>(w + 1) * WR);
                    int code = 0;
                    if (wa < wb && ks < ks0 + ctx + rows[wb - 1].t + 1) {
                        bool pure = true;                                 // no row of another request in the wave
                        for (size_t x = static_cast<size_t>(w) * WR;
                             x < std::min(rows.size(), static_cast<size_t>(w + 1) * WR); ++x)
                            if (rows[x].req >= 0 && rows[x].req != rq) pure = false;
                        const bool below = ke <= ks0 + ctx + rows[wa].t + 1;
                        code = (pure && below && ke - ks == BN) ? 2 : 1;
                    } else if (all_waves) {
                        code = 1;
                    }
                    if (code) { o.weight += 1; if (issued) *issued += static_cast<int64_t>(WR) * BN; }
                    flags |= code << (2 * w);
                }
                if (flags == 0) continue;
                o.kv.push_back(static_cast<int32_t>(ks));
                o.kv.push_back(static_cast<int32_t>(ke - ks) | (flags << 8));
            }
        }
        i = j;
    }
    return o;
}

void emit_sched(std::vector<TileOut>& tiles, const std::vector<int32_t>& order, Builder& b,
                DeviceTables::PrefillSched& s) {
    std::vector<int32_t> desc, rq, rlo, rhi, kv;
    for (int32_t idx : order) {
        TileOut& t = tiles[idx];
        desc.push_back(static_cast<int32_t>(kv.size() / 2));
        desc.push_back(static_cast<int32_t>(t.kv.size() / 2));
        desc.push_back(t.n_rows);
        desc.push_back(0);
        rq.insert(rq.end(), t.row_q.begin(), t.row_q.end());
        rlo.insert(rlo.end(), t.row_lo.begin(), t.row_lo.end());
        rhi.insert(rhi.end(), t.row_hi.begin(), t.row_hi.end());
        kv.insert(kv.end(), t.kv.begin(), t.kv.end());
    }
    s.n_tiles = static_cast<int32_t>(order.size());
    s.tiles = b.add(desc);
    s.row_q = b.add(rq); s.row_lo = b.add(rlo); s.row_hi = b.add(rhi);
    s.kvtiles = b.add(kv);
}

void build_prefill(const pk_plan& plan, const std::vector<int64_t>& q_start,
                   const std::vector<int64_t>& kv_start, Builder& b, DeviceTables& t) {
    constexpr int BM = kPrefillBM;
    // packed: tiles over each group's packed row stream
    {
        std::vector<TileOut> tiles;
        for (const Group& g : plan.groups) {
            std::vector<QRow> rows;
            for (const Member& m : g.members) {
                for (int32_t x = 0; x < plan.q_lens[m.req]; ++x) {
                    rows.push_back({m.req, x});
                    if (rows.size() == BM) {
                        tiles.push_back(make_tile(plan, q_start, kv_start, rows, false, &t.packed.issued_pairs));
                        rows.clear();
                    }
                }
            }
            if (!rows.empty())
                tiles.push_back(make_tile(plan, q_start, kv_start, rows, false, &t.packed.issued_pairs));
        }
        std::vector<int32_t> order(tiles.size());
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
            return tiles[x].weight > tiles[y].weight;                    // longest first
        });
        emit_sched(tiles, order, b, t.packed);
    }
    // padded: request-aligned grid (request, tile) sized by the longest request
    {
        int32_t max_tiles = 0;
        for (int32_t i = 0; i < plan.n; ++i)
            max_tiles = std::max(max_tiles, (plan.q_lens[i] + BM - 1) / BM);
        std::vector<TileOut> tiles;
        for (int32_t i = 0; i < plan.n; ++i) {
            for (int32_t tt = 0; tt < max_tiles; ++tt) {
                std::vector<QRow> rows;
                for (int32_t x = tt * BM; x < std::min(plan.q_lens[i], (tt + 1) * BM); ++x)
                    rows.push_back({i, x});
                tiles.push_back(make_tile(plan, q_start, kv_start, rows, true, &t.padded.issued_pairs));
            }
        }
        std::vector<int32_t> order(tiles.size());
        std::iota(order.begin(), order.end(), 0);
        emit_sched(tiles, order, b, t.padded);
    }
}

}  // namespace

size_t kv_buf_bytes(const pk_plan& plan, int Hkv, int d, int dtype) {
    const size_t elem = dtype == PK_F32 ? 4 : 2;
    return static_cast<size_t>(plan.buf_tokens) * Hkv * d * 2 * elem;
}

void build_tables(const pk_plan& plan, int Hq, int Hkv, int d, int dtype, DeviceTables& t) {
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
    if (plan.decode_only) build_decode(plan, Hq, Hkv, b, t);
    build_prefill(plan, q_start, kv_start, b, t);
    t.host.resize((t.host.size() + 63) / 64 * 64, 0);
    t.tables_bytes = t.host.size() * sizeof(int32_t);
    t.partial_offset = t.tables_bytes;
    t.partial_bytes = static_cast<size_t>(t.n_dec_parts) * Hq * (static_cast<size_t>(d) + 1) * sizeof(float);
    t.total_bytes = (t.partial_offset + t.partial_bytes + 255) / 256 * 256;
}

}  // namespace pk
