// Host side of the attention planner: the choice of the key-range pieces from a simulated schedule, the counts the
// launches need, and a host twin of the device list builder.  Plain C++ (no HIP), see attn_plan.h.
#include "attn_plan.h"

#include <algorithm>
#include <cmath>
#include <functional>
#include <queue>
#include <vector>

namespace cs {

void attn_plan_capacity(const AttnTune &tune, int64_t max_T, int64_t max_B, int G, int Hkv, int64_t *max_tiles,
                        int64_t *max_items) {
    int64_t tiles = (int64_t)Hkv * ((G * max_T + ATTN_BM - 1) / ATTN_BM + max_B);
    *max_tiles = tiles;
    *max_items = 3 * tiles + 4 * tune.target_items;     // candidates that need more are not considered
}

namespace {
struct UnitShape { int tiles, nc; };
struct Candidate { int cpi, equalize; };

UnitPlan shape_plan(const UnitShape &t, Candidate cd) {
    UnitPlan p;
    p.n_qt = t.tiles; p.nc_max = t.nc;       // n_qt holds Hkv * n_qt here (Hkv = 1 in the calls below)
    int n = t.nc > cd.cpi ? plan_ceil_div(t.nc, cd.cpi) : 1;
    bool clamped = n > ATTN_MAX_SPLIT;
    p.n_split = clamped ? ATTN_MAX_SPLIT : n;
    p.piece = (cd.equalize || clamped) ? plan_ceil_div(std::max(t.nc, 1), p.n_split) : cd.cpi;
    return p;
}

// Cost of an item beside its chunks, in chunk-times: filling the pipeline, loading q, writing the result - rows of the
// output (whole tiles) or fp32 partial results (pieces).  From the uniform 64-trace batch: whole tiles 424 us, halves
// 411 us + 26 us of merging per layer.
constexpr float ITEM_OVERHEAD_WHOLE = 6.0f, ITEM_OVERHEAD_PIECE = 8.0f;

// Items, partial slots and the largest per-XCD item count of a candidate; lens (optional) receives the
// per-XCD item costs (chunks + overhead) in dispatch order.  Same arithmetic as the list builder.
void candidate_counts(const std::vector<UnitShape> &tr, Candidate cd, int64_t n_tiles, int64_t work_total,
                      AttnPlanCounts *r, std::vector<float> *lens /* [8] */) {
    r->n_items = 0; r->n_part_slots = 0; r->max_xcd_items = 0;
    int tile_lo[9] = {0}, seg_base[9] = {0};
    int tile_base = 0, rest_base = 0;
    long long work_base = 0;
    std::vector<UnitPlan> plans;
    plans.reserve(tr.size());
    for (const UnitShape &t : tr) {
        UnitPlan p = shape_plan(t, cd);
        plans.push_back(p);
        plan_xcd_starts(p, 1, tile_base, rest_base, work_base, work_total, tile_lo, seg_base);
        r->n_items += (int64_t)t.tiles * p.n_split;
        if (p.n_split > 1) r->n_part_slots += (int64_t)t.tiles * p.n_split;
        tile_base += t.tiles; rest_base += t.tiles * (p.n_split - 1);
        work_base += (long long)t.tiles * t.nc;
    }
    tile_lo[8] = (int)n_tiles;
    seg_base[8] = (int)r->n_items;
    for (int x = 0; x < 8; ++x) r->max_xcd_items = std::max<int64_t>(r->max_xcd_items, seg_base[x + 1] - seg_base[x]);
    if (!lens) return;
    std::vector<float> rest_lens[8];
    int ti = 0;
    for (size_t i = 0; i < tr.size(); ++i)
        for (int j = 0; j < tr[i].tiles; ++j, ++ti) {
            int x = 7;
            while (x > 0 && tile_lo[x] > ti) --x;
            const UnitPlan &p = plans[i];
            const float ov = p.n_split > 1 ? ITEM_OVERHEAD_PIECE : ITEM_OVERHEAD_WHOLE;
            lens[x].push_back((float)std::min(p.piece, p.nc_max) + ov);
            for (int sp = 1; sp < p.n_split; ++sp)
                rest_lens[x].push_back((float)std::max(0, std::min(p.piece, p.nc_max - sp * p.piece)) + ov);
        }
    for (int x = 0; x < 8; ++x) lens[x].insert(lens[x].end(), rest_lens[x].begin(), rest_lens[x].end());
}

// Makespan of the item list of the busiest XCD, in chunk-times (the time a workgroup takes for one chunk while its CU
// holds two workgroups).  An XCD has slots / 8 workgroup slots, two per CU; items are handed out in list order as
// slots free up.  A workgroup that has its CU to itself runs faster - measured about 1.5 times - which decides the
// value of a last round that does not fill the chip: 96 equal items on 64 slots take 1.67 rounds, not 2.
double simulate(const std::vector<float> *lens, int slots) {
    constexpr double ALONE = 1.5;
    const int n_cu = std::max(1, slots / 16);
    int x_busy = 0;
    double most = -1;
    for (int x = 0; x < 8; ++x) {
        double w = 0;
        for (float len : lens[x]) w += len;
        if (w > most) { most = w; x_busy = x; }
    }
    const std::vector<float> &q = lens[x_busy];
    std::vector<double> rem(2 * (size_t)n_cu, -1.0);    // remaining work of slot s of CU c at rem[2 c + s]; < 0: empty
    size_t next = 0;
    // free slots are filled in list order, emptier CUs first (the dispatcher spreads workgroups over the CUs)
    auto fill = [&]() {
        while (next < q.size()) {
            int pick = -1, pick_busy = 3;
            for (int c = 0; c < n_cu; ++c) {
                const int busy = (rem[2 * c] >= 0) + (rem[2 * c + 1] >= 0);
                if (busy < 2 && busy < pick_busy) { pick = rem[2 * c] < 0 ? 2 * c : 2 * c + 1; pick_busy = busy; }
            }
            if (pick < 0) break;
            rem[pick] = (double)q[next++];
        }
    };
    fill();
    double now = 0.0;
    for (;;) {
        double dt = -1.0;
        for (int c = 0; c < n_cu; ++c) {
            const double speed = (rem[2 * c] >= 0 && rem[2 * c + 1] >= 0) ? 1.0 : ALONE;
            for (int s = 0; s < 2; ++s)
                if (rem[2 * c + s] >= 0 && (dt < 0 || rem[2 * c + s] / speed < dt)) dt = rem[2 * c + s] / speed;
        }
        if (dt < 0) break;
        now += dt;
        for (int c = 0; c < n_cu; ++c) {
            const double speed = (rem[2 * c] >= 0 && rem[2 * c + 1] >= 0) ? 1.0 : ALONE;
            for (int s = 0; s < 2; ++s)
                if (rem[2 * c + s] >= 0) {
                    rem[2 * c + s] -= dt * speed;
                    if (rem[2 * c + s] <= 1e-9) rem[2 * c + s] = -1.0;   // done: the slot is free
                }
        }
        fill();
    }
    return now;
}
}  // namespace

// Choice of the pieces: equal pieces with a split factor 1..4 of the average tile, or front-loaded
// pieces of 1.07x / 1.2x the per-slot share of all chunks (and of twice that share: half as many pieces); the
// candidate with the smallest simulated makespan plus the cost of its merge pass wins.  The merge pass is a launch
// (about 4 chunk-times) plus the partial results it reads back, 64 KiB written and read per piece: measured 26 us for
// 1536 pieces and 90 us for about 4000, against about 1.9 us per chunk-time of the attention kernel - 0.01 chunk-times
// per piece.  (With a flat 8 chunk-times the ragged 128-trace batch was cut into pieces whose merge cost 2.5 ms per
// pass to save 1 ms of attention.)
AttnPlanCounts attn_plan_counts(const AttnTune &tune, const int32_t *h_cu, const int32_t *h_plens, int B, int T,
                                const int32_t *h_group_start, int n_units, int G, int Hkv, int last_only) {
    AttnPlanCounts r = {};
    if (!h_group_start || last_only) n_units = B;
    std::vector<UnitShape> tr;
    tr.reserve(n_units);
    int64_t total = 0, n_tiles = 0;
    int nc_longest = 0;
    for (int i = 0; i < n_units; ++i) {
        AttnUnit u = plan_unit(h_cu, h_plens, h_group_start, n_units, i, B, T, 1 << 30, last_only);
        UnitPlan p = unit_plan(u, G, 1 << 30, 1, last_only);
        tr.push_back({Hkv * p.n_qt, p.nc_max});
        total += (int64_t)Hkv * p.n_qt * p.nc_max;
        n_tiles += (int64_t)Hkv * p.n_qt;
        if (p.n_qt > 0) nc_longest = std::max(nc_longest, p.nc_max);
    }
    r.n_tiles = n_tiles;
    r.total_chunks = total;
    double avg = n_tiles > 0 ? (double)total / (double)n_tiles : 1.0;
    int64_t slots = tune.target_items;
    int64_t cap_items = 3 * n_tiles + 4 * slots;
    std::vector<Candidate> cands;
    auto equal_cpi = [&](int sp) { return sp == 1 ? (1 << 30) : std::max<int>(tune.min_chunks, (int)((avg + sp - 1) / sp)); };
    auto front_cpi = [&](double f) { return std::max<int>(tune.min_chunks, (int)std::ceil(f * (double)total / (double)slots)); };
    if (tune.force_split >= 1 && tune.force_split <= 4) cands.push_back({equal_cpi(tune.force_split), 1});
    else if (tune.force_split == 5) cands.push_back({front_cpi(1.07), 0});
    else {
        for (int sp = 1; sp <= 4; ++sp) {
            if (sp > 1 && avg / sp < tune.min_chunks) break;
            cands.push_back({equal_cpi(sp), 1});
        }
        for (double f : {1.07, 1.2, 2.14, 2.4})
            if (front_cpi(f) < nc_longest) cands.push_back({front_cpi(f), 0});
    }
    double best = 1e300;
    Candidate pick = {1 << 30, 1};
    for (size_t i = 0; i < cands.size(); ++i) {
        AttnPlanCounts c = {};
        std::vector<float> lens[8];
        candidate_counts(tr, cands[i], n_tiles, total, &c, lens);
        if (c.n_items > cap_items && cands.size() > 1 && cands[i].cpi != (1 << 30)) continue;
        double est = simulate(lens, (int)slots) + (c.n_part_slots > 0 ? 4.0 + 0.01 * (double)c.n_part_slots : 0.0);
        if (est < best) { best = est; pick = cands[i]; }
    }
    r.chunks_per_item = pick.cpi;
    r.equalize = pick.equalize;
    candidate_counts(tr, pick, n_tiles, total, &r, nullptr);
    return r;
}

void attn_plan_host(const int32_t *cu, const int32_t *plens, const int32_t *group_start, int n_units, int B, int T,
                    int max_L, int G, int Hkv, int cpi, int equalize, int last_only, int max_tiles, int max_items,
                    AttnTile *tiles, AttnItem *items, int32_t *counts) {
    if (!group_start || last_only) n_units = B;
    // pass 0 adds up the chunks (the XCD cuts depend on the total), pass 1 places the cuts, pass 2 writes the lists
    long long work_total = 0;
    int tile_lo[9] = {0}, seg_base[9] = {0};
    int total_tiles = 0, total_rest = 0;
    for (int pass = 0; pass < 3; ++pass) {
        int tile_base = 0, rest_base = 0, slot_base = 0;
        long long work_base = 0;
        for (int i = 0; i < n_units; ++i) {
            AttnUnit u = plan_unit(cu, plens, group_start, n_units, i, B, T, max_L, last_only);
            UnitPlan p = unit_plan(u, G, cpi, equalize, last_only);
            int my_tiles = Hkv * p.n_qt;
            if (pass == 1) plan_xcd_starts(p, Hkv, tile_base, rest_base, work_base, work_total, tile_lo, seg_base);
            if (pass == 2)
                plan_emit_unit(cu, T, u, G, Hkv, p, tile_base, rest_base, slot_base, tile_lo, seg_base, last_only, max_tiles,
                               max_items, tiles, items);
            tile_base += my_tiles;
            rest_base += my_tiles * (p.n_split - 1);
            slot_base += p.n_split > 1 ? my_tiles * p.n_split : 0;
            work_base += (long long)my_tiles * p.nc_max;
        }
        if (pass == 0) work_total = work_base;
        if (pass == 1) { tile_lo[8] = tile_base; seg_base[8] = tile_base + rest_base; }
        total_tiles = tile_base;
        total_rest = rest_base;
    }
    counts[0] = std::min(total_tiles, max_tiles);
    counts[1] = std::min(total_tiles + total_rest, max_items);
    for (int x = 0; x < 9; ++x) counts[2 + x] = std::min(seg_base[x], max_items);
}

}  // namespace cs
