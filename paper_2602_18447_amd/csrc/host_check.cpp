// Host-side checker, meant to be built with AddressSanitizer and UBSan (no GPU needed): drives the attention
// planner (attn_plan.h / attn_plan.cpp) and the library's host arithmetic that sizes and carves device memory
// (workspace layout, split-K planes, validators, through the C ABI) over the five benchmark shapes and a few
// thousand seeded random batches, and checks the properties whose violation would become an out-of-bounds access
// on the device: every index in range, every key range covered exactly once, slices disjoint.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../../include/confspec.h"
#include "../../include/confspec_ops.h"
#include "../../include/confspec_static.h"
#include "attn_plan.h"

namespace cs {   // decode_bf16.hip: slices and workgroups of a generation step's projection
void dec_gemm_plan(int K, int n_ct, int *S, int *nwg);
size_t dec_gemm_plane_bytes(int K, int n_ct);
}

static int g_fail = 0;
#define CHECK(cond, ...)                                                         \
    do {                                                                         \
        if (!(cond)) {                                                           \
            if (++g_fail <= 20) { printf("FAIL %s:%d %s  ", __FILE__, __LINE__, #cond); printf(__VA_ARGS__); printf("\n"); } \
        }                                                                        \
    } while (0)

struct Batch {
    std::vector<int32_t> cu, plens, groups;   // groups empty = every trace on its own
    int B() const { return (int)plens.size(); }
    int T() const { return cu.back(); }
};

// One plan (all rows or last rows) of one batch: counts from the host planner, lists from the host twin of the
// device builder, then the invariants.
static void check_plan(const cs::AttnTune &tune, const Batch &b, int G, int Hkv, int last_only, const char *what) {
    const int B = b.B(), T = b.T();
    const int32_t *gs = b.groups.empty() ? nullptr : b.groups.data();
    const int n_units = b.groups.empty() ? B : (int)b.groups.size() - 1;
    cs::AttnPlanCounts pc = cs::attn_plan_counts(tune, b.cu.data(), b.plens.data(), B, T, gs, n_units, G, Hkv, last_only);
    int64_t cap_tiles = 0, cap_items = 0;
    cs::attn_plan_capacity(tune, T, B, G, Hkv, &cap_tiles, &cap_items);
    // the planner's own choice always fits the workspace bound; a forced split factor may not (the pass then refuses
    // the call with CONFSPEC_E_WORKSPACE before anything is launched)
    CHECK(pc.n_tiles <= cap_tiles && (pc.n_items <= cap_items || tune.force_split != 0),
          "%s: plan %lld tiles %lld items exceeds capacity %lld / %lld", what, (long long)pc.n_tiles, (long long)pc.n_items,
          (long long)cap_tiles, (long long)cap_items);
    // exact-size arrays with guard entries behind them: a write past the counted size is an ASan error
    std::vector<cs::AttnTile> tiles((size_t)std::max<int64_t>(pc.n_tiles, 1));
    std::vector<cs::AttnItem> items((size_t)std::max<int64_t>(pc.n_items, 1));
    for (auto &it : items) it.tile = -7;
    int32_t counts[11];
    int max_L = 0;
    for (int v : b.plens) max_L = std::max(max_L, v);
    cs::attn_plan_host(b.cu.data(), b.plens.data(), gs, n_units, B, T, max_L, G, Hkv, pc.chunks_per_item, pc.equalize, last_only,
                       (int)pc.n_tiles, (int)pc.n_items, tiles.data(), items.data(), counts);
    CHECK(counts[0] == pc.n_tiles && counts[1] == pc.n_items, "%s: builder wrote %d tiles %d items, planner counted %lld / %lld", what,
          counts[0], counts[1], (long long)pc.n_tiles, (long long)pc.n_items);
    CHECK(counts[2] == 0 && counts[10] == pc.n_items, "%s: XCD ranges do not span the item list", what);
    int64_t max_seg = 0;
    for (int x = 0; x < 8; ++x) {
        CHECK(counts[2 + x] <= counts[3 + x], "%s: XCD %d range is negative", what, x);
        max_seg = std::max<int64_t>(max_seg, counts[3 + x] - counts[2 + x]);
    }
    CHECK(max_seg == pc.max_xcd_items, "%s: largest XCD range %lld, planner said %lld", what, (long long)max_seg, (long long)pc.max_xcd_items);
    // per tile: pieces cover [0, nc) exactly once, in order of part slots; indices in range
    std::vector<std::vector<std::pair<int, int>>> cover((size_t)pc.n_tiles);
    std::vector<char> slot_used((size_t)std::max<int64_t>(pc.n_part_slots, 1), 0);
    for (int64_t i = 0; i < pc.n_items; ++i) {
        const cs::AttnItem &it = items[(size_t)i];
        CHECK(it.tile >= 0 && it.tile < pc.n_tiles, "%s: item %lld never written or tile %d out of range", what, (long long)i, it.tile);
        if (it.tile < 0 || it.tile >= pc.n_tiles) continue;
        const cs::AttnTile &t = tiles[(size_t)it.tile];
        CHECK(it.b0 == t.b0 && it.c == t.c && it.row0 == t.row0 && it.b_end == t.b_end, "%s: item / tile mismatch", what);
        CHECK(it.b0 >= 0 && it.b0 < it.b_end && it.b_end <= B && it.c >= 0 && it.c < Hkv, "%s: unit [%d, %d) head %d", what, it.b0, it.b_end, it.c);
        int rows = G * (b.cu[it.b_end] - b.cu[it.b0]);
        CHECK(it.row0 >= 0 && it.row0 < rows, "%s: row0 %d of %d rows", what, it.row0, rows);
        CHECK(it.chunk_begin >= 0 && it.chunk_begin <= it.chunk_end, "%s: chunk range [%d, %d)", what, it.chunk_begin, it.chunk_end);
        if (t.n_splits > 1) {
            CHECK(it.part_slot >= t.part_base && it.part_slot < t.part_base + t.n_splits && it.part_slot < pc.n_part_slots,
                  "%s: part slot %d (base %d, %d pieces, %lld slots)", what, it.part_slot, t.part_base, t.n_splits, (long long)pc.n_part_slots);
            if (it.part_slot >= 0 && it.part_slot < pc.n_part_slots) {
                CHECK(!slot_used[(size_t)it.part_slot], "%s: part slot %d used twice", what, it.part_slot);
                slot_used[(size_t)it.part_slot] = 1;
            }
        } else {
            CHECK(it.part_slot == -1, "%s: unsplit tile with part slot %d", what, it.part_slot);
        }
        cover[(size_t)it.tile].push_back({it.chunk_begin, it.chunk_end});
    }
    for (int64_t ti = 0; ti < pc.n_tiles; ++ti) {
        const cs::AttnTile &t = tiles[(size_t)ti];
        auto &cv = cover[(size_t)ti];
        CHECK((int)cv.size() == t.n_splits, "%s: tile %lld has %zu items, %d pieces", what, (long long)ti, cv.size(), t.n_splits);
        std::sort(cv.begin(), cv.end());
        // the chunks this tile must see, computed here from the definition
        int L = b.plens[t.b0], S_tot = b.cu[t.b_end] - b.cu[t.b0];
        int n_pc = (L + 63) / 64, need;
        if (last_only) {
            need = n_pc + (S_tot + 63) / 64;
            CHECK(t.b_end == t.b0 + 1 && t.row0 == (S_tot - 1) * G, "%s: last-row tile of trace %d at row %d", what, t.b0, t.row0);
        } else {
            int r_last = std::min(t.row0 + 127, G * S_tot - 1);
            int tok_lo = b.cu[t.b0] + t.row0 / G, tok_hi = b.cu[t.b0] + r_last / G;
            int tr = t.b0;
            while (b.cu[tr + 1] <= tok_lo) ++tr;          // trace of the tile's first row
            need = n_pc + (tok_hi - b.cu[tr] + 1 + 63) / 64;
            CHECK(t.row0 % 128 == 0, "%s: tile row0 %d", what, t.row0);
        }
        int at = 0;
        for (auto &p : cv) {
            CHECK(p.first == at || p.first == p.second, "%s: tile %lld pieces leave a gap or overlap at chunk %d (next piece [%d, %d))", what,
                  (long long)ti, at, p.first, p.second);
            if (p.second > p.first) at = p.second;
        }
        CHECK(at == need, "%s: tile %lld covered up to chunk %d, needs %d", what, (long long)ti, at, need);
    }
    // every row of every unit belongs to exactly one tile per kv head
    if (!last_only) {
        int64_t rows_total = 0, rows_tiled = 0;
        for (int u = 0; u < n_units; ++u) {
            int b0 = gs ? gs[u] : u, b1 = gs ? gs[u + 1] : u + 1;
            rows_total += (int64_t)Hkv * G * (b.cu[b1] - b.cu[b0]);
        }
        for (auto &t : tiles)
            if (pc.n_tiles > 0) rows_tiled += std::min(128, G * (b.cu[t.b_end] - b.cu[t.b0]) - t.row0);
        CHECK(rows_total == rows_tiled, "%s: %lld rows, %lld in tiles", what, (long long)rows_total, (long long)rows_tiled);
    }
}

static Batch uniform_batch(int B, int L, int S) {
    Batch b;
    b.cu.push_back(0);
    for (int i = 0; i < B; ++i) { b.plens.push_back(L); b.cu.push_back(b.cu.back() + S); }
    return b;
}

static void check_library(const confspec_model_cfg &cfg, const Batch &b, const char *what) {
    confspec_ctx *ctx = nullptr;
    int rc = confspec_create(&cfg, 0, &ctx);
    CHECK(rc == CONFSPEC_OK && ctx, "%s: create rc %d", what, rc);
    if (!ctx) return;
    size_t ws = 0, need = 0;
    CHECK(confspec_workspace_bytes(ctx, b.T(), b.B(), 0, &ws) == CONFSPEC_OK && ws % 256 == 0 && ws > 0, "%s: workspace %zu", what, ws);
    // the device pointers are never dereferenced by the calls below; any non-null value passes the null checks
    const int32_t *dev = reinterpret_cast<const int32_t *>(uintptr_t(0x1000));
    confspec_batch cb = {b.B(), b.T(), dev, dev, dev, b.cu.data(), b.plens.data()};
    CHECK(confspec_static_scratch_need(ctx, &cb, &need) == CONFSPEC_OK && need % 256 == 0 && need <= ws,
          "%s: exact layout %zu vs bound %zu", what, need, ws);
    // slices of both layouts: aligned, inside the total, disjoint
    for (int exact = 0; exact < 2; ++exact) {
        size_t off[64], len[64];
        int32_t n = 64;
        size_t total = 0;
        rc = confspec_op_workspace_slices(ctx, b.T(), b.B(), exact ? &cb : nullptr, off, len, &n, &total);
        CHECK(rc == CONFSPEC_OK && n > 10 && n <= 64, "%s: slices rc %d n %d", what, rc, n);
        if (rc != CONFSPEC_OK) continue;
        CHECK(total == (exact ? need : ws), "%s: slices total %zu", what, total);
        std::vector<std::pair<size_t, size_t>> v;
        for (int i = 0; i < n; ++i) {
            CHECK(off[i] % 256 == 0 && off[i] + len[i] <= total, "%s: slice %d [%zu, +%zu) of %zu", what, i, off[i], len[i], total);
            if (len[i]) v.push_back({off[i], len[i]});
        }
        std::sort(v.begin(), v.end());
        for (size_t i = 1; i < v.size(); ++i)
            CHECK(v[i - 1].first + v[i - 1].second <= v[i].first, "%s: slices overlap at %zu", what, v[i].first);
    }
    // split-K planes: the bytes asked for are a whole number (2..64) of [M, N] fp32 planes, or none
    const int qw = cfg.n_q_heads * cfg.head_dim, kw = cfg.n_kv_heads * cfg.head_dim;
    const int shapes[4][2] = {{qw + 2 * kw, cfg.d_model}, {cfg.d_model, qw}, {2 * cfg.d_ffn, cfg.d_model}, {cfg.d_model, cfg.d_ffn}};
    for (int M : {1, 7, b.B(), 128, 129, 300, b.T()})
        for (auto &s : shapes)
            for (int terms = 1; terms <= 3; ++terms) {
                size_t bytes = confspec_op_gemm_scratch_bytes(ctx, M, s[0], s[1], terms);
                size_t plane = (size_t)M * s[0] * 4;
                CHECK(bytes % plane == 0 && (bytes == 0 || (bytes / plane >= 2 && bytes / plane <= 64)), "%s: split-K bytes %zu for M %d N %d K %d", what,
                      bytes, M, s[0], s[1]);
            }
    // validators: malformed batches are rejected before anything else is touched
    std::vector<int32_t> bad_cu = b.cu;
    bad_cu[1] = bad_cu[0];                                   // an empty suffix
    confspec_batch bad = cb;
    bad.h_cu_suffix = bad_cu.data();
    CHECK(confspec_static_scratch_need(ctx, &bad, &need) == CONFSPEC_E_OUT_OF_RANGE, "%s: empty suffix accepted", what);
    bad = cb;
    bad.T = b.T() + 1;
    CHECK(confspec_static_scratch_need(ctx, &bad, &need) == CONFSPEC_E_OUT_OF_RANGE, "%s: wrong T accepted", what);
    confspec_destroy(ctx);
}

int main() {
    cs::AttnTune tune;
    const confspec_model_cfg draft = {28, 1536, 12, 2, 128, 8960, 151936, 1e6f, 1e-6f, CONFSPEC_DTYPE_BF16};
    const confspec_model_cfg target = {64, 5120, 40, 8, 128, 27648, 152064, 1e6f, 1e-6f, CONFSPEC_DTYPE_BF16};
    // the benchmark shapes
    struct Named { const char *name; Batch b; int G, Hkv; const confspec_model_cfg *cfg; };
    std::vector<Named> named;
    named.push_back({"config 2", uniform_batch(32, 2048, 96), 6, 2, &draft});
    named.push_back({"config 3", uniform_batch(64, 8192, 128), 6, 2, &draft});
    {
        std::mt19937 rng(1004);
        Batch b;
        b.cu.push_back(0);
        for (int i = 0; i < 128; ++i) {
            b.plens.push_back(512 + (int)(rng() % (16384 - 512 + 1)));
            b.cu.push_back(b.cu.back() + 32 + (int)(rng() % 225));
        }
        named.push_back({"config 4 (same ranges)", b, 6, 2, &draft});
    }
    named.push_back({"config 5", uniform_batch(16, 4096, 96), 5, 8, &target});
    named.push_back({"one-token batch", uniform_batch(32, 2048, 1), 6, 2, &draft});
    for (auto &nb : named) {
        check_plan(tune, nb.b, nb.G, nb.Hkv, 0, nb.name);
        check_plan(tune, nb.b, nb.G, nb.Hkv, 1, nb.name);
        check_library(*nb.cfg, nb.b, nb.name);
    }
    // seeded random batches: head groupings, lengths on and around page / chunk / tile borders, shared-context groups,
    // every planner setting
    std::mt19937 rng(20260218);
    const int special[] = {0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1023, 1024, 4095, 4096, 16384};
    const int heads[][2] = {{6, 2}, {1, 8}, {5, 8}, {2, 2}, {12, 1}, {4, 4}, {3, 3}};
    for (int iter = 0; iter < 4000; ++iter) {
        Batch b;
        int B = 1 + (int)(rng() % (iter % 50 == 0 ? 300 : 24));
        b.cu.push_back(0);
        for (int i = 0; i < B; ++i) {
            int L = (rng() & 1) ? special[rng() % 19] : (int)(rng() % 3000);
            int S = (rng() % 5 == 0) ? 1 : 1 + (int)(rng() % 300);
            b.plens.push_back(L);
            b.cu.push_back(b.cu.back() + S);
        }
        if (iter % 3 == 0) {          // groups of consecutive traces with one context length
            b.groups.push_back(0);
            while (b.groups.back() < B) {
                int w = 1 + (int)(rng() % 5);
                int lo = b.groups.back(), hi = std::min(B, lo + w);
                for (int i = lo + 1; i < hi; ++i) b.plens[i] = b.plens[lo];
                b.groups.push_back(hi);
            }
        }
        const int *h = heads[rng() % 7];
        cs::AttnTune t = tune;
        t.force_split = (int)(rng() % 6);
        t.min_chunks = 1 + (int)(rng() % 8);
        t.target_items = 64 << (rng() % 5);
        char what[64];
        snprintf(what, sizeof what, "random batch %d", iter);
        check_plan(t, b, h[0], h[1], 0, what);
        check_plan(t, b, h[0], h[1], 1, what);
        if (iter % 200 == 0) check_library(draft, b, what);
    }
    // slices of the generation step's projections: every k-tile in exactly one slice of at most 24, at most 256
    // column groups (one arrival counter each) and no more than there are column tiles, planes sized for the slices
    for (int iter = 0; iter < 20000; ++iter) {
        int K = 64 * (1 + (int)(rng() % 600)), n_ct = 1 + (int)(rng() % 12000);
        if (iter < 8) {
            const int shapes[8][2] = {{1536, 128}, {1536, 96}, {1536, 1120}, {8960, 96}, {5120, 448}, {5120, 320}, {5120, 3456}, {27648, 320}};
            K = shapes[iter][0]; n_ct = shapes[iter][1];
        }
        int S = 0, nwg = 0;
        cs::dec_gemm_plan(K, n_ct, &S, &nwg);
        const int nk = K / 64;
        bool ok = S >= 1 && S <= nk && nwg >= 1 && nwg <= n_ct && nwg <= 256 && (nk + S - 1) / S <= 24;
        int covered = 0;
        for (int sl = 0; ok && sl < S; ++sl) {
            int k0 = (int)((long)sl * nk / S), k1 = (int)((long)(sl + 1) * nk / S);
            ok = k1 > k0 && k1 - k0 <= 24 && k0 == covered;
            covered = k1;
        }
        ok = ok && covered == nk;
        size_t pb = cs::dec_gemm_plane_bytes(K, n_ct);
        ok = ok && pb == (S > 1 ? (size_t)S * 32 * n_ct * 16 * 4 : 0);
        if (!ok) { printf("dec_gemm_plan(K=%d, n_ct=%d) -> S=%d nwg=%d planes=%zu\n", K, n_ct, S, nwg, pb); ++g_fail; }
    }
    if (g_fail) { printf("host_check: %d check(s) failed\n", g_fail); return 1; }
    printf("host_check: ok\n");
    return 0;
}
