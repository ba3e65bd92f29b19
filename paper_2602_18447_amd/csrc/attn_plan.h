// Work description of the attention kernels and the arithmetic that builds it, shared by the host planner
// (attn_plan.cpp: counts, the choice of the pieces, and a host twin of the list builder for checks on the CPU) and the
// device planner (attn_plan_kernel in attn_bf16.hip).  Plain integer code: no HIP types, so that it also compiles as
// ordinary C++ for a sanitizer build of the host side.
#pragma once
#include <stdint.h>

#if defined(__HIP__)
#define CS_HD __host__ __device__
#else
#define CS_HD
#endif

namespace cs {

// One item = one q-row tile of one (context unit, kv head) over one range of 64-key chunks.
// A context unit is a run of consecutive traces b0 .. b_end-1 that verify candidate steps on top of the same cached
// context (tree-structured drafting, Section 4.3: the candidates of one step); a unit of one trace is the plain case.
// The rows of a unit are all (suffix token, q head of the kv head's group) pairs of its traces, flattened token-major:
// row = (token - cu[b0]) * G + g.  Keys of a tile come as a list of 64-key chunks: first the chunks of the shared
// context (keys 0 .. L-1 through the block table of trace b0), then the chunks of the suffix keys its rows can see -
// the packed suffix tokens from the start of the trace that holds the tile's first row up to the tile's last token.
struct AttnItem {
    int32_t b0;           // first trace of the unit (owner of the context: block-table row, prefix length)
    int32_t c;            // kv head
    int32_t row0;         // first row of the tile in the unit's flattened row space
    int32_t chunk_begin;  // first chunk of the tile's chunk list (inclusive)
    int32_t chunk_end;    // last chunk (exclusive)
    int32_t part_slot;    // >= 0: write fp32 partials to this slot; -1: write the final output
    int32_t tile;         // index into the tile list
    int32_t b_end;        // one past the last trace of the unit
};
struct AttnTile {
    int32_t b0, c, row0;
    int32_t part_base;    // first partial slot of this tile
    int32_t n_splits;     // number of items covering this tile
    int32_t b_end;
    int32_t pad[2];
};

constexpr int ATTN_BM = 128;      // q rows per tile: 4 wavefronts x 32 rows
constexpr int ATTN_THREADS = 256;
constexpr int ATTN_BN = 64;       // keys per chunk
constexpr int ATTN_MAX_SPLIT = 32;

struct AttnTune {
    int target_items = 512;   // concurrent workgroup slots the planner assumes
    int min_chunks = 4;       // shortest piece of a tile the planner cuts (one-token batches: 4 is 2.6 % faster than 8)
    int force_split = 0;      // 0 = choose by the makespan estimate, 1..4 = fixed split factor, 5 = front-loaded pieces
    int kernel = 0;           // 0 = software-pipelined main loop; 1 = the register-staged main loop
};

// Host-side mirror of the planner's counting pass (same arithmetic as the device code).
struct AttnPlanCounts {
    int64_t n_tiles, n_items, n_part_slots, total_chunks;
    int64_t max_xcd_items;      // largest number of items any of the 8 XCDs gets
    int32_t chunks_per_item;
    int32_t equalize;           // 1: equal pieces per tile, 0: pieces of chunks_per_item, remainder last
};

CS_HD inline int plan_ceil_div(int a, int b) { return (a + b - 1) / b; }
CS_HD inline int plan_min(int a, int b) { return a < b ? a : b; }
CS_HD inline int plan_max(int a, int b) { return a > b ? a : b; }
CS_HD inline int plan_clamp(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// A context unit as the planner sees it.
struct AttnUnit {
    int b0, b_end;   // traces
    int L;           // cached context length (of trace b0)
    int S_tot;       // suffix tokens of all its traces
    int S_max;       // longest suffix among its traces
};
// Unit i of a batch.  group_start (may be null: every trace is its own unit) holds n_units + 1 trace indices;
// last_only plans (the last suffix position of each trace only) always take every trace as its own unit.
CS_HD inline AttnUnit plan_unit(const int32_t *cu, const int32_t *plens, const int32_t *group_start, int n_units, int i,
                                int B, int T, int max_L, int last_only) {
    AttnUnit u;
    if (group_start && !last_only) {
        u.b0 = plan_clamp(group_start[i], 0, B - 1);
        u.b_end = plan_clamp(group_start[i + 1], u.b0 + 1, B);
    } else {
        u.b0 = i;
        u.b_end = i + 1;
    }
    u.L = plan_clamp(plens[u.b0], 0, max_L);
    int c0 = plan_clamp(cu[u.b0], 0, T);
    u.S_tot = plan_max(plan_clamp(cu[u.b_end], 0, T) - c0, 0);
    u.S_max = 0;
    for (int b = u.b0; b < u.b_end; ++b)
        u.S_max = plan_max(u.S_max, plan_clamp(cu[b + 1], 0, T) - plan_clamp(cu[b], 0, T));
    return u;
}
// Offset, in suffix tokens from the unit's first token, at which the trace that holds token tok_rel starts.
CS_HD inline int plan_member_start(const int32_t *cu, int T, const AttnUnit &u, int tok_rel) {
    int base = plan_clamp(cu[u.b0], 0, T), s = 0;
    for (int b = u.b0; b < u.b_end; ++b) {
        int e = plan_clamp(cu[b + 1], 0, T) - base;
        if (tok_rel < e) return s;
        s = e;
    }
    return s;
}

// Every tile of a unit is cut into n_split pieces of `piece` chunks (the last piece takes what is
// left and may be empty for the unit's shorter tiles).  Two ways to choose the pieces:
//   equal pieces : n_split = ceil(nc / cpi), piece = ceil(nc / n_split);
//   front-loaded : piece = cpi, so that the first pieces are long and a short remainder follows.
struct UnitPlan {
    int n_qt;      // q-row tiles per kv head
    int n_split;   // pieces of every tile of this unit
    int nc_max;    // upper bound of the chunks of any of its tiles
    int piece;     // chunks per piece
};
CS_HD inline UnitPlan unit_plan(const AttnUnit &u, int G, int cpi, int equalize, int last_only) {
    UnitPlan p;
    p.n_qt = u.S_tot > 0 ? (last_only ? 1 : plan_ceil_div(G * u.S_tot, ATTN_BM)) : 0;
    // a tile that starts inside one trace and ends in a later one sees the first trace's tokens from its start
    int extra = (u.b_end - u.b0 > 1) ? ATTN_BM / G + 1 : 0;
    p.nc_max = plan_ceil_div(u.L, ATTN_BN) + plan_ceil_div(u.S_max + extra, ATTN_BN);
    int n = p.nc_max > cpi ? plan_ceil_div(p.nc_max, cpi) : 1;
    bool clamped = n > ATTN_MAX_SPLIT;
    p.n_split = clamped ? ATTN_MAX_SPLIT : n;
    p.piece = (equalize || clamped) ? plan_ceil_div(plan_max(p.nc_max, 1), p.n_split) : cpi;
    return p;
}
// Chunks of tile m of a unit: the context's chunks plus those of the suffix keys the tile's rows can see.
CS_HD inline int tile_chunks(const int32_t *cu, int T, const AttnUnit &u, int G, int m, int last_only) {
    int n_pc = plan_ceil_div(u.L, ATTN_BN);
    if (last_only) return n_pc + plan_ceil_div(u.S_tot, ATTN_BN);
    int r_last = plan_min(m * ATTN_BM + ATTN_BM - 1, G * u.S_tot - 1);
    int tok_lo = (m * ATTN_BM) / G, tok_hi = r_last / G;
    return n_pc + plan_ceil_div(tok_hi - plan_member_start(cu, T, u, tok_lo) + 1, ATTN_BN);
}
// XCD x takes the contiguous range of tiles [tile_lo[x], tile_lo[x+1]); the cuts are placed where the
// running sum of chunks (every tile of a unit counted with the unit's bound) passes x/8 of the total.
// A cut that falls inside (or at the end of) this unit's tiles is written here, together with the number
// of items in front of it: the tiles before it plus their pieces other than the first.
CS_HD inline void plan_xcd_starts(const UnitPlan &p, int Hkv, int tile_base, int rest_base, long long work_base,
                                  long long work_total, int *tile_lo, int *seg_base) {
    int my_tiles = Hkv * p.n_qt;
    if (my_tiles <= 0 || p.nc_max <= 0) return;
    long long work_end = work_base + (long long)my_tiles * p.nc_max;
    for (int x = 1; x < 8; ++x) {
        long long target = (x * work_total + 7) / 8;
        if (target > work_base && target <= work_end) {
            int j = (int)((target - work_base + p.nc_max - 1) / p.nc_max);   // 1 .. my_tiles
            tile_lo[x] = tile_base + j;
            seg_base[x] = tile_base + j + rest_base + j * (p.n_split - 1);
        }
    }
}

// Tiles and items of one unit.  tile_base / rest_base / slot_base: tiles, pieces other than the first,
// and partial slots of all earlier units.  The item list is built per XCD (workgroup id % 8 selects the XCD, each
// XCD takes a contiguous range of tiles so that the row tiles of one unit and kv head share an L2): first the
// first pieces of all its tiles, then all the other pieces.  Workgroups are dispatched in id order, so the long
// pieces start first and the short ones fill the gaps when slots free up (longest-first list scheduling).
CS_HD inline void plan_emit_unit(const int32_t *cu, int T, const AttnUnit &u, int G, int Hkv, const UnitPlan &p,
                                 int tile_base, int rest_base, int slot_base, const int *tile_lo, const int *seg_base,
                                 int last_only, int max_tiles, int max_items, AttnTile *tiles, AttnItem *items) {
    for (int c = 0; c < Hkv; ++c)
        for (int m = 0; m < p.n_qt; ++m) {
            int local = c * p.n_qt + m;
            int ti = tile_base + local;
            int pbase = p.n_split > 1 ? slot_base + local * p.n_split : -1;
            int row0 = last_only ? (u.S_tot - 1) * G : m * ATTN_BM;
            if (ti < max_tiles) {
                AttnTile t;
                t.b0 = u.b0; t.c = c; t.row0 = row0; t.part_base = pbase; t.n_splits = p.n_split; t.b_end = u.b_end;
                t.pad[0] = t.pad[1] = 0;
                tiles[ti] = t;
            }
            int x = 7;
            while (x > 0 && tile_lo[x] > ti) --x;
            int lo = tile_lo[x], hi = tile_lo[x + 1];
            int rest_before = rest_base + local * (p.n_split - 1);   // other pieces of all earlier tiles
            int rest_lo = seg_base[x] - lo;                          // the same count at the start of the range
            int nc = tile_chunks(cu, T, u, G, m, last_only);
            for (int sp = 0; sp < p.n_split; ++sp) {
                int idx = sp == 0 ? seg_base[x] + (ti - lo) : seg_base[x] + (hi - lo) + (rest_before - rest_lo) + sp - 1;
                if (idx < 0 || idx >= max_items || pbase + sp >= max_items) continue;
                AttnItem it;
                it.b0 = u.b0; it.c = c; it.row0 = row0;
                it.chunk_begin = plan_min(sp * p.piece, nc);
                it.chunk_end = sp == p.n_split - 1 ? nc : plan_min((sp + 1) * p.piece, nc);
                it.part_slot = p.n_split > 1 ? pbase + sp : -1;
                it.tile = ti; it.b_end = u.b_end;
                items[idx] = it;
            }
        }
}

// ---- host planner (attn_plan.cpp) ----
// Choice of the pieces and the resulting counts.  h_group_start: null, or n_units + 1 trace indices (see plan_unit).
AttnPlanCounts attn_plan_counts(const AttnTune &tune, const int32_t *h_cu, const int32_t *h_plens, int B, int T,
                                const int32_t *h_group_start, int n_units, int G, int Hkv, int last_only);
// Upper bounds used to size the workspace for any batch of up to max_T tokens in max_B traces.
void attn_plan_capacity(const AttnTune &tune, int64_t max_T, int64_t max_B, int G, int Hkv, int64_t *max_tiles,
                        int64_t *max_items);
// Host twin of attn_plan_kernel: the same lists from the same functions, for checks on the CPU.
// counts[0] = tiles, counts[1] = items, counts[2 + x] = first item of XCD x (x = 0..8).
void attn_plan_host(const int32_t *cu, const int32_t *plens, const int32_t *group_start, int n_units, int B, int T,
                    int max_L, int G, int Hkv, int cpi, int equalize, int last_only, int max_tiles, int max_items,
                    AttnTile *tiles, AttnItem *items, int32_t *counts);

}  // namespace cs
