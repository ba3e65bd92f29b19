// Grouped-query causal attention of suffix queries over the paged prefix cache plus the suffix's own
// keys, bf16 operands on the gfx950 matrix cores, fp32 online softmax.
//
// Decomposition.  All G query heads that share one kv head are folded into the row dimension: a
// trace with S suffix tokens contributes G*S rows per kv head, flattened position-major
// (row = t*G + g), cut into tiles of 128 rows; one wavefront owns 32 rows.  The key range of a tile
// is cut into 64-key chunks, and - to balance ragged batches and fill 256 CUs - into several work
// items whose partial (max, sum, unnormalised output) results are merged by a second kernel in a
// fixed order.
//
// Per chunk a workgroup stages K as [key][hd] and V transposed as [hd][key] in LDS.  Scores are
// computed transposed, S^T = K . Q^T (keys on MFMA rows, queries on columns), so each lane owns one
// query column: the running max / sum and the rescale of the output accumulator are lane-local
// apart from one exchange between lane l and l+32.  The rows of each 32-key block are fed to the
// MFMA in a permuted order chosen so that the probabilities a lane ends up holding are 8
// consecutive keys per k-step: they are used as the B operand of O^T += V^T . P^T straight from
// registers, and the matching A operand is a single 16-byte read of the transposed V tile.
#include "kernels.h"
#include <algorithm>
#include <cmath>
#include <queue>
#include <vector>

namespace cs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int HD = 128;
constexpr int K_STRIDE = 136;             // elements per K row in LDS (128 + 8 pad = 272 bytes)
constexpr int VT_STRIDE = 72;             // elements per V^T row in LDS (64 + 8 pad = 144 bytes)
constexpr int K_TILE = ATTN_BN * K_STRIDE;
constexpr int VT_TILE = HD * VT_STRIDE;
constexpr int ATTN_STAGE = K_TILE + VT_TILE;   // elements per stage
constexpr int ATTN_SMEM_BYTES = 2 * ATTN_STAGE * 2;

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- planning: identical arithmetic on host (counts only) and device (counts + lists) ----
// Every tile of a trace is cut into n_split pieces of `piece` chunks (the last piece takes what is
// left and may be empty for the trace's shorter tiles).  Two ways to choose the pieces:
//   equal pieces : n_split = ceil(nc / cpi), piece = ceil(nc / n_split);
//   front-loaded : piece = cpi, so that the first pieces are long and a short remainder follows.
// The item list is built per XCD (workgroup id % 8 selects the XCD, each XCD takes a contiguous range
// of tiles so that the row tiles of one trace and kv head share an L2): first the first pieces of all
// its tiles, then all the other pieces.  Workgroups are dispatched in id order, so the long pieces
// start first and the short ones fill the gaps when slots free up (longest-first list scheduling).
constexpr int ATTN_MAX_SPLIT = 32;
struct TracePlan {
    int n_qt;      // q-row tiles per kv head
    int n_split;   // pieces of every tile of this trace
    int nc_max;    // chunks of the trace's last tile
    int piece;     // chunks per piece
};
// last_only: the plan covers the last suffix position of each trace only (its G rows per kv head form
// one tile that starts at row (S-1)*G), which is all the last decoder layer has to produce.
__host__ __device__ inline TracePlan trace_plan(int L, int S, int G, int cpi, int equalize, int last_only) {
    TracePlan p;
    p.n_qt = S > 0 ? (last_only ? 1 : ceil_div(G * S, ATTN_BM)) : 0;
    p.nc_max = ceil_div(L + S, ATTN_BN);
    int n = p.nc_max > cpi ? ceil_div(p.nc_max, cpi) : 1;
    bool clamped = n > ATTN_MAX_SPLIT;
    p.n_split = clamped ? ATTN_MAX_SPLIT : n;
    p.piece = (equalize || clamped) ? ceil_div(max(p.nc_max, 1), p.n_split) : cpi;
    return p;
}
__host__ __device__ inline int tile_chunks(int L, int S, int G, int m) {
    int r_last = min(m * ATTN_BM + ATTN_BM - 1, G * S - 1);
    return ceil_div(L + r_last / G + 1, ATTN_BN);
}
// XCD x takes the contiguous range of tiles [tile_lo[x], tile_lo[x+1]); the cuts are placed where the
// running sum of chunks (every tile of a trace counted with the trace's longest) passes x/8 of the total.
// A cut that falls inside (or at the end of) this trace's tiles is written here, together with the number
// of items in front of it: the tiles before it plus their pieces other than the first.
__host__ __device__ inline void plan_xcd_starts(const TracePlan &p, int Hkv, int tile_base, int rest_base,
                                                long long work_base, long long work_total, int *tile_lo,
                                                int *seg_base) {
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

// Tiles and items of one trace.  tile_base / rest_base / slot_base: tiles, pieces other than the first,
// and partial slots of all earlier traces.
__host__ __device__ inline void plan_emit_trace(int b, int L, int S, int G, int Hkv, const TracePlan &p, int tile_base,
                                                int rest_base, int slot_base, const int *tile_lo, const int *seg_base,
                                                int last_only, int max_tiles, int max_items, AttnTile *tiles,
                                                AttnItem *items) {
    for (int c = 0; c < Hkv; ++c)
        for (int m = 0; m < p.n_qt; ++m) {
            int local = c * p.n_qt + m;
            int ti = tile_base + local;
            int pbase = p.n_split > 1 ? slot_base + local * p.n_split : -1;
            int row0 = last_only ? (S - 1) * G : m * ATTN_BM;
            if (ti < max_tiles) {
                AttnTile t;
                t.b = b; t.c = c; t.row0 = row0; t.part_base = pbase; t.n_splits = p.n_split;
                t.pad[0] = t.pad[1] = t.pad[2] = 0;
                tiles[ti] = t;
            }
            int x = 7;
            while (x > 0 && tile_lo[x] > ti) --x;
            int lo = tile_lo[x], hi = tile_lo[x + 1];
            int rest_before = rest_base + local * (p.n_split - 1);   // other pieces of all earlier tiles
            int rest_lo = seg_base[x] - lo;                          // the same count at the start of the range
            int nc = last_only ? p.nc_max : tile_chunks(L, S, G, m);
            for (int sp = 0; sp < p.n_split; ++sp) {
                int idx = sp == 0 ? seg_base[x] + (ti - lo) : seg_base[x] + (hi - lo) + (rest_before - rest_lo) + sp - 1;
                if (idx < 0 || idx >= max_items || pbase + sp >= max_items) continue;
                AttnItem it;
                it.b = b; it.c = c; it.row0 = row0;
                it.chunk_begin = min(sp * p.piece, nc);
                it.chunk_end = sp == p.n_split - 1 ? nc : min((sp + 1) * p.piece, nc);
                it.part_slot = p.n_split > 1 ? pbase + sp : -1;
                it.tile = ti; it.pad = 0;
                items[idx] = it;
            }
        }
}

void attn_plan_capacity(const AttnTune &tune, int64_t max_T, int64_t max_B, int G, int Hkv, int64_t *max_tiles,
                        int64_t *max_items) {
    int64_t tiles = (int64_t)Hkv * ((G * max_T + ATTN_BM - 1) / ATTN_BM + max_B);
    *max_tiles = tiles;
    *max_items = 3 * tiles + 4 * tune.target_items;     // candidates that need more are not considered
}

namespace {
struct TraceShape { int tiles, nc; };
struct Candidate { int cpi, equalize; };

// Items, partial slots and the largest per-XCD item count of a candidate; lens (optional) receives the
// per-XCD piece lengths in dispatch order.  Same arithmetic as the device planner.
void candidate_counts(const std::vector<TraceShape> &tr, Candidate cd, int64_t n_tiles, int64_t work_total,
                      AttnPlanCounts *r, std::vector<int> *lens /* [8] */) {
    r->n_items = 0; r->n_part_slots = 0; r->max_xcd_items = 0;
    int tile_lo[9] = {0}, seg_base[9] = {0};
    int tile_base = 0, rest_base = 0;
    long long work_base = 0;
    std::vector<TracePlan> plans;
    plans.reserve(tr.size());
    for (const TraceShape &t : tr) {
        TracePlan p;
        p.n_qt = t.tiles; p.nc_max = t.nc;       // n_qt holds Hkv * n_qt here (Hkv = 1 below)
        int n = t.nc > cd.cpi ? ceil_div(t.nc, cd.cpi) : 1;
        bool clamped = n > ATTN_MAX_SPLIT;
        p.n_split = clamped ? ATTN_MAX_SPLIT : n;
        p.piece = (cd.equalize || clamped) ? ceil_div(std::max(t.nc, 1), p.n_split) : cd.cpi;
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
    std::vector<int> rest_lens[8];
    int ti = 0;
    for (size_t i = 0; i < tr.size(); ++i)
        for (int j = 0; j < tr[i].tiles; ++j, ++ti) {
            int x = 7;
            while (x > 0 && tile_lo[x] > ti) --x;
            const TracePlan &p = plans[i];
            lens[x].push_back(std::min(p.piece, p.nc_max));
            for (int sp = 1; sp < p.n_split; ++sp)
                rest_lens[x].push_back(std::max(0, std::min(p.piece, p.nc_max - sp * p.piece)));
        }
    for (int x = 0; x < 8; ++x) lens[x].insert(lens[x].end(), rest_lens[x].begin(), rest_lens[x].end());
}

// Makespan of longest-first list scheduling on slots/8 workgroup slots per XCD, in chunk-times.
double simulate(const std::vector<int> *lens, int slots) {
    int per_xcd = std::max(1, slots / 8);
    double worst = 0;
    for (int x = 0; x < 8; ++x) {
        std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
        for (int i = 0; i < per_xcd; ++i) free_at.push(0.0);
        double end = 0;
        for (int len : lens[x]) {
            double t0 = free_at.top();
            free_at.pop();
            double t1 = t0 + len + 1.5;          // 1.5: loading q, writing the result
            free_at.push(t1);
            end = std::max(end, t1);
        }
        worst = std::max(worst, end);
    }
    return worst;
}
}  // namespace

// Choice of the pieces: equal pieces with a split factor 1..4 of the average tile, or front-loaded
// pieces of 1.07x / 1.2x the per-slot share of all chunks; the candidate with the smallest simulated
// makespan (+ 8 chunk-times for the merge pass when anything is split) wins.
AttnPlanCounts attn_plan_counts(const AttnTune &tune, const int32_t *h_cu, const int32_t *h_plens, int B, int G, int Hkv,
                                int last_only) {
    const int g_target_items = tune.target_items, g_min_chunks = tune.min_chunks, g_force_split = tune.force_split;
    AttnPlanCounts r = {};
    std::vector<TraceShape> tr;
    tr.reserve(B);
    int64_t total = 0, n_tiles = 0;
    int nc_longest = 0;
    for (int b = 0; b < B; ++b) {
        int S = h_cu[b + 1] - h_cu[b], L = h_plens[b];
        TracePlan p = trace_plan(L, S, G, 1 << 30, 1, last_only);
        tr.push_back({Hkv * p.n_qt, p.nc_max});
        total += (int64_t)Hkv * p.n_qt * p.nc_max;
        n_tiles += (int64_t)Hkv * p.n_qt;
        if (p.n_qt > 0) nc_longest = std::max(nc_longest, p.nc_max);
    }
    r.n_tiles = n_tiles;
    r.total_chunks = total;
    double avg = n_tiles > 0 ? (double)total / (double)n_tiles : 1.0;
    int64_t slots = g_target_items;
    int64_t cap_items = 3 * n_tiles + 4 * slots;
    std::vector<Candidate> cands;
    auto equal_cpi = [&](int sp) { return sp == 1 ? (1 << 30) : std::max<int>(g_min_chunks, (int)((avg + sp - 1) / sp)); };
    auto front_cpi = [&](double f) { return std::max<int>(g_min_chunks, (int)std::ceil(f * (double)total / (double)slots)); };
    if (g_force_split >= 1 && g_force_split <= 4) cands.push_back({equal_cpi(g_force_split), 1});
    else if (g_force_split == 5) cands.push_back({front_cpi(1.07), 0});
    else {
        for (int sp = 1; sp <= 4; ++sp) {
            if (sp > 1 && avg / sp < g_min_chunks) break;
            cands.push_back({equal_cpi(sp), 1});
        }
        for (double f : {1.07, 1.2})
            if (front_cpi(f) < nc_longest) cands.push_back({front_cpi(f), 0});
    }
    double best = 1e300;
    Candidate pick = {1 << 30, 1};
    for (size_t i = 0; i < cands.size(); ++i) {
        AttnPlanCounts c = {};
        std::vector<int> lens[8];
        candidate_counts(tr, cands[i], n_tiles, total, &c, lens);
        if (c.n_items > cap_items && cands.size() > 1 && cands[i].cpi != (1 << 30)) continue;
        double est = simulate(lens, (int)slots) + (c.n_part_slots > 0 ? 8.0 : 0.0);
        if (est < best) { best = est; pick = cands[i]; }
    }
    r.chunks_per_item = pick.cpi;
    r.equalize = pick.equalize;
    candidate_counts(tr, pick, n_tiles, total, &r, nullptr);
    return r;
}

// counts[0] = tiles, counts[1] = items, counts[2 + x] = first item of XCD x (x = 0..8; [10] = items)
__global__ __launch_bounds__(256) void attn_plan_kernel(const int32_t *__restrict__ cu,
                                                         const int32_t *__restrict__ plens, int B, int T, int max_L,
                                                         int G, int Hkv, int cpi, int equalize, int last_only,
                                                         int max_tiles, int max_items, AttnTile *__restrict__ tiles,
                                                         AttnItem *__restrict__ items, int32_t *__restrict__ counts) {
    __shared__ int s_tiles[257], s_rest[257], s_slots[257];
    __shared__ long long s_work[257];
    __shared__ int carry[3];
    __shared__ long long carry_work;
    __shared__ int tile_lo[9], seg_base[9];
    int tid = threadIdx.x;
    // pass 0 adds up tiles and chunks (the XCD cuts depend on the totals), pass 1 places the cuts and
    // finds where each XCD's items start, pass 2 writes the lists
    long long work_total = 0;
    for (int pass = 0; pass < 3; ++pass) {
        if (tid == 0) { carry[0] = carry[1] = carry[2] = 0; carry_work = 0; }
        __syncthreads();
        for (int base = 0; base < B; base += 256) {
            int b = base + tid;
            int L = 0, S = 0;
            TracePlan p = {0, 1, 0, 1};
            if (b < B) {
                int c0 = min(max(cu[b], 0), T), c1 = min(max(cu[b + 1], 0), T);
                S = max(c1 - c0, 0);
                L = min(max(plens[b], 0), max_L);
                p = trace_plan(L, S, G, cpi, equalize, last_only);
            }
            int my_tiles = Hkv * p.n_qt;
            s_tiles[tid + 1] = my_tiles;
            s_rest[tid + 1] = my_tiles * (p.n_split - 1);
            s_slots[tid + 1] = p.n_split > 1 ? my_tiles * p.n_split : 0;
            s_work[tid + 1] = (long long)my_tiles * p.nc_max;
            __syncthreads();
            if (tid == 0) {  // serial exclusive scan of the entries of this batch of traces (at most 256)
                s_tiles[0] = carry[0];
                s_rest[0] = carry[1];
                s_slots[0] = carry[2];
                s_work[0] = carry_work;
                int n = min(256, B - base);
                for (int i = 1; i <= n; ++i) {
                    s_tiles[i] += s_tiles[i - 1];
                    s_rest[i] += s_rest[i - 1];
                    s_slots[i] += s_slots[i - 1];
                    s_work[i] += s_work[i - 1];
                }
                s_tiles[256] = s_tiles[n]; s_rest[256] = s_rest[n]; s_slots[256] = s_slots[n]; s_work[256] = s_work[n];
            }
            __syncthreads();
            int tile_base = s_tiles[tid], rest_base = s_rest[tid], slot_base = s_slots[tid];
            if (pass == 1 && b < B)
                plan_xcd_starts(p, Hkv, tile_base, rest_base, s_work[tid], work_total, tile_lo, seg_base);
            if (pass == 2 && b < B)
                plan_emit_trace(b, L, S, G, Hkv, p, tile_base, rest_base, slot_base, tile_lo, seg_base, last_only,
                                max_tiles, max_items, tiles, items);
            __syncthreads();
            if (tid == 0) { carry[0] = s_tiles[256]; carry[1] = s_rest[256]; carry[2] = s_slots[256]; carry_work = s_work[256]; }
            __syncthreads();
        }
        if (pass == 0) {
            work_total = carry_work;
            if (tid < 9) { tile_lo[tid] = 0; seg_base[tid] = 0; }
        }
        if (pass == 1 && tid == 0) { tile_lo[8] = carry[0]; seg_base[8] = carry[0] + carry[1]; }
        __syncthreads();
    }
    if (tid == 0) {
        counts[0] = min(carry[0], max_tiles);
        counts[1] = min(carry[0] + carry[1], max_items);
    }
    if (tid < 9) counts[2 + tid] = min(seg_base[tid], max_items);
}

hipError_t launch_attn_plan(const int32_t *cu, const int32_t *plens, int B, int T, int max_L, int G, int Hkv,
                            int chunks_per_item, int equalize, int last_only, int max_tiles, int max_items,
                            AttnTile *tiles, AttnItem *items, int32_t *counts, hipStream_t s) {
    attn_plan_kernel<<<1, 256, 0, s>>>(cu, plens, B, T, max_L, G, Hkv, chunks_per_item, equalize, last_only,
                                       max_tiles, max_items, tiles, items, counts);
    return hipGetLastError();
}

// Four consecutive output values in the requested activation format: 1 = bf16, 2 = bf16 hi at o and the
// bf16 remainder row_w elements further, 3 = IEEE half.
__device__ __forceinline__ void store_out4(bf16 *o, size_t row_w, int fmt, const float *v) {
    if (fmt == 3) {
        union { __half h[4]; uint2 u; } ph;
#pragma unroll
        for (int j = 0; j < 4; ++j) ph.h[j] = to_half_sat(v[j]);
        *reinterpret_cast<uint2 *>(o) = ph.u;
        return;
    }
    union { bf16 h[4]; uint2 u; } pk, pl;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        pk.h[j] = __float2bfloat16(v[j]);
        pl.h[j] = __float2bfloat16(v[j] - __bfloat162float(pk.h[j]));
    }
    *reinterpret_cast<uint2 *>(o) = pk.u;
    if (fmt == 2) *reinterpret_cast<uint2 *>(o + row_w) = pl.u;
}

// ---- the attention kernel ----
// PRECISE: q, the suffix keys / values and the probabilities are each carried as two bf16 terms
// (hi + lo); products hi*hi, hi*lo and lo*hi are accumulated (lo*lo is below fp32 resolution of the
// sum).  Cached prefix keys / values are exact bf16 values and need no second term.  Used for the
// first layer(s), where score noise from rounding q and k is amplified by every later layer.
template <bool PRECISE>
__global__ __launch_bounds__(ATTN_THREADS, PRECISE ? 1 : 2) void attn_bf16_kernel(AttnArgs a, const AttnItem *__restrict__ items,
                                                                  const int32_t *__restrict__ counts, int n_items_host,
                                                                  float *__restrict__ part_o,
                                                                  float *__restrict__ part_ml) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __bf16 *smem = reinterpret_cast<__bf16 *>(smem_raw);
    constexpr int STAGE = PRECISE ? 2 * ATTN_STAGE : ATTN_STAGE;   // PRECISE: [K | Vt | K_lo | Vt_lo]

    // workgroup id % 8 is the XCD; each XCD walks its own range of the item list in order
    int n_items = min(counts[1], n_items_host);
    int xcd = blockIdx.x & 7;
    int it_idx = counts[2 + xcd] + (blockIdx.x >> 3);
    if (it_idx >= min(counts[3 + xcd], n_items)) return;
    AttnItem item = items[it_idx];

    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (item.chunk_begin >= item.chunk_end) {
        // a split that received no chunks: mark its rows as "nothing seen" for the merge
        if (item.part_slot >= 0 && tid < ATTN_BM) {
            size_t row_slot = (size_t)item.part_slot * ATTN_BM + tid;
            part_ml[row_slot * 2] = -INFINITY;
            part_ml[row_slot * 2 + 1] = 0.f;
        }
        return;
    }
    int half = lane >> 5, lq = lane & 31;
    int G = a.Hq / a.Hkv;
    int b = min(max(item.b, 0), a.B - 1), c = min(max(item.c, 0), a.Hkv - 1);
    int cu_b = min(max(a.cu[b], 0), a.T - 1);
    int S = min(max(a.cu[b + 1] - cu_b, 1), a.T - cu_b);
    int L = min(max(a.plens[b], 0), a.max_blocks * 16);
    int n_rows = G * S;

    // Four wavefronts of 32 query rows each.  A wave whose rows all lie past the end of the trace
    // still loads and synchronises with the others but skips the matrix work.
    int wave_row0 = item.row0 + wave * 32;
    bool wave_active = wave_row0 < n_rows;             // wave-uniform
    int r = wave_row0 + lq;
    bool row_valid = r < n_rows;
    int rc = min(r, n_rows - 1);
    int t = rc / G, g = rc - t * G;
    int limit = L + t;                                          // last visible key of this lane's query
    int wave_first_limit = L + min(wave_row0, n_rows - 1) / G;

    const bf16 *q_row = reinterpret_cast<const bf16 *>(a.q) + ((size_t)(cu_b + t) * a.Hq + c * G + g) * HD;
    bf16x8 qf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(q_row + ks * 16 + half * 8);
    bf16x8 qf_lo[PRECISE ? 8 : 1];
    if constexpr (PRECISE) {
        const bf16 *ql_row = reinterpret_cast<const bf16 *>(a.q_lo) + ((size_t)(cu_b + t) * a.Hq + c * G + g) * HD;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf_lo[ks] = *reinterpret_cast<const bf16x8 *>(ql_row + ks * 16 + half * 8);
    }

    const bf16 *kp = reinterpret_cast<const bf16 *>(a.k_pages), *vp = reinterpret_cast<const bf16 *>(a.v_pages);
    const bf16 *ks_ = reinterpret_cast<const bf16 *>(a.ksuf), *vs_ = reinterpret_cast<const bf16 *>(a.vsuf);

    // Loader roles (every thread stages 4 K vectors and 4 V vectors per chunk).
    // K: load i of a thread takes key slot tid/16 of page i of the chunk, 16-byte vector tid%16.
    // V: a thread takes keys 4*v_kq..+3 (one page) x hd 8*v_g..+7, transposed on the way into LDS.
    int k_dst[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) k_dst[i] = ((tid >> 4) + 16 * i) * K_STRIDE + (tid & 15) * 8;
    int v_kq = lane & 15, v_g = wave * 4 + (lane >> 4);
    int v_dst = K_TILE + (8 * v_g) * VT_STRIDE + 4 * v_kq;
    const int32_t *bt = a.block_table + (size_t)b * a.max_blocks;        // wave-uniform
    const size_t page_elems = (size_t)a.Hkv * 16 * HD;
    const int k_in_page = (c * 16 + (tid >> 4)) * HD + (tid & 15) * 8;
    const int v_in_page = (c * 16 + 4 * (v_kq & 3)) * HD + v_g * 8;
    const int v_page_sel = v_kq >> 2;
    const int max_page = a.max_blocks - 1;

    // Physical block ids of the 4 pages of a chunk, fetched two chunks ahead: lanes 0..3 each load one
    // table entry into ids_v, the ids are broadcast with readlane right before the chunk's loads.
    int ids_v = 0;
    int ids[4];
    auto fetch_ids = [&](int ch) {
        int pg = min(4 * ch + (lane & 3), max_page);
        ids_v = bt[pg];
    };
    auto bcast_ids = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            ids[i] = min(max(__builtin_amdgcn_readlane(ids_v, i), 0), a.n_blocks - 1);
    };
    // Row of key j for chunks that touch the suffix or the end of the trace: page row for j < L, else
    // suffix row (clamped to the last one: such keys are masked for every query).
    auto row_general = [&](const bf16 *pages, const bf16 *suf, int j) -> const bf16 * {
        int jp = min(j, max(L - 1, 0));
        int id = min(max(bt[min(jp >> 4, max_page)], 0), a.n_blocks - 1);
        const bf16 *pp = pages + ((size_t)id * a.Hkv + c) * 16 * HD + (jp & 15) * HD;
        int ts = min(max(j - L, 0), S - 1);
        const bf16 *sp = suf + ((size_t)(cu_b + ts) * a.Hkv + c) * HD;
        return j < L ? pp : sp;
    };

    u32x4 k_reg[4], v_reg[4];
    u32x4 kl_reg[PRECISE ? 4 : 1], vl_reg[PRECISE ? 4 : 1];
    const bf16 *ksl_ = reinterpret_cast<const bf16 *>(a.ksuf_lo), *vsl_ = reinterpret_cast<const bf16 *>(a.vsuf_lo);
    // lo term of key / value row j: zero for cached rows, the lo plane of the suffix otherwise
    auto load_lo = [&](const bf16 *suf_lo, int j, int vec_off) -> u32x4 {
        u32x4 z = {0u, 0u, 0u, 0u};
        if (j < L) return z;
        int ts = min(j - L, S - 1);
        return *reinterpret_cast<const u32x4 *>(suf_lo + ((size_t)(cu_b + ts) * a.Hkv + c) * HD + vec_off);
    };
    auto load_chunk = [&](int ch) {
        int j0 = ch * ATTN_BN;
        if (j0 + ATTN_BN <= L) {          // uniform: the whole chunk lies in the cached prefix
#pragma unroll
            for (int i = 0; i < 4; ++i)
                k_reg[i] = *reinterpret_cast<const u32x4 *>(kp + (size_t)ids[i] * page_elems + k_in_page);
            int vid = v_page_sel == 0 ? ids[0] : v_page_sel == 1 ? ids[1] : v_page_sel == 2 ? ids[2] : ids[3];
            const bf16 *vb = vp + (size_t)vid * page_elems + v_in_page;
#pragma unroll
            for (int i = 0; i < 4; ++i) v_reg[i] = *reinterpret_cast<const u32x4 *>(vb + i * HD);
        } else {
            const bf16 *kr[4], *vr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                kr[i] = row_general(kp, ks_, j0 + (tid >> 4) + 16 * i) + (tid & 15) * 8;
                vr[i] = row_general(vp, vs_, j0 + 4 * v_kq + i) + v_g * 8;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                k_reg[i] = *reinterpret_cast<const u32x4 *>(kr[i]);
                v_reg[i] = *reinterpret_cast<const u32x4 *>(vr[i]);
            }
            if constexpr (PRECISE) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    kl_reg[i] = load_lo(ksl_, j0 + (tid >> 4) + 16 * i, (tid & 15) * 8);
                    vl_reg[i] = load_lo(vsl_, j0 + 4 * v_kq + i, v_g * 8);
                }
            }
        }
    };
    auto store_tiles = [&](__bf16 *base, const u32x4 (&kr)[4], const u32x4 (&vr)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4 *>(base + k_dst[i]) = kr[i];
        // 4 keys x 8 hd  ->  8 rows of 4 keys
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint2 lo, hi;
            // one byte permute per output word (low halves of two keys, high halves of two keys)
            lo.x = __builtin_amdgcn_perm(vr[1][d], vr[0][d], 0x05040100u);
            lo.y = __builtin_amdgcn_perm(vr[3][d], vr[2][d], 0x05040100u);
            hi.x = __builtin_amdgcn_perm(vr[1][d], vr[0][d], 0x07060302u);
            hi.y = __builtin_amdgcn_perm(vr[3][d], vr[2][d], 0x07060302u);
            *reinterpret_cast<uint2 *>(base + v_dst + (2 * d) * VT_STRIDE) = lo;
            *reinterpret_cast<uint2 *>(base + v_dst + (2 * d + 1) * VT_STRIDE) = hi;
        }
    };
    // ch: the chunk held in the registers (its lo tiles exist only if it touches the suffix)
    auto store_chunk = [&](int stage, int ch) {
        __bf16 *base = smem + stage * STAGE;
        store_tiles(base, k_reg, v_reg);
        if constexpr (PRECISE) {
            if (ch * ATTN_BN + ATTN_BN > L) store_tiles(base + ATTN_STAGE, kl_reg, vl_reg);
        }
    };

    f32x16 acc_o[4];
#pragma unroll
    for (int hb = 0; hb < 4; ++hb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[hb][e] = 0.f;
    float m_run = -INFINITY, m_ref = -INFINITY, l_run = 0.f;   // true max, exponent reference, sum (vs m_ref)
    const float sc = a.scale * 1.44269504088896340736f;   // scores in log2 units

    // K operand row (key) for MFMA row lq, see the header comment: pi(m)
    int pi_m = 16 * (lq >> 4) + 8 * ((lq >> 2) & 1) + 4 * ((lq >> 3) & 1) + (lq & 3);
    int k_frag = pi_m * K_STRIDE + half * 8;
    int v_frag = K_TILE + lq * VT_STRIDE + half * 8;

    int ch0 = item.chunk_begin, ch1 = item.chunk_end;
    fetch_ids(ch0);
    bcast_ids();
    load_chunk(ch0);
    fetch_ids(ch0 + 1);
    store_chunk(0, ch0);      // waits for every load issued so far, the Q fragments included
    __syncthreads();
    for (int ch = ch0; ch < ch1; ++ch) {
        int stage = (ch - ch0) & 1;
        bool more = ch + 1 < ch1;
        if (more) {
            bcast_ids();            // ids of chunk ch+1, fetched during the previous iteration
            load_chunk(ch + 1);
            fetch_ids(ch + 2);
        }
        // keep the consumers of these loads (the LDS stores below) behind the MFMA work of this chunk
        __builtin_amdgcn_sched_barrier(0);
        const __bf16 *base = smem + stage * STAGE;
        const bool has_lo = PRECISE && (ch * ATTN_BN + ATTN_BN > L);   // uniform

        if (wave_active) {
            f32x16 acc_s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc_s[kb][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    bf16x8 kf = *reinterpret_cast<const bf16x8 *>(base + kb * 32 * K_STRIDE + k_frag + ks * 16);
                    acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[kb], 0, 0, 0);
                    if constexpr (PRECISE)
                        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf_lo[ks], acc_s[kb], 0, 0, 0);
                }
            if (has_lo) {
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        bf16x8 kf = *reinterpret_cast<const bf16x8 *>(base + ATTN_STAGE + kb * 32 * K_STRIDE + k_frag + ks * 16);
                        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[kb], 0, 0, 0);
                    }
            }
            // register e of block kb holds key  ch*64 + 32*kb + 16*(e>>3) + 8*half + (e&7)
            if (ch * ATTN_BN + ATTN_BN - 1 > wave_first_limit) {      // wave-uniform: causal mask needed
                int key0 = ch * ATTN_BN + 8 * half;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (key0 + 32 * kb + 16 * (e >> 3) + (e & 7) > limit) acc_s[kb][e] = -INFINITY;
            }
            float mloc = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) mloc = fmaxf(mloc, acc_s[kb][e]);
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
            float m_new = fmaxf(m_run, mloc * sc);     // true running max, log2 units
            m_run = m_new;
            // Lazy rescale: the exponent reference m_ref only follows the running max when some query of
            // the wave has moved more than 8 (a factor 256) above it; until then probabilities may exceed
            // 1, which bf16 / fp32 hold without loss, and the accumulators need no per-chunk rescale.
            if (__builtin_amdgcn_ballot_w64(m_new > m_ref + 8.0f) != 0) {
                float off_old = (m_ref == -INFINITY) ? 0.f : m_ref;
                float off_new = (m_new == -INFINITY) ? 0.f : m_new;
                float alpha = __builtin_amdgcn_exp2f(off_old - off_new);
                m_ref = m_new;
                l_run *= alpha;
#pragma unroll
                for (int hb = 0; hb < 4; ++hb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc_o[hb][e] *= alpha;
            }
            float neg_off = (m_ref == -INFINITY) ? 0.f : -m_ref;
            float psum = 0.f;
            bf16x8 pf[2][2];
            bf16x8 pf_lo[PRECISE ? 2 : 1][2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float p = __builtin_amdgcn_exp2f(fmaf(acc_s[kb][e], sc, neg_off));
                    psum += p;
                    __bf16 ph = (__bf16)p;
                    pf[kb][e >> 3][e & 7] = ph;
                    if constexpr (PRECISE) pf_lo[kb][e >> 3][e & 7] = (__bf16)(p - (float)ph);
                }
            l_run += psum;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int hb = 0; hb < 4; ++hb) {
                        bf16x8 vf = *reinterpret_cast<const bf16x8 *>(base + v_frag + hb * 32 * VT_STRIDE + kb * 32 + s2 * 16);
                        acc_o[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][s2], acc_o[hb], 0, 0, 0);
                        if constexpr (PRECISE)
                            acc_o[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf_lo[kb][s2], acc_o[hb], 0, 0, 0);
                    }
            if (has_lo) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                        for (int hb = 0; hb < 4; ++hb) {
                            bf16x8 vf = *reinterpret_cast<const bf16x8 *>(base + ATTN_STAGE + v_frag + hb * 32 * VT_STRIDE + kb * 32 + s2 * 16);
                            acc_o[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][s2], acc_o[hb], 0, 0, 0);
                        }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) store_chunk(stage ^ 1, ch + 1);
        __syncthreads();
    }

    float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    // acc_o[hb][e]: hd = 32*hb + 8*(e>>2) + 4*half + (e&3), query = lq
    if (item.part_slot < 0) {
        if (row_valid) {
            float inv = 1.0f / l_tot;
            size_t row_w = (size_t)a.Hq * HD;
            bf16 *o_row = reinterpret_cast<bf16 *>(a.out) + (size_t)(cu_b + t) * row_w * (a.out_terms == 2 ? 2 : 1) +
                          (c * G + g) * HD;
#pragma unroll
            for (int hb = 0; hb < 4; ++hb)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    float v4[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) v4[j] = acc_o[hb][q4 * 4 + j] * inv;
                    store_out4(o_row + 32 * hb + 8 * q4 + 4 * half, row_w, a.out_terms, v4);
                }
        }
    } else {
        size_t row_slot = (size_t)item.part_slot * ATTN_BM + wave * 32 + lq;
        if (wave_active) {
            float *po = part_o + row_slot * HD;
#pragma unroll
            for (int hb = 0; hb < 4; ++hb)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    float4 v = make_float4(acc_o[hb][q4 * 4], acc_o[hb][q4 * 4 + 1], acc_o[hb][q4 * 4 + 2],
                                           acc_o[hb][q4 * 4 + 3]);
                    *reinterpret_cast<float4 *>(po + 32 * hb + 8 * q4 + 4 * half) = v;
                }
        }
        if (half == 0) {
            part_ml[row_slot * 2] = wave_active ? m_ref : -INFINITY;
            part_ml[row_slot * 2 + 1] = l_tot;
        }
    }
}

// Merge the splits of each tile in split order (fixed order: results are run-to-run identical).
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a, const AttnTile *__restrict__ tiles,
                                                          const int32_t *__restrict__ counts, int n_tiles_host,
                                                          const float *__restrict__ part_o,
                                                          const float *__restrict__ part_ml) {
    // One workgroup merges 8 rows of a tile: thread = (row, 4-float column), so every load of a
    // split's partial is independent of the others.
    constexpr int ROWS_PER_WG = 8, WGS_PER_TILE = ATTN_BM / ROWS_PER_WG;
    int n_tiles = min(counts[0], n_tiles_host);
    int tile_idx = blockIdx.x / WGS_PER_TILE;
    if (tile_idx >= n_tiles) return;
    AttnTile tile = tiles[tile_idx];
    if (tile.n_splits <= 1 || tile.part_base < 0) return;
    int G = a.Hq / a.Hkv;
    int b = min(max(tile.b, 0), a.B - 1), c = min(max(tile.c, 0), a.Hkv - 1);
    int cu_b = min(max(a.cu[b], 0), a.T - 1);
    int S = min(max(a.cu[b + 1] - cu_b, 1), a.T - cu_b);
    int n_rows = G * S;
    {
        int row = (blockIdx.x % WGS_PER_TILE) * ROWS_PER_WG + (threadIdx.x >> 5), hv = threadIdx.x & 31;
        int r = tile.row0 + row;
        if (r >= n_rows) return;
        float m_tot = -INFINITY;
        float l = 0.f;
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
        if (tile.n_splits == 2) {
            // the common case, same arithmetic as the loop below with every load issued before the first use
            size_t rs0 = (size_t)tile.part_base * ATTN_BM + row, rs1 = rs0 + ATTN_BM;
            float2 ml0 = *reinterpret_cast<const float2 *>(part_ml + rs0 * 2);
            float2 ml1 = *reinterpret_cast<const float2 *>(part_ml + rs1 * 2);
            float4 v0 = *reinterpret_cast<const float4 *>(part_o + rs0 * HD + hv * 4);
            float4 v1 = *reinterpret_cast<const float4 *>(part_o + rs1 * HD + hv * 4);
            m_tot = fmaxf(fmaxf(m_tot, ml0.x), ml1.x);
            if (ml0.x != -INFINITY) {
                float w = __builtin_amdgcn_exp2f(ml0.x - m_tot);
                l += w * ml0.y;
                o.x += w * v0.x; o.y += w * v0.y; o.z += w * v0.z; o.w += w * v0.w;
            }
            if (ml1.x != -INFINITY) {
                float w = __builtin_amdgcn_exp2f(ml1.x - m_tot);
                l += w * ml1.y;
                o.x += w * v1.x; o.y += w * v1.y; o.z += w * v1.z; o.w += w * v1.w;
            }
        } else {
            for (int s = 0; s < tile.n_splits; ++s)
                m_tot = fmaxf(m_tot, part_ml[((size_t)(tile.part_base + s) * ATTN_BM + row) * 2]);
            for (int s = 0; s < tile.n_splits; ++s) {
                size_t rs = (size_t)(tile.part_base + s) * ATTN_BM + row;
                float m_s = part_ml[rs * 2], l_s = part_ml[rs * 2 + 1];
                if (m_s == -INFINITY) continue;   // this split saw no visible key for the row
                float w = __builtin_amdgcn_exp2f(m_s - m_tot);
                float4 v = *reinterpret_cast<const float4 *>(part_o + rs * HD + hv * 4);
                l += w * l_s;
                o.x += w * v.x; o.y += w * v.y; o.z += w * v.z; o.w += w * v.w;
            }
        }
        float inv = 1.0f / l;
        int t = r / G, g = r - t * G;
        size_t row_w = (size_t)a.Hq * HD;
        bf16 *o_row = reinterpret_cast<bf16 *>(a.out) + (size_t)(cu_b + t) * row_w * (a.out_terms == 2 ? 2 : 1) +
                      (c * G + g) * HD;
        float vals[4] = {o.x * inv, o.y * inv, o.z * inv, o.w * inv};
        store_out4(o_row + hv * 4, row_w, a.out_terms, vals);
    }
}

template <bool PRECISE>
static hipError_t launch_attn_variant(const AttnArgs &a, const AttnItem *items, const int32_t *counts, int n_items_host,
                                      int max_xcd_items, float *part_o, float *part_ml, hipStream_t s) {
    constexpr int smem = PRECISE ? 2 * ATTN_SMEM_BYTES : ATTN_SMEM_BYTES;
    static std::atomic<uint32_t> attr_done{0};
    if (hipError_t e = set_dynamic_lds_once(attr_done, reinterpret_cast<const void *>(attn_bf16_kernel<PRECISE>), smem);
        e != hipSuccess)
        return e;
    int grid = 8 * max_xcd_items;
    attn_bf16_kernel<PRECISE><<<grid, ATTN_THREADS, smem, s>>>(a, items, counts, n_items_host, part_o, part_ml);
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnTune &tune, const AttnArgs &a, const AttnItem *items, const int32_t *counts,
                            int n_items_host, int max_xcd_items, float *part_o, float *part_ml, hipStream_t s) {
    if (n_items_host <= 0 || max_xcd_items <= 0) return hipSuccess;
    bool precise = a.q_lo && a.ksuf_lo && a.vsuf_lo;
    return precise ? launch_attn_variant<true>(a, items, counts, n_items_host, max_xcd_items, part_o, part_ml, s)
                   : launch_attn_variant<false>(a, items, counts, n_items_host, max_xcd_items, part_o, part_ml, s);
}

hipError_t launch_attn_merge(const AttnArgs &a, const AttnTile *tiles, const int32_t *counts, int n_tiles_host,
                             const float *part_o, const float *part_ml, hipStream_t s) {
    if (n_tiles_host <= 0) return hipSuccess;
    attn_merge_kernel<<<n_tiles_host * (ATTN_BM / 8), 256, 0, s>>>(a, tiles, counts, n_tiles_host, part_o, part_ml);
    return hipGetLastError();
}

}  // namespace cs
