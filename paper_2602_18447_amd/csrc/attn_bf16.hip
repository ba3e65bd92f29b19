// Grouped-query causal attention of suffix queries over the paged context cache plus the suffix's own
// keys, bf16 operands on the gfx950 matrix cores, fp32 online softmax.
//
// Decomposition.  All G query heads that share one kv head are folded into the row dimension: a context
// unit (one trace, or a run of traces whose candidate steps sit on the same cached context) with S suffix
// tokens contributes G*S rows per kv head, flattened token-major (row = t*G + g), cut into tiles of 128
// rows; one wavefront owns 32 rows.  The keys of a tile are a list of 64-key chunks - the chunks of the
// context, then the chunks of the suffix tokens its rows can see (attn_plan.h) - and, to balance ragged
// batches and fill 256 CUs, that list is cut into several work items whose partial (max, sum,
// unnormalised output) results are merged by a second kernel in a fixed order.
//
// Scores are computed transposed, S^T = K . Q^T (keys on MFMA rows, queries on columns), so each lane owns
// one query column: the running max / sum and the rescale of the output accumulator are lane-local apart
// from one exchange between lane l and l+32, and the probabilities a lane ends up holding are directly the
// B operand of O^T += V^T . P^T.
//
// Two main loops:
//  * attn_pipe_kernel (default): K and V chunks travel global -> LDS directly (no staging registers, no
//    transposition on the way), V^T fragments come from transposing LDS reads, and the loop is software
//    pipelined inside each wavefront: the score MFMAs of chunk i+1 are issued between the softmax
//    instructions of chunk i, so the matrix pipe and the vector ALU of a SIMD work at the same time.
//  * attn_staged_kernel (the two-term variant of the first layer(s); selectable for measurements): chunks go
//    through registers, V is transposed with byte permutes on the way into LDS.
#include "kernels.h"
#include <type_traits>
#include <utility>

namespace cs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define CS_GLOBAL_AS __attribute__((address_space(1)))
#define CS_LDS_AS __attribute__((address_space(3)))
// vmcnt(n) only (expcnt / lgkmcnt left unconstrained), gfx9 encoding of s_waitcnt
#define CS_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

constexpr int HD = 128;

// max(a, b, c) in one instruction.  The scores come straight from the matrix pipe, and fmaxf() would first put each
// of them through a canonicalising v_max (three instructions per score pair instead of one).
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// f(integral_constant<int, 0>{}), ..., f(integral_constant<int, N - 1>{}): a loop whose index is a compile-time
// constant in every round (no loop is left for the optimizer to unroll or not)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// ---- device planner: the lists of attn_plan.h, built from the device copies of the lengths ----
// counts[0] = tiles, counts[1] = items, counts[2 + x] = first item of XCD x (x = 0..8; [10] = items)
__global__ __launch_bounds__(256) void attn_plan_kernel(const int32_t *__restrict__ cu,
                                                         const int32_t *__restrict__ plens,
                                                         const int32_t *__restrict__ group_start, int n_units, int B,
                                                         int T, int max_L, int G, int Hkv, int cpi, int equalize,
                                                         int last_only, int max_tiles, int max_items,
                                                         AttnTile *__restrict__ tiles, AttnItem *__restrict__ items,
                                                         int32_t *__restrict__ counts) {
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
        for (int base = 0; base < n_units; base += 256) {
            int i = base + tid;
            AttnUnit u = {0, 1, 0, 0, 0};
            UnitPlan p = {0, 1, 0, 1};
            if (i < n_units) {
                u = plan_unit(cu, plens, group_start, n_units, i, B, T, max_L, last_only);
                p = unit_plan(u, G, cpi, equalize, last_only);
            }
            int my_tiles = Hkv * p.n_qt;
            s_tiles[tid + 1] = my_tiles;
            s_rest[tid + 1] = my_tiles * (p.n_split - 1);
            s_slots[tid + 1] = p.n_split > 1 ? my_tiles * p.n_split : 0;
            s_work[tid + 1] = (long long)my_tiles * p.nc_max;
            __syncthreads();
            if (tid == 0) {  // serial exclusive scan of the entries of this batch of units (at most 256)
                s_tiles[0] = carry[0];
                s_rest[0] = carry[1];
                s_slots[0] = carry[2];
                s_work[0] = carry_work;
                int n = min(256, n_units - base);
                for (int k = 1; k <= n; ++k) {
                    s_tiles[k] += s_tiles[k - 1];
                    s_rest[k] += s_rest[k - 1];
                    s_slots[k] += s_slots[k - 1];
                    s_work[k] += s_work[k - 1];
                }
                s_tiles[256] = s_tiles[n]; s_rest[256] = s_rest[n]; s_slots[256] = s_slots[n]; s_work[256] = s_work[n];
            }
            __syncthreads();
            int tile_base = s_tiles[tid], rest_base = s_rest[tid], slot_base = s_slots[tid];
            if (pass == 1 && i < n_units)
                plan_xcd_starts(p, Hkv, tile_base, rest_base, s_work[tid], work_total, tile_lo, seg_base);
            if (pass == 2 && i < n_units)
                plan_emit_unit(cu, T, u, G, Hkv, p, tile_base, rest_base, slot_base, tile_lo, seg_base, last_only,
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

hipError_t launch_attn_plan(const int32_t *cu, const int32_t *plens, const int32_t *group_start, int n_units, int B,
                            int T, int max_L, int G, int Hkv, int chunks_per_item, int equalize, int last_only,
                            int max_tiles, int max_items, AttnTile *tiles, AttnItem *items, int32_t *counts,
                            hipStream_t s) {
    if (!group_start || last_only) { group_start = nullptr; n_units = B; }
    attn_plan_kernel<<<1, 256, 0, s>>>(cu, plens, group_start, n_units, B, T, max_L, G, Hkv, chunks_per_item, equalize,
                                       last_only, max_tiles, max_items, tiles, items, counts);
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

// What every kernel below derives from its item: the unit, its rows, the tile's key list.
struct ItemGeom {
    int b0, c, cu0, n_rows, L, n_pc, k_start, G;
};
__device__ __forceinline__ ItemGeom item_geom(const AttnArgs &a, int ib0, int ib_end, int ic, int row0) {
    ItemGeom g;
    g.G = a.Hq / a.Hkv;
    g.b0 = min(max(ib0, 0), a.B - 1);
    int b1 = min(max(ib_end, g.b0 + 1), a.B);
    g.c = min(max(ic, 0), a.Hkv - 1);
    g.cu0 = min(max(a.cu[g.b0], 0), a.T - 1);
    int cu1 = min(max(a.cu[b1], g.cu0 + 1), a.T);
    g.n_rows = g.G * (cu1 - g.cu0);
    g.L = min(max(a.plens[g.b0], 0), a.max_blocks * 16);
    g.n_pc = (g.L + ATTN_BN - 1) / ATTN_BN;
    // first suffix key of the tile: the first token of the trace that holds the tile's first row
    int tok_lo = g.cu0 + min(max(row0, 0), g.n_rows - 1) / g.G;
    int tr_lo = min(max(a.tok_trace[tok_lo], g.b0), b1 - 1);
    g.k_start = min(max(a.cu[tr_lo], g.cu0), tok_lo);
    return g;
}

// End of an item: the normalised output rows (item covers its tile's whole key list), or the fp32 partial
// result of a piece for the merge.  acc_o[hb][e]: hd = 32*hb + 8*(e>>2) + 4*half + (e&3), query = the lane's row.
__device__ __forceinline__ void finish_item(const AttnArgs &a, const AttnItem &item, const f32x16 (&acc_o)[4], float l_run,
                                            float m_ref, bool wave_active, bool row_valid, int wave, int lq, int half,
                                            int token, int head, float *__restrict__ part_o, float *__restrict__ part_ml) {
    float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (item.part_slot < 0) {
        if (row_valid) {
            float inv = 1.0f / l_tot;
            size_t row_w = (size_t)a.Hq * HD;
            bf16 *o_row = reinterpret_cast<bf16 *>(a.out) + (size_t)token * row_w * (a.out_terms == 2 ? 2 : 1) + head * HD;
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

// =================================================================================================
// Software-pipelined main loop.
//
// LDS: two stages of K and two of V, each [64 keys][128 hd] bf16 in 256-byte rows without padding.  A
// wavefront fills 16 keys of a chunk with four direct loads (1 KiB = 4 rows each; in a context chunk those 16
// keys are one 16-token page).  Bank conflicts are avoided by permuting the 16-byte vectors inside a row:
// K keeps vector v of key k at slot v ^ (k & 15) (the score MFMAs read 16 consecutive keys at one v),
// V keeps it at slot v ^ (4 * (k & 3)) (32 lanes of a transposing read touch 4 consecutive keys x 64 contiguous
// bytes: each key in its own quarter of the 256-byte bank space).
// The lane that fills a slot fetches the matching global vector.
//
// Transposing reads (ds_read_b64_tr_b16): in a group of 16 lanes, lane i supplies the address of 4 consecutive
// 16-bit elements and receives element i % 4 of what lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4 addressed.  With
// lane 4 j + q pointing at V[key j][hd 4 q .. 4 q + 3] of a 4-key x 16-hd block, lane i receives
// V[key 0 .. 3][hd i]: four consecutive k-values of the A operand of O^T += V^T . P^T for its hd row.
//
// Pipeline, iteration i (chunk i of the item): wait for K(i+1) and V(i), barrier, start the direct loads of K(i+2)
// and V(i+1) into the stages that chunk i's score product and chunk i-1's value product have released; then
// S(i+1) = K(i+1) . Q^T on the matrix pipe while the vector ALU turns S(i) into probabilities, then
// O^T += V(i)^T . P(i)^T.
constexpr int PIPE_TILE_BYTES = ATTN_BN * HD * 2;          // one K or V stage: 16 KiB
constexpr int PIPE_SMEM_BYTES = 4 * PIPE_TILE_BYTES;       // K0 K1 V0 V1

__global__ __launch_bounds__(ATTN_THREADS, 2) void attn_pipe_kernel(AttnArgs a, const AttnItem *__restrict__ items,
                                                                    const int32_t *__restrict__ counts, int n_items_host,
                                                                    float *__restrict__ part_o,
                                                                    float *__restrict__ part_ml) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // workgroup id % 8 is the XCD; each XCD walks its own range of the item list in order
    int n_items = min(counts[1], n_items_host);
    int xcd = blockIdx.x & 7;
    int it_idx = counts[2 + xcd] + (blockIdx.x >> 3);
    if (it_idx >= min(counts[3 + xcd], n_items)) return;
    AttnItem item = items[it_idx];
    // the item is the same for every lane: keep it (and everything derived from it) in scalar registers, so that
    // loads at addresses derived from it - block-table entries, lengths - are scalar loads
    item.b0 = __builtin_amdgcn_readfirstlane(item.b0);
    item.c = __builtin_amdgcn_readfirstlane(item.c);
    item.row0 = __builtin_amdgcn_readfirstlane(item.row0);
    item.chunk_begin = __builtin_amdgcn_readfirstlane(item.chunk_begin);
    item.chunk_end = __builtin_amdgcn_readfirstlane(item.chunk_end);
    item.part_slot = __builtin_amdgcn_readfirstlane(item.part_slot);
    item.b_end = __builtin_amdgcn_readfirstlane(item.b_end);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (item.chunk_begin >= item.chunk_end) {
        // a piece that received no chunks: mark its rows as "nothing seen" for the merge
        if (item.part_slot >= 0 && tid < ATTN_BM) {
            size_t row_slot = (size_t)item.part_slot * ATTN_BM + tid;
            part_ml[row_slot * 2] = -INFINITY;
            part_ml[row_slot * 2 + 1] = 0.f;
        }
        return;
    }
    const int half = lane >> 5, lq = lane & 31;
    const ItemGeom ge = item_geom(a, item.b0, item.b_end, item.c, item.row0);
    const int G = ge.G, c = ge.c, L = ge.L, n_pc = ge.n_pc;

    // Four wavefronts of 32 query rows each.  A wave whose rows all lie past the end of the unit still
    // loads and synchronises with the others but skips the matrix work.
    const int wave_row0 = item.row0 + wave * 32;
    const bool wave_active = wave_row0 < ge.n_rows;             // wave-uniform
    const int r = wave_row0 + lq;
    const bool row_valid = r < ge.n_rows;
    const int rc = min(r, ge.n_rows - 1);
    const int tt = rc / G, g = rc - tt * G;
    const int token = ge.cu0 + tt;                              // packed suffix token of this lane's query
    // suffix keys visible to it: the packed tokens klo .. token (its own trace up to itself)
    const int klo = min(max(a.cu[min(max(a.tok_trace[token], ge.b0), a.B - 1)], ge.cu0), token);

    const bf16 *q_row = reinterpret_cast<const bf16 *>(a.q) + ((size_t)token * a.Hq + c * G + g) * HD;
    bf16x8 qf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(q_row + ks * 16 + half * 8);

    // ---- direct loads: wave w fills keys 16 w .. 16 w + 15 of a chunk, instruction j keys 4 j .. 4 j + 3 of those
    const bf16 *kp = reinterpret_cast<const bf16 *>(a.k_pages), *vp = reinterpret_cast<const bf16 *>(a.v_pages);
    const bf16 *ks_ = reinterpret_cast<const bf16 *>(a.ksuf), *vs_ = reinterpret_cast<const bf16 *>(a.vsuf);
    const int32_t *bt = a.block_table + (size_t)ge.b0 * a.max_blocks;
    const int last_page = max((L + 15) / 16 - 1, 0);
    const int lrow = lane >> 4, lpos = lane & 15;
    // element offsets inside a key row of the vector this lane fetches (the slot permutation above)
    int k_vec[4], v_vec[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int key = 4 * j + lrow;                                  // key & 15 (the wave's 16 keys start at a multiple of 16)
        k_vec[j] = (lpos ^ key) * 8;
        v_vec[j] = (lpos ^ (4 * (key & 3))) * 8;
    }
    // byte offsets of this lane's four vectors inside a page's rows of this kv head (context chunks)
    unsigned k_poff[4], v_poff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        k_poff[j] = ((4 * j + lrow) * HD + k_vec[j]) * 2;
        v_poff[j] = ((4 * j + lrow) * HD + v_vec[j]) * 2;
    }
    // Block-table entries: this wave needs page `wave` of every context chunk.  Lane l holds the entry of chunk
    // ids_first + l; the vector is refilled once every 64 chunks (a load whose wait coincides with the wait at the top
    // of an iteration), and an entry is picked with a lane read.
    int ids_vec = 0, ids_first = -(1 << 30);
    auto page_id = [&](int u) -> int {                           // wave-uniform
        if (u - ids_first >= 64 || u < ids_first) {              // uniform branch
            ids_first = u;
            ids_vec = bt[min(4 * (u + lane) + wave, last_page)];
        }
        return min(max(__builtin_amdgcn_readlane(ids_vec, u - ids_first), 0), a.n_blocks - 1);
    };
    // The direct loads are issued from inline assembly: the compiler then does not know that LDS is being written
    // behind its back, and does not put a wait for all of them in front of the transposing LDS reads (which it cannot
    // tell apart from the stage being filled).  Their completion is waited for explicitly (vmcnt) at the top of every
    // iteration, followed by the workgroup barrier.
    const unsigned lds_base = (unsigned)(size_t)(CS_LDS_AS unsigned char *)smem;
    auto dma16 = [&](const bf16 *src, unsigned lds_dst) {      // 64 lanes x 16 bytes -> lds_dst + 16 * lane
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_dst), "v"(src) : "memory");
    };
    // the same from a wave-uniform base address plus a 32-bit byte offset per lane (no address arithmetic per lane)
    auto dma16_base = [&](const bf16 *base, unsigned off, unsigned lds_dst) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_dst), "v"(off), "s"(base) : "memory");
    };
    auto issue = [&](const bf16 *pages, const bf16 *suf, const int (&vec)[4], const unsigned (&poff)[4], int u, int id,
                     int stage_idx) __attribute__((always_inline)) {
        unsigned dst = lds_base + stage_idx * PIPE_TILE_BYTES + wave * 4096;
        if (u < n_pc) {
            const bf16 *base = pages + ((size_t)id * a.Hkv + c) * 16 * HD;      // scalar
#pragma unroll
            for (int j = 0; j < 4; ++j) dma16_base(base, poff[j], dst + j * 1024);
        } else {
            int k0 = ge.k_start + ATTN_BN * (u - n_pc) + 16 * wave + lrow;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int kt = min(k0 + 4 * j, a.T - 1);               // tokens past the end are masked for every query
                dma16(suf + ((size_t)kt * a.Hkv + c) * HD + vec[j], dst + j * 1024);
            }
        }
    };
    // stage indices: K stages 0, 1; V stages 2, 3
    auto k_stage = [&](int i) -> unsigned char * { return smem + (i & 1) * PIPE_TILE_BYTES; };

    // ---- fragment addresses
    // K: MFMA row lq of block kb = key 32 kb + lq; k-step ks reads vector 2 ks + half of that key
    int k_off[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) k_off[ks] = lq * 256 + (((2 * ks + half) ^ (lq & 15)) << 4);
    // V^T: group gi = lane / 16 serves hd rows 16 (gi & 1) .. + 15 of a 32-row block for k-group gi / 2 (= half);
    // lane i of the group points at key 4 half + i / 4 (+ 8 for the second read), hd 4 (i % 4) .. + 3
    const int li = lane & 15, gi = lane >> 4;
    const int v_key = 4 * half + (li >> 2);                      // (key & 7) of the rows this lane addresses
    int v_off[4];
#pragma unroll
    for (int hb = 0; hb < 4; ++hb) {
        int vec = 4 * hb + 2 * (gi & 1) + ((li & 3) >> 1);       // 16-byte vector of hd 32 hb + 16 (gi & 1) + 4 (li & 3)
        v_off[hb] = v_key * 256 + ((vec ^ (4 * (v_key & 3))) << 4) + ((li & 1) << 3);
    }

    f32x16 acc_o[4];
#pragma unroll
    for (int hb = 0; hb < 4; ++hb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[hb][e] = 0.f;
    float m_run = -INFINITY, m_ref = -INFINITY, l_run = 0.f;   // true max, exponent reference, sum (vs m_ref)
    const float sc = a.scale * 1.44269504088896340736f;        // scores in log2 units

    const int u0 = item.chunk_begin, n = item.chunk_end - item.chunk_begin;

    // S^T block kb of a chunk: acc[kb][e] = score of key 32 kb + 8 (e >> 2) + 4 half + (e & 3), query lq.
    // MFMA q of the 16 of a chunk: k-step q / 2, key block q % 2.
    auto score_mfma = [&](f32x16 (&acc)[2], const unsigned char *kst, int q) {
        int ks = q >> 1, kb = q & 1;
        bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kst + kb * 32 * 256 + k_off[ks]);
        acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc[kb], 0, 0, 0);
    };
    auto zero2 = [&](f32x16 (&acc)[2]) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[kb][e] = 0.f;
    };

    // ---- prologue: K(0), V(0), K(1) in flight; S(0) computed without anything to overlap with
    int id_v = 0, id_k = 0, id_n = 0;                            // page ids: chunk i+1 (V), i+2 (K), i+3 (prefetched)
    {
        int id0 = u0 < n_pc ? page_id(u0) : 0;
        issue(kp, ks_, k_vec, k_poff, u0, id0, 0);
        issue(vp, vs_, v_vec, v_poff, u0, id0, 2);
        id_v = (n > 1 && u0 + 1 < n_pc) ? page_id(u0 + 1) : 0;
        if (n > 1) issue(kp, ks_, k_vec, k_poff, u0 + 1, id_v, 1);
        id_k = (n > 2 && u0 + 2 < n_pc) ? page_id(u0 + 2) : 0;
        id_n = (n > 3 && u0 + 3 < n_pc) ? page_id(u0 + 3) : 0;
    }
    f32x16 s_a[2], s_b[2];       // raw scores of two consecutive chunks; the roles alternate from iteration to iteration
    zero2(s_a);
    if (n > 1) CS_WAIT_VMCNT(8); else CS_WAIT_VMCNT(4);          // K(0) has landed (this wave's part)
    __syncthreads();
    if (wave_active) {
#pragma unroll
        for (int q = 0; q < 16; ++q) score_mfma(s_a, k_stage(0), q);
    }

    // One iteration.  Compile-time arguments: the parity of i (it fixes the LDS stages: K(i+1) is read from K stage
    // 1 - parity, V(i) from V stage parity) and whether chunk i + 1 exists (its scores are then computed under chunk
    // i's softmax, into s_nxt).
    auto iteration = [&](int i, f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2], auto parity_tag, auto more_tag) __attribute__((always_inline)) {
        constexpr int par = decltype(parity_tag)::value;
        constexpr bool more = decltype(more_tag)::value;
        const int u = u0 + i;
        // page id of chunk i + 4 (a scalar load, asked for before the wait so that it arrives under it)
        const int id_new = (i + 4 < n && u + 4 < n_pc) ? page_id(u + 4) : 0;
        CS_WAIT_VMCNT(0);
        __syncthreads();      // K(i+1) and V(i) are in LDS; nobody reads K(i) or V(i-1) any more
        if (i + 2 < n) issue(kp, ks_, k_vec, k_poff, u + 2, id_k, par);
        if constexpr (more) issue(vp, vs_, v_vec, v_poff, u + 1, id_v, 3 - par);
        id_v = id_k;
        id_k = id_n;
        id_n = id_new;
        const unsigned char *kst = smem + (1 - par) * PIPE_TILE_BYTES, *vst = smem + (2 + par) * PIPE_TILE_BYTES;

        if (wave_active) {
            // -- masks of chunk i: the tail of the context, or the visibility window of the suffix tokens
            if (u >= n_pc) {
                int kt0 = ge.k_start + ATTN_BN * (u - n_pc) + 4 * half;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        int kt = kt0 + 32 * kb + 8 * (e >> 2) + (e & 3);
                        if (kt < klo || kt > token) s_cur[kb][e] = -INFINITY;
                    }
            } else if (u * ATTN_BN + ATTN_BN > L) {
                int j0 = u * ATTN_BN + 4 * half;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (j0 + 32 * kb + 8 * (e >> 2) + (e & 3) >= L) s_cur[kb][e] = -INFINITY;
            }
            // The chunk is 32 steps of one MFMA each: steps 0..15 the score MFMAs of chunk i+1 (k-step s / 2, key
            // block s % 2), steps 16..31 the value MFMAs of chunk i (key block, k-step, hd block).  The operand of step
            // s + 2 is requested from LDS before the MFMA of step s is issued, and a slice of chunk i's softmax
            // follows each MFMA: the row maximum in steps 0..3, the probabilities of key block 0 in steps 4..15 (in
            // time for step 16), those of key block 1 in steps 16..23 (in time for step 24).
            bf16x8 fr[3];
            auto fetch = [&](auto st_tag) __attribute__((always_inline)) {     // operand of step st into fr[st % 3]
                constexpr int st = decltype(st_tag)::value;
                if constexpr (st < 16) {
                    if constexpr (more) fr[st % 3] = *reinterpret_cast<const bf16x8 *>(kst + (st & 1) * 32 * 256 + k_off[st >> 1]);
                } else if constexpr (st < 32) {
                    constexpr int idx = st - 16, kb = idx >> 3, s2 = (idx >> 2) & 1, hb = idx & 3;
                    // two transposing reads: keys 32 kb + 16 s2 + 4 half + 0..3 and + 8
                    const unsigned char *p0 = vst + (32 * kb + 16 * s2) * 256 + v_off[hb];
                    i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CS_LDS_AS i16x4 *)p0);
                    i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CS_LDS_AS i16x4 *)(p0 + 8 * 256));
                    i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    fr[st % 3] = __builtin_bit_cast(bf16x8, both);
                }
            };
            float mloc = -INFINITY, neg_off = 0.f, psum = 0.f;
            bf16x8 pf[2][2];
            fetch(std::integral_constant<int, 0>{});
            fetch(std::integral_constant<int, 1>{});
            __builtin_amdgcn_sched_barrier(0);
            static_for<32>([&](auto st_tag) __attribute__((always_inline)) {
                constexpr int st = decltype(st_tag)::value;
                fetch(std::integral_constant<int, st + 2>{});
                if constexpr (st < 16) {
                    if constexpr (more) {
                        if constexpr (st < 2) {
                            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                            s_nxt[st & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st % 3], qf[st >> 1], zero, 0, 0, 0);
                        } else {
                            s_nxt[st & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st % 3], qf[st >> 1], s_nxt[st & 1], 0, 0, 0);
                        }
                    }
                } else {
                    constexpr int idx = st - 16;
                    acc_o[idx & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st % 3], pf[idx >> 3][(idx >> 2) & 1], acc_o[idx & 3], 0, 0, 0);
                }
                if constexpr (st < 4) {
#pragma unroll
                    for (int e = 4 * st; e < 4 * st + 4; ++e) mloc = max3(mloc, s_cur[0][e], s_cur[1][e]);
                    if constexpr (st == 3) {
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
                        neg_off = (m_ref == -INFINITY) ? 0.f : -m_ref;
                    }
                } else if constexpr (st < 16) {
                    constexpr int e0 = ((st - 4) * 16) / 12, e1 = ((st - 3) * 16) / 12;
#pragma unroll
                    for (int e = e0; e < e1; ++e) {
                        float p = __builtin_amdgcn_exp2f(fmaf(s_cur[0][e], sc, neg_off));
                        psum += p;
                        pf[0][e >> 3][e & 7] = (__bf16)p;
                    }
                } else if constexpr (st < 24) {
#pragma unroll
                    for (int e = 2 * (st - 16); e < 2 * (st - 16) + 2; ++e) {
                        float p = __builtin_amdgcn_exp2f(fmaf(s_cur[1][e], sc, neg_off));
                        psum += p;
                        pf[1][e >> 3][e & 7] = (__bf16)p;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            l_run += psum;
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    {
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, 1>;
        int i = 0;
        for (; i + 2 < n; i += 2) {
            iteration(i, s_a, s_b, P0{}, std::true_type{});
            iteration(i + 1, s_b, s_a, P1{}, std::true_type{});
        }
        if (n - i == 2) {
            iteration(i, s_a, s_b, P0{}, std::true_type{});
            iteration(i + 1, s_b, s_a, P1{}, std::false_type{});
        } else {
            iteration(i, s_a, s_b, P0{}, std::false_type{});
        }
    }

    finish_item(a, item, acc_o, l_run, m_ref, wave_active, row_valid, wave, lq, half, token, c * G + g, part_o, part_ml);
}

// =================================================================================================
// Register-staged main loop.  Per chunk a workgroup stages K as [key][hd] and V transposed as [hd][key] in
// LDS through registers (the next chunk's loads are in flight while the current one is multiplied).  The rows
// of each 32-key block are fed to the score MFMA in a permuted order chosen so that the probabilities a
// lane ends up holding are 8 consecutive keys per k-step, and the matching A operand of the value product is
// a single 16-byte read of the transposed V tile.
//
// PRECISE: q, the suffix keys / values and the probabilities are each carried as two bf16 terms
// (hi + lo); products hi*hi, hi*lo and lo*hi are accumulated (lo*lo is below fp32 resolution of the
// sum).  Cached context keys / values are exact bf16 values and need no second term.  Used for the
// first layer(s), where score noise from rounding q and k is amplified by every later layer.
constexpr int K_STRIDE = 136;             // elements per K row in LDS (128 + 8 pad = 272 bytes)
constexpr int VT_STRIDE = 72;             // elements per V^T row in LDS (64 + 8 pad = 144 bytes)
constexpr int K_TILE = ATTN_BN * K_STRIDE;
constexpr int VT_TILE = HD * VT_STRIDE;
constexpr int ATTN_STAGE = K_TILE + VT_TILE;   // elements per stage
constexpr int ATTN_SMEM_BYTES = 2 * ATTN_STAGE * 2;

template <bool PRECISE>
__global__ __launch_bounds__(ATTN_THREADS, PRECISE ? 1 : 2) void attn_staged_kernel(AttnArgs a, const AttnItem *__restrict__ items,
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
    const ItemGeom ge = item_geom(a, item.b0, item.b_end, item.c, item.row0);
    const int G = ge.G, c = ge.c, L = ge.L, n_pc = ge.n_pc, n_rows = ge.n_rows;

    // Four wavefronts of 32 query rows each.  A wave whose rows all lie past the end of the trace
    // still loads and synchronises with the others but skips the matrix work.
    int wave_row0 = item.row0 + wave * 32;
    bool wave_active = wave_row0 < n_rows;             // wave-uniform
    int r = wave_row0 + lq;
    bool row_valid = r < n_rows;
    int rc = min(r, n_rows - 1);
    int tt = rc / G, g = rc - tt * G;
    const int token = ge.cu0 + tt;                              // packed suffix token of this lane's query
    // suffix keys visible to it: the packed tokens klo .. token (its own trace up to itself)
    const int klo = min(max(a.cu[min(max(a.tok_trace[token], ge.b0), a.B - 1)], ge.cu0), token);

    const bf16 *q_row = reinterpret_cast<const bf16 *>(a.q) + ((size_t)token * a.Hq + c * G + g) * HD;
    bf16x8 qf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(q_row + ks * 16 + half * 8);
    bf16x8 qf_lo[PRECISE ? 8 : 1];
    if constexpr (PRECISE) {
        const bf16 *ql_row = reinterpret_cast<const bf16 *>(a.q_lo) + ((size_t)token * a.Hq + c * G + g) * HD;
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
    const int32_t *bt = a.block_table + (size_t)ge.b0 * a.max_blocks;     // wave-uniform
    const size_t page_elems = (size_t)a.Hkv * 16 * HD;
    const int k_in_page = (c * 16 + (tid >> 4)) * HD + (tid & 15) * 8;
    const int v_in_page = (c * 16 + 4 * (v_kq & 3)) * HD + v_g * 8;
    const int v_page_sel = v_kq >> 2;
    const int max_page = max((L + 15) / 16 - 1, 0);

    // Physical block ids of the 4 pages of a context chunk, fetched two chunks ahead: lanes 0..3 each load one
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
    // Row of key k (0..63) of chunk u when the chunk is not a whole context chunk: the context's last, partly
    // filled chunk (rows past L - 1 are clamped to it: such keys are masked for every query), or a chunk of
    // suffix tokens (clamped to the last token of the batch, likewise masked).
    auto row_general = [&](const bf16 *pages, const bf16 *suf, int u, int k) -> const bf16 * {
        if (u < n_pc) {
            int jp = min(u * ATTN_BN + k, max(L - 1, 0));
            int id = min(max(bt[min(jp >> 4, max_page)], 0), a.n_blocks - 1);
            return pages + ((size_t)id * a.Hkv + c) * 16 * HD + (jp & 15) * HD;
        }
        int kt = min(ge.k_start + ATTN_BN * (u - n_pc) + k, a.T - 1);
        return suf + ((size_t)kt * a.Hkv + c) * HD;
    };

    u32x4 k_reg[4], v_reg[4];
    u32x4 kl_reg[PRECISE ? 4 : 1], vl_reg[PRECISE ? 4 : 1];
    const bf16 *ksl_ = reinterpret_cast<const bf16 *>(a.ksuf_lo), *vsl_ = reinterpret_cast<const bf16 *>(a.vsuf_lo);
    auto load_chunk = [&](int u) {
        if (u < n_pc && u * ATTN_BN + ATTN_BN <= L) {          // uniform: a whole chunk of the cached context
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
                kr[i] = row_general(kp, ks_, u, (tid >> 4) + 16 * i) + (tid & 15) * 8;
                vr[i] = row_general(vp, vs_, u, 4 * v_kq + i) + v_g * 8;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                k_reg[i] = *reinterpret_cast<const u32x4 *>(kr[i]);
                v_reg[i] = *reinterpret_cast<const u32x4 *>(vr[i]);
            }
            if constexpr (PRECISE) {
                if (u >= n_pc) {                               // second terms exist for suffix tokens only
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        kl_reg[i] = *reinterpret_cast<const u32x4 *>(row_general(ksl_, ksl_, u, (tid >> 4) + 16 * i) + (tid & 15) * 8);
                        vl_reg[i] = *reinterpret_cast<const u32x4 *>(row_general(vsl_, vsl_, u, 4 * v_kq + i) + v_g * 8);
                    }
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
    // u: the chunk held in the registers (its lo tiles exist only for chunks of suffix tokens)
    auto store_chunk = [&](int stage, int u) {
        __bf16 *base = smem + stage * STAGE;
        store_tiles(base, k_reg, v_reg);
        if constexpr (PRECISE) {
            if (u >= n_pc) store_tiles(base + ATTN_STAGE, kl_reg, vl_reg);
        }
    };

    f32x16 acc_o[4];
#pragma unroll
    for (int hb = 0; hb < 4; ++hb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[hb][e] = 0.f;
    float m_run = -INFINITY, m_ref = -INFINITY, l_run = 0.f;   // true max, exponent reference, sum (vs m_ref)
    const float sc = a.scale * 1.44269504088896340736f;   // scores in log2 units

    // K operand row (key) for MFMA row lq, see the comment above the kernel: pi(m)
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
        const bool has_lo = PRECISE && ch >= n_pc;   // uniform

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
            // register e of block kb holds key 32*kb + 16*(e>>3) + 8*half + (e&7) of the chunk
            if (ch >= n_pc) {                 // suffix tokens: visible from the start of the query's trace up to the query
                int kt0 = ge.k_start + ATTN_BN * (ch - n_pc) + 8 * half;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        int kt = kt0 + 32 * kb + 16 * (e >> 3) + (e & 7);
                        if (kt < klo || kt > token) acc_s[kb][e] = -INFINITY;
                    }
            } else if (ch * ATTN_BN + ATTN_BN > L) {      // the context's last, partly filled chunk
                int j0 = ch * ATTN_BN + 8 * half;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (j0 + 32 * kb + 16 * (e >> 3) + (e & 7) >= L) acc_s[kb][e] = -INFINITY;
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

    finish_item(a, item, acc_o, l_run, m_ref, wave_active, row_valid, wave, lq, half, token, c * G + g, part_o, part_ml);
}

// Merge the pieces of each tile in piece order (fixed order: results are run-to-run identical).
// One workgroup merges 32 rows of a tile: thread = (row, 16 of the 128 output columns).  The partial results of a
// piece are four independent 16-byte loads per thread; the loop over the pieces runs two pieces per round with all
// eight loads issued before the first use, so the kernel streams the partial results rather than waiting for them.
constexpr int MERGE_ROWS = 32;
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a, const AttnTile *__restrict__ tiles,
                                                          const int32_t *__restrict__ counts, int n_tiles_host,
                                                          const float *__restrict__ part_o,
                                                          const float *__restrict__ part_ml) {
    constexpr int WGS_PER_TILE = ATTN_BM / MERGE_ROWS;
    int n_tiles = min(counts[0], n_tiles_host);
    int tile_idx = blockIdx.x / WGS_PER_TILE;
    if (tile_idx >= n_tiles) return;
    AttnTile tile = tiles[tile_idx];
    if (tile.n_splits <= 1 || tile.part_base < 0) return;
    int G = a.Hq / a.Hkv;
    int b0 = min(max(tile.b0, 0), a.B - 1), b1 = min(max(tile.b_end, b0 + 1), a.B), c = min(max(tile.c, 0), a.Hkv - 1);
    int cu_b = min(max(a.cu[b0], 0), a.T - 1);
    int n_rows = G * (min(max(a.cu[b1], cu_b + 1), a.T) - cu_b);
    const int row = (blockIdx.x % WGS_PER_TILE) * MERGE_ROWS + (threadIdx.x >> 3), hv = threadIdx.x & 7;
    const int r = tile.row0 + row;
    if (r >= n_rows) return;
    const int ns = tile.n_splits;
    // the largest reference exponent over the pieces
    float m_tot = -INFINITY;
    for (int s = 0; s < ns; ++s) m_tot = fmaxf(m_tot, part_ml[((size_t)(tile.part_base + s) * ATTN_BM + row) * 2]);
    float l = 0.f;
    float4 o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    auto piece_ptr = [&](int s) { return part_o + ((size_t)(tile.part_base + s) * ATTN_BM + row) * HD + hv * 16; };
    auto add_piece = [&](float2 ml, const float4 (&v)[4]) {
        if (ml.x == -INFINITY) return;   // this piece saw no visible key for the row
        float w = __builtin_amdgcn_exp2f(ml.x - m_tot);
        l += w * ml.y;
#pragma unroll
        for (int j = 0; j < 4; ++j) { o[j].x += w * v[j].x; o[j].y += w * v[j].y; o[j].z += w * v[j].z; o[j].w += w * v[j].w; }
    };
    int s = 0;
    for (; s + 1 < ns; s += 2) {
        float4 v0[4], v1[4];
        const float4 *p0 = reinterpret_cast<const float4 *>(piece_ptr(s)), *p1 = reinterpret_cast<const float4 *>(piece_ptr(s + 1));
#pragma unroll
        for (int j = 0; j < 4; ++j) { v0[j] = p0[j]; v1[j] = p1[j]; }
        float2 ml0 = *reinterpret_cast<const float2 *>(part_ml + ((size_t)(tile.part_base + s) * ATTN_BM + row) * 2);
        float2 ml1 = *reinterpret_cast<const float2 *>(part_ml + ((size_t)(tile.part_base + s + 1) * ATTN_BM + row) * 2);
        add_piece(ml0, v0);
        add_piece(ml1, v1);
    }
    if (s < ns) {
        float4 v0[4];
        const float4 *p0 = reinterpret_cast<const float4 *>(piece_ptr(s));
#pragma unroll
        for (int j = 0; j < 4; ++j) v0[j] = p0[j];
        float2 ml0 = *reinterpret_cast<const float2 *>(part_ml + ((size_t)(tile.part_base + s) * ATTN_BM + row) * 2);
        add_piece(ml0, v0);
    }
    float inv = 1.0f / l;
    int t = r / G, g = r - t * G;
    size_t row_w = (size_t)a.Hq * HD;
    bf16 *o_row = reinterpret_cast<bf16 *>(a.out) + (size_t)(cu_b + t) * row_w * (a.out_terms == 2 ? 2 : 1) + (c * G + g) * HD;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float vals[4] = {o[j].x * inv, o[j].y * inv, o[j].z * inv, o[j].w * inv};
        store_out4(o_row + hv * 16 + 4 * j, row_w, a.out_terms, vals);
    }
}

template <bool PRECISE>
static hipError_t launch_staged(const AttnArgs &a, const AttnItem *items, const int32_t *counts, int n_items_host,
                                int max_xcd_items, float *part_o, float *part_ml, hipStream_t s) {
    constexpr int smem = PRECISE ? 2 * ATTN_SMEM_BYTES : ATTN_SMEM_BYTES;
    static std::atomic<uint32_t> attr_done{0};
    if (hipError_t e = set_dynamic_lds_once(attr_done, reinterpret_cast<const void *>(attn_staged_kernel<PRECISE>), smem);
        e != hipSuccess)
        return e;
    attn_staged_kernel<PRECISE><<<8 * max_xcd_items, ATTN_THREADS, smem, s>>>(a, items, counts, n_items_host, part_o, part_ml);
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnTune &tune, const AttnArgs &a, const AttnItem *items, const int32_t *counts,
                            int n_items_host, int max_xcd_items, int avg_chunks, float *part_o, float *part_ml, hipStream_t s) {
    if (n_items_host <= 0 || max_xcd_items <= 0) return hipSuccess;
    bool precise = a.q_lo && a.ksuf_lo && a.vsuf_lo;
    if (precise) return launch_staged<true>(a, items, counts, n_items_host, max_xcd_items, part_o, part_ml, s);
    // Short items (one-token batches cut into pieces of a few chunks): the pipelined loop's prologue and epilogue -
    // three chunk loads and an unoverlapped score product before the first iteration - weigh more than its steady
    // state gains; the register-staged loop is the faster one there (22.5 against 30.8 us per layer at 32 x 2048).
    if (tune.kernel == 1 || (tune.kernel == 0 && avg_chunks < 12))
        return launch_staged<false>(a, items, counts, n_items_host, max_xcd_items, part_o, part_ml, s);
    static std::atomic<uint32_t> attr_done{0};
    if (hipError_t e = set_dynamic_lds_once(attr_done, reinterpret_cast<const void *>(attn_pipe_kernel), PIPE_SMEM_BYTES);
        e != hipSuccess)
        return e;
    attn_pipe_kernel<<<8 * max_xcd_items, ATTN_THREADS, PIPE_SMEM_BYTES, s>>>(a, items, counts, n_items_host, part_o, part_ml);
    return hipGetLastError();
}

hipError_t launch_attn_merge(const AttnArgs &a, const AttnTile *tiles, const int32_t *counts, int n_tiles_host,
                             const float *part_o, const float *part_ml, hipStream_t s) {
    if (n_tiles_host <= 0) return hipSuccess;
    attn_merge_kernel<<<n_tiles_host * (ATTN_BM / MERGE_ROWS), 256, 0, s>>>(a, tiles, counts, n_tiles_host, part_o, part_ml);
    return hipGetLastError();
}

}  // namespace cs
