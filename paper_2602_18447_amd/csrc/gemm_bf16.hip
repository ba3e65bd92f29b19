// bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores: C[M,N] = A[M,K] . W[N,K]^T.
//
// Both operands are K-contiguous, which is exactly the per-lane operand shape of the 16-bit MFMAs: 8 consecutive k of
// one row / column per lane (v_mfma_f32_32x32x16: row lane % 32, k-group lane / 32; v_mfma_f32_16x16x32: row lane % 16,
// k-group lane / 16).
//
// Data path.  Operand tiles travel global -> LDS directly (buffer_load_dwordx4 ... lds): no staging registers, no
// ds_write instructions, the wave keeps issuing MFMAs while the data lands.  One such instruction fills 1 KiB of LDS in
// lane order, i.e. 8 tile rows of 64 k (128 bytes) each; its address is a scalar buffer resource (the tile's first row),
// a per-lane 32-bit offset that never changes and the k-tile's offset in a scalar register, so issuing one costs no
// vector instruction.  Rows are unpadded; instead the 16-byte k-vector g of row r is kept at position g ^ ((r >> 1) & 7)
// of its row (the lane that fills a position fetches the matching global vector), so the 16 lanes of one ds_read_b128
// phase - 16 consecutive rows, same k-vector - hit 16 different 4-bank groups.
// Two pipelines: 256 x 256 tiles run 16x16x32 MFMAs on a ring of five half-stage LDS units with the loads spread between
// the MFMAs (described where it is written); the smaller tiles, of which a CU holds two independent workgroups, keep two
// (or four) whole stages: the loads of the next k-tile(s) are issued right behind the barrier that frees their stage.
// Barriers inside the k loops are bare s_barrier instructions with explicit waits: __syncthreads() carries fences that
// make the compiler wait for every outstanding direct load.
//
// Epilogues: plain fp32 store, fp32 residual add in place, or SwiGLU on interleaved gate/up columns
// with a bf16 result; each wavefront transposes its accumulators through LDS so that global memory is
// touched in 16-byte pieces per lane.
//
// Two-term activations.  With a_terms == 2 the A operand is [M, 2K]: columns 0..K-1 hold the bf16
// rounding of the activation ("hi") and K..2K-1 the bf16 rounding of what that rounding lost
// ("lo"); the k loop then runs over both halves against the same W, so the fp32 accumulator receives
// (hi + lo) . W - the product with a 16-bit-mantissa activation.  With out_terms == 2 the SwiGLU
// epilogue writes its result in the same [M, 2F] hi | lo form for the next GEMM.
//
// Operand formats.  The activation format a_fmt / out_fmt is 1 (bf16), 2 (two bf16 terms, above) or
// 3 (fp16: both A and W hold IEEE half values and the f16 MFMA is used; three more mantissa bits than
// bf16 at the same cost, for layers whose weights have been converted).
#include "kernels.h"
#include <algorithm>
#include <cmath>

namespace cs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

#define CS_GLOBAL_AS __attribute__((address_space(1)))
#define CS_LDS_AS __attribute__((address_space(3)))

// one 32x32x16 MFMA on 16-bit operands held as bf16x8 bit patterns: bf16 or (F16) IEEE half
template <bool F16>
__device__ inline f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// one 16x16x32 MFMA: the same flops per cycle as the 32x32x16 one at a lower energy per flop - with random operands the
// matrix pipe alone sustains about 2.08 PFLOP/s with it against 1.85 PFLOP/s (the clock the chip holds under load differs)
template <bool F16>
__device__ inline f32x4 mma16(bf16x8 a, bf16x8 b, f32x4 c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// vmcnt(n) only (expcnt / lgkmcnt left unconstrained), gfx9 encoding of s_waitcnt
#define CS_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// Workgroup barrier without the fences of __syncthreads().  Those fences make the compiler wait for every outstanding
// direct load (a direct load writes LDS), which would cut the prefetch depth of a multi-stage pipeline to one k-tile
// whatever count the explicit wait in front of the barrier names.  The waits that matter are stated next to each use.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
// vmcnt(n) and lgkmcnt(0): at most n direct loads of this wavefront in flight, all of its LDS reads returned
#define CS_WAIT_VMCNT_LDS(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (0 << 8))

// Tiles that keep their operands in a ring of five half-stages (see the kernel) and the dynamic LDS of a tile shape
constexpr bool ring_tile(int BM, int BN, int BK) { return BM == 256 && BN == 256 && BK == 64; }
constexpr int gemm_lds_bytes(int BM, int BN, int BK, int NS) { return ring_tile(BM, BN, BK) ? 5 * BM * BK * 2 : NS * (BM + BN) * BK * 2; }

// BK: k extent of one LDS stage (64 or 32 elements); NS: number of LDS stages.  NS - 1 k-tiles are
// kept in flight: (64, 2) has the fewest barriers, (32, 4) the deepest prefetch for the same LDS budget.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NS, int EPI, int A_FMT>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W,
                                                         void *out_v, int M, int N, int K,
                                                         int tiles_m, int tiles_n, int n_base, int group_m, int out_fmt, RopeArgs rope,
                                                         PrefetchArgs pf) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's name (buffer resources are a device-side type)
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int A_TERMS = A_FMT == 2 ? 2 : 1;
    constexpr bool F16 = A_FMT == 3;
    const int out_terms = out_fmt == 2 ? 2 : 1;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;   // wave tile
    constexpr int MI = WM / 32, NI = WN / 32;             // 32x32 MFMA blocks per wave
    constexpr int ROWB = BK * 2;                          // bytes of one tile row in LDS
    constexpr int VPR = ROWB / 16;                        // 16-byte k-vectors per row (8 or 4)
    constexpr int RPD = 1024 / ROWB;                      // rows filled by one 1 KiB direct load (8 or 16)
    constexpr int A_DMA = BM / (RPD * NW), B_DMA = BN / (RPD * NW);   // direct loads per wave per k-tile
    constexpr int PER_TILE = A_DMA + B_DMA;
    constexpr int STAGE = (BM + BN) * ROWB;               // bytes
    static_assert(BK == 64 || BK == 32, "BK");
    static_assert(BM % (RPD * NW) == 0 && BN % (RPD * NW) == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert(EPI != EPI_SWIGLU || WN % 64 == 0, "SwiGLU needs a gate/up column pair inside one wave tile");
    static_assert(EPI != EPI_ROPE || WN == 64, "the rotation pairs of a head half fill a 64-column wave tile");
    static_assert(NS >= 2 && NS <= 5, "stages");
    static_assert(MI * NI >= 2, "a k-step has at least two MFMAs");
    // 256 x 256 tiles take the loop that reads a k-tile's first operands during the previous tile's last k-step
    // 256 x 256 tiles: 16x16x32 MFMAs, operands in a ring of five half-stage units (NS == 5 counts those units)
    constexpr bool M16 = ring_tile(BM, BN, BK);
    static_assert(!M16 || (WAVES_M == 2 && WAVES_N == 4 && NS == 5), "256 x 256 tiles run 8 wavefronts on the ring of five units");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // XCD-aware tile order: consecutive workgroup ids land on different XCDs, so give each XCD a
    // contiguous range of the tile list.  The list walks the tile grid in bands of group_m tile rows,
    // tile_m fastest inside a band, so the workgroups that share one L2 at any time cover a roughly
    // square block of tiles (group_m x resident/group_m): what they fetch together is
    // group_m A panels + resident/group_m W panels, the minimum for that many tiles.
    int n_tiles = tiles_m * tiles_n;
    int bid = blockIdx.x;
    int per = (n_tiles + 7) >> 3;
    int lid = (bid & 7) * per + (bid >> 3);
    if (lid >= n_tiles) return;   // uniform per workgroup: no barrier is skipped by a subset
    int band = lid / (group_m * tiles_n), in_band = lid - band * group_m * tiles_n;
    int band_rows = min(group_m, tiles_m - band * group_m);
    int tm = band * group_m + in_band % band_rows, tn = in_band / band_rows;
    int m0 = tm * BM, n0 = n_base + tn * BN;   // a launch may cover the column range [n_base, n_base + tiles_n * BN) only

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: LDS targets of the direct loads are then scalar too
    int wy = wave / WAVES_N, wx = wave % WAVES_N;

    // Direct-load roles: instruction j of wave w fills rows RPD*(w + NW*j) .. of an operand tile; lane s
    // sits at row s / VPR, position s % VPR and fetches the k-vector that the swizzle puts there.
    // Swizzle: position = k-vector ^ ((row >> 1) & 7) for 128-byte rows, ^ ((row >> 2) & 3) for 64-byte
    // rows; either way 16 consecutive rows at one k-vector cover all 64 banks once.  A rows past M
    // are clamped (fetched twice, never stored to the output).
    // The loads are buffer loads: a scalar resource per operand that starts at the tile's first row, a 32-bit byte
    // offset per lane that is the same for every k-tile, and the k-tile's offset in a scalar register - no vector
    // instruction is needed to issue one.  (Offsets stay below 256 rows x 2 K x 2 bytes.)
    auto swz = [](int row) { return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
    const int rl = lane / VPR, ph = lane % VPR;
    const int lda = K * A_TERMS;
    const __amdgpu_buffer_rsrc_t a_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16 *>(A + (size_t)m0 * lda), 0, -1, 0x00020000);
    const __amdgpu_buffer_rsrc_t b_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16 *>(W + (size_t)n0 * K), 0, -1, 0x00020000);
    int a_off[A_DMA], b_off[B_DMA];
#pragma unroll
    for (int j = 0; j < A_DMA; ++j) {
        int row = RPD * (wave + NW * j) + rl;
        int g = ph ^ swz(row);
        a_off[j] = (min(m0 + row, M - 1) - m0) * lda * 2 + g * 16;
    }
#pragma unroll
    for (int j = 0; j < B_DMA; ++j) {
        int row = RPD * (wave + NW * j) + rl;
        int g = ph ^ swz(row);
        b_off[j] = row * K * 2 + g * 16;
    }
    int nk_w = K / BK;             // k-tiles of W
    int nk_all = nk_w * A_TERMS;   // k-tiles of the loop: with two-term A, the hi and the lo tile of every W k-tile
    // Split-K launches (gridDim.y > 1, plain-store epilogue only): slice y takes the k-tiles y, y + s, y + 2s, ...
    // (s = gridDim.y) and writes its partial product to the y-th [M, N] plane of the output.  The slices of a tile run
    // at the same time on the same XCD and walk the k range together, so at any moment they ask for s adjacent 128-byte
    // lines of an operand row rather than lines a slice length apart (worth 0.4 % of a pass against contiguous slices).
    const int kstep = gridDim.y;
    const int kb = blockIdx.y;
    const int nk = (nk_all - kb + kstep - 1) / kstep;
    if (EPI == EPI_STORE_F32) out_v = reinterpret_cast<float *>(out_v) + (size_t)blockIdx.y * M * N;
    // load j (A: 0 .. A_DMA-1, then W) of k-tile kt into LDS stage `stage`
    auto issue_one = [&](int stage, int kt, int j) __attribute__((always_inline)) {
        // Two-term A: k-tile kt pairs W k-tile kt / 2 with the hi (even kt) or lo (odd kt) half of A, so a W k-tile is
        // asked for twice in a row (the second time it is still in L2) rather than once per sweep over K.
        int kw = A_TERMS == 2 ? kt >> 1 : kt;
        int ka = (A_TERMS == 2 && (kt & 1)) ? nk_w + kw : kw;
        unsigned char *base = smem + stage * STAGE;
        if (j < A_DMA)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rs, (CS_LDS_AS void *)(base + (wave + NW * j) * 1024), 16, a_off[j < A_DMA ? j : 0],
                                                     ka * ROWB, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rs, (CS_LDS_AS void *)(base + BM * ROWB + (wave + NW * (j - A_DMA)) * 1024), 16,
                                                     b_off[j >= A_DMA ? j - A_DMA : 0], kw * ROWB, 0, 0);
    };
    auto issue_loads = [&](int stage, int kt) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < PER_TILE; ++j) issue_one(stage, kt, j);
    };

    f32x16 acc[M16 ? 1 : MI][M16 ? 1 : NI];
#pragma unroll
    for (int i = 0; i < (M16 ? 1 : MI); ++i)
#pragma unroll
        for (int j = 0; j < (M16 ? 1 : NI); ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    // 16x16 blocks: acc16[i][j][e] = C[16 i + 4 (lane / 16) + e][16 j + lane % 16] of the wave tile
    constexpr int MI16 = M16 ? WM / 16 : 1, NI16 = M16 ? WN / 16 : 1;
    f32x4 acc16[MI16][NI16];
#pragma unroll
    for (int i = 0; i < MI16; ++i)
#pragma unroll
        for (int j = 0; j < NI16; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc16[i][j][e] = 0.f;

    // MFMA operand reads: row (lane % 32) of each 32-row block, k-vector 2 ks + lane / 32
    const int half = lane >> 5;
    const int arow = wy * WM + (lane & 31), brow = wx * WN + (lane & 31);
    const int a_base = arow * ROWB, a_sw = swz(arow);          // rows 32 apart share the swizzle value
    const int b_base = BM * ROWB + brow * ROWB, b_sw = swz(brow);

    // MFMA q of a k-step: accumulator block (q / NI, q % NI)
    auto mfma_range = [&](const bf16x8 (&a_)[MI], const bf16x8 (&b_)[NI], int q0, int q1) __attribute__((always_inline)) {
#pragma unroll
        for (int q = q0; q < q1; ++q) acc[q / NI][q % NI] = mma<F16>(a_[q / NI], b_[q % NI], acc[q / NI][q % NI]);
    };
    constexpr int KS = BK / 16;   // k-steps of a k-tile
    constexpr int EARLY = 2;      // MFMAs of a k-step issued before the next step's operand reads
    if constexpr (M16) {
        // 256 x 256 tile, 8 wavefronts of 128 x 64, 16x16x32 MFMAs.  A k-tile is 16 slots (k half ks2 = slot / 8, 16-row
        // block i = slot % 8) of four MFMAs each (the four 16-column blocks).  Operands: the four W fragments of a k half
        // are double-buffered, the A fragments go through a ring of four (the one of slot s + 3 is requested in slot s);
        // an A fragment is row lane % 16 of its block, 16-byte k-vector 4 ks2 + lane / 16, at the swizzled position.
        // One barrier per k-tile, in front of slot 13: before it a wavefront has requested its last operands of the
        // k-tile (slot 15's in slot 12) and waits for them and for its own direct loads of the next k-tile; after it the
        // next k-tile is complete in LDS (its first operands are read in slots 13 - 15: the matrix pipe does not drain at
        // the tile boundary) and the LDS of the current one is free for direct loads.
        // The direct loads are issued one at a time between the MFMAs: a burst of them queues at the CU's one address
        // unit, and the wavefronts then wait at their load instructions instead of issuing MFMAs (measured with time stamps:
        // a third of a k-tile).  To give every load time to land although they are issued evenly, LDS holds 2.5 k-tiles: a
        // unit is the A or the W part of a k-tile (32 KiB, 4 loads per wavefront), unit u of the stream A(0) W(0) A(1) W(1)
        // .. lives in ring slot u % 5 of the 160 KiB, so the whole of k-tile t+1 and the A part of k-tile t+2 are in flight
        // while k-tile t is multiplied.  One load in every second slot: 13, 15 of k-tile t and 1, 3 of k-tile t+1 make unit
        // 2t+5 (into the slot of A(t), free since the barrier), 5 .. 11 of k-tile t+1 make unit 2t+6 (slot of W(t)); each
        // has at least 10 slots to land.  At the barrier of k-tile t everything up to unit 2t+3 must have landed: direct
        // loads complete in order, so at most the four loads of unit 2t+4 may be outstanding.
        static_assert(A_DMA == 4 && B_DMA == 4, "256 x 256 tile, 8 wavefronts");
        constexpr int UNIT = BM * ROWB;   // 32 KiB: the A or the W part of a k-tile
        const int l16 = lane & 15, kq = lane >> 4;
        const int sw16 = (l16 >> 1) & 7;                                   // blocks start at multiples of 16 rows
        const int a_row_off = (wy * WM + l16) * ROWB, b_row_off = (wx * WN + l16) * ROWB;
        int kv_off[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) kv_off[h] = ((4 * h + kq) ^ sw16) * 16;
        bf16x8 a16[4], b16[2][4];
        // this lane's fragment offsets inside a unit for the two k halves; per k-tile they are added to the units' bases
        // once (five additions), every read is then that pointer plus a constant
        int a_lane[2], b_lane[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) { a_lane[h] = a_row_off + kv_off[h]; b_lane[h] = b_row_off + kv_off[h]; }
        auto read_a = [&](const unsigned char *pa, int s) __attribute__((always_inline)) {   // slot s; pa: the k half's pointer
            a16[s & 3] = *reinterpret_cast<const bf16x8 *>(pa + (s & 7) * 16 * ROWB);
        };
        auto read_b = [&](const unsigned char *pb, int h, int j) __attribute__((always_inline)) {
            b16[h][j] = *reinterpret_cast<const bf16x8 *>(pb + j * 16 * ROWB);
        };
        // direct load j of the A (w == 0) or W (w == 1) part of k-tile t of this workgroup's loop into LDS at dst
        auto issue = [&](int t, int w, int j, unsigned char *dst) __attribute__((always_inline)) {
            const int kt = kb + t * kstep;
            const int kw = A_TERMS == 2 ? kt >> 1 : kt;
            const int ka = (A_TERMS == 2 && (kt & 1)) ? nk_w + kw : kw;
            if (w) __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rs, (CS_LDS_AS void *)(dst + (wave + NW * j) * 1024), 16, b_off[j], kw * ROWB, 0, 0);
            else __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rs, (CS_LDS_AS void *)(dst + (wave + NW * j) * 1024), 16, a_off[j], ka * ROWB, 0, 0);
        };
        // LDS position of unit u = 2 t + w: ring slot u % 5
        auto unit_ptr = [&](int u) -> unsigned char * { return smem + (u % 5) * UNIT; };
        const int n_units = 2 * nk;
#pragma unroll
        for (int u = 0; u < 5; ++u)
            if (u < n_units) {
#pragma unroll
                for (int j = 0; j < 4; ++j) issue(u >> 1, u & 1, j, unit_ptr(u));
            }
        // units 0 and 1 have landed when at most the later ones are outstanding
        if (n_units >= 5) CS_WAIT_VMCNT_LDS(12);
        else if (n_units >= 4) CS_WAIT_VMCNT_LDS(8);
        else CS_WAIT_VMCNT_LDS(0);
        wg_barrier();
#pragma unroll
        for (int s = 0; s < 3; ++s) read_a(smem + a_lane[0], s);
#pragma unroll
        for (int j = 0; j < 4; ++j) read_b(smem + UNIT + b_lane[0], 0, j);
        int sl0 = 0;   // ring slot of unit 2 ki (the A part of the current k-tile); the following units in the next slots
        for (int ki = 0; ki < nk; ++ki) {
            auto next_slot = [](int v) { return v == 4 ? 0 : v + 1; };
            const int sl1 = next_slot(sl0), sl2 = next_slot(sl1), sl3 = next_slot(sl2), sl4 = next_slot(sl3);   // units 2 ki + 1 .. + 4
            unsigned char *const u0 = smem + sl0 * UNIT, *const u3 = smem + sl3 * UNIT, *const u4 = smem + sl4 * UNIT;
            const unsigned char *ua = u0, *ub = smem + sl1 * UNIT;
            const unsigned char *pa0 = ua + a_lane[0], *pa1 = ua + a_lane[1], *pb1 = ub + b_lane[1];
            const unsigned char *npa0 = smem + sl2 * UNIT + a_lane[0], *npb0 = u3 + b_lane[0];
            const bool more = ki + 1 < nk;   // uniform
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                __builtin_amdgcn_sched_barrier(0);
                if (s == 13 && more) {
                    if (2 * ki + 4 < n_units) CS_WAIT_VMCNT_LDS(4);
                    else CS_WAIT_VMCNT_LDS(0);
                    wg_barrier();
                }
                // the direct load of this slot, if any: unit and load index
                int lu = -1, lj = 0;
                unsigned char *ldst = u0;                      // unit 2 ki + 5 takes the slot of unit 2 ki
                if (s == 13 || s == 15) { lu = 2 * ki + 5; lj = (s - 13) >> 1; }
                else if (s == 1 || s == 3) { lu = ki >= 1 ? 2 * ki + 3 : -1; lj = 2 + (s >> 1); ldst = u3; }
                else if (s >= 5 && s <= 11 && (s & 1)) { lu = ki >= 1 ? 2 * ki + 4 : -1; lj = (s - 5) >> 1; ldst = u4; }
                const int i = s & 7, h = s >> 3;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    __builtin_amdgcn_sched_barrier(0);
                    acc16[i][j] = mma16<F16>(a16[s & 3], b16[h][j], acc16[i][j]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (j == 0) {                              // A fragment of slot s + 3
                        if (s + 3 < 16) read_a(s + 3 < 8 ? pa0 : pa1, s + 3);
                        else if (more) read_a(npa0, s + 3 - 16);
                    }
                    if (j == 1) {                              // W fragments of the next k half
                        if (s >= 4 && s < 8) read_b(pb1, 1, s - 4);
                        else if (s >= 13 && s < 15 && more) read_b(npb0, 0, 2 * (s - 13));
                    }
                    if (j == 2 && s >= 13 && s < 15 && more) read_b(npb0, 0, 2 * (s - 13) + 1);
                    if (j == 3 && lu >= 0 && lu < n_units) issue(lu >> 1, lu & 1, lj, ldst);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            sl0 = sl2;
        }
    } else
    {
    // Pipeline: k-tiles kt+1 .. kt+NS-1 are in flight while k-tile kt is multiplied.  Direct loads
    // complete in order per wave, so "at most PER_TILE * r outstanding" means this wave's part of tile
    // kt has landed when r tiles were issued after it; the barrier extends that to every wave and also
    // tells that everybody is done with the stage the next loads will overwrite.
#pragma unroll
    for (int t = 0; t < NS - 1; ++t)
        if (t < nk) issue_loads(t, kb + t * kstep);
    for (int ki = 0; ki < nk; ++ki) {
        const int kt = kb + ki * kstep;
        int after = min(NS - 2, nk - 1 - ki);
        if (after >= 2) CS_WAIT_VMCNT_LDS(2 * PER_TILE);
        else if (after == 1) CS_WAIT_VMCNT_LDS(PER_TILE);
        else CS_WAIT_VMCNT_LDS(0);
        wg_barrier();
        const unsigned char *cur = smem + (ki % NS) * STAGE;
        bf16x8 af[2][MI], bfr[2][NI];
        auto read_frags = [&](int buf, int ks) {
            int ga = ((2 * ks + half) ^ a_sw) * 16, gb = ((2 * ks + half) ^ b_sw) * 16;
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[buf][i] = *reinterpret_cast<const bf16x8 *>(cur + a_base + i * 32 * ROWB + ga);
#pragma unroll
            for (int j = 0; j < NI; ++j)
                bfr[buf][j] = *reinterpret_cast<const bf16x8 *>(cur + b_base + j * 32 * ROWB + gb);
        };
        // The first operands of this k-tile are requested before the next tile's loads are issued, so
        // their LDS latency passes under the address arithmetic of those loads.  Inside a k-step the
        // operands of the next step are requested after the first MFMAs and have the rest of the step to
        // arrive: the one wait in front of a step's first MFMA then only covers reads issued most of a
        // step earlier.  The scheduling barriers pin that order (left alone, the compiler sinks the reads
        // to save registers, and every group of MFMAs waits out its own LDS latency).
        read_frags(0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (ki + NS - 1 < nk) issue_loads((ki + NS - 1) % NS, kt + (NS - 1) * kstep);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            __builtin_amdgcn_sched_barrier(0);
            mfma_range(af[ks & 1], bfr[ks & 1], 0, EARLY);
            __builtin_amdgcn_sched_barrier(0);
            if (ks + 1 < KS) read_frags((ks + 1) & 1, ks + 1);
            __builtin_amdgcn_sched_barrier(0);
            mfma_range(af[ks & 1], bfr[ks & 1], EARLY, MI * NI);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    }

    // ---- epilogue.  The accumulator layout of a 32x32 block gives a lane one column and 16 rows, so
    // stores straight from it are 2- or 4-byte pieces per lane, and the store path retires a wavefront
    // instruction in about 16 cycles whatever its width.  Each wavefront therefore transposes one 32-row
    // block at a time through a private piece of LDS (the operand stages are dead by now) and moves
    // 16 bytes per lane to and from global memory.
    // Warm-up of memory the next kernel will read (the down projection's weights while the gate/up projection, which
    // leaves HBM idle, finishes a tile): every workgroup reads its slice once, front to back, so the data is in the
    // last-level cache when that kernel's strided tile loads ask for it.  The values are not used.
    constexpr int PF_VEC = 5;
    u32x4 pfv[PF_VEC];
    const bool do_pf = EPI == EPI_SWIGLU && pf.n16 != 0;
    if (do_pf) {
        constexpr unsigned NTHR = 64 * NW;
        unsigned per = min((pf.n16 + (unsigned)n_tiles - 1) / (unsigned)n_tiles, (unsigned)PF_VEC * NTHR);
        unsigned base = (unsigned)lid * per;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(pf.ptr);
#pragma unroll
        for (int i = 0; i < PF_VEC; ++i) {
            unsigned off = (unsigned)i * NTHR + (unsigned)tid;
            u32x4 z = {0u, 0u, 0u, 0u};
            pfv[i] = (off < per && base + off < pf.n16) ? src[base + off] : z;
        }
    }
    constexpr int WNO = (EPI == EPI_SWIGLU) ? WN / 2 : WN;   // output columns of a wave tile
    // staging row stride in words: the row groups of a write (two, 4 rows apart, for 32x32 blocks; four for 16x16 blocks)
    // hit disjoint banks with 4 * SROW % 64 == 32 or 16
    constexpr int SROW = M16 ? WNO + 4 : WNO + 8;
    static_assert(NW * 32 * SROW * 4 <= gemm_lds_bytes(BM, BN, BK, NS), "epilogue staging does not fit the operand stages");
    __syncthreads();                                         // every wavefront is done with the operand stages
    float *stg = reinterpret_cast<float *>(smem) + wave * 32 * SROW;
    const int col_l = lane & 31, row_l = (lane >> 5) * 4;    // C layout: column lane%32, rows 8*(e/4) + 4*(lane/32) + e%4
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        if constexpr (M16) {
            // rows 32 i .. 32 i + 31 of the wave tile are the 16-row blocks 2 i and 2 i + 1
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float *srow = stg + (16 * i2 + 4 * (lane >> 4) + e) * SROW + (lane & 15);
                    if (EPI == EPI_SWIGLU) {
                        // columns 64 c .. 64 c + 31 hold gate values and the 32 after them the matching up values
#pragma unroll
                        for (int j = 0; j < NI16; ++j)
                            if ((j & 3) < 2) {
                                float gte = acc16[2 * i + i2][j][e], up = acc16[2 * i + i2][j + 2][e];
                                srow[(j >> 2) * 32 + (j & 1) * 16] = gte * __builtin_amdgcn_rcpf(1.0f + __expf(-gte)) * up;
                            }
                    } else {
#pragma unroll
                        for (int j = 0; j < NI16; ++j) srow[j * 16] = acc16[2 * i + i2][j][e];
                    }
                }
        } else
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float *srow = stg + ((e >> 2) * 8 + row_l + (e & 3)) * SROW + col_l;
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int j = 0; j < NI; j += 2) {
                    // silu(g) * u with the hardware reciprocal (1 ulp): far below the bf16 rounding of the result,
                    // and a third of the instructions of an IEEE division
                    float gte = acc[i][j][e], up = acc[i][j + 1][e];
                    srow[(j >> 1) * 32] = gte * __builtin_amdgcn_rcpf(1.0f + __expf(-gte)) * up;
                }
            } else {
#pragma unroll
                for (int j = 0; j < NI; ++j) srow[j * 32] = acc[i][j][e];
            }
        }
        // LDS operations of one wavefront execute in order; the fence keeps the compiler from moving the
        // reads of other lanes' values above the writes.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int mrow0 = m0 + wy * WM + i * 32;
        if (EPI == EPI_SWIGLU) {
            constexpr int LPR = WNO / 8, RP = 64 / LPR;      // lanes per output row (8 bf16 each), rows per pass
            bf16 *out = reinterpret_cast<bf16 *>(out_v);
            const int Fo = N >> 1;
            const int f0 = ((n0 + wx * WN) >> 1) + (lane % LPR) * 8;
#pragma unroll
            for (int p = 0; p < 32 / RP; ++p) {
                int r = p * RP + lane / LPR, m = mrow0 + r;
                const f32x4 *src = reinterpret_cast<const f32x4 *>(stg + r * SROW + (lane % LPR) * 8);
                f32x4 v0 = src[0], v1 = src[1];
                float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                if (m < M) {
                    bf16 *dst = out + (size_t)m * Fo * out_terms + f0;
                    unsigned hi[8];
                    if (out_fmt == 3) {
#pragma unroll
                        for (int q = 0; q < 8; ++q) hi[q] = __half_as_ushort(to_half_sat(v[q]));
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q) hi[q] = __bfloat16_as_ushort(__float2bfloat16(v[q]));
                    }
                    u32x4 ph = {hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16)};
                    *reinterpret_cast<u32x4 *>(dst) = ph;
                    if (out_fmt == 2) {
                        unsigned lo[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q)
                            lo[q] = __bfloat16_as_ushort(
                                __float2bfloat16(v[q] - __bfloat162float(__ushort_as_bfloat16((unsigned short)hi[q]))));
                        u32x4 pl = {lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16)};
                        *reinterpret_cast<u32x4 *>(dst + Fo) = pl;
                    }
                }
            }
        } else if (EPI == EPI_ROPE) {
            // Staged columns 0..31 are columns c0..c0+31 of a head and columns 32..63 their rotation partners
            // c0+64.. (c0 = 0 or 32).  A lane takes 8 columns of a row and the 8 partners.
            const int n_w = n0 + wx * WN;
            const int head = n_w >> 7, c0 = ((n_w >> 6) & 1) * 32 + (lane & 3) * 8;
            const bool is_q = head < rope.Hq, is_v = head >= rope.Hq + rope.Hkv;
            const int hh = is_q ? head : is_v ? head - rope.Hq - rope.Hkv : head - rope.Hq;
            const int heads = is_q ? rope.Hq : rope.Hkv;
            bf16 *dst_hi = reinterpret_cast<bf16 *>(is_q ? rope.q : is_v ? rope.v : rope.k);
            bf16 *dst_lo = reinterpret_cast<bf16 *>(is_q ? rope.q_lo : is_v ? rope.v_lo : rope.k_lo);
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                int r = p * 16 + (lane >> 2), m = mrow0 + r;
                const f32x4 *sa = reinterpret_cast<const f32x4 *>(stg + r * SROW + (lane & 3) * 8);
                const f32x4 *sb = reinterpret_cast<const f32x4 *>(stg + r * SROW + 32 + (lane & 3) * 8);
                f32x4 a0 = sa[0], a1 = sa[1], b0 = sb[0], b1 = sb[1];
                if (m < M) {
                    float va[8] = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                    float vb[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
                    if (!is_v) {
                        const f32x4 *cp = reinterpret_cast<const f32x4 *>(rope.cos_t + (size_t)m * 64 + c0);
                        const f32x4 *sp = reinterpret_cast<const f32x4 *>(rope.sin_t + (size_t)m * 64 + c0);
                        f32x4 c_0 = cp[0], c_1 = cp[1], s_0 = sp[0], s_1 = sp[1];
                        float cs[8] = {c_0[0], c_0[1], c_0[2], c_0[3], c_1[0], c_1[1], c_1[2], c_1[3]};
                        float sn[8] = {s_0[0], s_0[1], s_0[2], s_0[3], s_1[0], s_1[1], s_1[2], s_1[3]};
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            float lo_ = va[q], hi_ = vb[q];
                            va[q] = lo_ * cs[q] - hi_ * sn[q];
                            vb[q] = hi_ * cs[q] + lo_ * sn[q];
                        }
                    }
                    size_t o = ((size_t)m * heads + hh) * 128 + c0;
                    unsigned ha[8], hb[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        ha[q] = __bfloat16_as_ushort(__float2bfloat16(va[q]));
                        hb[q] = __bfloat16_as_ushort(__float2bfloat16(vb[q]));
                    }
                    u32x4 pa = {ha[0] | (ha[1] << 16), ha[2] | (ha[3] << 16), ha[4] | (ha[5] << 16), ha[6] | (ha[7] << 16)};
                    u32x4 pb = {hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16), hb[4] | (hb[5] << 16), hb[6] | (hb[7] << 16)};
                    *reinterpret_cast<u32x4 *>(dst_hi + o) = pa;
                    *reinterpret_cast<u32x4 *>(dst_hi + o + 64) = pb;
                    if (dst_lo) {
                        unsigned la[8], lb[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            la[q] = __bfloat16_as_ushort(__float2bfloat16(va[q] - __bfloat162float(__ushort_as_bfloat16((unsigned short)ha[q]))));
                            lb[q] = __bfloat16_as_ushort(__float2bfloat16(vb[q] - __bfloat162float(__ushort_as_bfloat16((unsigned short)hb[q]))));
                        }
                        u32x4 qa = {la[0] | (la[1] << 16), la[2] | (la[3] << 16), la[4] | (la[5] << 16), la[6] | (la[7] << 16)};
                        u32x4 qb = {lb[0] | (lb[1] << 16), lb[2] | (lb[3] << 16), lb[4] | (lb[5] << 16), lb[6] | (lb[7] << 16)};
                        *reinterpret_cast<u32x4 *>(dst_lo + o) = qa;
                        *reinterpret_cast<u32x4 *>(dst_lo + o + 64) = qb;
                    }
                }
            }
        } else {
            constexpr int LPR = WNO / 4, RP = 64 / LPR;      // lanes per output row (4 floats each), rows per pass
            float *out = reinterpret_cast<float *>(out_v);
#pragma unroll
            for (int p = 0; p < 32 / RP; ++p) {
                int r = p * RP + lane / LPR, m = mrow0 + r;
                f32x4 v = *reinterpret_cast<const f32x4 *>(stg + r * SROW + (lane % LPR) * 4);
                if (m < M) {
                    f32x4 *dst = reinterpret_cast<f32x4 *>(out + (size_t)m * N + n0 + wx * WN + (lane % LPR) * 4);
                    if (EPI == EPI_RESID_F32) v += *dst;
                    *dst = v;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if (do_pf) {
#pragma unroll
        for (int i = 0; i < PF_VEC; ++i) asm volatile("" ::"v"(pfv[i]));   // the loads must not be dropped as unused
    }
#endif
}

// The number of activation terms is a template parameter, so the one-term and the two-term launches
// are different kernels (and show up under different names in a kernel trace).
// Launches the kernel on the column range [n_base, n_base + n_cols) of the N columns.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NS, int EPI, int A_FMT>
static hipError_t launch_inst(const GemmTune &tune, const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int n_base,
                              int n_cols, int out_terms, hipStream_t s, const RopeArgs *rope = nullptr,
                              const PrefetchArgs *pf = nullptr) {
    constexpr int smem = gemm_lds_bytes(BM, BN, BK, NS);
    static std::atomic<uint32_t> attr_done{0};
    auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, BK, NS, EPI, A_FMT>;
    if (hipError_t e = set_dynamic_lds_once(attr_done, reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
    int tiles_m = (M + BM - 1) / BM, tiles_n = n_cols / BN;
    int n_tiles = tiles_m * tiles_n;
    int grid = ((n_tiles + 7) / 8) * 8;
    // Workgroups of one XCD that run at the same time: its share of the tiles, at most 32 CUs x the
    // workgroups that fit one CU's 160 KiB of LDS.  A square block of that many tiles, weighted by the
    // tile's aspect, has sqrt(resident * BN / BM) rows.
    int group_m = tune.group_m;
    if (group_m <= 0) {
        int fit = 160 * 1024 / smem;
        int resident = std::min((n_tiles + 7) / 8, 32 * std::max(fit, 1));
        group_m = (int)std::lround(std::sqrt((double)resident * BN / BM));
    }
    group_m = std::max(1, std::min(group_m, tiles_m));
    kern<<<grid, 64 * WAVES_M * WAVES_N, smem, s>>>(A, W, out, M, N, K, tiles_m, tiles_n, n_base, group_m, out_terms,
                                                    rope ? *rope : RopeArgs{}, pf ? *pf : PrefetchArgs{});
    return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NS, int EPI>
static hipError_t launch_tile(const GemmTune &tune, const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int n_base,
                              int n_cols, int a_fmt, int out_fmt, hipStream_t s, const RopeArgs *rope = nullptr,
                              const PrefetchArgs *pf = nullptr) {
    if (a_fmt == 2)
        return launch_inst<BM, BN, WAVES_M, WAVES_N, BK, NS, EPI, 2>(tune, A, W, out, M, N, K, n_base, n_cols, out_fmt, s, rope, pf);
    if (a_fmt == 3) {
        // fp16 operands: built for the tile shapes the default choice uses
        constexpr bool has_f16 = (BK == 64 && NS == 2 && ((BM == 128 && BN == 128 && WAVES_M == 2 && WAVES_N == 2) ||
                                                            (BM == 192 && BN == 96 && WAVES_M == 2 && WAVES_N == 3))) ||
                                 (BM == 256 && BN == 256 && WAVES_M == 2);
        if constexpr (has_f16)
            return launch_inst<BM, BN, WAVES_M, WAVES_N, BK, NS, EPI, 3>(tune, A, W, out, M, N, K, n_base, n_cols, out_fmt, s, rope, pf);
        else
            return hipErrorInvalidValue;
    }
    return launch_inst<BM, BN, WAVES_M, WAVES_N, BK, NS, EPI, 1>(tune, A, W, out, M, N, K, n_base, n_cols, out_fmt, s, rope, pf);
}

// Tile ids: 1 = 128x128 / 4 waves, 4 = 256x256 / 8 waves, 7 = 192x96 / 6 waves (2 x 3, wave tile 96 x 32; for
// N % 96 == 0 and no SwiGLU); all with 64-element k-tiles in 2 stages.  Measured on the draft-model shapes: 4 is the
// fastest for the wide gate/up projection, 1 or 7 for the others.
// 256 x 256 tiles (one workgroup per CU, rounds of 256) or 128 x 128 tiles (two per CU, rounds of 512) for an output
// that is not split?  Measured time per k-tile of a round: 1.4 us for the large tile however full the round is; for the
// small tile 1.1 us for a full round, 0.73 us when every CU holds at most one workgroup, in between linearly.
static bool prefer_256_tiles(int M, int N) {
    if (N % 256 != 0) return false;
    long t128 = (long)((M + 127) / 128) * (N / 128), t256 = (long)((M + 255) / 256) * (N / 256);
    long rem = t128 % 512;
    double c128 = (double)(t128 / 512) * 1.1 + (rem == 0 ? 0.0 : rem <= 256 ? 0.73 : 0.73 + (double)(rem - 256) / 256.0 * 0.37);
    double c256 = (double)((t256 + 255) / 256) * 1.4;
    return c256 < c128;
}

template <int EPI>
static hipError_t launch_epi(const GemmTune &tune, const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int a_terms,
                             int out_terms, hipStream_t s, const PrefetchArgs *pf = nullptr) {
    int tile = tune.tile;
    if (tile == 0) {
        // Wide outputs take 256x256 tiles, one workgroup per CU, in rounds of 256 tiles.  A last round
        // that would be less than half full costs as much as a full one, so those columns are cut off
        // and done by a second launch with 128x128 tiles (two workgroups per CU), which is shorter.
        int tm = (M + 255) / 256, tn = N / 256;
        long t256 = (long)tm * tn;
        if (!prefer_256_tiles(M, N)) {
            // 128x128 tiles run two per CU; a count a little above 256 leaves most CUs with one workgroup, which
            // runs at well under the rate of two.  If the same output is at most 256 tiles of 192x96 (the same
            // flop per staged byte), one such tile per CU is the better cut: 3072 x 1536 = 288 -> 256 tiles.
            if constexpr (EPI != EPI_SWIGLU) {
                long t128 = (long)((M + 127) / 128) * (N / 128), t192 = (long)((M + 191) / 192) * (N / 96);
                if (N % 96 == 0 && t128 > 256 && t128 <= 384 && t192 <= 256)
                    return launch_tile<192, 96, 2, 3, 64, 2, EPI>(tune, A, W, out, M, N, K, 0, N, a_terms, out_terms, s);
            }
            return launch_tile<128, 128, 2, 2, 64, 2, EPI>(tune, A, W, out, M, N, K, 0, N, a_terms, out_terms, s);
        }
        long rounds = t256 / 256;
        int n1 = tn;
        if (rounds >= 1 && t256 - rounds * 256 > 0) {
            int full = (int)(rounds * 256 / tm);             // tile columns that fill whole rounds
            if ((long)(tn - full) * tm <= 128) n1 = full;
        }
        if (n1 > 0) {
            hipError_t e = launch_tile<256, 256, 2, 4, 64, 5, EPI>(tune, A, W, out, M, N, K, 0, n1 * 256, a_terms, out_terms, s, nullptr, pf);
            if (e != hipSuccess) return e;
        }
        if (n1 < tn)
            return launch_tile<128, 128, 2, 2, 64, 2, EPI>(tune, A, W, out, M, N, K, n1 * 256, N - n1 * 256, a_terms,
                                                           out_terms, s);
        return hipSuccess;
    }
    if (tile == 4 && N % 256 != 0) tile = 1;
    if (tile == 7 && (N % 96 != 0 || EPI == EPI_SWIGLU)) tile = 1;
    switch (tile) {
        case 4: return launch_tile<256, 256, 2, 4, 64, 5, EPI>(tune, A, W, out, M, N, K, 0, N, a_terms, out_terms, s);
        case 7:
            if constexpr (EPI != EPI_SWIGLU) return launch_tile<192, 96, 2, 3, 64, 2, EPI>(tune, A, W, out, M, N, K, 0, N, a_terms, out_terms, s);
            else return hipErrorInvalidValue;   // not reached: a SwiGLU column pair needs 64-column wave tiles
        default: return launch_tile<128, 128, 2, 2, 64, 2, EPI>(tune, A, W, out, M, N, K, 0, N, a_terms, out_terms, s);
    }
}

// ---- split-K for short outputs -----------------------------------------------------------------
// With M <= 128 there is one tile row, so a [M, N] output gives N / 128 workgroups, each walking all of
// K: a few CUs work for a long time.  Instead the k range is cut into slices, every (tile, slice) pair
// is a workgroup that stores its partial product, and a second kernel adds the slices in a fixed order
// and applies the epilogue.
//
// A second case: a long k range (K_total >= 4096) over an output that 128 x 128 tiles do cover but 256 x 256 tiles
// fill only a third to a sixth of the chip with.  Tiles of 128 or 192 x 96 are bound by the rate at which their operands
// arrive from the L2 (a 256 x 256 tile needs half the bytes per flop), so there the k range is cut into 3..6 slices of
// 256 x 256 tiles, one workgroup per CU, and the reduction pass that follows costs less than the tiles gain
// (3072 x 1536 x 8960: 97 us with 3 slices against 106 us for 256 tiles of 192 x 96, and the reduction can also
// normalise the rows for the next GEMM).  From 256 k-tiles on two slices pay as well (1536 x 5120 x 27648).
// *big_tile says which case applies.
int gemm_splitk_factor(const GemmTune &tune, int M, int N, int K_total, bool *big_tile) {
    if (big_tile) *big_tile = false;
    if (N % 128 != 0) return 1;
    int tiles = ((M + 127) / 128) * (N / 128), nk = K_total / 64;
    if (tune.splitk > 0) return std::max(1, std::min(tune.splitk, nk / 4));
    if (M > 128 && tiles >= 256) {                       // enough 128 x 128 tiles to fill the chip without a split
        int t256 = ((M + 255) / 256) * (N / 256);
        int s = t256 > 0 ? 256 / t256 : 0;
        if (big_tile && N % 256 == 0 && nk >= 64 && s >= (nk >= 256 ? 2 : 3) && s <= 6 && t256 * s >= 192) {
            *big_tile = true;
            return s;
        }
        return 1;
    }
    if (big_tile && M > 256 && N % 256 == 0 && nk >= 64) {
        // Few tiles, more than 256 rows and a long k range: again 256 x 256 tiles, one workgroup per CU (d_model 5120,
        // d_ffn 27648 over 480 rows: 38.9 ms per pass against 45.6 ms with 128 x 128 tiles; 288 rows: equal; 192 rows:
        // 28.7 against 24.6 ms, hence the row bound).
        int t256 = ((M + 255) / 256) * (N / 256);
        int s = std::min(std::min(256 / t256, nk / 4), 64);
        if (s >= 2) {
            *big_tile = true;
            return s;
        }
    }
    int want = (384 + tiles / 2) / tiles;                // about 384 workgroups
    // at least 4 k-tiles per slice; 2 for the 32-row tile, whose four LDS stages keep a short slice streaming
    int s = std::min(want, nk / ((M <= 32 && tune.short_tile) ? 2 : 4));
    return std::max(1, std::min(s, 64));
}
size_t gemm_splitk_bytes(const GemmTune &tune, int M, int N, int K_total) {
    bool big;
    int s = gemm_splitk_factor(tune, M, N, K_total, &big);
    return s > 1 ? (size_t)s * M * N * 4 : 0;
}
// Largest gemm_splitk_bytes over all row counts up to max_M (the factor changes with the number of row tiles).
size_t gemm_splitk_max_bytes(const GemmTune &tune, int max_M, int N, int K_total) {
    size_t best = 0;
    for (int tm = 1; tm <= (max_M + 127) / 128; ++tm)
        best = std::max(best, gemm_splitk_bytes(tune, std::min(tm * 128, max_M), N, K_total));
    return best;
}

template <int EPI>
__global__ void splitk_reduce_kernel(const float *__restrict__ part, int splits, int M, int N, void *__restrict__ out_v,
                                     int out_terms) {
    // one thread per 4 output columns of one row
    int n_out = EPI == EPI_SWIGLU ? N / 2 : N;
    int c4 = (blockIdx.x * blockDim.x + threadIdx.x) * 4, r = blockIdx.y;
    if (c4 >= n_out) return;
    size_t plane = (size_t)M * N;
    if (EPI == EPI_SWIGLU) {
        int gc = 64 * (c4 / 32) + c4 % 32;               // packed column of the gate value; its up value is 32 further
        f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = g;
#pragma unroll 4
        for (int sp = 0; sp < splits; ++sp) {
            const float *p = part + sp * plane + (size_t)r * N + gc;
            g += *reinterpret_cast<const f32x4 *>(p);
            u += *reinterpret_cast<const f32x4 *>(p + 32);
        }
        bf16 *out = reinterpret_cast<bf16 *>(out_v) + (size_t)r * n_out * (out_terms == 2 ? 2 : 1) + c4;
        unsigned hi[4], lo[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float act = g[q] * __builtin_amdgcn_rcpf(1.0f + __expf(-g[q])) * u[q];
            if (out_terms == 3) {
                hi[q] = __half_as_ushort(to_half_sat(act));
                lo[q] = 0;
            } else {
                bf16 h = __float2bfloat16(act);
                hi[q] = __bfloat16_as_ushort(h);
                lo[q] = __bfloat16_as_ushort(__float2bfloat16(act - __bfloat162float(h)));
            }
        }
        uint2 ph = {hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
        *reinterpret_cast<uint2 *>(out) = ph;
        if (out_terms == 2) {
            uint2 pl = {lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
            *reinterpret_cast<uint2 *>(out + n_out) = pl;
        }
    } else {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int sp = 0; sp < splits; ++sp)
            acc += *reinterpret_cast<const f32x4 *>(part + sp * plane + (size_t)r * N + c4);
        f32x4 *dst = reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(out_v) + (size_t)r * N + c4);
        if (EPI == EPI_RESID_F32) acc += *dst;
        *dst = acc;
    }
}

// Sum of the split-K slices of a QKV projection made with the reordered weight rows (see RopeArgs), rotation
// of q and k, and the q / k / v split.  Inside a head the reordered columns are [0..31 | 64..95 | 32..63 | 96..127]
// of the original order, so a column and its rotation partner lie 32 apart.  One thread per 4 columns + 4 partners.
__global__ void splitk_reduce_rope_kernel(const float *__restrict__ part, int splits, int M, int N, RopeArgs rope) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x, m = blockIdx.y;
    int per_row = (N / 128) * 16;
    if (idx >= per_row) return;
    int head = idx >> 4, g = (idx >> 3) & 1, j = idx & 7;
    int pc = head * 128 + g * 64 + j * 4, c0 = g * 32 + j * 4;
    size_t plane = (size_t)M * N;
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = a;
#pragma unroll 4
    for (int sp = 0; sp < splits; ++sp) {
        const float *p = part + sp * plane + (size_t)m * N + pc;
        a += *reinterpret_cast<const f32x4 *>(p);
        b += *reinterpret_cast<const f32x4 *>(p + 32);
    }
    const bool is_q = head < rope.Hq, is_v = head >= rope.Hq + rope.Hkv;
    const int hh = is_q ? head : is_v ? head - rope.Hq - rope.Hkv : head - rope.Hq;
    const int heads = is_q ? rope.Hq : rope.Hkv;
    bf16 *dst_hi = reinterpret_cast<bf16 *>(is_q ? rope.q : is_v ? rope.v : rope.k);
    bf16 *dst_lo = reinterpret_cast<bf16 *>(is_q ? rope.q_lo : is_v ? rope.v_lo : rope.k_lo);
    if (!is_v) {
        f32x4 c = *reinterpret_cast<const f32x4 *>(rope.cos_t + (size_t)m * 64 + c0);
        f32x4 sn = *reinterpret_cast<const f32x4 *>(rope.sin_t + (size_t)m * 64 + c0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float lo_ = a[q], hi_ = b[q];
            a[q] = lo_ * c[q] - hi_ * sn[q];
            b[q] = hi_ * c[q] + lo_ * sn[q];
        }
    }
    size_t o = ((size_t)m * heads + hh) * 128 + c0;
    unsigned ha[4], hb[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        ha[q] = __bfloat16_as_ushort(__float2bfloat16(a[q]));
        hb[q] = __bfloat16_as_ushort(__float2bfloat16(b[q]));
    }
    *reinterpret_cast<uint2 *>(dst_hi + o) = uint2{ha[0] | (ha[1] << 16), ha[2] | (ha[3] << 16)};
    *reinterpret_cast<uint2 *>(dst_hi + o + 64) = uint2{hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16)};
    if (dst_lo) {
        unsigned la[4], lb[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            la[q] = __bfloat16_as_ushort(__float2bfloat16(a[q] - __bfloat162float(__ushort_as_bfloat16((unsigned short)ha[q]))));
            lb[q] = __bfloat16_as_ushort(__float2bfloat16(b[q] - __bfloat162float(__ushort_as_bfloat16((unsigned short)hb[q]))));
        }
        *reinterpret_cast<uint2 *>(dst_lo + o) = uint2{la[0] | (la[1] << 16), la[2] | (la[3] << 16)};
        *reinterpret_cast<uint2 *>(dst_lo + o + 64) = uint2{lb[0] | (lb[1] << 16), lb[2] | (lb[3] << 16)};
    }
}

// Split-K slices of a residual projection summed in their fixed order, added to the residual stream, and the RMSNorm
// of the updated row (the operand of the next projection) taken in the same kernel: one workgroup per row keeps the
// row in registers between the two steps.  N <= 6144, N % 4 == 0.  Output formats as in the RMSNorm kernel:
// terms 1 bf16, 2 hi | lo, 3 fp16.
__global__ __launch_bounds__(256) void splitk_reduce_resid_norm_kernel(const float *__restrict__ part, int splits, int M, int N,
                                                                        float *__restrict__ x, const bf16 *__restrict__ g,
                                                                        bf16 *__restrict__ h, float eps, int terms) {
    constexpr int NV = 6;
    __shared__ float red[4];
    int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    size_t plane = (size_t)M * N;
    const int nv = N >> 2;
    f32x4 v[NV];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int j = tid + 256 * i;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if (j < nv) {
            const float *p0 = part + (size_t)r * N + 4 * j;
#pragma unroll 8
            for (int sp = 0; sp < splits; ++sp) acc += *reinterpret_cast<const f32x4 *>(p0 + sp * plane);
            f32x4 *dst = reinterpret_cast<f32x4 *>(x + (size_t)r * N + 4 * j);
            acc += *dst;
            *dst = acc;
        }
        v[i] = acc;
        ss += acc[0] * acc[0] + acc[1] * acc[1] + acc[2] * acc[2] + acc[3] * acc[3];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    float rinv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)N + eps);
    bf16 *o = h + (size_t)r * N * (terms == 2 ? 2 : 1);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int j = tid + 256 * i;
        if (j >= nv) continue;
        int c = j << 2;
        uint2 gp = *reinterpret_cast<const uint2 *>(g + c);
        float gv[4] = {__uint_as_float(gp.x << 16), __uint_as_float(gp.x & 0xffff0000u), __uint_as_float(gp.y << 16),
                       __uint_as_float(gp.y & 0xffff0000u)};
        unsigned hi[4], lo[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float y = v[i][q] * rinv * gv[q];
            if (terms == 3) {
                hi[q] = __half_as_ushort(to_half_sat(y));
                lo[q] = 0;
            } else {
                bf16 hh = __float2bfloat16(y);
                hi[q] = __bfloat16_as_ushort(hh);
                lo[q] = __bfloat16_as_ushort(__float2bfloat16(y - __bfloat162float(hh)));
            }
        }
        *reinterpret_cast<uint2 *>(o + c) = uint2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
        if (terms == 2) *reinterpret_cast<uint2 *>(o + N + c) = uint2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
    }
}

template <int A_FMT, int BT, int WAVES_N>
static hipError_t launch_splitk_tiles(const GemmTune &tune, const bf16 *A, const bf16 *W, float *part, int M, int N, int K,
                                      int splits, hipStream_t s) {
    constexpr int SBK = 64, SNS = BT == 256 ? 5 : 2;
    constexpr int smem = gemm_lds_bytes(BT, BT, SBK, SNS);
    static std::atomic<uint32_t> attr_done{0};
    auto kern = gemm_bf16_kernel<BT, BT, 2, WAVES_N, SBK, SNS, EPI_STORE_F32, A_FMT>;
    if (hipError_t e = set_dynamic_lds_once(attr_done, reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
    int tiles_m = (M + BT - 1) / BT, tiles_n = N / BT;
    dim3 grid(((tiles_m * tiles_n + 7) / 8) * 8, splits);
    // tile order as in launch_inst: the tiles an XCD works on at one time (its share of the list; every slice of a tile
    // lands on the same XCD) form a roughly square block, so that they ask the fabric for the fewest operand panels
    int group_m = tune.group_m;
    if (group_m <= 0) group_m = (int)std::lround(std::sqrt((double)std::min((tiles_m * tiles_n + 7) / 8, 32 * std::max(160 * 1024 / smem, 1))));
    group_m = std::max(1, std::min(group_m, tiles_m));
    kern<<<grid, 128 * WAVES_N, smem, s>>>(A, W, part, M, N, K, tiles_m, tiles_n, 0, group_m, 1, RopeArgs{}, PrefetchArgs{});
    return hipGetLastError();
}

// At most 32 rows (a generation step with one token per trace, the last layer's one row per trace): 32 x 128 tiles
// with four LDS stages, so that a workgroup keeps three k-tiles of its weight panel (60 KiB) in flight - such a
// product is a stream of the weight matrix, and the 128-row tile's two stages leave it latency-bound.
template <int A_FMT>
static hipError_t launch_splitk_short(const GemmTune &tune, const bf16 *A, const bf16 *W, float *part, int M, int N, int K,
                                      int splits, hipStream_t s) {
    constexpr int BM = 32, BN = 128, NS = 4;
    constexpr int smem = NS * (BM + BN) * 64 * 2;
    static std::atomic<uint32_t> attr_done{0};
    auto kern = gemm_bf16_kernel<BM, BN, 1, 2, 64, NS, EPI_STORE_F32, A_FMT>;
    if (hipError_t e = set_dynamic_lds_once(attr_done, reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
    int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    dim3 grid(((tiles_m * tiles_n + 7) / 8) * 8, splits);
    kern<<<grid, 128, smem, s>>>(A, W, part, M, N, K, tiles_m, tiles_n, 0, 1, 1, RopeArgs{}, PrefetchArgs{});
    return hipGetLastError();
}

// The partial products of the k slices, one [M, N] fp32 plane per slice; big_tile: 256 x 256 tiles, else 128 x 128.
static hipError_t launch_splitk_main(const GemmTune &tune, const bf16 *A, const bf16 *W, float *part, int M, int N, int K,
                                     int a_terms, int splits, bool big_tile, hipStream_t s) {
    if (big_tile)
        return a_terms == 2   ? launch_splitk_tiles<2, 256, 4>(tune, A, W, part, M, N, K, splits, s)
               : a_terms == 3 ? launch_splitk_tiles<3, 256, 4>(tune, A, W, part, M, N, K, splits, s)
                              : launch_splitk_tiles<1, 256, 4>(tune, A, W, part, M, N, K, splits, s);
    if (M <= 32 && tune.short_tile)
        return a_terms == 2   ? launch_splitk_short<2>(tune, A, W, part, M, N, K, splits, s)
               : a_terms == 3 ? launch_splitk_short<3>(tune, A, W, part, M, N, K, splits, s)
                              : launch_splitk_short<1>(tune, A, W, part, M, N, K, splits, s);
    return a_terms == 2   ? launch_splitk_tiles<2, 128, 2>(tune, A, W, part, M, N, K, splits, s)
           : a_terms == 3 ? launch_splitk_tiles<3, 128, 2>(tune, A, W, part, M, N, K, splits, s)
                          : launch_splitk_tiles<1, 128, 2>(tune, A, W, part, M, N, K, splits, s);
}

hipError_t launch_gemm_bf16(const GemmTune &tune, const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int epi,
                            int a_terms, int out_terms, float *splitk_ws, size_t splitk_ws_bytes, hipStream_t s,
                            const PrefetchArgs *pf, const NormAfter *norm, bool *norm_done) {
    if (norm_done) *norm_done = false;
    int k_total = K * (a_terms == 2 ? 2 : 1);
    bool big = false;
    int splits = tune.tile == 0 ? gemm_splitk_factor(tune, M, N, k_total, &big) : 1;
    if (splits > 1 && splitk_ws && gemm_splitk_bytes(tune, M, N, k_total) <= splitk_ws_bytes) {
        hipError_t e = launch_splitk_main(tune, A, W, splitk_ws, M, N, K, a_terms, splits, big, s);
        if (e != hipSuccess) return e;
        int n_out = epi == EPI_SWIGLU ? N / 2 : N;
        dim3 grid((n_out / 4 + 255) / 256, M);
        if (epi == EPI_RESID_F32 && norm && norm->g && norm->h && N % 4 == 0 && N <= 6144 &&
            ((((uintptr_t)norm->g | (uintptr_t)norm->h) & 7) == 0)) {
            splitk_reduce_resid_norm_kernel<<<M, 256, 0, s>>>(splitk_ws, splits, M, N, reinterpret_cast<float *>(out),
                                                              reinterpret_cast<const bf16 *>(norm->g),
                                                              reinterpret_cast<bf16 *>(norm->h), norm->eps, norm->terms);
            if (norm_done) *norm_done = true;
            return hipGetLastError();
        }
        if (epi == EPI_STORE_F32) splitk_reduce_kernel<EPI_STORE_F32><<<grid, 256, 0, s>>>(splitk_ws, splits, M, N, out, out_terms);
        else if (epi == EPI_RESID_F32) splitk_reduce_kernel<EPI_RESID_F32><<<grid, 256, 0, s>>>(splitk_ws, splits, M, N, out, out_terms);
        else splitk_reduce_kernel<EPI_SWIGLU><<<grid, 256, 0, s>>>(splitk_ws, splits, M, N, out, out_terms);
        return hipGetLastError();
    }
    if (epi == EPI_STORE_F32) return launch_epi<EPI_STORE_F32>(tune, A, W, out, M, N, K, a_terms, out_terms, s);
    if (epi == EPI_RESID_F32) return launch_epi<EPI_RESID_F32>(tune, A, W, out, M, N, K, a_terms, out_terms, s);
    return launch_epi<EPI_SWIGLU>(tune, A, W, out, M, N, K, a_terms, out_terms, s, pf);
}

// QKV projection with the rotation in the epilogue (see RopeArgs): the default tile choice, both shapes
// have 64-column wave tiles.
hipError_t launch_gemm_bf16_rope(const GemmTune &tune, const bf16 *A, const bf16 *W_perm, int M, int N, int K, int a_terms,
                                 const RopeArgs &rope, float *splitk_ws, size_t splitk_ws_bytes, hipStream_t s) {
    int k_total = K * (a_terms == 2 ? 2 : 1);
    bool big = false;
    int splits = tune.tile == 0 ? gemm_splitk_factor(tune, M, N, k_total, &big) : 1;
    if (splits > 1 && splitk_ws && gemm_splitk_bytes(tune, M, N, k_total) <= splitk_ws_bytes) {
        hipError_t e = launch_splitk_main(tune, A, W_perm, splitk_ws, M, N, K, a_terms, splits, big, s);
        if (e != hipSuccess) return e;
        dim3 grid(((N / 128) * 16 + 255) / 256, M);
        splitk_reduce_rope_kernel<<<grid, 256, 0, s>>>(splitk_ws, splits, M, N, rope);
        return hipGetLastError();
    }
    if (prefer_256_tiles(M, N)) {
        // as in launch_epi: a last round of 256 x 256 tiles that would be less than half full goes to a second launch with
        // 128 x 128 tiles (18606 rows x 2048 columns: 584 tiles = 2 rounds + 72 tiles)
        int tm = (M + 255) / 256, tn = N / 256, n1 = tn;
        long t256 = (long)tm * tn, rounds = t256 / 256;
        if (rounds >= 1 && t256 - rounds * 256 > 0) {
            int full = (int)(rounds * 256 / tm);
            if ((long)(tn - full) * tm <= 128) n1 = full;
        }
        if (n1 > 0) {
            hipError_t e = launch_tile<256, 256, 2, 4, 64, 5, EPI_ROPE>(tune, A, W_perm, nullptr, M, N, K, 0, n1 * 256, a_terms, 1, s, &rope);
            if (e != hipSuccess || n1 == tn) return e;
        }
        return launch_tile<128, 128, 2, 2, 64, 2, EPI_ROPE>(tune, A, W_perm, nullptr, M, N, K, n1 * 256, N - n1 * 256, a_terms, 1, s, &rope);
    }
    return launch_tile<128, 128, 2, 2, 64, 2, EPI_ROPE>(tune, A, W_perm, nullptr, M, N, K, 0, N, a_terms, 1, s, &rope);
}

}  // namespace cs
