// bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores: C[M,N] = A[M,K] . W[N,K]^T.
//
// Both operands are K-contiguous, which is exactly the per-lane operand shape of
// v_mfma_f32_32x32x16_bf16 (lane l supplies 8 consecutive k of row/column l%32, k-group l/32).
//
// Data path.  Operand tiles travel global -> LDS directly (global_load_lds_dwordx4): no staging
// registers, no ds_write instructions, the wave keeps issuing MFMAs while the data lands.  One such
// instruction fills 1 KiB of LDS in lane order, i.e. 8 tile rows of 64 k (128 bytes) each.  Rows are
// unpadded; instead the 16-byte k-vector g of row r is kept at position g ^ ((r >> 1) & 7) of its row
// (the lane that fills a position fetches the matching global vector), so the 16 lanes of one
// ds_read_b128 phase - 16 consecutive rows, same k-vector - hit 16 different 4-bank groups.
// Two LDS stages: the loads of k-tile i+1 are issued right after the barrier that frees their stage
// and have the whole MFMA phase of k-tile i to complete; one vmcnt wait + barrier per k-tile.
//
// Epilogues: plain fp32 store, fp32 residual add in place, or SwiGLU on interleaved gate/up columns
// with a bf16 result.
//
// Two-term activations.  With a_terms == 2 the A operand is [M, 2K]: columns 0..K-1 hold the bf16
// rounding of the activation ("hi") and K..2K-1 the bf16 rounding of what that rounding lost
// ("lo"); the k loop then runs over both halves against the same W, so the fp32 accumulator receives
// (hi + lo) . W - the product with a 16-bit-mantissa activation.  With out_terms == 2 the SwiGLU
// epilogue writes its result in the same [M, 2F] hi | lo form for the next GEMM.
#include "kernels.h"

namespace cs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define CS_GLOBAL_AS __attribute__((address_space(1)))
#define CS_LDS_AS __attribute__((address_space(3)))

struct GemmTune {
    int tile;   // 0 = heuristic; see launch_epi for the ids
};
static GemmTune g_gemm_tune = {0};
void gemm_set_tile(int t) { g_gemm_tune.tile = t; }

// vmcnt(n) only (expcnt / lgkmcnt left unconstrained), gfx9 encoding of s_waitcnt
#define CS_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// BK: k extent of one LDS stage (64 or 32 elements); NS: number of LDS stages.  NS - 1 k-tiles are
// kept in flight: (64, 2) has the fewest barriers, (32, 4) the deepest prefetch for the same LDS budget.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NS, int EPI, int A_TERMS>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W,
                                                         void *__restrict__ out_v, int M, int N, int K,
                                                         int tiles_m, int tiles_n, int out_terms) {
    constexpr int NW = WAVES_M * WAVES_N;
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
    static_assert(NS >= 2 && NS <= 4, "stages");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // XCD-aware tile order: consecutive workgroup ids land on different XCDs, so give each XCD a
    // contiguous range of tiles; inside a range tile_m runs fastest, so neighbours share a W tile.
    int n_tiles = tiles_m * tiles_n;
    int bid = blockIdx.x;
    int per = (n_tiles + 7) >> 3;
    int lid = (bid & 7) * per + (bid >> 3);
    if (lid >= n_tiles) return;   // uniform per workgroup: no barrier is skipped by a subset
    int tm = lid % tiles_m, tn = lid / tiles_m;
    int m0 = tm * BM, n0 = tn * BN;

    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int wy = wave / WAVES_N, wx = wave % WAVES_N;

    // Direct-load roles: instruction j of wave w fills rows RPD*(w + NW*j) .. of an operand tile; lane s
    // sits at row s / VPR, position s % VPR and fetches the k-vector that the swizzle puts there.
    // Swizzle: position = k-vector ^ ((row >> 1) & 7) for 128-byte rows, ^ ((row >> 2) & 3) for 64-byte
    // rows; either way 16 consecutive rows at one k-vector cover all 64 banks once.  A rows past M
    // are clamped (fetched twice, never stored to the output).
    auto swz = [](int row) { return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
    const int rl = lane / VPR, ph = lane % VPR;
    const int lda = K * A_TERMS;
    const char *a_src[A_DMA], *b_src[B_DMA];
#pragma unroll
    for (int j = 0; j < A_DMA; ++j) {
        int row = RPD * (wave + NW * j) + rl;
        int g = ph ^ swz(row);
        a_src[j] = reinterpret_cast<const char *>(A + (size_t)min(m0 + row, M - 1) * lda + g * 8);
    }
#pragma unroll
    for (int j = 0; j < B_DMA; ++j) {
        int row = RPD * (wave + NW * j) + rl;
        int g = ph ^ swz(row);
        b_src[j] = reinterpret_cast<const char *>(W + (size_t)(n0 + row) * K + g * 8);
    }
    int nk_w = K / BK;             // k-tiles of W
    int nk = nk_w * A_TERMS;       // k-tiles of A: hi half, then lo half
    auto issue_loads = [&](int stage, int kt) {
        int kw = (A_TERMS == 2 && kt >= nk_w) ? kt - nk_w : kt;     // W wraps around for the lo half
        unsigned char *base = smem + stage * STAGE;
#pragma unroll
        for (int j = 0; j < A_DMA; ++j)
            __builtin_amdgcn_global_load_lds((const CS_GLOBAL_AS void *)(a_src[j] + (size_t)kt * ROWB),
                                             (CS_LDS_AS void *)(base + (wave + NW * j) * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < B_DMA; ++j)
            __builtin_amdgcn_global_load_lds((const CS_GLOBAL_AS void *)(b_src[j] + (size_t)kw * ROWB),
                                             (CS_LDS_AS void *)(base + BM * ROWB + (wave + NW * j) * 1024), 16, 0, 0);
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // MFMA operand reads: row (lane % 32) of each 32-row block, k-vector 2 ks + lane / 32
    const int half = lane >> 5;
    const int arow = wy * WM + (lane & 31), brow = wx * WN + (lane & 31);
    const int a_base = arow * ROWB, a_sw = swz(arow);          // rows 32 apart share the swizzle value
    const int b_base = BM * ROWB + brow * ROWB, b_sw = swz(brow);

    // Pipeline: k-tiles kt+1 .. kt+NS-1 are in flight while k-tile kt is multiplied.  Direct loads
    // complete in order per wave, so "at most PER_TILE * r outstanding" means this wave's part of tile
    // kt has landed when r tiles were issued after it; the barrier extends that to every wave and also
    // tells that everybody is done with the stage the next loads will overwrite.
#pragma unroll
    for (int t = 0; t < NS - 1; ++t)
        if (t < nk) issue_loads(t, t);
    for (int kt = 0; kt < nk; ++kt) {
        int after = min(NS - 2, nk - 1 - kt);
        if (after >= 2) CS_WAIT_VMCNT(2 * PER_TILE);
        else if (after == 1) CS_WAIT_VMCNT(PER_TILE);
        else CS_WAIT_VMCNT(0);
        __syncthreads();
        if (kt + NS - 1 < nk) issue_loads((kt + NS - 1) % NS, kt + NS - 1);
        const unsigned char *cur = smem + (kt % NS) * STAGE;
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
        read_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) read_frags((ks + 1) & 1, ks + 1);   // next k-step's operands
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
        }
    }

    // C layout of one 32x32 block: lane holds column lane%32, rows 8*(e/4) + 4*(lane/32) + e%4.
    int col_l = lane & 31, row_l = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            int m = m0 + wy * WM + i * 32 + (e >> 2) * 8 + row_l + (e & 3);
            if (m >= M) continue;
            if (EPI == EPI_SWIGLU) {
                bf16 *out = reinterpret_cast<bf16 *>(out_v);
                int Fo = N >> 1;
#pragma unroll
                for (int j = 0; j < NI; j += 2) {
                    float gte = acc[i][j][e], up = acc[i][j + 1][e];
                    float act = gte / (1.0f + __expf(-gte)) * up;
                    int f = ((n0 + wx * WN + j * 32) >> 1) + col_l;
                    bf16 hi = __float2bfloat16(act);
                    size_t o = (size_t)m * Fo * out_terms + f;
                    out[o] = hi;
                    if (out_terms == 2) out[o + Fo] = __float2bfloat16(act - __bfloat162float(hi));
                }
            } else {
                float *out = reinterpret_cast<float *>(out_v);
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    size_t o = (size_t)m * N + n0 + wx * WN + j * 32 + col_l;
                    if (EPI == EPI_RESID_F32) out[o] += acc[i][j][e];
                    else out[o] = acc[i][j][e];
                }
            }
        }
    }
}

// The number of activation terms is a template parameter, so the one-term and the two-term launches
// are different kernels (and show up under different names in a kernel trace).
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NS, int EPI, int A_TERMS>
static hipError_t launch_inst(const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int out_terms,
                              hipStream_t s) {
    constexpr int smem = NS * (BM + BN) * BK * 2;
    static bool attr_set = false;
    auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, BK, NS, EPI, A_TERMS>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    int n_tiles = tiles_m * tiles_n;
    int grid = ((n_tiles + 7) / 8) * 8;
    kern<<<grid, 64 * WAVES_M * WAVES_N, smem, s>>>(A, W, out, M, N, K, tiles_m, tiles_n, out_terms);
    return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NS, int EPI>
static hipError_t launch_tile(const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int a_terms,
                              int out_terms, hipStream_t s) {
    if (a_terms == 2) return launch_inst<BM, BN, WAVES_M, WAVES_N, BK, NS, EPI, 2>(A, W, out, M, N, K, out_terms, s);
    return launch_inst<BM, BN, WAVES_M, WAVES_N, BK, NS, EPI, 1>(A, W, out, M, N, K, out_terms, s);
}

// Tile ids: 1 = 128x128 / 4 waves, 2 = 256x256 / 4 waves, 3 = 256x128 / 4 waves, 4 = 256x256 / 8 waves
// (all BK 64 x 2 stages); 5 = 128x128 / 4 waves and 6 = 256x256 / 8 waves with BK 32 x 4 stages.
// Measured on the draft-model shapes: 4 is the fastest for the wide gate/up projection, 1 for the
// others; the deeper pipelines (5, 6) pay more barriers than they hide latency.
template <int EPI>
static hipError_t launch_epi(const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int a_terms,
                             int out_terms, hipStream_t s) {
    int tile = g_gemm_tune.tile;
    if (tile == 0) {
        long t256 = (long)((M + 255) / 256) * (N / 256);
        tile = (N % 256 == 0 && t256 >= 192) ? 4 : 1;
    }
    if ((tile == 2 || tile == 4 || tile == 6) && N % 256 != 0) tile = 1;
    switch (tile) {
        case 2: return launch_tile<256, 256, 2, 2, 64, 2, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
        case 3: return launch_tile<256, 128, 2, 2, 64, 2, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
        case 4: return launch_tile<256, 256, 2, 4, 64, 2, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
        case 5: return launch_tile<128, 128, 2, 2, 32, 4, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
        case 6: return launch_tile<256, 256, 2, 4, 32, 4, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
        default: return launch_tile<128, 128, 2, 2, 64, 2, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
    }
}

hipError_t launch_gemm_bf16(const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int epi, int a_terms,
                            int out_terms, hipStream_t s) {
    if (epi == EPI_STORE_F32) return launch_epi<EPI_STORE_F32>(A, W, out, M, N, K, a_terms, out_terms, s);
    if (epi == EPI_RESID_F32) return launch_epi<EPI_RESID_F32>(A, W, out, M, N, K, a_terms, out_terms, s);
    return launch_epi<EPI_SWIGLU>(A, W, out, M, N, K, a_terms, out_terms, s);
}

}  // namespace cs
