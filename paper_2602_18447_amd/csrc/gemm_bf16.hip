// bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores: C[M,N] = A[M,K] . W[N,K]^T.
//
// Both operands are K-contiguous, which is exactly the per-lane operand shape of
// v_mfma_f32_32x32x16_bf16 (lane l supplies 8 consecutive k of row/column l%32, k-group l/32), so
// tiles go global -> registers -> LDS as 16-byte vectors and come back out of LDS as 16-byte MFMA
// operands with no shuffling.  LDS rows are padded from 128 to 144 bytes so that the 16 lanes of one
// ds_read_b128 phase hit 16 different 4-bank groups.  Two LDS stages: the global loads of k-tile
// i+1 are issued before the MFMAs of k-tile i and written to the other stage afterwards, one
// barrier per k-tile.
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
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int GEMM_BK = 64;
constexpr int GEMM_LDS_STRIDE = 72;  // elements per LDS row: 64 + 8 pad (144 bytes)

struct GemmTune {
    int tile;   // 0 = heuristic, 1 = 128x128, 2 = 256x256, 3 = 256x128
};
static GemmTune g_gemm_tune = {0};
void gemm_set_tile(int t) { g_gemm_tune.tile = t; }

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W,
                                                         void *__restrict__ out_v, int M, int N, int K,
                                                         int tiles_m, int tiles_n, int a_terms, int out_terms) {
    constexpr int WM = BM / 2, WN = BN / 2;     // 2 x 2 waves
    constexpr int MI = WM / 32, NI = WN / 32;   // 32x32 MFMA blocks per wave
    constexpr int A_VEC = BM / 32, B_VEC = BN / 32;  // 16-byte vectors per thread per k-tile
    constexpr int STAGE = (BM + BN) * GEMM_LDS_STRIDE;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __bf16 *smem = reinterpret_cast<__bf16 *>(smem_raw);

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
    int wy = wave >> 1, wx = wave & 1;

    const u32x4 *a_src[A_VEC];
    const u32x4 *b_src[B_VEC];
    int a_dst[A_VEC], b_dst[B_VEC];
#pragma unroll
    for (int i = 0; i < A_VEC; ++i) {
        int v = tid + 256 * i, r = v >> 3, kv = v & 7;
        int row = min(m0 + r, M - 1);
        a_src[i] = reinterpret_cast<const u32x4 *>(A + (size_t)row * K * a_terms + kv * 8);
        a_dst[i] = r * GEMM_LDS_STRIDE + kv * 8;
    }
#pragma unroll
    for (int i = 0; i < B_VEC; ++i) {
        int v = tid + 256 * i, r = v >> 3, kv = v & 7;
        b_src[i] = reinterpret_cast<const u32x4 *>(W + (size_t)(n0 + r) * K + kv * 8);
        b_dst[i] = BM * GEMM_LDS_STRIDE + r * GEMM_LDS_STRIDE + kv * 8;
    }

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    u32x4 a_reg[A_VEC], b_reg[B_VEC];
    int nk_w = K / GEMM_BK;        // k-tiles of W
    int nk = nk_w * a_terms;       // k-tiles of A: hi half, then lo half
    // prologue: k-tile 0 -> stage 0
#pragma unroll
    for (int i = 0; i < A_VEC; ++i) a_reg[i] = a_src[i][0];
#pragma unroll
    for (int i = 0; i < B_VEC; ++i) b_reg[i] = b_src[i][0];
#pragma unroll
    for (int i = 0; i < A_VEC; ++i) *reinterpret_cast<u32x4 *>(smem + a_dst[i]) = a_reg[i];
#pragma unroll
    for (int i = 0; i < B_VEC; ++i) *reinterpret_cast<u32x4 *>(smem + b_dst[i]) = b_reg[i];
    __syncthreads();

    int a_frag = (wy * WM + (lane & 31)) * GEMM_LDS_STRIDE + (lane >> 5) * 8;
    int b_frag = BM * GEMM_LDS_STRIDE + (wx * WN + (lane & 31)) * GEMM_LDS_STRIDE + (lane >> 5) * 8;

    for (int kt = 0; kt < nk; ++kt) {
        int cur = (kt & 1) * STAGE, nxt = ((kt + 1) & 1) * STAGE;
        bool more = kt + 1 < nk;
        if (more) {
            int ka = kt + 1, kw = ka >= nk_w ? ka - nk_w : ka;   // W wraps around for the lo half
            int ko = ka * (GEMM_BK / 8), kwo = kw * (GEMM_BK / 8);  // in u32x4 units
#pragma unroll
            for (int i = 0; i < A_VEC; ++i) a_reg[i] = a_src[i][ko];
#pragma unroll
            for (int i = 0; i < B_VEC; ++i) b_reg[i] = b_src[i][kwo];
        }
#pragma unroll
        for (int ks = 0; ks < GEMM_BK / 16; ++ks) {
            bf16x8 af[MI], bfr[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[i] = *reinterpret_cast<const bf16x8 *>(smem + cur + a_frag + i * 32 * GEMM_LDS_STRIDE + ks * 16);
#pragma unroll
            for (int j = 0; j < NI; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8 *>(smem + cur + b_frag + j * 32 * GEMM_LDS_STRIDE + ks * 16);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < A_VEC; ++i) *reinterpret_cast<u32x4 *>(smem + nxt + a_dst[i]) = a_reg[i];
#pragma unroll
            for (int i = 0; i < B_VEC; ++i) *reinterpret_cast<u32x4 *>(smem + nxt + b_dst[i]) = b_reg[i];
        }
        __syncthreads();
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

template <int BM, int BN, int EPI>
static hipError_t launch_tile(const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int a_terms,
                              int out_terms, hipStream_t s) {
    constexpr int smem = 2 * (BM + BN) * GEMM_LDS_STRIDE * 2;
    static bool attr_set = false;
    auto kern = gemm_bf16_kernel<BM, BN, EPI>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    int n_tiles = tiles_m * tiles_n;
    int grid = ((n_tiles + 7) / 8) * 8;
    kern<<<grid, 256, smem, s>>>(A, W, out, M, N, K, tiles_m, tiles_n, a_terms, out_terms);
    return hipGetLastError();
}

template <int EPI>
static hipError_t launch_epi(const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int a_terms,
                             int out_terms, hipStream_t s) {
    int tile = g_gemm_tune.tile;
    if (tile == 0) {
        long t256 = (long)((M + 255) / 256) * (N / 256);
        tile = (N % 256 == 0 && t256 >= 192) ? 2 : 1;
    }
    if (tile == 2 && N % 256 == 0) return launch_tile<256, 256, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
    if (tile == 3) return launch_tile<256, 128, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
    return launch_tile<128, 128, EPI>(A, W, out, M, N, K, a_terms, out_terms, s);
}

hipError_t launch_gemm_bf16(const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int epi, int a_terms,
                            int out_terms, hipStream_t s) {
    if (epi == EPI_STORE_F32) return launch_epi<EPI_STORE_F32>(A, W, out, M, N, K, a_terms, out_terms, s);
    if (epi == EPI_RESID_F32) return launch_epi<EPI_RESID_F32>(A, W, out, M, N, K, a_terms, out_terms, s);
    return launch_epi<EPI_SWIGLU>(A, W, out, M, N, K, a_terms, out_terms, s);
}

}  // namespace cs
