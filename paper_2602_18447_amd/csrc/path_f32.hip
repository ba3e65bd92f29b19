// fp32 storage path (small correctness configuration): an LDS-tiled FMA GEMM and a
// wavefront-per-row attention.  Both keep every product and sum in fp32.
#include "kernels.h"

namespace cs {

// ------------------------------------------------------------------------------------------------
// C[M,N] = A[M,K] . W[N,K]^T, 64x64x16 tiles, 256 threads, 4x4 outputs per thread at a stride of 16
// (rows ty+16i, columns tx+16j).  N % 64 == 0, K % 16 == 0, any M.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ W,
                                                        float *__restrict__ out, int M, int N, int K) {
    __shared__ float As[16][64 + 4];
    __shared__ float Ws[16][64 + 4];
    int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    int lr = tid >> 2, lk = (tid & 3) << 2;  // loader: row lr, k offset lk..lk+3
    float acc[4][4] = {};
    int arow = min(m0 + lr, M - 1);          // rows past M are clamped on load and dropped on store
    const float *ap = A + (size_t)arow * K + lk;
    const float *wp = W + (size_t)(n0 + lr) * K + lk;
    for (int k0 = 0; k0 < K; k0 += 16) {
        float4 av = *(const float4 *)(ap + k0);
        float4 wv = *(const float4 *)(wp + k0);
        As[lk + 0][lr] = av.x; As[lk + 1][lr] = av.y; As[lk + 2][lr] = av.z; As[lk + 3][lr] = av.w;
        Ws[lk + 0][lr] = wv.x; Ws[lk + 1][lr] = wv.y; Ws[lk + 2][lr] = wv.z; Ws[lk + 3][lr] = wv.w;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty + 16 * i]; b[i] = Ws[k][tx + 16 * i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + ty + 16 * i;
        if (m >= M) continue;
        if (EPI == EPI_SWIGLU) {
            // columns tx, tx+16 are gate entries; tx+32, tx+48 their up partners
            int Fo = N >> 1;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float gte = acc[i][j], up = acc[i][j + 2];
                float act = gte / (1.0f + expf(-gte)) * up;
                out[(size_t)m * Fo + (n0 >> 1) + tx + 16 * j] = act;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                size_t o = (size_t)m * N + n0 + tx + 16 * j;
                if (EPI == EPI_RESID_F32) out[o] += acc[i][j];
                else out[o] = acc[i][j];
            }
        }
    }
}

hipError_t launch_gemm_f32(const float *A, const float *W, void *out, int M, int N, int K, int epi,
                           hipStream_t s) {
    dim3 grid(N / 64, (M + 63) / 64);
    float *o = (float *)out;
    if (epi == EPI_STORE_F32) gemm_f32_kernel<EPI_STORE_F32><<<grid, 256, 0, s>>>(A, W, o, M, N, K);
    else if (epi == EPI_RESID_F32) gemm_f32_kernel<EPI_RESID_F32><<<grid, 256, 0, s>>>(A, W, o, M, N, K);
    else gemm_f32_kernel<EPI_SWIGLU><<<grid, 256, 0, s>>>(A, W, o, M, N, K);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Attention, one wavefront per (suffix row, q head).  Keys are visited 64 at a time: each lane
// scores one key (full head_dim dot from global memory), the wave keeps a running max / sum
// (online softmax), then the 64 probabilities are broadcast lane by lane while every lane
// accumulates its own 1 or 2 output dimensions.
__device__ __forceinline__ const float *key_row(const AttnArgs &a, const float *pages, const float *suf, int b,
                                                int L, int cu_b, int c, int j) {
    if (j < L) {
        int blk = a.block_table[(size_t)b * a.max_blocks + j / a.block_size];
        blk = min(max(blk, 0), a.n_blocks - 1);
        return pages + (((size_t)blk * a.Hkv + c) * a.block_size + (j % a.block_size)) * a.hd;
    }
    int t = min(cu_b + (j - L), a.T - 1);
    return suf + ((size_t)t * a.Hkv + c) * a.hd;
}

__global__ __launch_bounds__(256) void attn_f32_kernel(AttnArgs a, const int32_t *__restrict__ tok_trace,
                                                        const int32_t *__restrict__ tok_pos) {
    __shared__ float q_s[4][128];
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    long w = (long)blockIdx.x * 4 + wave;
    long total = (long)a.T * a.Hq;
    bool active = w < total;
    int t = active ? (int)(w / a.Hq) : 0;
    int h = active ? (int)(w % a.Hq) : 0;
    int G = a.Hq / a.Hkv, c = h / G;
    int b = min(max(tok_trace[t], 0), a.B - 1);
    int cu_b = min(max(a.cu[b], 0), a.T - 1);
    int L = min(max(a.plens[b], 0), a.max_blocks * a.block_size);
    int n_keys = min(tok_pos[t], L + a.T - 1) + 1;   // keys 0 .. pos inclusive
    const float *q = (const float *)a.q + ((size_t)t * a.Hq + h) * a.hd;
    for (int i = lane; i < a.hd; i += 64) q_s[wave][i] = q[i] * a.scale;
    __syncthreads();
    if (!active) return;
    const float *kp = (const float *)a.k_pages, *vp = (const float *)a.v_pages;
    const float *ks = (const float *)a.ksuf, *vs = (const float *)a.vsuf;
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int j0 = 0; j0 < n_keys; j0 += 64) {
        int j = j0 + lane;
        float sc = -INFINITY;
        if (j < n_keys) {
            const float4 *kr = (const float4 *)key_row(a, kp, ks, b, L, cu_b, c, j);
            float acc = 0.f;
            for (int i = 0; i < a.hd / 4; ++i) {
                float4 kv = kr[i];
                acc += q_s[wave][4 * i] * kv.x + q_s[wave][4 * i + 1] * kv.y + q_s[wave][4 * i + 2] * kv.z +
                       q_s[wave][4 * i + 3] * kv.w;
            }
            sc = acc;
        }
        float mx = sc;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        float m_new = fmaxf(m, mx);           // finite: key j0 is always visible
        float alpha = expf(m - m_new);
        float p = (j < n_keys) ? expf(sc - m_new) : 0.f;
        float ps = p;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ps += __shfl_xor(ps, o, 64);
        l = l * alpha + ps;
        o0 *= alpha;
        o1 *= alpha;
        int cnt = min(64, n_keys - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            float pj = __shfl(p, jj, 64);
            const float *vr = key_row(a, vp, vs, b, L, cu_b, c, j0 + jj);
            o0 = fmaf(pj, vr[lane], o0);
            if (a.hd > 64) o1 = fmaf(pj, vr[lane + 64], o1);
        }
        m = m_new;
    }
    float *out = (float *)a.out + ((size_t)t * a.Hq + h) * a.hd;
    if (lane < a.hd) out[lane] = o0 / l;
    if (a.hd > 64) out[lane + 64] = o1 / l;
}

hipError_t launch_attn_f32(const AttnArgs &a, const int32_t *tok_trace, const int32_t *tok_pos, hipStream_t s) {
    long total = (long)a.T * a.Hq;
    int blocks = (int)((total + 3) / 4);
    attn_f32_kernel<<<blocks, 256, 0, s>>>(a, tok_trace, tok_pos);
    return hipGetLastError();
}

}  // namespace cs
