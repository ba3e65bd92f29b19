// Bandwidth-bound helper kernels of the verification pass: token bookkeeping, rotary table,
// embedding gather, RMSNorm, rotary split of the QKV projection, gate/up row interleave and the
// fused last-position verdict head (norm + verdict-row dots + softmax + threshold gate).
#include "kernels.h"

namespace cs {

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16>(bf16 v) { return __bfloat162float(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return __float2bfloat16(v); }  // RNE

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ------------------------------------------------------------------------------------------------
// token -> (trace, absolute position); last suffix row of each trace.  All indices are clamped to
// the host-validated bounds so that inconsistent device arrays cannot cause out-of-range accesses.
__global__ void prep_kernel(const int32_t *__restrict__ cu, const int32_t *__restrict__ plens, int B, int T,
                            int max_L, int32_t *__restrict__ tok_trace, int32_t *__restrict__ tok_pos,
                            int32_t *__restrict__ last_row) {
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) {
        int lo = 0, hi = B - 1;  // largest b with cu[b] <= t
        while (lo < hi) {
            int mid = (lo + hi + 1) >> 1;
            if (cu[mid] <= t) lo = mid; else hi = mid - 1;
        }
        int L = min(max(plens[lo], 0), max_L);
        int off = min(max(t - cu[lo], 0), T - 1);
        tok_trace[t] = lo;
        tok_pos[t] = L + off;
    }
    if (t < B) last_row[t] = min(max(cu[t + 1] - 1, 0), T - 1);
}

hipError_t launch_prep(const int32_t *cu, const int32_t *plens, int B, int T, int max_L, int32_t *tok_trace,
                       int32_t *tok_pos, int32_t *last_row, hipStream_t s) {
    int n = T > B ? T : B;
    prep_kernel<<<(n + 255) / 256, 256, 0, s>>>(cu, plens, B, T, max_L, tok_trace, tok_pos, last_row);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// cos/sin of pos * theta^(-2i/hd), evaluated in double so that positions in the tens of thousands
// keep full fp32 accuracy after the final rounding.
__global__ void rope_table_kernel(const int32_t *__restrict__ tok_pos, int T, int half, double log_theta,
                                  float *__restrict__ cos_t, float *__restrict__ sin_t) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= T * half) return;
    int t = idx / half, i = idx - t * half;
    double inv_freq = exp(-log_theta * (double)i / (double)half);  // theta^(-2i/hd), hd = 2*half
    double phi = (double)tok_pos[t] * inv_freq;
    double sv, cv;
    sincos(phi, &sv, &cv);
    cos_t[idx] = (float)cv;
    sin_t[idx] = (float)sv;
}

hipError_t launch_rope_table(const int32_t *tok_pos, int T, int hd, float theta, float *cos_t, float *sin_t,
                             hipStream_t s) {
    int half = hd / 2;
    int n = T * half;
    rope_table_kernel<<<(n + 255) / 256, 256, 0, s>>>(tok_pos, T, half, log((double)theta), cos_t, sin_t);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void embed_kernel(const int32_t *__restrict__ ids, const T *__restrict__ E, float *__restrict__ x,
                             int n_tok, int d, int vocab) {
    int t = blockIdx.x;
    int id = min(max(ids[t], 0), vocab - 1);
    const T *row = E + (size_t)id * d;
    float *dst = x + (size_t)t * d;
    for (int j = threadIdx.x; j < d; j += blockDim.x) dst[j] = to_f32<T>(row[j]);
}

hipError_t launch_embed(int dtype, const int32_t *ids, const void *E, float *x, int T, int d, int vocab,
                        hipStream_t s) {
    if (dtype == 0) embed_kernel<float><<<T, 256, 0, s>>>(ids, (const float *)E, x, T, d, vocab);
    else embed_kernel<bf16><<<T, 256, 0, s>>>(ids, (const bf16 *)E, x, T, d, vocab);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// RMSNorm: one wavefront per row, fp32 statistics, output rounded to the storage type.  With
// terms == 2 the row is written as hi | lo: the rounded value, then the rounding of the remainder;
// with terms == 3 (16-bit storage only) it is written as IEEE half values.
template <typename T>
__device__ __forceinline__ void store_terms(T *o, int c, int d, int terms, float v) {
    if (sizeof(T) == 2 && terms == 3) {
        reinterpret_cast<__half *>(o)[c] = to_half_sat(v);
        return;
    }
    T hi = from_f32<T>(v);
    o[c] = hi;
    if (terms == 2) o[d + c] = from_f32<T>(v - to_f32<T>(hi));
}

template <typename T>
__global__ void rmsnorm_kernel(const float *__restrict__ x, const T *__restrict__ g, T *__restrict__ out,
                               int n_rows, int d, float eps, int terms) {
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int row = blockIdx.x * (blockDim.x >> 6) + wave;
    if (row >= n_rows) return;
    const float4 *xr = (const float4 *)(x + (size_t)row * d);
    int nv = d >> 2;
    float ss = 0.f;
    for (int j = lane; j < nv; j += 64) {
        float4 v = xr[j];
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = wave_sum(ss);
    float r = 1.0f / sqrtf(ss / (float)d + eps);
    T *o = out + (size_t)row * d * (terms == 2 ? 2 : 1);
    for (int j = lane; j < nv; j += 64) {
        float4 v = xr[j];
        int c = j << 2;
        store_terms<T>(o, c + 0, d, terms, v.x * r * to_f32<T>(g[c + 0]));
        store_terms<T>(o, c + 1, d, terms, v.y * r * to_f32<T>(g[c + 1]));
        store_terms<T>(o, c + 2, d, terms, v.z * r * to_f32<T>(g[c + 2]));
        store_terms<T>(o, c + 3, d, terms, v.w * r * to_f32<T>(g[c + 3]));
    }
}

// 16-bit outputs, rows of at most NV * 256 elements: the row stays in registers between the two sweeps (every
// load of a lane is in flight at once), gains are read 4 at a time and the outputs leave as 8-byte stores.
// Same arithmetic, in the same order, as the generic kernel above.
template <int NV>
__global__ __launch_bounds__(256) void rmsnorm_bf16_rows_kernel(const float *__restrict__ x, const bf16 *__restrict__ g,
                                                                bf16 *__restrict__ out, int n_rows, int d, float eps, int terms) {
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int row = blockIdx.x * 4 + wave;
    if (row >= n_rows) return;
    const float4 *xr = (const float4 *)(x + (size_t)row * d);
    const int nv = d >> 2;
    float4 v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int j = lane + 64 * i;
        v[i] = j < nv ? xr[j] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    ss = wave_sum(ss);
    float r = 1.0f / sqrtf(ss / (float)d + eps);
    bf16 *o = out + (size_t)row * d * (terms == 2 ? 2 : 1);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int j = lane + 64 * i;
        if (j >= nv) continue;
        int c = j << 2;
        uint2 gp = *reinterpret_cast<const uint2 *>(g + c);
        float gv[4] = {__uint_as_float(gp.x << 16), __uint_as_float(gp.x & 0xffff0000u), __uint_as_float(gp.y << 16),
                       __uint_as_float(gp.y & 0xffff0000u)};
        float y[4] = {v[i].x * r * gv[0], v[i].y * r * gv[1], v[i].z * r * gv[2], v[i].w * r * gv[3]};
        unsigned hi[4], lo[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (terms == 3) {
                hi[q] = __half_as_ushort(to_half_sat(y[q]));
                lo[q] = 0;
            } else {
                bf16 h = __float2bfloat16(y[q]);
                hi[q] = __bfloat16_as_ushort(h);
                lo[q] = __bfloat16_as_ushort(__float2bfloat16(y[q] - __bfloat162float(h)));
            }
        }
        *reinterpret_cast<uint2 *>(o + c) = uint2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
        if (terms == 2) *reinterpret_cast<uint2 *>(o + d + c) = uint2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
    }
}

hipError_t launch_rmsnorm(int dtype, const float *x, const void *g, void *out, int T, int d, float eps,
                          int terms, hipStream_t s) {
    int blocks = (T + 3) / 4;
    const bool vec = d % 4 == 0 && (((uintptr_t)g | (uintptr_t)out) & 7) == 0;   // 8-byte gain loads and output stores
    if (dtype == 0) {
        rmsnorm_kernel<float><<<blocks, 256, 0, s>>>(x, (const float *)g, (float *)out, T, d, eps, 1);
    } else if (!vec) {
        rmsnorm_kernel<bf16><<<blocks, 256, 0, s>>>(x, (const bf16 *)g, (bf16 *)out, T, d, eps, terms);
    } else if (d <= 8 * 256) {
        rmsnorm_bf16_rows_kernel<8><<<blocks, 256, 0, s>>>(x, (const bf16 *)g, (bf16 *)out, T, d, eps, terms);
    } else if (d <= 24 * 256) {
        rmsnorm_bf16_rows_kernel<24><<<blocks, 256, 0, s>>>(x, (const bf16 *)g, (bf16 *)out, T, d, eps, terms);
    } else {
        rmsnorm_kernel<bf16><<<blocks, 256, 0, s>>>(x, (const bf16 *)g, (bf16 *)out, T, d, eps, terms);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Row gather: dst row b = src row rows[b]; one workgroup per row, 16 bytes per lane per step.
__global__ void gather_rows_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst,
                                   const int32_t *__restrict__ rows, int n_src_rows, size_t row16) {
    int b = blockIdx.x;
    int r = min(max(rows ? rows[b] : b, 0), n_src_rows - 1);
    for (size_t i = threadIdx.x; i < row16; i += blockDim.x) dst[(size_t)b * row16 + i] = src[(size_t)r * row16 + i];
}

hipError_t launch_gather_rows(const void *src, void *dst, const int32_t *rows, int n_rows, int n_src_rows,
                              size_t row_bytes, hipStream_t s) {
    gather_rows_kernel<<<n_rows, 256, 0, s>>>((const u32x4_t *)src, (u32x4_t *)dst, rows, n_src_rows, row_bytes / 16);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Write-back of suffix keys and values into the paged cache: suffix token i of trace b (i < n_append[b]) goes to
// logical row L_b + i of that trace, found through the block table.  One workgroup per suffix token; a row of one
// kv head is row16 16-byte vectors.
__global__ void kv_append_kernel(const u32x4_t *__restrict__ ksuf, const u32x4_t *__restrict__ vsuf,
                                 u32x4_t *__restrict__ k_pages, u32x4_t *__restrict__ v_pages,
                                 const int32_t *__restrict__ table, const int32_t *__restrict__ cu,
                                 const int32_t *__restrict__ plens, const int32_t *__restrict__ n_append,
                                 const int32_t *__restrict__ tok_trace, int B, int T, int Hkv, int row16, int block_size,
                                 int max_blocks, int n_blocks) {
    int t = blockIdx.x;
    int b = min(max(tok_trace[t], 0), B - 1);
    int i = t - cu[b];
    if (i < 0 || i >= n_append[b]) return;
    int row = plens[b] + i;
    if (row < 0 || row >= max_blocks * block_size) return;
    int blk = min(max(table[(size_t)b * max_blocks + row / block_size], 0), n_blocks - 1);
    int slot = row % block_size;
    for (int e = threadIdx.x; e < Hkv * row16; e += blockDim.x) {
        int c = e / row16, j = e - c * row16;
        size_t src = ((size_t)t * Hkv + c) * row16 + j;
        size_t dst = (((size_t)blk * Hkv + c) * block_size + slot) * row16 + j;
        k_pages[dst] = ksuf[src];
        v_pages[dst] = vsuf[src];
    }
}

hipError_t launch_kv_append(const void *ksuf, const void *vsuf, void *k_pages, void *v_pages, const int32_t *table,
                            const int32_t *cu, const int32_t *plens, const int32_t *n_append, const int32_t *tok_trace,
                            int B, int T, int Hkv, size_t head_row_bytes, int block_size, int max_blocks, int n_blocks,
                            hipStream_t s) {
    kv_append_kernel<<<T, 128, 0, s>>>((const u32x4_t *)ksuf, (const u32x4_t *)vsuf, (u32x4_t *)k_pages, (u32x4_t *)v_pages,
                                       table, cu, plens, n_append, tok_trace, B, T, Hkv, (int)(head_row_bytes / 16),
                                       block_size, max_blocks, n_blocks);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Rotate q and k heads (half-split pairing) and split the fp32 QKV projection into q, suffix-k and
// suffix-v buffers of the storage type.
template <typename T>
__global__ void rope_split_kernel(const float *__restrict__ qkv, const float *__restrict__ cos_t,
                                  const float *__restrict__ sin_t, T *__restrict__ q, T *__restrict__ ksuf,
                                  T *__restrict__ vsuf, T *__restrict__ q_lo, T *__restrict__ k_lo,
                                  T *__restrict__ v_lo, int n_tok, int Hq, int Hkv, int hd) {
    int half = hd >> 1;
    int heads = Hq + 2 * Hkv;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long total = (long)n_tok * heads * half;
    if (idx >= total) return;
    int i = (int)(idx % half);
    int h = (int)((idx / half) % heads);
    int t = (int)(idx / ((long)half * heads));
    const float *src = qkv + ((size_t)t * heads + h) * hd;
    float lo = src[i], hi = src[i + half];
    T *dst, *dst_lo;
    if (h < Hq) {
        size_t o = ((size_t)t * Hq + h) * hd;
        dst = q + o; dst_lo = q_lo ? q_lo + o : nullptr;
    } else if (h < Hq + Hkv) {
        size_t o = ((size_t)t * Hkv + (h - Hq)) * hd;
        dst = ksuf + o; dst_lo = k_lo ? k_lo + o : nullptr;
    } else {
        size_t o = ((size_t)t * Hkv + (h - Hq - Hkv)) * hd;
        dst = vsuf + o; dst_lo = v_lo ? v_lo + o : nullptr;
    }
    if (h < Hq + Hkv) {
        float c = cos_t[(size_t)t * half + i], sn = sin_t[(size_t)t * half + i];
        float a = lo * c - hi * sn;
        float b = hi * c + lo * sn;
        lo = a;
        hi = b;
    }
    T r0 = from_f32<T>(lo), r1 = from_f32<T>(hi);
    dst[i] = r0;
    dst[i + half] = r1;
    if (dst_lo) {
        dst_lo[i] = from_f32<T>(lo - to_f32<T>(r0));
        dst_lo[i + half] = from_f32<T>(hi - to_f32<T>(r1));
    }
}

hipError_t launch_rope_split(int dtype, const float *qkv, const float *cos_t, const float *sin_t, void *q,
                             void *ksuf, void *vsuf, void *q_lo, void *k_lo, void *v_lo, int T, int Hq, int Hkv,
                             int hd, hipStream_t s) {
    long total = (long)T * (Hq + 2 * Hkv) * (hd / 2);
    int blocks = (int)((total + 255) / 256);
    if (dtype == 0)
        rope_split_kernel<float><<<blocks, 256, 0, s>>>(qkv, cos_t, sin_t, (float *)q, (float *)ksuf, (float *)vsuf,
                                                        nullptr, nullptr, nullptr, T, Hq, Hkv, hd);
    else
        rope_split_kernel<bf16><<<blocks, 256, 0, s>>>(qkv, cos_t, sin_t, (bf16 *)q, (bf16 *)ksuf, (bf16 *)vsuf,
                                                       (bf16 *)q_lo, (bf16 *)k_lo, (bf16 *)v_lo, T, Hq, Hkv, hd);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Gate/up interleave: packed row p holds gate row f = 32*(p/64) + p%32 when p%64 < 32, else the up
// row of the same f.  A 64-column output tile slice then carries 32 (gate, up) pairs.
template <typename T>
__global__ void pack_gate_up_kernel(const T *__restrict__ src, T *__restrict__ dst, int F, int d) {
    int p = blockIdx.x;
    int blk = p >> 6, w = p & 63;
    int f = (blk << 5) + (w & 31);
    const T *s = src + (size_t)((w < 32) ? f : F + f) * d;
    T *o = dst + (size_t)p * d;
    for (int j = threadIdx.x; j < d; j += blockDim.x) o[j] = s[j];
}

hipError_t launch_pack_gate_up(int dtype, const void *src, void *dst, int F, int d, hipStream_t s) {
    if (dtype == 0) pack_gate_up_kernel<float><<<2 * F, 256, 0, s>>>((const float *)src, (float *)dst, F, d);
    else pack_gate_up_kernel<bf16><<<2 * F, 256, 0, s>>>((const bf16 *)src, (bf16 *)dst, F, d);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Row order of the QKV weight for the GEMM epilogue that rotates in registers: inside every 128-row head
// the blocks of 32 rows go [0, 2, 1, 3], i.e. new row p holds old row p for p in [0,32) and [96,128),
// old row p + 32 for p in [32,64) and old row p - 32 for p in [64,96).
__global__ void permute_heads_kernel(const bf16 *__restrict__ src, bf16 *__restrict__ dst, int d) {
    int p = blockIdx.x, in_head = p & 127, blk = in_head >> 5;
    int q = (blk == 1) ? p + 32 : (blk == 2) ? p - 32 : p;
    const u32x4_t *s = reinterpret_cast<const u32x4_t *>(src + (size_t)q * d);
    u32x4_t *o = reinterpret_cast<u32x4_t *>(dst + (size_t)p * d);
    for (int j = threadIdx.x; j < d / 8; j += blockDim.x) o[j] = s[j];
}

hipError_t launch_permute_heads(const void *src, void *dst, int n_heads, int d, hipStream_t s) {
    permute_heads_kernel<<<n_heads * 128, 256, 0, s>>>((const bf16 *)src, (bf16 *)dst, d);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// bf16 -> IEEE half, element by element (every bf16 value inside the half range converts exactly; smaller
// magnitudes land on the half subnormal grid, larger ones saturate to the largest finite half).
__global__ void bf16_to_f16_kernel(const bf16 *__restrict__ src, __half *__restrict__ dst, size_t n) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float v = __bfloat162float(src[i]);
        v = fminf(fmaxf(v, -65504.f), 65504.f);
        dst[i] = __float2half_rn(v);
    }
}

hipError_t launch_bf16_to_f16(const void *src, void *dst, size_t n, hipStream_t s) {
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    bf16_to_f16_kernel<<<(unsigned)blocks, 256, 0, s>>>((const bf16 *)src, (__half *)dst, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Verdict head: for each trace, RMSNorm of the last suffix row, dot with the n_verdict LM-head rows,
// softmax over those logits, argmax (lowest index on ties), confidence and the threshold gate.
// The [vocab, d] LM-head GEMM is never formed.
template <typename T>
__global__ void verdict_kernel(const float *__restrict__ x, const int32_t *__restrict__ last_row,
                               const T *__restrict__ g, const T *__restrict__ lm, VerdictArgs va, int B, int n_tok,
                               int d, float eps, float *__restrict__ logits, float *__restrict__ conf,
                               int32_t *__restrict__ verdict, uint8_t *__restrict__ accept) {
    __shared__ float red[4];
    __shared__ float z_s[8];
    int b = blockIdx.x;
    int row = min(max(last_row ? last_row[b] : b, 0), n_tok - 1);
    const float *xr = x + (size_t)row * d;
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += blockDim.x) ss += xr[j] * xr[j];
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    float tot = red[0] + red[1] + red[2] + red[3];
    float r = 1.0f / sqrtf(tot / (float)d + eps);
    __syncthreads();
    for (int v = 0; v < va.n_verdict; ++v) {
        const T *wr = lm + (size_t)va.ids[v] * d;
        float acc = 0.f;
        for (int j = threadIdx.x; j < d; j += blockDim.x) acc += (xr[j] * r * to_f32<T>(g[j])) * to_f32<T>(wr[j]);
        acc = wave_sum(acc);
        if (lane == 0) red[wave] = acc;
        __syncthreads();
        if (threadIdx.x == 0) z_s[v] = red[0] + red[1] + red[2] + red[3];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        int best = 0;
        float zmax = z_s[0];
        for (int v = 1; v < va.n_verdict; ++v)
            if (z_s[v] > zmax) { zmax = z_s[v]; best = v; }
        float den = 0.f;
        for (int v = 0; v < va.n_verdict; ++v) {
            logits[(size_t)b * va.n_verdict + v] = z_s[v];
            den += expf(z_s[v] - zmax);
        }
        float c = 1.0f / den;  // probability of the argmax entry
        conf[b] = c;
        verdict[b] = best;
        for (int i = 0; i < va.n_tau; ++i) accept[(size_t)i * B + b] = (c >= va.tau[i]) ? 1 : 0;
    }
}

// Full-vocabulary statistics of one row of logits: arg max (lowest index on ties), its logit, and
// lse = log sum_v exp z_v.  With verdict logits (fp32, n_verdict per row) also the largest full-vocabulary
// probability among the verdict tokens, exp(max_v z_v - lse).  One workgroup of 1024 threads per row, one pass:
// every thread keeps (max, index of the max, sum of exp(z - max)) over its elements, read four at a time where the
// row allows it, and the triples are merged pairwise; rescaling a sum when its reference maximum moves is the only
// difference from the two-pass definition.
struct HeadAcc {
    float m;     // largest logit seen
    int idx;     // its index, the lowest on ties
    float s;     // sum of exp(z - m) over the elements seen
};
__device__ __forceinline__ void head_acc_add(HeadAcc &a, float v, int j) {
    if (v > a.m) {                       // j grows within a thread, so a strict comparison keeps the lowest index
        a.s = a.s * __expf(a.m - v) + 1.0f;   // exp(-inf) = 0 for the first element
        a.m = v;
        a.idx = j;
    } else if (a.m > -INFINITY) {
        a.s += __expf(v - a.m);
    }
}
__device__ __forceinline__ HeadAcc head_acc_merge(const HeadAcc &a, const HeadAcc &b) {
    if (b.m == -INFINITY) return a;
    if (a.m == -INFINITY) return b;
    HeadAcc r;
    bool take_b = b.m > a.m || (b.m == a.m && b.idx < a.idx);
    r.m = take_b ? b.m : a.m;
    r.idx = take_b ? b.idx : a.idx;
    r.s = a.s * __expf(a.m - r.m) + b.s * __expf(b.m - r.m);
    return r;
}
constexpr int HEAD_REDUCE_THREADS = 1024;
__global__ __launch_bounds__(HEAD_REDUCE_THREADS) void head_reduce_kernel(const float *__restrict__ logits, int V,
                                                                           const float *__restrict__ verdict_logits, int n_verdict,
                                                                           int32_t *__restrict__ token, float *__restrict__ max_logit,
                                                                           float *__restrict__ lse, float *__restrict__ conf_full) {
    constexpr int NWAVES = HEAD_REDUCE_THREADS / 64;
    __shared__ float s_m[NWAVES], s_s[NWAVES];
    __shared__ int s_i[NWAVES];
    int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *z = logits + (size_t)b * V;
    HeadAcc acc = {-INFINITY, 0x7fffffff, 0.f};
    if ((V & 3) == 0 && (reinterpret_cast<uintptr_t>(z) & 15) == 0) {
        const float4 *z4 = reinterpret_cast<const float4 *>(z);
        int n4 = V >> 2;
#pragma unroll 4
        for (int j = threadIdx.x; j < n4; j += HEAD_REDUCE_THREADS) {
            float4 v = z4[j];
            head_acc_add(acc, v.x, 4 * j);
            head_acc_add(acc, v.y, 4 * j + 1);
            head_acc_add(acc, v.z, 4 * j + 2);
            head_acc_add(acc, v.w, 4 * j + 3);
        }
    } else {
        for (int j = threadIdx.x; j < V; j += HEAD_REDUCE_THREADS) head_acc_add(acc, z[j], j);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        HeadAcc o = {__shfl_xor(acc.m, off), __shfl_xor(acc.idx, off), __shfl_xor(acc.s, off)};
        acc = head_acc_merge(acc, o);
    }
    if (lane == 0) { s_m[wave] = acc.m; s_i[wave] = acc.idx; s_s[wave] = acc.s; }
    __syncthreads();
    if (threadIdx.x == 0) {
        HeadAcc t = {s_m[0], s_i[0], s_s[0]};
        for (int w = 1; w < NWAVES; ++w) t = head_acc_merge(t, HeadAcc{s_m[w], s_i[w], s_s[w]});
        float l = t.m + logf(t.s);
        token[b] = t.idx;
        max_logit[b] = t.m;
        lse[b] = l;
        if (conf_full && verdict_logits) {
            float zv = verdict_logits[(size_t)b * n_verdict];
            for (int v = 1; v < n_verdict; ++v) zv = fmaxf(zv, verdict_logits[(size_t)b * n_verdict + v]);
            conf_full[b] = expf(zv - l);
        }
    }
}

hipError_t launch_head_reduce(const float *logits, int B, int V, const float *verdict_logits, int n_verdict, int32_t *token,
                              float *max_logit, float *lse, float *conf_full, hipStream_t s) {
    head_reduce_kernel<<<B, HEAD_REDUCE_THREADS, 0, s>>>(logits, V, verdict_logits, n_verdict, token, max_logit, lse, conf_full);
    return hipGetLastError();
}

hipError_t launch_verdict(int dtype, const float *x, const int32_t *last_row, const void *final_norm,
                          const void *lm_head, VerdictArgs va, int B, int T, int d, float eps, float *logits,
                          float *conf, int32_t *verdict, uint8_t *accept, hipStream_t s) {
    if (dtype == 0)
        verdict_kernel<float><<<B, 256, 0, s>>>(x, last_row, (const float *)final_norm, (const float *)lm_head, va, B,
                                                T, d, eps, logits, conf, verdict, accept);
    else
        verdict_kernel<bf16><<<B, 256, 0, s>>>(x, last_row, (const bf16 *)final_norm, (const bf16 *)lm_head, va, B, T,
                                               d, eps, logits, conf, verdict, accept);
    return hipGetLastError();
}

}  // namespace cs
