// Kernels shaped for a generation step (Algorithm 1: the generate calls of Stage 1 and of the Stage 3 fallback): one
// new token per trace, at most 32 traces, so every projection is 32 activation rows against a weight matrix that is
// read exactly once, and attention has one query row per head.  Such a step is a stream of weights and cached
// keys / values from HBM; what these kernels are built around is keeping that stream going and touching it once.
//
// Projections (dec_gemm_kernel).  A workgroup of 8 wavefronts walks a list of 16-column tiles of the weight matrix
// over one k range of at most 24 k-tiles of 64.  Wavefront w owns the k-tiles w, w + 8, w + 16 of that range: it
// fetches exactly the activation k-tiles it will multiply (32 rows; kept in LDS, or in registers as MFMA operands
// for the long stream of the language-model head), and streams the matching weight k-tiles (16 rows x 128 bytes)
// through a private ring of LDS slots filled by direct global -> LDS loads, so the main loop has no workgroup barrier
// and every wavefront always has its ring's worth of weight k-tiles in flight, across tile borders.
// Per column tile the 8 partial 32 x 16 products are added in wavefront order through LDS and the epilogue runs on
// the sum: rotary embedding + q / k / v split (+ the write-back of the new key / value row into the paged cache),
// SwiGLU, the residual update, or the running arg max / log-sum-exp of the language-model head.
// A k range longer than 24 k-tiles is cut into slices that run as separate workgroups; they leave fp32 partial planes,
// and the workgroup that finishes a column group last (a counter per group) adds the planes in slice order and runs
// the epilogue - the order of the additions is fixed, whoever performs them, so results are bit-identical from run to
// run.  The RMSNorm in front of the QKV and gate/up projections costs no kernel and no pass over the rows: 1 / rms is a
// factor per row, so it commutes with the projection.  The residual projection that precedes writes, next to the fp32
// residual rows, the 16-bit operand x * g (g: the gain of the norm that follows) and the sum of squares of its 16
// columns of every row; the consuming projection multiplies x * g as it is and scales its result rows by
// 1 / sqrt(sum of the partial sums / d + eps) in the epilogue.
//
// Values that workgroups hand to each other inside one launch (partial planes, attention partials) travel as
// device-scope relaxed atomic stores and loads, which are written through to, and served from, the memory side of the
// per-XCD L2 caches; the arrival counter is bumped only after the stores are acknowledged.  No cache is written back or
// invalidated as a whole (a device-wide fence per workgroup costs tens of microseconds per launch here).
//
// Attention (dec_attn_kernel).  One workgroup per (trace, kv head, piece of 256 keys); each of its 8 wavefronts takes
// 32 keys = two 16-token pages: the keys straight into registers, the values global -> LDS in one go, so a CU with two
// workgroups has 256 KiB of keys / values on the way at any time.  Scores and the value product run on the
// 16 x 16 x 32 MFMA with the G query rows of the kv head in the 16-row operand; q and the probabilities are carried
// as two bf16 terms (the matrix work is negligible here, so the extra precision is free).  The pieces of a
// (trace, kv head) leave (max, sum, O) partials; the workgroup that finishes last merges them in piece order.
#include "kernels.h"
#include <algorithm>

namespace cs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

#define CS_LDS_AS __attribute__((address_space(3)))

namespace {

constexpr int DEC_THREADS = 512, DEC_WAVES = 8;
constexpr int DEC_KW = 3;                    // k-tiles a wavefront owns at most (24 per slice / 8 wavefronts)
constexpr int DEC_XT = 4096;                 // one activation k-tile: 32 rows x 128 bytes = two ring slots
constexpr int DEC_WT = 2048;                 // one weight k-tile: 16 rows x 128 bytes = one ring slot
constexpr int DEC_RED = DEC_WAVES * 32 * 16 * 4;           // 16 KiB: the 8 partial products of a column tile
// Two layouts of the 160 KiB.  Resident activations (XREG = false): the slice's activation k-tiles (up to 96 KiB) stay
// in LDS and every wavefront has a ring of 3 weight slots; the activations and the first weight k-tiles are requested
// together, so the stream starts with the kernel.  Activations in registers (XREG = true): a wavefront's share of the
// rows goes through its ring once into registers and the ring has 8 slots (16 KiB in flight per wavefront); the
// stream starts one L2 round trip later, which pays for long streams and is what lets two-term activations fit.
template <bool XREG> constexpr int dec_nslot() { return XREG ? 8 : 3; }
template <bool XREG> constexpr int dec_ring_bytes() { return DEC_WAVES * dec_nslot<XREG>() * DEC_WT; }
static_assert(DEC_MAX_KT == DEC_KW * DEC_WAVES && 2 * DEC_KW <= dec_nslot<true>() - 2, "activation k-tiles are staged in the ring");

template <bool F16>
__device__ inline f32x4 mma16(bf16x8 a, bf16x8 b, f32x4 c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// 64 lanes x 16 bytes from per-lane global addresses into LDS at lds_dst + 16 * lane (lds_dst wave-uniform).  Issued
// from inline assembly with a memory clobber: the compiler neither reorders LDS accesses across it nor waits for it;
// completion is waited for explicitly with dec_wait_vm.
__device__ inline void dma16(const void *src, unsigned lds_dst) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_dst), "v"(src) : "memory");
}
// at most n vector memory operations of this wavefront still outstanding (they complete in issue order)
template <int N>
__device__ inline void dec_wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ inline void dec_wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory"); }

// Cross-workgroup hand-over inside one launch (see the head of the file).
__device__ inline void xwg_store(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ inline float xwg_load(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// Every thread calls it after its hand-over stores: waits until they are acknowledged, then counts the workgroup in.
// Returns true (to all threads) for the workgroup that arrives last of n; that one also clears the counter.
__device__ inline bool xwg_arrive_last(int32_t *cnt, int n, volatile int *flag, int tid) {
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
    __syncthreads();
    if (tid == 0) {
        int last = atomicAdd(cnt, 1) == n - 1;
        if (last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = last;
    }
    __syncthreads();
    return *flag != 0;
}

__device__ inline unsigned pack_bf16x2(float a, float b) {
    return (unsigned)__bfloat16_as_ushort(__float2bfloat16(a)) | ((unsigned)__bfloat16_as_ushort(__float2bfloat16(b)) << 16);
}
__device__ inline unsigned short to_fmt(float v, int fmt) {   // fmt 3: IEEE half (saturating), else bf16
    return fmt == 3 ? __half_as_ushort(to_half_sat(v)) : __bfloat16_as_ushort(__float2bfloat16(v));
}

}  // namespace

// ---- control block of a step: the arrival counters, zero at the start of every step -------------------------------
// ctl[DEC_CTL_ATTN ..]   one per (trace, kv head): pieces of the attention kernel
// ctl[DEC_CTL_TILE ..]   one per column group of a sliced projection
__global__ void dec_init_kernel(int32_t *__restrict__ ctl, int n_ctl) {
    for (int i = threadIdx.x; i < n_ctl; i += blockDim.x) ctl[i] = 0;
}

hipError_t launch_dec_init(int32_t *ctl, hipStream_t s) {
    dec_init_kernel<<<1, 256, 0, s>>>(ctl, DEC_CTL_INTS);
    return hipGetLastError();
}

// ---- projections ----------------------------------------------------------------------------------------------------
// The two 8-row groups of weight rows behind column tile t (accumulator columns 0..7 and 8..15).
__device__ inline void dec_tile_rows(int epi, int t, int perm, int &rA, int &rB) {
    if (epi == DEC_EPI_SWIGLU) {            // 8 gate rows and the 8 up rows of the same activations (groups of 32 interleaved)
        int f0 = 8 * t;
        rA = 64 * (f0 >> 5) + (f0 & 31);
        rB = rA + 32;
    } else if (epi == DEC_EPI_ROPE) {       // 8 columns of a head's first half and their rotation partners
        int head = t >> 3, o0 = 8 * (t & 7);
        int p = perm ? (o0 < 32 ? o0 : 32 + o0) : o0;   // reordered heads: [0..31 | 64..95 | 32..63 | 96..127]
        rA = head * 128 + p;
        rB = rA + (perm ? 32 : 64);
    } else {
        rA = 16 * t;
        rB = rA + 8;
    }
}

// Epilogue of one element (row, accumulator column c of tile t) of a projection; called by all 512 threads together.
template <int EPI>
__device__ inline void dec_epilogue(const DecGemm &a, int t, int row, int c, float v) {
    const bool live = row < a.M;
    if constexpr (EPI == DEC_EPI_RESID) {
        const int N = a.n_ct * 16, col = t * 16 + c;
        float xn = 0.f;
        if (live) {
            float *p = a.x + (size_t)row * N + col;
            xn = *p + v;
            *p = xn;
        }
        if (a.xg_out) {
            // for the projection that follows: the operand x * g in its 16-bit format, and this tile's share of the
            // row's sum of squares (added over the tile's 16 columns in a fixed butterfly order)
            float sq = xn * xn;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) sq += __shfl_xor(sq, off);
            if (live) {
                reinterpret_cast<unsigned short *>(a.xg_out)[(size_t)row * N + col] = to_fmt(xn * __bfloat162float(a.g_next[col]), a.xg_fmt);
                if (c == 0) a.ssq_out[t * DEC_MAX_ROWS + row] = sq;
            }
        }
    } else if constexpr (EPI == DEC_EPI_SWIGLU) {
        // columns 0..7 hold gate values, 8..15 the up values of the same activations
        float up = __shfl_xor(v, 8);
        if (live && c < 8) {
            float act = v * __builtin_amdgcn_rcpf(1.0f + __expf(-v)) * up;
            reinterpret_cast<unsigned short *>(a.act)[(size_t)row * (a.n_ct * 8) + t * 8 + c] = to_fmt(act, a.act_fmt);
        }
    } else {
        // columns 0..7: columns o .. o + 7 of the head's first half; 8..15: their rotation partners o + 64
        const RopeArgs &r = a.rope;
        float other = __shfl_xor(v, 8);
        const int head = t >> 3, o = 8 * (t & 7) + (c & 7);
        const bool is_q = head < r.Hq, is_v = head >= r.Hq + r.Hkv;
        const int hh = is_q ? head : is_v ? head - r.Hq - r.Hkv : head - r.Hq;
        const int heads = is_q ? r.Hq : r.Hkv;
        if (!live) return;
        float out = v;
        if (!is_v) {
            float cs = r.cos_t[(size_t)row * 64 + o], sn = r.sin_t[(size_t)row * 64 + o];
            out = c < 8 ? v * cs - other * sn : v * cs + other * sn;
        }
        const int col = c < 8 ? o : o + 64;
        const size_t idx = ((size_t)row * heads + hh) * 128 + col;
        bf16 hi = __float2bfloat16(out);
        reinterpret_cast<bf16 *>(is_q ? r.q : is_v ? r.v : r.k)[idx] = hi;
        if (is_q) {
            if (r.q_lo) reinterpret_cast<bf16 *>(r.q_lo)[idx] = __float2bfloat16(out - __bfloat162float(hi));
        } else if (a.n_append && a.n_append[row] > 0) {
            // the token joins the context: its key / value row goes to row L_b of the trace's pages
            int pos = a.plens[row];
            if (pos >= 0 && pos < a.max_blocks * 16) {
                int blk = min(max(a.table[(size_t)row * a.max_blocks + (pos >> 4)], 0), a.n_blocks - 1);
                reinterpret_cast<bf16 *>(is_v ? a.v_pages : a.k_pages)[(((size_t)blk * r.Hkv + hh) * 16 + (pos & 15)) * 128 + col] = hi;
            }
        }
    }
}

// Running (max, first index of the max, sum of exp(z - max)) of a row of logits.
struct DecHeadAcc {
    float m;
    int idx;
    float s;
};
__device__ inline DecHeadAcc dec_head_merge(DecHeadAcc a, DecHeadAcc b) {   // lowest index on equal maxima
    DecHeadAcc r;
    const bool a_first = a.m > b.m || (a.m == b.m && a.idx < b.idx);
    r.m = a_first ? a.m : b.m;
    r.idx = a_first ? a.idx : b.idx;
    r.s = (a.m == -INFINITY ? 0.f : a.s * __expf(a.m - r.m)) + (b.m == -INFINITY ? 0.f : b.s * __expf(b.m - r.m));
    return r;
}

template <int EPI, bool F16, bool NORMX, int TERMS, bool XREG>
__global__ __launch_bounds__(DEC_THREADS) void dec_gemm_kernel(DecGemm a) {
    static_assert(XREG || TERMS == 1, "two-term activations only fit in registers");
    constexpr int NSLOT = dec_nslot<XREG>();
    constexpr int SLOT0 = XREG ? 2 * DEC_KW : 0;                        // slot of unit 0
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = blockIdx.x / a.nwg, j = blockIdx.x - s * a.nwg;       // k slice, column group
    const int nk = a.K >> 6;
    const int kt0 = (int)((long)s * nk / a.S), kt1 = (int)((long)(s + 1) * nk / a.S);
    const int nks = kt1 - kt0;                                          // k-tiles of this slice (<= 24)
    const int nkw = nks > wave ? (nks - wave + DEC_WAVES - 1) / DEC_WAVES : 0;   // ... owned by this wavefront (<= 3)
    const int n_my = (a.n_ct - j + a.nwg - 1) / a.nwg;                  // column tiles j, j + nwg, ...
    const int total = n_my * nkw;                                       // (tile, k-tile) units of this wavefront

    // LDS: [resident activations: nks k-tiles] [rings: 8 wavefronts x NSLOT slots] [red]
    const int x_bytes = XREG ? 0 : nks * DEC_XT;
    unsigned char *xs = smem;
    unsigned char *ring = smem + x_bytes + wave * NSLOT * DEC_WT;       // this wavefront's slots
    float *red = reinterpret_cast<float *>(smem + x_bytes + dec_ring_bytes<XREG>());
    volatile int *s_last = reinterpret_cast<volatile int *>(red);       // arrival flag (after the main loop, red is free)
    const unsigned lds0 = (unsigned)(size_t)(CS_LDS_AS unsigned char *)smem;
    const unsigned ring0 = (unsigned)(size_t)(CS_LDS_AS unsigned char *)ring;

    // Direct-load roles: one instruction fills 8 rows x 128 bytes; lane l sits at row l / 8, 16-byte slot l % 8 and
    // fetches the k-vector that the swizzle (slot = vector ^ ((row >> 1) & 7), row counted inside the tile) puts there.
    const int lr = lane >> 3, lslot = lane & 7;
    // Unit u = (column tile u / nkw, the wavefront's k-tile u % nkw) goes through slot (SLOT0 + u) % NSLOT.
    auto issue_unit = [&](int u) {
        int ti = u / nkw, i = u - ti * nkw;
        int t = j + ti * a.nwg, kt = kt0 + wave + DEC_WAVES * i;
        int rA, rB;
        dec_tile_rows(EPI, t, a.perm, rA, rB);
        unsigned dst = ring0 + ((u + SLOT0) % NSLOT) * DEC_WT;
        int vecA = lslot ^ ((lr >> 1) & 7), vecB = lslot ^ (((8 + lr) >> 1) & 7);
        dma16(a.W + (size_t)(rA + lr) * a.K + (size_t)kt * 64 + vecA * 8, dst);
        dma16(a.W + (size_t)(rB + lr) * a.K + (size_t)kt * 64 + vecB * 8, dst + 1024);
    };
    // activation k-tile i of this wavefront (term: 0 = hi, 1 = lo half of a two-term row) to LDS address dst
    auto issue_x = [&](int i, int term, unsigned dst) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            int row = 8 * r4 + lr;
            int vec = lslot ^ ((row >> 1) & 7);
            const bf16 *src = a.X + (size_t)min(row, a.M - 1) * a.ldx + (size_t)term * a.K +
                              (size_t)(kt0 + wave + DEC_WAVES * i) * 64 + vec * 8;      // rows past M repeat the last row
            dma16(src, dst + r4 * 1024);
        }
    };
    // fragment addresses: 16 x 16 x 32 MFMA, lane l supplies row l % 16 and the k-vector l / 16 of a 32-wide k-step
    const int fr = lane & 15, fg = lane >> 4;
    int w_off[2], x_off[2][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        w_off[ks] = fr * 128 + (((4 * ks + fg) ^ ((fr >> 1) & 7)) << 4);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            int row = 16 * rb + fr;
            x_off[ks][rb] = row * 128 + (((4 * ks + fg) ^ ((row >> 1) & 7)) << 4);
        }
    }
    bf16x8 xf[TERMS][DEC_KW][2][2];                                     // XREG: the wavefront's activations as operands
    if constexpr (XREG) {
        // through slots 0..5 into registers, once per term; the first two weight units are on their way in slots 6, 7
#pragma unroll
        for (int term = 0; term < TERMS; ++term) {
#pragma unroll
            for (int i = 0; i < DEC_KW; ++i)
                if (i < nkw) issue_x(i, term, ring0 + i * DEC_XT);
            if (term == 0) {
                if (0 < total) issue_unit(0);
                if (1 < total) issue_unit(1);
            }
            // the staged k-tiles were issued before the weight units of this term (if any): they land first
            if (term == 0 && total >= 2) dec_wait_vm<4>();
            else if (term == 0 && total == 1) dec_wait_vm<2>();
            else dec_wait_vm<0>();
#pragma unroll
            for (int i = 0; i < DEC_KW; ++i)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb)
                        xf[term][i][ks][rb] = i < nkw ? *reinterpret_cast<const bf16x8 *>(ring + i * DEC_XT + x_off[ks][rb]) : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            dec_wait_lds();
        }
#pragma unroll
        for (int u = 2; u < NSLOT; ++u)
            if (u < total) issue_unit(u);
    } else {
        // resident: the wavefront's k-tiles into their places, then the first weight units (in order: the activations
        // have landed whenever a unit has)
        for (int i = 0; i < nkw; ++i) issue_x(i, 0, lds0 + (wave + DEC_WAVES * i) * DEC_XT);
#pragma unroll
        for (int u = 0; u < NSLOT; ++u)
            if (u < total) issue_unit(u);
    }

    const int row = tid >> 4, c = tid & 15;                             // this thread's element of a 32 x 16 tile
    // NORMX: the operand is x * g without the 1 / rms factor of its row; the factor comes from the partial sums of
    // squares the preceding projection left (one per 16 columns of the row), added in a fixed order: the 16 lanes of
    // a row take every 16th partial, then a butterfly.
    // (the partials are requested here and added up in front of the first epilogue, under the main loop's loads)
    float rinv = 1.0f, sqv[8];
    if constexpr (NORMX) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sqv[e] = c + 16 * e < a.ssq_n ? a.ssq_in[(c + 16 * e) * DEC_MAX_ROWS + min(row, a.M - 1)] : 0.f;
    }
    DecHeadAcc hacc = {-INFINITY, 0x7fffffff, 0.f};                     // HEAD: this thread's columns so far
    const size_t plane = (size_t)DEC_MAX_ROWS * a.n_ct * 16;
    int u = 0;
    for (int ti = 0; ti < n_my; ++ti) {
        const int t = j + ti * a.nwg;
        f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int i = 0; i < DEC_KW; ++i) {
            if (i < nkw) {
                const int after = min(NSLOT - 1, total - 1 - u);        // units issued after this one
                switch (after) {
                    case 7: dec_wait_vm<14>(); break;
                    case 6: dec_wait_vm<12>(); break;
                    case 5: dec_wait_vm<10>(); break;
                    case 4: dec_wait_vm<8>(); break;
                    case 3: dec_wait_vm<6>(); break;
                    case 2: dec_wait_vm<4>(); break;
                    case 1: dec_wait_vm<2>(); break;
                    default: dec_wait_vm<0>(); break;
                }
                const unsigned char *wsl = ring + ((u + SLOT0) % NSLOT) * DEC_WT;
                bf16x8 wf[2];
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) wf[ks] = *reinterpret_cast<const bf16x8 *>(wsl + w_off[ks]);
                if constexpr (!XREG) {
                    const unsigned char *xt = xs + (wave + DEC_WAVES * i) * DEC_XT;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        xf[0][i][ks][0] = *reinterpret_cast<const bf16x8 *>(xt + x_off[ks][0]);
                        xf[0][i][ks][1] = *reinterpret_cast<const bf16x8 *>(xt + x_off[ks][1]);
                    }
                }
                dec_wait_lds();                                         // the slot is in registers: refill it
                if (u + NSLOT < total) issue_unit(u + NSLOT);
#pragma unroll
                for (int term = 0; term < TERMS; ++term)
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        acc[0] = mma16<F16>(xf[term][i][ks][0], wf[ks], acc[0]);
                        acc[1] = mma16<F16>(xf[term][i][ks][1], wf[ks], acc[1]);
                    }
                ++u;
            }
        }
        // accumulator layout: column lane % 16, rows 16 rb + 4 (lane / 16) + e
        float *mine = red + wave * 512;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int e = 0; e < 4; ++e) mine[(16 * rb + 4 * fg + e) * 16 + fr] = acc[rb][e];
        __syncthreads();
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < DEC_WAVES; ++w) v += red[w * 512 + tid];   // wavefront order: fixed
        __syncthreads();                                                // red is free for the next tile
        if constexpr (NORMX) {
            if (ti == 0) {
                float sq = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) sq += sqv[e];
                for (int i = c + 128; i < a.ssq_n; i += 16) sq += a.ssq_in[i * DEC_MAX_ROWS + min(row, a.M - 1)];
#pragma unroll
                for (int off = 8; off >= 1; off >>= 1) sq += __shfl_xor(sq, off);
                rinv = 1.0f / sqrtf(sq / (float)a.K + a.eps);
            }
        }
        if constexpr (EPI == DEC_EPI_HEAD) {
            // logit of (row, vocabulary entry 16 t + c): into the thread's running statistics (its entries ascend)
            const int idx = 16 * t + c;
            if (v > hacc.m) {
                hacc.s = (hacc.m == -INFINITY ? 0.f : hacc.s * __expf(hacc.m - v)) + 1.0f;
                hacc.m = v;
                hacc.idx = idx;
            } else {
                hacc.s += __expf(v - hacc.m);
            }
        } else {
            if (a.S > 1) xwg_store(a.planes + (size_t)s * plane + (size_t)row * (a.n_ct * 16) + t * 16 + c, v);
            else dec_epilogue<EPI>(a, t, row, c, v * rinv);
        }
    }
    if constexpr (EPI == DEC_EPI_HEAD) {
        // the 16 threads of a row, then one record per (workgroup, row) for the kernel that finishes the rows
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) {
            DecHeadAcc o = {__shfl_xor(hacc.m, off), __shfl_xor(hacc.idx, off), __shfl_xor(hacc.s, off)};
            hacc = dec_head_merge(hacc, o);
        }
        if (c == 0) {
            float *rec = a.head_part + ((size_t)j * DEC_MAX_ROWS + row) * 4;
            rec[0] = hacc.m;
            rec[1] = __int_as_float(hacc.idx);
            rec[2] = hacc.s;
        }
        return;
    }
    if (a.S > 1) {
        // the slices of column group j: the last one to arrive adds the planes in slice order
        if (!xwg_arrive_last(a.tile_cnt + j, a.S, s_last, tid)) return;
        for (int ti = 0; ti < n_my; ++ti) {
            const int t = j + ti * a.nwg;
            const float *p = a.planes + (size_t)row * (a.n_ct * 16) + t * 16 + c;
            float v = 0.f;
            for (int sp = 0; sp < a.S; sp += 8) {                       // eight loads in flight, added in slice order
                float pv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) pv[e] = sp + e < a.S ? xwg_load(p + (size_t)(sp + e) * plane) : 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) v += pv[e];
            }
            dec_epilogue<EPI>(a, t, row, c, v * rinv);
        }
    }
}

// The rows of the language-model head: the records of all workgroups of dec_gemm_kernel<DEC_EPI_HEAD> merged in
// workgroup order per row (one wavefront per row).
__global__ __launch_bounds__(64) void dec_head_final_kernel(const float *__restrict__ part, int nwg, const float *__restrict__ verdict_logits,
                                                             int n_verdict, int32_t *__restrict__ token, float *__restrict__ max_logit,
                                                             float *__restrict__ lse, float *__restrict__ conf_full) {
    const int b = blockIdx.x, lane = threadIdx.x;
    DecHeadAcc acc = {-INFINITY, 0x7fffffff, 0.f};
    for (int g = lane; g < nwg; g += 64) {
        const float *rec = part + ((size_t)g * DEC_MAX_ROWS + b) * 4;
        acc = dec_head_merge(acc, DecHeadAcc{rec[0], __float_as_int(rec[1]), rec[2]});
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        DecHeadAcc o = {__shfl_xor(acc.m, off), __shfl_xor(acc.idx, off), __shfl_xor(acc.s, off)};
        acc = dec_head_merge(acc, o);
    }
    if (lane == 0) {
        float l = acc.m + logf(acc.s);
        token[b] = acc.idx;
        max_logit[b] = acc.m;
        lse[b] = l;
        if (conf_full && verdict_logits) {
            float zv = verdict_logits[(size_t)b * n_verdict];
            for (int v = 1; v < n_verdict; ++v) zv = fmaxf(zv, verdict_logits[(size_t)b * n_verdict + v]);
            conf_full[b] = expf(zv - l);
        }
    }
}

hipError_t launch_dec_head_final(const float *part, int nwg, int B, const float *verdict_logits, int n_verdict, int32_t *token,
                                 float *max_logit, float *lse, float *conf_full, hipStream_t s) {
    dec_head_final_kernel<<<B, 64, 0, s>>>(part, nwg, verdict_logits, n_verdict, token, max_logit, lse, conf_full);
    return hipGetLastError();
}

// Slices and workgroups of a projection.  A k range that fits one slice is never cut (no partial planes, no counters):
// one workgroup per CU, each with its share of the column tiles.  A longer one is cut into S slices of at most 24
// k-tiles, and S x nwg workgroups run in rounds of 256.  The choice minimises a model of the launch, in units of one
// column tile over 8 k-tiles (16 KiB of weights per workgroup, about 0.7 us at the rate a CU streams them):
//   rounds x (4 + tiles per workgroup x units per tile)   a workgroup's fixed cost (activations, first weights) is 4
//   + tiles per workgroup x ceil(S / 8) x 2                 the last slice of a column group to arrive adds the S planes of
//                                                           its tiles, eight loads at a time, alone
// Few column groups with many slices leave that last sum to a handful of workgroups (d_ffn 27648 as 32 slices x 8
// groups: 200 us per projection); many small workgroups pay the fixed cost once per round.
void dec_gemm_plan(int K, int n_ct, int *S_out, int *nwg_out) {
    const int nk = K / 64;
    const int s_min = (nk + DEC_MAX_KT - 1) / DEC_MAX_KT;
    if (s_min == 1) {
        *S_out = 1;
        *nwg_out = std::min(n_ct, 256);
        return;
    }
    double best = -1;
    int best_s = s_min, best_g = 1;
    for (int S = s_min; S <= std::min(nk, 2 * s_min + 2); ++S) {
        const double units = (double)((nk + S - 1) / S) / 8.0;     // the weights a workgroup streams per tile
        for (int g = 8; g <= 256; g += 8) {        // multiples of 8: the slices of a column group share an XCD, and with it an L2
            const int gg = std::min(g, n_ct);
            const int tiles = (n_ct + gg - 1) / gg;
            const long rounds = ((long)S * gg + 255) / 256;
            const double cost = (double)rounds * (4.0 + tiles * units) + tiles * ((S + 7) / 8) * 2.0;
            if (best < 0 || cost < best) { best = cost; best_s = S; best_g = gg; }
            if (gg == n_ct) break;
        }
    }
    *S_out = best_s;
    *nwg_out = best_g;
}
size_t dec_gemm_plane_bytes(int K, int n_ct) {
    int S, nwg;
    dec_gemm_plan(K, n_ct, &S, &nwg);
    return S > 1 ? (size_t)S * DEC_MAX_ROWS * n_ct * 16 * 4 : 0;
}

template <int EPI, bool F16, bool NORMX, int TERMS, bool XREG = false>
static hipError_t launch_dec_gemm_inst(const DecGemm &a, hipStream_t s) {
    static std::atomic<uint32_t> attr_done{0};
    auto kern = dec_gemm_kernel<EPI, F16, NORMX, TERMS, XREG>;
    constexpr int max_smem = (XREG ? 0 : DEC_MAX_KT * DEC_XT) + dec_ring_bytes<XREG>() + DEC_RED;     // 160 / 144 KiB
    if (hipError_t e = set_dynamic_lds_once(attr_done, reinterpret_cast<const void *>(kern), max_smem); e != hipSuccess) return e;
    const int nk = a.K / 64;
    const int smem = (XREG ? 0 : (nk + a.S - 1) / a.S * DEC_XT) + dec_ring_bytes<XREG>() + DEC_RED;
    kern<<<a.S * a.nwg, DEC_THREADS, smem, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_dec_gemm(const DecGemm &a, int epi, bool f16, hipStream_t s) {
    const int nk = a.K / 64;
    if (a.M < 1 || a.M > DEC_MAX_ROWS || a.K % 64 != 0 || a.S < 1 || a.nwg < 1 || a.nwg > 256 || a.n_ct < a.nwg ||
        (nk + a.S - 1) / a.S > DEC_MAX_KT || a.S > nk || (a.S > 1 && (!a.planes || !a.tile_cnt)))
        return hipErrorInvalidValue;
    const bool nx = a.ssq_in != nullptr;      // the operand lacks the 1 / rms factor of its rows
    if (!a.X || (nx && a.ssq_n < 1)) return hipErrorInvalidValue;
    switch (epi) {
        case DEC_EPI_ROPE:
            if (nx) return f16 ? launch_dec_gemm_inst<DEC_EPI_ROPE, true, true, 1>(a, s) : launch_dec_gemm_inst<DEC_EPI_ROPE, false, true, 1>(a, s);
            return f16 ? launch_dec_gemm_inst<DEC_EPI_ROPE, true, false, 1>(a, s) : launch_dec_gemm_inst<DEC_EPI_ROPE, false, false, 1>(a, s);
        case DEC_EPI_SWIGLU:
            if (nx) return f16 ? launch_dec_gemm_inst<DEC_EPI_SWIGLU, true, true, 1>(a, s) : launch_dec_gemm_inst<DEC_EPI_SWIGLU, false, true, 1>(a, s);
            return f16 ? launch_dec_gemm_inst<DEC_EPI_SWIGLU, true, false, 1>(a, s) : launch_dec_gemm_inst<DEC_EPI_SWIGLU, false, false, 1>(a, s);
        case DEC_EPI_RESID:
            if (nx) return hipErrorInvalidValue;
            return f16 ? launch_dec_gemm_inst<DEC_EPI_RESID, true, false, 1>(a, s) : launch_dec_gemm_inst<DEC_EPI_RESID, false, false, 1>(a, s);
        case DEC_EPI_HEAD:      // two-term bf16 rows [M, 2 K] against the bf16 head, one k slice
            if (nx || f16 || a.S != 1 || !a.head_part) return hipErrorInvalidValue;
            return launch_dec_gemm_inst<DEC_EPI_HEAD, false, false, 2, true>(a, s);
    }
    return hipErrorInvalidValue;
}

// ---- attention ------------------------------------------------------------------------------------------------------
// One workgroup of 8 wavefronts per (trace, kv head, piece of n_iter x 256 keys); in each round of 256 keys wavefront
// w takes the two 16-token pages 2 w, 2 w + 1 and keeps a running (max, sum, O) over its rounds.  Keys go straight from global memory into the registers of the score product's first
// operand (lane l: token l % 16 of a page, head-dim elements 32 ks + 8 (l / 16) .. + 7), values go global -> LDS
// (8 KiB per wavefront, rows of 256 bytes) and come back through transposing reads as the first operand of
// O^T += V^T . P^T.  The 16-byte vector v of token k sits at slot v ^ (2 (k & 7)) of its row, so that the 32 bytes x 8
// consecutive tokens that half a wavefront reads at a time fall into different banks; the lane that fills a slot
// fetches the matching global vector.
// Transposing reads (ds_read_b64_tr_b16): in a group of 16 lanes, lane i supplies the address of 4 consecutive 16-bit
// elements and receives element i % 4 of what lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4 addressed.
// The last piece of a trace is short (with L a multiple of 256 it holds the new token only); the grid starts with the
// last pieces, so they finish while the full pieces are still streaming instead of after them.
constexpr int DEC_ATTN_THREADS = 512, DEC_ATTN_WAVES = 8;
constexpr int DEC_ATTN_WAVE_LDS = 8192;
constexpr int DEC_ATTN_SMEM = DEC_ATTN_WAVES * DEC_ATTN_WAVE_LDS;
static_assert(DEC_PIECE == 32 * DEC_ATTN_WAVES, "a piece is two pages per wavefront");

// MULTI: the workgroup makes a.n_iter rounds (otherwise exactly one: the compiler then knows that nothing is carried
// into the round, which keeps the kernel at 96 registers and two workgroups on a CU; the loop form needs 144).
template <bool MULTI>
__global__ __launch_bounds__(DEC_ATTN_THREADS, MULTI ? 1 : 2) void dec_attn_kernel(DecAttn a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __shared__ volatile int s_last;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // grid: x = (piece, kv head), pieces from the last one of the longest trace down; y = trace.  Everything a
    // workgroup needs to find its keys follows from its indices and one load of the trace's length.
    const int h = blockIdx.x % a.Hkv, b = blockIdx.y;
    const int p = a.max_pieces - 1 - blockIdx.x / a.Hkv;
    const int L = min(max(a.plens[b], 0), a.max_L);                     // keys 0 .. L-1 are cached, key L is the new token
    const int n_iter = MULTI ? a.n_iter : 1;
    const int piece_keys = DEC_PIECE * n_iter;                          // a workgroup makes n_iter rounds of 256 keys
    const int n_p = L / piece_keys + 1;                                 // pieces over the L + 1 keys
    if (p >= n_p) return;                                               // uniform: a shorter trace
    const int pi = b * a.max_pieces + p;                                // index of the piece's partial results
    const int G = a.G;
    unsigned char *vst = smem + wave * DEC_ATTN_WAVE_LDS;
    const unsigned lds_v = (unsigned)(size_t)(CS_LDS_AS unsigned char *)vst;

    const int fr = lane & 15, fg = lane >> 4;
    float m_w = -INFINITY, l_w = 0.f;                                   // running maximum (log2 units) and sum of this wavefront
    f32x4 o_acc[8];
#pragma unroll
    for (int hb = 0; hb < 8; ++hb) o_acc[hb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bool active = piece_keys * p + 32 * wave <= L;                // wave-uniform: the wavefront sees at least one key
    for (int it = 0; it < n_iter; ++it) {
        const int key0 = piece_keys * p + DEC_PIECE * it + 32 * wave;   // this wavefront's 32 keys of this round
        if (key0 > L) break;                                            // wave-uniform; later rounds lie further out
        // A token at or past L comes from the new token's row (token L itself; later ones are masked), so page rows
        // that were never written are not read.
        const bf16 *ks_row = a.ksuf + ((size_t)b * a.Hkv + h) * 128, *vs_row = a.vsuf + ((size_t)b * a.Hkv + h) * 128;
        const int lrow = lane >> 4, lslot = lane & 15;
        bf16x8 kf[2][4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const int pg = (key0 >> 4) + kb;
            int id = 0;
            if (pg * 16 < L) id = min(max(a.table[(size_t)b * a.max_blocks + min(pg, a.max_blocks - 1)], 0), a.n_blocks - 1);
            const size_t page = ((size_t)id * a.Hkv + h) * 16 * 128;
            // values: instruction jj fills tokens 4 jj .. 4 jj + 3 of the page; lane l: token 4 jj + l / 16, slot l % 16
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int kl = 4 * jj + lrow;
                const int vvec = lslot ^ (2 * (kl & 7));
                dma16(pg * 16 + kl < L ? a.v_pages + page + kl * 128 + vvec * 8 : vs_row + vvec * 8, lds_v + kb * 4096 + jj * 1024);
            }
            // keys: token fr of the page, 16 bytes per k-step
            const bf16 *krow = pg * 16 + fr < L ? a.k_pages + page + fr * 128 : ks_row;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) kf[kb][ks] = *reinterpret_cast<const bf16x8 *>(krow + 32 * ks + 8 * fg);
        }
        // q operand: lane l holds query row l % 16 (rows >= G are zero), head-dim elements 32 ks + 8 (l / 16) .. + 7
        // (fetched in every round rather than kept: with it live across the loop the kernel needs more than 128
        // registers and a CU holds one workgroup instead of two)
        bf16x8 q_hi[4], q_lo[4];
        {
            const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
            const size_t qo = ((size_t)b * a.Hq + (size_t)h * G + min(fr, G - 1)) * 128;
    #pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                q_hi[ks] = fr < G ? *reinterpret_cast<const bf16x8 *>(a.q + qo + 32 * ks + 8 * fg) : zero;
                q_lo[ks] = (fr < G && a.q_lo) ? *reinterpret_cast<const bf16x8 *>(a.q_lo + qo + 32 * ks + 8 * fg) : zero;
            }
        }
        // scores: S^T[token][query row]; lane l ends up with query row l % 16, tokens 4 (l / 16) + e of each page
        f32x4 sc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                sc[kb] = mma16<false>(kf[kb][ks], q_hi[ks], sc[kb]);
                sc[kb] = mma16<false>(kf[kb][ks], q_lo[ks], sc[kb]);
            }
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = (key0 + 16 * kb + 4 * fg + e <= L) ? sc[kb][e] * a.scale_log2 : -INFINITY;
                sc[kb][e] = v;
                mx = fmaxf(mx, v);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // running maximum: finite from the first round on (token key0 <= L is visible to every query row)
        const float m_new = fmaxf(m_w, mx);
        const float alpha = m_w == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_w - m_new);
        m_w = m_new;
        float ps = 0.f, pv[8];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float pr = __builtin_amdgcn_exp2f(sc[kb][e] - m_new);
                pv[4 * kb + e] = pr;
                ps += pr;
            }
        ps += __shfl_xor(ps, 16);
        ps += __shfl_xor(ps, 32);
        l_w = l_w * alpha + ps;
        if (it > 0) {
#pragma unroll
            for (int hb = 0; hb < 8; ++hb) o_acc[hb] *= alpha;
        }
        // probabilities as the second operand of O^T += V^T . P^T: k index 8 (l / 16) + i <-> token 4 (l / 16) + i of
        // page 0 (i < 4) or page 1 (i >= 4), which is what the lane already holds; two bf16 terms
        bf16x8 p_hi, p_lo;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __bf16 hi = (__bf16)pv[i];
            p_hi[i] = hi;
            p_lo[i] = (__bf16)(pv[i] - (float)hi);
        }
        dec_wait_vm<0>();                                // the values have landed
        // V^T operand: group l / 16 reads tokens 4 (l / 16) .. + 3 of a page; lane i of the group points at token
        // i / 4, head-dim elements 16 hb + 4 (i % 4) .. + 3 and receives the four tokens of element 16 hb + i
        const int vrow = 4 * fg + (fr >> 2), q4 = fr & 3;
#pragma unroll
        for (int hb = 0; hb < 8; ++hb) {
            const unsigned char *p0 = vst + vrow * 256 + (((2 * hb + (q4 >> 1)) ^ (2 * (vrow & 7))) << 4) + ((q4 & 1) << 3);
            i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CS_LDS_AS i16x4 *)p0);
            i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CS_LDS_AS i16x4 *)(p0 + 4096));
            bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            o_acc[hb] = mma16<false>(vf, p_hi, o_acc[hb]);
            o_acc[hb] = mma16<false>(vf, p_lo, o_acc[hb]);
        }
        dec_wait_lds();                                  // the value region may be refilled (or reused below)
    }
    // ---- the eight wavefronts' results, combined in wavefront order.  Each leaves O [8 rows][128] fp32, then max and
    // sum per row, in its own value region (its own reads of that region are complete).
    float *om = reinterpret_cast<float *>(vst);
    if (active && fr < G) {
#pragma unroll
        for (int hb = 0; hb < 8; ++hb)
            *reinterpret_cast<f32x4 *>(om + fr * 128 + 16 * hb + 4 * fg) = o_acc[hb];   // rows 16 hb + 4 (l / 16) + e
    }
    if (fg == 0 && fr < DEC_MAX_G) {
        om[1024 + fr] = active ? m_w : -INFINITY;
        om[1040 + fr] = active ? l_w : 0.f;
    }
    __syncthreads();
    const int hd = tid & 127;
    const size_t item = (size_t)pi * a.Hkv + h;
    auto store_out = [&](int jq, float v) {
        const int Hq = a.Hq;
        unsigned short *o = reinterpret_cast<unsigned short *>(a.out);
        if (a.out_fmt == 2) {
            size_t base = (size_t)b * 2 * Hq * 128 + ((size_t)h * G + jq) * 128 + hd;
            bf16 hi = __float2bfloat16(v);
            o[base] = __bfloat16_as_ushort(hi);
            o[base + (size_t)Hq * 128] = __bfloat16_as_ushort(__float2bfloat16(v - __bfloat162float(hi)));
        } else {
            o[((size_t)b * Hq + (size_t)h * G + jq) * 128 + hd] = to_fmt(v, a.out_fmt);
        }
    };
    for (int jq = tid >> 7; jq < G; jq += 4) {
        float mw[DEC_ATTN_WAVES], M = -INFINITY;
#pragma unroll
        for (int w = 0; w < DEC_ATTN_WAVES; ++w) {
            mw[w] = reinterpret_cast<const float *>(smem + w * DEC_ATTN_WAVE_LDS)[1024 + jq];
            M = fmaxf(M, mw[w]);
        }
        float acc = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < DEC_ATTN_WAVES; ++w) {
            if (mw[w] == -INFINITY) continue;            // a wavefront past the end left nothing
            const float *ow = reinterpret_cast<const float *>(smem + w * DEC_ATTN_WAVE_LDS);
            float wgt = __builtin_amdgcn_exp2f(mw[w] - M);
            acc += wgt * ow[jq * 128 + hd];
            l += wgt * ow[1040 + jq];
        }
        if (n_p == 1) {
            store_out(jq, acc / l);
        } else {
            xwg_store(a.part_o + (item * DEC_MAX_G + jq) * 128 + hd, acc);
            if (hd == 0) {
                xwg_store(a.part_ml + (item * DEC_MAX_G + jq) * 2, M);
                xwg_store(a.part_ml + (item * DEC_MAX_G + jq) * 2 + 1, l);
            }
        }
    }
    if (n_p == 1) return;
    // ---- the pieces of this (trace, kv head): the last one to arrive merges them in piece order
    int32_t *cnt = a.ctl + DEC_CTL_ATTN + b * a.Hkv + h;
    if (!xwg_arrive_last(cnt, n_p, &s_last, tid)) return;
    // maxima and sums of all pieces into LDS (every thread needs them), then the weighted sums, 16 loads in flight
    float *ml = reinterpret_cast<float *>(smem);                        // [n_p][8][2]
    const size_t item0 = (size_t)b * a.max_pieces * a.Hkv + h;
    const int n_ml = min(n_p, DEC_ATTN_SMEM / (DEC_MAX_G * 2 * 4));     // pieces whose (max, sum) fit LDS: 1024
    for (int i = tid; i < n_ml * DEC_MAX_G * 2; i += DEC_ATTN_THREADS) {
        int pp = i / (DEC_MAX_G * 2), r = i - pp * (DEC_MAX_G * 2);
        ml[i] = (r >> 1) < G ? xwg_load(a.part_ml + (item0 + (size_t)pp * a.Hkv) * DEC_MAX_G * 2 + r) : 0.f;
    }
    __syncthreads();
    for (int jq = tid >> 7; jq < G; jq += 4) {
        float M = -INFINITY;
        for (int pp = 0; pp < n_ml; ++pp) M = fmaxf(M, ml[(pp * DEC_MAX_G + jq) * 2]);
        float acc = 0.f, l = 0.f;
        for (int p0 = 0; p0 < n_ml; p0 += 16) {
            float ov[16];
#pragma unroll
            for (int e = 0; e < 16; ++e)
                ov[e] = p0 + e < n_ml ? xwg_load(a.part_o + ((item0 + (size_t)(p0 + e) * a.Hkv) * DEC_MAX_G + jq) * 128 + hd) : 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                if (p0 + e < n_ml) {
                    float wgt = __builtin_amdgcn_exp2f(ml[((p0 + e) * DEC_MAX_G + jq) * 2] - M);
                    acc += wgt * ov[e];
                    l += wgt * ml[((p0 + e) * DEC_MAX_G + jq) * 2 + 1];
                }
            }
        }
        store_out(jq, acc / l);
    }
}

// Rounds of 256 keys a workgroup makes: the fewest (a power of two up to 16) that keep the grid at about two workgroups
// per CU - with many (trace, kv head) pairs, pieces of 256 keys make several rounds of short workgroups whose fixed
// costs (dispatch, lengths and page ids, the merge) add up (16 traces x 8 kv heads x 4096 keys: 67 us per layer).
int dec_attn_rounds(int B, int Hkv, int max_L) {
    int n = 1;
    while (n < 16 && (long)B * Hkv * (max_L / (DEC_PIECE * n) + 1) > 640) n *= 2;
    return n;
}

// a.n_iter from dec_attn_rounds; a.max_pieces: pieces of the longest trace, max_L / (DEC_PIECE * n_iter) + 1
hipError_t launch_dec_attn(const DecAttn &a, hipStream_t s) {
    if (a.B < 1 || a.B > DEC_MAX_ROWS || a.G < 1 || a.G > DEC_MAX_G || a.Hkv < 1 || a.B * a.Hkv > DEC_CTL_TILE - DEC_CTL_ATTN ||
        a.n_iter < 1 || a.max_pieces != a.max_L / (DEC_PIECE * a.n_iter) + 1 || a.max_pieces > DEC_ATTN_SMEM / (DEC_MAX_G * 2 * 4))
        return hipErrorInvalidValue;
    static std::atomic<uint32_t> attr_one{0}, attr_multi{0};
    const dim3 grid(a.max_pieces * a.Hkv, a.B);
    if (a.n_iter == 1) {
        if (hipError_t e = set_dynamic_lds_once(attr_one, reinterpret_cast<const void *>(dec_attn_kernel<false>), DEC_ATTN_SMEM); e != hipSuccess)
            return e;
        dec_attn_kernel<false><<<grid, DEC_ATTN_THREADS, DEC_ATTN_SMEM, s>>>(a);
    } else {
        if (hipError_t e = set_dynamic_lds_once(attr_multi, reinterpret_cast<const void *>(dec_attn_kernel<true>), DEC_ATTN_SMEM); e != hipSuccess)
            return e;
        dec_attn_kernel<true><<<grid, DEC_ATTN_THREADS, DEC_ATTN_SMEM, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace cs
