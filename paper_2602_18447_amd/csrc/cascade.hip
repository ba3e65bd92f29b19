// Two-tier cascade over the drafted steps of a batch of requests (Section 4.2, Eq. 4; Algorithm 1, Stage 2; candidate
// trees: Section 4.3, Eq. 5):
// selection and compaction of the traces the large model has to see, and the walk over each request's steps
// once both models have spoken.  The two forward passes themselves are confspec_verify calls.
#include "kernels.h"
#include <math.h>

namespace cs {

// Which traces can the walk of Stage 2 escalate?  A candidate is looked at only if the step it continues was chosen,
// and it goes to the large model if its small-model confidence is below gamma.  Before the large model has run,
// "chosen" is unknown for the escalated steps, but a confident rejection by the small model is final: nothing that
// continues such a step is ever reached.  keep[b] is the small model's gate bit (confidence >= gamma).
// parent (may be null): the trace that b continues, -1 for a first-layer candidate; null = every request is a chain.
// One thread per request walks its traces in index order (parents come first); open_flag is per-trace scratch.
// Then an exclusive scan over the traces compacts the selected ones.
__device__ __forceinline__ int parent_of(const int32_t *parent, int b, int lo) {
    int p = parent ? parent[b] : (b > lo ? b - 1 : -1);
    return (p >= lo && p < b) ? p : -1;          // anything else counts as "continues the context itself"
}

__global__ __launch_bounds__(256) void cascade_select_kernel(const uint8_t *__restrict__ keep, const int32_t *__restrict__ verdict_d,
                                                              const int32_t *__restrict__ req_start, const int32_t *__restrict__ parent,
                                                              int R, int B, const int32_t *__restrict__ cu,
                                                              const int32_t *__restrict__ plens, int T, uint8_t *open_flag,
                                                              uint8_t *__restrict__ target_ran,
                                                              int32_t *__restrict__ pos_of, int32_t *__restrict__ sel_idx,
                                                              int32_t *__restrict__ cu_out, int32_t *__restrict__ plens_out,
                                                              int32_t *__restrict__ n_out) {
    __shared__ int s_cnt[257], s_tok[257];
    __shared__ int carry[2];
    int tid = threadIdx.x;
    for (int r = tid; r < R; r += 256) {
        int lo = min(max(req_start[r], 0), B), hi = min(max(req_start[r + 1], lo), B);
        for (int b = lo; b < hi; ++b) {
            int p = parent_of(parent, b, lo);
            bool open = p < 0 ? true : (open_flag[p] != 0 && !(keep[p] != 0 && verdict_d[p] != 0));
            open_flag[b] = open ? 1 : 0;
            target_ran[b] = (open && keep[b] == 0) ? 1 : 0;
        }
    }
    if (tid == 0) carry[0] = carry[1] = 0;
    __syncthreads();            // also orders the target_ran writes of this block before the reads below
    for (int base = 0; base < B; base += 256) {
        int b = base + tid;
        int flag = 0, S = 0;
        if (b < B) {
            flag = target_ran[b];
            int c0 = min(max(cu[b], 0), T), c1 = min(max(cu[b + 1], c0), T);
            S = c1 - c0;
        }
        s_cnt[tid + 1] = flag;
        s_tok[tid + 1] = flag ? S : 0;
        __syncthreads();
        if (tid == 0) {
            s_cnt[0] = carry[0];
            s_tok[0] = carry[1];
            int n = min(256, B - base);
            for (int i = 1; i <= n; ++i) { s_cnt[i] += s_cnt[i - 1]; s_tok[i] += s_tok[i - 1]; }
            carry[0] = s_cnt[n];
            carry[1] = s_tok[n];
        }
        __syncthreads();
        if (b < B) {
            if (flag) {
                int p = s_cnt[tid];
                pos_of[b] = p;
                sel_idx[p] = b;
                cu_out[p] = s_tok[tid];
                plens_out[p] = plens[b];
            } else {
                pos_of[b] = -1;
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        cu_out[carry[0]] = carry[1];
        n_out[0] = carry[0];
        n_out[1] = carry[1];
    }
}

// Suffix ids and block-table rows of the selected traces, in compact order: one workgroup per trace.
__global__ __launch_bounds__(256) void cascade_gather_kernel(const int32_t *__restrict__ pos_of, const int32_t *__restrict__ cu,
                                                              const int32_t *__restrict__ cu_out,
                                                              const int32_t *__restrict__ ids, int32_t *__restrict__ ids_out,
                                                              const int32_t *__restrict__ table, int32_t *__restrict__ table_out,
                                                              int max_blocks, int T) {
    int b = blockIdx.x, p = pos_of[b];
    if (p < 0) return;
    int c0 = min(max(cu[b], 0), T), c1 = min(max(cu[b + 1], c0), T);
    int o0 = cu_out[p];
    for (int i = threadIdx.x; i < c1 - c0; i += blockDim.x)
        if (o0 + i < T) ids_out[o0 + i] = ids[c0 + i];
    for (int i = threadIdx.x; i < max_blocks; i += blockDim.x) table_out[(size_t)p * max_blocks + i] = table[(size_t)b * max_blocks + i];
}

// The walk of Stage 2 per request, with both models' decisions known (a chain: accept until the first rejection; a
// tree: among the accepted candidates that continue the chosen step take the most confident one, Eq. 5); and the
// large model's results scattered back to the traces of the full batch.
__global__ __launch_bounds__(256) void cascade_merge_kernel(const uint8_t *__restrict__ keep, const int32_t *__restrict__ verdict_d,
                                                             const float *__restrict__ conf_d, const int32_t *__restrict__ pos_of,
                                                             const float *__restrict__ conf_t_c, const int32_t *__restrict__ verdict_t_c,
                                                             const int32_t *__restrict__ req_start, const int32_t *__restrict__ parent,
                                                             int R, int B, int n_target,
                                                             float *__restrict__ conf_t, int32_t *__restrict__ verdict_t,
                                                             int32_t *__restrict__ decision, uint8_t *__restrict__ escalated,
                                                             uint8_t *__restrict__ selected, float *__restrict__ conf_used,
                                                             int32_t *__restrict__ accepted) {
    int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < B) {
        int p = pos_of[gid];
        bool has = p >= 0 && p < n_target;
        conf_t[gid] = has ? conf_t_c[p] : NAN;
        verdict_t[gid] = has ? verdict_t_c[p] : -1;
    }
    if (gid < R) {
        int lo = min(max(req_start[gid], 0), B), hi = min(max(req_start[gid + 1], lo), B);
        for (int b = lo; b < hi; ++b) {
            decision[b] = -1;
            escalated[b] = 0;
            if (selected) selected[b] = 0;
            if (conf_used) conf_used[b] = NAN;
        }
        int m = 0, cur = -1;
        for (int depth = 0; depth < hi - lo; ++depth) {          // a chosen node has a larger index than its parent
            int best = -1;
            float best_p = 0.f;
            for (int b = max(cur + 1, lo); b < hi; ++b) {
                if (parent_of(parent, b, lo) != cur) continue;
                int v;
                float pu;
                if (keep[b]) {
                    v = verdict_d[b];
                    pu = conf_d[b];
                } else {
                    int p = pos_of[b];
                    bool has = p >= 0 && p < n_target;           // selected by construction
                    v = has ? verdict_t_c[p] : -1;
                    pu = has ? conf_t_c[p] : NAN;
                    escalated[b] = 1;
                }
                decision[b] = v;
                if (conf_used) conf_used[b] = pu;
                if (v == 0 && (best < 0 || pu > best_p)) {
                    best = b;
                    best_p = pu;
                }
            }
            if (best < 0) break;
            if (selected) selected[best] = 1;
            ++m;
            cur = best;
        }
        accepted[gid] = m;
    }
}

hipError_t launch_cascade_select(const uint8_t *keep, const int32_t *verdict_d, const int32_t *req_start, const int32_t *parent,
                                 int R, int B, const int32_t *cu, const int32_t *plens, int T, uint8_t *open_flag,
                                 uint8_t *target_ran, int32_t *pos_of, int32_t *sel_idx, int32_t *cu_out, int32_t *plens_out,
                                 int32_t *n_out, hipStream_t s) {
    cascade_select_kernel<<<1, 256, 0, s>>>(keep, verdict_d, req_start, parent, R, B, cu, plens, T, open_flag, target_ran,
                                            pos_of, sel_idx, cu_out, plens_out, n_out);
    return hipGetLastError();
}

hipError_t launch_cascade_gather(const int32_t *pos_of, const int32_t *cu, const int32_t *cu_out, const int32_t *ids,
                                 int32_t *ids_out, const int32_t *table, int32_t *table_out, int max_blocks, int B, int T,
                                 hipStream_t s) {
    cascade_gather_kernel<<<B, 256, 0, s>>>(pos_of, cu, cu_out, ids, ids_out, table, table_out, max_blocks, T);
    return hipGetLastError();
}

hipError_t launch_cascade_merge(const uint8_t *keep, const int32_t *verdict_d, const float *conf_d, const int32_t *pos_of,
                                const float *conf_t_c, const int32_t *verdict_t_c, const int32_t *req_start,
                                const int32_t *parent, int R, int B, int n_target, float *conf_t, int32_t *verdict_t,
                                int32_t *decision, uint8_t *escalated, uint8_t *selected, float *conf_used, int32_t *accepted,
                                hipStream_t s) {
    int n = B > R ? B : R;
    cascade_merge_kernel<<<(n + 255) / 256, 256, 0, s>>>(keep, verdict_d, conf_d, pos_of, conf_t_c, verdict_t_c, req_start,
                                                          parent, R, B, n_target, conf_t, verdict_t, decision, escalated,
                                                          selected, conf_used, accepted);
    return hipGetLastError();
}

}  // namespace cs
