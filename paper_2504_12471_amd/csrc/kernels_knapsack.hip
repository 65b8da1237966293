// Bi-level knapsack selection on the GPU: DPSearching (Alg. 2) for the p_f stage and the p_o
// stage of every knapsack, then the merge of KnapsackScheduling (Alg. 1).
//
// One workgroup runs one (knapsack, stage) DP.  Items are processed one after another (the
// recurrence is sequential in i); the capacities w = 0..C of one item are spread over the
// threads.  Only two rows of the value table are kept (fp64, in the workspace); what the
// backtracking phase needs - whether T[i][w] differs from T[i-1][w] - is recorded per cell as
// one byte.  Each cell is one fp64 add and one compare, in the order the algorithm writes
// them, so the table equals a sequential CPU evaluation bit for bit.
#include "d2ft_common.h"

namespace d2ft {


__global__ __launch_bounds__(256) void knapsack_dp_kernel(KnapsackArgs a) {
    const int prob = blockIdx.x;           // knapsack * 2 + stage
    const int k = prob >> 1, stage = prob & 1;
    const int n = a.n_items;
    const int c = stage == 0 ? a.cost_fwd[k] + a.cost_bwd[k] : a.cost_fwd[k];   // W_b or W_f of Alg. 1
    const int C = stage == 0 ? a.cap_full[k] : a.cap_fwd[k];
    const double* score = (stage == 0 ? a.score_full : a.score_fwd) + (long)k * n;
    double* prev = a.rows + (long)prob * 2 * a.stride;
    double* cur = prev + a.stride;
    uint8_t* changed = a.changed + (long)prob * n * a.stride;
    uint8_t* sel = a.selected + (long)prob * n;

    for (int w = threadIdx.x; w <= C; w += blockDim.x) prev[w] = 0.0;
    for (int i = threadIdx.x; i < n; i += blockDim.x) sel[i] = 0;
    __syncthreads();

    // phase 1: fill
    for (int i = 1; i <= n; ++i) {
        const double s = score[i - 1];
        uint8_t* ch = changed + (long)(i - 1) * a.stride;
        for (int w = threadIdx.x; w <= C; w += blockDim.x) {
            const double keep = prev[w];
            double v = keep;
            if (w >= c) {
                const double take = __dadd_rn(prev[w - c], s);
                v = take > keep ? take : keep;
            }
            cur[w] = v;
            ch[w] = (v != keep) ? 1 : 0;
        }
        __syncthreads();
        double* t = prev;
        prev = cur;
        cur = t;
    }

    // phase 2: backtracking
    if (threadIdx.x == 0) {
        int i = n, w = C;
        while (i > 0 && w > 0) {
            if (changed[(long)(i - 1) * a.stride + w]) {
                sel[i - 1] = 1;
                w -= c;
            }
            i -= 1;
        }
    }
}

// merge of Alg. 1: both or only p_f -> 1, only p_o -> 2, neither -> 3
__global__ void knapsack_merge_kernel(const uint8_t* __restrict__ selected, uint8_t* __restrict__ ops, int n_knapsacks,
                                      int n_items) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)n_knapsacks * n_items) return;
    const int k = (int)(idx / n_items), i = (int)(idx % n_items);
    const uint8_t pf = selected[((long)k * 2 + 0) * n_items + i];
    const uint8_t po = selected[((long)k * 2 + 1) * n_items + i];
    ops[idx] = pf ? D2FT_OP_FULL : (po ? D2FT_OP_FWD : D2FT_OP_SKIP);
}

hipError_t launch_knapsack(const KnapsackArgs& a, uint8_t* ops_dev, hipStream_t s) {
    hipLaunchKernelGGL(knapsack_dp_kernel, dim3(a.n_knapsacks * 2), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long total = (long)a.n_knapsacks * a.n_items;
    hipLaunchKernelGGL(knapsack_merge_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a.selected,
                       ops_dev, a.n_knapsacks, a.n_items);
    return hipGetLastError();
}

}  // namespace d2ft
