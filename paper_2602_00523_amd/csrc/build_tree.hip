// sage_build_tree: entropy-guided adaptive tree construction (Sec. 3.2: Eq. 10 depth, Eq. 11 width,
// Eq. 12 per-level width decay, recursive expansion with the depth-adaptive threshold, node cap).
//
// The result is defined by the order of the recursive expansion (depth-first, ranks ascending, global node
// cap), which is inherently serial over at most 64 nodes, so one lane per sequence walks an explicit stack in
// LDS while the rest of its wave only helps with the coalesced write-out.  All real arithmetic is IEEE fp32
// with round-to-nearest add/mul/div and no fused multiply-add (this file is compiled with contraction off
// and uses the explicit *_rn intrinsics), so the integer outcome is reproducible bit for bit.
#include "sage_internal.h"

namespace {

struct Frame {
    int node;     // node being expanded
    int next_r;   // next candidate rank to try
    int width;    // W_l of this expansion
    float theta;  // theta_l of the level being created
};

__global__ __launch_bounds__(64) void build_tree_kernel(
    const float* __restrict__ topk_renorm, const float* __restrict__ alpha, const int* __restrict__ topk_idx, int k,
    sage_tree_params prm, int* __restrict__ n_nodes, int* __restrict__ parent, int* __restrict__ depth,
    int* __restrict__ rank, uint64_t* __restrict__ anc_mask, float* __restrict__ cum_prob,
    int* __restrict__ node_token) {
    __shared__ float s_pt[SAGE_MAX_TOPK];
    __shared__ int s_parent[SAGE_MAX_NODES], s_depth[SAGE_MAX_NODES], s_rank[SAGE_MAX_NODES];
    __shared__ float s_cum[SAGE_MAX_NODES];
    __shared__ uint64_t s_mask[SAGE_MAX_NODES];
    __shared__ Frame s_stack[SAGE_MAX_DEPTH + 1];
    __shared__ int s_n;

    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    if (lane < k) s_pt[lane] = topk_renorm[static_cast<long>(b) * k + lane];
    __syncthreads();

    if (lane == 0) {
        const float a = alpha[b];
        // Eq. 10 / Eq. 11, rounded half up
        const float Df = floorf(__fadd_rn(__fadd_rn((float)prm.d_min, __fmul_rn(a, (float)(prm.d_max - prm.d_min))), 0.5f));
        float W = floorf(__fadd_rn(
            __fadd_rn((float)prm.w_min, __fmul_rn(__fsub_rn(1.0f, a), (float)(prm.w_max - prm.w_min))), 0.5f));
        if (W > (float)k) W = (float)k;
        // alpha is a confidence in [0,1]; anything else is clamped to the stack's capacity rather than trusted
        const int D = Df >= (float)SAGE_MAX_DEPTH ? SAGE_MAX_DEPTH : (Df >= 0.0f ? (int)Df : 0);

        s_parent[0] = -1; s_depth[0] = 0; s_rank[0] = -1; s_cum[0] = 1.0f; s_mask[0] = 1ull;
        int n = 1;
        int sp = 0;
        if (D >= 1) {
            int w1 = (int)W;
            if (w1 > k) w1 = k;
            s_stack[0] = Frame{0, 0, w1, __fdiv_rn(__fmul_rn(0.1f, 1.0f), Df)};
            sp = 1;
        }
        while (sp > 0 && n < prm.n_max) {
            Frame& f = s_stack[sp - 1];
            if (f.next_r >= f.width) { --sp; continue; }
            const int r = f.next_r++;
            const int u = f.node;
            const float c = __fmul_rn(s_cum[u], s_pt[r]);
            if (c > f.theta) {
                const int v = n++;
                const int l = s_depth[u] + 1;
                s_parent[v] = u; s_depth[v] = l; s_rank[v] = r; s_cum[v] = c;
                s_mask[v] = s_mask[u] | (1ull << v);
                const int l2 = l + 1;                       // level that expanding v would create
                if (l2 <= D) {
                    // Eq. 12 with the parent's cumulative path probability, at least one candidate
                    const float w = floorf(__fmul_rn(__fdiv_rn(W, (float)l2), __fadd_rn(0.5f, c)));
                    int wl = (int)w;
                    if (wl < 1) wl = 1;
                    if (wl > k) wl = k;
                    s_stack[sp++] = Frame{v, 0, wl, __fdiv_rn(__fmul_rn(0.1f, (float)l2), Df)};
                }
            }
        }
        s_n = n;
    }
    __syncthreads();

    const int n = s_n;
    const long base = static_cast<long>(b) * SAGE_MAX_NODES;
    if (lane < n) {
        parent[base + lane] = s_parent[lane];
        depth[base + lane] = s_depth[lane];
        rank[base + lane] = s_rank[lane];
        anc_mask[base + lane] = s_mask[lane];
        if (cum_prob) cum_prob[base + lane] = s_cum[lane];
        if (node_token) node_token[base + lane] = lane == 0 ? -1 : topk_idx[static_cast<long>(b) * k + s_rank[lane]];
    }
    if (lane == 0) n_nodes[b] = n;
}

}  // namespace

extern "C" int sage_build_tree(const float* topk_renorm, const float* alpha, const int* topk_idx, int B, int k,
                               const sage_tree_params* params, int* n_nodes, int* parent, int* depth, int* rank,
                               uint64_t* anc_mask, float* cum_prob, int* node_token, void* stream) {
    if (!topk_renorm || !alpha || !params || !n_nodes || !parent || !depth || !rank || !anc_mask) return SAGE_INVALID_ARG;
    if (node_token && !topk_idx) return SAGE_INVALID_ARG;
    const sage_tree_params p = *params;
    if (B < 0 || k != p.k || k < 1 || k > SAGE_MAX_TOPK) return SAGE_INVALID_ARG;
    if (p.n_max < 1 || p.n_max > SAGE_MAX_NODES) return SAGE_INVALID_ARG;
    if (p.d_min < 1 || p.d_min > p.d_max || p.d_max > SAGE_MAX_DEPTH) return SAGE_INVALID_ARG;
    if (p.w_min < 1 || p.w_min > p.w_max || p.w_max > k) return SAGE_INVALID_ARG;
    if (B == 0) return SAGE_OK;
    hipLaunchKernelGGL(build_tree_kernel, dim3(B), dim3(64), 0, sage::as_stream(stream), topk_renorm, alpha, topk_idx,
                       k, p, n_nodes, parent, depth, rank, anc_mask, cum_prob, node_token);
    return sage::launch_status();
}
