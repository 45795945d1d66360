// sage_build_tree: entropy-guided adaptive tree construction (Sec. 3.2: Eq. 10 depth, Eq. 11 width,
// Eq. 12 per-level width decay, recursive expansion with the depth-adaptive threshold, node cap).
//
// The result is defined by the order of the recursive expansion (depth-first, ranks ascending, global node
// cap), which is inherently serial over at most 64 nodes, so one wave64 per sequence walks it with wave-uniform
// control flow and keeps everything in registers:
//   lane r   holds candidate probability P~[r]; the candidates of an expansion are tested in one ballot;
//   lane l   holds theta_l = 0.1 l / D and W / l of level l (the divisions are done once, in parallel);
//   lane v   holds the fields of node v (parent, depth, rank, cumulative probability, ancestor mask);
//   lane s   holds the parked frame of stack depth s (node being expanded, candidates not yet tried).
// All real arithmetic is IEEE fp32 with round-to-nearest add/mul/div and no fused multiply-add (this file is
// compiled with contraction off and uses the explicit *_rn intrinsics), so the integer outcome is reproducible
// bit for bit.
#include "sage_internal.h"

namespace {

__device__ __forceinline__ float lane_read(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ int lane_read(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ uint64_t lane_read(uint64_t v, int lane) {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(v), lane);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(v >> 32), lane);
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

__global__ __launch_bounds__(64) void build_tree_kernel(
    const float* __restrict__ topk_renorm, const float* __restrict__ alpha, const int* __restrict__ topk_idx, int k,
    sage_tree_params prm, const int* __restrict__ d_max_seq, int* __restrict__ n_nodes, int* __restrict__ parent, int* __restrict__ depth,
    int* __restrict__ rank, uint64_t* __restrict__ anc_mask, float* __restrict__ cum_prob,
    int* __restrict__ node_token) {
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    const float pt = lane < k ? topk_renorm[static_cast<long>(b) * k + lane] : 0.0f;
    const int tok = (topk_idx && lane < k) ? topk_idx[static_cast<long>(b) * k + lane] : -1;
    const float a = alpha[b];

    // the maximum depth of Eq. 10 is per sequence when adaptive history tracking (Sec. 3.3) maintains one
    int d_max = prm.d_max;
    if (d_max_seq) d_max = min(max(d_max_seq[b], prm.d_min), SAGE_MAX_DEPTH);
    // Eq. 10 / Eq. 11, rounded half up
    const float Df = floorf(__fadd_rn(__fadd_rn((float)prm.d_min, __fmul_rn(a, (float)(d_max - prm.d_min))), 0.5f));
    float W = floorf(__fadd_rn(__fadd_rn((float)prm.w_min, __fmul_rn(__fsub_rn(1.0f, a), (float)(prm.w_max - prm.w_min))), 0.5f));
    if (W > (float)k) W = (float)k;
    // alpha is a confidence in [0,1]; anything else is clamped to the stack's capacity rather than trusted
    const int D = Df >= (float)SAGE_MAX_DEPTH ? SAGE_MAX_DEPTH : (Df >= 0.0f ? (int)Df : 0);

    // per-level constants, lane l <-> level l
    const float lvl = (float)(lane > 0 ? lane : 1);
    const float theta_l = __fdiv_rn(__fmul_rn(0.1f, lvl), Df);     // depth-adaptive threshold
    const float per_level_l = __fdiv_rn(W, lvl);                   // W / l of Eq. 12

    // node fields, lane v <-> node v (the root is node 0)
    int nd_parent = -1, nd_depth = 0, nd_rank = -1, nd_token = -1;
    float nd_cum = 1.0f;
    uint64_t nd_mask = 1ull;

    // parked frames, lane s <-> stack depth s
    int st_node = 0;
    uint64_t st_rest = 0;

    int n = 1;
    int sp = 0;
    int f_node = 0, f_depth = 0;                     // frame being expanded (uniform)
    float f_cum = 1.0f;
    uint64_t f_nmask = 1ull;
    uint64_t f_rest = 0;                             // candidates of this expansion not yet tried (bit r = rank r)
    if (D >= 1) {
        int w1 = (int)W;
        if (w1 > k) w1 = k;
        f_rest = __ballot(lane < w1 && __fmul_rn(1.0f, pt) > lane_read(theta_l, 1));
    }
    while (n < prm.n_max) {
        if (f_rest == 0) {                           // this expansion is exhausted: resume the parent's
            if (sp == 0) break;
            --sp;
            f_node = lane_read(st_node, sp);
            f_rest = lane_read(st_rest, sp);
            f_cum = lane_read(nd_cum, f_node);
            f_depth = lane_read(nd_depth, f_node);
            f_nmask = lane_read(nd_mask, f_node);
            continue;
        }
        const int r = __builtin_ctzll(f_rest);       // lowest untried rank that passes the threshold
        f_rest &= f_rest - 1;
        const float c = __fmul_rn(f_cum, lane_read(pt, r));
        const int v = n++;
        const int l = f_depth + 1;
        const uint64_t vm = f_nmask | (1ull << v);
        if (lane == v) {
            nd_parent = f_node; nd_depth = l; nd_rank = r; nd_cum = c; nd_mask = vm;
        }
        const int tok_r = lane_read(tok, r);
        if (lane == v) nd_token = tok_r;
        const int l2 = l + 1;                        // level that expanding v creates
        if (l2 <= D) {
            // Eq. 12 with the parent's cumulative path probability, at least one candidate
            const float w = floorf(__fmul_rn(lane_read(per_level_l, l2), __fadd_rn(0.5f, c)));
            int wl = (int)w;
            if (wl < 1) wl = 1;
            if (wl > k) wl = k;
            const uint64_t pass = __ballot(lane < wl && __fmul_rn(c, pt) > lane_read(theta_l, l2));
            if (lane == sp) { st_node = f_node; st_rest = f_rest; }
            ++sp;
            f_node = v; f_depth = l; f_cum = c; f_nmask = vm; f_rest = pass;
        }
    }

    const long base = static_cast<long>(b) * SAGE_MAX_NODES;
    if (lane < n) {
        parent[base + lane] = nd_parent;
        depth[base + lane] = nd_depth;
        rank[base + lane] = nd_rank;
        anc_mask[base + lane] = nd_mask;
        if (cum_prob) cum_prob[base + lane] = nd_cum;
        if (node_token) node_token[base + lane] = nd_token;
    }
    if (lane == 0) n_nodes[b] = n;
}

}  // namespace

extern "C" int sage_build_tree(const float* topk_renorm, const float* alpha, const int* topk_idx, int B, int k,
                               const sage_tree_params* params, const int* d_max_seq, int* n_nodes, int* parent,
                               int* depth, int* rank, uint64_t* anc_mask, float* cum_prob, int* node_token, void* stream) {
    if (!topk_renorm || !alpha || !params || !n_nodes || !parent || !depth || !rank || !anc_mask) return SAGE_INVALID_ARG;
    if (node_token && !topk_idx) return SAGE_INVALID_ARG;
    const sage_tree_params p = *params;
    if (B < 0 || k != p.k || k < 1 || k > SAGE_MAX_TOPK) return SAGE_INVALID_ARG;
    if (p.n_max < 1 || p.n_max > SAGE_MAX_NODES) return SAGE_INVALID_ARG;
    if (p.d_min < 1 || p.d_min > p.d_max || p.d_max > SAGE_MAX_DEPTH) return SAGE_INVALID_ARG;
    if (p.w_min < 1 || p.w_min > p.w_max || p.w_max > k) return SAGE_INVALID_ARG;
    if (B == 0) return SAGE_OK;
    hipLaunchKernelGGL(build_tree_kernel, dim3(B), dim3(64), 0, sage::as_stream(stream), topk_renorm, alpha, topk_idx,
                       k, p, d_max_seq, n_nodes, parent, depth, rank, anc_mask, cum_prob, node_token);
    return sage::launch_status();
}
