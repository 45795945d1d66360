// The tree rule of sage_build_tree as a wave-level device function, shared by the kernel that runs it on its own
// (build_tree.hip) and by the kernel that runs it right after the top-k second pass (fused_steps.hip).
//
// entropy-guided adaptive tree construction (Sec. 3.2: Eq. 10 depth, Eq. 11 width,
// Eq. 12 per-level width decay, recursive expansion with the depth-adaptive threshold, node cap).
//
// The result is defined by the order of the recursive expansion (depth-first, ranks ascending, global node
// cap), which is inherently serial over at most 64 nodes, so one wave64 per sequence walks it with wave-uniform
// control flow and keeps everything in registers:
//   lane r   holds candidate probability P~[r]; the candidates of an expansion are tested in one ballot;
//   lane l   holds theta_l = 0.1 l / D and W / l of level l (the divisions are done once, in parallel);
//   lane v   holds the fields of node v (parent, depth, rank, cumulative probability, ancestor mask);
//   lane s   holds the parked frame of stack depth s (node being expanded, candidates not yet tried).
// All real arithmetic is IEEE fp32 with round-to-nearest add/mul/div and no fused multiply-add (every operation goes
// through a helper whose body is compiled with contraction off, whatever the including file's setting), so the
// integer outcome is reproducible bit for bit.
#pragma once
#include "sage_internal.h"

namespace sage {
namespace tree {

// Separately rounded fp32 operations: the pragma keeps the compiler from fusing a product into a following sum.
__device__ __forceinline__ float add_rn(float a, float b) {
#pragma clang fp contract(off)
    return a + b;
}
__device__ __forceinline__ float sub_rn(float a, float b) {
#pragma clang fp contract(off)
    return a - b;
}
__device__ __forceinline__ float mul_rn(float a, float b) {
#pragma clang fp contract(off)
    return a * b;
}
__device__ __forceinline__ float div_rn(float a, float b) {
#pragma clang fp contract(off)
    return a / b;
}

__device__ __forceinline__ float lane_read(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ int lane_read(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ uint64_t lane_read(uint64_t v, int lane) {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(v), lane);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(v >> 32), lane);
    return (static_cast<uint64_t>(hi) << 32) | lo;
}


// One wave64 builds the tree of sequence b.  pt = renormalised probability of candidate `lane` (0 past k), tok = its
// token id (-1 when none are given), a = the sequence's confidence (wave-uniform).
__device__ __forceinline__ void build_tree_wave(int b, int lane, float pt, int tok, float a, int k, const sage_tree_params& prm,
                                                const int* __restrict__ d_max_seq, int* __restrict__ n_nodes,
                                                int* __restrict__ parent, int* __restrict__ depth, int* __restrict__ rank,
                                                uint64_t* __restrict__ anc_mask, float* __restrict__ cum_prob,
                                                int* __restrict__ node_token) {

    // The confidence and the depth limit are the same in every lane, but arrive through per-lane loads or lane
    // exchanges; said explicitly, everything that steers the walk below (depth, width, node count, stack pointer, the
    // candidate masks) lives in scalar registers and the walk branches on scalar conditions instead of masking lanes.
    a = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a)));
    // the maximum depth of Eq. 10 is per sequence when adaptive history tracking (Sec. 3.3) maintains one
    int d_max = prm.d_max;
    if (d_max_seq) d_max = min(max(__builtin_amdgcn_readfirstlane(d_max_seq[b]), prm.d_min), SAGE_MAX_DEPTH);
    // Eq. 10 / Eq. 11, rounded half up
    const float Df = floorf(add_rn(add_rn((float)prm.d_min, mul_rn(a, (float)(d_max - prm.d_min))), 0.5f));
    float W = floorf(add_rn(add_rn((float)prm.w_min, mul_rn(sub_rn(1.0f, a), (float)(prm.w_max - prm.w_min))), 0.5f));
    if (W > (float)k) W = (float)k;
    // alpha is a confidence in [0,1]; anything else is clamped to the stack's capacity rather than trusted
    const int D = Df >= (float)SAGE_MAX_DEPTH ? SAGE_MAX_DEPTH : (Df >= 0.0f ? (int)Df : 0);

    // per-level constants, lane l <-> level l
    const float lvl = (float)(lane > 0 ? lane : 1);
    const float theta_l = div_rn(mul_rn(0.1f, lvl), Df);     // depth-adaptive threshold
    const float per_level_l = div_rn(W, lvl);                   // W / l of Eq. 12

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
        f_rest = __ballot(lane < w1 && mul_rn(1.0f, pt) > lane_read(theta_l, 1));
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
        const float c = mul_rn(f_cum, lane_read(pt, r));
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
            const float w = floorf(mul_rn(lane_read(per_level_l, l2), add_rn(0.5f, c)));
            int wl = (int)w;
            if (wl < 1) wl = 1;
            if (wl > k) wl = k;
            const uint64_t pass = __ballot(lane < wl && mul_rn(c, pt) > lane_read(theta_l, l2));
            if (pass != 0) {                         // v has candidates: park this frame and expand v (a node without any
                if (lane == sp) { st_node = f_node; st_rest = f_rest; }   // would be left again at once: same tree)
                ++sp;
                f_node = v; f_depth = l; f_cum = c; f_nmask = vm; f_rest = pass;
            }
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

}  // namespace tree
}  // namespace sage
