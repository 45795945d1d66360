// sage_build_tree as a launch of its own: one wave64 per sequence runs the tree rule (build_tree_device.h) on the
// renormalised top-k probabilities and the confidence that sage_entropy_topk left in memory.
#include "build_tree_device.h"

namespace {

__global__ __launch_bounds__(64) void build_tree_kernel(
    const float* __restrict__ topk_renorm, const float* __restrict__ alpha, const int* __restrict__ topk_idx, int k,
    sage_tree_params prm, const int* __restrict__ d_max_seq, int* __restrict__ n_nodes, int* __restrict__ parent, int* __restrict__ depth,
    int* __restrict__ rank, uint64_t* __restrict__ anc_mask, float* __restrict__ cum_prob,
    int* __restrict__ node_token) {
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    const float pt = lane < k ? topk_renorm[static_cast<long>(b) * k + lane] : 0.0f;
    const int tok = (topk_idx && lane < k) ? topk_idx[static_cast<long>(b) * k + lane] : -1;
    sage::tree::build_tree_wave(b, lane, pt, tok, alpha[b], k, prm, d_max_seq, n_nodes, parent, depth, rank, anc_mask, cum_prob,
                                node_token);
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
