// sage_verify_accept as a launch of its own: one wave64 per sequence runs the acceptance rule
// (verify_accept_device.h) on the target's greedy tokens that sage_entropy_topk left in memory.
#include "verify_accept_device.h"

namespace {

__global__ __launch_bounds__(64) void verify_accept_kernel(
    const int* __restrict__ token, const int* __restrict__ target_argmax, const int* __restrict__ parent,
    const int* __restrict__ depth, const uint64_t* __restrict__ anc_mask, const int* __restrict__ n_nodes,
    int path_cap, int* __restrict__ accept_len, int* __restrict__ best_node, int* __restrict__ path_nodes,
    int* __restrict__ out_tokens) {
    __shared__ sage::accept::AcceptShared sh;
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    const long base = static_cast<long>(b) * SAGE_MAX_NODES;
    int n = n_nodes[b];
    n = n < 1 ? 1 : (n > SAGE_MAX_NODES ? SAGE_MAX_NODES : n);
    const bool valid = i < n;
    const int par = valid ? parent[base + i] : -1;
    const int tok = valid ? token[base + i] : 0;
    const int tgt = valid ? target_argmax[base + i] : 0;
    const int dep = valid ? depth[base + i] : 0;
    const uint64_t am = valid ? anc_mask[base + i] : 0;
    const int tgt_par = (valid && par >= 0 && par < n) ? target_argmax[base + par] : 0;
    sage::accept::verify_accept_wave(b, i, n, par, tok, dep, am, tgt, tgt_par, path_cap, sh, accept_len, best_node, path_nodes,
                                     out_tokens);
}

}  // namespace

extern "C" int sage_verify_accept(const int* token, const int* target_argmax, const int* parent, const int* depth,
                                  const uint64_t* anc_mask, const int* n_nodes, int B, int path_cap,
                                  int* accept_len, int* best_node, int* path_nodes, int* out_tokens, void* stream) {
    if (!token || !target_argmax || !parent || !depth || !anc_mask || !n_nodes || !accept_len || !best_node ||
        !path_nodes || !out_tokens)
        return SAGE_INVALID_ARG;
    if (B < 0 || path_cap < 1) return SAGE_INVALID_ARG;
    if (B == 0) return SAGE_OK;
    hipLaunchKernelGGL(verify_accept_kernel, dim3(B), dim3(64), 0, sage::as_stream(stream), token, target_argmax,
                       parent, depth, anc_mask, n_nodes, path_cap, accept_len, best_node, path_nodes, out_tokens);
    return sage::launch_status();
}
