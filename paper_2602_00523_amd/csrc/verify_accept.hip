// sage_verify_accept: acceptance under greedy decoding (Sec. 2.2 "longest prefix matching the target's
// predictions"; Sec. 3.3 Phase 2 "all draft tokens along the path match"; Def. 4.1).
//
// One wave64 per sequence, lane i = tree node i.  The per-node match bits are gathered with one ballot;
// node i is accepted iff its ancestor-or-self mask has no unmatched bit, so the prefix-AND along every
// root-to-node path costs one 64-bit AND per lane.  The best node is a wave-wide max over
// (depth, lowest index); the path is read off the best node's mask.
#include "sage_internal.h"

namespace {

__global__ __launch_bounds__(64) void verify_accept_kernel(
    const int* __restrict__ token, const int* __restrict__ target_argmax, const int* __restrict__ parent,
    const int* __restrict__ depth, const uint64_t* __restrict__ anc_mask, const int* __restrict__ n_nodes,
    int path_cap, int* __restrict__ accept_len, int* __restrict__ best_node, int* __restrict__ path_nodes,
    int* __restrict__ out_tokens) {
    __shared__ int slot_node[SAGE_MAX_NODES];
    __shared__ int slot_token[SAGE_MAX_NODES];
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

    bool match = false;
    if (valid) match = (i == 0) || (par >= 0 && par < n && tok == target_argmax[base + par]);
    const uint64_t matched = __ballot(match);
    const bool accepted = valid && ((am & ~matched) == 0) && ((am >> i) & 1);

    // max over (depth, then lowest index); the root (depth 0) is always accepted
    int key = accepted ? (dep * SAGE_MAX_NODES + (SAGE_MAX_NODES - 1 - i)) : -1;
    for (int off = 32; off > 0; off >>= 1) key = max(key, __shfl_xor(key, off));
    const int best = SAGE_MAX_NODES - 1 - (key % SAGE_MAX_NODES);
    const int tau = key / SAGE_MAX_NODES;
    const uint64_t path_mask = __shfl(am, best);

    slot_node[i] = -1;
    slot_token[i] = -1;
    __syncthreads();
    if (valid && ((path_mask >> i) & 1) && dep >= 0 && dep < SAGE_MAX_NODES) {
        slot_node[dep] = i;
        if (dep >= 1) slot_token[dep - 1] = tok;     // draft token of the path node at depth dep
    }
    if (i == best && tau < SAGE_MAX_NODES) slot_token[tau] = tgt;   // bonus token: the target's choice at best
    __syncthreads();

    const long obase = static_cast<long>(b) * path_cap;
    for (int j = i; j < path_cap; j += SAGE_MAX_NODES) {
        path_nodes[obase + j] = (j < SAGE_MAX_NODES && j <= tau) ? slot_node[j] : -1;
        out_tokens[obase + j] = (j < SAGE_MAX_NODES && j <= tau) ? slot_token[j] : -1;
    }
    if (i == 0) {
        accept_len[b] = tau;
        best_node[b] = best;
    }
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
