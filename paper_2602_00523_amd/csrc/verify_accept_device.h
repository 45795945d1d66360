// The acceptance rule of sage_verify_accept as a wave-level device function: the prefix-AND of the per-node match bits
// along every root-to-node path, deepest fully matched node wins (Sec. 2.2; Sec. 3.3 Phase 2; Def. 4.1), shared by the
// kernel that runs it on its own (verify_accept.hip) and by the kernel that first finishes the target's argmax
// (fused_steps.hip).
//
// One wave64 per sequence, lane i = tree node i.  The per-node match bits are gathered with one ballot;
// node i is accepted iff its ancestor-or-self mask has no unmatched bit, so the prefix-AND along every
// root-to-node path costs one 64-bit AND per lane.  The best node is a wave-wide max over
// (depth, lowest index); the path is read off the best node's mask.
#pragma once
#include "sage_internal.h"

namespace sage {
namespace accept {

// LDS of one accepting wave: path slots by depth.
struct AcceptShared {
    int slot_node[SAGE_MAX_NODES];
    int slot_token[SAGE_MAX_NODES];
};

// Orders this wave's LDS writes before its later LDS reads (one wave: no workgroup barrier involved).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Lane i holds node i's fields (par, tok, dep, am; anything for i >= n) and tgt = the target's greedy token at node i;
// tgt_of_parent = the target's greedy token at node i's parent (anything when the parent is out of range).
// Returns tau (wave-uniform); the path nodes stay in sh.slot_node[0..tau].
__device__ __forceinline__ int verify_accept_wave(int b, int i, int n, int par, int tok, int dep, uint64_t am, int tgt,
                                                   int tgt_of_parent, int path_cap, AcceptShared& sh,
                                                   int* __restrict__ accept_len, int* __restrict__ best_node,
                                                   int* __restrict__ path_nodes, int* __restrict__ out_tokens) {
    const bool valid = i < n;
    bool match = false;
    if (valid) match = (i == 0) || (par >= 0 && par < n && tok == tgt_of_parent);
    const uint64_t matched = __ballot(match);
    const bool accepted = valid && ((am & ~matched) == 0) && ((am >> i) & 1);

    // max over (depth, then lowest index); the root (depth 0) is always accepted
    const int own_key = accepted ? (dep * SAGE_MAX_NODES + (SAGE_MAX_NODES - 1 - i)) : -1;
    const int key = static_cast<int>(sage::wave_max_u32(static_cast<uint32_t>(own_key + 1))) - 1;   // the root makes it >= 0
    const int best = __builtin_amdgcn_readfirstlane(SAGE_MAX_NODES - 1 - (key % SAGE_MAX_NODES));
    const int tau = key / SAGE_MAX_NODES;
    const uint64_t path_mask = sage::lane_value(am, best);

    sh.slot_node[i] = -1;
    sh.slot_token[i] = -1;
    wave_lds_sync();
    if (valid && ((path_mask >> i) & 1) && dep >= 0 && dep < SAGE_MAX_NODES) {
        sh.slot_node[dep] = i;
        if (dep >= 1) sh.slot_token[dep - 1] = tok;  // draft token of the path node at depth dep
    }
    wave_lds_sync();
    if (i == best && tau < SAGE_MAX_NODES) sh.slot_token[tau] = tgt;   // bonus token: the target's choice at best
    wave_lds_sync();

    const long obase = static_cast<long>(b) * path_cap;
    for (int j = i; j < path_cap; j += SAGE_MAX_NODES) {
        path_nodes[obase + j] = (j < SAGE_MAX_NODES && j <= tau) ? sh.slot_node[j] : -1;
        out_tokens[obase + j] = (j < SAGE_MAX_NODES && j <= tau) ? sh.slot_token[j] : -1;
    }
    if (i == 0) {
        accept_len[b] = tau;
        best_node[b] = best;
    }
    return tau;
}

}  // namespace accept
}  // namespace sage
