// Planning of the next tree for one sequence as a workgroup-level device function: the second pass of the draft row's
// top-k (Eq. 7-9) followed, in wave 0, by the tree rule (Sec. 3.2, Eq. 10-12).  Shared by the kernel that runs it as a
// launch of its own (fused_steps.hip) and by the attention launch that carries it along (tree_attention_bf16.hip), so
// that both produce the same bits.
#pragma once
#include "build_tree_device.h"
#include "topk_device.h"

namespace sage {

// Everything sage_build_tree_from_slices passes to its kernel.
struct PlanArgs {
    int k, nunits;
    const topk::UnitStats* stats;
    const uint64_t* keys;
    float* entropy; int* topk_idx; float* topk_prob; float* topk_renorm; float* topk_entropy; float* alpha;
    sage_tree_params prm;
    const int* d_max_seq;
    int* n_nodes; int* parent; int* depth; int* rank; uint64_t* anc_mask; float* cum_prob; int* node_token;
};

// Called by all WG_THREADS threads of a workgroup; sh as for topk::merge_row.
template <int OWN, int WG_THREADS, class Shared>
__device__ __forceinline__ void plan_sequence(int b, const PlanArgs& pl, Shared& sh) {
    topk::MergedRow r;
    if (!topk::merge_row<OWN, WG_THREADS>(b, pl.k, pl.nunits, pl.stats, pl.keys, sh, pl.entropy, pl.topk_idx, pl.topk_prob,
                                          pl.topk_renorm, pl.topk_entropy, pl.alpha, r))
        return;
    const int lane = threadIdx.x;                    // wave 0
    tree::build_tree_wave(b, lane, lane < pl.k ? r.q : 0.0f, lane < pl.k ? r.idx : -1, r.alpha, pl.k, pl.prm, pl.d_max_seq,
                          pl.n_nodes, pl.parent, pl.depth, pl.rank, pl.anc_mask, pl.cum_prob, pl.node_token);
}

}  // namespace sage
