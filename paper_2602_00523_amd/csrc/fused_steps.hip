// The second pass of sage_entropy_topk folded into the launch that consumes its result.  A step of the method is a
// chain of small dependent launches (Alg. 1: plan the tree from the draft distribution, verify, accept), each of which
// costs a few microseconds of launch and memory latency however little it computes; these entry points remove two of
// them without changing a single result:
//   sage_build_tree_from_slices     = second pass over the draft rows (Eq. 7-9) + the tree rule (Sec. 3.2, Eq. 10-12),
//   sage_verify_accept_from_slices  = second pass over the target rows (greedy token per node, Sec. 2.2) + acceptance.
// Both read the workspace that sage_entropy_topk_slices filled and run exactly the device code of the separate calls
// (topk_device.h, build_tree_device.h, verify_accept_device.h), so their outputs are bit-identical to the unfused
// sequence sage_entropy_topk -> sage_build_tree / sage_verify_accept.
//   sage_verify_accept_close_from_slices = the latter followed, in the same launch, by what closes the step (Alg. 1
// Phase 3, Sec. 3.3: path commit, length advance, history update; the device code of commit_device.h).
#include "commit_device.h"
#include "plan_device.h"
#include "verify_accept_device.h"

using namespace sage::topk;

namespace {

// One workgroup per sequence: merge the sequence's draft row, then wave 0 builds its tree from the winners it holds.
template <int OWN>
__global__ __launch_bounds__(MERGE_THREADS) void plan_kernel(int k, int nunits, const UnitStats* __restrict__ stats,
                                                             const uint64_t* __restrict__ keys, float* __restrict__ entropy,
                                                             int* __restrict__ topk_idx, float* __restrict__ topk_prob,
                                                             float* __restrict__ topk_renorm, float* __restrict__ topk_entropy,
                                                             float* __restrict__ alpha, sage_tree_params prm,
                                                             const int* __restrict__ d_max_seq, int* __restrict__ n_nodes,
                                                             int* __restrict__ parent, int* __restrict__ depth,
                                                             int* __restrict__ rank, uint64_t* __restrict__ anc_mask,
                                                             float* __restrict__ cum_prob, int* __restrict__ node_token) {
    __shared__ MergeShared<OWN> sh;
    const sage::PlanArgs pl{k,        nunits,      stats,        keys,  entropy, topk_idx,  topk_prob, topk_renorm, topk_entropy,
                            alpha,    prm,         d_max_seq,    n_nodes, parent, depth,    rank,      anc_mask,    cum_prob,
                            node_token};
    sage::plan_sequence<OWN, MERGE_THREADS>(blockIdx.x, pl, sh);
}

// One workgroup of 16 waves per sequence.  Wave w finishes the k = 1 reduction of the target rows of nodes w, w+16, ...
// (log-sum-exp of the slice statistics in the order merge_row uses, maximum of the slice candidates); the greedy tokens
// meet in LDS and wave 0 runs the acceptance rule on them.
constexpr int ACCEPT_WAVES = 16;
constexpr int ROWS_PER_WAVE = SAGE_MAX_NODES / ACCEPT_WAVES;
// What closes the step, for the kernel instantiated with CLOSE (sage_verify_accept_close_from_slices).
struct CloseArgs {
    const unsigned char* Kt; const unsigned char* Vt; unsigned char* Kc; unsigned char* Vc;
    const int64_t* kv_start; int* kv_len; int* hist; int* count; const int* d_max_in; int* d_max_out; float* avg_out;
    long kv_token_stride, kv_head_stride;
    int esz, Hkv, d, kv_capacity, window, d_floor, d_cap;
    float lo, hi;
};
template <int OWN, bool CLOSE>
__global__ __launch_bounds__(64 * ACCEPT_WAVES) void accept_kernel(const int* __restrict__ n_nodes, int nunits,
                                                                   const UnitStats* __restrict__ stats,
                                                                   const uint64_t* __restrict__ keys,
                                                                   const int* __restrict__ token, const int* __restrict__ parent,
                                                                   const int* __restrict__ depth,
                                                                   const uint64_t* __restrict__ anc_mask, int path_cap,
                                                                   float* __restrict__ entropy, int* __restrict__ target_argmax,
                                                                   int* __restrict__ accept_len, int* __restrict__ best_node,
                                                                   int* __restrict__ path_nodes, int* __restrict__ out_tokens,
                                                                   CloseArgs cl) {
    __shared__ int s_tgt[SAGE_MAX_NODES];
    __shared__ int s_tau;
    __shared__ sage::accept::AcceptShared sh;
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const long base = static_cast<long>(b) * SAGE_MAX_NODES;
    int n = n_nodes[b];
    n = n < 1 ? 1 : (n > SAGE_MAX_NODES ? SAGE_MAX_NODES : n);

    // wave 0 asks for its node fields now, so they arrive while the reductions run
    int par = -1, tok = 0, dep = 0;
    uint64_t am = 0;
    if (wave == 0 && lane < n) {
        par = parent[base + lane];
        tok = token[base + lane];
        dep = depth[base + lane];
        am = anc_mask[base + lane];
    }

    // ---- with few lists per lane all of this wave's rows are requested before the first one is reduced (one memory
    //      round trip); with many, a row at a time, to stay within the register file
    constexpr bool AHEAD = OWN <= 4;
    constexpr int HELD = AHEAD ? ROWS_PER_WAVE : 1;
    UnitStats st[HELD][OWN];
    uint64_t ky[HELD][OWN];
    auto request = [&](int j, int slot) __attribute__((always_inline)) {
        const int node = wave + j * ACCEPT_WAVES;
        const long row = base + node;
#pragma unroll
        for (int i = 0; i < OWN; ++i) {
            const int c = lane + 64 * i;
            const bool live = node < n && c < nunits;
            st[slot][i] = live ? stats[row * nunits + c] : UnitStats{-INFINITY, 0.f, 0.f, 0.f};
            ky[slot][i] = live ? keys[row * nunits + c] : 0ull;
        }
    };
    if (AHEAD) {
#pragma unroll
        for (int j = 0; j < ROWS_PER_WAVE; ++j) request(j, j);
    }
#pragma unroll
    for (int jj = 0; jj < ROWS_PER_WAVE; ++jj) {
        const int node = wave + jj * ACCEPT_WAVES;
        if (node >= n) continue;                     // wave-uniform
        if (!AHEAD) request(jj, 0);
        const int j = AHEAD ? jj : 0;
        float m, Z, Tm;
        combine_unit_stats<OWN>(st[j], lane, nunits, m, Z, Tm);
        Key best = key_unpack(ky[j][0]);
#pragma unroll
        for (int i = 1; i < OWN; ++i) best = key_max(best, key_unpack(ky[j][i]));
        const Key g = wave_max_key(best);
        if (lane == 0) {
            const int idx = key_index(g);
            s_tgt[node] = idx;
            target_argmax[base + node] = idx;
            if (entropy) entropy[base + node] = logf(Z) + Tm / Z;
        }
    }
    __syncthreads();
    if (wave != 0 && !CLOSE) return;
    if (wave == 0) {
        const int tgt = lane < n ? s_tgt[lane] : 0;
        const int tgt_par = (lane < n && par >= 0 && par < n) ? s_tgt[par] : 0;
        const int tau = sage::accept::verify_accept_wave(b, lane, n, par, tok, dep, am, tgt, tgt_par, path_cap, sh, accept_len,
                                                         best_node, path_nodes, out_tokens);
        if (CLOSE && lane == 0) s_tau = tau;
    }
    if (!CLOSE) return;
    // ---- the accepted path joins the cache, the length advances, the history moves the depth limit: what
    //      sage_close_step does, here with the path still in LDS and all 16 waves copying
    __syncthreads();
    const int tau = s_tau;
    const int len_b = cl.kv_len[b];
    for (int j = 0; j <= tau && j < path_cap; ++j)
        sage::closing::commit_row(cl.Kt, cl.Vt, cl.Kc, cl.Vc, cl.esz, cl.Hkv, cl.d, cl.kv_start, len_b, cl.kv_capacity,
                                  cl.kv_token_stride, cl.kv_head_stride, sh.slot_node[j], j, b);
    __syncthreads();                                 // every thread has read the old length
    if (threadIdx.x == 0) cl.kv_len[b] = sage::closing::advanced_len(len_b, tau, cl.kv_capacity);
    if (wave == 1)
        sage::closing::history_wave(b, lane, tau, cl.window, cl.lo, cl.hi, cl.d_floor, cl.d_cap, cl.hist, cl.count, cl.d_max_in,
                                    cl.d_max_out, cl.avg_out);
}

}  // namespace

// Argument checks of sage_build_tree_from_slices; fills what its kernel takes.  Shared with the attention call that
// carries the planning along (tree_attention.hip).
namespace sage {
int plan_args_from_slices(void* slices, int vocab, int B, int k, const sage_tree_params* params, const int* d_max_seq,
                          float* entropy, int* topk_idx, float* topk_prob, float* topk_renorm, float* topk_entropy,
                          float* alpha, int* n_nodes, int* parent, int* depth, int* rank, uint64_t* anc_mask, float* cum_prob,
                          int* node_token, PlanArgs* out) {
    if (!slices || !params || !topk_idx || !n_nodes || !parent || !depth || !rank || !anc_mask) return SAGE_INVALID_ARG;
    const sage_tree_params p = *params;
    if (B < 0 || vocab < 1 || k != p.k || k < 1 || k > SAGE_MAX_TOPK || k > vocab) return SAGE_INVALID_ARG;
    if (p.n_max < 1 || p.n_max > SAGE_MAX_NODES) return SAGE_INVALID_ARG;
    if (p.d_min < 1 || p.d_min > p.d_max || p.d_max > SAGE_MAX_DEPTH) return SAGE_INVALID_ARG;
    if (p.w_min < 1 || p.w_min > p.w_max || p.w_max > k) return SAGE_INVALID_ARG;
    if (!aligned(slices, 16)) return SAGE_INVALID_ARG;
    if (B > 65535) return SAGE_UNSUPPORTED;
    UnitStats* stats;
    uint64_t* keys;
    int nunits;
    topk_workspace_layout(B, vocab, slices, &stats, &keys, &nunits);
    if (nunits > topk_max_units()) return SAGE_UNSUPPORTED;
    *out = PlanArgs{k,     nunits, stats,     keys,   entropy, topk_idx, topk_prob, topk_renorm, topk_entropy,
                    alpha, p,      d_max_seq, n_nodes, parent, depth,    rank,      anc_mask,    cum_prob,
                    node_token};
    return SAGE_OK;
}

int launch_plan(const PlanArgs& a, int B, hipStream_t s) {
    if (a.nunits <= 256)
        hipLaunchKernelGGL(plan_kernel<4>, dim3(B), dim3(MERGE_THREADS), 0, s, a.k, a.nunits, a.stats, a.keys, a.entropy, a.topk_idx,
                           a.topk_prob, a.topk_renorm, a.topk_entropy, a.alpha, a.prm, a.d_max_seq, a.n_nodes, a.parent, a.depth,
                           a.rank, a.anc_mask, a.cum_prob, a.node_token);
    else
        hipLaunchKernelGGL(plan_kernel<MAX_OWN>, dim3(B), dim3(MERGE_THREADS), 0, s, a.k, a.nunits, a.stats, a.keys, a.entropy,
                           a.topk_idx, a.topk_prob, a.topk_renorm, a.topk_entropy, a.alpha, a.prm, a.d_max_seq, a.n_nodes, a.parent,
                           a.depth, a.rank, a.anc_mask, a.cum_prob, a.node_token);
    return launch_status();
}
}  // namespace sage

extern "C" int sage_build_tree_from_slices(void* slices, int vocab, int B, int k, const sage_tree_params* params,
                                           const int* d_max_seq, float* entropy, int* topk_idx, float* topk_prob,
                                           float* topk_renorm, float* topk_entropy, float* alpha, int* n_nodes, int* parent,
                                           int* depth, int* rank, uint64_t* anc_mask, float* cum_prob, int* node_token,
                                           void* stream) {
    sage::PlanArgs a;
    const int rc = sage::plan_args_from_slices(slices, vocab, B, k, params, d_max_seq, entropy, topk_idx, topk_prob, topk_renorm,
                                               topk_entropy, alpha, n_nodes, parent, depth, rank, anc_mask, cum_prob, node_token, &a);
    if (rc != SAGE_OK || B == 0) return rc;
    return sage::launch_plan(a, B, sage::as_stream(stream));
}

extern "C" int sage_verify_accept_from_slices(void* slices, int vocab, const int* token, const int* parent, const int* depth,
                                              const uint64_t* anc_mask, const int* n_nodes, int B, int path_cap,
                                              float* entropy, int* target_argmax, int* accept_len, int* best_node,
                                              int* path_nodes, int* out_tokens, void* stream) {
    if (!slices || !token || !parent || !depth || !anc_mask || !n_nodes || !target_argmax || !accept_len || !best_node ||
        !path_nodes || !out_tokens)
        return SAGE_INVALID_ARG;
    if (B < 0 || vocab < 1 || path_cap < 1) return SAGE_INVALID_ARG;
    if (!sage::aligned(slices, 16)) return SAGE_INVALID_ARG;
    if (static_cast<long>(B) * SAGE_MAX_NODES > 65535) return SAGE_UNSUPPORTED;   // the limit of the call that fills `slices`
    UnitStats* stats;
    uint64_t* keys;
    int nunits;
    sage::topk_workspace_layout(B * SAGE_MAX_NODES, vocab, slices, &stats, &keys, &nunits);
    if (nunits > sage::topk_max_units()) return SAGE_UNSUPPORTED;
    if (B == 0) return SAGE_OK;
    hipStream_t s = sage::as_stream(stream);
    if (nunits <= 256)
        hipLaunchKernelGGL((accept_kernel<4, false>), dim3(B), dim3(64 * ACCEPT_WAVES), 0, s, n_nodes, nunits, stats, keys, token,
                           parent, depth, anc_mask, path_cap, entropy, target_argmax, accept_len, best_node, path_nodes, out_tokens,
                           CloseArgs{});
    else
        hipLaunchKernelGGL((accept_kernel<MAX_OWN, false>), dim3(B), dim3(64 * ACCEPT_WAVES), 0, s, n_nodes, nunits, stats, keys,
                           token, parent, depth, anc_mask, path_cap, entropy, target_argmax, accept_len, best_node, path_nodes,
                           out_tokens, CloseArgs{});
    return sage::launch_status();
}

extern "C" int sage_verify_accept_close_from_slices(
    void* slices, int vocab, const int* token, const int* parent, const int* depth, const uint64_t* anc_mask, const int* n_nodes,
    int B, int path_cap, float* entropy, int* target_argmax, int* accept_len, int* best_node, int* path_nodes, int* out_tokens,
    const void* Kt, const void* Vt, void* Kc, void* Vc, int dtype, int Hkv, int d, const int64_t* kv_start, int* kv_len,
    int kv_capacity, long kv_token_stride, long kv_head_stride, int window, float lo, float hi, int d_floor, int d_cap, int* hist,
    int* count, const int* d_max_in, int* d_max_out, float* avg_out, void* stream) {
    if (!slices || !token || !parent || !depth || !anc_mask || !n_nodes || !target_argmax || !accept_len || !best_node ||
        !path_nodes || !out_tokens)
        return SAGE_INVALID_ARG;
    if (!Kt || !Vt || !Kc || !Vc || !kv_start || !kv_len || !hist || !count || !d_max_in || !d_max_out) return SAGE_INVALID_ARG;
    if (B < 0 || vocab < 1 || path_cap < 1 || Hkv < 1 || d < 1 || kv_capacity < 0) return SAGE_INVALID_ARG;
    if (dtype != SAGE_F32 && dtype != SAGE_BF16) return SAGE_INVALID_ARG;
    if (kv_head_stride < d || kv_token_stride < d) return SAGE_INVALID_ARG;
    const int esz = dtype == SAGE_F32 ? 4 : 2;
    if ((static_cast<long>(d) * esz) % 16 != 0 || (kv_token_stride * esz) % 16 != 0 || (kv_head_stride * esz) % 16 != 0)
        return SAGE_INVALID_ARG;
    if (!sage::aligned(slices, 16) || !sage::aligned(Kt, 16) || !sage::aligned(Vt, 16) || !sage::aligned(Kc, 16) ||
        !sage::aligned(Vc, 16))
        return SAGE_INVALID_ARG;
    if (window < 1 || window > 64 || d_floor < 1 || d_floor > d_cap || d_cap > SAGE_MAX_DEPTH || !(lo <= hi))
        return SAGE_INVALID_ARG;
    if (static_cast<long>(B) * SAGE_MAX_NODES > 65535 || path_cap > SAGE_MAX_NODES) return SAGE_UNSUPPORTED;
    UnitStats* stats;
    uint64_t* keys;
    int nunits;
    sage::topk_workspace_layout(B * SAGE_MAX_NODES, vocab, slices, &stats, &keys, &nunits);
    if (nunits > sage::topk_max_units()) return SAGE_UNSUPPORTED;
    if (B == 0) return SAGE_OK;
    CloseArgs cl;
    cl.Kt = static_cast<const unsigned char*>(Kt); cl.Vt = static_cast<const unsigned char*>(Vt);
    cl.Kc = static_cast<unsigned char*>(Kc); cl.Vc = static_cast<unsigned char*>(Vc);
    cl.kv_start = kv_start; cl.kv_len = kv_len; cl.hist = hist; cl.count = count; cl.d_max_in = d_max_in; cl.d_max_out = d_max_out;
    cl.avg_out = avg_out; cl.kv_token_stride = kv_token_stride; cl.kv_head_stride = kv_head_stride;
    cl.esz = esz; cl.Hkv = Hkv; cl.d = d; cl.kv_capacity = kv_capacity; cl.window = window; cl.d_floor = d_floor; cl.d_cap = d_cap;
    cl.lo = lo; cl.hi = hi;
    hipStream_t s = sage::as_stream(stream);
    if (nunits <= 256)
        hipLaunchKernelGGL((accept_kernel<4, true>), dim3(B), dim3(64 * ACCEPT_WAVES), 0, s, n_nodes, nunits, stats, keys, token,
                           parent, depth, anc_mask, path_cap, entropy, target_argmax, accept_len, best_node, path_nodes, out_tokens, cl);
    else
        hipLaunchKernelGGL((accept_kernel<MAX_OWN, true>), dim3(B), dim3(64 * ACCEPT_WAVES), 0, s, n_nodes, nunits, stats, keys,
                           token, parent, depth, anc_mask, path_cap, entropy, target_argmax, accept_len, best_node, path_nodes,
                           out_tokens, cl);
    return sage::launch_status();
}
