// Device-side pieces of the top-k second pass, shared by the kernels that run it on its own (entropy_topk.hip) and by
// the kernels that fold it into the step that consumes its result (fused_steps.hip): wave-wide reductions, the per-row
// merge of slice statistics and candidate lists, Eq. 7-9 on the winners.
#pragma once
#include "topk_common.h"

namespace sage {
namespace topk {

constexpr int MERGE_THREADS = 256;
constexpr int MERGE_LDS_KEYS = 6144;     // lists are staged in LDS when they fit (48 KB)
constexpr int MAX_OWN = 16;              // lists per lane in the second pass: up to 1024 slices = 1M logits

// The wave-wide reductions of sage_internal.h, under this namespace's names.
using sage::wave_max;
using sage::wave_max_u32;
using sage::wave_sum;

// A key is reduced in two passes: the value code first, then the index code among the lanes that hold the winning value.
__device__ __forceinline__ Key wave_max_key(Key k) {
    const uint32_t hi = wave_max_u32(k.hi);
    const uint64_t holders = __ballot(k.hi == hi);
    uint32_t lo;
    if (__builtin_popcountll(holders) == 1)          // the usual case: no second reduction, just fetch the winner's index
        lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(k.lo), __builtin_ctzll(holders)));
    else
        lo = wave_max_u32(k.hi == hi ? k.lo : 0u);
    return Key{hi, lo};
}
__device__ __forceinline__ bool row_is_valid(int row, const int* n_valid, int rows_per_group) {
    if (!n_valid) return true;
    return (row % rows_per_group) < n_valid[row / rows_per_group];
}

// Log-sum-exp combination of slice statistics held OWN per lane (lane owns slices lane, lane + 64, ...): the row's
// maximum m and the sums Z, T relative to it, in every lane.  One definition for every kernel that finishes a row, so
// that they agree to the bit.
template <int OWN>
__device__ __forceinline__ void combine_unit_stats(const UnitStats (&u)[OWN], int lane, int nunits, float& m, float& Z, float& Tm) {
    m = -INFINITY;
#pragma unroll
    for (int i = 0; i < OWN; ++i)
        if (lane + 64 * i < nunits) m = fmaxf(m, u[i].m);
    m = wave_max(m);
    Z = 0.f;
    Tm = 0.f;
#pragma unroll
    for (int i = 0; i < OWN; ++i) {
        if (lane + 64 * i < nunits && u[i].m > -INFINITY) {
            const float dlt = m - u[i].m;
            const float w = __builtin_amdgcn_exp2f(dlt * -1.4426950408889634f);
            Z += w * u[i].Z;
            Tm += w * (u[i].T + u[i].Z * dlt);
        }
    }
    Z = wave_sum(Z);
    Tm = wave_sum(Tm);
}

// LDS of one merging workgroup.  merge_row takes any type with these members (keys, stats, row_m, row_Z; LDS_KEYS =
// how many keys fit), so a kernel with another LDS budget can bring a smaller one.
template <int OWN> struct MergeShared {
    static constexpr int LDS_KEYS = MERGE_LDS_KEYS;
    uint64_t keys[MERGE_LDS_KEYS];
    UnitStats stats[64 * OWN];
    float row_m, row_Z;                  // the row's maximum and sum, from the wave that combines the statistics
};

// Short form of candidate `pos` of list `unit`: 16-bit value code, then the candidate's place among all lists, inverted.
// It orders candidates exactly like the full key when every value is a widened bf16 (the low half of such a value's
// code is all zeros or all ones, a function of the sign) and lists are in index order with at most 16 entries each:
// equal values then rank by (list, position in the list), which is index order.  0 = no candidate.
constexpr int SHORT_MAX_K = 16;
__device__ __forceinline__ bool key_is_widened_bf16(Key k) {
    return key_none(k) || (k.hi & 0xFFFFu) == ((k.hi & 0x80000000u) ? 0u : 0xFFFFu);
}
__device__ __forceinline__ uint32_t short_key(Key k, int unit, int pos) {
    return key_none(k) ? 0u : ((k.hi & 0xFFFF0000u) | (0xFFFFu - static_cast<uint32_t>(unit * SHORT_MAX_K + pos)));
}

// What wave 0 holds once a row is merged: lane j < k owns winner j (token index, probability, renormalised probability);
// alpha (Eq. 9) is wave-uniform.
struct MergedRow {
    int idx;
    float p, q, alpha;
};

// Second pass for one row, called by all WG_THREADS threads of a workgroup (at least two waves): combine the slice
// statistics, k-way merge of the per-slice sorted key lists, Eq. 7-9.  OWN = lists per lane (lane owns lists lane,
// lane+64, ...); the head of every owned list stays in registers and only the lane whose list wins a round fetches its
// next entry.  Writes the row's outputs (null pointers are skipped) and returns true in wave 0, whose lanes receive
// `out`; the other waves only help staging and return false.  Every thread passes the same two workgroup barriers.
template <int OWN, int WG_THREADS = MERGE_THREADS, class Shared>
__device__ __forceinline__ bool merge_row(int row, int k, int nunits, const UnitStats* __restrict__ stats,
                                          const uint64_t* __restrict__ keys, Shared& sh, float* __restrict__ entropy,
                                          int* __restrict__ topk_idx, float* __restrict__ topk_prob,
                                          float* __restrict__ topk_renorm, float* __restrict__ topk_entropy,
                                          float* __restrict__ alpha, MergedRow& out) {
    constexpr int THREADS = WG_THREADS;
    uint64_t* s_keys = sh.keys;
    UnitStats* s_stats = sh.stats;
    const int tid = threadIdx.x;
    const UnitStats* st = stats + static_cast<long>(row) * nunits;
    const uint64_t* kk = keys + static_cast<long>(row) * nunits * k;
    const int total = nunits * k;
    const bool in_lds = total <= Shared::LDS_KEYS;
    // ---- the whole workgroup stages statistics and lists in LDS, eight independent loads per thread at a time; while
    //      doing so it finds out whether the short form of the keys may be used for the selection rounds
    const bool short_possible = in_lds && k <= SHORT_MAX_K && nunits * SHORT_MAX_K < 0x10000;
    int all_bf16 = 1;
    for (int c = tid; c < nunits; c += THREADS) s_stats[c] = st[c];
    if (in_lds) {
        for (int i0 = tid; i0 < total; i0 += THREADS * 8) {
            uint64_t tmp[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) tmp[j] = (i0 + j * THREADS < total) ? kk[i0 + j * THREADS] : 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int at = i0 + j * THREADS;
                if (at < total) {
                    s_keys[at] = tmp[j];
                    all_bf16 &= key_is_widened_bf16(key_unpack(tmp[j])) ? 1 : 0;
                }
            }
        }
    }
    const bool use_short = __syncthreads_and(all_bf16) != 0 && short_possible;
    // Two serial chains that do not depend on each other run side by side: wave 1 combines the slice statistics (and
    // stores the row's entropy), wave 0 selects the k winners; they meet before Eq. 7-9, which wave 0 evaluates.
    const int lane = tid & 63;
    if (tid >= 64) {
        if (tid < 128) {
            UnitStats mine_stats[OWN];
#pragma unroll
            for (int i = 0; i < OWN; ++i)
                mine_stats[i] = lane + 64 * i < nunits ? s_stats[lane + 64 * i] : UnitStats{-INFINITY, 0.f, 0.f, 0.f};
            float m, Z, Tm;
            combine_unit_stats<OWN>(mine_stats, lane, nunits, m, Z, Tm);
            if (lane == 0) {
                sh.row_m = m;
                sh.row_Z = Z;
                if (entropy) entropy[row] = logf(Z) + Tm / Z;
            }
        }
        __syncthreads();
        return false;                                // wave 0 finishes the row
    }

    Key mine = Key{0, 0};                            // lane j keeps winner j
    if (use_short) {
        // the same tournament on the 32-bit form: one wave reduction per round, the next entry of every list already
        // in a register when its head wins
        uint32_t h[OWN], nx[OWN];
        int cur[OWN];
#pragma unroll
        for (int i = 0; i < OWN; ++i) {
            const int c = lane + 64 * i;
            h[i] = c < nunits ? short_key(key_unpack(s_keys[c * k]), c, 0) : 0u;
            nx[i] = (c < nunits && k > 1) ? short_key(key_unpack(s_keys[c * k + 1]), c, 1) : 0u;
            cur[i] = 0;
        }
        uint32_t mine_short = 0;
        for (int round = 0; round < k; ++round) {
            uint32_t best = h[0];
#pragma unroll
            for (int i = 1; i < OWN; ++i) best = max(best, h[i]);
            const uint32_t g = wave_max_u32(best);
            if (lane == round) mine_short = g;
            if (g != 0 && best == g && round + 1 < k) {
#pragma unroll
                for (int i = 0; i < OWN; ++i) {
                    if (h[i] == g) {
                        h[i] = nx[i];
                        const int after = ++cur[i] + 1;
                        nx[i] = after < k ? short_key(key_unpack(s_keys[(lane + 64 * i) * k + after]), lane + 64 * i, after) : 0u;
                    }
                }
            }
        }
        if (mine_short != 0) {
            const int place = static_cast<int>(0xFFFFu - (mine_short & 0xFFFFu));
            mine = key_unpack(s_keys[(place / SHORT_MAX_K) * k + place % SHORT_MAX_K]);
        }
    } else {
        Key head[OWN];
        int cursor[OWN];
#pragma unroll
        for (int i = 0; i < OWN; ++i) {
            const int c = lane + 64 * i;
            head[i] = c < nunits ? key_unpack(in_lds ? s_keys[c * k] : kk[static_cast<long>(c) * k]) : Key{0, 0};
            cursor[i] = 0;
        }
        for (int round = 0; round < k; ++round) {
            Key best = head[0];
#pragma unroll
            for (int i = 1; i < OWN; ++i) best = key_max(best, head[i]);
            const Key g = wave_max_key(best);
            if (lane == round) mine = g;
            if (!key_none(g) && key_equal(best, g) && round + 1 < k) {   // the owning lane advances the winning list
#pragma unroll
                for (int i = 0; i < OWN; ++i) {
                    if (key_equal(head[i], g)) {
                        const int nxt = ++cursor[i];
                        const long at = static_cast<long>(lane + 64 * i) * k + nxt;
                        head[i] = nxt < k ? key_unpack(in_lds ? s_keys[at] : kk[at]) : Key{0, 0};
                    }
                }
            }
        }
    }

    __syncthreads();                                 // the statistics are combined
    const float m = sh.row_m, Z = sh.row_Z;
    const bool have = lane < k;
    const float x = have ? key_value(mine) : -INFINITY;
    const float p = have ? expf(x - m) / Z : 0.f;
    const float mass = wave_sum(p);
    const float q = have ? p / mass : 0.f;
    const float hk = wave_sum(q > 0.f ? -q * logf(q) : 0.f);
    float a = (k == 1) ? 1.0f : 1.0f - hk / logf(static_cast<float>(k));
    a = fminf(fmaxf(a, 0.0f), 1.0f);
    if (have) {
        const long o = static_cast<long>(row) * k + lane;
        topk_idx[o] = key_index(mine);
        if (topk_prob) topk_prob[o] = p;
        if (topk_renorm) topk_renorm[o] = q;
    }
    if (lane == 0) {
        if (topk_entropy) topk_entropy[row] = hk;
        if (alpha) alpha[row] = a;
    }
    out.idx = have ? key_index(mine) : -1;
    out.p = p;
    out.q = q;
    out.alpha = a;
    return true;
}

}  // namespace topk
}  // namespace sage
