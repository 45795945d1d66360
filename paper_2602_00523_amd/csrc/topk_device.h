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

// Wave-wide maximum, result in every lane: four rotations inside each row of 16 lanes, then the 16-lane and
// 32-lane swaps combine the four rows.  A key is reduced in two passes: the value code first, then the index
// code among the lanes that hold the winning value.
template <int CTRL> __device__ __forceinline__ uint32_t u_dpp(uint32_t v) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, u_dpp<0x128>(v));         // row_ror:8
    v = max(v, u_dpp<0x124>(v));         // row_ror:4
    v = max(v, u_dpp<0x122>(v));         // row_ror:2
    v = max(v, u_dpp<0x121>(v));         // row_ror:1
    auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = max(a[0], a[1]);
    a = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return max(a[0], a[1]);
}
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
template <int CTRL> __device__ __forceinline__ float f_dpp(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += f_dpp<0x128>(v); v += f_dpp<0x124>(v); v += f_dpp<0x122>(v); v += f_dpp<0x121>(v);
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(a[0]) + __uint_as_float(a[1]);
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, f_dpp<0x128>(v)); v = fmaxf(v, f_dpp<0x124>(v)); v = fmaxf(v, f_dpp<0x122>(v)); v = fmaxf(v, f_dpp<0x121>(v));
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
}

__device__ __forceinline__ bool row_is_valid(int row, const int* n_valid, int rows_per_group) {
    if (!n_valid) return true;
    return (row % rows_per_group) < n_valid[row / rows_per_group];
}

// LDS of one merging workgroup.
template <int OWN> struct MergeShared {
    uint64_t keys[MERGE_LDS_KEYS];
    UnitStats stats[64 * OWN];
};

// What wave 0 holds once a row is merged: lane j < k owns winner j (token index, probability, renormalised probability);
// alpha (Eq. 9) is wave-uniform.
struct MergedRow {
    int idx;
    float p, q, alpha;
};

// Second pass for one row, called by all MERGE_THREADS threads of a workgroup: combine the slice statistics, k-way
// merge of the per-slice sorted key lists, Eq. 7-9.  OWN = lists per lane (lane owns lists lane, lane+64, ...); the
// head of every owned list stays in registers and only the lane whose list wins a round fetches its next entry.
// Writes the row's outputs (null pointers are skipped) and returns true in wave 0, whose lanes receive `out`; the other
// waves only help staging and return false.
template <int OWN>
__device__ __forceinline__ bool merge_row(int row, int k, int nunits, const UnitStats* __restrict__ stats,
                                          const uint64_t* __restrict__ keys, MergeShared<OWN>& sh, float* __restrict__ entropy,
                                          int* __restrict__ topk_idx, float* __restrict__ topk_prob,
                                          float* __restrict__ topk_renorm, float* __restrict__ topk_entropy,
                                          float* __restrict__ alpha, MergedRow& out) {
    constexpr int THREADS = MERGE_THREADS;
    uint64_t* s_keys = sh.keys;
    UnitStats* s_stats = sh.stats;
    const int tid = threadIdx.x;
    const UnitStats* st = stats + static_cast<long>(row) * nunits;
    const uint64_t* kk = keys + static_cast<long>(row) * nunits * k;
    const int total = nunits * k;
    const bool in_lds = total <= MERGE_LDS_KEYS;
    // ---- the whole workgroup stages statistics and lists in LDS, eight independent loads per thread at a time
    for (int c = tid; c < nunits; c += THREADS) s_stats[c] = st[c];
    if (in_lds) {
        for (int i0 = tid; i0 < total; i0 += THREADS * 8) {
            uint64_t tmp[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) tmp[j] = (i0 + j * THREADS < total) ? kk[i0 + j * THREADS] : 0;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (i0 + j * THREADS < total) s_keys[i0 + j * THREADS] = tmp[j];
        }
    }
    __syncthreads();
    if (tid >= 64) return false;                     // wave 0 finishes the row
    const int lane = tid;

    Key head[OWN];
    int cursor[OWN];
#pragma unroll
    for (int i = 0; i < OWN; ++i) {
        const int c = lane + 64 * i;
        head[i] = c < nunits ? key_unpack(in_lds ? s_keys[c * k] : kk[static_cast<long>(c) * k]) : Key{0, 0};
        cursor[i] = 0;
    }
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < OWN; ++i)
        if (lane + 64 * i < nunits) m = fmaxf(m, s_stats[lane + 64 * i].m);
    m = wave_max(m);
    float Z = 0.f, Tm = 0.f;
#pragma unroll
    for (int i = 0; i < OWN; ++i) {
        if (lane + 64 * i < nunits) {
            const UnitStats u = s_stats[lane + 64 * i];
            if (u.m > -INFINITY) {
                const float dlt = m - u.m;
                const float w = expf(-dlt);
                Z += w * u.Z;
                Tm += w * (u.T + u.Z * dlt);
            }
        }
    }
    Z = wave_sum(Z);
    Tm = wave_sum(Tm);
    if (lane == 0 && entropy) entropy[row] = logf(Z) + Tm / Z;

    Key mine = Key{0, 0};                            // lane j keeps winner j
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
