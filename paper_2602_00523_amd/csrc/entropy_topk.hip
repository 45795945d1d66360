// sage_entropy_topk: softmax statistics, top-k and confidence over vocabulary-sized logits
// (Sec. 3.1: Eq. 7 renormalised top-k, Eq. 8 its entropy, Eq. 9 confidence; Eq. 1 softmax) and, with k = 1,
// the target's greedy token per tree node (Sec. 2.2 / Def. 4.1).
//
// HBM-bound: every logit is read exactly once with 16-byte loads.  Pass 1: each WAVE owns a slice of UNIT
// logits of one row, held in registers; it extracts the slice's k best entries under the total order (value
// descending, index ascending) by k rounds of a wave-wide maximum on a 64-bit composite key, done with DPP row
// rotations and the 16/32-lane swaps (no LDS, no workgroup barrier), and reduces the slice's softmax statistics
//   Z = sum exp(x - m),  T = sum exp(x - m) (m - x)   so that   H = ln Z + T / Z   (both terms >= 0).
// Pass 2 (one wave per row) combines the slice statistics by log-sum-exp, merges the sorted per-slice lists with
// a k-round tournament over the list heads (lists staged in LDS), and evaluates Eq. 7-9 on the k winners.
#include "sage_internal.h"
#include "topk_common.h"
#include "topk_device.h"

using namespace sage::topk;

namespace {

constexpr int THREADS = 256;
constexpr int EPT = 16;                  // logits per lane
constexpr int UNIT = 64 * EPT;           // logits per wave
constexpr int WAVES = THREADS / 64;

template <typename T> struct Loader;
template <> struct Loader<float> {
    static constexpr int VEC = 4;   // elements per 16-byte load
    using Raw = float4;
    __device__ static Raw fetch(const float* p) { return *reinterpret_cast<const float4*>(p); }
    __device__ static void unpack(Raw v, float* out) { out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w; }
    __device__ static float one(const float* p) { return *p; }
};
template <> struct Loader<uint16_t> {
    static constexpr int VEC = 8;
    using Raw = uint4;
    __device__ static Raw fetch(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }
    __device__ static void unpack(Raw v, float* out) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static float one(const uint16_t* p) { return sage::bf16_bits_to_float(*p); }
};

// Pass 1 for k = 1 (many rows, one candidate per slice): one wave per (slice, row), 16 logits per lane.  HBM-bound,
// so the arithmetic per logit is kept to a compare-and-select for the argmax (strictly greater in index order keeps
// the lowest index among equals, the same total order as the composite key) and, once the slice maximum is known,
// one exp2 and two fused multiply-adds for the statistics.  Differences to the maximum are capped at 87, where
// exp is below 2^-125: a -inf logit or a padding slot then adds about 1e-38 instead of 0 to sums that are >= 1.
//
// The 16-byte loads of a (row, slice) are requested by request_unit and consumed by reduce_unit, so that a wave that
// walks several rows can have the next row's loads in flight while it reduces the current one.
template <typename T, int NV>
__device__ __forceinline__ void request_unit(const T* __restrict__ rowp, int base, int lane, int vocab,
                                             typename Loader<T>::Raw (&raw)[NV]) {
    using L = Loader<T>;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int e0 = base + (j * 64 + lane) * L::VEC;
        if (e0 + L::VEC <= vocab) raw[j] = L::fetch(rowp + e0);      // the ragged end is read element by element later
    }
}
template <typename T, int NV>
__device__ __forceinline__ void reduce_unit(const T* __restrict__ rowp, int base, int lane, int vocab,
                                            const typename Loader<T>::Raw (&raw)[NV], UnitStats* __restrict__ stat_out,
                                            uint64_t* __restrict__ key_out) {
    using L = Loader<T>;
    constexpr int VEC = L::VEC;
    float v[EPT];
    int first[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int e0 = base + (j * 64 + lane) * VEC;
        first[j] = e0;
        if (e0 + VEC <= vocab) {
            L::unpack(raw[j], v + j * VEC);
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[j * VEC + e] = (e0 + e < vocab) ? L::one(rowp + e0 + e) : -INFINITY;
        }
    }

    // ---- this lane's best candidate, then the slice's
    float bv = v[0];
    int bi = first[0];
#pragma unroll
    for (int s = 1; s < EPT; ++s) {
        const int idx = first[s / VEC] + (s % VEC);
        const bool better = v[s] > bv;                       // indices ascend with s: equal values keep the earlier one
        bv = better ? v[s] : bv;
        bi = better ? idx : bi;
    }
    const Key g = wave_max_key(bi < vocab ? make_key(bv, bi) : Key{0, 0});   // a lane past the end starts past the end
    const float unit_max = key_none(g) ? -INFINITY : key_value(g);
    if (lane == 0) *key_out = key_pack(g);

    // ---- softmax statistics of the slice relative to its own maximum
    float Z = 0.f, Tm = 0.f;
    if (unit_max > -INFINITY) {
#pragma unroll
        for (int s = 0; s < EPT; ++s) {
            const float dlt = fminf(unit_max - v[s], 87.0f);
            const float e = __builtin_amdgcn_exp2f(dlt * -1.4426950408889634f);
            Z += e;
            Tm = fmaf(e, dlt, Tm);
        }
    }
    Z = wave_sum(Z);
    Tm = wave_sum(Tm);
    if (lane == 0) *stat_out = UnitStats{unit_max, Z, Tm, 0.f};
}

// Every row is valid (n_valid == null): grid (slices / 4, rows).
template <typename T>
__global__ __launch_bounds__(THREADS) void slice_kernel(const T* __restrict__ logits, int vocab, long row_stride, int nunits,
                                                        UnitStats* __restrict__ stats, uint64_t* __restrict__ keys) {
    constexpr int NV = EPT / Loader<T>::VEC;
    const int row = blockIdx.y;
    const int unit = blockIdx.x * WAVES + (threadIdx.x >> 6);
    if (unit >= nunits) return;
    const int lane = threadIdx.x & 63;
    const T* rowp = logits + static_cast<long>(row) * row_stride;
    typename Loader<T>::Raw raw[NV];
    request_unit<T, NV>(rowp, unit * UNIT, lane, vocab, raw);
    const long o = static_cast<long>(row) * nunits + unit;
    reduce_unit<T, NV>(rowp, unit * UNIT, lane, vocab, raw, stats + o, keys + o);
}

// Rows in groups of which only the first n_valid[group] count (the target rows of a tree): grid (slices / 4, phases,
// groups).  A workgroup walks the live rows phase, phase + phases, ... of its group, the next row's loads in flight
// while the current one is reduced, so rows past n_valid cost no workgroup of their own.
constexpr int ROW_PHASES = 16;
template <typename T>
__device__ __forceinline__ void slice_rows_block(const T* __restrict__ logits, int vocab, long row_stride,
                                                 const int* __restrict__ n_valid, int rows_per_group, int rows, int nunits,
                                                 UnitStats* __restrict__ stats, uint64_t* __restrict__ keys, int block_x,
                                                 int phase, int phases, int group) {
    constexpr int NV = EPT / Loader<T>::VEC;
    const int unit = block_x * WAVES + (threadIdx.x >> 6);
    const int n = min(n_valid[group], min(rows_per_group, rows - group * rows_per_group));   // the last group may be short
    int r = phase;
    if (unit >= nunits || r >= n) return;
    const int lane = threadIdx.x & 63;
    const int base = unit * UNIT;
    const long row0 = static_cast<long>(group) * rows_per_group;
    typename Loader<T>::Raw cur[NV], nxt[NV];
    request_unit<T, NV>(logits + (row0 + r) * row_stride, base, lane, vocab, cur);
    while (true) {
        const int rn = r + phases;
        const bool more = rn < n;                            // wave-uniform
        if (more) request_unit<T, NV>(logits + (row0 + rn) * row_stride, base, lane, vocab, nxt);
        const long o = (row0 + r) * nunits + unit;
        reduce_unit<T, NV>(logits + (row0 + r) * row_stride, base, lane, vocab, cur, stats + o, keys + o);
        if (!more) break;
        for (int j = 0; j < NV; ++j) cur[j] = nxt[j];
        r = rn;
    }
}
template <typename T>
__global__ __launch_bounds__(THREADS) void slice_rows_kernel(const T* __restrict__ logits, int vocab, long row_stride,
                                                             const int* __restrict__ n_valid, int rows_per_group, int rows,
                                                             int nunits, UnitStats* __restrict__ stats,
                                                             uint64_t* __restrict__ keys) {
    slice_rows_block<T>(logits, vocab, row_stride, n_valid, rows_per_group, rows, nunits, stats, keys, blockIdx.x, blockIdx.y,
                        gridDim.y, blockIdx.z);
}

// Pass 1 for bf16 logits and 1 < k <= 16 (the draft row of a step; pure latency, so the serial selection rounds are
// kept as short as they can be): the same decomposition as the generic kernel below, but the rounds run on ONE
// 32-bit word per candidate, (16-bit value code << 16) | (1024 - position in the slice), whose order is the total
// order (value descending, index ascending) inside a slice; 0 = no candidate.  Each wave selects the k best of its
// 256 logits, wave 0 then selects the k best of the 4k survivors held one per lane.
constexpr int FAST_MAX_K = 16;
__device__ __forceinline__ void slice_topk_bf16_block(const uint16_t* __restrict__ logits, int vocab, long row_stride, int k,
                                                      const int* __restrict__ n_valid, int rows_per_group, int nunits,
                                                      UnitStats* __restrict__ stats, uint64_t* __restrict__ keys, int unit,
                                                      int row) {
    __shared__ uint32_t s_list[WAVES * FAST_MAX_K];
    __shared__ float s_red[3][WAVES];
    if (!row_is_valid(row, n_valid, rows_per_group)) return;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const uint16_t* rowp = logits + static_cast<long>(row) * row_stride;
    const int local0 = threadIdx.x * 4;
    const int e0 = unit * UNIT + local0;

    float v[4];
    if (e0 + 4 <= vocab) {
        const uint2 q = *reinterpret_cast<const uint2*>(rowp + e0);
        v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xFFFF0000u);
        v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xFFFF0000u);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (e0 + e < vocab) ? Loader<uint16_t>::one(rowp + e0 + e) : -INFINITY;
    }
    uint32_t cand[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        cand[e] = (e0 + e < vocab) ? ((sortable(v[e]) & 0xFFFF0000u) | static_cast<uint32_t>(UNIT - (local0 + e))) : 0u;

    uint32_t mine = 0, top = 0;                      // lane j keeps the wave's winner of round j
    for (int round = 0; round < k; ++round) {
        const uint32_t g = wave_max_u32(max(max(cand[0], cand[1]), max(cand[2], cand[3])));
        if (round == 0) top = g;
#pragma unroll
        for (int e = 0; e < 4; ++e) cand[e] = (cand[e] == g) ? 0u : cand[e];
        if (lane == round) mine = g;
    }
    if (lane < k) s_list[wave * k + lane] = mine;
    // a bf16 value's 32-bit code is its 16-bit code followed by sixteen zeros (non-negative) or ones (negative)
    auto full_code = [](uint32_t key) { return (key & 0xFFFF0000u) | ((key & 0x80000000u) ? 0u : 0xFFFFu); };
    const float wmax = top ? unsortable(full_code(top)) : -INFINITY;
    float Z = 0.f, Tm = 0.f;
    if (wmax > -INFINITY) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float dlt = wmax - v[e];
            const float ex = __builtin_amdgcn_exp2f(dlt * -1.4426950408889634f);   // exactly 0 for a -inf logit
            Z += ex;
            Tm += (ex > 0.f) ? ex * dlt : 0.f;
        }
    }
    Z = wave_sum(Z);
    Tm = wave_sum(Tm);
    if (lane == 0) { s_red[0][wave] = wmax; s_red[1][wave] = Z; s_red[2][wave] = Tm; }
    __syncthreads();
    if (wave != 0) return;

    uint32_t key = lane < WAVES * k ? s_list[lane] : 0u;
    uint32_t out = 0;
    for (int round = 0; round < k; ++round) {
        const uint32_t g = wave_max_u32(key);
        key = (key == g) ? 0u : key;
        if (lane == round) out = g;
    }
    if (lane < k) {
        const Key full = out ? Key{full_code(out), 0xFFFFFFFFu - static_cast<uint32_t>(unit * UNIT + UNIT - static_cast<int>(out & 0xFFFFu))}
                             : Key{0, 0};
        keys[(static_cast<long>(row) * nunits + unit) * k + lane] = key_pack(full);
    }
    if (lane == 0) {
        float m = fmaxf(fmaxf(s_red[0][0], s_red[0][1]), fmaxf(s_red[0][2], s_red[0][3]));
        float z = 0.f, t = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            if (s_red[0][w] > -INFINITY) {
                const float dlt = m - s_red[0][w];
                const float sc = expf(-dlt);
                z += sc * s_red[1][w];
                t += sc * (s_red[2][w] + s_red[1][w] * dlt);
            }
        }
        stats[static_cast<long>(row) * nunits + unit] = UnitStats{m, z, t, 0.f};
    }
}
__global__ __launch_bounds__(THREADS) void slice_topk_bf16_kernel(const uint16_t* __restrict__ logits, int vocab, long row_stride,
                                                                  int k, const int* __restrict__ n_valid, int rows_per_group,
                                                                  int nunits, UnitStats* __restrict__ stats,
                                                                  uint64_t* __restrict__ keys) {
    slice_topk_bf16_block(logits, vocab, row_stride, k, n_valid, rows_per_group, nunits, stats, keys, blockIdx.x, blockIdx.y);
}

// Pass 1 for k > 1 (few rows, latency matters more than bandwidth): one WORKGROUP per slice, 4 logits per lane.
// Each wave extracts the k best of its 256 logits; wave 0 then merges the four sorted lists.
template <typename T>
__device__ __forceinline__ void slice_topk_block(const T* __restrict__ logits, int vocab, long row_stride, int k,
                                                 const int* __restrict__ n_valid, int rows_per_group, int nunits,
                                                 UnitStats* __restrict__ stats, uint64_t* __restrict__ keys, int unit, int row) {
    __shared__ uint64_t s_list[WAVES][SAGE_MAX_TOPK];
    __shared__ float s_red[3][WAVES];
    if (!row_is_valid(row, n_valid, rows_per_group)) return;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const T* rowp = logits + static_cast<long>(row) * row_stride;
    const int e0 = unit * UNIT + threadIdx.x * 4;

    float v[4];
    if (e0 + 4 <= vocab) {
        if constexpr (sizeof(T) == 4) {
            const float4 q = *reinterpret_cast<const float4*>(rowp + e0);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
            const uint2 q = *reinterpret_cast<const uint2*>(rowp + e0);
            v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xFFFF0000u);
            v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xFFFF0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (e0 + e < vocab) ? Loader<T>::one(rowp + e0 + e) : -INFINITY;
    }
    Key cand[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) cand[e] = (e0 + e < vocab) ? make_key(v[e], e0 + e) : Key{0, 0};

    Key mine = Key{0, 0};                            // lane j keeps the wave's winner of round j
    Key top = Key{0, 0};
    for (int round = 0; round < k; ++round) {
        const Key best = key_max(key_max(cand[0], cand[1]), key_max(cand[2], cand[3]));
        const Key g = wave_max_key(best);
        if (round == 0) top = g;
        if (!key_none(g)) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (key_equal(cand[e], g)) cand[e] = Key{0, 0};
        }
        if (lane == round) mine = g;
    }
    if (lane < k) s_list[wave][lane] = key_pack(mine);
    // softmax statistics relative to the wave's maximum, combined across the four waves below
    const float wmax = key_none(top) ? -INFINITY : key_value(top);
    float Z = 0.f, Tm = 0.f;
    if (wmax > -INFINITY) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float dlt = wmax - v[e];
            const float ex = expf(-dlt);
            Z += ex;
            Tm += (ex > 0.f) ? ex * dlt : 0.f;
        }
    }
    Z = wave_sum(Z);
    Tm = wave_sum(Tm);
    if (lane == 0) { s_red[0][wave] = wmax; s_red[1][wave] = Z; s_red[2][wave] = Tm; }
    __syncthreads();
    if (wave != 0) return;

    // ---- wave 0: merge the four sorted lists (lane w < 4 owns list w) and the four statistics
    int cursor = 0;
    Key head = lane < WAVES ? key_unpack(s_list[lane][0]) : Key{0, 0};
    Key out = Key{0, 0};
    for (int round = 0; round < k; ++round) {
        const Key g = wave_max_key(head);
        if (lane == round) out = g;
        if (lane < WAVES && !key_none(g) && key_equal(head, g)) {
            ++cursor;
            head = cursor < k ? key_unpack(s_list[lane][cursor]) : Key{0, 0};
        }
    }
    if (lane < k) keys[(static_cast<long>(row) * nunits + unit) * k + lane] = key_pack(out);
    if (lane == 0) {
        float m = fmaxf(fmaxf(s_red[0][0], s_red[0][1]), fmaxf(s_red[0][2], s_red[0][3]));
        float z = 0.f, t = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            if (s_red[0][w] > -INFINITY) {
                const float dlt = m - s_red[0][w];
                const float sc = expf(-dlt);
                z += sc * s_red[1][w];
                t += sc * (s_red[2][w] + s_red[1][w] * dlt);
            }
        }
        stats[static_cast<long>(row) * nunits + unit] = UnitStats{m, z, t, 0.f};
    }
}
template <typename T>
__global__ __launch_bounds__(THREADS) void slice_topk_kernel(const T* __restrict__ logits, int vocab, long row_stride, int k,
                                                             const int* __restrict__ n_valid, int rows_per_group, int nunits,
                                                             UnitStats* __restrict__ stats, uint64_t* __restrict__ keys) {
    slice_topk_block<T>(logits, vocab, row_stride, k, n_valid, rows_per_group, nunits, stats, keys, blockIdx.x, blockIdx.y);
}

// Two first passes in one launch (sage_entropy_topk_slices_pair): the k = 1 pass over grouped rows (job A, the grid
// of slice_rows_kernel) with the k > 1 pass over a few rows (job B) in slabs of workgroups ahead of it.  A step is a
// chain of dependent launches, each a few microseconds whatever it computes; two passes that do not depend on each
// other share one.  FAST: job B takes the 32-bit rounds (bf16, k <= 16).
struct PairJob {
    const void* logits; long row_stride; int rows, k, nunits;
    UnitStats* stats; uint64_t* keys;
};
template <typename T, bool FAST>
__global__ __launch_bounds__(THREADS) void slice_pair_kernel(const T* __restrict__ logits_a, int vocab, long row_stride_a,
                                                             const int* __restrict__ n_valid_a, int rows_per_group_a,
                                                             int rows_a, int nunits, UnitStats* __restrict__ stats_a,
                                                             uint64_t* __restrict__ keys_a, int slabs_b, const PairJob b) {
    if (static_cast<int>(blockIdx.z) < slabs_b) {            // workgroup-uniform
        const int lin = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
        if (lin >= b.nunits * b.rows) return;
        const int row = lin / b.nunits, unit = lin - row * b.nunits;
        if constexpr (FAST)
            slice_topk_bf16_block(static_cast<const uint16_t*>(b.logits), vocab, b.row_stride, b.k, nullptr, 1, b.nunits, b.stats,
                                  b.keys, unit, row);
        else
            slice_topk_block<T>(static_cast<const T*>(b.logits), vocab, b.row_stride, b.k, nullptr, 1, b.nunits, b.stats, b.keys,
                                unit, row);
        return;
    }
    slice_rows_block<T>(logits_a, vocab, row_stride_a, n_valid_a, rows_per_group_a, rows_a, nunits, stats_a, keys_a, blockIdx.x,
                        blockIdx.y, gridDim.y, static_cast<int>(blockIdx.z) - slabs_b);
}

// Pass 2 as a launch of its own: one workgroup per row (see merge_row).
template <int OWN>
__global__ __launch_bounds__(MERGE_THREADS) void merge_kernel(int k, const int* __restrict__ n_valid, int rows_per_group, int nunits,
                                                              const UnitStats* __restrict__ stats, const uint64_t* __restrict__ keys,
                                                              float* __restrict__ entropy, int* __restrict__ topk_idx,
                                                              float* __restrict__ topk_prob, float* __restrict__ topk_renorm,
                                                              float* __restrict__ topk_entropy, float* __restrict__ alpha) {
    __shared__ MergeShared<OWN> sh;
    const int row = blockIdx.x;
    if (!row_is_valid(row, n_valid, rows_per_group)) return;
    MergedRow r;
    merge_row<OWN>(row, k, nunits, stats, keys, sh, entropy, topk_idx, topk_prob, topk_renorm, topk_entropy, alpha, r);
}

inline int num_units(int vocab) { return (vocab + UNIT - 1) / UNIT; }
inline size_t stats_bytes(int rows, int vocab) {
    size_t b = static_cast<size_t>(rows) * num_units(vocab) * sizeof(UnitStats);
    return (b + 255) & ~static_cast<size_t>(255);
}

}  // namespace

namespace sage {

int topk_max_units() { return 64 * MAX_OWN; }

// Pass 2 for `rows` rows whose `nunits` slices each left UnitStats and k sorted keys in stats / keys ([row][unit]).
void topk_merge(int rows, int k, const int* n_valid, int rows_per_group, int nunits, const UnitStats* stats,
                const uint64_t* keys, float* entropy, int* topk_idx, float* topk_prob, float* topk_renorm,
                float* topk_entropy, float* alpha, hipStream_t s) {
    if (nunits <= 256)
        hipLaunchKernelGGL(merge_kernel<4>, dim3(rows), dim3(MERGE_THREADS), 0, s, k, n_valid, rows_per_group, nunits, stats, keys,
                           entropy, topk_idx, topk_prob, topk_renorm, topk_entropy, alpha);
    else
        hipLaunchKernelGGL(merge_kernel<MAX_OWN>, dim3(rows), dim3(MERGE_THREADS), 0, s, k, n_valid, rows_per_group, nunits, stats,
                           keys, entropy, topk_idx, topk_prob, topk_renorm, topk_entropy, alpha);
}

}  // namespace sage

extern "C" size_t sage_entropy_topk_workspace_bytes(int rows, int vocab, int k) {
    if (rows < 0 || vocab < 1 || k < 1) return 0;
    return stats_bytes(rows, vocab) + static_cast<size_t>(rows) * num_units(vocab) * k * sizeof(uint64_t) + 256;
}

namespace sage {

// Where the first pass leaves its results inside a workspace of sage_entropy_topk_workspace_bytes(rows, vocab, k).
void topk_workspace_layout(int rows, int vocab, void* workspace, UnitStats** stats, uint64_t** keys, int* nunits) {
    *stats = static_cast<UnitStats*>(workspace);
    *keys = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + stats_bytes(rows, vocab));
    *nunits = num_units(vocab);
}

}  // namespace sage

// Argument checks of a first pass; SAGE_OK means it may be launched (rows == 0: there is nothing to launch).
static int check_first_pass(const void* logits, int dtype, int rows, int vocab, long row_stride, int k, const int* n_valid,
                            int rows_per_group, void* workspace, size_t workspace_bytes) {
    if (!logits || !workspace) return SAGE_INVALID_ARG;
    if (rows < 0 || vocab < 1 || k < 1 || k > SAGE_MAX_TOPK || k > vocab || row_stride < vocab) return SAGE_INVALID_ARG;
    if (dtype != SAGE_F32 && dtype != SAGE_BF16) return SAGE_INVALID_ARG;
    if (n_valid && rows_per_group < 1) return SAGE_INVALID_ARG;
    const size_t esz = dtype == SAGE_F32 ? 4 : 2;
    if (!sage::aligned(logits, 16) || (static_cast<size_t>(row_stride) * esz) % 16 != 0 || !sage::aligned(workspace, 16))
        return SAGE_INVALID_ARG;
    const int nunits = num_units(vocab);
    if (nunits > 64 * MAX_OWN) return SAGE_UNSUPPORTED;
    if (rows > 65535) return SAGE_UNSUPPORTED;
    if (workspace_bytes < sage_entropy_topk_workspace_bytes(rows, vocab, k)) return SAGE_WORKSPACE_TOO_SMALL;
    return SAGE_OK;
}

// Argument checks and the first pass, common to sage_entropy_topk and sage_entropy_topk_slices.
static int run_first_pass(const void* logits, int dtype, int rows, int vocab, long row_stride, int k, const int* n_valid,
                          int rows_per_group, void* workspace, size_t workspace_bytes, hipStream_t s) {
    const int rc = check_first_pass(logits, dtype, rows, vocab, row_stride, k, n_valid, rows_per_group, workspace, workspace_bytes);
    if (rc != SAGE_OK || rows == 0) return rc;
    const int nunits = num_units(vocab);
    UnitStats* stats = static_cast<UnitStats*>(workspace);
    uint64_t* keys = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + stats_bytes(rows, vocab));
    if (k == 1 && !n_valid) {                        // many rows, one round: a wave per slice, 16 logits per lane
        const dim3 grid((nunits + WAVES - 1) / WAVES, rows);
        if (dtype == SAGE_F32)
            hipLaunchKernelGGL(slice_kernel<float>, grid, dim3(THREADS), 0, s, static_cast<const float*>(logits), vocab,
                               row_stride, nunits, stats, keys);
        else
            hipLaunchKernelGGL(slice_kernel<uint16_t>, grid, dim3(THREADS), 0, s, static_cast<const uint16_t*>(logits),
                               vocab, row_stride, nunits, stats, keys);
    } else if (k == 1) {                             // grouped rows: workgroups walk the live rows of their group
        const int groups = (rows + rows_per_group - 1) / rows_per_group;
        const dim3 grid((nunits + WAVES - 1) / WAVES, rows_per_group < ROW_PHASES ? rows_per_group : ROW_PHASES, groups);
        if (dtype == SAGE_F32)
            hipLaunchKernelGGL(slice_rows_kernel<float>, grid, dim3(THREADS), 0, s, static_cast<const float*>(logits), vocab,
                               row_stride, n_valid, rows_per_group, rows, nunits, stats, keys);
        else
            hipLaunchKernelGGL(slice_rows_kernel<uint16_t>, grid, dim3(THREADS), 0, s, static_cast<const uint16_t*>(logits),
                               vocab, row_stride, n_valid, rows_per_group, rows, nunits, stats, keys);
    } else {                                         // k rounds: a workgroup per slice, 4 logits per lane
        const dim3 grid(nunits, rows);
        if (dtype == SAGE_F32)
            hipLaunchKernelGGL(slice_topk_kernel<float>, grid, dim3(THREADS), 0, s, static_cast<const float*>(logits), vocab,
                               row_stride, k, n_valid, rows_per_group, nunits, stats, keys);
        else if (k <= FAST_MAX_K)
            hipLaunchKernelGGL(slice_topk_bf16_kernel, grid, dim3(THREADS), 0, s, static_cast<const uint16_t*>(logits), vocab,
                               row_stride, k, n_valid, rows_per_group, nunits, stats, keys);
        else
            hipLaunchKernelGGL(slice_topk_kernel<uint16_t>, grid, dim3(THREADS), 0, s, static_cast<const uint16_t*>(logits),
                               vocab, row_stride, k, n_valid, rows_per_group, nunits, stats, keys);
    }
    return sage::launch_status();
}

extern "C" int sage_entropy_topk(const void* logits, int dtype, int rows, int vocab, long row_stride, int k,
                                 const int* n_valid, int rows_per_group, float* entropy, int* topk_idx,
                                 float* topk_prob, float* topk_renorm, float* topk_entropy, float* alpha,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    if (!topk_idx) return SAGE_INVALID_ARG;
    hipStream_t s = sage::as_stream(stream);
    const int rc = run_first_pass(logits, dtype, rows, vocab, row_stride, k, n_valid, rows_per_group, workspace, workspace_bytes, s);
    if (rc != SAGE_OK || rows == 0) return rc;
    UnitStats* stats;
    uint64_t* keys;
    int nunits;
    sage::topk_workspace_layout(rows, vocab, workspace, &stats, &keys, &nunits);
    sage::topk_merge(rows, k, n_valid, rows_per_group, nunits, stats, keys, entropy, topk_idx, topk_prob, topk_renorm,
                     topk_entropy, alpha, s);
    return sage::launch_status();
}

extern "C" int sage_entropy_topk_slices(const void* logits, int dtype, int rows, int vocab, long row_stride, int k,
                                        const int* n_valid, int rows_per_group, void* workspace, size_t workspace_bytes,
                                        void* stream) {
    return run_first_pass(logits, dtype, rows, vocab, row_stride, k, n_valid, rows_per_group, workspace, workspace_bytes,
                          sage::as_stream(stream));
}

extern "C" int sage_entropy_topk_slices_pair(const void* logits_a, int rows_a, long row_stride_a, const int* n_valid_a,
                                             int rows_per_group_a, void* workspace_a, size_t workspace_a_bytes,
                                             const void* logits_b, int rows_b, long row_stride_b, int k_b, void* workspace_b,
                                             size_t workspace_b_bytes, int dtype, int vocab, void* stream) {
    if (!n_valid_a || k_b < 2) return SAGE_INVALID_ARG;      // job A is the grouped k = 1 pass, job B a k > 1 pass
    int rc = check_first_pass(logits_a, dtype, rows_a, vocab, row_stride_a, 1, n_valid_a, rows_per_group_a, workspace_a,
                              workspace_a_bytes);
    if (rc != SAGE_OK) return rc;
    rc = check_first_pass(logits_b, dtype, rows_b, vocab, row_stride_b, k_b, nullptr, 1, workspace_b, workspace_b_bytes);
    if (rc != SAGE_OK) return rc;
    hipStream_t s = sage::as_stream(stream);
    if (rows_a == 0 || rows_b == 0) {                        // one job is empty: the other one's own launch
        if (rows_a) return run_first_pass(logits_a, dtype, rows_a, vocab, row_stride_a, 1, n_valid_a, rows_per_group_a, workspace_a,
                                          workspace_a_bytes, s);
        return run_first_pass(logits_b, dtype, rows_b, vocab, row_stride_b, k_b, nullptr, 1, workspace_b, workspace_b_bytes, s);
    }
    const int nunits = num_units(vocab);
    UnitStats* stats_a = static_cast<UnitStats*>(workspace_a);
    uint64_t* keys_a = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace_a) + stats_bytes(rows_a, vocab));
    PairJob b;
    b.logits = logits_b; b.row_stride = row_stride_b; b.rows = rows_b; b.k = k_b; b.nunits = nunits;
    b.stats = static_cast<UnitStats*>(workspace_b);
    b.keys = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace_b) + stats_bytes(rows_b, vocab));
    const int groups = (rows_a + rows_per_group_a - 1) / rows_per_group_a;
    const int gx = (nunits + WAVES - 1) / WAVES, gy = rows_per_group_a < ROW_PHASES ? rows_per_group_a : ROW_PHASES;
    const long blocks_b = static_cast<long>(nunits) * rows_b;
    const long slabs_b = (blocks_b + static_cast<long>(gx) * gy - 1) / (static_cast<long>(gx) * gy);
    if (slabs_b + groups > 65535) return SAGE_UNSUPPORTED;
    const dim3 grid(gx, gy, static_cast<unsigned>(slabs_b + groups));
    if (dtype == SAGE_F32)
        hipLaunchKernelGGL((slice_pair_kernel<float, false>), grid, dim3(THREADS), 0, s, static_cast<const float*>(logits_a), vocab,
                           row_stride_a, n_valid_a, rows_per_group_a, rows_a, nunits, stats_a, keys_a, static_cast<int>(slabs_b), b);
    else if (k_b <= FAST_MAX_K)
        hipLaunchKernelGGL((slice_pair_kernel<uint16_t, true>), grid, dim3(THREADS), 0, s, static_cast<const uint16_t*>(logits_a),
                           vocab, row_stride_a, n_valid_a, rows_per_group_a, rows_a, nunits, stats_a, keys_a,
                           static_cast<int>(slabs_b), b);
    else
        hipLaunchKernelGGL((slice_pair_kernel<uint16_t, false>), grid, dim3(THREADS), 0, s, static_cast<const uint16_t*>(logits_a),
                           vocab, row_stride_a, n_valid_a, rows_per_group_a, rows_a, nunits, stats_a, keys_a,
                           static_cast<int>(slabs_b), b);
    return sage::launch_status();
}
