// sage_entropy_topk: softmax statistics, top-k and confidence over vocabulary-sized logits
// (Sec. 3.1: Eq. 7 renormalised top-k, Eq. 8 its entropy, Eq. 9 confidence; Eq. 1 softmax) and, with k = 1,
// the target's greedy token per tree node (Sec. 2.2 / Def. 4.1).
//
// HBM-bound: every logit is read exactly once with 16-byte loads.  Pass 1 splits each row into chunks of
// CHUNK logits, one workgroup per (chunk, row): the chunk lives in registers, the workgroup selects its k best
// entries under the total order (value descending, index ascending) by k rounds of wave-shuffle argmax on a
// 64-bit composite key, and reduces the softmax statistics (m, Z, T) of the chunk, where
//   Z = sum exp(x - m),  T = sum exp(x - m) (m - x)   so that   H = ln Z + T / Z   (both terms >= 0).
// Pass 2 (one wave per row) combines the chunk statistics by log-sum-exp, merges the sorted per-chunk lists
// with a k-round tournament over the list heads, and evaluates Eq. 7-9 on the k winners.
#include "sage_internal.h"

namespace {

constexpr int THREADS = 256;
constexpr int EPT = 16;                  // logits per thread
constexpr int CHUNK = THREADS * EPT;     // logits per workgroup
constexpr int WAVES = THREADS / 64;

struct ChunkStats { float m, Z, T, pad; };

// Order-preserving map float -> uint32 (larger float -> larger code); -0 is folded into +0 so that equal
// values compare equal before the index tie-break.
__device__ __forceinline__ uint32_t sortable(float v) {
    uint32_t u = __float_as_uint(v);
    if (u == 0x80000000u) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unsortable(uint32_t s) {
    uint32_t u = (s & 0x80000000u) ? (s & 0x7FFFFFFFu) : ~s;
    return __uint_as_float(u);
}
// key: high word = value code, low word = ~index, so a larger key is a better candidate; 0 = no candidate.
__device__ __forceinline__ uint64_t make_key(float v, int idx) {
    return (static_cast<uint64_t>(sortable(v)) << 32) | static_cast<uint32_t>(0xFFFFFFFFu - static_cast<uint32_t>(idx));
}
__device__ __forceinline__ int key_index(uint64_t key) { return static_cast<int>(0xFFFFFFFFu - static_cast<uint32_t>(key)); }
__device__ __forceinline__ float key_value(uint64_t key) { return unsortable(static_cast<uint32_t>(key >> 32)); }

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int off) {
    uint32_t lo = __shfl_xor(static_cast<uint32_t>(v), off);
    uint32_t hi = __shfl_xor(static_cast<uint32_t>(v >> 32), off);
    return (static_cast<uint64_t>(hi) << 32) | lo;
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
    for (int off = 32; off > 0; off >>= 1) {
        uint64_t o = shfl_xor_u64(v, off);
        v = o > v ? o : v;
    }
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__device__ __forceinline__ bool row_is_valid(int row, const int* n_valid, int rows_per_group) {
    if (!n_valid) return true;
    return (row % rows_per_group) < n_valid[row / rows_per_group];
}

template <typename T> struct Loader;
template <> struct Loader<float> {
    static constexpr int VEC = 4;   // elements per 16-byte load
    __device__ static void load(const float* p, float* out) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
    __device__ static float one(const float* p) { return *p; }
};
template <> struct Loader<uint16_t> {
    static constexpr int VEC = 8;
    __device__ static void load(const uint16_t* p, float* out) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static float one(const uint16_t* p) { return sage::bf16_bits_to_float(*p); }
};

template <typename T>
__global__ __launch_bounds__(THREADS) void chunk_kernel(const T* __restrict__ logits, int vocab, long row_stride, int k,
                                                        const int* __restrict__ n_valid, int rows_per_group, int nchunks,
                                                        ChunkStats* __restrict__ stats, uint64_t* __restrict__ keys) {
    using L = Loader<T>;
    constexpr int VEC = L::VEC;
    constexpr int NV = EPT / VEC;
    __shared__ uint64_t s_key[WAVES];
    __shared__ float s_sum[2][WAVES];

    const int row = blockIdx.y;
    const int chunk = blockIdx.x;
    if (!row_is_valid(row, n_valid, rows_per_group)) return;
    const int tid = threadIdx.x;
    const T* rowp = logits + static_cast<long>(row) * row_stride;
    const int base = chunk * CHUNK;

    float v[EPT];
    int first[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int e0 = base + (j * THREADS + tid) * VEC;
        first[j] = e0;
        if (e0 + VEC <= vocab) {
            L::load(rowp + e0, v + j * VEC);
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[j * VEC + e] = (e0 + e < vocab) ? L::one(rowp + e0 + e) : -INFINITY;
        }
    }

    // ---- k rounds of workgroup-wide argmax on the composite key
    uint32_t taken = 0;
    float chunk_max = -INFINITY;
    uint64_t* out_keys = keys + (static_cast<long>(row) * nchunks + chunk) * k;
    for (int round = 0; round < k; ++round) {
        uint64_t best = 0;
        int best_slot = -1;
#pragma unroll
        for (int s = 0; s < EPT; ++s) {
            const int idx = first[s / VEC] + (s % VEC);
            const uint64_t key = (idx < vocab && !((taken >> s) & 1)) ? make_key(v[s], idx) : 0;
            if (key > best) { best = key; best_slot = s; }
        }
        uint64_t w = wave_max_u64(best);
        if ((tid & 63) == 0) s_key[tid >> 6] = w;
        __syncthreads();
        uint64_t g = s_key[0];
#pragma unroll
        for (int i = 1; i < WAVES; ++i) g = s_key[i] > g ? s_key[i] : g;
        __syncthreads();
        if (g != 0 && best == g) taken |= 1u << best_slot;
        if (round == 0) chunk_max = (g != 0) ? key_value(g) : -INFINITY;
        if (tid == 0) out_keys[round] = g;
    }

    // ---- softmax statistics of the chunk relative to its own maximum
    float Z = 0.f, Tm = 0.f;
    if (chunk_max > -INFINITY) {
#pragma unroll
        for (int s = 0; s < EPT; ++s) {
            const float dlt = chunk_max - v[s];          // >= 0, +inf for padding and -inf logits
            const float e = expf(-dlt);
            Z += e;
            Tm += (e > 0.f) ? e * dlt : 0.f;
        }
    }
    Z = wave_sum(Z);
    Tm = wave_sum(Tm);
    if ((tid & 63) == 0) { s_sum[0][tid >> 6] = Z; s_sum[1][tid >> 6] = Tm; }
    __syncthreads();
    if (tid == 0) {
        float z = 0.f, t = 0.f;
#pragma unroll
        for (int i = 0; i < WAVES; ++i) { z += s_sum[0][i]; t += s_sum[1][i]; }
        stats[static_cast<long>(row) * nchunks + chunk] = ChunkStats{chunk_max, z, t, 0.f};
    }
}

// One wave per row: combine chunk statistics, k-way merge of the per-chunk sorted key lists, Eq. 7-9.
__global__ __launch_bounds__(64) void merge_kernel(int k, const int* __restrict__ n_valid, int rows_per_group, int nchunks,
                                                   const ChunkStats* __restrict__ stats, const uint64_t* __restrict__ keys,
                                                   float* __restrict__ entropy, int* __restrict__ topk_idx,
                                                   float* __restrict__ topk_prob, float* __restrict__ topk_renorm,
                                                   float* __restrict__ topk_entropy, float* __restrict__ alpha) {
    const int row = blockIdx.x;
    if (!row_is_valid(row, n_valid, rows_per_group)) return;
    const int lane = threadIdx.x;
    const ChunkStats* st = stats + static_cast<long>(row) * nchunks;
    const uint64_t* kk = keys + static_cast<long>(row) * nchunks * k;

    float m = -INFINITY;
    for (int c = lane; c < nchunks; c += 64) m = fmaxf(m, st[c].m);
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float Z = 0.f, Tm = 0.f;
    for (int c = lane; c < nchunks; c += 64) {
        const ChunkStats s = st[c];
        if (s.m > -INFINITY) {
            const float dlt = m - s.m;
            const float w = expf(-dlt);
            Z += w * s.Z;
            Tm += w * (s.T + s.Z * dlt);
        }
    }
    Z = wave_sum(Z);
    Tm = wave_sum(Tm);
    if (lane == 0 && entropy) entropy[row] = logf(Z) + Tm / Z;

    // tournament over list heads; lane owns chunks lane, lane+64, ... and a cursor per owned chunk
    constexpr int MAX_OWN = 16;                      // supports nchunks <= 1024
    unsigned char cursor[MAX_OWN];
#pragma unroll
    for (int i = 0; i < MAX_OWN; ++i) cursor[i] = 0;
    uint64_t mine = 0;                               // the winner this lane reports: lane j keeps winner j
    for (int round = 0; round < k; ++round) {
        uint64_t best = 0;
        int best_own = -1;
#pragma unroll
        for (int i = 0; i < MAX_OWN; ++i) {
            const int c = lane + 64 * i;
            if (c < nchunks && cursor[i] < k) {
                const uint64_t key = kk[static_cast<long>(c) * k + cursor[i]];
                if (key > best) { best = key; best_own = i; }
            }
        }
        const uint64_t g = wave_max_u64(best);
        if (g != 0 && best == g) {
#pragma unroll
            for (int i = 0; i < MAX_OWN; ++i)
                if (i == best_own) cursor[i]++;
        }
        if (lane == round) mine = g;
    }

    const bool have = lane < k;
    const float x = have ? key_value(mine) : -INFINITY;
    const float p = have ? expf(x - m) / Z : 0.f;
    const float mass = wave_sum(p);
    const float q = have ? p / mass : 0.f;
    const float hk = wave_sum(q > 0.f ? -q * logf(q) : 0.f);
    if (have) {
        const long o = static_cast<long>(row) * k + lane;
        topk_idx[o] = key_index(mine);
        if (topk_prob) topk_prob[o] = p;
        if (topk_renorm) topk_renorm[o] = q;
    }
    if (lane == 0) {
        if (topk_entropy) topk_entropy[row] = hk;
        if (alpha) {
            float a = (k == 1) ? 1.0f : 1.0f - hk / logf(static_cast<float>(k));
            alpha[row] = fminf(fmaxf(a, 0.0f), 1.0f);
        }
    }
}

inline int num_chunks(int vocab) { return (vocab + CHUNK - 1) / CHUNK; }
inline size_t stats_bytes(int rows, int vocab) {
    size_t b = static_cast<size_t>(rows) * num_chunks(vocab) * sizeof(ChunkStats);
    return (b + 255) & ~static_cast<size_t>(255);
}

}  // namespace

extern "C" size_t sage_entropy_topk_workspace_bytes(int rows, int vocab, int k) {
    if (rows < 0 || vocab < 1 || k < 1) return 0;
    return stats_bytes(rows, vocab) + static_cast<size_t>(rows) * num_chunks(vocab) * k * sizeof(uint64_t) + 256;
}

extern "C" int sage_entropy_topk(const void* logits, int dtype, int rows, int vocab, long row_stride, int k,
                                 const int* n_valid, int rows_per_group, float* entropy, int* topk_idx,
                                 float* topk_prob, float* topk_renorm, float* topk_entropy, float* alpha,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    if (!logits || !topk_idx || !workspace) return SAGE_INVALID_ARG;
    if (rows < 0 || vocab < 1 || k < 1 || k > SAGE_MAX_TOPK || k > vocab || row_stride < vocab) return SAGE_INVALID_ARG;
    if (dtype != SAGE_F32 && dtype != SAGE_BF16) return SAGE_INVALID_ARG;
    if (n_valid && rows_per_group < 1) return SAGE_INVALID_ARG;
    const size_t esz = dtype == SAGE_F32 ? 4 : 2;
    if (!sage::aligned(logits, 16) || (static_cast<size_t>(row_stride) * esz) % 16 != 0 || !sage::aligned(workspace, 16))
        return SAGE_INVALID_ARG;
    const int nchunks = num_chunks(vocab);
    if (nchunks > 1024) return SAGE_UNSUPPORTED;
    if (rows > 65535) return SAGE_UNSUPPORTED;
    if (workspace_bytes < sage_entropy_topk_workspace_bytes(rows, vocab, k)) return SAGE_WORKSPACE_TOO_SMALL;
    if (rows == 0) return SAGE_OK;

    ChunkStats* stats = static_cast<ChunkStats*>(workspace);
    uint64_t* keys = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + stats_bytes(rows, vocab));
    hipStream_t s = sage::as_stream(stream);
    const dim3 grid(nchunks, rows);
    if (dtype == SAGE_F32)
        hipLaunchKernelGGL(chunk_kernel<float>, grid, dim3(THREADS), 0, s, static_cast<const float*>(logits), vocab,
                           row_stride, k, n_valid, rows_per_group, nchunks, stats, keys);
    else
        hipLaunchKernelGGL(chunk_kernel<uint16_t>, grid, dim3(THREADS), 0, s, static_cast<const uint16_t*>(logits), vocab,
                           row_stride, k, n_valid, rows_per_group, nchunks, stats, keys);
    if (hipGetLastError() != hipSuccess) return SAGE_LAUNCH_FAILED;
    hipLaunchKernelGGL(merge_kernel, dim3(rows), dim3(64), 0, s, k, n_valid, rows_per_group, nchunks, stats, keys, entropy,
                       topk_idx, topk_prob, topk_renorm, topk_entropy, alpha);
    return sage::launch_status();
}
