// Pieces shared by the kernels that reduce vocabulary-sized rows to softmax statistics and top-k candidates
// (stored logits in entropy_topk.hip, logits computed on the fly in lm_head_topk.hip) and by their common second pass.
#pragma once
#include "sage_internal.h"

namespace sage {
namespace topk {

// Softmax statistics of a slice relative to its own maximum m: Z = sum exp(x - m), T = sum exp(x - m) (m - x).
struct UnitStats { float m, Z, T, pad; };

// Order-preserving map float -> uint32 (larger float -> larger code); -0 is folded into +0 so that equal
// values compare equal before the index tie-break.
__host__ __device__ __forceinline__ uint32_t sortable(float v) {
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    if (u == 0x80000000u) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__host__ __device__ __forceinline__ float unsortable(uint32_t s) {
    uint32_t u = (s & 0x80000000u) ? (s & 0x7FFFFFFFu) : ~s;
    return __builtin_bit_cast(float, u);
}
// key: high word = value code, low word = ~index, so a larger key is a better candidate; 0 = no candidate.
struct Key { uint32_t hi, lo; };
__host__ __device__ __forceinline__ Key make_key(float v, int idx) { return Key{sortable(v), 0xFFFFFFFFu - static_cast<uint32_t>(idx)}; }
__host__ __device__ __forceinline__ bool key_less(Key a, Key b) { return a.hi < b.hi || (a.hi == b.hi && a.lo < b.lo); }
__host__ __device__ __forceinline__ bool key_equal(Key a, Key b) { return a.hi == b.hi && a.lo == b.lo; }
__host__ __device__ __forceinline__ bool key_none(Key a) { return (a.hi | a.lo) == 0; }
__host__ __device__ __forceinline__ Key key_max(Key a, Key b) { return key_less(a, b) ? b : a; }
__host__ __device__ __forceinline__ int key_index(Key k) { return static_cast<int>(0xFFFFFFFFu - k.lo); }
__host__ __device__ __forceinline__ float key_value(Key k) { return unsortable(k.hi); }
__host__ __device__ __forceinline__ uint64_t key_pack(Key k) { return (static_cast<uint64_t>(k.hi) << 32) | k.lo; }
__host__ __device__ __forceinline__ Key key_unpack(uint64_t v) { return Key{static_cast<uint32_t>(v >> 32), static_cast<uint32_t>(v)}; }

}  // namespace topk

int topk_max_units();
void topk_workspace_layout(int rows, int vocab, void* workspace, topk::UnitStats** stats, uint64_t** keys, int* nunits);
void topk_merge(int rows, int k, const int* n_valid, int rows_per_group, int nunits, const topk::UnitStats* stats,
                const uint64_t* keys, float* entropy, int* topk_idx, float* topk_prob, float* topk_renorm,
                float* topk_entropy, float* alpha, hipStream_t s);

}  // namespace sage
