// Device-side pieces of the calls that close a step (Alg. 1 Phase 3: the accepted tokens join the context; Sec. 3.3
// adaptive history tracking), shared by the kernels of commit_history.hip and by the kernel that runs them right after
// the acceptance rule (fused_steps.hip).
#pragma once
#include "sage_internal.h"

namespace sage {
namespace closing {

// The workgroup copies the K row and the V row of `node`, path entry j of sequence b (Hkv heads x d elements each), to
// cache position len_b + j in 16-byte pieces.
__device__ __forceinline__ void commit_row(
    const unsigned char* __restrict__ Kt, const unsigned char* __restrict__ Vt, unsigned char* __restrict__ Kc,
    unsigned char* __restrict__ Vc, int esz, int Hkv, int d, const int64_t* __restrict__ kv_start, int len_b,
    int kv_capacity, long kv_token_stride, long kv_head_stride, int node, int j, int b) {
    const long pos = static_cast<long>(len_b) + j;
    if (node < 0 || node >= SAGE_MAX_NODES || pos >= kv_capacity) return;      // never read or write out of range
    const int pieces = d * esz / 16;                                           // 16-byte pieces of one head's row
    const long src_row = (static_cast<long>(b) * SAGE_MAX_NODES + node) * Hkv * d * esz;
    const long dst_tok = (kv_start[b] + pos) * kv_token_stride * esz;
    for (int t = threadIdx.x; t < Hkv * pieces; t += blockDim.x) {
        const int g = t / pieces, c = t % pieces;
        const long src = src_row + (static_cast<long>(g) * d * esz) + c * 16;
        const long dst = dst_tok + static_cast<long>(g) * kv_head_stride * esz + c * 16;
        *reinterpret_cast<uint4*>(Kc + dst) = *reinterpret_cast<const uint4*>(Kt + src);
        *reinterpret_cast<uint4*>(Vc + dst) = *reinterpret_cast<const uint4*>(Vt + src);
    }
}

__device__ __forceinline__ int advanced_len(int len_b, int tau, int kv_capacity) {
    const long n = static_cast<long>(len_b) + tau + 1;                        // the root and the tau accepted tokens
    return n > kv_capacity ? kv_capacity : static_cast<int>(n);
}

// One wave for sequence b: lane i holds window slot i.  The new depth limit goes to d_max_out (which may be d_max_in).
__device__ __forceinline__ void history_wave(int b, int lane, int tau, int window, float lo, float hi, int d_floor, int d_cap,
                                             int* __restrict__ hist, int* __restrict__ count, const int* d_max_in,
                                             int* d_max_out, float* __restrict__ avg_out) {
    int* h = hist + static_cast<long>(b) * window;
    const int cnt = count[b];
    const int slot = cnt % window;
    const int n = min(cnt + 1, window);
    int v = 0;
    if (lane < n) v = (lane == slot) ? tau : h[lane];
    const int sum = static_cast<int>(sage::wave_sum_u32(static_cast<uint32_t>(v)));
    if (lane == 0) {
        h[slot] = tau;
        count[b] = cnt + 1;
        const float fs = static_cast<float>(sum), fn = static_cast<float>(n);
        if (avg_out) avg_out[b] = __fdiv_rn(fs, fn);
        int dm = d_max_in[b];
        if (fs < __fmul_rn(lo, fn)) dm -= 1;                                   // strictly below the lower threshold
        else if (fs > __fmul_rn(hi, fn)) dm += 1;                              // strictly above the upper one
        d_max_out[b] = min(max(dm, d_floor), d_cap);
    }
}

}  // namespace closing
}  // namespace sage
