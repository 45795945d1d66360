// sage_commit_path / sage_advance_kv_len: the accepted tokens join the context (Alg. 1 Phase 3, Sec. 2.2): their
// keys and values are appended to the KV cache and the sequence length advances.
// sage_update_history: adaptive history tracking (Sec. 3.3; window and thresholds of Sec. 5 "Implementation
// details"): a sliding window of acceptance lengths steers the maximum tree depth of every sequence.
// All three are byte/integer work of a few KB per step: one small kernel each, no workspace; sage_close_step does the
// three in one launch.
#include "commit_device.h"

using namespace sage::closing;

namespace {

// One workgroup per (path slot j, sequence b).
__global__ __launch_bounds__(256) void commit_path_kernel(
    const unsigned char* __restrict__ Kt, const unsigned char* __restrict__ Vt, unsigned char* __restrict__ Kc,
    unsigned char* __restrict__ Vc, int esz, int Hkv, int d, const int64_t* __restrict__ kv_start,
    const int* __restrict__ kv_len, int kv_capacity, long kv_token_stride, long kv_head_stride,
    const int* __restrict__ path_nodes, const int* __restrict__ accept_len, int path_cap) {
    const int j = blockIdx.x, b = blockIdx.y;
    if (j > accept_len[b] || j >= path_cap) return;
    commit_row(Kt, Vt, Kc, Vc, esz, Hkv, d, kv_start, kv_len[b], kv_capacity, kv_token_stride, kv_head_stride,
               path_nodes[static_cast<long>(b) * path_cap + j], j, b);
}

__global__ void advance_kv_len_kernel(int* __restrict__ kv_len, const int* __restrict__ accept_len, int B, int kv_capacity) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    kv_len[b] = advanced_len(kv_len[b], accept_len[b], kv_capacity);
}

__global__ __launch_bounds__(64) void update_history_kernel(const int* __restrict__ accept_len, int window, float lo, float hi,
                                                            int d_floor, int d_cap, int* __restrict__ hist,
                                                            int* __restrict__ count, int* d_max, float* __restrict__ avg_out) {
    history_wave(blockIdx.x, threadIdx.x, accept_len[blockIdx.x], window, lo, hi, d_floor, d_cap, hist, count, d_max, d_max,
                 avg_out);
}

// sage_close_step: one workgroup per sequence does what the three kernels above do, in their order: every path row is
// copied against the old length (read once, before anything is written), then thread 0 advances the length and wave 0
// updates the history.
__global__ __launch_bounds__(256) void close_step_kernel(
    const unsigned char* __restrict__ Kt, const unsigned char* __restrict__ Vt, unsigned char* __restrict__ Kc,
    unsigned char* __restrict__ Vc, int esz, int Hkv, int d, const int64_t* __restrict__ kv_start, int* kv_len,
    int kv_capacity, long kv_token_stride, long kv_head_stride, const int* __restrict__ path_nodes,
    const int* __restrict__ accept_len, int path_cap, int window, float lo, float hi, int d_floor, int d_cap,
    int* __restrict__ hist, int* __restrict__ count, const int* d_max_in, int* d_max_out, float* __restrict__ avg_out) {
    const int b = blockIdx.x;
    const int tau = accept_len[b];
    const int len_b = kv_len[b];
    for (int j = 0; j <= tau && j < path_cap; ++j)
        commit_row(Kt, Vt, Kc, Vc, esz, Hkv, d, kv_start, len_b, kv_capacity, kv_token_stride, kv_head_stride,
                   path_nodes[static_cast<long>(b) * path_cap + j], j, b);
    __syncthreads();                                                           // every thread has read the old length
    if (threadIdx.x == 0) kv_len[b] = advanced_len(len_b, tau, kv_capacity);
    if (threadIdx.x < 64) history_wave(b, threadIdx.x, tau, window, lo, hi, d_floor, d_cap, hist, count, d_max_in, d_max_out, avg_out);
}

}  // namespace

extern "C" int sage_commit_path(const void* Kt, const void* Vt, void* Kc, void* Vc, int dtype, int B, int Hkv, int d,
                                const int64_t* kv_start, const int* kv_len, int kv_capacity, long kv_token_stride,
                                long kv_head_stride, const int* path_nodes, const int* accept_len, int path_cap,
                                void* stream) {
    if (!Kt || !Vt || !Kc || !Vc || !kv_start || !kv_len || !path_nodes || !accept_len) return SAGE_INVALID_ARG;
    if (dtype != SAGE_F32 && dtype != SAGE_BF16) return SAGE_INVALID_ARG;
    if (B < 0 || Hkv < 1 || d < 1 || path_cap < 1 || kv_capacity < 0) return SAGE_INVALID_ARG;
    if (kv_head_stride < d || kv_token_stride < d) return SAGE_INVALID_ARG;
    const int esz = dtype == SAGE_F32 ? 4 : 2;
    if ((static_cast<long>(d) * esz) % 16 != 0 || (kv_token_stride * esz) % 16 != 0 || (kv_head_stride * esz) % 16 != 0)
        return SAGE_INVALID_ARG;
    if (!sage::aligned(Kt, 16) || !sage::aligned(Vt, 16) || !sage::aligned(Kc, 16) || !sage::aligned(Vc, 16))
        return SAGE_INVALID_ARG;
    if (B > 65535 || path_cap > SAGE_MAX_NODES) return SAGE_UNSUPPORTED;
    if (B == 0) return SAGE_OK;
    hipLaunchKernelGGL(commit_path_kernel, dim3(path_cap, B), dim3(256), 0, sage::as_stream(stream),
                       static_cast<const unsigned char*>(Kt), static_cast<const unsigned char*>(Vt),
                       static_cast<unsigned char*>(Kc), static_cast<unsigned char*>(Vc), esz, Hkv, d, kv_start, kv_len,
                       kv_capacity, kv_token_stride, kv_head_stride, path_nodes, accept_len, path_cap);
    return sage::launch_status();
}

extern "C" int sage_advance_kv_len(int* kv_len, const int* accept_len, int B, int kv_capacity, void* stream) {
    if (!kv_len || !accept_len || B < 0 || kv_capacity < 0) return SAGE_INVALID_ARG;
    if (B == 0) return SAGE_OK;
    hipLaunchKernelGGL(advance_kv_len_kernel, dim3((B + 255) / 256), dim3(256), 0, sage::as_stream(stream), kv_len,
                       accept_len, B, kv_capacity);
    return sage::launch_status();
}

extern "C" int sage_update_history(const int* accept_len, int B, int window, float lo, float hi, int d_floor, int d_cap,
                                   int* hist, int* count, int* d_max, float* avg_out, void* stream) {
    if (!accept_len || !hist || !count || !d_max || B < 0) return SAGE_INVALID_ARG;
    if (window < 1 || window > 64 || d_floor < 1 || d_floor > d_cap || d_cap > SAGE_MAX_DEPTH || !(lo <= hi))
        return SAGE_INVALID_ARG;
    if (B == 0) return SAGE_OK;
    hipLaunchKernelGGL(update_history_kernel, dim3(B), dim3(64), 0, sage::as_stream(stream), accept_len, window, lo, hi,
                       d_floor, d_cap, hist, count, d_max, avg_out);
    return sage::launch_status();
}

extern "C" int sage_close_step(const void* Kt, const void* Vt, void* Kc, void* Vc, int dtype, int B, int Hkv, int d,
                               const int64_t* kv_start, int* kv_len, int kv_capacity, long kv_token_stride,
                               long kv_head_stride, const int* path_nodes, const int* accept_len, int path_cap, int window,
                               float lo, float hi, int d_floor, int d_cap, int* hist, int* count, const int* d_max_in,
                               int* d_max_out, float* avg_out, void* stream) {
    if (!Kt || !Vt || !Kc || !Vc || !kv_start || !kv_len || !path_nodes || !accept_len) return SAGE_INVALID_ARG;
    if (!hist || !count || !d_max_in || !d_max_out) return SAGE_INVALID_ARG;
    if (dtype != SAGE_F32 && dtype != SAGE_BF16) return SAGE_INVALID_ARG;
    if (B < 0 || Hkv < 1 || d < 1 || path_cap < 1 || kv_capacity < 0) return SAGE_INVALID_ARG;
    if (kv_head_stride < d || kv_token_stride < d) return SAGE_INVALID_ARG;
    const int esz = dtype == SAGE_F32 ? 4 : 2;
    if ((static_cast<long>(d) * esz) % 16 != 0 || (kv_token_stride * esz) % 16 != 0 || (kv_head_stride * esz) % 16 != 0)
        return SAGE_INVALID_ARG;
    if (!sage::aligned(Kt, 16) || !sage::aligned(Vt, 16) || !sage::aligned(Kc, 16) || !sage::aligned(Vc, 16))
        return SAGE_INVALID_ARG;
    if (window < 1 || window > 64 || d_floor < 1 || d_floor > d_cap || d_cap > SAGE_MAX_DEPTH || !(lo <= hi))
        return SAGE_INVALID_ARG;
    if (B > 65535 || path_cap > SAGE_MAX_NODES) return SAGE_UNSUPPORTED;
    if (B == 0) return SAGE_OK;
    hipLaunchKernelGGL(close_step_kernel, dim3(B), dim3(256), 0, sage::as_stream(stream),
                       static_cast<const unsigned char*>(Kt), static_cast<const unsigned char*>(Vt),
                       static_cast<unsigned char*>(Kc), static_cast<unsigned char*>(Vc), esz, Hkv, d, kv_start, kv_len,
                       kv_capacity, kv_token_stride, kv_head_stride, path_nodes, accept_len, path_cap, window, lo, hi, d_floor,
                       d_cap, hist, count, d_max_in, d_max_out, avg_out);
    return sage::launch_status();
}
