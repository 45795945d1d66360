// sage_tree_attention, fp32 instantiation: tree-masked GQA attention of the verify pass (Sec. 2.2 tree mask;
// Alg. 1 Phase 2) in plain fp32 FMA arithmetic.  Used for small full-precision shapes; the bf16 MFMA kernel
// carries the 72B-shape workloads.
//
// One workgroup per (node, query head, sequence).  Keys are taken 256 at a time: lane = key for the scores
// (q broadcast from LDS, the key row read with 16-byte loads), then thread = (output dimension, slice of the block's
// keys) for the probability-weighted sum of values (coalesced across the dimension, eight independent loads in
// flight per thread), with an online softmax across blocks; the key slices are summed through LDS at the end.
// The tree's own keys form the last block, admitted by the node's ancestor-or-self mask.
#include "sage_internal.h"

namespace {

constexpr int THREADS = 256;

__device__ __forceinline__ float block_reduce(float v, float* s_red, bool is_max) {
    v = is_max ? sage::wave_max(v) : sage::wave_sum(v);
    __syncthreads();                         // s_red may still be read from a previous reduction
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int i = 1; i < THREADS / 64; ++i) r = is_max ? fmaxf(r, s_red[i]) : r + s_red[i];
    return r;
}

__global__ __launch_bounds__(THREADS) void tree_attention_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ Kc, const float* __restrict__ Vc,
    const float* __restrict__ Kt, const float* __restrict__ Vt, float* __restrict__ O, int Hq, int Hkv, int d,
    const int64_t* __restrict__ kv_start, const int* __restrict__ kv_len, long kv_token_stride, long kv_head_stride,
    const uint64_t* __restrict__ anc_mask, const int* __restrict__ n_nodes, const int* __restrict__ first_node, float scale) {
    __shared__ float s_q[256];
    __shared__ float s_p[THREADS];
    __shared__ float s_red[THREADS / 64];

    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    int n = n_nodes[b];
    n = n < 1 ? 1 : (n > SAGE_MAX_NODES ? SAGE_MAX_NODES : n);   // a tree always has its root
    int first = first_node ? first_node[b] : 0;             // rows of earlier nodes are not asked for
    first = first < 0 ? 0 : (first > n - 1 ? n - 1 : first);
    if (i >= n || i < first) return;
    const int tid = threadIdx.x;
    const int g = h / (Hq / Hkv);
    const int L = kv_len[b] > 0 ? kv_len[b] : 0;
    const long qoff = ((static_cast<long>(b) * SAGE_MAX_NODES + i) * Hq + h) * d;
    const uint64_t mask = anc_mask[static_cast<long>(b) * SAGE_MAX_NODES + i];
    if (tid < d) s_q[tid] = Q[qoff + tid];
    __syncthreads();

    const float* kbase = Kc + kv_start[b] * kv_token_stride + static_cast<long>(g) * kv_head_stride;
    const float* vbase = Vc + kv_start[b] * kv_token_stride + static_cast<long>(g) * kv_head_stride;
    const float* ktree = Kt + (static_cast<long>(b) * SAGE_MAX_NODES * Hkv + g) * d;
    const float* vtree = Vt + (static_cast<long>(b) * SAGE_MAX_NODES * Hkv + g) * d;
    const long tree_stride = static_cast<long>(Hkv) * d;

    const int dpad = d <= 64 ? 64 : (d <= 128 ? 128 : 256);  // threads per key slice in the value pass
    const int nslices = THREADS / dpad;
    const int dim = tid % dpad, slice = tid / dpad;
    float m = -INFINITY, l = 0.f, acc = 0.f;
    const int nblocks = (L + THREADS - 1) / THREADS + 1;     // cache blocks, then one block of tree keys
    for (int blk = 0; blk < nblocks; ++blk) {
        const bool tree = (blk == nblocks - 1);
        const int j = tree ? tid : blk * THREADS + tid;
        const bool admitted = tree ? (tid < n && ((mask >> tid) & 1)) : (j < L);
        const float* krow = tree ? ktree + j * tree_stride : kbase + j * kv_token_stride;
        float s = -INFINITY;
        if (admitted) {
            float a = 0.f;
            for (int c = 0; c < d; c += 4) {
                const float4 kv = *reinterpret_cast<const float4*>(krow + c);
                a = fmaf(s_q[c], kv.x, a);
                a = fmaf(s_q[c + 1], kv.y, a);
                a = fmaf(s_q[c + 2], kv.z, a);
                a = fmaf(s_q[c + 3], kv.w, a);
            }
            s = a * scale;
        }
        const float bm = block_reduce(s, s_red, true);
        const float m_new = fmaxf(m, bm);
        if (m_new == -INFINITY) continue;                    // nothing admitted so far (uniform across the workgroup)
        const float p = admitted ? expf(s - m_new) : 0.f;
        const float corr = (m == -INFINITY) ? 0.f : expf(m - m_new);
        const float bl = block_reduce(p, s_red, false);
        l = l * corr + bl;
        m = m_new;
        __syncthreads();                                     // previous block's s_p fully consumed
        s_p[tid] = p;
        __syncthreads();
        acc *= corr;
        if (dim < d) {
            const int cnt = tree ? n : min(THREADS, L - blk * THREADS);
            const float* vcol = (tree ? vtree : vbase + static_cast<long>(blk) * THREADS * kv_token_stride) + dim;
            const long vstride = tree ? tree_stride : kv_token_stride;
            int t = slice;
            for (; t + 7 * nslices < cnt; t += 8 * nslices) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = vcol[(t + u * nslices) * vstride];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const float pt = s_p[t + u * nslices];
                    acc = (pt != 0.f) ? fmaf(pt, v[u], acc) : acc;
                }
            }
            for (; t < cnt; t += nslices) {
                const float pt = s_p[t];
                if (pt != 0.f) acc = fmaf(pt, vcol[t * vstride], acc);
            }
        }
    }
    __syncthreads();                                         // s_p is free: sum the key slices
    s_p[tid] = acc;
    __syncthreads();
    if (tid < d) {
        float sum = 0.f;
        for (int sl = 0; sl < nslices; ++sl) sum += s_p[tid + sl * dpad];
        O[qoff + tid] = sum / l;
    }
}

}  // namespace

namespace sage {

int tree_attention_f32(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O, int B,
                       int Hq, int Hkv, int d, const int64_t* kv_start, const int* kv_len, long kv_token_stride,
                       long kv_head_stride, const uint64_t* anc_mask, const int* n_nodes, const int* first_node,
                       float scale, hipStream_t stream) {
    if (d < 4 || d > 256 || (d % 4) != 0) return SAGE_UNSUPPORTED;
    if ((kv_token_stride % 4) != 0 || (kv_head_stride % 4) != 0) return SAGE_INVALID_ARG;
    if (Hq > 65535 || B > 65535) return SAGE_UNSUPPORTED;
    hipLaunchKernelGGL(tree_attention_f32_kernel, dim3(SAGE_MAX_NODES, Hq, B), dim3(THREADS), 0, stream,
                       static_cast<const float*>(Q), static_cast<const float*>(Kc), static_cast<const float*>(Vc),
                       static_cast<const float*>(Kt), static_cast<const float*>(Vt), static_cast<float*>(O), Hq, Hkv, d,
                       kv_start, kv_len, kv_token_stride, kv_head_stride, anc_mask, n_nodes, first_node, scale);
    return launch_status();
}

}  // namespace sage
