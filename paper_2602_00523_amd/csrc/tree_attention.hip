// sage_tree_attention entry point: argument checks and dispatch to the fp32 FMA kernel or the bf16 MFMA kernel.
// Operation: attention of the verify pass under the tree mask (Sec. 2.2; Alg. 1 Phase 2).
// sage_tree_attention_with_plan: the same, with the planning of the next tree (Sec. 3.1-3.2) riding in the launch.
#include <mutex>

#include "plan_device.h"
#include "sage_internal.h"

namespace sage {
int tree_attention_f32(const void*, const void*, const void*, const void*, const void*, void*, int, int, int, int,
                       const int64_t*, const int*, long, long, const uint64_t*, const int*, const int*, float, hipStream_t);
int tree_attention_bf16(const void*, const void*, const void*, const void*, const void*, void*, int, int, int, int,
                        const int64_t*, const int*, int, long, long, const uint64_t*, const int*, const int*, float, void*,
                        size_t, hipStream_t, const PlanArgs*);
bool attention_bf16_can_carry_plan(const PlanArgs&);
size_t attention_bf16_workspace_bytes(int B, int Hkv, int G, int max_kv_len);
int plan_args_from_slices(void*, int, int, int, const sage_tree_params*, const int*, float*, int*, float*, float*, float*, float*,
                          int*, int*, int*, int*, uint64_t*, float*, int*, PlanArgs*);
int launch_plan(const PlanArgs&, int, hipStream_t);
}  // namespace sage

// Checks common to both entry points; SAGE_OK means the call may be dispatched.
static int check_attention_args(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, const void* O,
                                int dtype, int B, int Hq, int Hkv, int d, const int64_t* kv_start, const int* kv_len,
                                int max_kv_len, long kv_token_stride, long kv_head_stride, const uint64_t* anc_mask,
                                const int* n_nodes, float scale) {
    if (!Q || !Kc || !Vc || !Kt || !Vt || !O || !kv_start || !kv_len || !anc_mask || !n_nodes) return SAGE_INVALID_ARG;
    if (B < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || d < 1 || max_kv_len < 0) return SAGE_INVALID_ARG;
    if (kv_head_stride < d || kv_token_stride < d) return SAGE_INVALID_ARG;
    if (!(scale > 0.0f) || !(scale < 3.0e38f)) return SAGE_INVALID_ARG;
    if (dtype != SAGE_F32 && dtype != SAGE_BF16) return SAGE_INVALID_ARG;
    return SAGE_OK;
}

extern "C" size_t sage_tree_attention_workspace_bytes(int dtype, int B, int Hq, int Hkv, int d, int max_kv_len) {
    (void)d;
    if (dtype != SAGE_BF16 || B < 1 || Hkv < 1 || Hq < Hkv || max_kv_len < 0) return 256;
    return sage::attention_bf16_workspace_bytes(B, Hkv, Hq / Hkv, max_kv_len) + 256;
}

extern "C" int sage_tree_attention(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O,
                                   int dtype, int B, int Hq, int Hkv, int d, const int64_t* kv_start, const int* kv_len,
                                   int max_kv_len, long kv_token_stride, long kv_head_stride, const uint64_t* anc_mask,
                                   const int* n_nodes, const int* first_node, float scale, void* workspace,
                                   size_t workspace_bytes, void* stream) {
    const int rc = check_attention_args(Q, Kc, Vc, Kt, Vt, O, dtype, B, Hq, Hkv, d, kv_start, kv_len, max_kv_len, kv_token_stride,
                                        kv_head_stride, anc_mask, n_nodes, scale);
    if (rc != SAGE_OK || B == 0) return rc;
    hipStream_t s = sage::as_stream(stream);
    if (dtype == SAGE_F32)
        return sage::tree_attention_f32(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, kv_token_stride,
                                        kv_head_stride, anc_mask, n_nodes, first_node, scale, s);
    if (!workspace) return SAGE_INVALID_ARG;
    return sage::tree_attention_bf16(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, max_kv_len, kv_token_stride,
                                     kv_head_stride, anc_mask, n_nodes, first_node, scale, workspace, workspace_bytes, s, nullptr);
}

// ---- sage_tree_attention_static: the same call for callers that cannot hand over a workspace they allocated
// (code under graph capture, serving loops that must not call the allocator).  The split partials go to a
// file-scope device array instead.  In host code the array's name only stands for the symbol: its device address
// is looked up once per device and every use below goes through that address.
#define SAGE_STATIC_SCRATCH_BYTES (40u << 20)
static __device__ __align__(256) unsigned char scratch[SAGE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex scratch_lock;
void* scratch_ptr[MAX_DEVICES];          // per device: every GPU holds its own copy of the array at its own address

// Device address of `scratch` on the current device (looked up on the first call there); nullptr on failure.
void* scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}
}  // namespace

extern "C" size_t sage_tree_attention_static_scratch_bytes(void) { return SAGE_STATIC_SCRATCH_BYTES; }

extern "C" int sage_tree_attention_static(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O,
                                          int dtype, int B, int Hq, int Hkv, int d, const int64_t* kv_start,
                                          const int* kv_len, int max_kv_len, long kv_token_stride, long kv_head_stride,
                                          const uint64_t* anc_mask, const int* n_nodes, float scale, void* stream) {
    const int rc = check_attention_args(Q, Kc, Vc, Kt, Vt, O, dtype, B, Hq, Hkv, d, kv_start, kv_len, max_kv_len, kv_token_stride,
                                        kv_head_stride, anc_mask, n_nodes, scale);
    if (rc != SAGE_OK || B == 0) return rc;
    hipStream_t s = sage::as_stream(stream);
    if (dtype == SAGE_F32)               // no scratch in this path
        return sage::tree_attention_f32(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, kv_token_stride,
                                        kv_head_stride, anc_mask, n_nodes, nullptr, scale, s);
    // sizes whose partials do not fit the array are refused, nothing is enqueued
    if (sage_tree_attention_workspace_bytes(dtype, B, Hq, Hkv, d, max_kv_len) > SAGE_STATIC_SCRATCH_BYTES)
        return SAGE_WORKSPACE_TOO_SMALL;
    void* ws = scratch_of_current_device();
    if (!ws) return SAGE_LAUNCH_FAILED;
    // Every partial slot the merge reads is written by the main kernel of the same call first, so nothing of an earlier
    // call's contents has to be cleared.
    return sage::tree_attention_bf16(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, max_kv_len, kv_token_stride,
                                     kv_head_stride, anc_mask, n_nodes, nullptr, scale, ws, SAGE_STATIC_SCRATCH_BYTES, s, nullptr);
}

extern "C" int sage_tree_attention_with_plan(
    const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O, int dtype, int B, int Hq, int Hkv,
    int d, const int64_t* kv_start, const int* kv_len, int max_kv_len, long kv_token_stride, long kv_head_stride,
    const uint64_t* anc_mask, const int* n_nodes, float scale, void* workspace, size_t workspace_bytes, void* slices, int vocab,
    int k, const sage_tree_params* params, const int* d_max_seq, float* entropy, int* topk_idx, float* topk_prob,
    float* topk_renorm, float* topk_entropy, float* alpha, int* next_n_nodes, int* next_parent, int* next_depth, int* next_rank,
    uint64_t* next_anc_mask, float* next_cum_prob, int* next_node_token, void* stream) {
    int rc = check_attention_args(Q, Kc, Vc, Kt, Vt, O, dtype, B, Hq, Hkv, d, kv_start, kv_len, max_kv_len, kv_token_stride,
                                  kv_head_stride, anc_mask, n_nodes, scale);
    if (rc != SAGE_OK) return rc;
    sage::PlanArgs pl;
    rc = sage::plan_args_from_slices(slices, vocab, B, k, params, d_max_seq, entropy, topk_idx, topk_prob, topk_renorm, topk_entropy,
                                     alpha, next_n_nodes, next_parent, next_depth, next_rank, next_anc_mask, next_cum_prob,
                                     next_node_token, &pl);
    if (rc != SAGE_OK) return rc;
    // the tree being planned is the next step's: it must not be the one this attention reads
    if (next_n_nodes == n_nodes || next_anc_mask == anc_mask) return SAGE_INVALID_ARG;
    if (dtype == SAGE_BF16 && !workspace) return SAGE_INVALID_ARG;
    if (B == 0) return SAGE_OK;
    hipStream_t s = sage::as_stream(stream);
    if (dtype == SAGE_BF16 && sage::attention_bf16_can_carry_plan(pl))
        return sage::tree_attention_bf16(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, max_kv_len, kv_token_stride,
                                         kv_head_stride, anc_mask, n_nodes, nullptr, scale, workspace, workspace_bytes, s, &pl);
    // fp32, or candidate lists too long for the planning workgroup's LDS: the two launches one after the other
    rc = dtype == SAGE_F32 ? sage::tree_attention_f32(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, kv_token_stride,
                                                      kv_head_stride, anc_mask, n_nodes, nullptr, scale, s)
                           : sage::tree_attention_bf16(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, max_kv_len,
                                                       kv_token_stride, kv_head_stride, anc_mask, n_nodes, nullptr, scale,
                                                       workspace, workspace_bytes, s, nullptr);
    if (rc != SAGE_OK) return rc;
    return sage::launch_plan(pl, B, s);
}

extern "C" const char* sage_build_info(void) { return "libsage_hip gfx950 (MI355X), hand-written HIP"; }
