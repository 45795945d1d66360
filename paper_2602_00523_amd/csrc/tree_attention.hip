// sage_tree_attention entry point: argument checks and dispatch to the fp32 FMA kernel or the bf16 MFMA kernel.
// Operation: attention of the verify pass under the tree mask (Sec. 2.2; Alg. 1 Phase 2).
#include "sage_internal.h"

namespace sage {
int tree_attention_f32(const void*, const void*, const void*, const void*, const void*, void*, int, int, int, int,
                       const int64_t*, const int*, long, long, const uint64_t*, const int*, float, hipStream_t);
int tree_attention_bf16(const void*, const void*, const void*, const void*, const void*, void*, int, int, int, int,
                        const int64_t*, const int*, int, long, long, const uint64_t*, const int*, float, void*, size_t,
                        hipStream_t);
size_t attention_bf16_workspace_bytes(int B, int Hkv, int G, int max_kv_len);
}  // namespace sage

extern "C" size_t sage_tree_attention_workspace_bytes(int dtype, int B, int Hq, int Hkv, int d, int max_kv_len) {
    (void)d;
    if (dtype != SAGE_BF16 || B < 1 || Hkv < 1 || Hq < Hkv || max_kv_len < 0) return 256;
    return sage::attention_bf16_workspace_bytes(B, Hkv, Hq / Hkv, max_kv_len) + 256;
}

extern "C" int sage_tree_attention(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O,
                                   int dtype, int B, int Hq, int Hkv, int d, const int64_t* kv_start, const int* kv_len,
                                   int max_kv_len, long kv_token_stride, long kv_head_stride, const uint64_t* anc_mask,
                                   const int* n_nodes, float scale, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    if (!Q || !Kc || !Vc || !Kt || !Vt || !O || !kv_start || !kv_len || !anc_mask || !n_nodes) return SAGE_INVALID_ARG;
    if (B < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || d < 1 || max_kv_len < 0) return SAGE_INVALID_ARG;
    if (kv_head_stride < d || kv_token_stride < d) return SAGE_INVALID_ARG;
    if (!(scale > 0.0f) || !(scale < 3.0e38f)) return SAGE_INVALID_ARG;
    if (dtype != SAGE_F32 && dtype != SAGE_BF16) return SAGE_INVALID_ARG;
    if (B == 0) return SAGE_OK;
    hipStream_t s = sage::as_stream(stream);
    if (dtype == SAGE_F32)
        return sage::tree_attention_f32(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, kv_token_stride,
                                        kv_head_stride, anc_mask, n_nodes, scale, s);
    if (!workspace) return SAGE_INVALID_ARG;
    return sage::tree_attention_bf16(Q, Kc, Vc, Kt, Vt, O, B, Hq, Hkv, d, kv_start, kv_len, max_kv_len, kv_token_stride,
                                     kv_head_stride, anc_mask, n_nodes, scale, workspace, workspace_bytes, s);
}

extern "C" const char* sage_build_info(void) { return "libsage_hip gfx950 (MI355X), hand-written HIP"; }
