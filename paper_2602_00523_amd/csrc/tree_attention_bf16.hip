// sage_tree_attention, bf16 MFMA instantiation (head_dim 128): tree-masked GQA attention of the target's
// verify pass (Sec. 2.2 tree mask; Alg. 1 Phase 2) against a long KV cache plus the tree's own keys.
//
// Formulation.  All query rows that share a KV head (node i, head-in-group hg -> row m = i*G + hg, up to 512
// rows) are processed together so each K/V byte is fetched from HBM once.  Everything is computed transposed:
//   S^T = K Q^T   (tokens x rows):  A operand = K rows straight from the cache layout (16-byte reads),
//                                   B operand = Q rows held in registers for the whole kernel;
//   O^T = V^T P^T (dims x rows):    A operand = V^T from LDS, B operand = P^T.
// In the 32x32 MFMA accumulator layout a lane owns ONE query row (column lane%32) and 16 tokens of it, so the
// softmax max/sum are in-register reductions plus a single cross-half exchange, the rescale factor is a per-lane
// scalar, and the accumulator registers of S^T are, as they stand, the B operand of the PV product (the token
// order inside a k-block is whatever the accumulator layout says; V^T is staged in LDS in that same order).
//
// Decomposition (decided on the device from n_nodes/kv_len, so no host round trip): a workgroup of 4 waves
// owns (sequence, KV head, group of 4 column tiles = 128 query rows, KV split); wave w owns column tile w of
// the group.  Workgroups of one KV head are congruent modulo the KV-head count, which with 8 KV heads pins a
// head to one XCD and its L2: column groups of the same split re-read K/V from that L2, not from HBM.
// K/V tiles of 64 tokens are double-buffered in LDS (register-staged loads one tile ahead; V is transposed in
// registers on the way in).  Each workgroup writes an un-normalised partial (max, sum, O^T); a second kernel
// merges the splits in a fixed order (deterministic, no float atomics) and writes bf16.
#include "sage_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;                  // head_dim
constexpr int TILE = 64;                // tokens per LDS stage
constexpr int THREADS = 256;
constexpr int CT_PER_WG = 4;            // column tiles (of 32 query rows) per workgroup
constexpr int ROWS_PER_WG = CT_PER_WG * 32;
constexpr int K_ROW_B = 272;            // LDS bytes per K token row (256 + 16 pad: 17 x 16 B, conflict-free b128 reads)
constexpr int V_ROW_B = 144;            // LDS bytes per V^T dim row (128 + 16 pad: 9 x 16 B)
constexpr int K_BYTES = TILE * K_ROW_B;
constexpr int V_BYTES = D * V_ROW_B;
constexpr int STAGE_BYTES = K_BYTES + V_BYTES;
constexpr int PART_FLOATS = D + 2;      // per query row: O^T[128] in LDS-row order, then max, sum

struct Params {
    const uint16_t* Q; const uint16_t* Kc; const uint16_t* Vc; const uint16_t* Kt; const uint16_t* Vt;
    uint16_t* O;
    const int64_t* kv_start; const int* kv_len; const uint64_t* anc_mask; const int* n_nodes;
    float* part;                         // [B][Hkv][nslot][ROWS_PER_WG][PART_FLOATS]
    long kv_token_stride, kv_head_stride;
    int B, Hq, Hkv, G, nslot;
    float scale_log2e;                   // softmax scale times log2(e): probabilities are exp2 of scaled differences
};

// How one (sequence, KV head) is cut into workgroups; evaluated identically by both kernels.
struct Split {
    int n, rows, col_groups, tiles, tiles_per_split, nsplit;
};
__device__ __forceinline__ Split make_split(int n_nodes, int kv_len, int G, int nslot) {
    Split s;
    s.n = n_nodes < 1 ? 1 : (n_nodes > SAGE_MAX_NODES ? SAGE_MAX_NODES : n_nodes);
    s.rows = s.n * G;
    s.col_groups = (s.rows + ROWS_PER_WG - 1) / ROWS_PER_WG;
    const int L = kv_len > 0 ? kv_len : 0;
    s.tiles = (L + TILE - 1) / TILE + 1;                    // cache tiles, then one tile holding the tree's keys
    int max_split = nslot / s.col_groups;
    if (max_split < 1) max_split = 1;
    s.tiles_per_split = (s.tiles + max_split - 1) / max_split;
    s.nsplit = (s.tiles + s.tiles_per_split - 1) / s.tiles_per_split;
    return s;
}

__device__ __forceinline__ bf16x8 lds_frag(const unsigned char* p) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p));
}

__global__ __launch_bounds__(THREADS, 2) void tree_attention_bf16_kernel(const Params prm) {
    __shared__ __align__(16) unsigned char smem[2 * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r32 = lane & 31;           // MFMA row (A) / column (B, C) owned by this lane
    const int half = lane >> 5;

    int id = blockIdx.x;
    const int g = id % prm.Hkv; id /= prm.Hkv;
    const int slot = id % prm.nslot;
    const int b = id / prm.nslot;
    const int L = prm.kv_len[b] > 0 ? prm.kv_len[b] : 0;
    const Split sp = make_split(prm.n_nodes[b], L, prm.G, prm.nslot);
    if (sp.col_groups > prm.nslot) return;                  // host guarantees nslot >= the largest group count
    const int cg = slot % sp.col_groups;
    const int split = slot / sp.col_groups;
    if (split >= sp.nsplit) return;
    const int t_begin = split * sp.tiles_per_split;
    const int t_end = min(sp.tiles, t_begin + sp.tiles_per_split);
    const int tree_tile = sp.tiles - 1;

    // ---- this lane's query row
    const int m = cg * ROWS_PER_WG + wave * 32 + r32;       // row within the KV head
    const int node = m / prm.G;
    const bool row_valid = m < sp.rows;
    const bool wave_active = (cg * ROWS_PER_WG + wave * 32) < sp.rows;
    const uint64_t tree_mask = row_valid ? prm.anc_mask[static_cast<long>(b) * SAGE_MAX_NODES + node] : 0ull;

    bf16x8 qf[8];
    {
        const uint16_t* qrow = prm.Q + ((static_cast<long>(b) * SAGE_MAX_NODES + node) * prm.Hq + g * prm.G + (m % prm.G)) * D;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row_valid) v = *reinterpret_cast<const uint4*>(qrow + kk * 16 + half * 8);
            qf[kk] = __builtin_bit_cast(bf16x8, v);
        }
    }

    // ---- loader roles: waves 0,1 stage K (8 rows x 16 chunks per instruction), waves 2,3 stage V transposed
    const bool k_loader = wave < 2;
    const int lu = tid & 127;
    const int chunk = lu & 15;                               // 16-byte chunk (8 dims) of a 256-byte row
    const int lgrp = lu >> 4;                                // K: token row within each group of 8; V: position group
    const uint16_t* cache_base = (k_loader ? prm.Kc : prm.Vc) + prm.kv_start[b] * prm.kv_token_stride +
                                 static_cast<long>(g) * prm.kv_head_stride + chunk * 8;
    const uint16_t* tree_base = (k_loader ? prm.Kt : prm.Vt) + (static_cast<long>(b) * SAGE_MAX_NODES * prm.Hkv + g) * D + chunk * 8;
    const long tree_stride = static_cast<long>(prm.Hkv) * D;

    uint4 stage[8];
    auto issue_loads = [&](int tile) {
        const bool is_tree = (tile == tree_tile);
        const int base = tile * TILE;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int t;                                          // token within the tile
            if (k_loader) {
                t = i * 8 + lgrp;
            } else {                                        // position group lgrp = (sub, j, h); element i of the k-block
                t = 32 * (lgrp >> 2) + 16 * ((lgrp >> 1) & 1) + 8 * (i >> 2) + 4 * (lgrp & 1) + (i & 3);
            }
            const uint16_t* src;
            if (is_tree) {
                src = tree_base + min(t, sp.n - 1) * tree_stride;           // rows past n are masked; keep the read in range
            } else {
                src = cache_base + static_cast<long>(min(base + t, L - 1)) * prm.kv_token_stride;
            }
            stage[i] = *reinterpret_cast<const uint4*>(src);
        }
    };
    auto store_stage = [&](int buf) {
        unsigned char* kb = smem + buf * STAGE_BYTES;
        unsigned char* vb = kb + K_BYTES;
        if (k_loader) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                *reinterpret_cast<uint4*>(kb + (i * 8 + lgrp) * K_ROW_B + chunk * 16) = stage[i];
        } else {
            // 8x8 transpose of 16-bit elements: stage[e] holds dims chunk*8..+7 of token e; row dd of the result
            // holds tokens 0..7 of dim chunk*8+dd.  LDS row order is dd*16 + chunk (consecutive rows per store).
            auto dw = [&](int e, int q) -> uint32_t {      // dims 2q, 2q+1 of token e
                return q == 0 ? stage[e].x : q == 1 ? stage[e].y : q == 2 ? stage[e].z : stage[e].w;
            };
#pragma unroll
            for (int dd = 0; dd < 8; ++dd) {
                const uint32_t sel = (dd & 1) ? 0x07060302u : 0x05040100u;
                uint4 o;
                o.x = __builtin_amdgcn_perm(dw(1, dd / 2), dw(0, dd / 2), sel);
                o.y = __builtin_amdgcn_perm(dw(3, dd / 2), dw(2, dd / 2), sel);
                o.z = __builtin_amdgcn_perm(dw(5, dd / 2), dw(4, dd / 2), sel);
                o.w = __builtin_amdgcn_perm(dw(7, dd / 2), dw(6, dd / 2), sel);
                *reinterpret_cast<uint4*>(vb + (dd * 16 + chunk) * V_ROW_B + lgrp * 16) = o;
            }
        }
    };

    f32x16 acc[4];                                           // O^T: 4 tiles of 32 LDS rows x this lane's query row
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
    float m_run = -INFINITY;                                 // running max of raw (unscaled) scores
    float l_run = 0.f;                                       // this lane's share of the running sum
    const float c = prm.scale_log2e;

    issue_loads(t_begin);
    store_stage(0);
    __syncthreads();

    for (int tile = t_begin; tile < t_end; ++tile) {
        const int buf = (tile - t_begin) & 1;
        const bool has_next = tile + 1 < t_end;
        if (has_next) issue_loads(tile + 1);

        if (wave_active) {
            const unsigned char* kb = smem + buf * STAGE_BYTES;
            const unsigned char* vb = kb + K_BYTES;
            f32x16 s[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[sub][i] = 0.f;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const bf16x8 a = lds_frag(kb + (sub * 32 + r32) * K_ROW_B + kk * 32 + half * 16);
                    s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s[sub], 0, 0, 0);
                }
            }
            // ---- admit keys: cache positions below kv_len; tree nodes in this row's ancestor-or-self mask
            const bool is_tree = (tile == tree_tile);
            if (is_tree || tile * TILE + TILE > L) {
                uint64_t admit;
                if (is_tree) {
                    admit = tree_mask;
                } else {
                    const int left = L - tile * TILE;        // 1..63 valid tokens
                    admit = (1ull << left) - 1ull;
                }
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int t = 32 * sub + 8 * (i >> 2) + 4 * half + (i & 3);
                        if (!((admit >> t) & 1)) s[sub][i] = -INFINITY;
                    }
            }
            // ---- online softmax for this lane's query row
            float tmax = s[0][0];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, s[sub][i]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float m_new = fmaxf(m_run, tmax);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float corr = __builtin_amdgcn_exp2f((m_run - m_safe) * c);   // 0 on the first admitted tile
            const float neg_mc = -m_safe * c;
            float psum = 0.f;
            bf16x8 pf[4];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    bf16x8 frag;
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[sub][8 * j + e], c, neg_mc));
                        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[sub][8 * j + e + 1], c, neg_mc));
                        psum += p0 + p1;
                        const f32x2 pp = {p0, p1};
                        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
                        frag[e] = pb[0];
                        frag[e + 1] = pb[1];
                    }
                    pf[sub * 2 + j] = frag;
                }
            l_run = l_run * corr + psum;
            m_run = m_new;
            if (__any(corr != 1.0f)) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[dt][i] *= corr;
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int kbk = 0; kbk < 4; ++kbk) {
                    const bf16x8 a = lds_frag(vb + (dt * 32 + r32) * V_ROW_B + kbk * 32 + half * 16);
                    acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[kbk], acc[dt], 0, 0, 0);
                }
        }

        if (has_next) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- un-normalised partial for this (split, query row); LDS-row order of dims, merged by the second kernel
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (row_valid) {
        float* out = prm.part + (((static_cast<long>(b) * prm.Hkv + g) * prm.nslot + slot) * ROWS_PER_WG + wave * 32 + r32) * PART_FLOATS;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = make_float4(acc[dt][4 * q], acc[dt][4 * q + 1], acc[dt][4 * q + 2], acc[dt][4 * q + 3]);
                *reinterpret_cast<float4*>(out + dt * 32 + 8 * q + 4 * half) = v;
            }
        if (half == 0) {
            out[D] = m_run;
            out[D + 1] = l_tot;
        }
    }
}

// Merge the splits of one (sequence, node, query head) in split order and write bf16.
__global__ __launch_bounds__(D) void tree_attention_merge_kernel(const Params prm) {
    __shared__ uint16_t s_out[D];
    const int node = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int L = prm.kv_len[b] > 0 ? prm.kv_len[b] : 0;
    const Split sp = make_split(prm.n_nodes[b], L, prm.G, prm.nslot);
    if (node >= sp.n || sp.col_groups > prm.nslot) return;
    const int g = h / prm.G;
    const int m = node * prm.G + (h % prm.G);
    const int cg = m / ROWS_PER_WG;
    const int row = m % ROWS_PER_WG;
    const int p = threadIdx.x;                               // LDS-row index of the partial
    const float c = prm.scale_log2e;
    const float* base = prm.part + ((static_cast<long>(b) * prm.Hkv + g) * prm.nslot) * ROWS_PER_WG * PART_FLOATS;

    float m_all = -INFINITY;
    for (int s = 0; s < sp.nsplit; ++s) {
        const float* part = base + (static_cast<long>(s * sp.col_groups + cg) * ROWS_PER_WG + row) * PART_FLOATS;
        m_all = fmaxf(m_all, part[D]);
    }
    float l_all = 0.f, o = 0.f;
    for (int s = 0; s < sp.nsplit; ++s) {
        const float* part = base + (static_cast<long>(s * sp.col_groups + cg) * ROWS_PER_WG + row) * PART_FLOATS;
        const float ms = part[D];
        if (ms == -INFINITY) continue;
        const float w = __builtin_amdgcn_exp2f((ms - m_all) * c);
        l_all += w * part[D + 1];
        o += w * part[p];
    }
    const int dim = (p & 15) * 8 + (p >> 4);                 // LDS row dd*16 + chunk holds dim chunk*8 + dd
    s_out[dim] = sage::float_to_bf16_bits(o / l_all);
    __syncthreads();
    prm.O[((static_cast<long>(b) * SAGE_MAX_NODES + node) * prm.Hq + h) * D + p] = s_out[p];
}

}  // namespace

namespace sage {

// Number of workgroup slots per (sequence, KV head): enough to cover the device about twice, never more than
// one slot per tile and column group, never fewer than the largest possible number of column groups.
int attention_bf16_slots(int B, int Hkv, int G, int max_kv_len) {
    const int max_groups = (SAGE_MAX_NODES * G + ROWS_PER_WG - 1) / ROWS_PER_WG;
    const int tiles = (max_kv_len + TILE - 1) / TILE + 1;
    long want = 512 / (static_cast<long>(B > 0 ? B : 1) * Hkv);
    if (want < max_groups) want = max_groups;
    const long cap = static_cast<long>(tiles) * max_groups;
    if (want > cap) want = cap;
    return static_cast<int>(want);
}

size_t attention_bf16_workspace_bytes(int B, int Hkv, int G, int max_kv_len) {
    const size_t slots = attention_bf16_slots(B, Hkv, G, max_kv_len);
    return static_cast<size_t>(B) * Hkv * slots * ROWS_PER_WG * PART_FLOATS * sizeof(float);
}

int tree_attention_bf16(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O, int B,
                        int Hq, int Hkv, int d, const int64_t* kv_start, const int* kv_len, int max_kv_len,
                        long kv_token_stride, long kv_head_stride, const uint64_t* anc_mask, const int* n_nodes,
                        float scale, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    const int G = Hq / Hkv;
    if (d != D || !(G == 1 || G == 2 || G == 4 || G == 8 || G == 16)) return SAGE_UNSUPPORTED;
    if ((kv_token_stride % 8) != 0 || (kv_head_stride % 8) != 0) return SAGE_INVALID_ARG;
    if (!aligned(Q, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(Kt, 16) || !aligned(Vt, 16) || !aligned(workspace, 16))
        return SAGE_INVALID_ARG;
    if (workspace_bytes < attention_bf16_workspace_bytes(B, Hkv, G, max_kv_len)) return SAGE_WORKSPACE_TOO_SMALL;
    if (Hq > 65535 || B > 65535) return SAGE_UNSUPPORTED;

    Params p;
    p.Q = static_cast<const uint16_t*>(Q); p.Kc = static_cast<const uint16_t*>(Kc); p.Vc = static_cast<const uint16_t*>(Vc);
    p.Kt = static_cast<const uint16_t*>(Kt); p.Vt = static_cast<const uint16_t*>(Vt); p.O = static_cast<uint16_t*>(O);
    p.kv_start = kv_start; p.kv_len = kv_len; p.anc_mask = anc_mask; p.n_nodes = n_nodes;
    p.part = static_cast<float*>(workspace);
    p.kv_token_stride = kv_token_stride; p.kv_head_stride = kv_head_stride;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = G;
    p.nslot = attention_bf16_slots(B, Hkv, G, max_kv_len);
    p.scale_log2e = scale * 1.4426950408889634f;

    const long blocks = static_cast<long>(B) * p.nslot * Hkv;
    if (blocks > 0x7FFFFFFFL) return SAGE_UNSUPPORTED;
    hipLaunchKernelGGL(tree_attention_bf16_kernel, dim3(static_cast<unsigned>(blocks)), dim3(THREADS), 0, stream, p);
    if (hipGetLastError() != hipSuccess) return SAGE_LAUNCH_FAILED;
    hipLaunchKernelGGL(tree_attention_merge_kernel, dim3(SAGE_MAX_NODES, Hq, B), dim3(D), 0, stream, p);
    return launch_status();
}

}  // namespace sage
