// sage_tree_attention, bf16 MFMA instantiation (head_dim 128): tree-masked GQA attention of the target's
// verify pass (Sec. 2.2 tree mask; Alg. 1 Phase 2) against a long KV cache plus the tree's own keys.
//
// Formulation.  All query rows that share a KV head (node i, head-in-group hg -> row m = i*G + hg, up to 512
// rows at G = 8) are processed together so each K/V byte is fetched from HBM once.  Everything is computed transposed:
//   S^T = K Q^T   (tokens x rows):  A operand = K rows as stored in the cache (16-byte LDS reads),
//                                   B operand = Q rows, brought in through LDS once and held in registers
//                                   for the whole kernel;
//   O^T = V^T P^T (dims x rows):    A operand = V^T, read from row-major V in LDS with the transposing
//                                   64-bit LDS read of gfx950, B operand = P^T.
// In the 32x32 MFMA accumulator layout a lane owns ONE query row (column lane%32) and 16 tokens of it per 32-token
// half tile, so the softmax sums are in-register, the rescale factor is a per-lane scalar, and the accumulator
// registers of S^T are, as they stand, the B operand of the PV product (the token order inside a 16-token k-block
// is whatever the accumulator layout says; the V^T reads follow that order).
//
// Decomposition (decided on the device from n_nodes/kv_len, so no host round trip): a workgroup of 8 waves owns
// (sequence, KV head, group of up to 8 column tiles = 256 query rows, KV split); wave w owns column tile w (32 query
// rows) and processes whole 64-token tiles for it, so nothing is shared between waves but the K/V stages, and a wave's
// partial result is complete for its rows.  What bounds this kernel is how many bytes per second ONE compute unit can
// pull in (about 24-32 GB/s when the data comes from HBM, the latency of a miss times what a CU can keep in flight;
// every workgroup that shares a tile through L2 still waits out the first one's miss), not the matrix pipe: so a tile
// that has been brought into LDS must serve as many query rows as registers allow, and a tree of up to 32 nodes (G = 8)
// is one group.  With 2..64 sequences the splits are equal ranges of one list of all sequences' tiles, so ragged lengths
// leave no CU idle (see the kernel).  The KV head is the fastest grid index, so in launch order the workgroups of one KV
// head are congruent modulo the KV-head count, which with 8 KV heads pins a head to one XCD and its L2: the two groups
// of a 64-node tree re-read K/V from that L2, not from HBM.  Each workgroup writes an un-normalised partial (max, sum
// in fp32, O^T in bf16); a second kernel merges the splits in a fixed order (deterministic, no float atomics) and
// writes bf16.
//
// Data movement.  K/V tiles of 64 tokens go from global memory straight into LDS (16-byte LDS-direct loads, no
// staging registers; issued through inline assembly, see lds_direct_load16) through a 4-stage ring, three tiles
// ahead of the MFMAs.  A wave-level load writes 1 KB of contiguous LDS; it carries four tokens that are 16 apart,
// and the 1 KB groups are padded so that consecutive tokens are staggered across the banks (conflict-free reads
// with compile-time offsets, see the layout constants).  Every stage is its own LDS object, so every stage address
// is a compile-time constant.  The ancestor masks and the Q rows take the same road ahead of the first tiles, so
// that no load of the kernel returns into a register and every wait on the vector-memory counter is a counted one
// (which is also why these kernels must not spill: the build checks that they use no scratch memory).
//
// Softmax.  The reference maximum of a row is only moved by rebase(): the usual tile costs no maximum at all.
// Probabilities are exp2 of the scaled differences to the reference, rounded to bf16 (the B operand of PV); their sum,
// taken over the rounded values with a two-element dot product, doubles as the overflow check.  The final
// normalisation uses the same reference for numerator and denominator, so the result does not depend on it.
#include <type_traits>

#include "plan_device.h"
#include "sage_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) unsigned char lds_byte;
#define LDS_AS __attribute__((address_space(3)))

constexpr int D = 128;                  // head_dim
constexpr int TILE = 64;                // tokens per LDS stage
constexpr int THREADS = 512;
constexpr int CT_PER_WG = 8;            // column tiles (of 32 query rows) per workgroup: one per wave
constexpr int ROWS_PER_WG = CT_PER_WG * 32;
constexpr int ROW_B = 256;              // bytes of one token row (128 bf16)
// LDS stage layout: token t of a tile sits at (t % 16) * GROUP + (t / 16) * ROW_B, where a group is the 1 KB that
// one wave-level LDS-direct load writes (tokens t, t+16, t+32, t+48) plus padding.  The padding staggers
// consecutive tokens across the banks: 16 bytes for K (read 16 consecutive tokens x one 16-byte chunk at a time),
// 64 bytes for V (read 4 consecutive tokens x 64 bytes at a time).  All per-fragment offsets are compile-time.
constexpr int K_GROUP = 4 * ROW_B + 16;
constexpr int V_GROUP = 4 * ROW_B + 64;
constexpr int K_STAGE_B = 16 * K_GROUP;
constexpr int V_STAGE_B = 16 * V_GROUP;
constexpr int STAGES = 4;
constexpr int LOADS_PER_TILE = 2 * TILE * ROW_B / (THREADS * 16);   // LDS-direct loads per thread per tile (K and V)
// A partial: per query row O^T[128] in bf16, then max and sum in fp32.
constexpr int PART_ROW_B = D * 2 + 16;   // (8 bytes of padding keep the rows 16-byte aligned)
constexpr int PART_SLOT_B = ROWS_PER_WG * PART_ROW_B;
constexpr int EPI_ROW_B = PART_ROW_B;    // a parked row of the epilogue has the layout of a partial row
static_assert(32 * EPI_ROW_B <= K_STAGE_B && 32 * EPI_ROW_B <= V_STAGE_B, "a stage buffer holds a wave's epilogue block");
constexpr float RAISE_MIN = 4.0f;       // rebase() raises a row's reference maximum only past 2^4 ...
constexpr float REBASE_SUM = 512.0f;    // ... which bounds a lane's 32 probabilities of a tile by this sum afterwards

struct Params {
    const uint16_t* Q; const uint16_t* Kc; const uint16_t* Vc; const uint16_t* Kt; const uint16_t* Vt;
    uint16_t* O;
    const int64_t* kv_start; const int* kv_len; const uint64_t* anc_mask; const int* n_nodes;
    const int* first_node;               // nullable: rows are computed for nodes first_node[b] .. n_nodes[b] - 1 only
    unsigned char* part;                 // [B][Hkv][nslot] slots of PART_SLOT_B bytes; batched launches: [Hkv][nslot]
    long kv_token_stride, kv_head_stride;
    int B, Hq, Hkv, G, nslot, min_tiles_per_split;
    int nrange;                          // batched launches: ranges (workgroups) per KV head
    int merge_phases;                    // merge workgroups per (sequence, KV head)
    float scale_log2e;                   // softmax scale times log2(e): probabilities are exp2 of scaled differences
};

// How one (sequence, KV head) is cut into workgroups; evaluated identically by both kernels.
struct Split {
    int n, first, rows, col_groups, tiles, tiles_per_split, nsplit;
};
// the first node whose rows are computed: inside [0, n), so that a call always has a row
__device__ __forceinline__ int clamp_first(int first, int n) { return first < 0 ? 0 : (first > n - 1 ? n - 1 : first); }
__device__ __forceinline__ Split make_split(int n_nodes, int first_node, int kv_len, int G, int nslot, int min_tps) {
    Split s;
    s.n = n_nodes < 1 ? 1 : (n_nodes > SAGE_MAX_NODES ? SAGE_MAX_NODES : n_nodes);
    s.first = clamp_first(first_node, s.n);
    s.rows = (s.n - s.first) * G;
    s.col_groups = (s.rows + ROWS_PER_WG - 1) / ROWS_PER_WG;
    const int L = kv_len > 0 ? kv_len : 0;
    s.tiles = (L + TILE - 1) / TILE + 1;                    // cache tiles, then one tile holding the tree's keys
    int max_split = nslot / s.col_groups;
    if (max_split < 1) max_split = 1;
    s.tiles_per_split = max(min_tps, (s.tiles + max_split - 1) / max_split);
    s.nsplit = (s.tiles + s.tiles_per_split - 1) / s.tiles_per_split;
    return s;
}

// Batched decomposition: lane b of a wave holds the shape of sequence b.  Every (sequence, column group) segment
// occupies SEG_COST_TILES + tiles positions of one line per KV head (the first SEG_COST_TILES stand for the prologue and
// epilogue a pass costs, about that many tile steps); the line of `total` positions is cut into ranges of q, so a
// workgroup whose range starts several segments gets fewer tiles.  Evaluated identically by both kernels.
constexpr int SEG_COST_TILES = 4;
struct BatchShape {
    int n, first, L, tiles, col_groups, start_lo, start_hi;  // per lane (sequence)
    int total, q;                                            // wave-uniform
};
__device__ __forceinline__ int wave_sum_i32(int v) { return static_cast<int>(sage::wave_sum_u32(static_cast<uint32_t>(v))); }
__device__ __forceinline__ BatchShape make_batch_shape(const Params& prm, int lane) {
    BatchShape bs;
    bs.n = 1; bs.first = 0; bs.L = 0; bs.tiles = 0; bs.col_groups = 0; bs.start_lo = 0; bs.start_hi = 0;
    if (lane < prm.B) {
        const int nn = prm.n_nodes[lane];
        const int len = prm.kv_len[lane];
        const int64_t st = prm.kv_start[lane];
        bs.n = nn < 1 ? 1 : (nn > SAGE_MAX_NODES ? SAGE_MAX_NODES : nn);
        bs.first = prm.first_node ? clamp_first(prm.first_node[lane], bs.n) : 0;
        bs.L = len > 0 ? len : 0;
        bs.tiles = (bs.L + TILE - 1) / TILE + 1;             // cache tiles, then one tile holding the tree's keys
        bs.col_groups = ((bs.n - bs.first) * prm.G + ROWS_PER_WG - 1) / ROWS_PER_WG;
        bs.start_lo = static_cast<int>(static_cast<uint32_t>(st));
        bs.start_hi = static_cast<int>(st >> 32);
    }
    bs.total = wave_sum_i32((bs.tiles + SEG_COST_TILES) * bs.col_groups);   // tiles = 0 in lanes past the batch, so is col_groups
    bs.q = max(prm.min_tiles_per_split, (bs.total + prm.nrange - 1) / prm.nrange);
    return bs;
}

// s_waitcnt on the vector-memory counter only (expcnt and lgkmcnt fields left at "no wait")
template <int N> __device__ __forceinline__ void wait_vm() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Workgroup barrier of the stage ring.  __syncthreads() would also fence, and a workgroup-scope release makes the
// compiler wait for every LDS-direct load still in flight, which is exactly what the ring must not do: each
// thread has already waited for its own share of the tile (wait_vm), LDS needs no cache maintenance, so the bare
// barrier is enough; the wavefront-scope fences only pin the order of memory operations around it.
__device__ __forceinline__ void stage_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// max / sum of a value with its partner in the other 32-lane half (both halves receive the result)
__device__ __forceinline__ float cross_half_max(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float cross_half_sum(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// BATCH = false: one sequence per launch slot, every (sequence, KV head) cut into equal splits (see make_split).
// BATCH = true (2..64 sequences): the tiles of all sequences form one list per KV head (sequence-major, then column
// group), cut into prm.nrange equal ranges; a workgroup owns one range and runs one pass (prologue, tile loop,
// epilogue) per (sequence, column group) segment its range touches, so ragged lengths cannot unbalance the launch.
// The leading arguments repeat fields of prm: explicit scalar arguments are preloaded into registers at wave launch
// (the library is built with kernel-argument preloading), so the first thing a workgroup does, fetching its sequence's
// length and node count, does not wait for a fetch of the argument block first.
template <bool BATCH>
__device__ __forceinline__ void attention_workgroup(const int* __restrict__ kv_len_arg, const int* __restrict__ n_nodes_arg,
                                                    const int* __restrict__ first_node_arg,
                                                    const int64_t* __restrict__ kv_start_arg, int nslot_arg, int min_tps_arg,
                                                    int G_arg, const Params& prm, const int first_slab) {
    // one LDS object per stage and operand (see header)
    __shared__ __align__(1024) unsigned char sK0[K_STAGE_B];
    __shared__ __align__(1024) unsigned char sK1[K_STAGE_B];
    __shared__ __align__(1024) unsigned char sK2[K_STAGE_B];
    __shared__ __align__(1024) unsigned char sK3[K_STAGE_B];
    __shared__ __align__(1024) unsigned char sV0[V_STAGE_B];
    __shared__ __align__(1024) unsigned char sV1[V_STAGE_B];
    __shared__ __align__(1024) unsigned char sV2[V_STAGE_B];
    __shared__ __align__(1024) unsigned char sV3[V_STAGE_B];
    __shared__ uint64_t s_mask[ROWS_PER_WG];
#define SK(i) ((i) == 0 ? sK0 : (i) == 1 ? sK1 : (i) == 2 ? sK2 : sK3)
#define SV(i) ((i) == 0 ? sV0 : (i) == 1 ? sV1 : (i) == 2 ? sV2 : sV3)

    const int lane = threadIdx.x & 63;   // (run_segment derives its own copies)

    // grid = (KV head, slot or range, sequence): the KV head is the fastest index of the launch order, and no index
    // costs a division
    const int g = blockIdx.x;
    const int id = static_cast<int>(blockIdx.y) - first_slab;   // slabs before first_slab belong to somebody else
    const int inv_G = (65536 + G_arg - 1) / G_arg;           // (m * inv_G) >> 16 == m / G for the rows of a KV head

    // One pass over tiles [t_begin, t_end) of sequence b for column group cg; the un-normalised partial goes to out_base.
    // (seq_rows rows, of nodes first_v .. seq_n - 1)
    auto run_segment = [&](const int b_v, const int L_v, const int seq_n_v, const int first_v, const int seq_rows_v, const int cg_v, const int t_begin_v,
                           const int t_end_v, const int tree_tile_v, const long kv_start_v, unsigned char* const out_base_v)
                           __attribute__((always_inline)) {
    // every argument is wave-uniform; said to the compiler (the batched walk derives them through lane reads), so that
    // everything computed from them stays in scalar registers
    auto uni = [](int v) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(v); };
    auto uni64 = [&](uint64_t v) __attribute__((always_inline)) {
        return (static_cast<uint64_t>(static_cast<uint32_t>(uni(static_cast<int>(v >> 32)))) << 32) |
               static_cast<uint32_t>(uni(static_cast<int>(static_cast<uint32_t>(v))));
    };
    const int b = uni(b_v), L = uni(L_v), seq_n = uni(seq_n_v), seq_rows = uni(seq_rows_v), cg = uni(cg_v);
    const int node0 = uni(first_v);
    const int t_begin = uni(t_begin_v), t_end = uni(t_end_v), tree_tile = uni(tree_tile_v);
    const long kv_start_b = static_cast<long>(uni64(static_cast<uint64_t>(kv_start_v)));
    unsigned char* const out_base = reinterpret_cast<unsigned char*>(uni64(reinterpret_cast<uint64_t>(out_base_v)));
    if (BATCH) __syncthreads();                              // the previous segment's epilogue has left the stage buffers
    // A batched workgroup calls this in a loop.  Everything below that depends only on the thread index would be
    // loop-invariant, and the compiler hoists all of it out of the loop and keeps it alive across the whole pass (some
    // fifty registers more than the pass itself needs, which does not fit).  The thread index is therefore made opaque
    // per pass, and its derived values are recomputed (a handful of instructions).
    int tid = static_cast<int>(threadIdx.x);
    if (BATCH) asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, so LDS stage addresses stay scalar
    const int r32 = lane & 31;           // MFMA row (A) / column (B, C) owned by this lane
    const int half = lane >> 5;
    // ---- wave roles: wave w owns column tile w of the group (32 query rows) and processes whole tiles for it; with up
    // to four column tiles every computing wave has a SIMD to itself
    const int group_rows = min(ROWS_PER_WG, seq_rows - cg * ROWS_PER_WG);
    const int group_ct = (group_rows + 31) / 32;             // 1..8 column tiles in this group
    const bool wide = group_ct > 4;                          // Q needs two stages of the ring on its way in
    const bool wave_active = wave < group_ct;
    const int m_local = wave * 32 + r32;                     // this lane's query row within the group

    // ---- loader: instruction i of wave w copies tokens r, r+16, r+32, r+48 (r = 2w + i) of K and of V, 1 KB of
    //      LDS each: lane l fills chunk l%16 of token r + 16 (l/16).  Addresses are a wave-uniform tile base in scalar
    //      registers plus a 32-bit per-lane offset that is the same for every full tile, so a tile costs no vector
    //      address arithmetic.
    const int ld_tok = (lane >> 4) * 16 + wave * 2;          // token within the tile for i = 0 (i = 1: the next one)
    const unsigned ld_chunk_b = (lane & 15) * 16;
    const unsigned char* k_cache = reinterpret_cast<const unsigned char*>(
        prm.Kc + kv_start_b * prm.kv_token_stride + static_cast<long>(g) * prm.kv_head_stride);
    const unsigned char* v_cache = reinterpret_cast<const unsigned char*>(
        prm.Vc + kv_start_b * prm.kv_token_stride + static_cast<long>(g) * prm.kv_head_stride);
    const unsigned char* k_tree = reinterpret_cast<const unsigned char*>(
        prm.Kt + (static_cast<long>(b) * SAGE_MAX_NODES * prm.Hkv + g) * D);
    const unsigned char* v_tree = reinterpret_cast<const unsigned char*>(
        prm.Vt + (static_cast<long>(b) * SAGE_MAX_NODES * prm.Hkv + g) * D);
    const unsigned cache_row_b = static_cast<unsigned>(prm.kv_token_stride) * 2u;   // host: 64 rows fit 32 bits
    const unsigned tree_row_b = static_cast<unsigned>(prm.Hkv) * D * 2u;
    const unsigned ld_off0 = static_cast<unsigned>(ld_tok) * cache_row_b + ld_chunk_b;
    const unsigned ld_off1 = ld_off0 + cache_row_b;

    auto issue_loads = [&](int tile, auto stc) __attribute__((always_inline)) {
        constexpr int ST = decltype(stc)::value;
        LDS_AS unsigned char* k_dst = (LDS_AS unsigned char*)(&SK(ST)[wave * 2 * K_GROUP]);
        LDS_AS unsigned char* v_dst = (LDS_AS unsigned char*)(&SV(ST)[wave * 2 * V_GROUP]);
        const bool is_tree = (tile == tree_tile);
        if (tile >= t_end) {
            // Nothing left to fetch, but every step issues the same number of loads, so the wait for a tile is one fixed
            // count on every path.  Four loads of one valid 16-byte piece (served by L2) into the free stage.
            const unsigned char* any = reinterpret_cast<const unsigned char*>(prm.Q);
            sage::lds_direct_load16(any, 0u, k_dst);
            sage::lds_direct_load16(any, 0u, v_dst);
            sage::lds_direct_load16(any, 0u, k_dst + K_GROUP);
            sage::lds_direct_load16(any, 0u, v_dst + V_GROUP);
        } else if (!is_tree && tile * TILE + TILE <= L) {    // full cache tile
            const unsigned char* kb = k_cache + static_cast<long>(tile) * TILE * cache_row_b;
            const unsigned char* vb = v_cache + static_cast<long>(tile) * TILE * cache_row_b;
            sage::lds_direct_load16(kb, ld_off0, k_dst);
            sage::lds_direct_load16(vb, ld_off0, v_dst);
            sage::lds_direct_load16(kb, ld_off1, k_dst + K_GROUP);
            sage::lds_direct_load16(vb, ld_off1, v_dst + V_GROUP);
        } else {                                             // ragged tail or the tree's keys: rows past the end are
            const unsigned char* kb = is_tree ? k_tree : k_cache + static_cast<long>(tile) * TILE * cache_row_b;   // masked later,
            const unsigned char* vb = is_tree ? v_tree : v_cache + static_cast<long>(tile) * TILE * cache_row_b;   // reads stay in range
            const unsigned row_b = is_tree ? tree_row_b : cache_row_b;
            const int last = is_tree ? seq_n - 1 : L - 1 - tile * TILE;
            const unsigned o0 = static_cast<unsigned>(min(ld_tok, last)) * row_b + ld_chunk_b;
            const unsigned o1 = static_cast<unsigned>(min(ld_tok + 1, last)) * row_b + ld_chunk_b;
            sage::lds_direct_load16(kb, o0, k_dst);
            sage::lds_direct_load16(vb, o0, v_dst);
            sage::lds_direct_load16(kb, o1, k_dst + K_GROUP);
            sage::lds_direct_load16(vb, o1, v_dst + V_GROUP);
        }
    };
    // Everything the prologue needs from memory goes straight into LDS, requested back to back in this order: the rows'
    // ancestor masks, the Q rows (into the ring's last stage, idle until the first tile step refills it; a group of more
    // than four column tiles also borrows the third stage, whose tile is then requested one step later), the first
    // tiles.  No load returns into a register, so the compiler never waits on the vector-memory counter here and the
    // only waits are the counted ones: loads complete in order, so masks and Q have landed once no more than the tile
    // loads are outstanding, and the first tile is processed while the following ones are still arriving.
    // Rows past the group's last one repeat that row (their results are never written).
    auto row_of = [&](int local) __attribute__((always_inline)) {      // row `local` of this group -> (node, head in group)
        const int mm = min(cg * ROWS_PER_WG + local, seq_rows - 1);
        const int nd = (mm * inv_G) >> 16;                               // exact for mm < 64 G, G <= 16
        return make_int2(node0 + nd, mm - nd * prm.G);
    };
    {
        // wave w brings both words of the masks of its rows 32 w + lane / 2
        const int2 r = row_of(wave * 32 + (lane >> 1));
        sage::lds_direct_load4(
            reinterpret_cast<const unsigned char*>(prm.anc_mask + static_cast<long>(b) * SAGE_MAX_NODES + r.x) + (lane & 1) * 4,
            (LDS_AS unsigned char*)(&s_mask[wave * 32]));
    }
    // Q rows as blocks of 64 in the layout of a K tile (K buffer) and of a V tile (V buffer): row q of a block sits at
    // (q % 16) * GROUP + (q / 16) * ROW_B.  Blocks 0, 1 -> stage 3; blocks 2, 3 (wide groups only) -> stage 2.
    auto issue_q = [&](auto blkc) __attribute__((always_inline)) {
        constexpr int BLK = decltype(blkc)::value;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int2 r = row_of(BLK * 64 + wave * 2 + i + 16 * (lane >> 4));
            const unsigned char* src = reinterpret_cast<const unsigned char*>(
                prm.Q + ((static_cast<long>(b) * SAGE_MAX_NODES + r.x) * prm.Hq + g * prm.G + r.y) * D) + ld_chunk_b;
            unsigned char* buf = BLK == 0 ? sK3 : BLK == 1 ? sV3 : BLK == 2 ? sK2 : sV2;
            const int group_b = (BLK & 1) ? V_GROUP : K_GROUP;
            sage::lds_direct_load16(src, (LDS_AS unsigned char*)(&buf[(wave * 2 + i) * group_b]));
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    using I4 = std::integral_constant<int, 4>;
    issue_q(I0{});
    issue_q(I1{});
    if (wide) {
        issue_q(I2{});
        issue_q(I3{});
    }
    issue_loads(t_begin, I0{});
    issue_loads(t_begin + 1, I1{});
    if (wide) {
        wait_vm<2 * LOADS_PER_TILE>();                       // this thread's mask and Q loads have landed
    } else {
        issue_loads(t_begin + 2, I2{});
        wait_vm<3 * LOADS_PER_TILE>();
    }
    stage_barrier();                                         // ... everyone's have
    bf16x8 qf[8];                                            // this lane's query row: the B operand of every score MFMA
    {
        const int q = (wave & 1) * 32 + r32;                 // row within its block of 64
        const int blk = wave >> 1;
        const lds_byte* qb = blk == 0 ? (const lds_byte*)sK3 : blk == 1 ? (const lds_byte*)sV3 : blk == 2 ? (const lds_byte*)sK2
                                                                                                       : (const lds_byte*)sV2;
        qb += (q & 15) * ((blk & 1) ? V_GROUP : K_GROUP) + (q >> 4) * ROW_B + half * 16;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, *(const LDS_AS uint4*)(qb + kk * 32));
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);                      // lgkmcnt(0): Q is in registers before this wave reaches the
                                                             // barrier after which its stages are refilled

    // ---- per-lane LDS read offsets.  K fragment (sub, kk): token r32 of 32-token half `sub`, chunk 2kk + half
    //      -> k_lane + sub * 2 * ROW_B + 32 kk.
    const int k_lane = (r32 & 15) * K_GROUP + (r32 >> 4) * ROW_B + half * 16;
    // V^T fragment (dt, jj, u): k-block jj (16 tokens); the 16-lane group q = lane/16 reads tokens 16jj + 8u + 4(q/2) + s/4
    // and dims dt*32 + 16(q%2) + 4(s%4) .. +3  (s = lane%16); after the transposing read lane s holds dim dt*32+16(q%2)+s.
    // Offset: v_lane + jj * ROW_B + u * 8 * V_GROUP + dt * 64.
    int v_lane;
    {
        const int q = lane >> 4, s16 = lane & 15;
        v_lane = (4 * (q >> 1) + (s16 >> 2)) * V_GROUP + (2 * (q & 1) + ((s16 & 3) >> 1)) * 16 + 8 * (s16 & 1);
    }

    f32x16 acc[4];                                           // O^T: 4 tiles of 32 dims x this lane's query row
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
    float m_ref = -INFINITY;                                 // reference maximum of raw (unscaled) scores
    float neg_mc = 0.f;                                      // -m_ref * c, 0 while there is no reference yet
    float l_run = 0.f;                                       // this lane's share of the running sum
    const float c = prm.scale_log2e;
    f32x16 sc[2];                                            // scores of the tile's two 32-token halves
    bf16x8 pf[4];                                            // P^T of the tile's four 16-token k-blocks, the B operand of PV
    bf16x8 ka[8], va[2][4];                                  // K fragments of a half tile; V^T fragments of two dim tiles

    // The pieces of a tile step: scores (S^T = K Q^T, MFMA), softmax (VALU), PV (MFMA).  The LDS reads of a piece are
    // issued in batches ahead of the arithmetic that hides their latency; the scheduling fences keep the compiler from
    // sinking them back next to their uses, where every MFMA group would wait out a full LDS round trip.
    auto read_k = [&](const lds_byte* kb, auto subc, auto firstc) __attribute__((always_inline)) {
        constexpr int SUB = decltype(subc)::value;
        constexpr int FIRST = decltype(firstc)::value;        // dims FIRST*16 .. FIRST*16 + 63
#pragma unroll
        for (int kk = FIRST; kk < FIRST + 4; ++kk)
            ka[kk] = __builtin_bit_cast(bf16x8, *(const LDS_AS uint4*)(kb + k_lane + SUB * 2 * ROW_B + kk * 32));
    };
    auto read_v = [&](const lds_byte* vb, auto dt0c) __attribute__((always_inline)) {
        constexpr int DT0 = decltype(dt0c)::value;            // dims DT0*32 .. DT0*32 + 63, all four k-blocks
#pragma unroll
        for (int dt = DT0; dt < DT0 + 2; ++dt)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const lds_byte* p0 = vb + v_lane + jj * ROW_B + dt * 64;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_AS bf16x4*)p0);
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_AS bf16x4*)(p0 + 8 * V_GROUP));
                va[dt - DT0][jj] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
    };
    auto score_mfma = [&](auto subc, auto firstc) __attribute__((always_inline)) {
        constexpr int SUB = decltype(subc)::value;
        constexpr int FIRST = decltype(firstc)::value;
        if (FIRST == 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sc[SUB][i] = 0.f;
        }
#pragma unroll
        for (int kk = FIRST; kk < FIRST + 4; ++kk) sc[SUB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qf[kk], sc[SUB], 0, 0, 0);
    };
    // admit keys: cache positions below kv_len; tree nodes in this row's ancestor-or-self mask
    auto score_mask = [&](int tile) __attribute__((always_inline)) {
        const bool is_tree = (tile == tree_tile);
        if (!(is_tree || tile * TILE + TILE > L)) return;
        uint64_t admit;
        if (is_tree) {
            admit = s_mask[m_local];
        } else {
            const int left = L - tile * TILE;                // 1..63 valid tokens
            admit = (1ull << left) - 1ull;
        }
        // token of accumulator register i of half `sub`: 32 sub + 8 (i/4) + 4 half + i%4
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const uint32_t adm = static_cast<uint32_t>(admit >> (4 * half + 32 * sub));
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (!((adm >> (8 * (i >> 2) + (i & 3))) & 1u)) sc[sub][i] = -INFINITY;
        }
    };
    // probabilities of k-block JJ: sc[JJ / 2][8 (JJ % 2) .. + 7] -> pf[JJ]; returns sum + the block's rounded probabilities
    auto probs = [&](auto jjc, float sum) __attribute__((always_inline)) {
        constexpr int JJ = decltype(jjc)::value;
        const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
        bf16x8 frag;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const f32x2 pp = {__builtin_amdgcn_exp2f(fmaf(sc[JJ >> 1][8 * (JJ & 1) + e], c, neg_mc)),
                              __builtin_amdgcn_exp2f(fmaf(sc[JJ >> 1][8 * (JJ & 1) + e + 1], c, neg_mc))};
            const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
            frag[e] = pb[0];
            frag[e + 1] = pb[1];
            sum = __builtin_amdgcn_fdot2_f32_bf16(pb, ones, sum, false);
        }
        pf[JJ] = frag;
        return sum;
    };
    auto all_probs = [&]() __attribute__((always_inline)) { return probs(I3{}, probs(I2{}, probs(I1{}, probs(I0{}, 0.f)))); };
    // Move the reference maximum of the rows that need it to the row maximum of the current tile (both 32-lane halves of
    // a row decide alike) and rescale what has been accumulated so far.
    auto rebase = [&]() __attribute__((always_inline)) {
        float tmax = fmaxf(sc[0][0], sc[1][0]);
#pragma unroll
        for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, fmaxf(sc[0][i], sc[1][i]));
        tmax = cross_half_max(tmax);
        const bool raise = (m_ref == -INFINITY) ? (tmax > -INFINITY) : ((tmax - m_ref) * c > RAISE_MIN);
        if (__any(raise)) {
            const float m_new = raise ? tmax : m_ref;
            const float corr = !raise ? 1.f : (m_ref == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_ref - m_new) * c);
            m_ref = m_new;
            neg_mc = -m_ref * c;                             // raise implies a finite maximum
            if (!raise && m_ref == -INFINITY) neg_mc = 0.f;
            l_run *= corr;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[dt][i] *= corr;
        }
    };
    // Back to rebase() when a lane's sum says its probabilities may have overflowed, or when a lane has no reference yet:
    // the pass's first tile, or every key so far was masked for its half of the row.
    auto overflow = [&](float sum) __attribute__((always_inline)) {
        return __any(!(sum <= REBASE_SUM) || m_ref == -INFINITY) != 0;
    };
    // O^T += V^T P^T for the 64 dims whose fragments are in va (four k-blocks of 16 tokens)
    auto pv_mfma = [&](auto dt0c) __attribute__((always_inline)) {
        constexpr int DT0 = decltype(dt0c)::value;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int dt = DT0; dt < DT0 + 2; ++dt)
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt - DT0][jj], pf[jj], acc[dt], 0, 0, 0);
    };
#define FENCE() __builtin_amdgcn_sched_barrier(0)

    auto process = [&](int tile, int first, auto stc) __attribute__((always_inline)) {
        constexpr int ST = decltype(stc)::value;
        if (first && wide) {
            wait_vm<1 * LOADS_PER_TILE>();                   // (the third tile is not on its way yet)
            stage_barrier();                                 // tile 0 has landed; everyone has read Q out of stages 2, 3
            issue_loads(tile + 2, std::integral_constant<int, (ST + 2) % STAGES>{});
        } else {
            wait_vm<2 * LOADS_PER_TILE>();                   // this thread's part of `tile` has landed (two tiles may fly)
            stage_barrier();                                 // ... everyone's has, and the stage read last step is free
        }
        issue_loads(tile + 3, std::integral_constant<int, (ST + 3) % STAGES>{});
        if (!wave_active) return;

        const lds_byte* kst = (const lds_byte*)(SK(ST));
        const lds_byte* vst = (const lds_byte*)(SV(ST));
        read_k(kst, I0{}, I0{});
        read_k(kst, I0{}, I4{});
        FENCE();
        score_mfma(I0{}, I0{});
        FENCE();
        read_k(kst, I1{}, I0{});                             // the second half's fragments follow the first's through the
        FENCE();                                             // same registers, one batch of four behind the MFMAs
        score_mfma(I0{}, I4{});
        FENCE();
        read_k(kst, I1{}, I4{});
        FENCE();
        score_mfma(I1{}, I0{});
        FENCE();
        read_v(vst, I0{});                                   // V reads go out between the score MFMAs and land
        FENCE();                                             // during the softmax
        score_mfma(I1{}, I4{});
        FENCE();
        score_mask(tile);
        float sum = all_probs();
        if (overflow(sum)) {
            rebase();
            sum = all_probs();
        }
        l_run += sum;
        pv_mfma(I0{});
        FENCE();
        read_v(vst, I2{});
        FENCE();
        pv_mfma(I2{});
    };
    for (int tile = t_begin; tile < t_end; tile += STAGES) {    // no path reaches a step without the steps before it
        process(tile, tile == t_begin, I0{});
        if (tile + 1 >= t_end) break;
        process(tile + 1, 0, I1{});
        if (tile + 2 >= t_end) break;
        process(tile + 2, 0, I2{});
        if (tile + 3 >= t_end) break;
        process(tile + 3, 0, I3{});
    }
#undef FENCE

    const float l_tot = cross_half_sum(l_run);
    wait_vm<0>();                                            // the placeholder loads of the last steps have landed too

    // ---- epilogue: a wave's block (O^T in bf16, max, sum) is complete for its 32 rows.  It goes through the wave's own
    // piece of a stage buffer as [32 rows][EPI_ROW_B bytes], transposed on the way: written 8 bytes (4 dims) at a time from
    // the accumulator layout, read back and stored to the partial in row order, for the second kernel to merge.
    __syncthreads();                                         // all stages are idle now
    if (wave_active) {
        unsigned char* blk = wave < 4 ? SK(wave) : SV(wave - 4);
        unsigned char* mine = blk + r32 * EPI_ROW_B;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 v = {acc[dt][4 * q], acc[dt][4 * q + 1], acc[dt][4 * q + 2], acc[dt][4 * q + 3]};
                *reinterpret_cast<bf16x4*>(mine + (dt * 32 + 8 * q + 4 * half) * 2) = __builtin_convertvector(v, bf16x4);
            }
        if (half == 0) *reinterpret_cast<float2*>(mine + D * 2) = make_float2(m_ref, l_tot);
        // (a wave's LDS operations complete in order, and the reads below wait for them: no barrier inside a wave)
        const int rows_here = min(32, group_rows - wave * 32);
        unsigned char* out = out_base + static_cast<long>(wave) * 32 * PART_ROW_B;
        // parked rows and partial rows have the same pitch, so the wave's block goes out as one contiguous copy of
        // rows_here * 17 chunks of 16 bytes (16 of O^T, one of max and sum), 64 chunks per store instruction
        const int last_chunk = rows_here * (PART_ROW_B / 16);
#pragma unroll
        for (int i = 0; i < 9; ++i) {
            const int ch = lane + 64 * i;
            if (ch < last_chunk)
                *reinterpret_cast<uint4*>(out + ch * 16) = *reinterpret_cast<const uint4*>(blk + ch * 16);
        }
    }
    };   // run_segment

    if (!BATCH) {
        const int slot = id;
        const int b = blockIdx.z;
        // the three per-sequence words are requested together and waited for once: the empty statement needs all of
        // them in scalar registers at one point (readfirstlane: uniform values, wherever the compiler loaded them)
        int len_b = __builtin_amdgcn_readfirstlane(kv_len_arg[b]);
        int n_b = __builtin_amdgcn_readfirstlane(n_nodes_arg[b]);
        const int64_t start_w = kv_start_arg[b];
        int start_lo = __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(start_w)));
        int start_hi = __builtin_amdgcn_readfirstlane(static_cast<int>(start_w >> 32));
        int f_b = first_node_arg ? __builtin_amdgcn_readfirstlane(first_node_arg[b]) : 0;   // (a uniform branch on an argument)
        asm("" : "+s"(len_b), "+s"(n_b), "+s"(start_lo), "+s"(start_hi), "+s"(f_b));
        const long start_b = (static_cast<long>(start_hi) << 32) | static_cast<uint32_t>(start_lo);
        const int L = len_b > 0 ? len_b : 0;
        const Split sp = make_split(n_b, f_b, L, G_arg, nslot_arg, min_tps_arg);
        if (sp.col_groups > nslot_arg) return;              // host guarantees nslot >= the largest group count
        const int cg = slot % sp.col_groups;
        const int split = slot / sp.col_groups;
        if (split >= sp.nsplit) return;
        const int t_begin = split * sp.tiles_per_split;
        const int t_end = min(sp.tiles, t_begin + sp.tiles_per_split);
        run_segment(b, L, sp.n, sp.first, sp.rows, cg, t_begin, t_end, sp.tiles - 1, start_b,
                    prm.part + ((static_cast<long>(b) * prm.Hkv + g) * prm.nslot + slot) * PART_SLOT_B);
    } else {
        const BatchShape bs = make_batch_shape(prm, lane);  // lane b holds sequence b
        const int r0 = id * bs.q;                            // this workgroup's range of the tile list
        const int r1 = min(bs.total, r0 + bs.q);
        if (r0 >= r1) return;
        int first = 0, groups_before = 0;                    // first position / number of segments of the sequences before b
        for (int b = 0; b < prm.B && first < r1; ++b) {
            const int tiles_b = __builtin_amdgcn_readlane(bs.tiles, b);
            const int cgs_b = __builtin_amdgcn_readlane(bs.col_groups, b);
            const int seg_len = tiles_b + SEG_COST_TILES;
            if (first + seg_len * cgs_b > r0) {
                const int n_b = __builtin_amdgcn_readlane(bs.n, b);
                const int f_b = __builtin_amdgcn_readlane(bs.first, b);
                const int L_b = __builtin_amdgcn_readlane(bs.L, b);
                const long start_b = (static_cast<long>(__builtin_amdgcn_readlane(bs.start_hi, b)) << 32) |
                                     static_cast<uint32_t>(__builtin_amdgcn_readlane(bs.start_lo, b));
                for (int cg = 0; cg < cgs_b; ++cg) {
                    const int tile0 = first + cg * seg_len + SEG_COST_TILES;      // position of the segment's first tile
                    const int lo = max(r0, tile0), hi = min(r1, tile0 + tiles_b);
                    if (lo < hi)
                        run_segment(b, L_b, n_b, f_b, (n_b - f_b) * prm.G, cg, lo - tile0, hi - tile0, tiles_b - 1, start_b,
                                    prm.part + (static_cast<long>(g) * prm.nslot + id + groups_before + cg) * PART_SLOT_B);
                }
            }
            first += seg_len * cgs_b;
            groups_before += cgs_b;
        }
    }
#undef SK
#undef SV
}

template <bool BATCH>
__global__ __launch_bounds__(THREADS) void tree_attention_bf16_kernel(const int* __restrict__ kv_len_arg,
                                                                      const int* __restrict__ n_nodes_arg,
                                                                      const int* __restrict__ first_node_arg,
                                                                      const int64_t* __restrict__ kv_start_arg, int nslot_arg,
                                                                      int min_tps_arg, int G_arg, const Params prm) {
    attention_workgroup<BATCH>(kv_len_arg, n_nodes_arg, first_node_arg, kv_start_arg, nslot_arg, min_tps_arg, G_arg, prm, 0);
}

// The same launch carrying the planning of the next tree along (sage_tree_attention_with_plan): the grid has extra
// slabs of workgroups ahead of the attention's own (blockIdx.y < plan_slabs), one workgroup of which per sequence runs
// sage_build_tree_from_slices' work for that sequence, with LDS of its own, while the attention workgroups stream the
// cache.  The two halves share nothing: the tree being planned is the next step's, not the one whose mask the
// attention reads.  A step is a chain of dependent launches and planning is two of them; inside this launch it costs
// no launch and, as long as it is shorter than the attention, no time.  The planning slabs come first in launch order:
// when the attention's own workgroups fill every CU, the one that has to wait for a free CU is then the attention's
// last (a sequence's final split, seldom a full one), and it waits for the short planning workgroup, not the other
// way round.
constexpr int PLAN_LDS_KEYS = 2400;     // what the 160 KB of a CU leave beside the attention's stages (k = 16 at 152064 tokens: 2384)
constexpr int PLAN_OWN = 4;              // slices per lane: up to 256 slices per draft row
struct PlanShared {
    static constexpr int LDS_KEYS = PLAN_LDS_KEYS;
    uint64_t* keys;
    sage::topk::UnitStats* stats;
    float& row_m;
    float& row_Z;
};
template <bool BATCH>
__global__ __launch_bounds__(THREADS) void tree_attention_plan_kernel(const int* __restrict__ kv_len_arg,
                                                                      const int* __restrict__ n_nodes_arg,
                                                                      const int64_t* __restrict__ kv_start_arg, int nslot_arg,
                                                                      int min_tps_arg, int G_arg, int plan_slabs,
                                                                      const Params prm, const sage::PlanArgs pl) {
    if (static_cast<int>(blockIdx.y) < plan_slabs) {        // workgroup-uniform
        __shared__ uint64_t p_keys[PLAN_LDS_KEYS];
        __shared__ sage::topk::UnitStats p_stats[64 * PLAN_OWN];
        __shared__ float p_row[2];
        // one sequence per launch slot: the slab's first workgroup of sequence blockIdx.z; batches: slab workgroups in turn
        const int b = BATCH ? static_cast<int>(blockIdx.y * gridDim.x + blockIdx.x)
                            : (blockIdx.x == 0 ? static_cast<int>(blockIdx.z) : prm.B);
        if (b >= prm.B) return;
        PlanShared sh{p_keys, p_stats, p_row[0], p_row[1]};
        sage::plan_sequence<PLAN_OWN, THREADS>(b, pl, sh);
        return;
    }
    attention_workgroup<BATCH>(kv_len_arg, n_nodes_arg, nullptr, kv_start_arg, nslot_arg, min_tps_arg, G_arg, prm, plan_slabs);   // a verify pass: every node
}

// Merge the splits of one (sequence, node, query head) in split order and write bf16.  One wave per row:
// lane = split for the (max, sum) pairs and their weights, lane = pair of output dims for the accumulation.
// Every partial of the row is requested before the first one is used, so the merge costs one memory round trip.
// ROWS = rows (waves) per workgroup.  MAXS = splits handled per pass (one per lane for the (max, sum) pairs, one
// register each for the accumulation); the host picks the smallest instantiation that covers the launch's slot
// count, which keeps the register count, and with it the number of resident waves, in proportion to the work.
constexpr int MERGE_ROWS_SINGLE = 4;     // one sequence: many small workgroups spread best over the CUs
constexpr int MERGE_ROWS_BATCH = 4;      // (16 rows per workgroup measured 6 % slower on the ragged batch of 8)
constexpr int MERGE_PHASES_BATCH = 32;   // batches: workgroups per (sequence, KV head), each walking the live rows; a
                                         // single sequence gets a wave per possible row (fewer measured no faster)
template <int MAXS, bool BATCH, int ROWS>
__global__ __launch_bounds__(64 * ROWS) void tree_attention_merge_kernel(const int* __restrict__ kv_len_arg,
                                                                         const int* __restrict__ n_nodes_arg, int nslot_arg,
                                                                         int min_tps_arg, int G_arg, int phases_arg,
                                                                         const Params prm) {
    static_assert(MAXS <= 32, "one split per lane, one register per split");
    // As in the main kernel, a KV head's blocks are congruent modulo the KV-head count, so with 8 KV heads they run on
    // the XCD whose L2 still holds that head's partials.  Rows of a KV head are numbered as there: node * G + head-in-group.
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // a row's address is wave-uniform: scalar registers
    const int g = blockIdx.x;                                // grid = (KV head, phase, sequence), as in the main kernel
    const float c = prm.scale_log2e;

    // one row: `first_row` = the row in the first of its nsplit partials, stride_b = bytes to the next one.  Addresses are
    // the uniform row pointer plus 32-bit offsets (a launch's partials span far less than 4 GB from any row), which
    // keeps the address arithmetic of up to 32 loads per lane off the critical path of this latency-bound kernel.
    auto merge_row = [&](int b, int node, int hg, const unsigned char* first_row, unsigned stride_b, int nsplit_v) __attribute__((always_inline)) {
        // wave-uniform by construction; said to the compiler, which cannot see it through the lane exchanges of a batch
        const uintptr_t first_v = reinterpret_cast<uintptr_t>(first_row);
        const uintptr_t first =
            (static_cast<uintptr_t>(static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(first_v >> 32)))) << 32) |
            static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(first_v)));   // (the builtin returns int)
        stride_b = __builtin_amdgcn_readfirstlane(stride_b);
        const int nsplit = __builtin_amdgcn_readfirstlane(nsplit_v);
        float2 o = make_float2(0.f, 0.f);
        float m_all = -INFINITY, l_all = 0.f;
        for (int s0 = 0; s0 < nsplit; s0 += MAXS) {           // MAXS splits at a time
            const int cnt = min(MAXS, nsplit - s0);
            float ms = -INFINITY, ls = 0.f;
            // The row's partials of this pass as one buffer: uniform base (partial s0), 32-bit offsets, and a size that ends
            // with the row's extent in its last split, so that a load for a split past the last one is answered with zeros
            // by the bounds check instead of by memory.  One add and one load instruction per split.
            typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
            const __amdgpu_buffer_rsrc_t rows = __builtin_amdgcn_make_buffer_rsrc(
                reinterpret_cast<unsigned char*>(first + static_cast<size_t>(s0) * stride_b), 0,
                static_cast<int>(static_cast<unsigned>(cnt - 1) * stride_b + PART_ROW_B), 0x00020000);
            {
                const u32x2 pair = __builtin_amdgcn_raw_buffer_load_b64(rows, static_cast<unsigned>(lane) * stride_b + D * 2u, 0, 0);
                ms = lane < cnt ? __uint_as_float(pair[0]) : -INFINITY;
                ls = lane < cnt ? __uint_as_float(pair[1]) : 0.f;
            }
            unsigned v[MAXS];                                // two bf16 output dims of split s
            unsigned off = 4u * lane;                        // the whole offset goes through the per-lane operand: that one is
#pragma unroll                                               // bounds-checked, the scalar offset operand is not
            for (int s = 0; s < MAXS; ++s) {
                v[s] = __builtin_amdgcn_raw_buffer_load_b32(rows, off, 0, 0);
                off += stride_b;
            }
            __builtin_amdgcn_sched_barrier(0);               // every load is out before the first wait: one round trip
            const float m_blk = sage::wave_max(ms);
            const float m_new = fmaxf(m_all, m_blk);
            const float keep = (m_all == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_all - m_new) * c);
            const float w = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((ms - m_new) * c);
            l_all = l_all * keep + sage::wave_sum(w * ls);
            o.x *= keep; o.y *= keep;
            m_all = m_new;
#pragma unroll
            for (int s = 0; s < MAXS; ++s) {
                const float ws = sage::lane_value(w, s);        // split s's weight, through a scalar register
                o.x += ws * __uint_as_float(v[s] << 16);
                o.y += ws * __uint_as_float(v[s] & 0xFFFF0000u);
            }
        }
        const float inv = 1.0f / l_all;
        const uint32_t packed = static_cast<uint32_t>(sage::float_to_bf16_bits(o.x * inv)) |
                                (static_cast<uint32_t>(sage::float_to_bf16_bits(o.y * inv)) << 16);
        reinterpret_cast<uint32_t*>(prm.O + ((static_cast<long>(b) * SAGE_MAX_NODES + node) * prm.Hq + g * prm.G + hg) * D)[lane] = packed;
    };

    // blockIdx = (KV head, phase, sequence); a wave walks the live rows phase * ROWS + wave, + phases * ROWS,
    // ... of its (sequence, KV head), so that rows of nodes past n_nodes cost no workgroup of their own
    const int phases = phases_arg;
    const int phase = blockIdx.y;
    const int b = blockIdx.z;
    if (!BATCH) {
        int len_b = __builtin_amdgcn_readfirstlane(kv_len_arg[b]);   // requested together, waited for once
        int n_b = __builtin_amdgcn_readfirstlane(n_nodes_arg[b]);
        int f_b = prm.first_node ? __builtin_amdgcn_readfirstlane(prm.first_node[b]) : 0;
        asm("" : "+s"(len_b), "+s"(n_b), "+s"(f_b));
        const int L = len_b > 0 ? len_b : 0;
        const Split sp = make_split(n_b, f_b, L, G_arg, nslot_arg, min_tps_arg);
        if (sp.col_groups > nslot_arg) return;
        const unsigned char* base = prm.part + ((static_cast<long>(b) * prm.Hkv + g) * prm.nslot) * PART_SLOT_B;
        for (int m = phase * ROWS + wave; m < sp.rows; m += phases * ROWS)
            merge_row(b, sp.first + m / prm.G, m % prm.G, base + (static_cast<long>(m / ROWS_PER_WG) * ROWS_PER_WG + m % ROWS_PER_WG) * PART_ROW_B,
                      static_cast<unsigned>(sp.col_groups) * static_cast<unsigned>(PART_SLOT_B), sp.nsplit);
    } else {
        const BatchShape bs = make_batch_shape(prm, lane);
        const int first_b = __builtin_amdgcn_readlane(bs.first, b);
        const int live = (__builtin_amdgcn_readlane(bs.n, b) - first_b) * prm.G;
        const int tiles_b = __builtin_amdgcn_readlane(bs.tiles, b);
        const int before = wave_sum_i32(lane < b ? (bs.tiles + SEG_COST_TILES) * bs.col_groups : 0);
        const int groups_before = wave_sum_i32(lane < b ? bs.col_groups : 0);
        for (int m = phase * ROWS + wave; m < live; m += phases * ROWS) {
            const int cg = m / ROWS_PER_WG;
            const int u0 = before + cg * (tiles_b + SEG_COST_TILES) + SEG_COST_TILES;   // first tile of segment (b, cg)
            const int s_first = u0 / bs.q;
            merge_row(b, first_b + m / prm.G, m % prm.G,
                      prm.part + (static_cast<long>(g) * prm.nslot + s_first + groups_before + cg) * PART_SLOT_B + (m % ROWS_PER_WG) * PART_ROW_B,
                      static_cast<unsigned>(PART_SLOT_B), (u0 + tiles_b - 1) / bs.q - s_first + 1);
        }
    }
}

}  // namespace

namespace sage {

// Launch shape.  A single sequence (and batches of more than 64): slots = workgroups per (sequence, KV head); a slot is
// (KV split, column group); the sequence is cut into about one 8-wave workgroup per CU (one round, no tail).
// Batches of 2..64 sequences: the tile list of all sequences is cut into `nrange` ranges per KV head, about one
// workgroup per CU in total whatever the lengths turn out to be on the device; a range is at least MIN_RANGE_TILES
// tiles (every pass pays a few microseconds of prologue and epilogue), and the partial slots of a KV head are one per
// range plus one per (sequence, column group), the most that range and segment boundaries can produce together.
constexpr int MAX_BATCH_LANES = 64;      // a lane per sequence in make_batch_shape
constexpr int MIN_RANGE_TILES = 8;      // positions of the line, pass cost included
struct LaunchShape { int nslot, min_tiles_per_split, nrange; bool batch; };
LaunchShape attention_bf16_shape(int B, int Hkv, int G, int max_kv_len) {
    const int max_groups = (SAGE_MAX_NODES * G + ROWS_PER_WG - 1) / ROWS_PER_WG;
    const int tiles = (max_kv_len + TILE - 1) / TILE + 1;
    LaunchShape sh;
    sh.batch = B >= 2 && B <= MAX_BATCH_LANES;
    sh.nrange = 0;
    if (sh.batch) {
        long want = 256 / Hkv;
        if (want < 1) want = 1;
        const long cap = (static_cast<long>(B) * (tiles + SEG_COST_TILES) * max_groups + MIN_RANGE_TILES - 1) / MIN_RANGE_TILES;
        if (want > cap) want = cap;
        sh.nrange = static_cast<int>(want);
        sh.min_tiles_per_split = MIN_RANGE_TILES;
        sh.nslot = sh.nrange + B * max_groups;
        return sh;
    }
    if (B <= 1) {
        long want = 256 / Hkv;
        if (want < max_groups) want = max_groups;
        const long cap = static_cast<long>(tiles) * max_groups;
        if (want > cap) want = cap;
        sh.nslot = static_cast<int>(want);
        sh.min_tiles_per_split = 1;
    } else {
        const double est_tiles = 0.6 * B * Hkv * static_cast<double>(tiles);    // ragged batches average below the maximum
        long tps = static_cast<long>(est_tiles / 256.0) + 1;       // about one workgroup per CU in total
        if (tps < 4) tps = 4;
        if (tps > tiles) tps = tiles;
        sh.min_tiles_per_split = static_cast<int>(tps);
        sh.nslot = static_cast<int>((tiles + tps - 1) / tps) * max_groups;
    }
    if (sh.nslot > 256) sh.nslot = 256;               // the merge handles any count; this bounds the workspace
    if (sh.nslot < max_groups) sh.nslot = max_groups;
    return sh;
}

size_t attention_bf16_workspace_bytes(int B, int Hkv, int G, int max_kv_len) {
    const LaunchShape sh = attention_bf16_shape(B, Hkv, G, max_kv_len);
    return (sh.batch ? static_cast<size_t>(1) : static_cast<size_t>(B)) * Hkv * sh.nslot * static_cast<size_t>(PART_SLOT_B);
}

// Whether the attention launch can carry this planning along: the lists of a draft row must fit the LDS the planning
// workgroup has, and a lane holds at most PLAN_OWN slices.
bool attention_bf16_can_carry_plan(const PlanArgs& pl) {
    return pl.nunits <= 64 * PLAN_OWN && pl.nunits * pl.k <= PLAN_LDS_KEYS;
}

// plan == nullptr: the attention alone.  Otherwise the caller has checked attention_bf16_can_carry_plan(*plan).
int tree_attention_bf16(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt, void* O, int B,
                        int Hq, int Hkv, int d, const int64_t* kv_start, const int* kv_len, int max_kv_len,
                        long kv_token_stride, long kv_head_stride, const uint64_t* anc_mask, const int* n_nodes,
                        const int* first_node, float scale, void* workspace, size_t workspace_bytes, hipStream_t stream,
                        const PlanArgs* plan) {
    const int G = Hq / Hkv;
    if (d != D || G < 1 || G > 16) return SAGE_UNSUPPORTED;   // 64 nodes x 16 heads per KV head = 8 groups of 128 rows
    if ((kv_token_stride % 8) != 0 || (kv_head_stride % 8) != 0) return SAGE_INVALID_ARG;
    if (kv_token_stride > (1L << 24)) return SAGE_UNSUPPORTED;   // the byte offsets inside a 64-token tile are 32-bit
    if (!aligned(Q, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(Kt, 16) || !aligned(Vt, 16) || !aligned(workspace, 16))
        return SAGE_INVALID_ARG;
    if (workspace_bytes < attention_bf16_workspace_bytes(B, Hkv, G, max_kv_len)) return SAGE_WORKSPACE_TOO_SMALL;
    if (Hq > 65535 || B > 65535) return SAGE_UNSUPPORTED;

    Params p;
    p.Q = static_cast<const uint16_t*>(Q); p.Kc = static_cast<const uint16_t*>(Kc); p.Vc = static_cast<const uint16_t*>(Vc);
    p.Kt = static_cast<const uint16_t*>(Kt); p.Vt = static_cast<const uint16_t*>(Vt); p.O = static_cast<uint16_t*>(O);
    p.kv_start = kv_start; p.kv_len = kv_len; p.anc_mask = anc_mask; p.n_nodes = n_nodes;
    p.first_node = plan ? nullptr : first_node;
    p.part = static_cast<unsigned char*>(workspace);
    p.kv_token_stride = kv_token_stride; p.kv_head_stride = kv_head_stride;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = G;
    const LaunchShape sh = attention_bf16_shape(B, Hkv, G, max_kv_len);
    p.nslot = sh.nslot;
    p.min_tiles_per_split = sh.min_tiles_per_split;
    p.scale_log2e = scale * 1.4426950408889634f;

    p.nrange = sh.nrange;
    const int own_slabs = sh.batch ? p.nrange : p.nslot;
    const dim3 block(THREADS);
    if (plan) {
        // planning workgroups in slabs of their own ahead of the attention's: one slab whose first workgroup of every
        // sequence plans (one sequence per launch slot), or as many slabs as B workgroups need (batches)
        const int plan_slabs = sh.batch ? (B + Hkv - 1) / Hkv : 1;
        const dim3 grid(Hkv, plan_slabs + own_slabs, sh.batch ? 1 : B);
        if (sh.batch)
            hipLaunchKernelGGL(tree_attention_plan_kernel<true>, grid, block, 0, stream, kv_len, n_nodes, kv_start, p.nslot,
                               p.min_tiles_per_split, G, plan_slabs, p, *plan);
        else
            hipLaunchKernelGGL(tree_attention_plan_kernel<false>, grid, block, 0, stream, kv_len, n_nodes, kv_start, p.nslot,
                               p.min_tiles_per_split, G, plan_slabs, p, *plan);
    } else {
        const dim3 grid(Hkv, own_slabs, sh.batch ? 1 : B);
        if (sh.batch)
            hipLaunchKernelGGL(tree_attention_bf16_kernel<true>, grid, block, 0, stream, kv_len, n_nodes, first_node, kv_start, p.nslot,
                               p.min_tiles_per_split, G, p);
        else
            hipLaunchKernelGGL(tree_attention_bf16_kernel<false>, grid, block, 0, stream, kv_len, n_nodes, first_node, kv_start, p.nslot,
                               p.min_tiles_per_split, G, p);
    }
    if (hipGetLastError() != hipSuccess) return SAGE_LAUNCH_FAILED;
    const int mrows = sh.batch ? MERGE_ROWS_BATCH : MERGE_ROWS_SINGLE;
    const int row_blocks = (SAGE_MAX_NODES * G + mrows - 1) / mrows;
    const int want_phases = sh.batch ? MERGE_PHASES_BATCH : row_blocks;
    p.merge_phases = row_blocks < want_phases ? row_blocks : want_phases;
    const dim3 mgrid(Hkv, p.merge_phases, B), mblock(64 * mrows);
    const int max_tiles = (max_kv_len + TILE - 1) / TILE + 1;
    int most = sh.batch ? p.nrange : p.nslot;         // upper bound of the splits of a row: no more than slots, or tiles
    if (most > max_tiles) most = max_tiles;
    // more than 32 splits take several passes of 32: 64 register pairs per lane cost more in resident waves than the
    // second round trip does
    if (sh.batch) {
        if (most <= 8) hipLaunchKernelGGL((tree_attention_merge_kernel<8, true, MERGE_ROWS_BATCH>), mgrid, mblock, 0, stream, kv_len, n_nodes, p.nslot,
                               p.min_tiles_per_split, G, p.merge_phases, p);
        else if (most <= 16) hipLaunchKernelGGL((tree_attention_merge_kernel<16, true, MERGE_ROWS_BATCH>), mgrid, mblock, 0, stream, kv_len, n_nodes, p.nslot,
                               p.min_tiles_per_split, G, p.merge_phases, p);
        else hipLaunchKernelGGL((tree_attention_merge_kernel<32, true, MERGE_ROWS_BATCH>), mgrid, mblock, 0, stream, kv_len, n_nodes, p.nslot,
                               p.min_tiles_per_split, G, p.merge_phases, p);
    } else {
        if (most <= 8) hipLaunchKernelGGL((tree_attention_merge_kernel<8, false, MERGE_ROWS_SINGLE>), mgrid, mblock, 0, stream, kv_len, n_nodes, p.nslot,
                               p.min_tiles_per_split, G, p.merge_phases, p);
        else if (most <= 16) hipLaunchKernelGGL((tree_attention_merge_kernel<16, false, MERGE_ROWS_SINGLE>), mgrid, mblock, 0, stream, kv_len, n_nodes, p.nslot,
                               p.min_tiles_per_split, G, p.merge_phases, p);
        else hipLaunchKernelGGL((tree_attention_merge_kernel<32, false, MERGE_ROWS_SINGLE>), mgrid, mblock, 0, stream, kv_len, n_nodes, p.nslot,
                               p.min_tiles_per_split, G, p.merge_phases, p);
    }
    return launch_status();
}

}  // namespace sage
