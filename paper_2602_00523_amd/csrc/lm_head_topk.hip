// sage_lm_head_topk: the target's greedy token and softmax statistics per row (Sec. 2.2 / Def. 4.1, Eq. 1) taken
// straight from the output projection, logits = hidden . weight^T, so that the rows x vocabulary logits never
// exist in memory.  The weight matrix ([vocab, dim] bf16, 2.5 GB at the 72B shape) is fetched from HBM once per call:
// up to 128 live rows go through it in a single pass; with more, the workgroups that push different blocks of rows
// through the same weight tiles are neighbours on one XCD and run side by side, so that the first of them fetches a
// tile from HBM and the others find it in that XCD's L2.  Rows that n_valid marks dead are left out before the blocks
// are formed (the live rows of all groups are packed into dense blocks), so a batch of partly filled trees costs its
// live rows only.  The hidden rows (1 MB per block of 64) are read once per workgroup from L2.
//
// A workgroup of 4 waves owns T consecutive 64-row vocabulary tiles and R blocks of 64 hidden rows and keeps the
// logits of ALL of them in registers (R T accumulators of 32 x 32 per wave; with one wave per SIMD a wave has 512
// registers).  The loop runs over chunks of 128 hidden elements on the outside and the T tiles on the inside, so a
// hidden chunk is fetched once and its MFMA operands stay in registers for T steps, while the weight tiles (64 rows x
// 256 B) stream from global memory straight into LDS through a ring of 8 (R = 1) or 7 (R = 2) stages, all but one of
// them ahead of the MFMAs, in the same padded layout as the attention kernel's K tiles (conflict-free 16-byte reads
// with compile-time offsets).  Wave (vt, rt) accumulates logits^T[32 vocabulary rows of half vt][32 hidden rows of
// half rt] per row block with v_mfma_f32_32x32x16_bf16 (A = weight rows, B = hidden rows, both as stored), so a lane
// owns one hidden row per block and 16 vocabulary entries of it per tile.  After the last chunk every lane folds its
// 16 T logits into statistics of its row (maximum m, Z = sum exp(x - m), T = sum exp(x - m)(m - x), best (value,
// index) key); the four partial statistics of a row are combined through LDS and written as one "slice" per
// (row, unit), in the format of the stored-logits first pass, whose second pass finishes the row.
//
// The launch has at most one workgroup per CU (a workgroup fills a CU's LDS); each stays resident and walks the work
// items (unit, live row block) id, id + grid, ..., so a block without live rows costs nothing: as workgroups of their
// own such blocks were measured to cost about as much as live ones (a 512-row call with 64 live rows took 1.3 ms
// instead of 0.44).
#include <type_traits>

#include "sage_internal.h"
#include "topk_common.h"

using namespace sage::topk;

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) unsigned char lds_byte;
#define LDS_AS __attribute__((address_space(3)))

constexpr int TILE_V = 64;               // vocabulary rows per tile
constexpr int TILE_R = 64;               // hidden rows per launch block
constexpr int CHUNK = 128;               // hidden elements per stage
constexpr int ROW_B = CHUNK * 2;         // bytes of one row of a stage
constexpr int THREADS = 256;
constexpr int MAX_K = 16;                // largest candidate list per row
constexpr int CUS = 256;                 // compute units of the MI355X: workgroups of a launch that stay resident
constexpr int MAX_STAGES = 8;          // weight ring: all but one stage in flight per workgroup
// stage layout: row t at (t % 16) * GROUP + (t / 16) * ROW_B; a group is the 1 KB one wave-level LDS-direct load
// writes (rows t, t+16, t+32, t+48) plus 16 bytes, which staggers consecutive rows across the banks
constexpr int GROUP = 4 * ROW_B + 16;
constexpr int STAGE_B = 16 * GROUP;
constexpr int LOADS_PER_TILE = TILE_V * ROW_B / (THREADS * 16);       // 16-byte loads per thread and tile

struct Params {
    const unsigned char* hidden; const unsigned char* weight;
    long hidden_stride_b, weight_stride_b;
    int rows, dim, vocab, k, nunits, ntiles;
    int row_blocks;                      // blocks of 64 or 128 (packed live) rows, one workgroup each per unit
    const int* n_valid; int rows_per_group;
    UnitStats* stats; uint64_t* keys;    // [rows][nunits]
};

template <int N> __device__ __forceinline__ void wait_vm() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// wait until at most `tiles` tiles' worth of this thread's loads are outstanding (0..7)
__device__ __forceinline__ void wait_vm_tiles(int tiles) {
    switch (tiles) {
        case 0: wait_vm<0>(); break;
        case 1: wait_vm<1 * LOADS_PER_TILE>(); break;
        case 2: wait_vm<2 * LOADS_PER_TILE>(); break;
        case 3: wait_vm<3 * LOADS_PER_TILE>(); break;
        case 4: wait_vm<4 * LOADS_PER_TILE>(); break;
        case 5: wait_vm<5 * LOADS_PER_TILE>(); break;
        case 6: wait_vm<6 * LOADS_PER_TILE>(); break;
        default: wait_vm<7 * LOADS_PER_TILE>(); break;
    }
}
// bare barrier with wavefront-scope fences (a workgroup-scope release would wait for every load in flight)
__device__ __forceinline__ void stage_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// R = blocks of 64 hidden rows a workgroup pushes through its weight tiles (R * T accumulators per wave).  R = 2 is for
// launches with more than 64 rows: when every CU reads its weight tiles through L2 at once the chip delivers about
// 46 GB/s per CU, which at 64 rows per workgroup (64 flops per byte) caps the call near 700 TFLOP/s whatever the MFMAs
// could do; two row blocks per workgroup halve the bytes per flop.  The second hidden stage costs one weight stage.
// TOPK: k candidates per (row, unit) instead of one (the draft side of Sec. 3.1, whose rows are few): after the fold, k
// rounds pick the best remaining logit of every row in the total order (value descending, index ascending).  A round
// scans the lane's 16 T logits for the best one that comes after the previous winner, combines the four lanes of a row
// (lane halves by a swap, vocabulary halves through LDS) and writes the winner as key j of the unit's sorted list.
template <int T, int R, bool TOPK>
__global__ __launch_bounds__(THREADS) void lm_head_kernel(const Params prm) {
    static_assert(!TOPK || R == 1, "the candidate rounds are written for one row block");
    // The ring position of a step must be a compile-time constant (every stage is its own LDS object, so that loads
    // in flight into one stage are known not to alias reads of another): step t of chunk kc uses stage
    // (kc T + t) mod STAGES, which is static once the chunk loop is unrolled UNROLL times.
    constexpr int STAGES = R == 1 ? 8 : 7;
    constexpr int AHEAD = STAGES - 1;
    constexpr int UNROLL = STAGES == 7 ? (T % 7 == 0 ? 1 : 7)
                                       : (T % 8 == 0) ? 1 : (T % 4 == 0) ? 2 : (T % 2 == 0) ? 4 : 8;
    static_assert((UNROLL * T) % STAGES == 0 && STAGES <= MAX_STAGES && R >= 1 && R <= 2, "ring positions must be static");
    constexpr int ROWS = R * TILE_R;                         // hidden rows of this workgroup
    __shared__ __align__(16) unsigned char sW0[STAGE_B];
    __shared__ __align__(16) unsigned char sW1[STAGE_B];
    __shared__ __align__(16) unsigned char sW2[STAGE_B];
    __shared__ __align__(16) unsigned char sW3[STAGE_B];
    __shared__ __align__(16) unsigned char sW4[STAGE_B];
    __shared__ __align__(16) unsigned char sW5[STAGE_B];
    __shared__ __align__(16) unsigned char sW6[STAGE_B];
    __shared__ __align__(16) unsigned char sW7[STAGE_B];
    __shared__ __align__(16) unsigned char sH0[STAGE_B];    // the current hidden chunk (read into registers in step 0)
    __shared__ float s_part[ROWS][4][3];                     // per hidden row: 4 partial (m, Z, T)
    __shared__ uint64_t s_key[ROWS][4];
    __shared__ int s_row[ROWS];                              // hidden row behind each of this block's slots, -1 = none
    __shared__ int s_cnt[THREADS];
    __shared__ uint64_t s_sel[TOPK ? 2 : 1][TOPK ? TILE_R : 1][2];   // candidate rounds: a row's winner per vocabulary half
    unsigned char* const sH1 = sW7;                          // R = 2: the ring has seven stages, the eighth buffer holds the second row block's chunk
#define SW(i) ((i) == 0 ? sW0 : (i) == 1 ? sW1 : (i) == 2 ? sW2 : (i) == 3 ? sW3 : (i) == 4 ? sW4 : (i) == 5 ? sW5 : (i) == 6 ? sW6 : sW7)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, half = lane >> 5;
    const int vt = wave & 1, rt = wave >> 1;
    // ---- the rows of block rb: slot j is live row number ROWS rb + j, counted over the groups in order.  Fills s_row
    // and returns the number of live rows of the whole call (the same in every thread).
    auto map_rows = [&](int rb) __attribute__((always_inline)) {
        int live = prm.rows;
        if (prm.n_valid == nullptr) {
            if (tid < ROWS) s_row[tid] = rb * ROWS + tid < prm.rows ? rb * ROWS + tid : -1;
        } else {
            const int groups = (prm.rows + prm.rows_per_group - 1) / prm.rows_per_group;
            const int want = rb * ROWS + tid;                // (threads past ROWS only help to load the counts)
            int before = 0, found = -1;
            for (int g0 = 0; g0 < groups; g0 += THREADS) {   // uniform trip count
                const int g = g0 + tid;
                s_cnt[tid] = g < groups ? max(0, min(prm.n_valid[g], min(prm.rows_per_group, prm.rows - g * prm.rows_per_group))) : 0;
                __syncthreads();
                const int here = min(THREADS, groups - g0);
                for (int j = 0; j < here; ++j) {
                    const int c = s_cnt[j];
                    if (found < 0 && want < before + c) found = (g0 + j) * prm.rows_per_group + (want - before);
                    before += c;
                }
                __syncthreads();
            }
            if (tid < ROWS) s_row[tid] = found;
            live = before;
        }
        __syncthreads();
        return live;
    };
    // A workgroup stays on its CU and takes work items (unit, row block) id, id + grid size, ...; only blocks that hold
    // live rows are items.  Workgroup ids go round-robin over the 8 XCDs and the row blocks of one unit are consecutive
    // items of one XCD, so they run side by side and share the unit's weight tiles through that XCD's L2.
    const int live_blocks = (map_rows(0) + ROWS - 1) / ROWS;
    const int items = ((prm.nunits + 7) / 8) * 8 * live_blocks;
    for (int item = blockIdx.x; item < items; item += gridDim.x) {
    const int slot = item >> 3;
    const int unit = (slot / live_blocks) * 8 + (item & 7);
    const int rb = slot % live_blocks;
    if (unit >= prm.nunits) continue;                        // (uniform)
    if (item != static_cast<int>(blockIdx.x) || rb != 0) map_rows(rb);
    const bool second = R == 2 && s_row[R == 2 ? TILE_R : 0] >= 0;   // (uniform) the second row block has live rows
    // this unit's tiles: an even share of the vocabulary, at most T; missing ones are phantom steps that re-read one
    // row (an L2 hit) and whose logits are masked, so that every unit runs the same step sequence
    const int tile_begin = static_cast<int>(static_cast<long>(unit) * prm.ntiles / prm.nunits);
    const int tile_end = static_cast<int>(static_cast<long>(unit + 1) * prm.ntiles / prm.nunits);
    const int v_end = min(prm.vocab, tile_end * TILE_V);     // one past this unit's last vocabulary row
    const int nchunk = prm.dim / CHUNK;
    const int nsteps = nchunk * T;

    // ---- loader: instruction i of wave w copies rows r, r+16, r+32, r+48 (r = 4w + i) of a 64-row tile: lane l fills
    // chunk l%16 of row r + 16 (l/16).  Vocabulary rows past the end (the last unit's missing tiles, a partial last
    // tile) re-read the last valid row; their results are masked.
    const int ld_row = (lane >> 4) * 16 + wave * 4;
    const unsigned ld_chunk_b = (lane & 15) * 16;
    // (a slot without a row re-reads the block's first row)
    const unsigned char* w_base = prm.weight + static_cast<long>(tile_begin) * TILE_V * prm.weight_stride_b;
    const int rows_mine = v_end - tile_begin * TILE_V;       // vocabulary rows of this unit (>= 1)
    const int full_tiles = rows_mine / TILE_V;               // tiles that need no clamping
    // per-lane pointers into the first tile / first chunk; a step adds one wave-uniform offset to them.  (The offset is
    // made opaque to the compiler, which would otherwise keep a separate address pair per tile and load alive across
    // the whole loop: 8 registers instead of 8 T.)
    const unsigned char* w_ptr[4];
    const unsigned char* h_ptr[R][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        w_ptr[i] = w_base + static_cast<long>(ld_row + i) * prm.weight_stride_b + ld_chunk_b;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int hr = s_row[r * TILE_R + ld_row + i] >= 0 ? s_row[r * TILE_R + ld_row + i] : s_row[0];
            h_ptr[r][i] = prm.hidden + static_cast<long>(hr) * prm.hidden_stride_b + ld_chunk_b;
        }
    }

    auto issue_w = [&](int kc, int t, auto stc) __attribute__((always_inline)) {
        constexpr int ST = decltype(stc)::value;
        LDS_AS unsigned char* dst = (LDS_AS unsigned char*)(&SW(ST)[wave * 4 * GROUP]);
        if (t < full_tiles) {
            long off = static_cast<long>(t) * TILE_V * prm.weight_stride_b + static_cast<long>(kc) * ROW_B;
            asm volatile("" : "+s"(off));
#pragma unroll
            for (int i = 0; i < 4; ++i) sage::lds_direct_load16(reinterpret_cast<const unsigned char*>(w_ptr[i] + off), dst + i * GROUP);
        } else {
            const unsigned char* wb = w_base + static_cast<long>(kc) * ROW_B;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const long r = min(t * TILE_V + ld_row + i, rows_mine - 1);
                sage::lds_direct_load16(reinterpret_cast<const unsigned char*>(wb + r * prm.weight_stride_b + ld_chunk_b), dst + i * GROUP);
            }
        }
    };
    // (every row block is requested, live or not, so that the number of loads in flight is the same on every path)
    auto issue_h = [&](int kc) __attribute__((always_inline)) {
        long off = static_cast<long>(kc) * ROW_B;
        asm volatile("" : "+s"(off));
#pragma unroll
        for (int r = 0; r < R; ++r) {
            LDS_AS unsigned char* dst = (LDS_AS unsigned char*)(&(r == 0 ? sH0 : sH1)[wave * 4 * GROUP]);
#pragma unroll
            for (int i = 0; i < 4; ++i) sage::lds_direct_load16(reinterpret_cast<const unsigned char*>(h_ptr[r][i] + off), dst + i * GROUP);
        }
    };

    // ---- per-lane read offsets: fragment kk of row r32 of this wave's half: chunk 2kk + half
    const int w_lane = (r32 & 15) * GROUP + (2 * vt + (r32 >> 4)) * ROW_B + half * 16;
    const int h_lane = (r32 & 15) * GROUP + (2 * rt + (r32 >> 4)) * ROW_B + half * 16;

    f32x16 acc[R][T];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[r][t][i] = 0.f;
    bf16x8 hb_frag[R][8];                                    // this wave's hidden rows of the current chunk (B operands)

    // one hidden chunk: T steps; J = kc mod UNROLL fixes the ring positions
    auto chunk = [&](int kc, auto jc) __attribute__((always_inline)) {
        constexpr int J = decltype(jc)::value;
        auto step = [&](auto tc) __attribute__((always_inline)) {
            constexpr int t = decltype(tc)::value;
            constexpr int ST = (J * T + t) % STAGES;
            const int s = kc * T + t;
            // This thread's loads of step s have landed; younger ones may stay in flight (the counter retires loads in
            // order): the weight tiles of the next AHEAD - 1 steps and, during steps 2..AHEAD of a chunk, the next
            // hidden chunk, requested in step 1.  Step 0 also needs the hidden chunk itself, which only the weight
            // tiles requested after it (steps 2..T-1 of the previous chunk) are younger than.
            int younger = min(AHEAD - 1, nsteps - 1 - s);
            if (t >= 2 && t <= AHEAD && kc + 1 < nchunk) younger += R;   // (a hidden chunk is R tiles' worth of loads)
            if (t == 0 && kc > 0) younger = min(younger, max(0, min(T - 2, nsteps - AHEAD - ((kc - 1) * T + 2))));
            wait_vm_tiles(younger);
            stage_barrier();                                 // ... for every wave, and the stage read last step is free
            if (s + AHEAD < nsteps) {
                constexpr int ta = (t + AHEAD) % T;
                issue_w(kc + (t + AHEAD) / T, ta, std::integral_constant<int, (ST + AHEAD) % STAGES>{});
            }
            if (t == 1 && kc + 1 < nchunk) issue_h(kc + 1);  // every wave has taken its fragments of chunk kc in step 0
            if (t == 0) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const lds_byte* hst = (const lds_byte*)(r == 0 ? sH0 : sH1) + h_lane;
#pragma unroll
                    for (int kk = 0; kk < 8; ++kk) hb_frag[r][kk] = __builtin_bit_cast(bf16x8, *(const LDS_AS uint4*)(hst + kk * 32));
                }
            }
            const lds_byte* wst = (const lds_byte*)(SW(ST)) + w_lane;
            bf16x8 a[8];
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) a[kk] = __builtin_bit_cast(bf16x8, *(const LDS_AS uint4*)(wst + kk * 32));
            __builtin_amdgcn_sched_barrier(0);
            if (R == 1 || !second) {
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], hb_frag[0][kk], acc[0][t], 0, 0, 0);
            } else {                                         // two independent chains, interleaved
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], hb_frag[0][kk], acc[0][t], 0, 0, 0);
                    acc[R - 1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], hb_frag[R - 1][kk], acc[R - 1][t], 0, 0, 0);
                }
            }
        };
        [&]<int... Is>(std::integer_sequence<int, Is...>) __attribute__((always_inline)) {
            (step(std::integral_constant<int, Is>{}), ...);
        }(std::make_integer_sequence<int, T>{});
    };

    static_assert(T >= 2 && AHEAD + R <= 8, "prologue below issues the first AHEAD steps; waits count up to seven tiles");
    issue_h(0);
    [&]<int... Is>(std::integer_sequence<int, Is...>) __attribute__((always_inline)) {
        ((Is < nsteps ? issue_w(Is / T, Is % T, std::integral_constant<int, Is % STAGES>{}) : (void)0), ...);
    }(std::make_integer_sequence<int, AHEAD>{});
    for (int kc = 0; kc < nchunk; kc += UNROLL) {
        [&]<int... Js>(std::integer_sequence<int, Js...>) __attribute__((always_inline)) {
            ((kc + Js < nchunk ? chunk(kc + Js, std::integral_constant<int, Js>{}) : (void)0), ...);
        }(std::make_integer_sequence<int, UNROLL>{});
    }

    // ---- fold the logits into softmax statistics and the best candidate of this lane's hidden row (per row block), and
    // park the four partial statistics of every hidden row (two lane halves x two vocabulary halves) in LDS
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r > 0 && !second) break;
        float m_run = -INFINITY, Z = 0.f, Tm = 0.f;
        Key best = Key{0, 0};
#pragma unroll
        for (int t = 0; t < T; ++t) {
            // vocabulary index of accumulator register i: tile*64 + 32 vt + 8 (i/4) + 4 half + i%4
            const int v0 = (tile_begin + t) * TILE_V + 32 * vt + 4 * half;
            float x[16];
            float tmax = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int v = v0 + 8 * (i >> 2) + (i & 3);
                x[i] = v < v_end ? acc[r][t][i] : -INFINITY;
                tmax = fmaxf(tmax, x[i]);
                if (v < v_end) best = key_max(best, make_key(x[i], v));
            }
            if (tmax > m_run) {                              // move the statistics to the new maximum
                if (m_run > -INFINITY) {
                    const float dlt = tmax - m_run;
                    const float sc = expf(-dlt);
                    Tm = (Tm + dlt * Z) * sc;
                    Z *= sc;
                }
                m_run = tmax;
            }
            if (m_run > -INFINITY) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float dlt = m_run - x[i];          // >= 0, +inf for masked entries
                    const float e = expf(-dlt);
                    Z += e;
                    Tm += (e > 0.f) ? e * dlt : 0.f;
                }
            }
        }
        const int hr = r * TILE_R + rt * 32 + r32;
        s_part[hr][vt * 2 + half][0] = m_run;
        s_part[hr][vt * 2 + half][1] = Z;
        s_part[hr][vt * 2 + half][2] = Tm;
        s_key[hr][vt * 2 + half] = key_pack(best);
    }
    __syncthreads();
    if (tid < ROWS && s_row[tid] >= 0) {
        float m = -INFINITY;
        Key bk = Key{0, 0};
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            m = fmaxf(m, s_part[tid][p][0]);
            bk = key_max(bk, key_unpack(s_key[tid][p]));
        }
        float z = 0.f, t = 0.f;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const float mp = s_part[tid][p][0];
            if (mp > -INFINITY) {
                const float dlt = m - mp;
                const float sc = expf(-dlt);
                z += sc * s_part[tid][p][1];
                t += sc * (s_part[tid][p][2] + s_part[tid][p][1] * dlt);
            }
        }
        const long o = static_cast<long>(s_row[tid]) * prm.nunits + unit;
        prm.stats[o] = UnitStats{m, z, t, 0.f};
        if (!TOPK) prm.keys[o] = key_pack(bk);
    }
    if constexpr (TOPK) {
        const int hr = rt * 32 + r32;
        const int row = s_row[hr];
        // the statistics are done: the logits give way, in place, to their order-preserving codes (0 = not a candidate:
        // past the unit's end, or -inf), so that a round costs one 64-bit compare pair per logit
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int v0 = (tile_begin + t) * TILE_V + 32 * vt + 4 * half;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int v = v0 + 8 * (i >> 2) + (i & 3);
                const float x = acc[0][t][i];
                acc[0][t][i] = __uint_as_float((v < v_end && x > -INFINITY) ? sortable(x) : 0u);
            }
        }
        uint64_t prev = ~0ull;                               // the previous winner: candidates come after it in the order
        for (int j = 0; j < prm.k; ++j) {
            uint64_t best = 0xFFFFFFFFull;                   // (code 0, lowest index word): below every candidate
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint32_t lo0 = 0xFFFFFFFFu - static_cast<uint32_t>((tile_begin + t) * TILE_V + 32 * vt + 4 * half);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint64_t key = (static_cast<uint64_t>(__float_as_uint(acc[0][t][i])) << 32) | (lo0 - (8 * (i >> 2) + (i & 3)));
                    best = (key < prev && key > best) ? key : best;
                }
            }
            Key mine = (best >> 32) == 0 ? Key{0, 0} : key_unpack(best);
            {                                                // the other lane half of this row
                const auto hi = __builtin_amdgcn_permlane32_swap(mine.hi, mine.hi, false, false);
                const auto lo = __builtin_amdgcn_permlane32_swap(mine.lo, mine.lo, false, false);
                mine = key_max(Key{hi[0], lo[0]}, Key{hi[1], lo[1]});
            }
            if (half == 0) s_sel[j & 1][hr][vt] = key_pack(mine);
            __syncthreads();                                 // (rounds alternate between two buffers: one barrier per round)
            const Key w = key_max(key_unpack(s_sel[j & 1][hr][0]), key_unpack(s_sel[j & 1][hr][1]));
            if (vt == 0 && half == 0 && row >= 0)
                prm.keys[(static_cast<long>(row) * prm.nunits + unit) * prm.k + j] = key_pack(w);
            prev = key_none(w) ? 0ull : key_pack(w);         // an exhausted unit: nothing comes after
        }
    }
    __syncthreads();                                         // the next item rewrites s_row and s_part
    }   // work items
#undef SW
}

inline size_t align256(size_t b) { return (b + 255) & ~static_cast<size_t>(255); }

// Launch shape: R * T <= 10 accumulators per wave (more do not fit the register file without spills).  Up to 64 rows:
// one row block, T = 5 or 10 tiles per workgroup and about one workgroup per CU, each with an even share of the tiles; a
// vocabulary too large for that takes more workgroups (several rounds).  More rows: two row blocks and T = 5.
struct Shape { int nunits, tiles_per_unit, ntiles, rows_per_wg; };
inline Shape launch_shape(int vocab, int rows) {
    Shape sh;
    sh.ntiles = (vocab + TILE_V - 1) / TILE_V;
    sh.rows_per_wg = rows > TILE_R ? 2 * TILE_R : TILE_R;
    sh.tiles_per_unit = (rows > TILE_R || sh.ntiles <= 5 * 256) ? 5 : 10;
    const int need = (sh.ntiles + sh.tiles_per_unit - 1) / sh.tiles_per_unit;
    sh.nunits = need > 256 ? need : (sh.ntiles < 256 ? sh.ntiles : 256);
    return sh;
}

}  // namespace

extern "C" size_t sage_lm_head_topk_workspace_bytes(int rows, int vocab, int k) {
    if (rows < 0 || vocab < 1 || k < 1) return 0;
    const Shape sh = launch_shape(vocab, rows);
    return align256(static_cast<size_t>(rows) * sh.nunits * sizeof(UnitStats)) +
           static_cast<size_t>(rows) * sh.nunits * k * sizeof(uint64_t) + 256;
}

extern "C" int sage_lm_head_topk(const void* hidden, const void* weight, int dtype, int rows, int dim, int vocab,
                                 long hidden_stride, long weight_stride, int k, const int* n_valid, int rows_per_group,
                                 float* entropy, int* topk_idx, float* topk_prob, float* topk_renorm,
                                 float* topk_entropy, float* alpha, void* workspace, size_t workspace_bytes, void* stream) {
    if (!hidden || !weight || !topk_idx || !workspace) return SAGE_INVALID_ARG;
    if (rows < 0 || dim < 1 || vocab < 1 || k < 1 || hidden_stride < dim || weight_stride < dim) return SAGE_INVALID_ARG;
    if (dtype != SAGE_F32 && dtype != SAGE_BF16) return SAGE_INVALID_ARG;
    if (n_valid && rows_per_group < 1) return SAGE_INVALID_ARG;
    if (k > SAGE_MAX_TOPK || k > vocab) return SAGE_INVALID_ARG;
    if (dtype != SAGE_BF16 || dim % CHUNK != 0) return SAGE_UNSUPPORTED;
    if (k > MAX_K || (k > 1 && rows > TILE_R)) return SAGE_UNSUPPORTED;   // candidate lists: the draft side, few rows
    if ((hidden_stride % 8) != 0 || (weight_stride % 8) != 0 || !sage::aligned(hidden, 16) || !sage::aligned(weight, 16) ||
        !sage::aligned(workspace, 16))
        return SAGE_INVALID_ARG;
    if (weight_stride > (1L << 24) || hidden_stride > (1L << 24)) return SAGE_UNSUPPORTED;
    if (rows > (1 << 20)) return SAGE_UNSUPPORTED;                                            // grid size
    if (workspace_bytes < sage_lm_head_topk_workspace_bytes(rows, vocab, k)) return SAGE_WORKSPACE_TOO_SMALL;
    if (rows == 0) return SAGE_OK;
    const Shape sh = launch_shape(vocab, rows);
    if (sh.nunits > sage::topk_max_units()) return SAGE_UNSUPPORTED;

    Params p;
    p.hidden = static_cast<const unsigned char*>(hidden);
    p.weight = static_cast<const unsigned char*>(weight);
    p.hidden_stride_b = hidden_stride * 2;
    p.weight_stride_b = weight_stride * 2;
    p.rows = rows; p.dim = dim; p.vocab = vocab; p.k = k; p.nunits = sh.nunits; p.ntiles = sh.ntiles;
    p.row_blocks = (rows + sh.rows_per_wg - 1) / sh.rows_per_wg;
    p.n_valid = n_valid; p.rows_per_group = rows_per_group;
    p.stats = static_cast<UnitStats*>(workspace);
    p.keys = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) +
                                         align256(static_cast<size_t>(rows) * sh.nunits * sizeof(UnitStats)));
    hipStream_t s = sage::as_stream(stream);
    const int most = ((sh.nunits + 7) / 8) * 8 * p.row_blocks;   // work items if every row is live
    const dim3 grid(most < CUS ? most : CUS);                // a workgroup fills a CU's LDS: one resident workgroup per CU
    if (sh.rows_per_wg > TILE_R) hipLaunchKernelGGL((lm_head_kernel<5, 2, false>), grid, dim3(THREADS), 0, s, p);
    else if (k > 1 && sh.tiles_per_unit == 5) hipLaunchKernelGGL((lm_head_kernel<5, 1, true>), grid, dim3(THREADS), 0, s, p);
    else if (k > 1) hipLaunchKernelGGL((lm_head_kernel<10, 1, true>), grid, dim3(THREADS), 0, s, p);
    else if (sh.tiles_per_unit == 5) hipLaunchKernelGGL((lm_head_kernel<5, 1, false>), grid, dim3(THREADS), 0, s, p);
    else hipLaunchKernelGGL((lm_head_kernel<10, 1, false>), grid, dim3(THREADS), 0, s, p);
    if (hipGetLastError() != hipSuccess) return SAGE_LAUNCH_FAILED;
    sage::topk_merge(rows, k, n_valid, rows_per_group, sh.nunits, p.stats, p.keys, entropy, topk_idx, topk_prob, topk_renorm,
                     topk_entropy, alpha, s);
    return sage::launch_status();
}
