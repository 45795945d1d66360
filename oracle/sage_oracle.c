/*
 * SAGE CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct implementation of the four per-step
 * operations of entropy-guided adaptive speculative decoding, written from the
 * paper's definitions.  It exists so that the HIP library can be checked
 * against something that shares no code with it.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.
 *
 *   O1 oracle_entropy_topk   Sec. 3.1, Eq. (7) renormalised top-k, Eq. (8)
 *                            entropy, Eq. (9) confidence; plus the full-vocab
 *                            Shannon entropy of softmax(logits), Eq. (1).
 *   O2 oracle_build_tree     Sec. 3.2, Eq. (10) depth, Eq. (11) width,
 *                            Eq. (12) per-level width decay, the recursive
 *                            expansion paragraph and the formal membership
 *                            rule that follows it.
 *   O3 oracle_tree_attention Sec. 2.2 (tree attention mask: a draft token
 *                            attends to its ancestors) applied to ordinary
 *                            softmax attention of the target's verify pass,
 *                            Alg. 1 Phase 2.
 *   O4 oracle_verify_accept  Sec. 2.2 (longest matching prefix, advance
 *                            tau+1), Sec. 3.3 Phase 2, Def. 4.1 (greedy match).
 *   O5 oracle_commit_path    Alg. 1 Phase 3 / Sec. 2.2: the accepted tokens join
 *      oracle_advance_kv_len the context, i.e. their keys and values are appended
 *                            to the KV cache and the sequence length advances.
 *   O6 oracle_update_history Sec. 3.3 "Adaptive History Tracking" with the window
 *                            and thresholds of Sec. 5 "Implementation details".
 *   O7 oracle_lm_head_topk   O1 applied to logits that are not stored but defined
 *                            as hidden . weight^T (the target's output projection,
 *                            Eq. 1 / Sec. 2.2: the distribution the greedy token of
 *                            Def. 4.1 is taken from).
 *
 * Arithmetic: O1 and O3 are plain definitions and are evaluated in fp64 from
 * the exact input bits (bf16/fp32 widened exactly), two-pass softmax, no
 * tiling, no online rescaling.  O2 is a heuristic procedure whose integer
 * outcome depends on rounding, so its real arithmetic is IEEE fp32 with the
 * four basic operations only, evaluated left to right, no fused multiply-add
 * (compile with -ffp-contract=off); that is the precision the decision is
 * defined in for both sides.  O4 and O5 are integer/byte-only.  O6 compares a
 * sum of small integers with threshold * count in fp32 (both exact for the
 * paper's thresholds).
 *
 * Pins (tests marked "not gpu"): closed forms for O1 (uniform -> ln V, one-hot
 * -> 0, shift invariance, library sort for the top-k order), brute-force
 * enumeration of the membership rule for O2, textbook causal attention for O3
 * on chain trees, brute-force path enumeration for O4; for O5 the attention of
 * a lone root over the extended cache must equal the tree attention of the
 * deepest accepted node before the commit (O3 is the independent witness); O7
 * against a library matrix product followed by O1, and closed forms; for
 * O6 hand-computed depth sequences for constant and step-change acceptance
 * lengths and a full-history recomputation of the moving average.
 * parity unpinned: the integerisation of Eq. (10)/(11)/(12) in O2 (the paper
 * gives real-valued formulas only); pinned at the end-points and by
 * monotonicity only.
 *
 * OpenMP is used only across independent rows / (sequence, node, head) units.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MAX_NODES 64

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Exact widening of one stored element to double. */
static double load_elem(const void* base, int dtype, long i) {
    if (dtype == ORACLE_F32) return (double)((const float*)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------ O1 */

typedef struct { double v; int i; } val_idx;

/* Total order used for Top_k: larger logit first, equal logits by lower index. */
static int cmp_desc_then_index(const void* a, const void* b) {
    const val_idx* x = (const val_idx*)a;
    const val_idx* y = (const val_idx*)b;
    if (x->v > y->v) return -1;
    if (x->v < y->v) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

/*
 * Per row x[0..V): P = softmax(x) (Eq. 1), H = -sum P ln P in nats with
 * 0 ln 0 = 0; Top_k = first k indices of the full sort by (x desc, index asc);
 * Ptilde = P_topk / sum P_topk (Eq. 7); Htilde = -sum Ptilde ln Ptilde (Eq. 8);
 * alpha = 1 - Htilde / ln k clamped to [0,1] (Eq. 9), alpha = 1 when k = 1.
 * Rows are grouped in groups of rows_per_group; when n_valid is given only the
 * first n_valid[g] rows of group g are computed, the others are left untouched.
 */
int oracle_entropy_topk(const void* logits, int dtype, int rows, int vocab, long row_stride, int k,
                        const int* n_valid, int rows_per_group,
                        double* entropy, int* topk_idx, double* topk_prob, double* topk_renorm,
                        double* topk_entropy, double* alpha) {
    if (!logits || rows < 0 || vocab < 1 || k < 1 || k > vocab) return 1;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < rows; ++r) {
        if (n_valid) {
            int g = r / rows_per_group, j = r % rows_per_group;
            if (j >= n_valid[g]) continue;
        }
        val_idx* s = (val_idx*)malloc(sizeof(val_idx) * (size_t)vocab);
        if (!s) { status = 4; continue; }
        double m = -INFINITY;
        for (int i = 0; i < vocab; ++i) {
            s[i].v = load_elem(logits, dtype, (long)r * row_stride + i);
            s[i].i = i;
            if (s[i].v > m) m = s[i].v;
        }
        double Z = 0.0;
        for (int i = 0; i < vocab; ++i) Z += exp(s[i].v - m);
        double H = 0.0;
        for (int i = 0; i < vocab; ++i) {
            double p = exp(s[i].v - m) / Z;
            if (p > 0.0) H -= p * log(p);
        }
        entropy[r] = H;

        qsort(s, (size_t)vocab, sizeof(val_idx), cmp_desc_then_index);
        double mass = 0.0;
        for (int j = 0; j < k; ++j) {
            double p = exp(s[j].v - m) / Z;
            topk_idx[(long)r * k + j] = s[j].i;
            topk_prob[(long)r * k + j] = p;
            mass += p;
        }
        double Hk = 0.0;
        for (int j = 0; j < k; ++j) {
            double q = topk_prob[(long)r * k + j] / mass;
            topk_renorm[(long)r * k + j] = q;
            if (q > 0.0) Hk -= q * log(q);
        }
        topk_entropy[r] = Hk;
        double a = (k == 1) ? 1.0 : 1.0 - Hk / log((double)k);
        if (a < 0.0) a = 0.0;
        if (a > 1.0) a = 1.0;
        alpha[r] = a;
        free(s);
    }
    return status;
}

/* ------------------------------------------------------------------ O2 */

typedef struct {
    int d_min, d_max, w_min, w_max, k, n_max;
} oracle_tree_params;

typedef struct {
    const float* ptilde; /* renormalised top-k of this sequence, descending */
    int k, n_max, D;
    float W;             /* integerised width, kept as a float value */
    int n;
    int* parent; int* depth; int* rank; uint64_t* mask; float* cum;
} tree_state;

/*
 * Expand node u (depth l-1, cumulative path probability cum[u]) into level l.
 * Level 1 uses W undecayed; deeper levels use Eq. (12) with the parent's
 * cumulative probability, integerised as min(k, max(1, floor(.))).  A
 * candidate of rank r < W_l joins the tree iff its cumulative probability
 * exceeds theta_l = 0.1*l/D (strict); a joined node is expanded at once
 * (depth-first, ranks ascending).  Nothing is added once n_max nodes exist.
 */
static void expand(tree_state* t, int u) {
    int l = t->depth[u] + 1;
    if (l > t->D) return;
    int Wl;
    if (l == 1) {
        Wl = (int)t->W;
    } else {
        float per_level = t->W / (float)l;
        float boost = 0.5f + t->cum[u];
        float w = floorf(per_level * boost);
        Wl = (int)w;
        if (Wl < 1) Wl = 1;
    }
    if (Wl > t->k) Wl = t->k;
    float theta = (0.1f * (float)l) / (float)t->D;
    for (int r = 0; r < Wl; ++r) {
        if (t->n >= t->n_max) return;
        float c = t->cum[u] * t->ptilde[r];
        if (c > theta) {
            int v = t->n++;
            t->parent[v] = u;
            t->depth[v] = l;
            t->rank[v] = r;
            t->cum[v] = c;
            t->mask[v] = t->mask[u] | ((uint64_t)1 << v);
            expand(t, v);
        }
    }
}

/*
 * Per sequence b: D = round-half-up of Eq. (10), W = round-half-up of Eq. (11)
 * capped at k; root = node 0 (parent -1, depth 0, rank -1, cum 1); nodes are
 * emitted in creation order (DFS pre-order), so parent[v] < v.  Arrays are
 * [B, 64]; entries at or beyond n_nodes[b] are left untouched.  When the
 * candidates' vocabulary ids topk_idx [B,k] are given, node_token[v] is the
 * id of the candidate node v stands for (root -1).  When d_max_seq [B] is
 * given, sequence b uses d_max_seq[b] (clamped to [d_min, 31]) as the D_max of
 * Eq. (10): the maximum depth that adaptive history tracking maintains.
 */
int oracle_build_tree(const float* topk_renorm, const float* alpha, const int* topk_idx, int B, int k,
                      const oracle_tree_params* p, const int* d_max_seq,
                      int* n_nodes, int* parent, int* depth, int* rank, uint64_t* anc_mask,
                      float* cum_prob, int* node_token) {
    if (!topk_renorm || !alpha || !p || B < 0) return 1;
    if (p->k != k || k < 1 || p->n_max < 1 || p->n_max > ORACLE_MAX_NODES) return 1;
    if (p->d_min < 1 || p->d_min > p->d_max || p->w_min < 1 || p->w_min > p->w_max || p->w_max > k) return 1;
    for (int b = 0; b < B; ++b) {
        float a = alpha[b];
        int d_max = p->d_max;
        if (d_max_seq) {
            d_max = d_max_seq[b];
            if (d_max < p->d_min) d_max = p->d_min;
            if (d_max > 31) d_max = 31;
        }
        float D = floorf(((float)p->d_min + a * (float)(d_max - p->d_min)) + 0.5f);
        float W = floorf(((float)p->w_min + (1.0f - a) * (float)(p->w_max - p->w_min)) + 0.5f);
        if (W > (float)k) W = (float)k;
        float cum_local[ORACLE_MAX_NODES];
        tree_state t;
        t.ptilde = topk_renorm + (long)b * k;
        t.k = k; t.n_max = p->n_max; t.D = (int)D; t.W = W; t.n = 1;
        t.parent = parent + (long)b * ORACLE_MAX_NODES;
        t.depth = depth + (long)b * ORACLE_MAX_NODES;
        t.rank = rank + (long)b * ORACLE_MAX_NODES;
        t.mask = anc_mask + (long)b * ORACLE_MAX_NODES;
        t.cum = cum_prob ? cum_prob + (long)b * ORACLE_MAX_NODES : cum_local;
        t.parent[0] = -1; t.depth[0] = 0; t.rank[0] = -1; t.cum[0] = 1.0f; t.mask[0] = 1;
        expand(&t, 0);
        n_nodes[b] = t.n;
        /* a node stands for the candidate of its rank: its draft token is that candidate's vocabulary id */
        if (node_token && topk_idx) {
            node_token[(long)b * ORACLE_MAX_NODES] = -1;
            for (int v = 1; v < t.n; ++v)
                node_token[(long)b * ORACLE_MAX_NODES + v] = topk_idx[(long)b * k + t.rank[v]];
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ O3 */

/*
 * For sequence b, tree node i < n_nodes[b], query head h (kv head g = h / G):
 * keys are every cache position j < kv_len[b] and every tree node t whose bit
 * is set in anc_mask[b][i] (ancestor-or-self); score = scale * q.k; softmax
 * over that union; output = sum of probabilities times values.  Layouts:
 * Q, O [B,64,Hq,d]; Kt, Vt [B,64,Hkv,d]; cache element (b, j, g, c) at
 * (kv_start[b] + j) * kv_token_stride + g * kv_head_stride + c.
 * Output is fp64, not rounded to the storage type.
 */
int oracle_tree_attention(const void* Q, const void* Kc, const void* Vc, const void* Kt, const void* Vt,
                          double* O, int dtype, int B, int Hq, int Hkv, int d,
                          const long* kv_start, const int* kv_len,
                          long kv_token_stride, long kv_head_stride,
                          const uint64_t* anc_mask, const int* n_nodes, double scale) {
    if (!Q || !Kt || !Vt || !O || Hkv < 1 || Hq % Hkv != 0 || d < 1) return 1;
    const int G = Hq / Hkv;
    long units = (long)B * ORACLE_MAX_NODES * Hq;
#pragma omp parallel for schedule(dynamic, 4)
    for (long u = 0; u < units; ++u) {
        int h = (int)(u % Hq);
        int i = (int)((u / Hq) % ORACLE_MAX_NODES);
        int b = (int)(u / ((long)Hq * ORACLE_MAX_NODES));
        if (i >= n_nodes[b]) continue;
        int g = h / G;
        int L = kv_len[b];
        long qoff = (((long)b * ORACLE_MAX_NODES + i) * Hq + h) * d;
        uint64_t mask = anc_mask[(long)b * ORACLE_MAX_NODES + i];
        int nt = n_nodes[b];
        double* s = (double*)malloc(sizeof(double) * (size_t)(L + ORACLE_MAX_NODES));
        double m = -INFINITY;
        for (int j = 0; j < L; ++j) {
            long koff = (kv_start[b] + j) * kv_token_stride + (long)g * kv_head_stride;
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += load_elem(Q, dtype, qoff + c) * load_elem(Kc, dtype, koff + c);
            s[j] = scale * acc;
            if (s[j] > m) m = s[j];
        }
        for (int t = 0; t < nt; ++t) {
            if (!((mask >> t) & 1)) { s[L + t] = -INFINITY; continue; }
            long koff = (((long)b * ORACLE_MAX_NODES + t) * Hkv + g) * d;
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += load_elem(Q, dtype, qoff + c) * load_elem(Kt, dtype, koff + c);
            s[L + t] = scale * acc;
            if (s[L + t] > m) m = s[L + t];
        }
        double Z = 0.0;
        for (int j = 0; j < L + nt; ++j) Z += exp(s[j] - m);
        double* out = O + qoff;
        for (int c = 0; c < d; ++c) out[c] = 0.0;
        for (int j = 0; j < L; ++j) {
            double p = exp(s[j] - m) / Z;
            long voff = (kv_start[b] + j) * kv_token_stride + (long)g * kv_head_stride;
            for (int c = 0; c < d; ++c) out[c] += p * load_elem(Vc, dtype, voff + c);
        }
        for (int t = 0; t < nt; ++t) {
            if (!((mask >> t) & 1)) continue;
            double p = exp(s[L + t] - m) / Z;
            long voff = (((long)b * ORACLE_MAX_NODES + t) * Hkv + g) * d;
            for (int c = 0; c < d; ++c) out[c] += p * load_elem(Vt, dtype, voff + c);
        }
        free(s);
    }
    return 0;
}

/* ------------------------------------------------------------------ O4 */

/*
 * Per sequence: node i > 0 matches iff its draft token equals the target's
 * greedy token at its parent; a node is accepted iff it and every ancestor
 * match (walked through parent pointers); the result is the deepest accepted
 * node, ties to the lowest index; tau = its depth; the emitted tokens are the
 * tau draft tokens on the root-to-best path followed by the target's greedy
 * token at the best node.  path_nodes/out_tokens are [B, path_cap], padded -1.
 */
int oracle_verify_accept(const int* token, const int* target_argmax, const int* parent, const int* depth,
                         const int* n_nodes, int B, int path_cap,
                         int* accept_len, int* best_node, int* path_nodes, int* out_tokens) {
    if (!token || !target_argmax || !parent || !depth || !n_nodes || path_cap < 1) return 1;
    for (int b = 0; b < B; ++b) {
        const int* tok = token + (long)b * ORACLE_MAX_NODES;
        const int* tgt = target_argmax + (long)b * ORACLE_MAX_NODES;
        const int* par = parent + (long)b * ORACLE_MAX_NODES;
        const int* dep = depth + (long)b * ORACLE_MAX_NODES;
        int n = n_nodes[b];
        int best = 0;
        for (int i = 1; i < n; ++i) {
            int accepted = 1;
            for (int v = i; v > 0; v = par[v])
                if (tok[v] != tgt[par[v]]) accepted = 0;
            if (accepted && dep[i] > dep[best]) best = i;
        }
        int tau = dep[best];
        if (tau + 1 > path_cap) return 1;
        accept_len[b] = tau;
        best_node[b] = best;
        int* path = path_nodes + (long)b * path_cap;
        int* out = out_tokens + (long)b * path_cap;
        for (int j = 0; j < path_cap; ++j) { path[j] = -1; out[j] = -1; }
        for (int v = best; v >= 0; v = par[v]) path[dep[v]] = v;
        for (int j = 1; j <= tau; ++j) out[j - 1] = tok[path[j]];
        out[tau] = tgt[best];
    }
    return 0;
}

/* ------------------------------------------------------------------ O5 */

static size_t elem_size(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

/*
 * One layer's share of committing the accepted path.  For sequence b with
 * tau = accept_len[b] and path = path_nodes[b][0..tau] (root first, as
 * verify_accept emits it), the key and value rows of the tau + 1 path nodes
 * (the root, whose K/V is not in the cache yet, and the tau accepted draft
 * tokens) are copied, bytes unchanged, to cache positions kv_len[b] + j,
 * j = 0..tau.  The bonus token has no K/V yet: it is the next step's root.
 * Positions at or beyond kv_capacity are not written.  kv_len is not changed
 * here (every layer commits against the same old length).
 */
int oracle_commit_path(const void* Kt, const void* Vt, void* Kc, void* Vc, int dtype, int B, int Hkv, int d,
                       const int64_t* kv_start, const int* kv_len, int kv_capacity,
                       long kv_token_stride, long kv_head_stride,
                       const int* path_nodes, const int* accept_len, int path_cap) {
    if (!Kt || !Vt || !Kc || !Vc || !kv_start || !kv_len || !path_nodes || !accept_len) return 1;
    if (B < 0 || Hkv < 1 || d < 1 || path_cap < 1 || kv_capacity < 0) return 1;
    const size_t es = elem_size(dtype);
    for (int b = 0; b < B; ++b) {
        const int tau = accept_len[b];
        if (tau < 0 || tau + 1 > path_cap) return 1;
        for (int j = 0; j <= tau; ++j) {
            const int node = path_nodes[(long)b * path_cap + j];
            const long pos = (long)kv_len[b] + j;
            if (node < 0 || node >= ORACLE_MAX_NODES) return 1;
            if (pos >= kv_capacity) break;
            for (int g = 0; g < Hkv; ++g) {
                const size_t src = ((((size_t)b * ORACLE_MAX_NODES + node) * Hkv + g) * d) * es;
                const size_t dst = (size_t)((kv_start[b] + pos) * kv_token_stride + (long)g * kv_head_stride) * es;
                memcpy((char*)Kc + dst, (const char*)Kt + src, (size_t)d * es);
                memcpy((char*)Vc + dst, (const char*)Vt + src, (size_t)d * es);
            }
        }
    }
    return 0;
}

/* After every layer has committed: the sequence grows by the root and the tau accepted tokens. */
int oracle_advance_kv_len(int* kv_len, const int* accept_len, int B, int kv_capacity) {
    if (!kv_len || !accept_len || B < 0) return 1;
    for (int b = 0; b < B; ++b) {
        long n = (long)kv_len[b] + accept_len[b] + 1;
        kv_len[b] = n > kv_capacity ? kv_capacity : (int)n;
    }
    return 0;
}

/* ------------------------------------------------------------------ O6 */

/*
 * Adaptive history tracking.  Per sequence: the step's acceptance length is
 * pushed into a sliding window of the last `window` values (a ring: slot =
 * count mod window); the moving average runs over the values present (fewer
 * than `window` during the first steps).  Average below `lo` (strictly): the
 * maximum depth drops by one, not below d_floor; average above `hi`
 * (strictly): it rises by one, not above d_cap; in between it stays.  The
 * comparison is sum < lo * n, resp. sum > hi * n, in fp32.
 */
int oracle_update_history(const int* accept_len, int B, int window, float lo, float hi, int d_floor, int d_cap,
                          int* hist, int* count, int* d_max, float* avg_out) {
    if (!accept_len || !hist || !count || !d_max || B < 0 || window < 1 || window > 64) return 1;
    if (d_floor < 1 || d_floor > d_cap || !(lo <= hi)) return 1;
    for (int b = 0; b < B; ++b) {
        int* h = hist + (long)b * window;
        h[count[b] % window] = accept_len[b];
        count[b] += 1;
        const int n = count[b] < window ? count[b] : window;
        int sum = 0;
        for (int i = 0; i < n; ++i) sum += h[i];
        const float fs = (float)sum, fn = (float)n;
        if (avg_out) avg_out[b] = fs / fn;
        int dm = d_max[b];
        if (fs < lo * fn) dm -= 1;
        else if (fs > hi * fn) dm += 1;
        if (dm < d_floor) dm = d_floor;
        if (dm > d_cap) dm = d_cap;
        d_max[b] = dm;
    }
    return 0;
}

/* ------------------------------------------------------------------ O7 */

/*
 * O1 on logits x[r][v] = sum_c hidden[r][c] * weight[v][c], evaluated in fp64
 * from the exact stored bits (hidden [rows, dim], weight [vocab, dim], both
 * row-major with the given row strides, same storage type).  The logits are
 * never rounded to a storage type: the statistics and the order are those of
 * the fp64 products.  Row groups and n_valid as in O1.
 */
int oracle_lm_head_topk(const void* hidden, const void* weight, int dtype, int rows, int dim, int vocab,
                        long hidden_stride, long weight_stride, int k, const int* n_valid, int rows_per_group,
                        double* entropy, int* topk_idx, double* topk_prob, double* topk_renorm,
                        double* topk_entropy, double* alpha, double* logits_out) {
    if (!hidden || !weight || rows < 0 || dim < 1 || vocab < 1 || k < 1 || k > vocab) return 1;
    for (int r = 0; r < rows; ++r) {
        if (n_valid) {
            int g = r / rows_per_group, j = r % rows_per_group;
            if (j >= n_valid[g]) continue;
        }
        val_idx* s = (val_idx*)malloc(sizeof(val_idx) * (size_t)vocab);
        double* h = (double*)malloc(sizeof(double) * (size_t)dim);
        if (!s || !h) { free(s); free(h); return 4; }
        for (int c = 0; c < dim; ++c) h[c] = load_elem(hidden, dtype, (long)r * hidden_stride + c);
#pragma omp parallel for schedule(static)
        for (int v = 0; v < vocab; ++v) {
            double x = 0.0;
            for (int c = 0; c < dim; ++c) x += h[c] * load_elem(weight, dtype, (long)v * weight_stride + c);
            s[v].v = x;
            s[v].i = v;
        }
        if (logits_out)
            for (int v = 0; v < vocab; ++v) logits_out[(long)r * vocab + v] = s[v].v;
        double m = -INFINITY;
        for (int v = 0; v < vocab; ++v) if (s[v].v > m) m = s[v].v;
        double Z = 0.0;
        for (int v = 0; v < vocab; ++v) Z += exp(s[v].v - m);
        double H = 0.0;
        for (int v = 0; v < vocab; ++v) {
            double p = exp(s[v].v - m) / Z;
            if (p > 0.0) H -= p * log(p);
        }
        entropy[r] = H;
        qsort(s, (size_t)vocab, sizeof(val_idx), cmp_desc_then_index);
        double mass = 0.0;
        for (int j = 0; j < k; ++j) {
            double p = exp(s[j].v - m) / Z;
            topk_idx[(long)r * k + j] = s[j].i;
            topk_prob[(long)r * k + j] = p;
            mass += p;
        }
        double Hk = 0.0;
        for (int j = 0; j < k; ++j) {
            double q = topk_prob[(long)r * k + j] / mass;
            topk_renorm[(long)r * k + j] = q;
            if (q > 0.0) Hk -= q * log(q);
        }
        topk_entropy[r] = Hk;
        double a = (k == 1) ? 1.0 : 1.0 - Hk / log((double)k);
        alpha[r] = a < 0.0 ? 0.0 : (a > 1.0 ? 1.0 : a);
        free(s);
        free(h);
    }
    return 0;
}
