/*
 * DySpec CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of the three operations of one DySpec
 * speculative step, written from the paper (arXiv 2410.11744):
 *
 *   oracle_build_tree   greedy fixed-budget token-tree construction (Algorithm 1,
 *                       Section 4.2 and Appendix A.1)
 *   oracle_tree_attn    attention of the tree tokens over prefix + ancestors under
 *                       the ancestor mask (Section 2, "Tree Attention")
 *   oracle_verify       multi-candidate tree rejection sampling (Algorithm 3,
 *                       Appendix A.3)
 *   oracle_softmax_stats / oracle_accept_ratio_all   per-row softmax normalisers and
 *                       the conditional acceptance ratio of every node (inner loop of
 *                       Algorithm 3 with every earlier sibling rejected)
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this
 * file.  It shares no code with the GPU library and neither includes the other.
 *
 * Random numbers: every draw is a uniform in [0,1) with 24 bits, produced either by
 * Philox4x32-10 (Salmon et al., SC'11) from a counter that names the draw by the path
 * of sibling ranks leading to it, or taken from caller-supplied tables (tests use the
 * tables to integrate the algorithm's output law exactly).
 *
 * Pins (see tests/test_oracle_*.py): Philox known answers; closed form of every slot
 * value (Appendix D); greedy = max-weight connected subtree (Appendix D.1); chain tree
 * = causal attention; one child = plain speculative sampling (Section 2); exact output
 * law on trees of 1-4 nodes; 10^6-trial marginals at V = 8; a temperature-0 target =
 * the limit of small temperatures = following the target's argmax token down the tree.
 * The sample PATH for a given seed (which token, which accept) is fixed by this
 * file's own conventions (inverse CDF in ascending token order, the counter layout)
 * and is "parity unpinned" by the paper.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the attention routines spread independent rows over. */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sets the number of threads for the attention routines (timing only: results do not depend
 * on it, every row is computed by one thread on its own). */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------ Philox4x32-10 */

static void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;  /* multipliers (SC'11, Table 2) */
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;  /* Weyl key increments          */
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out)
{
    philox4x32_10(ctr, key, out);
}

enum { KIND_PATH = 0, KIND_BUILD = 1, KIND_ACCEPT = 2, KIND_RESID = 3 };

typedef struct { uint32_t lo, hi; } pathkey;

/* Source of uniforms.  mode 0: Philox keyed by (seed; path key, rank, kind).
 * mode 1: tables indexed by node creation index. */
typedef struct {
    int mode;
    uint64_t seed;
    const double* u_build;   /* [N]: draw used when node i is created            */
    const double* u_accept;  /* [N]: draw used when node i is tested             */
    const double* u_resid;   /* [N]: draw used when the walk stops at node i     */
} draw_source;

static double philox_u01(uint64_t seed, pathkey pk, uint32_t rank, uint32_t kind)
{
    uint32_t ctr[4] = { pk.lo, pk.hi, rank, kind };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    philox4x32_10(ctr, key, w);
    return (double)(w[0] >> 8) * (1.0 / 16777216.0);
}

static pathkey child_key(uint64_t seed, pathkey pk, uint32_t rank)
{
    uint32_t ctr[4] = { pk.lo, pk.hi, rank, KIND_PATH };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    philox4x32_10(ctr, key, w);
    pathkey c = { w[0], w[1] };
    return c;
}

static pathkey root_key(uint32_t seq) { pathkey r = { seq, 0u }; return r; }

double oracle_u01(uint64_t seed, uint32_t pk_lo, uint32_t pk_hi, uint32_t rank, uint32_t kind)
{
    pathkey pk = { pk_lo, pk_hi };
    return philox_u01(seed, pk, rank, kind);
}

/* ------------------------------------------------------------------ softmax rows */

/* p = softmax(logits / temp) in fp64; returns m = max(logits)/temp and writes
 * s = sum exp(logits/temp - m).
 * temp == 0 is the limit temp -> 0+ (Section 5, the temperature-0 target rows of the
 * result tables): all mass on the largest logit, the smallest index winning a tie.  Then
 * the return value is that largest raw logit and s is the index that holds it. */
static double softmax_row(const float* logits, int V, double temp, double* p, double* s_out)
{
    if (temp == 0.0) {
        int a = 0;
        for (int x = 1; x < V; ++x) if (logits[x] > logits[a]) a = x;
        for (int x = 0; x < V; ++x) p[x] = 0.0;
        p[a] = 1.0;
        if (s_out) *s_out = (double)a;
        return (double)logits[a];
    }
    double m = -INFINITY;
    for (int x = 0; x < V; ++x) { double z = (double)logits[x] / temp; if (z > m) m = z; }
    double s = 0.0;
    for (int x = 0; x < V; ++x) { p[x] = exp((double)logits[x] / temp - m); s += p[x]; }
    for (int x = 0; x < V; ++x) p[x] /= s;
    if (s_out) *s_out = s;
    return m;
}

void oracle_softmax(const float* logits, int V, double temp, double* p)
{
    softmax_row(logits, V, temp, p, NULL);
}

/* stats[4*i + {0,1,2,3}] = (max_d, sumexp_d, max_t, sumexp_t) for row i; at temp_t == 0
 * the last two are (largest raw target logit, its index) */
void oracle_softmax_stats(const float* draft_logits, const float* target_logits, int n_rows,
                          int V, double temp_d, double temp_t, double* stats)
{
    double* p = (double*)malloc(sizeof(double) * (size_t)V);
    for (int i = 0; i < n_rows; ++i) {
        double s;
        stats[4 * i + 0] = softmax_row(draft_logits + (size_t)i * V, V, temp_d, p, &s);
        stats[4 * i + 1] = s;
        stats[4 * i + 2] = softmax_row(target_logits + (size_t)i * V, V, temp_t, p, &s);
        stats[4 * i + 3] = s;
    }
    free(p);
}

/* Inverse CDF over non-negative weights w[0..V) in ascending index: smallest y with
 * sum_{x<=y} w[x] > u*W.  Zero-weight entries are never chosen.  *margin receives the
 * distance of u*W to the nearest edge of y's interval, divided by W. */
static int inverse_cdf(const double* w, int V, double u, double* W_out, double* margin)
{
    double W = 0.0;
    for (int x = 0; x < V; ++x) W += w[x];
    double target = u * W, cum = 0.0;
    int y = -1, last = -1;
    double lo = 0.0, hi = 0.0;
    for (int x = 0; x < V; ++x) {
        if (w[x] > 0.0) last = x;
        double next = cum + w[x];
        if (next > target) { y = x; lo = cum; hi = next; break; }
        cum = next;
    }
    if (y < 0) { y = last; lo = hi = target; }   /* rounding at the very top edge */
    if (W_out) *W_out = W;
    if (margin) {
        double a = target - lo, b = hi - target;
        *margin = (W > 0.0) ? (a < b ? a : b) / W : 0.0;
    }
    return y;
}

/* ------------------------------------------------------------------ Algorithm 1 */

/*
 * Greedy expansion with budget n_budget rows INCLUDING the root (row 0).
 * draft_logits[i*V ..] is the draft model's distribution over the token that follows
 * node i (i = creation index; row 0 follows the prefix).
 *
 * A "slot" is one expandable position: (parent p, number of children p already has,
 * estimated value v).  Each step takes the slot of largest v (earliest-created on a
 * tie), samples a token from p's draft distribution with p's earlier children removed
 * and renormalised, creates the node, and opens the two slots Algorithm 1 pushes:
 * next sibling with v*(1-R[y]) and first child with v*R[y].  Slots with v <= 0 are
 * never opened.
 *
 * Outputs (size n_budget unless noted): parent, token, sib_rank, first_child,
 * next_sibling (sampling order, -1 = none), depth, est_value (v of the slot the node
 * was sampled from; 1 for the root), mask [n_budget * mask_words] (bit i of row j set
 * iff i is an ancestor of j or i == j), margin_pop / margin_cdf per created node
 * (relative margin of the arg-max and of the inverse-CDF decision that produced it).
 * Rows >= *n_built keep parent = token = -1 and a mask row holding only their own bit.
 */
static void build_tree_core(const float* draft_logits, int V, int n_budget, double temp,
                            const draw_source* src, uint32_t seq,
                            int32_t* parent, int32_t* token, int32_t* sib_rank,
                            int32_t* first_child, int32_t* next_sibling, int32_t* depth,
                            double* est_value, uint64_t* mask, int mask_words,
                            int32_t* n_built, double* margin_pop, double* margin_cdf)
{
    int N = n_budget;
    int max_slots = 2 * N + 2;
    int32_t* slot_parent = (int32_t*)malloc(sizeof(int32_t) * max_slots);
    double* slot_value = (double*)malloc(sizeof(double) * max_slots);
    char* slot_live = (char*)calloc(max_slots, 1);
    int32_t* n_children = (int32_t*)calloc(N, sizeof(int32_t));
    int32_t* last_child = (int32_t*)malloc(sizeof(int32_t) * N);
    pathkey* pk = (pathkey*)malloc(sizeof(pathkey) * N);
    double* w = (double*)malloc(sizeof(double) * (size_t)V);
    int n_slots = 0;

    for (int i = 0; i < N; ++i) {
        parent[i] = -1; token[i] = -1; sib_rank[i] = 0; first_child[i] = -1;
        next_sibling[i] = -1; depth[i] = 0; est_value[i] = 0.0; last_child[i] = -1;
        margin_pop[i] = INFINITY; margin_cdf[i] = INFINITY;
        for (int k = 0; k < mask_words; ++k) mask[(size_t)i * mask_words + k] = 0;
        mask[(size_t)i * mask_words + i / 64] = 1ull << (i % 64);
    }
    est_value[0] = 1.0;
    pk[0] = root_key(seq);
    slot_parent[0] = 0; slot_value[0] = 1.0; slot_live[0] = 1; n_slots = 1;

    int n = 1;
    while (n < N) {
        /* pop: live slot of largest value, earliest-created on ties */
        int best = -1; double v_best = 0.0, v_second = 0.0;
        for (int s = 0; s < n_slots; ++s) {
            if (!slot_live[s]) continue;
            if (best < 0 || slot_value[s] > v_best) {
                if (best >= 0) v_second = v_best;
                best = s; v_best = slot_value[s];
            } else if (slot_value[s] > v_second) {
                v_second = slot_value[s];
            }
        }
        if (best < 0) break;                       /* frontier is empty */
        slot_live[best] = 0;
        int p = slot_parent[best];
        double v = v_best;

        /* residual draft distribution of p: earlier children removed */
        softmax_row(draft_logits + (size_t)p * V, V, temp, w, NULL);
        for (int c = first_child[p]; c >= 0; c = next_sibling[c]) w[token[c]] = 0.0;

        int rank = n_children[p];
        double u = (src->mode == 0) ? philox_u01(src->seed, pk[p], (uint32_t)rank, KIND_BUILD)
                                    : src->u_build[n];
        double W, mc;
        int y = inverse_cdf(w, V, u, &W, &mc);
        if (y < 0 || !(W > 0.0)) break;            /* nothing left to sample under p */
        double Ry = w[y] / W;

        int i = n++;
        parent[i] = p; token[i] = y; sib_rank[i] = rank; depth[i] = depth[p] + 1;
        est_value[i] = v;
        margin_pop[i] = (v_best > 0.0) ? (v_best - v_second) / v_best : 0.0;
        margin_cdf[i] = mc;
        if (last_child[p] < 0) first_child[p] = i; else next_sibling[last_child[p]] = i;
        last_child[p] = i; n_children[p] = rank + 1;
        pk[i] = (src->mode == 0) ? child_key(src->seed, pk[p], (uint32_t)rank) : root_key(0);
        for (int k = 0; k < mask_words; ++k)
            mask[(size_t)i * mask_words + k] |= mask[(size_t)p * mask_words + k];

        double v0 = v * Ry;            /* first child of the new node       */
        double v1 = v * (1.0 - Ry);    /* next sampling at the same position */
        if (v1 > 0.0) { slot_parent[n_slots] = p; slot_value[n_slots] = v1; slot_live[n_slots] = 1; ++n_slots; }
        if (v0 > 0.0) { slot_parent[n_slots] = i; slot_value[n_slots] = v0; slot_live[n_slots] = 1; ++n_slots; }
    }
    *n_built = n;
    free(slot_parent); free(slot_value); free(slot_live); free(n_children);
    free(last_child); free(pk); free(w);
}

void oracle_build_tree(const float* draft_logits, int V, int n_budget, double temp,
                       uint64_t seed, uint32_t seq,
                       int32_t* parent, int32_t* token, int32_t* sib_rank,
                       int32_t* first_child, int32_t* next_sibling, int32_t* depth,
                       double* est_value, uint64_t* mask, int mask_words,
                       int32_t* n_built, double* margin_pop, double* margin_cdf)
{
    draw_source src = { 0, seed, NULL, NULL, NULL };
    build_tree_core(draft_logits, V, n_budget, temp, &src, seq, parent, token, sib_rank,
                    first_child, next_sibling, depth, est_value, mask, mask_words,
                    n_built, margin_pop, margin_cdf);
}

void oracle_build_tree_explicit(const float* draft_logits, int V, int n_budget, double temp,
                                const double* u_build,
                                int32_t* parent, int32_t* token, int32_t* sib_rank,
                                int32_t* first_child, int32_t* next_sibling, int32_t* depth,
                                double* est_value, uint64_t* mask, int mask_words,
                                int32_t* n_built, double* margin_pop, double* margin_cdf)
{
    draw_source src = { 1, 0, u_build, NULL, NULL };
    build_tree_core(draft_logits, V, n_budget, temp, &src, 0, parent, token, sib_rank,
                    first_child, next_sibling, depth, est_value, mask, mask_words,
                    n_built, margin_pop, margin_cdf);
}

/* Ancestor mask from a parent array alone (parents precede children). */
void oracle_ancestor_mask(const int32_t* parent, int N, uint64_t* mask, int mask_words)
{
    for (int j = 0; j < N; ++j) {
        for (int k = 0; k < mask_words; ++k) mask[(size_t)j * mask_words + k] = 0;
        for (int a = j; a >= 0; a = parent[a])
            mask[(size_t)j * mask_words + a / 64] |= 1ull << (a % 64);
    }
}

/* ------------------------------------------------------------------ tree attention */

/*
 * One output row: query (node j, head h) against all P prefix keys and the tree keys
 * i with mask bit (j,i) set; softmax over the visible keys; weighted sum of values.
 * Layouts: q [N,Hq,d]; k_prefix,v_prefix [P,Hkv,d]; k_tree,v_tree [N,Hkv,d];
 * query head h reads KV head h / (Hq/Hkv).
 */
static void attn_row(const float* q, const float* kp, const float* vp, const float* kt,
                     const float* vt, const uint64_t* mask, int mask_words,
                     int N, int P, int Hq, int Hkv, int d, double scale,
                     int j, int h, double* out_row, double* score_buf)
{
    int g = h / (Hq / Hkv);
    const float* qv = q + ((size_t)j * Hq + h) * d;
    double m = -INFINITY;
    for (int k = 0; k < P + N; ++k) {
        int visible = 1;
        const float* kv;
        if (k < P) kv = kp + ((size_t)k * Hkv + g) * d;
        else {
            int i = k - P;
            visible = (int)((mask[(size_t)j * mask_words + i / 64] >> (i % 64)) & 1ull);
            kv = kt + ((size_t)i * Hkv + g) * d;
        }
        if (!visible) { score_buf[k] = -INFINITY; continue; }
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += (double)qv[c] * (double)kv[c];
        s *= scale;
        score_buf[k] = s;
        if (s > m) m = s;
    }
    double denom = 0.0;
    for (int k = 0; k < P + N; ++k) {
        score_buf[k] = (score_buf[k] == -INFINITY) ? 0.0 : exp(score_buf[k] - m);
        denom += score_buf[k];
    }
    for (int c = 0; c < d; ++c) out_row[c] = 0.0;
    for (int k = 0; k < P + N; ++k) {
        if (score_buf[k] == 0.0) continue;
        const float* vv = (k < P) ? vp + ((size_t)k * Hkv + g) * d
                                  : vt + ((size_t)(k - P) * Hkv + g) * d;
        double pk_ = score_buf[k] / denom;
        for (int c = 0; c < d; ++c) out_row[c] += pk_ * (double)vv[c];
    }
}

/* All rows: out [N,Hq,d] fp64. */
void oracle_tree_attn(const float* q, const float* kp, const float* vp, const float* kt,
                      const float* vt, const uint64_t* mask, int mask_words,
                      int N, int P, int Hq, int Hkv, int d, double scale, double* out)
{
#pragma omp parallel
    {
        double* buf = (double*)malloc(sizeof(double) * (size_t)(P + N));
#pragma omp for collapse(2) schedule(static)
        for (int j = 0; j < N; ++j)
            for (int h = 0; h < Hq; ++h)
                attn_row(q, kp, vp, kt, vt, mask, mask_words, N, P, Hq, Hkv, d, scale, j, h,
                         out + ((size_t)j * Hq + h) * d, buf);
        free(buf);
    }
}

/* Selected rows only: out [n_rows, d]; rows_j / rows_h name (node, head). */
void oracle_tree_attn_rows(const float* q, const float* kp, const float* vp, const float* kt,
                           const float* vt, const uint64_t* mask, int mask_words,
                           int N, int P, int Hq, int Hkv, int d, double scale,
                           int n_rows, const int32_t* rows_j, const int32_t* rows_h, double* out)
{
#pragma omp parallel
    {
        double* buf = (double*)malloc(sizeof(double) * (size_t)(P + N));
#pragma omp for schedule(static)
        for (int r = 0; r < n_rows; ++r)
            attn_row(q, kp, vp, kt, vt, mask, mask_words, N, P, Hq, Hkv, d, scale,
                     rows_j[r], rows_h[r], out + (size_t)r * d, buf);
        free(buf);
    }
}

/* ------------------------------------------------------------------ Algorithm 3 */

/*
 * Walk from the root.  At the current node: D = draft row, R = target row; for each
 * child in sampling order draw c in [0,1) and accept iff c*D[y] < R[y]; on a reject
 * R <- norm(max(R-D,0)) (with D as it was before this child is removed), D[y] <- 0,
 * stop scanning if nothing is left in D, else D <- norm(D).  When no child is accepted
 * the step's last token is sampled from R and the walk ends.  When the walk reaches a
 * node without children it ends; with emit_bonus != 0 one more token is sampled from
 * that node's target row (the printed algorithm returns without it: final_token = -1).
 *
 * accepted_nodes[0..*n_accepted) = accepted node indices in order (root excluded).
 * tested_margin[i] = |c - R[y]/D[y]| for every child i that was tested, else +inf.
 * *resid_margin = inverse-CDF margin of the final sample (+inf if none was drawn).
 * *stop_node = node at which the walk ended.
 */
static void verify_core(const float* draft_logits, const float* target_logits, int V, int N,
                        const int32_t* token, const int32_t* first_child,
                        const int32_t* next_sibling, double temp_d, double temp_t,
                        int emit_bonus, const draw_source* src, uint32_t seq,
                        int32_t* accepted_nodes, int32_t* n_accepted, int32_t* final_token,
                        int32_t* stop_node, double* tested_margin, double* resid_margin)
{
    double* D = (double*)malloc(sizeof(double) * (size_t)V);
    double* R = (double*)malloc(sizeof(double) * (size_t)V);
    for (int i = 0; i < N; ++i) tested_margin[i] = INFINITY;
    *resid_margin = INFINITY;
    *n_accepted = 0;
    *final_token = -1;

    int cur = 0;
    pathkey pk_cur = root_key(seq);
    for (;;) {
        softmax_row(target_logits + (size_t)cur * V, V, temp_t, R, NULL);
        if (first_child[cur] < 0) {                     /* accepted a leaf */
            if (emit_bonus) {
                double u = (src->mode == 0) ? philox_u01(src->seed, pk_cur, 0, KIND_RESID)
                                            : src->u_resid[cur];
                *final_token = inverse_cdf(R, V, u, NULL, resid_margin);
            }
            break;
        }
        softmax_row(draft_logits + (size_t)cur * V, V, temp_d, D, NULL);
        int next = -1;
        uint32_t rank = 0;
        pathkey pk_next = pk_cur;
        for (int n = first_child[cur]; n >= 0; n = next_sibling[n], ++rank) {
            int y = token[n];
            pathkey pk_n = (src->mode == 0) ? child_key(src->seed, pk_cur, rank) : pk_cur;
            double c = (src->mode == 0) ? philox_u01(src->seed, pk_n, 0, KIND_ACCEPT)
                                        : src->u_accept[n];
            tested_margin[n] = (D[y] > 0.0) ? fabs(c - R[y] / D[y]) : INFINITY;
            if (c * D[y] < R[y]) { next = n; pk_next = pk_n; break; }
            /* reject: residual target, then remove y from the draft */
            double mass = 0.0;
            for (int x = 0; x < V; ++x) { double r = R[x] - D[x]; mass += (r > 0.0) ? r : 0.0; }
            if (mass > 0.0)
                for (int x = 0; x < V; ++x) { double r = R[x] - D[x]; R[x] = (r > 0.0) ? r / mass : 0.0; }
            D[y] = 0.0;
            double left = 0.0;
            for (int x = 0; x < V; ++x) left += D[x];
            if (!(left > 0.0)) break;                   /* D is all zero */
            for (int x = 0; x < V; ++x) D[x] /= left;
        }
        if (next < 0) {
            double u = (src->mode == 0) ? philox_u01(src->seed, pk_cur, 0, KIND_RESID)
                                        : src->u_resid[cur];
            *final_token = inverse_cdf(R, V, u, NULL, resid_margin);
            break;
        }
        accepted_nodes[(*n_accepted)++] = next;
        cur = next; pk_cur = pk_next;
    }
    *stop_node = cur;
    free(D); free(R);
}

void oracle_verify(const float* draft_logits, const float* target_logits, int V, int N,
                   const int32_t* token, const int32_t* first_child, const int32_t* next_sibling,
                   double temp_d, double temp_t, int emit_bonus, uint64_t seed, uint32_t seq,
                   int32_t* accepted_nodes, int32_t* n_accepted, int32_t* final_token,
                   int32_t* stop_node, double* tested_margin, double* resid_margin)
{
    draw_source src = { 0, seed, NULL, NULL, NULL };
    verify_core(draft_logits, target_logits, V, N, token, first_child, next_sibling, temp_d,
                temp_t, emit_bonus, &src, seq, accepted_nodes, n_accepted, final_token,
                stop_node, tested_margin, resid_margin);
}

void oracle_verify_explicit(const float* draft_logits, const float* target_logits, int V, int N,
                            const int32_t* token, const int32_t* first_child,
                            const int32_t* next_sibling, double temp_d, double temp_t,
                            int emit_bonus, const double* u_accept, const double* u_resid,
                            int32_t* accepted_nodes, int32_t* n_accepted, int32_t* final_token,
                            int32_t* stop_node, double* tested_margin, double* resid_margin)
{
    draw_source src = { 1, 0, NULL, u_accept, u_resid };
    verify_core(draft_logits, target_logits, V, N, token, first_child, next_sibling, temp_d,
                temp_t, emit_bonus, &src, 0, accepted_nodes, n_accepted, final_token,
                stop_node, tested_margin, resid_margin);
}

/*
 * The inner loop of Algorithm 3 run to the end at EVERY node that has children, as if
 * each child in turn were rejected: ratio[n] = R_k[y]/D_k[y] seen by child n when it is
 * tested (its acceptance probability is min(1, ratio)); ratio of the root = 0.
 * This is what the walk would see at any node it reaches, so it is a deterministic
 * function of the two logit tables and the tree.
 */
void oracle_accept_ratio_all(const float* draft_logits, const float* target_logits, int V, int N,
                             const int32_t* token, const int32_t* first_child,
                             const int32_t* next_sibling, double temp_d, double temp_t,
                             double* ratio)
{
    double* D = (double*)malloc(sizeof(double) * (size_t)V);
    double* R = (double*)malloc(sizeof(double) * (size_t)V);
    for (int i = 0; i < N; ++i) ratio[i] = 0.0;
    for (int cur = 0; cur < N; ++cur) {
        if (first_child[cur] < 0) continue;
        softmax_row(target_logits + (size_t)cur * V, V, temp_t, R, NULL);
        softmax_row(draft_logits + (size_t)cur * V, V, temp_d, D, NULL);
        for (int n = first_child[cur]; n >= 0; n = next_sibling[n]) {
            int y = token[n];
            ratio[n] = (D[y] > 0.0) ? R[y] / D[y] : INFINITY;
            double mass = 0.0;
            for (int x = 0; x < V; ++x) { double r = R[x] - D[x]; mass += (r > 0.0) ? r : 0.0; }
            if (mass > 0.0)
                for (int x = 0; x < V; ++x) { double r = R[x] - D[x]; R[x] = (r > 0.0) ? r / mass : 0.0; }
            D[y] = 0.0;
            double left = 0.0;
            for (int x = 0; x < V; ++x) left += D[x];
            if (!(left > 0.0)) break;
            for (int x = 0; x < V; ++x) D[x] /= left;
        }
    }
    free(D); free(R);
}

/*
 * Monte-Carlo driver used by the marginal test: n_trials independent steps with seeds
 * seed0, seed0+1, ...; each builds a tree of n_budget rows from the same logit tables
 * and verifies it.  counts_first[x] += 1 when the first token the step emits is x
 * (token of the first accepted node, or the final token when nothing was accepted);
 * counts_pair[x*V + z] += 1 when the step emits at least two tokens x, z.
 */
void oracle_monte_carlo(const float* draft_logits, const float* target_logits, int V,
                        int n_budget, double temp_d, double temp_t, uint64_t seed0,
                        int64_t n_trials, int64_t* counts_first, int64_t* counts_pair,
                        int64_t* total_accepted)
{
    int N = n_budget, words = (N + 63) / 64;
    int32_t* i32 = (int32_t*)malloc(sizeof(int32_t) * N * 8);
    int32_t *parent = i32, *token = i32 + N, *rank = i32 + 2 * N, *fc = i32 + 3 * N,
            *ns = i32 + 4 * N, *depth = i32 + 5 * N, *acc = i32 + 6 * N;
    double* f64 = (double*)malloc(sizeof(double) * N * 4);
    uint64_t* mask = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)N * words);
    *total_accepted = 0;
    for (int64_t t = 0; t < n_trials; ++t) {
        int32_t nb, na, fin, stop; double rm;
        oracle_build_tree(draft_logits, V, N, temp_d, seed0 + (uint64_t)t, 0, parent, token, rank,
                          fc, ns, depth, f64, mask, words, &nb, f64 + N, f64 + 2 * N);
        oracle_verify(draft_logits, target_logits, V, N, token, fc, ns, temp_d, temp_t, 1,
                      seed0 + (uint64_t)t, 0, acc, &na, &fin, &stop, f64 + 3 * N, &rm);
        int first = (na > 0) ? token[acc[0]] : fin;
        counts_first[first] += 1;
        int second = (na > 1) ? token[acc[1]] : (na == 1 ? fin : -1);
        if (second >= 0) counts_pair[(size_t)first * V + second] += 1;
        *total_accepted += na;
    }
    free(i32); free(f64); free(mask);
}
