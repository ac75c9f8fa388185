// Vocabulary softmax of every tree row and multi-candidate tree rejection sampling
// (Algorithm 3, Appendix A.3; one-candidate rule of Section 2) for gfx950.
//
// Algorithm 3 as printed is a serial walk that does O(V) work at every node it visits.
// What it computes at a node p -- the ratio R[y]/D[y] seen by each child of p after its
// earlier siblings were rejected, and the residual R left when all children fail --
// depends only on p's two logit rows and p's children, not on the random draws.  So one
// workgroup per tree row computes these for ALL rows at once, reading each logit row from
// HBM exactly once into registers (the data-parallel pass), and a one-thread-per-sequence
// walk then follows the accepted path with one Philox draw per tested child.
#include "vocab_common.h"

namespace dyspec {

struct VerifyShared {
    CdfScratch cdf;
    float fred[kWaves * 2];
    int ranks[DYSPEC_MAX_NODES];
    uint2 pk;
};

template <bool VEC>
__global__ __launch_bounds__(kBlock) void verify_rows_kernel(
    const float* __restrict__ draft_logits, const float* __restrict__ target_logits, int V,
    SeqArgs sa, dyspec_tree tree, uint64_t seed, int emit_bonus,
    float* __restrict__ row_stats, float* __restrict__ accept_ratio, int* __restrict__ resid_token)
{
    __shared__ VerifyShared sh;
    const int tid = threadIdx.x;
    const int row = blockIdx.x;
    const int seq = find_seq(sa, row);
    const int base = sa.node_off[seq];
    const int p = row - base;
    const float inv_td = 1.0f / sa.temp_d[seq], inv_tt = 1.0f / sa.temp_t[seq];

    // path key of p: ranks up to the root, then keys back down (one thread; a few Philox calls)
    if (tid == 0) {
        int depth = 0;
        for (int a = p; a > 0 && depth < DYSPEC_MAX_NODES; a = tree.parent[base + a])
            sh.ranks[depth++] = tree.sib_rank[base + a];
        uint2 pk = root_key((uint32_t)seq);
        for (int k = depth - 1; k >= 0; --k) pk = child_key(seed, pk, (uint32_t)sh.ranks[k]);
        sh.pk = pk;
        if (p == 0) accept_ratio[row] = 0.0f;
    }

    float D[kMaxSeg][4], R[kMaxSeg][4];
    load_row<VEC>(draft_logits + (size_t)row * V, V, D);
    load_row<VEC>(target_logits + (size_t)row * V, V, R);

    // ---- softmax of both rows: z = logit / T, m = max z, e = exp(z - m), s = sum e
    float mx[2] = { -INFINITY, -INFINITY };
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            D[j][e] *= inv_td; R[j][e] *= inv_tt;
            mx[0] = fmaxf(mx[0], D[j][e]); mx[1] = fmaxf(mx[1], R[j][e]);
        }
    block_max<2>(mx, sh.fred);
    float sm[2] = { 0.0f, 0.0f };
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            D[j][e] = expf(D[j][e] - mx[0]); R[j][e] = expf(R[j][e] - mx[1]);   // exp(-inf) = 0 past V
            sm[0] += D[j][e]; sm[1] += R[j][e];
        }
    block_sum<float, 2>(sm, sh.fred);
    if (tid == 0) {
        float4 st = make_float4(mx[0], sm[0], mx[1], sm[1]);
        *reinterpret_cast<float4*>(row_stats + 4 * (size_t)row) = st;
    }
    {
        const float id = 1.0f / sm[0], it = 1.0f / sm[1];
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) { D[j][e] *= id; R[j][e] *= it; }
    }

    // ---- children of p in sampling order, each as if all earlier ones were rejected
    const int N = sa.node_off[seq + 1] - base;
    int c = tree.first_child[row];
    const bool leaf = c < 0;
    for (int guard = 0; c >= 0 && guard < N; ++guard) {      // a node has fewer than N children
        const int y = tree.token[base + c];
        const bool mine = y >= 0 && y < V && ((y % kSeg) >> 2) == tid;
        float res[2] = { 0.0f, 0.0f };              // mass of relu(R-D), mass left in D
        float dy_old = 0.0f;
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float d = D[j][e], r = R[j][e];
                if (mine && j == y / kSeg && e == (y & 3)) {
                    accept_ratio[base + c] = (d > 0.0f) ? r / d : (r > 0.0f ? INFINITY : 0.0f);
                    dy_old = d;
                    D[j][e] = 0.0f;                  // y leaves the draft AFTER R-D used it
                }
                res[0] += fmaxf(r - d, 0.0f);
                res[1] += D[j][e];
            }
        block_sum<float, 2>(res, sh.fred);
        if (res[0] > 0.0f) {                         // else R == D: keep R (no reject can reach here)
            const float ir = 1.0f / res[0];
#pragma unroll
            for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float d = (mine && j == y / kSeg && e == (y & 3)) ? dy_old : D[j][e];
                    R[j][e] = fmaxf(R[j][e] - d, 0.0f) * ir;
                }
        }
        c = tree.next_sibling[base + c];
        if (!(res[1] > 0.0f)) {                      // D is empty: later children are not tried
            if (tid == 0)
                for (int k = 0; c >= 0 && k < N; ++k, c = tree.next_sibling[base + c]) accept_ratio[base + c] = -1.0f;
            break;
        }
        const float il = 1.0f / res[1];
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) D[j][e] *= il;
    }

    // ---- token emitted if the walk stops here
    if (leaf && !emit_bonus) {
        if (tid == 0) resid_token[row] = -1;
        return;
    }
    __syncthreads();
    const double u = (double)u01(seed, sh.pk, 0u, KIND_RESID);
    double W, wy;
    const int y = block_inverse_cdf<float>(R, u, &sh.cdf, &W, &wy);
    if (tid == 0) resid_token[row] = y;
}

// One thread per sequence follows the accepted path (the while/for loops of Algorithm 3).
__global__ void verify_walk_kernel(SeqArgs sa, dyspec_tree tree, uint64_t seed,
                                   const float* __restrict__ accept_ratio,
                                   const int* __restrict__ resid_token,
                                   int* __restrict__ accepted_nodes, int* __restrict__ n_accepted,
                                   int* __restrict__ final_token, float* __restrict__ min_margin)
{
    const int seq = blockIdx.x * blockDim.x + threadIdx.x;
    if (seq >= sa.n_seq) return;
    const int base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - base;
    int cur = 0, na = 0;
    uint2 pk = root_key((uint32_t)seq);
    float margin = INFINITY;
    for (int steps = 0; steps < N; ++steps) {        // a path has fewer than N edges
        int next = -1;
        uint2 pk_next = pk;
        uint32_t rank = 0;
        for (int n = tree.first_child[base + cur]; n >= 0 && (int)rank < N; n = tree.next_sibling[base + n], ++rank) {
            const float ratio = accept_ratio[base + n];
            if (ratio < 0.0f) break;                 // draft distribution exhausted before n
            const uint2 pk_n = child_key(seed, pk, rank);
            const float c = u01(seed, pk_n, 0u, KIND_ACCEPT);
            margin = fminf(margin, fabsf(c - ratio));
            if (c < ratio) { next = n; pk_next = pk_n; break; }
        }
        if (next < 0) break;
        accepted_nodes[base + na++] = next;
        cur = next; pk = pk_next;
    }
    n_accepted[seq] = na;
    final_token[seq] = resid_token[base + cur];
    min_margin[seq] = margin;
}

hipError_t launch_verify(const float* draft_logits, const float* target_logits, int V,
                         const SeqArgs& sa, const dyspec_tree& tree, uint64_t seed, int emit_bonus,
                         float* row_stats, float* accept_ratio, int* resid_token,
                         int* accepted_nodes, int* n_accepted, int* final_token,
                         float* min_margin, hipStream_t stream)
{
    const int rows = sa.node_off[sa.n_seq];
    if (V % 4 == 0)
        verify_rows_kernel<true><<<rows, kBlock, 0, stream>>>(draft_logits, target_logits, V, sa, tree, seed,
                                                              emit_bonus, row_stats, accept_ratio, resid_token);
    else
        verify_rows_kernel<false><<<rows, kBlock, 0, stream>>>(draft_logits, target_logits, V, sa, tree, seed,
                                                               emit_bonus, row_stats, accept_ratio, resid_token);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    verify_walk_kernel<<<1, DYSPEC_MAX_SEQ, 0, stream>>>(sa, tree, seed, accept_ratio, resid_token,
                                                         accepted_nodes, n_accepted, final_token, min_margin);
    return hipGetLastError();
}

}  // namespace dyspec
