// Token tree construction with a threshold (Algorithm 2, Section 4.4, Appendix A.2) for gfx950.
//
// The tree grows level by level.  Within a level the nodes are independent: every node whose
// estimated value is at or above the threshold draws children from its own draft row, without
// replacement, for as long as the value of the next draw stays at or above the threshold.
// That is the data-parallel form of the builder: one 512-thread workgroup per node of the
// level (threshold_expand_kernel), all of them at once, each keeping its row's 4-token
// weight sums in registers so that a draw costs a segment pick, one workgroup scan and the
// update of one sum -- the arithmetic of the greedy builder, draw for draw.  Nodes are
// numbered in creation order (level by level, parents in order, children in sampling order),
// which a workgroup cannot know while its neighbours are still drawing, so children go to a
// per-level pool first and threshold_commit_kernel (one workgroup per sequence) scans the
// counts, cuts at the row capacity and writes the tree rows, links, path keys, values and
// ancestor masks.  The host reads the level's size back after every commit: it sizes the next
// grid and ends the loop.  Draft row of a node = its row index, as for Algorithm 1.
#include "draft_row.h"
#include "lane_ops.h"

namespace dyspec {

// Workspace, in doubles, for rows = sum of capacities N_s:
//   child_value[rows]   value of a node's own first draw (v * d[y]); root 1
//   pool_v0[pool], pool_v[pool]   per drawn child: v * d[y], and the value v it was drawn at
//   pk[rows] (uint2), counts[rows] (int), pool_token[pool] (int), state[4 * n_seq] (int)
// pool = sum over sequences of N_s^2 / 4 + N_s entries: a level with F nodes and R rows left
// holds at most F * R children and F <= N - R.
struct ThresholdWs {
    double* child_value;
    double* pool_v0;
    double* pool_v;
    uint2* pk;
    int* counts;
    int* pool_token;
    int* state;          // per sequence: level begin, level end, rows left at level begin, unused
    long long pool_off[DYSPEC_MAX_SEQ + 1];
};

static size_t pool_entries(int N) { return (size_t)N * N / 4 + N; }

size_t build_threshold_workspace_bytes(const SeqArgs& sa)
{
    const size_t rows = sa.node_off[sa.n_seq];
    size_t pool = 0;
    for (int s = 0; s < sa.n_seq; ++s) pool += pool_entries(sa.node_off[s + 1] - sa.node_off[s]);
    return rows * 8 + pool * 16 + rows * 8 + rows * 4 + pool * 4 + (size_t)sa.n_seq * 16 + 64;
}

static ThresholdWs carve(void* workspace, const SeqArgs& sa)
{
    ThresholdWs w;
    const size_t rows = sa.node_off[sa.n_seq];
    size_t pool = 0;
    for (int s = 0; s < sa.n_seq; ++s) {
        w.pool_off[s] = (long long)pool;
        pool += pool_entries(sa.node_off[s + 1] - sa.node_off[s]);
    }
    w.pool_off[sa.n_seq] = (long long)pool;
    char* p = static_cast<char*>(workspace);
    w.child_value = reinterpret_cast<double*>(p); p += rows * 8;
    w.pool_v0 = reinterpret_cast<double*>(p); p += pool * 8;
    w.pool_v = reinterpret_cast<double*>(p); p += pool * 8;
    w.pk = reinterpret_cast<uint2*>(p); p += rows * 8;
    w.counts = reinterpret_cast<int*>(p); p += rows * 4;
    w.pool_token = reinterpret_cast<int*>(p); p += pool * 4;
    w.state = reinterpret_cast<int*>(p);
    return w;
}

struct ThresholdArgs {
    double t[DYSPEC_MAX_SEQ];
};

__global__ __launch_bounds__(256) void threshold_init_kernel(SeqArgs sa, dyspec_tree tree, float* __restrict__ est_value,
                                                             uint64_t* __restrict__ anc_mask, int mask_words,
                                                             int* __restrict__ n_built, ThresholdWs w)
{
    const int seq = blockIdx.x;
    const int base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - base;
    for (int i = threadIdx.x; i < N; i += 256) {
        tree.parent[base + i] = -1; tree.token[base + i] = -1; tree.sib_rank[base + i] = 0;
        tree.first_child[base + i] = -1; tree.next_sibling[base + i] = -1; tree.depth[base + i] = 0;
        est_value[base + i] = (i == 0) ? 1.0f : 0.0f;
        for (int k = 0; k < mask_words; ++k)
            anc_mask[(size_t)(base + i) * mask_words + k] = (k == i / 64) ? (1ull << (i % 64)) : 0ull;
        w.counts[base + i] = 0;
    }
    if (threadIdx.x == 0) {
        if (N > 0) {
            w.child_value[base] = 1.0;
            w.pk[base] = root_key((uint32_t)seq);
        }
        w.state[4 * seq + 0] = 0;                       // the first level is the root alone
        w.state[4 * seq + 1] = min(N, 1);
        w.state[4 * seq + 2] = max(N - 1, 0);
        w.state[4 * seq + 3] = 0;
        n_built[seq] = min(N, 1);
    }
}

struct ExpandShared {
    double red[kWaves * kMaxSeg];       // workgroup sums at set-up
    double wave_tot[kWaves];            // per draw: the waves' sums of the picked segment
    double wy, old_sum, new_sum;        // per draw: the drawn token's weight, its thread's sum before and after
    int y, owner;                       // the drawn token, the thread that held it
    int last_live[kWaves];              // last thread of each wave with weight left, -1: none
    float fred[kWaves];
    float u_draw[DYSPEC_MAX_BUILD_NODES];     // the uniform draws of this node's samplings, by child rank
};

// One workgroup per node of the current level: blockIdx.x = position in the level.  The node's
// row of logits and a drawn-already bitmap live in LDS (dynamic: 4 bytes per token, 1 bit per
// token), the threads' 4-token weight sums in registers, segment total j in lanes j, j + 16, ...
// A draw is: segment pick (a 16-lane scan), a scan of the 512 sums of that segment (DPP, one
// barrier); the waves' totals tell every thread which wave holds the crossing; that wave finds
// the owning thread with a ballot, computes its four weights in four lanes and finishes the draw
// (one barrier); every thread then updates its copy of the totals.  The uniform draws of all
// samplings of the node (functions of its path key and the child rank) are made at set-up.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void threshold_expand_kernel(const float* __restrict__ draft_logits, int V, SeqArgs sa,
                                                                  ThresholdArgs ta, uint64_t seed, ThresholdWs w)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn[];
    __shared__ ExpandShared sh;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int seq = blockIdx.y;
    const int base = sa.node_off[seq];
    const int lvl_begin = w.state[4 * seq + 0], lvl_end = w.state[4 * seq + 1], left = w.state[4 * seq + 2];
    const int f = blockIdx.x;
    const int p = lvl_begin + f;
    if (p >= lvl_end) return;                           // uniform over the workgroup
    const double t = ta.t[seq];
    double v = w.child_value[base + p];
    if (!(v >= t) || left <= 0) {                       // below the threshold: no draw, the row is not even read
        if (tid == 0) w.counts[base + p] = 0;
        return;
    }
    const double inv_temp = 1.0 / (double)sa.temp_d[seq];
    const float* __restrict__ row = draft_logits + (size_t)(base + p) * V;
    const uint2 pk_p = w.pk[base + p];
    const size_t pool0 = (size_t)w.pool_off[seq] + (size_t)f * left;
    const int Vpad = (V + 31) & ~31;
    float* const row_lds = reinterpret_cast<float*>(dyn);
    uint32_t* const gone = reinterpret_cast<uint32_t*>(dyn + (size_t)Vpad * 4);
    for (int i = tid; i < Vpad; i += kBlock) row_lds[i] = (i < V) ? row[i] : -INFINITY;
    for (int i = tid; i < Vpad / 32; i += kBlock) gone[i] = 0u;

    for (int c = tid; c < left; c += kBlock) sh.u_draw[c] = u01(seed, pk_p, (uint32_t)c, KIND_BUILD);

    double m, seg[kMaxSeg], tot[kMaxSeg];
    row_segment_sums<VEC>(row, V, inv_temp, 0ull, sh.fred, &m, seg);
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) tot[j] = seg[j];
    block_sum<double, kMaxSeg>(tot, sh.red);
    double my_tot = 0.0;                                // total of segment lane % 16
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) if (j == (lane & 15)) my_tot = tot[j];
    __syncthreads();                                    // the row, the bitmap and the draws are in LDS for everyone

    int count = 0;
    while (v >= t && count < left) {
        const double u = (double)sh.u_draw[count];
        const SegPick pk = pick_segment_lanes(my_tot, u);
        if (!(pk.W > 0.0)) break;                       // nothing left to sample under p
        double mine = 0.0;
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j) if (j == pk.js) mine = seg[j];
        // ---- inclusive scan of the sums of segment js in thread order
        const double inc = wave_scan_dpp(mine);
        if (lane == kWave - 1) sh.wave_tot[wave] = inc;
        __syncthreads();
        // the waves' totals, one per lane (lanes 0..7 of every row of 16), scanned the same way
        const double wt = (lane & 8) ? 0.0 : sh.wave_tot[lane & 7];
        double wc = wt;
        wc += dpp_or_zero<0x111>(wc);
        wc += dpp_or_zero<0x112>(wc);
        wc += dpp_or_zero<0x114>(wc);
        const double before = readlane_f64(dpp_or_zero<0x111>(wc), wave);
        const uint32_t past = (uint32_t)__ballot(pk.cum_js + wc > pk.target) & 0xffu;
        int kw = past ? __builtin_ctz(past) : -1;       // first wave whose running total is past u * W
        const double incl = before + inc;
        const unsigned long long live = __ballot(mine > 0.0);
        int fixed_owner = -1;
        if (kw < 0) {
            // rounding at the very top: the last thread with weight left (the same in every thread)
            if (lane == 0) sh.last_live[wave] = live ? wave * kWave + 63 - __builtin_clzll(live) : -1;
            __syncthreads();
#pragma unroll
            for (int k = 0; k < kWaves; ++k) if (sh.last_live[k] >= 0) fixed_owner = sh.last_live[k];
            if (fixed_owner < 0) break;                 // the totals held rounding dust only
            kw = fixed_owner / kWave;
        }
        if (wave == kw) {
            // the wave's total is positive, so a thread with weight exists: the first one past the
            // target, else (the scan's rounding) the last one with weight
            const unsigned long long hit = __ballot(mine > 0.0 && pk.cum_js + incl > pk.target);
            const int ol = fixed_owner >= 0 ? fixed_owner % kWave : hit ? __builtin_ctzll(hit) : 63 - __builtin_clzll(live);
            const int tok0 = pk.js * kSeg + 4 * (kw * kWave + ol);      // first of the owner's four tokens
            double wgt = 0.0;                           // lanes 0..3: one weight each
            if (lane < 4) {
                const int idx = tok0 + lane;
                const bool there = idx < V && !((gone[idx >> 5] >> (idx & 31)) & 1u);
                if (there) wgt = token_weight(row_lds[idx], inv_temp, m);
            }
            const double w4v[4] = { readlane_f64(wgt, 0), readlane_f64(wgt, 1), readlane_f64(wgt, 2), readlane_f64(wgt, 3) };
            double run = readlane_f64(pk.cum_js + (incl - mine), ol), wy = 0.0, wlast = 0.0;
            int y = -1, ylast = -1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                run += w4v[e];
                if (w4v[e] > 0.0) { ylast = tok0 + e; wlast = w4v[e]; }
                if (y < 0 && w4v[e] > 0.0 && run > pk.target) { y = tok0 + e; wy = w4v[e]; }
            }
            if (y < 0) { y = ylast; wy = wlast; }
            const int ey = y - tok0;
            if (lane == 0) {
                sh.y = y; sh.wy = wy; sh.owner = kw * kWave + ol;
                sh.old_sum = (w4v[0] + w4v[1]) + (w4v[2] + w4v[3]);
                sh.new_sum = ((ey == 0 ? 0.0 : w4v[0]) + (ey == 1 ? 0.0 : w4v[1])) + ((ey == 2 ? 0.0 : w4v[2]) + (ey == 3 ? 0.0 : w4v[3]));
            }
        }
        __syncthreads();
        // ---- every thread updates its copy of the state
        const int y = sh.y;
        if (y < 0) break;
        const double wy = sh.wy, old_sum = sh.old_sum, new_sum = sh.new_sum;
        if (tid == sh.owner) {
#pragma unroll
            for (int j = 0; j < kMaxSeg; ++j) if (j == pk.js) seg[j] = new_sum;
        }
        if ((lane & 15) == pk.js) my_tot = (my_tot - old_sum) + new_sum;
        const double dy = wy / pk.W;
        if (tid == 0) {
            gone[y >> 5] |= 1u << (y & 31);             // read again one barrier from here at the earliest
            w.pool_token[pool0 + count] = y;
            w.pool_v[pool0 + count] = v;
            w.pool_v0[pool0 + count] = v * dy;
        }
        v = v * (1.0 - dy);
        ++count;
    }
    if (tid == 0) w.counts[base + p] = count;
}

struct CommitShared {
    int excl[DYSPEC_MAX_BUILD_NODES + 1];
    int scan[kWaves];
};

// One workgroup per sequence: numbers the level's children in creation order, cuts at the
// capacity, writes their rows and makes them the next level.
__global__ __launch_bounds__(kBlock) void threshold_commit_kernel(SeqArgs sa, uint64_t seed, dyspec_tree tree,
                                                                  float* __restrict__ est_value, uint64_t* anc_mask,
                                                                  int mask_words, int* __restrict__ n_built, ThresholdWs w)
{
    __shared__ CommitShared sh;
    const int tid = threadIdx.x;
    const int seq = blockIdx.x;
    const int base = sa.node_off[seq];
    const int lvl_begin = w.state[4 * seq + 0], lvl_end = w.state[4 * seq + 1], left = w.state[4 * seq + 2];
    const int F = lvl_end - lvl_begin;
    if (F <= 0) return;
    // exclusive scan of the children counts over the level, two nodes per thread (F <= 1024)
    const int f0 = 2 * tid, f1 = 2 * tid + 1;
    const int c0 = f0 < F ? w.counts[base + lvl_begin + f0] : 0;
    const int c1 = f1 < F ? w.counts[base + lvl_begin + f1] : 0;
    int excl;
    const int incl = block_scan_inclusive<int>(c0 + c1, sh.scan, &excl);
    if (f0 <= F) sh.excl[f0] = excl;
    if (f1 <= F) sh.excl[f1] = excl + c0;
    if (tid == kBlock - 1 && F == 2 * kBlock) sh.excl[F] = incl;
    __syncthreads();
    const int total = sh.excl[F];
    const int M = min(total, left);                     // rows that still fit
    for (int k = tid; k < M; k += kBlock) {
        // node of the level that drew child k: last f with excl[f] <= k
        int lo = 0, hi = F - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (sh.excl[mid] <= k) lo = mid; else hi = mid - 1;
        }
        const int fpos = lo, rank = k - sh.excl[fpos];
        const int p = lvl_begin + fpos, i = lvl_end + k;
        const size_t e = (size_t)w.pool_off[seq] + (size_t)fpos * left + rank;
        const int n_kids = min(sh.excl[fpos + 1], M) - sh.excl[fpos];      // children of p that fit
        tree.parent[base + i] = p;
        tree.token[base + i] = w.pool_token[e];
        tree.sib_rank[base + i] = rank;
        tree.depth[base + i] = tree.depth[base + p] + 1;
        tree.next_sibling[base + i] = (rank + 1 < n_kids) ? i + 1 : -1;
        if (rank == 0) tree.first_child[base + p] = i;
        est_value[base + i] = (float)w.pool_v[e];
        w.child_value[base + i] = w.pool_v0[e];
        w.pk[base + i] = child_key(seed, w.pk[base + p], (uint32_t)rank);
        w.counts[base + i] = 0;
        for (int q = 0; q < mask_words; ++q)
            anc_mask[(size_t)(base + i) * mask_words + q] =
                anc_mask[(size_t)(base + p) * mask_words + q] | ((q == i / 64) ? (1ull << (i % 64)) : 0ull);
    }
    __syncthreads();
    if (tid == 0) {
        w.state[4 * seq + 0] = lvl_end;
        w.state[4 * seq + 1] = lvl_end + M;
        w.state[4 * seq + 2] = left - M;
        n_built[seq] = lvl_end + M;
    }
}

// the expanding workgroups keep a row of logits and a token bitmap in dynamic LDS: raised to the
// largest vocabulary once
hipError_t prepare_build_threshold()
{
    static std::atomic<unsigned long long> done_vec{0}, done_scalar{0};
    constexpr int bytes = DYSPEC_MAX_VOCAB * 4 + DYSPEC_MAX_VOCAB / 8;
    hipError_t e = raise_dynamic_lds_once(reinterpret_cast<const void*>(&threshold_expand_kernel<true>), bytes, done_vec);
    if (e != hipSuccess) return e;
    return raise_dynamic_lds_once(reinterpret_cast<const void*>(&threshold_expand_kernel<false>), bytes, done_scalar);
}

hipError_t launch_build_threshold(const float* draft_logits, int V, const SeqArgs& sa, const double* threshold,
                                  uint64_t seed, const dyspec_tree& tree, float* est_value, uint64_t* anc_mask,
                                  int mask_words, int* n_built, int* n_levels, void* workspace, hipStream_t stream)
{
    const ThresholdWs w = carve(workspace, sa);
    ThresholdArgs ta;
    for (int s = 0; s < sa.n_seq; ++s) ta.t[s] = threshold[s];
    // the expanding workgroups keep their row (4 bytes per token) and a bitmap (1 bit per token) in LDS
    const int Vpad = (V + 31) & ~31;
    const size_t dyn_bytes = (size_t)Vpad * 4 + Vpad / 8;
    const hipError_t ea = prepare_build_threshold();
    if (ea != hipSuccess) return ea;
    threshold_init_kernel<<<sa.n_seq, 256, 0, stream>>>(sa, tree, est_value, anc_mask, mask_words, n_built, w);
    // (Launching eight levels at a time without a look from the host in between, over a grid sized for
    // the widest level possible, was measured and is slower: a launch of workgroups that find
    // nothing to do costs about as much as the look it saves -- 70B table 1.06 against 1.00 ms, the
    // 13B table, two levels deep, 0.60 against 0.50 ms.)
    int widest = 1;
    for (int s = 0; s < sa.n_seq; ++s) widest = max(widest, sa.node_off[s + 1] - sa.node_off[s]);
    int frontier = widest > 1 ? 1 : 0, levels = 0;      // widest level over the sequences: the roots, if a row is left
    int state[4 * DYSPEC_MAX_SEQ];
    // a level adds at least one row or ends the loop, so this runs at most max N times
    while (frontier > 0) {
        if (V % 4 == 0)
            threshold_expand_kernel<true><<<dim3(frontier, sa.n_seq), kBlock, dyn_bytes, stream>>>(draft_logits, V, sa, ta, seed, w);
        else
            threshold_expand_kernel<false><<<dim3(frontier, sa.n_seq), kBlock, dyn_bytes, stream>>>(draft_logits, V, sa, ta, seed, w);
        threshold_commit_kernel<<<sa.n_seq, kBlock, 0, stream>>>(sa, seed, tree, est_value, anc_mask, mask_words, n_built, w);
        hipError_t e = hipMemcpyAsync(state, w.state, sizeof(int) * 4 * sa.n_seq, hipMemcpyDeviceToHost, stream);
        if (e != hipSuccess) return e;
        e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return e;
        ++levels;
        frontier = 0;
        for (int s = 0; s < sa.n_seq; ++s)
            if (state[4 * s + 2] > 0) frontier = max(frontier, state[4 * s + 1] - state[4 * s + 0]);
    }
    if (n_levels) *n_levels = levels;
    return hipGetLastError();
}

}  // namespace dyspec
