// Greedy fixed-budget token-tree construction (Algorithm 1, Section 4.2, Appendix A.1)
// and the ancestor bitmask of tree attention (Section 2) for gfx950.
//
// One 512-thread workgroup builds one sequence's tree without leaving the GPU.  The
// paper keeps the expandable slots in a heap on the host; here the frontier (at most two
// new slots per node) lives in LDS or in registers and the pop is a workgroup arg-max, which
// costs less than a heap's pointer chasing at these sizes.  A draw needs the parent's residual draft
// distribution: fp64 softmax weights summed four tokens at a time, a workgroup sum and scan
// of those sums for the inverse CDF.  fp64 keeps every discrete decision (which slot, which
// token) equal to an fp64 evaluation of the algorithm except at relative margins near 1e-13.
//
// With a workspace the O(vocabulary) part leaves the serial loop: draft_row_sums_kernel (one
// workgroup per row, all rows at once) stores every row's maximum and the totals of its kMaxSeg
// segments, and the builder (build_tree_cached_kernel) keeps the totals current in LDS and a bit
// per drawn token in the workspace.  A draw picks the segment from the totals, makes one trip to
// global memory (each thread fetches its four logits and its drawn-already bits of the picked
// segment and recomputes their four weights, a 16th of a row pass) and passes two barriers.  Without a
// workspace the builder (build_tree_kernel) recomputes the sums of the parent's row for every
// draw; both ways take the same decisions and build the same tree.
#include "draft_row.h"
#include "lane_ops.h"

namespace dyspec {

constexpr int kMaxSlots = 2 * DYSPEC_MAX_BUILD_NODES + 2;

// Workspace of the cached form, per row (doubles): kMaxSeg segment totals, the row maximum
// (already divided by the temperature), and one bit per token: drawn at this position already
// (its weight is no longer in the totals).
constexpr int kGoneWords = DYSPEC_MAX_VOCAB / 32;
constexpr int kRowSumDoubles = kMaxSeg + 8 + kGoneWords / 2;
__host__ __device__ inline double* ws_totals(double* ws, int row) { return ws + (size_t)row * kRowSumDoubles; }
__host__ __device__ inline double* ws_rowmax(double* ws, int row) { return ws_totals(ws, row) + kMaxSeg; }
__host__ __device__ inline uint32_t* ws_gone(double* ws, int row) { return reinterpret_cast<uint32_t*>(ws_totals(ws, row) + kMaxSeg + 8); }

// Data-parallel part (the draft softmax of every node, Algorithm 1's model call output):
// one workgroup per row writes the row's segment totals and maximum and clears its drawn bits.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void draft_row_sums_kernel(const float* __restrict__ draft_logits, int V, SeqArgs sa,
                                                                double* __restrict__ ws)
{
    __shared__ float fred[kWaves];
    __shared__ double red[kWaves * kMaxSeg];
    const int row = blockIdx.x;
    const int seq = find_seq(sa, row);
    const double inv_temp = 1.0 / (double)sa.temp_d[seq];
    double m, seg[kMaxSeg];
    row_segment_sums<VEC>(draft_logits + (size_t)row * V, V, inv_temp, 0ull, fred, &m, seg);
    block_sum<double, kMaxSeg>(seg, red);
    if (threadIdx.x < kMaxSeg) {
        double t = 0.0;
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j) if (j == (int)threadIdx.x) t = seg[j];
        ws_totals(ws, row)[threadIdx.x] = t;
    }
    if (threadIdx.x == 0) *ws_rowmax(ws, row) = m;
    for (int w = threadIdx.x; w < kGoneWords; w += kBlock) ws_gone(ws, row)[w] = 0u;
}

// LDS state of the form without a workspace.
struct BuildShared {
    double slot_value[kMaxSlots];       // < 0: closed
    int slot_parent[kMaxSlots];
    int n_children[DYSPEC_MAX_BUILD_NODES];
    int last_child[DYSPEC_MAX_BUILD_NODES];
    int token[DYSPEC_MAX_BUILD_NODES];
    int first_child[DYSPEC_MAX_BUILD_NODES];
    int next_sibling[DYSPEC_MAX_BUILD_NODES];
    int depth[DYSPEC_MAX_BUILD_NODES];
    uint2 pk[DYSPEC_MAX_BUILD_NODES];
    CdfScratch cdf;
    double best_v[kWaves];
    int best_i[kWaves];
    float fred[kWaves];
    int n_slots;
    int pick;
};

// Initial state of a sequence's tree in global memory: every row unbuilt.
__device__ __forceinline__ void init_tree_rows(int base, int N, const dyspec_tree& tree, float* __restrict__ est_value,
                                               uint64_t* __restrict__ anc_mask, int mask_words)
{
    for (int i = threadIdx.x; i < N; i += kBlock) {
        tree.parent[base + i] = -1; tree.token[base + i] = -1; tree.sib_rank[base + i] = 0;
        tree.first_child[base + i] = -1; tree.next_sibling[base + i] = -1; tree.depth[base + i] = 0;
        est_value[base + i] = (i == 0) ? 1.0f : 0.0f;
        for (int w = 0; w < mask_words; ++w)
            anc_mask[(size_t)(base + i) * mask_words + w] = (w == i / 64) ? (1ull << (i % 64)) : 0ull;
    }
}

// ... and in LDS, with the root's slot open.  Ends with a barrier.
__device__ __forceinline__ void init_tree_state(BuildShared& sh, int seq, int base, int N, const dyspec_tree& tree,
                                                float* __restrict__ est_value, uint64_t* __restrict__ anc_mask, int mask_words)
{
    const int tid = threadIdx.x;
    init_tree_rows(base, N, tree, est_value, anc_mask, mask_words);
    for (int i = tid; i < N; i += kBlock) {
        sh.n_children[i] = 0; sh.last_child[i] = -1; sh.token[i] = -1;
        sh.first_child[i] = -1; sh.next_sibling[i] = -1; sh.depth[i] = 0;
    }
    for (int s = tid; s < kMaxSlots; s += kBlock) sh.slot_value[s] = -1.0;
    __syncthreads();
    if (tid == 0) {
        sh.slot_value[0] = 1.0; sh.slot_parent[0] = 0; sh.n_slots = 1;
        sh.pk[0] = root_key((uint32_t)seq);
    }
    __syncthreads();
}

// Thread 0's bookkeeping for new node i = child number `rank` of p with token y, taken from a slot
// of value v (Algorithm 1: the node's estimated acceptance rate).
__device__ __forceinline__ void append_node(BuildShared& sh, const dyspec_tree& tree, float* __restrict__ est_value,
                                            uint2 key, int base, int p, int i, int rank, int y, double v)
{
    sh.token[i] = y; sh.depth[i] = sh.depth[p] + 1;
    if (sh.last_child[p] < 0) { sh.first_child[p] = i; tree.first_child[base + p] = i; }
    else { sh.next_sibling[sh.last_child[p]] = i; tree.next_sibling[base + sh.last_child[p]] = i; }
    sh.last_child[p] = i; sh.n_children[p] = rank + 1;
    sh.pk[i] = key;
    tree.parent[base + i] = p; tree.token[base + i] = y; tree.sib_rank[base + i] = rank;
    tree.depth[base + i] = sh.depth[i];
    est_value[base + i] = (float)v;
}

// The form without a workspace: the sums of the parent's row are recomputed for every draw.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void build_tree_kernel(
    const float* __restrict__ draft_logits, int V, SeqArgs sa, uint64_t seed,
    dyspec_tree tree, float* __restrict__ est_value, uint64_t* __restrict__ anc_mask,
    int mask_words, int* __restrict__ n_built)
{
    __shared__ BuildShared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = blockIdx.x;
    const int base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - base;
    const double inv_temp = 1.0 / (double)sa.temp_d[seq];
    init_tree_state(sh, seq, base, N, tree, est_value, anc_mask, mask_words);

    int n = 1;
    while (n < N) {
        // ---- pop: open slot of largest value, earliest-opened on ties
        const int n_slots = sh.n_slots;
        double bv = -1.0; int bi = 0x7fffffff;
        for (int s = tid; s < n_slots; s += kBlock) {
            const double v = sh.slot_value[s];
            if (v > bv) { bv = v; bi = s; }           // s ascends: ties keep the earlier slot
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double ov = __shfl_xor(bv, o, kWave);
            const int oi = __shfl_xor(bi, o, kWave);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { sh.best_v[wave] = bv; sh.best_i[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            double v = sh.best_v[0]; int i = sh.best_i[0];
            for (int w = 1; w < kWaves; ++w)
                if (sh.best_v[w] > v || (sh.best_v[w] == v && sh.best_i[w] < i)) { v = sh.best_v[w]; i = sh.best_i[w]; }
            sh.pick = (v > 0.0) ? i : -1;
        }
        __syncthreads();
        const int pick = sh.pick;
        if (pick < 0) break;                           // frontier is empty
        const int p = sh.slot_parent[pick];
        const double v = sh.slot_value[pick];
        const int rank = sh.n_children[p];

        // ---- draw the token from the residual draft distribution of p (softmax weights with
        //      the earlier children's tokens removed)
        const double u = (double)u01(seed, sh.pk[p], (uint32_t)rank, KIND_BUILD);
        const float* __restrict__ row = draft_logits + (size_t)(base + p) * V;
        // bit k of `gone` marks this thread's k-th token as already drawn at this position
        uint64_t gone = 0ull;
        for (int c = sh.first_child[p]; c >= 0; c = sh.next_sibling[c]) {
            const int yc = sh.token[c];
            if (((yc % kSeg) >> 2) == tid) gone |= 1ull << (4 * (yc / kSeg) + (yc & 3));
        }
        double m, seg[kMaxSeg], W, wy;
        row_segment_sums<VEC>(row, V, inv_temp, gone, sh.fred, &m, seg);
        const int y = block_inverse_cdf_seg(seg, u, &sh.cdf, &W, &wy, [&](int j, int e) -> double {
            const int idx = tok_index(j, e);
            const bool live = idx < V && !((gone >> (4 * j + e)) & 1ull);
            return live ? token_weight(row[idx], inv_temp, m) : 0.0;
        });
        if (y < 0) break;                              // nothing left to sample under p

        // ---- append node n, open its two slots
        const int i = n;
        if (tid == 0) {
            const double Ry = wy / W;
            sh.slot_value[pick] = -1.0;
            append_node(sh, tree, est_value, child_key(seed, sh.pk[p], (uint32_t)rank), base, p, i, rank, y, v);
            const double v0 = v * Ry, v1 = v * (1.0 - Ry);
            int ns = sh.n_slots;
            if (v1 > 0.0) { sh.slot_value[ns] = v1; sh.slot_parent[ns] = p; ++ns; }   // next sampling at this position
            if (v0 > 0.0) { sh.slot_value[ns] = v0; sh.slot_parent[ns] = i; ++ns; }   // first child of the new node
            sh.n_slots = ns;
        }
        if (tid < mask_words) {
            const uint64_t up = anc_mask[(size_t)(base + p) * mask_words + tid];
            anc_mask[(size_t)(base + i) * mask_words + tid] = up | ((tid == i / 64) ? (1ull << (i % 64)) : 0ull);
        }
        ++n;
        __syncthreads();
    }
    if (tid == 0) n_built[seq] = n;
}

// The form with a workspace.  State of a row in LDS: its kMaxSeg segment totals and its maximum,
// kRowState doubles that follow each other in the workspace as well (the workspace's copy of the
// totals is not kept current).
//
// The open slots live in registers: slot s belongs to thread s % kBlock, which keeps its value,
// its (parent, rank) and the uniform draw of its sampling.  Every thread knows the slot being
// drawn from, its parent p, the rank of the child to draw and the draw u.
//
// A draw takes two barriers.  Lanes read p's segment totals from LDS (one each) and pick the
// segment with a 16-lane scan; every thread fetches, in one trip to global memory, its four
// logits of that segment and the word with their drawn-already bits.  While those loads
// are in flight each wave finds the best of its other open slots (DPP maximum and a ballot).
// Every thread computes its four weights (drawn tokens: 0) and their sum, in the order the
// pre-pass summed them; the sums are scanned (barrier 1).  The waves' totals tell every thread
// which wave holds the crossing; that wave finds the thread (the owner) with a ballot, takes the
// owner's four weights, finishes the draw (token, weight), has
// the owner store its bits and writes the segment's new total.  Meanwhile three
// other waves compute the path key of the new node and the draws of the two slots the draw
// opens (functions of p and rank only) and reduce the waves' bests to the best open slot outside
// this draw (barrier 2).  Every thread then computes the values of the two new slots, keeps them
// if they are its own, and picks the next slot among those two and the best of the rest; single
// lanes of different waves write the node down.
constexpr int kRowState = kMaxSeg + 1;
struct CachedShared {
    int last_child[DYSPEC_MAX_BUILD_NODES];
    int depth[DYSPEC_MAX_BUILD_NODES];
    uint2 pk[DYSPEC_MAX_BUILD_NODES];         // path keys of the nodes
    double wave_tot[kWaves];            // per draw: the waves' sums of the picked segment
    int last_live[kWaves];              // last thread of each wave with weight left, -1: none
    uint2 next_key;                     // path key of the node this draw makes
    float next_u[2];                    // draws of the two slots it opens
    double best_v[kWaves];              // per wave: its best open slot outside the current draw,
    int best_i[kWaves];                 //   the slot's index,
    int best_pr[kWaves];                //   its parent | rank << 10
    float best_u[kWaves];               //   and its draw
    double rest_v;                      // the best of those
    int rest_i, rest_pr;
    float rest_u;
    double draw_wy;                     // the drawn token and its weight
    int draw_y;
};
// LDS a workgroup may use on gfx950, less a margin; what CachedShared leaves of it holds the row states
constexpr size_t kLdsPerWorkgroup = 160 * 1024 - 1024;
static_assert(sizeof(CachedShared) + (size_t)DYSPEC_MAX_BUILD_NODES * kRowState * sizeof(double) <= kLdsPerWorkgroup,
              "the row states of the largest tree fit in LDS");
// A tree of N rows opens at most 2N - 1 slots (the root's, then two per draw): SLOTS of them per thread,
// 1 for N <= 256, 2 for N <= 512, 4 beyond.
constexpr int slots_per_thread(int n) { return n <= kBlock / 2 ? 1 : n <= kBlock ? 2 : 4; }
static_assert(4 * kBlock >= 2 * DYSPEC_MAX_BUILD_NODES - 1, "four slots per thread hold the largest tree's");
static_assert(DYSPEC_MAX_BUILD_NODES <= 1024 && DYSPEC_MAX_VOCAB <= (1 << 21), "a slot's parent and rank share one word");

template <bool VEC, int SLOTS>
__global__ __launch_bounds__(kBlock) void build_tree_cached_kernel(
    const float* __restrict__ draft_logits, int V, SeqArgs sa, uint64_t seed,
    dyspec_tree tree, float* __restrict__ est_value, uint64_t* __restrict__ anc_mask,
    int mask_words, int* __restrict__ n_built, double* ws)
{
    __shared__ CachedShared sh;
    extern __shared__ double row_state[];              // [N][kRowState]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = blockIdx.x;
    const int base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - base;
    const double inv_temp = 1.0 / (double)sa.temp_d[seq];
    for (int x = tid; x < N * kRowState; x += kBlock)
        row_state[x] = ws_totals(ws, base + x / kRowState)[x % kRowState];
    init_tree_rows(base, N, tree, est_value, anc_mask, mask_words);
    for (int i = tid; i < N; i += kBlock) { sh.last_child[i] = -1; sh.depth[i] = 0; }
    const uint2 key_root = root_key((uint32_t)seq);
    const float u_root = u01(seed, key_root, 0u, KIND_BUILD);
    if (tid == 0) sh.pk[0] = key_root;
    __syncthreads();

    // this thread's slots tid, tid + kBlock, ...: value (< 0: closed), parent | rank << 10, draw
    double my_v[SLOTS];
    int my_pr[SLOTS];
    float my_u[SLOTS];
#pragma unroll
    for (int k = 0; k < SLOTS; ++k) { my_v[k] = -1.0; my_pr[k] = 0; my_u[k] = 0.f; }
    if (tid == 0) { my_v[0] = 1.0; my_u[0] = u_root; }              // the root's slot
    auto set_slot = [&](int s, double v, int pr, float u) {
        if (tid == s % kBlock) {
#pragma unroll
            for (int k = 0; k < SLOTS; ++k)
                if (k == s / kBlock) { my_v[k] = v; my_pr[k] = pr; my_u[k] = u; }
        }
    };

    int n = 1, n_slots = 1;
    // the slot to draw from (known to every thread): the root's at first
    int pick = 0, p = 0, rank = 0;
    double v = 1.0, u = (double)u_root;
    while (n < N) {
        // the parent's mask word, needed when the node is appended: on its way during the draw
        const int mtid = tid - 4 * kWave;              // a wave that writes nothing else down
        uint64_t up = 0ull;
        if (mtid >= 0 && mtid < mask_words) up = anc_mask[(size_t)(base + p) * mask_words + mtid];

        // ---- draw the token from the residual draft distribution of p
        const float* __restrict__ row = draft_logits + (size_t)(base + p) * V;
        // (ws is written by this kernel and not declared restrict or const, so these are
        //  ordinary vector loads and stores; a bit word or a mask word is only ever re-read
        //  by the wave that wrote it)
        const double my_tot = row_state[p * kRowState + (lane & 15)];
        const double m = row_state[p * kRowState + kMaxSeg];
        const SegPick pk = pick_segment_lanes(my_tot, u);
        const double W = pk.W;
        if (!(W > 0.0)) break;                         // nothing left to sample under p
        const int tok_mine = pk.js * kSeg + 4 * tid;   // this thread's four tokens of the segment
        uint32_t* const gone_word = ws_gone(ws, base + p) + tok_mine / 32;
        const uint32_t gone = *gone_word;
        float lg[4];
        if constexpr (VEC) {
            const float4 x = tok_mine < V ? *reinterpret_cast<const float4*>(row + tok_mine) : make_float4(0.f, 0.f, 0.f, 0.f);
            lg[0] = x.x; lg[1] = x.y; lg[2] = x.z; lg[3] = x.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) lg[e] = tok_mine + e < V ? row[tok_mine + e] : 0.f;
        }
        // ---- while the loads are on their way: 1 / W for the slot values, and the best of this
        //      wave's open slots other than the one being drawn from (for the next pop)
        const double inv_W = 1.0 / W;
        {
            double bv = -1.0; int bi = 0x7fffffff, bpr = 0; float bu = 0.f;
#pragma unroll
            for (int k = 0; k < SLOTS; ++k)
                if (my_v[k] > bv && tid + k * kBlock != pick) { bv = my_v[k]; bi = tid + k * kBlock; bpr = my_pr[k]; bu = my_u[k]; }
            const double wv = wave_max_dpp(bv);        // largest value of the wave
            int wl;                                    // (a wave without an open slot: every lane holds -1, any will do)
            const int wi = first_of_equals(wv > 0.0 ? __ballot(bv == wv) : 1ull, bi, &wl);
            const int wpr = __builtin_amdgcn_readlane(bpr, wl);
            const float wu = readlane_f32(bu, wl);
            if (lane == 0) { sh.best_v[wave] = wv; sh.best_i[wave] = wi; sh.best_pr[wave] = wpr; sh.best_u[wave] = wu; }
        }
        // ---- this thread's four weights of the segment (a drawn token has none) and their sum,
        //      associated as the pre-pass did: the totals in LDS are sums of exactly these
        double w4[4];
        {
            double z[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) z[e] = fma((double)lg[e], inv_temp, -m);
            exp_nonpos_x4(z, w4);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (tok_mine + e >= V || ((gone >> (tok_mine % 32 + e)) & 1u)) w4[e] = 0.0;
        }
        const double mine = (w4[0] + w4[1]) + (w4[2] + w4[3]);
        // ---- inclusive scan of the 512 sums in thread order
        const double inc = wave_scan_dpp(mine);
        if (lane == kWave - 1) sh.wave_tot[wave] = inc;
        __syncthreads();                               // barrier 1 of 2
        // the waves' totals, one per lane (lanes 0..7 of every row of 16), scanned like the totals
        const double wt = (lane & 8) ? 0.0 : sh.wave_tot[lane & 7];
        double wc = wt;
        wc += dpp_or_zero<0x111>(wc);
        wc += dpp_or_zero<0x112>(wc);
        wc += dpp_or_zero<0x114>(wc);
        const double before = readlane_f64(dpp_or_zero<0x111>(wc), __builtin_amdgcn_readfirstlane(wave));
        // first wave whose running total is past u * W
        const uint32_t past = (uint32_t)__ballot(pk.cum_js + wc > pk.target) & 0xffu;
        int kw = past ? __builtin_ctz(past) : -1;
        const double incl = before + inc;
        const unsigned long long live = __ballot(mine > 0.0);
        int fixed_owner = -1;
        if (kw < 0) {
            // rounding at the very top: the last thread with weight left (the same in every thread)
            if (lane == 0) sh.last_live[wave] = live ? wave * kWave + 63 - __builtin_clzll(live) : -1;
            __syncthreads();
#pragma unroll
            for (int k = 0; k < kWaves; ++k) if (sh.last_live[k] >= 0) fixed_owner = sh.last_live[k];
            if (fixed_owner < 0) break;                // nothing left to sample under p
            kw = fixed_owner / kWave;
        }
        // ---- three waves that do not hold the crossing: the path key of the node this draw makes
        //      and the uniform draws of the two slots it opens (functions of p and rank only); the
        //      best open slot outside this draw (the winner among the waves' bests)
        if (wave == ((kw + 1) & 7) && lane == 0) sh.next_u[0] = u01(seed, sh.pk[p], (uint32_t)rank + 1u, KIND_BUILD);
        if (wave == ((kw + 2) & 7) && lane == 0) {
            const uint2 key_i = child_key(seed, sh.pk[p], (uint32_t)rank);
            sh.next_key = key_i;
            sh.next_u[1] = u01(seed, key_i, 0u, KIND_BUILD);
        }
        if (wave == ((kw + 3) & 7)) {
            const double cv = sh.best_v[lane & 7];     // lane l looks at wave l % 8
            const int ci = sh.best_i[lane & 7], cpr = sh.best_pr[lane & 7];
            const float cu = sh.best_u[lane & 7];
            double rv = cv;
            rv = fmax(rv, dpp_or_zero<kDppXor1>(rv));
            rv = fmax(rv, dpp_or_zero<kDppXor2>(rv));
            rv = fmax(rv, dpp_or_zero<kDppHalfMirror>(rv));
            rv = readlane_f64(rv, 0);
            int el;
            const int ri = first_of_equals(rv > 0.0 ? __ballot(cv == rv) & 0xffull : 1ull, ci, &el);
            const int rpr = __builtin_amdgcn_readlane(cpr, el);
            const float ru = readlane_f32(cu, el);
            if (lane == 0) { sh.rest_v = rv; sh.rest_i = ri; sh.rest_pr = rpr; sh.rest_u = ru; }
        }
        if (wave == kw) {
            // the wave's total is positive (it moved the running sum past the target), so a thread
            // with weight exists; after the first one past the target, else (the scan's rounding
            // can put the crossing on a thread without weight) the last one with weight
            const unsigned long long hit = __ballot(mine > 0.0 && pk.cum_js + incl > pk.target);
            const int ol = fixed_owner >= 0 ? fixed_owner % kWave : hit ? __builtin_ctzll(hit) : 63 - __builtin_clzll(live);
            const int tok0 = pk.js * kSeg + 4 * (kw * kWave + ol);
            // every lane of the wave finishes the draw with the owner's four weights: the token
            // among the four, what is left of their sum
            const double w4v[4] = { readlane_f64(w4[0], ol), readlane_f64(w4[1], ol), readlane_f64(w4[2], ol), readlane_f64(w4[3], ol) };
            double run = readlane_f64(pk.cum_js + (incl - mine), ol), wy = 0.0, wlast = 0.0;
            int y = -1, ylast = -1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                run += w4v[e];
                if (w4v[e] > 0.0) { ylast = tok0 + e; wlast = w4v[e]; }
                if (y < 0 && w4v[e] > 0.0 && run > pk.target) { y = tok0 + e; wy = w4v[e]; }
            }
            if (y < 0) { y = ylast; wy = wlast; }
            if (lane == 0) { sh.draw_y = y; sh.draw_wy = wy; }
            if (y >= 0) {
                // the sum that held y and the total of its segment lose y's weight
                const int ey = y - tok0;
                const double left = ((ey == 0 ? 0.0 : w4v[0]) + (ey == 1 ? 0.0 : w4v[1])) + ((ey == 2 ? 0.0 : w4v[2]) + (ey == 3 ? 0.0 : w4v[3]));
                if (lane == ol) *gone_word = gone | (1u << (tok0 % 32 + ey));
                const double wsum = wave_sum_dpp(lane == ol ? left : mine);     // the wave's sums again, the owner's replaced
                double t = (lane & 15) == kw ? wsum : wt;                       // lanes 0..7: the waves' totals now
                t += dpp_or_zero<kDppXor1>(t);
                t += dpp_or_zero<kDppXor2>(t);
                t += dpp_or_zero<kDppHalfMirror>(t);
                if (lane == 0) row_state[p * kRowState + pk.js] = t;
            }
        }
        __syncthreads();                               // barrier 2 of 2
        const int y = sh.draw_y;
        const double wy = sh.draw_wy;
        const float u_a = sh.next_u[0], u_b = sh.next_u[1];
        double nv = sh.rest_v; int ni = sh.rest_i, npr = sh.rest_pr; float nu = sh.rest_u;
        if (y < 0) break;                              // nothing left to sample under p
        // ---- node n: close the slot, open its two slots
        const int i = n;
        // R[y] = wy / W: with the correctly rounded 1 / W at hand, a product and one correction step
        // give the correctly rounded quotient; the last token of a row has R[y] = 1 exactly
        double Ry = wy * inv_W;
        Ry = fma(fma(-W, Ry, wy), inv_W, Ry);
        if (wy == W) Ry = 1.0;
        const double v0 = v * Ry, v1 = v * (1.0 - Ry);
        set_slot(pick, -1.0, 0, 0.f);
        // ---- the node is written down by single lanes of waves with nothing else to store
        if (tid == 0) {                                // links
            const int prev = sh.last_child[p];
            if (prev < 0) tree.first_child[base + p] = i; else tree.next_sibling[base + prev] = i;
            sh.last_child[p] = i;
            sh.pk[i] = sh.next_key;
        }
        if (tid == 3 * kWave) {                        // the node's own row
            const int dep = sh.depth[p] + 1;
            sh.depth[i] = dep;
            tree.parent[base + i] = p; tree.token[base + i] = y; tree.sib_rank[base + i] = rank;
            tree.depth[base + i] = dep;
            est_value[base + i] = (float)v;
        }
        if (mtid >= 0 && mtid < mask_words)
            anc_mask[(size_t)(base + i) * mask_words + mtid] = up | ((mtid == i / 64) ? (1ull << (i % 64)) : 0ull);
        ++n;
        // ---- the two new slots, and the next pop: the best slot outside this draw or one of the
        //      new ones (largest value, earliest-opened on ties: the new ones are the latest)
        if (v1 > 0.0) {                                // next sampling at this position
            const int pr_a = p | ((rank + 1) << 10);
            if (v1 > nv) { nv = v1; ni = n_slots; npr = pr_a; nu = u_a; }
            set_slot(n_slots++, v1, pr_a, u_a);
        }
        if (v0 > 0.0) {                                // first child of the new node
            if (v0 > nv) { nv = v0; ni = n_slots; npr = i; nu = u_b; }
            set_slot(n_slots++, v0, i, u_b);
        }
        if (!(nv > 0.0)) break;                        // frontier is empty
        pick = ni; p = npr & 1023; rank = npr >> 10; v = nv; u = (double)nu;
    }
    if (tid == 0) n_built[seq] = n;
}

// the cached builder keeps kRowState doubles per row in dynamic LDS: raised to the largest tree once
hipError_t prepare_build_tree()
{
    static std::atomic<unsigned long long> done[6] = { {0}, {0}, {0}, {0}, {0}, {0} };
    constexpr int bytes = DYSPEC_MAX_BUILD_NODES * kRowState * (int)sizeof(double);
    const void* const kernels[6] = {
        reinterpret_cast<const void*>(&build_tree_cached_kernel<true, 1>), reinterpret_cast<const void*>(&build_tree_cached_kernel<true, 2>),
        reinterpret_cast<const void*>(&build_tree_cached_kernel<true, 4>), reinterpret_cast<const void*>(&build_tree_cached_kernel<false, 1>),
        reinterpret_cast<const void*>(&build_tree_cached_kernel<false, 2>), reinterpret_cast<const void*>(&build_tree_cached_kernel<false, 4>) };
    for (int k = 0; k < 6; ++k) {
        const hipError_t e = raise_dynamic_lds_once(kernels[k], bytes, done[k]);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <bool VEC>
static void launch_cached(int slots, int n_seq, size_t dyn_bytes, hipStream_t stream, const float* draft_logits, int V, const SeqArgs& sa,
                          uint64_t seed, const dyspec_tree& tree, float* est_value, uint64_t* anc_mask, int mask_words, int* n_built,
                          double* ws)
{
    if (slots == 1)
        build_tree_cached_kernel<VEC, 1><<<n_seq, kBlock, dyn_bytes, stream>>>(draft_logits, V, sa, seed, tree, est_value, anc_mask, mask_words, n_built, ws);
    else if (slots == 2)
        build_tree_cached_kernel<VEC, 2><<<n_seq, kBlock, dyn_bytes, stream>>>(draft_logits, V, sa, seed, tree, est_value, anc_mask, mask_words, n_built, ws);
    else
        build_tree_cached_kernel<VEC, 4><<<n_seq, kBlock, dyn_bytes, stream>>>(draft_logits, V, sa, seed, tree, est_value, anc_mask, mask_words, n_built, ws);
}

size_t build_tree_workspace_bytes(int total_rows) { return (size_t)total_rows * kRowSumDoubles * sizeof(double); }

hipError_t launch_build_tree(const float* draft_logits, int V, const SeqArgs& sa, uint64_t seed,
                             const dyspec_tree& tree, float* est_value, uint64_t* anc_mask,
                             int mask_words, int* n_built, void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    const int rows = sa.node_off[sa.n_seq];
    double* ws = static_cast<double*>(workspace);
    const bool cached = ws != nullptr && workspace_bytes >= build_tree_workspace_bytes(rows);
    if (cached) {
        int widest = 0;
        for (int s = 0; s < sa.n_seq; ++s) widest = max(widest, sa.node_off[s + 1] - sa.node_off[s]);
        const size_t dyn_bytes = (size_t)widest * kRowState * sizeof(double);
        const hipError_t ea = prepare_build_tree();
        if (ea != hipSuccess) return ea;
        if (V % 4 == 0) {
            draft_row_sums_kernel<true><<<rows, kBlock, 0, stream>>>(draft_logits, V, sa, ws);
            launch_cached<true>(slots_per_thread(widest), sa.n_seq, dyn_bytes, stream, draft_logits, V, sa, seed, tree, est_value, anc_mask,
                                mask_words, n_built, ws);
        } else {
            draft_row_sums_kernel<false><<<rows, kBlock, 0, stream>>>(draft_logits, V, sa, ws);
            launch_cached<false>(slots_per_thread(widest), sa.n_seq, dyn_bytes, stream, draft_logits, V, sa, seed, tree, est_value, anc_mask,
                                 mask_words, n_built, ws);
        }
    } else if (V % 4 == 0) {
        build_tree_kernel<true><<<sa.n_seq, kBlock, 0, stream>>>(draft_logits, V, sa, seed, tree, est_value,
                                                                 anc_mask, mask_words, n_built);
    } else {
        build_tree_kernel<false><<<sa.n_seq, kBlock, 0, stream>>>(draft_logits, V, sa, seed, tree, est_value,
                                                                  anc_mask, mask_words, n_built);
    }
    return hipGetLastError();
}

}  // namespace dyspec
