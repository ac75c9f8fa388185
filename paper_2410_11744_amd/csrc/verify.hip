// Vocabulary softmax statistics of every tree row and multi-candidate tree rejection
// sampling (Algorithm 3, Appendix A.3; one-candidate rule of Section 2) for gfx950.
//
// Two kernels.  The statistics kernel is the data-parallel part: it reads every tree row's
// draft and target logits from HBM once and reduces each to (max, sum-exp), the normalisers
// every later probability needs (a streaming form for V % 4 == 0, a plain one workgroup per
// row form otherwise).  verify_walk_kernel is Algorithm 3 itself,
// one workgroup per sequence walking from the root: the first child of a node is tested
// from two logits and the row statistics alone; only after a rejection are the node's two
// rows brought into registers (normalised with the statistics, no reduction) for the residual
// updates R <- norm(max(R-D,0)), D[y] <- 0, D <- norm(D), one workgroup reduction per
// rejected child, stopping at the first accepted one.  Tree links and statistics of the
// sequence are staged in LDS so the walk chases pointers there, not in HBM.
//
// A target temperature of 0 (the temperature-0 rows of Section 5's tables) makes the target
// row all mass on its largest logit, the smallest index winning a tie.  For such a sequence
// the statistics pass stores (largest raw target logit, its index) in place of (max, sum-exp)
// and the walk builds its target row from that index instead of reading the logits; every
// other step of Algorithm 3 runs unchanged.
#include "vocab_common.h"

namespace dyspec {

// (value, index) pairs ordered by larger value, then smaller index
__device__ __forceinline__ void better_of(float& m, int& i, float m2, int i2)
{
    if (m2 > m || (m2 == m && i2 < i)) { m = m2; i = i2; }
}

// Largest value and the first index holding it over a workgroup of NW waves; every thread
// brings its own best pair.  The result is valid in thread 0.
template <int NW>
__device__ __forceinline__ void block_argmax(float& m, int& i, float* red_m, int* red_i)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) better_of(m, i, __shfl_xor(m, o, kWave), __shfl_xor(i, o, kWave));
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) { red_m[wave] = m; red_i[wave] = i; }
    __syncthreads();
    if (threadIdx.x == 0) {
        m = red_m[0]; i = red_i[0];
        for (int w = 1; w < NW; ++w) better_of(m, i, red_m[w], red_i[w]);
    }
}

template <bool VEC, typename T>
__global__ __launch_bounds__(kBlock) void softmax_stats_kernel(
    const T* __restrict__ draft_logits, const T* __restrict__ target_logits, int V,
    SeqArgs sa, float* __restrict__ row_stats, float* __restrict__ accept_ratio)
{
    __shared__ float fred[kWaves * 2];
    __shared__ int ired[kWaves];
    const int row = blockIdx.x;
    const int seq = find_seq(sa, row);
    const bool greedy = sa.temp_t[seq] == 0.0f;
    const float inv_td = 1.0f / sa.temp_d[seq], inv_tt = greedy ? 1.0f : 1.0f / sa.temp_t[seq];
    float D[kMaxSeg][4], R[kMaxSeg][4];
    load_row<VEC, T>(draft_logits + (size_t)row * V, V, D);
    load_row<VEC, T>(target_logits + (size_t)row * V, V, R);
    float top = -INFINITY;
    int top_i = 0;
    if (greedy) {
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (R[j][e] > top) { top = R[j][e]; top_i = tok_index(j, e); }   // ascending index per thread
        block_argmax<kWaves>(top, top_i, fred, ired);
        __syncthreads();
    }
    float mx[2] = { -INFINITY, -INFINITY };
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            D[j][e] *= inv_td; R[j][e] *= inv_tt;
            mx[0] = fmaxf(mx[0], D[j][e]); mx[1] = fmaxf(mx[1], R[j][e]);
        }
    block_max<2>(mx, fred);
    float sm[2] = { 0.0f, 0.0f };
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sm[0] += expf(D[j][e] - mx[0]); sm[1] += expf(R[j][e] - mx[1]);   // exp(-inf) = 0 past V
        }
    block_sum<float, 2>(sm, fred);
    if (threadIdx.x == 0) {
        *reinterpret_cast<float4*>(row_stats + 4 * (size_t)row) =
            greedy ? make_float4(mx[0], sm[0], top, (float)top_i) : make_float4(mx[0], sm[0], mx[1], sm[1]);
        accept_ratio[row] = (row == sa.node_off[seq]) ? 0.0f : -2.0f;      // -2: not tested by the walk
    }
}

// Streaming form of the statistics pass for V % 4 == 0: one workgroup of 256 threads per
// (row, table), so a 512-row batch puts 1024 independent 128 KB streams on the chip.  Each
// thread keeps a running (max, sum) pair over its 16-byte pieces, eight pieces in flight, and
// raises its reference once per batch of 32 values (33 exponentials per 32 values); pairs are
// merged with (m, s) + (m', s') = (M, s 2^{c(m-M)} + s' 2^{c(m'-M)}), M = max(m, m').  The
// maximum is taken over the raw logits, so max * (1/T) is rounded exactly as the plain
// two-pass form rounds it.
constexpr int kStatThreads = 256;
constexpr int kStatUnroll = 8;

__device__ __forceinline__ void merge_stat(float& m, float& s, float m2, float s2, float c)
{
    const float M = fmaxf(m, m2);
    if (M == -INFINITY) return;                                  // both empty
    s = s * __builtin_amdgcn_exp2f((m - M) * c) + s2 * __builtin_amdgcn_exp2f((m2 - M) * c);
    m = M;
}

__global__ __launch_bounds__(kStatThreads) void softmax_stats_stream_kernel(
    const float* __restrict__ draft_logits, const float* __restrict__ target_logits, int V,
    SeqArgs sa, float* __restrict__ row_stats, float* __restrict__ accept_ratio)
{
    __shared__ float red[2 * (kStatThreads / kWave)];
    const int row = blockIdx.x, table = blockIdx.y;
    const int seq = find_seq(sa, row);
    const float4* __restrict__ x = reinterpret_cast<const float4*>((table ? target_logits : draft_logits) + (size_t)row * V);
    const int n4 = V / 4;
    if (table == 1 && sa.temp_t[seq] == 0.0f) {                  // whole workgroup takes this branch
        __shared__ int ired[kStatThreads / kWave];
        float top = -INFINITY;
        int top_i = 0;
        for (int i0 = threadIdx.x; i0 < n4; i0 += kStatThreads * kStatUnroll) {
            float4 v[kStatUnroll];
#pragma unroll
            for (int u = 0; u < kStatUnroll; ++u) {
                const int i = i0 + u * kStatThreads;
                v[u] = (i < n4) ? x[i] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            }
#pragma unroll
            for (int u = 0; u < kStatUnroll; ++u) {              // ascending index per thread
                const int i = 4 * (i0 + u * kStatThreads);
                if (v[u].x > top) { top = v[u].x; top_i = i; }
                if (v[u].y > top) { top = v[u].y; top_i = i + 1; }
                if (v[u].z > top) { top = v[u].z; top_i = i + 2; }
                if (v[u].w > top) { top = v[u].w; top_i = i + 3; }
            }
        }
        block_argmax<kStatThreads / kWave>(top, top_i, red, ired);
        if (threadIdx.x == 0)
            *reinterpret_cast<float2*>(row_stats + 4 * (size_t)row + 2) = make_float2(top, (float)top_i);
        return;
    }
    const float inv_t = 1.0f / (table ? sa.temp_t[seq] : sa.temp_d[seq]);
    const float c = inv_t * 1.4426950408889634f;
    float m = -INFINITY, s = 0.0f;
    for (int i0 = threadIdx.x; i0 < n4; i0 += kStatThreads * kStatUnroll) {
        float4 v[kStatUnroll];
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) {
            const int i = i0 + u * kStatThreads;
            v[u] = (i < n4) ? x[i] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        }
        float cm = -INFINITY;
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) cm = fmaxf(fmaxf(cm, fmaxf(v[u].x, v[u].y)), fmaxf(v[u].z, v[u].w));
        const float M = fmaxf(m, cm);
        if (M == -INFINITY) continue;                            // nothing but -inf logits so far
        float acc = s * __builtin_amdgcn_exp2f((m - M) * c);
        const float Mc = M * c;
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) {
            acc += __builtin_amdgcn_exp2f(fmaf(v[u].x, c, -Mc)) + __builtin_amdgcn_exp2f(fmaf(v[u].y, c, -Mc));
            acc += __builtin_amdgcn_exp2f(fmaf(v[u].z, c, -Mc)) + __builtin_amdgcn_exp2f(fmaf(v[u].w, c, -Mc));
        }
        s = acc;
        m = M;
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) merge_stat(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave), c);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) { red[2 * wave] = m; red[2 * wave + 1] = s; }
    __syncthreads();
    if (threadIdx.x == 0) {
        m = red[0]; s = red[1];
#pragma unroll
        for (int w = 1; w < kStatThreads / kWave; ++w) merge_stat(m, s, red[2 * w], red[2 * w + 1], c);
        *reinterpret_cast<float2*>(row_stats + 4 * (size_t)row + 2 * table) = make_float2(m * inv_t, s);
        if (table == 0) accept_ratio[row] = (row == sa.node_off[seq]) ? 0.0f : -2.0f;   // -2: not tested by the walk
    }
}

// Sixteen bytes of a logits row: four fp32 or eight bf16 values.
template <typename T> struct Piece;
template <> struct Piece<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void unpack(const uint4& r, float (&f)[4])
    {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
};
template <> struct Piece<__bf16> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void unpack(const uint4& r, float (&f)[8])
    {
        f[0] = bf16_bits_to_float(r.x & 0xffffu); f[1] = bf16_bits_to_float(r.x >> 16);
        f[2] = bf16_bits_to_float(r.y & 0xffffu); f[3] = bf16_bits_to_float(r.y >> 16);
        f[4] = bf16_bits_to_float(r.z & 0xffffu); f[5] = bf16_bits_to_float(r.z >> 16);
        f[6] = bf16_bits_to_float(r.w & 0xffffu); f[7] = bf16_bits_to_float(r.w >> 16);
    }
};

// The streaming form for tables of type T read in 16-byte pieces; V a multiple of the values in
// a piece.  (fp32 tables take the kernel above, written out for four values per piece.)
template <typename T>
__global__ __launch_bounds__(kStatThreads) void softmax_stats_stream_pieces_kernel(
    const T* __restrict__ draft_logits, const T* __restrict__ target_logits, int V,
    SeqArgs sa, float* __restrict__ row_stats, float* __restrict__ accept_ratio)
{
    constexpr int PN = Piece<T>::N;
    __shared__ float red[2 * (kStatThreads / kWave)];
    const int row = blockIdx.x, table = blockIdx.y;
    const int seq = find_seq(sa, row);
    // pieces are fetched as float4 (one 16-byte load each; the bits are taken apart afterwards)
    const float4* __restrict__ x = reinterpret_cast<const float4*>((table ? target_logits : draft_logits) + (size_t)row * V);
    const int n16 = V / PN;
    // a piece past the end re-reads the last piece and is then set to -inf
    auto fetch = [&](int i) __attribute__((always_inline)) { return x[min(i, n16 - 1)]; };
    auto open_piece = [&](const float4& r, bool valid, float (&f)[PN]) __attribute__((always_inline)) {
        Piece<T>::unpack(make_uint4(__float_as_uint(r.x), __float_as_uint(r.y), __float_as_uint(r.z), __float_as_uint(r.w)), f);
#pragma unroll
        for (int e = 0; e < PN; ++e) f[e] = valid ? f[e] : -INFINITY;
    };
    if (table == 1 && sa.temp_t[seq] == 0.0f) {                  // whole workgroup takes this branch
        __shared__ int ired[kStatThreads / kWave];
        float top = -INFINITY;
        int top_i = 0;
        for (int i0 = threadIdx.x; i0 < n16; i0 += kStatThreads * kStatUnroll) {
            float4 v[kStatUnroll];
#pragma unroll
            for (int u = 0; u < kStatUnroll; ++u) v[u] = fetch(i0 + u * kStatThreads);
#pragma unroll
            for (int u = 0; u < kStatUnroll; ++u) {              // ascending index per thread
                const int i = PN * (i0 + u * kStatThreads);
                float f[PN];
                open_piece(v[u], i0 + u * kStatThreads < n16, f);
#pragma unroll
                for (int e = 0; e < PN; ++e) if (f[e] > top) { top = f[e]; top_i = i + e; }
            }
        }
        block_argmax<kStatThreads / kWave>(top, top_i, red, ired);
        if (threadIdx.x == 0)
            *reinterpret_cast<float2*>(row_stats + 4 * (size_t)row + 2) = make_float2(top, (float)top_i);
        return;
    }
    const float inv_t = 1.0f / (table ? sa.temp_t[seq] : sa.temp_d[seq]);
    const float c = inv_t * 1.4426950408889634f;
    float m = -INFINITY, s = 0.0f;
    for (int i0 = threadIdx.x; i0 < n16; i0 += kStatThreads * kStatUnroll) {
        float4 v[kStatUnroll];
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) v[u] = fetch(i0 + u * kStatThreads);
        float f[kStatUnroll][PN];
        float cm = -INFINITY;
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) {
            open_piece(v[u], i0 + u * kStatThreads < n16, f[u]);
#pragma unroll
            for (int e = 0; e < PN; e += 2) cm = fmaxf(cm, fmaxf(f[u][e], f[u][e + 1]));
        }
        const float M = fmaxf(m, cm);
        if (M == -INFINITY) continue;                            // nothing but -inf logits so far
        float acc = s * __builtin_amdgcn_exp2f((m - M) * c);
        const float Mc = M * c;
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u)
#pragma unroll
            for (int e = 0; e < PN; e += 2)
                acc += __builtin_amdgcn_exp2f(fmaf(f[u][e], c, -Mc)) + __builtin_amdgcn_exp2f(fmaf(f[u][e + 1], c, -Mc));
        s = acc;
        m = M;
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) merge_stat(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave), c);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) { red[2 * wave] = m; red[2 * wave + 1] = s; }
    __syncthreads();
    if (threadIdx.x == 0) {
        m = red[0]; s = red[1];
#pragma unroll
        for (int w = 1; w < kStatThreads / kWave; ++w) merge_stat(m, s, red[2 * w], red[2 * w + 1], c);
        *reinterpret_cast<float2*>(row_stats + 4 * (size_t)row + 2 * table) = make_float2(m * inv_t, s);
        if (table == 0) accept_ratio[row] = (row == sa.node_off[seq]) ? 0.0f : -2.0f;   // -2: not tested by the walk
    }
}

struct WalkShared {
    CdfScratch cdf;
    float fred[kWaves * 2];
    int token[DYSPEC_MAX_NODES];
    int first_child[DYSPEC_MAX_NODES];
    int next_sibling[DYSPEC_MAX_NODES];
    float4 stats[DYSPEC_MAX_NODES];
    float bcast[2];
};

template <bool VEC, typename T>
__global__ __launch_bounds__(kBlock) void verify_walk_kernel(
    const T* __restrict__ draft_logits, const T* __restrict__ target_logits, int V,
    SeqArgs sa, dyspec_tree tree, uint64_t seed, int emit_bonus,
    const float* __restrict__ row_stats, float* __restrict__ accept_ratio,
    int* __restrict__ accepted_nodes, int* __restrict__ n_accepted,
    int* __restrict__ final_token, float* __restrict__ min_margin)
{
    __shared__ WalkShared sh;
    const int tid = threadIdx.x;
    const int seq = blockIdx.x;
    const int base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - base;
    const bool greedy = sa.temp_t[seq] == 0.0f;                  // target row = all mass on stats.w
    const float inv_td = 1.0f / sa.temp_d[seq], inv_tt = greedy ? 1.0f : 1.0f / sa.temp_t[seq];
    for (int i = tid; i < N; i += kBlock) {
        sh.token[i] = tree.token[base + i];
        sh.first_child[i] = tree.first_child[base + i];
        sh.next_sibling[i] = tree.next_sibling[base + i];
        sh.stats[i] = *reinterpret_cast<const float4*>(row_stats + 4 * (size_t)(base + i));
    }
    __syncthreads();

    // probability of token y under row `node`: draft (.x) and target (.y)
    auto prob_pair = [&](int node, int y) {
        const float4 st = sh.stats[node];
        const float d = expf(logit_to_float(draft_logits[(size_t)(base + node) * V + y]) * inv_td - st.x) / st.y;
        const float r = greedy ? ((float)y == st.w ? 1.0f : 0.0f)
                               : expf(logit_to_float(target_logits[(size_t)(base + node) * V + y]) * inv_tt - st.z) / st.w;
        return make_float2(d, r);
    };
    auto ratio_of = [](float d, float r) { return (d > 0.0f) ? r / d : (r > 0.0f ? INFINITY : 0.0f); };

    int cur = 0, na = 0, fin = -1;
    uint2 pk = root_key((uint32_t)seq);
    float margin = INFINITY;
    for (int steps = 0; steps < N; ++steps) {            // a path has fewer than N edges
        int c = sh.first_child[cur];
        const bool leaf = c < 0 || c >= N;
        int next = -1;
        uint2 pk_next = pk;
        bool rows_loaded = false;
        float D[kMaxSeg][4], R[kMaxSeg][4];
        auto load_rows = [&](bool want_draft) {
            const float4 st = sh.stats[cur];
            if (!greedy) load_row<VEC, T>(target_logits + (size_t)(base + cur) * V, V, R);
            if (want_draft) load_row<VEC, T>(draft_logits + (size_t)(base + cur) * V, V, D);
            const float id = 1.0f / st.y, it = greedy ? 0.0f : 1.0f / st.w;
            const int top = greedy ? (int)st.w : -1;
#pragma unroll
            for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    R[j][e] = greedy ? (tok_index(j, e) == top ? 1.0f : 0.0f) : expf(R[j][e] * inv_tt - st.z) * it;
                    D[j][e] = want_draft ? expf(D[j][e] * inv_td - st.x) * id : 0.0f;
                }
        };
        if (!leaf) {
            // ---- first child: two logits and the row statistics decide
            {
                const int y = sh.token[c];
                const bool y_ok = y >= 0 && y < V;
                const float2 pr = y_ok ? prob_pair(cur, y) : make_float2(0.0f, 0.0f);
                const float ratio = ratio_of(pr.x, pr.y);
                const uint2 pk_n = child_key(seed, pk, 0u);
                const float u = u01(seed, pk_n, 0u, KIND_ACCEPT);
                margin = fminf(margin, fabsf(u - ratio));
                if (tid == 0) accept_ratio[base + c] = ratio;
                if (u < ratio) { next = c; pk_next = pk_n; }
            }
            // ---- rejected: bring the rows in and update the residuals child by child
            if (next < 0) {
                load_rows(true);
                rows_loaded = true;
                uint32_t rank = 0;
                for (int guard = 0; c >= 0 && c < N && guard < N; ++guard) {
                    const int y = sh.token[c];
                    const bool mine = y >= 0 && y < V && ((y % kSeg) >> 2) == tid;
                    if (rank > 0) {
                        // ratio seen by this child after its earlier siblings were rejected
                        if (mine) {
#pragma unroll
                            for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (j == y / kSeg && e == (y & 3)) { sh.bcast[0] = D[j][e]; sh.bcast[1] = R[j][e]; }
                        }
                        if (!(y >= 0 && y < V) && tid == 0) { sh.bcast[0] = 0.0f; sh.bcast[1] = 0.0f; }
                        __syncthreads();
                        const float ratio = ratio_of(sh.bcast[0], sh.bcast[1]);
                        const uint2 pk_n = child_key(seed, pk, rank);
                        const float u = u01(seed, pk_n, 0u, KIND_ACCEPT);
                        margin = fminf(margin, fabsf(u - ratio));
                        if (tid == 0) accept_ratio[base + c] = ratio;
                        if (u < ratio) { next = c; pk_next = pk_n; break; }
                    }
                    // reject child c: R <- norm(max(R-D,0)) with D as it stands, then y leaves D
                    float res[2] = { 0.0f, 0.0f };          // mass of relu(R-D), mass left in D
                    float dy_old = 0.0f;
#pragma unroll
                    for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float d = D[j][e], r = R[j][e];
                            if (mine && j == y / kSeg && e == (y & 3)) { dy_old = d; D[j][e] = 0.0f; }
                            res[0] += fmaxf(r - d, 0.0f);
                            res[1] += D[j][e];
                        }
                    block_sum<float, 2>(res, sh.fred);
                    if (res[0] > 0.0f) {                     // else R == D: keep R (no reject can reach here)
                        const float ir = 1.0f / res[0];
#pragma unroll
                        for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float d = (mine && j == y / kSeg && e == (y & 3)) ? dy_old : D[j][e];
                                R[j][e] = fmaxf(R[j][e] - d, 0.0f) * ir;
                            }
                    }
                    c = sh.next_sibling[c];
                    ++rank;
                    if (!(res[1] > 0.0f)) {                  // D is empty: later children are not tried
                        if (tid == 0)
                            for (int k = 0, cc = c; cc >= 0 && cc < N && k < N; ++k, cc = sh.next_sibling[cc])
                                accept_ratio[base + cc] = -1.0f;
                        break;
                    }
                    const float il = 1.0f / res[1];
#pragma unroll
                    for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
                        for (int e = 0; e < 4; ++e) D[j][e] *= il;
                }
            }
        }
        if (next >= 0) {
            if (tid == 0) accepted_nodes[base + na] = next;
            ++na;
            cur = next; pk = pk_next;
            continue;
        }
        // ---- the walk stops at cur: emit a token from what is left of the target row
        if (leaf && !emit_bonus) { fin = -1; break; }
        if (!rows_loaded) load_rows(false);
        __syncthreads();
        const double u = (double)u01(seed, pk, 0u, KIND_RESID);
        double W, wy;
        fin = block_inverse_cdf<float>(R, u, &sh.cdf, &W, &wy);
        break;
    }
    if (tid == 0) {
        n_accepted[seq] = na;
        final_token[seq] = fin;
        min_margin[seq] = margin;
    }
}

template <typename T>
static hipError_t launch_verify_t(const T* draft_logits, const T* target_logits, int V,
                                  const SeqArgs& sa, const dyspec_tree& tree, uint64_t seed, int emit_bonus,
                                  float* row_stats, float* accept_ratio, int* accepted_nodes, int* n_accepted,
                                  int* final_token, float* min_margin, hipStream_t stream)
{
    const int rows = sa.node_off[sa.n_seq];
    // statistics: the streaming form wants whole 16-byte pieces; the walk's row loads four tokens per thread
    if (V % Piece<T>::N == 0) {
        if constexpr (sizeof(T) == 4)
            softmax_stats_stream_kernel<<<dim3(rows, 2), kStatThreads, 0, stream>>>(draft_logits, target_logits, V, sa, row_stats, accept_ratio);
        else
            softmax_stats_stream_pieces_kernel<T><<<dim3(rows, 2), kStatThreads, 0, stream>>>(draft_logits, target_logits, V, sa, row_stats, accept_ratio);
    }
    else if (V % 4 == 0)
        softmax_stats_kernel<true, T><<<rows, kBlock, 0, stream>>>(draft_logits, target_logits, V, sa, row_stats, accept_ratio);
    else
        softmax_stats_kernel<false, T><<<rows, kBlock, 0, stream>>>(draft_logits, target_logits, V, sa, row_stats, accept_ratio);
    if (V % 4 == 0)
        verify_walk_kernel<true, T><<<sa.n_seq, kBlock, 0, stream>>>(draft_logits, target_logits, V, sa, tree, seed, emit_bonus,
                                                                     row_stats, accept_ratio, accepted_nodes, n_accepted,
                                                                     final_token, min_margin);
    else
        verify_walk_kernel<false, T><<<sa.n_seq, kBlock, 0, stream>>>(draft_logits, target_logits, V, sa, tree, seed, emit_bonus,
                                                                      row_stats, accept_ratio, accepted_nodes, n_accepted,
                                                                      final_token, min_margin);
    return hipGetLastError();
}

hipError_t launch_verify(const void* draft_logits, const void* target_logits, bool bf16_logits, int V,
                         const SeqArgs& sa, const dyspec_tree& tree, uint64_t seed, int emit_bonus,
                         float* row_stats, float* accept_ratio, int* accepted_nodes, int* n_accepted,
                         int* final_token, float* min_margin, hipStream_t stream)
{
    if (bf16_logits)
        return launch_verify_t(static_cast<const __bf16*>(draft_logits), static_cast<const __bf16*>(target_logits), V, sa, tree,
                               seed, emit_bonus, row_stats, accept_ratio, accepted_nodes, n_accepted, final_token, min_margin, stream);
    return launch_verify_t(static_cast<const float*>(draft_logits), static_cast<const float*>(target_logits), V, sa, tree,
                           seed, emit_bonus, row_stats, accept_ratio, accepted_nodes, n_accepted, final_token, min_margin, stream);
}

}  // namespace dyspec
