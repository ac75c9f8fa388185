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
#include "lane_ops.h"

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

// exp(x) for x <= 0 through the hardware's exp2 (inputs below -126/log2(e) give 0, which is what a
// probability that small is here): one multiply and one v_exp_f32, about 1e-7 |x| of relative
// error, against some twenty instructions of the library routine -- a thread turns 128 logits
// into probabilities per visited node.
__device__ __forceinline__ float exp_fast(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }

// Inverse CDF over a register-resident row of weights (the step's last token): the smallest token
// index y, in the order (segment, thread, element), whose cumulative weight exceeds u * W.  Sums
// are fp64.  The threads' sixteen segment sums are staged in LDS (`stage`: kStageDoubles doubles);
// wave w totals segments 2w and 2w+1 from there; every thread reads the sixteen totals and picks
// the segment; each wave scans its 64 sums of that segment across lanes; the eight wave totals
// tell every thread which wave holds the crossing, and that wave finds the owning thread with a
// ballot; the owner walks its four weights.  Three barriers.  Every thread gets y (-1 when W == 0).
constexpr int kStageDoubles = kMaxSeg * kBlock + kMaxSeg;
struct DrawScratch {
    double wave_tot[kWaves];
    int last_live[kWaves];
    int y;
};
__device__ __forceinline__ int draw_from_row(const float (&w)[kMaxSeg][4], double u, DrawScratch* sc, double* stage)
{
    static_assert(kMaxSeg == 2 * kWaves, "two segments per wave");
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j)
        stage[j * kBlock + tid] = ((double)w[j][0] + (double)w[j][1]) + ((double)w[j][2] + (double)w[j][3]);
    __syncthreads();
    double* const totals = stage + kMaxSeg * kBlock;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int j = 2 * wave + k;
        double a = 0.0;
#pragma unroll
        for (int i = 0; i < kBlock / kWave; ++i) a += stage[j * kBlock + i * kWave + lane];
        a = wave_sum_dpp(a);
        if (lane == 0) totals[j] = a;
    }
    __syncthreads();
    double tot[kMaxSeg];
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) tot[j] = totals[j];
    const SegPick pk = pick_segment(tot, u);
    if (!(pk.W > 0.0)) return -1;                            // uniform
    const double mine = stage[pk.js * kBlock + tid];
    const double inc = wave_scan_dpp(mine);                  // inclusive, in lane order
    const unsigned long long live = __ballot(mine > 0.0);
    if (lane == kWave - 1) sc->wave_tot[wave] = inc;
    if (lane == 0) sc->last_live[wave] = live ? wave * kWave + 63 - __builtin_clzll(live) : -1;
    __syncthreads();
    // the first wave whose running total is past the target; with none (rounding at the very top)
    // the last thread that has weight
    double before = 0.0, run = pk.cum_js;
    int kw = -1, fixed_owner = -1;
#pragma unroll
    for (int k = 0; k < kWaves; ++k) {
        const double t = sc->wave_tot[k];
        if (kw < 0 && run + t > pk.target) { kw = k; before = run - pk.cum_js; }
        run += t;
        if (sc->last_live[k] >= 0) fixed_owner = sc->last_live[k];
    }
    if (kw >= 0) fixed_owner = -1;
    else if (fixed_owner >= 0) kw = fixed_owner / kWave;
    if (wave == kw) {
        const unsigned long long hit = __ballot(mine > 0.0 && pk.cum_js + before + inc > pk.target);
        const int ol = fixed_owner >= 0 ? fixed_owner % kWave : hit ? __builtin_ctzll(hit) : 63 - __builtin_clzll(live);
        if (lane == ol) {
            // this thread's four weights of the picked segment (sixteen uniform compares pick the registers)
            float w4[4] = { 0.0f, 0.0f, 0.0f, 0.0f };
#pragma unroll
            for (int jj = 0; jj < kMaxSeg; ++jj)
                if (jj == pk.js) { w4[0] = w[jj][0]; w4[1] = w[jj][1]; w4[2] = w[jj][2]; w4[3] = w[jj][3]; }
            double c = pk.cum_js + before + (inc - mine);
            int y = -1, ylast = -1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                c += (double)w4[e];
                if (w4[e] > 0.0f) ylast = tok_index(pk.js, e);
                if (y < 0 && w4[e] > 0.0f && c > pk.target) y = tok_index(pk.js, e);
            }
            sc->y = y >= 0 ? y : ylast;
        }
    } else if (kw < 0 && tid == 0) {
        sc->y = -1;                                          // the totals held rounding dust only
    }
    __syncthreads();
    return sc->y;
}

// LDS of the walk.  Static part: scratch of the reductions.  Dynamic part: the draft row of the
// node being decided, as unnormalised weights exp(logit/T - max) indexed by token (what is left of
// D after the children rejected so far is D_lds[x] * scale), then the sequence's tree links as
// 16-bit values (tokens < 32768, nodes < 2048; -1 = none).  The target row R stays in registers.
struct WalkShared {
    DrawScratch draw;
    float fred[kWaves * 2];
    float bcast[2];
};
// (the row's place also stages the partial sums of the final draw: at least kStageDoubles doubles)
__host__ __device__ __forceinline__ size_t walk_row_bytes(int V)
{
    const size_t row = (size_t)((V + 3) & ~3) * sizeof(float), stage = (size_t)kStageDoubles * sizeof(double);
    return row > stage ? row : stage;
}
static size_t walk_lds_bytes(int V, int widest) { return walk_row_bytes(V) + 3 * (size_t)((widest + 7) & ~7) * sizeof(short); }

template <bool VEC, typename T>
__global__ __launch_bounds__(kBlock) void verify_walk_kernel(
    const T* __restrict__ draft_logits, const T* __restrict__ target_logits, int V,
    SeqArgs sa, dyspec_tree tree, uint64_t seed, int emit_bonus,
    const float* __restrict__ row_stats, float* __restrict__ accept_ratio,
    int* __restrict__ accepted_nodes, int* __restrict__ n_accepted,
    int* __restrict__ final_token, float* __restrict__ min_margin)
{
    __shared__ WalkShared sh;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn[];
    const int tid = threadIdx.x;
    const int seq = blockIdx.x;
    const int base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - base;
    const bool greedy = sa.temp_t[seq] == 0.0f;                  // target row = all mass on stats.w
    const float inv_td = 1.0f / sa.temp_d[seq], inv_tt = greedy ? 1.0f : 1.0f / sa.temp_t[seq];
    float* const D_lds = reinterpret_cast<float*>(dyn);
    const int Npad = (N + 7) & ~7;
    short* const l_token = reinterpret_cast<short*>(dyn + walk_row_bytes(V));
    short* const l_child = l_token + Npad;
    short* const l_next = l_child + Npad;
    for (int i = tid; i < N; i += kBlock) {
        const int tk = tree.token[base + i], fc = tree.first_child[base + i], ns = tree.next_sibling[base + i];
        l_token[i] = (short)((tk >= 0 && tk < V) ? tk : -1);     // anything else is no token: ratio 0
        l_child[i] = (short)((fc >= 0 && fc < N) ? fc : -1);
        l_next[i] = (short)((ns >= 0 && ns < N) ? ns : -1);
    }
    __syncthreads();

    auto ratio_of = [](float d, float r) { return (d > 0.0f) ? r / d : (r > 0.0f ? INFINITY : 0.0f); };

    int cur = 0, na = 0, fin = -1;
    uint2 pk = root_key((uint32_t)seq);
    float margin = INFINITY;
    for (int steps = 0; steps < N; ++steps) {            // a path has fewer than N edges
        int c = l_child[cur];
        const bool leaf = c < 0;
        int next = -1;
        uint2 pk_next = pk;
        bool rows_loaded = false;
        float R[kMaxSeg][4];
        // the node's statistics: one 16-byte load, on its way together with the first child's logits
        const float4 st = *reinterpret_cast<const float4*>(row_stats + 4 * (size_t)(base + cur));
        float scale_d = 0.0f;                             // what is left of D = D_lds * scale_d
        // R <- softmax of the target row (registers); with want_draft, D_lds <- the draft row's weights
        auto load_rows = [&](bool want_draft) {
            float X[kMaxSeg][4];
            if (want_draft) {
                load_row<VEC, T>(draft_logits + (size_t)(base + cur) * V, V, X);
#pragma unroll
                for (int j = 0; j < kMaxSeg; ++j) {
                    const int i0 = tok_index(j, 0);
                    if (i0 < V)                           // V is padded to a multiple of 4 in LDS; logits past V read as -inf
                        *reinterpret_cast<float4*>(D_lds + i0) = make_float4(exp_fast(X[j][0] * inv_td - st.x), exp_fast(X[j][1] * inv_td - st.x),
                                                                             exp_fast(X[j][2] * inv_td - st.x), exp_fast(X[j][3] * inv_td - st.x));
                }
                scale_d = 1.0f / st.y;
            }
            if (!greedy) load_row<VEC, T>(target_logits + (size_t)(base + cur) * V, V, R);
            const float it = greedy ? 0.0f : 1.0f / st.w;
            const int top = greedy ? (int)st.w : -1;
#pragma unroll
            for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    R[j][e] = greedy ? (tok_index(j, e) == top ? 1.0f : 0.0f) : exp_fast(R[j][e] * inv_tt - st.z) * it;
        };
        if (!leaf) {
            // ---- first child: two logits and the row statistics decide
            {
                const int y = l_token[c];
                float d = 0.0f, r = 0.0f;
                if (y >= 0) {
                    d = exp_fast(logit_to_float(draft_logits[(size_t)(base + cur) * V + y]) * inv_td - st.x) / st.y;
                    r = greedy ? ((float)y == st.w ? 1.0f : 0.0f)
                               : exp_fast(logit_to_float(target_logits[(size_t)(base + cur) * V + y]) * inv_tt - st.z) / st.w;
                }
                const float ratio = ratio_of(d, r);
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
                __syncthreads();                              // D_lds is complete
                uint32_t rank = 0;
                for (int guard = 0; c >= 0 && guard < N; ++guard) {
                    const int y = l_token[c];
                    const float dy = y >= 0 ? D_lds[y] : 0.0f;        // the same word for every thread
                    if (rank > 0) {
                        // ratio seen by this child after its earlier siblings were rejected: R[y] sits in one
                        // thread's registers
                        if (y >= 0 && ((y % kSeg) >> 2) == tid) {
#pragma unroll
                            for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (j == y / kSeg && e == (y & 3)) sh.bcast[1] = R[j][e];
                        }
                        if (y < 0 && tid == 0) sh.bcast[1] = 0.0f;
                        __syncthreads();
                        const float ratio = ratio_of(dy * scale_d, sh.bcast[1]);
                        const uint2 pk_n = child_key(seed, pk, rank);
                        const float u = u01(seed, pk_n, 0u, KIND_ACCEPT);
                        margin = fminf(margin, fabsf(u - ratio));
                        if (tid == 0) accept_ratio[base + c] = ratio;
                        if (u < ratio) { next = c; pk_next = pk_n; break; }
                    }
                    // reject child c: R <- norm(max(R-D,0)) with D as it stands, then y leaves D
                    float res[2] = { 0.0f, 0.0f };          // mass of relu(R-D); weight in D_lds
#pragma unroll
                    for (int j = 0; j < kMaxSeg; ++j) {
                        const int i0 = tok_index(j, 0);
                        if (i0 < V) {
                            const float4 dv = *reinterpret_cast<const float4*>(D_lds + i0);
                            res[0] += fmaxf(fmaf(-scale_d, dv.x, R[j][0]), 0.0f) + fmaxf(fmaf(-scale_d, dv.y, R[j][1]), 0.0f);
                            res[0] += fmaxf(fmaf(-scale_d, dv.z, R[j][2]), 0.0f) + fmaxf(fmaf(-scale_d, dv.w, R[j][3]), 0.0f);
                            res[1] += (dv.x + dv.y) + (dv.z + dv.w);
                        }
                    }
                    block_sum<float, 2>(res, sh.fred);
                    if (res[0] > 0.0f) {                     // else R == D: keep R (no reject can reach here)
                        const float ir = 1.0f / res[0];
#pragma unroll
                        for (int j = 0; j < kMaxSeg; ++j) {
                            const int i0 = tok_index(j, 0);
                            if (i0 < V) {
                                const float4 dv = *reinterpret_cast<const float4*>(D_lds + i0);
                                R[j][0] = fmaxf(fmaf(-scale_d, dv.x, R[j][0]), 0.0f) * ir;
                                R[j][1] = fmaxf(fmaf(-scale_d, dv.y, R[j][1]), 0.0f) * ir;
                                R[j][2] = fmaxf(fmaf(-scale_d, dv.z, R[j][2]), 0.0f) * ir;
                                R[j][3] = fmaxf(fmaf(-scale_d, dv.w, R[j][3]), 0.0f) * ir;
                            }
                        }
                    }
                    __syncthreads();                          // every thread has read D_lds as it stood
                    if (tid == 0 && y >= 0) D_lds[y] = 0.0f;  // y leaves D
                    const float left = res[1] - dy;           // weight left in D
                    c = l_next[c];
                    ++rank;
                    if (!(left > 0.0f)) {                     // D is empty: later children are not tried
                        if (tid == 0)
                            for (int k = 0, cc = c; cc >= 0 && k < N; ++k, cc = l_next[cc])
                                accept_ratio[base + cc] = -1.0f;
                        break;
                    }
                    scale_d = 1.0f / left;                    // D <- norm(D), kept as a factor
                    __syncthreads();                          // the removal is visible before D_lds is read again
                }
            }
        }
        if (next >= 0) {
            if (tid == 0) accepted_nodes[base + na] = next;
            ++na;
            cur = next; pk = pk_next;
            __syncthreads();                                  // D_lds and the scratch are free for the next node
            continue;
        }
        // ---- the walk stops at cur: emit a token from what is left of the target row
        if (leaf && !emit_bonus) { fin = -1; break; }
        if (!rows_loaded) load_rows(false);
        __syncthreads();
        const double u = (double)u01(seed, pk, 0u, KIND_RESID);
        fin = draw_from_row(R, u, &sh.draw, reinterpret_cast<double*>(dyn));     // the draft row's place in LDS is free now
        break;
    }
    if (tid == 0) {
        n_accepted[seq] = na;
        final_token[seq] = fin;
        min_margin[seq] = margin;
    }
}

// the walk keeps a draft row and the tree links in dynamic LDS: raised to the largest once
hipError_t prepare_verify()
{
    static std::atomic<unsigned long long> done[4] = { {0}, {0}, {0}, {0} };
    const int bytes = (int)walk_lds_bytes(DYSPEC_MAX_VOCAB, DYSPEC_MAX_NODES);
    hipError_t e = raise_dynamic_lds_once(reinterpret_cast<const void*>(&verify_walk_kernel<true, float>), bytes, done[0]);
    if (e == hipSuccess) e = raise_dynamic_lds_once(reinterpret_cast<const void*>(&verify_walk_kernel<false, float>), bytes, done[1]);
    if (e == hipSuccess) e = raise_dynamic_lds_once(reinterpret_cast<const void*>(&verify_walk_kernel<true, __bf16>), bytes, done[2]);
    if (e == hipSuccess) e = raise_dynamic_lds_once(reinterpret_cast<const void*>(&verify_walk_kernel<false, __bf16>), bytes, done[3]);
    return e;
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
    int widest = 1;
    for (int s = 0; s < sa.n_seq; ++s) widest = max(widest, sa.node_off[s + 1] - sa.node_off[s]);
    const size_t dyn = walk_lds_bytes(V, widest);
    const hipError_t ep = prepare_verify();
    if (ep != hipSuccess) return ep;
    if (V % 4 == 0)
        verify_walk_kernel<true, T><<<sa.n_seq, kBlock, dyn, stream>>>(draft_logits, target_logits, V, sa, tree, seed, emit_bonus,
                                                                       row_stats, accept_ratio, accepted_nodes, n_accepted,
                                                                       final_token, min_margin);
    else
        verify_walk_kernel<false, T><<<sa.n_seq, kBlock, dyn, stream>>>(draft_logits, target_logits, V, sa, tree, seed, emit_bonus,
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
