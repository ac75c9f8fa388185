// Tree attention (Section 2, "Tree Attention"; Appendix C) for gfx950.
//
// Two kernels:
//  * tree_attn_mfma_kernel: bf16, head_dim 64/128, matrix cores.  All G = Hq/Hkv query
//    heads of a KV head are folded into the row dimension (row = node*G + head), so the
//    prefix K/V stream of a KV head is read once per 128-row tile and every byte feeds
//    128 rows of MFMA work.  The tree part reuses the same tiles with the ancestor
//    bitmask applied to the score registers; 64-key tree tiles no row of the wave can see
//    are skipped (the paper's kernel skips empty 32x32 blocks of the mask).
//  * tree_attn_simple_kernel: one wavefront per (row, head), any head_dim <= 256, fp32 or
//    bf16 storage with fp32 arithmetic.  Used for fp32 tensors.
#include "dyspec_device.h"

namespace dyspec {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// =====================================================================================
// Matrix-core kernel
// =====================================================================================
//
// Workgroup = 4 waves = one tile of 128 rows of one (sequence, KV head).  Wave w owns the
// 64-row half (w & 1) and every second 64-key tile ((w >> 1) picks even or odd tiles); the
// two waves of a row half merge their (max, sum, accumulator) through LDS at the end.
// Per 64-key tile a wave computes S^T = K Q^T (keys x queries, so that each lane holds one
// query column and P = exp(S^T) is already in the register layout the second product wants
// as its B operand), the online softmax, and O^T += V^T P^T.  A key tile staged in LDS is
// read by two waves, a Q fragment stays in registers for the whole kernel.

constexpr int kRowsPerWG = 128;
constexpr int kKeysPerTile = 64;
constexpr int kAttnThreads = 256;

template <int D> struct AttnLds {
    static constexpr int kStrideK = D + 8;       // bf16 per K row in LDS: 16-byte reads of 32 rows hit all banks
    static constexpr int kStrideV = D + 16;      // bf16 per V row: rows 4 apart land 32 banks apart
    static constexpr int kTileElems = kKeysPerTile * (kStrideK + kStrideV);
    static constexpr int kStageElems = 2 * kTileElems;   // an even and an odd tile per pipeline stage
    static constexpr int kBytes = 2 * kStageElems * 2;   // two stages
};

__device__ __forceinline__ uint32_t pack_lo(uint32_t w0, uint32_t w1) { return __builtin_amdgcn_perm(w1, w0, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t w0, uint32_t w1) { return __builtin_amdgcn_perm(w1, w0, 0x07060302u); }

template <int D>
__global__ __launch_bounds__(kAttnThreads) void tree_attn_mfma_kernel(AttnArgs a, SeqArgs sa)
{
    using L = AttnLds<D>;
    constexpr int KK = D / 16;                   // k-steps of the QK^T product
    constexpr int DG = D / 64;                   // 64-wide groups of the head dimension
    constexpr int CH = D / 8;                    // 16-byte chunks per K/V row
    constexpr int RPP = kAttnThreads / CH;       // rows staged per pass of the workgroup
    constexpr int NPASS = kKeysPerTile / RPP;    // passes per matrix
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    __bf16* lds = reinterpret_cast<__bf16*>(lds_raw);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, g = lane >> 5;
    const int wq = wave & 1, wk = wave >> 1;

    // ---- which tile
    const int kvh = blockIdx.x % a.Hkv;
    const int tile = blockIdx.x / a.Hkv;
    int seq = 0;
    while (seq + 1 < sa.n_seq && tile >= a.tile_off[seq + 1]) ++seq;
    const int node_base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - node_base;
    const int P = sa.prefix_len[seq];
    const long long kv_base = sa.kv_off[seq];
    const int G = a.Hq / a.Hkv;
    const int rows = G * N;
    const int r0 = (tile - a.tile_off[seq]) * kRowsPerWG;

    const int nTp = (P + kKeysPerTile - 1) / kKeysPerTile;
    const int r_last = min(rows - 1, r0 + kRowsPerWG - 1);
    const int nTt = (r_last / G) / kKeysPerTile + 1;      // tree tiles up to the largest node of this row tile
    const int nT = nTp + nTt;
    const int nIt = (nT + 1) / 2;

    const __bf16* kp = static_cast<const __bf16*>(a.kp);
    const __bf16* vp = static_cast<const __bf16*>(a.vp);
    const __bf16* kt = static_cast<const __bf16*>(a.kt);
    const __bf16* vt = static_cast<const __bf16*>(a.vt);
    const size_t kv_row = (size_t)a.Hkv * D;

    // ---- Q fragments (B operand: lane holds query n, head-dim slice 16*kk + 8*g .. +7)
    bf16x8 qf[2][KK];
    int rq[2];
    const uint64_t* mrow[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int r = r0 + 64 * wq + 32 * qb + n;
        rq[qb] = r;
        const int rc = min(r, rows - 1);
        const int j = rc / G, h = kvh * G + rc % G;
        const __bf16* qrow = static_cast<const __bf16*>(a.q) + ((size_t)(node_base + j) * a.Hq + h) * D;
        mrow[qb] = a.mask + (size_t)(node_base + j) * a.mask_words;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            qf[qb][kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * g);
    }

    floatx16 acc[DG][2][2];                      // [d group][even/odd d][query block]
#pragma unroll
    for (int dg = 0; dg < DG; ++dg)
#pragma unroll
        for (int par = 0; par < 2; ++par)
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[dg][par][qb][i] = 0.0f;
    float m_run[2] = { -1e30f, -1e30f }, l_run[2] = { 0.0f, 0.0f };
    const float c2 = a.scale * 1.4426950408889634f;     // scores are used as exp2(c2 * s)

    // ---- staging: thread copies chunk (tid % CH) of rows (tid / CH + RPP*i)
    const int s_chunk = tid % CH, s_row = tid / CH;
    uint4 stage[4][NPASS];
    auto load_stage = [&](int it) {
#pragma unroll
        for (int mm = 0; mm < 4; ++mm) {
            const int t = 2 * it + (mm >> 1);
            const bool isV = mm & 1;
#pragma unroll
            for (int i = 0; i < NPASS; ++i) {
                const int row = s_row + RPP * i;
                const __bf16* src = nullptr;
                if (t < nTp) {
                    const int key = t * kKeysPerTile + row;
                    if (key < P) src = (isV ? vp : kp) + ((size_t)(kv_base + key)) * kv_row + (size_t)kvh * D;
                } else if (t < nT) {
                    const int key = (t - nTp) * kKeysPerTile + row;
                    if (key < N) src = (isV ? vt : kt) + ((size_t)(node_base + key)) * kv_row + (size_t)kvh * D;
                }
                stage[mm][i] = src ? *reinterpret_cast<const uint4*>(src + 8 * s_chunk) : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_stage = [&](int buf) {
        __bf16* base = lds + buf * L::kStageElems;
#pragma unroll
        for (int mm = 0; mm < 4; ++mm) {
            __bf16* tb = base + (mm >> 1) * L::kTileElems + ((mm & 1) ? kKeysPerTile * L::kStrideK : 0);
            const int stride = (mm & 1) ? L::kStrideV : L::kStrideK;
#pragma unroll
            for (int i = 0; i < NPASS; ++i)
                *reinterpret_cast<uint4*>(tb + (s_row + RPP * i) * stride + 8 * s_chunk) = stage[mm][i];
        }
    };

    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int it = 0; it < nIt; ++it) {
        if (it + 1 < nIt) load_stage(it + 1);

        const int t = 2 * it + wk;
        if (t < nT) {
            // ---- visibility of this tile's 64 keys for the lane's two queries
            uint64_t vis[2] = { ~0ull, ~0ull };
            bool need_mask = false;
            if (t >= nTp) {
                vis[0] = mrow[0][t - nTp];
                vis[1] = mrow[1][t - nTp];
                need_mask = true;
            } else if ((t + 1) * kKeysPerTile > P) {
                const int live = P - t * kKeysPerTile;              // 1..63
                vis[0] = vis[1] = (1ull << live) - 1ull;
                need_mask = true;
            }
            if (__any((vis[0] | vis[1]) != 0ull)) {
                const __bf16* Ks = lds + (it & 1) * L::kStageElems + wk * L::kTileElems;
                const __bf16* Vs = Ks + kKeysPerTile * L::kStrideK;

                // ---- S^T = K Q^T : [key block a][query block qb]
                floatx16 S[2][2];
#pragma unroll
                for (int ka = 0; ka < 2; ++ka)
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) S[ka][qb][i] = 0.0f;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    bf16x8 kf[2];
#pragma unroll
                    for (int ka = 0; ka < 2; ++ka)
                        kf[ka] = *reinterpret_cast<const bf16x8*>(Ks + (32 * ka + n) * L::kStrideK + 16 * kk + 8 * g);
#pragma unroll
                    for (int ka = 0; ka < 2; ++ka)
#pragma unroll
                        for (int qb = 0; qb < 2; ++qb)
                            S[ka][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ka], qf[qb][kk], S[ka][qb], 0, 0, 0);
                }

                // ---- mask + online softmax.  Register i of a 32x32 block holds key row
                //      8*(i/4) + 4*g + i%4 of the block, query column n.
                bf16x8 pb[2][2][2];                   // [query block][key block][16-key step]
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    if (need_mask) {
#pragma unroll
                        for (int ka = 0; ka < 2; ++ka) {
                            const uint32_t v32 = (uint32_t)(vis[qb] >> (32 * ka + 4 * g));
#pragma unroll
                            for (int i = 0; i < 16; ++i)
                                if (!((v32 >> (8 * (i / 4) + (i % 4))) & 1u)) S[ka][qb][i] = -INFINITY;
                        }
                    }
                    float mx = -INFINITY;
#pragma unroll
                    for (int ka = 0; ka < 2; ++ka)
#pragma unroll
                        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[ka][qb][i]);
                    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
                    if (__any(mx > m_run[qb])) {
                        const float m_new = fmaxf(m_run[qb], mx);
                        const float alpha = exp2f((m_run[qb] - m_new) * c2);
                        m_run[qb] = m_new;
                        l_run[qb] *= alpha;
#pragma unroll
                        for (int dg = 0; dg < DG; ++dg)
#pragma unroll
                            for (int par = 0; par < 2; ++par)
#pragma unroll
                                for (int i = 0; i < 16; ++i) acc[dg][par][qb][i] *= alpha;
                    }
                    const float mc = m_run[qb] * c2;
                    float ls = 0.0f;
#pragma unroll
                    for (int ka = 0; ka < 2; ++ka)
#pragma unroll
                        for (int i = 0; i < 16; i += 2) {
                            const float p0 = exp2f(fmaf(S[ka][qb][i], c2, -mc));
                            const float p1 = exp2f(fmaf(S[ka][qb][i + 1], c2, -mc));
                            ls += p0 + p1;
                            floatx2 pp = { p0, p1 };
                            const bf16x2 pc = __builtin_convertvector(pp, bf16x2);
                            pb[qb][ka][i / 8][i % 8] = pc[0];
                            pb[qb][ka][i / 8][i % 8 + 1] = pc[1];
                        }
                    l_run[qb] += ls;
                }

                // ---- O^T += V^T P^T.  k-slot (g, e) of step (ka, ts) is key
                //      32*ka + 8*(2*ts + e/4) + 4*g + e%4, as in the P registers.
#pragma unroll
                for (int ka = 0; ka < 2; ++ka)
#pragma unroll
                    for (int ts = 0; ts < 2; ++ts) {
#pragma unroll
                        for (int dg = 0; dg < DG; ++dg) {
                            uint32_t w[8];
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                const int key = 32 * ka + 8 * (2 * ts + e / 4) + 4 * g + e % 4;
                                w[e] = *reinterpret_cast<const uint32_t*>(Vs + key * L::kStrideV + 64 * dg + 2 * n);
                            }
                            union { uint32_t u[4]; bf16x8 v; } fe, fo;
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                fe.u[j] = pack_lo(w[2 * j], w[2 * j + 1]);
                                fo.u[j] = pack_hi(w[2 * j], w[2 * j + 1]);
                            }
#pragma unroll
                            for (int qb = 0; qb < 2; ++qb) {
                                acc[dg][0][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fe.v, pb[qb][ka][ts], acc[dg][0][qb], 0, 0, 0);
                                acc[dg][1][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo.v, pb[qb][ka][ts], acc[dg][1][qb], 0, 0, 0);
                            }
                        }
                    }
            }
        }

        if (it + 1 < nIt) store_stage((it + 1) & 1);
        __syncthreads();
    }

    // ---- merge the two key halves of each row half through LDS, normalise, store
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) l_run[qb] += __shfl_xor(l_run[qb], 32, kWave);
    float* xs = reinterpret_cast<float*>(lds_raw);           // [wq][register][lane]
    constexpr int NR = DG * 2 * 2 * 16 + 4;
    if (wk == 1) {
        float* dst = xs + (size_t)wq * NR * kWave + lane;
        int r = 0;
#pragma unroll
        for (int dg = 0; dg < DG; ++dg)
#pragma unroll
            for (int par = 0; par < 2; ++par)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) dst[(r++) * kWave] = acc[dg][par][qb][i];
        dst[(r++) * kWave] = m_run[0]; dst[(r++) * kWave] = m_run[1];
        dst[(r++) * kWave] = l_run[0]; dst[(r++) * kWave] = l_run[1];
    }
    __syncthreads();
    if (wk == 0) {
        const float* src = xs + (size_t)wq * NR * kWave + lane;
        float f0[2], f1[2], inv[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float m1 = src[(NR - 4 + qb) * kWave], l1 = src[(NR - 2 + qb) * kWave];
            const float m = fmaxf(m_run[qb], m1);
            f0[qb] = exp2f((m_run[qb] - m) * c2);
            f1[qb] = exp2f((m1 - m) * c2);
            inv[qb] = 1.0f / (l_run[qb] * f0[qb] + l1 * f1[qb]);
        }
        int r = 0;
#pragma unroll
        for (int dg = 0; dg < DG; ++dg)
#pragma unroll
            for (int par = 0; par < 2; ++par)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float o1 = src[(r++) * kWave];
                        acc[dg][par][qb][i] = (acc[dg][par][qb][i] * f0[qb] + o1 * f1[qb]) * inv[qb];
                    }
        // register i of block (dg, par) is head-dim index 64*dg + 2*(8*(i/4) + 4*g + i%4) + par
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (rq[qb] >= rows) continue;
            const int j = rq[qb] / G, h = kvh * G + rq[qb] % G;
            __bf16* orow = static_cast<__bf16*>(a.out) + ((size_t)(node_base + j) * a.Hq + h) * D;
#pragma unroll
            for (int dg = 0; dg < DG; ++dg)
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    union { bf16x2 p[4]; uint4 v; } o;
#pragma unroll
                    for (int ii = 0; ii < 4; ++ii) {
                        floatx2 pr = { acc[dg][0][qb][4 * ib + ii], acc[dg][1][qb][4 * ib + ii] };
                        o.p[ii] = __builtin_convertvector(pr, bf16x2);
                    }
                    *reinterpret_cast<uint4*>(orow + 64 * dg + 2 * (8 * ib + 4 * g)) = o.v;
                }
        }
    }
}

// =====================================================================================
// Simple kernel: one wavefront per (row, head); plain online softmax in fp32.
// =====================================================================================

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<__bf16>(__bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ __bf16 from_f32<__bf16>(float v) { return (__bf16)v; }

constexpr int kSimpleWaves = 4;
constexpr int kSimpleMaxD = 256;

template <typename T>
__global__ __launch_bounds__(kSimpleWaves* kWave) void tree_attn_simple_kernel(AttnArgs a, SeqArgs sa, int total_rows)
{
    __shared__ float q_s[kSimpleWaves][kSimpleMaxD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    long long wid = (long long)blockIdx.x * kSimpleWaves + wave;
    const bool active = wid < (long long)total_rows * a.Hq;
    if (!active) wid = 0;                                     // idle waves still reach the barrier
    const int row = (int)(wid / a.Hq), h = (int)(wid % a.Hq);
    const int seq = find_seq(sa, row);
    const int node_base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - node_base, P = sa.prefix_len[seq];
    const int d = a.d;
    const int kvh = h / (a.Hq / a.Hkv);
    const size_t kv_row = (size_t)a.Hkv * d;
    const T* kp = static_cast<const T*>(a.kp) + (size_t)sa.kv_off[seq] * kv_row + (size_t)kvh * d;
    const T* vp = static_cast<const T*>(a.vp) + (size_t)sa.kv_off[seq] * kv_row + (size_t)kvh * d;
    const T* kt = static_cast<const T*>(a.kt) + (size_t)node_base * kv_row + (size_t)kvh * d;
    const T* vt = static_cast<const T*>(a.vt) + (size_t)node_base * kv_row + (size_t)kvh * d;
    const T* qrow = static_cast<const T*>(a.q) + ((size_t)row * a.Hq + h) * d;
    const uint64_t* mrow = a.mask + (size_t)row * a.mask_words;

    for (int c = lane; c < d; c += kWave) q_s[wave][c] = to_f32<T>(qrow[c]);
    __syncthreads();
    if (!active) return;

    float acc[kSimpleMaxD / kWave] = { 0.f, 0.f, 0.f, 0.f };
    float m = -INFINITY, l = 0.0f;
    for (int k0 = 0; k0 < P + N; k0 += kWave) {
        const int k = k0 + lane;
        bool visible = false;
        const T* krow = nullptr;
        if (k < P) { visible = true; krow = kp + (size_t)k * kv_row; }
        else if (k < P + N) {
            const int i = k - P;
            visible = (mrow[i >> 6] >> (i & 63)) & 1ull;
            krow = kt + (size_t)i * kv_row;
        }
        float s = -INFINITY;
        if (visible) {
            float dot = 0.0f;
            for (int c = 0; c < d; ++c) dot = fmaf(q_s[wave][c], to_f32<T>(krow[c]), dot);
            s = dot * a.scale;
        }
        const float m_new = fmaxf(m, wave_max(s));
        if (m_new == -INFINITY) continue;                    // nothing visible so far
        const float p = visible ? expf(s - m_new) : 0.0f;
        const float corr = expf(m - m_new);                  // exp(-inf) = 0 on the first chunk
        l = l * corr + wave_sum(p);
        m = m_new;
#pragma unroll
        for (int i = 0; i < kSimpleMaxD / kWave; ++i) acc[i] *= corr;
        for (int tkey = 0; tkey < kWave; ++tkey) {
            const float pt = __shfl(p, tkey, kWave);
            if (pt == 0.0f) continue;                        // wave-uniform: also skips keys past the end
            const int kk = k0 + tkey;
            const T* vrow = (kk < P) ? vp + (size_t)kk * kv_row : vt + (size_t)(kk - P) * kv_row;
#pragma unroll
            for (int i = 0; i < kSimpleMaxD / kWave; ++i) {
                const int c = lane + kWave * i;
                if (c < d) acc[i] = fmaf(pt, to_f32<T>(vrow[c]), acc[i]);
            }
        }
    }
    T* orow = static_cast<T*>(a.out) + ((size_t)row * a.Hq + h) * d;
    const float inv = 1.0f / l;
#pragma unroll
    for (int i = 0; i < kSimpleMaxD / kWave; ++i) {
        const int c = lane + kWave * i;
        if (c < d) orow[c] = from_f32<T>(acc[i] * inv);
    }
}

hipError_t launch_tree_attn(AttnArgs a, const SeqArgs& sa, int dtype, bool force_simple, hipStream_t stream)
{
    const int total_rows = sa.node_off[sa.n_seq];
    const int G = a.Hq / a.Hkv;
    if (dtype == DYSPEC_BF16 && !force_simple && (a.d == 128 || a.d == 64)) {
        int tiles = 0;
        for (int s = 0; s < sa.n_seq; ++s) {
            a.tile_off[s] = tiles;
            tiles += (G * (sa.node_off[s + 1] - sa.node_off[s]) + kRowsPerWG - 1) / kRowsPerWG;
        }
        a.tile_off[sa.n_seq] = tiles;
        if (tiles == 0) return hipSuccess;
        if (a.d == 128) {
            static bool attr_set = false;
            if (!attr_set) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tree_attn_mfma_kernel<128>),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, AttnLds<128>::kBytes);
                if (e != hipSuccess) return e;
                attr_set = true;
            }
            tree_attn_mfma_kernel<128><<<tiles * a.Hkv, kAttnThreads, AttnLds<128>::kBytes, stream>>>(a, sa);
        } else {
            static bool attr_set = false;
            if (!attr_set) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tree_attn_mfma_kernel<64>),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, AttnLds<64>::kBytes);
                if (e != hipSuccess) return e;
                attr_set = true;
            }
            tree_attn_mfma_kernel<64><<<tiles * a.Hkv, kAttnThreads, AttnLds<64>::kBytes, stream>>>(a, sa);
        }
        return hipGetLastError();
    }
    if (total_rows == 0) return hipSuccess;
    const long long waves = (long long)total_rows * a.Hq;
    const int blocks = (int)((waves + kSimpleWaves - 1) / kSimpleWaves);
    if (dtype == DYSPEC_BF16)
        tree_attn_simple_kernel<__bf16><<<blocks, kSimpleWaves * kWave, 0, stream>>>(a, sa, total_rows);
    else
        tree_attn_simple_kernel<float><<<blocks, kSimpleWaves * kWave, 0, stream>>>(a, sa, total_rows);
    return hipGetLastError();
}

}  // namespace dyspec
