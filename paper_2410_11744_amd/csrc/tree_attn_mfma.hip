// Tree attention on the matrix cores (Section 2, "Tree Attention"; Appendix C) for gfx950:
// bf16 tensors, head_dim 64 or 128, fp32 accumulation.
//
// Row folding.  All G = Hq/Hkv query heads that share a KV head are folded into the row
// dimension (row = node*G + head), so a workgroup tile of 128 rows streams the prefix K/V
// of its KV head once and every K/V byte feeds 128 rows of MFMA work; the tree part reuses
// the same machinery with the ancestor bitmask applied to the score registers, and 64-key
// tree tiles that no row of the wave can see are skipped (the paper's kernel skips empty
// 32x32 blocks of the mask).
//
// Workgroup = 4 waves, one per SIMD.  Wave w owns the 64-row half (w & 1) and every second
// 64-key tile ((w >> 1) picks even or odd tiles); the two waves of a row half merge their
// (max, sum, accumulator) through LDS at the end.  Per 32-key block a wave computes
// S^T = K Q^T (keys x queries: each lane then holds one query column, and exp(S^T) is
// already in the register layout the second product wants as its B operand), the online
// softmax, and O^T += V^T P^T.  The reference maximum of the softmax is raised lazily (only
// when a score would push exp2 past 2^kLazy), so the accumulators are rescaled a handful of
// times per row instead of once per block.
//
// Staging.  K/V tiles go from HBM/L2 to LDS with direct loads (global_load_lds_dwordx4: lane
// i of a wave writes LDS bytes [16*i, 16*i+16) past a wave-uniform base), double buffered,
// without passing through registers; the loads of the next stage are in flight while the
// current one is consumed.  Rows sit unpadded in LDS; 16-byte chunks of a row are
// XOR-swizzled so that the 16-byte K reads and the 4-byte V reads of a wave spread over all
// 64 banks.
#include <utility>

#include "dyspec_device.h"

namespace dyspec {

// Compile-time loop: f(integral_constant<int, 0>), ..., f(integral_constant<int, N-1>).
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(1))) const void* global_ptr;
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v* lds_short4;

constexpr int kRowsPerWG = 128;
constexpr int kKeysPerTile = 64;
#ifndef DYSPEC_ATTN_QB
#define DYSPEC_ATTN_QB 1
#endif
constexpr int kQB = DYSPEC_ATTN_QB;   // 32-row query blocks per wave (see the kernel)
constexpr float kLazy = 8.0f;        // accumulators are rescaled only when exp2 would pass 2^kLazy

// v_exp_f32 without the denormal-range fix-up: inputs below -126 give 0, which is what the
// softmax wants.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// One wave-wide direct load: lane i moves 16 bytes from (base + voff_i) to LDS byte
// lds_base + 16*i.  Issued as inline assembly so that the compiler does not pair every later
// LDS read with a wait for these loads; the caller waits (wait_direct_loads) before the
// barrier that publishes the stage.
__device__ __forceinline__ void direct_load_16(const void* base, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(voff), "s"(base) : "m0", "memory");
}
__device__ __forceinline__ void wait_direct_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return (uint32_t)(size_t)(lds_ptr)(p);
}

// max of three without the NaN-quieting moves fmaxf would add in front
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

template <int D> struct Geo {
    static constexpr int kRowBytes = 2 * D;
    static constexpr int kChunks = D / 8;                        // 16-byte chunks per row
    static constexpr int kRowsPerLoad = 1024 / kRowBytes;        // rows one wave-wide direct load covers
    static constexpr int kMatBytes = kKeysPerTile * kRowBytes;   // one K or V tile
    static constexpr int kStageBytes = 4 * kMatBytes;            // K,V of the even tile, K,V of the odd tile
    static constexpr int kLdsBytes = 2 * kStageBytes;
    static constexpr int kLoadsPerMat = kKeysPerTile / kRowsPerLoad;
    // chunk c of K row r sits at chunk position c ^ swz_k(r); of V row r at c ^ swz_v(r)
    __device__ static __forceinline__ int swz_k(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
    __device__ static __forceinline__ int swz_v(int r) { return D == 128 ? ((r & 3) << 2) : 0; }
};

// QB = 32-row query blocks per wave.  QB = 2: 4 waves, one per SIMD, 512 registers each.
// QB = 1: 8 waves, two per SIMD with 256 registers each, so the matrix work of one wave hides
// behind the vector work of the other; every K/V byte is then read from LDS by four waves.
template <int D, int QB>
__global__ __launch_bounds__(64 * 2 * (4 / QB)) void tree_attn_mfma_kernel(AttnArgs a, SeqArgs sa)
{
    using L = Geo<D>;
    constexpr int NWQ = 4 / QB;                  // waves along the row dimension
    constexpr int NW = 2 * NWQ;                  // waves per workgroup
    constexpr int KK = D / 16;                   // k-steps of the QK^T product
    constexpr int DB = D / 32;                   // 32-wide blocks of the head dimension
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, g = lane >> 5;
    const int wq = wave % NWQ, wk = wave / NWQ;

    // ---- which tile
    const int kvh = blockIdx.x % a.Hkv;
    const int tile = blockIdx.x / a.Hkv;
    int seq = 0;
    while (seq + 1 < sa.n_seq && tile >= a.tile_off[seq + 1]) ++seq;
    const int node_base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - node_base;
    const int P = sa.prefix_len[seq];
    const int G = a.Hq / a.Hkv;
    const int rows = G * N;
    const int r0 = (tile - a.tile_off[seq]) * kRowsPerWG;

    const int nTp = (P + kKeysPerTile - 1) / kKeysPerTile;
    const int r_last = min(rows - 1, r0 + kRowsPerWG - 1);
    const int nTt = (r_last / G) / kKeysPerTile + 1;      // tree tiles up to the largest node of this row tile
    const int nT = nTp + nTt;
    const int nIt = (nT + 1) / 2;

    const size_t kv_row_bytes = (size_t)a.Hkv * D * 2;
    const char* kp = static_cast<const char*>(a.kp) + (size_t)sa.kv_off[seq] * kv_row_bytes + (size_t)kvh * D * 2;
    const char* vp = static_cast<const char*>(a.vp) + (size_t)sa.kv_off[seq] * kv_row_bytes + (size_t)kvh * D * 2;
    const char* kt = static_cast<const char*>(a.kt) + (size_t)node_base * kv_row_bytes + (size_t)kvh * D * 2;
    const char* vt = static_cast<const char*>(a.vt) + (size_t)node_base * kv_row_bytes + (size_t)kvh * D * 2;

    // ---- Q fragments (B operand: lane holds query n, head-dim slice 16*kk + 8*g .. +7)
    bf16x8 qf[QB][KK];
    int rq[QB];
    const uint64_t* mrow[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int r = r0 + 32 * QB * wq + 32 * qb + n;
        rq[qb] = r;
        const int rc = min(r, rows - 1);
        const int j = rc / G, h = kvh * G + rc % G;
        const __bf16* qrow = static_cast<const __bf16*>(a.q) + ((size_t)(node_base + j) * a.Hq + h) * D;
        mrow[qb] = a.mask + (size_t)(node_base + j) * a.mask_words;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            qf[qb][kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * g);
    }

    floatx16 acc[DB][QB];                        // O^T: [32-wide head-dim block][query block]
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[db][qb][i] = 0.0f;
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -1e30f; l_run[qb] = 0.0f; }
    const float c2 = a.scale * 1.4426950408889634f;     // scores are used as exp2(c2 * s)

    // ---- direct-load plan: a stage holds four matrices (0: K of the even tile, 1: V of the
    //      even tile, 2: K odd, 3: V odd) of kLoadsPerMat wave-wide loads each; wave w fills
    //      loads [LPW*part, LPW*part + LPW) of matrix w / (NW/4).  Lane i of load x writes row
    //      position R = kRowsPerLoad*x + i/kChunks, chunk position i % kChunks, so it must fetch
    //      chunk (i % kChunks) ^ swz(R) of that key row; with these swizzles the lane's byte
    //      offset depends on x mod 4 only.
    constexpr int LPW = L::kLoadsPerMat / (NW / 4);
    const int ld_mm = wave / (NW / 4), ld_x0 = (wave % (NW / 4)) * LPW;
    const bool ld_is_v = ld_mm & 1;
    const int ld_lrow = lane / L::kChunks, ld_cpos = lane % L::kChunks;
    int ld_voff[4];                               // byte offset of the lane's chunk for x mod 4
#pragma unroll
    for (int xm = 0; xm < 4; ++xm) {
        const int row = L::kRowsPerLoad * xm + ld_lrow;
        const int c = ld_cpos ^ (ld_is_v ? L::swz_v(row) : L::swz_k(row));
        ld_voff[xm] = ld_lrow * (int)kv_row_bytes + 16 * c;
    }
    const char* const st_prefix = ld_is_v ? vp : kp;
    const char* const st_tree = ld_is_v ? vt : kt;
    unsigned char* const st_dst = lds + ld_mm * L::kMatBytes + ld_x0 * 1024;
    // (captures by value: a conditional between variables captured by reference would be a
    //  conditional between addresses and force them into scratch memory)
    auto issue_stage = [=](int it) {
        const int t = 2 * it + (ld_mm >> 1);                     // the tile this wave stages
        if (t >= nT) return;                                     // odd tile past the end: nobody reads it
        unsigned char* dst0 = st_dst + (it & 1) * L::kStageBytes;
        const bool prefix = t < nTp;
        const char* region = prefix ? st_prefix : st_tree;
        const int key0 = (prefix ? t : t - nTp) * kKeysPerTile;
        const int limit = prefix ? P : N;
        if (key0 + kKeysPerTile <= limit) {                      // whole tile in range: uniform base + lane offset
            const char* base = region + (size_t)(key0 + L::kRowsPerLoad * ld_x0) * kv_row_bytes;
            static_for<LPW>([=](auto xc) {
                constexpr int x = decltype(xc)::value;
                direct_load_16(base + (size_t)(L::kRowsPerLoad * x) * kv_row_bytes, (uint32_t)ld_voff[x & 3],
                               lds_address(dst0) + x * 1024);
            });
        } else {
            // rows past the end read row 0 of the region (a key every query may see, so its
            // values are as finite as the result itself); their scores are masked out
            static_for<LPW>([=](auto xc) {
                constexpr int x = decltype(xc)::value;
                const int rowx = L::kRowsPerLoad * (ld_x0 + x);
                const int key = key0 + rowx + ld_lrow;
                const uint32_t off = (key < limit) ? (uint32_t)(key0 + rowx) * (uint32_t)kv_row_bytes + (uint32_t)ld_voff[x & 3]
                                                   : (uint32_t)(ld_voff[x & 3] - ld_lrow * (int)kv_row_bytes);
                direct_load_16(region, off, lds_address(dst0) + x * 1024);
            });
        }
    };

    // ---- LDS read offsets of this lane
    int k_off[KK];                               // K fragment of k-step kk, key row n (+32*ka rows)
    {
        const int h = g ^ L::swz_k(n);           // (2*kk + g) ^ swz == (2*kk) ^ (g ^ swz)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) k_off[kk] = n * L::kRowBytes + (((2 * kk) ^ h) << 4);
    }
    // V^T fragments come from the LDS transpose read (ds_read_b64_tr_b16).  Measured lane
    // layout of that instruction, per group of 16 lanes: lane i supplies the address of four
    // consecutive 16-bit elements M_i[0..3] and receives { M_{4j + i/4}[i % 4] : j = 0..3 }.
    // So lanes s = 4j + r of a group point at key row (base + j), columns 4r..4r+3 of a
    // 16-column slab, and lane i of the group gets column i of that slab for the four keys:
    // exactly four consecutive k-slots of an MFMA A operand whose row is head-dim index i.
    // Groups 0/1 of a half-wave take columns 0-15 / 16-31 of the 32-wide block, half-waves
    // (g) take key rows +0 / +4, matching the k-slot order of the P registers.
    int v_off[DB];                               // byte offset of the lane's 8-byte piece for block db
    {
        const int sl = lane & 15, grp = (lane >> 4) & 1;
        const int row = (sl >> 2) + 4 * g;       // + 8*(2*ts + half) + 32*ka rows added at the read
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * grp + ((sl & 3) >> 1);
            v_off[db] = row * L::kRowBytes + ((chunk ^ L::swz_v(row)) << 4) + 8 * (sl & 1);
        }
    }

    // Visibility words of a tile's 64 keys for the lane's two queries: all ones inside the
    // prefix, the low bits for a ragged last prefix tile, the ancestor-mask word for a tree
    // tile.  They are fetched one iteration ahead, BEFORE that iteration's direct loads are
    // issued, so that the wait the compiler places at their first use finds nothing in flight.
    uint64_t vis_next[QB];
    auto fetch_vis = [=](int t, uint64_t (&v)[QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) v[qb] = (t >= nTp && t < nT) ? mrow[qb][t - nTp] : ~0ull;
    };
    fetch_vis(wk, vis_next);
    issue_stage(0);
    wait_direct_loads();
    __syncthreads();

    for (int it = 0; it < nIt; ++it) {
        uint64_t vis[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            vis[qb] = vis_next[qb];
            asm volatile("" : "+v"(vis[qb]));                     // first use of the prefetched words
        }
        fetch_vis(2 * (it + 1) + wk, vis_next);
        if (it + 1 < nIt) issue_stage(it + 1);

        const int t = 2 * it + wk;
        if (t < nT) {
            bool need_mask = t >= nTp;
            if (t < nTp && (t + 1) * kKeysPerTile > P) {
                const int live = P - t * kKeysPerTile;              // 1..63
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) vis[qb] = (1ull << live) - 1ull;
                need_mask = true;
            }
            uint64_t vis_any = 0;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) vis_any |= vis[qb];
            if (__any(vis_any != 0ull)) {
                const unsigned char* Ks = lds + (it & 1) * L::kStageBytes + 2 * wk * L::kMatBytes;
                const unsigned char* Vs = Ks + L::kMatBytes;

                // ---- S^T = K Q^T for the two 32-key blocks of the tile: independent
                //      accumulation chains, so consecutive MFMAs never wait on each other
                floatx16 S[2][QB];
                const floatx16 zero16 = { 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0 };
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    bf16x8 kf[2];
#pragma unroll
                    for (int ka = 0; ka < 2; ++ka)
                        kf[ka] = *reinterpret_cast<const bf16x8*>(Ks + 32 * ka * L::kRowBytes + k_off[kk]);
#pragma unroll
                    for (int ka = 0; ka < 2; ++ka)
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
                            S[ka][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ka], qf[qb][kk], kk == 0 ? zero16 : S[ka][qb], 0, 0, 0);
                }

                // ---- mask + online softmax.  Register i of a 32x32 block holds key row
                //      8*(i/4) + 4*g + i%4 of the block, query column n.
                bf16x8 pb[QB][2][2];                      // [query block][key block][16-key step]
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
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
                        for (int i = 0; i < 16; i += 2) mx = max3(mx, S[ka][qb][i], S[ka][qb][i + 1]);
                    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
                    // The reference maximum only has to keep exp2 in range, so it is raised
                    // lazily: the accumulators are rescaled only when a score tops it by kLazy.
                    if (__any(mx * c2 > m_run[qb] * c2 + kLazy)) {
                        const float m_new = fmaxf(m_run[qb], mx);
                        const float alpha = fast_exp2((m_run[qb] - m_new) * c2);
                        m_run[qb] = m_new;
                        l_run[qb] *= alpha;
                        if (__any(alpha != 0.0f && alpha != 1.0f)) {   // alpha 0: accumulators still 0
#pragma unroll
                            for (int db = 0; db < DB; ++db)
#pragma unroll
                                for (int i = 0; i < 16; ++i) acc[db][qb][i] *= alpha;
                        }
                    }
                    const float mc = m_run[qb] * c2;
                    float ls = 0.0f;
#pragma unroll
                    for (int ka = 0; ka < 2; ++ka)
#pragma unroll
                        for (int i = 0; i < 16; i += 2) {
                            const float p0 = fast_exp2(fmaf(S[ka][qb][i], c2, -mc));
                            const float p1 = fast_exp2(fmaf(S[ka][qb][i + 1], c2, -mc));
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
                    for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                        for (int db = 0; db < DB; ++db) {
                            union { short4v h[2]; bf16x8 v; } f;
#pragma unroll
                            for (int half = 0; half < 2; ++half) {
                                const int krow = 32 * ka + 8 * (2 * ts + half);      // + s/4 + 4*g in v_off
                                f.h[half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                    (lds_short4)(Vs + krow * L::kRowBytes + v_off[db]));
                            }
#pragma unroll
                            for (int qb = 0; qb < QB; ++qb)
                                acc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v, pb[qb][ka][ts], acc[db][qb], 0, 0, 0);
                        }
            }
        }
        wait_direct_loads();
        __syncthreads();
    }

    // ---- merge the two key halves of each row half through LDS, normalise, store
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] += __shfl_xor(l_run[qb], 32, kWave);
    float* xs = reinterpret_cast<float*>(lds);               // [wq][register][lane]
    constexpr int NR = DB * QB * 16 + 2 * QB;
    if (wk == 1) {
        float* dst = xs + (size_t)wq * NR * kWave + lane;
        int r = 0;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int i = 0; i < 16; ++i) dst[(r++) * kWave] = acc[db][qb][i];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) dst[(r++) * kWave] = m_run[qb];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) dst[(r++) * kWave] = l_run[qb];
    }
    __syncthreads();
    if (wk == 0) {
        const float* src = xs + (size_t)wq * NR * kWave + lane;
        float f0[QB], f1[QB], inv[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float m1 = src[(NR - 2 * QB + qb) * kWave], l1 = src[(NR - QB + qb) * kWave];
            const float m = fmaxf(m_run[qb], m1);
            f0[qb] = exp2f((m_run[qb] - m) * c2);
            f1[qb] = exp2f((m1 - m) * c2);
            inv[qb] = 1.0f / (l_run[qb] * f0[qb] + l1 * f1[qb]);
        }
        int r = 0;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float o1 = src[(r++) * kWave];
                    acc[db][qb][i] = (acc[db][qb][i] * f0[qb] + o1 * f1[qb]) * inv[qb];
                }
        // register i of block db is head-dim index 32*db + 8*(i/4) + 4*g + i%4
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if (rq[qb] >= rows) continue;
            const int j = rq[qb] / G, h = kvh * G + rq[qb] % G;
            __bf16* orow = static_cast<__bf16*>(a.out) + ((size_t)(node_base + j) * a.Hq + h) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    union { bf16x2 p[2]; uint2 v; } o;
#pragma unroll
                    for (int ii = 0; ii < 2; ++ii) {
                        floatx2 pr = { acc[db][qb][4 * ib + 2 * ii], acc[db][qb][4 * ib + 2 * ii + 1] };
                        o.p[ii] = __builtin_convertvector(pr, bf16x2);
                    }
                    *reinterpret_cast<uint2*>(orow + 32 * db + 8 * ib + 4 * g) = o.v;
                }
        }
    }
}

template <int D, int QB>
static hipError_t launch_one(const AttnArgs& a, const SeqArgs& sa, int tiles, hipStream_t stream)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tree_attn_mfma_kernel<D, QB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Geo<D>::kLdsBytes);
    if (e != hipSuccess) return e;
    tree_attn_mfma_kernel<D, QB><<<tiles * a.Hkv, 64 * 2 * (4 / QB), Geo<D>::kLdsBytes, stream>>>(a, sa);
    return hipGetLastError();
}

hipError_t launch_tree_attn_mfma(AttnArgs a, const SeqArgs& sa, hipStream_t stream)
{
    const int G = a.Hq / a.Hkv;
    int tiles = 0;
    for (int s = 0; s < sa.n_seq; ++s) {
        a.tile_off[s] = tiles;
        tiles += (G * (sa.node_off[s + 1] - sa.node_off[s]) + kRowsPerWG - 1) / kRowsPerWG;
    }
    a.tile_off[sa.n_seq] = tiles;
    if (tiles == 0) return hipSuccess;
    return a.d == 128 ? launch_one<128, kQB>(a, sa, tiles, stream) : launch_one<64, kQB>(a, sa, tiles, stream);
}

}  // namespace dyspec
