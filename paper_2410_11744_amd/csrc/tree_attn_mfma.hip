// Tree attention on the matrix cores (Section 2, "Tree Attention"; Appendix C) for gfx950:
// bf16 tensors, head_dim 64 or 128, fp32 accumulation.
//
// Row folding.  All G = Hq/Hkv query heads that share a KV head are folded into the row
// dimension (row = node*G + head), so a workgroup tile of 128 rows streams the prefix K/V
// of its KV head once and every K/V byte feeds 128 rows of MFMA work; the tree part reuses
// the same machinery with the ancestor bitmask applied to the numerators.  Tree tiles (64
// keys) in which no query of the workgroup sees a key are left out of the walk altogether,
// and a wave does nothing for a 32-key half none of its own queries can see (the paper's
// kernel skips empty 32x32 blocks of the mask).
//
// Workgroup = 8 waves, two per SIMD.  Wave w owns the 32-row block (w & 3) and every second
// 64-key tile ((w >> 2) picks even or odd tiles); the two waves of a row block merge their
// (max, sum, accumulator) through LDS at the end.  Per 32-key half tile a wave computes
// S^T = K Q^T (keys x queries: each lane then holds one query column, and exp(S^T) is
// already in the register layout the second product wants as its B operand), the softmax
// numerators, and O^T += V^T P^T.
//
// Software pipeline.  The vector work of the softmax and the matrix work run in different
// pipes of a SIMD, but they overlap reliably only when both waves of the SIMD interleave them
// finely (a few vector instructions per MFMA: a wave's vector work runs behind the other
// wave's MFMA), so the loop is skewed by half tiles: a half step runs the exponentials of half
// h while the matrix pipe does the second product of half h-1 and the first product of half
// h+1; one scheduling group holds one MFMA, the LDS reads of an MFMA a few slots ahead, and
// a few vector instructions.
//
// Lazy maximum.  Numerators are computed against the running reference maximum without
// looking at the half's own maximum first; only when a lane's sum over the half leaves the
// safe range (the half is then recomputed, rarely) is the reference raised and the
// accumulators rescaled.
//
// Staging.  K/V tiles go from HBM/L2 to LDS with direct loads (global_load_lds_dwordx4: lane
// i of a wave writes LDS bytes [16*i, 16*i+16) past a wave-uniform base), two slots per
// matrix, without passing through registers; in the middle of step i (after the only
// barrier of the step) the loads of K of tile i+2 and V of tile i+1 start, spread over the
// following half step so that they drain while the matrix pipe works.  Rows sit unpadded in
// LDS; 16-byte chunks of a row are XOR-swizzled so that the 16-byte K reads and the
// transposing V reads of a wave spread over all 64 banks.
#include <utility>

#include <atomic>
#include <cstdlib>
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
template <typename F>
__device__ __forceinline__ void with_bool(bool b, F&& f)
{
    if (b) f(std::true_type{}); else f(std::false_type{});
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(1))) const void* global_ptr;
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v* lds_short4;
typedef __attribute__((address_space(3))) const bf16x8* lds_bf16x8;

#ifdef DYSPEC_STAMPS
// Timing build only: thread 0 of every workgroup records the 100 MHz wall clock at a few points.
__device__ unsigned long long g_stamps[8192 * 8];
__device__ unsigned g_stamp_slot;
#define STAMP(k) do { if (threadIdx.x == 0) stamp_row[k] = wall_clock64(); } while (0)
#else
#define STAMP(k) do { } while (0)
#endif

constexpr int kRowsPerWG = 128;
constexpr int kKeysPerTile = 64;
constexpr float kSumLimit = 1024.0f;      // a lane's tile sum above this raises the reference maximum
#ifndef DYSPEC_ATTN_LEAD
#define DYSPEC_ATTN_LEAD 2
#endif
constexpr int kLead = DYSPEC_ATTN_LEAD;   // fragment slots between an LDS read and the MFMAs that use it
#ifndef DYSPEC_ATTN_QB
#define DYSPEC_ATTN_QB 1
#endif
constexpr int kQB = DYSPEC_ATTN_QB;       // 32-row query blocks per wave (see the kernel)

// v_exp_f32 without the denormal-range fix-up: inputs below -126 give 0, which is what the
// softmax wants.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float and_bits(float x, int m) { return __int_as_float(__float_as_int(x) & m); }
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
    static constexpr int kSlotBytes = 2 * kMatBytes;             // a slot holds an even and an odd tile
    static constexpr int kVBase = 2 * kSlotBytes;                // K slots 0 and 1, then V slots 0 and 1
    static constexpr int kLdsBytes = 4 * kSlotBytes;
    static constexpr int kLoadsPerMat = kKeysPerTile / kRowsPerLoad;
    // chunk c of K row r sits at chunk position c ^ swz_k(r); of V row r at c ^ swz_v(r)
    __device__ static __forceinline__ int swz_k(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
    __device__ static __forceinline__ int swz_v(int r) { return D == 128 ? ((r & 3) << 2) : 0; }
};

// QB = 32-row query blocks per wave.  Every K/V fragment read from LDS feeds QB MFMAs, so
// QB = 2 halves the LDS traffic per flop: 4 waves, one per SIMD, with up to 512 registers each.
// QB = 1: 8 waves, two per SIMD, 256 registers each.  QB = 1 is what the library is built with:
// a wave alone on its SIMD does not hide its vector instructions behind its own MFMAs (measured
// at the 70B shape: 79.5 us per launch with QB = 2 against 71.1 us with QB = 1).
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
#ifdef DYSPEC_STAMPS
    unsigned long long* stamp_row = g_stamps;
    if (threadIdx.x == 0) { stamp_row = g_stamps + (size_t)(atomicAdd(&g_stamp_slot, 1u) % 8192u) * 8; stamp_row[7] = blockIdx.y; }
    STAMP(0);
#endif
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
    // Prefix split: this workgroup walks prefix tiles [p_begin, p_begin + nPl) and, if it is
    // the last split, the tree tiles as well; with a.tree_split the prefix is dealt to the other
    // splits only and the last one is left with the tree.
    const int split = blockIdx.y, n_split = a.splits;
    const int n_pref = max(n_split - a.tree_split, 1);
    const int share = (((nTp + n_pref - 1) / n_pref) + 1) & ~1;        // an even number of tiles
    const int p_begin = min(split * share, nTp);
    const int nPl = min(nTp - p_begin, share);
    const bool last_split = split == n_split - 1;
    const int nTt = last_split ? (r_last / G) / kKeysPerTile + 1 : 0;  // tree tiles up to the largest node of this row tile
    const int nT = nTp + nTt;                              // a tile index >= nT stands for "no tile"

    const size_t kv_row_bytes = (size_t)a.Hkv * D * 2;
    const int layer = blockIdx.z;                          // stacked layers: one grid plane each
    const size_t kvp_off = (size_t)layer * a.kvp_stride + (size_t)sa.kv_off[seq] * kv_row_bytes + (size_t)kvh * D * 2;
    const size_t kvt_off = (size_t)layer * a.kvt_stride + (size_t)node_base * kv_row_bytes + (size_t)kvh * D * 2;
    const char* kp = static_cast<const char*>(a.kp) + kvp_off;
    const char* vp = static_cast<const char*>(a.vp) + kvp_off;
    const char* kt = static_cast<const char*>(a.kt) + kvt_off;
    const char* vt = static_cast<const char*>(a.vt) + kvt_off;
    const __bf16* q_layer = reinterpret_cast<const __bf16*>(static_cast<const char*>(a.q) + (size_t)layer * a.q_stride);

    // ---- Q fragments (B operand: lane holds query n, head-dim slice 16*kk + 8*g .. +7).  The
    //      workgroup's 128 query rows come through LDS like a K tile (see the prologue) and are
    //      read into these registers once.
    static_assert(QB == 1, "the Q staging below is written for one query block per wave");
    bf16x8 qf[QB][KK];
    int rq[QB];
    const uint64_t* mrow[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        rq[qb] = r0 + 32 * QB * wq + 32 * qb + n;
        const int rc = min(rq[qb], rows - 1);
        mrow[qb] = a.mask + (size_t)(node_base + rc / G) * a.mask_words;
    }

    floatx16 acc[DB][QB];                        // O^T: [32-wide head-dim block][query block]
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[db][qb][i] = 0.0f;
    floatx16 S[2][QB];                           // scores of a 32-key half tile: half e in buffer e
    uint32_t pbw[2][QB][2][4];                   // numerators as bf16 pairs [buffer][query block][16-key step][word]
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -1e30f; l_run[qb] = 0.0f; }
    const float c2 = a.scale * 1.4426950408889634f;     // scores are used as exp2(c2 * s)

    // ---- direct-load plan.  Matrix mm (0: K of the even tile, 1: K odd, 2: V even, 3: V odd)
    //      takes kLoadsPerMat wave-wide loads, issued by NW/4 waves.  Lane i of load x writes row
    //      position R = kRowsPerLoad*x + i/kChunks, chunk position i % kChunks, so it must fetch
    //      chunk (i % kChunks) ^ swz(R) of that key row; with these swizzles the lane's byte
    //      offset depends on x mod 4 only.
    constexpr int LPW = L::kLoadsPerMat / (NW / 4);
    const int ld_mm = wave / (NW / 4), ld_x0 = (wave % (NW / 4)) * LPW;
    const bool ld_is_v = ld_mm >= 2;
    const int ld_par = ld_mm & 1;
    const int ld_lrow = lane / L::kChunks, ld_cpos = lane % L::kChunks;
    auto lane_offsets = [=](bool is_v, int (&voff)[4]) {
#pragma unroll
        for (int xm = 0; xm < 4; ++xm) {
            const int row = L::kRowsPerLoad * xm + ld_lrow;
            const int c = ld_cpos ^ (is_v ? L::swz_v(row) : L::swz_k(row));
            voff[xm] = ld_lrow * (int)kv_row_bytes + 16 * c;
        }
    };
    // Loads this wave's share of tile t (prefix or tree part of K or V) to LDS byte dst.
    // (captures by value: a conditional between variables captured by reference would be a
    //  conditional between addresses and force them into scratch memory)
    auto issue_tile = [=](const char* prefix_region, const char* tree_region, const int (&voff)[4], int t, uint32_t dst)
        __attribute__((always_inline)) {
        if (t >= nT) return;
        const bool prefix = t < nTp;
        const char* region = prefix ? prefix_region : tree_region;
        const int key0 = (prefix ? t : t - nTp) * kKeysPerTile;
        const int limit = prefix ? P : N;
        if (key0 + kKeysPerTile <= limit) {                      // whole tile in range: uniform base + lane offset
            const char* base = region + (size_t)(key0 + L::kRowsPerLoad * ld_x0) * kv_row_bytes;
            static_for<LPW>([=](auto xc) {
                constexpr int x = decltype(xc)::value;
                direct_load_16(base + (size_t)(L::kRowsPerLoad * x) * kv_row_bytes, (uint32_t)voff[x & 3], dst + x * 1024);
            });
        } else {
            // rows past the end read the last row of the region instead (finite values, as every row
            // of the tensor); their scores are masked out.  The tile's first row goes into the 64-bit
            // base, so the 32-bit lane offset stays below 64 rows whatever the prefix length.
            const char* base = region + (size_t)key0 * kv_row_bytes;
            static_for<LPW>([=](auto xc) {
                constexpr int x = decltype(xc)::value;
                const int rowx = L::kRowsPerLoad * (ld_x0 + x);
                const int back = max(key0 + rowx + ld_lrow - (limit - 1), 0);        // rows past the last one
                const uint32_t off = (uint32_t)(rowx - back) * (uint32_t)kv_row_bytes + (uint32_t)voff[x & 3];
                direct_load_16(base, off, dst + x * 1024);
            });
        }
    };
    const uint32_t lds0 = lds_address(lds);
    // steady state: this wave's matrix, the lane offsets for it, and its place in an LDS slot
    int ld_voff[4];
    lane_offsets(ld_is_v, ld_voff);
    const char* const st_prefix = ld_is_v ? vp : kp;
    const char* const st_tree = ld_is_v ? vt : kt;
    const uint32_t st_dst = lds0 + (ld_is_v ? L::kVBase : 0) + ld_par * L::kMatBytes + ld_x0 * 1024;
    uint32_t none32[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) none32[qb] = 0u;

    // ---- LDS read addresses of this lane (the LDS base and the even/odd tile choice of the wave folded in)
    int k_off[KK];                               // K fragment of k-step kk, key row n of a half tile
    {
        const int h = g ^ L::swz_k(n);           // (2*kk + g) ^ swz == (2*kk) ^ (g ^ swz)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) k_off[kk] = (int)lds0 + wk * L::kMatBytes + n * L::kRowBytes + (((2 * kk) ^ h) << 4);
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
        const int row = (sl >> 2) + 4 * g;       // + 8*(2*ts + half) rows (+32 for an upper half) added at the read
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * grp + ((sl & 3) >> 1);
            v_off[db] = (int)lds0 + L::kVBase + wk * L::kMatBytes + row * L::kRowBytes + ((chunk ^ L::swz_v(row)) << 4) + 8 * (sl & 1);
        }
    }

    // Visibility words of a tile's 64 keys for the lane's queries: all ones inside the prefix,
    // the low bits for a ragged last prefix tile, the ancestor-mask word for a tree tile,
    // zero for a tile that does not exist.
    auto fetch_vis = [=](int t, uint64_t (&v)[QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) v[qb] = (t >= nTp && t < nT) ? mrow[qb][t - nTp] : ~0ull;
    };
    auto fix_vis = [=](int t, uint64_t v) -> uint64_t {
        if (t >= nT) return 0ull;
        if (t < nTp && (t + 1) * kKeysPerTile > P) return (1ull << (P - t * kKeysPerTile)) - 1ull;
        return v;
    };

    // ---- one half step of the skewed loop, for the 32-key half e of tile i (SP = i & 1 is the
    //      LDS slot of tile i).  HS: numerators of this half from S[e] into pbw[e]; HP: second
    //      product of the previous half (pbw[e^1]); HQ: first product of the next half into
    //      S[e^1]; MK: this half needs its mask (vis32: the lane's 32 visibility bits >> 4g).
    //      The previous half is the upper half of tile i-1 (slot SP^1) for e = 0 and the lower
    //      half of tile i for e = 1; the next half is the upper half of tile i for e = 0 and
    //      the lower half of tile i+1 (slot SP^1) for e = 1.
    const floatx16 zero16 = { 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0 };
    float ls_half[QB];                           // the lane's sums of numerators of the half just done
    //      LD: this wave's LPW direct loads of a whole tile (ld_base: its first row for this wave,
    //      ld_dst: LDS byte) are issued one per two slots, so that they drain while the matrix
    //      pipe works instead of queueing up behind the barrier.
    auto half_step = [&](auto hp_c, auto hq_c, auto hs_c, auto mk_c, auto ld_c, auto sp_c, auto e_c,
                         const uint32_t (&vis32)[QB], const char* ld_base, uint32_t ld_dst) __attribute__((always_inline)) {
        constexpr bool LD = decltype(ld_c)::value;
        constexpr bool HP = decltype(hp_c)::value, HQ = decltype(hq_c)::value;
        constexpr bool HS = decltype(hs_c)::value, MK = decltype(mk_c)::value;
        constexpr int SP = decltype(sp_c)::value, E = decltype(e_c)::value, O = E ^ 1;
        constexpr int NP2 = 2 * DB, NQ2 = KK;                      // fragments per half: second, first product
        static_assert(NP2 == NQ2, "the interleave below alternates the two products");
        constexpr int NS = (HP ? NP2 : 0) + (HQ ? NQ2 : 0);       // fragment slots (QB MFMAs each) of this half step
        constexpr int kVsrc = (E == 0 ? (SP ^ 1) : SP) * L::kSlotBytes + 32 * O * L::kRowBytes;
        constexpr int kKsrc = (E == 0 ? SP : (SP ^ 1)) * L::kSlotBytes + 32 * O * L::kRowBytes;
        float mc[QB], ls[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { mc[qb] = m_run[qb] * c2; ls[qb] = 0.0f; }
        // Register i of a 32x32 score block holds key row 8*(i/4) + 4*g + i%4, query column n.
        // Vector work on pair p = scores 2p, 2p+1 of a query block: F (two fma: the exponents),
        // X (two exponentials), M (mask, only for masked halves), C (round the pair to bf16 and
        // store it as a numerator word), D (add the pair to the row sum).  A wave issues
        // in order and a dependent vector instruction waits for its operand, so the stages of a
        // pair sit in different items: item h (two per pair) holds X(p) and D(p-1) when even,
        // M(p), F(p+1) and C(p) when odd; F of the first pair comes before item 0, D of the last
        // pair after the last item.  Nothing inside an item depends on anything else in it.
        constexpr int NPAIR = 8 * QB;
        float ft[NPAIR][2], pt[NPAIR][2];
        auto stage_f = [&](auto kc) __attribute__((always_inline)) {
            constexpr int k = decltype(kc)::value, qb = k / 8, i = 2 * (k % 8);
            ft[k][0] = fmaf(S[E][qb][i], c2, -mc[qb]);
            ft[k][1] = fmaf(S[E][qb][i + 1], c2, -mc[qb]);
        };
        auto stage_d = [&](auto kc) __attribute__((always_inline)) {
            constexpr int k = decltype(kc)::value, qb = k / 8;
            // Two plain adds of the fp32 numerators (after the mask, before the rounding to bf16).  The
            // dot-product instruction that would sum the rounded pair in one go holds back the matrix
            // pipe: measured, one v_dot2c_f32_bf16 per two MFMAs costs about seven cycles per MFMA,
            // two v_add_f32 nothing.  Sum of unrounded against product of rounded numerators: a relative
            // difference below 2^-9, the size of the bf16 rounding of the output itself.
            ls[qb] += pt[k][0];
            ls[qb] += pt[k][1];
        };
        auto valu_item = [&](auto hc) __attribute__((always_inline)) {
            constexpr int h = decltype(hc)::value, k = h / 2, qb = k / 8, p = k % 8, i = 2 * p;
            if constexpr (h % 2 == 0) {
                pt[k][0] = fast_exp2(ft[k][0]);
                pt[k][1] = fast_exp2(ft[k][1]);
                if constexpr (k > 0) stage_d(std::integral_constant<int, k - 1>{});
            } else {
                float p0 = pt[k][0], p1 = pt[k][1];
                if constexpr (MK) {
                    p0 = and_bits(p0, __builtin_amdgcn_sbfe((int)vis32[qb], 8 * (i / 4) + (i % 4), 1));
                    p1 = and_bits(p1, __builtin_amdgcn_sbfe((int)vis32[qb], 8 * (i / 4) + (i % 4) + 1, 1));
                }
                if constexpr (k + 1 < NPAIR) stage_f(std::integral_constant<int, k + 1>{});
                floatx2 pp = { p0, p1 };
                uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, bf16x2));
                asm volatile("" : "+v"(w));                    // keep the conversion in this scheduling group
                if constexpr (MK) { pt[k][0] = p0; pt[k][1] = p1; }
                pbw[E][qb][p / 4][p % 4] = w;
            }
        };
        if constexpr (HS) stage_f(std::integral_constant<int, 0>{});
        if constexpr (NS > 0) {
            // with both products, even slots belong to the first product and odd slots to the second
            // (the score chain then ends one MFMA before the half step does, so the next half
            // step does not start by waiting for its scores)
            bf16x8 fr[NS];
            auto read_slot = [&](auto sc) __attribute__((always_inline)) {
                constexpr int s = decltype(sc)::value;
                constexpr bool isP = HP && (!HQ || s % 2 == 1);
                constexpr int idx = (HP && HQ) ? s / 2 : s;
                if constexpr (isP) {
                    // k-slot (g, e) of step ts is key 8*(2*ts + e/4) + 4*g + e%4 of the half
                    constexpr int ts = idx / DB, db = idx % DB;
                    union { short4v h[2]; bf16x8 v; } f;
#pragma unroll
                    for (int half = 0; half < 2; ++half)
                        f.h[half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (lds_short4)(uint32_t)(kVsrc + 8 * (2 * ts + half) * L::kRowBytes + v_off[db]));
                    fr[s] = f.v;
                } else {
                    fr[s] = *(lds_bf16x8)(uint32_t)(kKsrc + k_off[idx]);
                }
            };
            auto mfma_slot = [&](auto sc) __attribute__((always_inline)) {
                constexpr int s = decltype(sc)::value;
                constexpr bool isP = HP && (!HQ || s % 2 == 1);
                constexpr int idx = (HP && HQ) ? s / 2 : s;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    if constexpr (isP) {
                        constexpr int ts = idx / DB, db = idx % DB;
                        union { uint32_t w[4]; bf16x8 v; } b;
#pragma unroll
                        for (int w = 0; w < 4; ++w) b.w[w] = pbw[O][qb][ts][w];
                        acc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[s], b.v, acc[db][qb], 0, 0, 0);
                    } else {
                        if constexpr (idx == 0)
                            S[O][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[s], qf[qb][idx], zero16, 0, 0, 0);
                        else
                            S[O][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[s], qf[qb][idx], S[O][qb], 0, 0, 0);
                    }
                }
            };
            constexpr int IPS = 16 * QB / NS;                  // items of vector work per slot
            constexpr int LEVERY = 2 * LPW <= NS ? 2 : 1;      // a direct load every second slot, or every slot
            static_assert(!LD || LEVERY * LPW <= NS, "the loads of a step fit its upper half step");
            static_for<(kLead < NS ? kLead : NS)>([&](auto sc) { read_slot(sc); });
            static_for<NS>([&](auto sc) {
                constexpr int s = decltype(sc)::value;
                if constexpr (s + kLead < NS) read_slot(std::integral_constant<int, s + kLead>{});
                mfma_slot(sc);
                if constexpr (LD && s % LEVERY == 0 && s / LEVERY < LPW)
                    direct_load_16(ld_base + (size_t)(L::kRowsPerLoad * (s / LEVERY)) * kv_row_bytes,
                                   (uint32_t)ld_voff[(s / LEVERY) & 3], ld_dst + (s / LEVERY) * 1024);
                if constexpr (HS)
                    static_for<IPS>([&](auto hc) { valu_item(std::integral_constant<int, s * IPS + decltype(hc)::value>{}); });
                __builtin_amdgcn_sched_barrier(0);
            });
        } else if constexpr (HS) {
            static_for<16 * QB>(valu_item);
        }
        if constexpr (HS) {
            stage_d(std::integral_constant<int, NPAIR - 1>{});
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) ls_half[qb] = ls[qb];
        }
    };
    // Rare: some score of half e tops the reference maximum by too much (always so for the
    // first half a wave sees).  Raise the reference to the true maximum, rescale what has been
    // accumulated (the second product of the previous half is complete here), and redo this
    // half's numerators.
    auto redo_half = [&](auto e_c, bool mk, const uint32_t (&vis32)[QB]) __attribute__((always_inline)) {
        constexpr int E = decltype(e_c)::value;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float sm[16];
#pragma unroll
            for (int i = 0; i < 16; ++i)
                sm[i] = (mk && !((vis32[qb] >> (8 * (i / 4) + (i % 4))) & 1u)) ? -INFINITY : S[E][qb][i];
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; i += 2) mx = max3(mx, sm[i], sm[i + 1]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float m_new = fmaxf(m_run[qb], mx);
            const float alpha = fast_exp2((m_run[qb] - m_new) * c2);
            m_run[qb] = m_new;
            l_run[qb] *= alpha;
            if (__any(alpha != 0.0f && alpha != 1.0f)) {       // alpha 0: accumulators still 0
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[db][qb][i] *= alpha;
            }
            const float mc2 = m_run[qb] * c2;
            float ls = 0.0f;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float p0 = fast_exp2(fmaf(sm[i], c2, -mc2));
                const float p1 = fast_exp2(fmaf(sm[i + 1], c2, -mc2));
                floatx2 pp = { p0, p1 };
                const bf16x2 pc = __builtin_convertvector(pp, bf16x2);
                ls += p0;
                ls += p1;
                pbw[E][qb][i / 8][(i / 2) % 4] = __builtin_bit_cast(uint32_t, pc);
            }
            ls_half[qb] = ls;
        }
    };
    // A half step of the steady state: all three parts, then the (rare) raise of the reference.
    auto run_half = [&](auto mk_c, auto ld_c, auto sp_c, auto e_c, const uint32_t (&vis32)[QB], const char* ld_base,
                        uint32_t ld_dst) __attribute__((always_inline)) {
        half_step(std::true_type{}, std::true_type{}, std::true_type{}, mk_c, ld_c, sp_c, e_c, vis32, ld_base, ld_dst);
        bool high = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) high |= !(ls_half[qb] <= kSumLimit);
        if (__any(high)) redo_half(e_c, decltype(mk_c)::value, vis32);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) l_run[qb] += ls_half[qb];
    };

    // ---- prologue.  Tree tiles in which no query of the workgroup sees any key are left out of
    //      the walk: every wave ballots its queries' mask words per tile and the waves OR the
    //      results into one LDS word (bit tt = tree tile tt).  With four or more prefix tiles
    //      ahead of the tree this happens while the first loads (K of walk positions 0..3, V of
    //      positions 0 and 1, all prefix) are in flight; with fewer, the first loads reach into
    //      the tree, so the set is agreed on first, when it can shorten the walk at all.
    uint32_t* const tile_flag = reinterpret_cast<uint32_t*>(lds + L::kLdsBytes);
    auto ballot_tiles = [=]() __attribute__((always_inline)) {
        if (wk != 0) return;                               // the wk == 1 waves hold the same rows
        uint32_t mine = 0u;
        for (int tt = 0; tt < nTt; ++tt) {
            uint64_t w = 0ull;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) w |= mrow[qb][tt];
            if (__any(w != 0ull)) mine |= 1u << tt;
        }
        if (lane == 0) atomicOr(tile_flag, mine);
    };
    const bool squeeze = nPl >= 4;                         // set agreed on behind the first loads
    const bool squeeze_first = !squeeze && nTt > 4 - nPl;  // set agreed on before them
    uint32_t first_set = nTt ? 0xffffffffu >> (32 - nTt) : 0u;
    if (squeeze_first) {
        if (tid == 0) *tile_flag = 0u;
        __syncthreads();
        ballot_tiles();
        __syncthreads();
        first_set = (uint32_t)__builtin_amdgcn_readfirstlane((int)*tile_flag);
        __syncthreads();                                   // everyone has read it before it is cleared again
    }
    // k-th tree tile (in ascending order) of a set
    auto kth_tile = [=](uint32_t set, int k) __attribute__((always_inline)) -> int {
        if (k >= __builtin_popcount(set)) return nT;
        for (int j = 0; j < k; ++j) set &= set - 1u;
        return nTp + __builtin_ctz(set);
    };
    // positions 0..3 of the walk: prefix tiles, then the tree tiles known so far
    auto first_tiles = [=](int v) __attribute__((always_inline)) -> int {
        return v < nPl ? p_begin + v : kth_tile(first_set, v - nPl);
    };
    // The workgroup's 128 query rows go to LDS first, into V slot 1 (which no V tile needs before the
    // middle of step 0), laid out like two K tiles: row R at R * kRowBytes, chunks swizzled as K's.
    // A row past the end repeats the last one.
    const uint32_t q_lds = lds0 + L::kVBase + L::kSlotBytes;
    {
        constexpr int QLW = (2 * kKeysPerTile / L::kRowsPerLoad) / NW;     // wave-wide loads per wave
        const char* q_seq = reinterpret_cast<const char*>(q_layer) + (size_t)node_base * a.Hq * D * 2;
#pragma unroll
        for (int x = 0; x < QLW; ++x) {
            const int X = wave * QLW + x;
            const int R = X * L::kRowsPerLoad + ld_lrow;
            const int rc = min(r0 + R, rows - 1);
            const int j = rc / G, h = kvh * G + rc % G;
            const uint32_t off = (uint32_t)(j * a.Hq + h) * (uint32_t)(D * 2) + 16u * (uint32_t)(ld_cpos ^ L::swz_k(R));
            direct_load_16(q_seq, off, q_lds + X * 1024);
        }
    }
    // K of walk positions 0..3 (position mm = 2*slot + parity, two waves per matrix) and V of
    // positions 0 and 1.  Waves 0..3 hold what the first product needs (positions 0 and 1 of K) and
    // issue it now; waves 4..7 hold the rest and issue it behind the next barrier, so that it queues
    // up in the CU's address path after the urgent loads instead of among them.
    static_assert(NW == 8, "the prologue's load plan is written for eight waves");
    auto issue_first_loads = [=]() __attribute__((always_inline)) {
        int voff_k[4];
        lane_offsets(false, voff_k);
        issue_tile(kp, kt, voff_k, first_tiles(ld_mm), lds0 + ld_mm * L::kMatBytes + ld_x0 * 1024);
        if (ld_is_v) issue_tile(st_prefix, st_tree, ld_voff, first_tiles(ld_par), st_dst);
    };
    if (!ld_is_v) issue_first_loads();
    // The steady-state half step always runs all three parts; what it reads for a half that does
    // not exist must therefore be harmless.  The numerators start as zeros, and so do numerators of
    // masked keys; the V rows they meet must be finite: V slot 1 holds the query rows until a V tile
    // replaces them, a matrix of slot 0 whose walk position does not exist is cleared here.  K of a
    // tile that does not exist is whatever the slot held, and the scores it gives are masked.
    {
        const uint4 z = { 0u, 0u, 0u, 0u };
#pragma unroll
        for (int par = 0; par < 2; ++par)
            if (first_tiles(par) >= nT)
                for (int x = tid; x < L::kMatBytes / 16; x += 64 * NW)
                    reinterpret_cast<uint4*>(lds + L::kVBase + par * L::kMatBytes)[x] = z;
        if (tid == 0) *tile_flag = 0u;
#pragma unroll
        for (int bu = 0; bu < 2; ++bu)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                    for (int w = 0; w < 4; ++w) pbw[bu][qb][ts][w] = 0u;
    }
    __syncthreads();
    if (ld_is_v) issue_first_loads();
    if (squeeze) ballot_tiles();
    // The first product needs the query rows and K of walk positions 0 and 1, which waves 0..3
    // loaded (every wave its share of the query rows first).  Waves 4..7 went on to K of positions
    // 2, 3 and V of positions 0, 1, needed from the middle of step 0 on: they wait for their query
    // rows only, i.e. until just the 2 * LPW loads issued after those are still in flight.
    {
        const bool later_all = ld_is_v && first_tiles(ld_mm) < nT && first_tiles(ld_par) < nT;
        if (later_all) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * LPW) : "memory");
        else wait_direct_loads();
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int R = 32 * wq + n;
        qf[0][kk] = *(lds_bf16x8)(uint32_t)(q_lds + R * L::kRowBytes + (((2 * kk + g) ^ L::swz_k(R)) << 4));
    }
    const uint32_t active = squeeze ? (uint32_t)__builtin_amdgcn_readfirstlane((int)*tile_flag) : first_set;
    const int nAct = __builtin_popcount(active);
    const int nIt = (nPl + nAct + 1) / 2;                  // tiles per wave (the last odd one may not exist)
    // position v in the walk -> tile index (this split's prefix tiles, then the tree tiles of the set)
    auto tile_of = [=](int v) __attribute__((always_inline)) -> int {
        return v < nPl ? p_begin + v : kth_tile(active, v - nPl);
    };
    STAMP(1);
    // first product of the lower half of tile 0 (K slot 0) into S[0]
    half_step(std::false_type{}, std::true_type{}, std::false_type{}, std::false_type{}, std::false_type{},
              std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, none32, nullptr, 0u);

    // ---- step i: lower half of tile i; barrier; loads of K(i+2) and V(i+1) into the slots
    //      the lower half was the last to read; upper half of tile i
    auto issue_step_loads = [=](int i) __attribute__((always_inline)) {
        issue_tile(st_prefix, st_tree, ld_voff, tile_of(ld_is_v ? 2 * (i + 1) + ld_par : 2 * (i + 2) + ld_par),
                   st_dst + ((ld_is_v ? i + 1 : i) & 1) * L::kSlotBytes);
    };
    // Plain steps: positions 2i and 2i+1 of the walk are whole prefix tiles (no mask), and the tiles
    // the step loads -- positions up to 2(i+2)+1 -- are whole tiles of the prefix or of the tree (a
    // uniform base per load, spread over the upper half step) or do not exist (then a whole prefix
    // tile is loaded in their place: finite values under numerators that are all zero).
    const int nWholeP = min(nPl, max(P / kKeysPerTile - p_begin, 0));      // whole prefix tiles at the head of the walk
    int posRagged = 0x3fffffff;                                            // first place in the walk with a ragged tile
    if (nTt > 0 && nTt * kKeysPerTile > N && ((active >> (nTt - 1)) & 1u)) posRagged = nPl + nAct - 1;
    if (nWholeP < nPl) posRagged = nWholeP;
    const int nPlain = min(nWholeP / 2, max(posRagged - 4, 0) / 2);
    auto plain_load_base = [=](int ii) __attribute__((always_inline)) -> const char* {
        const int tl = tile_of(ld_is_v ? 2 * (ii + 1) + ld_par : 2 * (ii + 2) + ld_par);
        const bool tree = tl >= nTp && tl < nT;
        const int key0 = (tl >= nT ? p_begin : tree ? tl - nTp : tl) * kKeysPerTile;
        return (tree ? st_tree : st_prefix) + (size_t)(key0 + L::kRowsPerLoad * ld_x0) * kv_row_bytes;
    };
    int i = 0;
    for (; i + 1 < nPlain; i += 2) {
        static_for<2>([&](auto sp_c) {
            const int ii = i + decltype(sp_c)::value;
            run_half(std::false_type{}, std::false_type{}, sp_c, std::integral_constant<int, 0>{}, none32, nullptr, 0u);
            wait_direct_loads();
            __syncthreads();
            run_half(std::false_type{}, std::true_type{}, sp_c, std::integral_constant<int, 1>{}, none32, plain_load_base(ii),
                     st_dst + ((ld_is_v ? ii + 1 : ii) & 1) * L::kSlotBytes);
        });
    }
    STAMP(2);
    // The rest: ragged prefix tile, tree tiles (ancestor mask), tiles that do not exist (all
    // masked), until the second product of the last real half has run.  A half step does
    // something only if this wave's queries see a key of the half itself or of a neighbour
    // (whose second or first product it carries); otherwise it just clears its numerators.
    uint64_t visC[QB], visN[QB];
    {
        const int tc = tile_of(2 * i + wk), tn = tile_of(2 * i + 2 + wk);
        fetch_vis(tc, visC);
        fetch_vis(tn, visN);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            visC[qb] = fix_vis(tc, visC[qb]);
            visN[qb] = fix_vis(tn, visN[qb]);
        }
    }
    auto any_half = [&](const uint64_t (&v)[QB], int hi) __attribute__((always_inline)) -> bool {
        uint32_t x = 0u;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) x |= (uint32_t)(v[qb] >> (32 * hi));
        return __any(x != 0u);
    };
    auto masked_half = [&](auto sp_c, auto e_c, bool act, const uint32_t (&v32)[QB]) __attribute__((always_inline)) {
        if (act) {
            run_half(std::true_type{}, std::false_type{}, sp_c, e_c, v32, nullptr, 0u);
        } else {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                    for (int w = 0; w < 4; ++w) pbw[decltype(e_c)::value][qb][ts][w] = 0u;
        }
    };
    bool aP1 = true;                                         // the upper half of the last plain tile
    if (2 * i >= nPl + nAct) {
        // nothing left to walk (a split of whole prefix tiles that the plain loop has finished; i is
        // even here): only the second product of the last upper half is outstanding
        half_step(std::true_type{}, std::false_type{}, std::false_type{}, std::false_type{}, std::false_type{},
                  std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, none32, nullptr, 0u);
        wait_direct_loads();                                 // the last plain step's loads land before LDS is reused below
        i = nIt + 1;
    }
    for (; i <= nIt; i += 2) {
        static_for<2>([&](auto sp_c) {
            const int ii = i + decltype(sp_c)::value;
            const int t2 = tile_of(2 * ii + wk + 4);
            uint64_t visL[QB];
            fetch_vis(t2, visL);
            const bool aC0 = any_half(visC, 0), aC1 = any_half(visC, 1), aN0 = any_half(visN, 0);
            uint32_t v32[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) v32[qb] = (uint32_t)visC[qb] >> (4 * g);
            masked_half(sp_c, std::integral_constant<int, 0>{}, aP1 || aC0 || aC1, v32);
            wait_direct_loads();
            __syncthreads();
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) asm volatile("" : "+v"(visL[qb]));
            issue_step_loads(ii);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) v32[qb] = (uint32_t)(visC[qb] >> 32) >> (4 * g);
            masked_half(sp_c, std::integral_constant<int, 1>{}, aC0 || aC1 || aN0, v32);
            aP1 = aC1;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                visC[qb] = visN[qb];
                visN[qb] = fix_vis(t2, visL[qb]);
            }
        });
    }
    __syncthreads();                                         // every LDS read is done before the merge reuses it
    STAMP(3);

    // ---- merge the two key halves of each row block through LDS, normalise, store
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
                for (int i2 = 0; i2 < 16; ++i2) dst[(r++) * kWave] = acc[db][qb][i2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) dst[(r++) * kWave] = m_run[qb];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) dst[(r++) * kWave] = l_run[qb];
    }
    __syncthreads();
    // Row blocks are finished by the wk == 0 waves: (m_all, l_all) and the unnormalised rows, both key
    // halves merged.  Register i of block db is head-dim index 32*db + 8*(i/4) + 4*g + i%4.
    float m_all[QB], l_all[QB];
    if (wk == 0) {
        const float* src = xs + (size_t)wq * NR * kWave + lane;
        float f0[QB], f1[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float m1 = src[(NR - 2 * QB + qb) * kWave], l1 = src[(NR - QB + qb) * kWave];
            const float m = fmaxf(m_run[qb], m1);
            f0[qb] = exp2f((m_run[qb] - m) * c2);
            f1[qb] = exp2f((m1 - m) * c2);
            m_all[qb] = m;
            l_all[qb] = l_run[qb] * f0[qb] + l1 * f1[qb];
        }
        int r = 0;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int i2 = 0; i2 < 16; ++i2) {
                    const float o1 = src[(r++) * kWave];
                    acc[db][qb][i2] = acc[db][qb][i2] * f0[qb] + o1 * f1[qb];
                }
    }
    STAMP(4);
    if (n_split > 1) {
        // Prefix split.  Every workgroup leaves its normalised rows (bf16) and their (max, sum) in the
        // workspace, in register layout (word k of lane l at k*64 + l: each store of a wave is one
        // 512-byte run), then arrives at the counter of its (layer, row tile, KV head).  The one that
        // arrives last reads all parts and finishes the rows.  The counter wraps to zero with the
        // last arrival, so the next launch finds it as this one did.
        // Parts are written and read with device-scope atomic accesses (relaxed): they go to the
        // level of the memory system all workgroups share, whichever XCD they run on, without the
        // cache-wide write-back and invalidate a device-scope fence around plain accesses costs.
        static_assert(QB == 1, "the part layout assumes one query block per wave");
        constexpr int W2 = DB * 4;                              // 64-bit words of packed bf16 per lane
        constexpr int PW2 = attn_part_words(D) / 2;             // 64-bit words per (group, split)
        const size_t group = (size_t)layer * gridDim.x + blockIdx.x;
        unsigned long long* const parts = reinterpret_cast<unsigned long long*>(a.part) + group * n_split * PW2 +
                                          (size_t)wq * (W2 + 1) * kWave + lane;
        auto pack2 = [](float x, float y) -> uint32_t {
            floatx2 v = { x, y };
            return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
        };
        if (wk == 0) {
            unsigned long long* const mine = parts + (size_t)split * PW2;
            const float inv = l_all[0] > 0.0f ? 1.0f / l_all[0] : 0.0f;     // a split without keys: weight 0, rows 0
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    const uint32_t lo = pack2(acc[db][0][4 * ib] * inv, acc[db][0][4 * ib + 1] * inv);
                    const uint32_t hi = pack2(acc[db][0][4 * ib + 2] * inv, acc[db][0][4 * ib + 3] * inv);
                    __hip_atomic_store(mine + (db * 4 + ib) * kWave, ((unsigned long long)hi << 32) | lo, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
            __hip_atomic_store(mine + W2 * kWave, ((unsigned long long)__float_as_uint(l_all[0]) << 32) | __float_as_uint(m_all[0]),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // every store of the workgroup has been acknowledged before its arrival is counted
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (tid == 0) {
            const unsigned before = __builtin_amdgcn_atomic_inc32(a.counters + group, (unsigned)n_split - 1u, __ATOMIC_RELAXED, "agent");
            *tile_flag = before == (unsigned)n_split - 1u;
        }
        __syncthreads();
        STAMP(5);
        if (*tile_flag == 0u) return;                          // uniform over the workgroup
        // All parts come from memory, this workgroup's own too, and are summed in split order: the
        // result does not depend on which workgroup happened to arrive last.  All eight waves take
        // part: wave (wq, wk) finishes head-dim blocks [wk*DB/2, (wk+1)*DB/2) of row block wq, with
        // the loads of four splits in flight at a time.
        constexpr int HW = W2 / 2;                              // 64-bit words per lane and split in this wave's half
        auto ld = [&](int z, int k) -> unsigned long long {
            return __hip_atomic_load(parts + (size_t)z * PW2 + k * kWave, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        float M = -1e30f, Lsum = 0.0f;
        float o[HW][4];
#pragma unroll
        for (int k = 0; k < HW; ++k)
#pragma unroll
            for (int e = 0; e < 4; ++e) o[k][e] = 0.0f;
        // ZB splits per trip to memory (a trip costs about as much as a step of the walk)
        auto add_batch = [&](auto zb_c, int z0) __attribute__((always_inline)) {
            constexpr int ZB = decltype(zb_c)::value;
            unsigned long long w[ZB][HW + 1];
#pragma unroll
            for (int dz = 0; dz < ZB; ++dz) {
                if (z0 + dz < n_split) {                       // uniform: a part past the end is not fetched
#pragma unroll
                    for (int k = 0; k < HW; ++k) w[dz][k] = ld(z0 + dz, wk * HW + k);
                    w[dz][HW] = ld(z0 + dz, W2);
                } else {                                       // and stands in with maximum -1e30, weight 0 below
#pragma unroll
                    for (int k = 0; k < HW; ++k) w[dz][k] = 0ull;
                    w[dz][HW] = (unsigned long long)__float_as_uint(-1e30f);
                }
            }
            float Mb = M;                                      // the reference maximum moves up with the batch
#pragma unroll
            for (int dz = 0; dz < ZB; ++dz) Mb = fmaxf(Mb, __uint_as_float((uint32_t)w[dz][HW]));
            const float up = exp2f((M - Mb) * c2);
            M = Mb;
            Lsum *= up;
#pragma unroll
            for (int k = 0; k < HW; ++k)
#pragma unroll
                for (int e = 0; e < 4; ++e) o[k][e] *= up;
#pragma unroll
            for (int dz = 0; dz < ZB; ++dz) {
                const float mz = __uint_as_float((uint32_t)w[dz][HW]), lz = __uint_as_float((uint32_t)(w[dz][HW] >> 32));
                const float wz = z0 + dz < n_split ? exp2f((mz - M) * c2) * lz : 0.0f;   // normalised rows: weight times sum
                Lsum += wz;
#pragma unroll
                for (int k = 0; k < HW; ++k) {
                    const uint32_t lo = (uint32_t)w[dz][k], hi = (uint32_t)(w[dz][k] >> 32);
                    o[k][0] = fmaf(wz, __uint_as_float(lo << 16), o[k][0]);
                    o[k][1] = fmaf(wz, __uint_as_float(lo & 0xffff0000u), o[k][1]);
                    o[k][2] = fmaf(wz, __uint_as_float(hi << 16), o[k][2]);
                    o[k][3] = fmaf(wz, __uint_as_float(hi & 0xffff0000u), o[k][3]);
                }
            }
        };
        if (n_split <= 4) {
            add_batch(std::integral_constant<int, 4>{}, 0);
        } else {
            for (int z0 = 0; z0 < n_split; z0 += 8) add_batch(std::integral_constant<int, 8>{}, z0);
        }
        // The rows leave as in the unsplit case below: staged in LDS (each wave its half rows, in its own
        // half of its row block's part of the merge buffer, which nobody reads any more) and written as
        // whole 2*D/2-byte runs with streaming stores.
        {
            const float inv = 1.0f / Lsum;                     // a row past the end: never read back
            constexpr int kHalfBytes = D;                      // D/2 bf16 values
            constexpr int kPitch = kHalfBytes + 16;
            static_assert(2 * 32 * kPitch <= NR * kWave * (int)sizeof(float), "both halves fit in the row block's merge area");
            char* const stage = reinterpret_cast<char*>(xs + (size_t)wq * NR * kWave) + wk * 32 * kPitch;
#pragma unroll
            for (int k = 0; k < HW; ++k) {
                const int db = (wk * HW + k) / 4, ib = (wk * HW + k) % 4;
                uint2 v;
                v.x = pack2(o[k][0] * inv, o[k][1] * inv);
                v.y = pack2(o[k][2] * inv, o[k][3] * inv);
                *reinterpret_cast<uint2*>(stage + n * kPitch + (32 * db + 8 * ib + 4 * g) * 2 - wk * kHalfBytes) = v;
            }
            constexpr int CPH = kHalfBytes / 16;               // 16-byte chunks per half row
            char* const out_layer = static_cast<char*>(a.out) + (size_t)layer * a.q_stride;
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int t = 0; t < 32 * CPH / kWave; ++t) {
                const int c = lane + kWave * t, rn = c / CPH, cc = c % CPH;
                const int r = r0 + 32 * wq + rn;
                if (r >= rows) continue;
                const uint4 v = *reinterpret_cast<const uint4*>(stage + rn * kPitch + cc * 16);
                const int j = r / G, h = kvh * G + r % G;
                const u32x4 vv = { v.x, v.y, v.z, v.w };
                __builtin_nontemporal_store(vv, reinterpret_cast<u32x4*>(out_layer + (((size_t)(node_base + j) * a.Hq + h) * D) * 2 +
                                                                          wk * kHalfBytes + cc * 16));
            }
        }
        STAMP(6);
        return;
    }
    if (wk == 0) {
        // The wave's 32 finished rows go through LDS so that they leave as whole rows: in register
        // layout a store instruction writes 16 bytes of each of 32 rows, staged it writes four rows
        // end to end.  The staging area is the wave's own part of the merge buffer above, which only
        // this wave has read and nobody writes again; rows are 16 bytes apart from a multiple of 256
        // so that the 8-byte writes of a column of lanes spread over the banks.
        static_assert(QB == 1, "one query block per wave");
        constexpr int kPitch = D * 2 + 16;
        static_assert(32 * kPitch <= NR * kWave * (int)sizeof(float), "the rows fit in the wave's merge area");
        char* const stage = reinterpret_cast<char*>(xs + (size_t)wq * NR * kWave);
        const float inv = 1.0f / l_all[0];                     // a row past the end: never read back
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                union { bf16x2 p[2]; uint2 v; } o;
#pragma unroll
                for (int ii = 0; ii < 2; ++ii) {
                    floatx2 pr = { acc[db][0][4 * ib + 2 * ii] * inv, acc[db][0][4 * ib + 2 * ii + 1] * inv };
                    o.p[ii] = __builtin_convertvector(pr, bf16x2);
                }
                *reinterpret_cast<uint2*>(stage + n * kPitch + (32 * db + 8 * ib + 4 * g) * 2) = o.v;
            }
        constexpr int CPR = D * 2 / 16;                        // 16-byte chunks per row
        char* const out_layer = static_cast<char*>(a.out) + (size_t)layer * a.q_stride;
#pragma unroll
        for (int t = 0; t < 32 * CPR / kWave; ++t) {
            const int c = lane + kWave * t, rn = c / CPR, cc = c % CPR;
            const int r = r0 + 32 * wq + rn;
            if (r >= rows) continue;
            const uint4 v = *reinterpret_cast<const uint4*>(stage + rn * kPitch + cc * 16);
            const int j = r / G, h = kvh * G + r % G;
            // whole rows, streamed: all workgroups finish together, so what stays dirty in L2 is written
            // back after the last of them, with nothing left to overlap it
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 vv = { v.x, v.y, v.z, v.w };
            __builtin_nontemporal_store(vv, reinterpret_cast<u32x4*>(out_layer + (((size_t)(node_base + j) * a.Hq + h) * D) * 2 + cc * 16));
        }
    }
}

hipError_t prepare_tree_attn()
{
    static std::atomic<unsigned long long> done128{0}, done64{0};
    hipError_t e = raise_dynamic_lds_once(reinterpret_cast<const void*>(&tree_attn_mfma_kernel<128, kQB>), Geo<128>::kLdsBytes + 16, done128);
    if (e != hipSuccess) return e;
    return raise_dynamic_lds_once(reinterpret_cast<const void*>(&tree_attn_mfma_kernel<64, kQB>), Geo<64>::kLdsBytes + 16, done64);
}

template <int D, int QB>
static hipError_t launch_one(const AttnArgs& a, const SeqArgs& sa, int tiles, hipStream_t stream)
{
    const hipError_t e = prepare_tree_attn();              // the kernel needs more dynamic LDS than the default limit
    if (e != hipSuccess) return e;
    tree_attn_mfma_kernel<D, QB><<<dim3(tiles * a.Hkv, a.splits, a.layers), 64 * 2 * (4 / QB), Geo<D>::kLdsBytes + 16, stream>>>(a, sa);
    return hipGetLastError();
}

static int row_tiles(const SeqArgs& sa, int G, int* tile_off)
{
    int tiles = 0;
    for (int s = 0; s < sa.n_seq; ++s) {
        if (tile_off) tile_off[s] = tiles;
        tiles += (G * (sa.node_off[s + 1] - sa.node_off[s]) + kRowsPerWG - 1) / kRowsPerWG;
    }
    if (tile_off) tile_off[sa.n_seq] = tiles;
    return tiles;
}

// The kernel's parallelism is (row tiles) x (KV heads) x layers, one workgroup per CU at a time;
// when that leaves most of the 256 CUs idle (narrow trees, few KV heads) the prefix is split
// until the workgroups fill the chip once, as long as every split keeps at least four 64-key
// tiles of every sequence's prefix, and into at most eight parts (what the finishing workgroup
// fetches in one trip to memory).  Measured per layer: 1024 keys over 32 workgroups run best in 4
// parts, 2048 keys over 80 in 3, 4096 keys over 16 in 8.
//
// The split that also walks the tree ends last (a tree tile goes through the masked loop and
// costs about two prefix tiles).  If one more workgroup per group still fits on the chip and
// within the eight parts, the tree gets a split of its own when that shortens the longest walk
// of the batch, counted in prefix tiles.
AttnCut tree_attn_cut(const SeqArgs& sa, int Hq, int Hkv, int layers)
{
    const int groups = row_tiles(sa, Hq / Hkv, nullptr) * Hkv * layers;
    if (groups == 0) return { 1, 0 };
    int min_tiles = 1 << 30;
    for (int s = 0; s < sa.n_seq; ++s) min_tiles = min(min_tiles, (sa.prefix_len[s] + kKeysPerTile - 1) / kKeysPerTile);
    const int by_work = 256 / groups, by_prefix = min_tiles / 4;
    int splits = max(1, min(min(by_work, by_prefix), 8));
    int tree_split = 0;
    if ((size_t)groups * sizeof(unsigned) > kAttnCounterBytes) splits = 1;     // one arrival counter per group
    if (splits > 1) {
        // longest walk of the batch, in prefix tiles, for `parts` workgroups per group
        auto longest = [&](int parts, bool own) {
            int worst = 0;
            for (int s = 0; s < sa.n_seq; ++s) {
                const int nTp = (sa.prefix_len[s] + kKeysPerTile - 1) / kKeysPerTile;
                const int nTt = (sa.node_off[s + 1] - sa.node_off[s] + kKeysPerTile - 1) / kKeysPerTile;
                const int n_pref = own ? parts - 1 : parts;
                const int share = (((nTp + n_pref - 1) / n_pref) + 1) & ~1;
                const int last = max(0, min(nTp - (parts - 1) * share, share));       // prefix tiles of the last split
                worst = max(worst, own ? max(min(share, nTp), 2 * nTt) : max(min(share, nTp), last + 2 * nTt));
            }
            return worst;
        };
        const int shared = longest(splits, false);
        if (splits + 1 <= min(by_work, 8) && longest(splits + 1, true) < shared) { ++splits; tree_split = 1; }
        else if (splits >= 3 && longest(splits, true) < shared) tree_split = 1;
    }
#ifdef DYSPEC_TUNING
    if (const char* e = getenv("DYSPEC_ATTN_SPLITS")) splits = max(1, min(atoi(e), min(min_tiles / 2, 32)));
    if (const char* e = getenv("DYSPEC_ATTN_TREE_SPLIT")) tree_split = atoi(e) != 0 && splits > 1;
    if ((size_t)groups * sizeof(unsigned) > kAttnCounterBytes) { splits = 1; tree_split = 0; }
#endif
    return { splits, tree_split };
}

size_t tree_attn_workspace_bytes(const SeqArgs& sa, int Hq, int Hkv, int d, int layers)
{
    const int splits = tree_attn_cut(sa, Hq, Hkv, layers).splits;
    if (splits <= 1) return 0;
    const size_t groups = (size_t)row_tiles(sa, Hq / Hkv, nullptr) * Hkv * layers;
    return kAttnCounterBytes + groups * splits * attn_part_words(d) * sizeof(uint32_t);
}

hipError_t launch_tree_attn_mfma(AttnArgs a, const SeqArgs& sa, void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    const int tiles = row_tiles(sa, a.Hq / a.Hkv, a.tile_off);
    if (tiles == 0) return hipSuccess;
    const AttnCut cut = tree_attn_cut(sa, a.Hq, a.Hkv, a.layers);
    a.splits = cut.splits; a.tree_split = cut.tree_split;
    const size_t need = tree_attn_workspace_bytes(sa, a.Hq, a.Hkv, a.d, a.layers);
    if (a.splits > 1 && (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<size_t>(workspace) & 15)))
        a.splits = 1, a.tree_split = 0;                        // no room for partial results: one workgroup walks it all
    if (a.splits > 1) {
        a.counters = static_cast<unsigned*>(workspace);
        a.part = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + kAttnCounterBytes);
    }
    return a.d == 128 ? launch_one<128, kQB>(a, sa, tiles, stream) : launch_one<64, kQB>(a, sa, tiles, stream);
}

#ifdef DYSPEC_STAMPS
extern "C" int dyspec_debug_read(void* host_dst)
{
    // copies the stamps out (waits for the device) and clears them for the next run
    unsigned zero = 0;
    static unsigned long long z[8192 * 8];
    hipError_t e = hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_stamps), sizeof(z));
    if (e == hipSuccess) e = hipMemcpyToSymbol(HIP_SYMBOL(g_stamp_slot), &zero, sizeof(zero));
    if (e == hipSuccess) e = hipMemcpyToSymbol(HIP_SYMBOL(g_stamps), z, sizeof(z));
    return (int)e;
}
#endif

}  // namespace dyspec
