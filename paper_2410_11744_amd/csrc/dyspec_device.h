// Device-side helpers shared by the gfx950 kernels: Philox4x32-10 draws named by the
// sibling-rank path, and workgroup reductions / scans for 1024-thread workgroups.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/dyspec.h"

namespace dyspec {

constexpr int kWave = 64;
constexpr int kBlock = 512;                   // threads per workgroup of the vocabulary kernels
constexpr int kWaves = kBlock / kWave;        // 8
constexpr int kSeg = 4 * kBlock;              // tokens per vocabulary segment (float4 per thread)
constexpr int kMaxSeg = DYSPEC_MAX_VOCAB / kSeg;   // 16

// Per-sequence scalars, passed to kernels by value.
struct SeqArgs {
    int n_seq;
    int node_off[DYSPEC_MAX_SEQ + 1];
    int prefix_len[DYSPEC_MAX_SEQ];
    long long kv_off[DYSPEC_MAX_SEQ];
    float temp_d[DYSPEC_MAX_SEQ];
    float temp_t[DYSPEC_MAX_SEQ];
};

// Arguments of the tree-attention kernels.
struct AttnArgs {
    const void* q; const void* kp; const void* vp; const void* kt; const void* vt;
    const uint64_t* mask; void* out;
    int mask_words, Hq, Hkv, d;
    float scale;
    int tile_off[DYSPEC_MAX_SEQ + 1];      // first row tile of each sequence (matrix-core kernel)
    // prefix split of the matrix-core kernel: split z of `splits` takes every sequence's prefix
    // tiles [z*c, (z+1)*c) (c: an even share), the last one the tree as well; with `tree_split`
    // the last split takes the tree alone and the prefix is dealt to the others.  With splits > 1
    // every workgroup leaves its normalised rows (bf16) and their (max, sum) in `part`, in the
    // register layout of the kernel, and bumps the arrival counter of its (layer, row tile, KV
    // head); the workgroup that arrives last merges all parts and writes the output rows.
    int splits, tree_split;
    uint32_t* part;                        // [layers * tiles * Hkv][splits][attn_part_words(d)]
    unsigned* counters;                    // [layers * tiles * Hkv], zero between launches
    // stacked layers (matrix-core kernel): layer l = blockIdx.z reads q/out, prefix K/V and
    // tree K/V at byte offsets l * stride from the base pointers; the mask is shared.
    int layers;
    long long q_stride, kvp_stride, kvt_stride;
};

// Launchers (one per source file); each returns the launch status.
hipError_t launch_build_tree(const float* draft_logits, int V, const SeqArgs& sa, uint64_t seed,
                             const dyspec_tree& tree, float* est_value, uint64_t* anc_mask,
                             int mask_words, int* n_built, void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t build_tree_workspace_bytes(int total_rows);
hipError_t launch_build_threshold(const float* draft_logits, int V, const SeqArgs& sa, const double* threshold,
                                  uint64_t seed, const dyspec_tree& tree, float* est_value, uint64_t* anc_mask,
                                  int mask_words, int* n_built, int* n_levels, void* workspace, hipStream_t stream);
size_t build_threshold_workspace_bytes(const SeqArgs& sa);
hipError_t launch_dfs_reorder(const SeqArgs& sa, const dyspec_tree& in, const dyspec_tree& out, int* order,
                              uint64_t* mask_out, int mask_words, hipStream_t stream);
hipError_t launch_verify(const void* draft_logits, const void* target_logits, bool bf16_logits, int V,
                         const SeqArgs& sa, const dyspec_tree& tree, uint64_t seed, int emit_bonus,
                         float* row_stats, float* accept_ratio, int* accepted_nodes, int* n_accepted,
                         int* final_token, float* min_margin, hipStream_t stream);
hipError_t launch_tree_attn(AttnArgs a, const SeqArgs& sa, int dtype, bool per_wave, void* workspace, size_t workspace_bytes,
                            hipStream_t stream);
hipError_t launch_tree_attn_mfma(AttnArgs a, const SeqArgs& sa, void* workspace, size_t workspace_bytes, hipStream_t stream);
// 32-bit words one workgroup of the matrix-core kernel leaves per split: 4 row blocks x 64 lanes x
// (d/4 packed bf16 pairs + max + sum)
constexpr int attn_part_words(int d) { return 4 * 64 * (d / 4 + 2); }
constexpr size_t kAttnCounterBytes = DYSPEC_ATTN_COUNTER_BYTES;     // arrival counters at the head of the workspace
// how the matrix-core kernel would like to cut this batch's walks, and the workspace that takes
struct AttnCut { int splits, tree_split; };
AttnCut tree_attn_cut(const SeqArgs& sa, int Hq, int Hkv, int layers);
size_t tree_attn_workspace_bytes(const SeqArgs& sa, int Hq, int Hkv, int d, int layers);

// Raises a kernel's dynamic-LDS limit to `bytes`, once per device (`done`: one bit per device,
// owned by the call site).  Touching the kernel this way also makes the runtime load its code.
inline hipError_t raise_dynamic_lds_once(const void* kernel, int bytes, std::atomic<unsigned long long>& done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// One-time set-up of each source file's kernels on the current device (what dyspec_init calls;
// the launchers do the same at first use).
hipError_t prepare_tree_attn();
hipError_t prepare_build_tree();
hipError_t prepare_build_threshold();
hipError_t prepare_verify();

enum : uint32_t { KIND_PATH = 0, KIND_BUILD = 1, KIND_ACCEPT = 2, KIND_RESID = 3 };

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies with the
// multipliers of the 4x32 variant, key bumped by the Weyl constants between rounds.
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
        c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
        k.x += 0x9E3779B9u;
        k.y += 0xBB67AE85u;
    }
    return c;
}

__device__ __forceinline__ uint2 seed_key(uint64_t seed)
{
    return make_uint2((uint32_t)seed, (uint32_t)(seed >> 32));
}

// Path key of the root of sequence `seq`, and of the child of rank `rank` under `pk`.
__device__ __forceinline__ uint2 root_key(uint32_t seq) { return make_uint2(seq, 0u); }

__device__ __forceinline__ uint2 child_key(uint64_t seed, uint2 pk, uint32_t rank)
{
    const uint4 w = philox4x32_10(make_uint4(pk.x, pk.y, rank, KIND_PATH), seed_key(seed));
    return make_uint2(w.x, w.y);
}

// Uniform in [0,1) with 24 bits; exact in fp32 and fp64.
__device__ __forceinline__ float u01(uint64_t seed, uint2 pk, uint32_t rank, uint32_t kind)
{
    const uint4 w = philox4x32_10(make_uint4(pk.x, pk.y, rank, kind), seed_key(seed));
    return (float)(w.x >> 8) * (1.0f / 16777216.0f);
}

// ---------------------------------------------------------------- wave primitives

template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// ---------------------------------------------------------------- workgroup primitives
// All take a scratch array in LDS with at least kWaves * K entries and must be called by
// every thread of a kBlock-thread workgroup.  They end with a barrier, so the scratch may
// be reused right after they return.

template <int K>
__device__ __forceinline__ void block_max(float (&v)[K], float* scratch)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const float m = wave_max(v[k]);
        if (lane == 0) scratch[wave * K + k] = m;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        float m = scratch[k];
        for (int w = 1; w < kWaves; ++w) m = fmaxf(m, scratch[w * K + k]);
        v[k] = m;
    }
    __syncthreads();
}

template <typename T, int K>
__device__ __forceinline__ void block_sum(T (&v)[K], T* scratch)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const T s = wave_sum(v[k]);
        if (lane == 0) scratch[wave * K + k] = s;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        T s = scratch[k];
        for (int w = 1; w < kWaves; ++w) s += scratch[w * K + k];   // fixed order: same in every thread
        v[k] = s;
    }
    __syncthreads();
}

// Inclusive scan over the threads of the workgroup in thread order; returns the inclusive
// prefix of the caller and writes the exclusive one.
template <typename T>
__device__ __forceinline__ T block_scan_inclusive(T v, T* scratch, T* exclusive)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    T inc = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const T up = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += up;
    }
    if (lane == kWave - 1) scratch[wave] = inc;
    __syncthreads();
    T base = 0;
    for (int w = 0; w < wave; ++w) base += scratch[w];
    __syncthreads();
    const T below = __shfl_up(inc, 1, kWave);
    *exclusive = base + (lane ? below : (T)0);
    return base + inc;
}

// Sequence that owns packed row `row`.
__device__ __forceinline__ int find_seq(const SeqArgs& sa, int row)
{
    int s = 0;
    while (s + 1 < sa.n_seq && row >= sa.node_off[s + 1]) ++s;
    return s;
}

}  // namespace dyspec
