// Vocabulary-row helpers for the tree builder and the verifier.
//
// A row of V <= 16*2048 values is held in registers by a 512-thread workgroup: thread t
// owns elements {2048*j + 4*t + e : j < 16, e < 4}, so every wave reads whole 1 KiB
// stretches of the row with 128-bit loads, and token order is (segment j, thread t,
// element e) lexicographic -- the order the inverse CDF walks.
#pragma once
#include "dyspec_device.h"

namespace dyspec {

__device__ __forceinline__ int tok_index(int j, int e) { return j * kSeg + 4 * (int)threadIdx.x + e; }

// Logit tables are fp32 or bf16.  A bf16 value is the upper half of the fp32 with the same value.
__device__ __forceinline__ float logit_to_float(float x) { return x; }
__device__ __forceinline__ float logit_to_float(__bf16 x) { return (float)x; }
__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// Load one logits row; positions >= V read as -inf.  VEC: V % 4 == 0 (a thread's four tokens are
// one aligned 16-byte (fp32) or 8-byte (bf16) load).
template <bool VEC, typename T>
__device__ __forceinline__ void load_row(const T* __restrict__ row, int V, float (&x)[kMaxSeg][4])
{
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) {
        const int i0 = tok_index(j, 0);
        if (VEC) {
            if (i0 < V) {
                if constexpr (sizeof(T) == 4) {
                    const float4 v = *reinterpret_cast<const float4*>(row + i0);
                    x[j][0] = v.x; x[j][1] = v.y; x[j][2] = v.z; x[j][3] = v.w;
                } else {
                    const uint2 v = *reinterpret_cast<const uint2*>(row + i0);
                    x[j][0] = bf16_bits_to_float(v.x & 0xffffu); x[j][1] = bf16_bits_to_float(v.x >> 16);
                    x[j][2] = bf16_bits_to_float(v.y & 0xffffu); x[j][3] = bf16_bits_to_float(v.y >> 16);
                }
            } else {
                x[j][0] = x[j][1] = x[j][2] = x[j][3] = -INFINITY;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) x[j][e] = (i0 + e < V) ? logit_to_float(row[i0 + e]) : -INFINITY;
        }
    }
}

struct CdfScratch {
    double red[kWaves * kMaxSeg];
    int owner;
    int last;
    int y;
    double wy;
};

// Inverse CDF over non-negative weights, in token order (segment j, thread t, element e):
// the smallest token index y with sum_{x<=y} w[x] > u*W, W = total weight; zero-weight tokens
// are never returned.  The row is known through its 4-token sums: seg[j] of thread t is
// weight(j,0) + ... + weight(j,3) for tokens tok_index(j, 0..3), tot[j] the sum of seg[j] over
// the workgroup.
struct SegPick {
    int js;             // segment that holds the crossing
    double cum_js;      // weight of the segments before it
    double W, target;   // total weight, u * W
};

// First level: which segment.  Pure function of the totals, the same in every thread.
__device__ __forceinline__ SegPick pick_segment(const double (&tot)[kMaxSeg], double u)
{
    SegPick pk;
    double W = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) W += tot[j];
    pk.W = W;
    pk.target = u * W;
    int js = -1, jlast = 0;
    double cum = 0.0, cum_js = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) {
        if (js < 0 && cum + tot[j] > pk.target) { js = j; cum_js = cum; }
        if (tot[j] > 0.0) jlast = j;
        if (js < 0) cum += tot[j];
    }
    if (js < 0) {                      // rounding at the very top: take the last live segment
        js = jlast;
        cum_js = 0.0;
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j) if (j < jlast) cum_js += tot[j];
    }
    pk.js = js;
    pk.cum_js = cum_js;
    return pk;
}

// Second level: scan of the threads' sums of segment pk.js (mine), then the owning thread
// walks its four tokens (weight(j, e), asked only by that thread, j == pk.js).  Needs W > 0.
// Every thread gets y and w[y].
template <typename F>
__device__ __forceinline__ int finish_inverse_cdf(const SegPick& pk, double mine, CdfScratch* sc, double* wy_out, F&& weight)
{
    if (threadIdx.x == 0) { sc->owner = 0x7fffffff; sc->last = -1; sc->y = -1; sc->wy = 0.0; }
    double excl;
    const double incl = block_scan_inclusive<double>(mine, sc->red, &excl);   // two barriers: the reset is visible
    if (mine > 0.0 && pk.cum_js + incl > pk.target) atomicMin(&sc->owner, (int)threadIdx.x);
    if (mine > 0.0) atomicMax(&sc->last, (int)threadIdx.x);
    __syncthreads();
    const int owner = (sc->owner != 0x7fffffff) ? sc->owner : sc->last;
    if ((int)threadIdx.x == owner) {
        double run = pk.cum_js + excl;
        int y = -1, ylast = -1;
        double wy = 0.0, wlast = 0.0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double we = weight(pk.js, e);
            run += we;
            if (we > 0.0) { ylast = tok_index(pk.js, e); wlast = we; }
            if (y < 0 && we > 0.0 && run > pk.target) { y = tok_index(pk.js, e); wy = we; }
        }
        if (y < 0) { y = ylast; wy = wlast; }
        sc->y = y;
        sc->wy = wy;
    }
    __syncthreads();
    const int y_all = sc->y;
    *wy_out = sc->wy;
    __syncthreads();                   // scratch may be reset by the next call from here on
    return y_all;
}

// Both levels from the threads' segment sums.  Every thread gets y (or -1 when W == 0), W
// and w[y].
template <typename F>
__device__ __forceinline__ int block_inverse_cdf_seg(const double (&seg_in)[kMaxSeg], double u, CdfScratch* sc,
                                                     double* W_out, double* wy_out, F&& weight)
{
    double tot[kMaxSeg];
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) tot[j] = seg_in[j];
    block_sum<double, kMaxSeg>(tot, sc->red);
    const SegPick pk = pick_segment(tot, u);
    *W_out = pk.W;
    if (!(pk.W > 0.0)) { *wy_out = 0.0; return -1; }
    double mine = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) if (j == pk.js) mine = seg_in[j];
    return finish_inverse_cdf(pk, mine, sc, wy_out, weight);
}

}  // namespace dyspec
