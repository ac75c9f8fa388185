// Vocabulary-row helpers for the tree builder and the verifier.
//
// A row of V <= 16*2048 values is held in registers by a 512-thread workgroup: thread t
// owns elements {4096*j + 4*t + e : j < 8, e < 4}, so every wave reads whole 1 KiB
// stretches of the row with 128-bit loads, and token order is (segment j, thread t,
// element e) lexicographic -- the order the inverse CDF walks.
#pragma once
#include "dyspec_device.h"

namespace dyspec {

__device__ __forceinline__ int tok_index(int j, int e) { return j * kSeg + 4 * (int)threadIdx.x + e; }

// Load one logits row; positions >= V read as -inf.  VEC: V % 4 == 0 (row is 16-byte aligned).
template <bool VEC>
__device__ __forceinline__ void load_row(const float* __restrict__ row, int V, float (&x)[kMaxSeg][4])
{
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) {
        const int i0 = tok_index(j, 0);
        if (VEC) {
            if (i0 < V) {
                const float4 v = *reinterpret_cast<const float4*>(row + i0);
                x[j][0] = v.x; x[j][1] = v.y; x[j][2] = v.z; x[j][3] = v.w;
            } else {
                x[j][0] = x[j][1] = x[j][2] = x[j][3] = -INFINITY;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) x[j][e] = (i0 + e < V) ? row[i0 + e] : -INFINITY;
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

// Inverse CDF over non-negative weights held one 4-token segment sum per (thread, j):
// seg[j] = weight(j,0) + ... + weight(j,3) for tokens tok_index(j, 0..3).  Returns the smallest
// token index y with sum_{x<=y} w[x] > u*W, W = total weight; zero-weight tokens are never
// returned.  Every thread gets y (or -1 when W == 0), W and w[y].  Only the thread that owns
// the crossing segment asks for single weights again (weight(j, e), j uniform in its loop).
template <typename F>
__device__ __forceinline__ int block_inverse_cdf_seg(const double (&seg_in)[kMaxSeg], double u, CdfScratch* sc,
                                                     double* W_out, double* wy_out, F&& weight)
{
    double seg[kMaxSeg];
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) seg[j] = seg_in[j];
    if (threadIdx.x == 0) { sc->owner = 0x7fffffff; sc->last = -1; sc->y = -1; sc->wy = 0.0; }
    block_sum<double, kMaxSeg>(seg, sc->red);

    double W = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) W += seg[j];
    *W_out = W;
    if (!(W > 0.0)) { *wy_out = 0.0; return -1; }
    const double target = u * W;

    int js = -1, jlast = 0;
    double cum = 0.0, cum_js = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) {
        if (js < 0 && cum + seg[j] > target) { js = j; cum_js = cum; }
        if (seg[j] > 0.0) jlast = j;
        if (js < 0) cum += seg[j];
    }
    if (js < 0) {                      // rounding at the very top: take the last live segment
        js = jlast;
        cum_js = 0.0;
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j) if (j < jlast) cum_js += seg[j];
    }
    double mine = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) if (j == js) mine = seg_in[j];

    double excl;
    const double incl = block_scan_inclusive<double>(mine, sc->red, &excl);
    if (mine > 0.0 && cum_js + incl > target) atomicMin(&sc->owner, (int)threadIdx.x);
    if (mine > 0.0) atomicMax(&sc->last, (int)threadIdx.x);
    __syncthreads();
    const int owner = (sc->owner != 0x7fffffff) ? sc->owner : sc->last;
    if ((int)threadIdx.x == owner) {
        double run = cum_js + excl;
        int y = -1, ylast = -1;
        double wy = 0.0, wlast = 0.0;
#pragma unroll
        for (int j = 0; j < kMaxSeg; ++j) {
            if (j != js) continue;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double we = weight(j, e);
                run += we;
                if (we > 0.0) { ylast = tok_index(j, e); wlast = we; }
                if (y < 0 && we > 0.0 && run > target) { y = tok_index(j, e); wy = we; }
            }
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

// The same over a register-resident row of weights.
template <typename T>
__device__ __forceinline__ int block_inverse_cdf(const T (&w)[kMaxSeg][4], double u,
                                                 CdfScratch* sc, double* W_out, double* wy_out)
{
    double seg[kMaxSeg];
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j)
        seg[j] = ((double)w[j][0] + (double)w[j][1]) + ((double)w[j][2] + (double)w[j][3]);
    return block_inverse_cdf_seg(seg, u, sc, W_out, wy_out, [&](int j, int e) {
        double r = 0.0;
#pragma unroll
        for (int jj = 0; jj < kMaxSeg; ++jj)
#pragma unroll
            for (int ee = 0; ee < 4; ++ee) if (jj == j && ee == e) r = (double)w[jj][ee];
        return r;
    });
}

}  // namespace dyspec
