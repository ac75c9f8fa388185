// fp64 softmax weights of a draft row for the tree builders (Algorithms 1 and 2): the weight
// of a token, and a workgroup's 4-token segment sums of a row with some tokens left out.
#pragma once
#include "vocab_common.h"

namespace dyspec {

// exp(z) for z <= 0 (a softmax weight relative to the row maximum) in fp64: z = n ln2 + r with
// |r| <= ln2 / 2, exp(r) by its Taylor series to degree 13 (truncation below 1e-17), scaled by
// 2^n.  Arguments below the normal range, -inf included, give 0.
static __device__ __attribute__((noinline)) double exp_nonpos(double z)
{
    if (!(z >= -708.0)) return 0.0;
    const double n = rint(z * 1.4426950408889634074);
    double r = fma(n, -6.93147180369123816490e-01, z);
    r = fma(n, -1.90821492927058770002e-10, r);
    double p = 1.0 / 6227020800.0;
    p = fma(p, r, 1.0 / 479001600.0);
    p = fma(p, r, 1.0 / 39916800.0);
    p = fma(p, r, 1.0 / 3628800.0);
    p = fma(p, r, 1.0 / 362880.0);
    p = fma(p, r, 1.0 / 40320.0);
    p = fma(p, r, 1.0 / 5040.0);
    p = fma(p, r, 1.0 / 720.0);
    p = fma(p, r, 1.0 / 120.0);
    p = fma(p, r, 1.0 / 24.0);
    p = fma(p, r, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)n);
}

// exp_nonpos of four arguments at once: the same operations per argument, interleaved so that
// the four dependent chains overlap (every result equals exp_nonpos of its argument bit for bit)
__device__ __forceinline__ void exp_nonpos_x4(const double (&z)[4], double (&out)[4])
{
    constexpr double c[13] = { 1.0 / 479001600.0, 1.0 / 39916800.0, 1.0 / 3628800.0, 1.0 / 362880.0, 1.0 / 40320.0, 1.0 / 5040.0,
                               1.0 / 720.0, 1.0 / 120.0, 1.0 / 24.0, 1.0 / 6.0, 0.5, 1.0, 1.0 };
    double n[4], r[4], p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        n[e] = rint(z[e] * 1.4426950408889634074);
        r[e] = fma(n[e], -6.93147180369123816490e-01, z[e]);
        r[e] = fma(n[e], -1.90821492927058770002e-10, r[e]);
        p[e] = 1.0 / 6227020800.0;
    }
#pragma unroll
    for (int k = 0; k < 13; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e) p[e] = fma(p[e], r[e], c[k]);
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = z[e] >= -708.0 ? ldexp(p[e], (int)n[e]) : 0.0;
}

// weight of one token of a row: exp(x / T - m), m the row maximum over T
__device__ __forceinline__ double token_weight(float x, double inv_temp, double m)
{
    return exp_nonpos(fma((double)x, inv_temp, -m));
}

// Row maximum (over T) and the 4-token segment sums of this thread for one draft row, with
// the tokens flagged in `gone` (bit 4j+e) left out.
template <bool VEC>
__device__ __forceinline__ void row_segment_sums(const float* __restrict__ row, int V, double inv_temp, uint64_t gone,
                                                 float* fred, double* m_out, double (&seg)[kMaxSeg])
{
    float x[kMaxSeg][4];
    load_row<VEC, float>(row, V, x);
    float mx[1] = { -INFINITY };
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx[0] = fmaxf(mx[0], x[j][e]);
    block_max<1>(mx, fred);
    const double m = (double)mx[0] * inv_temp;
    *m_out = m;
#pragma unroll
    for (int j = 0; j < kMaxSeg; ++j) {
        double z[4], w4[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) z[e] = fma((double)x[j][e], inv_temp, -m);
        exp_nonpos_x4(z, w4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool live = tok_index(j, e) < V && !((gone >> (4 * j + e)) & 1ull);
            if (!live) w4[e] = 0.0;
        }
        seg[j] = (w4[0] + w4[1]) + (w4[2] + w4[3]);
    }
}

}  // namespace dyspec
