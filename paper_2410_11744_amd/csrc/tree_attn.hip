// Tree attention (Section 2, "Tree Attention"; Appendix C) for gfx950: launcher, and the
// per-wavefront kernel (one wavefront per (row, head), any head_dim <= 256, fp32 or bf16
// storage with fp32 arithmetic) that serves fp32 tensors and odd head sizes.  The bf16
// matrix-core kernel lives in tree_attn_mfma.hip.
#include "dyspec_device.h"

namespace dyspec {

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

hipError_t launch_tree_attn(AttnArgs a, const SeqArgs& sa, int dtype, bool per_wave, void* workspace, size_t workspace_bytes,
                            hipStream_t stream)
{
    const int total_rows = sa.node_off[sa.n_seq];
    if (dtype == DYSPEC_BF16 && !per_wave && (a.d == 128 || a.d == 64))
        return launch_tree_attn_mfma(a, sa, workspace, workspace_bytes, stream);
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
