// Tree attention (Section 2, "Tree Attention"; Appendix C) for gfx950: launcher, and the
// per-row kernel (one workgroup per (row, head), any head_dim <= 256 in steps of 4, fp32 or bf16
// storage with fp32 arithmetic) that serves fp32 tensors and odd head sizes.  The bf16
// matrix-core kernel lives in tree_attn_mfma.hip.
#include "dyspec_device.h"

namespace dyspec {

// =====================================================================================
// Per-row kernel: one workgroup of four wavefronts per (row, head); online softmax in fp32.
//
// The keys of the row's walk are dealt to the wavefronts in runs of 64, and a wavefront's 64 lanes
// are four groups of 16.  Group g takes keys g, g+4, g+8, ... of the wavefront's run
// (prefix keys, then the tree keys the ancestor mask admits); inside a group lane i holds the
// 16-byte pieces i, i+16, ... of the head dimension (CH pieces, head_dim <= 64*CH), so a key or
// value row is read by 16 lanes as one contiguous run.  A score is the group's dot product
// (four DPP adds); every group keeps its own running (max, sum, output); the groups of a wavefront are
// merged with lane exchanges and the four wavefronts through LDS at the end.  16 / CH keys per group are in flight per trip to memory; the row's mask words are
// fetched once (lane w holds word w) so that no trip waits for a mask read first.
// =====================================================================================

template <typename T> struct Piece4;
template <> struct Piece4<float> {
    static __device__ __forceinline__ float4 load(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ __forceinline__ void store(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
};
template <> struct Piece4<__bf16> {
    static __device__ __forceinline__ float4 load(const __bf16* p)
    {
        const uint2 w = *reinterpret_cast<const uint2*>(p);
        return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xffff0000u));
    }
    static __device__ __forceinline__ void store(__bf16* p, float4 v)
    {
        typedef float f2 __attribute__((ext_vector_type(2)));
        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
        const f2 lo = { v.x, v.y }, hi = { v.z, v.w };
        uint2 w;
        w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, b2));
        w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, b2));
        *reinterpret_cast<uint2*>(p) = w;
    }
};

// sum over the 16 lanes of a group (a DPP row), the same in each of them
__device__ __forceinline__ float group_sum(float x)
{
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, false));   // row_half_mirror
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, false));   // row_mirror
    return x;
}

constexpr int kSimpleWaves = 4;

template <typename T, int CH>
__global__ __launch_bounds__(kSimpleWaves* kWave) void tree_attn_simple_kernel(AttnArgs a, SeqArgs sa)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = (int)(blockIdx.x / (unsigned)a.Hq), h = (int)(blockIdx.x % (unsigned)a.Hq);   // grid = rows * heads
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
    static_assert(DYSPEC_MAX_NODES / 64 <= kWave, "a row's mask words fit one per lane");
    const uint64_t mword = lane < a.mask_words ? a.mask[(size_t)row * a.mask_words + lane] : 0ull;
    const int grp = lane >> 4, li = lane & 15;
    constexpr int kKeysInFlight = 16 / CH;   // keys per group and trip to memory
    const int pieces = d / 4;                                  // 16-byte (fp32) or 8-byte (bf16) pieces per row

    float4 q4[CH];
    bool have[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        have[c] = li + 16 * c < pieces;
        q4[c] = have[c] ? Piece4<T>::load(qrow + 4 * (li + 16 * c)) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float4 acc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    float m = -INFINITY, l = 0.0f;

    const int total = P + N;
    for (int k0 = wave * 4 * kKeysInFlight; k0 < total; k0 += kSimpleWaves * 4 * kKeysInFlight) {
        float4 kq[kKeysInFlight][CH], vq[kKeysInFlight][CH];
        bool vis[kKeysInFlight];
#pragma unroll
        for (int u = 0; u < kKeysInFlight; ++u) {
            const int k = k0 + 4 * u + grp;
            const int i = k - P;
            const uint64_t mw = __shfl(mword, i >= 0 && i < N ? i >> 6 : 0, kWave);   // every lane takes part
            vis[u] = k < P || (k < total && ((mw >> (i & 63)) & 1ull));
            // a key the row does not see is read from tree row 0 (the root, a key of every row)
            // and weighted 0; a piece beyond head_dim is read from piece 0 and meets q = 0
            const size_t off = (k < P ? (size_t)k : (size_t)(vis[u] ? i : 0)) * kv_row;
            const T* krow = (k < P ? kp : kt) + off;
            const T* vrow = (k < P ? vp : vt) + off;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int piece = have[c] ? li + 16 * c : 0;
                kq[u][c] = Piece4<T>::load(krow + 4 * piece);
                vq[u][c] = Piece4<T>::load(vrow + 4 * piece);
            }
        }
        // scores of the trip first (independent chains), then one rescale for all of them
        float sc[kKeysInFlight];
        float m_new = m;
#pragma unroll
        for (int u = 0; u < kKeysInFlight; ++u) {
            float dot = 0.0f;
#pragma unroll
            for (int c = 0; c < CH; ++c)
                dot += (q4[c].x * kq[u][c].x + q4[c].y * kq[u][c].y) + (q4[c].z * kq[u][c].z + q4[c].w * kq[u][c].w);
            const float g = group_sum(dot);                    // every lane takes part
            sc[u] = vis[u] ? g * a.scale : -INFINITY;
            m_new = fmaxf(m_new, sc[u]);
        }
        if (m_new != -INFINITY) {                              // uniform over the group: it has seen a key
            const float corr = expf(m - m_new);                // 0 while m is still -inf
            l *= corr;
#pragma unroll
            for (int c = 0; c < CH; ++c) { acc[c].x *= corr; acc[c].y *= corr; acc[c].z *= corr; acc[c].w *= corr; }
#pragma unroll
            for (int u = 0; u < kKeysInFlight; ++u) {
                const float p = expf(sc[u] - m_new);           // 0 for a key the row does not see
                l += p;
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    acc[c].x = fmaf(p, vq[u][c].x, acc[c].x); acc[c].y = fmaf(p, vq[u][c].y, acc[c].y);
                    acc[c].z = fmaf(p, vq[u][c].z, acc[c].z); acc[c].w = fmaf(p, vq[u][c].w, acc[c].w);
                }
            }
            m = m_new;
        }
    }
    // ---- merge the wave's four groups (a group that saw no key has m = -inf, weight 0) ...
    float M = fmaxf(m, __shfl_xor(m, 16, kWave));
    M = fmaxf(M, __shfl_xor(M, 32, kWave));
    const float w = m == -INFINITY ? 0.0f : expf(m - M);
    float L = l * w;
    L += __shfl_xor(L, 16, kWave);
    L += __shfl_xor(L, 32, kWave);
    float o[CH][4];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        o[c][0] = acc[c].x * w; o[c][1] = acc[c].y * w; o[c][2] = acc[c].z * w; o[c][3] = acc[c].w * w;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[c][e] += __shfl_xor(o[c][e], 16, kWave);
            o[c][e] += __shfl_xor(o[c][e], 32, kWave);
        }
    }
    // ---- ... then the four waves, through LDS: wave 0 adds them up and writes the row
    __shared__ float part_ml[kSimpleWaves][2];
    __shared__ float4 part_o[kSimpleWaves][CH * 16];
    if (grp == 0) {
        if (li == 0) { part_ml[wave][0] = M; part_ml[wave][1] = L; }
#pragma unroll
        for (int c = 0; c < CH; ++c) part_o[wave][li + 16 * c] = make_float4(o[c][0], o[c][1], o[c][2], o[c][3]);
    }
    __syncthreads();
    if (wave != 0 || grp != 0) return;
    float Mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < kSimpleWaves; ++v) Mx = fmaxf(Mx, part_ml[v][0]);
    float wv[kSimpleWaves], Lx = 0.0f;
#pragma unroll
    for (int v = 0; v < kSimpleWaves; ++v) {
        wv[v] = part_ml[v][0] == -INFINITY ? 0.0f : expf(part_ml[v][0] - Mx);
        Lx += wv[v] * part_ml[v][1];
    }
    const float inv = 1.0f / Lx;                               // the root sees itself: Lx > 0
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        if (!have[c]) continue;
        float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int v = 0; v < kSimpleWaves; ++v) {
            const float4 t = part_o[v][li + 16 * c];
            r.x = fmaf(wv[v], t.x, r.x); r.y = fmaf(wv[v], t.y, r.y); r.z = fmaf(wv[v], t.z, r.z); r.w = fmaf(wv[v], t.w, r.w);
        }
        Piece4<T>::store(static_cast<T*>(a.out) + ((size_t)row * a.Hq + h) * d + 4 * (li + 16 * c),
                         make_float4(r.x * inv, r.y * inv, r.z * inv, r.w * inv));
    }
}

template <typename T>
static void launch_simple(const AttnArgs& a, const SeqArgs& sa, int blocks, hipStream_t stream)
{
    const int ch = (a.d / 4 + 15) / 16;                        // pieces per lane: head_dim <= 64, 128, 192, 256
    if (ch <= 1) tree_attn_simple_kernel<T, 1><<<blocks, kSimpleWaves * kWave, 0, stream>>>(a, sa);
    else if (ch == 2) tree_attn_simple_kernel<T, 2><<<blocks, kSimpleWaves * kWave, 0, stream>>>(a, sa);
    else if (ch == 3) tree_attn_simple_kernel<T, 3><<<blocks, kSimpleWaves * kWave, 0, stream>>>(a, sa);
    else tree_attn_simple_kernel<T, 4><<<blocks, kSimpleWaves * kWave, 0, stream>>>(a, sa);
}

hipError_t launch_tree_attn(AttnArgs a, const SeqArgs& sa, int dtype, bool per_wave, void* workspace, size_t workspace_bytes,
                            hipStream_t stream)
{
    const int total_rows = sa.node_off[sa.n_seq];
    if (dtype == DYSPEC_BF16 && !per_wave && (a.d == 128 || a.d == 64))
        return launch_tree_attn_mfma(a, sa, workspace, workspace_bytes, stream);
    if (total_rows == 0) return hipSuccess;
    const long long groups = (long long)total_rows * a.Hq;    // one workgroup per (row, head)
    if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
    const int blocks = (int)groups;
    if (dtype == DYSPEC_BF16)
        launch_simple<__bf16>(a, sa, blocks, stream);
    else
        launch_simple<float>(a, sa, blocks, stream);
    return hipGetLastError();
}

}  // namespace dyspec
