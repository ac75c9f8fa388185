// extern "C" boundary: host-side validation, then kernel launches.  See include/dyspec.h
// for the contract of every entry point.
#include <atomic>

#include "dyspec_device.h"

namespace dyspec {

static dyspec_status check_batch(const dyspec_batch* b, bool need_prefix, SeqArgs* sa, int max_nodes = DYSPEC_MAX_NODES)
{
    if (!b || !b->node_offset) return DYSPEC_BAD_ARG;
    if (b->n_seq < 1 || b->n_seq > DYSPEC_MAX_SEQ) return DYSPEC_BAD_SHAPE;
    if (need_prefix && (!b->prefix_len || !b->kv_offset)) return DYSPEC_BAD_ARG;
    if (b->node_offset[0] != 0) return DYSPEC_BAD_SHAPE;
    sa->n_seq = b->n_seq;
    for (int s = 0; s < b->n_seq; ++s) {
        const int n = b->node_offset[s + 1] - b->node_offset[s];
        if (n < 1 || n > max_nodes) return DYSPEC_BAD_SHAPE;
        sa->node_off[s] = b->node_offset[s];
        sa->prefix_len[s] = 0;
        sa->kv_off[s] = 0;
        sa->temp_d[s] = sa->temp_t[s] = 1.0f;
        if (need_prefix) {
            if (b->prefix_len[s] < 0 || b->kv_offset[s] < 0) return DYSPEC_BAD_SHAPE;
            if (b->kv_offset[s + 1] < b->kv_offset[s] + b->prefix_len[s]) return DYSPEC_BAD_SHAPE;
            sa->prefix_len[s] = b->prefix_len[s];
            sa->kv_off[s] = b->kv_offset[s];
        }
    }
    sa->node_off[b->n_seq] = b->node_offset[b->n_seq];
    return DYSPEC_OK;
}

// Address alignment the kernels' vector loads rely on (16-byte pieces of tensors and logit rows,
// 8-byte mask words, 4-byte tree arrays); checked here so that a misaligned pointer is an error
// code and never a faulting load.
static bool aligned(const void* p, size_t n) { return (reinterpret_cast<size_t>(p) & (n - 1)) == 0; }

static bool tree_aligned(const dyspec_tree* t)
{
    return aligned(t->parent, 4) && aligned(t->token, 4) && aligned(t->sib_rank, 4) && aligned(t->first_child, 4) &&
           aligned(t->next_sibling, 4) && aligned(t->depth, 4);
}

static bool tree_ok(const dyspec_tree* t)
{
    return t && t->parent && t->token && t->sib_rank && t->first_child && t->next_sibling && t->depth;
}

static int mask_words_of(const dyspec_batch* b)
{
    int mx = 1;
    for (int s = 0; s < b->n_seq; ++s) mx = max(mx, b->node_offset[s + 1] - b->node_offset[s]);
    return (mx + 63) / 64;
}

}  // namespace dyspec

using namespace dyspec;

// ---- the variant for callers that cannot allocate: partial results go to a static device array
//
// In host code the array's name is only a stand-in for the symbol; its device address comes from
// hipGetSymbolAddress, once per device (every GPU holds its own copy at its own address), and that
// address is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[DYSPEC_STATIC_SCRATCH_BYTES];

static hipError_t static_scratch_address(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> per_device[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = per_device[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // with `dev` current: this device's copy
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev].store(p, std::memory_order_release); // two racing first calls store the same address
    }
    *out = p;
    return hipSuccess;
}

extern "C" {

int32_t dyspec_mask_words(const dyspec_batch* batch)
{
    SeqArgs sa;
    if (check_batch(batch, false, &sa) != DYSPEC_OK) return 0;
    return mask_words_of(batch);
}

size_t dyspec_workspace_bytes(int32_t which, const dyspec_batch* batch, int32_t, int32_t n_q_heads, int32_t n_kv_heads,
                              int32_t head_dim)
{
    // the tree builder keeps the rows' segment sums there; tree attention its partial results
    // when it splits the prefix over several workgroups; verification needs none
    SeqArgs sa;
    if (which == DYSPEC_WS_BUILD_TREE)
        return check_batch(batch, false, &sa, DYSPEC_MAX_BUILD_NODES) == DYSPEC_OK ? build_tree_workspace_bytes(sa.node_off[sa.n_seq]) : 0;
    if (which == DYSPEC_WS_TREE_ATTN) {
        if (check_batch(batch, true, &sa) != DYSPEC_OK || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads != 0 ||
            (head_dim != 64 && head_dim != 128))
            return 0;
        return tree_attn_workspace_bytes(sa, n_q_heads, n_kv_heads, head_dim, 1);
    }
    return 0;
}

size_t dyspec_tree_attn_layers_workspace_bytes(const dyspec_batch* batch, int32_t n_layers, int32_t n_q_heads,
                                               int32_t n_kv_heads, int32_t head_dim)
{
    SeqArgs sa;
    if (check_batch(batch, true, &sa) != DYSPEC_OK || n_layers < 1 || n_q_heads < 1 || n_kv_heads < 1 ||
        n_q_heads % n_kv_heads != 0 || (head_dim != 64 && head_dim != 128))
        return 0;
    return tree_attn_workspace_bytes(sa, n_q_heads, n_kv_heads, head_dim, n_layers);
}

dyspec_status dyspec_init(void)
{
    void* scratch_address = nullptr;
    if (prepare_tree_attn() != hipSuccess || prepare_build_tree() != hipSuccess || prepare_build_threshold() != hipSuccess || prepare_verify() != hipSuccess ||
        static_scratch_address(&scratch_address) != hipSuccess)
        return DYSPEC_HIP_ERROR;
    return DYSPEC_OK;
}

const char* dyspec_status_string(dyspec_status s)
{
    switch (s) {
        case DYSPEC_OK: return "ok";
        case DYSPEC_BAD_ARG: return "bad argument";
        case DYSPEC_BAD_SHAPE: return "bad shape";
        case DYSPEC_UNSUPPORTED: return "unsupported dtype, head_dim or vocabulary";
        case DYSPEC_WORKSPACE_TOO_SMALL: return "workspace too small";
        case DYSPEC_HIP_ERROR: return "HIP error";
        default: return "unknown status";
    }
}

dyspec_status dyspec_build_tree(const float* draft_logits, int32_t vocab, const dyspec_batch* batch,
                                const float* draft_temp, uint64_t seed, const dyspec_tree* tree,
                                float* est_value, uint64_t* anc_mask, int32_t* n_built,
                                void* workspace, size_t workspace_bytes, void* hip_stream)
{
    SeqArgs sa;
    const dyspec_status st = check_batch(batch, false, &sa, DYSPEC_MAX_BUILD_NODES);
    if (st != DYSPEC_OK) return st;
    if (!draft_logits || !draft_temp || !tree_ok(tree) || !est_value || !anc_mask || !n_built) return DYSPEC_BAD_ARG;
    if (vocab < 1) return DYSPEC_BAD_ARG;
    if (vocab > DYSPEC_MAX_VOCAB) return DYSPEC_UNSUPPORTED;
    if (!aligned(draft_logits, 16) || !tree_aligned(tree) || !aligned(est_value, 4) || !aligned(anc_mask, 8) ||
        !aligned(n_built, 4) || (workspace && !aligned(workspace, 8)))
        return DYSPEC_BAD_ARG;
    for (int s = 0; s < sa.n_seq; ++s) {
        if (!(draft_temp[s] > 0.0f)) return DYSPEC_BAD_ARG;
        sa.temp_d[s] = draft_temp[s];
    }
    const hipError_t e = launch_build_tree(draft_logits, vocab, sa, seed, *tree, est_value, anc_mask,
                                           mask_words_of(batch), n_built, workspace, workspace_bytes,
                                           static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DYSPEC_OK : DYSPEC_HIP_ERROR;
}

size_t dyspec_build_tree_threshold_workspace_bytes(const dyspec_batch* batch)
{
    SeqArgs sa;
    return check_batch(batch, false, &sa, DYSPEC_MAX_BUILD_NODES) == DYSPEC_OK ? build_threshold_workspace_bytes(sa) : 0;
}

dyspec_status dyspec_build_tree_threshold(const float* draft_logits, int32_t vocab, const dyspec_batch* batch,
                                          const float* draft_temp, const double* threshold, uint64_t seed,
                                          const dyspec_tree* tree, float* est_value, uint64_t* anc_mask,
                                          int32_t* n_built, int32_t* n_levels, void* workspace,
                                          size_t workspace_bytes, void* hip_stream)
{
    SeqArgs sa;
    const dyspec_status st = check_batch(batch, false, &sa, DYSPEC_MAX_BUILD_NODES);
    if (st != DYSPEC_OK) return st;
    if (!draft_logits || !draft_temp || !threshold || !tree_ok(tree) || !est_value || !anc_mask || !n_built)
        return DYSPEC_BAD_ARG;
    if (vocab < 1) return DYSPEC_BAD_ARG;
    if (vocab > DYSPEC_MAX_VOCAB) return DYSPEC_UNSUPPORTED;
    if (!aligned(draft_logits, 16) || !tree_aligned(tree) || !aligned(est_value, 4) || !aligned(anc_mask, 8) ||
        !aligned(n_built, 4) || (workspace && !aligned(workspace, 8)))
        return DYSPEC_BAD_ARG;
    for (int s = 0; s < sa.n_seq; ++s) {
        if (!(draft_temp[s] > 0.0f) || !(threshold[s] > 0.0)) return DYSPEC_BAD_ARG;
        sa.temp_d[s] = draft_temp[s];
    }
    if (!workspace || workspace_bytes < build_threshold_workspace_bytes(sa)) return DYSPEC_WORKSPACE_TOO_SMALL;
    int levels = 0;
    const hipError_t e = launch_build_threshold(draft_logits, vocab, sa, threshold, seed, *tree, est_value, anc_mask,
                                                mask_words_of(batch), n_built, &levels, workspace,
                                                static_cast<hipStream_t>(hip_stream));
    if (n_levels) *n_levels = levels;
    return e == hipSuccess ? DYSPEC_OK : DYSPEC_HIP_ERROR;
}

dyspec_status dyspec_dfs_reorder(const dyspec_batch* batch, const dyspec_tree* tree, const dyspec_tree* tree_out,
                                 int32_t* order, uint64_t* anc_mask_out, void* hip_stream)
{
    SeqArgs sa;
    const dyspec_status st = check_batch(batch, false, &sa);
    if (st != DYSPEC_OK) return st;
    if (!tree_ok(tree) || !tree_ok(tree_out) || !order || !anc_mask_out) return DYSPEC_BAD_ARG;
    if (tree->parent == tree_out->parent || tree->token == tree_out->token || tree->first_child == tree_out->first_child ||
        tree->next_sibling == tree_out->next_sibling || tree->sib_rank == tree_out->sib_rank || tree->depth == tree_out->depth)
        return DYSPEC_BAD_ARG;                                   // not in place
    if (!tree_aligned(tree) || !tree_aligned(tree_out) || !aligned(order, 4) || !aligned(anc_mask_out, 8)) return DYSPEC_BAD_ARG;
    const hipError_t e = launch_dfs_reorder(sa, *tree, *tree_out, order, anc_mask_out, mask_words_of(batch),
                                            static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DYSPEC_OK : DYSPEC_HIP_ERROR;
}

// Shared body of the one-layer and the stacked-layers call.  Strides are in bytes.
static dyspec_status tree_attn_common(const void* q, const void* k_prefix, const void* v_prefix,
                                      const void* k_tree, const void* v_tree, const uint64_t* anc_mask,
                                      const dyspec_batch* batch, int32_t n_layers, long long q_stride,
                                      long long kvp_stride, long long kvt_stride, int32_t n_q_heads,
                                      int32_t n_kv_heads, int32_t head_dim, int32_t dtype, float softmax_scale,
                                      void* out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    SeqArgs sa;
    const dyspec_status st = check_batch(batch, true, &sa);
    if (st != DYSPEC_OK) return st;
    if (!q || !k_tree || !v_tree || !anc_mask || !out) return DYSPEC_BAD_ARG;
    bool any_prefix = false;
    for (int s = 0; s < sa.n_seq; ++s) any_prefix |= sa.prefix_len[s] > 0;
    if (any_prefix && (!k_prefix || !v_prefix)) return DYSPEC_BAD_ARG;
    if (n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads != 0) return DYSPEC_BAD_SHAPE;
    // the kernels address a sequence's query rows, and the 64 key rows of a tile, with 32-bit byte offsets
    if ((long long)DYSPEC_MAX_NODES * n_q_heads * (head_dim > 0 ? head_dim : 1) * 4 > 0x7fffffffLL) return DYSPEC_BAD_SHAPE;
    if (!(softmax_scale > 0.0f)) return DYSPEC_BAD_ARG;
    // 16-byte pieces of every tensor are loaded at once (and moved to LDS without passing through
    // registers); mask rows are 8-byte words; the workspace holds float4 partial rows
    if (!aligned(q, 16) || !aligned(k_prefix, 16) || !aligned(v_prefix, 16) || !aligned(k_tree, 16) || !aligned(v_tree, 16) ||
        !aligned(out, 16) || !aligned(anc_mask, 8) || (workspace && !aligned(workspace, 16)))
        return DYSPEC_BAD_ARG;
    bool force_simple = false;
    if (dtype == DYSPEC_BF16 || dtype == DYSPEC_BF16_WAVE) {
        force_simple = dtype == DYSPEC_BF16_WAVE;
        dtype = DYSPEC_BF16;
        if (!force_simple && head_dim != 64 && head_dim != 128) return DYSPEC_UNSUPPORTED;
        if (force_simple && (head_dim < 4 || head_dim > 256 || head_dim % 4)) return DYSPEC_UNSUPPORTED;
    } else if (dtype == DYSPEC_F32) {
        if (head_dim < 4 || head_dim > 256 || head_dim % 4) return DYSPEC_UNSUPPORTED;   // rows are read 4 values at a time
    } else {
        return DYSPEC_UNSUPPORTED;
    }
    AttnArgs a;
    a.q = q; a.kp = k_prefix; a.vp = v_prefix; a.kt = k_tree; a.vt = v_tree;
    a.mask = anc_mask; a.out = out;
    a.mask_words = mask_words_of(batch);
    a.Hq = n_q_heads; a.Hkv = n_kv_heads; a.d = head_dim; a.scale = softmax_scale;
    a.splits = 1; a.tree_split = 0; a.part = nullptr; a.counters = nullptr;
    a.layers = n_layers; a.q_stride = q_stride; a.kvp_stride = kvp_stride; a.kvt_stride = kvt_stride;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool one_launch = dtype == DYSPEC_BF16 && !force_simple;      // the matrix-core kernel takes a layer plane
    if (one_launch || n_layers == 1)
        return launch_tree_attn(a, sa, dtype, force_simple, workspace, workspace_bytes, stream) == hipSuccess
                   ? DYSPEC_OK : DYSPEC_HIP_ERROR;
    auto at = [](const void* p, long long off) { return p ? static_cast<const char*>(p) + off : nullptr; };
    for (int l = 0; l < n_layers; ++l) {                                 // the per-row kernels: one launch per layer
        AttnArgs b = a;
        b.layers = 1;
        b.q = at(q, l * q_stride); b.out = static_cast<char*>(out) + l * q_stride;
        b.kp = at(k_prefix, l * kvp_stride); b.vp = at(v_prefix, l * kvp_stride);
        b.kt = at(k_tree, l * kvt_stride); b.vt = at(v_tree, l * kvt_stride);
        if (launch_tree_attn(b, sa, dtype, force_simple, nullptr, 0, stream) != hipSuccess) return DYSPEC_HIP_ERROR;
    }
    return DYSPEC_OK;
}

dyspec_status dyspec_tree_attn(const void* q, const void* k_prefix, const void* v_prefix,
                               const void* k_tree, const void* v_tree, const uint64_t* anc_mask,
                               const dyspec_batch* batch, int32_t n_q_heads, int32_t n_kv_heads,
                               int32_t head_dim, int32_t dtype, float softmax_scale, void* out,
                               void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return tree_attn_common(q, k_prefix, v_prefix, k_tree, v_tree, anc_mask, batch, 1, 0, 0, 0, n_q_heads,
                            n_kv_heads, head_dim, dtype, softmax_scale, out, workspace, workspace_bytes, hip_stream);
}

dyspec_status dyspec_tree_attn_static_scratch(const void* q, const void* k_prefix, const void* v_prefix,
                                              const void* k_tree, const void* v_tree, const uint64_t* anc_mask,
                                              const dyspec_batch* batch, int32_t n_q_heads, int32_t n_kv_heads,
                                              int32_t head_dim, int32_t dtype, float softmax_scale, void* out,
                                              void* hip_stream)
{
    // how much the split this batch would get needs; 0 (no split, or a dtype / shape the checks
    // below refuse anyway) needs no scratch at all
    const size_t need = dtype == DYSPEC_BF16 ? dyspec_workspace_bytes(DYSPEC_WS_TREE_ATTN, batch, 0, n_q_heads, n_kv_heads, head_dim) : 0;
    if (need > DYSPEC_STATIC_SCRATCH_BYTES) return DYSPEC_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    if (need > 0 && static_scratch_address(&ws) != hipSuccess) return DYSPEC_HIP_ERROR;
    return tree_attn_common(q, k_prefix, v_prefix, k_tree, v_tree, anc_mask, batch, 1, 0, 0, 0, n_q_heads,
                            n_kv_heads, head_dim, dtype, softmax_scale, out, ws, need, hip_stream);
}

dyspec_status dyspec_tree_attn_layers(const void* q, const void* k_prefix, const void* v_prefix,
                                      const void* k_tree, const void* v_tree, const uint64_t* anc_mask,
                                      const dyspec_batch* batch, int32_t n_layers, int64_t q_layer_stride,
                                      int64_t kv_prefix_layer_stride, int64_t kv_tree_layer_stride,
                                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t dtype,
                                      float softmax_scale, void* out, void* workspace, size_t workspace_bytes,
                                      void* hip_stream)
{
    if (n_layers < 1 || n_layers > 65535) return DYSPEC_BAD_SHAPE;
    if (q_layer_stride < 0 || kv_prefix_layer_stride < 0 || kv_tree_layer_stride < 0) return DYSPEC_BAD_ARG;
    const long long elt = dtype == DYSPEC_F32 ? 4 : 2;
    // every layer's tensors stay 16-byte aligned
    if ((q_layer_stride * elt) % 16 || (kv_prefix_layer_stride * elt) % 16 || (kv_tree_layer_stride * elt) % 16)
        return DYSPEC_BAD_ARG;
    return tree_attn_common(q, k_prefix, v_prefix, k_tree, v_tree, anc_mask, batch, n_layers, q_layer_stride * elt,
                            kv_prefix_layer_stride * elt, kv_tree_layer_stride * elt, n_q_heads, n_kv_heads,
                            head_dim, dtype, softmax_scale, out, workspace, workspace_bytes, hip_stream);
}

static dyspec_status verify_common(const void* draft_logits, const void* target_logits, bool bf16_logits, int32_t vocab,
                                   const dyspec_batch* batch, const dyspec_tree* tree, const float* draft_temp,
                                   const float* target_temp, uint64_t seed, int32_t emit_bonus,
                                   float* row_stats, float* accept_ratio, int32_t* accepted_nodes,
                                   int32_t* n_accepted, int32_t* final_token, float* min_margin, void* hip_stream)
{
    SeqArgs sa;
    const dyspec_status st = check_batch(batch, false, &sa);
    if (st != DYSPEC_OK) return st;
    if (!draft_logits || !target_logits || !tree_ok(tree) || !draft_temp || !target_temp || !row_stats ||
        !accept_ratio || !accepted_nodes || !n_accepted || !final_token || !min_margin)
        return DYSPEC_BAD_ARG;
    if (vocab < 1) return DYSPEC_BAD_ARG;
    if (vocab > DYSPEC_MAX_VOCAB) return DYSPEC_UNSUPPORTED;
    if (!aligned(draft_logits, 16) || !aligned(target_logits, 16) || !tree_aligned(tree) || !aligned(row_stats, 16) ||
        !aligned(accept_ratio, 4) || !aligned(accepted_nodes, 4) || !aligned(n_accepted, 4) || !aligned(final_token, 4) ||
        !aligned(min_margin, 4))
        return DYSPEC_BAD_ARG;
    for (int s = 0; s < sa.n_seq; ++s) {
        if (!(draft_temp[s] > 0.0f) || !(target_temp[s] >= 0.0f)) return DYSPEC_BAD_ARG;   // target 0 = argmax row
        sa.temp_d[s] = draft_temp[s];
        sa.temp_t[s] = target_temp[s];
    }
    const hipError_t e = launch_verify(draft_logits, target_logits, bf16_logits, vocab, sa, *tree, seed, emit_bonus != 0,
                                       row_stats, accept_ratio, accepted_nodes, n_accepted, final_token,
                                       min_margin, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DYSPEC_OK : DYSPEC_HIP_ERROR;
}

dyspec_status dyspec_verify(const float* draft_logits, const float* target_logits, int32_t vocab,
                            const dyspec_batch* batch, const dyspec_tree* tree, const float* draft_temp,
                            const float* target_temp, uint64_t seed, int32_t emit_bonus,
                            float* row_stats, float* accept_ratio, int32_t* accepted_nodes,
                            int32_t* n_accepted, int32_t* final_token, float* min_margin,
                            void*, size_t, void* hip_stream)
{
    return verify_common(draft_logits, target_logits, false, vocab, batch, tree, draft_temp, target_temp, seed, emit_bonus,
                         row_stats, accept_ratio, accepted_nodes, n_accepted, final_token, min_margin, hip_stream);
}

dyspec_status dyspec_verify_bf16(const void* draft_logits, const void* target_logits, int32_t vocab,
                                 const dyspec_batch* batch, const dyspec_tree* tree, const float* draft_temp,
                                 const float* target_temp, uint64_t seed, int32_t emit_bonus,
                                 float* row_stats, float* accept_ratio, int32_t* accepted_nodes,
                                 int32_t* n_accepted, int32_t* final_token, float* min_margin,
                                 void*, size_t, void* hip_stream)
{
    return verify_common(draft_logits, target_logits, true, vocab, batch, tree, draft_temp, target_temp, seed, emit_bonus,
                         row_stats, accept_ratio, accepted_nodes, n_accepted, final_token, min_margin, hip_stream);
}

}  // extern "C"
