/*
 * dyspec.h -- C ABI of the MI355X (gfx950) library for one DySpec speculative step
 * (arXiv 2410.11744): greedy token-tree construction, tree-masked attention and
 * multi-candidate tree verification.
 *
 * Conventions shared by every entry point
 *  - Pointers marked DEVICE address HBM of the current HIP device; pointers marked HOST
 *    address ordinary host memory that is read before the call returns.  The caller owns
 *    every buffer; the library allocates nothing and keeps no state between calls.
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *    stream); calls return without synchronising.  Two calls that write the same buffers
 *    race unless ordered by the stream.  Apart from dyspec_build_tree_threshold (which
 *    waits for each level) a call enqueues kernel launches only -- no allocation, memset,
 *    copy or wait -- so, after dyspec_init() or one plain call on the device, calls may be
 *    recorded into a HIP graph on a capturing stream and replayed.
 *  - Errors are return codes (< 0).  Arguments are validated on the host before anything
 *    is launched; a call that returns an error has launched nothing.
 *  - Alignment of DEVICE pointers is part of that validation (DYSPEC_BAD_ARG otherwise):
 *    attention tensors, logit tables, row_stats and the tree-attention workspace 16 bytes;
 *    ancestor masks and the builders' workspaces 8 bytes; every other array 4 bytes.
 *  - A batch holds n_seq independent sequences packed back to back.  Sequence s owns tree
 *    rows [node_offset[s], node_offset[s+1]) of every per-node array and prefix rows
 *    [kv_offset[s], kv_offset[s] + prefix_len[s]) of k_prefix / v_prefix.  Row 0 of each
 *    tree is the root: the last committed token, whose logits open the tree
 *    (Section 4.2, first paragraph).  Node indices stored in the arrays (parent, links,
 *    accepted_nodes, mask bits) are LOCAL to the sequence.
 *  - Uniform random numbers come from Philox4x32-10 (Salmon et al., SC'11) with key =
 *    seed and a counter that names each draw by the path of sibling ranks from the root,
 *    so results do not depend on node numbering or on which kernel makes the draw.
 */
#ifndef DYSPEC_H
#define DYSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t dyspec_status;
enum {
    DYSPEC_OK = 0,
    DYSPEC_BAD_ARG = -1,             /* null pointer, non-positive size, temperature <= 0 ... */
    DYSPEC_BAD_SHAPE = -2,           /* offsets not increasing, heads not divisible, ...      */
    DYSPEC_UNSUPPORTED = -3,         /* dtype / head_dim / vocabulary outside the built kernels */
    DYSPEC_WORKSPACE_TOO_SMALL = -4,
    DYSPEC_HIP_ERROR = -5            /* a HIP call failed; hipGetLastError() still holds it   */
};

/* Tensor element types of dyspec_tree_attn.  DYSPEC_BF16_WAVE: bf16 storage handled by the
 * one-workgroup-per-(row, head) kernel (fp32 arithmetic, any head_dim <= 256 that is a multiple of 4) instead of the
 * matrix-core kernel. */
enum { DYSPEC_F32 = 0, DYSPEC_BF16 = 1, DYSPEC_BF16_WAVE = 0x101 };

#define DYSPEC_MAX_SEQ 64            /* sequences per call                                */
#define DYSPEC_MAX_NODES 2048        /* tree rows per sequence, root included (attention, reorder, verify) */
#define DYSPEC_MAX_BUILD_NODES 1024  /* ... for the two tree builders, whose per-tree state lives in LDS   */
#define DYSPEC_MAX_VOCAB 32768       /* vocabulary handled by the build / verify kernels  */

/* Ragged batch description; all three arrays are HOST memory. */
typedef struct {
    int32_t n_seq;                   /* 1 .. DYSPEC_MAX_SEQ                               */
    const int32_t* node_offset;      /* [n_seq+1] increasing, node_offset[0] = 0          */
    const int32_t* prefix_len;       /* [n_seq]   >= 0                                    */
    const int64_t* kv_offset;        /* [n_seq+1] first prefix row of each sequence       */
} dyspec_batch;

/* A packed batch of token trees; every array is DEVICE memory of length node_offset[n_seq].
 * Children of a node are linked in the order they were sampled, which is the order
 * verification must try them (Algorithm 3, loop over CurrentNode.branches). */
typedef struct {
    int32_t* parent;                 /* -1 for the root and for rows that were not built  */
    int32_t* token;                  /* -1 for the root                                   */
    int32_t* sib_rank;               /* 0 for a first child, 1 for the next sampling ...  */
    int32_t* first_child;            /* -1 = leaf                                         */
    int32_t* next_sibling;           /* -1 = last sampled child                           */
    int32_t* depth;                  /* 0 for the root                                    */
} dyspec_tree;

/* Words per row of the ancestor bitmask for this batch: ceil(max_s N_s / 64). */
int32_t dyspec_mask_words(const dyspec_batch* batch);

/* Bytes of DEVICE workspace the named call can use for this batch (0 = none). */
enum { DYSPEC_WS_BUILD_TREE = 0, DYSPEC_WS_TREE_ATTN = 1, DYSPEC_WS_VERIFY = 2 };
#define DYSPEC_ATTN_COUNTER_BYTES 4096   /* head of a tree-attention workspace: see dyspec_tree_attn */
size_t dyspec_workspace_bytes(int32_t which, const dyspec_batch* batch, int32_t vocab,
                              int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim);

const char* dyspec_status_string(dyspec_status s);

/*
 * dyspec_init -- optional one-time set-up on the CURRENT device: has the runtime load the
 * kernels, raises their dynamic-LDS limits, takes the address of the static scratch array.
 * Every entry point does what it needs of this at its first use; calling dyspec_init first
 * moves those few milliseconds out of the first calls of a latency-sensitive loop.  Launches
 * nothing, allocates nothing; idempotent and safe to call from several threads.
 */
dyspec_status dyspec_init(void);

/*
 * dyspec_build_tree -- greedy fixed-budget construction of the draft token tree
 * (Algorithm 1; Section 4.2; Appendix A.1) plus the tree-attention mask (Section 2).
 *
 * For each sequence, N = node_offset[s+1]-node_offset[s] rows are built, the root
 * included.  Starting from the single slot (parent = root, value 1), the slot with the
 * largest estimated value v is taken (earliest-opened slot on a tie); a token y is drawn
 * from the parent's draft distribution with the parent's earlier children removed and the
 * rest renormalised (R); the node is appended; the slots "next sampling at the same
 * position" with value v*(1-R[y]) and "first child of the new node" with value v*R[y] are
 * opened (slots of value 0 are not).  Draft distributions are softmax(draft_logits[i]/T_d),
 * where row i is the distribution that FOLLOWS node i (creation index): the table stands in
 * for the draft model call of Algorithm 1.  Arithmetic on values and distributions is fp64.
 * y is the smallest index whose cumulative residual weight exceeds u * (total weight),
 * u in [0,1) with 24 random bits.
 *
 *   draft_logits  DEVICE [sum N, vocab] fp32, row-major, base 16-byte aligned
 *   draft_temp    HOST   [n_seq] > 0
 *   tree          DEVICE outputs (all six arrays)
 *   est_value     DEVICE [sum N] fp32: v of the slot each node was drawn from (root: 1)
 *   anc_mask      DEVICE [sum N, mask_words] u64: bit i of row j set iff local node i is an
 *                 ancestor of local node j or i == j
 *   n_built       DEVICE [n_seq]: rows actually built (< N only if no slot of positive
 *                 value is left); later rows keep parent = token = -1 and their own mask bit
 *   workspace     DEVICE, dyspec_workspace_bytes(DYSPEC_WS_BUILD_TREE, ...) bytes, 8-byte
 *                 aligned, contents overwritten (about 4.2 KB per row): every row's
 *                 maximum and the totals of its 16 vocabulary segments, computed for all
 *                 rows at once before the serial expansion, and one bit per token drawn
 *                 from the row so far; a draw then touches a 16th of the parent's row.
 *                 NULL or fewer bytes: the expansion makes a pass over the parent's whole
 *                 row at every draw instead (same arithmetic, same tree, several times
 *                 slower).
 * vocab <= DYSPEC_MAX_VOCAB, N <= DYSPEC_MAX_BUILD_NODES (DYSPEC_BAD_SHAPE beyond).
 */
dyspec_status dyspec_build_tree(const float* draft_logits, int32_t vocab,
                                const dyspec_batch* batch, const float* draft_temp,
                                uint64_t seed, const dyspec_tree* tree, float* est_value,
                                uint64_t* anc_mask, int32_t* n_built,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * dyspec_build_tree_threshold -- construction of the draft token tree with a threshold
 * (Algorithm 2; Section 4.4, Appendix A.2), the level-by-level form of dyspec_build_tree.
 *
 * Per sequence, starting from the root alone (value 1): every node i of the current level
 * with value v_i >= t reads its draft row D = softmax(draft_logits[i]/T) and, while v_i >= t
 * and rows are left, draws y from D (inverse CDF as in dyspec_build_tree, the draw named by
 * the node's sibling-rank path and the number of children it already has), appends a child
 * with token y, estimated value v_i and own value v_i*D[y], then sets v_i <- v_i*(1-D[y]),
 * D[y] <- 0, D <- norm(D).  The children of a level are the next level.  The loop condition
 * is read as "at or above the threshold" (the listing prints the opposite sign; the text says
 * nodes above the threshold are extended).  Rows are numbered in creation order: level by
 * level, parents in row order, children in sampling order; construction stops when the
 * sequence's N rows (root included) exist.  With t = the smallest est_value a run of
 * dyspec_build_tree produced, the same tree results (Appendix A.1) when both give a node
 * the same draft row; here a node reads the row of its own index, so the two calls agree on
 * tables whose rows are alike.  Nodes of a level are expanded in parallel, one workgroup each.
 *
 *   threshold     HOST [n_seq] > 0 (the paper suggests about 1/N)
 *   n_levels      HOST out, may be NULL: levels expanded (the number of draft model calls
 *                 the paper's loop would make), the widest sequence counting
 *   workspace     DEVICE, 8-byte aligned, dyspec_build_tree_threshold_workspace_bytes()
 *                 bytes, REQUIRED (DYSPEC_WORKSPACE_TOO_SMALL otherwise)
 *   all other arguments, and the limits on vocab and N, as for dyspec_build_tree.
 * The call copies one small record per level back to the host and waits for it (it sizes
 * the next level's launch), so it returns with the tree complete and cannot be captured
 * in a graph.
 */
dyspec_status dyspec_build_tree_threshold(const float* draft_logits, int32_t vocab,
                                          const dyspec_batch* batch, const float* draft_temp,
                                          const double* threshold, uint64_t seed,
                                          const dyspec_tree* tree, float* est_value,
                                          uint64_t* anc_mask, int32_t* n_built, int32_t* n_levels,
                                          void* workspace, size_t workspace_bytes, void* hip_stream);
size_t dyspec_build_tree_threshold_workspace_bytes(const dyspec_batch* batch);

/*
 * dyspec_dfs_reorder -- block-sparsity friendly token order (Appendix "Block-Sparsity
 * Friendly Token Order"): renames the nodes of every built tree by their position in the
 * depth-first pre-order walk that visits children in sampling order.  Subtrees become
 * contiguous runs of rows, parents still precede children, and the ancestor mask of the renamed
 * tree has fewer non-empty 32x32 blocks for tree attention to visit.  Rows that were never
 * attached (n_built < N) follow the tree in index order.
 *
 *   tree           DEVICE inputs (all six arrays, as written by dyspec_build_tree)
 *   tree_out       DEVICE outputs, six arrays distinct from the inputs: the renamed tree
 *   order          DEVICE [sum N] i32: order[node_offset[s] + new] = old local index; the caller
 *                  gathers token-aligned tensors (q, k_tree, v_tree, logit rows) with it
 *   anc_mask_out   DEVICE [sum N, mask_words] u64: ancestor mask of the renamed tree
 * Verification of the renamed tree reads logit rows by the new indices (gathered tables), and
 * Philox draws are named by paths of sibling ranks, so its outcome does not change.
 */
dyspec_status dyspec_dfs_reorder(const dyspec_batch* batch, const dyspec_tree* tree,
                                 const dyspec_tree* tree_out, int32_t* order,
                                 uint64_t* anc_mask_out, void* hip_stream);

/*
 * dyspec_tree_attn -- one layer of tree attention (Section 2, "Tree Attention";
 * Appendix C for the block-sparse treatment of the tree part).
 *
 * For every tree row j and query head h:
 *   out[j,h,:] = softmax_k( scale * <q[j,h,:], K[k, h/G, :]> ) . V[k, h/G, :]
 * over all prefix keys of the sequence and over the tree keys i whose bit is set in
 * anc_mask row j; G = n_q_heads / n_kv_heads.
 *
 *   q, out            DEVICE [sum N, n_q_heads, head_dim]
 *   k_prefix,v_prefix DEVICE [kv rows, n_kv_heads, head_dim]
 *   k_tree, v_tree    DEVICE [sum N, n_kv_heads, head_dim]
 *   anc_mask          DEVICE [sum N, mask_words] as written by dyspec_build_tree.  Bit i of row j
 *                     may be set only for i <= j (an ancestor is created before its descendants,
 *                     so its row index is smaller, in creation order and in depth-first order
 *                     alike); the matrix-core path does not look at tree keys past the largest
 *                     row of a tile, so bits above the diagonal are ignored there
 *   dtype             DYSPEC_F32 (any head_dim <= 256, multiple of 4) or DYSPEC_BF16
 *                     (head_dim 64 or 128; matrix-core path, fp32 accumulation)
 * All tensors are dense row-major and 16-byte aligned (checked: DYSPEC_BAD_ARG).
 *   workspace         DEVICE, 16-byte aligned, dyspec_workspace_bytes(DYSPEC_WS_TREE_ATTN, ...)
 *                     bytes.  Non-zero only for batches whose (row tiles) x (KV heads) leave most
 *                     of the chip idle: the bf16 path then splits every prefix over several
 *                     workgroups; each leaves its share of every row there (bf16) and the one
 *                     that finishes last merges them, in the same launch.  The first
 *                     DYSPEC_ATTN_COUNTER_BYTES of the workspace are the arrival counters of
 *                     that hand-over: they must be ZERO when a call starts and every call
 *                     leaves them zero again, so a workspace is cleared once, after it is
 *                     allocated (hipMemset), and never again; the rest is overwritten.  NULL or
 *                     fewer bytes: no split (same result up to the bf16 rounding of the parts).  A
 *                     non-NULL workspace that is not 16-byte aligned is DYSPEC_BAD_ARG.
 */
dyspec_status dyspec_tree_attn(const void* q, const void* k_prefix, const void* v_prefix,
                               const void* k_tree, const void* v_tree,
                               const uint64_t* anc_mask, const dyspec_batch* batch,
                               int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                               int32_t dtype, float softmax_scale, void* out,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * dyspec_tree_attn_static_scratch -- dyspec_tree_attn for callers that cannot allocate device
 * memory and have none to hand over as a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same operation, arguments, kernels and results as
 * dyspec_tree_attn called with a workspace of dyspec_workspace_bytes(DYSPEC_WS_TREE_ATTN, ...)
 * bytes; the partial results of a split prefix go to an array of DYSPEC_STATIC_SCRATCH_BYTES that
 * is part of the library's device image (each GPU the library runs on holds its copy until the
 * process ends).  The call allocates and frees nothing.  A batch whose split needs more than
 * DYSPEC_STATIC_SCRATCH_BYTES is refused with DYSPEC_WORKSPACE_TOO_SMALL (nothing launched).
 * Every call on one GPU uses the same array: calls that overlap on one GPU (two streams, two
 * threads) race; order them, or give the overlapping ones dyspec_tree_attn with workspaces of
 * their own.  The arrival counters at the head of the array start as zeros with the device image
 * and every call leaves them zero; nothing else in it has to survive from one call to the next.
 */
#define DYSPEC_STATIC_SCRATCH_BYTES (8u << 20)
dyspec_status dyspec_tree_attn_static_scratch(const void* q, const void* k_prefix, const void* v_prefix,
                                              const void* k_tree, const void* v_tree,
                                              const uint64_t* anc_mask, const dyspec_batch* batch,
                                              int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                              int32_t dtype, float softmax_scale, void* out,
                                              void* hip_stream);

/*
 * dyspec_tree_attn_layers -- dyspec_tree_attn for n_layers stacked layers in one call
 * (the same operation as above, Section 2 "Tree Attention", once per layer; the tree and
 * its mask are the same in every layer of one speculative step, the tensors are not).
 * Layer l reads q, k_prefix/v_prefix and k_tree/v_tree at element offsets l * q_layer_stride,
 * l * kv_prefix_layer_stride and l * kv_tree_layer_stride from the base pointers and writes
 * out at l * q_layer_stride; within a layer the layout is that of dyspec_tree_attn.  Strides
 * are >= 0 and keep every layer 16-byte aligned.  The bf16 matrix-core path runs all layers
 * in ONE launch (workgroups of all layers fill the chip together, so short prefixes need
 * no split and pay one launch latency); other dtypes launch once per layer.  This is for
 * callers that hold all layers' tensors at once (benchmarks, layer-parallel schedules);
 * a model that computes layer l+1's Q from layer l's output calls dyspec_tree_attn.
 *   workspace  as for dyspec_tree_attn (its first DYSPEC_ATTN_COUNTER_BYTES zero when the call
 *              starts), dyspec_tree_attn_layers_workspace_bytes() bytes.
 *   n_layers   1 .. 65535
 */
dyspec_status dyspec_tree_attn_layers(const void* q, const void* k_prefix, const void* v_prefix,
                                      const void* k_tree, const void* v_tree,
                                      const uint64_t* anc_mask, const dyspec_batch* batch,
                                      int32_t n_layers, int64_t q_layer_stride,
                                      int64_t kv_prefix_layer_stride, int64_t kv_tree_layer_stride,
                                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                      int32_t dtype, float softmax_scale, void* out,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);
size_t dyspec_tree_attn_layers_workspace_bytes(const dyspec_batch* batch, int32_t n_layers,
                                               int32_t n_q_heads, int32_t n_kv_heads,
                                               int32_t head_dim);

/*
 * dyspec_verify -- vocabulary softmax of every tree row and multi-candidate tree
 * rejection sampling (Algorithm 3; Appendix A.3; Section 2 for the one-candidate rule).
 *
 * Data-parallel part, one workgroup per tree row p: the maximum and the sum of exponentials
 * of draft_logits[p]/T_d and of target_logits[p]/T_t (row_stats), i.e. the normalisers of
 * D = softmax(draft_logits[p]/T_d) and R = softmax(target_logits[p]/T_t).
 * Walk, one workgroup per sequence, from the root: for each child n of the current node in
 * sampling order, with token y: draw c uniform in [0,1); accept iff c < R[y]/D[y]
 * (equivalently c*D[y] < R[y]); on a reject R <- norm(max(R-D,0)) with D as it stands, then
 * D[y] <- 0 and D <- norm(D); the scan of the children ends early when D is empty.  Move to
 * the accepted child; when none is accepted sample the step's last token from R; when the
 * walk reaches a leaf sample it from the leaf's target row if emit_bonus != 0 (the printed
 * algorithm returns without it: final_token = -1).  The final token is the smallest index
 * whose cumulative probability exceeds u * (total), u in [0,1) with 24 random bits.
 * target_temp[s] == 0 (the temperature-0 target of Section 5's tables) is the limit
 * T_t -> 0+: R is all mass on the largest target logit of the row, the smallest index
 * winning a tie, so the walk follows the target's argmax token down the tree and the last
 * token is the argmax of the row where it stops; the draws are still taken, in the same order.
 *
 *   draft_logits, target_logits DEVICE [sum N, vocab] fp32 (row i = distribution after node i),
 *                               rows dense, base pointers 16-byte aligned
 *   draft_temp                  HOST [n_seq] > 0
 *   target_temp                 HOST [n_seq] >= 0, independent of draft_temp
 *   tree                        DEVICE inputs (token, first_child, next_sibling are read)
 *   row_stats    DEVICE [sum N,4] fp32: max and sum-exp of draft/T_d, then of target/T_t
 *                (rows of a sequence with T_t == 0: largest raw target logit, then its index)
 *   accept_ratio DEVICE [sum N] fp32: R[y]/D[y] seen by every child the walk tested (root: 0;
 *                -1: not tried because the draft distribution was exhausted; -2: never reached)
 *   accepted_nodes DEVICE [sum N] i32: per sequence, from its node_offset, the accepted
 *                  local node indices in order (root excluded); n_accepted [n_seq]
 *   final_token  DEVICE [n_seq]: token emitted where the walk stopped (-1 if none)
 *   min_margin   DEVICE [n_seq] fp32: smallest |c - accept_ratio| over tested children
 *   workspace, workspace_bytes  not used (verification needs no scratch memory); pass NULL, 0
 * Arithmetic is fp32.  vocab <= DYSPEC_MAX_VOCAB.
 */
dyspec_status dyspec_verify(const float* draft_logits, const float* target_logits,
                            int32_t vocab, const dyspec_batch* batch, const dyspec_tree* tree,
                            const float* draft_temp, const float* target_temp, uint64_t seed,
                            int32_t emit_bonus, float* row_stats, float* accept_ratio,
                            int32_t* accepted_nodes, int32_t* n_accepted, int32_t* final_token,
                            float* min_margin, void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/*
 * dyspec_verify_bf16 -- dyspec_verify on bf16 logit tables (DEVICE [sum N, vocab] bf16, rows
 * dense, base pointers 16-byte aligned): the same operation (Algorithm 3), every logit
 * widened to fp32 as it is read, half the bytes for the statistics pass.  All other
 * arguments, outputs and error behaviour as for dyspec_verify.
 */
dyspec_status dyspec_verify_bf16(const void* draft_logits, const void* target_logits,
                                 int32_t vocab, const dyspec_batch* batch, const dyspec_tree* tree,
                                 const float* draft_temp, const float* target_temp, uint64_t seed,
                                 int32_t emit_bonus, float* row_stats, float* accept_ratio,
                                 int32_t* accepted_nodes, int32_t* n_accepted, int32_t* final_token,
                                 float* min_margin, void* workspace, size_t workspace_bytes,
                                 void* hip_stream);

/*
 * Measurement helpers (no part of the method): ceilings to set beside the published peaks
 * of the chip, and the clock the chip runs at under load.  All only launch; the caller times
 * them (HIP events on hip_stream).
 *
 * dyspec_probe_mfma_bf16: 1024 workgroups of 8 waves, every wave `iterations` rounds of four
 * independent 32x32x16 bf16 MFMAs, no memory traffic.  random_operands != 0: operands with
 * random signs and mantissas and magnitudes in [0.25, 4) instead of a smooth ramp of small
 * values (the clock the chip sustains under matrix load depends on the data).  *flops (HOST)
 * receives the number of floating-point operations of the launch.  sink: DEVICE, one float,
 * never written in practice.
 *
 * dyspec_probe_clock: one wave that sleeps through `iterations` (1 .. 2^24) naps of about
 * 8000 cycles and then writes counters[0] = shader clock cycles and counters[1] = wall clock
 * ticks that went by (DEVICE, two uint64); *wall_clock_khz (HOST) receives the rate of the
 * wall clock counter.  Launched on a stream of its own next to other work it reports the
 * shader clock that work ran at: cycles / (ticks / rate).
 *
 * dyspec_probe_hbm_read: streams `bytes` (a multiple of 16, src DEVICE, 16-byte aligned) from
 * memory once with 16-byte loads, eight in flight per thread.
 */
dyspec_status dyspec_probe_mfma_bf16(int32_t iterations, int32_t random_operands, double* flops,
                                     float* sink, void* hip_stream);
dyspec_status dyspec_probe_clock(int32_t iterations, uint64_t* counters, int32_t* wall_clock_khz,
                                 void* hip_stream);
dyspec_status dyspec_probe_hbm_read(const void* src, size_t bytes, float* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DYSPEC_H */
