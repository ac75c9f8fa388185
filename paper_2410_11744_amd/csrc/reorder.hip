// Depth-first renaming of built token trees (Appendix "Block-Sparsity Friendly Token Order")
// for gfx950: new index = position in the pre-order walk that visits children in sampling
// order, so every subtree becomes a contiguous run of rows and the ancestor mask gathers
// into fewer 32x32 blocks.  One workgroup per sequence.  The walk itself is serial (one
// lane chases first_child / next_sibling / parent in LDS, about N steps); renaming the
// arrays and rebuilding the mask rows is spread over the workgroup.
#include "dyspec_device.h"

namespace dyspec {

constexpr int kReorderThreads = 256;

struct ReorderShared {
    int parent[DYSPEC_MAX_NODES];
    int first_child[DYSPEC_MAX_NODES];
    int next_sibling[DYSPEC_MAX_NODES];
    int rank[DYSPEC_MAX_NODES];        // old index -> new index
    int order[DYSPEC_MAX_NODES];       // new index -> old index
    int new_parent[DYSPEC_MAX_NODES];
};

__global__ __launch_bounds__(kReorderThreads) void dfs_reorder_kernel(SeqArgs sa, dyspec_tree in, dyspec_tree out,
                                                                      int* __restrict__ order_out,
                                                                      uint64_t* __restrict__ mask_out, int mask_words)
{
    __shared__ ReorderShared sh;
    const int tid = threadIdx.x;
    const int seq = blockIdx.x;
    const int base = sa.node_off[seq];
    const int N = sa.node_off[seq + 1] - base;
    // links outside [0, N) are read as "none", so a malformed tree cannot send the walk out of LDS
    auto link = [N](int v) { return (v >= 0 && v < N) ? v : -1; };
    for (int i = tid; i < N; i += kReorderThreads) {
        sh.parent[i] = link(in.parent[base + i]);
        sh.first_child[i] = link(in.first_child[base + i]);
        sh.next_sibling[i] = link(in.next_sibling[base + i]);
        sh.rank[i] = -1;
    }
    __syncthreads();
    if (tid == 0) {
        // pre-order without a stack: down to the first child, else along to the next sibling of
        // the nearest ancestor-or-self that has one
        // (a node met twice, or more than 2N climbing steps, can only come from links that do
        //  not form a tree: the walk stops there and the rest is appended as unattached rows)
        int n = 0, cur = 0, climbs = 0;
        while (cur >= 0 && n < N && sh.rank[cur] < 0) {
            sh.rank[cur] = n;
            sh.order[n++] = cur;
            int next = sh.first_child[cur];
            while (next < 0 && cur >= 0 && climbs <= 2 * N) {
                next = sh.next_sibling[cur];
                if (next < 0) { cur = sh.parent[cur]; ++climbs; }
            }
            cur = next;
        }
        // rows that were never attached to the tree follow it in index order
        for (int i = 0; i < N && n < N; ++i)
            if (sh.rank[i] < 0) { sh.rank[i] = n; sh.order[n++] = i; }
    }
    __syncthreads();
    auto renamed = [&](int old) { return old >= 0 ? sh.rank[old] : -1; };
    for (int j = tid; j < N; j += kReorderThreads) {
        const int o = sh.order[j];
        const int p = renamed(sh.parent[o]);
        sh.new_parent[j] = p;
        order_out[base + j] = o;
        out.parent[base + j] = p;
        out.first_child[base + j] = renamed(sh.first_child[o]);
        out.next_sibling[base + j] = renamed(sh.next_sibling[o]);
        out.token[base + j] = in.token[base + o];
        out.sib_rank[base + j] = in.sib_rank[base + o];
        out.depth[base + j] = in.depth[base + o];
    }
    __syncthreads();
    // mask row j: own bit and the bits of the chain of renamed parents (all smaller than j)
    for (int j = tid; j < N; j += kReorderThreads) {
        uint64_t* row = mask_out + (size_t)(base + j) * mask_words;
        for (int w = 0; w < mask_words; ++w) row[w] = 0ull;
        for (int a = j, prev = N; a >= 0 && a < prev; prev = a, a = sh.new_parent[a]) row[a >> 6] |= 1ull << (a & 63);
    }
}

hipError_t launch_dfs_reorder(const SeqArgs& sa, const dyspec_tree& in, const dyspec_tree& out, int* order,
                              uint64_t* mask_out, int mask_words, hipStream_t stream)
{
    dfs_reorder_kernel<<<sa.n_seq, kReorderThreads, 0, stream>>>(sa, in, out, order, mask_out, mask_words);
    return hipGetLastError();
}

}  // namespace dyspec
