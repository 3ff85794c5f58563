// The tier in front of the fast model: one decision tree on every flow (Section 3.1 of the
// paper: the "fastest" model filters the traffic before the fast one; Section 4.1: its leaves
// keep the class counts of their training samples, which give P(y|x) for the least-confidence
// score of Section 3.2).
//
// Work split: one lane owns one flow.  It copies the first n_features values of its row into
// a shared-memory column once (walking the row in place re-fetches its cache line at every
// level: with a full complement of waves the lines do not survive in the cache between two
// levels), then walks the tree on that column; the nodes of the upper levels sit in shared
// memory as 8-byte (threshold, feature) pairs.  The arg-max, its count and the leaf total
// depend on the leaf only, so a small launch reduces every leaf's counts to one 8-byte summary
// first and the walk ends with one load of it.  Blocks are persistent over tiles of flows.
// n_features smaller than the row (a tree on the first window only) shrinks both the bytes
// fetched and the tile.
#include "common.h"

namespace sf {
size_t tree_tier_bytes(uint32_t depth);
}

namespace {

constexpr uint32_t kLdsLevels = 12; // levels whose nodes are staged in shared memory (32 KB)

struct TreeArgs {
    const float* feat;
    uint32_t ld;
    uint32_t n_flows;
    uint32_t depth, n_classes, n_features;
    const uint16_t* node_feat;
    const float* node_thr;
    const uint16_t* leaf_count;
    uint2* nodes;   // workspace: [2^depth - 1] (threshold bits, feature index clamped into the row)
    uint2* summary; // workspace: [2^depth] (pred | top_count << 16, leaf_total)
    uint16_t* pred;
    uint16_t* top;
    uint16_t* total;
    uint16_t* leaf_idx;
};

// one thread per node and per leaf
__global__ __launch_bounds__(256) void tree_prepare(TreeArgs a)
{
    const uint32_t n_int = (1u << a.depth) - 1u, n_leaf = 1u << a.depth;
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g < n_int) {
        uint32_t f = a.node_feat[g];
        f = f < a.n_features ? f : a.n_features - 1u; // a bad index must not leave the row
        a.nodes[g] = make_uint2(__float_as_uint(a.node_thr[g]), f);
    }
    if (g < n_leaf) {
        const uint16_t* cnt = a.leaf_count + (size_t)g * a.n_classes;
        uint32_t best = 0, bestv = cnt[0], tot = 0;
        for (uint32_t c = 0; c < a.n_classes; ++c) {
            const uint32_t v = cnt[c];
            tot += v;
            if (v > bestv) { // strict: the lowest class wins a tie
                bestv = v;
                best = c;
            }
        }
        tot = tot < 65535u ? tot : 65535u; // totals beyond 16 bits are rejected by sf_validate_tree
        a.summary[g] = make_uint2(best | (bestv << 16), tot);
    }
}

// Block of 256 lanes.  Shared memory: the feature tile [n_features][256] (a lane's flow is a
// column, so its data-dependent reads never collide with another lane's), then the staged nodes.
// A lane reads and writes only its own column, so the tile needs no barrier.
__global__ __launch_bounds__(256) void tree_walk(TreeArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float* xT = reinterpret_cast<float*>(smem_raw);
    uint2* s_nodes = reinterpret_cast<uint2*>(xT + (size_t)a.n_features * 256u);
    const uint32_t lds_levels = a.depth < kLdsLevels ? a.depth : kLdsLevels;
    const uint32_t n_lds = (1u << lds_levels) - 1u;
    for (uint32_t q = threadIdx.x; q < n_lds; q += 256u) s_nodes[q] = a.nodes[q];
    __syncthreads();
    const uint32_t n_int = (1u << a.depth) - 1u, F = a.n_features;
    const bool vec = (a.ld & 3u) == 0 && (F & 3u) == 0 && (reinterpret_cast<uintptr_t>(a.feat) & 15u) == 0;
    float* col = xT + threadIdx.x;
    for (uint32_t base = blockIdx.x * 256u; base < a.n_flows; base += gridDim.x * 256u) {
        const uint32_t i = base + threadIdx.x;
        const bool live = i < a.n_flows;
        const float* x = a.feat + (size_t)(live ? i : a.n_flows - 1u) * a.ld; // idle lanes walk a valid row
        if (vec) {
            for (uint32_t q = 0; q < F / 4u; ++q) {
                const float4 v = reinterpret_cast<const float4*>(x)[q];
                col[(4 * q + 0) * 256u] = v.x;
                col[(4 * q + 1) * 256u] = v.y;
                col[(4 * q + 2) * 256u] = v.z;
                col[(4 * q + 3) * 256u] = v.w;
            }
        } else {
            for (uint32_t f = 0; f < F; ++f) col[f * 256u] = x[f];
        }
        uint32_t k = 0;
        for (uint32_t s = 0; s < lds_levels; ++s) {
            const uint2 nd = s_nodes[k];
            k = 2u * k + 1u + (col[nd.y * 256u] <= __uint_as_float(nd.x) ? 0u : 1u);
        }
        for (uint32_t s = lds_levels; s < a.depth; ++s) {
            const uint2 nd = a.nodes[k];
            k = 2u * k + 1u + (col[nd.y * 256u] <= __uint_as_float(nd.x) ? 0u : 1u);
        }
        if (live) {
            const uint32_t leaf = k - n_int;
            const uint2 sm = a.summary[leaf];
            a.pred[i] = (uint16_t)(sm.x & 0xFFFFu);
            a.top[i] = (uint16_t)(sm.x >> 16);
            a.total[i] = (uint16_t)sm.y;
            if (a.leaf_idx) a.leaf_idx[i] = (uint16_t)leaf;
        }
    }
}

// counts what sf_validate_tree reports: flags[0] split features outside the row, flags[1]
// leaves whose total does not fit 16 bits, flags[2] thresholds that are NaN
__global__ __launch_bounds__(256) void tree_check(TreeArgs a, uint32_t* flags)
{
    const uint32_t n_int = (1u << a.depth) - 1u, n_leaf = 1u << a.depth;
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g < n_int) {
        if (a.node_feat[g] >= a.n_features) atomicAdd(&flags[0], 1u);
        const float t = a.node_thr[g];
        if (t != t) atomicAdd(&flags[2], 1u);
    }
    if (g < n_leaf) {
        uint64_t tot = 0;
        for (uint32_t c = 0; c < a.n_classes; ++c) tot += a.leaf_count[(size_t)g * a.n_classes + c];
        if (tot > 65535u) atomicAdd(&flags[1], 1u);
    }
}

__global__ void flags_zero(uint32_t* flags)
{
    if (threadIdx.x < 3) flags[threadIdx.x] = 0;
}

int check_tree_args(sf_ctx* ctx, const char* who, const sf_tree* tree)
{
    if (!tree) return sf::fail(ctx, SF_EINVAL, "%s: tree is NULL", who);
    if (tree->depth < 1 || tree->depth > SF_MAX_TREE_DEPTH)
        return sf::fail(ctx, SF_EINVAL, "%s: depth %u outside 1..%d", who, tree->depth, SF_MAX_TREE_DEPTH);
    if (tree->n_classes < 1 || tree->n_classes > SF_MAX_CLASSES)
        return sf::fail(ctx, SF_EINVAL, "%s: n_classes %u outside 1..%d", who, tree->n_classes, SF_MAX_CLASSES);
    if (tree->n_features < 1 || tree->n_features > SF_MAX_FEATURES)
        return sf::fail(ctx, SF_EINVAL, "%s: n_features %u outside 1..%d", who, tree->n_features, SF_MAX_FEATURES);
    if (!tree->node_feat || !tree->node_thr || !tree->leaf_count)
        return sf::fail(ctx, SF_EINVAL, "%s: tree arrays missing", who);
    return SF_OK;
}

} // namespace

namespace sf {
size_t tree_tier_bytes(uint32_t depth)
{
    if (depth == 0 || depth > SF_MAX_TREE_DEPTH) return 0;
    return align_up((size_t)((1u << depth) - 1u) * sizeof(uint2)) + align_up((size_t)(1u << depth) * sizeof(uint2));
}
} // namespace sf

extern "C" int sf_fastest_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows,
                                const sf_tree* tree, uint16_t* pred, uint16_t* top_count, uint16_t* leaf_total,
                                uint16_t* leaf_idx)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_fastest_infer: ctx is NULL");
    {
        const int rc = check_tree_args(ctx, "sf_fastest_infer", tree);
        if (rc != SF_OK) return rc;
    }
    if (tree->n_features > feat_ld)
        return sf::fail(ctx, SF_EINVAL, "sf_fastest_infer: n_features %u > feat_ld %u", tree->n_features, feat_ld);
    if (n_flows == 0) return SF_OK;
    if (!feat || !pred || !top_count || !leaf_total)
        return sf::fail(ctx, SF_EINVAL, "sf_fastest_infer: feat, pred, top_count or leaf_total is NULL");

    sf::Carve ws(ctx);
    const uint32_t n_int = (1u << tree->depth) - 1u, n_leaf = 1u << tree->depth;
    uint2* nodes = (uint2*)ws.take((size_t)n_int * sizeof(uint2));
    uint2* summary = (uint2*)ws.take((size_t)n_leaf * sizeof(uint2));
    if (!nodes || !summary)
        return sf::fail(ctx, SF_ENOMEM, "sf_fastest_infer: workspace has %zu bytes, the tree needs %zu", ctx->ws_bytes,
                        sf::tree_tier_bytes(tree->depth) + sf::kFlagBytes);
    TreeArgs a;
    a.feat = feat;
    a.ld = feat_ld;
    a.n_flows = n_flows;
    a.depth = tree->depth;
    a.n_classes = tree->n_classes;
    a.n_features = tree->n_features;
    a.node_feat = tree->node_feat;
    a.node_thr = tree->node_thr;
    a.leaf_count = tree->leaf_count;
    a.nodes = nodes;
    a.summary = summary;
    a.pred = pred;
    a.top = top_count;
    a.total = leaf_total;
    a.leaf_idx = leaf_idx;
    tree_prepare<<<(n_leaf + 255) / 256, 256, 0, ctx->stream>>>(a);
    SF_LAUNCH_CHECK(ctx, "tree_prepare");
    const uint32_t lds_levels = tree->depth < kLdsLevels ? tree->depth : kLdsLevels;
    const size_t lds = (size_t)tree->n_features * 256 * sizeof(float) + (size_t)((1u << lds_levels) - 1u) * sizeof(uint2);
    SF_ALLOW_LDS(ctx, sf::kLdsTreeWalk, tree_walk);
    uint32_t grid = (n_flows + 255) / 256;
    uint32_t per_cu = (uint32_t)((160u * 1024u) / (lds + 256));
    per_cu = per_cu < 1 ? 1 : (per_cu > 8 ? 8 : per_cu);
    const uint32_t resident = (uint32_t)ctx->n_cu * per_cu; // as many blocks as fit the compute units at once
    if (grid > resident) grid = resident;
    tree_walk<<<grid, 256, lds, ctx->stream>>>(a);
    SF_LAUNCH_CHECK(ctx, "tree_walk");
    return SF_OK;
}

extern "C" int sf_validate_tree(sf_ctx* ctx, const sf_tree* tree)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_validate_tree: ctx is NULL");
    {
        const int rc = check_tree_args(ctx, "sf_validate_tree", tree);
        if (rc != SF_OK) return rc;
    }
    TreeArgs a = {};
    a.depth = tree->depth;
    a.n_classes = tree->n_classes;
    a.n_features = tree->n_features;
    a.node_feat = tree->node_feat;
    a.node_thr = tree->node_thr;
    a.leaf_count = tree->leaf_count;
    uint32_t* flags = ctx->d_flags + 16; // three counters of this check
    flags_zero<<<1, 64, 0, ctx->stream>>>(flags);
    SF_LAUNCH_CHECK(ctx, "flags_zero");
    tree_check<<<((1u << tree->depth) + 255) / 256, 256, 0, ctx->stream>>>(a, flags);
    SF_LAUNCH_CHECK(ctx, "tree_check");
    uint32_t h[3] = {0, 0, 0};
    SF_HIP(ctx, hipMemcpyAsync(h, flags, sizeof(h), hipMemcpyDeviceToHost, ctx->stream));
    SF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (h[0] || h[1] || h[2])
        return sf::fail(ctx, SF_EDATA,
                        "sf_validate_tree: %u split features outside the row, %u leaf totals above 65535, %u NaN thresholds",
                        h[0], h[1], h[2]);
    return SF_OK;
}
