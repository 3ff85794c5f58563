// Steps 2-3: the fast model (a hard-voting ensemble of perfect binary trees) on every flow
// (Section 3.1 of the paper) and the integer form of the least-confidence score of
// Section 3.2 (top_votes = max_y votes[y]; LC = 1 - top_votes / n_trees).
//
// Work split: one lane owns one flow.  Its feature row sits in shared memory as a column,
// [feature][lane], so the data-dependent feature fetch x[feat] of every lane of a wave lands
// in its own bank.  Nodes are re-packed once per call to 8 bytes (threshold, feature index
// and, on the last level, the two leaf labels), so that one 8-byte load serves one visit and
// no separate leaf-label fetch is needed.  Several trees are walked at once per lane to keep
// independent loads in flight.  Votes are integers in shared memory; nothing here rounds.
#include "common.h"

namespace {

struct __align__(8) PackedNode {
    float thr;
    uint32_t meta; // bits 0..15 feature; last level: bits 16..23 left label, 24..31 right label
};

__global__ __launch_bounds__(256) void pack_forest(uint32_t n_trees, uint32_t depth, uint32_t n_features,
                                                   uint32_t n_classes, const uint16_t* __restrict__ nf,
                                                   const float* __restrict__ nt, const uint8_t* __restrict__ ll,
                                                   PackedNode* __restrict__ out)
{
    const uint32_t n_int = (1u << depth) - 1u, stride = 1u << depth;
    const uint64_t total = (uint64_t)n_trees * stride;
    for (uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total;
         g += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t t = (uint32_t)(g >> depth), k = (uint32_t)(g & (stride - 1));
        PackedNode p;
        if (k < n_int) {
            uint32_t f = nf[(size_t)t * n_int + k];
            f = f < n_features ? f : n_features - 1; // clamp: a bad index must not leave the row
            uint32_t meta = f;
            const uint32_t first_last = (1u << (depth - 1)) - 1u;
            if (k >= first_last) {
                const uint32_t leaf = 2 * (k - first_last);
                uint32_t l0 = ll[(size_t)t * stride + leaf], l1 = ll[(size_t)t * stride + leaf + 1];
                l0 = l0 < n_classes ? l0 : n_classes - 1;
                l1 = l1 < n_classes ? l1 : n_classes - 1;
                meta |= (l0 << 16) | (l1 << 24);
            }
            p.thr = nt[(size_t)t * n_int + k];
            p.meta = meta;
        } else {
            p.thr = 0.f;
            p.meta = 0;
        }
        out[g] = p;
    }
}

struct FastArgs {
    const float* feat;
    uint32_t ld;
    uint32_t n_flows;
    uint32_t n_trees, depth, n_classes, n_features;
    const PackedNode* nodes;
    uint16_t* votes;
    uint16_t* pred;
    uint16_t* top;
    uint16_t* leaf_idx;
};

constexpr int kIlp = 4; // trees walked at once per lane

template <int BS, bool WANT_LEAF>
__global__ __launch_bounds__(BS) void forest_votes(FastArgs a)
{
    extern __shared__ float smem[];
    float* xT = smem;                                                     // [n_features][BS]
    uint32_t* vT = reinterpret_cast<uint32_t*>(smem + (size_t)a.n_features * BS); // [n_classes][BS]
    const uint32_t tid = threadIdx.x;
    const uint32_t i = blockIdx.x * BS + tid;
    const bool live = i < a.n_flows;
    const uint32_t row = live ? i : a.n_flows - 1; // idle lanes walk a valid row, write nothing
    const float* x = a.feat + (size_t)row * a.ld;
    const uint32_t F = a.n_features;
    if ((a.ld & 3u) == 0 && (F & 3u) == 0 && (reinterpret_cast<uintptr_t>(a.feat) & 15u) == 0) {
        for (uint32_t q = 0; q < F / 4; ++q) {
            const float4 v = reinterpret_cast<const float4*>(x)[q];
            xT[(4 * q + 0) * BS + tid] = v.x;
            xT[(4 * q + 1) * BS + tid] = v.y;
            xT[(4 * q + 2) * BS + tid] = v.z;
            xT[(4 * q + 3) * BS + tid] = v.w;
        }
    } else {
        for (uint32_t f = 0; f < F; ++f) xT[f * BS + tid] = x[f];
    }
    for (uint32_t c = 0; c < a.n_classes; ++c) vT[c * BS + tid] = 0;
    // each lane reads back only what it wrote itself: no barrier needed

    const uint32_t depth = a.depth;
    const uint32_t stride = 1u << depth;
    const uint32_t n_int = stride - 1u;
    const float* xcol = xT + tid;
    uint32_t* vcol = vT + tid;
    uint32_t t = 0;
    for (; t + kIlp <= a.n_trees; t += kIlp) {
        uint32_t k[kIlp];
        uint32_t lab[kIlp];
#pragma unroll
        for (int u = 0; u < kIlp; ++u) k[u] = 0;
        for (uint32_t lvl = 0; lvl < depth; ++lvl) {
            PackedNode nd[kIlp];
#pragma unroll
            for (int u = 0; u < kIlp; ++u) nd[u] = a.nodes[(size_t)(t + u) * stride + k[u]];
#pragma unroll
            for (int u = 0; u < kIlp; ++u) {
                const float xv = xcol[(nd[u].meta & 0xFFFFu) * BS];
                const bool left = xv <= nd[u].thr;
                k[u] = 2 * k[u] + (left ? 1u : 2u);
                lab[u] = left ? (nd[u].meta >> 16) & 0xFFu : nd[u].meta >> 24;
            }
        }
#pragma unroll
        for (int u = 0; u < kIlp; ++u) {
            vcol[lab[u] * BS] += 1;
            if (WANT_LEAF && live) a.leaf_idx[(size_t)i * a.n_trees + t + u] = (uint16_t)(k[u] - n_int);
        }
    }
    for (; t < a.n_trees; ++t) {
        uint32_t k = 0, lab = 0;
        for (uint32_t lvl = 0; lvl < depth; ++lvl) {
            const PackedNode nd = a.nodes[(size_t)t * stride + k];
            const float xv = xcol[(nd.meta & 0xFFFFu) * BS];
            const bool left = xv <= nd.thr;
            k = 2 * k + (left ? 1u : 2u);
            lab = left ? (nd.meta >> 16) & 0xFFu : nd.meta >> 24;
        }
        vcol[lab * BS] += 1;
        if (WANT_LEAF && live) a.leaf_idx[(size_t)i * a.n_trees + t] = (uint16_t)(k - n_int);
    }
    if (!live) return;
    uint32_t best = 0, bestv = vcol[0];
    if (a.votes) a.votes[(size_t)i * a.n_classes] = (uint16_t)bestv;
    for (uint32_t c = 1; c < a.n_classes; ++c) {
        const uint32_t v = vcol[c * BS];
        if (a.votes) a.votes[(size_t)i * a.n_classes + c] = (uint16_t)v;
        if (v > bestv) {
            bestv = v;
            best = c;
        }
    }
    a.pred[i] = (uint16_t)best;
    a.top[i] = (uint16_t)bestv;
}

template <int BS>
int launch_votes(sf_ctx* ctx, const FastArgs& a, size_t lds)
{
    const uint32_t grid = (a.n_flows + BS - 1) / BS;
    if (a.leaf_idx) {
        SF_HIP(ctx, hipFuncSetAttribute((const void*)forest_votes<BS, true>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        forest_votes<BS, true><<<grid, BS, lds, ctx->stream>>>(a);
    } else {
        SF_HIP(ctx, hipFuncSetAttribute((const void*)forest_votes<BS, false>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        forest_votes<BS, false><<<grid, BS, lds, ctx->stream>>>(a);
    }
    SF_LAUNCH_CHECK(ctx, "forest_votes");
    return SF_OK;
}

} // namespace

extern "C" int sf_fast_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows,
                             const sf_forest* forest, uint16_t* votes, uint16_t* pred, uint16_t* top_votes,
                             uint16_t* leaf_idx)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_fast_infer: ctx is NULL");
    if (!forest) return sf::fail(ctx, SF_EINVAL, "sf_fast_infer: forest is NULL");
    if (forest->depth < 1 || forest->depth > SF_MAX_TREE_DEPTH)
        return sf::fail(ctx, SF_EINVAL, "sf_fast_infer: depth %u outside 1..%d", forest->depth, SF_MAX_TREE_DEPTH);
    if (forest->n_trees < 1 || forest->n_trees > 65535)
        return sf::fail(ctx, SF_EINVAL, "sf_fast_infer: n_trees %u outside 1..65535", forest->n_trees);
    if (forest->n_classes < 1 || forest->n_classes > SF_MAX_CLASSES)
        return sf::fail(ctx, SF_EINVAL, "sf_fast_infer: n_classes %u outside 1..%d", forest->n_classes, SF_MAX_CLASSES);
    if (forest->n_features < 1 || forest->n_features > SF_MAX_FEATURES)
        return sf::fail(ctx, SF_EINVAL, "sf_fast_infer: n_features %u outside 1..%d", forest->n_features,
                        SF_MAX_FEATURES);
    if (forest->n_features > feat_ld)
        return sf::fail(ctx, SF_EINVAL, "sf_fast_infer: n_features %u > feat_ld %u", forest->n_features, feat_ld);
    if (!forest->node_feat || !forest->node_thr || !forest->leaf_label)
        return sf::fail(ctx, SF_EINVAL, "sf_fast_infer: forest arrays missing");
    if (n_flows == 0) return SF_OK;
    if (!feat || !pred || !top_votes) return sf::fail(ctx, SF_EINVAL, "sf_fast_infer: feat, pred or top_votes is NULL");

    sf::Carve ws(ctx);
    const size_t pack_bytes = sf::forest_pack_bytes(forest->n_trees, forest->depth);
    PackedNode* packed = (PackedNode*)ws.take(pack_bytes);
    if (!packed)
        return sf::fail(ctx, SF_ENOMEM, "sf_fast_infer: workspace has %zu bytes, packed forest needs %zu",
                        ctx->ws_bytes, pack_bytes + sf::kFlagBytes);
    {
        const uint64_t total = (uint64_t)forest->n_trees << forest->depth;
        uint64_t blocks = (total + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        pack_forest<<<(uint32_t)blocks, 256, 0, ctx->stream>>>(forest->n_trees, forest->depth, forest->n_features,
                                                               forest->n_classes, forest->node_feat, forest->node_thr,
                                                               forest->leaf_label, packed);
        SF_LAUNCH_CHECK(ctx, "pack_forest");
    }
    FastArgs a;
    a.feat = feat;
    a.ld = feat_ld;
    a.n_flows = n_flows;
    a.n_trees = forest->n_trees;
    a.depth = forest->depth;
    a.n_classes = forest->n_classes;
    a.n_features = forest->n_features;
    a.nodes = packed;
    a.votes = votes;
    a.pred = pred;
    a.top = top_votes;
    a.leaf_idx = leaf_idx;
    // bytes of shared memory per lane; two blocks per compute unit when they fit in 160 KB
    const size_t per_lane = ((size_t)a.n_features + a.n_classes) * 4;
    if (per_lane * 256 <= 80 * 1024) return launch_votes<256>(ctx, a, per_lane * 256);
    if (per_lane * 128 <= 80 * 1024) return launch_votes<128>(ctx, a, per_lane * 128);
    return launch_votes<64>(ctx, a, per_lane * 64);
}
