// Steps 2-3: the fast model (a hard-voting ensemble of perfect binary trees) on every flow
// (Section 3.1 of the paper) and the integer form of the least-confidence score of
// Section 3.2 (top_votes = max_y votes[y]; LC = 1 - top_votes / n_trees).
//
// Also here: the same walk over the flows of a list (the middle tier of a three-tier cascade)
// and the boosted-tree form of the fast model (Section 4.1), whose leaves hold margins.
//
// Work split: one lane owns one flow (or 2 or 4 lanes share one and split the trees, where
// shared memory would otherwise leave too few waves resident).  The flow's feature row sits in
// shared memory as a column, [feature][flow], so the data-dependent fetch x[feat] of every lane
// of a wave lands in its own bank.  The kernel here copies the rows of its tile into that
// layout; the walk itself and the packed record format are in forest_core.h.
#include "forest_core.h"

namespace {

using namespace sfforest;

__global__ __launch_bounds__(256) void pack_forest(uint32_t n_trees, uint32_t depth, uint32_t n_features,
                                                   const uint16_t* __restrict__ nf, const float* __restrict__ nt,
                                                   PairRec* __restrict__ out)
{
    const uint32_t n_int = (1u << depth) - 1u;
    const uint32_t n_rec = recs_upto(pair_levels(depth));
    const uint64_t total = (uint64_t)n_trees * n_rec;
    for (uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total;
         g += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t t = (uint32_t)(g / n_rec), r = (uint32_t)(g % n_rec);
        uint32_t j = 0;
        while (recs_upto(j + 1) <= r) ++j;                 // pair-level of record r
        const uint32_t pos = r - recs_upto(j);             // position within tree level 2j
        const uint32_t k0 = ((1u << (2u * j)) - 1u) + pos; // heap index of the record's top node
        const uint32_t ks[3] = {k0, 2u * k0 + 1u, 2u * k0 + 2u};
        float thr[3];
        uint32_t fe[3];
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            const bool have = ks[q] < n_int;               // odd depth: the last records have no children
            uint32_t f = have ? nf[(size_t)t * n_int + ks[q]] : 0u;
            fe[q] = f < n_features ? f : n_features - 1u;  // clamp: a bad index must not leave the row
            thr[q] = have ? nt[(size_t)t * n_int + ks[q]] : 0.f;
        }
        PairRec p;
        p.thr0 = thr[0];
        p.thr1 = thr[1];
        p.thr2 = thr[2];
        p.feats = pack_feats(fe[0], fe[1], fe[2]);
        out[g] = p;
    }
}

template <int BS, int S, bool WANT_LEAF, bool GBDT>
__global__ __launch_bounds__(BS) void forest_votes(FastArgs a)
{
    constexpr uint32_t FPB = BS / S;       // flows per block
    constexpr uint32_t FPW = 64 / S;       // flows per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const uint32_t F = a.n_features;
    float* xT = reinterpret_cast<float*>(smem_raw);                          // [F][FPB]
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t grp = lane / FPW;                       // which share of the trees this lane walks
    const uint32_t slot = wave * FPW + (lane % FPW);       // flow slot in the block's tile
    const uint32_t i = blockIdx.x * FPB + slot;
    uint32_t n = a.n_flows;
    if (a.idx_count) {
        const uint32_t c = *a.idx_count;
        n = c < n ? c : n;
        if (blockIdx.x * FPB >= n) return; // the list ends before this block's tile (whole block leaves)
    }
    const bool live = i < n;
    uint32_t row = live ? i : n - 1; // idle lanes walk a valid row, write nothing
    if (a.idx) {
        row = a.idx[row];
        row = row < a.n_rows ? row : a.n_rows - 1u; // a bad list entry must not leave the matrix
    }
    {
        // the S lanes of a flow each copy 1/S of its row into the flow's column
        const float* x = a.feat + (size_t)row * a.ld;
        if ((a.ld & 3u) == 0 && (F % (4u * S)) == 0 && (reinterpret_cast<uintptr_t>(a.feat) & 15u) == 0) {
            const uint32_t per = F / 4u / S;
            for (uint32_t q = grp * per; q < (grp + 1u) * per; ++q) {
                const float4 v = reinterpret_cast<const float4*>(x)[q];
                xT[(4 * q + 0) * FPB + slot] = v.x;
                xT[(4 * q + 1) * FPB + slot] = v.y;
                xT[(4 * q + 2) * FPB + slot] = v.z;
                xT[(4 * q + 3) * FPB + slot] = v.w;
            }
        } else {
            for (uint32_t f = grp; f < F; f += S) xT[f * FPB + slot] = x[f];
        }
    }
    forest_walk<BS, S, WANT_LEAF, GBDT, false, (S > 1 || !GBDT)>(a, xT, i, row, live);
}

template <int BS, int S, bool GBDT>
int launch_votes(sf_ctx* ctx, const FastArgs& a, size_t lds)
{
    const uint32_t fpb = BS / S;
    const uint32_t grid = (a.n_flows + fpb - 1) / fpb;
    constexpr int slot = sf::kLdsForest + (S == 1 ? 0 : (S == 2 ? 1 : 2)) * 4 + (GBDT ? 1 : 0);
    if (a.leaf_idx) {
        SF_ALLOW_LDS(ctx, slot + 2, (forest_votes<BS, S, true, GBDT>));
        forest_votes<BS, S, true, GBDT><<<grid, BS, lds, ctx->stream>>>(a);
    } else {
        SF_ALLOW_LDS(ctx, slot, (forest_votes<BS, S, false, GBDT>));
        forest_votes<BS, S, false, GBDT><<<grid, BS, lds, ctx->stream>>>(a);
    }
    SF_LAUNCH_CHECK(ctx, "forest_votes");
    return SF_OK;
}

} // namespace

namespace sf {
size_t forest_pack_bytes(uint32_t n_trees, uint32_t depth)
{
    if (n_trees == 0 || depth == 0 || depth > SF_MAX_TREE_DEPTH) return 0;
    return align_up((size_t)n_trees * recs_upto(pair_levels(depth)) * sizeof(PairRec));
}
} // namespace sf

namespace {

// the model as the kernels see it: hard-voting forest (leaf_label) or boosted trees (leaf_value, base)
struct TreeModel {
    uint32_t n_trees, depth, n_classes, n_features;
    const uint16_t* node_feat;
    const float* node_thr;
    const uint8_t* leaf_label;
    const float* leaf_value;
    const float* base;
    const void* packed; // records made earlier by sf_forest_pack / sf_gbdt_pack, or NULL
};

struct Outputs {
    uint16_t* votes;
    uint16_t* pred;
    uint16_t* top_votes;
    uint16_t* leaf_idx;
    uint16_t* labels;
    float* margins;
    float* score;
    int score_kind;
};

int pack_into(sf_ctx* ctx, const TreeModel& m, PairRec* out)
{
    const uint64_t total = (uint64_t)m.n_trees * recs_upto(pair_levels(m.depth));
    uint64_t blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    pack_forest<<<(uint32_t)blocks, 256, 0, ctx->stream>>>(m.n_trees, m.depth, m.n_features, m.node_feat, m.node_thr, out);
    SF_LAUNCH_CHECK(ctx, "pack_forest");
    return SF_OK;
}

int check_model(sf_ctx* ctx, const char* who, const TreeModel& m)
{
    if (m.depth < 1 || m.depth > SF_MAX_TREE_DEPTH)
        return sf::fail(ctx, SF_EINVAL, "%s: depth %u outside 1..%d", who, m.depth, SF_MAX_TREE_DEPTH);
    if (m.n_trees < 1 || m.n_trees > 65535) return sf::fail(ctx, SF_EINVAL, "%s: n_trees %u outside 1..65535", who, m.n_trees);
    if (m.n_features < 1 || m.n_features > SF_MAX_FEATURES)
        return sf::fail(ctx, SF_EINVAL, "%s: n_features %u outside 1..%d", who, m.n_features, SF_MAX_FEATURES);
    if (!m.node_feat || !m.node_thr) return sf::fail(ctx, SF_EINVAL, "%s: model arrays missing", who);
    return SF_OK;
}

// The model part of the kernel arguments: checks, the packed records (made into the workspace when the model
// carries none), the width of the vote counters, lanes per flow (*split) and the block's shared memory (*lds).
// check_only: stop after the argument checks (a call on zero flows launches nothing).
int setup_trees(sf_ctx* ctx, const char* who, const TreeModel& m, bool gbdt, uint32_t feat_ld, FastArgs& a, uint32_t* split_out,
                size_t* lds_out, bool check_only = false, bool one_lane_per_flow = false)
{
    if (m.depth < 1 || m.depth > SF_MAX_TREE_DEPTH)
        return sf::fail(ctx, SF_EINVAL, "%s: depth %u outside 1..%d", who, m.depth, SF_MAX_TREE_DEPTH);
    if (m.n_trees < 1 || m.n_trees > 65535) return sf::fail(ctx, SF_EINVAL, "%s: n_trees %u outside 1..65535", who, m.n_trees);
    if (m.n_classes < 1 || m.n_classes > SF_MAX_CLASSES)
        return sf::fail(ctx, SF_EINVAL, "%s: n_classes %u outside 1..%d", who, m.n_classes, SF_MAX_CLASSES);
    if (m.n_features < 1 || m.n_features > SF_MAX_FEATURES)
        return sf::fail(ctx, SF_EINVAL, "%s: n_features %u outside 1..%d", who, m.n_features, SF_MAX_FEATURES);
    if (m.n_features > feat_ld) return sf::fail(ctx, SF_EINVAL, "%s: n_features %u > feat_ld %u", who, m.n_features, feat_ld);
    if (!m.node_feat || !m.node_thr || (gbdt ? !m.leaf_value : !m.leaf_label))
        return sf::fail(ctx, SF_EINVAL, "%s: model arrays missing", who);
    if (check_only) return SF_OK;

    const PairRec* packed = (const PairRec*)m.packed;
    if (!packed) {
        sf::Carve ws(ctx);
        const size_t pack_bytes = sf::forest_pack_bytes(m.n_trees, m.depth);
        PairRec* mine = (PairRec*)ws.take(pack_bytes);
        if (!mine)
            return sf::fail(ctx, SF_ENOMEM, "%s: workspace has %zu bytes, packed trees need %zu", who, ctx->ws_bytes,
                            pack_bytes + sf::kFlagBytes);
        const int rc = pack_into(ctx, m, mine);
        if (rc != SF_OK) return rc;
        packed = mine;
    }
    a.leaf_value = m.leaf_value;
    a.base = m.base;
    a.n_trees = m.n_trees;
    a.depth = m.depth;
    a.n_classes = m.n_classes;
    a.n_features = m.n_features;
    a.recs = packed;
    a.leaf_label = m.leaf_label;
    // Shared memory per block of 256 lanes: a feature column per FLOW, the per-lane result column
    // (packed vote counters, or one binary32 margin per class) and the staged top records of
    // every tree.  With two lanes per flow three blocks (12 waves) stay resident instead of two,
    // which pays while the deep records of the trees in flight still fit the first-level cache
    // (measured: faster up to depth 10, slower at 12, where more waves mean more distinct trees
    // in flight and more cache misses).  Where even that leaves a single block resident (many
    // features, many classes, hundreds of trees), four lanes per flow bring back a second one
    // (measured on 500 trees x 128 features x 32 classes: 16.6 -> 11.2 ms).  Margins are summed in
    // tree order by one lane, so the boosted form never splits a flow.
    a.vote_bits = a.n_trees <= 255 ? 8u : 16u;
    const uint32_t result_words = gbdt ? a.n_classes : (a.n_classes * a.vote_bits + 31u) / 32u;
    const uint32_t full_pairs = m.depth / 2;
    size_t lds = 0;
    // for `split` lanes per flow: how many pair-levels of records fit, and the block's shared memory.
    // The top records may use what is left of a third, else of a half, else of the whole shared memory.
    auto plan = [&](uint32_t split) {
        const size_t fixed = ((size_t)a.n_features + result_words) * 4 * (256 / split);
        size_t budget = 160 * 1024 / 3 - 256;
        if (fixed + (size_t)a.n_trees * 16 > budget) budget = 80 * 1024 - 512;
        if (fixed + (size_t)a.n_trees * 16 > budget) budget = 160 * 1024 - 1024;
        uint32_t top_pairs = 0;
        while (top_pairs < full_pairs && fixed + (size_t)a.n_trees * recs_upto(top_pairs + 1) * 16 <= budget) ++top_pairs;
        a.top_pairs = top_pairs;
        lds = fixed + (size_t)a.n_trees * recs_upto(top_pairs) * 16;
    };
    // (one_lane_per_flow: the fused feature + forest kernel builds one flow per lane; with the feature matrix's
    // round trip gone that beats the separate kernels also where those would share a flow between two lanes:
    // 1,048,576 flows, 100 trees of depth 10: 0.45 ms against 0.11 + 0.40 ms)
    uint32_t split = (!gbdt && !one_lane_per_flow && a.n_trees >= 32 && recs_upto(pair_levels(m.depth)) * 16u <= 8192u) ? 2u : 1u;
    plan(split);
    if (split == 2 && lds > 80 * 1024) {
        plan(4);
        if (lds <= 80 * 1024)
            split = 4;
        else
            plan(2);
    }
    if (lds > 160 * 1024) return sf::fail(ctx, SF_EUNSUPPORTED, "%s: %zu bytes of shared memory needed", who, lds);
    *split_out = split;
    *lds_out = lds;
    return SF_OK;
}

// every entry point of this file: n_flows rows (all flows, or the capacity of the list idx)
int run_trees(sf_ctx* ctx, const char* who, const float* feat, uint32_t feat_ld, uint32_t n_flows, const uint32_t* idx,
              const uint32_t* idx_count, uint32_t n_rows, const TreeModel& m, bool gbdt, const Outputs& out)
{
    FastArgs a = {};
    uint32_t split = 1;
    size_t lds = 0;
    {
        const int rc = setup_trees(ctx, who, m, gbdt, feat_ld, a, &split, &lds, n_flows == 0);
        if (rc != SF_OK) return rc;
    }
    if (n_flows == 0) return SF_OK;
    if (!feat || !out.pred || (gbdt ? !out.score : !out.top_votes))
        return sf::fail(ctx, SF_EINVAL, "%s: feat, pred or %s is NULL", who, gbdt ? "score" : "top_votes");
    a.feat = feat;
    a.ld = feat_ld;
    a.n_flows = n_flows;
    a.idx = idx;
    a.idx_count = idx_count;
    a.n_rows = n_rows;
    a.labels = out.labels;
    a.margins = out.margins;
    a.score = out.score;
    a.score_kind = out.score_kind;
    a.votes = out.votes;
    a.pred = out.pred;
    a.top = out.top_votes;
    a.leaf_idx = out.leaf_idx;
    if (split == 4) return launch_votes<256, 4, false>(ctx, a, lds);
    if (gbdt) return launch_votes<256, 1, true>(ctx, a, lds);
    if (split == 2) return launch_votes<256, 2, false>(ctx, a, lds);
    return launch_votes<256, 1, false>(ctx, a, lds);
}

int run_forest(sf_ctx* ctx, const char* who, const float* feat, uint32_t feat_ld, uint32_t n_flows, const uint32_t* idx,
               const uint32_t* idx_count, uint32_t n_rows, const sf_forest* f, uint16_t* votes, uint16_t* pred,
               uint16_t* top_votes, uint16_t* leaf_idx, uint16_t* labels)
{
    if (!f) return sf::fail(ctx, SF_EINVAL, "%s: forest is NULL", who);
    const TreeModel m = {f->n_trees, f->depth, f->n_classes, f->n_features, f->node_feat, f->node_thr, f->leaf_label,
                         nullptr, nullptr, f->packed};
    const Outputs out = {votes, pred, top_votes, leaf_idx, labels, nullptr, nullptr, 0};
    return run_trees(ctx, who, feat, feat_ld, n_flows, idx, idx_count, n_rows, m, false, out);
}

} // namespace

namespace sf {
// the hard-voting forest as kernel arguments (for the fused feature + forest entry point)
int forest_setup(sf_ctx* ctx, const char* who, const sf_forest* f, uint32_t feat_ld, sfforest::FastArgs& a, uint32_t* split,
                 size_t* lds)
{
    if (!f) return fail(ctx, SF_EINVAL, "%s: forest is NULL", who);
    const TreeModel m = {f->n_trees, f->depth, f->n_classes, f->n_features, f->node_feat, f->node_thr, f->leaf_label,
                         nullptr, nullptr, f->packed};
    return setup_trees(ctx, who, m, false, feat_ld, a, split, lds, false, true);
}
} // namespace sf

extern "C" int sf_fast_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows,
                             const sf_forest* forest, uint16_t* votes, uint16_t* pred, uint16_t* top_votes,
                             uint16_t* leaf_idx)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_fast_infer: ctx is NULL");
    return run_forest(ctx, "sf_fast_infer", feat, feat_ld, n_flows, nullptr, nullptr, n_flows, forest, votes, pred,
                      top_votes, leaf_idx, nullptr);
}

extern "C" int sf_fast_infer_subset(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows,
                                    const uint32_t* idx, const uint32_t* idx_count, uint32_t idx_cap,
                                    const sf_forest* forest, uint16_t* votes, uint16_t* pred, uint16_t* top_votes,
                                    uint16_t* labels)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_fast_infer_subset: ctx is NULL");
    if (idx_cap && n_flows == 0) return sf::fail(ctx, SF_EINVAL, "sf_fast_infer_subset: a list over zero flows");
    if (idx_cap && (!idx || !idx_count)) return sf::fail(ctx, SF_EINVAL, "sf_fast_infer_subset: idx or idx_count is NULL");
    return run_forest(ctx, "sf_fast_infer_subset", feat, feat_ld, idx_cap, idx, idx_count, n_flows, forest, votes, pred,
                      top_votes, nullptr, labels);
}

extern "C" int sf_gbdt_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows, const sf_gbdt* model,
                             int score_kind, float* margins, uint16_t* pred, float* score, uint16_t* leaf_idx)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_gbdt_infer: ctx is NULL");
    if (!model) return sf::fail(ctx, SF_EINVAL, "sf_gbdt_infer: model is NULL");
    if (score_kind != SF_SCORE_LC && score_kind != SF_SCORE_ENTROPY)
        return sf::fail(ctx, SF_EINVAL, "sf_gbdt_infer: score_kind %d is neither SF_SCORE_LC nor SF_SCORE_ENTROPY", score_kind);
    const TreeModel m = {model->n_trees, model->depth, model->n_classes, model->n_features, model->node_feat,
                         model->node_thr, nullptr, model->leaf_value, model->base, model->packed};
    const Outputs out = {nullptr, pred, nullptr, leaf_idx, nullptr, margins, score, score_kind};
    return run_trees(ctx, "sf_gbdt_infer", feat, feat_ld, n_flows, nullptr, nullptr, n_flows, m, true, out);
}

extern "C" size_t sf_forest_packed_bytes(uint32_t n_trees, uint32_t depth) { return sf::forest_pack_bytes(n_trees, depth); }

extern "C" int sf_forest_pack(sf_ctx* ctx, const sf_forest* f, void* packed)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_forest_pack: ctx is NULL");
    if (!f || !packed) return sf::fail(ctx, SF_EINVAL, "sf_forest_pack: forest or packed is NULL");
    if ((uintptr_t)packed & 15u) return sf::fail(ctx, SF_EINVAL, "sf_forest_pack: packed is not 16-byte aligned");
    const TreeModel m = {f->n_trees, f->depth, f->n_classes, f->n_features, f->node_feat, f->node_thr, f->leaf_label,
                         nullptr, nullptr, nullptr};
    const int rc = check_model(ctx, "sf_forest_pack", m);
    return rc != SF_OK ? rc : pack_into(ctx, m, (PairRec*)packed);
}

extern "C" int sf_gbdt_pack(sf_ctx* ctx, const sf_gbdt* g, void* packed)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_gbdt_pack: ctx is NULL");
    if (!g || !packed) return sf::fail(ctx, SF_EINVAL, "sf_gbdt_pack: model or packed is NULL");
    if ((uintptr_t)packed & 15u) return sf::fail(ctx, SF_EINVAL, "sf_gbdt_pack: packed is not 16-byte aligned");
    const TreeModel m = {g->n_trees, g->depth, g->n_classes, g->n_features, g->node_feat, g->node_thr, nullptr,
                         g->leaf_value, g->base, nullptr};
    const int rc = check_model(ctx, "sf_gbdt_pack", m);
    return rc != SF_OK ? rc : pack_into(ctx, m, (PairRec*)packed);
}
