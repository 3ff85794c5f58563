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
// of a wave lands in its own bank.  What bounds the walk is gather throughput, of the caches'
// address path (a compute unit retires a 64-lane gather every 16 to 57 cycles, by how many
// cache lines it touches) and of shared memory alike, so the forest is re-packed once per call
// into 16-byte records that hold TWO levels: a node and both its children (three thresholds,
// three feature indices).  One 16-byte load then serves two visits.  Records form a quaternary
// heap per tree (record r has children 4r+1..4r+4); the records of the top levels of every tree
// are staged in shared memory, the deeper ones come through the cache; the leaf label is one
// byte load at the end.  Eight trees are walked at once per lane to keep independent loads in
// flight.  Votes are integers in shared memory; nothing in the voting form rounds.
#include "common.h"

namespace {

struct __align__(16) PairRec {
    float thr0, thr1, thr2; // node, its left child, its right child
    uint32_t feats;         // bits 0..7, 8..15, 16..23: their feature indices
};

__host__ __device__ inline uint32_t pair_levels(uint32_t depth) { return (depth + 1u) / 2u; }
__host__ __device__ inline uint32_t recs_upto(uint32_t j) { return ((1u << (2u * j)) - 1u) / 3u; } // (4^j-1)/3

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
        p.feats = fe[0] | (fe[1] << 8) | (fe[2] << 16);
        out[g] = p;
    }
}

struct FastArgs {
    const float* feat;
    uint32_t ld;
    uint32_t n_flows;          // rows to classify (the capacity of the list when idx is given)
    const uint32_t* idx;       // subset form: row j is flow idx[j]; NULL = row j is flow j
    const uint32_t* idx_count; // subset form: device-side length of idx
    uint32_t n_rows;           // subset form: rows of feat (list entries are clamped below it)
    uint16_t* labels;          // subset form, optional: labels[idx[j]] = pred of row j
    // boosted form: leaves hold margins instead of labels, tree t adds to class t % n_classes
    const float* leaf_value;   // [n_trees][2^depth]
    const float* base;         // [n_classes] initial margins, or NULL
    float* margins;            // optional [n][n_classes]
    float* score;              // [n]: LC or entropy of softmax(margins)
    int score_kind;
    uint32_t n_trees, depth, n_classes, n_features;
    uint32_t top_pairs; // pair-levels of every tree staged in shared memory
    uint32_t vote_bits; // width of one packed vote counter: 8 (n_trees <= 255) or 16
    const PairRec* recs;
    const uint8_t* leaf_label;
    uint16_t* votes;
    uint16_t* pred;
    uint16_t* top;
    uint16_t* leaf_idx;
};

constexpr int kIlp = 8; // trees walked at once per lane (measured: 4 and 16 are slower)

// BS lanes per block; S lanes share one flow, lane group g of S walks trees g, g+S, g+2S, ...
// Splitting a flow over S lanes divides the shared memory per lane by S (the feature tile is per
// flow), which is what limits the number of resident waves.
// GBDT = false: leaves are class labels and the flow's result is the vote count per class.
// GBDT = true (S must be 1): leaves are binary32 margins; the lane's shared-memory column holds
// one binary32 sum per class, started at the initial margin and extended tree by tree in tree
// order (each addition rounded on its own, so the sums are reproducible bit for bit); the
// epilogue turns them into softmax probabilities in binary64 and into the score of Section 3.2.
template <int BS, int S, bool WANT_LEAF, bool GBDT>
__global__ __launch_bounds__(BS) void forest_votes(FastArgs a)
{
    static_assert(!GBDT || S == 1, "margins are summed in tree order by one lane");
    constexpr uint32_t FPB = BS / S;       // flows per block
    constexpr uint32_t FPW = 64 / S;       // flows per wave
    constexpr uint32_t kColShift = FPB == 256 ? 10 : (FPB == 128 ? 9 : (FPB == 64 ? 8 : 7)); // log2(bytes per feature column)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const uint32_t F = a.n_features, C = a.n_classes, T = a.n_trees;
    const uint32_t top_recs = recs_upto(a.top_pairs);      // records per tree held in shared memory
    float* xT = reinterpret_cast<float*>(smem_raw);                          // [F][FPB]
    // vote counters, 32 / vote_bits classes per word, one column per FLOW: [vote_words][FPB]; the S lanes of
    // a flow add to it with shared-memory atomics (fields cannot carry into each other: a count is at most n_trees)
    const uint32_t per_shift = a.vote_bits == 8 ? 2u : 1u; // log2(counters per word)
    const uint32_t vote_words = GBDT ? C : (C + (1u << per_shift) - 1u) >> per_shift; // boosted: one float per class
    uint32_t* vT = reinterpret_cast<uint32_t*>(xT + (size_t)F * FPB);
    uint4* topT = reinterpret_cast<uint4*>(vT + (size_t)vote_words * FPB);   // [T][top_recs]
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
    if (GBDT) {
        for (uint32_t c = 0; c < C; ++c) vT[c * FPB + slot] = __float_as_uint(a.base ? a.base[c] : 0.f);
    } else {
        for (uint32_t c = grp; c < vote_words; c += S) vT[c * FPB + slot] = 0;
    }
    const uint32_t n_rec = recs_upto(pair_levels(a.depth));
    const uint4* recs = reinterpret_cast<const uint4*>(a.recs);
    for (uint32_t q = tid; q < T * top_recs; q += BS) {
        const uint32_t t = q / top_recs, r = q - t * top_recs;
        topT[q] = recs[(size_t)t * n_rec + r];
    }
    __syncthreads(); // the staged records and the feature columns are shared

    const uint32_t depth = a.depth;
    const uint32_t full_pairs = depth >> 1;
    const uint32_t lds_pairs = a.top_pairs < full_pairs ? a.top_pairs : full_pairs;
    const bool odd = depth & 1u;
    const char* xlane = reinterpret_cast<const char*>(xT) + slot * 4u; // the flow's column
    uint32_t* vcol = vT + slot;
    const uint32_t rec_bytes = n_rec * 16u, top_bytes = top_recs * 16u;
    const uint32_t leaf_base = recs_upto(full_pairs); // record index of position 0 on tree level 2*full_pairs
    const uint32_t n_leaf = 1u << depth;

    // two visits from one record; o is the byte offset of the record inside its tree.
    // One lane per flow (S = 1, eight or more waves per compute unit): the child's feature is fetched
    // after the parent's test (two shared-memory reads per record, the second dependent on the first):
    // the shared-memory pipe is the scarcer resource there and the resident waves cover the latency.
    // Lanes sharing a flow (S = 2: forests whose shared-memory needs leave few waves resident): all
    // three features up front (three independent reads), which is faster when latency binds.
#define SF_PAIR_STEP(REC, O)                                                                              \
    do {                                                                                                  \
        const uint32_t fw = (REC).w;                                                                      \
        const float x0 = *reinterpret_cast<const float*>(xlane + ((fw & 0xFFu) << kColShift));            \
        const bool r0 = !(x0 <= __uint_as_float((REC).x));                                                \
        if (S == 1) {                                                                                     \
            const uint32_t fc = r0 ? (fw >> 16) : ((fw >> 8) & 0xFFu);                                    \
            const float tc = __uint_as_float(r0 ? (REC).z : (REC).y);                                     \
            const float xc = *reinterpret_cast<const float*>(xlane + (fc << kColShift));                  \
            const bool rc = !(xc <= tc);                                                                  \
            (O) = 4u * (O) + (r0 ? 48u : 16u) + (rc ? 16u : 0u);                                          \
        } else {                                                                                          \
            const float x1 = *reinterpret_cast<const float*>(xlane + (((fw >> 8) & 0xFFu) << kColShift)); \
            const float x2 = *reinterpret_cast<const float*>(xlane + ((fw >> 16) << kColShift));          \
            const bool r1 = !(x1 <= __uint_as_float((REC).y));                                            \
            const bool r2 = !(x2 <= __uint_as_float((REC).z));                                            \
            const uint32_t inc_l = r1 ? 32u : 16u, inc_r = r2 ? 64u : 48u;                                \
            (O) = 4u * (O) + (r0 ? inc_r : inc_l);                                                        \
        }                                                                                                 \
    } while (0)

    // lane group g walks trees g, g+S, ...; every group runs the same number of rounds so that
    // the loop stays wave-uniform; a slot past the last tree repeats it and does not vote
    const uint32_t per_grp = (T + S - 1u) / S;
    for (uint32_t q0 = 0; q0 < per_grp; q0 += kIlp) {
        uint32_t o[kIlp], tt[kIlp];
        bool tv[kIlp];
#pragma unroll
        for (int u = 0; u < kIlp; ++u) {
            const uint32_t t = (q0 + u) * S + grp;
            o[u] = 0;
            tv[u] = q0 + u < per_grp && t < T;
            tt[u] = tv[u] ? t : T - 1u;
        }
        uint32_t j = 0;
        for (; j < lds_pairs; ++j) {
            uint4 rec[kIlp];
#pragma unroll
            for (int u = 0; u < kIlp; ++u)
                rec[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(topT) + tt[u] * top_bytes + o[u]);
#pragma unroll
            for (int u = 0; u < kIlp; ++u) SF_PAIR_STEP(rec[u], o[u]);
        }
        const char* gb = reinterpret_cast<const char*>(a.recs);
        for (; j < full_pairs; ++j) {
            uint4 rec[kIlp];
#pragma unroll
            for (int u = 0; u < kIlp; ++u)
                rec[u] = *reinterpret_cast<const uint4*>(gb + (size_t)tt[u] * rec_bytes + o[u]);
#pragma unroll
            for (int u = 0; u < kIlp; ++u) SF_PAIR_STEP(rec[u], o[u]);
        }
        uint32_t leaf[kIlp];
        if (odd) {
            // one level left: only the record's top node counts
            uint4 rec[kIlp];
#pragma unroll
            for (int u = 0; u < kIlp; ++u)
                rec[u] = *reinterpret_cast<const uint4*>(gb + (size_t)tt[u] * rec_bytes + o[u]);
#pragma unroll
            for (int u = 0; u < kIlp; ++u) {
                const float x0 = *reinterpret_cast<const float*>(xlane + ((rec[u].w & 0xFFu) << kColShift));
                const bool r0 = !(x0 <= __uint_as_float(rec[u].x));
                leaf[u] = 2u * ((o[u] >> 4) - leaf_base) + (r0 ? 1u : 0u);
            }
        } else {
#pragma unroll
            for (int u = 0; u < kIlp; ++u) leaf[u] = (o[u] >> 4) - leaf_base;
        }
        if (GBDT) {
            float val[kIlp];
#pragma unroll
            for (int u = 0; u < kIlp; ++u) val[u] = a.leaf_value[(size_t)tt[u] * n_leaf + leaf[u]];
#pragma unroll
            for (int u = 0; u < kIlp; ++u) { // ascending u = ascending tree: the order of the sum
                if (tv[u]) {
                    float* m = reinterpret_cast<float*>(&vcol[(tt[u] % C) * FPB]);
                    *m = *m + val[u];
                    if (WANT_LEAF && live) a.leaf_idx[(size_t)i * T + tt[u]] = (uint16_t)leaf[u];
                }
            }
            continue;
        }
        uint32_t lab[kIlp];
#pragma unroll
        for (int u = 0; u < kIlp; ++u) lab[u] = a.leaf_label[(size_t)tt[u] * n_leaf + leaf[u]];
#pragma unroll
        for (int u = 0; u < kIlp; ++u) {
            if (tv[u]) {
                const uint32_t l = lab[u] < C ? lab[u] : C - 1u; // clamp: a bad label must not leave the tile
                // only this lane touches its column; the add is one shared-memory instruction
                atomicAdd(&vcol[(l >> per_shift) * FPB], 1u << ((l & ((1u << per_shift) - 1u)) * a.vote_bits));
                if (WANT_LEAF && live) a.leaf_idx[(size_t)i * T + tt[u]] = (uint16_t)leaf[u];
            }
        }
    }
#undef SF_PAIR_STEP
    if (S > 1) __syncthreads(); // all lanes of a flow have added their votes before its first lane reads them
    if (!live || grp != 0) return;
    if (GBDT) {
        const float* mcol = reinterpret_cast<const float*>(vcol);
        uint32_t bc = 0;
        float bm = mcol[0];
        for (uint32_t c = 1; c < C; ++c) {
            const float m = mcol[c * FPB];
            if (m > bm) { // strict: the lowest class wins a tie
                bm = m;
                bc = c;
            }
        }
        double z = 0.0;
        for (uint32_t c = 0; c < C; ++c) z += exp((double)mcol[c * FPB] - (double)bm);
        double sc;
        if (a.score_kind == SF_SCORE_ENTROPY) {
            double h = 0.0;
            for (uint32_t c = 0; c < C; ++c) {
                const double p = exp((double)mcol[c * FPB] - (double)bm) / z;
                if (p > 0.0) h -= p * log(p);
            }
            sc = h;
        } else {
            sc = 1.0 - 1.0 / z; // the largest probability is exp(0) / z
        }
        if (a.margins)
            for (uint32_t c = 0; c < C; ++c) a.margins[(size_t)i * C + c] = mcol[c * FPB];
        a.pred[i] = (uint16_t)bc;
        a.score[i] = (float)sc;
        if (a.labels) a.labels[row] = (uint16_t)bc;
        return;
    }
    uint32_t best = 0, bestv = 0;
    const uint32_t vmask = (1u << a.vote_bits) - 1u;
    for (uint32_t w = 0; w < vote_words; ++w) {
        const uint32_t word = vT[w * FPB + slot];
        for (uint32_t k = 0; k < (1u << per_shift); ++k) {
            const uint32_t c = (w << per_shift) + k;
            if (c < C) {
                const uint32_t v = (word >> (k * a.vote_bits)) & vmask;
                if (a.votes) a.votes[(size_t)i * C + c] = (uint16_t)v;
                if (c == 0 || v > bestv) {
                    bestv = v;
                    best = c;
                }
            }
        }
    }
    a.pred[i] = (uint16_t)best;
    a.top[i] = (uint16_t)bestv;
    if (a.labels) a.labels[row] = (uint16_t)best;
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

// every entry point of this file: n_flows rows (all flows, or the capacity of the list idx)
int run_trees(sf_ctx* ctx, const char* who, const float* feat, uint32_t feat_ld, uint32_t n_flows, const uint32_t* idx,
              const uint32_t* idx_count, uint32_t n_rows, const TreeModel& m, bool gbdt, const Outputs& out)
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
    if (n_flows == 0) return SF_OK;
    if (!feat || !out.pred || (gbdt ? !out.score : !out.top_votes))
        return sf::fail(ctx, SF_EINVAL, "%s: feat, pred or %s is NULL", who, gbdt ? "score" : "top_votes");

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
    FastArgs a;
    a.feat = feat;
    a.ld = feat_ld;
    a.n_flows = n_flows;
    a.idx = idx;
    a.idx_count = idx_count;
    a.n_rows = n_rows;
    a.labels = out.labels;
    a.leaf_value = m.leaf_value;
    a.base = m.base;
    a.margins = out.margins;
    a.score = out.score;
    a.score_kind = out.score_kind;
    a.n_trees = m.n_trees;
    a.depth = m.depth;
    a.n_classes = m.n_classes;
    a.n_features = m.n_features;
    a.recs = packed;
    a.leaf_label = m.leaf_label;
    a.votes = out.votes;
    a.pred = out.pred;
    a.top = out.top_votes;
    a.leaf_idx = out.leaf_idx;
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
    uint32_t split = (!gbdt && a.n_trees >= 32 && recs_upto(pair_levels(m.depth)) * 16u <= 8192u) ? 2u : 1u;
    plan(split);
    if (split == 2 && lds > 80 * 1024) {
        plan(4);
        if (lds <= 80 * 1024)
            split = 4;
        else
            plan(2);
    }
    if (lds > 160 * 1024) return sf::fail(ctx, SF_EUNSUPPORTED, "%s: %zu bytes of shared memory needed", who, lds);
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
