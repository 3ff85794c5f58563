// Device code of steps 2-3 shared by the stand-alone forest kernel and the fused feature + forest kernel:
// the walk of a hard-voting ensemble of perfect binary trees (the fast model that sees every flow,
// Section 3.1 of the paper; boosted form: Section 4.1) over a tile of flows whose feature rows already sit
// in shared memory as columns [feature][flow], and the score of Section 3.2 (top_votes = max_y votes[y],
// LC = 1 - top_votes / n_trees; entropy or LC of the softmax for boosted trees).
//
// What bounds the walk is gather throughput, of the caches' address path (a compute unit retires a
// 64-lane gather every 16 to 57 cycles, by how many cache lines it touches) and of shared memory alike,
// so the forest is packed into 16-byte records that hold TWO levels: a node and both its children (three
// thresholds, three feature indices).  One 16-byte load then serves two visits.  Records form a quaternary
// heap per tree (record r has children 4r+1..4r+4); the records of the top levels of every tree are staged
// in shared memory, the deeper ones come through the cache; the leaf label is one byte load at the end.
// Eight trees are walked at once per lane to keep independent loads in flight.  Votes are integers in
// shared memory; nothing in the voting form rounds.
#pragma once

#include <type_traits>

#include "common.h"

namespace sfforest {

constexpr uint32_t kFeatRot = 10; // the word of feature indices is rotated left by this (see forest_walk)

struct __align__(16) PairRec {
    float thr0, thr1, thr2; // node, its left child, its right child
    uint32_t feats;         // their feature indices as 8-bit fields (f0 | f1 << 8 | f2 << 16), rotated left by kFeatRot
};

__host__ __device__ inline uint32_t pack_feats(uint32_t f0, uint32_t f1, uint32_t f2)
{
    const uint32_t w = f0 | (f1 << 8) | (f2 << 16);
    return (w << kFeatRot) | (w >> (32u - kFeatRot));
}

__host__ __device__ inline uint32_t pair_levels(uint32_t depth) { return (depth + 1u) / 2u; }
__host__ __device__ inline uint32_t recs_upto(uint32_t j) { return ((1u << (2u * j)) - 1u) / 3u; } // (4^j-1)/3

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
    // fused form: the tile's rows are written to feat_out only for flows the gate hands on
    // (top_votes < vmin, or vmin[pred] with one threshold per class)
    float* feat_out;
    uint32_t feat_out_ld;
    uint32_t feat_out16; // feat_out is 16-byte aligned and its leading dimension a multiple of 4
    uint32_t n_vmin;
    uint16_t vmin[SF_MAX_CLASSES];
};

// Trees walked at once per lane: groups of kIlp, and a last group of kIlpTail when at most that many trees are
// left (so that 100 trees take ten full groups and 125 twelve and a half, not thirteen of eight with four idle
// slots; measured on 100 trees of depth 12: 8 at a time 0.565 ms, 10 at a time 0.532, 12 0.565, 20 0.553).
constexpr int kIlp = 10, kIlpTail = 5;


// Shared memory of a block behind the feature tile xT ([n_features][FPB] floats, FPB = BS / S flows):
// vote counters (or margins), then the staged top records.
// BS lanes per block; S lanes share one flow, lane group g of S walks trees g, g+S, g+2S, ...
// GBDT = false: leaves are class labels and the flow's result is the vote count per class.
// GBDT = true (S must be 1): leaves are binary32 margins; the lane's shared-memory column holds
// one binary32 sum per class, started at the initial margin and extended tree by tree in tree
// order (each addition rounded on its own, so the sums are reproducible bit for bit); the
// epilogue turns them into softmax probabilities in binary64 and into the score of Section 3.2.
// KEEP_ROWS: the fused form (see FastArgs::feat_out).
// i: the row of the outputs this lane's flow owns; row: its row in the feature matrix (subset form);
// live: false for lanes past the end (they walk a valid tile column and write nothing).
// The caller has filled xT (no barrier needed before the call: this function synchronises the block
// before the first read of the tile).
template <int BS, int S, bool WANT_LEAF, bool GBDT, bool KEEP_ROWS, bool EAGER = (S > 1)>
__device__ __forceinline__ void forest_walk(const FastArgs& a, float* xT, uint32_t i, uint32_t row, bool live)
{
    static_assert(!GBDT || S == 1, "margins are summed in tree order by one lane");
    constexpr uint32_t FPB = BS / S;       // flows per block
    constexpr uint32_t FPW = 64 / S;       // flows per wave
    constexpr uint32_t kColShift = FPB == 256 ? 10 : (FPB == 128 ? 9 : (FPB == 64 ? 8 : 7)); // log2(bytes per feature column)
    const uint32_t F = a.n_features, C = a.n_classes, T = a.n_trees;
    const uint32_t top_recs = recs_upto(a.top_pairs);      // records per tree held in shared memory
    // vote counters, 32 / vote_bits classes per word, one column per FLOW: [vote_words][FPB]; the S lanes of
    // a flow add to it with shared-memory atomics (fields cannot carry into each other: a count is at most n_trees)
    const uint32_t per_shift = a.vote_bits == 8 ? 2u : 1u; // log2(counters per word)
    const uint32_t vote_words = GBDT ? C : (C + (1u << per_shift) - 1u) >> per_shift; // boosted: one float per class
    uint32_t* vT = reinterpret_cast<uint32_t*>(xT + (size_t)F * FPB);
    uint4* topT = reinterpret_cast<uint4*>(vT + (size_t)vote_words * FPB);   // [T][top_recs]
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t grp = lane / FPW;                       // which share of the trees this lane walks
    const uint32_t slot = wave * FPW + (lane % FPW);       // flow slot in the block's tile
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
    // The tile is read through absolute shared-memory addresses formed with bit operations: it heads the
    // block's shared memory, which in the kernels that use this walk is dynamic only, so the tile starts at
    // address 0 and "offset of the feature's row | offset of the flow's column" is the address.
    typedef __attribute__((address_space(3))) const float LdsFloat;
    const uint32_t tile_abs = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)reinterpret_cast<const char*>(xT);
    const uint32_t xl = tile_abs + slot * 4u; // address of the flow's column in the tile's first row
    uint32_t* vcol = vT + slot;
    const uint32_t rec_bytes = n_rec * 16u, top_bytes = top_recs * 16u;
    const uint32_t leaf_base = recs_upto(full_pairs); // record index of position 0 on tree level 2*full_pairs
    const uint32_t n_leaf = 1u << depth;

    // The three feature indices of a record sit in its last word as 8-bit fields, rotated so that the first
    // stands at bits 10..17: for a tile of 256 flows (a feature's row is 1024 bytes) masking the word gives
    // the byte offset of x[feature] in one operation, and a rotation by 8 or 16 bits brings a child's field
    // there.  Narrower tiles (two or four lanes per flow) rotate by one or two bits more.
    constexpr uint32_t kFieldMask = 0xFFu << kColShift;
    constexpr uint32_t kRot0 = kFeatRot - kColShift;
#define SF_FEAT_ROT(FW, SH) (*(LdsFloat*)(uintptr_t)((__builtin_amdgcn_alignbit((FW), (FW), (SH)) & kFieldMask) | xl))
#define SF_FEAT_0(FW) (kRot0 == 0u ? *(LdsFloat*)(uintptr_t)(((FW) & kFieldMask) | xl) : SF_FEAT_ROT(FW, kRot0))

    // two visits from one record; o is the byte offset of the record inside its tree.
    // EAGER = false: the child's feature is fetched after the parent's test (two shared-memory reads per
    // record, the second dependent on the first).  The record offset moves on as
    // 4 * o + 16 * (1 + 2 * right0 + right1) = ((o + sh) << 2) - 16 + 16 * right1 with sh = 8 or 16, the rotation
    // that selects the child's feature field.
    // EAGER = true: all three features up front (three independent reads), which is faster when latency
    // binds.  Which one wins is measured per kernel: lanes sharing a flow (few waves resident) and the
    // stand-alone vote kernel run eager (workload 2: 0.564 -> 0.543 ms), the fused feature + forest kernel
    // and the boosted form do not (0.531 against 0.570 ms, 0.72 against 0.78 ms).
#define SF_PAIR_STEP(REC, O)                                                                              \
    do {                                                                                                  \
        const uint32_t fw = (REC).w;                                                                      \
        const float x0 = SF_FEAT_0(fw);                                                                   \
        const bool r0 = !(x0 <= __uint_as_float((REC).x));                                                \
        if (!EAGER) {                                                                                     \
            const uint32_t sh = r0 ? 16u : 8u;                                                            \
            const float tc = __uint_as_float(r0 ? (REC).z : (REC).y);                                     \
            const float xc = SF_FEAT_ROT(fw, sh + kRot0);                                                 \
            const bool rc = !(xc <= tc);                                                                  \
            (O) = (((O) + sh) << 2) + (rc ? 0u : 0xFFFFFFF0u);                                            \
        } else {                                                                                          \
            const float x1 = SF_FEAT_ROT(fw, kRot0 + 8u);                                                 \
            const float x2 = SF_FEAT_ROT(fw, kRot0 + 16u);                                                \
            const bool r1 = !(x1 <= __uint_as_float((REC).y));                                            \
            const bool r2 = !(x2 <= __uint_as_float((REC).z));                                            \
            const uint32_t inc_l = r1 ? 32u : 16u, inc_r = r2 ? 64u : 48u;                                \
            (O) = 4u * (O) + (r0 ? inc_r : inc_l);                                                        \
        }                                                                                                 \
    } while (0)

    // lane group g walks trees g, g+S, ...; every group runs the same number of rounds so that
    // the loop stays wave-uniform; a slot past the last tree repeats it and does not vote
    const uint32_t per_grp = (T + S - 1u) / S;
    // one group: ILP trees from position q0 of the lane group's list
    auto walk_group = [&](auto ilp_tag, uint32_t q0) {
        constexpr int kIlp = decltype(ilp_tag)::value;
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
                const float x0 = SF_FEAT_0(rec[u].w);
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
            return;
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
    };
    {
        const uint32_t rem = per_grp % (uint32_t)kIlp;
        const bool short_tail = rem != 0 && rem <= (uint32_t)kIlpTail;
        const uint32_t full_end = short_tail ? per_grp - rem : per_grp; // (a longer tail runs as a full group with idle slots)
        uint32_t q0 = 0;
        for (; q0 < full_end; q0 += kIlp) walk_group(std::integral_constant<int, kIlp>{}, q0);
        if (short_tail) walk_group(std::integral_constant<int, kIlpTail>{}, q0);
    }
#undef SF_PAIR_STEP
#undef SF_FEAT_0
#undef SF_FEAT_ROT
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
    if (KEEP_ROWS) {
        // the features never left the chip: the row is written out only for a flow the gate hands on
        const uint32_t th = a.vmin[a.n_vmin > 1u ? (best < a.n_vmin ? best : a.n_vmin - 1u) : 0u];
        if (bestv < th) {
            float* dst = a.feat_out + (size_t)i * a.feat_out_ld;
            if (a.feat_out16) {
                for (uint32_t q = 0; q < F; q += 4u)
                    *reinterpret_cast<float4*>(dst + q) = make_float4(xT[(q + 0u) * FPB + slot], xT[(q + 1u) * FPB + slot],
                                                                    xT[(q + 2u) * FPB + slot], xT[(q + 3u) * FPB + slot]);
            } else {
                for (uint32_t q = 0; q < F; ++q) dst[q] = xT[q * FPB + slot];
            }
        }
    }
}

} // namespace sfforest
