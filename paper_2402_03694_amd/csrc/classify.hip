// All four steps behind one entry point, with steps 1-3 in ONE kernel: a block featurizes a tile of 256
// flows straight into the shared-memory columns the forest walk reads (Section 3.1 of the paper: the fast
// model sees every flow, from its first k packets) and walks the forest on them; the feature row of a
// flow leaves the chip only if the gate (Section 3.2) hands the flow on to the slow model.
//
// Why: the feature step is bound by vector arithmetic and by its memory pattern, the walk by gathers;
// with two blocks per compute unit one block's feature phase runs under the other's walk, and the
// feature matrix (256 bytes per flow written, then read again) is neither written nor read for the
// flows that stay with the fast model.
//
// Shared memory of a block: the tile [32 * windows][256] floats, behind it what the walk needs (vote
// counters, staged top records).  The sorting networks of the feature phase need a scratch column per
// lane; windows are computed from the last to the first, and every window but the first uses the
// first window's 32 columns (not written yet) as scratch, the first window the space behind the tile
// (the walk fills that only afterwards).
#include "featurize_core.h"
#include "forest_core.h"

namespace sf {
int forest_setup(sf_ctx* ctx, const char* who, const sf_forest* f, uint32_t feat_ld, sfforest::FastArgs& a, uint32_t* split,
                 size_t* lds);
}

namespace {

using namespace sfforest;

struct ClassifyArgs {
    uint32_t n_pkts;
    const uint32_t* off;
    const uint16_t* size;
    const float* iat;
    const uint8_t* dir;
    uint32_t n_windows;
    uint32_t depth[SF_MAX_WINDOWS];
    uint32_t wide_ok; // the packet arrays start on 16-byte (size, time) and 8-byte (direction) boundaries
    FastArgs fa;      // n_flows, model, outputs, gate; n_features = 32 * n_windows
};

template <int KMAX, bool KEEP_ROWS>
__global__ __launch_bounds__(256) void featurize_forest(ClassifyArgs c)
{
    constexpr uint32_t FPB = 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const FastArgs& a = c.fa;
    float* xT = reinterpret_cast<float*>(smem_raw); // [32 * windows][FPB]
    uint32_t* behind = reinterpret_cast<uint32_t*>(xT + (size_t)a.n_features * FPB);
    const uint32_t tid = threadIdx.x;
    const uint32_t i = blockIdx.x * FPB + tid;
    const bool live = i < a.n_flows;
    // a lane past the last flow works on the last flow (its loads stay inside the arrays) and writes nothing
    const uint32_t flow = live ? i : a.n_flows - 1u;
    uint32_t o, n;
    {
        uint32_t b = c.off[flow], e = c.off[flow + 1];
        b = b < c.n_pkts ? b : c.n_pkts; // clamp: malformed offsets must not leave the arrays
        e = e < c.n_pkts ? e : c.n_pkts;
        e = e < b ? b : e;
        o = b;
        n = e - b;
    }
    const uint32_t dmax = c.depth[c.n_windows - 1];
    const int avail = (int)(n < dmax ? n : dmax);
    float s[KMAX], t[KMAX];
    uint64_t dmask = 0;
    if (avail == KMAX && (o & 7u) == 0 && c.wide_ok) {
        // whole window present and 16-byte aligned (array bases included): wide loads
#pragma unroll
        for (int q = 0; q < KMAX / 8; ++q) {
            const uint4 sz = *reinterpret_cast<const uint4*>(c.size + o + 8 * q);
            const uint32_t w[4] = {sz.x, sz.y, sz.z, sz.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                s[8 * q + 2 * k] = (float)(w[k] & 0xFFFFu);
                s[8 * q + 2 * k + 1] = (float)(w[k] >> 16);
            }
            const float4 t0 = *reinterpret_cast<const float4*>(c.iat + o + 8 * q);
            const float4 t1 = *reinterpret_cast<const float4*>(c.iat + o + 8 * q + 4);
            t[8 * q + 0] = t0.x; t[8 * q + 1] = t0.y; t[8 * q + 2] = t0.z; t[8 * q + 3] = t0.w;
            t[8 * q + 4] = t1.x; t[8 * q + 5] = t1.y; t[8 * q + 6] = t1.z; t[8 * q + 7] = t1.w;
            const uint2 dd = *reinterpret_cast<const uint2*>(c.dir + o + 8 * q);
            const uint32_t dw[2] = {dd.x, dd.y};
#pragma unroll
            for (int k = 0; k < 8; ++k) dmask |= (uint64_t)((dw[k >> 2] >> (8 * (k & 3))) & 1u) << (8 * q + k);
        }
    } else {
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            if (j < avail) {
                s[j] = (float)c.size[o + j];
                t[j] = c.iat[o + j];
                dmask |= (uint64_t)(c.dir[o + j] & 1u) << j;
            } else {
                s[j] = 0.f;
                t[j] = 0.f;
            }
        }
    }
    // a time with its sign bit set anywhere in the wave: the order statistics take the general path
    uint32_t sign_bits = 0;
#pragma unroll
    for (int j = 0; j < KMAX; ++j) sign_bits |= __float_as_uint(t[j]);
    const bool signed_times = __any((int)(sign_bits >> 31));
    for (int w = (int)c.n_windows - 1; w >= 0; --w) {
        const int dw = (int)c.depth[w];
        const int m = avail < dw ? avail : dw;
        // every address below is the lane's own column: no two lanes (or waves) share a word
        uint32_t* col = (w > 0 ? reinterpret_cast<uint32_t*>(xT) : behind) + tid;
        float* dst = xT + (size_t)(32 * w) * FPB + tid;
        // the smallest network that covers every lane's window (wave-uniform choice)
        if (KMAX >= 16 && __any(m > 8))
            sffeat::window_stats<(KMAX >= 16 ? 16 : KMAX), KMAX>(s, t, dmask, m, signed_times, col, FPB, dst, FPB);
        else
            sffeat::window_stats<8, KMAX>(s, t, dmask, m, signed_times, col, FPB, dst, FPB);
    }
    __syncthreads(); // the space behind the tile is free: the walk may stage its records there
    forest_walk<256, 1, false, false, KEEP_ROWS>(a, xT, i, i, live);
}

template <int KMAX, bool KEEP_ROWS>
int launch_fused(sf_ctx* ctx, const ClassifyArgs& c, size_t lds, int slot)
{
    SF_ALLOW_LDS(ctx, slot, (featurize_forest<KMAX, KEEP_ROWS>));
    const uint32_t grid = (c.fa.n_flows + 255u) / 256u;
    featurize_forest<KMAX, KEEP_ROWS><<<grid, 256, lds, ctx->stream>>>(c);
    SF_LAUNCH_CHECK(ctx, "featurize_forest");
    return SF_OK;
}

// steps 1-3 for both entry points; keep_rows: feature rows of the flows the gate hands on are wanted
int run_features_and_forest(sf_ctx* ctx, const char* who, const sf_packets* pk, const sf_feat_cfg* cfg, const sf_forest* forest,
                            const uint16_t* host_vmin, uint32_t n_vmin, bool keep_rows, float* feat, uint32_t feat_ld,
                            uint16_t* pred, uint16_t* top_votes, uint16_t* labels, bool* labels_done)
{
    if (!pk || !cfg || !forest) return sf::fail(ctx, SF_EINVAL, "%s: packets, config or forest is NULL", who);
    if (!host_vmin || n_vmin < 1 || n_vmin > SF_MAX_CLASSES)
        return sf::fail(ctx, SF_EINVAL, "%s: host_vmin missing or n_vmin %u outside 1..%d", who, n_vmin, SF_MAX_CLASSES);
    if (cfg->n_windows < 1 || cfg->n_windows > SF_MAX_WINDOWS)
        return sf::fail(ctx, SF_EINVAL, "%s: n_windows %u outside 1..%d", who, cfg->n_windows, SF_MAX_WINDOWS);
    for (uint32_t w = 0; w < cfg->n_windows; ++w) {
        if (cfg->depth[w] < 1 || cfg->depth[w] > SF_MAX_DEPTH_PKTS)
            return sf::fail(ctx, SF_EINVAL, "%s: depth[%u] = %u outside 1..%d", who, w, cfg->depth[w], SF_MAX_DEPTH_PKTS);
        if (w && cfg->depth[w] <= cfg->depth[w - 1]) return sf::fail(ctx, SF_EINVAL, "%s: depths must be strictly increasing", who);
    }
    const uint32_t F = 32u * cfg->n_windows;
    if (keep_rows && feat_ld < F) return sf::fail(ctx, SF_EINVAL, "%s: feat_ld %u < %u", who, feat_ld, F);
    if (forest->n_features > F)
        return sf::fail(ctx, SF_EINVAL, "%s: the forest splits on %u features, the windows give %u", who, forest->n_features, F);
    if (pk->n_pkts >> 32) return sf::fail(ctx, SF_EINVAL, "%s: n_pkts exceeds 32-bit offsets", who);
    const uint32_t n = pk->n_flows;
    *labels_done = false;
    if (n == 0) return SF_OK;
    if (!pk->flow_off || !pred || !top_votes || (keep_rows && !feat))
        return sf::fail(ctx, SF_EINVAL, "%s: flow_off, feat, pred or top_votes is NULL", who);
    if (pk->n_pkts && (!pk->pkt_size || !pk->pkt_iat || !pk->pkt_dir)) return sf::fail(ctx, SF_EINVAL, "%s: packet arrays missing", who);

    // the forest with the tile's width (the walk's shared-memory layout follows the tile, not the model)
    sf_forest wide = *forest;
    wide.n_features = F;
    ClassifyArgs c = {};
    uint32_t split = 1;
    size_t lds = 0;
    const uint32_t dmax = cfg->depth[cfg->n_windows - 1];
    int rc = sf::forest_setup(ctx, who, &wide, F, c.fa, &split, &lds);
    if (rc != SF_OK) return rc;
    // scratch of the first window's sorting network behind the tile: one column per element
    uint32_t n0 = 8;
    while (n0 < cfg->depth[0] && n0 < 16u) n0 *= 2;
    const size_t lds_feat = (size_t)F * 1024 + (size_t)n0 * 1024;
    const bool fused = split == 1 && dmax <= 16 && (lds > lds_feat ? lds : lds_feat) <= 80 * 1024;
    if (!fused) {
        // shapes the fused kernel does not cover (windows deeper than 16 packets, whose registers would leave one
        // block per compute unit; forests that run several lanes per flow): the same results from the separate
        // kernels, with every feature row written
        if (!feat || feat_ld < F) return sf::fail(ctx, SF_EINVAL, "%s: this shape needs the feature matrix", who);
        rc = sf_featurize(ctx, pk, cfg, feat, feat_ld, nullptr);
        if (rc != SF_OK) return rc;
        return sf_fast_infer(ctx, feat, feat_ld, n, forest, nullptr, pred, top_votes, nullptr);
    }
    c.n_pkts = (uint32_t)pk->n_pkts;
    c.off = pk->flow_off;
    c.size = pk->pkt_size;
    c.iat = pk->pkt_iat;
    c.dir = pk->pkt_dir;
    c.n_windows = cfg->n_windows;
    for (int w = 0; w < SF_MAX_WINDOWS; ++w) c.depth[w] = w < (int)cfg->n_windows ? cfg->depth[w] : 0;
    c.wide_ok = (((uintptr_t)c.size | (uintptr_t)c.iat) & 15u) == 0 && ((uintptr_t)c.dir & 7u) == 0;
    c.fa.n_flows = n;
    c.fa.n_rows = n;
    c.fa.pred = pred;
    c.fa.top = top_votes;
    c.fa.labels = labels; // the label array starts as the fast prediction (Section 4.4); the slow model overwrites its flows
    *labels_done = labels != nullptr;
    c.fa.feat_out = feat;
    c.fa.feat_out_ld = feat_ld;
    c.fa.feat_out16 = ((uintptr_t)feat & 15u) == 0 && (feat_ld & 3u) == 0;
    c.fa.n_vmin = n_vmin;
    for (uint32_t k = 0; k < SF_MAX_CLASSES; ++k) c.fa.vmin[k] = host_vmin[k < n_vmin ? k : n_vmin - 1];
    if (lds_feat > lds) lds = lds_feat;
    const int base = sf::kLdsClassify + (keep_rows ? 2 : 0);
    if (dmax <= 8) return keep_rows ? launch_fused<8, true>(ctx, c, lds, base) : launch_fused<8, false>(ctx, c, lds, base);
    return keep_rows ? launch_fused<16, true>(ctx, c, lds, base + 1) : launch_fused<16, false>(ctx, c, lds, base + 1);
}

} // namespace

namespace {
// labels = pred for every flow (the separate kernels do not write labels: one small copy)
__global__ __launch_bounds__(256) void labels_from_pred(const uint16_t* __restrict__ pred, uint16_t* __restrict__ labels, uint32_t n)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) labels[i] = pred[i];
}
} // namespace

extern "C" int sf_featurize_fast_infer(sf_ctx* ctx, const sf_packets* pk, const sf_feat_cfg* cfg, const sf_forest* forest,
                                       const uint16_t* host_vmin, uint32_t n_vmin, float* feat, uint32_t feat_ld,
                                       uint16_t* pred, uint16_t* top_votes, uint16_t* labels)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_featurize_fast_infer: ctx is NULL");
    bool done = false;
    const int rc = run_features_and_forest(ctx, "sf_featurize_fast_infer", pk, cfg, forest, host_vmin, n_vmin, feat != nullptr, feat,
                                           feat_ld, pred, top_votes, labels, &done);
    if (rc != SF_OK || !labels || done || !pk || pk->n_flows == 0) return rc;
    uint32_t blocks = (pk->n_flows + 255u) / 256u;
    labels_from_pred<<<blocks > 4096u ? 4096u : blocks, 256, 0, ctx->stream>>>(pred, labels, pk->n_flows);
    SF_LAUNCH_CHECK(ctx, "labels_from_pred");
    return SF_OK;
}

extern "C" int sf_classify(sf_ctx* ctx, const sf_packets* pk, const sf_feat_cfg* cfg, const sf_forest* forest,
                           const uint16_t* host_vmin, uint32_t n_vmin, const sf_mlp* mlp, float* feat, uint32_t feat_ld,
                           uint16_t* pred, uint16_t* top_votes, uint32_t* esc_idx, uint32_t* esc_count, float* logits,
                           uint16_t* labels)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_classify: ctx is NULL");
    if (!cfg || !mlp || !pk) return sf::fail(ctx, SF_EINVAL, "sf_classify: packets, config or mlp is NULL");
    if (!esc_count) return sf::fail(ctx, SF_EINVAL, "sf_classify: esc_count is NULL");
    const bool raw = cfg->raw_pkts > 0;
    const uint32_t n = pk->n_flows;
    if (n && (!esc_idx || !labels)) return sf::fail(ctx, SF_EINVAL, "sf_classify: esc_idx or labels is NULL");
    bool labels_done = false;
    int rc = run_features_and_forest(ctx, "sf_classify", pk, cfg, forest, host_vmin, n_vmin, !raw, feat, feat_ld, pred, top_votes,
                                     labels, &labels_done);
    if (rc != SF_OK) return rc;
    rc = sf_route(ctx, top_votes, pred, n, host_vmin, n_vmin, esc_idx, esc_count);
    if (rc != SF_OK || n == 0) return rc;
    return sf_slow_infer(ctx, raw ? nullptr : feat, raw ? 0u : feat_ld, raw ? pk : nullptr, raw ? cfg : nullptr, esc_idx, esc_count, n,
                         n, mlp, labels_done ? nullptr : pred, logits, labels);
}
