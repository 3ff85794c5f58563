// Context life cycle, error text, workspace sizing and the device-side validators.
#include <cmath>
#include <cstring>
#include <new>

#include "common.h"

namespace sf {

static char g_err[512] = "";

void set_global_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int fail(sf_ctx* ctx, int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    if (ctx)
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    else
        vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

size_t route_scratch_bytes(uint32_t n_flows)
{
    (void)n_flows;
    return align_up(4096 * sizeof(uint32_t)); // per-block counts, block count is capped
}

size_t slow_row_bytes(uint32_t n_h1, uint32_t n_h2, int dtype)
{
    size_t el = dtype == SF_F32 ? 4 : 2;
    return ((size_t)n_h1 + n_h2) * el;
}

} // namespace sf

namespace sf {
size_t reordered_bytes(uint32_t N, uint32_t K); // slow_fused.hip
int route_static_init(sf_ctx* ctx);             // route.hip: address of this device's static block counts
}

extern "C" size_t sf_workspace_bytes(uint32_t max_flows, uint32_t n_trees, uint32_t tree_depth,
                                     uint32_t n_in, uint32_t n_h1, uint32_t n_h2)
{
    using namespace sf;
    size_t total = kFlagBytes;
    total = align_up(total) + forest_pack_bytes(n_trees, tree_depth);
    total = align_up(total) + route_scratch_bytes(max_flows);
    total = align_up(total) + tree_tier_bytes(SF_MAX_TREE_DEPTH); // the single-tree tier at any depth
    total = align_up(total) + kQuantileScratch;                   // histograms and state of sf_score_quantiles
    if (n_h1 || n_h2) {
        // operand-ordered copies of the three weight matrices
        total = align_up(total) + reordered_bytes(n_h1, n_in ? n_in : 1) + reordered_bytes(n_h2, n_h1 ? n_h1 : 1) +
                reordered_bytes(32, n_h2 ? n_h2 : 1) + 4 * kAlign;
        uint32_t rows = max_flows < kSlowWantRows ? max_flows : kSlowWantRows;
        if (rows < kSlowMinRows) rows = kSlowMinRows;
        total = align_up(total) + align_up((size_t)rows * slow_row_bytes(n_h1, n_h2, SF_F32)) + 2 * kAlign;
    }
    return align_up(total) + kAlign;
}

extern "C" int sf_create(sf_ctx** out, void* hip_stream, void* workspace, size_t workspace_bytes)
{
    if (!out) return sf::fail(nullptr, SF_EINVAL, "sf_create: out is NULL");
    *out = nullptr;
    if (!workspace || workspace_bytes < sf::kFlagBytes)
        return sf::fail(nullptr, SF_EINVAL, "sf_create: workspace missing or smaller than %zu bytes",
                        sf::kFlagBytes);
    if ((uintptr_t)workspace % sf::kAlign)
        return sf::fail(nullptr, SF_EINVAL, "sf_create: workspace is not 256-byte aligned");
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return sf::fail(nullptr, SF_EHIP, "sf_create: hipGetDevice failed: %s", hipGetErrorString(e));
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess)
        return sf::fail(nullptr, SF_EHIP, "sf_create: hipGetDeviceProperties failed: %s",
                        hipGetErrorString(e));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return sf::fail(nullptr, SF_EUNSUPPORTED, "sf_create: device is %s, the kernels are built for gfx950",
                        prop.gcnArchName);
    sf_ctx* c = new (std::nothrow) sf_ctx;
    if (!c) return sf::fail(nullptr, SF_ENOMEM, "sf_create: out of host memory");
    c->stream = (hipStream_t)hip_stream;
    c->ws = (char*)workspace;
    c->ws_bytes = workspace_bytes;
    c->device = dev;
    c->n_cu = prop.multiProcessorCount;
    c->d_flags = (uint32_t*)workspace;
    c->lds_ready = 0;
    c->err[0] = 0;
    // set-up for the entry point that uses the static scratch array: look its address up now, once per device
    const int rs = sf::route_static_init(c);
    if (rs != SF_OK) {
        sf::set_global_error("sf_create: %s", c->err);
        delete c;
        return rs;
    }
    *out = c;
    return SF_OK;
}

extern "C" void sf_destroy(sf_ctx* ctx) { delete ctx; }

extern "C" const char* sf_last_error(const sf_ctx* ctx) { return ctx ? ctx->err : sf::g_err; }

extern "C" uint32_t sf_vmin_from_theta(float theta, uint32_t n_trees)
{
    // a 24-bit significand times a 32-bit integer is exact in long double's 64-bit significand;
    // for n_trees < 2^29 it is exact in double as well
    long double p = (long double)theta * (long double)n_trees;
    long double c = ceill(p);
    if (!(c > 0.0L)) return 0;
    if (c > 65535.0L) return 65535;
    return (uint32_t)c;
}

// ---- validators -----------------------------------------------------------------------

namespace {

__global__ void check_packets(uint32_t n_flows, uint64_t n_pkts, const uint32_t* __restrict__ off,
                              const float* __restrict__ iat, const uint8_t* __restrict__ dir,
                              uint32_t* __restrict__ bad)
{
    uint64_t gid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    uint32_t b = 0;
    for (uint64_t i = gid; i <= n_flows; i += stride) {
        uint32_t o = off[i];
        if (i == 0 && o != 0) b |= 1;
        if (i == n_flows && o != n_pkts) b |= 2;
        if (i < n_flows && off[i + 1] < o) b |= 4;
    }
    for (uint64_t j = gid; j < n_pkts; j += stride) {
        if (dir[j] > 1) b |= 8;
        if (!(fabsf(iat[j]) <= 3.402823466e38f)) b |= 16;
    }
    if (b) atomicOr(bad, b);
}

__global__ void check_forest(uint64_t n_nodes, uint64_t n_leaves, uint32_t n_features,
                             uint32_t n_classes, const uint16_t* __restrict__ nf,
                             const uint8_t* __restrict__ ll, uint32_t* __restrict__ bad)
{
    uint64_t gid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    uint32_t b = 0;
    for (uint64_t i = gid; i < n_nodes; i += stride)
        if (nf[i] >= n_features) b |= 1;
    for (uint64_t i = gid; i < n_leaves; i += stride)
        if (ll[i] >= n_classes) b |= 2;
    if (b) atomicOr(bad, b);
}

__global__ void clear_word(uint32_t* w) { *w = 0; }

int read_flag(sf_ctx* ctx, uint32_t* d, uint32_t* h)
{
    SF_HIP(ctx, hipMemcpyAsync(h, d, 4, hipMemcpyDeviceToHost, ctx->stream));
    SF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return SF_OK;
}

} // namespace

extern "C" int sf_validate_packets(sf_ctx* ctx, const sf_packets* pk)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_validate_packets: ctx is NULL");
    if (!pk || !pk->flow_off) return sf::fail(ctx, SF_EINVAL, "sf_validate_packets: packets missing");
    if (pk->n_pkts && (!pk->pkt_size || !pk->pkt_iat || !pk->pkt_dir))
        return sf::fail(ctx, SF_EINVAL, "sf_validate_packets: packet arrays missing");
    if (pk->n_pkts >> 32) return sf::fail(ctx, SF_EINVAL, "sf_validate_packets: n_pkts exceeds 32-bit offsets");
    uint32_t* flag = ctx->d_flags + 8;
    clear_word<<<1, 1, 0, ctx->stream>>>(flag);
    check_packets<<<1024, 256, 0, ctx->stream>>>(pk->n_flows, pk->n_pkts, pk->flow_off, pk->pkt_iat,
                                                 pk->pkt_dir, flag);
    SF_LAUNCH_CHECK(ctx, "check_packets");
    uint32_t h = 0;
    int rc = read_flag(ctx, flag, &h);
    if (rc) return rc;
    if (h)
        return sf::fail(ctx, SF_EDATA,
                        "packet records violate the layout (mask 0x%x: 1 first offset, 2 last offset, "
                        "4 decreasing offsets, 8 direction, 16 non-finite time)", h);
    return SF_OK;
}

extern "C" int sf_validate_forest(sf_ctx* ctx, const sf_forest* f)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_validate_forest: ctx is NULL");
    if (!f || !f->node_feat || !f->node_thr || !f->leaf_label)
        return sf::fail(ctx, SF_EINVAL, "sf_validate_forest: forest arrays missing");
    if (f->depth < 1 || f->depth > SF_MAX_TREE_DEPTH)
        return sf::fail(ctx, SF_EINVAL, "sf_validate_forest: depth %u outside 1..%d", f->depth, SF_MAX_TREE_DEPTH);
    uint64_t nn = (uint64_t)f->n_trees * (((uint64_t)1 << f->depth) - 1);
    uint64_t nl = (uint64_t)f->n_trees * ((uint64_t)1 << f->depth);
    uint32_t* flag = ctx->d_flags + 9;
    clear_word<<<1, 1, 0, ctx->stream>>>(flag);
    check_forest<<<512, 256, 0, ctx->stream>>>(nn, nl, f->n_features, f->n_classes, f->node_feat,
                                               f->leaf_label, flag);
    SF_LAUNCH_CHECK(ctx, "check_forest");
    uint32_t h = 0;
    int rc = read_flag(ctx, flag, &h);
    if (rc) return rc;
    if (h)
        return sf::fail(ctx, SF_EDATA, "forest violates the layout (mask 0x%x: 1 feature index, 2 leaf label)", h);
    return SF_OK;
}
