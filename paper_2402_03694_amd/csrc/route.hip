// Step 4: the gate of Section 3.2 of the paper in integer form, and the compaction of the
// uncertain flows into an ascending index list.  Three forms of the gate share the kernels:
// votes against a threshold (universal or per predicted class), a leaf's class share against
// theta (the single-tree tier), and either of them over the rows of an earlier list (the
// second gate of a three-tier cascade, Section 3.1), which writes flow numbers, not rows.
//
// Two launches, no spinning between blocks: the first counts the escalated flows of each
// block's contiguous chunk; the second adds up the counts of the blocks before it, then
// re-evaluates the gate and writes the indices in order (a wave-level prefix sum of per-lane
// pop-counts gives each lane its write position).  The count stays on the device.
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "common.h"

namespace {

constexpr int kBlock = 256;
constexpr int kPerLane = 8;                // consecutive flows per lane per tile
constexpr int kTile = kBlock * kPerLane;   // flows per block per tile
constexpr uint32_t kMaxBlocks = 4096;

struct RouteArgs {
    const uint16_t* top;
    const uint16_t* pred;
    const uint16_t* total;     // ratio gate: per-row denominators (NULL = vote gate)
    float theta;               // ratio gate: escalate iff top / total < theta
    const float* score;        // score gate: a real-valued uncertainty per row (NULL = the integer gates)
    float score_thr;           // score gate: escalate iff score > score_thr
    const uint32_t* src_idx;   // rows are the entries of this list (NULL = rows are flows)
    const uint32_t* src_count; // device-side length of that list (n is then its capacity)
    uint32_t n;
    uint32_t chunk; // flows per block, a multiple of kTile
    uint32_t n_vmin;
    uint16_t vmin[SF_MAX_CLASSES];
    uint32_t* counts;
    uint32_t* esc_idx;
    uint32_t* esc_count;
};

// rows the gate runs over: the whole array, or as many as the earlier list holds
__device__ __forceinline__ uint32_t live_rows(const RouteArgs& a)
{
    if (!a.src_count) return a.n;
    const uint32_t c = *a.src_count;
    return c < a.n ? c : a.n;
}

// top / total < theta without rounding: binary32 theta times a 16-bit total is exact in binary64.
// A leaf without samples has no distribution; it escalates for any positive theta.
__device__ __forceinline__ bool ratio_below(uint32_t top, uint32_t total, float theta)
{
    if (total == 0) return theta > 0.f;
    return (double)top < (double)theta * (double)total;
}

// 8-bit mask of the lane's rows [base, base+8) that escalate; n = live_rows(a)
__device__ __forceinline__ uint32_t gate_mask(const RouteArgs& a, uint32_t n, uint32_t base)
{
    uint32_t m = 0;
    if (base >= n) return 0;
    if (a.score) {
        for (int k = 0; k < kPerLane; ++k) {
            const uint32_t i = base + k;
            if (i < n) m |= (a.score[i] > a.score_thr ? 1u : 0u) << k;
        }
        return m;
    }
    if (a.total) {
        for (int k = 0; k < kPerLane; ++k) {
            const uint32_t i = base + k;
            if (i < n) m |= (ratio_below(a.top[i], a.total[i], a.theta) ? 1u : 0u) << k;
        }
        return m;
    }
    if (base + kPerLane <= n && a.n_vmin == 1) {
        // base is a multiple of 8: the 16-byte load is aligned whenever top is
        uint16_t v[kPerLane];
        if ((reinterpret_cast<uintptr_t>(a.top) & 15u) == 0) {
            const uint4 w = *reinterpret_cast<const uint4*>(a.top + base);
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                v[2 * k] = (uint16_t)(ww[k] & 0xFFFFu);
                v[2 * k + 1] = (uint16_t)(ww[k] >> 16);
            }
        } else {
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) v[k] = a.top[base + k];
        }
        const uint16_t th = a.vmin[0];
#pragma unroll
        for (int k = 0; k < kPerLane; ++k) m |= (v[k] < th ? 1u : 0u) << k;
        return m;
    }
    for (int k = 0; k < kPerLane; ++k) {
        const uint32_t i = base + k;
        if (i < n) {
            uint16_t th = a.vmin[0];
            if (a.n_vmin > 1) {
                uint32_t p = a.pred[i];
                p = p < a.n_vmin ? p : a.n_vmin - 1;
                th = a.vmin[p];
            }
            m |= (a.top[i] < th ? 1u : 0u) << k;
        }
    }
    return m;
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

// exclusive prefix of v over the block and the block total; sm holds kBlock/64 + 1 words
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* sm, uint32_t& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t inc = wave_inclusive_scan(v);
    __syncthreads(); // sm may still be read from the previous tile
    if (lane == 63) sm[wave] = inc;
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) {
        const uint32_t s = sm[w];
        before += w < wave ? s : 0;
        tot += s;
    }
    total = tot;
    return before + inc - v;
}

__global__ __launch_bounds__(kBlock) void route_count(RouteArgs a)
{
    __shared__ uint32_t sm[kBlock / 64];
    const uint32_t begin = blockIdx.x * a.chunk;
    const uint32_t n = live_rows(a);
    uint32_t c = 0;
    for (uint32_t t = 0; t < a.chunk; t += kTile) c += __popc(gate_mask(a, n, begin + t + threadIdx.x * kPerLane));
    const uint32_t inc = wave_inclusive_scan(c);
    if ((threadIdx.x & 63) == 63) sm[threadIdx.x >> 6] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t tot = 0;
        for (int w = 0; w < kBlock / 64; ++w) tot += sm[w];
        a.counts[blockIdx.x] = tot;
    }
}

__global__ __launch_bounds__(kBlock) void route_scatter(RouteArgs a)
{
    __shared__ uint32_t sm[kBlock / 64];
    // sum of the counts of all earlier blocks (every lane ends up with the block-wide total)
    uint32_t part = 0;
    for (uint32_t b = threadIdx.x; b < blockIdx.x; b += kBlock) part += a.counts[b];
    uint32_t run;
    block_exclusive_scan(part, sm, run);
    const uint32_t begin = blockIdx.x * a.chunk;
    const uint32_t n = live_rows(a);
    for (uint32_t t = 0; t < a.chunk; t += kTile) {
        const uint32_t base = begin + t + threadIdx.x * kPerLane;
        const uint32_t m = gate_mask(a, n, base);
        uint32_t tile_total;
        uint32_t pos = run + block_exclusive_scan(__popc(m), sm, tile_total);
#pragma unroll
        for (int k = 0; k < kPerLane; ++k)
            if (m & (1u << k)) a.esc_idx[pos++] = a.src_idx ? a.src_idx[base + k] : base + k;
        run += tile_total;
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *a.esc_count = run;
}

__global__ void route_zero(uint32_t* esc_count) { *esc_count = 0; }

// ---- calibration: histogram of the integer score ------------------------------------------

constexpr uint32_t kHistLdsBins = 8192; // bins a block can keep in shared memory (32 KB)

__global__ __launch_bounds__(256) void hist_zero(uint32_t* hist, uint32_t bins)
{
    for (uint32_t b = blockIdx.x * blockDim.x + threadIdx.x; b < bins; b += gridDim.x * blockDim.x) hist[b] = 0;
}

// hist[v] += number of flows with top_votes == v (values above n_trees are counted in the last bin)
__global__ __launch_bounds__(256) void hist_scores(const uint16_t* __restrict__ top, uint32_t n, uint32_t bins,
                                                   uint32_t* __restrict__ hist)
{
    __shared__ uint32_t sh[kHistLdsBins];
    const bool local = bins <= kHistLdsBins;
    if (local) {
        for (uint32_t b = threadIdx.x; b < bins; b += blockDim.x) sh[b] = 0;
        __syncthreads();
    }
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
        uint32_t v = top[i];
        v = v < bins ? v : bins - 1u;
        if (local)
            atomicAdd(&sh[v], 1u);
        else
            atomicAdd(&hist[v], 1u);
    }
    if (local) {
        __syncthreads();
        for (uint32_t b = threadIdx.x; b < bins; b += blockDim.x)
            if (sh[b]) atomicAdd(&hist[b], sh[b]);
    }
}

// hist[((pred * bins) + top_votes) * 2 + wrong] += 1, wrong = (pred != truth); out-of-range values are clamped
__global__ __launch_bounds__(256) void hist_class_scores(const uint16_t* __restrict__ top, const uint16_t* __restrict__ pred,
                                                         const uint16_t* __restrict__ truth, uint32_t n, uint32_t bins,
                                                         uint32_t n_classes, uint32_t* __restrict__ hist)
{
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
        uint32_t v = top[i], c = pred[i];
        v = v < bins ? v : bins - 1u;
        c = c < n_classes ? c : n_classes - 1u;
        atomicAdd(&hist[((size_t)c * bins + v) * 2u + (pred[i] != truth[i] ? 1u : 0u)], 1u);
    }
}

// ---- calibration on a real-valued score: exact order statistics by radix selection on the device ------
// Three histogram passes over order-preserving 32-bit keys (11 + 11 + 10 bits); after each pass one small
// block finds the bin that holds the wanted rank and narrows the key prefix.  Everything stays on the
// device until the thresholds are read back.

// order-preserving 32-bit key of a binary32 value (negative values below positive ones)
__device__ __forceinline__ uint32_t float_key(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr uint32_t kSelBins = 2048;
constexpr uint32_t kMaxQuantiles = 256;

struct SelState {
    uint32_t prefix; // the key bits fixed so far (right-aligned)
    uint32_t rank;   // 1-based position of the wanted element among the scores that share the prefix
};

// hist[(key >> shift) & mask] += 1 for every score whose key has the state's prefix above prefix_shift
// (st == NULL: every score).  A block counts in shared memory; lanes of a wave with the same bin are
// counted with one add (scores cluster: most of a wave lands in a handful of bins).
__global__ __launch_bounds__(256) void sel_hist(const float* __restrict__ score, uint32_t n, uint32_t shift, uint32_t mask,
                                                uint32_t prefix_shift, const SelState* __restrict__ st,
                                                uint32_t* __restrict__ hist)
{
    __shared__ uint32_t sh[kSelBins];
    for (uint32_t b = threadIdx.x; b < kSelBins; b += blockDim.x) sh[b] = 0;
    __syncthreads();
    const bool all = st == nullptr;
    const uint32_t prefix = all ? 0u : st->prefix;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t rounded = (n + 63u) & ~63u; // whole waves stay in the loop together
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < rounded; i += (uint64_t)gridDim.x * blockDim.x) {
        bool in = i < n;
        const uint32_t key = in ? float_key(score[i]) : 0u;
        in = in && (all || (key >> prefix_shift) == prefix);
        const uint32_t bin = (key >> shift) & mask;
        unsigned long long todo = __ballot(in);
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const uint32_t lb = (uint32_t)__shfl((int)bin, leader, 64);
            const unsigned long long same = __ballot(in && bin == lb);
            if ((int)lane == leader) atomicAdd(&sh[lb], (uint32_t)__popcll(same));
            todo &= ~same;
        }
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < kSelBins; b += blockDim.x)
        if (sh[b]) atomicAdd(&hist[b], sh[b]);
}

// One block.  Finds the bin of hist[0..bins) that holds the state's rank, appends its `bits` bits to the
// prefix and reduces the rank to the position inside that bin.  first_rank != 0 starts a new selection
// (prefix empty, rank = first_rank).  clear (may be hist itself) is zero-filled for the next pass.
// out != NULL (last pass): the finished key is turned back into the binary32 value it encodes.
__global__ __launch_bounds__(256) void sel_pick(const uint32_t* __restrict__ hist, uint32_t bins, uint32_t bits,
                                                SelState* __restrict__ st, uint32_t first_rank, uint32_t* clear,
                                                float* __restrict__ out)
{
    __shared__ uint32_t sh[kSelBins];
    __shared__ uint32_t part[256];
    const uint32_t tid = threadIdx.x;
    for (uint32_t b = tid; b < kSelBins; b += 256u) sh[b] = b < bins ? hist[b] : 0u;
    __syncthreads();
    for (uint32_t b = tid; b < kSelBins; b += 256u) clear[b] = 0u;
    constexpr uint32_t per = kSelBins / 256u;
    uint32_t mine = 0;
    for (uint32_t k = 0; k < per; ++k) mine += sh[tid * per + k];
    part[tid] = mine;
    __syncthreads();
    for (uint32_t d = 1; d < 256u; d <<= 1) { // inclusive prefix sums over the threads' totals
        const uint32_t v = tid >= d ? part[tid - d] : 0u;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    const uint32_t rank = first_rank ? first_rank : st->rank;
    const uint32_t prefix = first_rank ? 0u : st->prefix;
    const uint32_t total = part[255];
    const uint32_t want = rank < 1u ? 1u : (rank > total ? total : rank); // total >= rank by construction
    const uint32_t incl = part[tid], excl = incl - mine;
    if (want > excl && want <= incl) { // exactly one thread
        uint32_t seen = excl, bin = tid * per;
        for (uint32_t k = 0; k < per; ++k) {
            if (seen + sh[tid * per + k] >= want) {
                bin = tid * per + k;
                break;
            }
            seen += sh[tid * per + k];
        }
        const uint32_t key = (prefix << bits) | bin;
        st->prefix = key;
        st->rank = want - seen;
        if (out) *out = __uint_as_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
    }
}

// shared launch of the two kernels; a.top, a.pred, a.total, a.theta, a.src_*, a.n, a.n_vmin and
// a.vmin are filled by the caller.  counts: kMaxBlocks words of device scratch, or NULL to take
// them from the context's workspace.
int launch_route(sf_ctx* ctx, const char* who, RouteArgs& a, uint32_t* esc_idx, uint32_t* esc_count,
                 uint32_t* counts = nullptr)
{
    if (!counts) {
        sf::Carve ws(ctx);
        // workspace contents do not outlive a call: every entry point carves from the start
        counts = (uint32_t*)ws.take(sf::route_scratch_bytes(a.n));
        if (!counts)
            return sf::fail(ctx, SF_ENOMEM, "%s: workspace too small for %zu bytes of block counts", who,
                            sf::route_scratch_bytes(a.n));
    }
    uint64_t tiles = ((uint64_t)a.n + kTile - 1) / kTile;
    uint64_t tiles_per_block = (tiles + kMaxBlocks - 1) / kMaxBlocks;
    a.chunk = (uint32_t)(tiles_per_block * kTile);
    const uint32_t grid = (uint32_t)((tiles + tiles_per_block - 1) / tiles_per_block);
    a.counts = counts;
    a.esc_idx = esc_idx;
    a.esc_count = esc_count;
    route_count<<<grid, kBlock, 0, ctx->stream>>>(a);
    SF_LAUNCH_CHECK(ctx, "route_count");
    route_scatter<<<grid, kBlock, 0, ctx->stream>>>(a);
    SF_LAUNCH_CHECK(ctx, "route_scatter");
    return SF_OK;
}

int zero_count(sf_ctx* ctx, uint32_t* esc_count)
{
    route_zero<<<1, 1, 0, ctx->stream>>>(esc_count);
    SF_LAUNCH_CHECK(ctx, "route_zero");
    return SF_OK;
}

int fill_vmin(sf_ctx* ctx, const char* who, RouteArgs& a, const uint16_t* host_vmin, uint32_t n_vmin)
{
    if (!host_vmin || n_vmin < 1 || n_vmin > SF_MAX_CLASSES)
        return sf::fail(ctx, SF_EINVAL, "%s: host_vmin missing or n_vmin %u outside 1..%d", who, n_vmin, SF_MAX_CLASSES);
    a.n_vmin = n_vmin;
    for (uint32_t c = 0; c < SF_MAX_CLASSES; ++c) a.vmin[c] = host_vmin[c < n_vmin ? c : n_vmin - 1];
    return SF_OK;
}

// ---- block counts for callers that cannot allocate ---------------------------------------------
// One array per GPU, part of the loaded code object, held until the process ends.  The name is a
// host-side stand-in for the symbol, not a device address: host code only ever uses the pointer
// that hipGetSymbolAddress returned for the device at hand.
static __device__ __align__(256) uint32_t scratch[kMaxBlocks];

constexpr int kMaxDevices = 64;
uint32_t* g_scratch_ptr[kMaxDevices]; // per device: address of that device's copy of scratch
std::mutex g_scratch_mu;

// the current device's copy of scratch, looked up once per device with that device current
int scratch_of_current_device(sf_ctx* ctx, uint32_t** out)
{
    int dev = -1;
    SF_HIP(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return sf::fail(ctx, SF_EUNSUPPORTED, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        uint32_t* p = nullptr;
        SF_HIP(ctx, hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
        if (!p) return sf::fail(ctx, SF_EHIP, "hipGetSymbolAddress returned no address for the static block counts");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SF_OK;
}

} // namespace

namespace sf {
int route_static_init(sf_ctx* ctx)
{
    uint32_t* p = nullptr;
    return scratch_of_current_device(ctx, &p);
}
} // namespace sf

extern "C" int sf_route(sf_ctx* ctx, const uint16_t* top_votes, const uint16_t* pred, uint32_t n_flows,
                        const uint16_t* host_vmin, uint32_t n_vmin, uint32_t* esc_idx, uint32_t* esc_count)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_route: ctx is NULL");
    RouteArgs a = {};
    {
        const int rc = fill_vmin(ctx, "sf_route", a, host_vmin, n_vmin);
        if (rc != SF_OK) return rc;
    }
    if (!esc_count) return sf::fail(ctx, SF_EINVAL, "sf_route: esc_count is NULL");
    if (n_flows == 0) return zero_count(ctx, esc_count);
    if (n_flows > (1u << 31)) return sf::fail(ctx, SF_EUNSUPPORTED, "sf_route: more than 2^31 flows per call");
    if (!top_votes || !esc_idx) return sf::fail(ctx, SF_EINVAL, "sf_route: top_votes or esc_idx is NULL");
    if (n_vmin > 1 && !pred) return sf::fail(ctx, SF_EINVAL, "sf_route: per-class thresholds need pred");
    a.top = top_votes;
    a.pred = pred;
    a.n = n_flows;
    return launch_route(ctx, "sf_route", a, esc_idx, esc_count);
}

extern "C" int sf_route_static(sf_ctx* ctx, const uint16_t* top_votes, const uint16_t* pred, uint32_t n_flows,
                               const uint16_t* host_vmin, uint32_t n_vmin, uint32_t* esc_idx, uint32_t* esc_count)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_route_static: ctx is NULL");
    RouteArgs a = {};
    {
        const int rc = fill_vmin(ctx, "sf_route_static", a, host_vmin, n_vmin);
        if (rc != SF_OK) return rc;
    }
    if (!esc_count) return sf::fail(ctx, SF_EINVAL, "sf_route_static: esc_count is NULL");
    if (n_flows > SF_ROUTE_STATIC_MAX_FLOWS)
        return sf::fail(ctx, SF_EUNSUPPORTED, "sf_route_static: %u flows, the static block counts cover at most %u per call",
                        n_flows, (unsigned)SF_ROUTE_STATIC_MAX_FLOWS);
    if (n_flows == 0) return zero_count(ctx, esc_count);
    if (!top_votes || !esc_idx) return sf::fail(ctx, SF_EINVAL, "sf_route_static: top_votes or esc_idx is NULL");
    if (n_vmin > 1 && !pred) return sf::fail(ctx, SF_EINVAL, "sf_route_static: per-class thresholds need pred");
    uint32_t* counts = nullptr;
    {
        const int rc = scratch_of_current_device(ctx, &counts);
        if (rc != SF_OK) return rc;
    }
    a.top = top_votes;
    a.pred = pred;
    a.n = n_flows;
    // nothing in the counts has to start at zero: route_count writes the entry of every block of this
    // launch and route_scatter reads only those
    return launch_route(ctx, "sf_route_static", a, esc_idx, esc_count, counts);
}

extern "C" int sf_route_ratio(sf_ctx* ctx, const uint16_t* top_count, const uint16_t* leaf_total, uint32_t n_flows,
                              float theta, uint32_t* esc_idx, uint32_t* esc_count)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_route_ratio: ctx is NULL");
    if (theta != theta) return sf::fail(ctx, SF_EINVAL, "sf_route_ratio: theta is NaN");
    if (!esc_count) return sf::fail(ctx, SF_EINVAL, "sf_route_ratio: esc_count is NULL");
    if (n_flows == 0) return zero_count(ctx, esc_count);
    if (n_flows > (1u << 31)) return sf::fail(ctx, SF_EUNSUPPORTED, "sf_route_ratio: more than 2^31 flows per call");
    if (!top_count || !leaf_total || !esc_idx)
        return sf::fail(ctx, SF_EINVAL, "sf_route_ratio: top_count, leaf_total or esc_idx is NULL");
    RouteArgs a = {};
    a.top = top_count;
    a.total = leaf_total;
    a.theta = theta;
    a.n = n_flows;
    a.n_vmin = 1;
    return launch_route(ctx, "sf_route_ratio", a, esc_idx, esc_count);
}

extern "C" int sf_route_score(sf_ctx* ctx, const float* score, uint32_t n_flows, float threshold, uint32_t* esc_idx,
                              uint32_t* esc_count)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_route_score: ctx is NULL");
    if (threshold != threshold) return sf::fail(ctx, SF_EINVAL, "sf_route_score: threshold is NaN");
    if (!esc_count) return sf::fail(ctx, SF_EINVAL, "sf_route_score: esc_count is NULL");
    if (n_flows == 0) return zero_count(ctx, esc_count);
    if (n_flows > (1u << 31)) return sf::fail(ctx, SF_EUNSUPPORTED, "sf_route_score: more than 2^31 flows per call");
    if (!score || !esc_idx) return sf::fail(ctx, SF_EINVAL, "sf_route_score: score or esc_idx is NULL");
    RouteArgs a = {};
    a.score = score;
    a.score_thr = threshold;
    a.n = n_flows;
    a.n_vmin = 1;
    return launch_route(ctx, "sf_route_score", a, esc_idx, esc_count);
}

extern "C" int sf_route_subset(sf_ctx* ctx, const uint16_t* top_votes, const uint16_t* pred, const uint32_t* idx,
                               const uint32_t* idx_count, uint32_t idx_cap, const uint16_t* host_vmin,
                               uint32_t n_vmin, uint32_t* esc_idx, uint32_t* esc_count)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_route_subset: ctx is NULL");
    RouteArgs a = {};
    {
        const int rc = fill_vmin(ctx, "sf_route_subset", a, host_vmin, n_vmin);
        if (rc != SF_OK) return rc;
    }
    if (!esc_count) return sf::fail(ctx, SF_EINVAL, "sf_route_subset: esc_count is NULL");
    if (idx_cap == 0) return zero_count(ctx, esc_count);
    if (idx_cap > (1u << 31)) return sf::fail(ctx, SF_EUNSUPPORTED, "sf_route_subset: more than 2^31 rows per call");
    if (!top_votes || !esc_idx || !idx || !idx_count)
        return sf::fail(ctx, SF_EINVAL, "sf_route_subset: top_votes, idx, idx_count or esc_idx is NULL");
    if (n_vmin > 1 && !pred) return sf::fail(ctx, SF_EINVAL, "sf_route_subset: per-class thresholds need pred");
    a.top = top_votes;
    a.pred = pred;
    a.src_idx = idx;
    a.src_count = idx_count;
    a.n = idx_cap;
    return launch_route(ctx, "sf_route_subset", a, esc_idx, esc_count);
}

// ---- calibration entry points ------------------------------------------------------------------

extern "C" int sf_score_histogram(sf_ctx* ctx, const uint16_t* top_votes, uint32_t n_flows, uint32_t n_trees,
                                  uint32_t* host_hist)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_score_histogram: ctx is NULL");
    if (!host_hist) return sf::fail(ctx, SF_EINVAL, "sf_score_histogram: host_hist is NULL");
    if (n_trees < 1 || n_trees > 65535) return sf::fail(ctx, SF_EINVAL, "sf_score_histogram: n_trees %u outside 1..65535", n_trees);
    const uint32_t bins = n_trees + 1u;
    if (n_flows == 0) {
        for (uint32_t b = 0; b < bins; ++b) host_hist[b] = 0;
        return SF_OK;
    }
    if (!top_votes) return sf::fail(ctx, SF_EINVAL, "sf_score_histogram: top_votes is NULL");
    sf::Carve ws(ctx);
    uint32_t* d_hist = (uint32_t*)ws.take((size_t)bins * 4);
    if (!d_hist) return sf::fail(ctx, SF_ENOMEM, "sf_score_histogram: workspace too small for %u bins", bins);
    hist_zero<<<(bins + 255) / 256, 256, 0, ctx->stream>>>(d_hist, bins);
    SF_LAUNCH_CHECK(ctx, "hist_zero");
    uint32_t blocks = (n_flows + 256 * 16 - 1) / (256 * 16);
    blocks = blocks > 2048 ? 2048 : blocks;
    hist_scores<<<blocks, 256, 0, ctx->stream>>>(top_votes, n_flows, bins, d_hist);
    SF_LAUNCH_CHECK(ctx, "hist_scores");
    SF_HIP(ctx, hipMemcpyAsync(host_hist, d_hist, (size_t)bins * 4, hipMemcpyDeviceToHost, ctx->stream));
    SF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return SF_OK;
}

extern "C" int sf_universal_thresholds(const uint32_t* host_hist, uint32_t n_trees, const double* host_q, uint32_t n_q,
                                       uint16_t* host_votes_at)
{
    if (!host_hist || !host_q || !host_votes_at || n_trees < 1 || n_trees > 65535) return SF_EINVAL;
    uint64_t n = 0;
    for (uint32_t v = 0; v <= n_trees; ++v) n += host_hist[v];
    if (n == 0) return SF_EINVAL;
    for (uint32_t j = 0; j < n_q; ++j) {
        // 1-based position ceil(q * n) in the ascending order of LC = descending order of top_votes
        double pos = std::ceil(host_q[j] * (double)n);
        if (!(pos >= 1.0)) pos = 1.0;
        if (pos > (double)n) pos = (double)n;
        const uint64_t want = (uint64_t)pos;
        uint64_t seen = 0;
        uint32_t v = n_trees;
        for (;; --v) {
            seen += host_hist[v];
            if (seen >= want || v == 0) break;
        }
        host_votes_at[j] = (uint16_t)v;
    }
    return SF_OK;
}

extern "C" uint32_t sf_vmin_for_target(const uint32_t* host_hist, uint32_t n_trees, double target_fraction,
                                       double* reached_fraction)
{
    if (!host_hist || n_trees < 1 || n_trees > 65535) return 0;
    uint64_t n = 0;
    for (uint32_t v = 0; v <= n_trees; ++v) n += host_hist[v];
    uint32_t best = 0;
    uint64_t best_below = 0, below = 0; // below = flows with top_votes < vmin
    // |below/n - target| compared exactly as |below - target*n| (same double product for every candidate)
    const double tn = target_fraction * (double)n;
    double best_d = tn < 0 ? -tn : tn;
    for (uint32_t vmin = 1; vmin <= n_trees + 1u; ++vmin) {
        below += host_hist[vmin - 1];
        double d = (double)below - tn;
        d = d < 0 ? -d : d;
        if (d < best_d) { // strict: on a tie the smaller fraction (found first) stays
            best_d = d;
            best = vmin;
            best_below = below;
        }
    }
    if (reached_fraction) *reached_fraction = n ? (double)best_below / (double)n : 0.0;
    return best;
}

extern "C" int sf_score_quantiles(sf_ctx* ctx, const float* score, uint32_t n_flows, const double* host_q, uint32_t n_q,
                                  float* host_thresholds)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_score_quantiles: ctx is NULL");
    if (!score || !host_q || !host_thresholds || n_flows == 0)
        return sf::fail(ctx, SF_EINVAL, "sf_score_quantiles: score, host_q or host_thresholds missing, or no flows");
    if (n_q == 0) return SF_OK;
    if (n_q > kMaxQuantiles) return sf::fail(ctx, SF_EUNSUPPORTED, "sf_score_quantiles: %u quantiles, at most %u per call", n_q, kMaxQuantiles);
    sf::Carve ws(ctx);
    uint32_t* hist_all = (uint32_t*)ws.take(kSelBins * 4);  // pass 1, shared by every quantile
    uint32_t* hist = (uint32_t*)ws.take(kSelBins * 4);      // passes 2 and 3 of the quantile at hand
    SelState* st = (SelState*)ws.take(sizeof(SelState));
    float* d_out = (float*)ws.take((size_t)n_q * 4);
    if (!hist_all || !hist || !st || !d_out)
        return sf::fail(ctx, SF_ENOMEM, "sf_score_quantiles: workspace too small for %zu bytes", sf::kQuantileScratch);
    uint32_t blocks = (n_flows + 256 * 16 - 1) / (256 * 16);
    blocks = blocks > 2048 ? 2048 : blocks;
    hist_zero<<<(2 * kSelBins + 255) / 256, 256, 0, ctx->stream>>>(hist_all, kSelBins);
    hist_zero<<<(2 * kSelBins + 255) / 256, 256, 0, ctx->stream>>>(hist, kSelBins);
    SF_LAUNCH_CHECK(ctx, "hist_zero");
    sel_hist<<<blocks, 256, 0, ctx->stream>>>(score, n_flows, 21u, 0x7FFu, 0u, nullptr, hist_all);
    SF_LAUNCH_CHECK(ctx, "sel_hist");
    for (uint32_t j = 0; j < n_q; ++j) {
        // 1-based position ceil(q * n) in the ascending order (Algorithm 1), clamped to 1..n
        double pos = std::ceil(host_q[j] * (double)n_flows);
        if (!(pos >= 1.0)) pos = 1.0;
        if (pos > (double)n_flows) pos = (double)n_flows;
        sel_pick<<<1, 256, 0, ctx->stream>>>(hist_all, kSelBins, 11u, st, (uint32_t)pos, hist, nullptr);
        sel_hist<<<blocks, 256, 0, ctx->stream>>>(score, n_flows, 10u, 0x7FFu, 21u, st, hist);
        sel_pick<<<1, 256, 0, ctx->stream>>>(hist, kSelBins, 11u, st, 0u, hist, nullptr);
        sel_hist<<<blocks, 256, 0, ctx->stream>>>(score, n_flows, 0u, 0x3FFu, 10u, st, hist);
        sel_pick<<<1, 256, 0, ctx->stream>>>(hist, 1024u, 10u, st, 0u, hist, d_out + j);
        SF_LAUNCH_CHECK(ctx, "sel_pick");
    }
    SF_HIP(ctx, hipMemcpyAsync(host_thresholds, d_out, (size_t)n_q * 4, hipMemcpyDeviceToHost, ctx->stream));
    SF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return SF_OK;
}

extern "C" int sf_class_score_histogram(sf_ctx* ctx, const uint16_t* top_votes, const uint16_t* pred, const uint16_t* truth,
                                        uint32_t n_flows, uint32_t n_trees, uint32_t n_classes, uint32_t* host_hist)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_class_score_histogram: ctx is NULL");
    if (!host_hist) return sf::fail(ctx, SF_EINVAL, "sf_class_score_histogram: host_hist is NULL");
    if (n_trees < 1 || n_trees > 65535 || n_classes < 1 || n_classes > SF_MAX_CLASSES)
        return sf::fail(ctx, SF_EINVAL, "sf_class_score_histogram: n_trees %u or n_classes %u out of range", n_trees, n_classes);
    const size_t words = (size_t)n_classes * (n_trees + 1u) * 2u;
    if (n_flows == 0) {
        for (size_t b = 0; b < words; ++b) host_hist[b] = 0;
        return SF_OK;
    }
    if (!top_votes || !pred || !truth) return sf::fail(ctx, SF_EINVAL, "sf_class_score_histogram: top_votes, pred or truth is NULL");
    sf::Carve ws(ctx);
    uint32_t* d_hist = (uint32_t*)ws.take(words * 4);
    if (!d_hist) return sf::fail(ctx, SF_ENOMEM, "sf_class_score_histogram: workspace too small for %zu bytes", words * 4);
    uint32_t zb = (uint32_t)((words + 255) / 256);
    hist_zero<<<zb > 4096 ? 4096 : zb, 256, 0, ctx->stream>>>(d_hist, (uint32_t)words);
    SF_LAUNCH_CHECK(ctx, "hist_zero");
    uint32_t blocks = (n_flows + 256 * 16 - 1) / (256 * 16);
    blocks = blocks > 2048 ? 2048 : blocks;
    hist_class_scores<<<blocks, 256, 0, ctx->stream>>>(top_votes, pred, truth, n_flows, n_trees + 1u, n_classes, d_hist);
    SF_LAUNCH_CHECK(ctx, "hist_class_scores");
    SF_HIP(ctx, hipMemcpyAsync(host_hist, d_hist, words * 4, hipMemcpyDeviceToHost, ctx->stream));
    SF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return SF_OK;
}

// assigned < target * n without rounding: target = m * 2^e with a 53-bit integer m, so the test is
// assigned < ceil(m * n / 2^-e) in integers
static bool below_target(uint64_t assigned, uint64_t n, double target)
{
    if (!(target > 0.0) || n == 0) return false;
    int e;
    const double fr = std::frexp(target, &e);
    const unsigned __int128 m = (unsigned __int128)(uint64_t)std::ldexp(fr, 53);
    e -= 53;
    unsigned __int128 rhs = m * n; // below 2^117
    if (e >= 0) return e > 10 ? true : assigned < (rhs << e);
    const int s = -e;
    if (s >= 127) return assigned < 1; // 0 < target * n < 1
    const unsigned __int128 up = (rhs + (((unsigned __int128)1 << s) - 1)) >> s; // ceil(rhs / 2^s)
    return assigned < up;
}

// Algorithm 2 on the histogram.  A class's candidates are its non-empty vote counts in ascending order
// (descending uncertainty); slopes dI / (dC + dI) are compared exactly by cross-multiplication.
extern "C" int sf_per_class_thresholds(const uint32_t* host_hist, uint32_t n_trees, uint32_t n_classes,
                                       double target_fraction, uint16_t* host_vmin, double* reached_fraction)
{
    if (!host_hist || !host_vmin || n_trees < 1 || n_trees > 65535 || n_classes < 1 || n_classes > SF_MAX_CLASSES)
        return SF_EINVAL;
    const uint32_t bins = n_trees + 1u;
    auto cell = [&](uint32_t c, uint32_t v, uint32_t wrong) -> uint64_t { return host_hist[((size_t)c * bins + v) * 2u + wrong]; };
    uint64_t n = 0;
    for (size_t b = 0; b < (size_t)n_classes * bins * 2u; ++b) n += host_hist[b];
    uint32_t next[SF_MAX_CLASSES]; // first vote count of the class not yet assigned
    for (uint32_t c = 0; c < n_classes; ++c) {
        next[c] = 0;
        host_vmin[c] = 0;
    }
    uint64_t assigned = 0;
    while (below_target(assigned, n, target_fraction)) {
        int best = -1;
        uint64_t best_i = 0, best_t = 1;
        uint32_t best_v = 0;
        for (uint32_t c = 0; c < n_classes; ++c) {
            uint32_t v = next[c];
            while (v < bins && cell(c, v, 0) + cell(c, v, 1) == 0) ++v; // empty vote counts are no candidates
            if (v >= bins) continue;
            const uint64_t di = cell(c, v, 1), dt = cell(c, v, 0) + di;
            // di / dt > best_i / best_t  <=>  di * best_t > best_i * dt   (counts below 2^32: no overflow)
            if (best < 0 || di * best_t > best_i * dt) {
                best = (int)c;
                best_i = di;
                best_t = dt;
                best_v = v;
            }
        }
        if (best < 0) break;
        next[best] = best_v + 1u;
        host_vmin[best] = (uint16_t)(best_v + 1u > 65535u ? 65535u : best_v + 1u);
        assigned += best_t;
    }
    if (reached_fraction) *reached_fraction = n ? (double)assigned / (double)n : 0.0;
    return SF_OK;
}
