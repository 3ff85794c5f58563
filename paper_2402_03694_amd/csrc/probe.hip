// Measurement aid, not a step of the method: what a 64-lane gather costs a compute unit.
// The tree walk of the fast model (Section 3.1 of the paper: it runs on every flow, so it sets the
// service rate) is bound by gathers, not by HBM; the benchmark prices it against the rates this
// probe measures on the device at hand.
//
// Every lane runs chains of dependent gathers (the loaded value feeds the next index), eight chains
// at once, as the walk keeps eight trees in flight.  Three access patterns, those of the walk:
//   0  shared memory, 4 bytes, lane-own column [row][lane] with a data-dependent row
//      (the fetch of x[feature]: never a bank conflict)
//   1  shared memory, 16 bytes at a data-dependent record index (the staged top levels of the trees)
//   2  global memory through the caches, 16 bytes at a data-dependent record index of a table of
//      2^table_log2 records (the deeper levels; 2 K records stay in the first-level cache, 128 K in
//      the second)
#include "common.h"

namespace {

constexpr int kProbeIlp = 8;
constexpr int kProbeBlock = 256;
// Shared memory per block is kept small (16 KB) so that eight blocks share a compute unit and the probe
// measures the pipe's throughput, not the latency of a few waves.
constexpr uint32_t kColRows = 16;     // rows of the per-lane column
constexpr uint32_t kLdsRecs = 1024;   // 16-byte records staged in shared memory

template <int KIND>
__global__ __launch_bounds__(kProbeBlock) void probe_gather(const uint4* __restrict__ table, uint32_t mask, uint32_t iters,
                                                            uint32_t* __restrict__ sink)
{
    // pattern 0 uses the array as [16][256] words, pattern 1 as 1024 records of four words
    __shared__ __attribute__((aligned(16))) uint32_t lds[kColRows * kProbeBlock];
    static_assert(kColRows * kProbeBlock == kLdsRecs * 4u, "one array serves both patterns");
    const uint32_t tid = threadIdx.x;
    if (KIND != 2) {
        const uint32_t words = KIND == 0 ? kColRows * kProbeBlock : kLdsRecs * 4u;
        const uint32_t* src = reinterpret_cast<const uint32_t*>(table);
        for (uint32_t i = tid; i < words; i += kProbeBlock) lds[i] = src[i & (4u * mask + 3u)];
        __syncthreads();
    }
    uint32_t idx[kProbeIlp];
#pragma unroll
    for (int u = 0; u < kProbeIlp; ++u) idx[u] = (tid * 37u + u * 7u + blockIdx.x) & mask;
    uint32_t acc = 0;
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kProbeIlp; ++u) {
            uint32_t v;
            if (KIND == 0) {
                v = lds[(idx[u] & (kColRows - 1u)) * kProbeBlock + tid];
            } else if (KIND == 1) {
                const uint4 r = reinterpret_cast<const uint4*>(lds)[idx[u] & (kLdsRecs - 1u)];
                v = r.x ^ r.y ^ r.z ^ r.w;
            } else {
                const uint4 r = table[idx[u]];
                v = r.x ^ r.y ^ r.z ^ r.w;
            }
            acc += v;
            idx[u] = (idx[u] * 5u + v + 1u) & mask; // the next index depends on the data
        }
    }
    sink[blockIdx.x * kProbeBlock + tid] = acc;
}

} // namespace

extern "C" int sf_probe_gather(sf_ctx* ctx, int kind, uint32_t table_log2, uint32_t iters, uint32_t blocks,
                               const void* table, uint32_t* sink, uint64_t* host_wave_gathers)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_probe_gather: ctx is NULL");
    if (kind < 0 || kind > 2) return sf::fail(ctx, SF_EINVAL, "sf_probe_gather: kind %d outside 0..2", kind);
    if (table_log2 < (kind == 2 ? 8u : 12u) || table_log2 > 24)
        return sf::fail(ctx, SF_EINVAL, "sf_probe_gather: table_log2 %u outside %u..24", table_log2, kind == 2 ? 8u : 12u);
    if (!table || !sink || iters == 0 || blocks == 0 || blocks > 65536)
        return sf::fail(ctx, SF_EINVAL, "sf_probe_gather: table or sink is NULL, or iters / blocks out of range");
    if ((uintptr_t)table & 15u) return sf::fail(ctx, SF_EINVAL, "sf_probe_gather: table is not 16-byte aligned");
    const uint32_t mask = (1u << table_log2) - 1u;
    const uint4* t = (const uint4*)table;
    if (kind == 0)
        probe_gather<0><<<blocks, kProbeBlock, 0, ctx->stream>>>(t, mask, iters, sink);
    else if (kind == 1)
        probe_gather<1><<<blocks, kProbeBlock, 0, ctx->stream>>>(t, mask, iters, sink);
    else
        probe_gather<2><<<blocks, kProbeBlock, 0, ctx->stream>>>(t, mask, iters, sink);
    SF_LAUNCH_CHECK(ctx, "probe_gather");
    if (host_wave_gathers) *host_wave_gathers = (uint64_t)blocks * (kProbeBlock / 64) * iters * kProbeIlp;
    return SF_OK;
}
