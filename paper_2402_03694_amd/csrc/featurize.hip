// Step 1: per-flow statistics of the first k packets (context length k, Section 3.1 of the
// paper) and the unpacking of raw header bits (Section 4.1).
//
// One lane owns one flow and keeps its packets in registers; the statistics of a window are
// computed by the shared device code in featurize_core.h (ordered sums, one sorting network and
// one merge stage per quantity for the order statistics), so the result does not depend on how
// flows are spread over lanes.  A block is one wave: its 64 feature rows are staged in shared
// memory per window and written out as full 128-byte runs.
#include "common.h"
#include "featurize_core.h"

namespace {

constexpr int kWave = 64;      // flows per block (one wave)
constexpr int kRow = 33;       // staged row stride in floats (32 + 1 keeps lanes on distinct banks)

struct FeatArgs {
    uint32_t n_flows;
    uint32_t n_pkts;
    const uint32_t* off;
    const uint16_t* size;
    const float* iat;
    const uint8_t* dir;
    uint32_t n_windows;
    uint32_t depth[SF_MAX_WINDOWS];
    float* feat;
    uint32_t ld;
    uint32_t wide_ok; // the packet arrays start on 16-byte (size, time) and 8-byte (direction) boundaries
    uint32_t store16; // feat is 16-byte aligned and ld a multiple of 4: rows can be written in 16-byte pieces
};

__device__ __forceinline__ void flow_range(const FeatArgs& a, uint32_t i, uint32_t& o, uint32_t& n)
{
    uint32_t b = a.off[i], e = a.off[i + 1];
    b = b < a.n_pkts ? b : a.n_pkts; // clamp: malformed offsets must not leave the arrays
    e = e < a.n_pkts ? e : a.n_pkts;
    e = e < b ? b : e;
    o = b;
    n = e - b;
}

// A flow's packet records as loaded by the wide path (whole deepest window present, 16-byte aligned)
template <int KMAX>
struct RawPackets {
    uint4 sz[KMAX / 8];
    float4 tm[KMAX / 4];
    uint2 dr[KMAX / 8];
};

template <int KMAX>
__device__ __forceinline__ void load_wide(const FeatArgs& a, uint32_t o, RawPackets<KMAX>& r)
{
#pragma unroll
    for (int c = 0; c < KMAX / 8; ++c) {
        r.sz[c] = *reinterpret_cast<const uint4*>(a.size + o + 8 * c);
        r.tm[2 * c] = *reinterpret_cast<const float4*>(a.iat + o + 8 * c);
        r.tm[2 * c + 1] = *reinterpret_cast<const float4*>(a.iat + o + 8 * c + 4);
        r.dr[c] = *reinterpret_cast<const uint2*>(a.dir + o + 8 * c);
    }
}

template <int KMAX>
__device__ __forceinline__ void decode_wide(const RawPackets<KMAX>& r, float (&s)[KMAX], float (&t)[KMAX], uint64_t& dmask)
{
    dmask = 0;
#pragma unroll
    for (int c = 0; c < KMAX / 8; ++c) {
        const uint32_t w[4] = {r.sz[c].x, r.sz[c].y, r.sz[c].z, r.sz[c].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            s[8 * c + 2 * k] = (float)(w[k] & 0xFFFFu);
            s[8 * c + 2 * k + 1] = (float)(w[k] >> 16);
        }
        const float4 t0 = r.tm[2 * c], t1 = r.tm[2 * c + 1];
        t[8 * c + 0] = t0.x; t[8 * c + 1] = t0.y; t[8 * c + 2] = t0.z; t[8 * c + 3] = t0.w;
        t[8 * c + 4] = t1.x; t[8 * c + 5] = t1.y; t[8 * c + 6] = t1.z; t[8 * c + 7] = t1.w;
        const uint32_t dw[2] = {r.dr[c].x, r.dr[c].y};
#pragma unroll
        for (int k = 0; k < 8; ++k) dmask |= (uint64_t)((dw[k >> 2] >> (8 * (k & 3))) & 1u) << (8 * c + k);
    }
}

// (second launch bound: waves per SIMD the register allocation aims for: three up to 16 packets per flow)
template <int KMAX>
__global__ __launch_bounds__(kWave, (KMAX <= 16 ? 3 : 1)) void featurize_wave(FeatArgs a)
{
    __shared__ uint32_t sort_col[KMAX * kWave]; // [rank][lane]
    __shared__ float tile[kWave * kRow];        // [lane][33]
    const uint32_t lane = threadIdx.x;
    const uint32_t tile0 = blockIdx.x * kWave;
    const uint32_t i = tile0 + lane;
    const bool live = i < a.n_flows;
    uint32_t o = 0, n = 0;
    if (live) flow_range(a, i, o, n);
    const uint32_t dmax = a.depth[a.n_windows - 1];
    const int avail = (int)(n < dmax ? n : dmax);
    float s[KMAX], t[KMAX];
    uint64_t dmask = 0;
    if (avail == KMAX && (o & 7u) == 0 && a.wide_ok) {
        // whole window present and 16-byte aligned (array bases included): wide loads
        RawPackets<KMAX> raw;
        load_wide<KMAX>(a, o, raw);
        decode_wide<KMAX>(raw, s, t, dmask);
    } else {
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            if (j < avail) {
                s[j] = (float)a.size[o + j];
                t[j] = a.iat[o + j];
                dmask |= (uint64_t)(a.dir[o + j] & 1u) << j;
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
    uint32_t* col = sort_col + lane;
    float* row = tile + lane * kRow;
    uint32_t rows = a.n_flows - tile0;
    rows = rows < (uint32_t)kWave ? rows : (uint32_t)kWave;
    for (uint32_t w = 0; w < a.n_windows; ++w) {
        const int dw = (int)a.depth[w];
        const int m = avail < dw ? avail : dw;
        // the smallest network that covers every lane's window (wave-uniform choice)
        if (KMAX >= 64 && __any(m > 32))
            sffeat::window_stats<(KMAX >= 64 ? 64 : KMAX), KMAX>(s, t, dmask, m, signed_times, col, kWave, row, 1u);
        else if (KMAX >= 32 && __any(m > 16))
            sffeat::window_stats<(KMAX >= 32 ? 32 : KMAX), KMAX>(s, t, dmask, m, signed_times, col, kWave, row, 1u);
        else if (KMAX >= 16 && __any(m > 8))
            sffeat::window_stats<(KMAX >= 16 ? 16 : KMAX), KMAX>(s, t, dmask, m, signed_times, col, kWave, row, 1u);
        else
            sffeat::window_stats<8, KMAX>(s, t, dmask, m, signed_times, col, kWave, row, 1u);
        __syncthreads();
        if (a.store16) {
            // eight lanes write one staged row (32 consecutive floats = one 128-byte run) as 16-byte pieces:
            // a store instruction of the wave covers eight rows
            const uint32_t c4 = (lane & 7u) * 4u;
            for (uint32_t r = lane >> 3; r < rows; r += 8u) {
                const float* src = tile + r * kRow + c4;
                *reinterpret_cast<float4*>(a.feat + (size_t)(tile0 + r) * a.ld + 32u * w + c4) =
                    make_float4(src[0], src[1], src[2], src[3]);
            }
        } else {
            // half a wave writes one staged row, a float per lane
            const uint32_t c = lane & 31u, half = lane >> 5;
            for (uint32_t r = half; r < rows; r += 2)
                a.feat[(size_t)(tile0 + r) * a.ld + 32u * w + c] = tile[r * kRow + c];
        }
        __syncthreads();
    }
}

// Raw header bits -> one byte per bit.  A thread unpacks one header word (32 features).
__global__ __launch_bounds__(256) void unpack_raw(uint32_t n_flows, uint32_t n_pkts, const uint32_t* __restrict__ off,
                                                  const uint32_t* __restrict__ hdr, uint32_t hdr_words,
                                                  uint32_t raw_pkts, uint32_t raw_bits, uint8_t* __restrict__ raw)
{
    const uint32_t words = (raw_bits + 31) / 32; // words per packet that carry features
    const uint64_t total = (uint64_t)n_flows * raw_pkts * words;
    for (uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total;
         g += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t wq = (uint32_t)(g % words);
        const uint64_t fp = g / words;
        const uint32_t j = (uint32_t)(fp % raw_pkts);
        const uint32_t i = (uint32_t)(fp / raw_pkts);
        uint32_t b = off[i], e = off[i + 1];
        b = b < n_pkts ? b : n_pkts;
        e = e < n_pkts ? e : n_pkts;
        const uint32_t n = e > b ? e - b : 0;
        const uint32_t word = j < n ? hdr[(size_t)(b + j) * hdr_words + wq] : 0u;
        uint8_t* dst = raw + ((size_t)i * raw_pkts + j) * raw_bits + 32u * wq;
        const uint32_t nb = raw_bits - 32u * wq < 32u ? raw_bits - 32u * wq : 32u;
        for (uint32_t k = 0; k < nb; ++k) {
            // feature bit 32*wq + k: byte k/8 of the word, bit 7-(k%8) of that byte
            dst[k] = (uint8_t)((word >> (8u * (k >> 3) + 7u - (k & 7u))) & 1u);
        }
    }
}

} // namespace

extern "C" int sf_featurize(sf_ctx* ctx, const sf_packets* pk, const sf_feat_cfg* cfg, float* feat,
                            uint32_t feat_ld, uint8_t* raw)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_featurize: ctx is NULL");
    if (!pk || !cfg) return sf::fail(ctx, SF_EINVAL, "sf_featurize: packets or config is NULL");
    if (cfg->n_windows < 1 || cfg->n_windows > SF_MAX_WINDOWS)
        return sf::fail(ctx, SF_EINVAL, "sf_featurize: n_windows %u outside 1..%d", cfg->n_windows, SF_MAX_WINDOWS);
    for (uint32_t w = 0; w < cfg->n_windows; ++w) {
        if (cfg->depth[w] < 1 || cfg->depth[w] > SF_MAX_DEPTH_PKTS)
            return sf::fail(ctx, SF_EINVAL, "sf_featurize: depth[%u] = %u outside 1..%d", w, cfg->depth[w],
                            SF_MAX_DEPTH_PKTS);
        if (w && cfg->depth[w] <= cfg->depth[w - 1])
            return sf::fail(ctx, SF_EINVAL, "sf_featurize: depths must be strictly increasing");
    }
    if (feat_ld < 32 * cfg->n_windows)
        return sf::fail(ctx, SF_EINVAL, "sf_featurize: feat_ld %u < %u", feat_ld, 32 * cfg->n_windows);
    if (pk->n_pkts >> 32) return sf::fail(ctx, SF_EINVAL, "sf_featurize: n_pkts exceeds 32-bit offsets");
    if (pk->n_flows == 0) return SF_OK;
    if (!feat || !pk->flow_off) return sf::fail(ctx, SF_EINVAL, "sf_featurize: feat or flow_off is NULL");
    if (pk->n_pkts && (!pk->pkt_size || !pk->pkt_iat || !pk->pkt_dir))
        return sf::fail(ctx, SF_EINVAL, "sf_featurize: packet arrays missing");
    if (raw) {
        if (!pk->pkt_hdr || pk->hdr_words == 0 || pk->hdr_words > SF_HDR_WORDS_MAX)
            return sf::fail(ctx, SF_EINVAL, "sf_featurize: raw output needs pkt_hdr with 1..%d words per packet",
                            SF_HDR_WORDS_MAX);
        if (cfg->raw_pkts == 0 || cfg->raw_bits == 0 || cfg->raw_bits > 32 * pk->hdr_words)
            return sf::fail(ctx, SF_EINVAL, "sf_featurize: raw_pkts/raw_bits do not fit the header words");
    }

    FeatArgs a;
    a.n_flows = pk->n_flows;
    a.n_pkts = (uint32_t)pk->n_pkts;
    a.off = pk->flow_off;
    a.size = pk->pkt_size;
    a.iat = pk->pkt_iat;
    a.dir = pk->pkt_dir;
    a.n_windows = cfg->n_windows;
    for (int w = 0; w < SF_MAX_WINDOWS; ++w) a.depth[w] = w < (int)cfg->n_windows ? cfg->depth[w] : 0;
    a.feat = feat;
    a.ld = feat_ld;
    a.wide_ok = (((uintptr_t)a.size | (uintptr_t)a.iat) & 15u) == 0 && ((uintptr_t)a.dir & 7u) == 0;
    a.store16 = ((uintptr_t)feat & 15u) == 0 && (feat_ld & 3u) == 0;
    const uint32_t dmax = cfg->depth[cfg->n_windows - 1];
    const uint32_t grid = (a.n_flows + kWave - 1) / kWave;
    if (dmax <= 8)
        featurize_wave<8><<<grid, kWave, 0, ctx->stream>>>(a);
    else if (dmax <= 16)
        featurize_wave<16><<<grid, kWave, 0, ctx->stream>>>(a);
    else if (dmax <= 32)
        featurize_wave<32><<<grid, kWave, 0, ctx->stream>>>(a);
    else
        featurize_wave<64><<<grid, kWave, 0, ctx->stream>>>(a);
    SF_LAUNCH_CHECK(ctx, "featurize");
    if (raw) {
        const uint64_t total = (uint64_t)a.n_flows * cfg->raw_pkts * ((cfg->raw_bits + 31) / 32);
        uint64_t blocks = (total + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        unpack_raw<<<(uint32_t)blocks, 256, 0, ctx->stream>>>(a.n_flows, a.n_pkts, pk->flow_off, pk->pkt_hdr,
                                                              pk->hdr_words, cfg->raw_pkts, cfg->raw_bits, raw);
        SF_LAUNCH_CHECK(ctx, "unpack_raw");
    }
    return SF_OK;
}
