// Step 1: per-flow statistics of the first k packets (context length k, Section 3.1 of the
// paper) and the unpacking of raw header bits (Section 4.1).
//
// One lane owns one flow and keeps its packets in registers.  Every binary32 operation is
// issued on its own, in packet order (the file is compiled without floating-point
// contraction), so the result does not depend on how flows are spread over lanes; a packet
// outside a group contributes +0.0 to that group's running sums, which leaves them unchanged.
// Order statistics (median, min, max) come from a compare-exchange sorting network over
// order-preserving integer keys, padded with the largest key; the element at a data-dependent
// rank is then read through a per-lane column of shared memory.  A block is one wave: its 64
// feature rows are staged in shared memory per window and written out as full 128-byte runs.
#include "common.h"

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
};

// float -> unsigned key with the same order (negative values: all bits flipped, others: sign set)
__device__ __forceinline__ uint32_t order_key(float x)
{
    const uint32_t b = __float_as_uint(x);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float from_key(uint32_t u)
{
    return __uint_as_float(u ^ ((u & 0x80000000u) ? 0x80000000u : 0xFFFFFFFFu));
}

// Batcher's odd-even merge sort as a fixed network; every index is a compile-time constant
// after unrolling, so the keys stay in registers.
template <int N>
__device__ __forceinline__ void sort_network(uint32_t (&a)[N])
{
#pragma unroll
    for (int p = 1; p < N; p <<= 1) {
#pragma unroll
        for (int k = p; k >= 1; k >>= 1) {
#pragma unroll
            for (int j = k % p; j + k < N; j += 2 * k) {
#pragma unroll
                for (int i = 0; i < k; ++i) {
                    if (i + j + k < N && (i + j) / (2 * p) == (i + j + k) / (2 * p)) {
                        const uint32_t lo = a[i + j] < a[i + j + k] ? a[i + j] : a[i + j + k];
                        const uint32_t hi = a[i + j] < a[i + j + k] ? a[i + j + k] : a[i + j];
                        a[i + j] = lo;
                        a[i + j + k] = hi;
                    }
                }
            }
        }
    }
}

__device__ __forceinline__ bool bit_of(uint64_t m, int j) { return (m >> j) & 1ull; }

// Order statistics of one (quantity, group): keys of the group's members, the rest padded.
template <int N, bool IS_TIME, int KMAX>
__device__ __forceinline__ void order_stats(const float (&x)[KMAX], uint64_t gm, int cg, uint32_t* col,
                                            float& mn, float& mx, float& med)
{
    uint32_t key[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        // packet sizes are >= 0, so their bit pattern already orders like the value
        const uint32_t k = IS_TIME ? order_key(x[i]) : __float_as_uint(x[i]);
        key[i] = bit_of(gm, i) ? k : 0xFFFFFFFFu;
    }
    sort_network<N>(key);
#pragma unroll
    for (int i = 0; i < N; ++i) col[i * kWave] = key[i];
    const int last = cg > 0 ? cg - 1 : 0;
    const uint32_t klo = col[(last >> 1) * kWave], khi = col[(cg >> 1) * kWave], kmx = col[last * kWave];
    mn = IS_TIME ? from_key(key[0]) : __uint_as_float(key[0]);
    mx = IS_TIME ? from_key(kmx) : __uint_as_float(kmx);
    const float lo = IS_TIME ? from_key(klo) : __uint_as_float(klo), hi = IS_TIME ? from_key(khi) : __uint_as_float(khi);
    const float two = lo + hi;
    med = (cg & 1) ? hi : two * 0.5f;
}

// The 32 statistics of one prefix window of m <= N packets, written to the lane's staged row.
template <int N, int KMAX>
__device__ __forceinline__ void window_stats(const float (&s)[KMAX], const float (&t)[KMAX], uint64_t dmask, int m,
                                             uint32_t* col, float* row)
{
    static_assert(N <= KMAX, "window network larger than the register file of the flow");
    const uint64_t valid = m >= 64 ? ~0ull : ((1ull << m) - 1ull);
    const uint64_t m1 = dmask & valid, m0 = ~dmask & valid;
    const int c1 = __popcll(m1), c0 = m - c1;
    // pass 1: ordered sums
    float sS0 = 0.f, sS1 = 0.f, sSa = 0.f, sT0 = 0.f, sT1 = 0.f, sTa = 0.f;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const bool v = bit_of(valid, j), d0 = bit_of(m0, j), d1 = bit_of(m1, j);
        const float a = s[j], b = t[j];
        sSa = sSa + (v ? a : 0.f);
        sS0 = sS0 + (d0 ? a : 0.f);
        sS1 = sS1 + (d1 ? a : 0.f);
        sTa = sTa + (v ? b : 0.f);
        sT0 = sT0 + (d0 ? b : 0.f);
        sT1 = sT1 + (d1 ? b : 0.f);
    }
    const float n0 = (float)(c0 > 0 ? c0 : 1), n1 = (float)(c1 > 0 ? c1 : 1), na = (float)(m > 0 ? m : 1);
    const float mS0 = sS0 / n0, mS1 = sS1 / n1, mSa = sSa / na;
    const float mT0 = sT0 / n0, mT1 = sT1 / n1, mTa = sTa / na;
    // pass 2: ordered sums of squared deviations
    float qS0 = 0.f, qS1 = 0.f, qSa = 0.f, qT0 = 0.f, qT1 = 0.f, qTa = 0.f;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const bool v = bit_of(valid, j), d0 = bit_of(m0, j), d1 = bit_of(m1, j);
        const float a = s[j], b = t[j];
        const float ea = a - mSa, eb = b - mTa;
        const float ea2 = ea * ea, eb2 = eb * eb;
        qSa = qSa + (v ? ea2 : 0.f);
        qTa = qTa + (v ? eb2 : 0.f);
        const float ga = a - (d1 ? mS1 : mS0), gb = b - (d1 ? mT1 : mT0);
        const float ga2 = ga * ga, gb2 = gb * gb;
        qS0 = qS0 + (d0 ? ga2 : 0.f);
        qS1 = qS1 + (d1 ? ga2 : 0.f);
        qT0 = qT0 + (d0 ? gb2 : 0.f);
        qT1 = qT1 + (d1 ? gb2 : 0.f);
    }
    // per group: assemble the ten statistics (for the larger networks the group index is a run-time
    // loop so that the sorting network is emitted twice, not six times)
    constexpr int kGroupUnroll = N <= 16 ? 3 : 1;
#pragma unroll kGroupUnroll
    for (int g = 0; g < 3; ++g) {
        const uint64_t gm = g == 0 ? m0 : (g == 1 ? m1 : valid);
        const int cg = g == 0 ? c0 : (g == 1 ? c1 : m);
        const float ng = g == 0 ? n0 : (g == 1 ? n1 : na);
        const float meanS = g == 0 ? mS0 : (g == 1 ? mS1 : mSa), meanT = g == 0 ? mT0 : (g == 1 ? mT1 : mTa);
        const float ssS = g == 0 ? qS0 : (g == 1 ? qS1 : qSa), ssT = g == 0 ? qT0 : (g == 1 ? qT1 : qTa);
        const float varS = ssS / ng, varT = ssT / ng;
        float mnS, mxS, medS, mnT, mxT, medT;
        order_stats<N, false, KMAX>(s, gm, cg, col, mnS, mxS, medS);
        order_stats<N, true, KMAX>(t, gm, cg, col, mnT, mxT, medT);
        const bool empty = cg == 0;
        float* o = row + 10 * g;
        o[0] = empty ? 0.f : meanS;
        o[1] = empty ? 0.f : sqrtf(varS);
        o[2] = empty ? 0.f : mnS;
        o[3] = empty ? 0.f : mxS;
        o[4] = empty ? 0.f : medS;
        o[5] = empty ? 0.f : meanT;
        o[6] = empty ? 0.f : sqrtf(varT);
        o[7] = empty ? 0.f : mnT;
        o[8] = empty ? 0.f : mxT;
        o[9] = empty ? 0.f : medT;
    }
    row[30] = sSa; // total bytes: every partial sum is an integer below 2^24, so this is exact
    row[31] = (float)m;
}

__device__ __forceinline__ void flow_range(const FeatArgs& a, uint32_t i, uint32_t& o, uint32_t& n)
{
    uint32_t b = a.off[i], e = a.off[i + 1];
    b = b < a.n_pkts ? b : a.n_pkts; // clamp: malformed offsets must not leave the arrays
    e = e < a.n_pkts ? e : a.n_pkts;
    e = e < b ? b : e;
    o = b;
    n = e - b;
}

template <int KMAX>
__global__ __launch_bounds__(kWave) void featurize_wave(FeatArgs a)
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
#pragma unroll
        for (int c = 0; c < KMAX / 8; ++c) {
            const uint4 sz = *reinterpret_cast<const uint4*>(a.size + o + 8 * c);
            const uint32_t w[4] = {sz.x, sz.y, sz.z, sz.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                s[8 * c + 2 * k] = (float)(w[k] & 0xFFFFu);
                s[8 * c + 2 * k + 1] = (float)(w[k] >> 16);
            }
            const float4 t0 = *reinterpret_cast<const float4*>(a.iat + o + 8 * c);
            const float4 t1 = *reinterpret_cast<const float4*>(a.iat + o + 8 * c + 4);
            t[8 * c + 0] = t0.x; t[8 * c + 1] = t0.y; t[8 * c + 2] = t0.z; t[8 * c + 3] = t0.w;
            t[8 * c + 4] = t1.x; t[8 * c + 5] = t1.y; t[8 * c + 6] = t1.z; t[8 * c + 7] = t1.w;
            const uint2 dd = *reinterpret_cast<const uint2*>(a.dir + o + 8 * c);
            const uint32_t dw[2] = {dd.x, dd.y};
#pragma unroll
            for (int k = 0; k < 8; ++k)
                dmask |= (uint64_t)((dw[k >> 2] >> (8 * (k & 3))) & 1u) << (8 * c + k);
        }
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
    uint32_t* col = sort_col + lane;
    float* row = tile + lane * kRow;
    uint32_t rows = a.n_flows - tile0;
    rows = rows < (uint32_t)kWave ? rows : (uint32_t)kWave;
    for (uint32_t w = 0; w < a.n_windows; ++w) {
        const int dw = (int)a.depth[w];
        const int m = avail < dw ? avail : dw;
        // the smallest network that covers every lane's window (wave-uniform choice)
        if (KMAX >= 64 && __any(m > 32))
            window_stats<(KMAX >= 64 ? 64 : KMAX), KMAX>(s, t, dmask, m, col, row);
        else if (KMAX >= 32 && __any(m > 16))
            window_stats<(KMAX >= 32 ? 32 : KMAX), KMAX>(s, t, dmask, m, col, row);
        else if (KMAX >= 16 && __any(m > 8))
            window_stats<(KMAX >= 16 ? 16 : KMAX), KMAX>(s, t, dmask, m, col, row);
        else
            window_stats<8, KMAX>(s, t, dmask, m, col, row);
        __syncthreads();
        // half a wave writes one staged row: 32 consecutive floats = one 128-byte run
        const uint32_t c = lane & 31u, half = lane >> 5;
        for (uint32_t r = half; r < rows; r += 2)
            a.feat[(size_t)(tile0 + r) * a.ld + 32u * w + c] = tile[r * kRow + c];
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
