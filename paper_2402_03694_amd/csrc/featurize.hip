// Step 1: per-flow statistics of the first k packets (context length k, Section 3.1 of the
// paper) and the unpacking of raw header bits (Section 4.1).
//
// One lane owns one flow.  Every binary32 operation is issued on its own, in packet order
// (the file is compiled without floating-point contraction), so the result does not depend
// on how flows are spread over lanes.  Medians come from stable ranks (the number of
// elements that sort before an element), which needs no data movement and no sort.
#include "common.h"

namespace {

constexpr int kLdsLanes = 64; // block size of the long-window variant

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
};

// Packet values of one flow: in registers (short windows) or in a column of shared memory.
template <int KMAX, bool LDS>
struct Vals;

template <int KMAX>
struct Vals<KMAX, false> {
    float s[KMAX], t[KMAX];
    __device__ __forceinline__ float S(int j) const { return s[j]; }
    __device__ __forceinline__ float T(int j) const { return t[j]; }
};

template <int KMAX>
struct Vals<KMAX, true> {
    const float* ps; // [j][lane]
    const float* pt;
    __device__ __forceinline__ float S(int j) const { return ps[j * kLdsLanes]; }
    __device__ __forceinline__ float T(int j) const { return pt[j * kLdsLanes]; }
};

struct Stat5 {
    float mean, sd, mn, mx, med;
};

__device__ __forceinline__ void store32(float* out, const float* f, bool vec)
{
    if (vec) {
#pragma unroll
        for (int q = 0; q < 8; ++q)
            reinterpret_cast<float4*>(out)[q] = make_float4(f[4 * q], f[4 * q + 1], f[4 * q + 2], f[4 * q + 3]);
    } else {
#pragma unroll
        for (int q = 0; q < 32; ++q) out[q] = f[q];
    }
}

// All 32 statistics of one prefix window of m packets.
template <int KMAX, bool LDS>
__device__ __forceinline__ void window_stats(const Vals<KMAX, LDS>& v, uint64_t dmask, int m, float* f)
{
    const int bound = LDS ? m : KMAX;
    // ---- pass 1: counts, ordered sums, min, max -------------------------------------------
    int cnt[3] = {0, 0, 0};
    float sumS[3] = {0.f, 0.f, 0.f}, sumT[3] = {0.f, 0.f, 0.f};
    float mnS[3] = {0.f, 0.f, 0.f}, mxS[3] = {0.f, 0.f, 0.f}, mnT[3] = {0.f, 0.f, 0.f}, mxT[3] = {0.f, 0.f, 0.f};
    float bytes = 0.f;
#pragma unroll
    for (int j = 0; j < bound; ++j) {
        if (j < m) {
            const float a = v.S(j), b = v.T(j);
            const int d = (int)((dmask >> j) & 1u);
            bytes = bytes + a;
#pragma unroll
            for (int g = 0; g < 3; ++g) {
                const bool in = g == 2 || d == g;
                if (in) {
                    const bool first = cnt[g] == 0;
                    sumS[g] = sumS[g] + a;
                    sumT[g] = sumT[g] + b;
                    mnS[g] = (first || a < mnS[g]) ? a : mnS[g];
                    mxS[g] = (first || a > mxS[g]) ? a : mxS[g];
                    mnT[g] = (first || b < mnT[g]) ? b : mnT[g];
                    mxT[g] = (first || b > mxT[g]) ? b : mxT[g];
                    cnt[g] += 1;
                }
            }
        }
    }
    float meanS[3], meanT[3];
#pragma unroll
    for (int g = 0; g < 3; ++g) {
        const float c = (float)(cnt[g] > 0 ? cnt[g] : 1);
        meanS[g] = sumS[g] / c;
        meanT[g] = sumT[g] / c;
    }
    // ---- pass 2: sum of squared deviations, in packet order ------------------------------
    float ssS[3] = {0.f, 0.f, 0.f}, ssT[3] = {0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < bound; ++j) {
        if (j < m) {
            const float a = v.S(j), b = v.T(j);
            const int d = (int)((dmask >> j) & 1u);
#pragma unroll
            for (int g = 0; g < 3; ++g) {
                const bool in = g == 2 || d == g;
                if (in) {
                    const float ta = a - meanS[g];
                    const float tb = b - meanT[g];
                    const float qa = ta * ta;
                    const float qb = tb * tb;
                    ssS[g] = ssS[g] + qa;
                    ssT[g] = ssT[g] + qb;
                }
            }
        }
    }
    // ---- medians from stable ranks --------------------------------------------------------
    int tlo[3], thi[3];
#pragma unroll
    for (int g = 0; g < 3; ++g) {
        thi[g] = cnt[g] >> 1;
        tlo[g] = (cnt[g] - 1) >> 1;
    }
    float loS[3] = {0.f, 0.f, 0.f}, hiS[3] = {0.f, 0.f, 0.f}, loT[3] = {0.f, 0.f, 0.f}, hiT[3] = {0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < bound; ++j) {
        if (j < m) {
            const float a = v.S(j), b = v.T(j);
            const int d = (int)((dmask >> j) & 1u);
            int raS = 0, raT = 0, rgS = 0, rgT = 0;
#pragma unroll
            for (int i = 0; i < bound; ++i) {
                if (i < m && i != j) {
                    const float ai = v.S(i), bi = v.T(i);
                    const bool same = (int)((dmask >> i) & 1u) == d;
                    const bool bS = i < j ? ai <= a : ai < a;
                    const bool bT = i < j ? bi <= b : bi < b;
                    raS += bS ? 1 : 0;
                    raT += bT ? 1 : 0;
                    rgS += (bS && same) ? 1 : 0;
                    rgT += (bT && same) ? 1 : 0;
                }
            }
            loS[2] = raS == tlo[2] ? a : loS[2];
            hiS[2] = raS == thi[2] ? a : hiS[2];
            loT[2] = raT == tlo[2] ? b : loT[2];
            hiT[2] = raT == thi[2] ? b : hiT[2];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const bool in = d == g;
                loS[g] = (in && rgS == tlo[g]) ? a : loS[g];
                hiS[g] = (in && rgS == thi[g]) ? a : hiS[g];
                loT[g] = (in && rgT == tlo[g]) ? b : loT[g];
                hiT[g] = (in && rgT == thi[g]) ? b : hiT[g];
            }
        }
    }
    // ---- assemble ------------------------------------------------------------------------
#pragma unroll
    for (int g = 0; g < 3; ++g) {
        const bool empty = cnt[g] == 0;
        const float c = (float)(empty ? 1 : cnt[g]);
        const float varS = ssS[g] / c, varT = ssT[g] / c;
        const bool odd = cnt[g] & 1;
        const float twoS = loS[g] + hiS[g], twoT = loT[g] + hiT[g];
        float* o = f + 10 * g;
        o[0] = empty ? 0.f : meanS[g];
        o[1] = empty ? 0.f : sqrtf(varS);
        o[2] = empty ? 0.f : mnS[g];
        o[3] = empty ? 0.f : mxS[g];
        o[4] = empty ? 0.f : (odd ? hiS[g] : twoS * 0.5f);
        o[5] = empty ? 0.f : meanT[g];
        o[6] = empty ? 0.f : sqrtf(varT);
        o[7] = empty ? 0.f : mnT[g];
        o[8] = empty ? 0.f : mxT[g];
        o[9] = empty ? 0.f : (odd ? hiT[g] : twoT * 0.5f);
    }
    f[30] = bytes;
    f[31] = (float)m;
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
__global__ __launch_bounds__(256) void featurize_reg(FeatArgs a)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.n_flows) return;
    uint32_t o, n;
    flow_range(a, i, o, n);
    const uint32_t dmax = a.depth[a.n_windows - 1];
    const int avail = (int)(n < dmax ? n : dmax);
    Vals<KMAX, false> v;
    uint64_t dmask = 0;
    if (avail == KMAX && (o & 7u) == 0) {
        // whole window present and 16-byte aligned: wide loads
#pragma unroll
        for (int c = 0; c < KMAX / 8; ++c) {
            const uint4 sz = *reinterpret_cast<const uint4*>(a.size + o + 8 * c);
            const uint32_t w[4] = {sz.x, sz.y, sz.z, sz.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                v.s[8 * c + 2 * k] = (float)(w[k] & 0xFFFFu);
                v.s[8 * c + 2 * k + 1] = (float)(w[k] >> 16);
            }
            const float4 t0 = *reinterpret_cast<const float4*>(a.iat + o + 8 * c);
            const float4 t1 = *reinterpret_cast<const float4*>(a.iat + o + 8 * c + 4);
            v.t[8 * c + 0] = t0.x; v.t[8 * c + 1] = t0.y; v.t[8 * c + 2] = t0.z; v.t[8 * c + 3] = t0.w;
            v.t[8 * c + 4] = t1.x; v.t[8 * c + 5] = t1.y; v.t[8 * c + 6] = t1.z; v.t[8 * c + 7] = t1.w;
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
                v.s[j] = (float)a.size[o + j];
                v.t[j] = a.iat[o + j];
                dmask |= (uint64_t)(a.dir[o + j] & 1u) << j;
            } else {
                v.s[j] = 0.f;
                v.t[j] = 0.f;
            }
        }
    }
    float* out = a.feat + (size_t)i * a.ld;
    const bool vec = (a.ld & 3u) == 0 && (reinterpret_cast<uintptr_t>(a.feat) & 15u) == 0;
#pragma unroll
    for (int w = 0; w < SF_MAX_WINDOWS; ++w) {
        if (w < (int)a.n_windows) {
            const int m = avail < (int)a.depth[w] ? avail : (int)a.depth[w];
            float f[32];
            window_stats<KMAX, false>(v, dmask, m, f);
            store32(out + 32 * w, f, vec);
        }
    }
}

// Long windows (up to 64 packets): the flow's values sit in a column of shared memory,
// [packet][lane], so that lane l always hits bank l % 32.
__global__ __launch_bounds__(kLdsLanes) void featurize_lds(FeatArgs a)
{
    __shared__ float ls[SF_MAX_DEPTH_PKTS * kLdsLanes];
    __shared__ float lt[SF_MAX_DEPTH_PKTS * kLdsLanes];
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.n_flows) return;
    uint32_t o, n;
    flow_range(a, i, o, n);
    const uint32_t dmax = a.depth[a.n_windows - 1];
    const int avail = (int)(n < dmax ? n : dmax);
    uint64_t dmask = 0;
    float* cs = ls + threadIdx.x;
    float* ct = lt + threadIdx.x;
    for (int j = 0; j < avail; ++j) {
        cs[j * kLdsLanes] = (float)a.size[o + j];
        ct[j * kLdsLanes] = a.iat[o + j];
        dmask |= (uint64_t)(a.dir[o + j] & 1u) << j;
    }
    Vals<SF_MAX_DEPTH_PKTS, true> v{cs, ct};
    float* out = a.feat + (size_t)i * a.ld;
    const bool vec = (a.ld & 3u) == 0 && (reinterpret_cast<uintptr_t>(a.feat) & 15u) == 0;
    for (int w = 0; w < (int)a.n_windows; ++w) {
        const int m = avail < (int)a.depth[w] ? avail : (int)a.depth[w];
        float f[32];
        window_stats<SF_MAX_DEPTH_PKTS, true>(v, dmask, m, f);
        store32(out + 32 * w, f, vec);
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
    const uint32_t dmax = cfg->depth[cfg->n_windows - 1];
    if (dmax <= 16) {
        const uint32_t bs = 256, grid = (a.n_flows + bs - 1) / bs;
        if (dmax <= 8)
            featurize_reg<8><<<grid, bs, 0, ctx->stream>>>(a);
        else
            featurize_reg<16><<<grid, bs, 0, ctx->stream>>>(a);
    } else {
        const uint32_t grid = (a.n_flows + kLdsLanes - 1) / kLdsLanes;
        featurize_lds<<<grid, kLdsLanes, 0, ctx->stream>>>(a);
    }
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
