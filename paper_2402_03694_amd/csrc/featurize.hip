// Step 1: per-flow statistics of the first k packets (context length k, Section 3.1 of the
// paper) and the unpacking of raw header bits (Section 4.1).
//
// One lane owns one flow and keeps its packets in registers; the statistics of a window are
// computed by the shared device code in featurize_core.h (ordered sums, one sorting network and
// one merge stage per quantity for the order statistics), so the result does not depend on how
// flows are spread over lanes.  A window of more than 32 packets is worked on by the whole wave
// (a sort across the lanes; see below).  A block is one wave: its 64 feature rows are staged in
// shared memory per window and written out as full 128-byte runs.
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

// ---- windows deeper than 32 packets ---------------------------------------------------------------------
// A lane keeps at most 32 packets in registers (a 64-element network per lane needs more registers than a
// lane has, and its straight-line code no longer fits the instruction cache).  A flow whose window holds
// more than 32 packets is worked on by the whole wave instead, in two steps:
//   order statistics  lane p holds packet p; six arrays (quantity x group, padded with the largest key) are
//                     sorted at once by a bitonic network across the lanes, and the flow's values are parked
//                     in shared memory;
//   ordered sums      for up to kSlots parked flows at once: six lanes per flow, each walking one
//                     (quantity, group) chain packet by packet.
// The arithmetic per value is the one of sffeat::window_stats.

constexpr uint32_t kSlots = 10;                 // flows whose chains run side by side (6 lanes each)
constexpr uint32_t kSlotWords = 2 * kWave + 8;  // parked per flow: 64 sizes, 64 times, then lane, packets, direction mask

__device__ __forceinline__ uint32_t lane_value(uint32_t x, int p) { return (uint32_t)__builtin_amdgcn_readlane((int)x, p); }

// the value of lane (lane ^ J): within four lanes and across half a row of 16 by a data-parallel move,
// otherwise through the shared-memory crossbar
template <uint32_t J>
__device__ __forceinline__ uint32_t from_lane_xor(uint32_t v)
{
    if (J == 1) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false);  // quad_perm [1,0,3,2]
    if (J == 2) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false);  // quad_perm [2,3,0,1]
    if (J == 8) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, false); // row_ror:8
    return (uint32_t)__shfl_xor((int)v, (int)J, kWave);
}

template <uint32_t K, uint32_t J>
__device__ __forceinline__ void sort6_step(uint32_t (&key)[6], uint32_t lane)
{
    const bool up = (lane & K) == 0; // (K = 64: every lane)
    const bool lower = (lane & J) == 0;
    uint32_t other[6];
#pragma unroll
    for (int c = 0; c < 6; ++c) other[c] = from_lane_xor<J>(key[c]);
#pragma unroll
    for (int c = 0; c < 6; ++c) {
        const uint32_t lo = key[c] < other[c] ? key[c] : other[c], hi = key[c] < other[c] ? other[c] : key[c];
        key[c] = lower == up ? lo : hi;
    }
}
template <uint32_t K, uint32_t J>
__device__ __forceinline__ void sort6_merge(uint32_t (&key)[6], uint32_t lane)
{
    sort6_step<K, J>(key, lane);
    if constexpr (J > 1) sort6_merge<K, J / 2>(key, lane);
}
// Six independent arrays of one key per lane, each sorted ascending by lane; the six exchanges of a step are
// issued together so that their latencies overlap.
__device__ __forceinline__ void wave_sort6(uint32_t (&key)[6], uint32_t lane)
{
    sort6_merge<2, 1>(key, lane);
    sort6_merge<4, 2>(key, lane);
    sort6_merge<8, 4>(key, lane);
    sort6_merge<16, 8>(key, lane);
    sort6_merge<32, 16>(key, lane);
    sort6_merge<64, 32>(key, lane);
}

// lane p's packet of a window of m packets that start at packet o (zeros past the window), as loaded: nothing
// is computed from it here, so that the request can be issued a whole flow ahead of its use
struct LanePacket {
    uint32_t sz, d;
    float tm;
};
__device__ __forceinline__ LanePacket long_flow_load(const FeatArgs& a, uint32_t o, int m, uint32_t lane)
{
    LanePacket r = {0u, 0u, 0.f};
    if ((int)lane < m) {
        r.sz = a.size[o + lane];
        r.tm = a.iat[o + lane];
        r.d = a.dir[o + lane];
    }
    return r;
}

// Sort keys of a window of m packets (32 < m <= 64), lane p holding packet p: array c = 3 * quantity + group,
// padded with the largest key; c0 / c1: packets of direction 0 / 1.  The values are parked in slot[] for the
// chains.  Every lane of the wave takes part, m and src_lane are the same in all of them.
__device__ __forceinline__ void long_flow_keys(const LanePacket& pk, int m, uint32_t src_lane, uint32_t lane, uint32_t* slot,
                                               uint32_t (&key)[6], int& c0, int& c1)
{
    const bool valid = (int)lane < m;
    const float sz = (float)pk.sz, tm = pk.tm;
    const uint32_t d = pk.d & 1u;
    const uint64_t vmask = __ballot(valid), m1 = __ballot(valid && d != 0), m0 = vmask & ~m1;
    c1 = __popcll(m1);
    c0 = m - c1;
    slot[lane] = __float_as_uint(sz);
    slot[kWave + lane] = __float_as_uint(tm);
    if (lane == 0u) {
        slot[2 * kWave + 0] = src_lane;
        slot[2 * kWave + 1] = (uint32_t)m;
        slot[2 * kWave + 2] = (uint32_t)m1;
        slot[2 * kWave + 3] = (uint32_t)(m1 >> 32);
    }
#pragma unroll
    for (uint32_t c = 0; c < 6u; ++c) {
        const uint32_t g = c % 3u, q = c / 3u;
        const uint64_t gm = g == 0 ? m0 : (g == 1 ? m1 : vmask);
        const bool in = (gm >> lane) & 1ull;
        key[c] = in ? (q ? sffeat::order_key(tm) : (uint32_t)sz) : 0xFFFFFFFFu;
    }
}

// Order statistics from the keys -> dst[10g + 5q + 2..4]
__device__ __forceinline__ void long_flow_order_stats(uint32_t (&key)[6], int m, int c0, int c1, uint32_t lane, float* dst)
{
    wave_sort6(key, lane);
#pragma unroll
    for (uint32_t c = 0; c < 6u; ++c) {
        const uint32_t g = c % 3u, q = c / 3u;
        const int cg = g == 0 ? c0 : (g == 1 ? c1 : m);
        const int last = cg > 0 ? cg - 1 : 0;
        const uint32_t k_mn = lane_value(key[c], 0), k_mx = lane_value(key[c], last);
        const uint32_t k_lo = lane_value(key[c], last >> 1), k_hi = lane_value(key[c], cg >> 1);
        const float mn = q ? sffeat::from_key(k_mn) : (float)k_mn, mx = q ? sffeat::from_key(k_mx) : (float)k_mx;
        const float lo = q ? sffeat::from_key(k_lo) : (float)k_lo, hi = q ? sffeat::from_key(k_hi) : (float)k_hi;
        const float two = lo + hi;
        if (lane == 0u) {
            dst[10u * g + 5u * q + 2u] = cg == 0 ? 0.f : mn;
            dst[10u * g + 5u * q + 3u] = cg == 0 ? 0.f : mx;
            dst[10u * g + 5u * q + 4u] = cg == 0 ? 0.f : ((cg & 1) ? hi : two * 0.5f);
        }
    }
}

// Means, standard deviations, byte and packet counts of the n_slots parked flows -> their staged rows
// (tile + lane_of_flow * kRow).  Lane 6k + c carries chain c (quantity c / 3, group c % 3) of slot k.
__device__ __forceinline__ void long_flow_chains(const uint32_t* park, uint32_t n_slots, uint32_t lane, float* tile)
{
    const uint32_t k = lane / 6u, c = lane - 6u * k;
    if (k >= n_slots) return;
    const uint32_t g = c % 3u, q = c / 3u;
    const uint32_t* slot = park + k * kSlotWords;
    const uint32_t src_lane = slot[2 * kWave + 0];
    const int m = (int)slot[2 * kWave + 1];
    const uint64_t m1 = (uint64_t)slot[2 * kWave + 2] | ((uint64_t)slot[2 * kWave + 3] << 32);
    const uint64_t valid = m >= 64 ? ~0ull : ((1ull << m) - 1ull);
    const uint64_t in_mask = g == 0 ? valid & ~m1 : (g == 1 ? m1 : valid);
    const int cg = __popcll(in_mask);
    const float ng = (float)(cg > 0 ? cg : 1);
    const float* x = reinterpret_cast<const float*>(slot) + q * kWave;
    float sum = 0.f;
    for (int p = 0; p < kWave; p += 4) {
        const float4 v = *reinterpret_cast<const float4*>(x + p);
        const uint32_t in4 = (uint32_t)(in_mask >> p) & 15u;
        sum = sum + ((in4 & 1u) ? v.x : 0.f);
        sum = sum + ((in4 & 2u) ? v.y : 0.f);
        sum = sum + ((in4 & 4u) ? v.z : 0.f);
        sum = sum + ((in4 & 8u) ? v.w : 0.f);
    }
    const float mean = sum / ng;
    float acc = 0.f;
    for (int p = 0; p < kWave; p += 4) {
        const float4 v = *reinterpret_cast<const float4*>(x + p);
        const uint32_t in4 = (uint32_t)(in_mask >> p) & 15u;
        const float d0 = v.x - mean, d1 = v.y - mean, d2 = v.z - mean, d3 = v.w - mean;
        const float e0 = d0 * d0, e1 = d1 * d1, e2 = d2 * d2, e3 = d3 * d3;
        acc = acc + ((in4 & 1u) ? e0 : 0.f);
        acc = acc + ((in4 & 2u) ? e1 : 0.f);
        acc = acc + ((in4 & 4u) ? e2 : 0.f);
        acc = acc + ((in4 & 8u) ? e3 : 0.f);
    }
    const float var = acc / ng;
    float* dst = tile + src_lane * kRow;
    dst[10u * g + 5u * q + 0u] = cg == 0 ? 0.f : mean;
    dst[10u * g + 5u * q + 1u] = cg == 0 ? 0.f : sqrtf(var);
    if (c == 2u) { // sizes, all packets
        dst[30] = sum;
        dst[31] = (float)m;
    }
}

// KMAX: packets a lane keeps in registers.  LONG: windows may be deeper than that (up to 64 packets); flows
// with more than KMAX packets in a window then go through long_window_stats.
// (second launch bound: waves per SIMD the register allocation aims for.  Three up to 16 packets per flow.
// Two with 32 packets in registers: the allocation then spills 28 registers per lane, and two waves that
// cover each other's memory latency still win: 1.75 -> 1.37 ms on 4,194,304 flows of 32 packets; three waves
// spill 160 registers and lose, 2.9 ms.  One where long flows go through the whole-wave path: that kernel's
// time is a single wave's latency, which spills only lengthen.)
template <int KMAX, bool LONG>
__global__ __launch_bounds__(kWave, (KMAX <= 16 ? 3 : (LONG ? 1 : 2))) void featurize_wave(FeatArgs a)
{
    static_assert(!LONG || KMAX == 32, "the whole-wave path takes over above 32 packets");
    __shared__ uint32_t sort_col[KMAX * kWave]; // [rank][lane]
    __shared__ float tile[kWave * kRow];        // [lane][33]
    const uint32_t lane = threadIdx.x;
    const uint32_t tile0 = blockIdx.x * kWave;
    const uint32_t i = tile0 + lane;
    const bool live = i < a.n_flows;
    uint32_t o = 0, n = 0;
    if (live) flow_range(a, i, o, n);
    const uint32_t dmax = a.depth[a.n_windows - 1];
    const int avail_w = (int)(n < dmax ? n : dmax);              // packets of the deepest window
    const int avail = avail_w < KMAX ? avail_w : KMAX;           // of which the lane holds in registers
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
        const int m_w = avail_w < dw ? avail_w : dw;
        const bool long_flow = LONG && m_w > KMAX;
        const int m = long_flow ? 0 : m_w; // (the lane's own result for such a flow is overwritten below)
        // the smallest network that covers every lane's window (wave-uniform choice)
        if (KMAX >= 32 && __any(m > 16))
            sffeat::window_stats<(KMAX >= 32 ? 32 : KMAX), KMAX>(s, t, dmask, m, signed_times, col, kWave, row, 1u);
        else if (KMAX >= 16 && __any(m > 8))
            sffeat::window_stats<(KMAX >= 16 ? 16 : KMAX), KMAX>(s, t, dmask, m, signed_times, col, kWave, row, 1u);
        else
            sffeat::window_stats<8, KMAX>(s, t, dmask, m, signed_times, col, kWave, row, 1u);
        if (LONG) {
            // (the sort scratch of the lanes' own windows is free by now: the long flows' values are parked there)
            static_assert(!LONG || kSlots * kSlotWords <= (uint32_t)KMAX * kWave, "parked flows fit the sort scratch");
            uint64_t todo = __ballot(long_flow);
            // the packets of the next long flow are requested while the current one is sorted
            int l = todo ? __ffsll((unsigned long long)todo) - 1 : 0;
            int m_l = todo ? (int)lane_value((uint32_t)m_w, l) : 0;
            LanePacket cur = long_flow_load(a, lane_value(o, l), m_l, lane);
            while (todo) {
                uint32_t n_slots = 0;
                while (todo && n_slots < kSlots) {
                    todo &= todo - 1ull;
                    const int l_next = todo ? __ffsll((unsigned long long)todo) - 1 : 0;
                    const int m_next = todo ? (int)lane_value((uint32_t)m_w, l_next) : 0;
                    uint32_t key[6];
                    int c0, c1;
                    long_flow_keys(cur, m_l, (uint32_t)l, lane, sort_col + n_slots * kSlotWords, key, c0, c1);
                    // (requested only now, behind the wait for the current flow's packets, and pinned here: the
                    // request then flies while the current flow is sorted)
                    __builtin_amdgcn_sched_barrier(0);
                    const LanePacket next = long_flow_load(a, lane_value(o, l_next), m_next, lane);
                    __builtin_amdgcn_sched_barrier(0);
                    long_flow_order_stats(key, m_l, c0, c1, lane, tile + l * kRow);
                    ++n_slots;
                    cur = next;
                    l = l_next;
                    m_l = m_next;
                }
                long_flow_chains(sort_col, n_slots, lane, tile);
            }
        }
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
        featurize_wave<8, false><<<grid, kWave, 0, ctx->stream>>>(a);
    else if (dmax <= 16)
        featurize_wave<16, false><<<grid, kWave, 0, ctx->stream>>>(a);
    else if (dmax <= 32)
        featurize_wave<32, false><<<grid, kWave, 0, ctx->stream>>>(a);
    else
        featurize_wave<32, true><<<grid, kWave, 0, ctx->stream>>>(a);
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
