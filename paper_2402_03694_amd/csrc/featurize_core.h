// Device code of step 1 shared by the stand-alone feature kernel and the fused feature + forest kernel:
// the 32 statistics of one prefix window of a flow whose packets sit in the lane's registers
// (context length k, Section 3.1 of the paper).
//
// Every binary32 operation is issued on its own, in packet order (the files that include this are
// compiled without floating-point contraction); a packet outside a group contributes +0.0 to that
// group's running sums, which leaves them unchanged.
//
// Order statistics (min, max, median of the two directions and of all packets) need sorted values.
// Instead of three sorting networks per quantity (one per group) there is ONE, on keys that carry the
// direction as their top bit and the value of a direction-1 packet complemented: after it the
// direction-0 packets stand first in ascending order, the direction-1 packets behind them in
// DESCENDING order, padding last.  Both directions' statistics are read from that array at
// data-dependent positions; the array, with padding read as the smallest value, is also a bitonic
// sequence (up, then down), so ONE merge stage (log2 N levels instead of a full network) sorts all
// packets together for the third group.  This needs values that order like non-negative integers
// below 2^W: packet sizes (W = 16) and non-negative times (W = 31, the binary32 bit pattern).  A wave
// that holds a time with its sign bit set takes the general path: three full networks on
// order-preserving keys.
//
// The element at a data-dependent rank is read through a per-lane column of shared memory
// (col[i * stride], stride = lanes that share the array, so every lane stays on its own bank).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sffeat {

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

__device__ __forceinline__ void cmp_swap(uint32_t& lo, uint32_t& hi)
{
    const uint32_t a = lo < hi ? lo : hi, b = lo < hi ? hi : lo;
    lo = a;
    hi = b;
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
                    if (i + j + k < N && (i + j) / (2 * p) == (i + j + k) / (2 * p)) cmp_swap(a[i + j], a[i + j + k]);
                }
            }
        }
    }
}

// Sorts a bitonic sequence (ascending, then descending) into ascending order: log2 N levels of N/2 exchanges.
template <int N>
__device__ __forceinline__ void bitonic_merge(uint32_t (&a)[N])
{
#pragma unroll
    for (int k = N / 2; k >= 1; k >>= 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if ((i & k) == 0) cmp_swap(a[i], a[i + k]);
        }
    }
}

__device__ __forceinline__ bool bit_of(uint64_t m, int j) { return (m >> j) & 1ull; }

// Order statistics of one quantity for the three groups (0: direction 0, 1: direction 1, 2: all packets).
// v[i]: the value of packet i as a non-negative integer below 2^W that orders like the value.  valid: the
// window's packets; m1: those of direction 1; m = c0 + c1 packets.  Results are such integers too; for an
// empty group they are meaningless (the caller writes zeros).  lo/hi: the two middle elements (equal for an
// odd count).
template <int N, int W>
__device__ __forceinline__ void order_stats3(const uint32_t (&v)[N], uint64_t valid, uint64_t m1, int m, int c0, int c1,
                                             uint32_t* col, uint32_t stride, uint32_t (&mn)[3], uint32_t (&mx)[3],
                                             uint32_t (&lo)[3], uint32_t (&hi)[3])
{
    constexpr uint32_t kMask = (1u << W) - 1u;            // W = 31: 0x7FFFFFFF
    constexpr uint32_t kPad = (1u << W) | kMask;          // the largest key; decodes to the value 0
    uint32_t key[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const uint32_t k = bit_of(m1, i) ? ((1u << W) | (v[i] ^ kMask)) : v[i];
        key[i] = bit_of(valid, i) ? k : kPad;
    }
    sort_network<N>(key);
#pragma unroll
    for (int i = 0; i < N; ++i) col[i * stride] = key[i];
    // direction 0: ascending at positions [0, c0)
    const int l0 = c0 > 0 ? c0 - 1 : 0;
    mn[0] = key[0];
    mx[0] = col[l0 * stride];
    lo[0] = col[(l0 >> 1) * stride];
    hi[0] = col[(c0 >> 1) * stride];
    // direction 1: descending at positions [c0, m); rank r (ascending) sits at position m - 1 - r
    const int l1 = c1 > 0 ? c1 - 1 : 0;
    const int top = m > 0 ? m - 1 : 0;
    const int p_mx = c0 < N ? c0 : N - 1; // c1 = 0 and c0 = N: the group is empty, any position will do
    mn[1] = col[top * stride] ^ kMask;    // (key & kMask) ^ kMask; the direction bit is cleared below
    mx[1] = col[p_mx * stride] ^ kMask;
    lo[1] = col[(top - (l1 >> 1)) * stride] ^ kMask;
    hi[1] = col[(top - (c1 >> 1) < 0 ? 0 : top - (c1 >> 1)) * stride] ^ kMask;
    mn[1] &= kMask;
    mx[1] &= kMask;
    lo[1] &= kMask;
    hi[1] &= kMask;
    // all packets: decode (padding becomes 0, the smallest value), merge; the padding then stands first
#pragma unroll
    for (int i = 0; i < N; ++i) key[i] = (key[i] & kMask) ^ ((key[i] >> W) ? kMask : 0u);
    bitonic_merge<N>(key);
#pragma unroll
    for (int i = 0; i < N; ++i) col[i * stride] = key[i];
    const int first = N - m; // number of padding elements
    const int la = m > 0 ? m - 1 : 0;
    const int f = first < N ? first : N - 1;
    mn[2] = col[f * stride];
    mx[2] = key[N - 1];
    lo[2] = col[(f + (la >> 1)) * stride];
    hi[2] = col[(f + (m >> 1) < N ? f + (m >> 1) : N - 1) * stride];
}

// General path for times with the sign bit set somewhere in the wave: one full network per group on
// order-preserving keys, padded with the largest key.
template <int N, int KMAX>
__device__ __forceinline__ void order_stats_signed(const float (&x)[KMAX], uint64_t gm, int cg, uint32_t* col, uint32_t stride,
                                                   float& mn, float& mx, float& lo, float& hi)
{
    uint32_t key[N];
#pragma unroll
    for (int i = 0; i < N; ++i) key[i] = bit_of(gm, i) ? order_key(x[i]) : 0xFFFFFFFFu;
    sort_network<N>(key);
#pragma unroll
    for (int i = 0; i < N; ++i) col[i * stride] = key[i];
    const int last = cg > 0 ? cg - 1 : 0;
    mn = from_key(key[0]);
    mx = from_key(col[last * stride]);
    lo = from_key(col[(last >> 1) * stride]);
    hi = from_key(col[(cg >> 1) * stride]);
}

// The 32 statistics of one prefix window of m <= N packets -> dst[k * ds], k = 10*g + 5*q + stat, then
// total bytes (k = 30) and packet count (k = 31).  Each result is stored as soon as it is known (the
// sorting networks need the registers).  signed_times: wave-uniform, some lane of the wave holds a time
// with its sign bit set.  dst and col must not overlap.
template <int N, int KMAX>
__device__ __forceinline__ void window_stats(const float (&s)[KMAX], const float (&t)[KMAX], uint64_t dmask, int m,
                                             bool signed_times, uint32_t* col, uint32_t stride, float* dst, uint32_t ds)
{
    static_assert(N <= KMAX, "window network larger than the register file of the flow");
    const uint64_t valid = m >= 64 ? ~0ull : ((1ull << m) - 1ull);
    const uint64_t m1 = dmask & valid, m0 = ~dmask & valid;
    const int c1 = __popcll(m1), c0 = m - c1;
    const bool e0 = c0 == 0, e1 = c1 == 0, ea = m == 0;
    {
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
            const float xa = a - mSa, xb = b - mTa;
            const float xa2 = xa * xa, xb2 = xb * xb;
            qSa = qSa + (v ? xa2 : 0.f);
            qTa = qTa + (v ? xb2 : 0.f);
            const float ga = a - (d1 ? mS1 : mS0), gb = b - (d1 ? mT1 : mT0);
            const float ga2 = ga * ga, gb2 = gb * gb;
            qS0 = qS0 + (d0 ? ga2 : 0.f);
            qS1 = qS1 + (d1 ? ga2 : 0.f);
            qT0 = qT0 + (d0 ? gb2 : 0.f);
            qT1 = qT1 + (d1 ? gb2 : 0.f);
        }
        const float vS0 = qS0 / n0, vS1 = qS1 / n1, vSa = qSa / na;
        const float vT0 = qT0 / n0, vT1 = qT1 / n1, vTa = qTa / na;
        dst[0 * ds] = e0 ? 0.f : mS0;
        dst[1 * ds] = e0 ? 0.f : sqrtf(vS0);
        dst[5 * ds] = e0 ? 0.f : mT0;
        dst[6 * ds] = e0 ? 0.f : sqrtf(vT0);
        dst[10 * ds] = e1 ? 0.f : mS1;
        dst[11 * ds] = e1 ? 0.f : sqrtf(vS1);
        dst[15 * ds] = e1 ? 0.f : mT1;
        dst[16 * ds] = e1 ? 0.f : sqrtf(vT1);
        dst[20 * ds] = ea ? 0.f : mSa;
        dst[21 * ds] = ea ? 0.f : sqrtf(vSa);
        dst[25 * ds] = ea ? 0.f : mTa;
        dst[26 * ds] = ea ? 0.f : sqrtf(vTa);
        dst[30 * ds] = sSa; // total bytes: every partial sum is an integer below 2^24, so this is exact
        dst[31 * ds] = (float)m;
    }
    // order statistics: sizes always as 16-bit integers (exact in binary32)
    {
        uint32_t v[N], a[3], b[3], c[3], d[3];
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = (uint32_t)s[i];
        order_stats3<N, 16>(v, valid, m1, m, c0, c1, col, stride, a, b, c, d);
#pragma unroll
        for (int g = 0; g < 3; ++g) {
            const int cg = g == 0 ? c0 : (g == 1 ? c1 : m);
            const float lo = (float)c[g], hi = (float)d[g];
            const float two = lo + hi;
            dst[(10 * g + 2) * ds] = cg == 0 ? 0.f : (float)a[g];
            dst[(10 * g + 3) * ds] = cg == 0 ? 0.f : (float)b[g];
            dst[(10 * g + 4) * ds] = cg == 0 ? 0.f : ((cg & 1) ? hi : two * 0.5f);
        }
    }
    if (!signed_times) {
        uint32_t v[N], a[3], b[3], c[3], d[3];
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = __float_as_uint(t[i]);
        order_stats3<N, 31>(v, valid, m1, m, c0, c1, col, stride, a, b, c, d);
#pragma unroll
        for (int g = 0; g < 3; ++g) {
            const int cg = g == 0 ? c0 : (g == 1 ? c1 : m);
            const float lo = __uint_as_float(c[g]), hi = __uint_as_float(d[g]);
            const float two = lo + hi;
            dst[(10 * g + 7) * ds] = cg == 0 ? 0.f : __uint_as_float(a[g]);
            dst[(10 * g + 8) * ds] = cg == 0 ? 0.f : __uint_as_float(b[g]);
            dst[(10 * g + 9) * ds] = cg == 0 ? 0.f : ((cg & 1) ? hi : two * 0.5f);
        }
    } else {
#pragma unroll 1
        for (int g = 0; g < 3; ++g) {
            const uint64_t gm = g == 0 ? m0 : (g == 1 ? m1 : valid);
            const int cg = g == 0 ? c0 : (g == 1 ? c1 : m);
            float mn, mx, lo, hi;
            order_stats_signed<N, KMAX>(t, gm, cg, col, stride, mn, mx, lo, hi);
            const float two = lo + hi;
            dst[(10 * g + 7) * ds] = cg == 0 ? 0.f : mn;
            dst[(10 * g + 8) * ds] = cg == 0 ? 0.f : mx;
            dst[(10 * g + 9) * ds] = cg == 0 ? 0.f : ((cg & 1) ? hi : two * 0.5f);
        }
    }
}

} // namespace sffeat
