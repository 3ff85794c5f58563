// Pieces shared by the layer-by-layer MLP kernels: the argument block of one layer and the
// builder of the A operand (8 consecutive K values of one escalated row as bfloat16), which reads
// a bfloat16 activation matrix, or gathers and standardises a feature row, or unpacks header bits.
#pragma once

#include "common.h"

namespace sfmlp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BM = 128; // rows per block
constexpr int BK = 64;  // K per main-loop step
constexpr int LDT = BK + 8; // shared-memory row stride (elements): 144 bytes keeps 16-byte
                            // reads of 8 consecutive rows on distinct banks

enum { A_BF16 = 0, A_FEAT = 1, A_RAW = 2 };

struct LayerArgs {
    // rows
    const uint32_t* esc_idx;  // row e reads the input row esc_idx[e] (clamped below n_rows) ...
    const uint32_t* scatter;  // ... and its label goes to labels[scatter[e]]; NULL = the same index
    const uint32_t* esc_count;
    uint32_t esc_cap;
    uint32_t row_begin; // first escalated row of this chunk
    uint32_t n_rows;    // rows of the input (feature matrix or flows of the packet arrays)
    uint32_t n_labels;  // entries of labels; a label index outside is not written
    // A operand
    const uint16_t* a_bf16; // [rows_in_chunk][lda]
    uint32_t lda;
    const float* feat;
    uint32_t feat_ld;
    const float* mu;
    const float* inv_sigma;
    float clamp;
    const uint32_t* off;
    const uint32_t* hdr;
    uint32_t hdr_words, raw_bits, raw_pkts, n_pkts;
    // weights
    const uint16_t* w; // [N][K] bfloat16 bit patterns
    const float* bias;
    uint32_t N, K;
    // output
    uint16_t* h_out; // [rows_in_chunk][ldh] bfloat16
    uint32_t ldh;
    float* logits;   // [esc_cap][N] or NULL
    uint16_t* labels;
};

static __device__ __forceinline__ uint16_t f32_to_bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16); // inf / nan: truncate
    u += 0x7FFFu + ((u >> 16) & 1u);                                  // round to nearest even
    return (uint16_t)(u >> 16);
}

static __device__ __forceinline__ uint32_t pack2(uint16_t lo, uint16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }

// the packets of a flow for the raw-bit input: first packet and count, clamped into the packet arrays
static __device__ __forceinline__ void raw_flow_range(const LayerArgs& a, uint32_t flow, uint32_t& b0, uint32_t& n)
{
    uint32_t e0 = a.off[flow + 1];
    b0 = a.off[flow];
    b0 = b0 < a.n_pkts ? b0 : a.n_pkts;
    e0 = e0 < a.n_pkts ? e0 : a.n_pkts;
    n = e0 > b0 ? e0 - b0 : 0;
}

// 8 consecutive raw-bit features [k, k+8) of a flow whose packets start at b0 (n of them) as bfloat16 0.0 / 1.0:
// feature k = raw_bits * packet + bit; bit b is bit 7-(b%8) of header byte b/8; zero past K and past the flow
static __device__ __forceinline__ uint4 raw_chunk_at(const LayerArgs& a, uint32_t b0, uint32_t n, uint32_t k)
{
    if (k >= a.K) return make_uint4(0, 0, 0, 0);
    uint16_t v[8];
    if ((a.raw_bits & 7u) == 0 && k + 8u <= a.K) {
        // the 8 features are the 8 bits of one header byte (k is a multiple of 8): one word load
        const uint32_t j = k / a.raw_bits, b = k - j * a.raw_bits, byte_i = b >> 3;
        uint32_t byte = 0;
        if (j < n) byte = (a.hdr[(size_t)(b0 + j) * a.hdr_words + (byte_i >> 2)] >> (8u * (byte_i & 3u))) & 0xFFu;
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = ((byte >> (7 - q)) & 1u) ? (uint16_t)0x3F80 : (uint16_t)0;
        return make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const uint32_t kk = k + q;
        uint16_t bit = 0;
        if (kk < a.K) {
            const uint32_t j = kk / a.raw_bits, b = kk - j * a.raw_bits;
            if (j < n) {
                const uint32_t byte_i = b >> 3;
                const uint32_t word = a.hdr[(size_t)(b0 + j) * a.hdr_words + (byte_i >> 2)];
                const uint32_t byte = (word >> (8u * (byte_i & 3u))) & 0xFFu;
                bit = (uint16_t)((byte >> (7u - (b & 7u))) & 1u);
            }
        }
        v[q] = bit ? (uint16_t)0x3F80 : (uint16_t)0; // bfloat16 1.0 or 0.0
    }
    return make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
}

// 8 consecutive K values [k, k+8) of escalated row e as bfloat16, zero past K.
template <int AMODE>
static __device__ __forceinline__ uint4 load_a_chunk(const LayerArgs& a, bool row_ok, uint32_t row_in_chunk,
                                              uint32_t flow, uint32_t k)
{
    uint4 out = make_uint4(0, 0, 0, 0);
    if (!row_ok || k >= a.K) return out;
    if (AMODE == A_BF16) {
        const uint16_t* p = a.a_bf16 + (size_t)row_in_chunk * a.lda + k;
        if (k + 8 <= a.K && (a.lda & 7u) == 0) return *reinterpret_cast<const uint4*>(p);
        uint16_t v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = k + q < a.K ? p[q] : (uint16_t)0;
        return make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
    }
    if (AMODE == A_FEAT) {
        const float* p = a.feat + (size_t)flow * a.feat_ld + k;
        float x[8];
        if (k + 8 <= a.K && (a.feat_ld & 3u) == 0 && (reinterpret_cast<uintptr_t>(a.feat) & 15u) == 0 && (k & 3u) == 0) {
            const float4 x0 = reinterpret_cast<const float4*>(p)[0], x1 = reinterpret_cast<const float4*>(p)[1];
            x[0] = x0.x; x[1] = x0.y; x[2] = x0.z; x[3] = x0.w;
            x[4] = x1.x; x[5] = x1.y; x[6] = x1.z; x[7] = x1.w;
        } else {
#pragma unroll
            for (int q = 0; q < 8; ++q) x[q] = k + q < a.K ? p[q] : 0.f;
        }
        uint16_t v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float z = x[q];
            if (a.mu && k + q < a.K) {
                const float d = z - a.mu[k + q];
                z = d * a.inv_sigma[k + q];
                z = z < -a.clamp ? -a.clamp : z;
                z = z > a.clamp ? a.clamp : z;
            }
            v[q] = k + q < a.K ? f32_to_bf16_bits(z) : (uint16_t)0;
        }
        return make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
    }
    // A_RAW
    uint32_t b0, n;
    raw_flow_range(a, flow, b0, n);
    return raw_chunk_at(a, b0, n, k);
}

static __device__ __forceinline__ bf16x8 as_bf16x8(uint4 u)
{
    union {
        uint4 u;
        bf16x8 b;
    } c;
    c.u = u;
    return c.b;
}


} // namespace sfmlp

namespace sf {
// operand-ordered copies of weight matrices (slow_fused.hip): out[(nb*KS + ks)*64 + lane] holds the 8
// values W[nb*32 + lane%32][ks*16 + 8*(lane/32) ..+8), K padded to a multiple of 64, zero outside
struct ReorderSpec {
    const void* w; // [N][K] bfloat16 bits, row-major
    uint32_t N, K;
    void* out;
};
size_t reordered_bytes(uint32_t N, uint32_t K);
int reorder_weights_async(sf_ctx* ctx, const ReorderSpec* specs, int n_specs); // at most 3 per launch
} // namespace sf
