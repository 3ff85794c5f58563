// Step 5: the slow model on the escalated flows only; its label replaces the fast one
// (Sections 3.1 and 4.4 of the paper).  The slow model is a 3-layer ReLU MLP.
//
// bfloat16 models run on the matrix cores: each layer is one tiled GEMM
// C[rows][N] = act(A[rows][K] * W[N][K]^T + b) built from 32x32x16 MFMA blocks with binary32
// accumulators.  Both operands are contiguous along K, which is exactly what an MFMA operand
// wants (each lane supplies 8 consecutive K values of one row or column).  The first layer
// builds its A tile on the fly from the escalated flows' feature rows (gather through the
// index list, standardise, clamp, round to bfloat16) or from packed header bits; the last
// layer adds the bias, finds the arg-max per row and scatters the label to the flow's slot.
// The row count comes from the device-side escalation count; blocks past it exit.
//
// binary32 models (small, used for the small workload) run on plain vector arithmetic.
#include "mlp_common.h"

namespace sf {
// fused single-kernel form for narrow hidden layers (slow_fused.hip)
bool slow_fused_ok(const sf_mlp* mlp, bool raw_input);
size_t slow_fused_ws_bytes(const sf_mlp* mlp);
int slow_fused(sf_ctx* ctx, void* ws, bool ws_is_ordered, const float* feat, uint32_t feat_ld, uint32_t n_rows,
               const uint32_t* esc_idx, const uint32_t* scatter, const uint32_t* esc_count, uint32_t esc_cap,
               uint32_t n_labels, const sf_mlp* mlp, float* logits, uint16_t* labels);
int order_all(sf_ctx* ctx, const sf_mlp* mlp, void* out);
// one hidden layer of any width on operand-ordered weights (slow_wide.hip)
int wide_layer(sf_ctx* ctx, int amode, const sfmlp::LayerArgs& a, const void* w_ordered, uint32_t rows_cap);
} // namespace sf

namespace {

using namespace sfmlp;

// 8 consecutive K values [k, k+8) of weight row n (row-major [N][K] bfloat16 bits), zero outside
__device__ __forceinline__ uint4 load_w_chunk(const LayerArgs& a, uint32_t n, uint32_t k)
{
    if (n >= a.N || k >= a.K) return make_uint4(0, 0, 0, 0);
    const uint16_t* p = a.w + (size_t)n * a.K + k;
    if (k + 8 <= a.K && (a.K & 7u) == 0 && (reinterpret_cast<uintptr_t>(a.w) & 15u) == 0)
        return *reinterpret_cast<const uint4*>(p);
    uint16_t v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = k + q < a.K ? p[q] : (uint16_t)0;
    return make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
}

// The last layer of a wide model: logits = A * W3^T + b3 on bfloat16 activations (at most BN classes), then the
// arg-max per row and the scatter of the label.  128 rows per block, four waves of 32 rows each.  K is walked
// in steps of 128; the operands of the next step are requested before the MFMAs of the current one, so that
// a launch with few blocks (a small batch) does not wait a whole memory latency per step.
constexpr int LBK = 128;      // K per step of the last layer
constexpr int LLDT = LBK + 8; // shared-memory row stride (elements): 272 bytes, 16-byte reads of 8 consecutive rows on distinct banks

template <int BN>
__global__ __launch_bounds__(256) void mlp_last_layer(LayerArgs a)
{
    constexpr int MI = 1, NI = BN / 32;   // a wave owns 32 rows x BN columns
    constexpr int WM = BM / 4;
    constexpr int A_CHUNKS = BM * LBK / 8 / 256; // 16-byte chunks per thread per step
    constexpr int B_CHUNKS = (BN * LBK / 8 + 255) / 256;
    constexpr int SM_AB = (BM + BN) * LLDT * 2;
    constexpr int SM_EPI = BM * (BN + 1) * 4;
    constexpr int SM_BYTES = SM_AB > SM_EPI ? SM_AB : SM_EPI;
    __shared__ __attribute__((aligned(16))) unsigned char smem[SM_BYTES];
    __shared__ uint32_t s_flow[BM];
    uint16_t* As = reinterpret_cast<uint16_t*>(smem);
    uint16_t* Bs = As + BM * LLDT;

    uint32_t total = *a.esc_count;
    total = total < a.esc_cap ? total : a.esc_cap;
    const uint32_t row0 = a.row_begin + blockIdx.x * BM; // first escalated row of this block
    if (row0 >= total) return;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wm = tid >> 6;

    if (tid < BM) // the index the row's label goes to
        s_flow[tid] = row0 + tid < total ? (a.scatter ? a.scatter[row0 + tid] : a.esc_idx[row0 + tid]) : 0u;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 ra[A_CHUNKS], rb[B_CHUNKS];
    auto fetch = [&](uint32_t k0) {
#pragma unroll
        for (int u = 0; u < A_CHUNKS; ++u) {
            const uint32_t c = tid + 256 * u, r = c / (LBK / 8), kq = c % (LBK / 8);
            ra[u] = load_a_chunk<A_BF16>(a, row0 + r < total, blockIdx.x * BM + r, 0u, k0 + kq * 8);
        }
#pragma unroll
        for (int u = 0; u < B_CHUNKS; ++u) {
            const uint32_t c = tid + 256 * u, r = c / (LBK / 8), kq = c % (LBK / 8);
            rb[u] = (r < (uint32_t)BN) ? load_w_chunk(a, r, k0 + kq * 8) : make_uint4(0, 0, 0, 0);
        }
    };
    fetch(0);
    for (uint32_t k0 = 0; k0 < a.K; k0 += LBK) {
        __syncthreads(); // previous step's fragment reads are done (first step: s_flow is in place)
#pragma unroll
        for (int u = 0; u < A_CHUNKS; ++u) {
            const uint32_t c = tid + 256 * u, r = c / (LBK / 8), kq = c % (LBK / 8);
            *reinterpret_cast<uint4*>(As + r * LLDT + kq * 8) = ra[u];
        }
#pragma unroll
        for (int u = 0; u < B_CHUNKS; ++u) {
            const uint32_t c = tid + 256 * u, r = c / (LBK / 8), kq = c % (LBK / 8);
            if (r < (uint32_t)BN) *reinterpret_cast<uint4*>(Bs + r * LLDT + kq * 8) = rb[u];
        }
        __syncthreads();
        if (k0 + LBK < a.K) fetch(k0 + LBK); // chunks past K read as zeros
        __builtin_amdgcn_sched_barrier(0);   // keep the requests ahead of the MFMAs
#pragma unroll
        for (int ks = 0; ks < LBK / 16; ++ks) {
            bf16x8 fa[MI], fb[NI];
            const uint32_t kofs = ks * 16 + (lane >> 5) * 8;
#pragma unroll
            for (int i = 0; i < MI; ++i)
                fa[i] = as_bf16x8(*reinterpret_cast<const uint4*>(As + (wm * WM + i * 32 + (lane & 31)) * LLDT + kofs));
#pragma unroll
            for (int j = 0; j < NI; ++j)
                fb[j] = as_bf16x8(*reinterpret_cast<const uint4*>(Bs + (j * 32 + (lane & 31)) * LLDT + kofs));
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // accumulator element v of lane l in a 32x32 block: row 8*(v/4) + 4*(l/32) + v%4, column l%32
    __syncthreads(); // operand tiles are dead; reuse the space for the logits tile
    float* Ls = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const uint32_t cl = j * 32 + (lane & 31);
            const float b = cl < a.N ? a.bias[cl] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t r = wm * WM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                Ls[r * (BN + 1) + cl] = acc[i][j][v] + b;
            }
        }
    __syncthreads();
    if (tid < BM && row0 + tid < total) {
        const float* lr = Ls + tid * (BN + 1);
        uint32_t best = 0;
        float bv = lr[0];
        for (uint32_t c = 0; c < a.N; ++c) {
            const float v = lr[c];
            if (a.logits) a.logits[(size_t)(row0 + tid) * a.N + c] = v;
            if (v > bv) {
                bv = v;
                best = c;
            }
        }
        if (s_flow[tid] < a.n_labels) a.labels[s_flow[tid]] = (uint16_t)best;
    }
}

// ---- binary32 model (plain vector arithmetic) ---------------------------------------------

struct F32Args {
    const uint32_t* esc_idx;
    const uint32_t* esc_count;
    uint32_t esc_cap, row_begin, rows_cap, n_rows;
    const float* feat;
    uint32_t feat_ld;
    const float* mu;
    const float* inv_sigma;
    float clamp;
    const uint32_t* off;
    const uint32_t* hdr;
    uint32_t hdr_words, raw_bits, raw_pkts, n_pkts;
    uint32_t n_in;
};

__global__ __launch_bounds__(256) void f32_input(F32Args a, float* __restrict__ z)
{
    uint32_t total = *a.esc_count;
    total = total < a.esc_cap ? total : a.esc_cap;
    if (a.row_begin >= total) return;
    uint32_t rows = total - a.row_begin;
    rows = rows < a.rows_cap ? rows : a.rows_cap;
    const uint64_t n = (uint64_t)rows * a.n_in;
    for (uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n; g += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t r = (uint32_t)(g / a.n_in), k = (uint32_t)(g % a.n_in);
        uint32_t flow = a.esc_idx[a.row_begin + r];
        flow = flow < a.n_rows ? flow : a.n_rows - 1u; // a bad list entry must not leave the input
        float v;
        if (a.feat) {
            v = a.feat[(size_t)flow * a.feat_ld + k];
            if (a.mu) {
                const float d = v - a.mu[k];
                v = d * a.inv_sigma[k];
                v = v < -a.clamp ? -a.clamp : v;
                v = v > a.clamp ? a.clamp : v;
            }
        } else {
            uint32_t b0 = a.off[flow], e0 = a.off[flow + 1];
            b0 = b0 < a.n_pkts ? b0 : a.n_pkts;
            e0 = e0 < a.n_pkts ? e0 : a.n_pkts;
            const uint32_t np = e0 > b0 ? e0 - b0 : 0;
            const uint32_t j = k / a.raw_bits, b = k - j * a.raw_bits;
            v = 0.f;
            if (j < np) {
                const uint32_t byte_i = b >> 3;
                const uint32_t word = a.hdr[(size_t)(b0 + j) * a.hdr_words + (byte_i >> 2)];
                v = (float)(((word >> (8u * (byte_i & 3u))) >> (7u - (b & 7u))) & 1u);
            }
        }
        z[g] = v;
    }
}

// out[r][o] = act(sum_k in[r][k] * w[o][k] + b[o]) in binary32, the sum taken in order of k (one multiply
// and one add per term, each rounded).  A block computes a 64 x 64 tile of outputs from K-slabs of 16 staged
// in shared memory; a thread owns a 4 x 4 patch (rows ty + 16 i, columns tx + 16 j).
constexpr int kF32Tile = 64, kF32Slab = 16;

__global__ __launch_bounds__(256) void f32_layer(const uint32_t* esc_count, uint32_t esc_cap, uint32_t row_begin,
                                                 uint32_t rows_cap, const float* __restrict__ in, uint32_t K,
                                                 const float* __restrict__ w, const float* __restrict__ bias,
                                                 uint32_t N, float* __restrict__ out, int relu)
{
    __shared__ float As[kF32Slab][kF32Tile + 1]; // [k][row]
    __shared__ float Ws[kF32Slab][kF32Tile + 1]; // [k][column]
    uint32_t total = *esc_count;
    total = total < esc_cap ? total : esc_cap;
    if (row_begin >= total) return;
    uint32_t rows = total - row_begin;
    rows = rows < rows_cap ? rows : rows_cap;
    const uint32_t r0 = blockIdx.x * kF32Tile, c0 = blockIdx.y * kF32Tile;
    if (r0 >= rows) return;
    const uint32_t tid = threadIdx.x, tx = tid & 15u, ty = tid >> 4;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (uint32_t k0 = 0; k0 < K; k0 += kF32Slab) {
        // 64 x 16 values of each operand, four per thread: element e -> (row e / 16, k e % 16)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t e = tid + 256u * q, rr = e >> 4, kk = e & 15u;
            const bool kin = k0 + kk < K;
            As[kk][rr] = (kin && r0 + rr < rows) ? in[(size_t)(r0 + rr) * K + k0 + kk] : 0.f;
            Ws[kk][rr] = (kin && c0 + rr < N) ? w[(size_t)(c0 + rr) * K + k0 + kk] : 0.f;
        }
        __syncthreads();
        const uint32_t kn = K - k0 < (uint32_t)kF32Slab ? K - k0 : (uint32_t)kF32Slab;
        for (uint32_t kk = 0; kk < kn; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t r = r0 + ty + 16 * i;
        if (r >= rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t o = c0 + tx + 16 * j;
            if (o < N) {
                const float y = acc[i][j] + bias[o];
                out[(size_t)r * N + o] = (relu && y < 0.f) ? 0.f : y;
            }
        }
    }
}

__global__ __launch_bounds__(256) void f32_argmax(const uint32_t* label_idx, const uint32_t* esc_count, uint32_t esc_cap,
                                                  uint32_t row_begin, uint32_t rows_cap, const float* __restrict__ lg,
                                                  uint32_t C, float* __restrict__ logits, uint16_t* __restrict__ labels,
                                                  uint32_t n_labels)
{
    uint32_t total = *esc_count;
    total = total < esc_cap ? total : esc_cap;
    if (row_begin >= total) return;
    uint32_t rows = total - row_begin;
    rows = rows < rows_cap ? rows : rows_cap;
    for (uint32_t r = blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += gridDim.x * blockDim.x) {
        const float* p = lg + (size_t)r * C;
        uint32_t best = 0;
        float bv = p[0];
        for (uint32_t c = 0; c < C; ++c) {
            const float v = p[c];
            if (logits) logits[(size_t)(row_begin + r) * C + c] = v;
            if (v > bv) {
                bv = v;
                best = c;
            }
        }
        const uint32_t dst = label_idx[row_begin + r];
        if (dst < n_labels) labels[dst] = (uint16_t)best;
    }
}

void launch_final(sf_ctx* ctx, const LayerArgs& a, uint32_t rows_cap)
{
    dim3 grid((rows_cap + BM - 1) / BM, 1);
    if (a.N <= 32)
        mlp_last_layer<32><<<grid, 256, 0, ctx->stream>>>(a);
    else
        mlp_last_layer<64><<<grid, 256, 0, ctx->stream>>>(a);
}

// labels = pred for every flow; the slow labels are scattered over it afterwards
__global__ __launch_bounds__(256) void copy_labels(const uint16_t* __restrict__ pred, uint16_t* __restrict__ labels, uint32_t n)
{
    const uint32_t base = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (base + 8 <= n && ((reinterpret_cast<uintptr_t>(pred) | reinterpret_cast<uintptr_t>(labels)) & 15u) == 0) {
        *reinterpret_cast<uint4*>(labels + base) = *reinterpret_cast<const uint4*>(pred + base);
    } else {
        for (uint32_t k = base; k < n && k < base + 8; ++k) labels[k] = pred[k];
    }
}

uint32_t pad64(uint32_t x) { return (x + 63u) / 64u * 64u; }

} // namespace

namespace {

// Both entry points.  esc_idx: input rows (of feat, n_rows of them, or flows of raw_src); scatter: where the
// labels go (NULL = esc_idx); n_flows: entries of labels.
int run_slow(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_rows, const sf_packets* raw_src,
             const sf_feat_cfg* raw_cfg, const uint32_t* esc_idx, const uint32_t* scatter, const uint32_t* esc_count,
             uint32_t esc_cap, uint32_t n_flows, const sf_mlp* mlp, const uint16_t* pred, float* logits, uint16_t* labels)
{
    if (!mlp) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: mlp is NULL");
    if (mlp->dtype != SF_F32 && mlp->dtype != SF_BF16) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: unknown dtype %d", mlp->dtype);
    if (!mlp->n_in || !mlp->n_h1 || !mlp->n_h2 || !mlp->n_classes)
        return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: a layer width is zero");
    if (mlp->n_classes > SF_MAX_CLASSES)
        return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: n_classes %u > %d", mlp->n_classes, SF_MAX_CLASSES);
    if (!mlp->w1 || !mlp->w2 || !mlp->w3 || !mlp->b1 || !mlp->b2 || !mlp->b3)
        return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: weights or biases missing");
    if ((mlp->mu == nullptr) != (mlp->inv_sigma == nullptr))
        return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: mu and inv_sigma come together");
    if (n_flows == 0) return SF_OK;
    if (pred && pred != labels) {
        // labels = the fast prediction for every flow, also when nothing escalates (Section 4.4: the fast
        // label stands unless the slow model replaces it)
        if (!labels) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: labels is NULL");
        uint32_t blocks = (n_flows + 2047) / 2048;
        copy_labels<<<blocks, 256, 0, ctx->stream>>>(pred, labels, n_flows);
        SF_LAUNCH_CHECK(ctx, "copy_labels");
    }
    if (esc_cap == 0 || n_rows == 0) return SF_OK;
    if ((feat == nullptr) == (raw_src == nullptr))
        return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: give exactly one of feat and raw_src");
    if (feat && mlp->n_in > feat_ld) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: n_in %u > feat_ld %u", mlp->n_in, feat_ld);
    if (raw_src) {
        if (!raw_cfg || !raw_src->pkt_hdr || !raw_src->flow_off || raw_src->hdr_words == 0)
            return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: raw input needs raw_cfg, flow_off and pkt_hdr");
        if (raw_cfg->raw_bits == 0 || raw_cfg->raw_bits > 32 * raw_src->hdr_words ||
            (uint64_t)raw_cfg->raw_pkts * raw_cfg->raw_bits != mlp->n_in)
            return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: raw_pkts*raw_bits must equal n_in and fit the header words");
        if (raw_src->n_flows != n_flows) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: raw_src->n_flows != n_flows");
        if (raw_src->n_pkts >> 32) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: n_pkts exceeds 32-bit offsets");
    }
    if (!esc_idx || !esc_count || !labels) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer: esc_idx, esc_count or labels is NULL");
    if (!scatter && esc_cap > n_flows) esc_cap = n_flows;

    sf::Carve ws(ctx);
    const bool bf = mlp->dtype == SF_BF16;
    if (sf::slow_fused_ok(mlp, raw_src != nullptr)) {
        if (mlp->ordered)
            return sf::slow_fused(ctx, const_cast<void*>(mlp->ordered), true, feat, feat_ld, n_rows, esc_idx, scatter, esc_count,
                                  esc_cap, n_flows, mlp, logits, labels);
        const size_t need = sf::slow_fused_ws_bytes(mlp);
        void* w = ws.take(need);
        if (!w) return sf::fail(ctx, SF_ENOMEM, "sf_slow_infer: workspace too small for %zu bytes of re-ordered weights", need);
        return sf::slow_fused(ctx, w, false, feat, feat_ld, n_rows, esc_idx, scatter, esc_count, esc_cap, n_flows, mlp, logits,
                              labels);
    }
    const void *w1o = nullptr, *w2o = nullptr;
    if (bf && mlp->ordered) {
        w1o = mlp->ordered;
        w2o = (const char*)mlp->ordered + sf::reordered_bytes(mlp->n_h1, mlp->n_in);
    } else if (bf) {
        // operand-ordered copies of the two hidden layers' weights
        void* o1 = ws.take(sf::reordered_bytes(mlp->n_h1, mlp->n_in));
        void* o2 = ws.take(sf::reordered_bytes(mlp->n_h2, mlp->n_h1));
        if (!o1 || !o2) return sf::fail(ctx, SF_ENOMEM, "sf_slow_infer: workspace too small for the re-ordered weights");
        const sf::ReorderSpec specs[2] = {{mlp->w1, mlp->n_h1, mlp->n_in, o1}, {mlp->w2, mlp->n_h2, mlp->n_h1, o2}};
        const int rc = sf::reorder_weights_async(ctx, specs, 2);
        if (rc != SF_OK) return rc;
        w1o = o1;
        w2o = o2;
    }
    const uint32_t ld1 = bf ? pad64(mlp->n_h1) : mlp->n_h1, ld2 = bf ? pad64(mlp->n_h2) : mlp->n_h2;
    const size_t row_bytes = bf ? ((size_t)ld1 + ld2) * 2 : ((size_t)mlp->n_in + ld1 + ld2 + mlp->n_classes) * 4;
    const size_t avail = ws.left() > 4 * sf::kAlign ? ws.left() - 4 * sf::kAlign : 0;
    uint64_t rows_cap = avail / row_bytes / BM * BM;
    if (rows_cap < sf::kSlowMinRows)
        return sf::fail(ctx, SF_ENOMEM, "sf_slow_infer: workspace holds %llu rows of hidden activations, need at least %u",
                        (unsigned long long)rows_cap, sf::kSlowMinRows);
    if (rows_cap > ((uint64_t)esc_cap + BM - 1) / BM * BM) rows_cap = ((uint64_t)esc_cap + BM - 1) / BM * BM;
    const uint32_t R = (uint32_t)rows_cap;

    if (bf) {
        uint16_t* h1 = (uint16_t*)ws.take((size_t)R * ld1 * 2);
        uint16_t* h2 = (uint16_t*)ws.take((size_t)R * ld2 * 2);
        if (!h1 || !h2) return sf::fail(ctx, SF_ENOMEM, "sf_slow_infer: workspace carve failed");
        for (uint32_t begin = 0; begin < esc_cap; begin += R) {
            LayerArgs a = {};
            a.esc_idx = esc_idx;
            a.scatter = scatter;
            a.esc_count = esc_count;
            a.esc_cap = esc_cap;
            a.row_begin = begin;
            a.n_rows = n_rows;
            a.n_labels = n_flows;
            a.labels = labels;
            // layer 1
            a.feat = feat;
            a.feat_ld = feat_ld;
            a.mu = mlp->mu;
            a.inv_sigma = mlp->inv_sigma;
            a.clamp = mlp->clamp;
            if (raw_src) {
                a.off = raw_src->flow_off;
                a.hdr = raw_src->pkt_hdr;
                a.hdr_words = raw_src->hdr_words;
                a.raw_bits = raw_cfg->raw_bits;
                a.raw_pkts = raw_cfg->raw_pkts;
                a.n_pkts = (uint32_t)raw_src->n_pkts;
            }
            a.w = (const uint16_t*)mlp->w1;
            a.bias = mlp->b1;
            a.N = mlp->n_h1;
            a.K = mlp->n_in;
            a.h_out = h1;
            a.ldh = ld1;
            {
                const int rc = sf::wide_layer(ctx, raw_src ? A_RAW : A_FEAT, a, w1o, R);
                if (rc != SF_OK) return rc;
            }
            // layer 2
            a.a_bf16 = h1;
            a.lda = ld1;
            a.w = (const uint16_t*)mlp->w2;
            a.bias = mlp->b2;
            a.N = mlp->n_h2;
            a.K = mlp->n_h1;
            a.h_out = h2;
            a.ldh = ld2;
            {
                const int rc = sf::wide_layer(ctx, A_BF16, a, w2o, R);
                if (rc != SF_OK) return rc;
            }
            // layer 3
            a.a_bf16 = h2;
            a.lda = ld2;
            a.w = (const uint16_t*)mlp->w3;
            a.bias = mlp->b3;
            a.N = mlp->n_classes;
            a.K = mlp->n_h2;
            a.h_out = nullptr;
            a.ldh = 0;
            a.logits = logits;
            launch_final(ctx, a, R);
            SF_LAUNCH_CHECK(ctx, "mlp_last_layer");
        }
        return SF_OK;
    }

    float* z = (float*)ws.take((size_t)R * mlp->n_in * 4);
    float* h1 = (float*)ws.take((size_t)R * ld1 * 4);
    float* h2 = (float*)ws.take((size_t)R * ld2 * 4);
    float* lg = (float*)ws.take((size_t)R * mlp->n_classes * 4);
    if (!z || !h1 || !h2 || !lg) return sf::fail(ctx, SF_ENOMEM, "sf_slow_infer: workspace carve failed");
    for (uint32_t begin = 0; begin < esc_cap; begin += R) {
        F32Args f = {};
        f.esc_idx = esc_idx;
        f.esc_count = esc_count;
        f.esc_cap = esc_cap;
        f.row_begin = begin;
        f.rows_cap = R;
        f.n_rows = n_rows;
        f.feat = feat;
        f.feat_ld = feat_ld;
        f.mu = mlp->mu;
        f.inv_sigma = mlp->inv_sigma;
        f.clamp = mlp->clamp;
        if (raw_src) {
            f.off = raw_src->flow_off;
            f.hdr = raw_src->pkt_hdr;
            f.hdr_words = raw_src->hdr_words;
            f.raw_bits = raw_cfg->raw_bits;
            f.raw_pkts = raw_cfg->raw_pkts;
            f.n_pkts = (uint32_t)raw_src->n_pkts;
        }
        f.n_in = mlp->n_in;
        auto blocks = [&](uint64_t n) { uint64_t b = (n + 255) / 256; return (uint32_t)(b > 16384 ? 16384 : (b ? b : 1)); };
        f32_input<<<blocks((uint64_t)R * mlp->n_in), 256, 0, ctx->stream>>>(f, z);
        SF_LAUNCH_CHECK(ctx, "f32_input");
        auto tiles = [&](uint32_t n_out) { return dim3((R + kF32Tile - 1) / kF32Tile, (n_out + kF32Tile - 1) / kF32Tile); };
        f32_layer<<<tiles(mlp->n_h1), 256, 0, ctx->stream>>>(esc_count, esc_cap, begin, R, z, mlp->n_in,
                                                                            (const float*)mlp->w1, mlp->b1, mlp->n_h1, h1, 1);
        SF_LAUNCH_CHECK(ctx, "f32_layer 1");
        f32_layer<<<tiles(mlp->n_h2), 256, 0, ctx->stream>>>(esc_count, esc_cap, begin, R, h1, mlp->n_h1,
                                                                            (const float*)mlp->w2, mlp->b2, mlp->n_h2, h2, 1);
        SF_LAUNCH_CHECK(ctx, "f32_layer 2");
        f32_layer<<<tiles(mlp->n_classes), 256, 0, ctx->stream>>>(
            esc_count, esc_cap, begin, R, h2, mlp->n_h2, (const float*)mlp->w3, mlp->b3, mlp->n_classes, lg, 0);
        SF_LAUNCH_CHECK(ctx, "f32_layer 3");
        f32_argmax<<<blocks(R), 256, 0, ctx->stream>>>(scatter ? scatter : esc_idx, esc_count, esc_cap, begin, R, lg,
                                                       mlp->n_classes, logits, labels, n_flows);
        SF_LAUNCH_CHECK(ctx, "f32_argmax");
    }
    return SF_OK;
}

} // namespace

extern "C" int sf_slow_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, const sf_packets* raw_src,
                             const sf_feat_cfg* raw_cfg, const uint32_t* esc_idx, const uint32_t* esc_count,
                             uint32_t esc_cap, uint32_t n_flows, const sf_mlp* mlp, const uint16_t* pred, float* logits,
                             uint16_t* labels)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_slow_infer: ctx is NULL");
    return run_slow(ctx, feat, feat_ld, n_flows, raw_src, raw_cfg, esc_idx, nullptr, esc_count, esc_cap, n_flows, mlp, pred,
                    logits, labels);
}

extern "C" int sf_slow_infer_pairs(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_rows,
                                   const uint32_t* pair_row, const uint32_t* pair_flow, const uint32_t* n_pairs,
                                   uint32_t pair_cap, uint32_t n_flows, const sf_mlp* mlp, float* logits, uint16_t* labels)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_slow_infer_pairs: ctx is NULL");
    if (!feat) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer_pairs: feat is NULL");
    if (pair_cap && n_flows && n_rows && !pair_flow) return sf::fail(ctx, SF_EINVAL, "sf_slow_infer_pairs: pair_flow is NULL");
    return run_slow(ctx, feat, feat_ld, n_rows, nullptr, nullptr, pair_row, pair_flow, n_pairs, pair_cap, n_flows, mlp,
                    nullptr, logits, labels);
}

extern "C" size_t sf_mlp_ordered_bytes(const sf_mlp* mlp)
{
    if (!mlp || mlp->dtype != SF_BF16 || !mlp->n_in || !mlp->n_h1 || !mlp->n_h2 || !mlp->n_classes) return 0;
    return sf::reordered_bytes(mlp->n_h1, mlp->n_in) + sf::reordered_bytes(mlp->n_h2, mlp->n_h1) +
           sf::reordered_bytes(32, mlp->n_h2);
}

extern "C" int sf_mlp_order(sf_ctx* ctx, const sf_mlp* mlp, void* ordered)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_mlp_order: ctx is NULL");
    if (!mlp || !ordered) return sf::fail(ctx, SF_EINVAL, "sf_mlp_order: mlp or ordered is NULL");
    if (mlp->dtype != SF_BF16) return sf::fail(ctx, SF_EINVAL, "sf_mlp_order: only bfloat16 models have an ordered copy");
    if (!mlp->n_in || !mlp->n_h1 || !mlp->n_h2 || !mlp->n_classes || mlp->n_classes > 32 || !mlp->w1 || !mlp->w2 || !mlp->w3)
        return sf::fail(ctx, SF_EINVAL, "sf_mlp_order: widths, class count (at most 32) or weights missing");
    if ((uintptr_t)ordered & 255u) return sf::fail(ctx, SF_EINVAL, "sf_mlp_order: ordered is not 256-byte aligned");
    return sf::order_all(ctx, mlp, ordered);
}
