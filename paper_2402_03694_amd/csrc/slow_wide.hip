// Step 5, one hidden layer of the slow model for any width (Sections 3.1 and 4.4 of the paper:
// the slow model runs on the escalated flows only): H_out = relu(A * W^T + b), bfloat16 in,
// binary32 MFMA accumulation, bfloat16 out.
//
// A block is eight waves and owns 128 rows x 512 output columns; wave w owns columns
// [64w, 64w+64) for all 128 rows (4x2 accumulators of v_mfma_f32_32x32x16_bf16, weight operand
// first, so a lane holds 4 consecutive columns of one row).  The A operand is streamed through
// shared memory in slabs of 64 K-values, double-buffered, one barrier per slab; it is built by
// the shared chunk loader (bfloat16 activations, gathered and standardised feature rows, or
// unpacked header bits).  The weight operand comes operand-ordered straight from the cache
// through a ring of register buffers, as in the fused kernel.  The output tile is staged in
// shared memory behind the slabs, 64 rows at a time, and written as whole 1 KB rows.
// A layer whose K fits the two slab buffers (K <= 128: a first layer on flow statistics), on enough rows
// to give every compute unit a 128-row block of its own (decided in the kernel from the device-side
// count), is run with one block per 128 rows that walks ALL column blocks: the input rows are gathered
// once and stay in shared memory, and the next column block's first weight operands are requested
// before the current one's epilogue, so that a block does not pay the gather, the weight latency and
// the write-out of every 128 x 512 tile one after the other (4,194,304 flows, 793 k rows through
// 128-2048-2048-32: 9.4 -> 8.4 ms for the whole slow step).
#include "mlp_common.h"

namespace sf {
int wide_layer(sf_ctx* ctx, int amode, const sfmlp::LayerArgs& a, const void* w_ordered, uint32_t rows_cap);
}

namespace {

using namespace sfmlp;

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int WBM = 128;          // rows per block
constexpr int WBN = 512;          // columns per block
constexpr int WWAVES = 8;
constexpr int WNI = 2, WMI = 4;   // 32-column / 32-row accumulator blocks per wave
constexpr int WSLAB = 64;         // K values per slab
constexpr int WLDS = WSLAB + 8;   // slab row stride (elements)
constexpr int WLDO = WBN + 8;     // output tile row stride (elements)
constexpr int WRING = 4;          // = k-steps per slab
constexpr int WHALF = WBM / 2;    // rows of the output tile staged at a time
constexpr size_t kSlabBytes = (size_t)2 * WBM * WLDS * 2;
constexpr size_t kWideLds = kSlabBytes + (size_t)WHALF * WLDO * 2 + WBM * 4; // two slabs, half an output tile, flow ids

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    union {
        bf16x2 b;
        uint32_t u;
    } c;
    c.b = __builtin_convertvector(v, bf16x2);
    return c.u;
}

template <int AMODE>
__global__ __launch_bounds__(WWAVES * 64) void mlp_wide_layer(LayerArgs a, const uint4* __restrict__ ws, uint32_t resident_min_rb)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* slab = reinterpret_cast<uint16_t*>(smem);                          // [2][128][WLDS]
    uint16_t* otile = reinterpret_cast<uint16_t*>(smem + kSlabBytes);            // [64][WLDO]
    uint32_t* s_flow = reinterpret_cast<uint32_t*>(smem + kSlabBytes + (size_t)WHALF * WLDO * 2); // [128]
    uint32_t total = *a.esc_count;
    total = total < a.esc_cap ? total : a.esc_cap;
    const uint32_t row0 = a.row_begin + blockIdx.x * WBM; // first escalated row of this block
    if (row0 >= total) return;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t nb_total = (a.N + 31u) / 32u;
    const uint32_t KS = (a.K + WSLAB - 1) / WSLAB * WRING; // k-steps, padded to whole slabs
    const uint32_t n_slabs = KS / WRING;
    // One column block per block (gridDim.y of them); or, when K fits the two slab buffers and the rows that
    // exist give every compute unit a row block of its own (resident_min_rb: 0 = never), the blocks of the
    // first column block walk all column blocks with the A operand resident, and the others leave.
    const uint32_t n_cb = gridDim.y;
    const uint32_t rb_count = (total - a.row_begin + WBM - 1u) / WBM; // (row0 < total, so total > row_begin)
    const bool resident = resident_min_rb != 0u && n_cb > 1u && rb_count >= resident_min_rb;
    if (resident && blockIdx.y != 0u) return;
    const uint32_t cb_first = resident ? 0u : blockIdx.y, cb_end = resident ? n_cb : blockIdx.y + 1u;

    if (AMODE != A_BF16) {
        if (tid < WBM) {
            uint32_t f = row0 + tid < total ? a.esc_idx[row0 + tid] : 0u;
            s_flow[tid] = f < a.n_rows ? f : a.n_rows - 1u; // a bad list entry must not leave the input
        }
        __syncthreads();
    }
    // two 16-byte chunks of the slab per thread: rows r, 8 k-values each
    const uint32_t cr[2] = {tid / (WSLAB / 8), (tid + WWAVES * 64) / (WSLAB / 8)};
    const uint32_t ck = (tid % (WSLAB / 8)) * 8u;
    // raw-bit input: where the two rows' flows start and how many packets they have, once (not per slab)
    uint32_t raw_b0[2] = {0u, 0u}, raw_n[2] = {0u, 0u};
    if (AMODE == A_RAW) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (row0 + cr[u] < total) raw_flow_range(a, s_flow[cr[u]], raw_b0[u], raw_n[u]); // (no packets: the row reads as zeros)
    }
    // slab sl of the A operand as this thread's two chunks
    auto fetch = [&](uint32_t sl, uint4 (&r)[2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (AMODE == A_RAW)
                r[u] = raw_chunk_at(a, raw_b0[u], raw_n[u], sl * WSLAB + ck);
            else
                r[u] = load_a_chunk<AMODE>(a, row0 + cr[u] < total, blockIdx.x * WBM + cr[u], AMODE != A_BF16 ? s_flow[cr[u]] : 0u,
                                           sl * WSLAB + ck);
        }
    };
    uint4 ra[2];
    for (uint32_t sl = 0; sl < (resident ? n_slabs : 1u); ++sl) {
        fetch(sl, ra);
#pragma unroll
        for (int u = 0; u < 2; ++u) *reinterpret_cast<uint4*>(slab + (sl & 1u) * (WBM * WLDS) + cr[u] * WLDS + ck) = ra[u];
    }

    // weight operands of a column block: a 32-column block past the end repeats the last one, its results are not
    // stored.  (A wave whose columns all lie past the end still runs the loop: a branch around the refills would
    // make the wait in front of the slab store, which is placed for the worst path, drain the whole ring once
    // per slab.)
    auto operands_of = [&](uint32_t cb, const uint4* (&w)[WNI]) {
#pragma unroll
        for (int j = 0; j < WNI; ++j) {
            const uint32_t nb = cb * (WBN / 32u) + wave * WNI + j;
            w[j] = ws + (size_t)(nb < nb_total ? nb : nb_total - 1u) * KS * 64u;
        }
    };
    const uint4* wl[WNI];
    operands_of(cb_first, wl);
    uint4 fb[WRING][WNI];
#pragma unroll
    for (int s = 0; s < WRING; ++s) {
#pragma unroll
        for (int j = 0; j < WNI; ++j) fb[s][j] = wl[j][s * 64 + lane];
        __builtin_amdgcn_sched_barrier(0); // ring order: keeps the counter waits inside the loop at "oldest load"
    }
    __syncthreads(); // slab 0 (resident: every slab) is in place

    for (uint32_t cb = cb_first; cb < cb_end; ++cb) {
        const uint32_t col0 = cb * WBN;
        const uint32_t nb0 = col0 / 32u + wave * WNI;
        // the ring goes on to the next column block's first k-steps (none: past the end, as within a block)
        const uint4* nwl[WNI];
        if (cb + 1u < cb_end) {
            operands_of(cb + 1u, nwl);
        } else {
#pragma unroll
            for (int j = 0; j < WNI; ++j) nwl[j] = wl[j] + (size_t)KS * 64u;
        }
        // accumulators start at the bias of their column
        f32x16 acc[WMI][WNI];
#pragma unroll
        for (int j = 0; j < WNI; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t col = (nb0 + j) * 32u + 8u * g + 4u * (lane >> 5);
                float b[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) b[q] = col + q < a.N ? a.bias[col + q] : 0.f;
#pragma unroll
                for (int i = 0; i < WMI; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[i][j][4 * g + q] = b[q];
            }

        for (uint32_t sl = 0; sl < n_slabs; ++sl) {
            const bool more = sl + 1 < n_slabs;
            if (more && !resident) fetch(sl + 1, ra);
            const uint4* src[WNI]; // this slab's refills: the next slab of the column block, or the next block's first
#pragma unroll
            for (int j = 0; j < WNI; ++j) src[j] = more ? wl[j] + (size_t)(sl + 1) * WRING * 64u : nwl[j];
            __builtin_amdgcn_sched_barrier(0);
            {
                const uint16_t* arow = slab + (sl & 1u) * (WBM * WLDS) + (lane & 31u) * WLDS + 8u * (lane >> 5);
#pragma unroll
                for (int s = 0; s < WRING; ++s) {
                    uint4 fa[WMI];
#pragma unroll
                    for (int i = 0; i < WMI; ++i) fa[i] = *reinterpret_cast<const uint4*>(arow + i * 32 * WLDS + s * 16);
#pragma unroll
                    for (int j = 0; j < WNI; ++j) {
                        const bf16x8 b = as_bf16x8(fb[s][j]);
#pragma unroll
                        for (int i = 0; i < WMI; ++i)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, as_bf16x8(fa[i]), acc[i][j], 0, 0, 0);
                    }
#pragma unroll
                    for (int j = 0; j < WNI; ++j) fb[s][j] = src[j][s * 64u + lane];
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (!resident) {
                if (more) {
#pragma unroll
                    for (int u = 0; u < 2; ++u)
                        *reinterpret_cast<uint4*>(slab + ((sl + 1) & 1u) * (WBM * WLDS) + cr[u] * WLDS + ck) = ra[u];
                }
                __syncthreads(); // the next slab is in place; nobody reads this one any more
            }
        }
#pragma unroll
        for (int j = 0; j < WNI; ++j) wl[j] = nwl[j];

        // epilogue: relu, bfloat16, stage 64 rows of the tile, then whole rows to memory
        // (a column block past the last real one holds a repeat of that block's results: stored as zeros)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int j = 0; j < WNI; ++j) {
                const bool real = nb0 + j < nb_total;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t cl = wave * 64u + j * 32u + 8u * g + 4u * (lane >> 5); // column inside the tile
#pragma unroll
                    for (int ih = 0; ih < WMI / 2; ++ih) {
                        const int i = half * (WMI / 2) + ih;
                        const uint32_t row = ih * 32u + (lane & 31u); // row inside the staged half
                        const float y0 = fmaxf(acc[i][j][4 * g + 0], 0.f), y1 = fmaxf(acc[i][j][4 * g + 1], 0.f);
                        const float y2 = fmaxf(acc[i][j][4 * g + 2], 0.f), y3 = fmaxf(acc[i][j][4 * g + 3], 0.f);
                        *reinterpret_cast<uint2*>(otile + row * WLDO + cl) =
                            real ? make_uint2(pack_bf16(y0, y1), pack_bf16(y2, y3)) : make_uint2(0u, 0u);
                    }
                }
            }
            __syncthreads();
            // 64 chunks of 8 columns per row; columns in [N, ldh) are padding and hold zeros
            for (uint32_t c = tid; c < WHALF * (WBN / 8); c += WWAVES * 64u) {
                const uint32_t rh = c / (WBN / 8), k = (c % (WBN / 8)) * 8u;
                const uint32_t r = half * WHALF + rh;
                if (row0 + r < total && col0 + k < a.ldh) {
                    const uint4 v = *reinterpret_cast<const uint4*>(otile + rh * WLDO + k);
                    uint16_t* dst = a.h_out + (size_t)(blockIdx.x * WBM + r) * a.ldh + col0 + k;
                    if (col0 + k + 8u <= a.ldh && (a.ldh & 7u) == 0) {
                        *reinterpret_cast<uint4*>(dst) = v;
                    } else {
                        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                        for (uint32_t q = 0; q < 8u && col0 + k + q < a.ldh; ++q) dst[q] = (uint16_t)(w[q >> 1] >> (16u * (q & 1u)));
                    }
                }
            }
            __syncthreads(); // the staged rows are out: the space may be written again
        }
    }
}

template <int AMODE>
int launch_wide(sf_ctx* ctx, const LayerArgs& a, const void* w_ordered, uint32_t rows_cap)
{
    SF_ALLOW_LDS(ctx, sf::kLdsWide + AMODE, mlp_wide_layer<AMODE>);
    // K up to two slabs: with enough rows, one block per 128 rows walks all column blocks (see the kernel)
    const uint32_t n_slabs = (a.K + WSLAB - 1) / WSLAB;
    const uint32_t resident_min_rb = n_slabs <= 2u ? (uint32_t)ctx->n_cu : 0u;
    dim3 grid((rows_cap + WBM - 1) / WBM, (a.ldh + WBN - 1) / WBN);
    mlp_wide_layer<AMODE><<<grid, WWAVES * 64, kWideLds, ctx->stream>>>(a, (const uint4*)w_ordered, resident_min_rb);
    SF_LAUNCH_CHECK(ctx, "mlp_wide_layer");
    return SF_OK;
}

} // namespace

namespace sf {

int wide_layer(sf_ctx* ctx, int amode, const sfmlp::LayerArgs& a, const void* w_ordered, uint32_t rows_cap)
{
    if (amode == A_BF16) return launch_wide<A_BF16>(ctx, a, w_ordered, rows_cap);
    if (amode == A_FEAT) return launch_wide<A_FEAT>(ctx, a, w_ordered, rows_cap);
    return launch_wide<A_RAW>(ctx, a, w_ordered, rows_cap);
}

} // namespace sf
