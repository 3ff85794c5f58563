// Step 5, fused form for hidden widths up to 512: the whole 3-layer MLP of a tile of 128
// escalated flows runs in one block without touching HBM between layers (Sections 3.1 and 4.4
// of the paper: only the uncertain flows reach the slow model, and its label replaces the fast
// one).
//
// A block is eight waves; wave w owns output columns [64w, 64w+64) of each hidden layer for
// all 128 rows, i.e. a 4x2 grid of 32x32 MFMA accumulators (128 accumulator registers).  The
// activations of the tile stay in shared memory ([128][520] bfloat16, 16-byte reads of 8
// consecutive rows fall on distinct banks); the weights are re-ordered once per call so that
// the 8 K-values a lane needs for an MFMA B operand are contiguous and a wave's operand is one
// contiguous kilobyte, and are then read straight from the cache into registers.  There is no
// barrier inside a layer's K loop.  The last layer (at most 32 classes) runs on all eight waves
// (four row blocks x two halves of K), followed by a per-row arg-max in registers and the
// scatter of the label.
// Blocks are persistent.  The rows that exist (the device-side escalation count) are cut into
// row blocks of 32 and dealt out evenly: every block gets a run of consecutive row blocks, the runs
// differ by at most one, and a block walks its run in tiles of four row blocks; what is left at
// the end of a run (one to three row blocks) is a last, lower tile (two row blocks high when that
// is enough), so the blocks finish together and few rows fill the whole device.
#include "mlp_common.h"

namespace sf {
bool slow_fused_ok(const sf_mlp* mlp, bool raw_input);
size_t slow_fused_ws_bytes(const sf_mlp* mlp);
int slow_fused(sf_ctx* ctx, void* ws, bool ws_is_ordered, const float* feat, uint32_t feat_ld, uint32_t n_rows,
               const uint32_t* esc_idx, const uint32_t* scatter, const uint32_t* esc_count, uint32_t esc_cap,
               uint32_t n_labels, const sf_mlp* mlp, float* logits, uint16_t* labels);
int order_all(sf_ctx* ctx, const sf_mlp* mlp, void* out);
} // namespace sf

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int FBM = 128;      // rows per tile
constexpr int HMAX = 512;     // widest hidden layer
constexpr int LDH = HMAX + 8; // activation row stride in elements
constexpr uint32_t kPadK = 64; // every K is padded to this (four k-steps of 16)

__host__ __device__ inline uint32_t up(uint32_t x, uint32_t m) { return (x + m - 1u) / m * m; }

struct FusedArgs {
    const uint32_t* esc_idx;  // row e reads feature row esc_idx[e] (clamped below n_rows) ...
    const uint32_t* scatter;  // ... and its label goes to labels[scatter[e]]; NULL = the same index
    const uint32_t* esc_count;
    uint32_t esc_cap;
    uint32_t n_rows, n_labels;
    const float* feat;
    uint32_t feat_ld;
    const float* mu;
    const float* inv_sigma;
    float clamp;
    uint32_t n_in, h1, h2, c;
    const uint4* w1s; // operand-ordered weights, see reorder_weights
    const uint4* w2s;
    const uint4* w3s;
    const float *b1, *b2, *b3;
    float* logits;
    uint16_t* labels;
};

__device__ __forceinline__ uint16_t to_bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16);
    u += 0x7FFFu + ((u >> 16) & 1u); // round to nearest even
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ bf16x8 as_frag(uint4 u)
{
    union {
        uint4 u;
        bf16x8 b;
    } c;
    c.u = u;
    return c.b;
}

// W[N][K] (row-major, bfloat16 bits) -> out[(nb * KS + ks) * 64 + lane] = the 8 values
// W[nb*32 + lane%32][ks*16 + 8*(lane/32) .. +8), zero outside; nb < NB, ks < KS.
// One launch re-orders all three layers.
struct ReorderJob {
    const uint16_t* w;
    uint32_t N, K, NB, KS;
    uint32_t first; // index of the job's first 16-byte element in the launch-wide numbering
    uint4* out;
};
struct ReorderArgs {
    ReorderJob job[3];
    uint32_t total;
};

__global__ __launch_bounds__(256) void reorder_weights(ReorderArgs r)
{
    for (uint32_t e = blockIdx.x * blockDim.x + threadIdx.x; e < r.total; e += gridDim.x * blockDim.x) {
        const int ji = e >= r.job[2].first ? 2 : (e >= r.job[1].first ? 1 : 0);
        const ReorderJob& jb = r.job[ji];
        const uint32_t g = e - jb.first;
        const uint32_t lane = g & 63u, t = g >> 6, ks = t % jb.KS, nb = t / jb.KS;
        const uint32_t n = nb * 32u + (lane & 31u), k0 = ks * 16u + 8u * (lane >> 5);
        uint16_t v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = (n < jb.N && k0 + q < jb.K) ? jb.w[(size_t)n * jb.K + k0 + q] : (uint16_t)0;
        jb.out[g] = make_uint4(v[0] | ((uint32_t)v[1] << 16), v[2] | ((uint32_t)v[3] << 16), v[4] | ((uint32_t)v[5] << 16),
                               v[6] | ((uint32_t)v[7] << 16));
    }
}

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// two floats -> two bfloat16 (round to nearest even) in one word
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

constexpr int kWaves = 8;  // waves per block
constexpr int kNI = 2;     // 32-column blocks per wave (64 columns)
constexpr int kMI = 4;     // 32-row blocks per wave in a full tile (all 128 rows)
constexpr int kRing = 4;   // weight operands of this many k-steps are in flight (K is padded to 16 * kRing)

// first kRing k-steps of a wave's weight operands (column blocks nb0 .. nb0+kNI, clamped to the last real one)
__device__ __forceinline__ void ring_fill(uint4 (&fb)[kRing][kNI], const uint4* __restrict__ ws, uint32_t KS, uint32_t nb0,
                                          uint32_t nb_total, uint32_t lane)
{
#pragma unroll
    for (int s = 0; s < kRing; ++s) {
#pragma unroll
        for (int j = 0; j < kNI; ++j) {
            const uint32_t nb = nb0 + j < nb_total ? nb0 + j : nb_total - 1u;
            fb[s][j] = ws[((size_t)nb * KS + s) * 64u + lane];
        }
        // ring order: the counter wait in front of an MFMA is placed for the worst order on any path
        // into the loop, and a fill issued out of order makes every k-step wait for the newest load
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The MFMA is issued with the WEIGHT operand first, so the 32x32 accumulator block holds the
// output transposed: element v of lane l is output column 8*(v/4) + 4*(l/32) + v%4 of
// activation row l%32.  Four consecutive v are four consecutive columns of one row, which lets
// the epilogue write 8 bytes at a time.
// acc[i][j] += W[cols of block nb0+j][K] * A[rows 32i..32i+32)[K]^T, KS a multiple of kRing.
// The weight operands sit in a ring of kRing register buffers; a buffer is refilled for k-step
// ks + kRing right after the MFMAs of k-step ks have been issued, so no load is waited for in the
// step that issues it and no register is copied.
// fb holds k-steps 0 .. kRing-1 of this layer on entry.  The last kRing refills of the loop fetch the
// first k-steps of the NEXT GEMM (operand array nws, nKS k-steps per column block, nnb_total column
// blocks), so that one starts without waiting for memory: its operands arrive during the epilogue
// in between.
template <int MI>
__device__ __forceinline__ void wave_gemm(const uint16_t* A, uint32_t lda, const uint4* __restrict__ ws, uint32_t KS,
                                          uint32_t nb0, uint32_t nb_total, uint32_t lane, f32x16 (&acc)[MI][kNI],
                                          uint4 (&fb)[kRing][kNI], const uint4* __restrict__ nws, uint32_t nKS,
                                          uint32_t nnb_total)
{
    if (nb0 >= nb_total) { // this wave has no columns in this layer
        ring_fill(fb, nws, nKS, nb0, nnb_total, lane);
        return;
    }
    const uint16_t* arow = A + (lane & 31u) * lda + 8u * (lane >> 5);
    // a column block past the end repeats the last one; its results are never used
    const uint4 *wl[kNI], *nwl[kNI];
#pragma unroll
    for (int j = 0; j < kNI; ++j) {
        const uint32_t nb = nb0 + j < nb_total ? nb0 + j : nb_total - 1u;
        wl[j] = ws + (size_t)nb * KS * 64u;
        const uint32_t nnb = nb0 + j < nnb_total ? nb0 + j : nnb_total - 1u;
        nwl[j] = nws + (size_t)nnb * nKS * 64u;
    }
    // the activation operands are double-buffered too: those of k-step ks+1 are read from shared
    // memory before the MFMAs of k-step ks are issued (H has 8 columns of padding, so the read
    // one step past the end stays inside the row)
    uint4 fa[2][MI];
#pragma unroll
    for (int i = 0; i < MI; ++i) fa[0][i] = *reinterpret_cast<const uint4*>(arow + (size_t)i * 32u * lda);
    for (uint32_t k0 = 0; k0 < KS; k0 += kRing) {
        // where this round's refills come from: further down this layer, or the start of the next
        // GEMM (a select between wave-uniform pointers: no branch around the loads, which would
        // make the counter waits drain the ring)
        const bool more = k0 + kRing < KS;
        const uint4* src[kNI];
#pragma unroll
        for (int j = 0; j < kNI; ++j) src[j] = more ? wl[j] + (size_t)(k0 + kRing) * 64u : nwl[j];
#pragma unroll
        for (int s = 0; s < kRing; ++s) {
            const uint32_t kn = k0 + s + 1u < KS ? k0 + s + 1u : k0 + s;
#pragma unroll
            for (int i = 0; i < MI; ++i)
                fa[(s + 1) & 1][i] = *reinterpret_cast<const uint4*>(arow + (size_t)i * 32u * lda + kn * 16u);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < kNI; ++j) {
                const bf16x8 b = as_frag(fb[s][j]);
#pragma unroll
                for (int i = 0; i < MI; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, as_frag(fa[s & 1][i]), acc[i][j], 0, 0, 0);
            }
            // refill for k-step k0 + s + kRing (or k-step s of the next GEMM)
#pragma unroll
            for (int j = 0; j < kNI; ++j) fb[s][j] = src[j][s * 64u + lane];
            // keep the refill here: left alone, the scheduler sinks it to just before its use
            // (to save registers) and every k-step then waits a full memory latency
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// H[row][col] = bfloat16(relu(acc)) for the wave's columns (the bias is already in acc).  Padding columns
// [n_valid, n_pad) inside the last real 32-column block come out as zeros by themselves (their weights and
// bias entries are zero); a column block past the last real one (nb_total) holds a repeat of that block's
// results in acc and is stored as zeros.
template <int MI>
__device__ __forceinline__ void store_hidden(uint16_t* H, const f32x16 (&acc)[MI][kNI], uint32_t n0, uint32_t n_pad,
                                             uint32_t nb_total, uint32_t lane)
{
#pragma unroll
    for (int j = 0; j < kNI; ++j) {
        const bool real = n0 / 32u + j < nb_total;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t col = n0 + j * 32u + 8u * g + 4u * (lane >> 5); // first of 4 consecutive columns
            if (col < n_pad) {
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const uint32_t row = i * 32u + (lane & 31u);
                    const float y0 = fmaxf(acc[i][j][4 * g + 0], 0.f), y1 = fmaxf(acc[i][j][4 * g + 1], 0.f);
                    const float y2 = fmaxf(acc[i][j][4 * g + 2], 0.f), y3 = fmaxf(acc[i][j][4 * g + 3], 0.f);
                    *reinterpret_cast<uint2*>(H + row * LDH + col) =
                        real ? make_uint2(pack_bf16(y0, y1), pack_bf16(y2, y3)) : make_uint2(0u, 0u);
                }
            }
        }
    }
}

// accumulators start at the bias of their column (element v of lane l is column
// 8*(v/4) + 4*(l/32) + v%4 of the 32-column block), so the epilogue has no add
template <int MI>
__device__ __forceinline__ void bias_acc(f32x16 (&acc)[MI][kNI], const float* sbias, uint32_t n0, uint32_t lane)
{
#pragma unroll
    for (int j = 0; j < kNI; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t col = n0 + j * 32u + 8u * g + 4u * (lane >> 5);
            const float4 b = col < (uint32_t)HMAX ? *reinterpret_cast<const float4*>(sbias + col) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                acc[i][j][4 * g + 0] = b.x;
                acc[i][j][4 * g + 1] = b.y;
                acc[i][j][4 * g + 2] = b.z;
                acc[i][j][4 * g + 3] = b.w;
            }
        }
}

constexpr uint32_t kNoFlow = 0xFFFFFFFFu;
// a bad list entry must not leave the feature matrix
__device__ __forceinline__ uint32_t clamp_row(uint32_t f, uint32_t n_rows) { return f < n_rows ? f : n_rows - 1u; }
constexpr int kXr = 2; // 8-value input chunks a thread can hold in registers for the next tile

// raw feature values [k, k+8) of one flow (zeros for a missing flow or past n_in)
__device__ __forceinline__ void load_chunk(const FusedArgs& a, uint32_t flow, uint32_t k, float (&z)[8])
{
#pragma unroll
    for (int q = 0; q < 8; ++q) z[q] = 0.f;
    if (flow == kNoFlow) return;
    const float* p = a.feat + (size_t)flow * a.feat_ld + k;
    if (k + 8u <= a.n_in && (a.feat_ld & 3u) == 0 && (reinterpret_cast<uintptr_t>(a.feat) & 15u) == 0) {
        const float4 x0 = reinterpret_cast<const float4*>(p)[0], x1 = reinterpret_cast<const float4*>(p)[1];
        z[0] = x0.x; z[1] = x0.y; z[2] = x0.z; z[3] = x0.w;
        z[4] = x1.x; z[5] = x1.y; z[6] = x1.z; z[7] = x1.w;
    } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) z[q] = k + q < a.n_in ? p[q] : 0.f;
    }
}

// standardise, clamp, round to bfloat16 and store one chunk of the input tile
// (s_mu / s_is: the input map in shared memory, zero / one past n_in; has_map false = identity)
__device__ __forceinline__ void store_chunk(bool has_map, const float* s_mu, const float* s_is, float clamp,
                                            uint16_t* dst, uint32_t k, float (&z)[8])
{
    if (has_map) {
        const float4 m0 = *reinterpret_cast<const float4*>(s_mu + k), m1 = *reinterpret_cast<const float4*>(s_mu + k + 4);
        const float4 i0 = *reinterpret_cast<const float4*>(s_is + k), i1 = *reinterpret_cast<const float4*>(s_is + k + 4);
        const float mu[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
        const float is[8] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const float d = z[q] - mu[q];
            float t = d * is[q];
            t = t < -clamp ? -clamp : t;
            z[q] = t > clamp ? clamp : t;
        }
    }
    *reinterpret_cast<uint4*>(dst) =
        make_uint4(pack_bf16(z[0], z[1]), pack_bf16(z[2], z[3]), pack_bf16(z[4], z[5]), pack_bf16(z[6], z[7]));
}

// Tile schedule of run_tiles (one block, eight waves, n_tiles consecutive tiles of MI row blocks):
//   top        the input tile is written from registers that were loaded during the previous
//              tile's last layer; the flow ids of the NEXT tile are requested
//   layer 1    MFMA, then the next tile's flow ids are parked in shared memory, epilogue -> H
//   layer 2    MFMA, epilogue -> H; the last layer's weight operands are requested
//   layer 3    the next tile's feature rows are requested (they arrive while layer 3 runs);
//              8 waves = MI row blocks x 2 halves of K (waves beyond that idle); halves are
//              summed through shared memory
// Rows from row_end on belong to another block (or do not exist): they read as zeros and nothing of
// theirs is stored.
struct FusedSmem {
    uint16_t* H;      // [128][LDH]; also the input tile
    uint32_t* s_flow; // [2][128]: this tile, next tile
    float *s_b1, *s_b2, *s_b3, *s_part, *s_mu, *s_is;
};

template <int MI>
__device__ __forceinline__ void run_tiles(const FusedArgs& a, const FusedSmem& m, uint32_t wave, uint32_t row_begin,
                                          uint32_t n_tiles, uint32_t row_end)
{
    constexpr uint32_t TM = MI * 32u; // rows per tile
    uint16_t* H = m.H;
    uint32_t* s_flow = m.s_flow;
    const uint32_t k1p = up(a.n_in, kPadK), k2p = up(a.h1, kPadK), k3p = up(a.h2, kPadK);
    const uint32_t ldx = k1p + 8; // input tile row stride
    const uint32_t n0 = wave * 32u * kNI;
    const uint32_t nb1 = up(a.h1, 32) / 32u, nb2 = up(a.h2, 32) / 32u;
    const uint32_t chunks = k1p / 8u;
    const bool in_regs = TM * chunks <= (uint32_t)kXr * kWaves * 64u; // the whole input tile fits the threads' registers
    const bool has_map = a.mu != nullptr;
    float xr[kXr][8];
    __syncthreads(); // the previous run of tiles (if any) is done with the tile and the flow ids
    {
        // first tile: flow ids and feature rows are fetched here, with nothing to overlap them
        // (the lane index behind an opaque barrier, as in the loop: nothing computed from it here is shared
        // with, and kept alive across, another run of tiles)
        uint32_t tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        if (tid < TM) s_flow[tid] = row_begin + tid < row_end ? clamp_row(a.esc_idx[row_begin + tid], a.n_rows) : kNoFlow;
        __syncthreads();
        if (in_regs) {
#pragma unroll
            for (int u = 0; u < kXr; ++u) {
                const uint32_t g = tid + u * kWaves * 64u, r = g / chunks, k = (g - r * chunks) * 8u;
                load_chunk(a, r < TM ? s_flow[r] : kNoFlow, k, xr[u]);
            }
        }
    }
    // weight operands of layer 1's first k-steps; from here on every GEMM leaves the ring filled for the next one
    uint4 fb[kRing][kNI];
    ring_fill(fb, a.w1s, k1p / 16u, wave * kNI, nb1, threadIdx.x & 63u);
    uint32_t cur = 0;
    for (uint32_t ti = 0; ti < n_tiles; ++ti) {
        const uint32_t row0 = row_begin + ti * TM;
        const uint32_t next_row0 = row0 + TM;
        const bool has_next = ti + 1u < n_tiles;
        // Re-read the lane index behind an opaque barrier in every tile: otherwise every per-lane
        // address of the tile body is hoisted out of this loop and spilled around the MFMA loops.
        uint32_t tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const uint32_t lane = tid & 63u;
        const uint32_t* flow_cur = s_flow + cur * FBM;
        uint32_t* flow_next = s_flow + (cur ^ 1u) * FBM;
        // flow ids of the next tile: requested now, parked in shared memory after layer 1
        uint32_t nf = kNoFlow;
        if (has_next && tid < TM && next_row0 + tid < row_end) nf = clamp_row(a.esc_idx[next_row0 + tid], a.n_rows);
        // input tile of this tile (H is free: the previous tile's last layer ended with a barrier)
        if (in_regs) {
#pragma unroll
            for (int u = 0; u < kXr; ++u) {
                const uint32_t g = tid + u * kWaves * 64u, r = g / chunks, k = (g - r * chunks) * 8u;
                if (r < TM) store_chunk(has_map, m.s_mu, m.s_is, a.clamp, H + r * ldx + k, k, xr[u]);
            }
        } else {
            for (uint32_t g = tid; g < TM * chunks; g += kWaves * 64u) {
                const uint32_t r = g / chunks, k = (g - r * chunks) * 8u;
                float z[8];
                load_chunk(a, flow_cur[r], k, z);
                store_chunk(has_map, m.s_mu, m.s_is, a.clamp, H + r * ldx + k, k, z);
            }
        }
        __syncthreads();

        f32x16 acc[MI][kNI];
        // layer 1
        bias_acc<MI>(acc, m.s_b1, n0, lane);
        wave_gemm<MI>(H, ldx, a.w1s, k1p / 16u, wave * kNI, nb1, lane, acc, fb, a.w2s, k2p / 16u, nb2);
        __syncthreads(); // every wave has read the input tile; H may be overwritten
        if (tid < TM) flow_next[tid] = nf;
        store_hidden<MI>(H, acc, n0, k2p, nb1, lane);
        __syncthreads();
        // layer 2
        bias_acc<MI>(acc, m.s_b2, n0, lane);
        // (the ring goes on to layer 1 of the next tile; after the last tile the fetch is not used)
        wave_gemm<MI>(H, LDH, a.w2s, k2p / 16u, wave * kNI, nb2, lane, acc, fb, a.w1s, k1p / 16u, nb1);
        __syncthreads();
        store_hidden<MI>(H, acc, n0, k3p, nb2, lane);
        // layer 3: wave = (row block rb, half kh of K); waves beyond MI x 2 only keep the barriers.  The hidden
        // accumulators are dead, so a whole half-layer of weight operands fits in registers; they are requested
        // before the barrier so that their latency overlaps it.
        const uint32_t rb = wave % (uint32_t)MI, kh = wave / (uint32_t)MI;
        const bool l3 = MI == kMI ? true : kh < 2u; // (eight waves: with four row blocks every wave has a share)
        const uint32_t KS3 = k3p / 16u, khalf = KS3 / 2u, kbeg = (l3 ? kh : 0u) * khalf; // KS3 is a multiple of 4
        uint4 wv[16];
        if (l3) {
#pragma unroll
            for (int s3 = 0; s3 < 16; ++s3)
                wv[s3] = a.w3s[(size_t)(kbeg + ((uint32_t)s3 < khalf ? (uint32_t)s3 : khalf - 1u)) * 64u + lane];
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        // the next tile's feature rows: requested now, consumed at the top of the next iteration
        if (has_next && in_regs) {
#pragma unroll
            for (int u = 0; u < kXr; ++u) {
                const uint32_t g = tid + u * kWaves * 64u, r = g / chunks, k = (g - r * chunks) * 8u;
                load_chunk(a, r < TM ? flow_next[r] : kNoFlow, k, xr[u]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        {
            f32x16 c3, c3b;
#pragma unroll
            for (int v = 0; v < 16; ++v) c3[v] = c3b[v] = 0.f;
            const uint16_t* arow = H + (rb * 32u + (lane & 31u)) * LDH + 8u * (lane >> 5);
            if (l3) {
                for (uint32_t kb = 0; kb < khalf; kb += 16u) {
                    if (kb) {
#pragma unroll
                        for (int s3 = 0; s3 < 16; ++s3)
                            wv[s3] = a.w3s[(size_t)(kbeg + (kb + s3 < khalf ? kb + s3 : khalf - 1u)) * 64u + lane];
                    }
#pragma unroll
                    for (int s3 = 0; s3 < 16; s3 += 2) {
                        if (kb + s3 < khalf)
                            c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                as_frag(wv[s3]), as_frag(*reinterpret_cast<const uint4*>(arow + (kbeg + kb + s3) * 16u)), c3, 0, 0, 0);
                        if (kb + s3 + 1 < khalf)
                            c3b = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                as_frag(wv[s3 + 1]), as_frag(*reinterpret_cast<const uint4*>(arow + (kbeg + kb + s3 + 1) * 16u)), c3b, 0, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) c3[v] += c3b[v];
            float* part = m.s_part + rb * (16 * 64);
            if (l3 && kh == 1u) {
#pragma unroll
                for (int v = 0; v < 16; ++v) part[v * 64 + lane] = c3[v];
            }
            __syncthreads(); // also: every wave is done reading H
            if (l3 && kh == 0u) {
                // the accumulator is transposed: lane l holds 16 classes of row l%32, lane l^32 the others
                const uint32_t r = rb * 32u + (lane & 31u);
                const bool row_ok = row0 + r < row_end;
                uint32_t best = kNoFlow;
                float bv = 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const uint32_t c = 8u * (v >> 2) + 4u * (lane >> 5) + (v & 3); // ascending in v
                    if (c < a.c) {
                        const float y = c3[v] + part[v * 64 + lane] + m.s_b3[c];
                        if (a.logits && row_ok) a.logits[(size_t)(row0 + r) * a.c + c] = y;
                        if (best == kNoFlow || y > bv) {
                            bv = y;
                            best = c;
                        }
                    }
                }
                // combine the two halves of the row: larger value wins, the lower class on a tie
                const float ov = __shfl_xor(bv, 32, 64);
                const uint32_t ob = (uint32_t)__shfl_xor((int)best, 32, 64);
                if (ob != kNoFlow && (best == kNoFlow || ov > bv || (ov == bv && ob < best))) best = ob;
                if (lane < 32u && row_ok) {
                    const uint32_t dst = a.scatter ? a.scatter[row0 + r] : flow_cur[r];
                    if (dst < a.n_labels) a.labels[dst] = (uint16_t)best;
                }
            }
        }
        cur ^= 1u;
    }
}

__global__ __launch_bounds__(kWaves * 64) void mlp_fused(FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    FusedSmem m;
    m.H = reinterpret_cast<uint16_t*>(smem);                                    // [128][LDH]; also the input tile
    m.s_flow = reinterpret_cast<uint32_t*>(smem + (size_t)FBM * LDH * 2);       // [2][128]: this tile, next tile
    m.s_b1 = reinterpret_cast<float*>(m.s_flow + 2 * FBM);                      // [HMAX], zero past h1
    m.s_b2 = m.s_b1 + HMAX;                                                     // [HMAX], zero past h2
    m.s_b3 = m.s_b2 + HMAX;                                                     // [32], zero past c
    m.s_part = m.s_b3 + 32;                                                     // [4][16][64] last-layer partial sums
    m.s_mu = m.s_part + 4 * 16 * 64;                                            // [HMAX] input map (0 / 1 if none)
    m.s_is = m.s_mu + HMAX;                                                     // [HMAX]
    // the wave index is the same in every lane: say so, and everything derived from it (column
    // block, weight pointers) lives in scalar registers
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t total = *a.esc_count;
    total = total < a.esc_cap ? total : a.esc_cap;
    // this block's run of row blocks: the runs of the grid differ by at most one row block
    const uint32_t rb_total = (total + 31u) / 32u;
    const uint32_t rb_lo = rb_total / gridDim.x, rb_rem = rb_total % gridDim.x;
    const uint32_t rb_first = blockIdx.x * rb_lo + (blockIdx.x < rb_rem ? blockIdx.x : rb_rem);
    const uint32_t rb_count = rb_lo + (blockIdx.x < rb_rem ? 1u : 0u);
    if (rb_count == 0) return;
    const uint32_t row_begin = rb_first * 32u;
    uint32_t row_end = (rb_first + rb_count) * 32u;
    row_end = row_end < total ? row_end : total;

    for (uint32_t q = threadIdx.x; q < (uint32_t)HMAX; q += kWaves * 64u) {
        m.s_b1[q] = q < a.h1 ? a.b1[q] : 0.f;
        m.s_b2[q] = q < a.h2 ? a.b2[q] : 0.f;
        if (q < 32u) m.s_b3[q] = q < a.c ? a.b3[q] : 0.f;
        m.s_mu[q] = (a.mu && q < a.n_in) ? a.mu[q] : 0.f;
        m.s_is[q] = (a.mu && q < a.n_in) ? a.inv_sigma[q] : 1.f;
    }
    // full tiles of four row blocks, then what is left: three row blocks run as a (masked) full tile, one or
    // two as a tile of half the height
    const uint32_t rest = rb_count % (uint32_t)kMI;
    const uint32_t n_full = rb_count / (uint32_t)kMI + (rest == 3u ? 1u : 0u);
    if (n_full) run_tiles<kMI>(a, m, wave, row_begin, n_full, row_end);
    if (rest == 1u || rest == 2u) run_tiles<2>(a, m, wave, row_begin + n_full * FBM, 1u, row_end);
}

constexpr size_t kFusedLds = (size_t)FBM * LDH * 2 + 2 * FBM * 4 + (4 * HMAX + 32) * 4 + 4 * 16 * 64 * 4;

} // namespace

namespace sf {

bool slow_fused_ok(const sf_mlp* m, bool raw_input)
{
    return m->dtype == SF_BF16 && !raw_input && m->n_in <= HMAX && m->n_h1 <= HMAX && m->n_h2 <= HMAX && m->n_classes <= 32;
}

// the kernel reads kRing k-steps past the end of a column block: keep that much padding behind the last one
static size_t sw_bytes(uint32_t N, uint32_t K) { return align_up((size_t)(up(N, 32) / 32) * (up(K, kPadK) / 16) * 64 * 16 + (size_t)kRing * 1024); }

size_t slow_fused_ws_bytes(const sf_mlp* m)
{
    return sw_bytes(m->n_h1, m->n_in) + sw_bytes(m->n_h2, m->n_h1) + sw_bytes(32, m->n_h2) + 3 * kAlign;
}

size_t reordered_bytes(uint32_t N, uint32_t K) { return sw_bytes(N, K); }

int reorder_weights_async(sf_ctx* ctx, const ReorderSpec* specs, int n_specs)
{
    if (n_specs < 1 || n_specs > 3) return fail(ctx, SF_EINVAL, "reorder_weights_async: 1..3 matrices per launch");
    ReorderArgs r;
    r.total = 0;
    for (int q = 0; q < 3; ++q) {
        const ReorderSpec& sp = specs[q < n_specs ? q : n_specs - 1];
        r.job[q].w = (const uint16_t*)sp.w;
        r.job[q].N = sp.N;
        r.job[q].K = sp.K;
        r.job[q].NB = up(sp.N, 32) / 32;
        r.job[q].KS = up(sp.K, kPadK) / 16;
        r.job[q].first = r.total;
        r.job[q].out = (uint4*)sp.out;
        if (q < n_specs) r.total += r.job[q].NB * r.job[q].KS * 64;
    }
    // jobs past n_specs start at r.total, so no element maps to them
    uint32_t blocks = (r.total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    reorder_weights<<<blocks, 256, 0, ctx->stream>>>(r);
    SF_LAUNCH_CHECK(ctx, "reorder_weights");
    return SF_OK;
}

// w1 | w2 | w3 in operand order, at the offsets every consumer uses (the last layer padded to 32 columns)
int order_all(sf_ctx* ctx, const sf_mlp* m, void* out)
{
    char* p = (char*)out;
    uint4* w1s = (uint4*)p;
    p += sw_bytes(m->n_h1, m->n_in);
    uint4* w2s = (uint4*)p;
    p += sw_bytes(m->n_h2, m->n_h1);
    uint4* w3s = (uint4*)p;
    const ReorderSpec specs[3] = {{m->w1, m->n_h1, m->n_in, w1s}, {m->w2, m->n_h2, m->n_h1, w2s},
                                  {m->w3, m->n_classes, m->n_h2, w3s}};
    return reorder_weights_async(ctx, specs, 3);
}

int slow_fused(sf_ctx* ctx, void* ws, bool ws_is_ordered, const float* feat, uint32_t feat_ld, uint32_t n_rows,
               const uint32_t* esc_idx, const uint32_t* scatter, const uint32_t* esc_count, uint32_t esc_cap,
               uint32_t n_labels, const sf_mlp* m, float* logits, uint16_t* labels)
{
    char* p = (char*)ws;
    uint4* w1s = (uint4*)p;
    p += sw_bytes(m->n_h1, m->n_in);
    uint4* w2s = (uint4*)p;
    p += sw_bytes(m->n_h2, m->n_h1);
    uint4* w3s = (uint4*)p;
    if (!ws_is_ordered) {
        const int rc = order_all(ctx, m, ws);
        if (rc != SF_OK) return rc;
    }
    FusedArgs a;
    a.esc_idx = esc_idx;
    a.scatter = scatter;
    a.esc_count = esc_count;
    a.esc_cap = esc_cap;
    a.n_rows = n_rows;
    a.n_labels = n_labels;
    a.feat = feat;
    a.feat_ld = feat_ld;
    a.mu = m->mu;
    a.inv_sigma = m->inv_sigma;
    a.clamp = m->clamp;
    a.n_in = m->n_in;
    a.h1 = m->n_h1;
    a.h2 = m->n_h2;
    a.c = m->n_classes;
    a.w1s = w1s;
    a.w2s = w2s;
    a.w3s = w3s;
    a.b1 = m->b1;
    a.b2 = m->b2;
    a.b3 = m->b3;
    a.logits = logits;
    a.labels = labels;
    SF_ALLOW_LDS(ctx, sf::kLdsFused, mlp_fused);
    const uint32_t rb_cap = (esc_cap + 31u) / 32u;
    uint32_t grid = (uint32_t)ctx->n_cu; // one block per compute unit (its shared memory fills the unit)
    if (grid > rb_cap) grid = rb_cap;
    if (grid == 0) grid = 1;
    mlp_fused<<<grid, kWaves * 64, kFusedLds, ctx->stream>>>(a);
    SF_LAUNCH_CHECK(ctx, "mlp_fused");
    return SF_OK;
}

} // namespace sf
