// The two queues in front of the slow model as device hash tables (Section 3.1 of the paper:
// queue 3 carries the flows the fast model hands on, queue 2 the features of their later
// packets, both keyed by flow ID; the slow model takes a flow when both are there; a record
// that finds no partner in the other queue is discarded after a timeout).
//
// One open-addressing table per side (linear probing, 16-byte slots: flow ID, value, stamp).
// A step first drops what has waited too long and packs the survivors (collect -> clear ->
// re-insert, so probe chains never carry deleted slots from one step to the next), then takes
// the arrivals of queue 3 (look up the other side's table: found -> emit the pair and remove it;
// not found -> insert on the own side), then those of queue 2 the same way.  The two sides run
// in separate launches, so a launch only ever removes from one table and inserts into the
// other; a record of one side therefore never meets a half-written record of the other.
// Every probe loop is bounded by the table size.
#include "common.h"

namespace sf {
size_t join_scratch_bytes(uint32_t cap_log2);
}

namespace {

constexpr unsigned long long kEmpty = 0ull;
constexpr unsigned long long kGone = ~0ull; // removed during this step; cleared by the next step's repack

struct Slot {
    unsigned long long id;
    uint32_t val;
    uint32_t stamp;
};

// stats words: 0 discarded after the timeout, 1 records that could not be stored (table full),
// 2 records whose flow ID was already waiting on their own side, 3 pairs that did not fit pair_cap
enum { kExpired = 0, kDropped = 1, kDuplicate = 2, kPairOverflow = 3 };

__device__ __forceinline__ uint32_t slot_of(unsigned long long id, uint32_t mask)
{
    // 64-bit finaliser (xor-shift-multiply), then the low bits
    id ^= id >> 33;
    id *= 0xff51afd7ed558ccdull;
    id ^= id >> 33;
    id *= 0xc4ceb9fe1a85ec53ull;
    id ^= id >> 33;
    return (uint32_t)id & mask;
}

// One atomic per wave instead of one per lane: the lanes for which want is set get consecutive positions
// base .. base + count - 1 (base from a single atomicAdd by the first of them).  All lanes that are active at
// the call take part; the result is meaningful only where want is set.
__device__ __forceinline__ uint32_t wave_claim(uint32_t* counter, bool want)
{
    const unsigned long long m = __ballot(want);
    if (m == 0) return 0;
    const uint32_t lane = threadIdx.x & 63u;
    const int leader = __ffsll((long long)m) - 1;
    uint32_t base = 0;
    if ((int)lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
    base = (uint32_t)__shfl((int)base, leader, 64);
    return base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}

__device__ __forceinline__ void wave_count(uint32_t* counter, bool want)
{
    const unsigned long long m = __ballot(want);
    if (m && (int)(threadIdx.x & 63u) == __ffsll((long long)m) - 1) atomicAdd(counter, (uint32_t)__popcll(m));
}

struct JoinArgs {
    Slot* table[2]; // [0] queue 3, [1] queue 2
    uint32_t* used[2]; // per side, one word per kChunk slots: non-zero once a record was stored there since the last sweep
    uint32_t mask;  // slots per table - 1
    uint32_t now, timeout;
    Slot* list;     // scratch: survivors, side s in list[s * slots ...]
    uint32_t* counters; // scratch: [0] survivors of side 0, [1] survivors of side 1
    uint32_t* n_pairs;
    uint32_t* pair_q3;
    uint32_t* pair_q2;
    uint32_t pair_cap;
    uint32_t* stats;
};

__global__ void join_zero(uint32_t* counters, uint32_t* n_pairs, uint32_t* stats)
{
    if (threadIdx.x < 2) counters[threadIdx.x] = 0;
    if (threadIdx.x == 2) *n_pairs = 0;
    if (stats && threadIdx.x >= 4 && threadIdx.x < 8) stats[threadIdx.x - 4] = 0;
}

// survivors of both tables -> list (side s occupies list[s * slots ...]); every slot is cleared.
// A wave takes kChunk consecutive slots of one side per trip and claims the list positions of all its
// survivors with ONE atomic (a counter that every wave of the grid adds to is the bottleneck otherwise:
// same-address atomics retire a few nanoseconds apart).
constexpr uint32_t kChunkTrips = 16;             // slots per lane per trip
constexpr uint32_t kChunk = 64u * kChunkTrips;   // slots per wave per trip

__global__ __launch_bounds__(256) void join_collect(JoinArgs a)
{
    const uint32_t slots = a.mask + 1u;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, n_waves = (gridDim.x * blockDim.x) >> 6;
    const uint32_t chunks_per_side = (slots + kChunk - 1u) / kChunk;
    for (uint32_t c = wave; c < 2u * chunks_per_side; c += n_waves) {
        const uint32_t side = c >= chunks_per_side ? 1u : 0u;
        const uint32_t first = (c - side * chunks_per_side) * kChunk;
        // nothing was stored in this stretch since it was last swept: every slot is still empty
        uint32_t* used = a.used[side] + (c - side * chunks_per_side);
        if (*used == 0u) continue; // the same word in every lane: the wave skips together
        if (lane == 0) *used = 0u; // the sweep below empties the stretch (the re-insert marks what it refills)
        Slot* t = a.table[side];
        // pass 1: who survives (one 64-bit lane mask per trip, the same in every lane)
        unsigned long long keep[kChunkTrips];
        uint32_t n_keep = 0, n_old = 0;
#pragma unroll
        for (uint32_t j = 0; j < kChunkTrips; ++j) {
            const uint32_t q = first + j * 64u + lane;
            bool live = false, old = false;
            if (q < slots) {
                const Slot v = t[q];
                live = v.id != kEmpty && v.id != kGone;
                old = live && (a.now - v.stamp > a.timeout); // unsigned: wraps like the tick counter
            }
            keep[j] = __ballot(live && !old);
            n_keep += (uint32_t)__popcll(keep[j]);
            n_old += (uint32_t)__popcll(__ballot(old));
        }
        uint32_t base = 0;
        if (lane == 0) {
            if (n_keep) base = atomicAdd(&a.counters[side], n_keep);
            if (n_old && a.stats) atomicAdd(&a.stats[kExpired], n_old);
        }
        base = (uint32_t)__shfl((int)base, 0, 64);
        // pass 2: move the survivors, clear every used slot
#pragma unroll
        for (uint32_t j = 0; j < kChunkTrips; ++j) {
            const uint32_t q = first + j * 64u + lane;
            if (q < slots) {
                const Slot v = t[q];
                if (v.id != kEmpty) {
                    if ((keep[j] >> lane) & 1ull)
                        a.list[(size_t)side * slots + base + (uint32_t)__popcll(keep[j] & ((1ull << lane) - 1ull))] = v;
                    t[q].id = kEmpty;
                }
            }
            base += (uint32_t)__popcll(keep[j]);
        }
    }
}

// claim a free slot of `table` for id (probing from its home slot) and fill it; false if the table is full.
// used: the side's occupancy words; the stretch of the claimed slot is marked (every writer stores the same 1).
__device__ __forceinline__ bool insert_slot(Slot* table, uint32_t* used, uint32_t mask, unsigned long long id, uint32_t val,
                                            uint32_t stamp, bool* duplicate)
{
    uint32_t p = slot_of(id, mask);
    for (uint32_t tries = 0; tries <= mask; ++tries, p = (p + 1u) & mask) {
        unsigned long long seen = table[p].id;
        if (seen == kEmpty) {
            seen = atomicCAS(&table[p].id, kEmpty, id);
            if (seen == kEmpty) {
                table[p].val = val;
                table[p].stamp = stamp;
                used[p / kChunk] = 1u;
                return true;
            }
        }
        if (seen == id) { // the same flow ID is already waiting (or arriving) on this side
            *duplicate = true;
            return true;
        }
    }
    return false;
}

__global__ __launch_bounds__(256) void join_reinsert(JoinArgs a)
{
    const uint32_t slots = a.mask + 1u;
    for (uint32_t side = 0; side < 2u; ++side) {
        const uint32_t n = a.counters[side];
        for (uint32_t g = blockIdx.x * blockDim.x + threadIdx.x; g < n; g += gridDim.x * blockDim.x) {
            const Slot v = a.list[(size_t)side * slots + g];
            bool dup = false;
            insert_slot(a.table[side], a.used[side], a.mask, v.id, v.val, v.stamp, &dup); // cannot fail: it fitted before
        }
    }
}

// arrivals of one side: SIDE 0 = queue 3 (own table 0, partner table 1), SIDE 1 = queue 2.
// what: 0 stored to wait, 1 matched, 2 no room (or a reserved ID), 3 already waiting on this side, 4 no record
template <int SIDE>
__device__ __forceinline__ void arrive_one(const JoinArgs& a, const unsigned long long* __restrict__ ids,
                                           const uint32_t* __restrict__ vals, uint32_t n, uint32_t g)
{
    Slot* own = a.table[SIDE];
    Slot* other = a.table[1 - SIDE];
    int what = 4;
    uint32_t val = 0, pair_val = 0;
    unsigned long long id = kEmpty;
    if (g < n) {
        id = ids[g];
        val = vals[g];
        what = 2; // stays so for the two reserved IDs, which cannot be stored
    }
    if (id != kEmpty && id != kGone) {
        // partner waiting on the other side?
        bool matched = false;
        uint32_t pv = 0;
        uint32_t p = slot_of(id, a.mask);
        for (uint32_t tries = 0; tries <= a.mask; ++tries, p = (p + 1u) & a.mask) {
            const unsigned long long seen = other[p].id;
            if (seen == kEmpty) break;
            if (seen == id) {
                // take it out; only one arrival can win the slot
                if (atomicCAS(&other[p].id, id, kGone) == id) {
                    pv = other[p].val;
                    matched = true;
                }
                break;
            }
        }
        bool dup = false, stored = true;
        if (!matched) stored = insert_slot(own, a.used[SIDE], a.mask, id, val, a.now, &dup);
        what = matched ? 1 : (!stored ? 2 : (dup ? 3 : 0));
        pair_val = pv;
    }
    // the wave's pairs take consecutive positions with one atomic
    const uint32_t at = wave_claim(a.n_pairs, what == 1);
    if (what == 1) {
        if (at < a.pair_cap) {
            a.pair_q3[at] = SIDE == 0 ? val : pair_val;
            a.pair_q2[at] = SIDE == 0 ? pair_val : val;
        }
    }
    if (a.stats) {
        wave_count(&a.stats[kPairOverflow], what == 1 && at >= a.pair_cap);
        wave_count(&a.stats[kDropped], what == 2);
        wave_count(&a.stats[kDuplicate], what == 3);
    }
}

template <int SIDE>
__global__ __launch_bounds__(256) void join_arrive(JoinArgs a, const unsigned long long* __restrict__ ids,
                                                   const uint32_t* __restrict__ vals, uint32_t n)
{
    const uint32_t rounded = (n + 63u) & ~63u; // whole waves stay in the loop together
    for (uint32_t g = blockIdx.x * blockDim.x + threadIdx.x; g < rounded; g += gridDim.x * blockDim.x)
        arrive_one<SIDE>(a, ids, vals, n, g);
}

// live records of one side -> arrays, in no particular order
__global__ __launch_bounds__(256) void join_dump(const Slot* __restrict__ table, uint32_t slots, unsigned long long* ids,
                                                 uint32_t* vals, uint32_t* stamps, uint32_t cap, uint32_t* count)
{
    for (uint32_t g = blockIdx.x * blockDim.x + threadIdx.x; g < slots; g += gridDim.x * blockDim.x) {
        const Slot v = table[g];
        if (v.id != kEmpty && v.id != kGone) {
            const uint32_t at = atomicAdd(count, 1u);
            if (at < cap) {
                ids[at] = v.id;
                if (vals) vals[at] = v.val;
                if (stamps) stamps[at] = v.stamp;
            }
        }
    }
}

__global__ void zero_word(uint32_t* w) { *w = 0; }

int check_table(sf_ctx* ctx, const char* who, const sf_join_table* t)
{
    if (!t || !t->slots) return sf::fail(ctx, SF_EINVAL, "%s: table missing", who);
    if (t->cap_log2 < 4 || t->cap_log2 > 28) return sf::fail(ctx, SF_EINVAL, "%s: cap_log2 %u outside 4..28", who, t->cap_log2);
    if ((uintptr_t)t->slots & 15u) return sf::fail(ctx, SF_EINVAL, "%s: table is not 16-byte aligned", who);
    return SF_OK;
}

uint32_t grid_for(uint64_t items)
{
    uint64_t b = (items + 255) / 256;
    return (uint32_t)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}

} // namespace

namespace sf {
size_t join_scratch_bytes(uint32_t cap_log2)
{
    if (cap_log2 < 4 || cap_log2 > 28) return 0;
    return align_up(((size_t)2 << cap_log2) * sizeof(Slot)) + kAlign; // survivor list of both sides + counters
}
} // namespace sf

// occupancy words per side (one per kChunk slots), padded to whole 16-byte units
static size_t used_words(uint32_t cap_log2) { return ((((size_t)1 << cap_log2) + kChunk - 1) / kChunk + 3) / 4 * 4; }

extern "C" size_t sf_join_table_bytes(uint32_t cap_log2)
{
    if (cap_log2 < 4 || cap_log2 > 28) return 0;
    return ((size_t)2 << cap_log2) * sizeof(Slot) + 2 * used_words(cap_log2) * sizeof(uint32_t);
}

extern "C" size_t sf_join_workspace_bytes(uint32_t cap_log2)
{
    const size_t b = sf::join_scratch_bytes(cap_log2);
    return b ? b + sf::kFlagBytes + sf::kAlign : 0;
}

extern "C" int sf_join_step(sf_ctx* ctx, const sf_join_table* table, uint32_t now, uint32_t timeout,
                            const uint64_t* q3_id, const uint32_t* q3_val, uint32_t n3, const uint64_t* q2_id,
                            const uint32_t* q2_val, uint32_t n2, uint32_t* pair_q3, uint32_t* pair_q2, uint32_t pair_cap,
                            uint32_t* n_pairs, uint32_t* stats)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_join_step: ctx is NULL");
    {
        const int rc = check_table(ctx, "sf_join_step", table);
        if (rc != SF_OK) return rc;
    }
    if (!n_pairs) return sf::fail(ctx, SF_EINVAL, "sf_join_step: n_pairs is NULL");
    if ((n3 && (!q3_id || !q3_val)) || (n2 && (!q2_id || !q2_val)))
        return sf::fail(ctx, SF_EINVAL, "sf_join_step: arrival arrays missing");
    if (pair_cap && (!pair_q3 || !pair_q2)) return sf::fail(ctx, SF_EINVAL, "sf_join_step: pair arrays missing");
    const uint32_t slots = 1u << table->cap_log2;
    sf::Carve ws(ctx);
    Slot* list = (Slot*)ws.take((size_t)2 * slots * sizeof(Slot));
    uint32_t* counters = (uint32_t*)ws.take(sf::kAlign);
    if (!list || !counters)
        return sf::fail(ctx, SF_ENOMEM, "sf_join_step: workspace has %zu bytes, a step on this table needs %zu",
                        ctx->ws_bytes, sf_join_workspace_bytes(table->cap_log2));
    JoinArgs a;
    a.table[0] = (Slot*)table->slots;
    a.table[1] = (Slot*)table->slots + slots;
    a.used[0] = (uint32_t*)((Slot*)table->slots + 2 * (size_t)slots);
    a.used[1] = a.used[0] + used_words(table->cap_log2);
    a.mask = slots - 1u;
    a.now = now;
    a.timeout = timeout;
    a.list = list;
    a.counters = counters;
    a.n_pairs = n_pairs;
    a.pair_q3 = pair_q3;
    a.pair_q2 = pair_q2;
    a.pair_cap = pair_cap;
    a.stats = stats;
    join_zero<<<1, 64, 0, ctx->stream>>>(counters, n_pairs, stats);
    SF_LAUNCH_CHECK(ctx, "join_zero");
    join_collect<<<grid_for(2ull * slots / kChunkTrips), 256, 0, ctx->stream>>>(a);
    SF_LAUNCH_CHECK(ctx, "join_collect");
    join_reinsert<<<grid_for(slots), 256, 0, ctx->stream>>>(a);
    SF_LAUNCH_CHECK(ctx, "join_reinsert");
    if (n3) {
        join_arrive<0><<<grid_for(n3), 256, 0, ctx->stream>>>(a, (const unsigned long long*)q3_id, q3_val, n3);
        SF_LAUNCH_CHECK(ctx, "join_arrive<3>");
    }
    if (n2) {
        join_arrive<1><<<grid_for(n2), 256, 0, ctx->stream>>>(a, (const unsigned long long*)q2_id, q2_val, n2);
        SF_LAUNCH_CHECK(ctx, "join_arrive<2>");
    }
    return SF_OK;
}

extern "C" int sf_join_pending(sf_ctx* ctx, const sf_join_table* table, int queue, uint64_t* ids, uint32_t* vals,
                               uint32_t* stamps, uint32_t cap, uint32_t* count)
{
    if (!ctx) return sf::fail(nullptr, SF_EINVAL, "sf_join_pending: ctx is NULL");
    {
        const int rc = check_table(ctx, "sf_join_pending", table);
        if (rc != SF_OK) return rc;
    }
    if (queue != 3 && queue != 2) return sf::fail(ctx, SF_EINVAL, "sf_join_pending: queue %d is neither 3 nor 2", queue);
    if (!count || (cap && !ids)) return sf::fail(ctx, SF_EINVAL, "sf_join_pending: count or ids is NULL");
    const uint32_t slots = 1u << table->cap_log2;
    zero_word<<<1, 1, 0, ctx->stream>>>(count);
    SF_LAUNCH_CHECK(ctx, "zero_word");
    join_dump<<<grid_for(slots), 256, 0, ctx->stream>>>((const Slot*)table->slots + (queue == 2 ? slots : 0), slots,
                                                         (unsigned long long*)ids, vals, stamps, cap, count);
    SF_LAUNCH_CHECK(ctx, "join_dump");
    return SF_OK;
}
