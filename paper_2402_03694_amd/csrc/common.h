// Shared host-side plumbing of the library: the context object, error reporting and the
// workspace carve-up.  No device code here.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <cstdio>

#include "serveflow.h"

struct sf_ctx {
    hipStream_t stream;
    char* ws;          // caller-owned device workspace
    size_t ws_bytes;
    int device;
    int n_cu;          // compute units of the device
    uint32_t* d_flags; // 64 words at the head of the workspace: validation counters etc.
    uint64_t lds_ready; // bit per kernel (sf::LdsSlot): its dynamic shared-memory limit has been raised
    char err[512];
};

namespace sf {

constexpr size_t kAlign = 256;
constexpr size_t kFlagBytes = 256; // head of the workspace, reserved for counters

inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

int fail(sf_ctx* ctx, int code, const char* fmt, ...);
void set_global_error(const char* fmt, ...);

// Workspace sub-allocator: hands out aligned slices after the flag words.
struct Carve {
    char* base;
    size_t cap, used;
    explicit Carve(sf_ctx* c) : base(c->ws), cap(c->ws_bytes), used(kFlagBytes) {}
    void* take(size_t bytes)
    {
        size_t at = align_up(used);
        if (at + bytes > cap) return nullptr;
        used = at + bytes;
        return base + at;
    }
    size_t left() const { return cap > align_up(used) ? cap - align_up(used) : 0; }
};

#define SF_HIP(ctx, call)                                                                   \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return sf::fail((ctx), SF_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define SF_LAUNCH_CHECK(ctx, what)                                                           \
    do {                                                                                     \
        hipError_t e_ = hipGetLastError();                                                   \
        if (e_ != hipSuccess)                                                                \
            return sf::fail((ctx), SF_EHIP, "launch of %s failed: %s", (what),               \
                            hipGetErrorString(e_));                                          \
    } while (0)

// Kernels that take more dynamic shared memory than the default limit have the limit raised to the
// whole of a compute unit's, once per context and kernel (the context remembers which).
constexpr int kLdsLimitBytes = 160 * 1024;
enum LdsSlot { kLdsForest = 0 /* 12 variants */, kLdsTreeWalk = 12, kLdsWide = 13 /* 3 operand modes */, kLdsFused = 16,
               kLdsClassify = 17 /* 2 window depths x rows kept or not */ };
#define SF_ALLOW_LDS(ctx, slot, func)                                                                         \
    do {                                                                                                      \
        if (!((ctx)->lds_ready & (1ull << (slot)))) {                                                         \
            SF_HIP((ctx), hipFuncSetAttribute((const void*)(func), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                              sf::kLdsLimitBytes));                                           \
            (ctx)->lds_ready |= 1ull << (slot);                                                               \
        }                                                                                                     \
    } while (0)

// Bytes each step needs from the workspace (also used by sf_workspace_bytes).
size_t forest_pack_bytes(uint32_t n_trees, uint32_t depth);
size_t route_scratch_bytes(uint32_t n_flows);
size_t tree_tier_bytes(uint32_t depth);
constexpr size_t kQuantileScratch = 32768; // histograms, selection state and results of sf_score_quantiles
size_t slow_row_bytes(uint32_t n_h1, uint32_t n_h2, int dtype);
constexpr uint32_t kSlowMinRows = 256;     // smallest row chunk sf_slow_infer can work with
constexpr uint32_t kSlowWantRows = 1 << 18; // chunk sf_workspace_bytes provisions for

} // namespace sf
