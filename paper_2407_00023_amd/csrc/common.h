// Shared host-side helpers of libprefixattn: error reporting, argument checks, and the
// device-side view of the flattened radix tree.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/prefixattn.h"

namespace pa {

// Records a message for pa_last_error() and returns `code`.
int fail(int code, const char* fmt, ...);

#define PA_HIP(expr)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) return pa::fail(PA_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define PA_REQUIRE(cond, ...)                                \
    do {                                                     \
        if (!(cond)) return pa::fail(PA_EINVAL, __VA_ARGS__); \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elt_size(int dtype) { return dtype == PA_F32 ? 4 : 2; }
inline bool shape_ok(int Hq, int Hkv, int D) {
    return Hkv > 0 && Hq > 0 && Hq % Hkv == 0 && (D == 64 || D == 128);
}

// Flattened radix tree in device memory.
//   Node n (0 = the empty virtual root) owns edge tokens edge_tok[node_start[n] .. +node_len[n])
//   and, in parallel, the KV slot of each of those tokens in edge_slot.
//   Children are found through one open-addressing hash table for the whole tree:
//   key = (parent node id << 32) | first token of the child's edge, value = child node id;
//   linear probing, empty key = all ones, capacity a power of two (mask = capacity - 1).
struct DeviceTree {
    const int32_t* edge_tok;
    const int32_t* edge_slot;
    const int32_t* node_start;
    const int32_t* node_len;
    const unsigned long long* ht_key;
    const int32_t* ht_val;
    uint32_t ht_mask;
    int32_t n_nodes;
};

constexpr unsigned long long kEmptyKey = ~0ull;

// 64-bit mix (splitmix64 finaliser) used identically by the host builder and the device lookup.
__host__ __device__ inline uint32_t hash_key(unsigned long long k) {
    k ^= k >> 30; k *= 0xbf58476d1ce4e5b9ull;
    k ^= k >> 27; k *= 0x94d049bb133111ebull;
    k ^= k >> 31;
    return static_cast<uint32_t>(k);
}

// Pool layout: [page][K=0 | V=1][kv head][token in page][D] elements.
// Element index of the first element of (slot, which, head).
__host__ __device__ inline int64_t pool_row(int64_t slot, int which, int g, int Hkv, int D, int page_size) {
    int64_t page = slot / page_size;
    int64_t o = slot - page * page_size;
    return (((page * 2 + which) * Hkv + g) * page_size + o) * D;
}

// Per-kernel event timing (profile.cpp).  A ProfScope around a launch records a start/stop event
// pair on the stream while profiling is switched on, and does nothing otherwise.
enum ProfKernel { kProfMatch = 0, kProfTiles, kProfExtend, kProfMerge, kProfExtendF32, kProfAppend, kProfGather, kProfKernels };
bool prof_begin(int kernel, hipStream_t stream, size_t* slot);
void prof_end(size_t slot, hipStream_t stream);
struct ProfScope {
    hipStream_t stream;
    size_t slot = 0;
    bool on;
    ProfScope(int kernel, hipStream_t s) : stream(s), on(prof_begin(kernel, s, &slot)) {}
    ~ProfScope() { if (on) prof_end(slot, stream); }
    ProfScope(const ProfScope&) = delete;
    ProfScope& operator=(const ProfScope&) = delete;
};

}  // namespace pa

// Internal: device view of an uploaded tree (PA_ESTATE if it is stale or was never uploaded).
int pa_tree_device(const pa_tree* tree, const pa::DeviceTree** out);
