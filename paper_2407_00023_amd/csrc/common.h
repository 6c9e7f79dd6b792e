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

// Entry of the positional index of the flattened tree (see DeviceTree).
struct __attribute__((aligned(32))) PathEntry {
    unsigned long long hash;  // of the token path up to and including the first token of the node's edge
    int32_t depth;            // depth of that token
    int32_t node;             // -1 = empty entry
    int32_t edge_start;       // index of the node's first edge token in edge_tok / edge_slot
    int32_t edge_len;
    int32_t parent;
    int32_t pad;
};

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
    int32_t n_tokens;  // edge tokens of all nodes together (as of the upload)
    // Second index, by position: a node is also reachable through the hash of the whole token path from
    // the root up to and including the FIRST token of its edge, together with the depth of that token.
    // A prompt can therefore look up every node boundary on its path at once from its own prefix hashes.
    //   ph_entry: open addressing, linear probing, empty = node -1, mask = ph_mask; one 32-byte entry holds
    //             everything a lookup needs, so that a probe is a single memory round trip
    //   node_endhash[n] = hash of the path up to and including the LAST token of the node's edge
    const PathEntry* ph_entry;
    const unsigned long long* node_endhash;
    uint32_t ph_mask;
};

constexpr unsigned long long kEmptyKey = ~0ull;

// 64-bit mix (splitmix64 finaliser) used identically by the host builder and the device lookup.
__host__ __device__ inline uint32_t hash_key(unsigned long long k) {
    k ^= k >> 30; k *= 0xbf58476d1ce4e5b9ull;
    k ^= k >> 27; k *= 0x94d049bb133111ebull;
    k ^= k >> 31;
    return static_cast<uint32_t>(k);
}

// Polynomial hash of a token path: h(empty) = 0, h(p + t) = h(p) * kPathHashBase + (uint32(t) + 1), mod 2^64.
constexpr unsigned long long kPathHashBase = 0x9E3779B97F4A7C15ull;  // odd
__host__ __device__ inline unsigned long long path_hash_push(unsigned long long h, int32_t tok) {
    return h * kPathHashBase + (static_cast<unsigned long long>(static_cast<uint32_t>(tok)) + 1ull);
}
__host__ __device__ inline uint32_t path_slot(unsigned long long h, int32_t depth) {
    return hash_key(h ^ (static_cast<unsigned long long>(static_cast<uint32_t>(depth)) * 0xD6E8FEB86659FD93ull));
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
// Byte offset, in the workspace of pa_extend_attention, of the two 64-bit counters of the clock probe (the header
// of the workspace is 256 bytes; the first 12 hold the work-list counts).
constexpr size_t kClockProbeOffset = 128;
bool prof_clock_enabled();

enum ProfKernel { kProfMatch = 0, kProfPlan, kProfExtend, kProfMerge, kProfExtendF32, kProfAppend, kProfGather, kProfCalibCopy, kProfCalibMfma, kProfKernels };
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
