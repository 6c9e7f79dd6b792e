// Batched longest-prefix match of prompts against the flattened radix tree.
//
// Algorithm 1 of the paper starts by matching the request to the radix tree and taking
// cached_len = the sum of the matched lengths along the path; Sec. 3.2 defines the match as
// "from the beginning until no match exists", a partly matched node counting for the
// tokens that do match.  One workgroup walks one request: the child of the current node is
// found through a 64-lane-wide probe of the hash table, then the whole workgroup compares
// the child's edge against the prompt, kTokPerRound tokens per round trip to memory, and
// copies the edge's KV slots into the output as it goes.
#include "common.h"

namespace pa {

constexpr int kMatchThreads = 1024;
constexpr int kMatchUnroll = 4;
constexpr int kTokPerRound = kMatchThreads * kMatchUnroll;
constexpr int kMatchWaves = kMatchThreads / 64;

// Child of `node` whose edge starts with `tok`, or -1.  Executed by a full wave; every lane returns the result.
__device__ __forceinline__ int32_t find_child(const DeviceTree& t, int32_t node, int32_t tok) {
    const unsigned long long key =
        (static_cast<unsigned long long>(static_cast<uint32_t>(node)) << 32) | static_cast<uint32_t>(tok);
    const int lane = threadIdx.x & 63;
    uint32_t h = hash_key(key) & t.ht_mask;
    // The table is at most half full, so an empty slot ends the probe sequence after few windows.
    for (uint32_t probed = 0; probed <= t.ht_mask; probed += 64) {
        const uint32_t idx = (h + lane) & t.ht_mask;
        const unsigned long long k = t.ht_key[idx];
        const unsigned long long hit = __ballot(k == key);
        if (hit) {
            const int src = __ffsll(static_cast<long long>(hit)) - 1;
            const int32_t v = t.ht_val[(h + src) & t.ht_mask];
            return v;
        }
        if (__ballot(k == kEmptyKey)) return -1;
        h = (h + 64) & t.ht_mask;
    }
    return -1;
}

__global__ __launch_bounds__(kMatchThreads) void match_prefixes_kernel(DeviceTree t, const int32_t* __restrict__ tokens,
                                                                      const int32_t* __restrict__ offsets,
                                                                      int32_t* __restrict__ prefix_len,
                                                                      int32_t* __restrict__ slot_idx) {
    __shared__ int32_t s_first_mismatch[2][kMatchWaves];
    const int r = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int32_t base = offsets[r];
    const int32_t n = offsets[r + 1] - base;
    const int32_t* __restrict__ prompt = tokens + base;
    int32_t* __restrict__ out_slots = slot_idx + base;

    int32_t pos = 0, node = 0;
    int round = 0;
    while (pos < n) {
        const int32_t child = find_child(t, node, prompt[pos]);
        if (child < 0) break;
        const int32_t es = t.node_start[child];
        const int32_t el = t.node_len[child];
        const int32_t lim = min(el, n - pos);  // tokens of this edge that can match at all
        int32_t matched = lim;                 // becomes the index of the first mismatch, if any
        for (int32_t c0 = 0; c0 < lim; c0 += kTokPerRound) {
            int32_t mine = INT32_MAX;
            int32_t et[kMatchUnroll], pt[kMatchUnroll], sl[kMatchUnroll];
#pragma unroll
            for (int u = 0; u < kMatchUnroll; ++u) {
                const int32_t k = c0 + u * kMatchThreads + tid;
                const bool in = k < lim;
                et[u] = in ? t.edge_tok[es + k] : 0;
                pt[u] = in ? prompt[pos + k] : 0;
                sl[u] = in ? t.edge_slot[es + k] : 0;
            }
#pragma unroll
            for (int u = kMatchUnroll - 1; u >= 0; --u) {
                const int32_t k = c0 + u * kMatchThreads + tid;
                if (k < lim) {
                    out_slots[pos + k] = sl[u];  // entries past the final match are unspecified by contract
                    if (et[u] != pt[u]) mine = k;
                }
            }
            // workgroup minimum of `mine`: wave reduction, then one LDS slot per wave (double-buffered by round)
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) mine = min(mine, __shfl_xor(mine, off));
            if (lane == 0) s_first_mismatch[round & 1][wave] = mine;
            __syncthreads();
            int32_t first = INT32_MAX;
#pragma unroll
            for (int w = 0; w < kMatchWaves; ++w) first = min(first, s_first_mismatch[round & 1][w]);
            ++round;
            if (first != INT32_MAX) { matched = first; break; }
        }
        pos += matched;
        if (matched < el) break;  // mismatch inside the edge, or the prompt ended inside it
        node = child;
    }
    if (tid == 0) prefix_len[r] = pos;
}

}  // namespace pa

extern "C" int pa_match_prefixes(const pa_tree* tree, const int32_t* tokens, const int32_t* offsets, int B,
                                 int32_t* prefix_len, int32_t* slot_idx, void* stream) {
    const pa::DeviceTree* view = nullptr;
    int rc = pa_tree_device(tree, &view);
    if (rc != PA_OK) return rc;
    PA_REQUIRE(B >= 0, "pa_match_prefixes: B = %d", B);
    if (B == 0) return PA_OK;
    PA_REQUIRE(offsets && prefix_len, "pa_match_prefixes: offsets or prefix_len is NULL");
    // tokens / slot_idx may be NULL only if every prompt is empty (offsets[B] == 0), which the host cannot see
    {
        pa::ProfScope prof(pa::kProfMatch, static_cast<hipStream_t>(stream));
        hipLaunchKernelGGL(pa::match_prefixes_kernel, dim3(B), dim3(pa::kMatchThreads), 0,
                           static_cast<hipStream_t>(stream), *view, tokens, offsets, prefix_len, slot_idx);
    }
    PA_HIP(hipGetLastError());
    return PA_OK;
}
