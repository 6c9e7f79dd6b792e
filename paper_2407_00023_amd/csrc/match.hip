// Batched longest-prefix match of prompts against the flattened radix tree.
//
// Algorithm 1 of the paper starts by matching the request to the radix tree and taking
// cached_len = the sum of the matched lengths along the path; Sec. 3.2 defines the match as
// running from the beginning until no match exists, a partly matched node counting for the
// tokens that do match.  A workgroup of 1024 threads walks a request's path.  The child of the
// current node is found through a 64-lane-wide probe of the (parent, first token) table.  If its edge is
// long, the whole workgroup compares it against the prompt, 4096 tokens per round trip to memory,
// copying the edge's KV slots to the output as it goes.  If it is short, the path is likely to run
// through many short nodes, and a window of prompt positions is resolved at once (below).  In small
// batches a long prompt gets a workgroup per window (further below).
#include <atomic>
#include <mutex>

#include "common.h"

namespace pa {

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
        const int32_t val = t.ht_val[idx];  // (fetched with the key, not after it: one round trip to memory, not two)
        const unsigned long long hit = __ballot(k == key);
        if (hit) {
            const int src = __ffsll(static_cast<long long>(hit)) - 1;
            return __shfl(val, src);
        }
        if (__ballot(k == kEmptyKey)) return -1;
        h = (h + 64) & t.ht_mask;
    }
    return -1;
}

// ---------------------------------------------------------------------------------------------------
// Windows: all node boundaries of a stretch of the prompt's path at once, instead of one node after the
// other (a step from node to node costs several dependent memory round trips; a path through a tree with
// many branch points has hundreds of nodes).
//
// The tree carries a second index: node -> (hash of the token path up to and including the first token
// of the node's edge, depth of that token).  A window is the kWin prompt positions from the current match
// position on.  The workgroup forms the prefix hash of the prompt at every position of the window (a scan
// seeded with the stored hash of the path that ends at the current node) and looks every (hash, position)
// up: a hit NOMINATES a node whose edge would start there.  The edges of all nominated nodes are compared
// with the prompt in parallel.  Then the nodes that really lie on the path are marked: hash collisions apart,
// the nominated nodes are the path's nodes in order, so each must be linked to the one nominated before it
// ("that one matched its whole edge, ends where this one starts, and is this one's parent"), starting from
// position 0, which holds the child found exactly; the path's nodes are those before the first broken link (a
// prefix maximum and a minimum over the workgroup, no walk along the chain).  The slots of all marked nodes are
// copied in parallel.  Whatever ends the chain (a mismatch, no nomination, a very long edge, a collision, the
// window's end), the loop head takes over from the last confirmed position with an exact child lookup, so the
// result never depends on the hash being free of collisions: a collision can only cost time.
// What a window costs (measured, 4,096 positions, a tree of 4,096 sequences): 3.6 us for the table probes (one
// 16-byte entry per position from a table far larger than any cache: the compute unit's memory pipeline takes
// about one such line per cycle, then a second trip for the hits), 2 us for the edge comparisons, 2 us for the
// marking, 1 us each for the scan, the child lookup and the slot copy.
// ---------------------------------------------------------------------------------------------------
constexpr int kWin = 1024;        // threads per workgroup
// kPos = prompt positions per thread and window (consecutive ones), kWinP = kWin * kPos positions per window: 2 / 2048
// for large batches (two workgroups fit a compute unit), 4 / 4096 for small ones (a window costs a fixed number of
// dependent round trips to memory, so a long prompt is done in fewer of them; 110 KB of LDS, one workgroup per unit)
constexpr int kQuadEdge = 16;     // edges with at most this many tokens to compare are compared by 4 lanes, in one round
constexpr int kGroupEdge = 64;    // ... with at most this many by 16 lanes, in one round
constexpr int kWaveEdge = 1024;   // ... by one wave, 256 tokens per round; longer ones by the whole workgroup
constexpr int kDirectEdge = 256;  // a next edge at least this long is compared directly, without opening a window
constexpr int kWideUnroll = 4;    // tokens per thread and round of a wave- or workgroup-wide comparison

// Several workgroups per request (small batches).  The hashes of a window depend on the prompt alone, so the windows
// of a long prompt need not wait for one another: workgroup w of a request resolves the window at the fixed place
// [w * kWinP, (w + 1) * kWinP) on its own - workgroup 0 the walk from the root as far as it begins a step inside the first
// window, the others one window each, from the first node nominated in it, their entry hash formed from the prompt's
// tokens before the window - and leaves a summary: where its chain begins, the parent its first node names, and where
// the walk would stand after it.  The workgroup that finishes last (a counter per request) joins the summaries in order
// - a window's chain is accepted if it begins exactly where the walk stands and names the walk's node as parent: the
// same exact link as inside a window - and walks on alone from where the chain of accepted windows ends.  Nobody waits
// for anybody.  Slot ids that a window writes before it is accepted are those of nodes whose whole path hashes like the
// prompt, confirmed token by token along their edges; the last workgroup's own writes come after all of them.
constexpr int kMaxW = 8;         // workgroups (windows) per request; a longer prompt's rest is walked by the last one
constexpr int kMultiMaxB = 64;   // batches of up to this many requests take this form
constexpr int kScratchSets = 64; // calls in flight at once on a device that may use it
struct MatchSummary {
    int32_t f_pos, f_parent;     // position of the first node of the chain (-1: none), the parent it names
    int32_t exit_pos, exit_cur;  // matched length and current node after the chain
    int32_t done;                // 1: the walk ends there (mismatch inside an edge, or no child)
    int32_t last_es, last_start; // the chain's last edge: index of its first token in the tree's arrays, its position
    int32_t pad;
};
struct MatchScratch {
    MatchSummary sum[kMultiMaxB][kMaxW];
    unsigned counter[kMultiMaxB];  // workgroups of the request that have finished; back to 0 with the last one
};

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits until the global stores of
// the slot ids are acknowledged, a long round trip the matcher has no reason to wait for.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int kPos, bool kMulti>
__global__ __launch_bounds__(kWin) void match_prefixes_pos_kernel(DeviceTree t, const int32_t* __restrict__ tokens,
                                                                 const int32_t* __restrict__ offsets,
                                                                 int32_t* __restrict__ prefix_len,
                                                                 int32_t* __restrict__ slot_idx, MatchScratch* scratch) {
    constexpr int kWinP = kWin * kPos;
    constexpr int kWaves = kWin / 64;
    __shared__ unsigned long long s_wtot[kWaves];
    // per window position: {candidate node or -1, its parent, its edge length, tokens of the edge that match the
    // prompt (-2 = not compared yet: very long edge)}
    __shared__ int4 s_rec[kWinP];
    __shared__ int32_t s_es[kWinP];      // index of the candidate's first edge token
    __shared__ int16_t s_list0[kWinP];   // window positions of candidates compared by 4 lanes
    __shared__ int16_t s_list[kWinP];    // ... by 16 lanes
    __shared__ int16_t s_list2[kWinP];   // ... by one wave
    __shared__ int16_t s_list3[16];      // ... by the whole workgroup (multi-workgroup form only)
    __shared__ int32_t s_wmax[kWaves], s_brk[kWaves], s_last[kWaves];
    __shared__ int32_t s_count0, s_count, s_count2, s_count3;
    __shared__ int32_t s_red[2][kWaves];
    __shared__ int32_t s_first[2];  // a lone window: position of its first nominated node and the parent it names
    __shared__ int32_t s_last_one;  // this workgroup is the last of its request to finish
    __shared__ int32_t s_sum[kMaxW * 8];  // ... and then holds the request's summaries here
    // (multi-workgroup form: the first workgroups of the grid are the requests' workgroups 0, which have the longest way
    // to go, then come all workgroups 1, and so on)
    const int n_req = kMulti ? gridDim.x / kMaxW : gridDim.x;
    const int r = blockIdx.x % n_req;
    const int w = blockIdx.x / n_req;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t base = offsets[r];
    const int32_t n = offsets[r + 1] - base;
    const int32_t* __restrict__ prompt = tokens + base;
    int32_t* __restrict__ out_slots = slot_idx + base;

    // With b = B^kPos (a thread's positions hash as one step of the scan): b^(2^k), and b^lane
    unsigned long long bp2[7];
    bp2[0] = 1ull;
#pragma unroll
    for (int i = 0; i < kPos; ++i) bp2[0] *= kPathHashBase;
#pragma unroll
    for (int k = 1; k < 7; ++k) bp2[k] = bp2[k - 1] * bp2[k - 1];
    unsigned long long bpow_lane = 1ull;
#pragma unroll
    for (int k = 0; k < 6; ++k)
        if (lane >> k & 1) bpow_lane *= bp2[k];

    int32_t pos = 0, cur = 0;        // matched so far; node whose edge ends at pos
    int red_round = 0;
    bool done = false;
    // What this workgroup's pass over the loop below is: 0 the whole walk (the only pass of the single-workgroup form, the
    // last workgroup's second pass otherwise), 1 the walk as long as it begins a step inside the first window, 2 one
    // window at a fixed place.
    // (a request takes one workgroup per window its prompt reaches into, kMaxW at most; the others leave at once, and a
    // prompt inside the first window is walked by its workgroup 0 as in the single-workgroup form)
    const int n_wg = !kMulti ? 1 : max(1, min(kMaxW, (n + kWinP - 1) / kWinP));
    if (w >= n_wg) return;
    int role = n_wg == 1 ? 0 : w == 0 ? 1 : 2;
    int32_t f_pos = role == 2 ? -1 : 0, f_parent = 0;
    int32_t last_es = 0, last_start = 0;  // the last edge walked: its first token in the tree's arrays, its position
    unsigned long long seed = 0ull;  // role 2: hash of the prompt before the window
    bool active = true;
    // Slot ids written by a lone window go straight through to memory (stores of device scope leave no dirty line in
    // this XCD's L2), so that waiting for them to be acknowledged is all it takes for the last workgroup's own writes to
    // come after them; a fence of device scope would write the whole L2 back and costs 100 us and more here.  (What the
    // walk from the root writes is exact whenever it is written and needs no such care.)
    auto put_slot = [&](int32_t at, int32_t v) __attribute__((always_inline)) {
        if (kMulti && role == 2) __hip_atomic_store(out_slots + at, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else out_slots[at] = v;
    };
    if (role == 2) {
        pos = w * kWinP;
        active = pos < n;
        if (active) {
            // The hash of the pos = kWin * L tokens before the window is sum_j (token_j + 1) B^(pos - 1 - j).  Thread t takes
            // the tokens t, t + kWin, t + 2 kWin, ... (neighbouring lanes read neighbouring tokens): its share is
            // B^(kWin - 1 - t) times a fold of its L tokens with B^kWin as the step; the shares are then joined in thread
            // order, a scan with B as the step.
            const int L = pos / kWin;  // = kPos * w
            int32_t tk[kPos * (kMaxW - 1)];
#pragma unroll
            for (int i = 0; i < kPos * (kMaxW - 1); ++i) tk[i] = i < L ? prompt[i * kWin + tid] : 0;  // (all loads out together)
            unsigned long long big = kPathHashBase;  // B^kWin
#pragma unroll
            for (int k = 0; k < 10; ++k) big *= big;
            static_assert(kWin == 1024, "B^kWin by ten squarings");
            unsigned long long c = 0ull;
#pragma unroll
            for (int i = 0; i < kPos * (kMaxW - 1); ++i)
                if (i < L) c = c * big + (static_cast<unsigned long long>(static_cast<uint32_t>(tk[i])) + 1ull);
            unsigned long long step = kPathHashBase;  // B^(2^k)
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                const unsigned long long left = __shfl_up(c, 1u << k);
                if (lane >= (1 << k)) c = left * step + c;
                step *= step;
            }
            if (lane == 63) s_wtot[wave] = c;
            lds_barrier();
            for (int v = 0; v < kWaves; ++v) seed = seed * step + s_wtot[v];  // (step = B^64 by now)
            lds_barrier();
        }
    }
    for (;;) {
    while (active && !done && pos < n && (role != 1 || pos < kWinP)) {
        // The next node, found exactly (child table keyed by parent and first token).  A long edge is compared
        // right away by the whole workgroup; a short one opens a window.  (A lone window has no node to start from: its
        // first node is whatever the hashes nominate first.)
        unsigned long long h = seed;  // hash of prompt[0 .. pos)
        int32_t child = -1, c_es = 0, c_len = 0;
        if (role != 2) {
            h = t.node_endhash[cur];  // (asked for ahead of its use below)
            child = find_child(t, cur, prompt[pos]);
            if (child < 0) {
                done = true;
                break;
            }
            c_es = t.node_start[child];
            c_len = t.node_len[child];
        }
        if (role != 2 && c_len >= kDirectEdge) {
            const int32_t lim = min(c_len, n - pos);
            int32_t m = lim;
            for (int32_t c0 = 0; c0 < lim; c0 += kWin * kWideUnroll) {
                int32_t et[kWideUnroll], pt[kWideUnroll], sl[kWideUnroll];
#pragma unroll
                for (int u = 0; u < kWideUnroll; ++u) {
                    const int32_t k = c0 + u * kWin + tid;
                    const bool in = k < lim;
                    et[u] = in ? t.edge_tok[c_es + k] : 0;
                    pt[u] = in ? prompt[pos + k] : 0;
                    sl[u] = in ? t.edge_slot[c_es + k] : 0;
                }
                int32_t mine = INT32_MAX;
#pragma unroll
                for (int u = kWideUnroll - 1; u >= 0; --u) {
                    const int32_t k = c0 + u * kWin + tid;
                    if (k < lim) {
                        put_slot(pos + k, sl[u]);  // entries past the final match are unspecified by contract
                        if (et[u] != pt[u]) mine = k;
                    }
                }
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) mine = min(mine, __shfl_xor(mine, off));
                if (lane == 0) s_red[red_round & 1][wave] = mine;
                lds_barrier();
                int32_t first = INT32_MAX;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) first = min(first, s_red[red_round & 1][w]);
                ++red_round;
                if (first != INT32_MAX) { m = first; break; }
            }
            last_es = c_es;
            last_start = pos;
            pos += m;
            if (m < c_len) {  // mismatch inside the edge, or the prompt ended inside it
                done = true;
                break;
            }
            cur = child;
            continue;
        }
        const int32_t w0 = pos;
        // (workgroup 0 of several nominates nodes inside the first window only, so that its chain ends where the next
        // workgroup's begins; edges are still compared to their end)
        const int32_t n_nom = role == 1 ? min(n, kWinP) : n;
        const int32_t rel0 = tid * kPos;  // this thread's first position in the window; its positions are rel0 + i
        // ---- A. prefix hashes of the window: inclusive scan of x -> x * B + (token + 1).  A thread folds its own
        // positions, then the scan runs over threads with B^kPos as the step: within a wave by shuffles, then
        // across waves ----
        unsigned long long loc[kPos];  // hash of this thread's positions 0 .. i
        {
            unsigned long long run = 0ull;
#pragma unroll
            for (int i = 0; i < kPos; ++i) {
                const int32_t p = w0 + rel0 + i;
                run = run * kPathHashBase + (p < n ? static_cast<unsigned long long>(static_cast<uint32_t>(prompt[p])) + 1ull : 0ull);
                loc[i] = run;
            }
        }
        unsigned long long c = loc[kPos - 1];
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const unsigned long long left = __shfl_up(c, 1u << k);
            if (lane >= (1 << k)) c = left * bp2[k] + c;
        }
        if (lane == 63) s_wtot[wave] = c;
        if (tid == 0) { s_count0 = 0; s_count = 0; s_count2 = 0; s_count3 = 0; }
        unsigned long long excl = __shfl_up(c, 1);  // hash of the wave's positions before this thread's
        if (lane == 0) excl = 0ull;
        lds_barrier();
        unsigned long long before = h;  // hash of everything before this wave's positions
        for (int v = 0; v < wave; ++v) before = before * bp2[6] + s_wtot[v];
        const unsigned long long upto = before * bpow_lane + excl;  // hash of prompt[0 .. w0 + rel0)
        // ---- B. candidates: nodes whose edge starts at p after exactly this prefix (by hash) ----
        {
            // (the first probe of every position of the thread goes out before any is looked at, both halves of the
            // entry: one round trip to memory for all of them; only a collision in the table costs another)
            unsigned long long hps[kPos];
            uint32_t ats[kPos];
            uint4 lo0[kPos];
            unsigned long long bi = 1ull;
#pragma unroll
            for (int i = 0; i < kPos; ++i) {
                bi *= kPathHashBase;
                const int32_t p = w0 + rel0 + i;
                hps[i] = upto * bi + loc[i];  // hash of prompt[0 .. p]
                ats[i] = path_slot(hps[i], p) & t.ph_mask;
                lo0[i] = make_uint4(0, 0, 0, 0xFFFFFFFFu);
                if (p < n_nom) lo0[i] = reinterpret_cast<const uint4*>(t.ph_entry + ats[i])[0];  // hash, depth, node
            }
#pragma unroll
            for (int i = 0; i < kPos; ++i) {
                const int32_t rel = rel0 + i, p = w0 + rel;
                const unsigned long long hp = hps[i];
                int4 rec = make_int4(-1, -1, 0, 0);
                if (p < n_nom) {
                    uint32_t at = ats[i];
                    uint4 lo = lo0[i];
                    for (uint32_t probes = 0; probes <= t.ph_mask; ++probes) {
                        const int32_t nd = static_cast<int32_t>(lo.w);
                        if (nd < 0) break;
                        const unsigned long long eh = (static_cast<unsigned long long>(lo.y) << 32) | lo.x;
                        if (eh == hp && static_cast<int32_t>(lo.z) == p) {
                            const uint4 hi = reinterpret_cast<const uint4*>(t.ph_entry + at)[1];  // edge start, length, parent
                            rec = make_int4(nd, static_cast<int32_t>(hi.z), static_cast<int32_t>(hi.y), -2);
                            s_es[rel] = static_cast<int32_t>(hi.x);
                            break;
                        }
                        at = (at + 1) & t.ph_mask;
                        lo = reinterpret_cast<const uint4*>(t.ph_entry + at)[0];
                    }
                }
                if (rel == 0 && role != 2) {  // position 0 holds the node found exactly above, whatever the probe said
                    rec = make_int4(child, cur, c_len, -2);
                    s_es[0] = c_es;
                }
                s_rec[rel] = rec;
                if (rec.x >= 0) {
                    const int32_t lim = min(rec.z, n - p);
                    if (lim <= kQuadEdge) s_list0[atomicAdd(&s_count0, 1)] = static_cast<int16_t>(rel);
                    else if (lim <= kGroupEdge) s_list[atomicAdd(&s_count, 1)] = static_cast<int16_t>(rel);
                    else if (lim <= kWaveEdge) s_list2[atomicAdd(&s_count2, 1)] = static_cast<int16_t>(rel);
                    else if (kMulti) {  // (a window of its own cannot hand a very long edge to a loop head: compared here)
                        const int at = atomicAdd(&s_count3, 1);
                        if (at < 16) s_list3[at] = static_cast<int16_t>(rel);
                    }
                }
            }
        }
        lds_barrier();
        // ---- C. compare the candidates' edges with the prompt, all candidates at once ----
        {
            const int n0 = s_count0, n1 = s_count, n2 = s_count2;
            for (int j = tid >> 2; j < n0; j += kWin / 4) {  // 4 lanes per candidate, one round of <= 16 tokens
                const int rel = s_list0[j], sub4 = tid & 3;
                const int32_t es = s_es[rel];
                const int32_t lim = min(s_rec[rel].z, n - (w0 + rel));
                bool bad[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int32_t k = sub4 + 4 * u, kk = min(k, lim - 1);
                    const int32_t a = t.edge_tok[es + kk], b = prompt[w0 + rel + kk];
                    bad[u] = (k < lim) & (a != b);
                }
                int32_t m = lim;
#pragma unroll
                for (int u = 3; u >= 0; --u) {
                    const unsigned mine = static_cast<unsigned>(__ballot(bad[u]) >> (lane & 60)) & 0xFu;
                    if (mine) m = 4 * u + __ffs(mine) - 1;
                }
                if (sub4 == 0) s_rec[rel].w = m;
            }
            const int sub = tid & 15;
            for (int j = tid >> 4; j < n1; j += kWin / 16) {  // 16 lanes per candidate, one round of <= 64 tokens
                const int rel = s_list[j];
                const int32_t es = s_es[rel];
                const int32_t lim = min(s_rec[rel].z, n - (w0 + rel));
                bool bad[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {  // (all loads go out before the first comparison: one round trip, not four)
                    const int32_t k = sub + 16 * u, kk = min(k, lim - 1);
                    const int32_t a = t.edge_tok[es + kk], b = prompt[w0 + rel + kk];
                    bad[u] = (k < lim) & (a != b);
                }
                int32_t m = lim;
#pragma unroll
                for (int u = 3; u >= 0; --u) {
                    const unsigned mine = static_cast<unsigned>(__ballot(bad[u]) >> (lane & 48)) & 0xFFFFu;
                    if (mine) m = 16 * u + __ffs(mine) - 1;
                }
                if (sub == 0) s_rec[rel].w = m;
            }
            for (int j = wave; j < n2; j += kWaves) {  // one wave per candidate, 256 tokens per round
                const int rel = s_list2[j];
                const int32_t es = s_es[rel];
                const int32_t lim = min(s_rec[rel].z, n - (w0 + rel));
                int32_t m = lim;
                for (int32_t c0 = 0; c0 < lim; c0 += 64 * kWideUnroll) {
                    bool bad[kWideUnroll];
#pragma unroll
                    for (int u = 0; u < kWideUnroll; ++u) {
                        const int32_t k = c0 + 64 * u + lane, kk = min(k, lim - 1);
                        const int32_t a = t.edge_tok[es + kk], b = prompt[w0 + rel + kk];
                        bad[u] = (k < lim) & (a != b);
                    }
                    int32_t first = -1;
#pragma unroll
                    for (int u = kWideUnroll - 1; u >= 0; --u) {
                        const unsigned long long bb = __ballot(bad[u]);
                        if (bb) first = c0 + 64 * u + __ffsll(static_cast<long long>(bb)) - 1;
                    }
                    if (first >= 0) { m = first; break; }
                }
                if (lane == 0) s_rec[rel].w = m;
            }
            if (kMulti) {  // very long edges, one after the other, 4,096 tokens per round by the whole workgroup
                const int n3 = min(s_count3, 16);
                for (int j = 0; j < n3; ++j) {
                    const int rel = s_list3[j];
                    const int32_t es = s_es[rel];
                    const int32_t lim = min(s_rec[rel].z, n - (w0 + rel));
                    int32_t m = lim;
                    for (int32_t c0 = 0; c0 < lim; c0 += kWin * kWideUnroll) {
                        bool bad[kWideUnroll];
#pragma unroll
                        for (int u = 0; u < kWideUnroll; ++u) {
                            const int32_t k = c0 + u * kWin + tid, kk = min(k, lim - 1);
                            const int32_t a = t.edge_tok[es + kk], b = prompt[w0 + rel + kk];
                            bad[u] = (k < lim) & (a != b);
                        }
                        int32_t mine = INT32_MAX;
#pragma unroll
                        for (int u = kWideUnroll - 1; u >= 0; --u)
                            if (bad[u]) mine = c0 + u * kWin + tid;
#pragma unroll
                        for (int off = 32; off > 0; off >>= 1) mine = min(mine, __shfl_xor(mine, off));
                        if (lane == 0) s_red[red_round & 1][wave] = mine;
                        lds_barrier();
                        int32_t first = INT32_MAX;
#pragma unroll
                        for (int v = 0; v < kWaves; ++v) first = min(first, s_red[red_round & 1][v]);
                        ++red_round;
                        if (first != INT32_MAX) { m = first; break; }
                    }
                    if (tid == 0) s_rec[rel].w = m;
                }
            }
        }
        lds_barrier();
        // ---- D. which candidates lie on the prompt's path.  A candidate's whole path hashes like the prompt up to its
        // position, so (hash collisions apart) the candidates ARE the path's nodes, in order, and each is the child
        // of the one before it.  Exactly that is checked: a candidate is linked if the candidate before it matched its
        // whole edge, ends where this one starts and is its parent.  The path's nodes in this window are the
        // candidates before the first one that is not linked; whatever broke the chain (the end of the match, a very
        // long edge left uncompared, a collision) is the loop head's business. ----
        int32_t candm[kPos];  // the last candidate at or before each of the thread's positions, among its own
        int4 recs[kPos];
        {
            int32_t run = -1;
#pragma unroll
            for (int i = 0; i < kPos; ++i) {
                recs[i] = s_rec[rel0 + i];
                run = max(run, recs[i].x >= 0 ? rel0 + i : -1);
                candm[i] = run;
            }
        }
        int32_t cm = candm[kPos - 1];
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const int32_t left = __shfl_up(cm, 1u << k);
            if (lane >= (1 << k)) cm = max(cm, left);
        }
        if (lane == 63) s_wmax[wave] = cm;
        int32_t cand_before = __shfl_up(cm, 1);  // last candidate before this thread's positions
        if (lane == 0) cand_before = -1;
        lds_barrier();
        for (int v = 0; v < wave; ++v) cand_before = max(cand_before, s_wmax[v]);
        int32_t brk = INT32_MAX;  // first candidate of this thread that is not linked
#pragma unroll
        for (int i = kPos - 1; i >= 0; --i) {
            const int rel = rel0 + i;
            if (recs[i].x >= 0) {
                const int32_t pc = i > 0 ? max(cand_before, candm[i - 1]) : cand_before;  // the candidate before this one
                if (pc >= 0) {
                    const int4 pr = s_rec[pc];
                    if (!(pr.w == pr.z && pc + pr.z == rel && recs[i].y == pr.x)) brk = rel;
                } else {  // the first of the window (position 0, except in a lone window): the chain begins here
                    s_first[0] = rel;
                    s_first[1] = recs[i].y;
                }
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) brk = min(brk, __shfl_xor(brk, off));
        if (lane == 0) s_brk[wave] = brk;
        lds_barrier();
        int32_t first_break = INT32_MAX;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) first_break = min(first_break, s_brk[v]);
        int32_t lastm = -1;  // last path node among the thread's positions
#pragma unroll
        for (int i = 0; i < kPos; ++i)
            if (recs[i].x >= 0 && rel0 + i < first_break) lastm = rel0 + i;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) lastm = max(lastm, __shfl_xor(lastm, off));
        if (lane == 0) s_last[wave] = lastm;
        lds_barrier();
        int32_t z = -1;  // last path node of the window
#pragma unroll
        for (int v = 0; v < kWaves; ++v) z = max(z, s_last[v]);
        // ---- E. slots of the matched positions: position i belongs to the last path node starting at or before it ----
#pragma unroll
        for (int i = 0; i < kPos; ++i) {
            const int rel = rel0 + i;
            const int32_t cv = rel < first_break ? max(cand_before, candm[i]) : z;
            if (cv >= 0) {
                const int4 cr = s_rec[cv];
                if (cr.w >= 0 && rel < cv + cr.w) put_slot(w0 + rel, t.edge_slot[s_es[cv] + (rel - cv)]);
            }
        }
        // ---- F. where the walk stands after this window (the same in every thread).  The loop head decides
        // what follows: the hash only nominated the nodes, the child table has the last word. ----
        if (z < 0) {  // (a lone window in which nothing was nominated)
            active = false;
        } else {
            const int4 zr = s_rec[z];
            if (zr.w < 0) {
                pos = w0 + z;  // very long edge, not compared here: the loop head takes it
                cur = zr.y;
                last_start = pos;
            } else {
                const int32_t m = zr.w;
                const int32_t es = s_es[z];
                last_es = es;
                last_start = w0 + z;
                // the part of the last node's edge that reaches past the window
                for (int32_t k = kWinP - z + tid; k < m; k += kWin) put_slot(w0 + z + k, t.edge_slot[es + k]);
                pos = w0 + z + m;
                if (m == zr.z) {
                    cur = zr.x;
                    // (every node that begins at a position of the window was nominated there: if nothing was where this
                    // edge ends, no child continues the walk, and the lookup that would say so is saved)
                    if (z + m < kWinP && pos < n_nom && s_rec[z + m].x < 0) done = true;
                } else if (m == 0) {
                    cur = zr.y;  // the nominated node is not the child (only a hash collision does that)
                } else {
                    done = true;  // mismatch inside the edge, or the prompt ended inside it
                }
            }
            if (pos == w0 && role != 2) done = true;  // cannot happen: position 0 holds a true child, whose first token matches
            if (role == 2) {
                f_pos = w0 + s_first[0];
                f_parent = s_first[1];
            }
        }
        lds_barrier();  // the window arrays are rebuilt next
        if (role == 2) break;  // one window only
    }
    if (!kMulti || role == 0) break;
    // ---- leave the summary; the last workgroup of the request to get here joins them ----
    if (role == 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's slot ids have arrived before the count says so
    lds_barrier();
    if (tid == 0) {
        int32_t* sm = reinterpret_cast<int32_t*>(&scratch->sum[r][w]);
        const int32_t vals[7] = {f_pos, f_parent, pos, cur, done ? 1 : 0, last_es, last_start};
#pragma unroll
        for (int i = 0; i < 7; ++i) __hip_atomic_store(sm + i, vals[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        s_last_one = atomicInc(&scratch->counter[r], n_wg - 1) == static_cast<unsigned>(n_wg - 1);
    }
    lds_barrier();
    if (!s_last_one) return;
    {
        // (fetched at once, by loads of device scope: past this XCD's L2, which may hold what the array said during an
        // earlier call)
        static_assert(sizeof(MatchSummary) == 8 * sizeof(int32_t), "eight words per summary");
        if (tid < n_wg * 8)
            s_sum[tid] = __hip_atomic_load(reinterpret_cast<int32_t*>(&scratch->sum[r][0]) + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lds_barrier();
        auto field = [&](int ww, int i) __attribute__((always_inline)) { return s_sum[ww * 8 + i]; };
        auto accept = [&](int ww) __attribute__((always_inline)) {
            pos = field(ww, 2);
            cur = field(ww, 3);
            done = field(ww, 4) != 0;
            last_es = field(ww, 5);
            last_start = field(ww, 6);
        };
        // A window that is no part of the walk may still have written slot ids below the walk's position: only a chain
        // that begins with a node nominated by a colliding hash does (no node of the path begins inside an edge).  What
        // it wrote there is put right from the edge the walk took.
        auto repair = [&](int ww) __attribute__((always_inline)) {
            const int32_t fp = field(ww, 0), ep = field(ww, 2);
            if (fp >= 0 && fp < pos)
                for (int32_t k = max(fp, last_start) + tid; k < min(ep, pos); k += kWin) out_slots[k] = t.edge_slot[last_es + (k - last_start)];
        };
        accept(0);
        int wlast = 0;  // the last window whose chain is part of the walk
        for (;;) {
            const int ww = min(pos / kWinP, n_wg);  // the window the walk stands in (n_wg: past all of them)
            for (int x = wlast + 1; x < ww; ++x) repair(x);  // (windows that lie inside the last edge)
            if (ww >= n_wg || ww == wlast) break;
            if (!done && pos < n && field(ww, 0) == pos && field(ww, 1) == cur && field(ww, 2) > pos) {
                accept(ww);  // the walk's next node begins this window's chain
                wlast = ww;
                continue;
            }
            // (the window nominated every node that begins in it: none where the walk stands means no child goes on)
            if (!done && pos < n && (field(ww, 0) < 0 || field(ww, 0) > pos)) done = true;
            repair(ww);
            break;  // the walk goes on by itself, if it goes on
        }
    }
    role = 0;
    active = true;
    }
    if (tid == 0) prefix_len[r] = pos;
}

}  // namespace pa

// Summaries and counters of the multi-workgroup form: part of the library's code object (each GPU holds its own copy;
// in host code the array's name is only a handle for hipGetSymbolAddress).  A call takes the next of kScratchSets sets,
// so that calls in flight at once on different streams do not meet in one (more than kScratchSets of them could).
static __device__ pa::MatchScratch g_match_scratch[pa::kScratchSets];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_ms_mu;
pa::MatchScratch* g_ms_ptr[kMaxDevices] = {};
std::atomic<unsigned> g_ms_next{0};

int match_scratch_of_current_device(pa::MatchScratch** out) {
    int dev = -1;
    PA_HIP(hipGetDevice(&dev));
    PA_REQUIRE(dev >= 0 && dev < kMaxDevices, "pa_match_prefixes: device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lk(g_ms_mu);
    if (g_ms_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        PA_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_match_scratch)));
        PA_REQUIRE(ptr != nullptr, "pa_match_prefixes: no address for the library's scratch array");
        g_ms_ptr[dev] = static_cast<pa::MatchScratch*>(ptr);
    }
    *out = g_ms_ptr[dev];
    return PA_OK;
}
}  // namespace

extern "C" int pa_match_prefixes(const pa_tree* tree, const int32_t* tokens, const int32_t* offsets, int B,
                                 int32_t* prefix_len, int32_t* slot_idx, void* stream) {
    const pa::DeviceTree* view = nullptr;
    int rc = pa_tree_device(tree, &view);
    if (rc != PA_OK) return rc;
    PA_REQUIRE(B >= 0, "pa_match_prefixes: B = %d", B);
    if (B == 0) return PA_OK;
    PA_REQUIRE(offsets && prefix_len, "pa_match_prefixes: offsets or prefix_len is NULL");
    // tokens / slot_idx may be NULL only if every prompt is empty (offsets[B] == 0), which the host cannot see
    // Several workgroups per request pay where a prompt's path has nodes in most of its windows.  Where the tree's edges
    // are longer than a window on average (a few long documents), a walk crosses whole windows inside one edge, compared
    // in one go by the workgroup that got there, and the others' work would only be waited for: one workgroup then.
    const bool multi = B <= pa::kMultiMaxB && static_cast<int64_t>(view->n_tokens) <= 4096ll * (view->n_nodes > 1 ? view->n_nodes - 1 : 1);
    pa::MatchScratch* scratch = nullptr;
    if (multi) {
        if ((rc = match_scratch_of_current_device(&scratch)) != PA_OK) return rc;
        scratch += g_ms_next.fetch_add(1) % pa::kScratchSets;
    }
    {
        pa::ProfScope prof(pa::kProfMatch, static_cast<hipStream_t>(stream));
        // Small batches: several workgroups per request.  Up to 256 requests: windows of 4,096 positions (every workgroup
        // has a compute unit of its own anyway).  Above: windows of 2,048, two workgroups per unit.
        if (multi)
            hipLaunchKernelGGL((pa::match_prefixes_pos_kernel<4, true>), dim3(B * pa::kMaxW), dim3(pa::kWin), 0,
                               static_cast<hipStream_t>(stream), *view, tokens, offsets, prefix_len, slot_idx, scratch);
        else if (B <= 256)
            hipLaunchKernelGGL((pa::match_prefixes_pos_kernel<4, false>), dim3(B), dim3(pa::kWin), 0, static_cast<hipStream_t>(stream),
                               *view, tokens, offsets, prefix_len, slot_idx, scratch);
        else
            hipLaunchKernelGGL((pa::match_prefixes_pos_kernel<2, false>), dim3(B), dim3(pa::kWin), 0, static_cast<hipStream_t>(stream),
                               *view, tokens, offsets, prefix_len, slot_idx, scratch);
    }
    PA_HIP(hipGetLastError());
    return PA_OK;
}
