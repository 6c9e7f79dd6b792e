// Extend attention on the bf16 matrix cores (MFMA 32x32x16, fp32 accumulate), gfx950.
//
// What is computed (Sec. 3.2 and Sec. 5 of the paper: only the missed tokens of a prompt
// are prefilled, the cached prefix KV is reused losslessly): extend row i of request r
// attends to the P_r prefix tokens, whose K/V rows are gathered from the paged pool
// through slot_idx, and causally to extend tokens 0..i.
//
// Decomposition.  The G = Hq/Hkv query heads of one KV head are packed with the extend
// rows into one row axis rho = i * G + (h mod G), so a K/V tile is read once per KV head.
// A workgroup of NW waves owns 32 * NW packed rows of one (request, KV head) and walks the
// key axis in tiles of kKT = 64 tokens: prefix positions first, then the extend tokens
// (the same loop; only the row address differs).  A planning kernel (extend_plan_kernel, one
// workgroup) builds the list of work items per launch - row tile x part of its key range - from
// the lengths on the device; the parts of a split tile are merged by a third kernel.
//
// Data movement.  K and V tiles go from global memory straight into LDS (16 bytes per
// lane, no register staging), one tile ahead of the arithmetic, into a ring of LDS
// buffers.  A wave's load lands as 1 KB of consecutive LDS bytes, so the bank-conflict
// swizzle is applied on the global-address side: the lane that owns LDS chunk c of a row
// fetches the row's chunk c ^ swizzle(row).
//
// MFMA formulation.  Scores are produced TRANSPOSED, S^T = K * Q^T, so that in the
// accumulator layout every lane holds one query row (column l % 32) and 16 of the 32
// keys of a block: row statistics of the online softmax are per-lane scalars plus one
// exchange between lane l and l ^ 32, and the probabilities are already laid out as the
// B operand of the second product O^T = V^T * P^T.  The V^T fragments are read from the
// row-major V tile with the transposing LDS read of gfx950.
//
// Two kinds of tile.  The general tile (general_block below) takes any mix of pool and extend rows, masks and
// ragged ends, and moves the running maximum; it runs for the first tile of a workgroup, where prefix and extend
// tokens meet, and on the causal diagonal.  Runs of consecutive tiles that need no mask (D = 128) execute as one
// assembly statement each (fast_run_d128.inc, written by gen_fast_run.py) with the running maximum frozen.
#include <hip/hip_bf16.h>

#include <atomic>
#include <cstdlib>
#include <mutex>
#include <type_traits>

#include "common.h"
#include "fp8_rows.h"

namespace pa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x32 __attribute__((ext_vector_type(32)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// fast_run_pool_d128 / fast_run_ext_d128: runs of steady-state tiles as assembly with fixed registers
#include "fast_run_d128.inc"

constexpr int kKT = 64;                  // key tokens per tile
constexpr int kStages = 2;               // LDS ring: one tile being read, one being filled
constexpr int kWgSlots = 512;            // workgroups resident at once: two on each of the 256 compute units
constexpr int kRounds = 2;               // the plan aims at about this many work items per workgroup slot (measured: with 3
                                         // long_doc_qa's kernel took 6 % longer - every item pays its start-up, its partial
                                         // results and their merge - with 1.5 its last round ran thin; the rest did not care)
constexpr int kRoundsStatic = 1;         // ... with the library's own scratch buffer as workspace (fewer partial results)
constexpr int kMinChunkTiles = 16;       // never split below this many key tiles (1,024 keys) per part (with 512 decode's
                                         // step took 3 % longer; nothing else splits that fine)
constexpr int kItemOverhead = 4;         // fixed cost of a work item, in key tiles (its prologue and epilogue)
constexpr int kMaxParts = 64;            // parts of one row tile at most
constexpr int kSortMax = 1024;           // up to this many requests are ordered (and their lengths staged in LDS)
constexpr int kTileLds = 3072;           // up to this many row tiles the planner keeps in LDS between its passes
constexpr int kPackMax = 256;            // batches of up to this many requests pack the left-over rows of requests
                                         // that share their prefix into common row tiles
constexpr int kPackMinPrefix = 512;      // ... if the shared prefix has at least this many keys
constexpr int kPackOwnCost = 2;          // ... and the members' own keys, which a shared tile walks in the general tile
                                         // for the few rows that see them, cost less than walking the prefix per member:
                                         // this factor x their sum <= (members - 1) x the shared prefix
constexpr float kRescaleThreshold = 8.f; // log2 units: the running maximum may lag the true one by this much
// The steady-state tiles (fast_run_*.inc) never move the running maximum: a run is left, for the general tile, when
// the probabilities of one lane and key block sum to more than 2^40.  The exponent range of fp32 and bf16 leaves that
// much room: a probability of 2^40 is as precise as one of 1, and what then underflows next to it is < 2^-100 of it.

struct ExtendPlan {
    int nw;          // waves per workgroup
    int rb;          // blocks of 32 packed rows per wave; a row tile has 32 * rb * nw packed rows
    int tiles_cap;   // upper bound on the number of (request, row tile) pairs
    int items_cap;   // upper bound on the number of work items (row tile x part of its key range)
    int parts_cap;   // upper bound on the number of items that belong to split tiles (they write partial results)
    int slots;       // workgroup slots per KV head
    int rounds;      // work items aimed at per workgroup slot
    int merge_cap;   // upper bound on the number of row tiles whose output rows are merged from partial results
    int pack;        // 1: left-over rows of requests with a common prefix may be packed (B <= kPackMax)
    int tile_parts;  // parts of one row tile at most
    size_t off_order, off_tile, off_aux, off_member, off_item, off_split, off_part_o, off_part_ml, total;
};

static inline size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

// Work list of one launch.  A row tile = up to 128 packed query rows (row = (extend token, query head of the group))
// of one request; a work item = a row tile x a contiguous part of its key range; one workgroup per (item, KV head).
// Workgroups cost about the same per key tile whatever the number of their rows, and the hardware starts them in
// index order as slots fall free, so the list is built for an even finish: requests with the same prefix together,
// the longest first, every tile cut into parts of about 1 / kRounds of a slot's share of the whole work.  (Cutting
// the end of the list finer still evens the finish further and was measured to gain nothing: while every slot is
// busy the chip is at its power limit, and the extra parts cost a merge.)  The bounds below follow from that rule
// (see extend_plan_kernel).
static ExtendPlan make_plan(int B, int64_t T, int64_t max_kv_len, int Hq, int Hkv, int D, int rounds = kRounds, int nw = 4) {
    ExtendPlan p{};
    p.rounds = rounds;
    const int G = Hq / Hkv;
    p.nw = nw;
    p.rb = 1;
    const int mt = 32 * p.rb * p.nw;
    const int64_t est = (T * G + mt - 1) / mt;
    p.pack = B <= kPackMax;
    p.tiles_cap = static_cast<int>(est + B);  // (packing only lowers the number of tiles)
    const int wg_slots = nw == 8 ? kWgSlots / 2 : kWgSlots;  // (workgroups of eight waves: one on a compute unit)
    p.slots = wg_slots / Hkv > 0 ? wg_slots / Hkv : 1;
    const int64_t by_rule = static_cast<int64_t>(p.slots) * rounds + 1;                  // sum of (parts - 1) over the tiles
    // (the key range of a shared tile holds the own keys of every member: of up to mt requests)
    const int64_t longest = p.pack ? max_kv_len * (B < mt ? (B > 0 ? B : 1) : mt) : max_kv_len;
    const int64_t per_tile = (longest / kKT) / kMinChunkTiles > 1 ? (longest / kKT) / kMinChunkTiles : 1;
    p.tile_parts = static_cast<int>(per_tile < kMaxParts ? per_tile : kMaxParts);
    const int64_t by_size = static_cast<int64_t>(p.tiles_cap) * p.tile_parts;
    p.items_cap = static_cast<int>(p.tiles_cap + (by_rule < by_size ? by_rule : by_size));
    const int64_t split_parts = 2 * by_rule < by_size ? 2 * by_rule : by_size;
    p.parts_cap = static_cast<int>(split_parts);
    p.merge_cap = static_cast<int>(split_parts / 2 + 1);
    p.off_order = 256;
    p.off_tile = p.off_order + up256(sizeof(int32_t) * (B > 0 ? B : 1));
    p.off_aux = p.off_tile + up256(sizeof(int4) * p.tiles_cap);
    p.off_member = p.off_aux + up256(sizeof(int4) * p.tiles_cap);
    p.off_item = p.off_member + up256(sizeof(int4) * 2 * (B > 0 ? B : 1));
    p.off_split = p.off_item + up256(sizeof(int4) * 3 * p.items_cap);
    p.off_part_o = p.off_split + up256(sizeof(int32_t) * (p.merge_cap + 1));
    const size_t units = static_cast<size_t>(p.parts_cap) * Hkv;
    p.off_part_ml = p.off_part_o + up256(units * mt * D * sizeof(float));
    p.total = p.off_part_ml + up256(units * mt * 2 * sizeof(float));
    return p;
}

constexpr int kPlanThreads = 1024;

// Exclusive prefix sums of up to three ints per thread over the workgroup of the planner (kPlanThreads threads):
// a shuffle scan inside each wave, then the 16 wave totals.  total[] receives the sums.
template <int N>
__device__ __forceinline__ void block_scan(int (&v)[N], int (&total)[N], int (*s_w)[kPlanThreads / 64 + 1]) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int x[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        x[i] = v[i];
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int y = __shfl_up(x[i], off);
            if (lane >= off) x[i] += y;
        }
    }
    __syncthreads();  // s_w may still be read from the call before
    if (lane == 63)
#pragma unroll
        for (int i = 0; i < N; ++i) s_w[i][w] = x[i];
    __syncthreads();
    if (tid < N) {
        int run = 0;
        for (int k = 0; k < kPlanThreads / 64; ++k) {
            const int c = s_w[tid][k];
            s_w[tid][k] = run;
            run += c;
        }
        s_w[tid][kPlanThreads / 64] = run;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < N; ++i) {
        v[i] = x[i] - v[i] + s_w[i][w];
        total[i] = s_w[i][kPlanThreads / 64];
    }
}

// ---------------------------------------------------------------------------------------
// The work list.  One workgroup.  hdr[0] = row tiles, hdr[1] = work items, hdr[2] = tiles to merge (listed in
// merge_tiles).
//   tile_tab[t] = (parts, index of its first partial result or -1, request, first packed row)
//   tile_aux[t] = (kind, first member, members, rows of the group)               (shared tiles; zeros otherwise)
//   item_tab[3 i ..] = (request, first packed row, first key, end key),
//                      (partial index or -1: writes the output, prefix length or common part, extend length or rows
//                       of the group, first extend token), (first slot-list entry, tile, first member, members or 0)
//   member_tab[2 m]     = (first row among the group's left-over rows, first extend token, first left-over row of
//                          the request, extend length)
//   member_tab[2 m + 1] = (keys of its prefix past the group's common part, its first slot-list entry, own keys
//                          (prefix part + extend tokens) of the group's members before it, 0)
// Everything a workgroup of the attention kernel needs sits in its item record: one dependent load, not four.
//
// Kinds of row tile.  Whole: rows of one request over all its keys.  With packing (B <= kPackMax, tables in LDS): the
// left-over rows of a request - those past its last full tile, fewer than a tile - cost a workgroup as much per
// key tile as a full tile, so where two or more requests share their whole prefix (at least kPackMinPrefix keys)
// their left-over rows are laid end to end and cut into shared tiles.  A shared tile walks the common prefix, every
// key of it visible to every row, and then the keys of each request that has rows in the tile, one request's
// after the other's, visible to that request's rows only (and causally).  Its members are the consecutive
// entries of member_tab whose rows meet the tile.
// Requests may also share only the first part of their prefixes (a decode batch: a common system and tool prompt, then
// tokens of each request's own).  Those whose rows make less than one tile, and whose whole prefix nobody shares, are
// grouped by the deepest of kProbes evenly spaced depths at which another such request has the same slot (slots name
// cached tokens: the same slot at a depth means the same tokens up to there); the group's common part is then
// measured exactly, by bisection over the slot lists against the group's first member.  A member's own keys in a
// shared tile are the rest of its prefix (pool rows through its own slot list) followed by its extend tokens.
// ---------------------------------------------------------------------------------------
constexpr int kTileWhole = 0, kTileShared = 1;

struct TileDesc {
    int kind, r, row0, kv_lo, kv_end, rows_total;  // rows_total: rows of the request, or of the group (shared)
    int member0, n_members;                        // shared tiles: the entries of member_tab whose rows meet the tile
    int common;                                    // shared tiles: keys that all members have in common
};

__global__ __launch_bounds__(kPlanThreads) void extend_plan_kernel(
    const int32_t* __restrict__ prefix_len, const int32_t* __restrict__ ext_len, const int32_t* __restrict__ ext_offsets,
    const int32_t* __restrict__ slot_offsets, const int32_t* __restrict__ slot_idx, int B, int G, int mt, int tiles_cap,
    int items_cap, int parts_cap, int merge_cap, int slot_items, int pack, int tile_parts, int32_t* __restrict__ hdr,
    int32_t* __restrict__ order, int4* __restrict__ tile_tab, int4* __restrict__ tile_aux, int4* __restrict__ member_tab,
    int4* __restrict__ item_tab, int32_t* __restrict__ merge_tiles) {
    __shared__ int s_w[3][kPlanThreads / 64 + 1];
    __shared__ int s_P[kSortMax], s_E[kSortMax];  // prefix and extend length of the request (staged when B <= kSortMax)
    __shared__ int s_key[kSortMax];               // keys of the request, prefix + extend length (-1: nothing to do)
    __shared__ int s_grp[kSortMax];               // slot of its last prefix token: equal for requests with the same prefix
    __shared__ int s_gkey[kSortMax];              // the most keys of any request of its group; later: first tile of a position
    __shared__ int s_order[kSortMax];             // position in the list -> request
    __shared__ int s_e0[kSortMax], s_so[kSortMax]; // first extend token and first slot-list entry of the request
    __shared__ int s_tpos[kTileLds];  // tile -> (list position << 12 | tile of the position)
    static_assert(kTileLds >= 3 * kSortMax, "the grouping borrows s_tpos");
    int* const s_first = s_tpos;               // first and middle slot of the request's prefix, the first request with
    int* const s_mid = s_tpos + kSortMax;      // the same prefix (before the tiles are laid out)
    int* const s_ldr = s_tpos + 2 * kSortMax;
    // packing (B <= kPackMax): per list position ...
    __shared__ int s_gid[kPackMax];     // its group (run of positions with the same prefix)
    __shared__ int s_R[kPackMax];       // first row of its left-over rows among the group's, -1: not packed
    __shared__ int s_nshared[kPackMax]; // shared tiles placed in front of its own tiles (the first position of a group)
    // ... and per group
    __shared__ int s_gn[kPackMax], s_gL[kPackMax];        // members, left-over rows
    __shared__ int s_gbase[kPackMax], s_gm0[kPackMax];    // rows / members of earlier groups
    __shared__ int s_gown0[kPackMax];                     // own keys of the members of earlier groups
    // ... and per member (packed request)
    __shared__ int s_mR[kPackMax], s_mE[kPackMax];        // first row among the group's left-over rows, keys of its own
    // ... and per request (B <= kPackMax)
    __shared__ int s_cut[kPackMax];                       // keys of its prefix that its group has in common
    __shared__ int s_kstar[kPackMax], s_lead[kPackMax], s_lcp[kPackMax];
    __shared__ int s_carry, s_maxP;
    const int tid = threadIdx.x;
    const bool staged = B <= kSortMax;
    auto P_of = [&](int r) { return staged ? s_P[r] : prefix_len[r]; };
    auto E_of = [&](int r) { return staged ? s_E[r] : ext_len[r]; };
    // Requests that share their whole prefix become neighbours (their workgroups then run at the same time and the
    // shared keys are served from L2); groups with the most keys first, inside a group the request with the most
    // keys first.  Beyond kSortMax requests the order stays as given.
    if (staged) {
        for (int r = tid; r < B; r += kPlanThreads) {
            const int P = prefix_len[r], so = slot_offsets[r];
            const int E = ext_len[r];
            s_P[r] = P;
            s_E[r] = E;
            s_key[r] = E > 0 ? P + E : -1;
            s_e0[r] = ext_offsets[r];
            s_so[r] = so;
            s_grp[r] = P > 0 ? slot_idx[so + P - 1] : -1 - r;
            s_first[r] = P > 0 ? slot_idx[so] : 0;
            s_mid[r] = P > 0 ? slot_idx[so + P / 2] : 0;
            s_ldr[r] = r;
        }
        __syncthreads();
        // Requests share their whole prefix if it has the same length and the same slots: the group is named by its
        // first request.  Slot lists that name the tokens of one prefix tree are equal as soon as their last slots
        // are; the length, the first and the middle slot are compared as well, so that lists of other origin that
        // merely end in the same slot stay apart.
        {
            const int tpr = max(1, kPlanThreads / B);
            const int r = tid / tpr, q_first = tid % tpr;
            if (r < B) {
                const int grp = s_grp[r], P = s_P[r], first = s_first[r], mid = s_mid[r];
                int lead = r;
#pragma unroll 4
                for (int q = q_first; q < r; q += tpr)
                    if (s_grp[q] == grp && s_P[q] == P && s_first[q] == first && s_mid[q] == mid) lead = min(lead, q);
                if (lead < r) atomicMin(&s_ldr[r], lead);
            }
            __syncthreads();
            for (int q = tid; q < B; q += kPlanThreads) s_grp[q] = s_ldr[q];  // (>= 0; a lone request names itself)
            __syncthreads();
        }
        if (pack && B <= kPackMax) {
            // groups of requests that share the first part of their prefixes (see above); four threads per request
            constexpr int kProbes = 12;
            static_assert(kProbes * kPackMax <= kTileLds, "the probes borrow s_tpos");
            int* s_probe = s_tpos;
            const int r = tid >> 2, sub = tid & 3;
            const bool on = r < B;
            auto sum4 = [](int x) { x += __shfl_xor(x, 1); return x + __shfl_xor(x, 2); };
            auto min4 = [](int x) { x = min(x, __shfl_xor(x, 1)); return min(x, __shfl_xor(x, 2)); };
            auto or4 = [](int x) { x |= __shfl_xor(x, 1); return x | __shfl_xor(x, 2); };  // (over a request's four threads)
            if (tid == 0) s_maxP = 0;
            if (on && sub == 0) s_cut[r] = s_P[r];
            __syncthreads();
            int same = 0;
            if (on)
#pragma unroll 8
                for (int q = sub; q < B; q += 4) same += s_grp[q] == s_grp[r];
            same = sum4(same);
            const bool cand = on && same == 1 && s_E[r] > 0 && s_E[r] * G < mt && s_P[r] >= kPackMinPrefix;
            if (cand && sub == 0) atomicMax(&s_maxP, s_P[r]);
            __syncthreads();
            const int maxP = s_maxP;
            if (maxP > 0) {  // (the same for every thread)
                const int ps = kPackMinPrefix * ((maxP + kProbes * kPackMinPrefix - 1) / (kProbes * kPackMinPrefix));
                if (on)
                    for (int k = sub; k < kProbes; k += 4) {
                        const int d = (k + 1) * ps;  // (who is no candidate, or shorter, matches nobody)
                        s_probe[r * kProbes + k] = cand && d <= s_P[r] ? slot_idx[s_so[r] + d - 1] : -1 - r;
                    }
                __syncthreads();
                // The deepest depth at which another candidate has the same slot.  Equal slots at a depth mean equal slots
                // at every depth above it: another request only matters if it also matches at the first depth not
                // matched so far.
                int depths = 0;
                if (cand)
                    for (int q0 = sub; q0 < B; q0 += 32) {  // eight other requests at a time
                        bool deeper = depths < kProbes;
                        while (deeper) {
                            const int mine = s_probe[r * kProbes + depths];
                            deeper = false;
#pragma unroll
                            for (int u = 0; u < 8; ++u) {  // (loads first, all of them; then the tests)
                                const int q = q0 + 4 * u;
                                const int theirs = s_probe[min(q, B - 1) * kProbes + depths];
                                deeper |= (q < B) & (q != r) & (theirs == mine);
                            }
                            depths += deeper;
                            deeper = deeper && depths < kProbes;
                        }
                    }
                depths = max(depths, __shfl_xor(depths, 1));
                depths = max(depths, __shfl_xor(depths, 2));
                const int kstar = depths - 1;
                if (on && sub == 0) s_kstar[r] = kstar;
                __syncthreads();
                // the group: the candidates that chose this depth and have this slot there; its first member leads
                int lead = B, members = 0;
                if (kstar >= 0) {
                    const int mine = s_probe[r * kProbes + kstar];
#pragma unroll 8
                    for (int q = sub; q < B; q += 4) {
                        const bool with_me = (s_kstar[q] == kstar) & (s_probe[q * kProbes + kstar] == mine);
                        lead = with_me ? min(lead, q) : lead;
                        members += with_me;
                    }
                }
                lead = min4(lead);
                members = sum4(members);
                const bool grouped = kstar >= 0 && members >= 2;
                int lcp = 0;
                if (grouped) {
                    // The slot lists agree on [0, lo); they differ at hi, or hi is where the shorter one (or the probe
                    // interval) ends.  The request's four threads look at four places between lo and hi at once.
                    const int d = (kstar + 1) * ps;
                    int lo = d, hi = min(min(s_P[r], s_P[lead]), d + ps);
                    const int32_t* a = slot_idx + s_so[r];
                    const int32_t* b = slot_idx + s_so[lead];
                    while (r != lead && lo < hi) {
                        const int span = hi - lo;
                        auto place = [&](int j) { return lo + static_cast<int>(static_cast<int64_t>(span) * (j + 1) / 5); };
                        const int x = place(sub);  // lo <= x < hi
                        const int first_off = __ffs(~or4((a[x] == b[x]) << sub) & 0xF) - 1;  // first place that differs, -1: none
                        const int new_lo = first_off == 0 ? lo : place((first_off < 0 ? 4 : first_off) - 1) + 1;
                        hi = first_off < 0 ? hi : place(first_off);
                        lo = new_lo;
                    }
                    lcp = hi;
                }
                if (on && sub == 0) {
                    s_lcp[r] = lcp;
                    s_lead[r] = grouped ? lead : -1;
                }
                __syncthreads();
                if (grouped) {
                    int cut = 0x7fffffff;
#pragma unroll 8
                    for (int q = sub; q < B; q += 4) {
                        const int theirs = s_lcp[q];
                        cut = s_lead[q] == lead ? min(cut, theirs) : cut;
                    }
                    cut = min4(cut);
                    // (lists of one prefix tree agree on [0, cut) once they agree at cut - 1; for lists of other origin
                    // three more places are compared, and a request that differs there stays on its own)
                    const int32_t* a = slot_idx + s_so[r];
                    const int32_t* b = slot_idx + s_so[lead];
                    const int at = sub == 0 ? 0 : sub == 1 ? cut / 3 : sub == 2 ? (2 * cut) / 3 : cut - 1;
                    const bool agree = or4((cut > 0 && a[at] != b[at]) ? 1 : 0) == 0;
                    if (sub == 0 && agree) {
                        s_cut[r] = cut;
                        s_grp[r] = -1 - lead;  // (no whole-prefix group has a negative name)
                    }
                }
                __syncthreads();
            }
        }
        // tpr threads per request r, each over its share of the other requests q
        const int tpr = max(1, kPlanThreads / B);
        const int r = tid / tpr, q_first = tid % tpr;
        const bool on = r < B;
        const int k = on ? s_key[r] : 0, grp = on ? s_grp[r] : 0;
        if (on && q_first == 0) {
            s_gkey[r] = k;
            s_order[r] = 0;  // (the rank of r is summed up here first)
        }
        __syncthreads();
        if (on) {
            int gk = -1;
#pragma unroll 8
            for (int q = q_first; q < B; q += tpr) {
                const int kq = s_key[q], gq = s_grp[q];
                gk = max(gk, gq == grp ? kq : -1);
            }
            atomicMax(&s_gkey[r], gk);
        }
        __syncthreads();
        int rank = 0;
        if (on) {
            const int gk = s_gkey[r];
#pragma unroll 8
            for (int q = q_first; q < B; q += tpr) {
                const int kq = s_key[q], gq = s_grp[q], gkq = s_gkey[q];
                // (group keys, group, keys, index) of q sorts before that of r: more keys first, lower ids first
                rank += (gkq > gk) | ((gkq == gk) & ((gq < grp) | ((gq == grp) & ((kq > k) | ((kq == k) & (q < r))))));
            }
            atomicAdd(&s_order[r], rank);
        }
        __syncthreads();
        if (on && q_first == 0) rank = s_order[r];
        __syncthreads();
        if (on && q_first == 0) s_order[rank] = r;
    } else {
        for (int r = tid; r < B; r += kPlanThreads) order[r] = r;
    }
    if (tid == 0) s_carry = 0;
    __syncthreads();
    // With few requests and few row tiles the passes below work on LDS copies; otherwise on the table in global
    // memory.
    const bool in_lds = staged && tiles_cap <= kTileLds;
    const bool packing = in_lds && pack && B <= kPackMax;
    int n_tiles;
    bool tiles_over;  // more row tiles than the launch was sized for: ext_len on the device exceeds the host's T
    if (in_lds) {
        // one thread per list position (B <= kPlanThreads here)
        const bool on = tid < B;
        const int r = on ? s_order[tid] : 0;
        const int P = on ? s_P[r] : 0, E = on ? s_E[r] : 0;
        const int rows = max(E, 0) * G, full = rows / mt, left = rows - full * mt;
        int nshared = 0;
        bool packed_me = false;  // this request's left-over rows go into shared tiles
        if (packing) {
            // groups: runs of positions with the same prefix
            const bool head = on && (tid == 0 || s_grp[s_order[tid - 1]] != s_grp[r]);
            if (tid < kPackMax) {
                s_gn[tid] = 0;
                s_gL[tid] = 0;
                s_gown0[tid] = 0;  // (first the sum of the group's own keys, later those of the groups before it)
            }
            int v[1] = {head ? 1 : 0}, total[1];
            block_scan<1>(v, total, s_w);
            const int gid = v[0] + (head ? 1 : 0) - 1;  // (block_scan ends with a barrier: the zeros above are in place)
            const int cut = on ? s_cut[r] : 0;  // (the whole prefix, unless the group shares only a first part of it)
            const bool cand = on && left > 0 && cut >= kPackMinPrefix;
            if (on) s_gid[tid] = gid;
            if (cand) {
                atomicAdd(&s_gn[gid], 1);
                atomicAdd(&s_gown0[gid], P - cut + E);
            }
            __syncthreads();
            // (requests with long extends behind a short common prefix stay on their own)
            const bool packed = cand && s_gn[gid] >= 2 &&
                                static_cast<int64_t>(kPackOwnCost) * s_gown0[gid] <= static_cast<int64_t>(s_gn[gid] - 1) * cut;
            packed_me = packed;
            int v2[3] = {packed ? left : 0, packed ? 1 : 0, packed ? P - cut + E : 0}, total2[3];
            block_scan<3>(v2, total2, s_w);
            if (head) {
                s_gbase[gid] = v2[0];
                s_gm0[gid] = v2[1];
                s_gown0[gid] = v2[2];
            }
            if (packed) atomicAdd(&s_gL[gid], left);
            __syncthreads();
            if (on) s_R[tid] = packed ? v2[0] - s_gbase[gid] : -1;
            if (packed) {
                member_tab[2 * v2[1]] = make_int4(v2[0] - s_gbase[gid], s_e0[r], full * mt, E);
                member_tab[2 * v2[1] + 1] = make_int4(P - cut, s_so[r], v2[2] - s_gown0[gid], 0);
                s_mR[v2[1]] = v2[0] - s_gbase[gid];
                s_mE[v2[1]] = P - cut + E;
            }
            if (head && s_gn[gid] >= 2) nshared = (s_gL[gid] + mt - 1) / mt;
            if (on) s_nshared[tid] = nshared;
        }
        int v[1] = {on ? nshared + full + (left > 0 && !packed_me ? 1 : 0) : 0}, total[1];
        block_scan<1>(v, total, s_w);
        if (on) s_gkey[tid] = v[0];  // (s_gkey is free again: the first tile of the position)
        __syncthreads();
        tiles_over = total[0] > tiles_cap;
        n_tiles = min(total[0], tiles_cap);
        for (int t = tid; t < n_tiles; t += kPlanThreads) {
            int lo = 0, hi = B;  // the last position whose first tile is <= t
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_gkey[mid] <= t) lo = mid; else hi = mid;
            }
            s_tpos[t] = (lo << 12) | (t - s_gkey[lo]);
        }
        __syncthreads();
    } else {
        for (int base = 0; base < B; base += kPlanThreads) {
            const int k = base + tid;
            int cnt = 0, r = 0;
            if (k < B) {
                r = staged ? s_order[k] : order[k];
                const int e = E_of(r);
                cnt = e > 0 ? (e * G + mt - 1) / mt : 0;
            }
            int v[1] = {cnt}, total[1];
            block_scan<1>(v, total, s_w);
            const int start = s_carry + v[0];
            for (int j = 0; j < cnt; ++j)  // a request's last rows - the most keys - first
                if (start + j < tiles_cap) tile_tab[start + j] = make_int4(1, -1, r, (cnt - 1 - j) * mt);
            __syncthreads();
            if (tid == 0) s_carry += total[0];
            __syncthreads();
        }
        tiles_over = s_carry > tiles_cap;
        n_tiles = min(s_carry, tiles_cap);
    }
    // what tile t is
    auto describe = [&](int t) {
        TileDesc d{};
        if (in_lds) {
            const int pos = s_tpos[t] >> 12;
            int j = s_tpos[t] & 0xFFF;
            const int r = s_order[pos];
            const int P = s_P[r], rows = s_E[r] * G, full = rows / mt;
            d.r = r;
            const int nshared = packing ? s_nshared[pos] : 0;
            if (j < nshared) {  // a shared tile of the group this position heads
                const int gid = s_gid[pos];
                const int m0 = s_gm0[gid], nm = s_gn[gid], L = s_gL[gid];
                d.kind = kTileShared;
                d.row0 = j * mt;
                d.rows_total = L;
                // the members whose rows meet rows [row0, row_end): the one holding row0 ... the one holding row_end - 1
                const int row_end = min(L, d.row0 + mt);
                int ka = 0, kb = 0;
                for (int k = 0; k < nm; ++k) {
                    ka = s_mR[m0 + k] <= d.row0 ? k : ka;
                    kb = s_mR[m0 + k] <= row_end - 1 ? k : kb;
                }
                int own = 0;
                for (int k = ka; k <= kb; ++k) own += s_mE[m0 + k];
                d.member0 = m0 + ka;
                d.n_members = kb - ka + 1;
                d.kv_lo = 0;
                d.common = s_cut[r];
                d.kv_end = d.common + own;
                return d;
            }
            j -= nshared;
            d.rows_total = rows;
            d.kv_lo = 0;
            d.kind = kTileWhole;
            // the request's last rows - the most keys - first: its left-over rows, if they were not packed, then the
            // full tiles from the last one down
            const bool own_left = rows > full * mt && !(packing && s_R[pos] >= 0);
            if (own_left) {
                if (j == 0) {
                    d.row0 = full * mt;
                    d.kv_end = P + (rows - 1) / G + 1;
                    return d;
                }
                --j;
            }
            d.row0 = (full - 1 - j) * mt;
            d.kv_end = P + (d.row0 + mt - 1) / G + 1;
            return d;
        }
        const int4 tt = tile_tab[t];
        d.kind = kTileWhole;
        d.r = tt.z;
        d.row0 = tt.w;
        d.rows_total = E_of(tt.z) * G;
        d.kv_lo = 0;
        d.kv_end = P_of(tt.z) + (tt.w + min(mt, d.rows_total - tt.w) - 1) / G + 1;
        return d;
    };
    // cost of a tile = its key tiles + a fixed overhead; thread i owns tiles [i * per, (i + 1) * per)
    const int per = (n_tiles + kPlanThreads - 1) / kPlanThreads;
    const int t_lo = min(n_tiles, tid * per), t_hi = min(n_tiles, t_lo + per);
    // (the three passes below look at the same tiles; the first of a thread's - with up to 1,024 tiles its only one -
    // is worked out once)
    const TileDesc d_first = t_lo < t_hi ? describe(t_lo) : TileDesc{};
    auto tile_desc = [&](int t) { return t == t_lo ? d_first : describe(t); };
    int my_cost = 0;
    for (int t = t_lo; t < t_hi; ++t) {
        const TileDesc d = tile_desc(t);
        my_cost += (d.kv_end - d.kv_lo + kKT - 1) / kKT + kItemOverhead;
    }
    int W;
    {
        int v[1] = {my_cost}, total[1];
        block_scan<1>(v, total, s_w);
        W = total[0];
    }
    // parts of a tile: its cost over the target cost of an item, rounded up from a quarter past a whole number (an item
    // of 1.5 targets at the end of the list is a tail of its own); never below kMinChunkTiles key tiles per part.
    // Summed over the tiles, parts - 1 stays below W / target = slot_items = slots * rounds (a tile of cost c adds at most
    // c / target - 1/4), which is what the capacities are sized for.
    const float target = fmaxf(static_cast<float>(W) / static_cast<float>(slot_items), 1.f);
    auto parts_of = [&](int K) {
        int n = static_cast<int>(static_cast<float>(K + kItemOverhead) / target + 0.75f);
        n = min(min(n, K / kMinChunkTiles), tile_parts);
        return max(n, 1);
    };
    // a tile's output rows come from partial results, joined by the merge kernel, if it is split
    int my_items = 0, my_parts = 0, my_merge = 0;
    for (int t = t_lo; t < t_hi; ++t) {
        const TileDesc d = tile_desc(t);
        const int n = parts_of((d.kv_end - d.kv_lo + kKT - 1) / kKT);
        my_items += n;
        my_parts += n > 1 ? n : 0;
        my_merge += n > 1;
    }
    int base3[3] = {my_items, my_parts, my_merge}, total3[3];
    block_scan<3>(base3, total3, s_w);
    int item0 = base3[0], part0 = base3[1], merge0 = base3[2];
    const int n_items = total3[0], n_merge = total3[2];
    // The capacities follow from the host's T and max_kv_len: a batch on the device that is larger than they say does
    // not fit.  Nothing is computed then (an empty list: no output row is written) and hdr[3] says so, which
    // pa_extend_status reports.
    const bool overflow = tiles_over || n_items > items_cap || total3[1] > parts_cap || n_merge > merge_cap;
    for (int t = t_lo; t < t_hi && !overflow; ++t) {
        const TileDesc d = tile_desc(t);
        const int K = (d.kv_end - d.kv_lo + kKT - 1) / kKT;
        const int n = parts_of(K);
        const bool partial = n > 1;
        tile_tab[t] = make_int4(n, partial ? part0 : -1, d.r, d.row0);
        tile_aux[t] = make_int4(d.kind, d.member0, d.n_members, d.kind == kTileShared ? d.rows_total : 0);
        if (partial) merge_tiles[merge0++] = t;
        const int r = d.r;
        const int e0 = staged ? s_e0[r] : ext_offsets[r];
        const int slot_off = staged ? s_so[r] : slot_offsets[r];
        const int P = d.kind == kTileShared ? d.common : P_of(r);
        const int e_or_rows = d.kind == kTileShared ? d.rows_total : E_of(r);
        for (int j = 0; j < n; ++j) {
            // (K < 2^24 key tiles and n <= 64 parts: the products fit 32 bits)
            const int lo = d.kv_lo + static_cast<int>(static_cast<unsigned>(K) * static_cast<unsigned>(j) / static_cast<unsigned>(n)) * kKT;
            const int hi = min(d.kv_end, d.kv_lo + static_cast<int>(static_cast<unsigned>(K) * static_cast<unsigned>(j + 1) / static_cast<unsigned>(n)) * kKT);
            int4* rec = item_tab + 3 * static_cast<size_t>(item0 + j);
            rec[0] = make_int4(r, d.row0, lo, hi);
            rec[1] = make_int4(partial ? part0 + j : -1, P, e_or_rows, e0);
            rec[2] = make_int4(slot_off, t, d.member0, d.n_members);
        }
        item0 += n;
        part0 += partial ? n : 0;
    }
    if (tid == 0) {
        hdr[0] = overflow ? 0 : n_tiles;
        hdr[1] = overflow ? 0 : n_items;
        hdr[2] = overflow ? 0 : n_merge;
        hdr[3] = overflow;
    }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    // round to nearest even; inputs are finite probabilities or outputs
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 v = {a, b};
    bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}

// XOR swizzles of the 16-byte chunks of a K/V row in LDS, chosen so that the two read patterns of the
// arithmetic are free of bank conflicts for 256-byte rows: K is read 16 bytes per lane down 16
// consecutive rows, V is read 8 bytes per lane across 64 bytes of 4 consecutive rows.
template <int D>
__device__ __forceinline__ int swz_k(int row) {
    return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D>
__device__ __forceinline__ int swz_v(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

// The V^T fragments come from the transposing LDS read ds_read_b64_tr_b16: within each group of 16 lanes the
// 16 x 4 16-bit values addressed by the lanes form a flat array F (lane-major); lane i of the group receives
// F[i], F[16 + i], F[32 + i], F[48 + i].

// Both halves of a query row (lanes l and l ^ 32) combined, in every lane, without going through LDS.
// v_permlane32_swap exchanges lanes 32..63 of its first operand with lanes 0..31 of its second: fed the
// same value x twice it leaves (x of the low half, x of the high half) in every lane.  Written as
// inline assembly (the compiler builtin folded its two results into one); the s_nop pairs cover the
// wait states the instruction needs after a VALU write of its operands and before a VALU read of them.
__device__ __forceinline__ void row_halves(float x, float& lo, float& hi) {
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    lo = a;
    hi = b;
}
__device__ __forceinline__ float row_max(float x) {
    float lo, hi;
    row_halves(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float row_sum(float x) {
    float lo, hi;
    row_halves(x, lo, hi);
    return lo + hi;
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence would make the compiler wait
// for every outstanding global->LDS load, including the ones meant to stay in flight.  Completion of
// the loads that must be visible is awaited explicitly (wait_vm_all) before the barrier.
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
// s_waitcnt vmcnt(0) (expcnt and lgkmcnt left alone), as the builtin so that the compiler's own wait
// bookkeeping sees it and does not repeat it later.
__device__ __forceinline__ void wait_vm_all() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");
}

// Direct global -> LDS load of 16 bytes per lane: lane l of the wave writes LDS bytes
// [lds_addr + 16 l, lds_addr + 16 l + 16) with the 16 bytes at its own global address g.  lds_addr is
// wave-uniform.  Issued as inline assembly so that the compiler does not see an LDS store in flight: it
// would otherwise wait for it before every later LDS read, and the load could not overlap the
// arithmetic on the other ring slot.  The explicit wait_vm_all() + wg_barrier() order it instead.
__device__ __forceinline__ void load_to_lds_16(const void* g, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory");
}
// The same with the global address given as a wave-uniform base plus a 32-bit unsigned byte offset per lane.
__device__ __forceinline__ void load_to_lds_16(const void* base, unsigned off, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_addr) : "memory");
}
// One byte per lane: lane l of the wave writes the 32-bit word at lds_addr + 4 l (the byte in its low 8 bits).
__device__ __forceinline__ void load_to_lds_1(const void* g, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_ubyte %0, off" ::"v"(g), "s"(lds_addr) : "memory");
}
__device__ __forceinline__ unsigned lds_address(const void* p) {
    return static_cast<unsigned>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const unsigned char*)(p)));
}

// KV8: the pool holds one-byte codes and row exponents (fp8_rows.h) instead of bfloat16; its rows are decoded into the
// bfloat16 tiles in LDS, and everything from there on is the same arithmetic.
template <int D, int NW, int RB, bool KV8>
__global__ __launch_bounds__(NW * 64, RB == 1 && NW == 4 ? 2 : 1) void extend_bf16_kernel(
    const __hip_bfloat16* __restrict__ q_ext, const __hip_bfloat16* __restrict__ k_ext,
    const __hip_bfloat16* __restrict__ v_ext, const __hip_bfloat16* __restrict__ pool, const signed char* __restrict__ pool_exp,
    const int32_t* __restrict__ slot_idx, int Hq, int Hkv, int page_size, int page_shift, unsigned page_magic,
    int page_mshift, int num_slots, int fast_ok, float scale_log2e, __hip_bfloat16* __restrict__ out, const int32_t* __restrict__ hdr,
    const int4* __restrict__ item_tab, const int4* __restrict__ member_tab, float* __restrict__ part_o,
    float* __restrict__ part_ml, unsigned long long* __restrict__ clk) {
    constexpr int WR = 32 * RB;              // packed query rows per wave (RB blocks of 32)
    constexpr int MT = WR * NW;              // packed query rows per workgroup
    constexpr int NB = D / 32;               // MFMA row blocks of the head dimension in O^T
    constexpr int KS = D / 16;               // k-slices of the QK^T product
    constexpr int CPR = D / 8;               // 16-byte chunks per K/V row
    constexpr int ROWB = D * 2;              // bytes per row
    constexpr int TILEB = kKT * ROWB;        // bytes of one K (or V) tile
    constexpr int STAGEB = 2 * TILEB;        // one ring slot: K tile, V tile
    constexpr int RPB = 1024 / ROWB;         // rows per 1 KB block (what one wave-wide 16-byte load fills)
    constexpr int UPW = kKT / RPB / NW;      // blocks per wave, tile and tensor
    static_assert(UPW >= 1, "tile too small for this many waves");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [kStages][K tile | V tile]

    // block -> (work item, kv head); the kv head varies fastest so that with 8 kv heads every XCD (blocks are
    // dealt round-robin to the 8 XCDs) serves one head and keeps its shared prefixes in L2
    const int g = blockIdx.x % Hkv;
    const int item = blockIdx.x / Hkv;
    if (item >= hdr[1]) return;
#ifdef PA_PROBE_DETAIL
    // (build option for experiments: where a workgroup's cycles go - clk[2..7] = cycles in runs of assembly tiles, tiles
    // done there, cycles in general tiles, their number, cycles before the key loop, cycles after it)
    const long long probe_t0 = clk ? clock64() : 0;
    long long probe_fast = 0, probe_gen = 0, probe_gen_issue = 0, probe_gen_math = 0, probe_single = 0, probe_single_issue = 0, probe_landed = 0;
    int probe_nfast = 0, probe_ngen = 0, probe_nsingle = 0;
#endif
    const int4 rec0 = item_tab[3 * static_cast<size_t>(item)], rec1 = item_tab[3 * static_cast<size_t>(item) + 1];
    const int4 rec2 = item_tab[3 * static_cast<size_t>(item) + 2];
    const int slot_off = rec2.x;
    const int row0 = rec0.y, kv_lo = rec0.z, kv_hi = rec0.w;
    const int part = rec1.x;  // index of this item's partial result; -1: the item covers all keys and writes the output
    const int P = rec1.y;  // keys of the prefix; in a shared tile: of the part of it that all members have in common
    const int G = Hq / Hkv;
    // a shared tile: left-over rows of n_members requests with this prefix, laid end to end; after the common keys
    // come the members' own: the rest of a member's prefix (if the group shares only a first part), then its extend
    // tokens; member after member
    const int member0 = __builtin_amdgcn_readfirstlane(rec2.z), n_members = __builtin_amdgcn_readfirstlane(rec2.w);
    const bool shared = n_members > 0;
    const int rows_total = shared ? rec1.z : rec1.z * G;
    const int rows_here = min(MT, rows_total - row0);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hh = lane >> 5;
    const int64_t e0 = rec1.w;
    const int32_t* __restrict__ slots = slot_idx + slot_off;

    // this lane's query rows: one per row block
    const bool wave_on = wave * WR < rows_here;
    // (the rows of a shared tile are their requests' last ones: no tile of its key range is skipped)
    const int wave_i_last = shared ? max(0, kv_hi - P) : (row0 + min(rows_here, wave * WR + WR) - 1) / G;
    bool row_ok[RB];
    int qi[RB], qh[RB];          // extend index and query head of the row
    int vis_end[RB];             // keys [.., vis_end) are visible to the row ...
    int vis_lo[RB];              // ... except, in a shared tile, the other members' extend tokens [P, vis_lo)
    int64_t e0_row[RB];          // first extend token of the row's request
    int blk_vis_min[RB];         // every row of the block sees keys [.., this)
    bool own_prefix = false;     // shared tile: some member has prefix keys of its own (uniform)
    // the members of a shared tile: where a member's own keys begin on the tile's key axis (and, one past the last
    // member, where they end), how many of them are prefix keys, its first slot-list entry, its first extend token
    // counted from this item's
    // (behind the K/V ring in the dynamic LDS, which thereby keeps its alignment)
    int* const s_mseg = reinterpret_cast<int*>(smem + kStages * STAGEB);
    int* const s_mown = s_mseg + (MT + 1);
    int* const s_mso = s_mown + MT;
    int* const s_mx0 = s_mso + MT;
    int* const s_wave_own = s_mx0 + MT;  // per wave: the key range that holds the own keys of its rows' members
    if (shared) {
        if (tid < n_members) {  // (a member has at least one row in the tile: there are at most MT)
            const int4 mem = member_tab[2 * (member0 + tid)], aux = member_tab[2 * (member0 + tid) + 1];
            const int at = P + aux.z - member_tab[2 * member0 + 1].z;
            s_mseg[tid] = at;
            s_mown[tid] = aux.x;
            s_mso[tid] = aux.y;
            s_mx0[tid] = mem.y - static_cast<int>(rec1.w);
            if (tid == n_members - 1) s_mseg[n_members] = at + aux.x + mem.w;
        }
        __syncthreads();
    }
    bf16x8 qreg[RB][KS];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        int rho = row0 + wave * WR + rb * 32 + n;
        row_ok[rb] = rho < rows_total;
        e0_row[rb] = e0;
        vis_lo[rb] = P;
        int own_row = 0;  // prefix keys of the row's request past the common part
        if (shared) {
            // whose row this is: the last member that starts at or before it; its place in that request; where
            // that member's extend tokens begin on the tile's key axis
            const int want = row_ok[rb] ? rho : member_tab[2 * member0].x;
            for (int k = 0; k < n_members; ++k) {
                const int4 mem = member_tab[2 * (member0 + k)];  // (same address in every lane)
                const int own = s_mown[k];
                own_prefix |= own > 0;
                if (mem.x <= want) {
                    e0_row[rb] = mem.y;
                    rho = mem.z + (want - mem.x);
                    vis_lo[rb] = s_mseg[k];
                    own_row = own;
                }
            }
        }
        qi[rb] = row_ok[rb] ? rho / G : 0;
        qh[rb] = g * G + (row_ok[rb] ? rho % G : 0);
        vis_end[rb] = min(kv_hi, vis_lo[rb] + own_row + qi[rb] + 1);
        blk_vis_min[rb] = shared ? min(kv_hi, P) : min(kv_hi, P + (row0 + wave * WR + rb * 32) / G + 1);
        const uint4* qp = reinterpret_cast<const uint4*>(q_ext + ((e0_row[rb] + qi[rb]) * Hq + qh[rb]) * static_cast<int64_t>(D));
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row_ok[rb]) v = qp[2 * s + hh];
            qreg[rb][s] = __builtin_bit_cast(bf16x8, v);
        }
    }

    // In a shared tile the keys past the common part concern one member each: the wave skips the arithmetic of a tile
    // that holds no key of the members its rows belong to (uniform over the wave).
    if (shared) {
        int wave_own_lo = 0x7fffffff, wave_own_hi = 0;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            wave_own_lo = min(wave_own_lo, vis_lo[rb]);
            wave_own_hi = max(wave_own_hi, vis_end[rb]);
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            wave_own_lo = min(wave_own_lo, __shfl_xor(wave_own_lo, off));
            wave_own_hi = max(wave_own_hi, __shfl_xor(wave_own_hi, off));
        }
        if (lane == 0) {  // (kept in LDS, not in registers: read, by this wave only, in the own-key part of a shared tile)
            s_wave_own[2 * wave] = wave_own_lo;
            s_wave_own[2 * wave + 1] = wave_own_hi;
        }
    }
    auto has_own_prefix = [&]() __attribute__((always_inline)) { return own_prefix; };

    // ---- global -> LDS tile loads.  Wave w fills blocks w * UPW + u: rows blk * RPB + lane / CPR, and the
    // lane lands on chunk position lane % CPR of its row.
    const int ld_pos = lane % CPR;
    const int ld_rowl = lane / CPR;
    const unsigned char* pool_g = reinterpret_cast<const unsigned char*>(pool) + static_cast<size_t>(g) * page_size * ROWB;
    const unsigned page_stride = 2u * Hkv * page_size * ROWB;  // bytes from one page to the next (< 4 GB, checked on the host)
    const unsigned v_off32 = static_cast<unsigned>(Hkv) * page_size * ROWB;      // from a K row to its V row
    const unsigned char* kx_g = reinterpret_cast<const unsigned char*>(k_ext) + (e0 * Hkv + g) * static_cast<int64_t>(ROWB);
    const unsigned char* vx_g = reinterpret_cast<const unsigned char*>(v_ext) + (e0 * Hkv + g) * static_cast<int64_t>(ROWB);
    const size_t x_stride = static_cast<size_t>(Hkv) * ROWB;  // bytes from one extend token to the next
    const unsigned smem_addr = __builtin_amdgcn_readfirstlane(lds_address(smem));
    int32_t sl_next[UPW];  // pool slots of the rows this lane loads in the tile after the one in flight

    // (first member of a shared tile whose own keys reach the tile asked for; the tiles are asked for in order)
    int cur_member = 0;
    auto member_at = [&](int cur, int p) __attribute__((always_inline)) {  // the member whose own keys hold key p >= P
        int k = cur;
        while (k + 1 < n_members && p >= s_mseg[k + 1]) ++k;
        return k;
    };
    auto load_slots = [&](int p0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            // positions past the end of the key range repeat the last valid one (see issue_tile)
            const int p = min(p0 + (wave * UPW + u) * RPB + ld_rowl, kv_hi - 1);
            int32_t sl = p < P ? slots[p] : 0;
            if (p >= P && has_own_prefix()) {
                // a key of some member's own: of its prefix (then its slot comes from its own list) or an extend token
                const int k = member_at(cur_member, p);  // (slots are asked for ahead of the tile being issued)
                const int q = p - s_mseg[k];
                if (q < s_mown[k]) sl = slot_idx[s_mso[k] + P + q];
            }
            sl_next[u] = sl;
        }
    };
    // Byte offset, inside its K (V) row, of the 16 bytes this lane fetches for block u.  Block u of the wave holds
    // rows 16 w + 4 u + lane / 16 (D = 128), so its swizzle differs from that of block 0 by an XOR with 4 u (K) or
    // u (V); for D = 64 (rows 16 w + 8 u + lane / 8) by an XOR with 4 u (K) or 2 u (V).
    const unsigned ld_koff0 = (ld_pos ^ swz_k<D>(wave * UPW * RPB + ld_rowl)) * 16;
    const unsigned ld_voff0 = (ld_pos ^ swz_v<D>(wave * UPW * RPB + ld_rowl)) * 16;
    // (Worked out where they are used, from a value the compiler cannot see through: left to itself it keeps all eight
    // of them as 64-bit addends, spills them, and each reload waits for the tile load issued just before it - eight
    // loads in a row, one memory round trip each.)
    auto opaque = [](unsigned x) __attribute__((always_inline)) {
        asm volatile("" : "+v"(x));
        return x;
    };
    auto ld_koff = [&](int u) __attribute__((always_inline)) { return opaque(ld_koff0) ^ (64u * u); };
    auto ld_voff = [&](int u) __attribute__((always_inline)) { return opaque(ld_voff0) ^ ((D == 128 ? 16u : 32u) * u); };
    // The next tile's loads, general: every lane takes its row from the pool (through the slot prefetched for it) or
    // from the extend tensors, by position; rows past the end of the key range repeat the last valid row (finite
    // values that the mask zeroes).  The page of a slot: a shift where the page size is a power of two
    // (page_shift >= 0), otherwise the exact quotient by a multiplication (see page_divider).
    auto issue = [&](int p0, int ring) __attribute__((always_inline)) {
        const unsigned sk = __builtin_amdgcn_readfirstlane(smem_addr + ring * STAGEB);  // wave-uniform (goes to M0)
        if (shared)
            while (cur_member + 1 < n_members && s_mseg[cur_member + 1] <= p0) ++cur_member;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int blk = wave * UPW + u;
            const int p = min(p0 + blk * RPB + ld_rowl, kv_hi - 1);
            bool ext = p >= P;
            const unsigned sl = static_cast<unsigned>(min(max(sl_next[u], 0), num_slots - 1));  // never outside the pool
            const unsigned pg = page_shift >= 0 ? sl >> page_shift : __umulhi(sl, page_magic) >> page_mshift;
            const size_t pool_off = static_cast<size_t>(pg) * page_stride +
                                    (sl - pg * static_cast<unsigned>(page_size)) * static_cast<unsigned>(ROWB);
            int64_t xrow = p - P;  // extend token, counted from the first one of the request of this item
            if (shared && ext) {
                // the member whose extend tokens hold key p, and that token relative to e0
                const int k = member_at(cur_member, p);
                const int q = p - s_mseg[k], own = s_mown[k];
                xrow = static_cast<int64_t>(s_mx0[k]) + (q - own);
                ext = q >= own;  // (a member's own prefix keys are pool rows: their slots were fetched by load_slots)
            }
            const size_t off = ext ? static_cast<size_t>(xrow) * x_stride : pool_off;
            const unsigned char* ka = (ext ? kx_g : pool_g) + off + ld_koff(u);
            const unsigned char* va = (ext ? vx_g : pool_g + v_off32) + off + ld_voff(u);
            load_to_lds_16(ka, sk + blk * 1024);
            load_to_lds_16(va, sk + TILEB + blk * 1024);
        }
    };

    // ---- fp8 pool.  A pool row arrives as its D codes, in the first half of the LDS bytes its bfloat16 form will take
    // (the lanes that would fetch the second half stay idle), and its exponent as one byte in a small staging area of
    // the wave; rows of the extend tensors arrive as before.  Once the loads have landed, landed8() turns the codes
    // into bfloat16 in place: the lanes of a row (one wave, in step) all read their 8 codes before any of them writes,
    // and no other wave touches the row until the barrier that follows.
    constexpr int EXPB = 256 * 2 * UPW;  // staging bytes per wave: one 32-bit word per lane, load block and tensor
    constexpr int EX_OFF = (kStages * STAGEB + (4 * MT + 1 + 2 * NW) * static_cast<int>(sizeof(int)) + 255) & ~255;
    const unsigned char* pool8_g = reinterpret_cast<const unsigned char*>(pool) + static_cast<size_t>(g) * page_size * D;
    const size_t page_stride8 = static_cast<size_t>(2) * Hkv * page_size * D;
    const size_t v_off8 = static_cast<size_t>(Hkv) * page_size * D;
    const signed char* exp_g = pool_exp + static_cast<size_t>(g) * page_size;
    const size_t exp_page = static_cast<size_t>(2) * Hkv * page_size, exp_v = static_cast<size_t>(Hkv) * page_size;
    int raw_mask = 0;  // bit u: this lane's row of load block u is a pool row (codes to be decoded)
    auto issue8 = [&](int p0, int ring) __attribute__((always_inline)) {
        const unsigned sk = __builtin_amdgcn_readfirstlane(smem_addr + ring * STAGEB);
        const unsigned ex = __builtin_amdgcn_readfirstlane(smem_addr + EX_OFF + wave * EXPB);
        if (shared)
            while (cur_member + 1 < n_members && s_mseg[cur_member + 1] <= p0) ++cur_member;
        raw_mask = 0;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int blk = wave * UPW + u;
            const int p = min(p0 + blk * RPB + ld_rowl, kv_hi - 1);
            bool ext = p >= P;
            const unsigned sl = static_cast<unsigned>(min(max(sl_next[u], 0), num_slots - 1));  // never outside the pool
            const unsigned pg = page_shift >= 0 ? sl >> page_shift : __umulhi(sl, page_magic) >> page_mshift;
            const unsigned o = sl - pg * static_cast<unsigned>(page_size);
            int64_t xrow = p - P;
            if (shared && ext) {
                const int k = member_at(cur_member, p);
                const int q = p - s_mseg[k], own = s_mown[k];
                xrow = static_cast<int64_t>(s_mx0[k]) + (q - own);
                ext = q >= own;
            }
            if (ext) {
                const size_t off = static_cast<size_t>(xrow) * x_stride;
                load_to_lds_16(kx_g + off + ld_koff(u), sk + blk * 1024);
                load_to_lds_16(vx_g + off + ld_voff(u), sk + TILEB + blk * 1024);
            } else {
                raw_mask |= 1 << u;
                if (ld_pos < CPR / 2) {
                    const unsigned char* ka = pool8_g + static_cast<size_t>(pg) * page_stride8 + o * static_cast<unsigned>(D) + ld_pos * 16;
                    load_to_lds_16(ka, sk + blk * 1024);
                    load_to_lds_16(ka + v_off8, sk + TILEB + blk * 1024);
                }
                if (ld_pos == 0) {
                    const signed char* ea = exp_g + static_cast<size_t>(pg) * exp_page + o;
                    load_to_lds_1(ea, ex + (2 * u) * 256);
                    load_to_lds_1(ea + exp_v, ex + (2 * u + 1) * 256);
                }
            }
        }
    };
    // the tile in ring slot `ring` has landed (this wave's loads have been waited for): decode this wave's pool rows
    auto landed8 = [&](int ring) __attribute__((always_inline)) {
        unsigned char* const sk = smem + ring * STAGEB;
        const int* const ex = reinterpret_cast<const int*>(smem + EX_OFF + wave * EXPB);
        uint2 kraw[UPW], vraw[UPW];
        int ke[UPW], ve[UPW];
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            if ((raw_mask >> u) & 1) {
                const unsigned char* row = sk + (wave * UPW + u) * 1024 + ld_rowl * ROWB;
                kraw[u] = *reinterpret_cast<const uint2*>(row + (ld_koff(u) >> 1));
                vraw[u] = *reinterpret_cast<const uint2*>(row + TILEB + (ld_voff(u) >> 1));
                ke[u] = ex[(2 * u) * 64 + (lane & ~(CPR - 1))];
                ve[u] = ex[(2 * u + 1) * 64 + (lane & ~(CPR - 1))];
            }
        }
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            if ((raw_mask >> u) & 1) {
                unsigned char* dst = sk + (wave * UPW + u) * 1024 + lane * 16;
                const float ks = fp8_scale(static_cast<int>(static_cast<signed char>(ke[u] & 0xFF)));
                const float vs = fp8_scale(static_cast<int>(static_cast<signed char>(ve[u] & 0xFF)));
                const uint2 ka = fp8_decode4(kraw[u].x, ks), kb = fp8_decode4(kraw[u].y, ks);
                const uint2 va = fp8_decode4(vraw[u].x, vs), vb = fp8_decode4(vraw[u].y, vs);
                *reinterpret_cast<uint4*>(dst) = make_uint4(ka.x, ka.y, kb.x, kb.y);
                *reinterpret_cast<uint4*>(dst + TILEB) = make_uint4(va.x, va.y, vb.x, vb.y);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the barrier that follows does not wait for LDS writes
    };
    auto issue_any = [&](int p0, int ring) __attribute__((always_inline)) {
        if constexpr (KV8) issue8(p0, ring);
        else issue(p0, ring);
    };

    f32x16 oacc[RB][NB];
    float m_run[RB], l_run[RB];  // running maximum (scaled, log2 domain) and this lane's share of the sum
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[rb][b][i] = 0.f;
    }

    // ---- LDS read addresses of this lane in the ring slot that holds the current tile (toggled after every tile).
    // K: row n (+32 for the second key block), 16-byte chunk 2 s + hh of the row.
    // V, transposing read: group lane i = 4 e + c reads key row 8 h2 + 4 hh + e (+ 16 cs + 32 mb) and 8 bytes at
    // head-dim offset 32 b + 16 par + 4 c.  The swizzles do not depend on mb / cs, which become immediates.
    typedef __attribute__((address_space(3))) const unsigned char lds_cbyte;
    lds_cbyte* lds = (lds_cbyte*)nullptr;  // k_rd / v_rd hold absolute LDS addresses
    unsigned k_rd[KS], v_rd[NB][2];
    {
        const int tr_e = (lane >> 2) & 3, tr_c = lane & 3, tr_par = (lane >> 4) & 1;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            k_rd[s] = smem_addr + n * ROWB + (((2 * s + hh) ^ swz_k<D>(n)) * 16);
            asm volatile("" : "+v"(k_rd[s]));  // keep it in a register instead of recomputing it every tile
        }
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                const int vrow = 8 * h2 + 4 * hh + tr_e;
                const int chunk16 = 4 * b + 2 * tr_par + (tr_c >> 1);
                v_rd[b][h2] = smem_addr + TILEB + vrow * ROWB + ((chunk16 ^ swz_v<D>(vrow)) * 16) + (tr_c & 1) * 8;
                asm volatile("" : "+v"(v_rd[b][h2]));
            }
    }
    const bf16x2_t ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};

    // ---- One block of 32 keys of the current tile, general: masks, any running maximum.  Kept small in registers
    // (one score block alive, no overlap of its phases inside the wave; the other wave of the SIMD fills the gaps):
    // it runs for the first tile, the tile where prefix and extend tokens meet, the tiles on the causal diagonal, and
    // wherever the hand-scheduled tile does not apply.  mb = 0 / 1: first / second block of the tile.
    auto general_block = [&](int p0, int mb, bool need_mask) __attribute__((always_inline)) {
        const unsigned off = static_cast<unsigned>(mb) * (32 * ROWB);
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 sacc[RB];
        // S^T = K Q^T: each K fragment read from LDS feeds RB MFMAs.  All fragments of the block are asked for before
        // the first product, so that their LDS round trips overlap instead of following one another.
        // (Written as assembly: the compiler, short of registers, otherwise reads one fragment at a time into the same four
        // registers, eight LDS round trips in a row.  Nothing else of this wave's is in flight on the LDS counter here:
        // the compiler's own LDS reads are awaited before they are used, and one wait for all eight follows.)
        bf16x8 kf[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("ds_read_b128 %0, %1" : "=v"(kf[s]) : "v"(k_rd[s] + off));
        if constexpr (KS == 8)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]), "+v"(kf[7]));
        else
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]));
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                sacc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qreg[rb][s], s == 0 ? zero16 : sacc[rb], 0, 0, 0);
        }
        const int pb0 = p0 + 32 * mb;
        uint32_t pb[RB][8];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            // the keys a row must not see (only where the block crosses a visibility limit)
            // (register i of the lane holds the key at offset 8 (i / 4) + i % 4 from the lane's first key of the block:
            // compared, without branches, against the row's limits counted from that key)
            if (need_mask && pb0 + 32 > blk_vis_min[rb]) {
                const int first = pb0 + 4 * hh;
                const int lim_end = vis_end[rb] - first;
                if (!shared) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) sacc[rb][i] = (8 * (i / 4) + (i % 4) < lim_end) ? sacc[rb][i] : -INFINITY;
                } else {
                    const int lim_p = P - first, lim_lo = vis_lo[rb] - first;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int o = 8 * (i / 4) + (i % 4);
                        const bool hide = (o >= lim_end) | ((o >= lim_p) & (o < lim_lo));
                        sacc[rb][i] = hide ? -INFINITY : sacc[rb][i];
                    }
                }
            }
            // row maximum of the block, in every lane of the row
            float mx = fmaxf(sacc[rb][0], sacc[rb][1]);
#pragma unroll
            for (int i = 2; i < 16; ++i) mx = fmaxf(mx, sacc[rb][i]);
            const float m_blk = row_max(mx) * scale_log2e;  // log2 domain (scale > 0)
            // The running maximum may lag the true one by kRescaleThreshold (probabilities then reach 2^threshold,
            // harmless in bf16/fp32).  If some row of the wave outgrew it by more, raise it and rescale what was
            // accumulated so far.  With a stable maximum this happens for the first block only.
            if (__any(m_blk > m_run[rb] + kRescaleThreshold)) {
                const float m_new = fmaxf(m_run[rb], m_blk);
                const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - ((m_new == -INFINITY) ? 0.f : m_new));
                l_run[rb] *= alpha;
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[rb][b][i] *= alpha;
                m_run[rb] = m_new;
            }
            // probabilities, packed to bf16 pairs (the B operand of the second product); the row sum takes the
            // ROUNDED probabilities, the values the numerator uses
            const float neg_m = (m_run[rb] == -INFINITY) ? 0.f : -m_run[rb];
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float a = __builtin_amdgcn_exp2f(fmaf(sacc[rb][i], scale_log2e, neg_m));
                const float b = __builtin_amdgcn_exp2f(fmaf(sacc[rb][i + 1], scale_log2e, neg_m));
                const uint32_t pk = pack_bf16x2(a, b);
                pb[rb][i / 2] = pk;
                acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pk), ones, acc, false);
            }
            l_run[rb] += acc;
        }
        // O^T += V^T P^T, 16 keys per MFMA: each V^T fragment feeds RB MFMAs
#pragma unroll
        for (int cs = 0; cs < 2; ++cs) {
            bf16x8 pop[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                pop[rb] = __builtin_bit_cast(bf16x8, make_uint4(pb[rb][cs * 4 + 0], pb[rb][cs * 4 + 1], pb[rb][cs * 4 + 2], pb[rb][cs * 4 + 3]));
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                s16x4 frag[2];
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2)
                    frag[h2] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(lds + (v_rd[b][h2] + off + cs * 16 * ROWB)));
                const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(frag[0], frag[1], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    oacc[rb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pop[rb], oacc[rb][b], 0, 0, 0);
            }
        }
    };

    // One tile, general: any mix of prefix and extend rows, masks, ragged ends, any page size.  from = 1: the first
    // key block is already accumulated; issue_next = false: the next tile's loads are already in flight.
    auto tile_general = [&](int p0, int ring, int from, bool issue_next) __attribute__((always_inline)) {
#ifdef PA_PROBE_DETAIL
        const long long probe_i0 = clk ? clock64() : 0;
#endif
        if (issue_next && p0 + kKT < kv_hi) {
            issue_any(p0 + kKT, ring ^ 1);  // the next tile flies during this tile's arithmetic
            load_slots(p0 + 2 * kKT);
        } else if (issue_next) {
            raw_mask = 0;  // (the last tile: nothing lands after it)
        }
#ifdef PA_PROBE_DETAIL
        const long long probe_i1 = clk ? clock64() : 0;
        probe_gen_issue += probe_i1 - probe_i0;
#endif
        const bool not_ours = shared && p0 >= P && (p0 >= s_wave_own[2 * wave + 1] || p0 + kKT <= s_wave_own[2 * wave]);
        if (wave_on && p0 <= P + wave_i_last && !not_ours) {
            bool need_mask = false;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) need_mask |= p0 + kKT > blk_vis_min[rb];
#pragma unroll 1
            for (int mb = from; mb < 2; ++mb) general_block(p0, mb, need_mask);
        }
#ifdef PA_PROBE_DETAIL
        if (clk) probe_gen_math += clock64() - probe_i1;
#endif
    };
    // 0: the tile at p0 takes the general code; 1 / 2: the hand-scheduled one, the next tile lying wholly in the
    // prefix / wholly in the extend tokens (its rows clamp to the last valid key).  Uniform over the wave.
    auto tile_kind = [&](int p0) __attribute__((always_inline)) -> int {
        if (!(fast_ok && D == 128 && RB == 1 && (NW == 4 || NW == 8) && (smem_addr & 255u) == 0)) return 0;
        bool no_mask = true;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) no_mask &= p0 + kKT <= blk_vis_min[rb];
        if (!(wave_on && p0 <= P + wave_i_last && no_mask)) return 0;
        const int first = min(p0 + kKT, kv_hi - 1), last = min(p0 + 2 * kKT - 1, kv_hi - 1);
        // (after the common keys of a shared tile come several requests' keys: never one run of extend tokens)
        // (fp8 pool: fast_ok bit 0 allows runs over the extend tokens, bit 1 runs over the pool)
        if (last < P) return !KV8 || (fast_ok & 2) ? 1 : 0;
        return (first >= P && !shared && (!KV8 || (fast_ok & 1))) ? 2 : 0;
    };

    // ---- prologue: first tile into ring slot 0 ----
    load_slots(kv_lo);
    issue_any(kv_lo, 0);
    load_slots(kv_lo + kKT);
    wait_vm_all();
    if constexpr (KV8) landed8(0);
    wg_barrier();

    // clock probe (benchmarks only): shader cycles and ticks of the constant 100 MHz counter across the key loop
    long long clk_c0 = 0, clk_w0 = 0;
    if (clk) {
        clk_c0 = clock64();
        clk_w0 = wall_clock64();
    }
    int p0 = kv_lo, ring = 0;  // the tile at p0 sits in ring slot `ring`
    // the LDS read addresses follow the ring: from slot `from_ring` to the other one
    auto move_read_addresses = [&](int from_ring) __attribute__((always_inline)) {
        const int d = from_ring ? -STAGEB : STAGEB;
#pragma unroll
        for (int s = 0; s < KS; ++s) k_rd[s] += d;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            v_rd[b][0] += d;
            v_rd[b][1] += d;
        }
    };
    // this wave's part of the next tile has landed, and so has everyone else's; nobody still reads the tile just
    // finished; then on to the next tile
    auto next_tile = [&]() __attribute__((always_inline)) {
        wait_vm_all();
        if constexpr (KV8) landed8(ring ^ 1);
        wg_barrier();
        move_read_addresses(ring);
        ring ^= 1;
        p0 += kKT;
    };
    // Tiles in assembly (D = 128; one statement, see fast_run_d128.inc).  A run: consecutive tiles that need no mask
    // and whose successors lie wholly in the prefix (mode 1, or 3 for pools of 4 GB and more) or wholly in the extend
    // tokens (2); it issues its tiles' loads itself.  A single tile: arithmetic only, with the keys a row must not see
    // hidden if there are any (5, else 4), the next tile's loads issued from here by the general code - for the tiles
    // that no run takes because of what their successor is (prefix and extend rows mixed) or because they touch the
    // causal diagonal; not in shared tiles (a second visibility bound).  Neither before the running maximum exists.
    auto single_tile_ok = [&](int p0) __attribute__((always_inline)) -> bool {
        return (fast_ok || KV8) && D == 128 && RB == 1 && NW == 4 && (smem_addr & 255u) == 0 && !shared && wave_on && p0 <= P + wave_i_last;
    };
    // The assembly tiles want a running maximum to start from, and any lower bound of the true one will do as long as it
    // is not 2^40 short (then the tile is handed to the general code, as always): the largest score of the first 32 keys,
    // where every row of the wave sees all of them.  The first tile then runs in assembly like the others (its first
    // key block is multiplied twice) instead of in the general code, which establishes the maximum otherwise.
    if constexpr (D == 128 && RB == 1 && NW == 4) {
        // (also in shared tiles: the keys of the common prefix are visible to every row)
        if ((fast_ok || KV8) && (smem_addr & 255u) == 0 && wave_on && kv_lo <= P + wave_i_last && kv_lo + 32 <= blk_vis_min[0] && kv_lo + 32 <= kv_hi) {
            const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            bf16x8 kf[KS];
#pragma unroll
            for (int s = 0; s < KS; ++s) asm volatile("ds_read_b128 %0, %1" : "=v"(kf[s]) : "v"(k_rd[s]));
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]), "+v"(kf[7]));
            f32x16 sacc = zero16;
#pragma unroll
            for (int s = 0; s < KS; ++s) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qreg[0][s], sacc, 0, 0, 0);
            float mx = fmaxf(sacc[0], sacc[1]);
#pragma unroll
            for (int i = 2; i < 16; ++i) mx = fmaxf(mx, sacc[i]);
            m_run[0] = row_max(mx) * scale_log2e;
        }
    }
    bool fast_allowed = true;
    while (p0 < kv_hi) {
        p0 = __builtin_amdgcn_readfirstlane(p0);  // wave-uniform, said so to the compiler
        ring = __builtin_amdgcn_readfirstlane(ring);
        int from = 0;
        bool issue_next = true;
        bool have_m = true;  // every row has a finite running maximum
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) have_m &= m_run[rb] != -INFINITY;
        int mode = 0, kind = 0;
        if (fast_allowed && __all(have_m)) {
            kind = tile_kind(p0);
            mode = kind == 1 ? (KV8 ? 6 : fast_ok == 2 ? 3 : 1) : kind == 2 ? 2 : single_tile_ok(p0) ? (p0 + kKT > blk_vis_min[0] ? 5 : 4) : 0;
        }
        if (mode != 0) {
            if constexpr (D == 128 && RB == 1 && (NW == 4 || (NW == 8 && !KV8))) {
                // Against the running maximum as it stands: scores never move it in there (a row's probabilities may
                // reach 2^40 instead), the output accumulators are touched by MFMAs only.
                int p_end = p0 + kKT;
                if (mode <= 3 || mode == 6) {
                    while (tile_kind(p_end) == kind) p_end += kKT;
                    raw_mask = 0;  // (fp8 pool: a run decodes what it loads itself)
                } else if (p0 + kKT < kv_hi) {
#ifdef PA_PROBE_DETAIL
                    const long long probe_s0 = clk ? clock64() : 0;
#endif
                    issue_any(p0 + kKT, ring ^ 1);
                    load_slots(p0 + 2 * kKT);
#ifdef PA_PROBE_DETAIL
                    if (clk) probe_single_issue += clock64() - probe_s0;
#endif
                } else {
                    raw_mask = 0;
                }
#ifdef PA_PROBE_DETAIL
                const long long probe_r0 = clk ? clock64() : 0;
#endif
                const int p_start = p0, ring_start = ring;
                int st = 0;
                const bf16x16 q01 = __builtin_shufflevector(qreg[0][0], qreg[0][1], 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                const bf16x16 q23 = __builtin_shufflevector(qreg[0][2], qreg[0][3], 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                const bf16x16 q45 = __builtin_shufflevector(qreg[0][4], qreg[0][5], 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                const bf16x16 q67 = __builtin_shufflevector(qreg[0][6], qreg[0][7], 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                const bf16x32 q_lo = __builtin_shufflevector(q01, q23, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18,
                                                             19, 20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31);
                const bf16x32 q_hi = __builtin_shufflevector(q45, q67, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18,
                                                             19, 20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31);
                // wave-uniform values, said so to the compiler (they go to scalar registers)
                auto uni = [](int x) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(x); };
                auto uni_ptr = [&](const void* q) __attribute__((always_inline)) {
                    const uint64_t a = reinterpret_cast<uint64_t>(q);
                    const uint64_t lo = static_cast<uint32_t>(uni(static_cast<int>(a))), hi = static_cast<uint32_t>(uni(static_cast<int>(a >> 32)));
                    return reinterpret_cast<const void*>(lo | (hi << 32));
                };
                // (mode 3: the pool is too large for 32-bit byte offsets; rows are then counted in units of 256 bytes)
                // (mode 6, the fp8 pool: strides of the codes and of the row exponents, and where the latter lie)
                const uint64_t exp_addr = reinterpret_cast<uint64_t>(exp_g);
                const i32x8 c = {uni(page_shift), uni(page_size - 1),
                                 uni(static_cast<int>(mode == 6 ? page_stride8 : mode == 3 ? page_stride / ROWB : page_stride)), uni(num_slots - 1),
                                 uni(P - 1), uni(static_cast<int>(mode == 6 ? exp_page : x_stride)),
                                 uni(mode == 6 ? static_cast<int>(exp_v) : kv_hi - 1 - P),
                                 uni(static_cast<int>(smem_addr) + wave * (UPW * 1024))};
                const i32x4 c2 = {uni(mode == 6 ? static_cast<int>(exp_addr) : 128), uni(mode == 6 ? static_cast<int>(exp_addr >> 32) : 192), uni(P),
                                  uni(__float_as_int(scale_log2e))};
                p0 = uni(p0);
                ring = uni(ring);
                p_end = uni(p_end);
                const int row_in_tile = wave * (UPW * RPB) + ld_rowl;
                const void* base_k = mode == 2 ? static_cast<const void*>(kx_g) : mode == 6 ? static_cast<const void*>(pool8_g) : static_cast<const void*>(pool_g);
                const void* base_v = mode == 2 ? static_cast<const void*>(vx_g) : mode == 6 ? static_cast<const void*>(pool8_g + v_off8) : static_cast<const void*>(pool_g + v_off32);
                const int lim = vis_end[0] - p0 - 4 * hh;
                if constexpr (KV8)  // (single tiles only; they end with this wave's loads landed and leave the barrier to the caller)
                    fast_tiles_d128_kv8(uni(mode), oacc[0][0], oacc[0][1], oacc[0][2], oacc[0][3], q_lo, q_hi, l_run[0], -m_run[0], sl_next,
                                        k_rd[0], v_rd[0][0], ld_koff0, ld_voff0, row_in_tile, p0, ring, st, p_end, uni_ptr(slots),
                                        uni_ptr(base_k), uni_ptr(base_v), lim, c, c2, uni(static_cast<int>(smem_addr) + EX_OFF + wave * EXPB));
                else if constexpr (NW == 4)
                    fast_tiles_d128(uni(mode), oacc[0][0], oacc[0][1], oacc[0][2], oacc[0][3], q_lo, q_hi, l_run[0], -m_run[0], sl_next,
                                    k_rd[0], v_rd[0][0], ld_koff0, ld_voff0, row_in_tile, p0, ring, st, p_end, uni_ptr(slots),
                                    uni_ptr(base_k), uni_ptr(base_v), lim, c, c2);
                else
                    fast_tiles_d128_w8(uni(mode), oacc[0][0], oacc[0][1], oacc[0][2], oacc[0][3], q_lo, q_hi, l_run[0], -m_run[0], sl_next,
                                       k_rd[0], v_rd[0][0], ld_koff0, ld_voff0, row_in_tile, p0, ring, st, p_end, uni_ptr(slots),
                                       uni_ptr(base_k), uni_ptr(base_v), lim, c, c2);
#ifdef PA_PROBE_DETAIL
                if (clk) {
                    if (mode <= 3 || mode == 6) {
                        probe_fast += clock64() - probe_r0;
                        probe_nfast += (p0 - p_start) / kKT;
                    } else {
                        probe_single += clock64() - probe_r0;
                        probe_nsingle += (p0 - p_start) / kKT;
                    }
                }
#endif
                if constexpr (KV8) {
                    if (mode == 6 && st != 0) raw_mask = (1 << UPW) - 1;  // left inside a tile: the next one's rows are still codes
                    if (st == 0 && mode != 6 && mode >= 4) {
#ifdef PA_PROBE_DETAIL
                        const long long probe_l0 = clk ? clock64() : 0;
#endif
                        landed8(ring);
#ifdef PA_PROBE_DETAIL
                        if (clk) probe_landed += clock64() - probe_l0;
#endif
                        wg_barrier();
                    }
                }
                if (((p0 - p_start) / kKT) & 1) move_read_addresses(ring_start);
                // (a run fetched slot ids from the common list only: where the tile they are for holds a member's own
                // prefix keys they are fetched again, from that member's list.  That tile is the next one, or, if the
                // run was left inside a tile - the next one's loads are in flight then - the one after it.)
                if ((mode <= 3 || mode == 6) && has_own_prefix()) {
                    const int pn = p0 + (st == 0 ? kKT : 2 * kKT);
                    if (pn + kKT > P) load_slots(pn);
                }
                if (st == 0) continue;
                // the tile outgrew the maximum: the general code does what is left of it, and stays (rare enough)
                from = st - 1;
                issue_next = false;
                fast_allowed = false;
            }
        }
#ifdef PA_PROBE_DETAIL
        const long long probe_g0 = clk ? clock64() : 0;
#endif
        tile_general(p0, ring, from, issue_next);
        next_tile();
#ifdef PA_PROBE_DETAIL
        if (clk) {
            probe_gen += clock64() - probe_g0;
            ++probe_ngen;
        }
#endif
    }
#ifdef PA_PROBE_DETAIL
    const long long probe_t1 = clk ? clock64() : 0;
#endif

    if (clk && blockIdx.x % 997 == 7 && tid == 0) {
        atomicAdd(clk, static_cast<unsigned long long>(clock64() - clk_c0));
        atomicAdd(clk + 1, static_cast<unsigned long long>(wall_clock64() - clk_w0));
    }
    // ---- epilogue: lane holds, for block b and register i, head-dim element 32 b + 8 (i / 4) + 4 hh + i % 4 ----
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const float l_row = row_sum(l_run[rb]);
        if (!row_ok[rb]) continue;
        if (part < 0) {
            const float inv = 1.f / l_row;
            __hip_bfloat16* orow = out + ((e0_row[rb] + qi[rb]) * Hq + qh[rb]) * static_cast<int64_t>(D);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    uint2 v;
                    v.x = pack_bf16x2(oacc[rb][b][4 * q4 + 0] * inv, oacc[rb][b][4 * q4 + 1] * inv);
                    v.y = pack_bf16x2(oacc[rb][b][4 * q4 + 2] * inv, oacc[rb][b][4 * q4 + 3] * inv);
                    *reinterpret_cast<uint2*>(orow + 32 * b + 8 * q4 + 4 * hh) = v;
                }
        } else {
            const size_t unit = static_cast<size_t>(part) * Hkv + g;
            const int lrow = wave * WR + rb * 32 + n;
            float* prow = part_o + (unit * MT + lrow) * D;
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *reinterpret_cast<float4*>(prow + 32 * b + 8 * q4 + 4 * hh) = make_float4(
                        oacc[rb][b][4 * q4 + 0], oacc[rb][b][4 * q4 + 1], oacc[rb][b][4 * q4 + 2], oacc[rb][b][4 * q4 + 3]);
            if (hh == 0) {
                part_ml[(unit * MT + lrow) * 2 + 0] = m_run[rb];
                part_ml[(unit * MT + lrow) * 2 + 1] = l_row;
            }
        }
    }
#ifdef PA_PROBE_DETAIL
    if (clk && blockIdx.x % 997 == 7 && tid == 0) {
        atomicAdd(clk + 2, static_cast<unsigned long long>(probe_fast));
        atomicAdd(clk + 3, static_cast<unsigned long long>(probe_nfast));
        atomicAdd(clk + 4, static_cast<unsigned long long>(probe_gen));
        atomicAdd(clk + 5, static_cast<unsigned long long>(probe_ngen));
        atomicAdd(clk + 6, static_cast<unsigned long long>(clk_c0 - probe_t0));
        atomicAdd(clk + 7, static_cast<unsigned long long>(clock64() - probe_t1));
        atomicAdd(clk + 8, static_cast<unsigned long long>(probe_gen_issue));
        atomicAdd(clk + 9, static_cast<unsigned long long>(probe_gen_math));
        atomicAdd(clk + 10, static_cast<unsigned long long>(probe_single));
        atomicAdd(clk + 11, static_cast<unsigned long long>(probe_nsingle));
        atomicAdd(clk + 12, static_cast<unsigned long long>(probe_single_issue));
        atomicAdd(clk + 13, static_cast<unsigned long long>(probe_landed));
    }
#endif
}

// Merge of the parts of a split tile: out = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s over the parts s.
template <int D>
__global__ __launch_bounds__(256) void extend_merge_kernel(const int32_t* __restrict__ ext_len,
                                                          const int32_t* __restrict__ ext_offsets, int Hq, int Hkv,
                                                          __hip_bfloat16* __restrict__ out,
                                                          const int32_t* __restrict__ hdr,
                                                          const int4* __restrict__ tile_tab,
                                                          const int4* __restrict__ tile_aux,
                                                          const int4* __restrict__ member_tab,
                                                          const int32_t* __restrict__ merge_tiles, int mt,
                                                          const float* __restrict__ part_o,
                                                          const float* __restrict__ part_ml) {
    constexpr int V4 = D / 4;           // 16-byte pieces per partial row
    constexpr int RPBK = 256 / V4;      // rows per pass of a block: one thread per (row, piece)
    const int G = Hq / Hkv;
    const int chunks = mt / RPBK;
    // a fixed grid strides over (tile to merge, kv head, chunk of rows): how many there are is known on the device only
    const int n_work = hdr[2] * Hkv * chunks;
    for (int w = blockIdx.x; w < n_work; w += gridDim.x) {
        const int chunk = w % chunks, g = (w / chunks) % Hkv;
        const int t = merge_tiles[w / (chunks * Hkv)];
        const int4 tt = tile_tab[t];
        const int4 aux = tile_aux[t];
        const int n_parts = tt.x, part0 = tt.y, row0 = tt.w;
        const bool shared = aux.x == kTileShared;
        const int rows_here = min(mt, (shared ? aux.w : ext_len[tt.z] * G) - row0);
        const int lrow = chunk * RPBK + threadIdx.x / V4, c = threadIdx.x % V4;
        if (lrow >= rows_here) continue;
        // whose row it is: the tile's request, or in a shared tile the last member that starts at or before it
        int64_t e0 = 0;
        int rho = row0 + lrow;
        if (shared) {
            for (int k = 0; k < aux.z; ++k) {
                const int4 mem = member_tab[2 * (aux.y + k)];
                if (mem.x <= row0 + lrow) {
                    e0 = mem.y;
                    rho = mem.z + (row0 + lrow - mem.x);
                }
            }
        } else {
            e0 = ext_offsets[tt.z];
        }
        float m = -INFINITY;
#pragma unroll 8
        for (int s = 0; s < n_parts; ++s) {
            const size_t at = (static_cast<size_t>(part0 + s) * Hkv + g) * mt + lrow;
            m = fmaxf(m, part_ml[at * 2]);
        }
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float l = 0.f;
#pragma unroll 4
        for (int s = 0; s < n_parts; ++s) {
            const size_t at = (static_cast<size_t>(part0 + s) * Hkv + g) * mt + lrow;
            const float2 ml = reinterpret_cast<const float2*>(part_ml)[at];
            const float wgt = (ml.x == -INFINITY) ? 0.f : exp2f(ml.x - m);
            l += wgt * ml.y;
            const float4 o = reinterpret_cast<const float4*>(part_o + at * D)[c];
            acc.x += wgt * o.x; acc.y += wgt * o.y; acc.z += wgt * o.z; acc.w += wgt * o.w;
        }
        const float inv = 1.f / l;
        __hip_bfloat16* orow = out + ((e0 + rho / G) * Hq + g * G + rho % G) * static_cast<int64_t>(D);
        uint2 v;
        v.x = pack_bf16x2(acc.x * inv, acc.y * inv);
        v.y = pack_bf16x2(acc.z * inv, acc.w * inv);
        reinterpret_cast<uint2*>(orow)[c] = v;
    }
}

// How the kernel divides a slot id (< 2^31) by the page size d.  A power of two: *shift = log2 d.  Otherwise
// *shift = -1 and slot / d = umulhi(slot, *magic) >> *mshift exactly: with l = ceil(log2 d), k = 31 + l and
// magic = floor(2^k / d) + 1 (< 2^32 since 2^l < 2 d), the error magic * d - 2^k is at most d <= 2^l = 2^(k - 31),
// which keeps the quotient exact for every numerator below 2^31; mshift = k - 32.
static void page_divider(int d, int* shift, unsigned* magic, int* mshift) {
    *shift = -1;
    *magic = 0;
    *mshift = 0;
    if ((d & (d - 1)) == 0) {
        *shift = 0;
        while ((1 << *shift) < d) ++*shift;
        return;
    }
    int l = 0;
    while ((int64_t{1} << l) < d) ++l;
    const int k = 31 + l;
    *magic = static_cast<unsigned>((static_cast<unsigned __int128>(1) << k) / static_cast<unsigned>(d) + 1);
    *mshift = k - 32;
}

template <int D, int NW, int RB, bool KV8>
static int launch_extend(const ExtendPlan& p, const void* q_ext, const void* k_ext, const void* v_ext,
                         const void* kv_pool, const int32_t* slot_idx, const int32_t* ext_len, const int32_t* ext_offsets,
                         int Hq, int Hkv, int page_size, int64_t num_slots, int64_t T_total, float scale_log2e, void* out,
                         const int32_t* hdr, const int4* tile_tab, const int4* tile_aux, const int4* member_tab,
                         const int4* item_tab, const int32_t* merge_tiles, float* part_o, float* part_ml,
                         unsigned long long* clk, hipStream_t stream) {
    // the K/V ring, and behind it the table of a shared tile's members (4 ints each, one int more) and 2 ints per wave
    // (fp8 pool: rounded up to 256 bytes, then one 32-bit word per lane, load block of a wave and tensor for the row exponents)
    constexpr size_t lds_plain = static_cast<size_t>(kStages) * 2 * kKT * D * 2 + (4 * 32 * RB * NW + 1 + 2 * NW) * sizeof(int);
    constexpr size_t lds_bytes = KV8 ? ((lds_plain + 255) & ~size_t{255}) + static_cast<size_t>(NW) * 256 * 2 * (kKT / (1024 / (D * 2)) / NW) : lds_plain;
    int page_shift = -1, page_mshift = 0;
    unsigned page_magic = 0;
    page_divider(page_size, &page_shift, &page_magic, &page_mshift);
    const dim3 grid(static_cast<unsigned>(p.items_cap) * Hkv);
#ifdef PA_PROBE_DETAIL
    // (experiments: more LDS per workgroup than it uses, so that only one fits a compute unit)
    const char* pad_env = getenv("PA_PROBE_LDS_PAD");
    const size_t lds_pad = pad_env ? static_cast<size_t>(atol(pad_env)) : 0;
    if (lds_pad)
        PA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&extend_bf16_kernel<D, NW, RB, KV8>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes + lds_pad)));
#else
    constexpr size_t lds_pad = 0;
#endif
    // The hand-scheduled tiles multiply in 24 bits and take a power-of-two page size.  They address pool rows by
    // 32-bit byte offsets where the pool is below 4 GB (1); by row numbers in units of 256 bytes, the byte address
    // formed in 64 bits, where it is larger (2: D = 128, a pool base aligned to 256 bytes, up to 64 GB).  The extend
    // tensors are addressed by 32-bit byte offsets in either case.
    const int64_t rowb = static_cast<int64_t>(D) * 2;
    const int64_t pool_bytes = num_slots * 2 * Hkv * rowb;
    const int64_t page_bytes = static_cast<int64_t>(page_size) * 2 * Hkv * rowb;
    const bool common_ok = page_shift >= 0 && num_slots / page_size < (1 << 24) && T_total < (1 << 24) &&
                           T_total * Hkv * rowb < (int64_t{1} << 32);
    const bool ok32 = common_ok && pool_bytes < (int64_t{1} << 32) && page_bytes < (1 << 24);
    const bool ok64 = common_ok && rowb == 256 && (reinterpret_cast<uintptr_t>(kv_pool) & 255u) == 0 &&
                      page_bytes / rowb < (1 << 24) && pool_bytes / rowb < (int64_t{1} << 28);
    // (fp8 pool: 1 = the extend tensors can be addressed by 32-bit offsets, all that its runs of tiles ask for)
    // (fp8 pool: bit 0 = the extend tensors can be addressed by 32-bit offsets, as the runs over extend tokens do; bit 1 =
    // so can the codes, with page numbers and page strides that fit the 24-bit multiplications of the runs over the pool)
    const bool ext_ok = T_total < (1 << 24) && T_total * Hkv * rowb < (int64_t{1} << 32);
    const bool pool8_ok = page_shift >= 0 && num_slots / page_size < (1 << 24) && pool_bytes / 2 < (int64_t{1} << 32) && page_bytes / 2 < (1 << 24);
    const int fast_ok = KV8 ? (ext_ok ? 1 : 0) | (pool8_ok ? 2 : 0) : ok32 ? 1 : ok64 ? 2 : 0;
    // (fp8 pool: the row exponents lie behind the codes)
    const signed char* pool_exp = KV8 ? static_cast<const signed char*>(kv_pool) + static_cast<size_t>(num_slots) * 2u * Hkv * D : nullptr;
    {
        ProfScope prof(kProfExtend, stream);
        hipLaunchKernelGGL((extend_bf16_kernel<D, NW, RB, KV8>), grid, dim3(NW * 64), lds_bytes + lds_pad, stream,
                           static_cast<const __hip_bfloat16*>(q_ext), static_cast<const __hip_bfloat16*>(k_ext),
                           static_cast<const __hip_bfloat16*>(v_ext), static_cast<const __hip_bfloat16*>(kv_pool), pool_exp, slot_idx,
                           Hq, Hkv, page_size, page_shift, page_magic, page_mshift, static_cast<int>(num_slots), fast_ok,
                           scale_log2e,
                           static_cast<__hip_bfloat16*>(out), hdr, item_tab, member_tab, part_o, part_ml, clk);
    }
    if (p.parts_cap > 0) {  // whether any tile was split is known on the device only: unsplit tiles leave at once
        ProfScope prof(kProfMerge, stream);
        const int64_t most = static_cast<int64_t>(p.merge_cap) * Hkv * ((32 * RB * NW) / (256 / (D / 4)));
        hipLaunchKernelGGL((extend_merge_kernel<D>), dim3(static_cast<unsigned>(most < 2048 ? most : 2048)), dim3(256), 0, stream,
                           ext_len, ext_offsets, Hq, Hkv, static_cast<__hip_bfloat16*>(out), hdr, tile_tab, tile_aux, member_tab,
                           merge_tiles, 32 * RB * NW, part_o, part_ml);
    }
    return PA_OK;
}

}  // namespace pa

// Process-wide switch: 0 = every request gets row tiles of its own (no grouping by equal slots).
static std::atomic<int> g_row_sharing{1};
extern "C" int pa_extend_set_row_sharing(int on) {
    g_row_sharing.store(on != 0);
    return PA_OK;
}

// Whether the last bf16 launch that used this workspace found room for its work list.
extern "C" int pa_extend_status(const void* workspace, void* stream) {
    PA_REQUIRE(workspace != nullptr, "pa_extend_status: workspace is NULL");
    int32_t hdr[4] = {0, 0, 0, 0};
    hipStream_t s = static_cast<hipStream_t>(stream);
    PA_HIP(hipMemcpyAsync(hdr, workspace, sizeof hdr, hipMemcpyDeviceToHost, s));
    PA_HIP(hipStreamSynchronize(s));
    if (hdr[3] != 0)
        return pa::fail(PA_EOVERFLOW, "pa_extend_attention: the batch on the device is larger than the T and max_kv_len "
                                      "the call was given; its work list did not fit and no output was written");
    return PA_OK;
}

// Waves per workgroup for a batch: eight (row tiles of 256 packed rows; a K/V tile then serves twice the rows and a
// wave issues half the loads per tile) where requests bring many rows, four (finer row tiles, two workgroups on a
// compute unit) otherwise.
static int waves_for(int B, int64_t T, int Hq, int Hkv, int D) {
#ifdef PA_PROBE_DETAIL
    if (const char* e = getenv("PA_PROBE_NW")) return atoi(e) == 8 && D == 128 ? 8 : 4;
#endif
    (void)B; (void)T; (void)Hq; (void)Hkv; (void)D;
    return 4;
}

size_t pa_extend_workspace_bytes_bf16(int B, int64_t T, int64_t max_kv_len, int Hq, int Hkv, int D) {
    const size_t a = pa::make_plan(B, T, max_kv_len, Hq, Hkv, D, pa::kRounds, 4).total;
    const size_t b = D == 128 ? pa::make_plan(B, T, max_kv_len, Hq, Hkv, D, pa::kRounds, 8).total : 0;
    return a > b ? a : b;
}

// The work of a bf16 call once its plan and its workspace are settled.
static int run_extend_bf16(pa::ExtendPlan p, const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                           const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                           const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T, int Hq, int Hkv, int D,
                           int page_size, int64_t num_slots, bool kv8, float scale, void* out, void* workspace, hipStream_t stream) {
    using namespace pa;
    if (!g_row_sharing.load()) p.pack = 0;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int32_t* hdr = reinterpret_cast<int32_t*>(ws);
    int32_t* order = reinterpret_cast<int32_t*>(ws + p.off_order);
    int4* tile_tab = reinterpret_cast<int4*>(ws + p.off_tile);
    int4* tile_aux = reinterpret_cast<int4*>(ws + p.off_aux);
    int4* member_tab = reinterpret_cast<int4*>(ws + p.off_member);
    int4* item_tab = reinterpret_cast<int4*>(ws + p.off_item);
    int32_t* merge_tiles = reinterpret_cast<int32_t*>(ws + p.off_split);
    float* part_o = reinterpret_cast<float*>(ws + p.off_part_o);
    float* part_ml = reinterpret_cast<float*>(ws + p.off_part_ml);
    // with the clock probe on, a few workgroups also add their cycle counts to two counters in the header
    unsigned long long* clk = prof_clock_enabled() ? reinterpret_cast<unsigned long long*>(ws + kClockProbeOffset) : nullptr;
    const int G = Hq / Hkv;
    const float scale_log2e = scale * 1.4426950408889634f;
    {
        ProfScope prof(kProfPlan, stream);
        hipLaunchKernelGGL(extend_plan_kernel, dim3(1), dim3(kPlanThreads), 0, stream, prefix_len, ext_len, ext_offsets, slot_offsets, slot_idx, B,
                           G, 32 * p.rb * p.nw, p.tiles_cap, p.items_cap, p.parts_cap, p.merge_cap, p.slots * p.rounds, p.pack, p.tile_parts, hdr, order,
                           tile_tab, tile_aux, member_tab, item_tab, merge_tiles);
    }
    if (kv8 && D == 64)
        launch_extend<64, 4, 1, true>(p, q_ext, k_ext, v_ext, kv_pool, slot_idx, ext_len, ext_offsets, Hq, Hkv, page_size, num_slots, T,
                             scale_log2e, out, hdr, tile_tab, tile_aux, member_tab, item_tab, merge_tiles, part_o, part_ml, clk, stream);
    else if (kv8)
        launch_extend<128, 4, 1, true>(p, q_ext, k_ext, v_ext, kv_pool, slot_idx, ext_len, ext_offsets, Hq, Hkv, page_size, num_slots, T,
                              scale_log2e, out, hdr, tile_tab, tile_aux, member_tab, item_tab, merge_tiles, part_o, part_ml, clk, stream);
    else if (D == 64)
        launch_extend<64, 4, 1, false>(p, q_ext, k_ext, v_ext, kv_pool, slot_idx, ext_len, ext_offsets, Hq, Hkv, page_size, num_slots, T,
                             scale_log2e, out, hdr, tile_tab, tile_aux, member_tab, item_tab, merge_tiles, part_o, part_ml, clk, stream);
    else if (p.nw == 8)
        launch_extend<128, 8, 1, false>(p, q_ext, k_ext, v_ext, kv_pool, slot_idx, ext_len, ext_offsets, Hq, Hkv, page_size, num_slots, T,
                              scale_log2e, out, hdr, tile_tab, tile_aux, member_tab, item_tab, merge_tiles, part_o, part_ml, clk, stream);
    else
        launch_extend<128, 4, 1, false>(p, q_ext, k_ext, v_ext, kv_pool, slot_idx, ext_len, ext_offsets, Hq, Hkv, page_size, num_slots, T,
                              scale_log2e, out, hdr, tile_tab, tile_aux, member_tab, item_tab, merge_tiles, part_o, part_ml, clk, stream);
    PA_HIP(hipGetLastError());
    return PA_OK;
}

static int check_bf16_args(float scale, int64_t num_slots, int page_size, int Hkv, int D) {
    PA_REQUIRE(scale > 0.f && scale < INFINITY, "pa_extend_attention: scale must be positive and finite");
    PA_REQUIRE(num_slots <= INT32_MAX, "pa_extend_attention: num_slots exceeds the int32 range of slot ids");
    PA_REQUIRE(static_cast<int64_t>(page_size) * Hkv * D * 4 < (int64_t{1} << 31), "pa_extend_attention: a page of %d tokens x %d heads is too large", page_size, Hkv);
    return PA_OK;
}

// Called by pa_extend_attention after argument validation.
int pa_extend_attention_bf16(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                             const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                             const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T, int64_t max_kv_len,
                             int Hq, int Hkv, int D, int page_size, int64_t num_slots, bool kv8, float scale, void* out,
                             void* workspace, size_t workspace_bytes, hipStream_t stream) {
    using namespace pa;
    if (const int rc = check_bf16_args(scale, num_slots, page_size, Hkv, D)) return rc;
    const ExtendPlan p = make_plan(B, T, max_kv_len, Hq, Hkv, D, kRounds, kv8 ? 4 : waves_for(B, T, Hq, Hkv, D));  // (sized for shared row tiles whether or not they are on)
    if (workspace_bytes < p.total || workspace == nullptr)
        return fail(PA_ENOMEM, "pa_extend_attention: workspace of %zu bytes given, %zu needed", workspace_bytes, p.total);
    PA_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, "pa_extend_attention: workspace must be 256-byte aligned");
    return run_extend_bf16(p, q_ext, k_ext, v_ext, kv_pool, slot_idx, slot_offsets, prefix_len, ext_len, ext_offsets, B, T, Hq,
                           Hkv, D, page_size, num_slots, kv8, scale, out, workspace, stream);
}

// ---------------------------------------------------------------------------------------
// The variant for callers that cannot allocate: its workspace is a buffer that is part of the library's code object.
// Every GPU that loads the library holds its own copy of the array at its own address; in host code the array's name
// is only a handle for hipGetSymbolAddress, never a device address.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
int scratch_of_current_device(void** out) {
    int dev = -1;
    PA_HIP(hipGetDevice(&dev));
    PA_REQUIRE(dev >= 0 && dev < kMaxDevices, "pa_extend_attention_static: device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        PA_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        PA_REQUIRE(ptr != nullptr && (reinterpret_cast<uintptr_t>(ptr) & 255u) == 0, "pa_extend_attention_static: bad scratch address");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PA_OK;
}
}  // namespace

// Called by pa_extend_attention_static after argument validation.
int pa_extend_attention_bf16_static(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                                    const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                                    const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T,
                                    int64_t max_kv_len, int Hq, int Hkv, int D, int page_size, int64_t num_slots,
                                    bool kv8, float scale, void* out, hipStream_t stream) {
    using namespace pa;
    if (const int rc = check_bf16_args(scale, num_slots, page_size, Hkv, D)) return rc;
    // (one work item per workgroup slot is aimed at instead of three: a third of the partial results at most)
    const ExtendPlan p = make_plan(B, T, max_kv_len, Hq, Hkv, D, kRoundsStatic, kv8 ? 4 : waves_for(B, T, Hq, Hkv, D));
    if (p.total > PA_STATIC_SCRATCH_BYTES)
        return fail(PA_ENOMEM, "pa_extend_attention_static: this batch needs %zu bytes of workspace, the library's own buffer holds %zu; "
                               "use pa_extend_attention with a workspace of the caller's", p.total, static_cast<size_t>(PA_STATIC_SCRATCH_BYTES));
    void* ws = nullptr;
    if (const int rc = scratch_of_current_device(&ws)) return rc;
    return run_extend_bf16(p, q_ext, k_ext, v_ext, kv_pool, slot_idx, slot_offsets, prefix_len, ext_len, ext_offsets, B, T, Hq,
                           Hkv, D, page_size, num_slots, kv8, scale, out, ws, stream);
}
