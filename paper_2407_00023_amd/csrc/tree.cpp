// Host-side radix tree of cached token sequences, its flattening, and the upload of the
// flat form to device memory.
//
// Sec. 3.2 ("global scheduler data structures") and Sec. 3.3 of the paper: insertion
// matches a sequence from the beginning until no match exists and adds the remainder as
// a new leaf; a node that matches only partly is split into matched part + remainder; a
// sequence that matches nothing becomes a new tree (here a child of an empty root).
#include <algorithm>
#include <cstring>
#include <deque>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "common.h"

namespace pa {

static thread_local std::string g_last_error;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

// Byte offsets of the arrays of the flat form (what the device sees) for given capacities.
struct FlatLayout {
    int64_t tok_cap = 0, node_cap = 0;
    uint64_t tab_cap = 0;  // entries of each hash table, a power of two
    size_t o_tok = 0, o_slot = 0, o_start = 0, o_len = 0, o_key = 0, o_val = 0, o_phe = 0, o_end = 0, total = 0;
    void set(int64_t tokens, int64_t nodes, uint64_t table) {
        auto up = [](size_t x) { return (x + 255) & ~size_t(255); };
        tok_cap = tokens;
        node_cap = nodes;
        tab_cap = table;
        o_tok = 0;
        o_slot = o_tok + up(static_cast<size_t>(tokens) * 4);
        o_start = o_slot + up(static_cast<size_t>(tokens) * 4);
        o_len = o_start + up(static_cast<size_t>(nodes) * 4);
        o_key = o_len + up(static_cast<size_t>(nodes) * 4);
        o_val = o_key + up(table * 8);
        o_phe = o_val + up(table * 4);
        o_end = o_phe + up(table * sizeof(PathEntry));
        total = o_end + up(static_cast<size_t>(nodes) * 8);
    }
};

constexpr unsigned long long kDeletedKey = ~0ull - 1;  // child table: an entry that was removed (never a real key)

struct Node {
    std::vector<int32_t> tok;   // edge tokens leading into this node
    std::vector<int32_t> slot;  // KV slot of each edge token
    std::unordered_map<int32_t, int32_t> child;  // first token of child's edge -> node id
    int32_t parent = -1;        // -1: the root, or a node that was evicted whole (its id waits for reuse)
    int32_t ref = 0;            // requests admitted and not yet released whose prompt runs through this node
    int64_t last = 0;           // time of the last admission that ran through this node
    std::vector<int64_t> hits;  // times of the admissions that ran through this node, increasing
};

}  // namespace pa

struct pa_tree {
    std::vector<pa::Node> nodes;
    std::vector<int32_t> free_nodes;  // ids of evicted nodes
    int64_t n_tokens = 0;
    // cache bookkeeping, once a pool is attached
    int64_t num_slots = 0;
    int32_t page_size = 0;
    std::vector<int32_t> free_pages;  // stack: the back is handed out next
    std::vector<int32_t> page_live;   // cached tokens per page
    int64_t clock = INT64_MIN;        // time of the last admission
    int64_t hit_window = 0;           // admission times older than clock - hit_window are forgotten (0: none is)
    std::deque<int64_t> admissions;   // times of the admissions, increasing
    // device mirror
    bool uploaded = false;
    int device = -1;
    void* d_blob = nullptr;
    size_t d_cap = 0;                 // bytes allocated at d_blob
    void* h_stage = nullptr;          // pinned host buffer the flat form is built in, kept between uploads
    size_t h_cap = 0;
    hipEvent_t copied = nullptr;      // recorded after the last copy out of h_stage (a whole upload)
    bool copy_pending = false;        // ... and not yet waited for
    // Partial uploads copy from one of two small pinned buffers, filled from h_stage at upload time, so that the
    // tree can go on changing (and h_stage with it) while the copies are in flight.
    void* h_xfer[2] = {nullptr, nullptr};
    size_t xfer_cap[2] = {0, 0};
    hipEvent_t xfer_done[2] = {nullptr, nullptr};
    bool xfer_pending[2] = {false, false};
    int xfer_next = 0;
    pa::DeviceTree view{};
    // The flat form in h_stage is kept up to date by every change of the tree (mirror_ok), so that an upload copies
    // only what changed since the last one (dirty byte ranges).  When a change does not fit the capacities of the
    // flat form, or too much of its token array is dead, mirror_ok goes false and the next upload rebuilds it.
    bool incremental = true;
    bool mirror_ok = false;
    pa::FlatLayout flat{};
    int64_t arena_end = 0, arena_holes = 0;  // tokens of the token array in use (live or dead), dead ones
    int64_t table_used = 0;                  // entries of each hash table in use (live or deleted)
    std::vector<int32_t> ht_pos, phe_pos, end_depth;  // per node: its entry in either table, depth of its last token
    std::vector<std::pair<size_t, size_t>> dirty;     // (offset, bytes) changed in h_stage since the last upload
    int64_t n_full_uploads = 0, n_incremental_uploads = 0, last_upload_bytes = 0;
    std::mutex mu;
};

extern "C" const char* pa_last_error(void) { return pa::g_last_error.c_str(); }

extern "C" int pa_tree_create(pa_tree** out) {
    PA_REQUIRE(out != nullptr, "pa_tree_create: out is NULL");
    pa_tree* t = new (std::nothrow) pa_tree();
    if (!t) return pa::fail(PA_ENOMEM, "pa_tree_create: out of host memory");
    t->nodes.emplace_back();  // node 0: empty virtual root
    *out = t;
    return PA_OK;
}

namespace pa {

static int32_t new_node(pa_tree* t) {
    if (!t->free_nodes.empty()) {
        const int32_t id = t->free_nodes.back();
        t->free_nodes.pop_back();
        t->nodes[id] = Node();
        return id;
    }
    t->nodes.emplace_back();
    return static_cast<int32_t>(t->nodes.size() - 1);
}

// Splits node c after its first k edge tokens (0 < k < length).  The TAIL keeps the id c - whoever holds c as the
// deepest node of a path still does - and a new node takes the head, between c and its old parent; both halves
// carry the pins and the access time.  Returns the head.
static int32_t split_node(pa_tree* t, int32_t c, int32_t k) {
    const int32_t h = new_node(t);  // may move the vector: no references across this call
    auto& nodes = t->nodes;
    Node& tail = nodes[c];
    Node& head = nodes[h];
    head.tok.assign(tail.tok.begin(), tail.tok.begin() + k);
    head.slot.assign(tail.slot.begin(), tail.slot.begin() + k);
    head.parent = tail.parent;
    head.ref = tail.ref;
    head.last = tail.last;
    head.hits = tail.hits;
    tail.tok.erase(tail.tok.begin(), tail.tok.begin() + k);
    tail.slot.erase(tail.slot.begin(), tail.slot.begin() + k);
    tail.parent = h;
    head.child.emplace(tail.tok[0], c);
    nodes[head.parent].child[head.tok[0]] = h;
    t->uploaded = false;
    return h;
}

// ---- keeping the flat form in step with the tree ----------------------------------------------------------------
struct FlatView {
    int32_t *tok, *slot, *start, *len, *val;
    unsigned long long *key, *end;
    PathEntry* phe;
};
static FlatView flat_view(pa_tree* t) {
    unsigned char* b = static_cast<unsigned char*>(t->h_stage);
    const FlatLayout& f = t->flat;
    return {reinterpret_cast<int32_t*>(b + f.o_tok),   reinterpret_cast<int32_t*>(b + f.o_slot),
            reinterpret_cast<int32_t*>(b + f.o_start), reinterpret_cast<int32_t*>(b + f.o_len),
            reinterpret_cast<int32_t*>(b + f.o_val),   reinterpret_cast<unsigned long long*>(b + f.o_key),
            reinterpret_cast<unsigned long long*>(b + f.o_end), reinterpret_cast<PathEntry*>(b + f.o_phe)};
}
template <class T>
static void mark(pa_tree* t, const T* first, size_t count) {
    const size_t off = static_cast<size_t>(reinterpret_cast<const unsigned char*>(first) - static_cast<unsigned char*>(t->h_stage));
    t->dirty.emplace_back(off, count * sizeof(T));
}
// May the flat form be changed now?  Not if it is stale anyway; and the copy of the last upload must be done with it.
static bool mirror_open(pa_tree* t) {
    if (!t->mirror_ok) return false;
    if (t->copy_pending) {
        if (hipEventSynchronize(t->copied) != hipSuccess) {
            (void)hipGetLastError();
            t->mirror_ok = false;
            return false;
        }
        t->copy_pending = false;
    }
    return true;
}
static int32_t child_table_put(pa_tree* t, FlatView& v, int32_t parent, int32_t first_tok, int32_t node) {
    const uint64_t mask = t->flat.tab_cap - 1;
    const unsigned long long key = (static_cast<unsigned long long>(static_cast<uint32_t>(parent)) << 32) | static_cast<uint32_t>(first_tok);
    uint64_t h = hash_key(key) & mask;
    while (v.key[h] != kEmptyKey) h = (h + 1) & mask;  // (deleted entries are not reused: a probe for a key stops at the first empty one)
    v.key[h] = key;
    v.val[h] = node;
    mark(t, v.key + h, 1);
    mark(t, v.val + h, 1);
    return static_cast<int32_t>(h);
}
static int32_t path_table_put(pa_tree* t, FlatView& v, unsigned long long hash, int32_t depth, int32_t node, int32_t parent) {
    const uint64_t mask = t->flat.tab_cap - 1;
    uint64_t at = path_slot(hash, depth) & mask;
    while (v.phe[at].node != -1) at = (at + 1) & mask;
    v.phe[at].hash = hash;
    v.phe[at].depth = depth;
    v.phe[at].node = node;
    v.phe[at].edge_start = v.start[node];
    v.phe[at].edge_len = v.len[node];
    v.phe[at].parent = parent;
    mark(t, v.phe + at, 1);
    return static_cast<int32_t>(at);
}
static unsigned long long hash_through(unsigned long long h, const std::vector<int32_t>& tok, size_t from, size_t to) {
    for (size_t i = from; i < to; ++i) h = path_hash_push(h, tok[i]);
    return h;
}

// A new leaf c (its tokens, slots and parent are set).
static void mirror_new_leaf(pa_tree* t, int32_t c) {
    if (!mirror_open(t)) return;
    const Node& nd = t->nodes[c];
    const int64_t len = static_cast<int64_t>(nd.tok.size());
    if (c >= t->flat.node_cap || t->arena_end + len + 64 > t->flat.tok_cap ||
        2 * static_cast<uint64_t>(t->table_used + 1) > t->flat.tab_cap) {
        t->mirror_ok = false;
        return;
    }
    FlatView v = flat_view(t);
    const int32_t p = nd.parent;
    std::memcpy(v.tok + t->arena_end, nd.tok.data(), static_cast<size_t>(len) * 4);
    std::memcpy(v.slot + t->arena_end, nd.slot.data(), static_cast<size_t>(len) * 4);
    mark(t, v.tok + t->arena_end, static_cast<size_t>(len));
    mark(t, v.slot + t->arena_end, static_cast<size_t>(len));
    v.start[c] = static_cast<int32_t>(t->arena_end);
    v.len[c] = static_cast<int32_t>(len);
    t->arena_end += len;
    const unsigned long long first_hash = path_hash_push(v.end[p], nd.tok[0]);
    v.end[c] = hash_through(first_hash, nd.tok, 1, nd.tok.size());
    t->end_depth[c] = t->end_depth[p] + static_cast<int32_t>(len);
    mark(t, v.start + c, 1);
    mark(t, v.len + c, 1);
    mark(t, v.end + c, 1);
    t->ht_pos[c] = child_table_put(t, v, p, nd.tok[0], c);
    t->phe_pos[c] = path_table_put(t, v, first_hash, t->end_depth[p], c, p);
    ++t->table_used;
}

// Node c was split after k tokens: c keeps the tail, the new node h holds the head (both already updated).
static void mirror_split(pa_tree* t, int32_t c, int32_t h, int32_t k) {
    if (!mirror_open(t)) return;
    if (h >= t->flat.node_cap || 2 * static_cast<uint64_t>(t->table_used + 1) > t->flat.tab_cap) {
        t->mirror_ok = false;
        return;
    }
    FlatView v = flat_view(t);
    const Node& head = t->nodes[h];
    const Node& tail = t->nodes[c];
    const int32_t p = head.parent;
    // the tokens stay where they are: the head is their first k, the tail the rest
    v.start[h] = v.start[c];
    v.len[h] = k;
    v.start[c] += k;
    v.len[c] -= k;
    v.end[h] = hash_through(v.end[p], head.tok, 0, head.tok.size());
    t->end_depth[h] = t->end_depth[p] + k;
    mark(t, v.start + h, 1);
    mark(t, v.len + h, 1);
    mark(t, v.end + h, 1);
    mark(t, v.start + c, 1);
    mark(t, v.len + c, 1);
    // the entries that led to c lead to the head now (same keys: same parent, same first token, same depth)
    t->ht_pos[h] = t->ht_pos[c];
    v.val[t->ht_pos[h]] = h;
    mark(t, v.val + t->ht_pos[h], 1);
    t->phe_pos[h] = t->phe_pos[c];
    PathEntry& eh = v.phe[t->phe_pos[h]];
    eh.node = h;
    eh.edge_len = k;
    mark(t, &eh, 1);
    // and the tail gets entries of its own under the head
    t->ht_pos[c] = child_table_put(t, v, h, tail.tok[0], c);
    t->phe_pos[c] = path_table_put(t, v, path_hash_push(v.end[h], tail.tok[0]), t->end_depth[h], c, h);
    ++t->table_used;
}

// Leaf c lost `removed` tokens from its tail and keeps some.
static void mirror_trim(pa_tree* t, int32_t c, int32_t removed) {
    if (!mirror_open(t)) return;
    FlatView v = flat_view(t);
    const Node& nd = t->nodes[c];
    v.len[c] = static_cast<int32_t>(nd.tok.size());
    v.end[c] = hash_through(v.end[nd.parent], nd.tok, 0, nd.tok.size());
    t->end_depth[c] -= removed;
    v.phe[t->phe_pos[c]].edge_len = v.len[c];
    mark(t, v.len + c, 1);
    mark(t, v.end + c, 1);
    mark(t, v.phe + t->phe_pos[c], 1);
    t->arena_holes += removed;
}

// Node c is gone (it held `removed` tokens when it went).
static void mirror_remove(pa_tree* t, int32_t c, int32_t removed) {
    if (!mirror_open(t)) return;
    FlatView v = flat_view(t);
    v.len[c] = 0;
    mark(t, v.len + c, 1);
    v.key[t->ht_pos[c]] = kDeletedKey;
    mark(t, v.key + t->ht_pos[c], 1);
    PathEntry& e = v.phe[t->phe_pos[c]];  // stays in its probe chain, matches nothing: no position is negative
    e.node = 0;
    e.depth = -1;
    e.edge_len = 0;
    mark(t, &e, 1);
    t->arena_holes += removed;
    // a token array that is mostly dead is compacted by the next full rebuild
    if (t->arena_holes > 4096 && 2 * t->arena_holes > t->arena_end) t->mirror_ok = false;
}

}  // namespace pa

extern "C" int pa_tree_insert(pa_tree* tree, const int32_t* tokens, const int32_t* slots, int32_t n,
                              int32_t* n_already_cached) {
    PA_REQUIRE(tree != nullptr, "pa_tree_insert: tree is NULL");
    PA_REQUIRE(n >= 0 && (n == 0 || (tokens && slots)), "pa_tree_insert: bad sequence (n=%d)", n);
    std::lock_guard<std::mutex> lk(tree->mu);
    if (tree->page_size > 0)
        return pa::fail(PA_ESTATE, "pa_tree_insert: a pool is attached, slots come from pa_tree_admit");
    auto& nodes = tree->nodes;
    int32_t cur = 0, pos = 0;
    try {
        while (pos < n) {
            auto it = nodes[cur].child.find(tokens[pos]);
            if (it == nodes[cur].child.end()) break;
            int32_t c = it->second;
            const int32_t elen = static_cast<int32_t>(nodes[c].tok.size());
            const int32_t lim = std::min(elen, n - pos);
            int32_t k = 1;  // first token equal by construction of the child map
            while (k < lim && nodes[c].tok[k] == tokens[pos + k]) ++k;
            if (k < elen) {
                if (pos + k == n) { pos = n; break; }  // the sequence ends inside this edge: nothing new to store
                cur = pa::split_node(tree, c, k);
                pa::mirror_split(tree, c, cur, k);
                pos += k;
                break;  // tokens[pos] differs from the tail's first token, so the walk ends here
            }
            pos += elen;
            cur = c;
        }
        if (n_already_cached) *n_already_cached = pos;
        if (pos < n) {
            const int32_t lid = pa::new_node(tree);
            nodes[lid].tok.assign(tokens + pos, tokens + n);
            nodes[lid].slot.assign(slots + pos, slots + n);
            nodes[lid].parent = cur;
            nodes[cur].child.emplace(tokens[pos], lid);
            tree->n_tokens += n - pos;
            tree->uploaded = false;
            pa::mirror_new_leaf(tree, lid);
        }
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_insert: out of host memory");
    }
    return PA_OK;
}

// ---------------------------------------------------------------------------------------------------------
// Cache bookkeeping around the hot path (Sec. 3.3: the local scheduler keeps, next to the prefix tree, the number
// of active requests sharing each node, and when memory is short evicts a node, or part of one if a part is
// enough, by the access time of the nodes' requests).  Pages follow the reading used for the workloads: the new
// part of a prompt receives whole pages, token t of it sits in slot page[t / p] * p + t % p.
// ---------------------------------------------------------------------------------------------------------
extern "C" int pa_tree_attach_pool(pa_tree* tree, int64_t num_slots, int page_size) {
    PA_REQUIRE(tree != nullptr, "pa_tree_attach_pool: tree is NULL");
    PA_REQUIRE(page_size >= 1 && num_slots >= page_size && num_slots % page_size == 0 && num_slots / page_size <= INT32_MAX &&
                   num_slots <= INT32_MAX,
               "pa_tree_attach_pool: num_slots %lld, page_size %d", static_cast<long long>(num_slots), page_size);
    std::lock_guard<std::mutex> lk(tree->mu);
    if (tree->n_tokens != 0 || tree->page_size != 0)
        return pa::fail(PA_ESTATE, "pa_tree_attach_pool: the tree must be empty and have no pool yet");
    try {
        const int32_t pages = static_cast<int32_t>(num_slots / page_size);
        tree->free_pages.resize(pages);
        for (int32_t i = 0; i < pages; ++i) tree->free_pages[i] = pages - 1 - i;  // page 0 is handed out first
        tree->page_live.assign(pages, 0);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_attach_pool: out of host memory");
    }
    tree->num_slots = num_slots;
    tree->page_size = page_size;
    return PA_OK;
}

extern "C" int pa_tree_free_slots(const pa_tree* tree, int64_t* free_slots) {
    PA_REQUIRE(tree != nullptr && free_slots != nullptr, "pa_tree_free_slots: NULL argument");
    *free_slots = static_cast<int64_t>(tree->free_pages.size()) * tree->page_size;
    return PA_OK;
}

extern "C" int pa_tree_admit(pa_tree* tree, const int32_t* tokens, int32_t n, int64_t now, int32_t* new_slots,
                             int32_t* n_cached, int64_t* handle) {
    PA_REQUIRE(tree != nullptr && handle != nullptr, "pa_tree_admit: NULL argument");
    PA_REQUIRE(n >= 1 && tokens && new_slots, "pa_tree_admit: bad prompt (n=%d)", n);
    std::lock_guard<std::mutex> lk(tree->mu);
    if (tree->page_size == 0) return pa::fail(PA_ESTATE, "pa_tree_admit: no pool attached");
    if (now <= tree->clock) return pa::fail(PA_EINVAL, "pa_tree_admit: time must increase from one admission to the next");
    auto& nodes = tree->nodes;
    const int32_t p = tree->page_size;
    try {
        // the cached part of the prompt; a prompt that ends inside an edge splits it there, so that pins are exact
        int32_t cur = 0, pos = 0;
        while (pos < n) {
            auto it = nodes[cur].child.find(tokens[pos]);
            if (it == nodes[cur].child.end()) break;
            const int32_t c = it->second;
            const int32_t elen = static_cast<int32_t>(nodes[c].tok.size());
            const int32_t lim = std::min(elen, n - pos);
            int32_t k = 1;
            while (k < lim && nodes[c].tok[k] == tokens[pos + k]) ++k;
            if (k < elen) {
                cur = pa::split_node(tree, c, k);
                pa::mirror_split(tree, c, cur, k);
                pos += k;
                break;
            }
            pos += elen;
            cur = c;
        }
        const int32_t rem = n - pos;
        const int64_t need = (static_cast<int64_t>(rem) + p - 1) / p;
        if (need > static_cast<int64_t>(tree->free_pages.size()))
            return pa::fail(PA_ENOMEM, "pa_tree_admit: %lld pages needed, %zu free (evict and try again)",
                            static_cast<long long>(need), tree->free_pages.size());
        if (rem > 0) {
            const int32_t lid = pa::new_node(tree);
            pa::Node& leaf = nodes[lid];
            leaf.tok.assign(tokens + pos, tokens + n);
            leaf.slot.resize(rem);
            int32_t page = -1;
            for (int32_t i = 0; i < rem; ++i) {
                if (i % p == 0) {
                    page = tree->free_pages.back();
                    tree->free_pages.pop_back();
                }
                leaf.slot[i] = page * p + i % p;
                ++tree->page_live[page];
                new_slots[pos + i] = leaf.slot[i];
            }
            leaf.parent = cur;
            nodes[cur].child.emplace(tokens[pos], lid);
            tree->n_tokens += rem;
            pa::mirror_new_leaf(tree, lid);
            cur = lid;
        }
        const bool forget = tree->hit_window > 0 && now > INT64_MIN + tree->hit_window;
        const int64_t horizon = forget ? now - tree->hit_window : INT64_MIN;  // times <= horizon are forgotten
        for (int32_t x = cur; x > 0; x = nodes[x].parent) {  // pin the path, and it is the most recently used now
            ++nodes[x].ref;
            nodes[x].last = now;
            auto& hits = nodes[x].hits;
            if (forget && !hits.empty() && hits.front() <= horizon)
                hits.erase(hits.begin(), std::upper_bound(hits.begin(), hits.end(), horizon));
            hits.push_back(now);
        }
        while (forget && !tree->admissions.empty() && tree->admissions.front() <= horizon) tree->admissions.pop_front();
        tree->admissions.push_back(now);
        tree->clock = now;
        tree->uploaded = false;
        if (n_cached) *n_cached = pos;
        *handle = cur;
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_admit: out of host memory");
    }
    return PA_OK;
}

extern "C" int pa_tree_release(pa_tree* tree, int64_t handle) {
    PA_REQUIRE(tree != nullptr, "pa_tree_release: tree is NULL");
    std::lock_guard<std::mutex> lk(tree->mu);
    auto& nodes = tree->nodes;
    PA_REQUIRE(handle > 0 && handle < static_cast<int64_t>(nodes.size()) && nodes[handle].ref > 0 && !nodes[handle].tok.empty(),
               "pa_tree_release: %lld is not the handle of an admitted request", static_cast<long long>(handle));
    for (int32_t x = static_cast<int32_t>(handle); x > 0; x = nodes[x].parent) {
        if (nodes[x].ref <= 0) return pa::fail(PA_ESTATE, "pa_tree_release: pin counts are inconsistent at node %d", x);
        --nodes[x].ref;
    }
    return PA_OK;
}

namespace pa {

struct EvictStep {
    int32_t node;    // a leaf that no admitted request runs through
    int32_t tokens;  // how many tokens it loses from its tail (all of them: the node goes)
};

// The eviction order: the least recently used leaf that no admitted request runs through goes first, from its
// tail, token by token, until enough whole pages are free: part of a node if a part is enough.  A parent whose
// children are all gone is a leaf in turn.  (Admission times are distinct, and an admission touches one path, so
// no two leaves share a time.)  Reads the tree only; pa_tree_evict applies the steps, pa_tree_evict_plan reports them.
// keep (may be NULL): node -> number of leading tokens that must stay (the cached part of a prompt about to be admitted).
static void plan_eviction(const pa_tree* tree, int64_t need_slots, const std::unordered_map<int32_t, int32_t>* keep,
                          std::vector<EvictStep>& steps, int64_t& freed) {
    const auto& nodes = tree->nodes;
    const int32_t p = tree->page_size;
    const int32_t nn = static_cast<int32_t>(nodes.size());
    std::vector<int32_t> kids(nn, 0);
    std::vector<char> gone(nn, 0);
    for (int32_t i = 0; i < nn; ++i) kids[i] = static_cast<int32_t>(nodes[i].child.size());
    std::unordered_map<int32_t, int32_t> live;  // page -> cached tokens left, for the pages touched so far
    int32_t done_partly = -1;                   // the one node of `keep` whose tail has been taken already
    freed = 0;
    while (freed < need_slots) {
        int32_t victim = -1;
        for (int32_t i = 1; i < nn; ++i) {
            const Node& nd = nodes[i];
            if (nd.tok.empty() || gone[i] || kids[i] != 0 || nd.ref != 0) continue;
            if (keep) {
                auto kp = keep->find(i);
                if (kp != keep->end() && (kp->second >= static_cast<int32_t>(nd.tok.size()) || done_partly == i)) continue;
            }
            if (victim < 0 || nd.last < nodes[victim].last) victim = i;
        }
        if (victim < 0) break;
        const Node& nd = nodes[victim];
        int32_t k = 0;
        int32_t len = static_cast<int32_t>(nd.tok.size());
        const int32_t full = len;
        if (keep) {
            auto kp = keep->find(victim);
            if (kp != keep->end()) len -= kp->second;  // only the tail past the part to keep
        }
        while (k < len && freed < need_slots) {
            const int32_t page = nd.slot[full - 1 - k] / p;
            auto it = live.find(page);
            if (it == live.end()) it = live.emplace(page, tree->page_live[page]).first;
            ++k;
            if (--it->second == 0) freed += p;
        }
        steps.push_back({victim, k});
        if (k == full) {
            gone[victim] = 1;
            --kids[nd.parent];
        } else if (k == len) {
            done_partly = victim;  // its head is to be kept: it stays a leaf, and has nothing more to give
        } else {
            break;  // a node that keeps its head: enough is free
        }
    }
}

}  // namespace pa

namespace pa {

// The cached part of a prompt as "tokens to keep" per node, and the slots its admission still needs.
static void keep_for_prompt(const pa_tree* tree, const int32_t* tokens, int32_t n,
                            std::unordered_map<int32_t, int32_t>& keep, int64_t& need_slots) {
    const auto& nodes = tree->nodes;
    int32_t cur = 0, pos = 0;
    while (pos < n) {
        auto it = nodes[cur].child.find(tokens[pos]);
        if (it == nodes[cur].child.end()) break;
        const int32_t c = it->second;
        const int32_t elen = static_cast<int32_t>(nodes[c].tok.size());
        const int32_t lim = std::min(elen, n - pos);
        int32_t k = 1;
        while (k < lim && nodes[c].tok[k] == tokens[pos + k]) ++k;
        keep.emplace(c, k);
        pos += k;
        if (k < elen) break;
        cur = c;
    }
    const int64_t p = tree->page_size;
    const int64_t pages = (static_cast<int64_t>(n - pos) + p - 1) / p;
    need_slots = std::max<int64_t>(0, pages * p - static_cast<int64_t>(tree->free_pages.size()) * p);
}

static int evict_locked(pa_tree* tree, int64_t need_slots, const std::unordered_map<int32_t, int32_t>* keep,
                        int64_t* freed_slots, int64_t* evicted_tokens) {
    auto& nodes = tree->nodes;
    const int32_t p = tree->page_size;
    int64_t freed = 0, planned = 0, gone = 0;
    std::vector<EvictStep> steps;
    plan_eviction(tree, need_slots, keep, steps, planned);
    for (const EvictStep& st : steps) {
        Node& nd = nodes[st.node];
        const int32_t first_tok = nd.tok.front();
        for (int32_t k = 0; k < st.tokens; ++k) {
            const int32_t page = nd.slot.back() / p;
            nd.tok.pop_back();
            nd.slot.pop_back();
            ++gone;
            if (--tree->page_live[page] == 0) {
                tree->free_pages.push_back(page);
                freed += p;
            }
        }
        if (nd.tok.empty()) {
            nodes[nd.parent].child.erase(first_tok);
            nd.parent = -1;
            nd.hits.clear();
            tree->free_nodes.push_back(st.node);
            mirror_remove(tree, st.node, st.tokens);
        } else {
            mirror_trim(tree, st.node, st.tokens);
        }
    }
    tree->n_tokens -= gone;
    if (gone) tree->uploaded = false;
    if (freed_slots) *freed_slots = freed;
    if (evicted_tokens) *evicted_tokens = gone;
    return PA_OK;
}

static int plan_locked(const pa_tree* tree, int64_t need_slots, const std::unordered_map<int32_t, int32_t>* keep,
                       int64_t since, int64_t cap, int32_t* node_tokens, int32_t* node_sharers, int64_t* n_nodes,
                       int64_t* n_requests) {
    std::vector<EvictStep> steps;
    int64_t freed = 0;
    plan_eviction(tree, need_slots, keep, steps, freed);
    // A node that goes whole, followed at once by its parent with the same count of sharers, is one entry: where
    // the tree happens to be cut along a path that the same requests used does not show in the result.
    std::vector<std::pair<int32_t, int32_t>> runs;  // (tokens, sharers)
    for (size_t k = 0; k < steps.size(); ++k) {
        const auto& hits = tree->nodes[steps[k].node].hits;
        const int32_t sharers = static_cast<int32_t>(hits.end() - std::upper_bound(hits.begin(), hits.end(), since));
        if (k > 0 && tree->nodes[steps[k - 1].node].parent == steps[k].node && runs.back().second == sharers)
            runs.back().first += steps[k].tokens;
        else
            runs.emplace_back(steps[k].tokens, sharers);
    }
    *n_nodes = static_cast<int64_t>(runs.size());
    if (n_requests)
        *n_requests = tree->admissions.end() - std::upper_bound(tree->admissions.begin(), tree->admissions.end(), since);
    if (static_cast<int64_t>(runs.size()) > cap)
        return fail(PA_ENOMEM, "pa_tree_evict_plan: %zu nodes, room for %lld", runs.size(), static_cast<long long>(cap));
    for (size_t k = 0; k < runs.size(); ++k) {
        node_tokens[k] = runs[k].first;
        node_sharers[k] = runs[k].second;
    }
    return PA_OK;
}

}  // namespace pa

extern "C" int pa_tree_evict(pa_tree* tree, int64_t need_slots, int64_t* freed_slots, int64_t* evicted_tokens) {
    PA_REQUIRE(tree != nullptr, "pa_tree_evict: tree is NULL");
    std::lock_guard<std::mutex> lk(tree->mu);
    if (tree->page_size == 0) return pa::fail(PA_ESTATE, "pa_tree_evict: no pool attached");
    try {
        return pa::evict_locked(tree, need_slots, nullptr, freed_slots, evicted_tokens);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_evict: out of host memory");
    }
}

extern "C" int pa_tree_evict_for(pa_tree* tree, const int32_t* tokens, int32_t n, int64_t* freed_slots,
                                 int64_t* evicted_tokens) {
    PA_REQUIRE(tree != nullptr && tokens != nullptr && n >= 1, "pa_tree_evict_for: bad argument");
    std::lock_guard<std::mutex> lk(tree->mu);
    if (tree->page_size == 0) return pa::fail(PA_ESTATE, "pa_tree_evict_for: no pool attached");
    try {
        std::unordered_map<int32_t, int32_t> keep;
        int64_t need = 0;
        pa::keep_for_prompt(tree, tokens, n, keep, need);
        return pa::evict_locked(tree, need, &keep, freed_slots, evicted_tokens);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_evict_for: out of host memory");
    }
}

extern "C" int pa_tree_evict_plan(const pa_tree* tree, int64_t need_slots, int64_t since, int64_t cap,
                                  int32_t* node_tokens, int32_t* node_sharers, int64_t* n_nodes, int64_t* n_requests) {
    PA_REQUIRE(tree != nullptr && n_nodes != nullptr, "pa_tree_evict_plan: NULL argument");
    PA_REQUIRE(cap >= 0 && (cap == 0 || (node_tokens && node_sharers)), "pa_tree_evict_plan: bad output arrays");
    std::lock_guard<std::mutex> lk(const_cast<pa_tree*>(tree)->mu);
    if (tree->page_size == 0) return pa::fail(PA_ESTATE, "pa_tree_evict_plan: no pool attached");
    try {
        return pa::plan_locked(tree, need_slots, nullptr, since, cap, node_tokens, node_sharers, n_nodes, n_requests);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_evict_plan: out of host memory");
    }
}

extern "C" int pa_tree_evict_plan_for(const pa_tree* tree, const int32_t* tokens, int32_t n, int64_t since, int64_t cap,
                                      int32_t* node_tokens, int32_t* node_sharers, int64_t* n_nodes,
                                      int64_t* n_requests) {
    PA_REQUIRE(tree != nullptr && n_nodes != nullptr && tokens != nullptr && n >= 1, "pa_tree_evict_plan_for: bad argument");
    PA_REQUIRE(cap >= 0 && (cap == 0 || (node_tokens && node_sharers)), "pa_tree_evict_plan_for: bad output arrays");
    std::lock_guard<std::mutex> lk(const_cast<pa_tree*>(tree)->mu);
    if (tree->page_size == 0) return pa::fail(PA_ESTATE, "pa_tree_evict_plan_for: no pool attached");
    try {
        std::unordered_map<int32_t, int32_t> keep;
        int64_t need = 0;
        pa::keep_for_prompt(tree, tokens, n, keep, need);
        return pa::plan_locked(tree, need, &keep, since, cap, node_tokens, node_sharers, n_nodes, n_requests);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_evict_plan_for: out of host memory");
    }
}

extern "C" int pa_tree_set_hit_window(pa_tree* tree, int64_t window) {
    PA_REQUIRE(tree != nullptr && window >= 0, "pa_tree_set_hit_window: bad argument");
    std::lock_guard<std::mutex> lk(tree->mu);
    tree->hit_window = window;
    return PA_OK;
}

extern "C" int pa_tree_stats(const pa_tree* tree, int64_t* n_nodes, int64_t* n_tokens) {
    PA_REQUIRE(tree != nullptr, "pa_tree_stats: tree is NULL");
    if (n_nodes) *n_nodes = static_cast<int64_t>(tree->nodes.size() - tree->free_nodes.size());
    if (n_tokens) *n_tokens = tree->n_tokens;
    return PA_OK;
}

static void release_device(pa_tree* t) {
    if (t->d_blob) {
        int prev = -1;
        if (hipGetDevice(&prev) == hipSuccess && prev != t->device && t->device >= 0) (void)hipSetDevice(t->device);
        (void)hipFree(t->d_blob);
        if (prev >= 0 && prev != t->device) (void)hipSetDevice(prev);
        t->d_blob = nullptr;
        t->d_cap = 0;
    }
    t->uploaded = false;
}

extern "C" int pa_tree_upload(pa_tree* tree, void* stream_) {
    PA_REQUIRE(tree != nullptr, "pa_tree_upload: tree is NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    std::lock_guard<std::mutex> lk(tree->mu);
    const auto& nodes = tree->nodes;
    const int64_t nn = static_cast<int64_t>(nodes.size());
    if (tree->n_tokens > INT32_MAX / 2 - 64 || nn > INT32_MAX / 8)
        return pa::fail(PA_EINVAL, "pa_tree_upload: tree too large for 32-bit indices");
    int cur_dev = -1;
    PA_HIP(hipGetDevice(&cur_dev));
    if (tree->copy_pending) {  // the copy before this one still reads the host buffer
        PA_HIP(hipEventSynchronize(tree->copied));
        tree->copy_pending = false;
    }
    if (!tree->copied) PA_HIP(hipEventCreateWithFlags(&tree->copied, hipEventDisableTiming));

    // ---- only what changed since the last upload ----
    if (tree->incremental && tree->mirror_ok && tree->d_blob && tree->device == cur_dev) {
        auto& dirty = tree->dirty;
        std::sort(dirty.begin(), dirty.end());
        // neighbours closer than 512 bytes go in one copy
        std::vector<std::pair<size_t, size_t>> runs;  // (offset, end)
        size_t bytes = 0;
        for (size_t i = 0; i < dirty.size();) {
            size_t lo = dirty[i].first, hi = lo + dirty[i].second;
            for (++i; i < dirty.size() && dirty[i].first <= hi + 512; ++i) hi = std::max(hi, dirty[i].first + dirty[i].second);
            runs.emplace_back(lo, hi);
            bytes += hi - lo;
        }
        dirty.clear();
        if (bytes) {
            // the runs are gathered into a transfer buffer (two take turns) and copied from there
            const int x = tree->xfer_next;
            tree->xfer_next ^= 1;
            if (tree->xfer_pending[x]) {  // the upload before the last one, long done as a rule
                PA_HIP(hipEventSynchronize(tree->xfer_done[x]));
                tree->xfer_pending[x] = false;
            }
            if (tree->xfer_cap[x] < bytes) {
                if (tree->h_xfer[x]) (void)hipHostFree(tree->h_xfer[x]);
                tree->h_xfer[x] = nullptr;
                tree->xfer_cap[x] = 0;
                const size_t want = bytes * 2 > (size_t(64) << 10) ? bytes * 2 : (size_t(64) << 10);
                if (hipHostMalloc(&tree->h_xfer[x], want, hipHostMallocDefault) != hipSuccess) {
                    (void)hipGetLastError();
                    tree->mirror_ok = false;
                    return pa::fail(PA_ENOMEM, "pa_tree_upload: %zu bytes of pinned host memory", want);
                }
                tree->xfer_cap[x] = want;
            }
            if (!tree->xfer_done[x]) PA_HIP(hipEventCreateWithFlags(&tree->xfer_done[x], hipEventDisableTiming));
            unsigned char* h = static_cast<unsigned char*>(tree->h_stage);
            unsigned char* d = static_cast<unsigned char*>(tree->d_blob);
            unsigned char* xb = static_cast<unsigned char*>(tree->h_xfer[x]);
            size_t at = 0;
            for (const auto& run : runs) {
                std::memcpy(xb + at, h + run.first, run.second - run.first);
                PA_HIP(hipMemcpyAsync(d + run.first, xb + at, run.second - run.first, hipMemcpyHostToDevice, stream));
                at += run.second - run.first;
            }
            PA_HIP(hipEventRecord(tree->xfer_done[x], stream));
            tree->xfer_pending[x] = true;
        }
        tree->view.n_nodes = static_cast<int32_t>(nn);
        tree->view.n_tokens = static_cast<int32_t>(tree->n_tokens);
        tree->uploaded = true;
        ++tree->n_incremental_uploads;
        tree->last_upload_bytes = static_cast<int64_t>(bytes);
        return PA_OK;
    }

    // ---- the whole flat form, rebuilt with room to grow ----
    tree->mirror_ok = false;
    tree->dirty.clear();
    const int64_t ntok = tree->n_tokens;
    uint64_t cap = 64;  // power of two >= 4 * (#nodes): at most half full after as many more entries; and at least 64
    while (cap < 4ull * static_cast<uint64_t>(nn)) cap <<= 1;  // so a 64-lane probe window never wraps onto itself
    tree->flat.set(ntok + ntok / 2 + 4096, nn + nn / 2 + 256, cap);
    const pa::FlatLayout& f = tree->flat;
    if (tree->h_cap < f.total) {
        if (tree->h_stage) (void)hipHostFree(tree->h_stage);
        tree->h_stage = nullptr;
        tree->h_cap = 0;
        if (hipHostMalloc(&tree->h_stage, f.total, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            return pa::fail(PA_ENOMEM, "pa_tree_upload: %zu bytes of pinned host memory", f.total);
        }
        tree->h_cap = f.total;
    }
    pa::FlatView v = pa::flat_view(tree);
    try {
        tree->ht_pos.assign(static_cast<size_t>(f.node_cap), -1);
        tree->phe_pos.assign(static_cast<size_t>(f.node_cap), -1);
        tree->end_depth.assign(static_cast<size_t>(f.node_cap), 0);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_upload: out of host memory");
    }
    const uint64_t mask = cap - 1;
    for (uint64_t i = 0; i < cap; ++i) {
        v.key[i] = pa::kEmptyKey;
        v.val[i] = -1;
    }
    std::memset(v.start, 0, static_cast<size_t>(f.node_cap) * 4);
    std::memset(v.len, 0, static_cast<size_t>(f.node_cap) * 4);
    std::memset(v.end, 0, static_cast<size_t>(f.node_cap) * 8);
    std::memset(v.phe, 0, cap * sizeof(pa::PathEntry));
    for (uint64_t i = 0; i < cap; ++i) v.phe[i].node = -1;

    int64_t cursor = 0, entries = 0;
    for (int64_t i = 0; i < nn; ++i) {
        const auto& nd = nodes[i];
        v.start[i] = static_cast<int32_t>(cursor);
        v.len[i] = static_cast<int32_t>(nd.tok.size());
        if (!nd.tok.empty()) {
            std::memcpy(v.tok + cursor, nd.tok.data(), nd.tok.size() * 4);
            std::memcpy(v.slot + cursor, nd.slot.data(), nd.slot.size() * 4);
        }
        cursor += static_cast<int64_t>(nd.tok.size());
        for (const auto& kv : nd.child) {
            const unsigned long long key =
                (static_cast<unsigned long long>(static_cast<uint32_t>(i)) << 32) | static_cast<uint32_t>(kv.first);
            uint64_t h = pa::hash_key(key) & mask;
            while (v.key[h] != pa::kEmptyKey) h = (h + 1) & mask;
            v.key[h] = key;
            v.val[h] = kv.second;
            tree->ht_pos[static_cast<size_t>(kv.second)] = static_cast<int32_t>(h);
            ++entries;
        }
    }
    std::memset(v.tok + cursor, 0, static_cast<size_t>(f.tok_cap - cursor) * 4);  // (edge reads may run past an edge's end)
    std::memset(v.slot + cursor, 0, static_cast<size_t>(f.tok_cap - cursor) * 4);

    // positional index: depth-first walk carrying the hash of the path so far (explicit stack: paths can be deep)
    try {
        struct Item { int32_t node; int32_t parent; int32_t depth; unsigned long long hash; };  // depth, hash: of the path BEFORE the node's edge
        std::vector<Item> stack;
        stack.push_back({0, -1, 0, 0ull});
        v.end[0] = 0ull;
        while (!stack.empty()) {
            const Item it = stack.back();
            stack.pop_back();
            const auto& nd = nodes[it.node];
            unsigned long long h = it.hash;
            if (it.node != 0) {
                const unsigned long long key = pa::path_hash_push(h, nd.tok[0]);
                uint64_t at = pa::path_slot(key, it.depth) & mask;
                while (v.phe[at].node != -1) at = (at + 1) & mask;
                v.phe[at].hash = key;
                v.phe[at].depth = it.depth;
                v.phe[at].node = it.node;
                v.phe[at].edge_start = v.start[it.node];
                v.phe[at].edge_len = v.len[it.node];
                v.phe[at].parent = it.parent;
                tree->phe_pos[static_cast<size_t>(it.node)] = static_cast<int32_t>(at);
                for (int32_t t : nd.tok) h = pa::path_hash_push(h, t);
                v.end[it.node] = h;
            }
            const int32_t end_depth = it.depth + static_cast<int32_t>(nd.tok.size());
            tree->end_depth[static_cast<size_t>(it.node)] = end_depth;
            for (const auto& kv : nd.child) stack.push_back({kv.second, it.node, end_depth, h});
        }
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_upload: out of host memory");
    }

    tree->uploaded = false;
    if (tree->d_blob == nullptr || tree->d_cap < f.total || tree->device != cur_dev) {
        release_device(tree);  // (hipFree waits for whatever still reads the old buffer)
        tree->device = cur_dev;
        void* fresh = nullptr;
        if (hipMalloc(&fresh, f.total) != hipSuccess) {
            (void)hipGetLastError();
            return pa::fail(PA_ENOMEM, "pa_tree_upload: hipMalloc of %zu bytes failed", f.total);
        }
        tree->d_blob = fresh;
        tree->d_cap = f.total;
    }
    void* d = tree->d_blob;
    PA_HIP(hipMemcpyAsync(d, tree->h_stage, f.total, hipMemcpyHostToDevice, stream));
    PA_HIP(hipEventRecord(tree->copied, stream));
    tree->copy_pending = true;
    unsigned char* b = static_cast<unsigned char*>(d);
    tree->view.edge_tok = reinterpret_cast<const int32_t*>(b + f.o_tok);
    tree->view.edge_slot = reinterpret_cast<const int32_t*>(b + f.o_slot);
    tree->view.node_start = reinterpret_cast<const int32_t*>(b + f.o_start);
    tree->view.node_len = reinterpret_cast<const int32_t*>(b + f.o_len);
    tree->view.ht_key = reinterpret_cast<const unsigned long long*>(b + f.o_key);
    tree->view.ht_val = reinterpret_cast<const int32_t*>(b + f.o_val);
    tree->view.ht_mask = static_cast<uint32_t>(cap - 1);
    tree->view.ph_entry = reinterpret_cast<const pa::PathEntry*>(b + f.o_phe);
    tree->view.node_endhash = reinterpret_cast<const unsigned long long*>(b + f.o_end);
    tree->view.ph_mask = static_cast<uint32_t>(cap - 1);
    tree->view.n_nodes = static_cast<int32_t>(nn);
    tree->view.n_tokens = static_cast<int32_t>(ntok);
    tree->uploaded = true;
    tree->mirror_ok = tree->incremental;
    tree->arena_end = cursor;
    tree->arena_holes = 0;
    tree->table_used = entries;
    ++tree->n_full_uploads;
    tree->last_upload_bytes = static_cast<int64_t>(f.total);
    return PA_OK;
}

extern "C" int pa_tree_set_incremental_upload(pa_tree* tree, int on) {
    PA_REQUIRE(tree != nullptr, "pa_tree_set_incremental_upload: tree is NULL");
    std::lock_guard<std::mutex> lk(tree->mu);
    tree->incremental = on != 0;
    if (!tree->incremental) {
        tree->mirror_ok = false;
        tree->dirty.clear();
    }
    return PA_OK;
}

extern "C" int pa_tree_upload_stats(const pa_tree* tree, int64_t* full, int64_t* incremental, int64_t* last_bytes) {
    PA_REQUIRE(tree != nullptr, "pa_tree_upload_stats: tree is NULL");
    if (full) *full = tree->n_full_uploads;
    if (incremental) *incremental = tree->n_incremental_uploads;
    if (last_bytes) *last_bytes = tree->last_upload_bytes;
    return PA_OK;
}

extern "C" int pa_tree_destroy(pa_tree* tree) {
    if (!tree) return PA_OK;
    if (tree->copied) {
        (void)hipEventSynchronize(tree->copied);
        (void)hipEventDestroy(tree->copied);
    }
    for (int x = 0; x < 2; ++x) {
        if (tree->xfer_done[x]) {
            (void)hipEventSynchronize(tree->xfer_done[x]);
            (void)hipEventDestroy(tree->xfer_done[x]);
        }
        if (tree->h_xfer[x]) (void)hipHostFree(tree->h_xfer[x]);
    }
    release_device(tree);
    if (tree->h_stage) (void)hipHostFree(tree->h_stage);
    delete tree;
    return PA_OK;
}

int pa_tree_device(const pa_tree* tree, const pa::DeviceTree** out) {
    if (!tree) return pa::fail(PA_EINVAL, "tree is NULL");
    if (!tree->uploaded)
        return pa::fail(PA_ESTATE, "tree not uploaded since its last insert (call pa_tree_upload)");
    *out = &tree->view;
    return PA_OK;
}
