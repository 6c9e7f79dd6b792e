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
    pa::DeviceTree view{};
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
    }
    t->uploaded = false;
}

extern "C" int pa_tree_upload(pa_tree* tree, void* stream_) {
    PA_REQUIRE(tree != nullptr, "pa_tree_upload: tree is NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    std::lock_guard<std::mutex> lk(tree->mu);
    const auto& nodes = tree->nodes;
    const int64_t nn = static_cast<int64_t>(nodes.size());
    if (tree->n_tokens > INT32_MAX - 64 || nn > INT32_MAX / 4)
        return pa::fail(PA_EINVAL, "pa_tree_upload: tree too large for 32-bit indices");

    // hash capacity: power of two >= 2 * (#edges), at least 64 so a 64-lane probe window never wraps onto itself
    uint64_t cap = 64;
    while (cap < 2ull * static_cast<uint64_t>(nn)) cap <<= 1;

    auto up = [](size_t x) { return (x + 255) & ~size_t(255); };
    const size_t ntok = static_cast<size_t>(tree->n_tokens);
    const size_t o_tok = 0;
    const size_t o_slot = o_tok + up((ntok + 64) * 4);
    const size_t o_start = o_slot + up((ntok + 64) * 4);
    const size_t o_len = o_start + up(nn * 4);
    const size_t o_key = o_len + up(nn * 4);
    const size_t o_val = o_key + up(cap * 8);
    const size_t o_phe = o_val + up(cap * 4);
    const size_t o_end = o_phe + up(cap * sizeof(pa::PathEntry));
    const size_t total = o_end + up(nn * 8);

    std::vector<unsigned char> blob;
    try {
        blob.assign(total, 0);
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_upload: out of host memory");
    }
    int32_t* h_tok = reinterpret_cast<int32_t*>(blob.data() + o_tok);
    int32_t* h_slot = reinterpret_cast<int32_t*>(blob.data() + o_slot);
    int32_t* h_start = reinterpret_cast<int32_t*>(blob.data() + o_start);
    int32_t* h_len = reinterpret_cast<int32_t*>(blob.data() + o_len);
    unsigned long long* h_key = reinterpret_cast<unsigned long long*>(blob.data() + o_key);
    int32_t* h_val = reinterpret_cast<int32_t*>(blob.data() + o_val);
    for (uint64_t i = 0; i < cap; ++i) { h_key[i] = pa::kEmptyKey; h_val[i] = -1; }

    int64_t cursor = 0;
    for (int64_t i = 0; i < nn; ++i) {
        const auto& nd = nodes[i];
        h_start[i] = static_cast<int32_t>(cursor);
        h_len[i] = static_cast<int32_t>(nd.tok.size());
        if (!nd.tok.empty()) {
            std::memcpy(h_tok + cursor, nd.tok.data(), nd.tok.size() * 4);
            std::memcpy(h_slot + cursor, nd.slot.data(), nd.slot.size() * 4);
        }
        cursor += static_cast<int64_t>(nd.tok.size());
        for (const auto& kv : nd.child) {
            const unsigned long long key =
                (static_cast<unsigned long long>(static_cast<uint32_t>(i)) << 32) | static_cast<uint32_t>(kv.first);
            uint64_t h = pa::hash_key(key) & (cap - 1);
            while (h_key[h] != pa::kEmptyKey) h = (h + 1) & (cap - 1);
            h_key[h] = key;
            h_val[h] = kv.second;
        }
    }

    // positional index: depth-first walk carrying the hash of the path so far (explicit stack: paths can be deep)
    pa::PathEntry* h_phe = reinterpret_cast<pa::PathEntry*>(blob.data() + o_phe);
    unsigned long long* h_end = reinterpret_cast<unsigned long long*>(blob.data() + o_end);
    for (uint64_t i = 0; i < cap; ++i) h_phe[i].node = -1;
    try {
        struct Item { int32_t node; int32_t parent; int32_t depth; unsigned long long hash; };  // depth, hash: of the path BEFORE the node's edge
        std::vector<Item> stack;
        stack.push_back({0, -1, 0, 0ull});
        h_end[0] = 0ull;
        while (!stack.empty()) {
            const Item it = stack.back();
            stack.pop_back();
            const auto& nd = nodes[it.node];
            unsigned long long h = it.hash;
            if (it.node != 0) {
                const unsigned long long key = pa::path_hash_push(h, nd.tok[0]);
                uint64_t at = pa::path_slot(key, it.depth) & (cap - 1);
                while (h_phe[at].node != -1) at = (at + 1) & (cap - 1);
                h_phe[at].hash = key;
                h_phe[at].depth = it.depth;
                h_phe[at].node = it.node;
                h_phe[at].edge_start = h_start[it.node];
                h_phe[at].edge_len = h_len[it.node];
                h_phe[at].parent = it.parent;
                for (int32_t t : nd.tok) h = pa::path_hash_push(h, t);
                h_end[it.node] = h;
            }
            const int32_t end_depth = it.depth + static_cast<int32_t>(nd.tok.size());
            for (const auto& kv : nd.child) stack.push_back({kv.second, it.node, end_depth, h});
        }
    } catch (const std::bad_alloc&) {
        return pa::fail(PA_ENOMEM, "pa_tree_upload: out of host memory");
    }

    release_device(tree);
    PA_HIP(hipGetDevice(&tree->device));
    void* d = nullptr;
    if (hipMalloc(&d, total) != hipSuccess) {
        (void)hipGetLastError();
        return pa::fail(PA_ENOMEM, "pa_tree_upload: hipMalloc of %zu bytes failed", total);
    }
    tree->d_blob = d;
    PA_HIP(hipMemcpyAsync(d, blob.data(), total, hipMemcpyHostToDevice, stream));
    PA_HIP(hipStreamSynchronize(stream));
    unsigned char* b = static_cast<unsigned char*>(d);
    tree->view.edge_tok = reinterpret_cast<const int32_t*>(b + o_tok);
    tree->view.edge_slot = reinterpret_cast<const int32_t*>(b + o_slot);
    tree->view.node_start = reinterpret_cast<const int32_t*>(b + o_start);
    tree->view.node_len = reinterpret_cast<const int32_t*>(b + o_len);
    tree->view.ht_key = reinterpret_cast<const unsigned long long*>(b + o_key);
    tree->view.ht_val = reinterpret_cast<const int32_t*>(b + o_val);
    tree->view.ht_mask = static_cast<uint32_t>(cap - 1);
    tree->view.ph_entry = reinterpret_cast<const pa::PathEntry*>(b + o_phe);
    tree->view.node_endhash = reinterpret_cast<const unsigned long long*>(b + o_end);
    tree->view.ph_mask = static_cast<uint32_t>(cap - 1);
    tree->view.n_nodes = static_cast<int32_t>(nn);
    tree->uploaded = true;
    return PA_OK;
}

extern "C" int pa_tree_destroy(pa_tree* tree) {
    if (!tree) return PA_OK;
    release_device(tree);
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
