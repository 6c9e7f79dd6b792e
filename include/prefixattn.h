/*
 * libprefixattn: prefix-cached "extend" prefill on one MI355X (gfx950).
 *
 * The paper (Preble, arXiv 2407.00023) schedules requests so that the KV of shared
 * prompt prefixes is computed once and reused; a request then costs only the prefill
 * of its missed tokens (Sec. 3.2, cost P of Algorithm 2).  This library is that
 * per-GPU computation: match each prompt against the radix tree of cached sequences,
 * run attention of the new tokens over the cached prefix KV plus themselves, and put
 * the new KV into the cache.
 *
 * Conventions
 *  - Every function returns PA_OK (0) or a negative error code and never throws or
 *    aborts; pa_last_error() returns a description of the most recent failure on the
 *    calling thread.
 *  - "host" / "device" says where a pointer must live.  Device buffers are owned by
 *    the caller (allocate them however you like, e.g. with PyTorch); the library owns
 *    only pa_tree objects (host structure and its device mirror).
 *  - Hot-path calls only enqueue work on `stream` (a hipStream_t passed as void*, NULL
 *    = the default stream); they do not synchronise and do not allocate.
 *  - All index arrays are int32.  Packed per-request arrays use an offsets array of
 *    B + 1 entries (offsets[0] = 0).
 *  - dtype: PA_F32 computes in fp32 throughout; PA_BF16 takes bf16 inputs, multiplies
 *    on the bf16 matrix cores with fp32 accumulation, keeps softmax in fp32, and
 *    writes bf16.  PA_BF16_KV8 is PA_BF16 for every tensor and all arithmetic, with the
 *    KV pool held in 8 bits per element (see "KV pool"): half the memory per cached token.
 *  - Supported shapes: D in {64, 128}; Hq a multiple of Hkv; page_size >= 1 dividing
 *    num_slots (any size, a power of two or not).  Tensor base pointers must be 16-byte aligned.
 */
#ifndef PREFIXATTN_H
#define PREFIXATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PA_OK 0
#define PA_EINVAL (-1) /* bad argument, shape or alignment */
#define PA_ENOMEM (-2) /* host or device allocation failed, or workspace too small */
#define PA_ESTATE (-3) /* tree not uploaded, or changed since the last upload */
#define PA_EHIP (-4)   /* HIP runtime error */
#define PA_EOVERFLOW (-5) /* the batch on the device is larger than the host-side sizes the call was given */

#define PA_F32 0
#define PA_BF16 1
#define PA_BF16_KV8 2 /* as PA_BF16, with the KV pool held in 8 bits per element (see "KV pool" below) */

typedef struct pa_tree pa_tree;

/* Text of the last error raised on this thread ("" if none).  Host. */
const char* pa_last_error(void);

/* ---------------------------------------------------------------------------------
 * Radix tree of cached token sequences (host side; not on the timed path).
 *
 * Sec. 3.2, "global scheduler data structures", and Sec. 3.3 (the per-GPU copy): a
 * radix tree over token ids.  Inserting a sequence matches it from the beginning until
 * no match exists and adds the rest as a new leaf; a node that matches only partly is
 * split into the matched part and the remainder; a sequence matching nothing starts a
 * new tree (here: a new child of one empty virtual root).
 * --------------------------------------------------------------------------------- */

/* Create an empty tree.  *out receives a handle owned by the library. */
int pa_tree_create(pa_tree** out);

/* Insert tokens[0..n) with the KV slot of each token (host pointers, copied).  A token
 * position already in the tree keeps the slot of its first insertion; slots passed for
 * such positions are ignored.  *n_already_cached (may be NULL) receives how many leading
 * tokens were present before the call.  Marks the device mirror stale. */
int pa_tree_insert(pa_tree* tree, const int32_t* tokens, const int32_t* slots, int32_t n,
                   int32_t* n_already_cached);

/* Bring the mirror on the current device up to date.  The flat form of the tree lives in a pinned
 * host buffer owned by the tree and follows every change of the tree as it happens (a new leaf
 * appends its tokens and adds two table entries, a split rewrites a few words, an eviction shortens
 * or deletes entries); an upload copies the byte ranges that changed since the last one, so its
 * cost follows the size of the change, not of the tree.  The first upload, and one after changes
 * that outgrew the room left in the flat form (it is rebuilt with half as much again) or left more
 * than half of its token array dead, copies everything.  Copies are enqueued on `stream` and the
 * call returns without waiting for them, so pa_match_prefixes calls that follow on the same stream
 * see the new tree; work that still reads the mirror on another stream must have finished before
 * the call.  Changed ranges are copied from a snapshot taken at the call, so the tree may change
 * again at once; only after an upload that copied everything does the next change of the tree wait
 * for the copy. */
int pa_tree_upload(pa_tree* tree, void* stream);

/* on = 0: every upload rebuilds and copies the whole flat form (for comparison).  Default: 1. */
int pa_tree_set_incremental_upload(pa_tree* tree, int on);

/* Uploads so far that copied everything / only the changes, and the bytes the last one copied
 * (each may be NULL). */
int pa_tree_upload_stats(const pa_tree* tree, int64_t* full, int64_t* incremental, int64_t* last_bytes);

/* Number of nodes (including the virtual root) and of stored tokens.  Either pointer may be NULL. */
int pa_tree_stats(const pa_tree* tree, int64_t* n_nodes, int64_t* n_tokens);

/* Free the tree and its device mirror.  NULL is allowed. */
int pa_tree_destroy(pa_tree* tree);

/* ---------------------------------------------------------------------------------
 * Cache bookkeeping on the host, the steps either side of the hot path (not timed with it).
 *
 * Sec. 3.3: the local scheduler keeps a prefix tree and the number of active requests sharing each
 * node; a new request is matched to the tree and the tree is updated; when memory is short a node,
 * or part of a node if a part is enough, is evicted by the access time of the requests (LRU).  The
 * paper says nothing of pages: as for the workloads, the new part of a prompt receives whole pages
 * and token t of it sits in slot page[t / page_size] * page_size + t % page_size.  All pointers are
 * host pointers.  Every call that changes the tree marks the device mirror stale (pa_tree_upload).
 * --------------------------------------------------------------------------------- */

/* Give the (still empty) tree a pool of num_slots slots in pages of page_size: from then on slots
 * come from pa_tree_admit (pa_tree_insert returns PA_ESTATE).  Page 0 is handed out first, freed
 * pages are reused last-freed-first. */
int pa_tree_attach_pool(pa_tree* tree, int64_t num_slots, int page_size);

/* Slots in pages that hold no cached token. */
int pa_tree_free_slots(const pa_tree* tree, int64_t* free_slots);

/* Admit a request: match tokens[0..n) (n >= 1) to the tree, store the part that is not cached in
 * freshly allocated pages, pin every node on the prompt's path (one more active request) and make
 * the path the most recently used (time `now`, which must grow from one admission to the next).
 * *n_cached (may be NULL) receives the number of cached leading tokens, new_slots[n_cached .. n)
 * the slots of the new tokens (what pa_append_kv needs; entries below n_cached are not written),
 * *handle what pa_tree_release takes.  PA_ENOMEM if the free pages do not suffice: nothing is
 * stored or pinned then (evict and call again). */
int pa_tree_admit(pa_tree* tree, const int32_t* tokens, int32_t n, int64_t now, int32_t* new_slots,
                  int32_t* n_cached, int64_t* handle);

/* The request of this handle has finished: its path is no longer pinned by it. */
int pa_tree_release(pa_tree* tree, int64_t handle);

/* Evict until at least need_slots slots are in free pages, or nothing evictable is left: the
 * least recently used leaf that no admitted request runs through goes first, from its tail,
 * token by token, and only as far as needed; a parent whose children are all gone is a leaf in
 * turn.  *freed_slots (may be NULL) receives the slots of the pages that became free,
 * *evicted_tokens (may be NULL) the number of tokens dropped from the tree. */
int pa_tree_evict(pa_tree* tree, int64_t need_slots, int64_t* freed_slots, int64_t* evicted_tokens);

/* Make room for a prompt about to be admitted: as pa_tree_evict with need_slots = the whole pages
 * its part that is not cached needs, less the free ones, and never dropping a token of its cached
 * part (a request must not evict the prefix it is about to reuse). */
int pa_tree_evict_for(pa_tree* tree, const int32_t* tokens, int32_t n, int64_t* freed_slots,
                      int64_t* evicted_tokens);

/* Admission times older than `window` before the latest admission are forgotten from then on
 * (0, the default: none is).  They are what pa_tree_evict_plan counts sharers from. */
int pa_tree_set_hit_window(pa_tree* tree, int64_t window);

/* What pa_tree_evict(tree, need_slots, ...) would drop, without dropping it (the eviction set behind the
 * second cost term of Sec. 3.2 and Algorithm 2).  node_tokens[k] receives the number
 * of tokens the k-th victim would lose (all of a node, or its tail), node_sharers[k] the number of
 * admissions later than time `since` whose prompt ran through that node (a node that goes whole
 * and is followed at once by its parent with the same count forms one entry with it: where a path
 * used by the same requests happens to be cut does not show); at most `cap` entries
 * are written, *n_nodes receives the number there are (PA_ENOMEM if it exceeds cap), and
 * *n_requests (may be NULL) the number of admissions later than `since` in the whole tree. */
int pa_tree_evict_plan(const pa_tree* tree, int64_t need_slots, int64_t since, int64_t cap, int32_t* node_tokens,
                       int32_t* node_sharers, int64_t* n_nodes, int64_t* n_requests);

/* The same for pa_tree_evict_for(tree, tokens, n, ...): the E of Algorithm 2 for this prompt. */
int pa_tree_evict_plan_for(const pa_tree* tree, const int32_t* tokens, int32_t n, int64_t since, int64_t cap,
                           int32_t* node_tokens, int32_t* node_sharers, int64_t* n_nodes, int64_t* n_requests);

/* ---------------------------------------------------------------------------------
 * Scheduling decisions on the host: plain functions over numbers the caller holds (all host
 * pointers; nothing here touches the GPU).  The matcher's prefix lengths are their input.
 * --------------------------------------------------------------------------------- */

/* Sec. 3.3, "waiting queue request ordering": with P priority groups a request belongs to the
 * group given by the cached share of its prompt, in whole P-ths (63 of 100 tokens cached, P = 10:
 * group 6).  Groups run from 0 to P; only a fully cached prompt is in group P. */
int pa_priority_group(int32_t cached_len, int32_t prompt_len, int32_t P, int32_t* group);

/* Sec. 3.3 and Algorithm 3: choose the next batch of at most n_pick requests from a waiting queue
 * given in arrival order (cached_len[i], prompt_len[i] of waiting request i).  Group p takes a share
 * of the picks in proportion to p (55 picks from full groups: 10 from group 10, 9 from group 9, ...,
 * 1 from group 1), by largest remainder, ties to the higher group; what a group cannot use is shared
 * out again the same way among the groups that still have requests; group 0 has weight 0 and fills
 * what the others leave.  Inside a group requests leave in arrival order.  picked[0 .. *n_picked)
 * (room for min(n_pick, n_waiting) entries) receives queue indices, higher groups first. */
int pa_priority_select(const int32_t* cached_len, const int32_t* prompt_len, int64_t n_waiting, int32_t P,
                       int64_t n_pick, int32_t* picked, int64_t* n_picked);

/* The two regression functions of Sec. 3.2 (time against token count, from profiling; the paper
 * prints no coefficients): PrefillTime(n) = prefill_per_token * n + prefill_base for n > 0, 0 for
 * n = 0, DecodeTime likewise.  default_output_len stands in for the average output length of a
 * GPU on which no request has finished inside the window. */
typedef struct pa_cost_model {
    double prefill_per_token, prefill_base, decode_per_token, decode_base, default_output_len;
} pa_cost_model;

/* Algorithm 2, load cost of one GPU for one new request: *L = sum over the n_hist requests of the
 * window of PrefillTime(hist_missed_len[r]) + DecodeTime(avg_output_len); *M = sum over the n_evict
 * nodes that would be evicted of PrefillTime(evict_tokens[j]) * evict_sharers[j] / n_requests
 * (0 if n_requests is 0); *P = PrefillTime(missed_len_k).  The cost is their sum. */
int pa_e2_load_cost(const pa_cost_model* model, const int32_t* hist_missed_len, int64_t n_hist,
                    double avg_output_len, const int32_t* evict_tokens, const int32_t* evict_sharers,
                    int64_t n_evict, int64_t n_requests, int32_t missed_len_k, double* L, double* M, double* P);

#define PA_EXPLOIT 0        /* sent to a GPU that caches the longest node of the matched path */
#define PA_EXPLORE_DECODE 1 /* sent to the GPU most loaded with decoding */
#define PA_EXPLORE_COST 2   /* sent to the GPU of lowest load cost */

/* Algorithm 1 for one request over n_gpus GPUs.  If the missed part (prompt_len - cached_len) is
 * shorter than the cached part, and on_longest_node[i] != 0 for some GPU (GPU i caches the longest
 * node of the matched path), the request goes to the flagged GPU of lowest cost[i].  Otherwise, if
 * the highest decode_ratio[i] exceeds imbal_r it goes there, else to the GPU of lowest cost[i].
 * Ties go to the lowest index. */
int pa_e2_schedule(int32_t prompt_len, int32_t cached_len, const uint8_t* on_longest_node, const double* cost,
                   const double* decode_ratio, double imbal_r, int32_t n_gpus, int32_t* gpu, int32_t* mode);

/* The flags pa_e2_schedule takes, from the cached lengths alone, for callers that keep one prefix tree
 * per GPU and no global tree with its nodes: the matched path (as long as the longest cached_len[i])
 * is cut where the GPUs' cached lengths differ, the longest piece (the first, if several are as long)
 * stands for the longest node, and on_longest_node[i] = 1 for the GPUs whose cache reaches its end.
 * All zero if nothing is cached anywhere. */
int pa_e2_longest_piece(const int32_t* cached_len, int32_t n_gpus, uint8_t* on_longest_node);

/* Per-GPU request history over the window H of Sec. 3.2 (first cost): what L and the decode ratio
 * are computed from.  Times are the caller's integers (any unit; the window is in the same unit);
 * a request counts at time `now` if now - window < its time <= now. */
typedef struct pa_history pa_history;
int pa_history_create(int32_t n_gpus, int64_t window, const pa_cost_model* model, pa_history** out);
int pa_history_destroy(pa_history* h);
/* A request with missed_len tokens to prefill was assigned to `gpu` at time `now`. */
int pa_history_assign(pa_history* h, int32_t gpu, int64_t now, int32_t missed_len);
/* A request on `gpu` finished at time `now` after output_len generated tokens. */
int pa_history_complete(pa_history* h, int32_t gpu, int64_t now, int32_t output_len);
/* *L as in pa_e2_load_cost over the window; *decode_ratio = decode time / (prefill + decode time)
 * of the window (0 if it is empty): the share of "decoding-phase" work on that GPU;
 * *n_requests the assignments in the window; *avg_output_len the average the decode time used.
 * Any of the four may be NULL.  Entries older than the window are dropped. */
int pa_history_gpu_load(pa_history* h, int32_t gpu, int64_t now, double* L, double* decode_ratio,
                        int64_t* n_requests, double* avg_output_len);

/* ---------------------------------------------------------------------------------
 * KV pool.  num_slots rows, each holding K and V of one token for all Hkv heads.  The
 * byte layout is private to the library: only pa_append_kv writes it and only
 * pa_extend_attention / pa_gather_kv read it.  The caller allocates
 * pa_kv_pool_bytes(...) bytes of device memory (16-byte aligned); contents of slots
 * never appended are never read for a request whose slot_idx does not name them.
 *
 * With PA_BF16_KV8 (Sec. 3.3: memory for KV decides what can stay cached; the paper fixes no
 * storage format, this one is the library's) a row - the D elements of one token, KV head and
 * K or V - is kept as D one-byte codes and one signed exponent byte k: the value stored is
 * decode(code) * 2^k, the code being the 8-bit floating-point format with 4 exponent bits
 * (bias 7), 3 mantissa bits, no infinities and largest value 448.  pa_append_kv chooses k as
 * the smallest integer with max|row| * 2^-k <= 448 (0 for a row of zeros, kept within
 * [-100, 119]) and rounds x * 2^-k to the nearest code, ties to the even mantissa, anything
 * still above 448 to 448.  Every stored value is exactly a finite bf16; pa_gather_kv returns
 * those values, and pa_extend_attention computes over them as PA_BF16 does over its pool.
 * Rows given to pa_append_kv must be finite.  The pool takes num_slots * 2 * Hkv * (D + 1)
 * bytes.
 * --------------------------------------------------------------------------------- */
size_t pa_kv_pool_bytes(int64_t num_slots, int Hkv, int D, int dtype, int page_size);

/* Bytes of device workspace pa_extend_attention needs for any batch with at most B
 * requests, T extend tokens in total and prefix_len[r] + ext_len[r] <= max_kv_len.
 * It holds the work list of the launch and the partial results of row tiles whose key range is
 * split over several workgroups; with bf16 at serving sizes the bound on the latter dominates
 * (about 135 MB for 8 KV heads of 128: 2 x 2 parts per workgroup slot, each 128 rows of fp32).
 * Returns 0 for invalid arguments. */
size_t pa_extend_workspace_bytes(int B, int64_t T, int64_t max_kv_len, int Hq, int Hkv, int D, int dtype);

/* ---------------------------------------------------------------------------------
 * The hot path.  All pointers below are DEVICE pointers unless marked otherwise.
 * --------------------------------------------------------------------------------- */

/* Longest-prefix match (Algorithm 1: "match R_k to the radix tree; cached_len = sum of
 * matched length"; Sec. 3.3: the local scheduler matches each new request to its tree).
 *
 * tokens     int32 [offsets[B]]  prompts of the B requests, packed
 * offsets    int32 [B + 1]
 * prefix_len int32 [B]           out: number of leading prompt tokens found in the tree.
 *                                The match is token-granular: it may end inside a tree
 *                                node (nothing is split) and may equal the prompt length.
 * slot_idx   int32 [offsets[B]]  out: slot_idx[offsets[r] + j] = KV slot of prompt token
 *                                j for j < prefix_len[r]; entries past that are
 *                                unspecified (never read by pa_extend_attention).
 * The tree must have been uploaded after its last insert (else PA_ESTATE).  B = 0 is a
 * no-op.  Read-only on the tree: concurrent matches on different streams are safe.  (For
 * batches of up to 64 requests, on a tree whose edges hold at most 4,096 tokens on average,
 * a prompt longer than 4,096 tokens is matched by several workgroups, which meet in one of
 * 64 small buffers of the library's own, taken in turn: more than 64 such calls in flight
 * at once on one device are not supported.) */
int pa_match_prefixes(const pa_tree* tree, const int32_t* tokens, const int32_t* offsets, int B,
                      int32_t* prefix_len, int32_t* slot_idx, void* stream);

/* Extend attention: the prefill of the missed tokens with the cached prefix reused
 * (Sec. 2.1 and Sec. 3.2: only non-cached tokens are computed; Sec. 5: prefix reuse is
 * lossless, so the result equals causal attention over the whole prompt).
 *
 * For request r with P = prefix_len[r], E = ext_len[r], extend row i < E and query head h
 * (KV head g = h / (Hq / Hkv)), the visible keys are the P prefix tokens, read from the
 * pool at slot_idx[slot_offsets[r] + j], j < P, followed by extend tokens 0..i:
 *     out[e0 + i, h, :] = sum_j softmax_j(scale * <q_ext[e0 + i, h, :], K_j[g, :]>) V_j[g, :]
 * with e0 = ext_offsets[r].
 *
 * q_ext        [T, Hq, D]   k_ext, v_ext  [T, Hkv, D]   out [T, Hq, D]   (dtype elements; bf16 with PA_BF16_KV8)
 * kv_pool      pool written by pa_append_kv with the same Hkv, D, dtype, page_size, num_slots
 * slot_idx, slot_offsets   as produced by pa_match_prefixes (slot_offsets = its offsets).  The bf16 path lets
 *                requests that share a prefix, or a first part of it, share row tiles, and finds them by comparing
 *                slots: two requests count as sharing positions [0, n) if their lists agree in length (whole
 *                prefixes) and at position n - 1 and at a few places before it.  Lists that name the cached tokens
 *                of one prefix tree (the matcher's, or lists built from a request's own slots as in chunked
 *                prefill: cached prefix + its earlier chunks) agree everywhere once they agree there.  For lists of
 *                any other origin, in which two requests may hold the same slot at the same position behind different
 *                slots, call pa_extend_set_row_sharing(0) first: every request then walks its own list only.
 * prefix_len, ext_len      int32 [B];  ext_offsets int32 [B + 1], ext_offsets[B] = T
 * T, max_kv_len  HOST values: total extend tokens, and an upper bound on
 *                prefix_len[r] + ext_len[r] (used to size the launch; a request exceeding
 *                it is still computed correctly, only less efficiently)
 * workspace    at least pa_extend_workspace_bytes(B, T, max_kv_len, ...) bytes, 256-byte aligned
 * Requests with ext_len[r] = 0 produce no output rows.  Prefix slots must lie in
 * [0, num_slots); a slot outside is clamped into the pool (no fault, result for that
 * request unspecified).  out must not alias the inputs. */
int pa_extend_attention(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                        const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                        const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T,
                        int64_t max_kv_len, int Hq, int Hkv, int D, int page_size, int64_t num_slots,
                        int dtype, float scale, void* out, void* workspace, size_t workspace_bytes,
                        void* stream);

/* pa_extend_attention for callers that cannot allocate device memory - code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc - and so cannot supply a workspace: the same computation with the same
 * arguments (minus workspace and workspace_bytes), its work list and partial results kept in a buffer of
 * PA_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the library runs on holds its copy from
 * the first use until the process ends).  The call allocates nothing and frees nothing.  To fit that buffer the
 * launch aims at one work item per workgroup slot instead of three, so long key ranges are cut into fewer parts
 * (results agree with pa_extend_attention within the tolerance of the dtype, bit for bit where no row tile is split);
 * a batch whose plan still does not fit is refused with PA_ENOMEM and a message that names both sizes, and nothing
 * is launched.  All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU - on different
 * streams or from different threads - race, and the caller must order them.  Nothing in the buffer has to be zero
 * beforehand (each call writes every word it later reads).  The very first call on a device looks the buffer's
 * address up (hipGetSymbolAddress); make it once outside any stream capture.  PA_F32 needs no workspace and simply runs. */
#define PA_STATIC_SCRATCH_BYTES (80u << 20)
int pa_extend_attention_static(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                               const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                               const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T,
                               int64_t max_kv_len, int Hq, int Hkv, int D, int page_size, int64_t num_slots,
                               int dtype, float scale, void* out, void* stream);

/* Whether the most recent bf16 pa_extend_attention launch that used `workspace` (device pointer) could lay out its
 * work.  The launch is sized from the host values T and max_kv_len; if ext_len on the device adds up to more
 * row tiles than T allows, or the key ranges to more parts than max_kv_len allows, the kernels compute nothing, write
 * no output row and leave a mark in the workspace.  This call waits for `stream`, reads the mark and returns
 * PA_EOVERFLOW if it is set, PA_OK otherwise.  (pa_extend_attention itself never waits for the device, so it cannot
 * report this.)  Undefined for a workspace that no bf16 launch has used. */
int pa_extend_status(const void* workspace, void* stream);

/* Process-wide switch for the bf16 path, on by default: on = 0 gives every request row tiles of its own, so that
 * nothing is concluded from equal slots in different requests' lists (see slot_idx above); slower where prefixes
 * are shared and rows are few.  Takes effect from the next pa_extend_attention call. */
int pa_extend_set_row_sharing(int on);

/* Cache the KV of newly computed tokens (Sec. 3.2: a prefix stays cached on its GPU from
 * its first assignment until eviction): pool[new_slots[t]] = (k_ext[t], v_ext[t]).
 * new_slots int32 [T], pairwise distinct and in [0, num_slots).  Distinctness is the
 * caller's responsibility (duplicate slots leave one of the rows, unspecified which); a
 * slot outside the pool is skipped. */
int pa_append_kv(void* kv_pool, const int32_t* new_slots, const void* k_ext, const void* v_ext, int64_t T,
                 int Hkv, int D, int page_size, int64_t num_slots, int dtype, void* stream);

/* Inverse of pa_append_kv, for tests and debugging (not on the timed path): copies the
 * pool rows of slots[0..n) into dense k_out, v_out [n, Hkv, D]. */
int pa_gather_kv(const void* kv_pool, const int32_t* slots, int64_t n, int Hkv, int D, int page_size,
                 int64_t num_slots, int dtype, void* k_out, void* v_out, void* stream);

/* ---------------------------------------------------------------------------------
 * Per-kernel timing for benchmarks (not part of the method).  While enabled, every kernel
 * the library launches is bracketed by two HIP events on its stream (this creates events on
 * first use, so do not enable it under stream capture).  pa_profile_enable(1) clears the
 * records and starts recording, pa_profile_enable(0) stops.  pa_profile_read waits for the
 * recorded events and returns the summed device time (ms) and the number of launches of one
 * kernel, named "match_prefixes", "extend_plan", "extend_attention", "extend_merge",
 * "extend_attention_f32", "append_kv", "gather_kv", "calib_copy" or "calib_mfma".  At most 65536 launches are recorded.
 * --------------------------------------------------------------------------------- */
int pa_profile_enable(int on);
int pa_profile_read(const char* kernel, double* total_ms, int64_t* launches);

/* Clock probe, for benchmarks: after pa_profile_enable(2) (timing plus the probe; the probed kernel reads
 * two clocks more per workgroup, so time it with pa_profile_enable(1)), a few workgroups of every bf16
 * extend-attention launch add the shader cycles and the ticks of the constant 100 MHz counter that pass across their key
 * loop to two counters in the workspace (device pointer, the one given to pa_extend_attention).
 * reset != 0 zeroes the counters; reset == 0 reads them: *shader_mhz = 100 * cycles / ticks, the clock
 * the kernel actually ran at (0 if nothing was recorded).  Synchronises the device. */
int pa_profile_clock(void* workspace, int reset, double* shader_mhz);

/* Calibration kernels, for benchmarks (not part of the method): what this GPU reaches on a plain streaming copy and on
 * a loop of nothing but bf16 MFMAs, to set a kernel's distance from the published peaks against.  Both are
 * asynchronous on the stream and are recorded by the per-kernel timing above as "calib_copy" and "calib_mfma".
 * pa_calib_copy: dst[0..bytes) = src[0..bytes) (device pointers, 16-byte aligned, bytes a multiple of 16); it moves
 * 2 * bytes.  pa_calib_mfma: 512 workgroups of four waves (two per compute unit) each run `iters` rounds of four
 * independent 32x32x16 bf16 MFMAs per wave; *flops (host) receives the flops of the launch.  out: device, 16-byte
 * aligned, at least 16,400 bytes; its first two 64-bit words receive the shader cycles and the ticks of the 100 MHz
 * constant counter that one wave spent in its loop (clock in MHz = 100 * cycles / ticks).  PA_EINVAL on bad arguments. */
int pa_calib_copy(void* dst, const void* src, size_t bytes, void* stream);
int pa_calib_mfma(void* out, size_t out_bytes, int iters, int64_t* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PREFIXATTN_H */
