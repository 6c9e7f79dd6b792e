/*
 * CPU oracle for the prefix-cached extend-prefill path.  TEST INFRASTRUCTURE ONLY:
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it; the
 * product (the HIP library) never does, and the two share no code.
 *
 * Everything here is the plain definition, written for checking by eye:
 *
 *  - Prefix match (paper Sec. 3.2 "global scheduler data structures", Sec. 3.3, and
 *    Algorithm 1's "match R_k to the radix tree; cached_len = sum of matched length"):
 *    a trie with ONE token per node.  Inserting a sequence walks from the root while
 *    the next token has a child, then adds one node per remaining token.  A position
 *    that already exists keeps the slot it was first given.  Matching a prompt walks
 *    the same way; the number of nodes visited is the matched length, and the slots
 *    stored on those nodes are the KV slots of the matched tokens.  A radix tree with
 *    node splitting represents the same set of prefixes, so it must return the same.
 *
 *  - Extend attention (the computation the paper prices as "prefill of the missed
 *    tokens", Sec. 3.2 cost P, with cached prefix KV reused losslessly, Sec. 5): for
 *    request r, extend row i, query head h (kv head g = h / (Hq/Hkv)) the visible keys
 *    are the P_r cached prefix tokens (rows of the pool at slot_idx[r][0..P_r)) followed
 *    by extend tokens 0..i.  score_j = scale * <q, k_j>; out = sum_j softmax(score)_j v_j.
 *    All arithmetic in fp64 on the stored input values (bf16 widened exactly).
 *
 *  - append_kv: pool[slot[t]] = (k_ext[t], v_ext[t]).
 *
 * No blocking, no online softmax, no reordering: one row at a time.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ trie */

typedef struct {
    int64_t n, cap;
    int32_t *token;        /* token on the edge into this node */
    int32_t *slot;         /* KV slot of that token (first insertion wins) */
    int64_t *first_child;  /* -1 if none */
    int64_t *next_sibling; /* -1 if none */
} ora_trie;

static int64_t trie_new_node(ora_trie *t, int32_t token, int32_t slot) {
    if (t->n == t->cap) {
        t->cap = t->cap ? t->cap * 2 : 1024;
        t->token = (int32_t *)realloc(t->token, t->cap * sizeof(int32_t));
        t->slot = (int32_t *)realloc(t->slot, t->cap * sizeof(int32_t));
        t->first_child = (int64_t *)realloc(t->first_child, t->cap * sizeof(int64_t));
        t->next_sibling = (int64_t *)realloc(t->next_sibling, t->cap * sizeof(int64_t));
    }
    int64_t id = t->n++;
    t->token[id] = token;
    t->slot[id] = slot;
    t->first_child[id] = -1;
    t->next_sibling[id] = -1;
    return id;
}

ora_trie *ora_trie_new(void) {
    ora_trie *t = (ora_trie *)calloc(1, sizeof(ora_trie));
    trie_new_node(t, -1, -1); /* node 0: the empty virtual root of the forest */
    return t;
}

void ora_trie_free(ora_trie *t) {
    if (!t) return;
    free(t->token); free(t->slot); free(t->first_child); free(t->next_sibling);
    free(t);
}

int64_t ora_trie_num_nodes(const ora_trie *t) { return t->n; }

static int64_t trie_child(const ora_trie *t, int64_t node, int32_t token) {
    for (int64_t c = t->first_child[node]; c >= 0; c = t->next_sibling[c])
        if (t->token[c] == token) return c;
    return -1;
}

/* returns how many leading tokens were already present */
int64_t ora_trie_insert(ora_trie *t, const int32_t *tok, const int32_t *slot, int64_t n) {
    int64_t node = 0, j = 0;
    for (; j < n; ++j) {
        int64_t c = trie_child(t, node, tok[j]);
        if (c < 0) break;
        node = c;
    }
    int64_t already = j;
    for (; j < n; ++j) {
        int64_t c = trie_new_node(t, tok[j], slot[j]);
        t->next_sibling[c] = t->first_child[node];
        t->first_child[node] = c;
        node = c;
    }
    return already;
}

/* prefix_len[r] and slot_idx[offsets[r] + j] for j < prefix_len[r]; other entries of
   slot_idx are set to -1. */
void ora_trie_match(const ora_trie *t, const int32_t *tokens, const int32_t *offsets, int B,
                    int32_t *prefix_len, int32_t *slot_idx) {
    for (int r = 0; r < B; ++r) {
        const int32_t *p = tokens + offsets[r];
        int32_t n = offsets[r + 1] - offsets[r];
        int64_t node = 0;
        int32_t j = 0;
        for (; j < n; ++j) {
            int64_t c = trie_child(t, node, p[j]);
            if (c < 0) break;
            slot_idx[offsets[r] + j] = t->slot[c];
            node = c;
        }
        prefix_len[r] = j;
        for (int32_t k = j; k < n; ++k) slot_idx[offsets[r] + k] = -1;
    }
}

/* ------------------------------------------------------------------ values */

/* dtype 0: float32 storage; dtype 1: bfloat16 bit patterns in uint16 */
static inline double load_val(const void *base, int64_t idx, int dtype) {
    if (dtype == 0) return (double)((const float *)base)[idx];
    uint32_t u = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static inline size_t elt_size(int dtype) { return dtype == 0 ? 4 : 2; }

/* ------------------------------------------------------------------ append_kv */

/* pool_k, pool_v: [num_slots][Hkv][D] in the oracle's own dense layout */
void ora_append_kv(void *pool_k, void *pool_v, const int32_t *new_slots, const void *k_ext,
                   const void *v_ext, int64_t T, int Hkv, int D, int dtype) {
    size_t row = (size_t)Hkv * D * elt_size(dtype);
    for (int64_t t = 0; t < T; ++t) {
        memcpy((char *)pool_k + (size_t)new_slots[t] * row, (const char *)k_ext + (size_t)t * row, row);
        memcpy((char *)pool_v + (size_t)new_slots[t] * row, (const char *)v_ext + (size_t)t * row, row);
    }
}

/* ------------------------------------------------------------------ fp8 KV rows */

/*
 * The fp8 form of the KV pool (a reading of this build, not of the paper, which stores no KV format: memory for KV
 * bounds what stays cached, Sec. 3.3).  A row = the D elements of one (token, KV head, K or V).  It is stored as D
 * codes in the 8-bit format with 4 exponent bits (bias 7), 3 mantissa bits, no infinities and largest value 448, and
 * one exponent k per row: stored value = decode(code) * 2^k.  k is the smallest integer with max|row| * 2^-k <= 448
 * (0 for a row of zeros, kept within [-100, 119]); code = x * 2^-k rounded to the nearest representable value, ties to
 * the one with an even mantissa, and what still exceeds 448 (only where k was cut at 119: values within a factor 1.14
 * of the largest bfloat16) becomes 448.  Every stored value is exactly a finite bfloat16, so the pool that attention
 * reads can be held, without loss, as the bfloat16 rows this function returns.
 */
static double e4m3_value(int code) { /* code 0..126 (sign apart); 127 would be NaN and is never produced */
    int e = code >> 3, m = code & 7;
    return e == 0 ? ldexp((double)m, -9) : ldexp(1.0 + m / 8.0, e - 7);
}

static int e4m3_nearest(double a) { /* 0 <= a <= 448 */
    /* the two neighbours of a among the 127 non-negative values, then nearest, ties to even */
    int lo = 0, hi = 126;
    while (hi - lo > 1) {
        int mid = (lo + hi) / 2;
        if (e4m3_value(mid) <= a) lo = mid; else hi = mid;
    }
    if (e4m3_value(hi) <= a) return hi;
    double dl = a - e4m3_value(lo), dh = e4m3_value(hi) - a;
    if (dl < dh) return lo;
    if (dh < dl) return hi;
    return (lo & 1) ? hi : lo;
}

/* rows: n rows of D bfloat16 bit patterns.  codes (n * D bytes, sign in bit 7), exps (n) and stored (n * D bfloat16
 * bit patterns of the stored values) may each be NULL. */
void ora_fp8_rows(const uint16_t *rows, int64_t n, int D, uint8_t *codes, int8_t *exps, uint16_t *stored) {
    for (int64_t r = 0; r < n; ++r) {
        double amax = 0.0;
        for (int d = 0; d < D; ++d) {
            double x = fabs(load_val(rows, r * D + d, 1));
            if (x > amax) amax = x;
        }
        int k = 0;
        if (amax > 0.0) {
            int e;
            double m = frexp(amax / 448.0, &e); /* amax / 448 = m * 2^e, 0.5 <= m < 1 */
            k = (m == 0.5) ? e - 1 : e;
            if (k < -100) k = -100;
            if (k > 119) k = 119;
        }
        if (exps) exps[r] = (int8_t)k;
        for (int d = 0; d < D; ++d) {
            double x = load_val(rows, r * D + d, 1);
            double y = ldexp(fabs(x), -k);
            int code = e4m3_nearest(y > 448.0 ? 448.0 : y);
            if (codes) codes[r * D + d] = (uint8_t)(code | (signbit(x) ? 0x80 : 0));
            if (stored) {
                float f = (float)(ldexp(e4m3_value(code), k) * (signbit(x) ? -1.0 : 1.0)); /* exact */
                uint32_t u;
                memcpy(&u, &f, 4);
                stored[r * D + d] = (uint16_t)(u >> 16); /* the low 16 bits are zero: at most 4 significant bits */
            }
        }
    }
}

/* ------------------------------------------------------------------ extend attention */

/* one output row: request r, extend row i, query head h -> out[D] */
static void attention_row(const void *q_ext, const void *k_ext, const void *v_ext, const void *pool_k,
                          const void *pool_v, const int32_t *slot_idx, const int32_t *slot_offsets,
                          const int32_t *prefix_len, const int32_t *ext_offsets, int Hq, int Hkv, int D,
                          int dtype, double scale, int r, int i, int h, double *out) {
    const int G = Hq / Hkv;
    const int g = h / G;
    const int P = prefix_len[r];
    const int nvis = P + i + 1;
    const int64_t e0 = ext_offsets[r];
    const int64_t qbase = ((e0 + i) * Hq + h) * (int64_t)D;
    double *s = (double *)malloc((size_t)nvis * sizeof(double));

    for (int j = 0; j < nvis; ++j) {
        const void *kb;
        int64_t kbase;
        if (j < P) { kb = pool_k; kbase = ((int64_t)slot_idx[slot_offsets[r] + j] * Hkv + g) * D; }
        else       { kb = k_ext;  kbase = ((e0 + (j - P)) * Hkv + g) * (int64_t)D; }
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += load_val(q_ext, qbase + d, dtype) * load_val(kb, kbase + d, dtype);
        s[j] = scale * dot;
    }
    double m = s[0];
    for (int j = 1; j < nvis; ++j) if (s[j] > m) m = s[j];
    double denom = 0.0;
    for (int j = 0; j < nvis; ++j) { s[j] = exp(s[j] - m); denom += s[j]; }
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    for (int j = 0; j < nvis; ++j) {
        const void *vb;
        int64_t vbase;
        if (j < P) { vb = pool_v; vbase = ((int64_t)slot_idx[slot_offsets[r] + j] * Hkv + g) * D; }
        else       { vb = v_ext;  vbase = ((e0 + (j - P)) * Hkv + g) * (int64_t)D; }
        for (int d = 0; d < D; ++d) out[d] += s[j] * load_val(vb, vbase + d, dtype);
    }
    for (int d = 0; d < D; ++d) out[d] /= denom;
    free(s);
}

/* Full output: out is double [T][Hq][D]. */
void ora_extend_attention(const void *q_ext, const void *k_ext, const void *v_ext, const void *pool_k,
                          const void *pool_v, const int32_t *slot_idx, const int32_t *slot_offsets,
                          const int32_t *prefix_len, const int32_t *ext_len, const int32_t *ext_offsets,
                          int B, int Hq, int Hkv, int D, int dtype, double scale, double *out) {
    for (int r = 0; r < B; ++r) {
        const int E = ext_len[r];
        const int64_t nrow = (int64_t)E * Hq;
#pragma omp parallel for schedule(dynamic, 4)
        for (int64_t x = 0; x < nrow; ++x) {
            int i = (int)(x / Hq), h = (int)(x % Hq);
            attention_row(q_ext, k_ext, v_ext, pool_k, pool_v, slot_idx, slot_offsets, prefix_len,
                          ext_offsets, Hq, Hkv, D, dtype, scale, r, i, h,
                          out + ((ext_offsets[r] + (int64_t)i) * Hq + h) * D);
        }
    }
}

/* Selected rows only: rows is int32 [n][3] = (r, i, h); out is double [n][D]. */
void ora_extend_attention_rows(const void *q_ext, const void *k_ext, const void *v_ext, const void *pool_k,
                               const void *pool_v, const int32_t *slot_idx, const int32_t *slot_offsets,
                               const int32_t *prefix_len, const int32_t *ext_offsets, int Hq, int Hkv, int D,
                               int dtype, double scale, const int32_t *rows, int64_t n, double *out) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t x = 0; x < n; ++x)
        attention_row(q_ext, k_ext, v_ext, pool_k, pool_v, slot_idx, slot_offsets, prefix_len, ext_offsets,
                      Hq, Hkv, D, dtype, scale, rows[3 * x], rows[3 * x + 1], rows[3 * x + 2], out + x * D);
}
