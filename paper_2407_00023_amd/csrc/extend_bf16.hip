// Extend attention on the bf16 matrix cores (MFMA 32x32x16, fp32 accumulate), gfx950.
//
// What is computed (Sec. 3.2 and Sec. 5 of the paper: only the missed tokens of a prompt
// are prefilled, the cached prefix KV is reused losslessly): extend row i of request r
// attends to the P_r prefix tokens, whose K/V rows are gathered from the paged pool
// through slot_idx, and causally to extend tokens 0..i.
//
// Decomposition.  The G = Hq/Hkv query heads of one KV head are packed with the extend
// rows into one row axis rho = i * G + (h mod G), so a K/V tile is read once per KV head.
// A workgroup (4 waves) owns kMT = 128 packed rows of one (request, KV head) and walks
// the key axis in tiles of kKT = 64 tokens: prefix positions first, then the extend
// tokens (the same loop; only the row address differs).  Optionally the key axis is cut
// into `nsplit` chunks handled by different workgroups, merged by a second kernel.
//
// MFMA formulation.  Scores are produced TRANSPOSED, S^T = K * Q^T, so that in the
// accumulator layout every lane holds one query row (column l % 32) and 16 of the 32
// tokens of a block: row statistics of the online softmax are per-lane scalars plus one
// exchange between lane l and l ^ 32, and the probabilities are already laid out as the
// B operand of the second product O^T = V^T * P^T.  V^T rows are formed from row-major V
// in LDS by reading 4 head-dim elements of 8 tokens and transposing 2-byte lanes in
// registers; head-dim element d = 4 * m + b belongs to row m of MFMA block b.
#include <hip/hip_bf16.h>

#include "common.h"

namespace pa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

constexpr int kMT = 128;  // packed query rows per workgroup (4 waves x 32)
constexpr int kKT = 64;   // key tokens per tile
constexpr int kThreads = 256;
constexpr int kTargetWorkgroups = 1024;  // split the key axis until about this many workgroups exist
constexpr int kMinChunk = 512;           // never split below this many keys per chunk

struct ExtendPlan {
    int tiles_cap;   // upper bound on the number of (request, row tile) pairs
    int nsplit;      // chunks of the key axis
    int chunk;       // keys per chunk (multiple of kKT)
    size_t off_req, off_row0, off_part_o, off_part_ml, total;
};

static inline size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

static ExtendPlan make_plan(int B, int64_t T, int64_t max_kv_len, int Hq, int Hkv, int D) {
    ExtendPlan p{};
    const int G = Hq / Hkv;
    const int64_t est = (T * G + kMT - 1) / kMT;
    p.tiles_cap = static_cast<int>(est + B);
    int64_t want = (kTargetWorkgroups + est * Hkv - 1) / (est * Hkv > 0 ? est * Hkv : 1);
    int64_t max_split = (max_kv_len + kMinChunk - 1) / kMinChunk;
    if (max_split < 1) max_split = 1;
    if (want > max_split) want = max_split;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    p.nsplit = static_cast<int>(want);
    int64_t chunk = (max_kv_len + p.nsplit - 1) / p.nsplit;
    chunk = (chunk + kKT - 1) / kKT * kKT;
    if (chunk < kKT) chunk = kKT;
    p.chunk = static_cast<int>(chunk);
    p.off_req = 256;
    p.off_row0 = p.off_req + up256(sizeof(int32_t) * p.tiles_cap);
    p.off_part_o = p.off_row0 + up256(sizeof(int32_t) * p.tiles_cap);
    const size_t units = p.nsplit > 1 ? static_cast<size_t>(p.tiles_cap) * p.nsplit * Hkv : 0;
    p.off_part_ml = p.off_part_o + up256(units * kMT * D * sizeof(float));
    p.total = p.off_part_ml + up256(units * kMT * 2 * sizeof(float));
    return p;
}

// ---------------------------------------------------------------------------------------
// Row-tile table: tile t -> (request, first packed row).  One workgroup; block-wide scan.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void extend_tiles_kernel(const int32_t* __restrict__ ext_len, int B, int G,
                                                          int tiles_cap, int32_t* __restrict__ n_tiles,
                                                          int32_t* __restrict__ tile_req,
                                                          int32_t* __restrict__ tile_row0) {
    __shared__ int s_scan[256];
    __shared__ int s_carry;
    const int tid = threadIdx.x;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int base = 0; base < B; base += 256) {
        const int r = base + tid;
        int cnt = 0;
        if (r < B) {
            const int e = ext_len[r];
            cnt = e > 0 ? (e * G + kMT - 1) / kMT : 0;
        }
        s_scan[tid] = cnt;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int v = tid >= off ? s_scan[tid - off] : 0;
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        const int start = s_carry + s_scan[tid] - cnt;
        for (int k = 0; k < cnt; ++k) {
            if (start + k < tiles_cap) {
                tile_req[start + k] = r;
                tile_row0[start + k] = k * kMT;
            }
        }
        __syncthreads();
        if (tid == 255) s_carry += s_scan[255];
        __syncthreads();
    }
    if (tid == 0) *n_tiles = min(s_carry, tiles_cap);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    // round to nearest even; inputs are finite probabilities or outputs
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    f32x2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

// Key range handled by split s of a tile whose visible keys are [0, kv_end).
__device__ __forceinline__ void split_range(int kv_end, int chunk, int nsplit, int s, int& n_act, int& lo, int& hi) {
    n_act = min(nsplit, (kv_end + chunk - 1) / chunk);
    lo = s * chunk;
    hi = (s == n_act - 1) ? kv_end : min(kv_end, (s + 1) * chunk);
}

// XOR swizzles of the 16-byte chunks of a K/V row in LDS, chosen so that the two read patterns below are
// free of bank conflicts for 256-byte rows: K is read 16 bytes per lane down 16 consecutive rows, V is
// read 8 bytes per lane across 64 bytes of 4 consecutive rows (the transposing LDS read).
template <int D>
__device__ __forceinline__ int swz_k(int row) {
    return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D>
__device__ __forceinline__ int swz_v(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes the 16 x 4 16-bit values
// addressed by the lanes form a flat array F (lane-major); lane i of the group receives F[i], F[16+i],
// F[32+i], F[48+i].
__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4*)(__attribute__((address_space(3))) unsigned char*)(p));
}

__device__ __forceinline__ float swap32(float x) {
    // value of the lane 32 away (the other half of the same query row)
    return __shfl_xor(x, 32);
}

constexpr float kRescaleThreshold = 8.f;  // log2 units: the running maximum may lag the true one by this much

template <int D>
__global__ __launch_bounds__(kThreads, 2) void extend_bf16_kernel(
    const __hip_bfloat16* __restrict__ q_ext, const __hip_bfloat16* __restrict__ k_ext,
    const __hip_bfloat16* __restrict__ v_ext, const __hip_bfloat16* __restrict__ pool,
    const int32_t* __restrict__ slot_idx, const int32_t* __restrict__ slot_offsets,
    const int32_t* __restrict__ prefix_len, const int32_t* __restrict__ ext_len,
    const int32_t* __restrict__ ext_offsets, int Hq, int Hkv, int page_size, int64_t num_slots, float scale_log2e,
    __hip_bfloat16* __restrict__ out, const int32_t* __restrict__ n_tiles, const int32_t* __restrict__ tile_req,
    const int32_t* __restrict__ tile_row0, int nsplit, int chunk, float* __restrict__ part_o,
    float* __restrict__ part_ml) {
    constexpr int NB = D / 32;               // MFMA row blocks of the head dimension in O^T
    constexpr int KS = D / 16;               // k-slices of the QK^T product
    constexpr int CPR = D / 8;               // 16-byte chunks per K/V row
    constexpr int ROWB = D * 2;              // bytes per row
    constexpr int TILEB = kKT * ROWB;        // bytes of one K (or V) tile
    constexpr int U = kKT * CPR / kThreads;  // 16-byte chunks each thread stages per tile and tensor
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2 buffers][K tile | V tile]

    // block -> (row tile, key split, kv head); the kv head varies fastest so that with 8 kv heads every
    // XCD (blocks are dealt round-robin to the 8 XCDs) serves one head and keeps its shared prefixes in L2
    const int g = blockIdx.x % Hkv;
    const int ts = blockIdx.x / Hkv;
    const int t = ts / nsplit;
    const int sp = ts - t * nsplit;
    if (t >= *n_tiles) return;
    const int r = tile_req[t];
    const int row0 = tile_row0[t];
    const int G = Hq / Hkv;
    const int P = prefix_len[r];
    const int E = ext_len[r];
    const int rows_total = E * G;
    const int rows_here = min(kMT, rows_total - row0);
    const int i_last = (row0 + rows_here - 1) / G;
    const int kv_end = P + i_last + 1;
    int n_act, kv_lo, kv_hi;
    split_range(kv_end, chunk, nsplit, sp, n_act, kv_lo, kv_hi);
    if (sp >= n_act) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int64_t e0 = ext_offsets[r];
    const int32_t* __restrict__ slots = slot_idx + slot_offsets[r];

    // this lane's query row
    const int rho = row0 + wave * 32 + n;
    const bool row_ok = rho < rows_total;
    const int qi = row_ok ? rho / G : 0;            // extend index of the row
    const int qh = g * G + (row_ok ? rho % G : 0);  // query head
    const bool wave_on = wave * 32 < rows_here;
    const int wave_i_first = (row0 + wave * 32) / G;
    const int wave_i_last = (row0 + min(rows_here, wave * 32 + 32) - 1) / G;
    const int wave_vis_min = min(kv_hi, P + wave_i_first + 1);  // every row of the wave sees keys [.., this)
    const int vis_end = min(kv_hi, P + qi + 1);                 // keys [.., vis_end) are visible to this row

    bf16x8 qreg[KS];
    {
        const uint4* qp = reinterpret_cast<const uint4*>(q_ext + ((e0 + qi) * Hq + qh) * static_cast<int64_t>(D));
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row_ok) v = qp[2 * s + hh];
            qreg[s] = __builtin_bit_cast(bf16x8, v);
        }
    }

    // ---- staging of one K/V tile: thread -> U (row, 16-byte column) pairs per tensor ----
    const int st_col = tid % CPR;
    const int st_row = tid / CPR;            // + u * (kThreads / CPR)
    constexpr int ST_ROWS = kThreads / CPR;  // rows covered per u
    uint4 st_k[U], st_v[U];
    int32_t sl_next[U];                      // pool slots of the tile after the staged one

    auto load_slots = [&](int p0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int p = p0 + st_row + u * ST_ROWS;
            sl_next[u] = (p < P && p < kv_hi) ? slots[p] : 0;
        }
    };
    auto issue_loads = [&](int p0) {  // consumes sl_next (slots of tile p0)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int p = p0 + st_row + u * ST_ROWS;
            uint4 kk = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
            if (p < kv_hi) {
                if (p < P) {
                    int64_t sl = sl_next[u];
                    sl = sl < 0 ? 0 : (sl >= num_slots ? num_slots - 1 : sl);
                    kk = reinterpret_cast<const uint4*>(pool + pool_row(sl, 0, g, Hkv, D, page_size))[st_col];
                    vv = reinterpret_cast<const uint4*>(pool + pool_row(sl, 1, g, Hkv, D, page_size))[st_col];
                } else {
                    const int64_t off = ((e0 + (p - P)) * Hkv + g) * static_cast<int64_t>(D);
                    kk = reinterpret_cast<const uint4*>(k_ext + off)[st_col];
                    vv = reinterpret_cast<const uint4*>(v_ext + off)[st_col];
                }
            }
            st_k[u] = kk;
            st_v[u] = vv;
        }
    };
    auto write_stage = [&](int buf) {
        unsigned char* sk = smem + buf * 2 * TILEB;
        unsigned char* sv = sk + TILEB;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = st_row + u * ST_ROWS;
            *reinterpret_cast<uint4*>(sk + row * ROWB + ((st_col ^ swz_k<D>(row)) * 16)) = st_k[u];
            *reinterpret_cast<uint4*>(sv + row * ROWB + ((st_col ^ swz_v<D>(row)) * 16)) = st_v[u];
        }
    };

    f32x16 oacc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[b][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;  // running maximum (scaled, log2 domain) and this lane's share of the sum

    // lane constants of the transposing V read: group lane i = 4 * e + c reads key row (4 * hh + e) + ..., and
    // 8 bytes at head-dim offset 32 * b + 16 * par + 4 * c
    const int tr_e = (lane >> 2) & 3, tr_c = lane & 3, tr_par = (lane >> 4) & 1;
    const bf16x2_t ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};

    // ---- prologue: first tile into buffer 0 ----
    load_slots(kv_lo);
    issue_loads(kv_lo);
    load_slots(kv_lo + kKT);
    write_stage(0);
    __syncthreads();

    int buf = 0;
    for (int p0 = kv_lo; p0 < kv_hi; p0 += kKT, buf ^= 1) {
        const bool more = p0 + kKT < kv_hi;
        if (more) {
            issue_loads(p0 + kKT);       // global loads of the next tile fly during this tile's arithmetic
            load_slots(p0 + 2 * kKT);
        }
        if (wave_on && p0 <= P + wave_i_last) {
            const unsigned char* sk = smem + buf * 2 * TILEB;
            const unsigned char* sv = sk + TILEB;
            // ---- S^T = K Q^T for two blocks of 32 keys ----
            f32x16 sacc[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[mb][i] = 0.f;
                const int krow = mb * 32 + n;
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const int pos = (2 * s + hh) ^ swz_k<D>(krow);
                    const uint4 kv = *reinterpret_cast<const uint4*>(sk + krow * ROWB + pos * 16);
                    sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kv), qreg[s], sacc[mb], 0, 0, 0);
                }
            }

            // ---- mask (only where the tile crosses a visibility limit), row maximum ----
            if (p0 + kKT > wave_vis_min) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int p = p0 + mb * 32 + 8 * (i / 4) + 4 * hh + (i % 4);
                        if (p >= vis_end) sacc[mb][i] = -INFINITY;
                    }
            }
            float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, fmaxf(sacc[0][i], sacc[1][i]));
            mx = fmaxf(mx, swap32(mx));
            const float m_tile = mx * scale_log2e;
            // The running maximum is only raised when some row of the wave outgrows it by the threshold;
            // until then probabilities are formed against the older, smaller maximum (they stay <= 2^threshold).
            if (__any(m_tile > m_run + kRescaleThreshold)) {
                const float m_new = fmaxf(m_run, m_tile);
                const float alpha = __builtin_amdgcn_exp2f(m_run - ((m_new == -INFINITY) ? 0.f : m_new));
                l_run *= alpha;
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
                m_run = m_new;
            }
            const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
            uint32_t pb[2][8];  // probabilities as packed bf16 pairs: the B operand of the second product
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float a = __builtin_amdgcn_exp2f(fmaf(sacc[mb][i], scale_log2e, neg_m));
                    const float b = __builtin_amdgcn_exp2f(fmaf(sacc[mb][i + 1], scale_log2e, neg_m));
                    const uint32_t pk = pack_bf16x2(a, b);
                    pb[mb][i / 2] = pk;
                    // the denominator sums the rounded probabilities, the same values the numerator uses
                    l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pk), ones, l_run, false);
                }

            // ---- O^T += V^T P^T, 16 keys per MFMA; V^T fragments come from the transposing LDS read ----
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int cs = 0; cs < 2; ++cs) {
                    const uint4 pv4 = make_uint4(pb[mb][cs * 4 + 0], pb[mb][cs * 4 + 1], pb[mb][cs * 4 + 2], pb[mb][cs * 4 + 3]);
                    const bf16x8 pop = __builtin_bit_cast(bf16x8, pv4);
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        s16x4 frag[2];
#pragma unroll
                        for (int h2 = 0; h2 < 2; ++h2) {
                            const int vrow = mb * 32 + cs * 16 + 8 * h2 + 4 * hh + tr_e;
                            const int chunk = 4 * b + 2 * tr_par + (tr_c >> 1);
                            frag[h2] = lds_read_tr16(sv + vrow * ROWB + ((chunk ^ swz_v<D>(vrow)) * 16) + (tr_c & 1) * 8);
                        }
                        typedef short s16x8 __attribute__((ext_vector_type(8)));
                        const s16x8 a8 = __builtin_shufflevector(frag[0], frag[1], 0, 1, 2, 3, 4, 5, 6, 7);
                        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a8), pop, oacc[b], 0, 0, 0);
                    }
                }
        }
        if (more) write_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds, for block b and register i, head-dim element 32 b + 8 (i / 4) + 4 hh + i % 4 ----
    l_run += swap32(l_run);
    if (!row_ok) return;
    if (n_act == 1) {
        const float inv = 1.f / l_run;
        __hip_bfloat16* orow = out + ((e0 + qi) * Hq + qh) * static_cast<int64_t>(D);
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                uint2 v;
                v.x = pack_bf16x2(oacc[b][4 * q4 + 0] * inv, oacc[b][4 * q4 + 1] * inv);
                v.y = pack_bf16x2(oacc[b][4 * q4 + 2] * inv, oacc[b][4 * q4 + 3] * inv);
                *reinterpret_cast<uint2*>(orow + 32 * b + 8 * q4 + 4 * hh) = v;
            }
    } else {
        const size_t unit = (static_cast<size_t>(t) * nsplit + sp) * Hkv + g;
        const int lrow = wave * 32 + n;
        float* prow = part_o + (unit * kMT + lrow) * D;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<float4*>(prow + 32 * b + 8 * q4 + 4 * hh) =
                    make_float4(oacc[b][4 * q4 + 0], oacc[b][4 * q4 + 1], oacc[b][4 * q4 + 2], oacc[b][4 * q4 + 3]);
        if (hh == 0) {
            part_ml[(unit * kMT + lrow) * 2 + 0] = m_run;
            part_ml[(unit * kMT + lrow) * 2 + 1] = l_run;
        }
    }
}

// Merge of the key-axis splits: out = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s.
template <int D>
__global__ __launch_bounds__(256) void extend_merge_kernel(const int32_t* __restrict__ prefix_len,
                                                          const int32_t* __restrict__ ext_len,
                                                          const int32_t* __restrict__ ext_offsets, int Hq, int Hkv,
                                                          __hip_bfloat16* __restrict__ out,
                                                          const int32_t* __restrict__ n_tiles,
                                                          const int32_t* __restrict__ tile_req,
                                                          const int32_t* __restrict__ tile_row0, int nsplit, int chunk,
                                                          const float* __restrict__ part_o,
                                                          const float* __restrict__ part_ml) {
    const int t = blockIdx.x, g = blockIdx.y;
    if (t >= *n_tiles) return;
    const int r = tile_req[t], row0 = tile_row0[t];
    const int G = Hq / Hkv;
    const int P = prefix_len[r], E = ext_len[r];
    const int rows_here = min(kMT, E * G - row0);
    const int kv_end = P + (row0 + rows_here - 1) / G + 1;
    int n_act, lo, hi;
    split_range(kv_end, chunk, nsplit, 0, n_act, lo, hi);
    if (n_act <= 1) return;
    const int64_t e0 = ext_offsets[r];
    constexpr int V4 = D / 4;
    for (int x = threadIdx.x; x < rows_here * V4; x += 256) {
        const int lrow = x / V4, c = x % V4;
        float m = -INFINITY;
        for (int s = 0; s < n_act; ++s) {
            const size_t unit = (static_cast<size_t>(t) * nsplit + s) * Hkv + g;
            m = fmaxf(m, part_ml[(unit * kMT + lrow) * 2]);
        }
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float l = 0.f;
        for (int s = 0; s < n_act; ++s) {
            const size_t unit = (static_cast<size_t>(t) * nsplit + s) * Hkv + g;
            const float ms = part_ml[(unit * kMT + lrow) * 2];
            const float w = (ms == -INFINITY) ? 0.f : exp2f(ms - m);
            l += w * part_ml[(unit * kMT + lrow) * 2 + 1];
            const float4 o = reinterpret_cast<const float4*>(part_o + (unit * kMT + lrow) * D)[c];
            acc.x += w * o.x; acc.y += w * o.y; acc.z += w * o.z; acc.w += w * o.w;
        }
        const float inv = 1.f / l;
        const int rho = row0 + lrow;
        __hip_bfloat16* orow = out + ((e0 + rho / G) * Hq + g * G + rho % G) * static_cast<int64_t>(D);
        uint2 v;
        v.x = pack_bf16x2(acc.x * inv, acc.y * inv);
        v.y = pack_bf16x2(acc.z * inv, acc.w * inv);
        reinterpret_cast<uint2*>(orow)[c] = v;
    }
}

}  // namespace pa

size_t pa_extend_workspace_bytes_bf16(int B, int64_t T, int64_t max_kv_len, int Hq, int Hkv, int D) {
    return pa::make_plan(B, T, max_kv_len, Hq, Hkv, D).total;
}

// Called by pa_extend_attention after argument validation.
int pa_extend_attention_bf16(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                             const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                             const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T, int64_t max_kv_len,
                             int Hq, int Hkv, int D, int page_size, int64_t num_slots, float scale, void* out,
                             void* workspace, size_t workspace_bytes, hipStream_t stream) {
    using namespace pa;
    const ExtendPlan p = make_plan(B, T, max_kv_len, Hq, Hkv, D);
    if (workspace_bytes < p.total || workspace == nullptr)
        return fail(PA_ENOMEM, "pa_extend_attention: workspace of %zu bytes given, %zu needed", workspace_bytes, p.total);
    PA_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, "pa_extend_attention: workspace must be 256-byte aligned");
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int32_t* n_tiles = reinterpret_cast<int32_t*>(ws);
    int32_t* tile_req = reinterpret_cast<int32_t*>(ws + p.off_req);
    int32_t* tile_row0 = reinterpret_cast<int32_t*>(ws + p.off_row0);
    float* part_o = reinterpret_cast<float*>(ws + p.off_part_o);
    float* part_ml = reinterpret_cast<float*>(ws + p.off_part_ml);
    const int G = Hq / Hkv;
    const float scale_log2e = scale * 1.4426950408889634f;

    {
        ProfScope prof(kProfTiles, stream);
        hipLaunchKernelGGL(extend_tiles_kernel, dim3(1), dim3(256), 0, stream, ext_len, B, G, p.tiles_cap, n_tiles,
                           tile_req, tile_row0);
    }
    const dim3 grid(static_cast<unsigned>(p.tiles_cap) * p.nsplit * Hkv);
    const size_t lds_bytes = 2u * 2u * kKT * D * 2u;  // two buffers of one K tile and one V tile
    const dim3 mgrid(p.tiles_cap, Hkv);
#define PA_LAUNCH_BF16(DD)                                                                                           \
    do {                                                                                                             \
        {                                                                                                            \
        ProfScope prof(kProfExtend, stream);                                                                         \
        hipLaunchKernelGGL(extend_bf16_kernel<DD>, grid, dim3(kThreads), lds_bytes, stream,                                 \
                           static_cast<const __hip_bfloat16*>(q_ext), static_cast<const __hip_bfloat16*>(k_ext),     \
                           static_cast<const __hip_bfloat16*>(v_ext), static_cast<const __hip_bfloat16*>(kv_pool),   \
                           slot_idx, slot_offsets, prefix_len, ext_len, ext_offsets, Hq, Hkv, page_size, num_slots,  \
                           scale_log2e, static_cast<__hip_bfloat16*>(out), n_tiles, tile_req, tile_row0, p.nsplit,   \
                           p.chunk, part_o, part_ml);                                                                \
        }                                                                                                            \
        if (p.nsplit > 1) {                                                                                          \
            ProfScope prof(kProfMerge, stream);                                                                      \
            hipLaunchKernelGGL(extend_merge_kernel<DD>, mgrid, dim3(256), 0, stream, prefix_len, ext_len,            \
                               ext_offsets, Hq, Hkv, static_cast<__hip_bfloat16*>(out), n_tiles, tile_req,           \
                               tile_row0, p.nsplit, p.chunk, part_o, part_ml);                                       \
        }                                                                                                            \
    } while (0)
    if (D == 64) PA_LAUNCH_BF16(64);
    else PA_LAUNCH_BF16(128);
#undef PA_LAUNCH_BF16
    PA_HIP(hipGetLastError());
    return PA_OK;
}
