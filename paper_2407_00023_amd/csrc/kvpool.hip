// KV pool: size, scatter of new rows (append_kv) and its inverse (gather_kv).
//
// Sec. 3.2 of the paper: once computed on a GPU, a prefix stays cached there until it is
// evicted; this is the write that puts the KV of newly computed tokens into the cache.
// Pure data movement: one 16-byte vector per thread, rows of D elements per (token, head).  With the fp8 pool
// (PA_BF16_KV8) the rows are bfloat16 on the caller's side and one-byte codes plus a row exponent in the pool.
#include "common.h"
#include "fp8_rows.h"

namespace pa {

// vectors of 16 bytes; row = D * elt bytes = vec_per_row vectors
template <bool kToPool>
__global__ __launch_bounds__(256) void kv_rows_kernel(uint4* __restrict__ pool, const int32_t* __restrict__ slots,
                                                      uint4* __restrict__ k_dense, uint4* __restrict__ v_dense,
                                                      int64_t n_tok, int Hkv, int vec_per_row, int page_size,
                                                      int64_t num_slots) {
    // one item = one 16-byte vector of one (token, K|V, head) row
    const int64_t per_tok = 2ll * Hkv * vec_per_row;
    const int64_t total = n_tok * per_tok;
    for (int64_t x = blockIdx.x * 256ll + threadIdx.x; x < total; x += gridDim.x * 256ll) {
        const int64_t t = x / per_tok;
        int rem = static_cast<int>(x - t * per_tok);
        const int which = rem / (Hkv * vec_per_row);
        rem -= which * Hkv * vec_per_row;
        const int g = rem / vec_per_row;
        const int c = rem - g * vec_per_row;
        const int64_t slot = slots[t];
        if (slot < 0 || slot >= num_slots) continue;  // never touch memory outside the pool
        // pool_row with D replaced by vec_per_row gives the index in 16-byte units
        const int64_t pidx = pool_row(slot, which, g, Hkv, vec_per_row, page_size) + c;
        uint4* dense = which ? v_dense : k_dense;
        const int64_t didx = (t * Hkv + g) * vec_per_row + c;
        if (kToPool) pool[pidx] = dense[didx];
        else dense[didx] = pool[pidx];
    }
}

// fp8 pool: D / 8 lanes share one row of D bfloat16; a lane holds 8 elements of it (16 bytes dense, 8 bytes of codes).
// Encoding needs the largest magnitude of the whole row first: a maximum over the row's lanes, which sit side by side
// in one wave.  `exps` = the int8 row exponents behind the codes.
template <int D, bool kToPool>
__global__ __launch_bounds__(256) void kv8_rows_kernel(uint2* __restrict__ pool, signed char* __restrict__ exps,
                                                       const int32_t* __restrict__ slots, uint4* __restrict__ k_dense,
                                                       uint4* __restrict__ v_dense, int64_t n_tok, int Hkv, int page_size,
                                                       int64_t num_slots) {
    constexpr int LPR = D / 8;  // lanes per row
    const int64_t per_tok = 2ll * Hkv * LPR;
    const int64_t total = n_tok * per_tok;
    for (int64_t x = blockIdx.x * 256ll + threadIdx.x; x < total; x += gridDim.x * 256ll) {
        const int64_t t = x / per_tok;
        int rem = static_cast<int>(x - t * per_tok);
        const int which = rem / (Hkv * LPR);
        rem -= which * Hkv * LPR;
        const int g = rem / LPR;
        const int c = rem - g * LPR;
        const int64_t slot = slots[t];
        const bool ok = slot >= 0 && slot < num_slots;  // never touch memory outside the pool (the whole row agrees)
        const int64_t row = pool_row(ok ? slot : 0, which, g, Hkv, 1, page_size);  // row number = index of its exponent
        uint4* dense = which ? v_dense : k_dense;
        const int64_t didx = (t * Hkv + g) * LPR + c;
        if (kToPool) {
            const uint4 in = dense[didx];
            const unsigned w[4] = {in.x, in.y, in.z, in.w};
            unsigned amax = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) amax = max(amax, max(w[i] & 0x7FFFu, (w[i] >> 16) & 0x7FFFu));
            // (the lanes of a row are LPR consecutive lanes, all of them in the loop together: total is a multiple of LPR)
#pragma unroll
            for (int off = 1; off < LPR; off <<= 1) amax = max(amax, static_cast<unsigned>(__shfl_xor(static_cast<int>(amax), off)));
            const int k = fp8_row_exponent(amax);
            unsigned o[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                o[i] = fp8_encode(w[2 * i] & 0xFFFFu, k) | (fp8_encode(w[2 * i] >> 16, k) << 8) |
                       (fp8_encode(w[2 * i + 1] & 0xFFFFu, k) << 16) | (fp8_encode(w[2 * i + 1] >> 16, k) << 24);
            if (ok) {
                pool[row * LPR + c] = make_uint2(o[0], o[1]);
                if (c == 0) exps[row] = static_cast<signed char>(k);
            }
        } else if (ok) {
            const uint2 in = pool[row * LPR + c];
            const float scale = fp8_scale(exps[row]);
            const uint2 a = fp8_decode4(in.x, scale), b = fp8_decode4(in.y, scale);
            dense[didx] = make_uint4(a.x, a.y, b.x, b.y);
        }
    }
}

static int check_pool_args(const char* fn, const void* pool, const void* slots, const void* k, const void* v, int64_t n,
                           int Hkv, int D, int page_size, int64_t num_slots, int dtype) {
    PA_REQUIRE(n >= 0, "%s: negative token count", fn);
    PA_REQUIRE(dtype == PA_F32 || dtype == PA_BF16 || dtype == PA_BF16_KV8, "%s: unknown dtype %d", fn, dtype);
    PA_REQUIRE(Hkv > 0 && (D == 64 || D == 128), "%s: unsupported shape Hkv=%d D=%d", fn, Hkv, D);
    PA_REQUIRE(page_size >= 1 && num_slots > 0 && num_slots % page_size == 0,
               "%s: page_size %d must divide num_slots %lld", fn, page_size, static_cast<long long>(num_slots));
    if (n == 0) return PA_OK;
    PA_REQUIRE(pool && slots && k && v, "%s: NULL pointer", fn);
    PA_REQUIRE(aligned16(pool) && aligned16(k) && aligned16(v), "%s: buffers must be 16-byte aligned", fn);
    return PA_OK;
}

static int grid_for(int64_t items) {
    int64_t blocks = (items + 255) / 256;
    const int64_t cap = 256 * 32;  // 32 workgroups per CU is plenty for a streaming copy
    return static_cast<int>(blocks < cap ? (blocks > 0 ? blocks : 1) : cap);
}

}  // namespace pa

extern "C" size_t pa_kv_pool_bytes(int64_t num_slots, int Hkv, int D, int dtype, int page_size) {
    if (num_slots <= 0 || Hkv <= 0 || D <= 0 || page_size <= 0 || num_slots % page_size != 0) return 0;
    if (dtype == PA_BF16_KV8) return static_cast<size_t>(num_slots) * 2u * Hkv * (static_cast<size_t>(D) + 1u);  // codes, then one exponent per row
    if (dtype != PA_F32 && dtype != PA_BF16) return 0;
    return static_cast<size_t>(num_slots) * 2u * Hkv * D * pa::elt_size(dtype);
}

// The fp8 pool as the kernels see it: codes, and the row exponents behind them.
template <int D, bool kToPool>
static void launch_kv8(void* pool, const int32_t* slots, void* k, void* v, int64_t n, int Hkv, int page_size,
                       int64_t num_slots, hipStream_t stream) {
    signed char* exps = static_cast<signed char*>(pool) + static_cast<size_t>(num_slots) * 2u * Hkv * D;
    hipLaunchKernelGGL((pa::kv8_rows_kernel<D, kToPool>), dim3(pa::grid_for(n * 2 * Hkv * (D / 8))), dim3(256), 0, stream,
                       static_cast<uint2*>(pool), exps, slots, static_cast<uint4*>(k), static_cast<uint4*>(v), n, Hkv,
                       page_size, num_slots);
}

extern "C" int pa_append_kv(void* kv_pool, const int32_t* new_slots, const void* k_ext, const void* v_ext, int64_t T,
                            int Hkv, int D, int page_size, int64_t num_slots, int dtype, void* stream) {
    int rc = pa::check_pool_args("pa_append_kv", kv_pool, new_slots, k_ext, v_ext, T, Hkv, D, page_size, num_slots, dtype);
    if (rc != PA_OK || T == 0) return rc;
    const int vpr = static_cast<int>(D * pa::elt_size(dtype) / 16);
    pa::ProfScope prof(pa::kProfAppend, static_cast<hipStream_t>(stream));
    if (dtype == PA_BF16_KV8) {
        if (D == 64) launch_kv8<64, true>(kv_pool, new_slots, const_cast<void*>(k_ext), const_cast<void*>(v_ext), T, Hkv, page_size, num_slots, static_cast<hipStream_t>(stream));
        else launch_kv8<128, true>(kv_pool, new_slots, const_cast<void*>(k_ext), const_cast<void*>(v_ext), T, Hkv, page_size, num_slots, static_cast<hipStream_t>(stream));
        PA_HIP(hipGetLastError());
        return PA_OK;
    }
    hipLaunchKernelGGL(pa::kv_rows_kernel<true>, dim3(pa::grid_for(T * 2 * Hkv * vpr)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<uint4*>(kv_pool), new_slots,
                       static_cast<uint4*>(const_cast<void*>(k_ext)), static_cast<uint4*>(const_cast<void*>(v_ext)), T,
                       Hkv, vpr, page_size, num_slots);
    PA_HIP(hipGetLastError());
    return PA_OK;
}

extern "C" int pa_gather_kv(const void* kv_pool, const int32_t* slots, int64_t n, int Hkv, int D, int page_size,
                            int64_t num_slots, int dtype, void* k_out, void* v_out, void* stream) {
    int rc = pa::check_pool_args("pa_gather_kv", kv_pool, slots, k_out, v_out, n, Hkv, D, page_size, num_slots, dtype);
    if (rc != PA_OK || n == 0) return rc;
    const int vpr = static_cast<int>(D * pa::elt_size(dtype) / 16);
    pa::ProfScope prof(pa::kProfGather, static_cast<hipStream_t>(stream));
    if (dtype == PA_BF16_KV8) {
        if (D == 64) launch_kv8<64, false>(const_cast<void*>(kv_pool), slots, k_out, v_out, n, Hkv, page_size, num_slots, static_cast<hipStream_t>(stream));
        else launch_kv8<128, false>(const_cast<void*>(kv_pool), slots, k_out, v_out, n, Hkv, page_size, num_slots, static_cast<hipStream_t>(stream));
        PA_HIP(hipGetLastError());
        return PA_OK;
    }
    hipLaunchKernelGGL(pa::kv_rows_kernel<false>, dim3(pa::grid_for(n * 2 * Hkv * vpr)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<uint4*>(const_cast<void*>(kv_pool)), slots,
                       static_cast<uint4*>(k_out), static_cast<uint4*>(v_out), n, Hkv, vpr, page_size, num_slots);
    PA_HIP(hipGetLastError());
    return PA_OK;
}
