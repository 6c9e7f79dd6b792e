// pa_extend_attention: argument validation and dispatch on dtype.
#include "common.h"

int pa_extend_attention_f32(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                            const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                            const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T, int Hq, int Hkv, int D,
                            int page_size, int64_t num_slots, float scale, void* out, hipStream_t stream);
int pa_extend_attention_bf16(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                             const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                             const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T, int64_t max_kv_len,
                             int Hq, int Hkv, int D, int page_size, int64_t num_slots, bool kv8, float scale, void* out,
                             void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t pa_extend_workspace_bytes_bf16(int B, int64_t T, int64_t max_kv_len, int Hq, int Hkv, int D);

extern "C" size_t pa_extend_workspace_bytes(int B, int64_t T, int64_t max_kv_len, int Hq, int Hkv, int D, int dtype) {
    if (B < 0 || T < 0 || max_kv_len < 0 || !pa::shape_ok(Hq, Hkv, D)) return 0;
    if (T > INT32_MAX / (Hq / Hkv) - 256 || max_kv_len > INT32_MAX / 2) return 0;
    if (dtype == PA_F32) return 256;  // the fp32 kernel needs no scratch; a non-zero size keeps "0 = invalid"
    if (dtype == PA_BF16 || dtype == PA_BF16_KV8) return pa_extend_workspace_bytes_bf16(B, T, max_kv_len, Hq, Hkv, D);
    return 0;
}

int pa_extend_attention_bf16_static(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                                    const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                                    const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T,
                                    int64_t max_kv_len, int Hq, int Hkv, int D, int page_size, int64_t num_slots,
                                    bool kv8, float scale, void* out, hipStream_t stream);

// What both entry points ask of their arguments.  *nothing_to_do: an empty batch (no pointer is looked at then).
static int check_extend_args(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                             const int32_t* slot_offsets, const int32_t* prefix_len, const int32_t* ext_len,
                             const int32_t* ext_offsets, int B, int64_t T, int64_t max_kv_len, int Hq, int Hkv, int D,
                             int page_size, int64_t num_slots, int dtype, const void* out, bool* nothing_to_do) {
    *nothing_to_do = false;
    PA_REQUIRE(dtype == PA_F32 || dtype == PA_BF16 || dtype == PA_BF16_KV8, "pa_extend_attention: unknown dtype %d", dtype);
    PA_REQUIRE(pa::shape_ok(Hq, Hkv, D), "pa_extend_attention: unsupported shape Hq=%d Hkv=%d D=%d", Hq, Hkv, D);
    PA_REQUIRE(B >= 0 && T >= 0 && max_kv_len >= 0, "pa_extend_attention: negative size");
    PA_REQUIRE(T <= INT32_MAX / (Hq / Hkv) - 256 && max_kv_len <= INT32_MAX / 2, "pa_extend_attention: batch too large for 32-bit row indices");
    PA_REQUIRE(page_size >= 1 && num_slots > 0 && num_slots % page_size == 0,
               "pa_extend_attention: page_size %d must divide num_slots %lld", page_size, static_cast<long long>(num_slots));
    if (B == 0 || T == 0) {
        *nothing_to_do = true;
        return PA_OK;
    }
    PA_REQUIRE(q_ext && k_ext && v_ext && kv_pool && slot_offsets && prefix_len && ext_len && ext_offsets && out,
               "pa_extend_attention: NULL pointer");
    PA_REQUIRE(pa::aligned16(q_ext) && pa::aligned16(k_ext) && pa::aligned16(v_ext) && pa::aligned16(kv_pool) &&
                   pa::aligned16(out), "pa_extend_attention: tensors must be 16-byte aligned");
    PA_REQUIRE(out != q_ext && out != k_ext && out != v_ext, "pa_extend_attention: out aliases an input");
    return PA_OK;
}

extern "C" int pa_extend_attention(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                                   const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                                   const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T,
                                   int64_t max_kv_len, int Hq, int Hkv, int D, int page_size, int64_t num_slots,
                                   int dtype, float scale, void* out, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    bool nothing = false;
    if (const int rc = check_extend_args(q_ext, k_ext, v_ext, kv_pool, slot_offsets, prefix_len, ext_len, ext_offsets, B, T,
                                         max_kv_len, Hq, Hkv, D, page_size, num_slots, dtype, out, &nothing))
        return rc;
    if (nothing) return PA_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == PA_F32)
        return pa_extend_attention_f32(q_ext, k_ext, v_ext, kv_pool, slot_idx, slot_offsets, prefix_len, ext_len,
                                       ext_offsets, B, T, Hq, Hkv, D, page_size, num_slots, scale, out, s);
    return pa_extend_attention_bf16(q_ext, k_ext, v_ext, kv_pool, slot_idx, slot_offsets, prefix_len, ext_len,
                                    ext_offsets, B, T, max_kv_len, Hq, Hkv, D, page_size, num_slots, dtype == PA_BF16_KV8, scale,
                                    out, workspace, workspace_bytes, s);
}

extern "C" int pa_extend_attention_static(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                                          const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                                          const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T,
                                          int64_t max_kv_len, int Hq, int Hkv, int D, int page_size, int64_t num_slots,
                                          int dtype, float scale, void* out, void* stream) {
    bool nothing = false;
    if (const int rc = check_extend_args(q_ext, k_ext, v_ext, kv_pool, slot_offsets, prefix_len, ext_len, ext_offsets, B, T,
                                         max_kv_len, Hq, Hkv, D, page_size, num_slots, dtype, out, &nothing))
        return rc;
    if (nothing) return PA_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == PA_F32)  // (the fp32 kernel uses no workspace at all)
        return pa_extend_attention_f32(q_ext, k_ext, v_ext, kv_pool, slot_idx, slot_offsets, prefix_len, ext_len,
                                       ext_offsets, B, T, Hq, Hkv, D, page_size, num_slots, scale, out, s);
    return pa_extend_attention_bf16_static(q_ext, k_ext, v_ext, kv_pool, slot_idx, slot_offsets, prefix_len, ext_len,
                                           ext_offsets, B, T, max_kv_len, Hq, Hkv, D, page_size, num_slots,
                                           dtype == PA_BF16_KV8, scale, out, s);
}
