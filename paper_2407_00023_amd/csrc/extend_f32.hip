// Extend attention, fp32 arithmetic throughout (the tiny correctness configuration).
//
// The computation is the one the paper prices as "prefill of the missed tokens" with the
// cached prefix reused losslessly (Sec. 3.2, Sec. 5): extend row i of request r sees the
// P_r cached prefix tokens (rows of the pool named by slot_idx) and extend tokens 0..i.
//
// One wavefront computes one output row (one extend token, one query head).  Keys are
// taken 64 at a time: lane j forms the score of key j, the wave reduces max and sum for
// the online softmax, then lane d accumulates output element d over the 64 keys.
#include "common.h"

namespace pa {

template <int D>
__global__ __launch_bounds__(256) void extend_f32_kernel(
    const float* __restrict__ q_ext, const float* __restrict__ k_ext, const float* __restrict__ v_ext,
    const float* __restrict__ pool, const int32_t* __restrict__ slot_idx, const int32_t* __restrict__ slot_offsets,
    const int32_t* __restrict__ prefix_len, const int32_t* __restrict__ ext_len,
    const int32_t* __restrict__ ext_offsets, int B, int64_t T, int Hq, int Hkv, int page_size, int64_t num_slots,
    float scale, float* __restrict__ out) {
    constexpr int DPL = D / 64;  // output elements per lane
    const int lane = threadIdx.x & 63;
    const int64_t row = blockIdx.x * 4ll + (threadIdx.x >> 6);  // (extend token, head)
    if (row >= T * Hq) return;
    const int64_t t = row / Hq;
    const int h = static_cast<int>(row - t * Hq);
    const int g = h / (Hq / Hkv);

    // request of extend token t: last r with ext_offsets[r] <= t
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (ext_offsets[mid] <= t) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int i = static_cast<int>(t - ext_offsets[r]);
    if (i >= ext_len[r]) return;  // inconsistent offsets: produce nothing rather than read out of range
    const int P = prefix_len[r];
    const int nvis = P + i + 1;
    const int32_t* __restrict__ slots = slot_idx + slot_offsets[r];
    const int64_t e0 = ext_offsets[r];

    float qreg[DPL];
#pragma unroll
    for (int x = 0; x < DPL; ++x) qreg[x] = q_ext[(t * Hq + h) * D + x * 64 + lane] * scale;

    float m = -INFINITY, l = 0.f;
    float acc[DPL];
#pragma unroll
    for (int x = 0; x < DPL; ++x) acc[x] = 0.f;

    for (int j0 = 0; j0 < nvis; j0 += 64) {
        const int j = j0 + lane;
        const bool vis = j < nvis;
        // element offsets of this lane's key row and value row; lanes past the end read a valid
        // dummy row (extend token 0 of the request) so that the whole wave stays convergent
        const float* kp = k_ext;
        int64_t koff = (e0 * Hkv + g) * static_cast<int64_t>(D), voff = koff;
        if (vis) {
            if (j < P) {
                int64_t sl = slots[j];
                sl = sl < 0 ? 0 : (sl >= num_slots ? num_slots - 1 : sl);
                kp = pool;
                koff = pool_row(sl, 0, g, Hkv, D, page_size);
                voff = pool_row(sl, 1, g, Hkv, D, page_size);
            } else {
                koff = voff = ((e0 + (j - P)) * Hkv + g) * static_cast<int64_t>(D);
            }
        }
        float s = 0.f;
        {
            const float4* k4 = reinterpret_cast<const float4*>(kp + koff);
#pragma unroll
            for (int c = 0; c < D / 4; ++c) {
                const float4 kk = k4[c];
                const int d = 4 * c;
                s += __shfl(qreg[d / 64], d % 64) * kk.x;
                s += __shfl(qreg[(d + 1) / 64], (d + 1) % 64) * kk.y;
                s += __shfl(qreg[(d + 2) / 64], (d + 2) % 64) * kk.z;
                s += __shfl(qreg[(d + 3) / 64], (d + 3) % 64) * kk.w;
            }
        }
        if (!vis) s = -INFINITY;
        float cm = s;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off));
        const float m_new = fmaxf(m, cm);
        const float alpha = expf(m - m_new);  // first chunk: exp(-inf) = 0
        const float p = vis ? expf(s - m_new) : 0.f;
        float ps = p;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off);
        l = l * alpha + ps;
        m = m_new;
#pragma unroll
        for (int x = 0; x < DPL; ++x) acc[x] *= alpha;
        const int cnt = min(64, nvis - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj);
            const bool in_pool = (j0 + jj) < P;
            const long long vo = __shfl(static_cast<long long>(voff), jj);
            const float* vrow = (in_pool ? pool : v_ext) + vo;
#pragma unroll
            for (int x = 0; x < DPL; ++x) acc[x] += pj * vrow[x * 64 + lane];
        }
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int x = 0; x < DPL; ++x) out[(t * Hq + h) * D + x * 64 + lane] = acc[x] * inv;
}

}  // namespace pa

// Called by pa_extend_attention after argument validation.
int pa_extend_attention_f32(const void* q_ext, const void* k_ext, const void* v_ext, const void* kv_pool,
                            const int32_t* slot_idx, const int32_t* slot_offsets, const int32_t* prefix_len,
                            const int32_t* ext_len, const int32_t* ext_offsets, int B, int64_t T, int Hq, int Hkv, int D,
                            int page_size, int64_t num_slots, float scale, void* out, hipStream_t stream) {
    const int64_t rows = T * Hq;
    const dim3 grid(static_cast<unsigned>((rows + 3) / 4)), block(256);
#define PA_LAUNCH_F32(DD)                                                                                        \
    hipLaunchKernelGGL(pa::extend_f32_kernel<DD>, grid, block, 0, stream, static_cast<const float*>(q_ext),      \
                       static_cast<const float*>(k_ext), static_cast<const float*>(v_ext),                       \
                       static_cast<const float*>(kv_pool), slot_idx, slot_offsets, prefix_len, ext_len,          \
                       ext_offsets, B, T, Hq, Hkv, page_size, num_slots, scale, static_cast<float*>(out))
    {
        pa::ProfScope prof(pa::kProfExtendF32, stream);
        if (D == 64) PA_LAUNCH_F32(64);
        else PA_LAUNCH_F32(128);
    }
#undef PA_LAUNCH_F32
    PA_HIP(hipGetLastError());
    return PA_OK;
}
