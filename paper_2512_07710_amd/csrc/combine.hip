// Weighted combine of the expert outputs back to token order.
//
// One block per token gathers the k expert-ordered fp32 rows named by inv_perm,
// accumulates w[t,j]*row in slot order with fp32 fused multiply-adds and rounds to
// bf16 once.  A gather per output token needs no atomics and is deterministic.
#include "moe_internal.hpp"

namespace moe355 {
namespace {

__device__ inline uint32_t f32_to_bf16_rne(float v) {
    uint32_t b = __float_as_uint(v);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (b >> 16) | 0x40;   // NaN stays NaN
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// KT > 0: k known at compile time, so the k row reads of a column group are all in flight before
// the first multiply-add; KT == 0: any k up to MAX_K.
template <int KT>
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ y_perm,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ topk_w, int T, int d, int k_rt,
                                                      uint16_t* __restrict__ y, float* __restrict__ y_f32) {
    __shared__ int32_t s_row[MAX_K];
    __shared__ float s_w[MAX_K];
    const int k = KT > 0 ? KT : k_rt;
    const int t = blockIdx.x;
    if (threadIdx.x < k) {
        s_row[threadIdx.x] = inv_perm[(size_t)t * k + threadIdx.x];
        s_w[threadIdx.x] = topk_w[(size_t)t * k + threadIdx.x];
    }
    __syncthreads();
    constexpr int KU = KT > 0 ? KT : 1;
    const float* src[KU];
    float w[KU];
    if (KT > 0) {
#pragma unroll
        for (int j = 0; j < KU; ++j) {
            const int row = s_row[j];
            src[j] = row < 0 ? nullptr : y_perm + (size_t)row * d;   // a slot whose expert id was invalid adds nothing
            w[j] = s_w[j];
        }
    }
    for (int c4 = threadIdx.x; c4 < d / 4; c4 += 256) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (KT > 0) {
            float4 v[KU];
#pragma unroll
            for (int j = 0; j < KU; ++j)
                v[j] = src[j] ? *reinterpret_cast<const float4*>(src[j] + (size_t)c4 * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int j = 0; j < KU; ++j) {
                if (!src[j]) continue;
                acc.x = fmaf(w[j], v[j].x, acc.x);
                acc.y = fmaf(w[j], v[j].y, acc.y);
                acc.z = fmaf(w[j], v[j].z, acc.z);
                acc.w = fmaf(w[j], v[j].w, acc.w);
            }
        } else {
            for (int j = 0; j < k; ++j) {
                const int row = s_row[j];
                if (row < 0) continue;
                const float wj = s_w[j];
                const float4 v = *reinterpret_cast<const float4*>(y_perm + (size_t)row * d + (size_t)c4 * 4);
                acc.x = fmaf(wj, v.x, acc.x);
                acc.y = fmaf(wj, v.y, acc.y);
                acc.z = fmaf(wj, v.z, acc.z);
                acc.w = fmaf(wj, v.w, acc.w);
            }
        }
        uint2 o;
        o.x = f32_to_bf16_rne(acc.x) | (f32_to_bf16_rne(acc.y) << 16);
        o.y = f32_to_bf16_rne(acc.z) | (f32_to_bf16_rne(acc.w) << 16);
        *reinterpret_cast<uint2*>(y + (size_t)t * d + (size_t)c4 * 4) = o;
        if (y_f32) *reinterpret_cast<float4*>(y_f32 + (size_t)t * d + (size_t)c4 * 4) = acc;   // the sums before rounding
    }
    (void)T;
}

}  // namespace

hipError_t launch_combine(moe_ctx* c, const float* y_perm, const int32_t* inv_perm, const float* topk_w,
                          uint16_t* y, float* y_f32) {
    const moe_dims& D = c->dims;
#define MOE_COMBINE(KT_)                                                                                  \
    hipLaunchKernelGGL(combine_kernel<KT_>, dim3(D.T), dim3(256), 0, c->stream, y_perm, inv_perm, topk_w, D.T, \
                       D.d, D.k, y, y_f32)
    switch (D.k) {
        case 1: MOE_COMBINE(1); break;
        case 2: MOE_COMBINE(2); break;
        case 4: MOE_COMBINE(4); break;
        case 6: MOE_COMBINE(6); break;
        case 8: MOE_COMBINE(8); break;
        default: MOE_COMBINE(0); break;
    }
#undef MOE_COMBINE
    return hipGetLastError();
}

}  // namespace moe355
