// Router GEMM fused with top-k selection and gate weights (routed mode).
//
// One block scores TT tokens against all E experts: logits are accumulated in
// fp32 from bf16 activations and fp32 router weights staged through LDS, then
// each wave picks the top k of a token with shuffle reductions (larger score
// wins, equal scores go to the lower expert index) and turns the k selected
// unbiased logits into softmax gate weights.
#include "moe_internal.hpp"

namespace moe355 {
namespace {

constexpr int TT = 16;    // tokens per block
constexpr int KC = 32;    // hidden columns staged per step
constexpr int WPAD = 4;   // row padding (floats) of the staged router tile

__device__ inline float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// EP: expert count padded to a power of two in [32,256]; 256/EP thread groups split each K step.
template <int EP>
__global__ __launch_bounds__(256) void route_kernel(const uint16_t* __restrict__ x,
                                                    const float* __restrict__ W,
                                                    const float* __restrict__ bias, int T, int d, int E,
                                                    int k, int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w) {
    constexpr int GRP = 256 / EP;      // thread groups sharing one expert column
    constexpr int CPG = KC / GRP;      // hidden columns per group per step (multiple of 4)
    static_assert(CPG % 4 == 0, "column split must keep float4 granularity");
    constexpr int VPT = (EP + 63) / 64;

    __shared__ float xs[TT][KC];
    // the staged router tile; the thread groups' partial sums reuse its storage afterwards
    constexpr int WS_FLOATS = EP * (KC + WPAD) > GRP * TT * EP ? EP * (KC + WPAD) : GRP * TT * EP;
    __shared__ float ws_raw[WS_FLOATS];
    float (*ws)[KC + WPAD] = reinterpret_cast<float (*)[KC + WPAD]>(ws_raw);
    __shared__ float logit[TT][EP + 1];

    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * TT;
    const int e = tid % EP;
    const int grp = tid / EP;

    float acc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) acc[t] = 0.f;

    for (int kc = 0; kc < d; kc += KC) {
        // activations: TT x KC bf16 = TT*KC/8 vectors of 8
        if (tid < TT * KC / 8) {
            const int t = tid / (KC / 8), c8 = tid % (KC / 8);
            uint4 v = make_uint4(0, 0, 0, 0);
            if (t0 + t < T) v = *reinterpret_cast<const uint4*>(x + (size_t)(t0 + t) * d + kc + c8 * 8);
            float* dst = &xs[t][c8 * 8];
            dst[0] = bf16_to_f32(v.x & 0xFFFF); dst[1] = bf16_to_f32(v.x >> 16);
            dst[2] = bf16_to_f32(v.y & 0xFFFF); dst[3] = bf16_to_f32(v.y >> 16);
            dst[4] = bf16_to_f32(v.z & 0xFFFF); dst[5] = bf16_to_f32(v.z >> 16);
            dst[6] = bf16_to_f32(v.w & 0xFFFF); dst[7] = bf16_to_f32(v.w >> 16);
        }
        // router weights: EP x KC floats, coalesced along the hidden axis
        for (int i = tid; i < EP * (KC / 4); i += 256) {
            const int r = i / (KC / 4), c4 = i % (KC / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < E) v = *reinterpret_cast<const float4*>(W + (size_t)r * d + kc + c4 * 4);
            *reinterpret_cast<float4*>(&ws[r][c4 * 4]) = v;
        }
        __syncthreads();
#pragma unroll
        for (int cc = 0; cc < CPG; cc += 4) {
            const int c = grp * CPG + cc;
            const float4 w4 = *reinterpret_cast<const float4*>(&ws[e][c]);
#pragma unroll
            for (int t = 0; t < TT; ++t) {
                const float4 x4 = *reinterpret_cast<const float4*>(&xs[t][c]);
                float a = acc[t];
                a = fmaf(x4.x, w4.x, a);
                a = fmaf(x4.y, w4.y, a);
                a = fmaf(x4.z, w4.z, a);
                a = fmaf(x4.w, w4.w, a);
                acc[t] = a;
            }
        }
        __syncthreads();
    }

    if (GRP == 1) {
#pragma unroll
        for (int t = 0; t < TT; ++t) logit[t][e] = acc[t];
    } else {
        float* part = ws_raw;                         // [GRP][TT][EP]
#pragma unroll
        for (int t = 0; t < TT; ++t) part[(grp * TT + t) * EP + e] = acc[t];
        __syncthreads();
        for (int i = tid; i < TT * EP; i += 256) {
            const int t = i / EP, ee = i % EP;
            float s = 0.f;
            for (int g = 0; g < GRP; ++g) s += part[(g * TT + t) * EP + ee];
            logit[t][ee] = s;
        }
    }
    __syncthreads();

    // ---- top-k and gate weights: one wave per token, four tokens in flight ----
    const int lane = tid & 63, wave = tid >> 6;
    for (int t = wave; t < TT; t += 4) {
        if (t0 + t >= T) break;                       // uniform per wave
        float sc[VPT];
        bool taken[VPT];
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            const int ee = lane + 64 * v;
            taken[v] = !(ee < E);
            sc[v] = 0.f;
            if (ee < E) sc[v] = logit[t][ee] + (bias ? bias[ee] : 0.f);
        }
        int my_idx = 0;
        float my_logit = 0.f;
        for (int j = 0; j < k; ++j) {
            float bs = 0.f;
            int bi = 0x7FFFFFFF;                      // "no candidate"
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
                const int ee = lane + 64 * v;
                if (!taken[v] && (bi == 0x7FFFFFFF || sc[v] > bs)) { bs = sc[v]; bi = ee; }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const float os = __shfl_xor(bs, off);
                const int oi = __shfl_xor(bi, off);
                const bool other_valid = oi != 0x7FFFFFFF;
                const bool mine_valid = bi != 0x7FFFFFFF;
                const bool take = other_valid && (!mine_valid || os > bs || (os == bs && oi < bi));
                if (take) { bs = os; bi = oi; }
            }
            // bi is now uniform across the wave
#pragma unroll
            for (int v = 0; v < VPT; ++v)
                if (lane + 64 * v == bi) taken[v] = true;
            if (lane == j) { my_idx = bi; my_logit = logit[t][bi]; }
        }
        // softmax over the k selected unbiased logits (lanes 0..k-1)
        float m = (lane < k) ? my_logit : -INFINITY;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
        float p = (lane < k) ? expf(my_logit - m) : 0.f;
        float s = p;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        if (lane < k) {
            topk_idx[(size_t)(t0 + t) * k + lane] = my_idx;
            topk_w[(size_t)(t0 + t) * k + lane] = p / s;
        }
    }
}

}  // namespace

hipError_t launch_route(moe_ctx* c, const uint16_t* x, const float* W_r, const float* bias,
                        int32_t* topk_idx, float* topk_w) {
    const moe_dims& D = c->dims;
    if (D.T == 0) return hipSuccess;
    const int grid = (D.T + TT - 1) / TT;
#define ROUTE_CASE(EP)                                                                           \
    hipLaunchKernelGGL((route_kernel<EP>), dim3(grid), dim3(256), 0, c->stream, x, W_r, bias, D.T, \
                       D.d, D.E, D.k, topk_idx, topk_w)
    if (D.E <= 32) ROUTE_CASE(32);
    else if (D.E <= 64) ROUTE_CASE(64);
    else if (D.E <= 128) ROUTE_CASE(128);
    else ROUTE_CASE(256);
#undef ROUTE_CASE
    return hipGetLastError();
}

}  // namespace moe355
