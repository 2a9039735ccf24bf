// Per-row, per-128-column FP8 (e4m3) quantisation of bf16 activations, with optional
// fan-out of each quantised row to several output rows (the expert-ordered layout).
//
// Sixteen lanes own one 128-column group: each loads 8 bf16 (16 bytes), the group
// maximum is reduced with four xor-shuffles, and scale = amax/448 and x/scale are
// computed with correctly rounded fp32 division so the codes are reproducible bit
// for bit.  The row is read once and written `fanout` times.  Scales are stored K-block
// major, scales[group][output row]: the layout the grouped GEMM reads them in.
#include "moe_internal.hpp"

namespace moe355 {
namespace {

__device__ inline float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ inline float clamp448(float v) { return fminf(fmaxf(v, -448.f), 448.f); }

// four fp32 -> four e4m3 codes packed little-endian (a in the low byte)
__device__ inline uint32_t pack4_e4m3(float a, float b, float c, float d) {
    int p = 0;
    p = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), p, false);
    p = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(c), clamp448(d), p, true);
    return (uint32_t)p;
}

__global__ __launch_bounds__(256) void quantize_rows_kernel(const uint16_t* __restrict__ x, int64_t rows_in,
                                                            int cols, const int32_t* __restrict__ dst_rows,
                                                            int fanout, uint8_t* __restrict__ q,
                                                            float* __restrict__ scales) {
    const int64_t rows_out = dst_rows ? rows_in * fanout : rows_in;
    const int vecs = cols / 8;                        // 16-byte vectors per row, a multiple of 16
    for (int64_t r = blockIdx.x; r < rows_in; r += gridDim.x) {
        const uint16_t* xr = x + r * cols;
        for (int v = threadIdx.x; v < vecs; v += 256) {
            const uint4 raw = *reinterpret_cast<const uint4*>(xr + (size_t)v * 8);
            float f[8] = {bf16lo(raw.x), bf16hi(raw.x), bf16lo(raw.y), bf16hi(raw.y),
                          bf16lo(raw.z), bf16hi(raw.z), bf16lo(raw.w), bf16hi(raw.w)};
            float amax = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[i]));
            // the 16 lanes of a group are consecutive and either all active or all inactive
            amax = fmaxf(amax, __shfl_xor(amax, 1));
            amax = fmaxf(amax, __shfl_xor(amax, 2));
            amax = fmaxf(amax, __shfl_xor(amax, 4));
            amax = fmaxf(amax, __shfl_xor(amax, 8));
            const float s = (amax == 0.f) ? 1.0f : amax / 448.0f;
            uint2 codes;
            codes.x = pack4_e4m3(f[0] / s, f[1] / s, f[2] / s, f[3] / s);
            codes.y = pack4_e4m3(f[4] / s, f[5] / s, f[6] / s, f[7] / s);
            const int g = v / 16;
            for (int j = 0; j < fanout; ++j) {
                const int64_t orow = dst_rows ? (int64_t)dst_rows[r * fanout + j] : r;
                if (orow < 0) continue;               // assignment skipped by the permutation
                *reinterpret_cast<uint2*>(q + orow * cols + (size_t)v * 8) = codes;
                if ((v & 15) == 0) scales[(int64_t)g * rows_out + orow] = s;
            }
        }
    }
}

}  // namespace

hipError_t launch_quantize(hipStream_t s, const uint16_t* x, int64_t rows_in, int32_t cols,
                           const int32_t* dst_rows, int32_t fanout, uint8_t* q, float* scales) {
    const int grid = (int)(rows_in < 65536 ? rows_in : 65536);
    hipLaunchKernelGGL(quantize_rows_kernel, dim3(grid), dim3(256), 0, s, x, rows_in, cols, dst_rows, fanout, q,
                       scales);
    return hipGetLastError();
}

}  // namespace moe355
