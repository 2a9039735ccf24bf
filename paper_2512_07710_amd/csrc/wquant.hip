// Block-wise FP8 (e4m3) quantisation of a bf16 weight matrix: one fp32 scale per 128x128 block.
//
// One workgroup per block.  Thread t owns 64 elements: row (t/2) of the block, columns
// (t%2)*64 .. +63, read as eight 16-byte vectors.  The block maximum goes through a wave
// reduction and four LDS words; scale = amax/448 and w/scale use correctly rounded fp32
// division so that codes and scales are reproducible bit for bit.  Each element is read once
// and written once: 3 bytes of HBM traffic per weight.
#include "moe_internal.hpp"

namespace moe355 {
namespace {

__device__ inline float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ inline float clamp448(float v) { return fminf(fmaxf(v, -448.f), 448.f); }
__device__ inline uint32_t pack4_e4m3(float a, float b, float c, float d) {
    int p = 0;
    p = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), p, false);
    p = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(c), clamp448(d), p, true);
    return (uint32_t)p;
}

__global__ __launch_bounds__(256) void quantize_blocks_kernel(const uint16_t* __restrict__ w, int64_t rows, int cols,
                                                              uint8_t* __restrict__ q, float* __restrict__ scales) {
    __shared__ float s_max[4];
    const int bj = blockIdx.x, tid = threadIdx.x;
    const int64_t bi = blockIdx.y;
    const int r = tid >> 1, c0 = (tid & 1) * 64;
    const size_t off = (size_t)(bi * QBLOCK + r) * cols + (size_t)bj * QBLOCK + c0;
    uint4 raw[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) raw[v] = *reinterpret_cast<const uint4*>(w + off + v * 8);
    float amax = 0.f;
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const uint32_t u[4] = {raw[v].x, raw[v].y, raw[v].z, raw[v].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) amax = fmaxf(amax, fmaxf(fabsf(bf16lo(u[i])), fabsf(bf16hi(u[i]))));
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m));
    if ((tid & 63) == 0) s_max[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    const float s = (amax == 0.f) ? 1.0f : amax / 448.0f;
    if (tid == 0) scales[(size_t)bi * (cols / QBLOCK) + bj] = s;
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const uint32_t u[4] = {raw[v].x, raw[v].y, raw[v].z, raw[v].w};
        uint2 codes;
        codes.x = pack4_e4m3(bf16lo(u[0]) / s, bf16hi(u[0]) / s, bf16lo(u[1]) / s, bf16hi(u[1]) / s);
        codes.y = pack4_e4m3(bf16lo(u[2]) / s, bf16hi(u[2]) / s, bf16lo(u[3]) / s, bf16hi(u[3]) / s);
        *reinterpret_cast<uint2*>(q + off + v * 8) = codes;
    }
}

}  // namespace

hipError_t launch_quantize_weights(hipStream_t s, const uint16_t* w, int64_t rows, int32_t cols, uint8_t* q,
                                   float* scales) {
    hipLaunchKernelGGL(quantize_blocks_kernel, dim3(cols / QBLOCK, (unsigned)(rows / QBLOCK)), dim3(256), 0, s, w, rows,
                       cols, q, scales);
    return hipGetLastError();
}

}  // namespace moe355
