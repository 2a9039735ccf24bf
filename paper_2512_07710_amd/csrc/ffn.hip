// Grouped block-scaled FP8 SwiGLU expert FFN on the CDNA4 matrix cores.
//
// Work is cut into tiles of TOK_TILE expert-sorted rows x FEAT_TILE output features;
// a small kernel turns offsets[] into the list of row tiles so ragged experts need no
// host round trip.  Both GEMMs run the same main loop:
//
//   for each 128-wide K block kb:
//       stage the weight rows and the activation rows of the tile in LDS (16-byte chunks,
//       XOR-swizzled by row so the 32-row operand reads are bank-conflict free)
//       partial = W_tile * X_tile^T  with two v_mfma_f32_32x32x64_f8f6f4 per 32x32 sub-tile
//       acc    += (xs[row,kb] * ws[feature block,kb]) * partial      (fp32, per lane)
//
// The matrix product is taken as (features x tokens): in the 32x32 accumulator layout
// a lane then owns ONE token column and 16 feature rows, so the per-token activation
// scale is a single scalar per lane and the per-row reductions of the epilogue
// (the 128-wide amax for re-quantising h) stay inside a lane plus one cross-half shuffle.
//
// GEMM1 computes gate and up projections for the same 128 features in one tile, applies
// h = silu(g)*u and writes h as e4m3 codes + one fp32 scale per (row, 128 features).
// GEMM2 multiplies h by W2 and writes fp32 rows in expert order.
#include "moe_internal.hpp"

namespace moe355 {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int KB = QBLOCK;              // K bytes staged per step (= one scale block)
constexpr int CHUNKS = KB / 16;         // 16-byte chunks per staged row

// ------------------------------------------------------------------ tile list
__global__ __launch_bounds__(256) void build_tiles(const int32_t* __restrict__ offsets, int E,
                                                   Tile* __restrict__ tiles, int32_t* __restrict__ n_tiles) {
    __shared__ int32_t s_n[MAX_E];
    const int tid = threadIdx.x;
    int start = 0, cnt = 0;
    if (tid < E) {
        start = offsets[tid];
        cnt = offsets[tid + 1] - start;
    }
    const int mine = (cnt + TOK_TILE - 1) / TOK_TILE;
    s_n[tid] = mine;
    __syncthreads();
    for (int off = 1; off < MAX_E; off <<= 1) {
        int add = (tid >= off) ? s_n[tid - off] : 0;
        __syncthreads();
        s_n[tid] += add;
        __syncthreads();
    }
    const int base = s_n[tid] - mine;
    for (int i = 0; i < mine; ++i) {
        Tile t;
        t.expert = tid;
        t.row0 = start + i * TOK_TILE;
        tiles[base + i] = t;
    }
    if (tid == MAX_E - 1) *n_tiles = s_n[tid];
}

// ------------------------------------------------------------------ helpers
__device__ inline int swz(int row, int chunk) { return row * KB + ((chunk ^ (row & 7)) << 4); }

// the 32 K-bytes a lane feeds to one 32x32x64 MFMA: row `row`, K half `half` of K step `ks`
__device__ inline v8i load_operand(const uint8_t* tile, int row, int ks, int half) {
    const int c0 = ks * 4 + half * 2;
    const uint4 lo = *reinterpret_cast<const uint4*>(tile + swz(row, c0));
    const uint4 hi = *reinterpret_cast<const uint4*>(tile + swz(row, c0 + 1));
    v8i r;
    r[0] = lo.x; r[1] = lo.y; r[2] = lo.z; r[3] = lo.w;
    r[4] = hi.x; r[5] = hi.y; r[6] = hi.z; r[7] = hi.w;
    return r;
}

__device__ inline float clamp448(float v) { return fminf(fmaxf(v, -448.f), 448.f); }

__device__ inline uint32_t pack4_e4m3(float a, float b, float c, float d) {
    int p = 0;
    p = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), p, false);
    p = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(c), clamp448(d), p, true);
    return (uint32_t)p;
}

// ------------------------------------------------------------------ GEMM kernel
// GATED = true : A rows are [W1 tile (128 rows); W3 tile (128 rows)], K = d, epilogue SwiGLU + quant
// GATED = false: A rows are the W2 tile (128 rows), K = F, epilogue fp32 store
//
// act  [N, K] u8, act_s [N, K/128] f32 : expert-sorted activations and their scales
// Wa (and Wb if GATED) [E, NOUT, K] u8 ; sa (sb) [E, NOUT/128, K/128] f32
template <bool GATED>
__global__ __launch_bounds__(256, 1) void ffn_gemm(const uint8_t* __restrict__ act,
                                                   const float* __restrict__ act_s,
                                                   const int32_t* __restrict__ offsets,
                                                   const Tile* __restrict__ tiles,
                                                   const int32_t* __restrict__ n_tiles,
                                                   const uint8_t* __restrict__ Wa, const uint8_t* __restrict__ Wb,
                                                   const float* __restrict__ sa, const float* __restrict__ sb,
                                                   int K, int NOUT, uint8_t* __restrict__ hq,
                                                   float* __restrict__ hs, float* __restrict__ y_perm) {
    constexpr int WROWS = GATED ? 2 * FEAT_TILE : FEAT_TILE;   // staged weight rows
    constexpr int WSUB = WROWS / 32;                           // 32-row sub-tiles of the weight tile
    constexpr int W_LOADS = WROWS * CHUNKS / 256;              // 16-byte chunks per thread per step
    constexpr int X_LOADS = TOK_TILE * CHUNKS / 256;

    __shared__ __attribute__((aligned(16))) uint8_t sW[WROWS * KB];
    __shared__ __attribute__((aligned(16))) uint8_t sX[TOK_TILE * KB];

    const int n_feat_tiles = NOUT / FEAT_TILE;
    const int tile_id = blockIdx.x / n_feat_tiles;
    const int ft = blockIdx.x % n_feat_tiles;
    if (tile_id >= *n_tiles) return;
    const Tile tile = tiles[tile_id];
    const int e = tile.expert;
    const int row_end = offsets[e + 1];
    const int f0 = ft * FEAT_TILE;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int nkb = K / KB;

    // ---- global -> register staging addresses (thread owns chunk `lc` of rows lr + 32*i)
    const int lc = tid & 7, lr = tid >> 3;
    const uint8_t* wsrc[W_LOADS];
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) {
        const int r = lr + 32 * i;
        const uint8_t* basep = (GATED && r >= FEAT_TILE) ? Wb : Wa;
        const int fr = f0 + (r % FEAT_TILE);
        wsrc[i] = basep + ((size_t)e * NOUT + fr) * (size_t)K + lc * 16;
    }
    const uint8_t* xsrc[X_LOADS];
#pragma unroll
    for (int i = 0; i < X_LOADS; ++i) {
        int p = tile.row0 + lr + 32 * i;
        p = min(p, row_end - 1);                               // rows past the segment repeat its last row
        xsrc[i] = act + (size_t)p * K + lc * 16;
    }
    // the token this lane accumulates, for its activation scale
    const int my_row = tile.row0 + wave * 32 + l32;
    const bool row_ok = my_row < row_end;
    const float* my_xs = act_s + (size_t)min(my_row, row_end - 1) * nkb;
    const float* sa_e = sa + ((size_t)e * (NOUT / QBLOCK) + ft) * nkb;
    const float* sb_e = GATED ? sb + ((size_t)e * (NOUT / QBLOCK) + ft) * nkb : nullptr;

    v16f acc[WSUB];
#pragma unroll
    for (int s = 0; s < WSUB; ++s)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[s][r] = 0.f;

    uint4 wreg[W_LOADS], xreg[X_LOADS];
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) wreg[i] = *reinterpret_cast<const uint4*>(wsrc[i]);
#pragma unroll
    for (int i = 0; i < X_LOADS; ++i) xreg[i] = *reinterpret_cast<const uint4*>(xsrc[i]);
    float xscale = my_xs[0];

    for (int kb = 0; kb < nkb; ++kb) {
        __syncthreads();                                       // previous step's operand reads are done
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i) *reinterpret_cast<uint4*>(sW + swz(lr + 32 * i, lc)) = wreg[i];
#pragma unroll
        for (int i = 0; i < X_LOADS; ++i) *reinterpret_cast<uint4*>(sX + swz(lr + 32 * i, lc)) = xreg[i];
        const float cur_xscale = xscale;
        __syncthreads();
        if (kb + 1 < nkb) {                                    // prefetch the next K block
            const size_t koff = (size_t)(kb + 1) * KB;
#pragma unroll
            for (int i = 0; i < W_LOADS; ++i) wreg[i] = *reinterpret_cast<const uint4*>(wsrc[i] + koff);
#pragma unroll
            for (int i = 0; i < X_LOADS; ++i) xreg[i] = *reinterpret_cast<const uint4*>(xsrc[i] + koff);
            xscale = my_xs[kb + 1];
        }
        const float scale_a = cur_xscale * sa_e[kb];
        const float scale_b = GATED ? cur_xscale * sb_e[kb] : 0.f;

        const int xrow = wave * 32 + l32;
        const v8i b0 = load_operand(sX, xrow, 0, half);
        const v8i b1 = load_operand(sX, xrow, 1, half);
#pragma unroll
        for (int s = 0; s < WSUB; ++s) {
            const int wrow = s * 32 + l32;
            const v8i a0 = load_operand(sW, wrow, 0, half);
            const v8i a1 = load_operand(sW, wrow, 1, half);
            v16f part;
#pragma unroll
            for (int r = 0; r < 16; ++r) part[r] = 0.f;
            part = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a0, b0, part, 0, 0, 0, 0, 0, 0);
            part = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a1, b1, part, 0, 0, 0, 0, 0, 0);
            const float sc = (GATED && s >= WSUB / 2) ? scale_b : scale_a;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[s][r] = fmaf(sc, part[r], acc[s][r]);
        }
    }

    // ---- epilogue.  Accumulator element (s, r) of this lane is feature
    //      f0 + (s % 4)*32 + (r/4)*8 + half*4 + (r%4) of token my_row.
    if (GATED) {
        constexpr int HS = WSUB / 2;
        float h[HS][16];
        float amax = 0.f;
#pragma unroll
        for (int s = 0; s < HS; ++s)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float g = acc[s][r], u = acc[s + HS][r];
                const float v = (g / (1.0f + expf(-g))) * u;
                h[s][r] = v;
                amax = fmaxf(amax, fabsf(v));
            }
        amax = fmaxf(amax, __shfl_xor(amax, 32));              // the other 64 features of this token
        const float sc = (amax == 0.f) ? 1.0f : amax / 448.0f;
        if (row_ok) {
            uint8_t* dst = hq + (size_t)my_row * NOUT + f0 + half * 4;
#pragma unroll
            for (int s = 0; s < HS; ++s)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const uint32_t code = pack4_e4m3(h[s][r4 * 4] / sc, h[s][r4 * 4 + 1] / sc,
                                                     h[s][r4 * 4 + 2] / sc, h[s][r4 * 4 + 3] / sc);
                    *reinterpret_cast<uint32_t*>(dst + s * 32 + r4 * 8) = code;
                }
            if (half == 0) hs[(size_t)my_row * (NOUT / QBLOCK) + ft] = sc;
        }
    } else {
        if (row_ok) {
            float* dst = y_perm + (size_t)my_row * NOUT + f0 + half * 4;
#pragma unroll
            for (int s = 0; s < WSUB; ++s)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const float4 v = make_float4(acc[s][r4 * 4], acc[s][r4 * 4 + 1], acc[s][r4 * 4 + 2],
                                                 acc[s][r4 * 4 + 3]);
                    *reinterpret_cast<float4*>(dst + s * 32 + r4 * 8) = v;
                }
        }
    }
}

}  // namespace

hipError_t launch_expert_ffn(moe_ctx* c, const uint8_t* xq, const float* xs, const int32_t* offsets,
                             const uint8_t* W1, const uint8_t* W3, const uint8_t* W2, const float* s1,
                             const float* s3, const float* s2, float* y_perm) {
    const moe_dims& D = c->dims;
    hipLaunchKernelGGL(build_tiles, dim3(1), dim3(256), 0, c->stream, offsets, D.E, c->tiles, c->n_tiles);
    hipEvent_t* ev = nullptr;
    if (c->profiling && c->prof_calls < PROF_MAX_CALLS) ev = c->prof_events + 3 * c->prof_calls++;
    if (ev) (void)hipEventRecord(ev[0], c->stream);
    const int grid1 = c->max_tiles * (D.F / FEAT_TILE);
    hipLaunchKernelGGL((ffn_gemm<true>), dim3(grid1), dim3(256), 0, c->stream, xq, xs, offsets, c->tiles,
                       c->n_tiles, W1, W3, s1, s3, D.d, D.F, c->hq, c->hs, (float*)nullptr);
    if (ev) (void)hipEventRecord(ev[1], c->stream);
    const int grid2 = c->max_tiles * (D.d / FEAT_TILE);
    hipLaunchKernelGGL((ffn_gemm<false>), dim3(grid2), dim3(256), 0, c->stream, c->hq, c->hs, offsets,
                       c->tiles, c->n_tiles, W2, (const uint8_t*)nullptr, s2, (const float*)nullptr, D.F,
                       D.d, (uint8_t*)nullptr, (float*)nullptr, y_perm);
    if (ev) (void)hipEventRecord(ev[2], c->stream);
    return hipGetLastError();
}

}  // namespace moe355
