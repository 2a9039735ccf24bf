// Grouped block-scaled FP8 SwiGLU expert FFN on the CDNA4 matrix cores.
//
// Work unit: a tile of TOK_TILE (256) expert-sorted rows x 256 staged weight rows.  A small
// kernel turns offsets[] into the list of work units (expert, first row, feature tile), so
// ragged experts need no host round trip, and orders it so that units sharing a weight tile
// are adjacent; blocks map onto the list so that each XCD (blockIdx % 8) walks a contiguous
// range and its L2 sees every weight tile once.
//
// Main loop, one iteration per 128-wide K block (= one scale block):
//   * both operand tiles are copied global -> LDS by direct-to-LDS loads (no staging
//     registers), double buffered, 16-byte chunks XOR-swizzled by row so that the 32-row
//     operand reads are bank-conflict free;
//   * partial = W_tile * X_tile^T with two v_mfma_f32_32x32x64_f8f6f4 per 32x32 sub-tile;
//   * acc += (xs[row,kb] * ws[feature block,kb]) * partial in fp32.
// The product is taken as (features x tokens): in the 32x32 accumulator layout a lane then
// owns ONE token column and 16 feature rows, so the activation scale is one scalar per lane
// and sub-tile, and the 128-wide amax of the epilogue is a lane-local reduction plus one
// cross-half shuffle and one exchange between the two waves that share a token.
//
// Eight waves per block: wave (wt, wf) owns 64 tokens x 128 staged weight rows (2 x 4
// sub-tiles): 6 operand sub-tiles feed 8 MFMA pairs, which keeps LDS reads under the
// 128 B/clk the LDS delivers.  Waves whose 64 tokens lie beyond the expert's last row skip
// their MFMAs, so a ragged tail costs a fraction of a tile.
//
// GEMM1: staged rows of wave wf are [64 gate rows | 64 up rows] of the same features;
//        epilogue h = silu(g)*u, re-quantised to e4m3 with one scale per (row, 128 features).
// GEMM2: staged rows are 256 consecutive output features; epilogue fp32 store.
#include "moe_internal.hpp"

namespace moe355 {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int KB = QBLOCK;                        // K bytes per stage (= one scale block)
constexpr int W_ROWS = 256;                       // staged weight rows per block
constexpr int X_ROWS = TOK_TILE;                  // staged activation rows per block (256)
constexpr int STAGE_BYTES = (W_ROWS + X_ROWS) * KB;   // 64 KiB
constexpr int NTHREADS = 512;
constexpr int NXCD = 8;

struct Work { int32_t expert; int32_t row0; int32_t ft; };

// ------------------------------------------------------------------ work list
// One thread per expert.  Full 256-row tiles of all experts come first, ordered (expert,
// feature tile, row tile); the ragged last tiles follow, ordered (expert, feature tile).
// Units that share a weight tile or an activation tile are thus neighbours AND do the same
// amount of work, so the blocks that run them side by side on one XCD advance in step and
// hit each other's lines in that XCD's L2 (a few K steps of skew already exceed what the L2
// retains, and the shared tile is then fetched again from HBM).
__global__ __launch_bounds__(256) void build_work(const int32_t* __restrict__ offsets, int E, int n_ft,
                                                  Work* __restrict__ work, int32_t* __restrict__ n_work) {
    __shared__ int32_t s_full[MAX_E];
    __shared__ int32_t s_tail[MAX_E];
    const int tid = threadIdx.x;
    int start = 0, cnt = 0;
    if (tid < E) {
        start = offsets[tid];
        cnt = offsets[tid + 1] - start;
    }
    const int full = cnt / TOK_TILE;
    const int tail = (cnt % TOK_TILE) ? 1 : 0;
    s_full[tid] = full;
    s_tail[tid] = tail;
    __syncthreads();
    for (int off = 1; off < MAX_E; off <<= 1) {
        const int a = (tid >= off) ? s_full[tid - off] : 0;
        const int b = (tid >= off) ? s_tail[tid - off] : 0;
        __syncthreads();
        s_full[tid] += a;
        s_tail[tid] += b;
        __syncthreads();
    }
    const int all_full = s_full[MAX_E - 1];
    const int base_full = (s_full[tid] - full) * n_ft;
    for (int f = 0; f < n_ft; ++f)
        for (int i = 0; i < full; ++i) {
            Work w;
            w.expert = tid;
            w.row0 = start + i * TOK_TILE;
            w.ft = f;
            work[base_full + f * full + i] = w;
        }
    if (tail) {
        const int base_tail = (all_full + s_tail[tid] - 1) * n_ft;
        for (int f = 0; f < n_ft; ++f) {
            Work w;
            w.expert = tid;
            w.row0 = start + full * TOK_TILE;
            w.ft = f;
            work[base_tail + f] = w;
        }
    }
    if (tid == MAX_E - 1) *n_work = (all_full + s_tail[tid]) * n_ft;
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

// Direct global -> LDS copies.  Lane i of the wave deposits its bytes at lds_addr + i*size;
// the global address is sbase + voff (per lane).  Completion is tracked by vmcnt; the
// compiler does not see these as memory operations of its own, so every wait on them is
// written out explicitly below.
__device__ inline void dma16(uint32_t lds_addr, uint32_t voff, const void* sbase) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}
__device__ inline void dma4(uint32_t lds_addr, uint32_t voff, const void* sbase) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}

__device__ inline float clamp448(float v) { return fminf(fmaxf(v, -448.f), 448.f); }

__device__ inline uint32_t pack4_e4m3(float a, float b, float c, float d) {
    int p = 0;
    p = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), p, false);
    p = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(c), clamp448(d), p, true);
    return (uint32_t)p;
}

// ------------------------------------------------------------------ GEMM kernel
// GATED = true : Wa = W1, Wb = W3 [E, NOUT, K]; feature tile = 128 features (gate + up rows)
// GATED = false: Wa = W2 [E, NOUT, K]; feature tile = 256 output features
// act [N, K] u8 and act_s [N, K/128] f32 are the expert-sorted activations and their scales.
template <bool GATED>
__global__ __launch_bounds__(NTHREADS, 1) void ffn_gemm(const uint8_t* __restrict__ act,
                                                        const float* __restrict__ act_s,
                                                        const int32_t* __restrict__ offsets,
                                                        const Work* __restrict__ work,
                                                        const int32_t* __restrict__ n_work,
                                                        const uint8_t* __restrict__ Wa,
                                                        const uint8_t* __restrict__ Wb,
                                                        const float* __restrict__ sa,
                                                        const float* __restrict__ sb, int K, int NOUT,
                                                        uint8_t* __restrict__ hq, float* __restrict__ hs,
                                                        float* __restrict__ y_perm) {
    constexpr int FT = GATED ? 128 : 256;                      // output features per tile
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    // [2 stages][W rows | X rows][128 B], then [2][256] activation scales, [256] dummy, [2][256] amax
    uint8_t* const s_stage = smem;
    float* const s_xs = reinterpret_cast<float*>(smem + 2 * STAGE_BYTES);
    float* const s_amax = s_xs + 3 * X_ROWS;

    // ---- which work unit: XCD x (= blockIdx % 8) walks the contiguous range [x*chunk, (x+1)*chunk)
    const int total = *n_work;
    const int chunk = (total + NXCD - 1) / NXCD;
    const int slot = blockIdx.x / NXCD;
    const int wi = (blockIdx.x % NXCD) * chunk + slot;
    if (slot >= chunk || wi >= total) return;
    const Work wk = work[wi];
    const int e = wk.expert;
    const int row_end = offsets[e + 1];
    const int f0 = wk.ft * FT;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wt = wave >> 1, wf = wave & 1;                   // token group (64 rows), weight-row half
    const int nkb = K / KB;
    const int nblk_out = NOUT / QBLOCK;

    // ---- DMA plan: wave w copies staged rows [w*64, w*64+64) of the 512 (W rows then X rows),
    //      8 instructions of 8 rows each; lane i -> row i/8, LDS chunk slot i%8.
    const uint8_t* dma_base;                                   // wave-uniform
    uint32_t dma_off[8];
    {
        const int sub = lane >> 3, cslot = lane & 7;
        if (wave < 4) {
            // staged W row r: GATED: wave 0,2 gate rows, wave 1,3 up rows of features f0 + (r/128)*64 + r%64
            const int r0 = wave * 64;
            const uint8_t* wbase = (GATED && (wave & 1)) ? Wb : Wa;
            dma_base = wbase + (size_t)e * NOUT * (size_t)K;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = r0 + j * 8 + sub;
                int f = GATED ? f0 + (r >> 7) * 64 + (r & 63) : f0 + r;
                f = min(f, NOUT - 1);
                dma_off[j] = (uint32_t)f * (uint32_t)K + ((cslot ^ (r & 7)) << 4);
            }
        } else {
            const int r0 = (wave - 4) * 64;
            dma_base = act;
            // rows past the expert's segment repeat its last row (never stored)
            const size_t first = (size_t)wk.row0 * K;
            dma_base += first;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = r0 + j * 8 + sub;
                const int p = min(wk.row0 + r, row_end - 1) - wk.row0;
                dma_off[j] = (uint32_t)p * (uint32_t)K + ((cslot ^ (r & 7)) << 4);
            }
        }
    }
    // activation scales of one K block: waves 4..7 copy 64 each; waves 0..3 issue a same-sized
    // copy into a dummy area so that every wave has the same number of copies in flight
    const float* xs_base = act_s + (size_t)wk.row0 * nkb;
    uint32_t xs_off;
    {
        const int r = ((wave & 3) * 64 + lane);
        const int p = min(wk.row0 + r, row_end - 1) - wk.row0;
        xs_off = (uint32_t)p * (uint32_t)nkb * 4u;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)smem;
    const uint32_t lds_rows = lds0 + wave * 64 * KB;           // this wave's rows inside a stage
    const uint32_t lds_xs = lds0 + 2 * STAGE_BYTES + (wave >= 4 ? 0 : 2 * X_ROWS * 4) + (wave & 3) * 64 * 4;

    auto issue_stage = [&](int kb, int buf) {
        const uint8_t* src = dma_base + (size_t)kb * KB;
        const uint32_t dst = lds_rows + buf * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < 8; ++j) dma16(dst + j * 8 * KB, dma_off[j], src);
        dma4(lds_xs + (wave >= 4 ? buf * X_ROWS * 4 : 0), xs_off, xs_base + kb);
    };

    // ---- weight scales of this wave's rows (wave-uniform -> scalar loads)
    const int blk_a = GATED ? wk.ft : min(wk.ft * 2 + wf, nblk_out - 1);
    const float* sa_e = sa + ((size_t)e * nblk_out + blk_a) * nkb;
    const float* sb_e = GATED ? sb + ((size_t)e * nblk_out + blk_a) * nkb : sa_e;

    const bool wave_active = wk.row0 + wt * 64 < row_end;      // wave-uniform

    v16f acc[4][2];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int ts = 0; ts < 2; ++ts)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[s][ts][r] = 0.f;

    float wsa_next = sa_e[0], wsb_next = sb_e[0];
    issue_stage(0, 0);
    for (int kb = 0; kb < nkb; ++kb) {
        const int buf = kb & 1;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // this wave's copies of stage kb landed
        __builtin_amdgcn_s_barrier();                          // everybody's landed; stage kb-1 fully consumed
        asm volatile("" ::: "memory");
        if (kb + 1 < nkb) issue_stage(kb + 1, buf ^ 1);
        if (wave_active) {
            const uint8_t* sW = s_stage + buf * STAGE_BYTES;
            const uint8_t* sX = sW + W_ROWS * KB;
            const float wsa = wsa_next, wsb = wsb_next;        // loaded one iteration ahead
            if (kb + 1 < nkb) {
                wsa_next = sa_e[kb + 1];
                wsb_next = sb_e[kb + 1];
            }
            v8i b[2][2];
            float sc_a[2], sc_b[2];
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                const int xrow = wt * 64 + ts * 32 + l32;
                b[ts][0] = load_operand(sX, xrow, 0, half);
                b[ts][1] = load_operand(sX, xrow, 1, half);
                const float xsc = s_xs[buf * X_ROWS + xrow];
                sc_a[ts] = xsc * wsa;
                sc_b[ts] = xsc * wsb;
            }
            // Software pipeline over the 8 (weight sub-tile s, token sub-tile ts) pairs: the two
            // MFMAs of pair i are issued before the 16 scale-FMAs of pair i-1, so the matrix
            // pipe works on pair i while the vector ALU folds pair i-1 into the accumulators.
            const int wrow0 = wf * 128 + l32;
            v8i a0 = load_operand(sW, wrow0, 0, half);
            v8i a1 = load_operand(sW, wrow0, 1, half);
            v16f zero;
#pragma unroll
            for (int r = 0; r < 16; ++r) zero[r] = 0.f;
            v16f prev = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a0, b[0][0], zero, 0, 0, 0, 0, 0, 0);
            prev = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a1, b[0][1], prev, 0, 0, 0, 0, 0, 0);
#pragma unroll
            for (int i = 1; i < 8; ++i) {
                const int s = i >> 1, ts = i & 1;
                if (ts == 0) {
                    a0 = load_operand(sW, wrow0 + s * 32, 0, half);
                    a1 = load_operand(sW, wrow0 + s * 32, 1, half);
                }
                __builtin_amdgcn_sched_barrier(0);
                v16f cur = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a0, b[ts][0], zero, 0, 0, 0, 0, 0, 0);
                cur = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a1, b[ts][1], cur, 0, 0, 0, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                const int ps = (i - 1) >> 1, pts = (i - 1) & 1;
                const float sc = (GATED && ps >= 2) ? sc_b[pts] : sc_a[pts];
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ps][pts][r] = fmaf(sc, prev[r], acc[ps][pts][r]);
                __builtin_amdgcn_sched_barrier(0);
                prev = cur;
            }
            {
                const float sc = GATED ? sc_b[1] : sc_a[1];
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[3][1][r] = fmaf(sc, prev[r], acc[3][1][r]);
            }
        }
    }

    // ---- epilogue.  Accumulator (s, ts, r) of this lane belongs to token
    //      row0 + wt*64 + ts*32 + l32 and staged weight row wf*128 + s*32 + (r/4)*8 + half*4 + r%4.
    if (GATED) {
        // gate rows s = 0,1 and up rows s = 2,3 of features f0 + wf*64 + (s&1)*32 + ...
        float h[2][2][16];
        float amax[2] = {0.f, 0.f};
        if (wave_active) {
#pragma unroll
            for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float g = acc[s][ts][r], u = acc[s + 2][ts][r];
                        const float v = (g / (1.0f + __expf(-g))) * u;
                        h[ts][s][r] = v;
                        amax[ts] = fmaxf(amax[ts], fabsf(v));
                    }
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                amax[ts] = fmaxf(amax[ts], __shfl_xor(amax[ts], 32));   // the lane pair covers 64 features
                if (half == 0) s_amax[wf * X_ROWS + wt * 64 + ts * 32 + l32] = amax[ts];
            }
        }
        __syncthreads();                                       // the other 64 features live in wave (wt, wf^1)
        if (wave_active) {
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                const int trow = wt * 64 + ts * 32 + l32;
                const int p = wk.row0 + trow;
                const float am = fmaxf(amax[ts], s_amax[(wf ^ 1) * X_ROWS + trow]);
                const float sc = (am == 0.f) ? 1.0f : am / 448.0f;
                if (p < row_end) {
                    uint8_t* dst = hq + (size_t)p * NOUT + f0 + wf * 64 + half * 4;
#pragma unroll
                    for (int s = 0; s < 2; ++s)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            const uint32_t code = pack4_e4m3(h[ts][s][r4 * 4] / sc, h[ts][s][r4 * 4 + 1] / sc,
                                                             h[ts][s][r4 * 4 + 2] / sc, h[ts][s][r4 * 4 + 3] / sc);
                            *reinterpret_cast<uint32_t*>(dst + s * 32 + r4 * 8) = code;
                        }
                    if (half == 0 && wf == 0) hs[(size_t)p * nblk_out + wk.ft] = sc;
                }
            }
        }
    } else {
        if (wave_active) {
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                const int p = wk.row0 + wt * 64 + ts * 32 + l32;
                if (p < row_end) {
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        const int fbase = f0 + wf * 128 + s * 32 + half * 4;
                        if (fbase < NOUT) {
                            float* dst = y_perm + (size_t)p * NOUT + fbase;
#pragma unroll
                            for (int r4 = 0; r4 < 4; ++r4) {
                                const float4 v = make_float4(acc[s][ts][r4 * 4], acc[s][ts][r4 * 4 + 1],
                                                             acc[s][ts][r4 * 4 + 2], acc[s][ts][r4 * 4 + 3]);
                                *reinterpret_cast<float4*>(dst + r4 * 8) = v;
                            }
                        }
                    }
                }
            }
        }
    }
}

constexpr size_t SMEM_BYTES = 2 * STAGE_BYTES + 5 * X_ROWS * sizeof(float);

}  // namespace

size_t ffn_work_bytes(int max_tiles, int F, int d) {
    return sizeof(Work) * (size_t)max_tiles * (size_t)(F / 128 + (d + 255) / 256);
}

hipError_t launch_expert_ffn(moe_ctx* c, const uint8_t* xq, const float* xs, const int32_t* offsets,
                             const uint8_t* W1, const uint8_t* W3, const uint8_t* W2, const float* s1,
                             const float* s3, const float* s2, float* y_perm) {
    const moe_dims& D = c->dims;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_gemm<true>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM_BYTES);
        hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_gemm<false>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM_BYTES);
        if (e1 != hipSuccess) return e1;
        if (e2 != hipSuccess) return e2;
        attr_set = true;
    }
    Work* work = reinterpret_cast<Work*>(c->tiles);
    hipEvent_t* ev = nullptr;
    if (c->profiling && c->prof_calls < PROF_MAX_CALLS) ev = c->prof_events + 3 * c->prof_calls++;

    const int nft1 = D.F / 128;
    const int nft2 = (D.d + 255) / 256;
    Work* work2 = work + (size_t)c->max_tiles * nft1;          // the down projection's list
    int32_t* n_work2 = c->n_tiles + 1;
    hipLaunchKernelGGL(build_work, dim3(1), dim3(256), 0, c->stream, offsets, D.E, nft1, work, c->n_tiles);
    hipLaunchKernelGGL(build_work, dim3(1), dim3(256), 0, c->stream, offsets, D.E, nft2, work2, n_work2);
    if (ev) (void)hipEventRecord(ev[0], c->stream);
    const int grid1 = ((c->max_tiles * nft1 + NXCD - 1) / NXCD) * NXCD;
    hipLaunchKernelGGL((ffn_gemm<true>), dim3(grid1), dim3(NTHREADS), SMEM_BYTES, c->stream, xq, xs, offsets,
                       work, c->n_tiles, W1, W3, s1, s3, D.d, D.F, c->hq, c->hs, (float*)nullptr);
    if (ev) (void)hipEventRecord(ev[1], c->stream);
    const int grid2 = ((c->max_tiles * nft2 + NXCD - 1) / NXCD) * NXCD;
    hipLaunchKernelGGL((ffn_gemm<false>), dim3(grid2), dim3(NTHREADS), SMEM_BYTES, c->stream, c->hq, c->hs,
                       offsets, work2, n_work2, W2, (const uint8_t*)nullptr, s2, (const float*)nullptr, D.F,
                       D.d, (uint8_t*)nullptr, (float*)nullptr, y_perm);
    if (ev) (void)hipEventRecord(ev[2], c->stream);
    return hipGetLastError();
}

}  // namespace moe355
