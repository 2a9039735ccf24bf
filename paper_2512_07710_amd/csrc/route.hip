// Router GEMM on the bf16 matrix cores, fused with top-k selection and gate weights.
//
// The fp32 router matrix is first split into three bf16 planes (hi + mid + lo reproduces
// every fp32 weight exactly), stored in the order the matrix cores consume them.  Since
// the activations are bf16 already, every product x*w_plane is exact in fp32 and the
// accumulated logit is as accurate as an fp32 FMA chain, at matrix-core speed.
//
// One block scores 128, 64 or 32 tokens against all experts.  Wave w owns a quarter of the
// (padded) experts: its weight operands come straight from global memory, fully
// coalesced, while the activation tile is staged through LDS and shared by
// the four waves.  The product is taken as (experts x tokens), so a lane owns one
// token column; each lane pair then extracts the k best of the wave's experts for its
// token with register scans and one cross-half shuffle per round (larger score wins,
// equal scores go to the lower expert index), and a final pass merges the four waves'
// candidates, applies the softmax over the k selected unbiased logits and writes out.
//
// Batches of at most 4096 tokens would give that kernel fewer blocks than half the compute units.
// They take 32-token tiles whose K loop is split over up to 16 blocks; each block writes its
// partial logits, and a second kernel (one wave per token) adds them up in split order and does
// the same selection with wave-wide reductions.
#include "moe_internal.hpp"

#include <type_traits>

namespace moe355 {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int NO_CAND = 0x7FFFFFFF;
// Batches of at most ROUTE_SPLIT_MAX_T tokens (fewer 32-token tiles than half the compute units) run the K loop
// split over up to ROUTE_MAX_SPLITS blocks per token tile: as many as bring the grid to about 256 blocks.
constexpr int ROUTE_SPLIT_MAX_T = 4096;
constexpr int ROUTE_MAX_SPLITS = 16;

__device__ inline uint32_t f32_to_bf16_rne_bits(float v) {
    const uint32_t b = __float_as_uint(v);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}
__device__ inline float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// W [E, d] fp32 -> planes in matrix-core operand order:
// [(expert sub-tile st, k step kk, plane p)][lane = half*32 + row][8 bf16], lane's 8 columns = kk*16 + half*8 + 0..7
__global__ __launch_bounds__(256) void split_router_weights(const float* __restrict__ W, int E, int E_pad, int d,
                                                            uint16_t* __restrict__ planes) {
    const int groups = d / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)E_pad * groups) return;
    const int e = (int)(idx / groups), g = (int)(idx % groups);
    float w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = 0.f;
    if (e < E) {
        const float4 a = *reinterpret_cast<const float4*>(W + (size_t)e * d + g * 8);
        const float4 b = *reinterpret_cast<const float4*>(W + (size_t)e * d + g * 8 + 4);
        w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
    }
    uint32_t p[3][8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t h0 = f32_to_bf16_rne_bits(w[j]);
        const float r1 = w[j] - bf16_bits_to_f32(h0);          // exact
        const uint32_t h1 = f32_to_bf16_rne_bits(r1);
        const float r2 = r1 - bf16_bits_to_f32(h1);            // exact, at most 8 significant bits left
        p[0][j] = h0; p[1][j] = h1; p[2][j] = f32_to_bf16_rne_bits(r2);
    }
    const int st = e >> 5, row = e & 31, kk = g >> 1, half = g & 1;
    const int nk = d / 16;
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) {
        uint4 v;
        v.x = p[pl][0] | (p[pl][1] << 16); v.y = p[pl][2] | (p[pl][3] << 16);
        v.z = p[pl][4] | (p[pl][5] << 16); v.w = p[pl][6] | (p[pl][7] << 16);
        const size_t off = ((((size_t)st * nk + kk) * 3 + pl) * 64 + half * 32 + row) * 8;
        *reinterpret_cast<uint4*>(planes + off) = v;
    }
}

// s_waitcnt vmcnt(n): the immediate has to be a literal in the asm text, so one case per value; n is known
// after unrolling and the switch folds away.  Values beyond the 6-bit field wait for everything.
__device__ inline void wait_vm(int n) {
    switch (n) {
        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
        case 1: asm volatile("s_waitcnt vmcnt(1)" ::: "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(3)" ::: "memory"); break;
        case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
        case 5: asm volatile("s_waitcnt vmcnt(5)" ::: "memory"); break;
        case 6: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
        case 7: asm volatile("s_waitcnt vmcnt(7)" ::: "memory"); break;
        case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
        case 9: asm volatile("s_waitcnt vmcnt(9)" ::: "memory"); break;
        case 10: asm volatile("s_waitcnt vmcnt(10)" ::: "memory"); break;
        case 11: asm volatile("s_waitcnt vmcnt(11)" ::: "memory"); break;
        case 12: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
        case 13: asm volatile("s_waitcnt vmcnt(13)" ::: "memory"); break;
        case 14: asm volatile("s_waitcnt vmcnt(14)" ::: "memory"); break;
        case 15: asm volatile("s_waitcnt vmcnt(15)" ::: "memory"); break;
        case 16: asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
        case 17: asm volatile("s_waitcnt vmcnt(17)" ::: "memory"); break;
        case 18: asm volatile("s_waitcnt vmcnt(18)" ::: "memory"); break;
        case 19: asm volatile("s_waitcnt vmcnt(19)" ::: "memory"); break;
        case 20: asm volatile("s_waitcnt vmcnt(20)" ::: "memory"); break;
        case 21: asm volatile("s_waitcnt vmcnt(21)" ::: "memory"); break;
        case 22: asm volatile("s_waitcnt vmcnt(22)" ::: "memory"); break;
        case 23: asm volatile("s_waitcnt vmcnt(23)" ::: "memory"); break;
        case 24: asm volatile("s_waitcnt vmcnt(24)" ::: "memory"); break;
        case 25: asm volatile("s_waitcnt vmcnt(25)" ::: "memory"); break;
        case 26: asm volatile("s_waitcnt vmcnt(26)" ::: "memory"); break;
        case 27: asm volatile("s_waitcnt vmcnt(27)" ::: "memory"); break;
        case 28: asm volatile("s_waitcnt vmcnt(28)" ::: "memory"); break;
        case 29: asm volatile("s_waitcnt vmcnt(29)" ::: "memory"); break;
        case 30: asm volatile("s_waitcnt vmcnt(30)" ::: "memory"); break;
        case 31: asm volatile("s_waitcnt vmcnt(31)" ::: "memory"); break;
        case 32: asm volatile("s_waitcnt vmcnt(32)" ::: "memory"); break;
        case 33: asm volatile("s_waitcnt vmcnt(33)" ::: "memory"); break;
        case 34: asm volatile("s_waitcnt vmcnt(34)" ::: "memory"); break;
        case 35: asm volatile("s_waitcnt vmcnt(35)" ::: "memory"); break;
        case 36: asm volatile("s_waitcnt vmcnt(36)" ::: "memory"); break;
        case 37: asm volatile("s_waitcnt vmcnt(37)" ::: "memory"); break;
        case 38: asm volatile("s_waitcnt vmcnt(38)" ::: "memory"); break;
        case 39: asm volatile("s_waitcnt vmcnt(39)" ::: "memory"); break;
        case 40: asm volatile("s_waitcnt vmcnt(40)" ::: "memory"); break;
        case 41: asm volatile("s_waitcnt vmcnt(41)" ::: "memory"); break;
        case 42: asm volatile("s_waitcnt vmcnt(42)" ::: "memory"); break;
        case 43: asm volatile("s_waitcnt vmcnt(43)" ::: "memory"); break;
        case 44: asm volatile("s_waitcnt vmcnt(44)" ::: "memory"); break;
        case 45: asm volatile("s_waitcnt vmcnt(45)" ::: "memory"); break;
        case 46: asm volatile("s_waitcnt vmcnt(46)" ::: "memory"); break;
        case 47: asm volatile("s_waitcnt vmcnt(47)" ::: "memory"); break;
        case 48: asm volatile("s_waitcnt vmcnt(48)" ::: "memory"); break;
        case 49: asm volatile("s_waitcnt vmcnt(49)" ::: "memory"); break;
        case 50: asm volatile("s_waitcnt vmcnt(50)" ::: "memory"); break;
        case 51: asm volatile("s_waitcnt vmcnt(51)" ::: "memory"); break;
        case 52: asm volatile("s_waitcnt vmcnt(52)" ::: "memory"); break;
        case 53: asm volatile("s_waitcnt vmcnt(53)" ::: "memory"); break;
        case 54: asm volatile("s_waitcnt vmcnt(54)" ::: "memory"); break;
        case 55: asm volatile("s_waitcnt vmcnt(55)" ::: "memory"); break;
        case 56: asm volatile("s_waitcnt vmcnt(56)" ::: "memory"); break;
        case 57: asm volatile("s_waitcnt vmcnt(57)" ::: "memory"); break;
        case 58: asm volatile("s_waitcnt vmcnt(58)" ::: "memory"); break;
        case 59: asm volatile("s_waitcnt vmcnt(59)" ::: "memory"); break;
        case 60: asm volatile("s_waitcnt vmcnt(60)" ::: "memory"); break;
        case 61: asm volatile("s_waitcnt vmcnt(61)" ::: "memory"); break;
        case 62: asm volatile("s_waitcnt vmcnt(62)" ::: "memory"); break;
        case 63: asm volatile("s_waitcnt vmcnt(63)" ::: "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
}
#define WAIT_VM(N) wait_vm(N)

// NS: 32-expert sub-tiles per wave (E_pad = 128*NS).  TS: 32-token sub-tiles per block (32*TS tokens):
// four for large batches, one when the batch would otherwise fill only a fraction of the compute units.
// KS: K steps (of 16 columns) per staged activation chunk = depth of the weight-operand ring (8 in every launch:
// with 4 the K loop of the small token tiles is a chain of L2 round trips).
// IDS = false: top-k selection.  IDS = true (ids-only Router Replay): the k expert ids of every token are
// given in logged_idx; their logits are picked out of the same accumulators and only the softmax is new.
// SPLIT = true (small batches, where one block per token tile would leave most compute units idle): block
// (x, y) runs only chunks [y*cps, (y+1)*cps) of the K loop and writes its partial logits to
// partial[y][token][expert]; route_finish_kernel adds the partials up and does the selection.
template <int NS, int TS, int KS, bool IDS, bool SPLIT = false>
__global__ __launch_bounds__(256, 1) void route_mfma_kernel(const uint16_t* __restrict__ x,
                                                            const uint16_t* __restrict__ planes,
                                                            const float* __restrict__ bias,
                                                            const int32_t* __restrict__ logged_idx, int T, int d,
                                                            int E, int k, int32_t* __restrict__ topk_idx,
                                                            float* __restrict__ topk_w,
                                                            float* __restrict__ partial, int cps) {
    constexpr int RT = 32 * TS;                                // tokens per block
    constexpr int PANELS = KS / 4;                             // a chunk is staged as panels of RT rows x 128 bytes (64 columns)
    constexpr int STAGE = PANELS * RT * 128;                   // bytes of one staged chunk
    constexpr int AH = KS - 1;                                 // K steps the weight loads run ahead
    constexpr int L = 3 * NS;                                  // weight loads per K step and wave
    constexpr int C = PANELS * TS;                             // activation copies per chunk and wave
    static_assert(KS == 4 || KS == 8, "a ring slot is a step's position inside its chunk");
    // two activation stages; the candidate lists [token][wave][MAX_K] of {logit, expert id} reuse the
    // storage afterwards
    __shared__ __attribute__((aligned(16))) uint8_t smem[RT * 4 * MAX_K * 8];
    static_assert(RT * 4 * MAX_K * 8 >= 2 * STAGE, "stages fit");
    static_assert(AH * L + C <= 63 && KS * L <= 63, "wait counts fit the 6-bit field");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int t0 = blockIdx.x * RT;
    const int nchunks_all = d / (16 * KS);
    const int kc_begin = SPLIT ? (int)blockIdx.y * cps : 0;
    const int nchunks = SPLIT ? min(nchunks_all, kc_begin + cps) : nchunks_all;   // this block's chunks: [kc_begin, nchunks)
    const int nk = nchunks * KS;                                                  // one past its last K step

    // activation staging by direct-to-LDS copies: wave w, copy j < TS brings rows (TS*w+j)*8 .. +7 of the chunk;
    // lane i -> row i/8, LDS chunk slot i%8, which receives global 16-byte chunk
    // slot ^ (row & 7) ^ ((row >> 3) & 1) (the operand reads then touch all 64 LDS banks evenly)
    uint32_t xoff[TS];
#pragma unroll
    for (int j = 0; j < TS; ++j) {
        const int row = (wave * TS + j) * 8 + (lane >> 3);
        const int t = min(t0 + row, T - 1);
        xoff[j] = (uint32_t)t * (uint32_t)d * 2u + ((((lane & 7) ^ (row & 7) ^ ((row >> 3) & 1))) << 4);
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)smem;
    auto issue_x = [&](int kc) {
        const uint8_t* src = reinterpret_cast<const uint8_t*>(x) + (size_t)kc * (KS * 32);
        const uint32_t dst = lds0 + (kc & 1) * STAGE + wave * TS * 1024;
#pragma unroll
        for (int pn = 0; pn < PANELS; ++pn)
#pragma unroll
            for (int j = 0; j < TS; ++j)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                             :: "s"(dst + pn * RT * 128 + j * 1024), "v"(xoff[j]), "s"(src + pn * 128) : "memory");
    };
    const v4i* wsrc[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s)
        wsrc[s] = reinterpret_cast<const v4i*>(planes) + ((size_t)(wave * NS + s) * (d / 16) * 3) * 64 + lane;

    // accumulators live in the accumulation registers for the whole K loop; the matrix instructions are
    // volatile asm with a memory clobber, so they and the loads around them stay in source order
    v16f acc[NS][TS];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int ts = 0; ts < TS; ++ts)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[s][ts][r] = 0.f;

    // Weight operands run KS - 1 K steps ahead of the matrix cores in a ring of KS register sets
    // (a K step is 16 columns; a staged activation chunk holds KS of them, so the ring slot of a
    // step is its position inside the chunk).
    v4i a[KS][NS][3];
    auto load_a = [&](int slot, int kk) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int p = 0; p < 3; ++p) a[slot][s][p] = wsrc[s][((size_t)kk * 3 + p) * 64];
    };
    issue_x(kc_begin);
#pragma unroll
    for (int i = 0; i < AH; ++i) load_a(i, kc_begin * KS + i);   // a block has at least one chunk = KS > AH steps

    // activation operands of one K step: TS reads of 16 bytes per lane from the staged chunk
    auto read_b = [&](v4i (&b)[TS], const uint8_t* stage, int ks) {
#pragma unroll
        for (int ts = 0; ts < TS; ++ts) {
            const int row = ts * 32 + l32;
            b[ts] = *reinterpret_cast<const v4i*>(stage + (ks >> 2) * RT * 128 + row * 128 +
                                                  ((((ks & 3) * 2 + half) ^ (row & 7) ^ ((row >> 3) & 1)) << 4));
        }
    };
    v4i b[2][TS];                                              // step ks multiplies out of b[ks & 1] while b[(ks+1) & 1] loads
    for (int kc = kc_begin; kc < nchunks; ++kc) {
        // chunk kc must have landed.  Vector-memory operations complete in issue order: after the copies
        // of chunk kc this wave has issued exactly KS K steps of weight loads (L each), except
        // before the first chunk.
        if (kc == kc_begin) WAIT_VM(0); else WAIT_VM(KS * L);
        __syncthreads();                                       // landed for everybody; chunk kc-1 fully consumed
        if (kc + 1 < nchunks) issue_x(kc + 1);
        const uint8_t* stage = smem + (kc & 1) * STAGE;
        read_b(b[0], stage, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int kk = kc * KS + ks;
            if (kk + AH < nk) load_a((ks + AH) % KS, kk + AH);
            // the next step's activation operands (same chunk: the last step of a chunk has none to fetch, the
            // next chunk's first operands are read behind the barrier above)
            if (ks + 1 < KS) read_b(b[(ks + 1) & 1], stage, ks + 1);
            // The weight operands of this K step were requested AH steps ago; vector-memory operations
            // complete in issue order, so "at most as many outstanding as were issued since" means they
            // have arrived.  (Written out by hand: the steady-state loop gets no automatic wait for
            // values loaded in an earlier iteration and consumed by asm.)
            // Issued since: the weight groups of the next AH steps (in the last chunk step ks is followed
            // by KS - 1 - ks groups only) and, for every step of a chunk but the last, the C copies of the
            // next chunk that went out at this chunk's top: those may all stay in flight.
            if (kc + 1 < nchunks) {
                if (ks < KS - 1) WAIT_VM(AH * L + C);
                else WAIT_VM(AH * L);
            } else {
                WAIT_VM((KS - 1 - ks) * L);
            }
            // this step's activation operands were requested one step ago: all LDS reads but the TS just issued
            // must have returned (the compiler cannot see this through the asm below, so it is written out)
            if (ks + 1 < KS) asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(TS) : "memory");
            else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int ts = 0; ts < TS; ++ts)
                        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
                                     : "+a"(acc[s][ts]) : "v"(a[ks][s][p]), "v"(b[ks & 1][ts]) : "memory");
        }
    }
    // the last matrix instructions must have left the pipe before the accumulators are read
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __syncthreads();                                           // all reads of the activation stages are done

    if (SPLIT) {
        // partial[y][t][e], t over the padded token tiles, e over the padded experts: a lane owns four consecutive experts
        const int T_pad = gridDim.x * RT, E_pad = 128 * NS;
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int ts = 0; ts < TS; ++ts)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int e = (wave * NS + s) * 32 + r4 * 8 + half * 4;
                    const size_t at = ((size_t)blockIdx.y * T_pad + t0 + ts * 32 + l32) * E_pad + e;
                    *reinterpret_cast<float4*>(partial + at) = make_float4(acc[s][ts][r4 * 4], acc[s][ts][r4 * 4 + 1],
                                                                           acc[s][ts][r4 * 4 + 2], acc[s][ts][r4 * 4 + 3]);
                }
        return;
    }

    if (IDS) {
        // every lane looks up the logged ids of its TS tokens among the experts it holds
        float* sel = reinterpret_cast<float*>(smem);           // [RT][MAX_K] logits of the logged ids
        for (int i = tid; i < RT * MAX_K; i += 256) sel[i] = 0.f;   // ids outside [0,E) keep logit 0
        __syncthreads();
#pragma unroll
        for (int ts = 0; ts < TS; ++ts) {
            const int tok = ts * 32 + l32;
            if (t0 + tok >= T) continue;
            const int32_t* ids = logged_idx + (size_t)(t0 + tok) * k;
            for (int j = 0; j < k; ++j) {
                const int id = ids[j];
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int e = (wave * NS + s) * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                        if (e == id && e < E) sel[tok * MAX_K + j] = acc[s][ts][r];
                    }
            }
        }
        __syncthreads();
        if (tid < RT && t0 + tid < T) {
            // loops over MAX_K slots with a compile-time index (slots >= k are skipped), so that the selected logits
            // stay in registers: an array indexed by a run-time j would live in scratch memory
            const int32_t* ids = logged_idx + (size_t)(t0 + tid) * k;
            float lg[MAX_K];
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < MAX_K; ++j)
                if (j < k) { lg[j] = sel[tid * MAX_K + j]; m = fmaxf(m, lg[j]); }
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < MAX_K; ++j)
                if (j < k) { lg[j] = expf(lg[j] - m); sum += lg[j]; }
#pragma unroll
            for (int j = 0; j < MAX_K; ++j)
                if (j < k) {
                    topk_idx[(size_t)(t0 + tid) * k + j] = ids[j];
                    topk_w[(size_t)(t0 + tid) * k + j] = lg[j] / sum;
                }
        }
        return;
    }

    // ---- per-wave top-k.  Lane (l32, half) holds, for token ts*32+l32, the logits of experts
    //      wave*32*NS + s*32 + (r/4)*8 + half*4 + (r%4), position pos = s*16 + r (ascending in the expert index).
    //      Candidates: cand[token][wave][j] = {logit, idx}.
    //      The selection scores (logit + bias; -inf for padded experts) are copied to vector registers once - the
    //      weight ring's registers are free by now - and a taken score is overwritten with -inf, so that a round is
    //      one scan "strictly larger wins" (3 instructions per score: ties keep the lower index) and one marking pass
    //      (2 per score), which with a bias also picks the winner's unbiased logit out of the accumulators.
    float2* cand = reinterpret_cast<float2*>(smem);
    float sc[NS][TS][16];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int e = (wave * NS + s) * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            const float be = bias ? bias[min(e, E - 1)] : 0.f;
#pragma unroll
            for (int ts = 0; ts < TS; ++ts) sc[s][ts][r] = e < E ? acc[s][ts][r] + be : -INFINITY;
        }
    auto extract = [&](auto with_bias) {
        constexpr bool WB = decltype(with_bias)::value;
        for (int j = 0; j < k; ++j) {
#pragma unroll
            for (int ts = 0; ts < TS; ++ts) {
                float bs = -INFINITY;
                int bpos = -1;
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = sc[s][ts][r];
                        if (v > bs) { bs = v; bpos = s * 16 + r; }
                    }
                const int bi = bpos < 0 ? NO_CAND
                                        : (wave * NS + (bpos >> 4)) * 32 + ((bpos & 15) >> 2) * 8 + half * 4 + (bpos & 3);
                // the partner lane holds the other half of the wave's experts for the same token
                const float os = __shfl_xor(bs, 32);
                const int oi = __shfl_xor(bi, 32);
                const bool mine = bi != NO_CAND && (oi == NO_CAND || bs > os || (bs == os && bi < oi));
                const int mark = mine ? bpos : -1;
                float bl = bs;                                 // without a bias the score is the logit
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const bool hit = mark == s * 16 + r;
                        if (WB && hit) bl = acc[s][ts][r];
                        sc[s][ts][r] = hit ? -INFINITY : sc[s][ts][r];
                    }
                const float ol = __shfl_xor(bl, 32);
                if (half == 0) {
                    float2 c;
                    c.x = mine ? bl : ol;
                    c.y = __int_as_float(mine ? bi : oi);
                    cand[((ts * 32 + l32) * 4 + wave) * MAX_K + j] = c;
                }
            }
        }
    };
    if (bias) extract(std::true_type{}); else extract(std::false_type{});
    __syncthreads();

    // ---- merge the four waves' candidates, softmax, store: one thread per token.  Every wave's list is already in
    //      selection order (descending score, lower index first), so the merge only compares the four list heads.
    if (tid < RT && t0 + tid < T) {
        const float2* mine = cand + (size_t)tid * 4 * MAX_K;
        int head0 = 0, head1 = 0, head2 = 0, head3 = 0;
        // slots are walked with a compile-time index (those >= k are skipped): the selected logits and ids stay in
        // registers, where an array indexed by a run-time j would live in scratch memory
        float sel_logit[MAX_K];
        float m = -INFINITY;
#pragma unroll
        for (int j = 0; j < MAX_K; ++j) {
            if (j >= k) continue;
            float bs = 0.f, bl = 0.f;
            int bi = NO_CAND, bw = 0;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const int h = w == 0 ? head0 : w == 1 ? head1 : w == 2 ? head2 : head3;
                if (h >= k) continue;
                const float2 c = mine[w * MAX_K + h];
                const int e = __float_as_int(c.y);
                if (e == NO_CAND) continue;                    // this wave's experts are used up
                const float sc = c.x + (bias ? bias[e] : 0.f);
                if (bi == NO_CAND || sc > bs || (sc == bs && e < bi)) { bs = sc; bl = c.x; bi = e; bw = w; }
            }
            head0 += bw == 0; head1 += bw == 1; head2 += bw == 2; head3 += bw == 3;
            sel_logit[j] = bl;
            topk_idx[(size_t)(t0 + tid) * k + j] = bi;
            m = fmaxf(m, bl);
        }
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < MAX_K; ++j)
            if (j < k) { sel_logit[j] = expf(sel_logit[j] - m); sum += sel_logit[j]; }
#pragma unroll
        for (int j = 0; j < MAX_K; ++j)
            if (j < k) topk_w[(size_t)(t0 + tid) * k + j] = sel_logit[j] / sum;
    }
}

// Second half of the split router: one wave per token adds the partial logits up in split order, then
// selects as the single-pass kernel does (larger score, then lower expert index; softmax over the k selected
// unbiased logits, exponentials summed in slot order) or, with logged ids, picks their logits.  Lane l holds
// experts l, l+64, l+128, l+192.
template <bool IDS>
__global__ __launch_bounds__(256) void route_finish_kernel(const float* __restrict__ partial, int splits, int T_pad,
                                                           int E_pad, const float* __restrict__ bias,
                                                           const int32_t* __restrict__ logged_idx, int T, int E, int k,
                                                           int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;                                        // wave-uniform
    float lg[4], sc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = lane + 64 * i;
        // all partials are requested before the first is added (a loop of load-then-add would pay one memory round trip
        // per split); they are added in split order, absent splits as zeros
        float part[ROUTE_MAX_SPLITS];
#pragma unroll
        for (int sp = 0; sp < ROUTE_MAX_SPLITS; ++sp)
            part[sp] = (e < E_pad && sp < splits) ? partial[((size_t)sp * T_pad + t) * E_pad + e] : 0.f;
        float v = 0.f;
#pragma unroll
        for (int sp = 0; sp < ROUTE_MAX_SPLITS; ++sp) v += part[sp];
        lg[i] = v;
        sc[i] = e < E ? v + (bias ? bias[e] : 0.f) : -INFINITY;
    }
    float sel = 0.f;                                           // lane j < k: the j-th selected logit
    for (int j = 0; j < k; ++j) {
        int be;
        if (IDS) {
            be = logged_idx[(size_t)t * k + j];
        } else {
            float bs = -INFINITY;
            be = NO_CAND;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (sc[i] > bs) { bs = sc[i]; be = lane + 64 * i; }       // ascending index: ties keep the lower one
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float os = __shfl_xor(bs, off);
                const int oe = __shfl_xor(be, off);
                if (os > bs || (os == bs && oe < be)) { bs = os; be = oe; }
            }
        }
        const bool valid = be >= 0 && be < E;                  // wave-uniform (ids outside [0,E) keep logit 0)
        const int slot = valid ? be >> 6 : 0;
        const float mine = slot == 0 ? lg[0] : slot == 1 ? lg[1] : slot == 2 ? lg[2] : lg[3];
        const float chosen = valid ? __shfl(mine, be & 63) : 0.f;
        if (!IDS && valid && lane == (be & 63)) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (i == slot) sc[i] = -INFINITY;
        }
        if (lane == j) sel = chosen;
        if (lane == 0) topk_idx[(size_t)t * k + j] = be;
    }
    float m = -INFINITY;
    for (int j = 0; j < k; ++j) m = fmaxf(m, __shfl(sel, j));
    float sum = 0.f;
    for (int j = 0; j < k; ++j) sum += expf(__shfl(sel, j) - m);
    if (lane < k) topk_w[(size_t)t * k + lane] = expf(sel - m) / sum;
}

}  // namespace

size_t route_workspace_bytes(int E, int d) {
    const int E_pad = E <= 128 ? 128 : 256;
    return (size_t)3 * E_pad * d * sizeof(uint16_t);
}


static int route_splits_for(int T) {
    const int tiles = (T + 31) / 32;
    const int s = 256 / tiles;
    return s < 1 ? 1 : s > ROUTE_MAX_SPLITS ? ROUTE_MAX_SPLITS : s;
}

size_t route_partial_bytes(int T, int E) {
    if (T < 1 || T > ROUTE_SPLIT_MAX_T || route_splits_for(T) < 2) return 0;
    const int E_pad = E <= 128 ? 128 : 256;
    const size_t T_pad = (size_t)((T + 31) / 32) * 32;
    return (size_t)route_splits_for(T) * T_pad * E_pad * sizeof(float);
}

hipError_t launch_route(moe_ctx* c, const uint16_t* x, const float* W_r, const float* bias,
                        const int32_t* logged_idx, int32_t* topk_idx, float* topk_w) {
    const moe_dims& D = c->dims;
    if (D.T == 0) return hipSuccess;
    const int E_pad = D.E <= 128 ? 128 : 256;
    const int64_t nthreads = (int64_t)E_pad * (D.d / 8);
    hipLaunchKernelGGL(split_router_weights, dim3((unsigned)((nthreads + 255) / 256)), dim3(256), 0, c->stream,
                       W_r, D.E, E_pad, D.d, c->router_planes);
    const int nchunks = D.d / 128;
    if (D.T <= ROUTE_SPLIT_MAX_T && c->route_partial && nchunks >= 2) {
        // small batch: 32-token tiles, the K loop of each split over enough blocks to occupy the chip
        const int tiles = (D.T + 31) / 32;
        int splits = route_splits_for(D.T);
        const int cps = (nchunks + splits - 1) / splits;       // chunks per block
        splits = (nchunks + cps - 1) / cps;                    // no empty block
        if (splits >= 2) {
            const dim3 grid(tiles, splits);
#define MOE_ROUTE_SPLIT(NS_)                                                                                       \
    hipLaunchKernelGGL((route_mfma_kernel<NS_, 1, 8, false, true>), grid, dim3(256), 0, c->stream, x, c->router_planes, \
                       bias, logged_idx, D.T, D.d, D.E, D.k, topk_idx, topk_w, c->route_partial, cps)
            if (E_pad == 128) MOE_ROUTE_SPLIT(1); else MOE_ROUTE_SPLIT(2);
#undef MOE_ROUTE_SPLIT
            const dim3 fgrid((D.T + 3) / 4);
            if (logged_idx)
                hipLaunchKernelGGL(route_finish_kernel<true>, fgrid, dim3(256), 0, c->stream, c->route_partial, splits,
                                   tiles * 32, E_pad, (const float*)nullptr, logged_idx, D.T, D.E, D.k, topk_idx, topk_w);
            else
                hipLaunchKernelGGL(route_finish_kernel<false>, fgrid, dim3(256), 0, c->stream, c->route_partial, splits,
                                   tiles * 32, E_pad, bias, logged_idx, D.T, D.E, D.k, topk_idx, topk_w);
            return hipGetLastError();
        }
    }
    // token tile: the largest of 128 / 64 / 32 rows that still gives every compute unit a block
    const int TS = D.T >= 256 * 128 ? 4 : D.T >= 256 * 64 ? 2 : 1;
    const int grid = (D.T + 32 * TS - 1) / (32 * TS);
#define MOE_ROUTE_LAUNCH(NS_, TS_, IDS_)                                                                    \
    hipLaunchKernelGGL((route_mfma_kernel<NS_, TS_, 8, IDS_>), dim3(grid), dim3(256), 0, c->stream, x,         \
                       c->router_planes, bias, logged_idx, D.T, D.d, D.E, D.k, topk_idx, topk_w, (float*)nullptr, 0)
#define MOE_ROUTE_TS(NS_, IDS_)                                                                             \
    do {                                                                                                    \
        if (TS == 4) MOE_ROUTE_LAUNCH(NS_, 4, IDS_);                                                        \
        else if (TS == 2) MOE_ROUTE_LAUNCH(NS_, 2, IDS_);                                                   \
        else MOE_ROUTE_LAUNCH(NS_, 1, IDS_);                                                                \
    } while (0)
    if (E_pad == 128) {
        if (logged_idx) MOE_ROUTE_TS(1, true); else MOE_ROUTE_TS(1, false);
    } else {
        if (logged_idx) MOE_ROUTE_TS(2, true); else MOE_ROUTE_TS(2, false);
    }
#undef MOE_ROUTE_TS
#undef MOE_ROUTE_LAUNCH
    return hipGetLastError();
}

}  // namespace moe355
