// Grouped block-scaled FP8 SwiGLU expert FFN on the CDNA4 matrix cores.
//
// Work unit: a tile of up to TOK_TILE (256) expert-sorted rows x 256 staged weight rows.  A
// small kernel turns offsets[] into the list of work units (expert, first row, feature tile,
// rows), so ragged experts need no host round trip, and orders it so that units sharing a
// weight tile are adjacent; blocks map onto the list so that each XCD (blockIdx % 8) walks a
// contiguous range and its L2 sees every weight tile once.
//
// Main loop, one iteration per 128-wide K block (= one scale block):
//   * both operand tiles are copied global -> LDS by direct-to-LDS loads (no staging
//     registers) into rings of three (weights) and two (activations) 32 KiB buffers, 16-byte
//     chunks XOR-swizzled by row so that the 32-row operand reads spread over all 64 banks;
//   * partial = W_tile * X_tile^T with two v_mfma_f32_32x32x64_f8f6f4 per 32x32 sub-tile;
//   * acc += (xs[kb][row] * ws[feature block,kb]) * partial in fp32.
// The product is taken as (features x tokens): in the 32x32 accumulator layout a lane then
// owns ONE token column and 16 feature rows, so the activation scale is one scalar per lane
// and sub-tile, and the 128-wide amax of the epilogue is a lane-local reduction plus one
// cross-half shuffle and one exchange between the two waves that share a token.
// Activation scales are K-block major ([K/128][rows]): the 32 lanes of a half-wave read 32
// consecutive floats of one plane.
//
// Eight waves per block: wave (wt, wf) owns 64 tokens x 128 staged weight rows (2 x 4
// sub-tiles): 6 operand sub-tiles feed 8 MFMA pairs.  Waves whose 64 tokens lie beyond the
// expert's last row skip their MFMAs, so a ragged tail costs a fraction of a tile.
//
// GEMM1: staged rows of wave wf are [64 gate rows | 64 up rows] of the same features;
//        epilogue h = silu(g)*u, re-quantised to e4m3 with one scale per (row, 128 features).
// GEMM2: staged rows are 256 consecutive output features; epilogue: fp32 rows, turned through LDS so
//        that every row is stored in contiguous 256-byte pieces.
#include "moe_internal.hpp"

namespace moe355 {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int KB = QBLOCK;                        // K bytes per stage (= one scale block)
constexpr int W_ROWS = 256;                       // staged weight rows per block
constexpr int X_ROWS = TOK_TILE;                  // staged activation rows per block (256)
constexpr int W_TILE = W_ROWS * KB;                // 32 KiB: one K block of the weight tile
constexpr int X_TILE = X_ROWS * KB;                // 32 KiB: one K block of the activation tile
constexpr int NW_BUF = 3, NX_BUF = 2;              // LDS ring depths
constexpr int X_RING = NW_BUF * W_TILE;            // byte offset of the activation ring
constexpr int NTHREADS = 512;
constexpr int NXCD = 8;
constexpr int NARROW_ROWS = 64;                     // tiles of at most this many rows take the narrow path of ffn_gemm

struct Work { int32_t expert; int32_t row0; int32_t ft; int32_t nrows; };

// ------------------------------------------------------------------ work list
// An expert with c rows gets ceil(c/256) row tiles, ordered (expert, feature tile, row tile).  Units
// that share a weight tile are thus neighbours and, when they do the same amount of work, the blocks
// that run them side by side on one XCD advance in step and hit each other's lines in that XCD's L2
// (a few K steps of skew already exceed what the L2 retains, and the shared tile is then fetched
// again from HBM).
// Block (e, l) writes the units of expert e into list l (0: gate/up, n_ft0 feature tiles; 1: down,
// n_ft1 feature tiles); every block recomputes the tile counts of all experts for its base index.
__global__ __launch_bounds__(256) void build_work(const int32_t* __restrict__ offsets, int E, int n_ft0, int n_ft1,
                                                  Work* __restrict__ work0, Work* __restrict__ work1,
                                                  int32_t* __restrict__ n_work) {
    __shared__ int32_t s_tiles[MAX_E];
    const int tid = threadIdx.x;
    const int e = blockIdx.x;
    const int n_ft = blockIdx.y == 0 ? n_ft0 : n_ft1;
    Work* const work = blockIdx.y == 0 ? work0 : work1;
    int nt_t = 0;
    if (tid < E) nt_t = (offsets[tid + 1] - offsets[tid] + TOK_TILE - 1) / TOK_TILE;
    s_tiles[tid] = nt_t;
    __syncthreads();
    for (int off = 1; off < MAX_E; off <<= 1) {            // inclusive scan
        const int a = (tid >= off) ? s_tiles[tid - off] : 0;
        __syncthreads();
        s_tiles[tid] += a;
        __syncthreads();
    }
    if (e == 0 && tid == 0) n_work[blockIdx.y] = s_tiles[MAX_E - 1] * n_ft;
    if (e >= E) return;
    const int start = offsets[e], cnt = offsets[e + 1] - start;
    const int nt = (cnt + TOK_TILE - 1) / TOK_TILE;
    if (nt == 0) return;
    const int base = (s_tiles[e] - nt) * n_ft;
    for (int idx = tid; idx < nt * n_ft; idx += 256) {
        const int f = idx / nt, i = idx - f * nt;
        // Down projection: experts with three or more tiles whose remainder is at most 128 rows get full tiles
        // plus one short tile: a short tile keeps half of the block's waves out of the matrix work and,
        // measured, costs 0.7 to 0.9 of a full one, less than making every tile of the expert ragged.
        // Otherwise, and always in the gate/up projection, the expert's G = ceil(cnt/64) groups of 64 rows (the
        // share of one wave pair) are dealt out evenly: tile i covers groups [i*G/nt, (i+1)*G/nt).  The tiles
        // that share a weight tile then advance in step and fetch it once, and only the expert's last group is partly
        // filled: splitting the ROWS evenly instead leaves a partly filled group in every tile, whose wave pair does a
        // full group's matrix work (3 % of the gate/up projection at 896..1152 rows per expert: the kernel runs at
        // the power cap, so matrix work that is thrown away costs time even where it hides behind other waves).
        // A tile that runs faster than the tiles it shares a weight tile with does not pay: it runs ahead and the
        // weight tile is fetched twice.  Measured for a remainder of at most 64 rows cut off as a NARROW tile (a fifth
        // of a full tile's time by itself): gate/up projection 8 % slower at 248..264 rows per expert, 3 % slower at
        // 896..1152.  Narrow tiles therefore arise only where an expert has at most 64 rows altogether.
        const bool short_tail = blockIdx.y == 1 && nt >= 3 && cnt - (nt - 1) * TOK_TILE <= TOK_TILE / 2;
        const int G = (cnt + 63) / 64;
        const int lo = short_tail ? i * TOK_TILE : min(cnt, 64 * (int)((int64_t)i * G / nt));
        const int hi = short_tail ? min(cnt, lo + TOK_TILE) : min(cnt, 64 * (int)((int64_t)(i + 1) * G / nt));
        Work w;
        w.expert = e;
        w.row0 = start + lo;
        w.ft = f;
        w.nrows = hi - lo;
        work[base + idx] = w;
    }
}

// ------------------------------------------------------------------ helpers
// Direct global -> LDS copies.  Lane i of the wave deposits its bytes at lds_addr + i*size;
// the global address is sbase + voff (per lane).  Completion is tracked by vmcnt; the
// compiler does not see these as memory operations of its own, so every wait on them is
// written out explicitly below.
__device__ inline void dma16(uint32_t lds_addr, uint32_t voff, const void* sbase) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}

// The matrix instructions are written as volatile asm so that they stay exactly where the
// source puts them: the schedule below relies on it.  T = A*B (first K half) and T += A*B.
__device__ inline void mfma_first(v16f& t, const v8i& a, const v8i& b) {
    asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, 0" : "=&v"(t) : "v"(a), "v"(b) : "memory");
}
__device__ inline void mfma_acc(v16f& t, const v8i& a, const v8i& b) {
    asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0" : "+v"(t) : "v"(a), "v"(b) : "memory");
}
// An empty volatile asm that "rewrites" x: uses of x after it cannot move above it, and
// values feeding x cannot move below it.
#define PIN(x) asm volatile("" : "+v"(x))

// the 32 K-bytes a lane feeds to one 32x32x64 MFMA, from a row's two swizzled 16-byte chunks
__device__ inline v8i lds_operand(const uint8_t* row, uint32_t o0, uint32_t o1) {
    const uint4 lo = *reinterpret_cast<const uint4*>(row + o0);
    const uint4 hi = *reinterpret_cast<const uint4*>(row + o1);
    v8i r;
    r[0] = lo.x; r[1] = lo.y; r[2] = lo.z; r[3] = lo.w;
    r[4] = hi.x; r[5] = hi.y; r[6] = hi.z; r[7] = hi.w;
    return r;
}

// ------------------------------------------------------------------ GEMM kernel
// GATED = true : Wa = W1, Wb = W3 [E, NOUT, K]; feature tile = 128 features (gate + up rows)
// GATED = false: Wa = W2 [E, NOUT, K]; feature tile = 256 output features
// act [N, K] u8 are the expert-sorted activations; act_s [K/128][N] f32 their scales, K-block major.
// GATHER (gate/up only): act [n_tok, K] is in TOKEN order and sorted row p reads the codes of token
// perm[p] / fan (clamped to the last token, so that a foreign perm cannot address outside act): the
// expert-ordered copy of the codes is never materialised.  The scales act_s
// [K/128][n_rows] are in sorted order in both cases (they are 1/128 of the data; a lane-scattered
// scale read per K step would cost more than it saves).
template <bool GATED, bool GATHER>
__global__ __launch_bounds__(NTHREADS, 1) void ffn_gemm(const uint8_t* __restrict__ act,
                                                        const float* __restrict__ act_s, int n_rows,
                                                        const int32_t* __restrict__ perm, int fan, int n_tok,
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
    // [3][256 weight rows][128 B] then [2][256 activation rows][128 B]: all 160 KiB.  The amax
    // exchange of the epilogue reuses the first bytes once the main loop is over.
    float* const s_amax = reinterpret_cast<float*>(smem);

    // ---- which work unit: XCD x (= blockIdx % 8) walks the contiguous range [x*chunk, (x+1)*chunk)
    const int total = *n_work;
    const int chunk = (total + NXCD - 1) / NXCD;
    const int slot = blockIdx.x / NXCD;
    const int wi = (blockIdx.x % NXCD) * chunk + slot;
    if (slot >= chunk || wi >= total) return;
    const Work wk = work[wi];
    const int e = wk.expert;
    const int row_end = wk.row0 + wk.nrows;                    // this tile's rows only
    const int f0 = wk.ft * FT;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wt = wave >> 1, wf = wave & 1;                   // token group (64 rows), weight-row half
    const int nkb = K / KB;
    const int nblk_out = NOUT / QBLOCK;

    // ---- copy plan: wave w brings staged weight rows [32w, 32w+32) and staged activation rows
    //      [32w, 32w+32) of every K block, 4 + 4 instructions of 8 rows each; lane i -> row i/8,
    //      LDS chunk slot i%8 which receives global chunk slot ^ (row & 7) ^ ((row >> 3) & 1): with that
    //      swizzle the 32-row x 16-byte operand reads below touch all 64 LDS banks evenly.
    //      Staged weight row r: GATED: features f0 + (r/128)*64 + r%64, gate (Wa) if (r/64)%2 == 0 else up (Wb).
    //      NARROW tiles (at most 64 rows, see below): wave w's 32 staged rows are 32 consecutive features of the tile
    //      (down projection) or, GATED, [16 gate rows | 16 up rows] of features f0 + 16w .. 16w+15.
    const bool narrow = wk.nrows <= NARROW_ROWS;               // block-uniform
    const uint8_t* w_base[2];                                  // wave-uniform: matrix of copy instructions 0,1 and 2,3
    uint32_t w_off[4], x_off[4];
    {
        const int sub = lane >> 3, cslot = lane & 7;
        const size_t we = (size_t)e * NOUT * (size_t)K;
        if (GATED && narrow) {
            w_base[0] = Wa + we;
            w_base[1] = Wb + we;
        } else {
            w_base[0] = w_base[1] = ((GATED && ((wave >> 1) & 1)) ? Wb : Wa) + we;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = wave * 32 + j * 8 + sub;
            int f = GATED ? (narrow ? f0 + wave * 16 + ((j * 8 + sub) & 15) : f0 + (r >> 7) * 64 + (r & 63)) : f0 + r;
            f = min(f, NOUT - 1);
            w_off[j] = (uint32_t)f * (uint32_t)K + ((cslot ^ (r & 7) ^ ((r >> 3) & 1)) << 4);
            const int p = min(wk.row0 + r, row_end - 1);      // rows past the tile repeat its last row
            const int src = GATHER ? (int)min((uint32_t)perm[p] / (uint32_t)fan, (uint32_t)(n_tok - 1)) : p - wk.row0;
            x_off[j] = (uint32_t)src * (uint32_t)K + ((cslot ^ (r & 7) ^ ((r >> 3) & 1)) << 4);
        }
    }
    const uint8_t* x_base = GATHER ? act : act + (size_t)wk.row0 * K;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)smem;
    const uint32_t lds_rows = lds0 + wave * 32 * KB;           // this wave's rows inside a tile buffer

    auto issue_w = [&](int kb, int wslot) {
        const uint32_t dst = lds_rows + wslot * W_TILE;
#pragma unroll
        for (int j = 0; j < 4; ++j) dma16(dst + j * 8 * KB, w_off[j], w_base[j >> 1] + (size_t)kb * KB);
    };
    auto issue_w1 = [&](int kb, int wslot, int j) {
        const uint32_t dst = lds_rows + wslot * W_TILE;
        dma16(dst + j * 8 * KB, w_off[j], w_base[j >> 1] + (size_t)kb * KB);
    };
    // 8-row activation copies that lie wholly beyond the expert's last row are not issued at all
    // (a ragged last tile then moves only the rows it has); wave-uniform
    const int x_copies = __builtin_amdgcn_readfirstlane(max(0, min(4, (row_end - wk.row0 - wave * 32 + 7) / 8)));
    // the skip is a scalar branch inside the asm: the compiler's control flow stays a straight line
#define X_COPY(KBLK, XSLOT, J)                                                                                  \
    asm volatile("s_cmp_gt_i32 %3, %4\n\ts_cbranch_scc0 .Lskipx%=\n\ts_mov_b32 m0, %0\n\ts_nop 0\n\t"           \
                 "global_load_lds_dwordx4 %1, %2\n.Lskipx%=:"                                                   \
                 :: "s"(lds_rows + X_RING + (XSLOT) * X_TILE + (J) * 8 * KB), "v"(x_off[J]),                    \
                    "s"(x_base + (size_t)(KBLK) * KB), "s"(x_copies), "n"(J) : "memory", "scc")
    auto issue_x = [&](int kb, int xslot) {
        X_COPY(kb, xslot, 0);
        X_COPY(kb, xslot, 1);
        X_COPY(kb, xslot, 2);
        X_COPY(kb, xslot, 3);
    };

    // ---- weight scales of this wave's rows (wave-uniform -> scalar loads)
    const int blk_a = GATED ? wk.ft : min(wk.ft * 2 + (narrow ? wave >> 2 : wf), nblk_out - 1);
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

    // Pipeline.  K block kb of the weight tile lives in ring slot kb % 3, of the activation tile in
    // slot kb % 2.  Each wave passes ONE barrier per K block, placed after its last LDS read of block
    // kb (before sub-tile product 6 of 8).  Behind that barrier block kb+1 is complete in LDS and the
    // slots of block kb are free.  The copies that refill them follow: activation block kb+2, then
    // weight block kb+3 - always in that order, so that "all but the newest four copies have landed" is
    // exactly "everything but the weight block two steps ahead".  They go out one behind each matrix
    // instruction (activations over products 6 and 7, weights over products 0 and 1 of the next step),
    // so that the wave does not sit at the issue of a copy while the queue drains (in two bursts of four
    // the gate/up projection ran 4 % slower).  Products 6 and 7 already fetch the first operands of
    // block kb+1 into registers.
    issue_x(0, 0);
    issue_w(0, 0);
    if (narrow) {
        // ---- NARROW tile: at most 64 rows.  In the layout above only the two waves of token group 0 would
        //      multiply, alone on their SIMDs, and such a tile costs 0.7 of a full one.  Here all eight waves work:
        //      wave w multiplies the 32 staged weight rows it copies itself by the tile's 64 token columns (two
        //      32x32 products, four matrix instructions per K block), so the matrix work is spread over every SIMD
        //      and the tile runs at the speed its weight tile streams in.  Same rings, same copy order, same
        //      barrier per K block as the full tiles; nothing is overlapped by hand - the copies are the bound.
        uint32_t offk[2][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                offk[ks][j] = (uint32_t)(((ks * 4 + half * 2 + j) ^ (l32 & 7) ^ ((l32 >> 3) & 1)) << 4);
        const uint32_t a_row = (uint32_t)(wave * 32 + l32) * KB;
        const uint32_t b_row = (uint32_t)(X_RING + l32 * KB);
        uint32_t xs_i[2];
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) xs_i[ts] = 4u * (uint32_t)min(wk.row0 + ts * 32 + l32, n_rows - 1);
        const size_t plane = (size_t)n_rows * 4;
        auto xs_load = [&](float& dst, int kb, int ts) {
            asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(xs_i[ts]),
                         "s"(reinterpret_cast<const uint8_t*>(act_s) + (size_t)kb * plane) : "memory");
        };
        float xs_n[2], xs_cur[2];
        xs_load(xs_n[0], 0, 0);
        xs_load(xs_n[1], 0, 1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) asm volatile("v_mov_b32 %0, %1" : "=v"(xs_cur[ts]) : "v"(xs_n[ts]));
        if (nkb > 1) {
            xs_load(xs_n[0], 1, 0);
            xs_load(xs_n[1], 1, 1);
            issue_x(1, 1);
            issue_w(1, 1);
        }
        if (nkb > 2) issue_w(2, 2);
        v16f an[2];
#pragma unroll
        for (int ts = 0; ts < 2; ++ts)
#pragma unroll
            for (int r = 0; r < 16; ++r) an[ts][r] = 0.f;
        int wslot = 0;
        for (int kb = 0; kb < nkb; ++kb) {
            const uint8_t* sW = smem + wslot * W_TILE + a_row;
            const uint8_t* sX = smem + b_row + (kb & 1) * X_TILE;
            v8i a[2], b[2][2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                a[ks] = lds_operand(sW, offk[ks][0], offk[ks][1]);
                b[0][ks] = lds_operand(sX, offk[ks][0], offk[ks][1]);
                b[1][ks] = lds_operand(sX + 32 * KB, offk[ks][0], offk[ks][1]);
            }
            const float wsa = sa_e[kb], wsb = sb_e[kb];
            v16f T0, T1;
            mfma_first(T0, a[0], b[0][0]);
            mfma_acc(T0, a[1], b[0][1]);
            mfma_first(T1, a[0], b[1][0]);
            mfma_acc(T1, a[1], b[1][1]);
            // this wave's reads of block kb are done (the operands are in registers): wait for the copies that must be
            // complete (all but the weight block two steps ahead), meet the other waves, refill the freed slots
            if (kb + 2 < nkb) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const float x0 = xs_cur[0], x1 = xs_cur[1];
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) asm volatile("v_mov_b32 %0, %1" : "=v"(xs_cur[ts]) : "v"(xs_n[ts]));
            if (kb + 2 < nkb) {
                xs_load(xs_n[0], kb + 2, 0);
                xs_load(xs_n[1], kb + 2, 1);
                issue_x(kb + 2, kb & 1);
            }
            if (kb + 3 < nkb) issue_w(kb + 3, wslot);
            // the four matrix instructions have left the pipe by now; a few wait states more cost nothing here
            asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
            PIN(T0);
            PIN(T1);
            // accumulator rows 0..15 of the product (registers 0..7) are gate rows, 16..31 (registers 8..15) up rows
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float w = (GATED && r >= 8) ? wsb : wsa;
                an[0][r] = fmaf(x0 * w, T0[r], an[0][r]);
                an[1][r] = fmaf(x1 * w, T1[r], an[1][r]);
            }
            PIN(an[0]);
            PIN(an[1]);
            wslot = (wslot == NW_BUF - 1) ? 0 : wslot + 1;
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();                          // every wave is done with the operand rings
        asm volatile("" ::: "memory");
        // ---- narrow epilogue.  Register r of an[ts] belongs to token row0 + ts*32 + l32 and staged row
        //      32w + (r/4)*8 + half*4 + r%4 of this wave.
        if (GATED) {
            // registers 0..7: gate of features f0 + 16w + (r/4)*8 + half*4 + r%4, registers 8..15: up of the same
            float h[2][8];
            float amax[2] = {0.f, 0.f};
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const float g = an[ts][r], u = an[ts][r + 8];
                    const float v = g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
                    h[ts][r] = v;
                    amax[ts] = fmaxf(amax[ts], fabsf(v));
                }
                amax[ts] = fmaxf(amax[ts], __shfl_xor(amax[ts], 32));
                if (half == 0) s_amax[wave * 64 + ts * 32 + l32] = amax[ts];
            }
            __syncthreads();                                   // the 128 features of a token's group live in all 8 waves
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                const int trow = ts * 32 + l32;
                const int p = wk.row0 + trow;
                float am = 0.f;
#pragma unroll
                for (int w = 0; w < 8; ++w) am = fmaxf(am, s_amax[w * 64 + trow]);
                const float sc = (am == 0.f) ? 1.0f : am / 448.0f;
                // the same correctly rounded quotient as in the full tiles' epilogue
                float inv = __builtin_amdgcn_rcpf(sc);
                inv = fmaf(fmaf(-sc, inv, 1.0f), inv, inv);
                const bool mid_range = sc > 1e-30f && sc < 1e30f;
                auto quot = [&](float hv) {
                    const float q0 = hv * inv;
                    return mid_range ? fmaf(fmaf(-q0, sc, hv), inv, q0) : hv / sc;
                };
                if (p < row_end) {
                    uint8_t* dst = hq + (size_t)p * NOUT + f0 + wave * 16 + half * 4;
#pragma unroll
                    for (int r4 = 0; r4 < 2; ++r4) {
                        int code = 0;
                        code = __builtin_amdgcn_cvt_pk_fp8_f32(quot(h[ts][r4 * 4]), quot(h[ts][r4 * 4 + 1]), code, false);
                        code = __builtin_amdgcn_cvt_pk_fp8_f32(quot(h[ts][r4 * 4 + 2]), quot(h[ts][r4 * 4 + 3]), code, true);
                        *reinterpret_cast<uint32_t*>(dst + r4 * 8) = (uint32_t)code;
                    }
                    if (half == 0 && wave == 0) hs[(size_t)wk.ft * n_rows + p] = sc;
                }
            }
        } else {
            // 64 rows x 256 features: 16-byte pieces straight from the accumulator layout (a narrow tile's output is small)
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                const int p = wk.row0 + ts * 32 + l32;
                if (p >= row_end) continue;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int fcol = f0 + wave * 32 + r4 * 8 + half * 4;
                    if (fcol < NOUT)
                        *reinterpret_cast<float4*>(y_perm + (size_t)p * NOUT + fcol) =
                            make_float4(an[ts][r4 * 4], an[ts][r4 * 4 + 1], an[ts][r4 * 4 + 2], an[ts][r4 * 4 + 3]);
                }
            }
        }
        return;
    }
    if (!wave_active) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (nkb > 1) { issue_x(1, 1); issue_w(1, 1); }
        if (nkb > 2) issue_w(2, 2);
        int wslot = 0;
        for (int kb = 0; kb < nkb; ++kb) {
            if (kb + 2 < nkb) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (kb + 2 < nkb) issue_x(kb + 2, kb & 1);
            if (kb + 3 < nkb) issue_w(kb + 3, wslot);
            wslot = (wslot == NW_BUF - 1) ? 0 : wslot + 1;
        }
    } else {
        // per-lane constants of the operand reads
        uint32_t offk[2][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                offk[ks][j] = (uint32_t)(((ks * 4 + half * 2 + j) ^ (l32 & 7) ^ ((l32 >> 3) & 1)) << 4);
        const uint32_t a_row = (uint32_t)(wf * 128 + l32) * KB;
        const uint32_t b_row = (uint32_t)(X_RING + (wt * 64 + l32) * KB);
        // activation scales of this lane's two token columns (K-block major: one plane per K block)
        uint32_t xs_i[2];                                      // byte offset of the lane's row inside a plane
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) xs_i[ts] = 4u * (uint32_t)min(wk.row0 + wt * 64 + ts * 32 + l32, n_rows - 1);
        const size_t plane = (size_t)n_rows * 4;
        // issued as asm (saddr + 32-bit lane offset); the data is only touched behind a vmcnt wait
        auto xs_load = [&](float& dst, int kb, int ts) {
            asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(xs_i[ts]),
                         "s"(reinterpret_cast<const uint8_t*>(act_s) + (size_t)kb * plane) : "memory");
        };
        float xs_n[2];
        xs_load(xs_n[0], 0, 0);
        xs_load(xs_n[1], 0, 1);
        float xs_cur[2];

        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) asm volatile("v_mov_b32 %0, %1" : "=v"(xs_cur[ts]) : "v"(xs_n[ts]));
        if (nkb > 1) {
            xs_load(xs_n[0], 1, 0);
            xs_load(xs_n[1], 1, 1);
            issue_x(1, 1);
            issue_w(1, 1);
        }
        if (nkb > 2) issue_w(2, 2);
        v8i b[2][2], a[2][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) a[0][ks] = lds_operand(smem + a_row, offk[ks][0], offk[ks][1]);
#pragma unroll
        for (int ts = 0; ts < 2; ++ts)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                b[ts][ks] = lds_operand(smem + b_row + ts * 32 * KB, offk[ks][0], offk[ks][1]);
        float sc[2][2];
        {
            const float wsa = sa_e[0], wsb = sb_e[0];
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                sc[ts][0] = xs_cur[ts] * wsa;
                sc[ts][1] = xs_cur[ts] * wsb;
            }
        }
        v16f T0, T1;
#pragma unroll
        for (int r = 0; r < 16; ++r) { T0[r] = 0.f; T1[r] = 0.f; }
        float sc_pend = 0.f;                                   // scale of the sub-tile product still held in T1

        // fold product `PS, PTS` (held in T0 for PTS == 0, T1 for PTS == 1) into its accumulator
#define FOLD(PS, PTS, SCV)                                                                      \
        do {                                                                                    \
            if ((PTS) == 0) {                                                                   \
                PIN(T0);                                                                        \
                _Pragma("unroll") for (int r = 0; r < 16; ++r)                                  \
                    acc[PS][0][r] = fmaf((SCV), T0[r], acc[PS][0][r]);                          \
            } else {                                                                            \
                PIN(T1);                                                                        \
                _Pragma("unroll") for (int r = 0; r < 16; ++r)                                  \
                    acc[PS][1][r] = fmaf((SCV), T1[r], acc[PS][1][r]);                          \
            }                                                                                   \
            PIN(acc[PS][PTS]);                                                                  \
        } while (0)

        int wslot = 0;                                         // ring slot of weight block kb
        for (int kb = 0; kb < nkb; ++kb) {
            const int wnext = (wslot == NW_BUF - 1) ? 0 : wslot + 1;
            const int wprev = (wslot == 0) ? NW_BUF - 1 : wslot - 1;             // slot of block kb-1 = of block kb+2
            const uint8_t* sW = smem + wslot * W_TILE + a_row;                   // block kb
            const uint8_t* sWn = smem + wnext * W_TILE + a_row;                  // block kb+1
            const uint8_t* sXn = smem + b_row + ((kb & 1) ^ 1) * X_TILE;         // block kb+1
            const int kn = min(kb + 1, nkb - 1);
            const float wsa_n = sa_e[kn], wsb_n = sb_e[kn];            // consumed at the end of this step
            // Eight sub-tile products, two MFMAs each.  The 16 scale-FMAs of product i-1 sit behind the
            // second MFMA of product i: by then its result has left the matrix pipe (two more MFMAs
            // have been issued since), and the vector ALU works in the shadow of the MFMA just issued.
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int s = i >> 1, ts = i & 1;
                if (i == 6) {
                    // all of this wave's reads of block kb have been issued; wait for them and for the
                    // copies that must be complete, then meet the other waves
                    if (kb + 2 < nkb) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
                    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2) asm volatile("v_mov_b32 %0, %1" : "=v"(xs_cur[t2]) : "v"(xs_n[t2]));
                }
                if (ts == 0) mfma_first(T0, a[s & 1][0], b[0][0]); else mfma_first(T1, a[s & 1][0], b[1][0]);
                // one copy behind every matrix instruction: weight block kb+2 over products 0 and 1
                if (i < 2 && kb >= 1 && kb + 2 < nkb) issue_w1(kb + 2, wprev, i * 2);
                if (i == 7 && kb + 2 < nkb) X_COPY(kb + 2, kb & 1, 2);
                if (ts == 0 && s < 3) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
                        a[(s + 1) & 1][ks] = lds_operand(sW + (s + 1) * 32 * KB, offk[ks][0], offk[ks][1]);
                }
                if (i == 6) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) a[0][ks] = lds_operand(sWn, offk[ks][0], offk[ks][1]);
                    if (kb + 2 < nkb) {
                        xs_load(xs_n[0], kb + 2, 0);
                        xs_load(xs_n[1], kb + 2, 1);
                        X_COPY(kb + 2, kb & 1, 0);
                    }
                }
                if (ts == 0) mfma_acc(T0, a[s & 1][1], b[0][1]); else mfma_acc(T1, a[s & 1][1], b[1][1]);
                if (i < 2 && kb >= 1 && kb + 2 < nkb) issue_w1(kb + 2, wprev, i * 2 + 1);
                if (i == 6 && kb + 2 < nkb) X_COPY(kb + 2, kb & 1, 1);
                if (i == 7 && kb + 2 < nkb) X_COPY(kb + 2, kb & 1, 3);
                if (i == 0) {
                    FOLD(3, 1, sc_pend);
                } else {
                    const int ps = (i - 1) >> 1, pts = (i - 1) & 1;
                    FOLD(ps, pts, sc[pts][(GATED && ps >= 2) ? 1 : 0]);
                }
                if (i == 6) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) b[0][ks] = lds_operand(sXn, offk[ks][0], offk[ks][1]);
                }
                if (i == 7) {
                    sc_pend = sc[1][GATED ? 1 : 0];
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2) {
                        sc[t2][0] = xs_cur[t2] * wsa_n;
                        sc[t2][1] = xs_cur[t2] * wsb_n;
                    }
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) b[1][ks] = lds_operand(sXn + 32 * KB, offk[ks][0], offk[ks][1]);
                }
            }
            wslot = wnext;
        }
        // the last product: wait out the matrix pipe, then fold it
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
        FOLD(3, 1, sc_pend);
#undef FOLD
#undef X_COPY
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                              // every wave is done with the operand rings
    asm volatile("" ::: "memory");

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
                        // silu(g)*u with the hardware reciprocal (1 ulp): far below the matrix cores' own error
                        const float v = g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
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
                // h / sc, correctly rounded, for 32 values per token: a reciprocal refined once, then the
                // quotient estimate corrected by its exact remainder (three instructions instead of a full
                // division each; equal to the division wherever sc is far from the ends of the fp32 range,
                // and the plain division elsewhere).  |h / sc| <= 448 up to one rounding, so no clamp.
                float inv = __builtin_amdgcn_rcpf(sc);
                inv = fmaf(fmaf(-sc, inv, 1.0f), inv, inv);
                const bool mid_range = sc > 1e-30f && sc < 1e30f;
                auto quot = [&](float hv) {
                    const float q0 = hv * inv;
                    return mid_range ? fmaf(fmaf(-q0, sc, hv), inv, q0) : hv / sc;
                };
                if (p < row_end) {
                    uint8_t* dst = hq + (size_t)p * NOUT + f0 + wf * 64 + half * 4;
#pragma unroll
                    for (int s = 0; s < 2; ++s)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            int code = 0;
                            code = __builtin_amdgcn_cvt_pk_fp8_f32(quot(h[ts][s][r4 * 4]), quot(h[ts][s][r4 * 4 + 1]), code, false);
                            code = __builtin_amdgcn_cvt_pk_fp8_f32(quot(h[ts][s][r4 * 4 + 2]), quot(h[ts][s][r4 * 4 + 3]), code, true);
                            *reinterpret_cast<uint32_t*>(dst + s * 32 + r4 * 8) = (uint32_t)code;
                        }
                    if (half == 0 && wf == 0) hs[(size_t)wk.ft * n_rows + p] = sc;
                }
            }
        }
    } else {
        // The accumulators hold 16-byte pieces of 64 different rows per store instruction, which the memory
        // pipeline would take as 64 separate requests.  Each wave therefore turns its 128 x 64 block through a
        // private LDS region (the operand rings are free now), 64 features at a time, and writes 256 contiguous
        // bytes of a row with every 16 lanes.
        if (wave_active) {
            constexpr int TS_STRIDE = 68;                      // floats per staged token row: 64 + 4 of padding
            float* const stage = reinterpret_cast<float*>(smem) + wave * (64 * TS_STRIDE);
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            const int s = hh * 2 + sl;
                            const float4 v = make_float4(acc[s][ts][r4 * 4], acc[s][ts][r4 * 4 + 1],
                                                         acc[s][ts][r4 * 4 + 2], acc[s][ts][r4 * 4 + 3]);
                            *reinterpret_cast<float4*>(stage + (ts * 32 + l32) * TS_STRIDE + sl * 32 + r4 * 8 + half * 4) = v;
                        }
                // the lanes of a wave run in step: once its own LDS writes have completed, every lane's have
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                const int fcol = f0 + wf * 128 + hh * 64;
                if (fcol < NOUT) {
#pragma unroll 4
                    for (int it = 0; it < 16; ++it) {
                        const int trow = it * 4 + (lane >> 4);
                        const float4 v = *reinterpret_cast<const float4*>(stage + trow * TS_STRIDE + (lane & 15) * 4);
                        const int p = wk.row0 + wt * 64 + trow;
                        if (p < row_end)
                            *reinterpret_cast<float4*>(y_perm + (size_t)p * NOUT + fcol + (lane & 15) * 4) = v;
                    }
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // all reads done before the region is rewritten
            }
        }
    }
}

constexpr size_t SMEM_BYTES = NW_BUF * W_TILE + NX_BUF * X_TILE;   // 160 KiB

}  // namespace

size_t ffn_work_bytes(int max_tiles, int F, int d) {
    return sizeof(Work) * (size_t)max_tiles * (size_t)(F / 128 + (d + 255) / 256);
}

static hipError_t set_lds_limits() {
    static bool attr_set = false;
    if (attr_set) return hipSuccess;
    const void* kernels[3] = {reinterpret_cast<const void*>(&ffn_gemm<true, false>),
                              reinterpret_cast<const void*>(&ffn_gemm<true, true>),
                              reinterpret_cast<const void*>(&ffn_gemm<false, false>)};
    for (const void* k : kernels) {
        hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM_BYTES);
        if (e != hipSuccess) return e;
    }
    attr_set = true;
    return hipSuccess;
}

// scales of the expert-sorted rows from the per-token scales: out[g][p] = in[g][perm[p] / fan]
__global__ __launch_bounds__(256) void gather_scales(const float* __restrict__ in, int T, const int32_t* __restrict__ perm,
                                                     int fan, int N, float* __restrict__ out) {
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= N) return;
    const size_t g = blockIdx.y;
    const uint32_t t = min((uint32_t)perm[p] / (uint32_t)fan, (uint32_t)(T - 1));
    out[g * N + p] = in[g * T + t];
}

// perm == nullptr: xq/xs are the expert-ordered activations [N,d], [d/128][N].
// perm != nullptr: xq/xs are in token order [T,d], [d/128][T]; sorted row p reads token perm[p] / k
//                  (the scales are first brought into sorted order in the context's workspace).
hipError_t launch_expert_ffn(moe_ctx* c, const uint8_t* xq, const float* xs, const int32_t* perm, const int32_t* offsets,
                             const uint8_t* W1, const uint8_t* W3, const uint8_t* W2, const float* s1,
                             const float* s3, const float* s2, float* y_perm) {
    const moe_dims& D = c->dims;
    hipError_t ea = set_lds_limits();
    if (ea != hipSuccess) return ea;
    Work* work = reinterpret_cast<Work*>(c->tiles);
    hipEvent_t* ev = nullptr;
    if (c->profiling && c->prof_calls < PROF_MAX_CALLS) ev = c->prof_events + 3 * c->prof_calls++;

    const int N = (int)((int64_t)D.T * D.k);
    const int nft1 = D.F / 128;
    const int nft2 = (D.d + 255) / 256;
    Work* work2 = work + (size_t)c->max_tiles * nft1;          // the down projection's list
    int32_t* n_work2 = c->n_tiles + 1;
    hipLaunchKernelGGL(build_work, dim3(D.E, 2), dim3(256), 0, c->stream, offsets, D.E, nft1, nft2, work, work2,
                       c->n_tiles);
    const int grid1 = ((c->max_tiles * nft1 + NXCD - 1) / NXCD) * NXCD;
    if (perm)
        hipLaunchKernelGGL(gather_scales, dim3((N + 255) / 256, D.d / QBLOCK), dim3(256), 0, c->stream, xs, D.T,
                           perm, D.k, N, c->xs_sorted);
    if (ev) (void)hipEventRecord(ev[0], c->stream);          // the timed interval is the GEMM kernel alone
    if (perm) {
        hipLaunchKernelGGL((ffn_gemm<true, true>), dim3(grid1), dim3(NTHREADS), SMEM_BYTES, c->stream, xq, c->xs_sorted, N,
                           perm, D.k, D.T, offsets, work, c->n_tiles, W1, W3, s1, s3, D.d, D.F, c->hq, c->hs,
                           (float*)nullptr);
    } else {
        hipLaunchKernelGGL((ffn_gemm<true, false>), dim3(grid1), dim3(NTHREADS), SMEM_BYTES, c->stream, xq, xs, N,
                           (const int32_t*)nullptr, 1, 1, offsets, work, c->n_tiles, W1, W3, s1, s3, D.d, D.F, c->hq,
                           c->hs, (float*)nullptr);
    }
    if (ev) (void)hipEventRecord(ev[1], c->stream);
    const int grid2 = ((c->max_tiles * nft2 + NXCD - 1) / NXCD) * NXCD;
    hipLaunchKernelGGL((ffn_gemm<false, false>), dim3(grid2), dim3(NTHREADS), SMEM_BYTES, c->stream, c->hq, c->hs,
                       N, (const int32_t*)nullptr, 1, 1, offsets, work2, n_work2, W2, (const uint8_t*)nullptr, s2,
                       (const float*)nullptr, D.F, D.d, (uint8_t*)nullptr, (float*)nullptr, y_perm);
    if (ev) (void)hipEventRecord(ev[2], c->stream);
    return hipGetLastError();
}

__global__ void set_row_range(int32_t* __restrict__ offsets2, int32_t rows) {
    offsets2[0] = 0;
    offsets2[1] = rows;
}

// Dense block-scaled FP8 linear layer: the down-projection kernel with a single "expert" that owns all rows.
hipError_t launch_linear(moe_ctx* c, const uint8_t* xq, const float* xs, int32_t rows, int32_t K, const uint8_t* Wq,
                         const float* ws, int32_t NOUT, float* y) {
    hipError_t ea = set_lds_limits();
    if (ea != hipSuccess) return ea;
    Work* work = reinterpret_cast<Work*>(c->tiles);
    int32_t* range = c->flags + 2;                             // {0, rows}
    int32_t* n_work = c->n_tiles + 2;
    const int nft = (NOUT + 255) / 256;
    hipLaunchKernelGGL(set_row_range, dim3(1), dim3(1), 0, c->stream, range, rows);
    hipLaunchKernelGGL(build_work, dim3(1, 1), dim3(256), 0, c->stream, range, 1, nft, nft, work, work, n_work);
    const int tiles = (rows + TOK_TILE - 1) / TOK_TILE;
    const int grid = ((tiles * nft + NXCD - 1) / NXCD) * NXCD;
    hipLaunchKernelGGL((ffn_gemm<false, false>), dim3(grid), dim3(NTHREADS), SMEM_BYTES, c->stream, xq, xs, rows,
                       (const int32_t*)nullptr, 1, 1, range, work, n_work, Wq, (const uint8_t*)nullptr, ws, (const float*)nullptr, K, NOUT, (uint8_t*)nullptr,
                       (float*)nullptr, y);
    return hipGetLastError();
}

}  // namespace moe355
