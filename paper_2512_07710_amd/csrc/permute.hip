// Stable counting sort of the T*k (token, slot) assignments by expert id.
//
// Three atomics-free kernels:
//   1. chunk_hist_rank: each block ranks PERM_CHUNK ids with wave ballots and per-wave
//      running counts in LDS, which yields the chunk's histogram and every entry's rank
//      among earlier equal ids of the chunk.
//   2. scan_chunks: one block turns the per-chunk histograms into exclusive prefix
//      sums over chunks (per expert) and the expert totals into offsets[0..E].
//   3. scatter: position = offsets[e] + prefix[chunk][e] + rank; writes perm/inv_perm.  Ids that come
//      from a log are also checked here: an id outside [0,E) raises flags[0], an id that repeats an
//      earlier slot of the same token raises flags[1] (the permutation is still the stable sort of
//      what was given).
// The result is unique (stable), so it can be compared bit for bit.  Batches of at most PERM_CHUNK
// assignments take one fused launch instead (permute_one_chunk).
#include "moe_internal.hpp"

#include <mutex>

namespace moe355 {
namespace {

// Scratch of moe_route_replay_noalloc: the per-chunk histograms of the three-kernel permutation, then two flag
// words.  A file-scope device array (every GPU the library runs on holds its own copy until the process ends)
// instead of a hipMalloc'ed workspace, so that the call allocates nothing.
constexpr int NOALLOC_MAX_N = 1 << 20;                                  // assignments (T*k) per call
constexpr int NOALLOC_COUNT_INTS = (NOALLOC_MAX_N / PERM_CHUNK) * MAX_E; // 512 chunks x 256 experts
constexpr int NOALLOC_FLAG_INTS = 64;
static __device__ __align__(256) int32_t scratch[NOALLOC_COUNT_INTS + NOALLOC_FLAG_INTS];   // 512.25 KiB

// Host code never passes `scratch` itself to a kernel (there the name is a host-side stand-in): the device
// address is asked for once per device and kept here.
constexpr int MAX_DEVICES = 64;
int32_t* scratch_addr[MAX_DEVICES] = {};
std::mutex scratch_mutex;

hipError_t scratch_on_current_device(int32_t** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_addr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_addr[dev] = static_cast<int32_t*>(p);
    }
    *out = scratch_addr[dev];
    return hipSuccess;
}

// Each of the four waves ranks a quarter of the chunk, 64 entries at a time: eight ballots (one per
// bit of the expert id) give every lane the set of lanes that hold the same id, its rank among them is
// a population count of the lower lanes, and the lowest lane of each set advances that expert's running
// count, kept per wave in LDS (read by the whole set, then written by one lane: LDS operations of a wave
// execute in order).  A second pass turns the per-wave counts into the chunk histogram and the per-wave
// bases.  Ids outside [0,E) are ranked among themselves; that rank is never used.
__global__ __launch_bounds__(256) void chunk_hist_rank(const int32_t* __restrict__ ids, int N, int E,
                                                       int32_t* __restrict__ chunk_counts,
                                                       int32_t* __restrict__ rank_out,
                                                       int32_t* __restrict__ ids_copy) {
    constexpr int PER_WAVE = PERM_CHUNK / 4;          // 512 entries, 8 steps of 64
    __shared__ int32_t s_cnt[4][MAX_E];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int base = blockIdx.x * PERM_CHUNK;
    for (int i = tid; i < 4 * MAX_E; i += 256) (&s_cnt[0][0])[i] = 0;
    __syncthreads();
    int32_t my_id[PER_WAVE / 64], my_rank[PER_WAVE / 64];
    const uint64_t lower = (1ull << lane) - 1ull;
#pragma unroll
    for (int st = 0; st < PER_WAVE / 64; ++st) {
        const int i = base + wave * PER_WAVE + st * 64 + lane;
        int32_t v = -1;
        if (i < N) {
            v = ids[i];
            if (ids_copy) ids_copy[i] = v;
        }
        const bool valid = v >= 0 && v < E;           // entries past the end and bad ids form a class of their own
        my_id[st] = v;
        const int key = v & (MAX_E - 1);
        uint64_t same = __ballot(valid);              // lanes past the end never match a valid lane
        if (!valid) same = ~same;
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const uint64_t bal = __ballot((key >> bit) & 1);
            same &= ((key >> bit) & 1) ? bal : ~bal;
        }
        const int before = s_cnt[wave][key];
        my_rank[st] = before + __popcll(same & lower);
        if (valid && (same & lower) == 0ull) s_cnt[wave][key] = before + __popcll(same);
    }
    __syncthreads();
    // thread e: per-wave bases (exclusive over waves) and the chunk total of expert e
    if (tid < MAX_E) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int c = s_cnt[w][tid];
            s_cnt[w][tid] = run;
            run += c;
        }
        if (tid < E) chunk_counts[(size_t)blockIdx.x * E + tid] = run;
    }
    __syncthreads();
#pragma unroll
    for (int st = 0; st < PER_WAVE / 64; ++st) {
        const int i = base + wave * PER_WAVE + st * 64 + lane;
        if (i < N) rank_out[i] = my_rank[st] + s_cnt[wave][my_id[st] & (MAX_E - 1)];
    }
}

__global__ __launch_bounds__(256) void scan_chunks(int32_t* __restrict__ chunk_counts, int n_chunks,
                                                   int E, int N, int32_t* __restrict__ offsets) {
    __shared__ int32_t s_tot[MAX_E];
    const int tid = threadIdx.x;
    int run = 0;
    if (tid < E) {
        int c = 0;
        for (; c + 8 <= n_chunks; c += 8) {
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = chunk_counts[(size_t)(c + u) * E + tid];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                chunk_counts[(size_t)(c + u) * E + tid] = run;
                run += v[u];
            }
        }
        for (; c < n_chunks; ++c) {
            const int v = chunk_counts[(size_t)c * E + tid];
            chunk_counts[(size_t)c * E + tid] = run;
            run += v;
        }
    }
    s_tot[tid] = (tid < E) ? run : 0;
    __syncthreads();
    // inclusive scan over experts (Hillis-Steele, 256 entries)
    for (int off = 1; off < MAX_E; off <<= 1) {
        int add = (tid >= off) ? s_tot[tid - off] : 0;
        __syncthreads();
        s_tot[tid] += add;
        __syncthreads();
    }
    if (tid < E) offsets[tid + 1] = s_tot[tid];
    if (tid == 0) offsets[0] = 0;
    (void)N;
}

__global__ __launch_bounds__(256) void scatter(const int32_t* __restrict__ ids, int N, int E,
                                               const int32_t* __restrict__ chunk_prefix,
                                               const int32_t* __restrict__ offsets,
                                               const float* __restrict__ w_in, float* __restrict__ w_copy,
                                               int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                                               int k, bool check_dups, int32_t* __restrict__ flags) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    if (w_copy) w_copy[i] = w_in[i];
    const int e = ids[i];
    if (e < 0 || e >= E) {
        flags[0] = 1;                                   // plain store; any writer stores the same value
        inv_perm[i] = -1;
        return;
    }
    if (check_dups) {
        const int first = i - i % k;                    // slot 0 of this assignment's token
        bool dup = false;
        for (int q = first; q < i; ++q) dup |= ids[q] == e;
        if (dup) flags[1] = 1;
    }
    const int chunk = i / PERM_CHUNK;
    const int pos = offsets[e] + chunk_prefix[(size_t)chunk * E + e] + inv_perm[i];   // inv_perm holds the rank
    inv_perm[i] = pos;
    perm[pos] = i;
}

// N <= PERM_CHUNK: the three steps in one block and one launch (decode-sized batches, where the launches
// themselves are most of the time).  Same ranking as chunk_hist_rank, then the scan over experts and the
// scatter from registers.
__global__ __launch_bounds__(256) void permute_one_chunk(const int32_t* __restrict__ ids, int N, int E,
                                                         int32_t* __restrict__ ids_copy,
                                                         const float* __restrict__ w_in, float* __restrict__ w_copy,
                                                         int32_t* __restrict__ offsets, int32_t* __restrict__ perm,
                                                         int32_t* __restrict__ inv_perm, int k, bool check_dups,
                                                         int32_t* __restrict__ flags) {
    constexpr int PER_WAVE = PERM_CHUNK / 4;
    __shared__ int32_t s_cnt[4][MAX_E];
    __shared__ int32_t s_off[MAX_E];                  // inclusive scan of the expert totals
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 4 * MAX_E; i += 256) (&s_cnt[0][0])[i] = 0;
    __syncthreads();
    int32_t my_id[PER_WAVE / 64], my_rank[PER_WAVE / 64];
    const uint64_t lower = (1ull << lane) - 1ull;
#pragma unroll
    for (int st = 0; st < PER_WAVE / 64; ++st) {
        const int i = wave * PER_WAVE + st * 64 + lane;
        int32_t v = -1;
        if (i < N) {
            v = ids[i];
            if (ids_copy) ids_copy[i] = v;
            if (w_copy) w_copy[i] = w_in[i];
        }
        const bool valid = v >= 0 && v < E;
        my_id[st] = v;
        const int key = v & (MAX_E - 1);
        uint64_t same = __ballot(valid);
        if (!valid) same = ~same;
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const uint64_t bal = __ballot((key >> bit) & 1);
            same &= ((key >> bit) & 1) ? bal : ~bal;
        }
        const int before = s_cnt[wave][key];
        my_rank[st] = before + __popcll(same & lower);
        if (valid && (same & lower) == 0ull) s_cnt[wave][key] = before + __popcll(same);
    }
    __syncthreads();
    {
        int run = 0;                                  // thread e: per-wave bases and the total of expert e
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int c = s_cnt[w][tid];
            s_cnt[w][tid] = run;
            run += c;
        }
        s_off[tid] = (tid < E) ? run : 0;
    }
    __syncthreads();
    for (int off = 1; off < MAX_E; off <<= 1) {       // inclusive scan over experts
        const int add = (tid >= off) ? s_off[tid - off] : 0;
        __syncthreads();
        s_off[tid] += add;
        __syncthreads();
    }
    if (tid < E) offsets[tid + 1] = s_off[tid];
    if (tid == 0) offsets[0] = 0;
#pragma unroll
    for (int st = 0; st < PER_WAVE / 64; ++st) {
        const int i = wave * PER_WAVE + st * 64 + lane;
        if (i >= N) continue;
        const int e = my_id[st];
        if (e < 0 || e >= E) {
            flags[0] = 1;
            inv_perm[i] = -1;
            continue;
        }
        if (check_dups) {
            const int first = i - i % k;
            bool dup = false;
            for (int q = first; q < i; ++q) dup |= ids[q] == e;
            if (dup) flags[1] = 1;
        }
        const int pos = (e ? s_off[e - 1] : 0) + s_cnt[wave][e] + my_rank[st];
        inv_perm[i] = pos;
        perm[pos] = i;
    }
}

__global__ void fill_i32(int32_t* __restrict__ p, int n, int32_t v) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

}  // namespace

// a fill kernel, not hipMemsetAsync: it stays correct when a caller records the call into a HIP graph
hipError_t launch_fill_i32(hipStream_t stream, int32_t* p, int n, int32_t v) {
    if (n > 0) hipLaunchKernelGGL(fill_i32, dim3((n + 255) / 256), dim3(256), 0, stream, p, n, v);
    return hipGetLastError();
}

hipError_t launch_permute(const permute_args& a, const int32_t* ids_in, int32_t* ids_copy, const float* w_in,
                          float* w_copy, int32_t* offsets, int32_t* perm, int32_t* inv_perm) {
    const int N = a.T * a.k;
    const int n_chunks = (N + PERM_CHUNK - 1) / PERM_CHUNK;
    if (n_chunks == 1) {
        hipLaunchKernelGGL(permute_one_chunk, dim3(1), dim3(256), 0, a.stream, ids_in, N, a.E, ids_copy, w_in, w_copy,
                           offsets, perm, inv_perm, a.k, a.check_dups, a.flags);
        return hipGetLastError();
    }
    if (n_chunks > 0)
        hipLaunchKernelGGL(chunk_hist_rank, dim3(n_chunks), dim3(256), 0, a.stream, ids_in, N, a.E,
                           a.chunk_counts, inv_perm, ids_copy);
    hipLaunchKernelGGL(scan_chunks, dim3(1), dim3(256), 0, a.stream, a.chunk_counts, n_chunks, a.E, N,
                       offsets);
    if (N > 0)
        hipLaunchKernelGGL(scatter, dim3((N + 255) / 256), dim3(256), 0, a.stream, ids_in, N, a.E,
                           a.chunk_counts, offsets, w_in, w_copy, perm, inv_perm, a.k, a.check_dups, a.flags);
    return hipGetLastError();
}

// Router Replay (copy of the log + stable permutation) whose only workspace is the static device array above.
// Overlapping calls on one GPU (two streams, two threads) share that array and race.
int route_replay_noalloc(hipStream_t stream, int32_t T, int32_t E, int32_t k, const int32_t* logged_idx,
                         const float* logged_w, int32_t* topk_idx, float* topk_w, int32_t* offsets, int32_t* perm,
                         int32_t* inv_perm, int32_t* id_flags) {
    if (T < 0 || E < 1 || E > MAX_E || k < 1 || k > E || k > MAX_K) return MOE_EINVAL;
    if ((int64_t)T * k > NOALLOC_MAX_N) return MOE_EINVAL;             // beyond the scratch array's capacity
    if (!offsets) return MOE_EINVAL;
    if (T > 0 && (!logged_idx || !logged_w || !topk_idx || !topk_w || !perm || !inv_perm)) return MOE_EINVAL;
    int32_t* base = nullptr;
    if (scratch_on_current_device(&base) != hipSuccess) return MOE_EHIP;
    int32_t* flags = id_flags ? id_flags : base + NOALLOC_COUNT_INTS;
    // the flags must start at zero (the histograms need no clearing: every chunk in use is rewritten in full)
    if (launch_fill_i32(stream, flags, 2, 0) != hipSuccess) return MOE_EHIP;
    if (T == 0) return launch_fill_i32(stream, offsets, E + 1, 0) == hipSuccess ? MOE_OK : MOE_EHIP;
    const permute_args a{stream, T, E, k, base, flags, true};
    int32_t* idx_copy = (topk_idx == logged_idx) ? nullptr : topk_idx;
    float* w_copy = (topk_w == logged_w) ? nullptr : topk_w;
    return launch_permute(a, logged_idx, idx_copy, logged_w, w_copy, offsets, perm, inv_perm) == hipSuccess ? MOE_OK
                                                                                                           : MOE_EHIP;
}

}  // namespace moe355
