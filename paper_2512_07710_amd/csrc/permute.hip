// Stable counting sort of the T*k (token, slot) assignments by expert id.
//
// Three atomics-free kernels:
//   1. chunk_hist_rank: each block stages PERM_CHUNK ids in LDS; thread e walks the
//      chunk in order and numbers the entries that name expert e, which yields the
//      chunk's histogram and every entry's rank among earlier equal ids of the chunk.
//   2. scan_chunks: one block turns the per-chunk histograms into exclusive prefix
//      sums over chunks (per expert) and the expert totals into offsets[0..E].
//   3. scatter: position = offsets[e] + prefix[chunk][e] + rank; writes perm/inv_perm.
// The result is unique (stable), so it can be compared bit for bit.
#include "moe_internal.hpp"

namespace moe355 {
namespace {

__global__ __launch_bounds__(256) void chunk_hist_rank(const int32_t* __restrict__ ids, int N, int E,
                                                       int32_t* __restrict__ chunk_counts,
                                                       int32_t* __restrict__ rank_out,
                                                       int32_t* __restrict__ ids_copy) {
    __shared__ int32_t s_id[PERM_CHUNK];
    __shared__ uint16_t s_rank[PERM_CHUNK];
    const int tid = threadIdx.x;
    const int base = blockIdx.x * PERM_CHUNK;
    const int len = min(PERM_CHUNK, N - base);
    for (int i = tid; i < PERM_CHUNK; i += 256) {
        int32_t v = -1;
        if (i < len) {
            v = ids[base + i];
            if (ids_copy) ids_copy[base + i] = v;
        }
        s_id[i] = v;
        s_rank[i] = 0;
    }
    __syncthreads();
    if (tid < E) {
        int cnt = 0;
        const int len4 = (len + 3) & ~3;              // padded entries hold -1 and never match
        for (int i = 0; i < len4; i += 4) {
            const int4 v = *reinterpret_cast<const int4*>(&s_id[i]);
            if (v.x == tid) s_rank[i] = (uint16_t)cnt++;
            if (v.y == tid) s_rank[i + 1] = (uint16_t)cnt++;
            if (v.z == tid) s_rank[i + 2] = (uint16_t)cnt++;
            if (v.w == tid) s_rank[i + 3] = (uint16_t)cnt++;
        }
        chunk_counts[(size_t)blockIdx.x * E + tid] = cnt;
    }
    __syncthreads();
    for (int i = tid; i < len; i += 256) rank_out[base + i] = s_rank[i];
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
                                               int32_t* __restrict__ flags) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    if (w_copy) w_copy[i] = w_in[i];
    const int e = ids[i];
    if (e < 0 || e >= E) {
        flags[0] = 1;                                   // plain store; any writer stores the same value
        inv_perm[i] = -1;
        return;
    }
    const int chunk = i / PERM_CHUNK;
    const int pos = offsets[e] + chunk_prefix[(size_t)chunk * E + e] + inv_perm[i];   // inv_perm holds the rank
    inv_perm[i] = pos;
    perm[pos] = i;
}

}  // namespace

hipError_t launch_permute(moe_ctx* c, const int32_t* ids_in, int32_t* ids_copy, const float* w_in,
                          float* w_copy, int32_t* offsets, int32_t* perm, int32_t* inv_perm) {
    const moe_dims& D = c->dims;
    const int N = D.T * D.k;
    const int n_chunks = (N + PERM_CHUNK - 1) / PERM_CHUNK;
    if (n_chunks > 0)
        hipLaunchKernelGGL(chunk_hist_rank, dim3(n_chunks), dim3(256), 0, c->stream, ids_in, N, D.E,
                           c->chunk_counts, inv_perm, ids_copy);
    hipLaunchKernelGGL(scan_chunks, dim3(1), dim3(256), 0, c->stream, c->chunk_counts, n_chunks, D.E, N,
                       offsets);
    if (N > 0)
        hipLaunchKernelGGL(scatter, dim3((N + 255) / 256), dim3(256), 0, c->stream, ids_in, N, D.E,
                           c->chunk_counts, offsets, w_in, w_copy, perm, inv_perm, c->flags);
    return hipGetLastError();
}

}  // namespace moe355
