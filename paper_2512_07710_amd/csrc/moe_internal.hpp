// Internal declarations shared by the HIP translation units of libmoe355.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "moe355.h"

namespace moe355 {

constexpr int QBLOCK = 128;        // quantisation group (activations 1x128, weights 128x128)
constexpr int PERM_CHUNK = 2048;   // assignments handled by one block of the permutation kernels
constexpr int TOK_TILE = 256;      // expert-sorted rows per GEMM tile
constexpr int MAX_E = 256;
constexpr int MAX_K = 16;
constexpr int PROF_MAX_CALLS = 512;


}  // namespace moe355

struct moe_ctx {
    moe_dims dims;
    hipStream_t stream;
    int device;
    int n_chunks;            // ceil(N / PERM_CHUNK)
    int max_tiles;           // upper bound on GEMM row tiles: N/TOK_TILE + E
    int32_t* chunk_counts;   // [n_chunks][E] per-chunk histograms, then their exclusive scans
    void* tiles;             // GEMM work lists (gate/up list, then down list)
    int32_t* n_tiles;        // [2] their lengths
    int32_t* flags;          // [4] flags[0] != 0: an expert id outside [0,E) was met; flags[1] != 0: a logged id repeated
                             //     inside a token; [2..3]: row range of a dense linear
    float* xs_sorted;        // [d/128][N] activation scales in sorted order (gathered FFN only)
    uint16_t* router_planes; // router weights split into three bf16 planes, matrix-core order
    float* route_partial;    // [splits][T padded to 32][E padded] partial logits of the split router (small batches only)
    uint8_t* hq;             // [N][F]
    float* hs;               // [N][F/128]
    // optional kernel timing: three events per recorded expert-FFN call
    bool profiling;
    int prof_calls;
    hipEvent_t* prof_events; // [3 * PROF_MAX_CALLS], created on first enable
};

namespace moe355 {

// logged_idx == nullptr: top-k selection; otherwise the ids are given and only the gate weights are computed
hipError_t launch_route(moe_ctx* c, const uint16_t* x, const float* W_r, const float* bias,
                        const int32_t* logged_idx, int32_t* topk_idx, float* topk_w);
// Permutation of T*k assignments over E experts on `stream`.  chunk_counts: ceil(T*k / PERM_CHUNK) * E ints of
// scratch; flags: two ints, [0] raised by an id outside [0,E), [1] (check_dups only) by a repeat inside a token.
struct permute_args {
    hipStream_t stream;
    int T, E, k;
    int32_t* chunk_counts;
    int32_t* flags;
    bool check_dups;
};
hipError_t launch_permute(const permute_args& a, const int32_t* ids_in, int32_t* ids_copy, const float* w_in,
                          float* w_copy, int32_t* offsets, int32_t* perm, int32_t* inv_perm);
// Router Replay with every byte of workspace in a static device array (permute.hip)
int route_replay_noalloc(hipStream_t stream, int32_t T, int32_t E, int32_t k, const int32_t* logged_idx,
                         const float* logged_w, int32_t* topk_idx, float* topk_w, int32_t* offsets, int32_t* perm,
                         int32_t* inv_perm, int32_t* id_flags);
hipError_t launch_probe_copy(hipStream_t stream, const void* src, void* dst, size_t bytes);
hipError_t launch_probe_mfma(hipStream_t stream, int blocks, int steps, bool scaled, float* sink);
hipError_t launch_fill_i32(hipStream_t stream, int32_t* p, int n, int32_t v);
hipError_t launch_quantize(hipStream_t s, const uint16_t* x, int64_t rows_in, int32_t cols,
                           const int32_t* dst_rows, int32_t fanout, uint8_t* q, float* scales);
hipError_t launch_expert_ffn(moe_ctx* c, const uint8_t* xq, const float* xs, const int32_t* perm, const int32_t* offsets,
                             const uint8_t* W1, const uint8_t* W3, const uint8_t* W2,
                             const float* s1, const float* s3, const float* s2, float* y_perm);
hipError_t launch_linear(moe_ctx* c, const uint8_t* xq, const float* xs, int32_t rows, int32_t K,
                         const uint8_t* Wq, const float* ws, int32_t NOUT, float* y);
hipError_t launch_quantize_weights(hipStream_t s, const uint16_t* w, int64_t rows, int32_t cols, uint8_t* q,
                                   float* scales);
size_t ffn_work_bytes(int max_tiles, int F, int d);
size_t route_workspace_bytes(int E, int d);
size_t route_partial_bytes(int T, int E);
hipError_t launch_combine(moe_ctx* c, const float* y_perm, const int32_t* inv_perm,
                          const float* topk_w, uint16_t* y, float* y_f32);

}  // namespace moe355
