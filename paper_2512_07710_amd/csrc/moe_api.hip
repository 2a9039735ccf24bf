// C-ABI entry points of libmoe355: argument validation, context and workspace.
#include "moe_internal.hpp"

#include <new>

using namespace moe355;

namespace {

inline int hip_rc(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_EHIP; }

// T == 0: the per-token arrays have no elements and may be null; offsets is all zeros
int route_empty(moe_ctx* c, int32_t* offsets) {
    if (!offsets) return MOE_EINVAL;
    return hip_rc(launch_fill_i32(c->stream, offsets, c->dims.E + 1, 0));
}

// The kernels address a row's bytes with 32-bit offsets from a 64-bit base: the router reads x at byte t*d*2,
// the gathering gate/up GEMM reads the token-order codes at byte t*d and every GEMM reads a weight matrix of
// one expert at byte f*K.  Shapes beyond those ranges are refused here instead of wrapping silently.
bool dims_ok(const moe_dims* d) {
    if (!d) return false;
    if (d->T < 0 || d->d <= 0 || d->F <= 0 || d->E <= 0 || d->k <= 0) return false;
    if (d->d % QBLOCK || d->F % QBLOCK) return false;
    if (d->E > MAX_E || d->k > d->E || d->k > MAX_K) return false;
    if ((int64_t)d->T * d->k > (int64_t)1 << 30) return false;
    if ((int64_t)d->T * d->d >= (int64_t)1 << 31) return false;
    if ((int64_t)d->F * d->d >= (int64_t)1 << 32) return false;
    return true;
}

permute_args perm_args(moe_ctx* c, bool check_dups) {
    return permute_args{c->stream, c->dims.T, c->dims.E, c->dims.k, c->chunk_counts, c->flags, check_dups};
}

}  // namespace

extern "C" {

const char* moe_version(void) { return "moe355 0.1 (gfx950)"; }

const char* moe_strerror(int code) {
    switch (code) {
        case MOE_OK: return "ok";
        case MOE_EINVAL: return "invalid argument";
        case MOE_EHIP: return "HIP runtime or launch error";
        case MOE_EBADIDS: return "expert id outside [0,E) or repeated inside a token";
        case MOE_ENOMEM: return "workspace allocation failed";
        default: return "unknown error";
    }
}

int moe_create(moe_ctx** out, const moe_dims* dims, void* hip_stream) {
    if (!out) return MOE_EINVAL;
    *out = nullptr;
    if (!dims_ok(dims)) return MOE_EINVAL;
    moe_ctx* c = new (std::nothrow) moe_ctx();
    if (!c) return MOE_ENOMEM;
    c->dims = *dims;
    c->stream = (hipStream_t)hip_stream;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return MOE_EHIP; }
    const int64_t N = (int64_t)dims->T * dims->k;
    c->n_chunks = (int)((N + PERM_CHUNK - 1) / PERM_CHUNK);
    if (c->n_chunks < 1) c->n_chunks = 1;
    c->max_tiles = (int)(N / TOK_TILE) + dims->E;
    const size_t nrow = (size_t)(N > 0 ? N : 1);
    bool ok = true;
    ok = ok && hipMalloc((void**)&c->chunk_counts, sizeof(int32_t) * (size_t)c->n_chunks * dims->E) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->tiles, ffn_work_bytes(c->max_tiles, dims->F, dims->d)) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->n_tiles, 4 * sizeof(int32_t)) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->flags, 4 * sizeof(int32_t)) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->router_planes, route_workspace_bytes(dims->E, dims->d)) == hipSuccess;
    if (route_partial_bytes(dims->T, dims->E))
        ok = ok && hipMalloc((void**)&c->route_partial, route_partial_bytes(dims->T, dims->E)) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->xs_sorted, nrow * (size_t)(dims->d / QBLOCK) * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->hq, nrow * (size_t)dims->F) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->hs, nrow * (size_t)(dims->F / QBLOCK) * sizeof(float)) == hipSuccess;
    ok = ok && launch_fill_i32(c->stream, c->flags, 4, 0) == hipSuccess;
    ok = ok && launch_fill_i32(c->stream, c->n_tiles, 4, 0) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        moe_destroy(c);
        return MOE_ENOMEM;
    }
    *out = c;
    return MOE_OK;
}

int moe_destroy(moe_ctx* c) {
    if (!c) return MOE_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    if (c->chunk_counts) (void)hipFree(c->chunk_counts);
    if (c->tiles) (void)hipFree(c->tiles);
    if (c->n_tiles) (void)hipFree(c->n_tiles);
    if (c->flags) (void)hipFree(c->flags);
    if (c->xs_sorted) (void)hipFree(c->xs_sorted);
    if (c->router_planes) (void)hipFree(c->router_planes);
    if (c->route_partial) (void)hipFree(c->route_partial);
    if (c->hq) (void)hipFree(c->hq);
    if (c->hs) (void)hipFree(c->hs);
    if (c->prof_events) {
        for (int i = 0; i < 3 * PROF_MAX_CALLS; ++i) (void)hipEventDestroy(c->prof_events[i]);
        delete[] c->prof_events;
    }
    delete c;
    return MOE_OK;
}

int moe_route(moe_ctx* c, const uint16_t* x, const float* W_r, const float* bias, int32_t k,
              int32_t* topk_idx, float* topk_w, int32_t* offsets, int32_t* perm, int32_t* inv_perm) {
    if (!c || k != c->dims.k) return MOE_EINVAL;
    if (c->dims.T == 0) return route_empty(c, offsets);
    if (!x || !W_r || !topk_idx || !topk_w || !offsets || !perm || !inv_perm) return MOE_EINVAL;
    hipError_t e = launch_route(c, x, W_r, bias, nullptr, topk_idx, topk_w);
    if (e != hipSuccess) return MOE_EHIP;
    return hip_rc(launch_permute(perm_args(c, false), topk_idx, nullptr, nullptr, nullptr, offsets, perm, inv_perm));
}

int moe_route_replay(moe_ctx* c, const uint16_t* x, const int32_t* logged_idx, const float* logged_w,
                     int32_t* topk_idx, float* topk_w, int32_t* offsets, int32_t* perm,
                     int32_t* inv_perm) {
    (void)x;
    if (!c) return MOE_EINVAL;
    if (c->dims.T == 0) return route_empty(c, offsets);
    if (!logged_idx || !logged_w || !topk_idx || !topk_w || !offsets || !perm || !inv_perm) return MOE_EINVAL;
    int32_t* idx_copy = (topk_idx == logged_idx) ? nullptr : topk_idx;
    float* w_copy = (topk_w == logged_w) ? nullptr : topk_w;
    return hip_rc(launch_permute(perm_args(c, true), logged_idx, idx_copy, logged_w, w_copy, offsets, perm, inv_perm));
}

int moe_route_replay_noalloc(void* hip_stream, int32_t T, int32_t E, int32_t k, const int32_t* logged_idx,
                             const float* logged_w, int32_t* topk_idx, float* topk_w, int32_t* offsets,
                             int32_t* perm, int32_t* inv_perm, int32_t* id_flags) {
    return route_replay_noalloc((hipStream_t)hip_stream, T, E, k, logged_idx, logged_w, topk_idx, topk_w, offsets, perm,
                                inv_perm, id_flags);
}

int moe_route_replay_ids(moe_ctx* c, const uint16_t* x, const float* W_r, const int32_t* logged_idx,
                         int32_t* topk_idx, float* topk_w, int32_t* offsets, int32_t* perm, int32_t* inv_perm) {
    if (!c) return MOE_EINVAL;
    if (c->dims.T == 0) return route_empty(c, offsets);
    if (!x || !W_r || !logged_idx || !topk_idx || !topk_w || !offsets || !perm || !inv_perm) return MOE_EINVAL;
    hipError_t e = launch_route(c, x, W_r, nullptr, logged_idx, topk_idx, topk_w);
    if (e != hipSuccess) return MOE_EHIP;
    return hip_rc(launch_permute(perm_args(c, true), topk_idx, nullptr, nullptr, nullptr, offsets, perm, inv_perm));
}

int moe_check_ids(moe_ctx* c) {
    if (!c) return MOE_EINVAL;
    int32_t h[4] = {0, 0, 0, 0};
    if (hipMemcpyAsync(h, c->flags, sizeof(h), hipMemcpyDeviceToHost, c->stream) != hipSuccess) return MOE_EHIP;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return MOE_EHIP;
    if (h[0] != 0 || h[1] != 0) {
        if (launch_fill_i32(c->stream, c->flags, 2, 0) != hipSuccess) return MOE_EHIP;
        return MOE_EBADIDS;
    }
    return MOE_OK;
}

int moe_quantize_fp8(moe_ctx* c, const uint16_t* x, int64_t rows_in, int32_t cols, int32_t block,
                     const int32_t* dst_rows, int32_t fanout, uint8_t* q, float* scales) {
    if (!c) return MOE_EINVAL;
    if (block != QBLOCK || cols <= 0 || cols % QBLOCK || rows_in < 0 || fanout < 1) return MOE_EINVAL;
    if (!dst_rows && fanout != 1) return MOE_EINVAL;
    if (rows_in * (int64_t)fanout > (int64_t)1 << 30) return MOE_EINVAL;
    if (rows_in == 0) return MOE_OK;
    if (!x || !q || !scales) return MOE_EINVAL;
    return hip_rc(launch_quantize(c->stream, x, rows_in, cols, dst_rows, fanout, q, scales));
}

int moe_quantize_weights_fp8(moe_ctx* c, const uint16_t* w, int64_t rows, int32_t cols, uint8_t* q, float* scales) {
    if (!c || !w || !q || !scales) return MOE_EINVAL;
    if (rows < 0 || cols <= 0 || rows % QBLOCK || cols % QBLOCK || rows / QBLOCK > 65535) return MOE_EINVAL;
    if (rows == 0) return MOE_OK;
    return hip_rc(launch_quantize_weights(c->stream, w, rows, cols, q, scales));
}

int moe_linear_fp8(moe_ctx* c, const uint8_t* xq, const float* xs, int32_t rows, int32_t K, const uint8_t* Wq,
                   const float* ws, int32_t NOUT, float* y) {
    if (!c || !xq || !xs || !Wq || !ws || !y) return MOE_EINVAL;
    if (rows < 0 || K <= 0 || NOUT <= 0 || K % QBLOCK || NOUT % QBLOCK) return MOE_EINVAL;
    if ((int64_t)NOUT * K >= (int64_t)1 << 32) return MOE_EINVAL;     // 32-bit byte offsets inside the weight matrix
    const int64_t units = ((int64_t)rows + TOK_TILE - 1) / TOK_TILE * ((NOUT + 255) / 256);
    const int64_t room = (int64_t)c->max_tiles * (c->dims.F / 128 + (c->dims.d + 255) / 256);
    if (units > room) return MOE_EINVAL;              // the context's work-list storage bounds the problem size
    if (rows == 0) return MOE_OK;
    return hip_rc(launch_linear(c, xq, xs, rows, K, Wq, ws, NOUT, y));
}

int moe_expert_ffn_fp8(moe_ctx* c, const uint8_t* xq, const float* xs, const int32_t* offsets,
                       const uint8_t* W1, const uint8_t* W3, const uint8_t* W2, const float* s1,
                       const float* s3, const float* s2, float* y_perm) {
    if (!c) return MOE_EINVAL;
    if (c->dims.T == 0) return MOE_OK;
    if (!xq || !xs || !offsets || !W1 || !W3 || !W2 || !s1 || !s3 || !s2 || !y_perm) return MOE_EINVAL;
    return hip_rc(launch_expert_ffn(c, xq, xs, nullptr, offsets, W1, W3, W2, s1, s3, s2, y_perm));
}

int moe_expert_ffn_fp8_gather(moe_ctx* c, const uint8_t* xq_tok, const float* xs_tok, const int32_t* perm,
                              const int32_t* offsets, const uint8_t* W1, const uint8_t* W3, const uint8_t* W2,
                              const float* s1, const float* s3, const float* s2, float* y_perm) {
    if (!c) return MOE_EINVAL;
    if (c->dims.T == 0) return MOE_OK;
    if (!xq_tok || !xs_tok || !perm || !offsets || !W1 || !W3 || !W2 || !s1 || !s3 || !s2 || !y_perm) return MOE_EINVAL;
    return hip_rc(launch_expert_ffn(c, xq_tok, xs_tok, perm, offsets, W1, W3, W2, s1, s3, s2, y_perm));
}

int moe_combine(moe_ctx* c, const float* y_perm, const int32_t* inv_perm, const float* topk_w,
                uint16_t* y, float* y_f32) {
    if (!c) return MOE_EINVAL;
    if (c->dims.T == 0) return MOE_OK;
    if (!y_perm || !inv_perm || !topk_w || !y) return MOE_EINVAL;
    return hip_rc(launch_combine(c, y_perm, inv_perm, topk_w, y, y_f32));
}

int moe_profile_enable(moe_ctx* c, int32_t on) {
    if (!c) return MOE_EINVAL;
    if (on && !c->prof_events) {
        c->prof_events = new (std::nothrow) hipEvent_t[3 * PROF_MAX_CALLS];
        if (!c->prof_events) return MOE_ENOMEM;
        for (int i = 0; i < 3 * PROF_MAX_CALLS; ++i)
            if (hipEventCreate(&c->prof_events[i]) != hipSuccess) return MOE_EHIP;
    }
    c->profiling = on != 0;
    c->prof_calls = 0;
    return MOE_OK;
}

int moe_profile_read(moe_ctx* c, float* ms, int32_t* calls) {
    if (!c || !ms || !calls) return MOE_EINVAL;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return MOE_EHIP;
    double a = 0.0, b = 0.0;
    for (int i = 0; i < c->prof_calls; ++i) {
        float t1 = 0.f, t2 = 0.f;
        if (hipEventElapsedTime(&t1, c->prof_events[3 * i], c->prof_events[3 * i + 1]) != hipSuccess) return MOE_EHIP;
        if (hipEventElapsedTime(&t2, c->prof_events[3 * i + 1], c->prof_events[3 * i + 2]) != hipSuccess) return MOE_EHIP;
        a += t1;
        b += t2;
    }
    *calls = c->prof_calls;
    ms[0] = c->prof_calls ? (float)(a / c->prof_calls) : 0.f;
    ms[1] = c->prof_calls ? (float)(b / c->prof_calls) : 0.f;
    c->prof_calls = 0;
    return MOE_OK;
}

int moe_probe_copy(moe_ctx* c, const void* src, void* dst, int64_t bytes) {
    if (!c || !src || !dst || bytes < 0 || bytes % 16) return MOE_EINVAL;
    return hip_rc(launch_probe_copy(c->stream, src, dst, (size_t)bytes));
}

int moe_probe_fp8_mfma(moe_ctx* c, int32_t blocks, int32_t steps, int32_t scaled, float* sink) {
    if (!c || !sink || blocks < 1 || blocks > 65536 || steps < 1 || steps > (1 << 24)) return MOE_EINVAL;
    return hip_rc(launch_probe_mfma(c->stream, blocks, steps, scaled != 0, sink));
}

int moe_debug_copy_hidden(moe_ctx* c, uint8_t* hq_out, float* hs_out) {
    if (!c || !hq_out || !hs_out) return MOE_EINVAL;
    const size_t N = (size_t)c->dims.T * c->dims.k;
    if (N == 0) return MOE_OK;
    if (hipMemcpyAsync(hq_out, c->hq, N * (size_t)c->dims.F, hipMemcpyDeviceToDevice, c->stream) != hipSuccess)
        return MOE_EHIP;
    return hip_rc(hipMemcpyAsync(hs_out, c->hs, N * (size_t)(c->dims.F / QBLOCK) * sizeof(float),
                                 hipMemcpyDeviceToDevice, c->stream));
}

}  // extern "C"
