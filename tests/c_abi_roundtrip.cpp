// A caller of the C ABI that knows nothing of Python or torch: plain hipMalloc'd
// buffers, the five shuffle calls, and checks that need no second
// implementation of the method.
//   1. Layout (section Dispatch, grouped layout): walking experts, source ranks and
//      tokens in that order and taking every token routed to the expert IS the
//      definition of the expert-major row order; each row must hold its token's bits.
//   2. Round trip (section Combine): identity experts and weights 1/2, 1/4, 1/4 make
//      every partial product and sum exact in fp32, so combine must return x bit for bit.
// Built by the repository's build step, run by the GPU test suite; exits 0 on success.
#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "flmoe.h"

#define HIP_OK(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));            \
            return 2;                                                                  \
        }                                                                              \
    } while (0)
#define FL_CALL(call)                                                                  \
    do {                                                                               \
        int c_ = (call);                                                               \
        if (c_ != FL_OK) {                                                             \
            std::fprintf(stderr, "%s: %s\n", #call, fl_moe_strerror(c_));              \
            return 3;                                                                  \
        }                                                                              \
    } while (0)

int main() {
    const int N = 4, E = 16, El = E / N, T = 48, K = 3, H = 512;
    const int nt[N] = {48, 17, 0, 33};   // ragged, one rank without tokens

    // a configuration the host must refuse: experts not divisible by ranks
    fl_moe_config bad;
    std::memset(&bad, 0, sizeof bad);
    bad.n_ranks = 4; bad.n_experts = 18; bad.max_tokens = T; bad.top_k = K; bad.hidden = H;
    bad.expert_align = 1;
    fl_moe_sizes sz;
    if (fl_moe_query_sizes(&bad, &sz) != FL_ERR_INVALID_ARG) {
        std::fprintf(stderr, "an invalid configuration was accepted\n");
        return 4;
    }

    fl_moe_config cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.n_ranks = N; cfg.n_experts = E; cfg.max_tokens = T; cfg.top_k = K; cfg.hidden = H;
    cfg.dispatch_dtype = FL_DTYPE_BF16; cfg.expert_align = 1;
    FL_CALL(fl_moe_query_sizes(&cfg, &sz));
    const int64_t cap = sz.expert_capacity_rows;

    // inputs: three distinct experts per token, finite bf16 bit patterns from a small generator
    std::vector<int32_t> indices((size_t)N * T * K);
    std::vector<float> weights((size_t)N * T * K);
    std::vector<uint16_t> x((size_t)N * T * H);
    for (int s = 0; s < N; ++s)
        for (int t = 0; t < T; ++t)
            for (int k = 0; k < K; ++k) {
                indices[((size_t)s * T + t) * K + k] = (7 * t + 3 * s + 5 * k) % E;   // 0, 5, 10 apart
                weights[((size_t)s * T + t) * K + k] = k == 0 ? 0.5f : 0.25f;
            }
    uint32_t state = 12345u;
    for (auto &v : x) {
        state = state * 1664525u + 1013904223u;
        const uint32_t sign = state >> 31, expo = 100 + (state >> 8) % 41, mant = (state >> 16) & 0x7f;
        v = (uint16_t)((sign << 15) | (expo << 7) | mant);
    }

    void *ws = nullptr, *d_x = nullptr, *d_ex = nullptr, *d_out = nullptr;
    int32_t *d_idx = nullptr, *d_nt = nullptr, *d_tpe = nullptr;
    float *d_w = nullptr;
    HIP_OK(hipMalloc(&ws, sz.workspace_bytes));
    HIP_OK(hipMalloc(&d_x, x.size() * 2));
    HIP_OK(hipMalloc(&d_ex, (size_t)N * cap * H * 2));
    HIP_OK(hipMalloc(&d_out, x.size() * 2));
    HIP_OK(hipMalloc((void **)&d_idx, indices.size() * 4));
    HIP_OK(hipMalloc((void **)&d_nt, N * 4));
    HIP_OK(hipMalloc((void **)&d_tpe, N * El * 4));
    HIP_OK(hipMalloc((void **)&d_w, weights.size() * 4));
    HIP_OK(hipMemcpy(d_x, x.data(), x.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_idx, indices.data(), indices.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_nt, nt, N * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_w, weights.data(), weights.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemset(d_out, 0xff, x.size() * 2));

    hipStream_t st;
    HIP_OK(hipStreamCreate(&st));
    fl_moe_ctx *ctx = nullptr;
    FL_CALL(fl_moe_create(&cfg, ws, sz.workspace_bytes, &ctx));
    // the route exchange needs all ranks at once; the payload calls are issued per half of the group
    FL_CALL(fl_moe_layout(ctx, 0, N, d_idx, d_nt, nullptr, st));
    for (int half = 0; half < 2; ++half) FL_CALL(fl_moe_dispatch_send(ctx, 2 * half, 2, d_x, st));
    for (int half = 0; half < 2; ++half) FL_CALL(fl_moe_dispatch_recv(ctx, 2 * half, 2, d_ex, nullptr, d_tpe, st));
    for (int half = 0; half < 2; ++half) FL_CALL(fl_moe_combine_send(ctx, 2 * half, 2, d_ex, st));
    for (int half = 0; half < 2; ++half) FL_CALL(fl_moe_combine_reduce(ctx, 2 * half, 2, d_w, d_out, st));
    int32_t status = -1;
    FL_CALL(fl_moe_status(ctx, &status, st));
    if (status != 0) {
        std::fprintf(stderr, "device status %d\n", status);
        return 5;
    }

    std::vector<uint16_t> ex((size_t)N * cap * H), out(x.size());
    std::vector<int32_t> tpe(N * El);
    HIP_OK(hipMemcpy(ex.data(), d_ex, ex.size() * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(out.data(), d_out, out.size() * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(tpe.data(), d_tpe, tpe.size() * 4, hipMemcpyDeviceToHost));

    long long rows_checked = 0;
    for (int d = 0; d < N; ++d) {
        int64_t row = 0;
        for (int j = 0; j < El; ++j) {
            int count = 0;
            for (int s = 0; s < N; ++s)
                for (int t = 0; t < nt[s]; ++t)
                    for (int k = 0; k < K; ++k)
                        if (indices[((size_t)s * T + t) * K + k] == d * El + j) {
                            const uint16_t *got = &ex[((size_t)d * cap + row) * H];
                            const uint16_t *want = &x[((size_t)s * T + t) * H];
                            if (std::memcmp(got, want, (size_t)H * 2) != 0) {
                                std::fprintf(stderr, "rank %d row %lld: not token (%d,%d)\n", d,
                                             (long long)row, s, t);
                                return 6;
                            }
                            ++row; ++count; ++rows_checked;
                        }
            if (tpe[d * El + j] != count) {
                std::fprintf(stderr, "tokens_per_expert[%d][%d] = %d, expected %d\n", d, j,
                             tpe[d * El + j], count);
                return 7;
            }
        }
    }
    for (int s = 0; s < N; ++s) {
        if (std::memcmp(&out[(size_t)s * T * H], &x[(size_t)s * T * H], (size_t)nt[s] * H * 2) != 0) {
            std::fprintf(stderr, "rank %d: combined output differs from the tokens\n", s);
            return 8;
        }
        for (size_t i = (size_t)(s * T + nt[s]) * H; i < (size_t)(s + 1) * T * H; ++i)
            if (out[i] != 0xffff) {
                std::fprintf(stderr, "rank %d: a row of an absent token was written\n", s);
                return 9;
            }
    }

    // 3. The layout step without context or workspace (fl_moe_layout_static, for callers that
    //    cannot allocate): its tokens_per_expert must equal the context's, its counts a plain
    //    histogram of the indices; called twice, the array inside the library being re-used.
    {
        const size_t sizes[10] = {(size_t)N * E, (size_t)N * N, (size_t)N * El, (size_t)N * (N + 1),
                                  (size_t)N * (N + 1), (size_t)N * (El + 1), (size_t)N * (N + 1),
                                  (size_t)N * T * K, (size_t)N, 1};
        size_t total = 0;
        for (size_t v : sizes) total += v;
        int32_t *d_tab = nullptr;
        HIP_OK(hipMalloc((void **)&d_tab, total * 4));
        int32_t *p[10];
        size_t at = 0;
        for (int i = 0; i < 10; ++i) { p[i] = d_tab + at; at += sizes[i]; }
        const fl_moe_layout_out lo = {p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7], p[8], p[9]};
        std::vector<int32_t> tab(total);
        for (int call = 0; call < 2; ++call) {
            HIP_OK(hipMemsetAsync(d_tab, 0x5a, total * 4, st));
            FL_CALL(fl_moe_layout_static(&cfg, d_idx, d_nt, &lo, st));
            HIP_OK(hipStreamSynchronize(st));
            HIP_OK(hipMemcpy(tab.data(), d_tab, total * 4, hipMemcpyDeviceToHost));
            const int32_t *counts = tab.data(), *tpe2 = tab.data() + (p[2] - d_tab);
            if (tab[p[9] - d_tab] != 0) { std::fprintf(stderr, "static layout: status %d\n", tab[p[9] - d_tab]); return 10; }
            for (int r = 0; r < N; ++r)
                if (tab[(p[8] - d_tab) + r] != 1) { std::fprintf(stderr, "static layout: plan_ok[%d]\n", r); return 11; }
            if (std::memcmp(tpe2, tpe.data(), tpe.size() * 4) != 0) {
                std::fprintf(stderr, "static layout: tokens_per_expert differs from the context's\n");
                return 12;
            }
            for (int s = 0; s < N; ++s)
                for (int e = 0; e < E; ++e) {
                    int c = 0;
                    for (int t = 0; t < nt[s]; ++t)
                        for (int k = 0; k < K; ++k) c += indices[((size_t)s * T + t) * K + k] == e;
                    if (counts[s * E + e] != c) { std::fprintf(stderr, "static layout: counts[%d][%d]\n", s, e); return 13; }
                }
        }
        fl_moe_config huge = cfg;
        huge.n_ranks = 32; huge.n_experts = 256; huge.max_tokens = 4096; huge.top_k = 8;
        if (fl_moe_layout_static(&huge, d_idx, d_nt, &lo, st) != FL_ERR_STATIC_LIMIT) {
            std::fprintf(stderr, "static layout: a configuration beyond the array was accepted\n");
            return 14;
        }
        HIP_OK(hipFree(d_tab));
    }

    FL_CALL(fl_moe_destroy(ctx));
    HIP_OK(hipStreamDestroy(st));
    HIP_OK(hipFree(ws)); HIP_OK(hipFree(d_x)); HIP_OK(hipFree(d_ex)); HIP_OK(hipFree(d_out));
    HIP_OK(hipFree(d_idx)); HIP_OK(hipFree(d_nt)); HIP_OK(hipFree(d_tpe)); HIP_OK(hipFree(d_w));
    std::printf("c abi roundtrip ok: %lld expert-major rows and %d tokens bit-exact\n", rows_checked,
                nt[0] + nt[1] + nt[2] + nt[3]);
    return 0;
}
