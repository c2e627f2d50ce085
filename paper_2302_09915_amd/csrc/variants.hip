// Variants of the weighting: combine weights renormalised over a token's k selected experts and
// the transpose of that map.  O(S*k) words, one thread per token, rows read and written as they
// lie in memory (a wavefront touches 64*k consecutive floats).
#include "internal.h"

namespace tamoe {

constexpr int kThreads = 256;

template <int KK>
__global__ __launch_bounds__(kThreads) void renorm_topk_kernel(const float* __restrict__ w, int64_t S, int k_arg,
                                                               float* __restrict__ out) {
    constexpr int KM = KK > 0 ? KK : TAMOE_MAX_K;
    const int k = KK > 0 ? KK : k_arg;
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= S) return;
    float v[KM];
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < KM; ++j) {
        v[j] = j < k ? w[t * k + j] : 0.0f;
        s += v[j];  // ascending j
    }
#pragma unroll
    for (int j = 0; j < KM; ++j)
        if (j < k) out[t * k + j] = v[j] / s;
}

template <int KK>
__global__ __launch_bounds__(kThreads) void renorm_topk_bwd_kernel(const float* __restrict__ w,
                                                                   const float* __restrict__ d_out, int64_t S,
                                                                   int k_arg, float* __restrict__ d_w) {
    constexpr int KM = KK > 0 ? KK : TAMOE_MAX_K;
    const int k = KK > 0 ? KK : k_arg;
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= S) return;
    float g[KM];
    float s = 0.0f, dot = 0.0f;
#pragma unroll
    for (int j = 0; j < KM; ++j) {
        const float v = j < k ? w[t * k + j] : 0.0f;
        g[j] = j < k ? d_out[t * k + j] : 0.0f;
        s += v;
        dot = fmaf(g[j], v, dot);
    }
    const float inv = 1.0f / s;
    const float shift = dot * inv * inv;
#pragma unroll
    for (int j = 0; j < KM; ++j)
        if (j < k) d_w[t * k + j] = fmaf(g[j], inv, -shift);
}

static int check_renorm(const char* fn, int64_t S, int k) {
    if (S < 0 || S * (int64_t)TAMOE_MAX_K >= ((int64_t)1 << 31))
        return fail(TAMOE_INVALID_ARG, "%s: S = %lld outside [0, 2^31 / %d)", fn, (long long)S, TAMOE_MAX_K);
    if (k < 1) return fail(TAMOE_INVALID_ARG, "%s: k = %d must be positive", fn, k);
    if (k > TAMOE_MAX_K) return fail(TAMOE_UNSUPPORTED, "%s: k = %d exceeds %d", fn, k, TAMOE_MAX_K);
    return TAMOE_OK;
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_renorm_topk(const float* topk_w, int64_t S, int k, float* out, void* stream) {
    const char* fn = "tamoe_renorm_topk";
    clear_error();
    int rc;
    if ((rc = check_renorm(fn, S, k)) != TAMOE_OK) return rc;
    if (S == 0) return TAMOE_OK;
    if ((rc = check_ptr(fn, "topk_w", topk_w, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "out", out, 4)) != TAMOE_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)ceil_div(S, kThreads)), block(kThreads);
    {
        TraceScope tr("renorm_topk_kernel", st);
        if (k == 1)
            renorm_topk_kernel<1><<<grid, block, 0, st>>>(topk_w, S, k, out);
        else if (k == 2)
            renorm_topk_kernel<2><<<grid, block, 0, st>>>(topk_w, S, k, out);
        else
            renorm_topk_kernel<0><<<grid, block, 0, st>>>(topk_w, S, k, out);
    }
    return check_launch(fn, "renorm_topk_kernel");
}

extern "C" int tamoe_renorm_topk_bwd(const float* topk_w, const float* d_out, int64_t S, int k, float* d_topk_w,
                                     void* stream) {
    const char* fn = "tamoe_renorm_topk_bwd";
    clear_error();
    int rc;
    if ((rc = check_renorm(fn, S, k)) != TAMOE_OK) return rc;
    if (S == 0) return TAMOE_OK;
    if ((rc = check_ptr(fn, "topk_w", topk_w, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "d_out", d_out, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "d_topk_w", d_topk_w, 4)) != TAMOE_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)ceil_div(S, kThreads)), block(kThreads);
    {
        TraceScope tr("renorm_topk_bwd_kernel", st);
        if (k == 1)
            renorm_topk_bwd_kernel<1><<<grid, block, 0, st>>>(topk_w, d_out, S, k, d_topk_w);
        else if (k == 2)
            renorm_topk_bwd_kernel<2><<<grid, block, 0, st>>>(topk_w, d_out, S, k, d_topk_w);
        else
            renorm_topk_bwd_kernel<0><<<grid, block, 0, st>>>(topk_w, d_out, S, k, d_topk_w);
    }
    return check_launch(fn, "renorm_topk_bwd_kernel");
}
