// tamoe_combine: y[t] = sum over the kept choices j of topk_w[t][j] * recv[slot[t][j]]
// (paper Section 3.1: the layer output aggregates the computed results).
//
// The 16-byte chunks of y are laid out flat over the threads, a few per thread, no loop and no
// LDS: a thread gathers the same chunk of the (up to k) source rows, accumulates in fp32 in
// ascending j with one fused multiply-add per term, rounds once to the storage type and writes
// the chunk of y.  Bound by HBM: d*b bytes read per kept pair, d*b written per token; the HBM
// latency is covered by the number of independent wavefronts, as in a plain copy.
#include "chunk.h"
#include "internal.h"

namespace tamoe {

constexpr int kThreads = 256;

// KK > 0: k is the compile-time constant KK; KK == 0: any k up to TAMOE_MAX_K.
// ROWU: a row is a multiple of 1 KiB, so the 64 chunks of a wavefront belong to one token and
// its slots and weights are read once per wavefront through the scalar unit.
// UNITW: every weight is 1 (the transpose of the scatter: dx[t] = sum of the rows its slots name).
template <int DT, int KK, int U, bool ROWU, bool UNITW>
__global__ __launch_bounds__(kThreads) void combine_kernel(const vec16* __restrict__ recv, int64_t K_rows,
                                                           const int32_t* __restrict__ slot,
                                                           const float* __restrict__ topk_w, int64_t total_chunks,
                                                           int k_arg, int cpr, int shift, vec16* __restrict__ y) {
    constexpr int KM = KK > 0 ? KK : TAMOE_MAX_K;
    const int k = KK > 0 ? KK : k_arg;
    const int64_t base = (int64_t)blockIdx.x * (kThreads * U) + threadIdx.x;
    vec16 v[U][KM];
    float wgt[U][KM];
    bool use[U][KM];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + (int64_t)u * kThreads;
#pragma unroll
        for (int j = 0; j < KM; ++j) use[u][j] = false;
        if (c < total_chunks) {
            int t, col;
            split_chunk(c, total_chunks, cpr, shift, t, col);
            if (ROWU) t = __builtin_amdgcn_readfirstlane(t);
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                if (j < k) {
                    const int32_t s = slot[(int64_t)t * k + j];
                    wgt[u][j] = UNITW ? 1.0f : topk_w[(int64_t)t * k + j];
                    use[u][j] = s >= 0 && (int64_t)s < K_rows;
                    if (use[u][j]) v[u][j] = __builtin_nontemporal_load(recv + (size_t)s * cpr + col);
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + (int64_t)u * kThreads;
        if (c >= total_chunks) continue;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KM; ++j)
            if (use[u][j]) Chunk<DT>::fma(acc, wgt[u][j], v[u][j]);
        __builtin_nontemporal_store(Chunk<DT>::pack(acc), y + c);
    }
}

template <int DT, int KK, int U>
static void launch_combine_k(const void* recv, int64_t K_rows, const int32_t* slot, const float* topk_w, int64_t S,
                             int k, int cpr, void* y, hipStream_t st) {
    const int64_t total = S * (int64_t)cpr;
    const dim3 grid((unsigned)ceil_div(total, kThreads * U)), block(kThreads);
    const vec16* r = static_cast<const vec16*>(recv);
    vec16* out = static_cast<vec16*>(y);
    const int shift = pow2_shift(cpr);
    const bool rowu = cpr % 64 == 0;
    if (topk_w != nullptr) {
        if (rowu)
            combine_kernel<DT, KK, U, true, false><<<grid, block, 0, st>>>(r, K_rows, slot, topk_w, total, k, cpr, shift, out);
        else
            combine_kernel<DT, KK, U, false, false><<<grid, block, 0, st>>>(r, K_rows, slot, topk_w, total, k, cpr, shift, out);
    } else {
        if (rowu)
            combine_kernel<DT, KK, U, true, true><<<grid, block, 0, st>>>(r, K_rows, slot, topk_w, total, k, cpr, shift, out);
        else
            combine_kernel<DT, KK, U, false, true><<<grid, block, 0, st>>>(r, K_rows, slot, topk_w, total, k, cpr, shift, out);
    }
}

// topk_w == nullptr: unit weights (tamoe_dispatch_bwd)
template <int DT>
static void launch_combine(const void* recv, int64_t K_rows, const int32_t* slot, const float* topk_w, int64_t S,
                           int k, int cpr, void* y, hipStream_t st) {
    TraceScope tr(topk_w != nullptr ? "combine_kernel" : "dispatch_bwd_kernel", st);
    if (k == 1)
        launch_combine_k<DT, 1, 2>(recv, K_rows, slot, topk_w, S, k, cpr, y, st);
    else if (k == 2)
        launch_combine_k<DT, 2, 1>(recv, K_rows, slot, topk_w, S, k, cpr, y, st);
    else
        launch_combine_k<DT, 0, 1>(recv, K_rows, slot, topk_w, S, k, cpr, y, st);
}

}  // namespace tamoe

using namespace tamoe;

static int combine_entry(const char* fn, const void* recv, int64_t K_rows, const int32_t* slot, const float* topk_w,
                         bool weighted, int dtype, int64_t S, int d, int k, void* y, void* stream) {
    clear_error();
    int rc;
    if (S < 0 || K_rows < 0) return fail(TAMOE_INVALID_ARG, "%s: S and K_rows must not be negative", fn);
    if (k <= 0) return fail(TAMOE_INVALID_ARG, "%s: k = %d must be positive", fn, k);
    if (k > TAMOE_MAX_K) return fail(TAMOE_UNSUPPORTED, "%s: k = %d exceeds the limit of %d", fn, k, TAMOE_MAX_K);
    if (S * (int64_t)k >= (int64_t)1 << 31) return fail(TAMOE_UNSUPPORTED, "%s: S*k does not fit int32", fn);
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if (S == 0) return TAMOE_OK;
    if (K_rows > 0 && (rc = check_ptr(fn, weighted ? "recv" : "d_send", recv, 16)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "slot", slot, 4)) != TAMOE_OK) return rc;
    if (weighted && (rc = check_ptr(fn, "topk_w", topk_w, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, weighted ? "y" : "d_x", y, 16)) != TAMOE_OK) return rc;
    const int cpr = d * elem_bytes(dtype) / 16;  // 16-byte chunks per row
    if (ceil_div(S * (int64_t)cpr, kThreads * 1) > 0x7fffffff)
        return fail(TAMOE_UNSUPPORTED, "%s: the output is too large for one launch", fn);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == TAMOE_F32)
        launch_combine<TAMOE_F32>(recv, K_rows, slot, weighted ? topk_w : nullptr, S, k, cpr, y, st);
    else if (dtype == TAMOE_F16)
        launch_combine<TAMOE_F16>(recv, K_rows, slot, weighted ? topk_w : nullptr, S, k, cpr, y, st);
    else
        launch_combine<TAMOE_BF16>(recv, K_rows, slot, weighted ? topk_w : nullptr, S, k, cpr, y, st);
    return check_launch(fn, "combine_kernel");
}

extern "C" int tamoe_combine(const void* recv, int64_t K_rows, const int32_t* slot, const float* topk_w, int dtype,
                             int64_t S, int d, int k, void* y, void* stream) {
    return combine_entry("tamoe_combine", recv, K_rows, slot, topk_w, true, dtype, S, d, k, y, stream);
}

extern "C" int tamoe_dispatch_bwd(const void* d_send, int64_t K_rows, const int32_t* slot, int dtype, int64_t S, int d,
                                  int k, void* d_x, void* stream) {
    return combine_entry("tamoe_dispatch_bwd", d_send, K_rows, slot, nullptr, false, dtype, S, d, k, d_x, stream);
}
