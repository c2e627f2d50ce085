// Backward of the path, for training with the auxiliary loss added to the train loss (paper
// Sections 3.1 and 4.3):
//   tamoe_gate_bwd     gradient to the gate scores through the softmax: from the combine weights
//                      and from l_topo (or l_aux), routing fixed
//   tamoe_combine_bwd  transpose of the combine: d_recv (weighted scatter of dy) and d_topk_w
//                      (one dot product per kept pair)
// (tamoe_dispatch_bwd, the transpose of the scatter, is the combine kernel with unit weights.)
#include <climits>

#include "chunk.h"
#include "internal.h"

namespace tamoe {

constexpr int kThreads = 256;

// ---- combine backward: one wavefront per token ------------------------------------------------
// The wavefront walks its row of dy in steps of 64 chunks (1 KiB), two steps per batch: all loads
// of a batch (dy and the k source rows of recv) are issued before anything is stored, because
// stores and loads retire in one order and a store-then-load loop would wait for the stores.
// d_w is a fixed-order sum: per lane over its chunks, then a butterfly over the lanes.
template <int DT, int KK>
__global__ __launch_bounds__(kThreads) void combine_bwd_kernel(const vec16* __restrict__ dy,
                                                               const vec16* __restrict__ recv, int64_t K_rows,
                                                               const int32_t* __restrict__ slot,
                                                               const float* __restrict__ topk_w, int64_t S, int k_arg,
                                                               int cpr, vec16* __restrict__ d_recv,
                                                               float* __restrict__ d_w) {
    constexpr int KM = KK > 0 ? KK : TAMOE_MAX_K;
    constexpr int UB = 2;
    const int k = KK > 0 ? KK : k_arg;
    const int lane = threadIdx.x & 63;
    const int64_t t64 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
    if (t64 >= S) return;  // whole wavefront
    const int t = __builtin_amdgcn_readfirstlane((int)t64);
    int32_t s[KM];
    float w[KM], dot[KM];
#pragma unroll
    for (int j = 0; j < KM; ++j) {
        s[j] = -1;
        w[j] = 0.f;
        dot[j] = 0.f;
        if (j < k) {
            const int32_t sj = slot[(int64_t)t * k + j];
            s[j] = (sj >= 0 && (int64_t)sj < K_rows) ? sj : -1;
            w[j] = topk_w[(int64_t)t * k + j];
        }
    }
    const vec16* grow = dy + (size_t)t * cpr;
    for (int c0 = 0; c0 < cpr; c0 += 64 * UB) {
        vec16 g[UB], r[UB][KM];
        bool ok[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int c = c0 + u * 64 + lane;
            ok[u] = c < cpr;
            if (ok[u]) {
                g[u] = __builtin_nontemporal_load(grow + c);
#pragma unroll
                for (int j = 0; j < KM; ++j)
                    if (s[j] >= 0) r[u][j] = __builtin_nontemporal_load(recv + (size_t)s[j] * cpr + c);
            }
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            if (!ok[u]) continue;
            const int c = c0 + u * 64 + lane;
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                if (s[j] < 0) continue;
                dot[j] = chunk_dot<DT>(g[u], r[u][j], dot[j]);
                float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                Chunk<DT>::fma(acc, w[j], g[u]);
                __builtin_nontemporal_store(Chunk<DT>::pack(acc), d_recv + (size_t)s[j] * cpr + c);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < KM; ++j) {
        if (j < k) {
            float v = dot[j];
            v += __shfl_xor(v, 32);
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 8);
            v += __shfl_xor(v, 4);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 1);
            if (lane == 0) d_w[(int64_t)t * k + j] = s[j] >= 0 ? v : 0.f;
        }
    }
}

// ---- gate backward: the accumulator layout of the gate's selection stage ----------------------
__device__ __forceinline__ int expert_at(int nb, int v, int half) {
    return nb * 32 + ((v >> 2) << 3) + (half << 2) + (v & 3);
}

// One wavefront per 32 tokens; lane l holds, for token (l & 31), the experts expert_at(nb, v, l>>5),
// and the lane pair (l, l^32) a token's whole score vector.
//   u[e]  = coef[e] + sum_j d_w[t][j] * [idx[t][j] == e],   coef[e] = scale * p[e] * c[e]
//   dl[e] = G[e] * (u[e] - sum_e' u[e'] G[e'])
template <int NB>
__global__ __launch_bounds__(kThreads) void gate_bwd_kernel(const float* __restrict__ logits,
                                                            const int32_t* __restrict__ idx,
                                                            const float* __restrict__ d_w,
                                                            const float* __restrict__ penalty,
                                                            const int32_t* __restrict__ c, float scale, int64_t S,
                                                            int N, int k, float* __restrict__ d_logits) {
    __shared__ float coef[NB * 32];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    for (int e = tid; e < NB * 32; e += kThreads)
        coef[e] = e < N ? scale * (penalty != nullptr ? penalty[e] : 1.0f) * (float)c[e] : 0.f;
    __syncthreads();
    const int64_t token = ((int64_t)blockIdx.x * 4 + wave) * 32 + (lane & 31);
    const bool token_ok = token < S;
    const int64_t tk = token_ok ? token : 0;

    int sel[TAMOE_MAX_K];
    float dwt[TAMOE_MAX_K];
#pragma unroll
    for (int j = 0; j < TAMOE_MAX_K; ++j) {
        sel[j] = -1;
        dwt[j] = 0.f;
        if (j < k && token_ok) {
            sel[j] = idx[tk * k + j];
            dwt[j] = d_w[tk * k + j];
        }
    }
    float sc[NB][16];
    float mx = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int e = expert_at(nb, v, half);
            sc[nb][v] = (token_ok && e < N) ? logits[(size_t)tk * N + e] : -INFINITY;
            mx = fmaxf(mx, sc[nb][v]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (!token_ok) mx = 0.f;
    float part = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            sc[nb][v] = __builtin_amdgcn_exp2f((sc[nb][v] - mx) * 1.44269504088896340736f);
            part += sc[nb][v];
        }
    const float den = part + __shfl_xor(part, 32);
    const float inv = token_ok ? 1.0f / den : 0.f;
    float ubar = 0.f;
    float u[NB][16];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int e = expert_at(nb, v, half);
            float uu = coef[e];
#pragma unroll
            for (int j = 0; j < TAMOE_MAX_K; ++j)
                if (j < k && sel[j] == e) uu += dwt[j];
            sc[nb][v] *= inv;  // G
            u[nb][v] = uu;
            ubar = __builtin_fmaf(uu, sc[nb][v], ubar);
        }
    ubar += __shfl_xor(ubar, 32);
    if (token_ok) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int e = expert_at(nb, v, half);
                if (e < N) d_logits[(size_t)token * N + e] = sc[nb][v] * (u[nb][v] - ubar);
            }
    }
}

template <int DT>
static void launch_combine_bwd(const void* dy, const void* recv, int64_t K_rows, const int32_t* slot,
                               const float* topk_w, int64_t S, int k, int cpr, void* d_recv, float* d_w,
                               hipStream_t st) {
    const dim3 grid((unsigned)ceil_div(S, kThreads / 64)), block(kThreads);
    const vec16* g = static_cast<const vec16*>(dy);
    const vec16* r = static_cast<const vec16*>(recv);
    vec16* o = static_cast<vec16*>(d_recv);
    TraceScope tr("combine_bwd_kernel", st);
    if (k == 1)
        combine_bwd_kernel<DT, 1><<<grid, block, 0, st>>>(g, r, K_rows, slot, topk_w, S, k, cpr, o, d_w);
    else if (k == 2)
        combine_bwd_kernel<DT, 2><<<grid, block, 0, st>>>(g, r, K_rows, slot, topk_w, S, k, cpr, o, d_w);
    else
        combine_bwd_kernel<DT, 0><<<grid, block, 0, st>>>(g, r, K_rows, slot, topk_w, S, k, cpr, o, d_w);
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_combine_bwd(const void* dy, const void* recv, int64_t K_rows, const int32_t* slot,
                                 const float* topk_w, int dtype, int64_t S, int d, int k, void* d_recv,
                                 float* d_topk_w, void* stream) {
    const char* fn = "tamoe_combine_bwd";
    clear_error();
    int rc;
    if (S < 0 || K_rows < 0) return fail(TAMOE_INVALID_ARG, "%s: S and K_rows must not be negative", fn);
    if (k <= 0) return fail(TAMOE_INVALID_ARG, "%s: k = %d must be positive", fn, k);
    if (k > TAMOE_MAX_K) return fail(TAMOE_UNSUPPORTED, "%s: k = %d exceeds the limit of %d", fn, k, TAMOE_MAX_K);
    if (S * (int64_t)k >= (int64_t)1 << 31) return fail(TAMOE_UNSUPPORTED, "%s: S*k does not fit int32", fn);
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if (S == 0) return TAMOE_OK;
    if ((rc = check_ptr(fn, "dy", dy, 16)) != TAMOE_OK) return rc;
    if (K_rows > 0 && (rc = check_ptr(fn, "recv", recv, 16)) != TAMOE_OK) return rc;
    if (K_rows > 0 && (rc = check_ptr(fn, "d_recv", d_recv, 16)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "slot", slot, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "topk_w", topk_w, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "d_topk_w", d_topk_w, 4)) != TAMOE_OK) return rc;
    const int cpr = d * elem_bytes(dtype) / 16;
    if (ceil_div(S, kThreads / 64) > 0x7fffffff) return fail(TAMOE_UNSUPPORTED, "%s: too many tokens for one launch", fn);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == TAMOE_F32)
        launch_combine_bwd<TAMOE_F32>(dy, recv, K_rows, slot, topk_w, S, k, cpr, d_recv, d_topk_w, st);
    else
        launch_combine_bwd<TAMOE_BF16>(dy, recv, K_rows, slot, topk_w, S, k, cpr, d_recv, d_topk_w, st);
    return check_launch(fn, "combine_bwd_kernel");
}

extern "C" int tamoe_gate_bwd(const float* logits, const int32_t* topk_idx, const float* d_topk_w,
                              const float* penalty, const int32_t* c_expert, float loss_scale, int64_t S, int N, int P,
                              int k, float* d_logits, void* stream) {
    const char* fn = "tamoe_gate_bwd";
    clear_error();
    int rc;
    if ((rc = check_shape(fn, S, N, P, k)) != TAMOE_OK) return rc;
    if (S == 0) return TAMOE_OK;
    if ((rc = check_ptr(fn, "logits", logits, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "topk_idx", topk_idx, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "d_topk_w", d_topk_w, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "c_expert", c_expert, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "d_logits", d_logits, 4)) != TAMOE_OK) return rc;
    if (penalty != nullptr && (rc = check_ptr(fn, "penalty", penalty, 4)) != TAMOE_OK) return rc;
    // d l_topo / d G[t][e] = loss_scale * N*P * p[e] * c[e] / S^2 (l_aux: no N*P, unit weights); the
    // part that does not depend on e is folded into one fp32 factor on the host, in double
    const float scale =
        (float)((double)loss_scale * (penalty != nullptr ? (double)N * (double)P : 1.0) / ((double)S * (double)S));
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)ceil_div(S, 128)), block(kThreads);
    {
        TraceScope tr("gate_bwd_kernel", st);
        if (N <= 32)
            gate_bwd_kernel<1><<<grid, block, 0, st>>>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits);
        else if (N <= 64)
            gate_bwd_kernel<2><<<grid, block, 0, st>>>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits);
        else
            gate_bwd_kernel<4><<<grid, block, 0, st>>>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits);
    }
    return check_launch(fn, "gate_bwd_kernel");
}
