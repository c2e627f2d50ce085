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
// The wavefront walks its row of dy in steps of 64 chunks (1 KiB), four steps per batch: all loads
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
    constexpr int UB = 4;
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

// ---- combine backward, rows of 64 * 2^n chunks (1 KiB .. 16 KiB), k <= 2 --------------------------
// One 16-byte chunk per thread, no loop: like the forward row movers, the thread issues its loads
// (dy and the k source rows), then its k stores.  A token's row spans cpr / 64 whole wavefronts of
// one workgroup; the dot products are reduced by a butterfly inside the wavefront and then summed
// over the row's wavefronts in ascending order by the row's first lane (fixed order).
template <int DT, int KK, int WG>
__global__ __launch_bounds__(WG) void combine_bwd_flat_kernel(const vec16* __restrict__ dy,
                                                              const vec16* __restrict__ recv, int64_t K_rows,
                                                              const int32_t* __restrict__ slot,
                                                              const float* __restrict__ topk_w, int64_t S, int shift,
                                                              vec16* __restrict__ d_recv, float* __restrict__ d_w) {
    __shared__ float part[WG / 64][KK];
    const int cpr = 1 << shift;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t c = (int64_t)blockIdx.x * WG + threadIdx.x;
    const int64_t tok = c >> shift;  // the same for the whole wavefront: cpr >= 64
    const bool live = tok < S;
    const int t = __builtin_amdgcn_readfirstlane(live ? (int)tok : 0);
    const int col = (int)c & (cpr - 1);
    int32_t s[KK];
    float w[KK], dot[KK];
#pragma unroll
    for (int j = 0; j < KK; ++j) {
        const int32_t sj = live ? slot[(int64_t)t * KK + j] : -1;
        s[j] = (sj >= 0 && (int64_t)sj < K_rows) ? sj : -1;
        w[j] = topk_w[(int64_t)t * KK + j];
        dot[j] = 0.f;
    }
    if (live) {
        const vec16 g = __builtin_nontemporal_load(dy + c);
        vec16 r[KK];
#pragma unroll
        for (int j = 0; j < KK; ++j)
            if (s[j] >= 0) r[j] = __builtin_nontemporal_load(recv + (size_t)s[j] * cpr + col);
#pragma unroll
        for (int j = 0; j < KK; ++j) {
            if (s[j] < 0) continue;
            dot[j] = chunk_dot<DT>(g, r[j], 0.f);
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            Chunk<DT>::fma(acc, w[j], g);
            __builtin_nontemporal_store(Chunk<DT>::pack(acc), d_recv + (size_t)s[j] * cpr + col);
        }
    }
#pragma unroll
    for (int j = 0; j < KK; ++j) {
        float v = dot[j];
        v += __shfl_xor(v, 32);
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 8);
        v += __shfl_xor(v, 4);
        v += __shfl_xor(v, 2);
        v += __shfl_xor(v, 1);
        if (lane == 0) part[wave][j] = v;
    }
    __syncthreads();
    const int wpr = cpr >> 6;  // wavefronts per row
    if (live && lane == 0 && (wave & (wpr - 1)) == 0) {
#pragma unroll
        for (int j = 0; j < KK; ++j) {
            float v = 0.f;
            for (int i = 0; i < wpr; ++i) v += part[wave + i][j];
            d_w[(int64_t)t * KK + j] = s[j] >= 0 ? v : 0.f;
        }
    }
}

// ---- gate backward ------------------------------------------------------------------------------
// value of lane (lane ^ MASK), MASK < 32, through the LDS crossbar
template <int MASK>
__device__ __forceinline__ float lane_xor(float v) {
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), (MASK << 10) | 0x1f));
}
template <int LPT>
__device__ __forceinline__ float group_max(float v) {
    if constexpr (LPT > 1) v = fmaxf(v, lane_xor<1>(v));
    if constexpr (LPT > 2) v = fmaxf(v, lane_xor<2>(v));
    if constexpr (LPT > 4) v = fmaxf(v, lane_xor<4>(v));
    if constexpr (LPT > 8) v = fmaxf(v, lane_xor<8>(v));
    if constexpr (LPT > 16) v = fmaxf(v, lane_xor<16>(v));
    return v;
}
template <int LPT>
__device__ __forceinline__ float group_sum(float v) {
    if constexpr (LPT > 1) v += lane_xor<1>(v);
    if constexpr (LPT > 2) v += lane_xor<2>(v);
    if constexpr (LPT > 4) v += lane_xor<4>(v);
    if constexpr (LPT > 8) v += lane_xor<8>(v);
    if constexpr (LPT > 16) v += lane_xor<16>(v);
    return v;
}

// A token's score row is spread over LPT consecutive lanes, four consecutive experts per lane
// (4*LPT >= N), so that a wavefront reads and writes whole rows contiguously; the three
// reductions of a row (max, sum of exponentials, sum of u*G) are butterflies over those lanes.
//   u[e]  = coef[e] + sum_j d_w[t][j] * [idx[t][j] == e],   coef[e] = scale * p[e] * c[e]
//   dl[e] = G[e] * (u[e] - sum_e' u[e'] G[e'])
// VEC: N is a multiple of 4, rows are 16-byte aligned and each lane moves one dwordx4.
template <int LPT, bool VEC>
__global__ __launch_bounds__(kThreads) void gate_bwd_kernel(const float* __restrict__ logits,
                                                            const int32_t* __restrict__ idx,
                                                            const float* __restrict__ d_w,
                                                            const float* __restrict__ penalty,
                                                            const int32_t* __restrict__ c, float scale, int64_t S,
                                                            int N, int k, float* __restrict__ d_logits) {
    __shared__ float coef[TAMOE_MAX_EXPERTS + 4];
    const int tid = threadIdx.x;
    for (int e = tid; e < TAMOE_MAX_EXPERTS + 4; e += kThreads)
        coef[e] = e < N ? scale * (penalty != nullptr ? penalty[e] : 1.0f) * (float)c[e] : 0.f;
    __syncthreads();
    const int64_t token = ((int64_t)blockIdx.x * kThreads + tid) / LPT;
    const int e0 = (tid % LPT) * 4;
    const bool token_ok = token < S;
    const int64_t tk = token_ok ? token : 0;
    const float* row = logits + (size_t)tk * N;

    float l[4];
    if (VEC) {
        const float4 q = (token_ok && e0 < N) ? *reinterpret_cast<const float4*>(row + e0)
                                             : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        l[0] = q.x; l[1] = q.y; l[2] = q.z; l[3] = q.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) l[i] = (token_ok && e0 + i < N) ? row[e0 + i] : -INFINITY;
    }
    float mx = group_max<LPT>(fmaxf(fmaxf(l[0], l[1]), fmaxf(l[2], l[3])));
    if (!token_ok) mx = 0.f;
    float g[4], part = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        g[i] = __builtin_amdgcn_exp2f((l[i] - mx) * 1.44269504088896340736f);
        part += g[i];
    }
    const float den = group_sum<LPT>(part);
    const float inv = token_ok ? 1.0f / den : 0.f;
    float u[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        g[i] *= inv;
        u[i] = coef[e0 + i];
    }
    for (int j = 0; j < k; ++j) {
        const int sel = token_ok ? idx[tk * k + j] : -1;
        const float dwt = token_ok ? d_w[tk * k + j] : 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] += (sel == e0 + i) ? dwt : 0.f;
    }
    float ub = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) ub = __builtin_fmaf(u[i], g[i], ub);
    const float ubar = group_sum<LPT>(ub);
    if (token_ok) {
        float* out = d_logits + (size_t)token * N;
        if (VEC) {
            if (e0 < N)
                *reinterpret_cast<float4*>(out + e0) =
                    make_float4(g[0] * (u[0] - ubar), g[1] * (u[1] - ubar), g[2] * (u[2] - ubar), g[3] * (u[3] - ubar));
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (e0 + i < N) out[e0 + i] = g[i] * (u[i] - ubar);
        }
    }
}

template <int LPT>
static void launch_gate_bwd(const float* logits, const int32_t* idx, const float* d_w, const float* penalty,
                            const int32_t* c, float scale, int64_t S, int N, int k, float* d_logits, hipStream_t st) {
    const dim3 grid((unsigned)ceil_div(S * LPT, kThreads)), block(kThreads);
    const bool vec = N % 4 == 0 && reinterpret_cast<uintptr_t>(logits) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(d_logits) % 16 == 0;
    if (vec)
        gate_bwd_kernel<LPT, true><<<grid, block, 0, st>>>(logits, idx, d_w, penalty, c, scale, S, N, k, d_logits);
    else
        gate_bwd_kernel<LPT, false><<<grid, block, 0, st>>>(logits, idx, d_w, penalty, c, scale, S, N, k, d_logits);
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
    const int shift = pow2_shift(cpr);
    if (k <= 2 && shift >= 6 && shift <= 10) {
        // rows of 1, 2, 4 KiB share a 256-thread workgroup; 8 and 16 KiB rows take one of their own
        const int wg = cpr <= 256 ? 256 : cpr;
        const dim3 fgrid((unsigned)ceil_div(S * (int64_t)cpr, wg)), fblock(wg);
#define TAMOE_FLAT(KK, WG) \
    combine_bwd_flat_kernel<DT, KK, WG><<<fgrid, fblock, 0, st>>>(g, r, K_rows, slot, topk_w, S, shift, o, d_w)
        if (k == 1) {
            if (wg == 256) TAMOE_FLAT(1, 256); else if (wg == 512) TAMOE_FLAT(1, 512); else TAMOE_FLAT(1, 1024);
        } else {
            if (wg == 256) TAMOE_FLAT(2, 256); else if (wg == 512) TAMOE_FLAT(2, 512); else TAMOE_FLAT(2, 1024);
        }
#undef TAMOE_FLAT
        return;
    }
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
    else if (dtype == TAMOE_F16)
        launch_combine_bwd<TAMOE_F16>(dy, recv, K_rows, slot, topk_w, S, k, cpr, d_recv, d_topk_w, st);
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
    if (ceil_div(S * 32, kThreads) > 0x7fffffff) return fail(TAMOE_UNSUPPORTED, "%s: too many tokens for one launch", fn);
    {
        TraceScope tr("gate_bwd_kernel", st);
        if (N <= 4)
            launch_gate_bwd<1>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits, st);
        else if (N <= 8)
            launch_gate_bwd<2>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits, st);
        else if (N <= 16)
            launch_gate_bwd<4>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits, st);
        else if (N <= 32)
            launch_gate_bwd<8>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits, st);
        else if (N <= 64)
            launch_gate_bwd<16>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits, st);
        else
            launch_gate_bwd<32>(logits, topk_idx, d_topk_w, penalty, c_expert, scale, S, N, k, d_logits, st);
    }
    return check_launch(fn, "gate_bwd_kernel");
}
