// tamoe_combine: y[t] = sum over the kept choices j of topk_w[t][j] * recv[slot[t][j]]
// (paper Section 3.1: the layer output aggregates the computed results).
//
// One workgroup per row tile of 4..64 tokens.  The 16-byte chunks of the tile are laid out flat
// over the threads; a thread gathers the same chunk of the (up to k) source rows, accumulates in
// fp32 in ascending j with one fused multiply-add per term, rounds once to the storage type and
// writes the chunk of y.  Bound by HBM: d*b bytes read per kept pair, d*b written per token.
#include "internal.h"

namespace tamoe {

constexpr int kThreads = 256;
constexpr int kMaxRowTile = 64;

template <int DT>
struct Chunk;

template <>
struct Chunk<TAMOE_F32> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void fma(float (&acc)[8], float w, vec16 v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(w, __uint_as_float(v[i]), acc[i]);
    }
    static __device__ __forceinline__ vec16 pack(const float (&acc)[8]) {
        vec16 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(acc[i]);
        return r;
    }
};

// fp32 -> bfloat16, round to nearest, ties to even (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <>
struct Chunk<TAMOE_BF16> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void fma(float (&acc)[8], float w, vec16 v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] = __builtin_fmaf(w, __uint_as_float(v[i] << 16), acc[2 * i]);
            acc[2 * i + 1] = __builtin_fmaf(w, __uint_as_float(v[i] & 0xffff0000u), acc[2 * i + 1]);
        }
    }
    static __device__ __forceinline__ vec16 pack(const float (&acc)[8]) {
        vec16 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = f32_to_bf16(acc[2 * i]) | (f32_to_bf16(acc[2 * i + 1]) << 16);
        return r;
    }
};

// KK > 0: k is the compile-time constant KK (all source loads of a chunk are issued together);
// KK == 0: any k up to TAMOE_MAX_K.
template <int DT, int KK, int U>
__global__ __launch_bounds__(kThreads) void combine_kernel(
    const vec16* __restrict__ recv, int64_t K_rows, const int32_t* __restrict__ slot,
    const float* __restrict__ topk_w, int64_t S, int k_arg, int row_tile, int cpr, vec16* __restrict__ y) {
    __shared__ int32_t s_slot[kMaxRowTile * TAMOE_MAX_K];
    __shared__ float s_w[kMaxRowTile * TAMOE_MAX_K];
    const int k = KK > 0 ? KK : k_arg;
    const int64_t t0 = (int64_t)blockIdx.x * row_tile;
    const int rows = (int)min((int64_t)row_tile, S - t0);
    for (int p = threadIdx.x; p < rows * k; p += kThreads) {
        const int32_t s = slot[t0 * k + p];
        s_slot[p] = (s >= 0 && (int64_t)s < K_rows) ? s : -1;
        s_w[p] = topk_w[t0 * k + p];
    }
    __syncthreads();

    const int total = rows * cpr;
    vec16* dst = y + (size_t)t0 * cpr;
    for (int base = 0; base < total; base += kThreads * U) {
        if constexpr (KK > 0) {
            vec16 v[U][KK];
            int32_t sl[U][KK];
            int row[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = base + u * kThreads + threadIdx.x;
                row[u] = -1;
                if (c < total) {
                    row[u] = c / cpr;
                    const int col = c - row[u] * cpr;
#pragma unroll
                    for (int j = 0; j < KK; ++j) {
                        sl[u][j] = s_slot[row[u] * KK + j];
                        if (sl[u][j] >= 0) v[u][j] = __builtin_nontemporal_load(recv + (size_t)sl[u][j] * cpr + col);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (row[u] < 0) continue;
                float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < KK; ++j)
                    if (sl[u][j] >= 0) Chunk<DT>::fma(acc, s_w[row[u] * KK + j], v[u][j]);
                __builtin_nontemporal_store(Chunk<DT>::pack(acc), dst + base + u * kThreads + threadIdx.x);
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = base + u * kThreads + threadIdx.x;
                if (c >= total) continue;
                const int r = c / cpr;
                const int col = c - r * cpr;
                float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                for (int j = 0; j < k; ++j) {
                    const int32_t s = s_slot[r * k + j];
                    if (s >= 0) Chunk<DT>::fma(acc, s_w[r * k + j], recv[(size_t)s * cpr + col]);
                }
                __builtin_nontemporal_store(Chunk<DT>::pack(acc), dst + c);
            }
        }
    }
}

template <int DT>
static void launch_combine(const void* recv, int64_t K_rows, const int32_t* slot, const float* topk_w, int64_t S,
                           int k, int rt, int cpr, void* y, hipStream_t st) {
    const dim3 grid((unsigned)ceil_div(S, rt)), block(kThreads);
    const vec16* r = static_cast<const vec16*>(recv);
    vec16* out = static_cast<vec16*>(y);
    TraceScope tr("combine_kernel", st);
    if (k == 1)
        combine_kernel<DT, 1, 4><<<grid, block, 0, st>>>(r, K_rows, slot, topk_w, S, k, rt, cpr, out);
    else if (k == 2)
        combine_kernel<DT, 2, 2><<<grid, block, 0, st>>>(r, K_rows, slot, topk_w, S, k, rt, cpr, out);
    else
        combine_kernel<DT, 0, 2><<<grid, block, 0, st>>>(r, K_rows, slot, topk_w, S, k, rt, cpr, out);
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_combine(const void* recv, int64_t K_rows, const int32_t* slot, const float* topk_w, int dtype,
                             int64_t S, int d, int k, void* y, void* stream) {
    const char* fn = "tamoe_combine";
    clear_error();
    int rc;
    if (S < 0 || K_rows < 0) return fail(TAMOE_INVALID_ARG, "%s: S and K_rows must not be negative", fn);
    if (k <= 0) return fail(TAMOE_INVALID_ARG, "%s: k = %d must be positive", fn, k);
    if (k > TAMOE_MAX_K) return fail(TAMOE_UNSUPPORTED, "%s: k = %d exceeds the limit of %d", fn, k, TAMOE_MAX_K);
    if (S * (int64_t)k >= (int64_t)1 << 31) return fail(TAMOE_UNSUPPORTED, "%s: S*k does not fit int32", fn);
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if (S == 0) return TAMOE_OK;
    if (K_rows > 0 && (rc = check_ptr(fn, "recv", recv, 16)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "slot", slot, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "topk_w", topk_w, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "y", y, 16)) != TAMOE_OK) return rc;
    const int row_bytes = d * elem_bytes(dtype);
    const int cpr = row_bytes / 16;
    if (cpr > 65536) return fail(TAMOE_UNSUPPORTED, "%s: rows longer than 1 MiB are not supported", fn);
    const int rt = row_tile(S, row_bytes);
    if (ceil_div(S, rt) > 0x7fffffff) return fail(TAMOE_UNSUPPORTED, "%s: too many row tiles", fn);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == TAMOE_F32)
        launch_combine<TAMOE_F32>(recv, K_rows, slot, topk_w, S, k, rt, cpr, y, st);
    else
        launch_combine<TAMOE_BF16>(recv, K_rows, slot, topk_w, S, k, rt, cpr, y, st);
    return check_launch(fn, "combine_kernel");
}
