// tamoe_regroup: the step right after the global exchange (paper Section 3.1: each expert
// receives a combined batch of tokens).  The receive buffer holds one chunk per source device,
// each chunk grouped by local expert; the experts need one contiguous batch each.  Regrouping is
// a permutation of P*E contiguous row segments (and its inverse before the return exchange): a
// pure copy, bound by HBM (2 * R * d * b bytes for R rows).
//
// Two launches: one workgroup turns the P*E counts into the two offset tables (source-major and
// expert-major) in the workspace; the copy kernel maps every 16-byte chunk to its segment by a
// binary search over at most 129 offsets held in LDS.
#include "internal.h"
#include "scan128.h"

namespace tamoe {

constexpr int kThreads = 256;
constexpr int kMaxSeg = TAMOE_MAX_EXPERTS;  // P * E <= 128

// tables[0 .. n]: offsets of the segments in source-major order g = s*E + e
// tables[kMaxSeg+1 .. ]: offsets of the same segments in expert-major order h = e*P + s
__global__ __launch_bounds__(kThreads) void regroup_offsets_kernel(const int32_t* __restrict__ cnt, int P, int E,
                                                                   int32_t* __restrict__ tables,
                                                                   int32_t* __restrict__ expert_offset) {
    __shared__ int32_t v[kMaxSeg], off[kMaxSeg + 1], tmp[2 * 128];
    const int n = P * E;
    const int t = threadIdx.x;
    if (t < n) v[t] = cnt[t] < 0 ? 0 : cnt[t];
    __syncthreads();
    exclusive_scan_128(v, off, tmp, n);
    if (t <= n) tables[t] = off[t];
    __syncthreads();
    if (t < n) {  // expert-major order: entry h = e*P + s holds segment g = s*E + e
        const int e = t / P, s = t - e * P;
        const int32_t c = cnt[s * E + e];
        v[t] = c < 0 ? 0 : c;
    }
    __syncthreads();
    exclusive_scan_128(v, off, tmp, n);
    if (t <= n) tables[kMaxSeg + 1 + t] = off[t];
    if (expert_offset != nullptr && t <= E) expert_offset[t] = off[t * P];
}

template <int U>
__global__ __launch_bounds__(kThreads) void regroup_copy_kernel(const vec16* __restrict__ in,
                                                                const int32_t* __restrict__ tables, int P, int E,
                                                                int64_t cap_rows, int cpr, int shift, int to_expert_major,
                                                                vec16* __restrict__ out) {
    __shared__ int32_t from_off[kMaxSeg + 1], to_off[kMaxSeg + 1];
    const int n = P * E;
    // the input is read in `from` order; the segment found there is looked up in `to` order
    const int32_t* from_tab = tables + (to_expert_major ? 0 : kMaxSeg + 1);
    const int32_t* to_tab = tables + (to_expert_major ? kMaxSeg + 1 : 0);
    for (int i = threadIdx.x; i <= n; i += kThreads) {
        from_off[i] = from_tab[i];
        to_off[i] = to_tab[i];
    }
    __syncthreads();
    const int64_t R = from_off[n] < cap_rows ? from_off[n] : cap_rows;
    const int64_t total = R * cpr;
    const int64_t base = (int64_t)blockIdx.x * (kThreads * U) + threadIdx.x;
    vec16 v[U];
    int64_t dst[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + (int64_t)u * kThreads;
        dst[u] = -1;
        if (c < total) {
            int row, col;
            split_chunk(c, total, cpr, shift, row, col);
            int lo = 0, hi = n;  // largest lo with from_off[lo] <= row (empty segments are skipped)
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (from_off[mid] <= row) lo = mid; else hi = mid;
            }
            // lo indexes the `from` order; the same segment in the `to` order
            int other;
            if (to_expert_major) { const int s = lo / E, e = lo - s * E; other = e * P + s; }
            else                 { const int e = lo / P, s = lo - e * P; other = s * E + e; }
            const int64_t drow = (int64_t)to_off[other] + (row - from_off[lo]);
            if (drow < cap_rows) {
                dst[u] = drow * cpr + col;
                v[u] = __builtin_nontemporal_load(in + c);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (dst[u] >= 0) __builtin_nontemporal_store(v[u], out + dst[u]);
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_regroup(const void* in, const int32_t* recv_count, int P, int E, int dtype, int d,
                             int64_t cap_rows, int to_expert_major, void* out, int32_t* expert_offset, void* ws,
                             size_t ws_bytes, void* stream) {
    const char* fn = "tamoe_regroup";
    clear_error();
    int rc;
    if (P <= 0 || E <= 0) return fail(TAMOE_INVALID_ARG, "%s: P = %d and E = %d must be positive", fn, P, E);
    if ((int64_t)P * E > kMaxSeg)
        return fail(TAMOE_UNSUPPORTED, "%s: P*E = %lld exceeds the limit of %d segments", fn, (long long)P * E, kMaxSeg);
    if (cap_rows < 0 || cap_rows >= ((int64_t)1 << 31))
        return fail(TAMOE_INVALID_ARG, "%s: cap_rows = %lld outside [0, 2^31)", fn, (long long)cap_rows);
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "recv_count", recv_count, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "ws", ws, 256)) != TAMOE_OK) return rc;
    const size_t need = 2 * (kMaxSeg + 1) * sizeof(int32_t);
    if (ws_bytes < need) return fail(TAMOE_WORKSPACE_TOO_SMALL, "%s: workspace has %zu bytes, %zu needed", fn, ws_bytes, need);
    if (cap_rows > 0) {
        if ((rc = check_ptr(fn, "in", in, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "out", out, 16)) != TAMOE_OK) return rc;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t* tables = static_cast<int32_t*>(ws);
    {
        TraceScope tr("regroup_offsets_kernel", st);
        regroup_offsets_kernel<<<dim3(1), dim3(kThreads), 0, st>>>(recv_count, P, E, tables, expert_offset);
    }
    if ((rc = check_launch(fn, "regroup_offsets_kernel")) != TAMOE_OK) return rc;
    if (cap_rows == 0) return TAMOE_OK;
    const int cpr = d * elem_bytes(dtype) / 16;
    // two chunks per thread: the offset tables are loaded once per 8 KiB instead of once per 4 KiB
    // (2 GiB: 377 -> 341 us; four chunks: 350 us)
    constexpr int kChunksPerThread = 2;
    const int64_t blocks = ceil_div(cap_rows * cpr, kThreads * kChunksPerThread);
    if (blocks > 0x7fffffff) return fail(TAMOE_UNSUPPORTED, "%s: the buffer is too large for one launch", fn);
    {
        TraceScope tr("regroup_copy_kernel", st);
        regroup_copy_kernel<kChunksPerThread><<<dim3((unsigned)blocks), dim3(kThreads), 0, st>>>(
            static_cast<const vec16*>(in), tables, P, E, cap_rows, cpr, pow2_shift(cpr), to_expert_major ? 1 : 0,
            static_cast<vec16*>(out));
    }
    return check_launch(fn, "regroup_copy_kernel");
}
