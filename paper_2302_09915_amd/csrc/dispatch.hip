// tamoe_dispatch: capacity-limited slot assignment by prefix scans, and the row scatter into the
// destination-grouped send buffer (paper Section 3.1: dispatched data [k*S, d], local capacity;
// Section 4.1: one merged delivery per destination device; Section 4.3: variable chunk sizes).
//
// Four launches (five for the fixed-size padded layout), no atomics on positions, so the result is
// the same on every run:
//   1. dispatch_count_kernel  pairs per (choice j, count tile of 1024 tokens, expert)
//   2. dispatch_scan_kernel   exclusive prefix of those counts in priority order (choice-major,
//                             then token order), kept = min(count, cap), expert offsets, rows per
//                             destination device
//   3. dispatch_slot_kernel   one workgroup per 64 tokens: recount the pairs of the count tile
//                             that precede them, rank the 64 tokens' own pairs, write slot[]
//   4. dispatch_copy_kernel   streams the rows: each thread owns one 16-byte chunk of x (two for
//                             k = 1), reads it once if its token has a kept choice and stores it
//                             to each of the token's slots.  No loop and no LDS: like a plain
//                             copy, the latency of HBM is covered by the number of independent
//                             wavefronts.
//   5. dispatch_pad_fill_kernel (tamoe_dispatch_padded only) zeroes every expert's unused rows.
//
// The copy is bound by HBM: it reads d*b bytes per token with a kept choice and writes d*b
// bytes per kept pair.  Chunks are laid out flat over the threads, so a wavefront always touches
// 1 KiB of consecutive bytes, whatever d is.
#include <algorithm>
#include <mutex>

#include "internal.h"
#include "scan128.h"

namespace tamoe {

constexpr int kThreads = 256;
constexpr int kSlotTile = 64;  // tokens per slot-assignment workgroup; divides kCountTile

// hist[j*N + e] += number of pairs p in [p_begin, p_end) with idx[p] == e, j = p mod k (LDS integer
// atomics).  Eight loads per thread are issued before the first is used: a loop that consumes each
// index as it arrives pays one memory round trip per iteration.
__device__ __forceinline__ void count_pairs(const int32_t* __restrict__ idx, int64_t p_begin, int64_t p_end, int k,
                                            int N, int32_t* hist) {
    constexpr int kBatch = 8;
    for (int64_t p0 = p_begin + threadIdx.x; p0 < p_end; p0 += (int64_t)kThreads * kBatch) {
        int32_t e[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int64_t p = p0 + (int64_t)i * kThreads;
            e[i] = p < p_end ? idx[p] : -1;
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int64_t p = p0 + (int64_t)i * kThreads;
            if (e[i] >= 0 && e[i] < N) atomicAdd(&hist[(int)(p % k) * N + e[i]], 1);
        }
    }
}

__global__ __launch_bounds__(kThreads) void dispatch_count_kernel(
    const int32_t* __restrict__ idx, int64_t S, int N, int k, int n_ct, int32_t* __restrict__ tile_count) {
    __shared__ int32_t hist[TAMOE_MAX_K * TAMOE_MAX_EXPERTS];
    const int ct = blockIdx.x;
    for (int q = threadIdx.x; q < k * N; q += kThreads) hist[q] = 0;
    __syncthreads();
    const int64_t p_begin = (int64_t)ct * kCountTile * k;
    int64_t p_end = p_begin + (int64_t)kCountTile * k;
    if (p_end > S * k) p_end = S * k;
    count_pairs(idx, p_begin, p_end, k, N, hist);
    __syncthreads();
    for (int q = threadIdx.x; q < k * N; q += kThreads) {
        const int j = q / N, e = q - j * N;
        tile_count[((size_t)j * n_ct + ct) * N + e] = hist[q];
    }
}

// kept rows per expert -> the three size outputs of tamoe_dispatch (kept and off in LDS)
__device__ __forceinline__ void write_sizes(const int32_t* kept, const int32_t* off, int N, int P,
                                            int32_t* __restrict__ kept_expert, int32_t* __restrict__ expert_offset,
                                            int32_t* __restrict__ send_count_dev) {
    const int t = threadIdx.x;
    if (t < N) kept_expert[t] = kept[t];
    if (expert_offset != nullptr && t <= N) expert_offset[t] = off[t];
    if (send_count_dev != nullptr && t < P) {
        const int E = N / P;
        send_count_dev[t] = off[(t + 1) * E] - off[t * E];
    }
}

// Pairs of expert e that may be kept: its capacity (none given: unlimited), and in the fixed-size
// layout (pad_C > 0) at most the pad_C rows that every expert owns.
__device__ __forceinline__ int32_t pair_limit(const int32_t* __restrict__ cap, int e, int pad_C) {
    int32_t c = cap != nullptr ? (cap[e] < 0 ? 0 : cap[e]) : 0x7fffffff;
    if (pad_C > 0 && c > pad_C) c = pad_C;
    return c;
}

// One workgroup of 1024 threads: thread (part, e) owns a contiguous eighth of expert e's
// entries.  Entry q = j * n_ct + ct; ascending q is the priority order.
constexpr int kScanThreads = 1024;
constexpr int kScanParts = kScanThreads / TAMOE_MAX_EXPERTS;

__global__ __launch_bounds__(kScanThreads) void dispatch_scan_kernel(
    int32_t* __restrict__ tile_count, const int32_t* __restrict__ cap, int N, int P, int n_entries, int pad_C,
    int32_t* __restrict__ kept_expert, int32_t* __restrict__ expert_offset,
    int32_t* __restrict__ send_count_dev) {
    __shared__ int32_t part_sum[kScanParts][TAMOE_MAX_EXPERTS];
    __shared__ int32_t kept[TAMOE_MAX_EXPERTS];
    __shared__ int32_t off[TAMOE_MAX_EXPERTS + 1];
    __shared__ int32_t tmp[2 * 128];
    const int e = threadIdx.x % TAMOE_MAX_EXPERTS;
    const int part = threadIdx.x / TAMOE_MAX_EXPERTS;
    const int per_part = (n_entries + kScanParts - 1) / kScanParts;
    const int q0 = part * per_part;
    const int q1 = min(n_entries, q0 + per_part);
    // Loads are issued in batches of kBatch (a loop that adds each value as it arrives would pay
    // one L2 round trip per entry); the first batch stays in registers for the second pass.
    constexpr int kBatch = 16;
    int32_t first[kBatch];
    int32_t sum = 0;
    if (e < N) {
#pragma unroll
        for (int i = 0; i < kBatch; ++i) first[i] = (q0 + i < q1) ? tile_count[(size_t)(q0 + i) * N + e] : 0;
#pragma unroll
        for (int i = 0; i < kBatch; ++i) sum += first[i];
        for (int q = q0 + kBatch; q < q1; q += kBatch) {
            int32_t v[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) v[i] = (q + i < q1) ? tile_count[(size_t)(q + i) * N + e] : 0;
#pragma unroll
            for (int i = 0; i < kBatch; ++i) sum += v[i];
        }
    }
    part_sum[part][e] = sum;
    __syncthreads();
    if (e < N) {
        int32_t run = 0;
        for (int pp = 0; pp < part; ++pp) run += part_sum[pp][e];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            if (q0 + i < q1) tile_count[(size_t)(q0 + i) * N + e] = run;
            run += first[i];
        }
        for (int q = q0 + kBatch; q < q1; q += kBatch) {
            int32_t v[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) v[i] = (q + i < q1) ? tile_count[(size_t)(q + i) * N + e] : 0;
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                if (q + i < q1) tile_count[(size_t)(q + i) * N + e] = run;
                run += v[i];
            }
        }
        if (part == 0) {
            int32_t total = 0;
#pragma unroll
            for (int pp = 0; pp < kScanParts; ++pp) total += part_sum[pp][e];
            const int32_t c = pair_limit(cap, e, pad_C);
            kept[e] = total < c ? total : c;
        }
    }
    __syncthreads();
    exclusive_scan_128(kept, off, tmp, N);
    write_sizes(kept, off, N, P, kept_expert, expert_offset, send_count_dev);
}

// One workgroup per 64 tokens: recounts the pairs of its count tile that precede them, ranks
// their own pairs and writes slot[].
__global__ __launch_bounds__(kThreads) void dispatch_slot_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ cap, const int32_t* __restrict__ tile_base,
    const int32_t* __restrict__ expert_offset, int64_t S, int N, int k, int n_ct, int pad_C,
    int32_t* __restrict__ slot) {
    __shared__ int32_t before[TAMOE_MAX_K * TAMOE_MAX_EXPERTS];
    __shared__ int32_t s_idx[kSlotTile * TAMOE_MAX_K];

    const int64_t t0 = (int64_t)blockIdx.x * kSlotTile;
    const int ct = (int)(t0 / kCountTile);
    const int64_t tile_begin = (int64_t)ct * kCountTile;
    const int rows = (int)min((int64_t)kSlotTile, S - t0);
    const int pairs = rows * k;

    for (int q = threadIdx.x; q < k * N; q += kThreads) before[q] = 0;
    for (int p = threadIdx.x; p < pairs; p += kThreads) s_idx[p] = idx[t0 * k + p];
    __syncthreads();
    // pairs of this count tile that come before these tokens (same choice j)
    count_pairs(idx, tile_begin * k, t0 * k, k, N, before);
    __syncthreads();
    for (int p = threadIdx.x; p < pairs; p += kThreads) {
        const int e = s_idx[p];
        const int tl = p / k, j = p - tl * k;
        int32_t sl = -1;
        if (e >= 0 && e < N) {
            int32_t pos = tile_base[((size_t)j * n_ct + ct) * N + e] + before[j * N + e];
            for (int tt = 0; tt < tl; ++tt) pos += (s_idx[tt * k + j] == e) ? 1 : 0;
            if (pos < pair_limit(cap, e, pad_C)) sl = (pad_C > 0 ? e * pad_C : expert_offset[e]) + pos;
        }
        slot[t0 * k + p] = sl;
    }
}

// KK > 0: k is the compile-time constant KK; KK == 0: any k up to TAMOE_MAX_K.
// ROWU: a row is a multiple of 1 KiB, so the 64 chunks of a wavefront belong to one token and
// its slots are read once per wavefront through the scalar unit.
// `shift` >= 0: cpr == 1 << shift, and the (token, column) split of a chunk index is a shift and a
// mask; otherwise it is a division (32-bit when the tensor has fewer than 2^32 chunks).
// STREAM: rows are written with streaming (nontemporal) stores; otherwise with ordinary ones, which
// leave them in the last-level cache.
template <int KK, int U, bool ROWU, bool STREAM>
__global__ __launch_bounds__(kThreads) void dispatch_copy_kernel(const vec16* __restrict__ x,
                                                                 const int32_t* __restrict__ slot,
                                                                 int64_t total_chunks, int k_arg, int cpr, int shift,
                                                                 vec16* __restrict__ send) {
    constexpr int KM = KK > 0 ? KK : TAMOE_MAX_K;
    const int k = KK > 0 ? KK : k_arg;
    const int64_t base = (int64_t)blockIdx.x * (kThreads * U) + threadIdx.x;
    vec16 v[U];
    int32_t sl[U][KM];
    int col[U];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + (int64_t)u * kThreads;
        live[u] = false;
        col[u] = 0;
        if (c < total_chunks) {
            int t;
            split_chunk(c, total_chunks, cpr, shift, t, col[u]);
            if (ROWU) t = __builtin_amdgcn_readfirstlane(t);
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                sl[u][j] = j < k ? slot[(int64_t)t * k + j] : -1;
                live[u] |= sl[u][j] >= 0;
            }
            if (live[u]) v[u] = __builtin_nontemporal_load(x + c);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!live[u]) continue;
#pragma unroll
        for (int j = 0; j < KM; ++j)
            if (sl[u][j] >= 0) {
                if (STREAM)
                    __builtin_nontemporal_store(v[u], send + (size_t)sl[u][j] * cpr + col[u]);
                else
                    send[(size_t)sl[u][j] * cpr + col[u]] = v[u];
            }
    }
}

template <int KK, int U>
static void launch_copy(const void* x, const int32_t* slot, int64_t S, int k, int cpr, void* send, hipStream_t st) {
    const int64_t total = S * (int64_t)cpr;
    const dim3 grid((unsigned)ceil_div(total, kThreads * U)), block(kThreads);
    const vec16* src = static_cast<const vec16*>(x);
    vec16* dst = static_cast<vec16*>(send);
    const int shift = pow2_shift(cpr);
    const bool stream = !send_stays_in_cache(S, k, cpr);
    if (cpr % 64 == 0) {
        if (stream)
            dispatch_copy_kernel<KK, U, true, true><<<grid, block, 0, st>>>(src, slot, total, k, cpr, shift, dst);
        else
            dispatch_copy_kernel<KK, U, true, false><<<grid, block, 0, st>>>(src, slot, total, k, cpr, shift, dst);
    } else {
        if (stream)
            dispatch_copy_kernel<KK, U, false, true><<<grid, block, 0, st>>>(src, slot, total, k, cpr, shift, dst);
        else
            dispatch_copy_kernel<KK, U, false, false><<<grid, block, 0, st>>>(src, slot, total, k, cpr, shift, dst);
    }
}

static void launch_dispatch_copy(const void* x, const int32_t* slot, int64_t S, int k, int cpr, void* send,
                                 hipStream_t st) {
    TraceScope tr("dispatch_copy_kernel", st);
    if (k == 1)
        launch_copy<1, 2>(x, slot, S, k, cpr, send, st);
    else if (k == 2)
        launch_copy<2, 1>(x, slot, S, k, cpr, send, st);
    else
        launch_copy<0, 1>(x, slot, S, k, cpr, send, st);
}

// Fixed-size layout: zero rows e*C + kept[e] .. (e+1)*C - 1 of every expert.  Workgroup (e, part)
// clears a contiguous share of expert e's unused chunks: stores only, so nothing waits on memory.
__global__ __launch_bounds__(kThreads) void dispatch_pad_fill_kernel(const int32_t* __restrict__ kept_expert, int cpr,
                                                                     int C, vec16* __restrict__ send) {
    const int e = blockIdx.x;
    const int32_t used = kept_expert[e];
    const int64_t n = (int64_t)(C - used) * cpr;                   // chunks to clear, >= 0
    const int64_t per = (n + gridDim.y - 1) / gridDim.y;
    const int64_t i0 = (int64_t)blockIdx.y * per;
    const int64_t i1 = i0 + per < n ? i0 + per : n;
    vec16* base = send + ((int64_t)e * C + used) * cpr;
    const vec16 zero = {0u, 0u, 0u, 0u};
    for (int64_t i = i0 + threadIdx.x; i < i1; i += kThreads) __builtin_nontemporal_store(zero, base + i);
}

// Shared body of tamoe_dispatch (pad_C == 0: packed rows, expert after expert) and
// tamoe_dispatch_padded (pad_C > 0: pad_C rows per expert, the unused ones zeroed).
// tile_count: device scratch of k * count_tiles(S) * N ints; every entry is written by the count
// kernel before it is read, so its content on entry does not matter.
static int dispatch_impl(const char* fn, const void* x, const int32_t* topk_idx, const int32_t* cap, int dtype,
                         int64_t S, int d, int N, int P, int k, int pad_C, void* send, int32_t* slot,
                         int32_t* kept_expert, int32_t* expert_offset, int32_t* send_count_dev,
                         int32_t* tile_count, void* stream) {
    int rc;
    const int64_t n_ct = count_tiles(S);
    if ((int64_t)k * n_ct > (int64_t)1 << 30)
        return fail(TAMOE_UNSUPPORTED, "%s: too many count tiles (%lld)", fn, (long long)n_ct);
    const int cpr = d * elem_bytes(dtype) / 16;  // 16-byte chunks per row
    if (S > 0 && ceil_div(S * (int64_t)cpr, kThreads * 1) > 0x7fffffff)
        return fail(TAMOE_UNSUPPORTED, "%s: x is too large for one launch", fn);

    hipStream_t st = static_cast<hipStream_t>(stream);

    if (n_ct > 0) {
        TraceScope tr("dispatch_count_kernel", st);
        dispatch_count_kernel<<<dim3((unsigned)n_ct), dim3(kThreads), 0, st>>>(topk_idx, S, N, k, (int)n_ct,
                                                                                tile_count);
        if ((rc = check_launch(fn, "dispatch_count_kernel")) != TAMOE_OK) return rc;
    }
    {
        TraceScope tr("dispatch_scan_kernel", st);
        dispatch_scan_kernel<<<dim3(1), dim3(kScanThreads), 0, st>>>(tile_count, cap, N, P, (int)(k * n_ct), pad_C,
                                                                      kept_expert, expert_offset, send_count_dev);
    }
    if ((rc = check_launch(fn, "dispatch_scan_kernel")) != TAMOE_OK) return rc;
    if (S > 0) {
        {
            TraceScope tr("dispatch_slot_kernel", st);
            dispatch_slot_kernel<<<dim3((unsigned)ceil_div(S, kSlotTile)), dim3(kThreads), 0, st>>>(
                topk_idx, cap, tile_count, expert_offset, S, N, k, (int)n_ct, pad_C, slot);
        }
        if ((rc = check_launch(fn, "dispatch_slot_kernel")) != TAMOE_OK) return rc;
        launch_dispatch_copy(x, slot, S, k, cpr, send, st);
        if ((rc = check_launch(fn, "dispatch_copy_kernel")) != TAMOE_OK) return rc;
    }
    if (pad_C > 0) {
        {
            // about 4096 workgroups in all, at most one per 4 KiB of an expert's rows
            const int64_t parts = std::max<int64_t>(1, std::min<int64_t>(ceil_div(4096, N),
                                                                         ceil_div((int64_t)pad_C * cpr, kThreads)));
            TraceScope tr("dispatch_pad_fill_kernel", st);
            dispatch_pad_fill_kernel<<<dim3((unsigned)N, (unsigned)parts), dim3(kThreads), 0, st>>>(
                kept_expert, cpr, pad_C, static_cast<vec16*>(send));
        }
        if ((rc = check_launch(fn, "dispatch_pad_fill_kernel")) != TAMOE_OK) return rc;
    }
    return TAMOE_OK;
}

// The pair-count table inside a caller's workspace, or NULL (error recorded) if the workspace is too small.
static int32_t* tile_count_in(const char* fn, void* ws, size_t ws_bytes, int64_t S, int N, int k) {
    const Workspace lay = workspace_layout(S, N, k);
    if (ws_bytes < lay.total) {
        fail(TAMOE_WORKSPACE_TOO_SMALL, "%s: workspace has %zu bytes, %zu needed", fn, ws_bytes, lay.total);
        return nullptr;
    }
    return reinterpret_cast<int32_t*>(static_cast<char*>(ws) + lay.tile_count);
}

// ---- scratch that lives in the library's own image (tamoe_dispatch_static) --------------------
// One copy of this array exists on every device the library's code object is loaded on, at an address of
// its own.  Host code must not use the array's name as a pointer: the per-device address is asked for
// once (first call on that device, with that device current) and kept.
constexpr int kStaticDevices = 64;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[TAMOE_STATIC_SCRATCH_BYTES];
static std::mutex g_scratch_lock;
static void* g_scratch_ptr[kStaticDevices] = {};

static int static_scratch(const char* fn, int32_t** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticDevices)
        return fail(TAMOE_HIP_ERROR, "%s: no current device (or device ordinal beyond %d)", fn, kStaticDevices - 1);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr)
            return fail(TAMOE_HIP_ERROR, "%s: hipGetSymbolAddress failed: %s", fn, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<int32_t*>(g_scratch_ptr[dev]);
    return TAMOE_OK;
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_dispatch_static(const void* x, const int32_t* topk_idx, const int32_t* cap, int dtype,
                                     int64_t S, int d, int N, int P, int k, void* send, int32_t* slot,
                                     int32_t* kept_expert, int32_t* expert_offset, int32_t* send_count_dev,
                                     void* stream) {
    const char* fn = "tamoe_dispatch_static";
    clear_error();
    int rc;
    if ((rc = check_shape(fn, S, N, P, k)) != TAMOE_OK) return rc;
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "cap", cap, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "kept_expert", kept_expert, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "expert_offset", expert_offset, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "send_count_dev", send_count_dev, 4)) != TAMOE_OK) return rc;
    if (S > 0) {
        if ((rc = check_ptr(fn, "x", x, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "topk_idx", topk_idx, 4)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "send", send, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "slot", slot, 4)) != TAMOE_OK) return rc;
    }
    const int64_t entries = (int64_t)k * count_tiles(S) * N;   // ints of scratch this shape needs
    if (entries * (int64_t)sizeof(int32_t) > (int64_t)TAMOE_STATIC_SCRATCH_BYTES)
        return fail(TAMOE_UNSUPPORTED,
                    "%s: k * ceil(S/%d) * N = %lld pair counters exceed the %d of the built-in scratch; "
                    "use tamoe_dispatch with a workspace",
                    fn, kCountTile, (long long)entries, (int)(TAMOE_STATIC_SCRATCH_BYTES / sizeof(int32_t)));
    int32_t* tile_count = nullptr;
    if ((rc = static_scratch(fn, &tile_count)) != TAMOE_OK) return rc;
    return dispatch_impl(fn, x, topk_idx, cap, dtype, S, d, N, P, k, 0, send, slot, kept_expert, expert_offset,
                         send_count_dev, tile_count, stream);
}

extern "C" int tamoe_dispatch(const void* x, const int32_t* topk_idx, const int32_t* cap, int dtype, int64_t S,
                              int d, int N, int P, int k, void* send, int32_t* slot, int32_t* kept_expert,
                              int32_t* expert_offset, int32_t* send_count_dev, void* ws, size_t ws_bytes,
                              void* stream) {
    const char* fn = "tamoe_dispatch";
    clear_error();
    int rc;
    if ((rc = check_shape(fn, S, N, P, k)) != TAMOE_OK) return rc;
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "cap", cap, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "kept_expert", kept_expert, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "expert_offset", expert_offset, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "send_count_dev", send_count_dev, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "ws", ws, 256)) != TAMOE_OK) return rc;
    if (S > 0) {
        if ((rc = check_ptr(fn, "x", x, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "topk_idx", topk_idx, 4)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "send", send, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "slot", slot, 4)) != TAMOE_OK) return rc;
    }
    int32_t* tile_count = tile_count_in(fn, ws, ws_bytes, S, N, k);
    if (tile_count == nullptr) return TAMOE_WORKSPACE_TOO_SMALL;
    return dispatch_impl(fn, x, topk_idx, cap, dtype, S, d, N, P, k, 0, send, slot, kept_expert, expert_offset,
                         send_count_dev, tile_count, stream);
}

extern "C" int tamoe_dispatch_padded(const void* x, const int32_t* topk_idx, const int32_t* cap, int dtype,
                                     int64_t S, int d, int N, int P, int k, int C, void* send, int32_t* slot,
                                     int32_t* kept_expert, void* ws, size_t ws_bytes, void* stream) {
    const char* fn = "tamoe_dispatch_padded";
    clear_error();
    int rc;
    if ((rc = check_shape(fn, S, N, P, k)) != TAMOE_OK) return rc;
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if (C <= 0 || (int64_t)N * C >= ((int64_t)1 << 31))
        return fail(TAMOE_INVALID_ARG, "%s: C = %d, N*C must lie in (0, 2^31)", fn, C);
    if (cap != nullptr && (rc = check_ptr(fn, "cap", cap, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "kept_expert", kept_expert, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "send", send, 16)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "ws", ws, 256)) != TAMOE_OK) return rc;
    if (S > 0) {
        if ((rc = check_ptr(fn, "x", x, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "topk_idx", topk_idx, 4)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "slot", slot, 4)) != TAMOE_OK) return rc;
    }
    int32_t* tile_count = tile_count_in(fn, ws, ws_bytes, S, N, k);
    if (tile_count == nullptr) return TAMOE_WORKSPACE_TOO_SMALL;
    return dispatch_impl(fn, x, topk_idx, cap, dtype, S, d, N, P, k, C, send, slot, kept_expert, nullptr, nullptr,
                         tile_count, stream);
}
