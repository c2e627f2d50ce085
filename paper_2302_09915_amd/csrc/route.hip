// tamoe_gate_dispatch: the forward path up to the send buffer in three launches (paper Section 3.1:
// gate, softmax, top-k, l_aux and local capacity; Section 4.1: one merged delivery per device;
// Section 4.3: l_topo, variable chunk sizes).  Same results as tamoe_gate + tamoe_aux_loss +
// tamoe_dispatch, which take seven.
//
//   1. the gate kernel (gate_tile.h) leaves, besides the selection, per gate workgroup b the number of
//      pairs per (expert e, choice j) and for every pair its position among the pairs of (b, e, j);
//   2. route_expert_kernel, one workgroup per expert: mean probability, count, the exclusive prefix of
//      the expert's pair counts in priority order (choice-major, then token order), kept rows; the
//      workgroup that finishes last adds expert offsets, rows per destination device and the loss;
//   3. route_copy_kernel: the scatter.  A pair's slot is offset[e] + prefix[e][j][b] + position, kept
//      iff prefix + position < cap[e]; every thread derives the slots of its token on the way to
//      moving its 16-byte chunk, and the thread with the row's first chunk writes them to slot[].
//      When the send buffer is too large to stay in the last-level cache (96 MiB) the slots are written
//      by route_slot_kernel (one thread per pair) and the rows are moved by the scatter of
//      tamoe_dispatch: a fourth launch, but a shorter scatter.
#include "internal.h"
#include "scan128.h"

namespace tamoe {

constexpr int kCopyThreads = 256;

// Sum of v over the lanes below this one plus its own (wavefront of 64) with data-parallel
// primitives: shifts by 1, 2, 4, 8 inside each row of 16 lanes (a lane without a source adds 0), then
// the last lane of row 0 (2) is added to row 1 (3) and the last lane of row 1 to rows 2 and 3.
__device__ __forceinline__ int32_t wave_inclusive_scan(int32_t v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// One workgroup per expert e: the exclusive prefix of the expert's pair counts in priority order (in
// place), its total, kept rows and mean probability.  A single workgroup for all experts would be a
// chain of memory round trips through one compute unit's few outstanding misses (measured: 27 us for
// 640 KiB on the large configuration); spread over N compute units each has two kilobytes to fetch.
// What needs every expert (offsets, rows per device, the loss) is done by the workgroup that
// finishes last: each publishes its three numbers, then takes a ticket from a counter that the gate
// kernel has reset; no workgroup waits for another.
constexpr int kExpertThreads = 256;

template <typename V>
__device__ __forceinline__ void publish(V* p, V v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename V>
__device__ __forceinline__ V observe(const V* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(kExpertThreads) void route_expert_kernel(
    const float* __restrict__ m_part, int32_t* __restrict__ tile_pairs, int n_blocks, int entries, int pitch, int N,
    int P, int64_t S, const float* __restrict__ penalty, float loss_scale, const int32_t* __restrict__ cap,
    float* m, int32_t* c_expert, int32_t* __restrict__ c_device, float* __restrict__ loss, int32_t* kept_expert,
    int32_t* __restrict__ expert_offset, int32_t* __restrict__ send_count_dev, uint32_t* done_counter) {
    constexpr int kWaves = kExpertThreads / 64;
    __shared__ int32_t wave_cnt[kWaves];
    __shared__ float wave_sum[kWaves];
    __shared__ int is_last;
    __shared__ int32_t total[TAMOE_MAX_EXPERTS];
    __shared__ int32_t kept[TAMOE_MAX_EXPERTS];
    __shared__ int32_t off[TAMOE_MAX_EXPERTS + 1];
    __shared__ int32_t tmp[2 * 128];
    __shared__ float term[TAMOE_MAX_EXPERTS];

    const int e = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    // pair counts of this expert, 1024 entries (16 bytes per thread) at a time
    int32_t* row = tile_pairs + (size_t)e * pitch;
    int32_t carry = 0;
    for (int q0 = 0; q0 < entries; q0 += 4 * kExpertThreads) {
        const int q = q0 + 4 * tid;
        int4 v = make_int4(0, 0, 0, 0);
        if (q < entries) v = *reinterpret_cast<const int4*>(row + q);
        // entries past the end of the row are padding of unknown content
        const int32_t a = q < entries ? v.x : 0, b = q + 1 < entries ? v.y : 0;
        const int32_t c = q + 2 < entries ? v.z : 0, d = q + 3 < entries ? v.w : 0;
        const int32_t s4 = a + b + c + d;
        const int32_t incl = wave_inclusive_scan(s4);
        if (lane == 63) wave_cnt[wave] = incl;
        __syncthreads();
        int32_t before = 0, piece = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            before += w < wave ? wave_cnt[w] : 0;
            piece += wave_cnt[w];
        }
        const int32_t first = carry + before + incl - s4;
        if (q < entries) *reinterpret_cast<int4*>(row + q) = make_int4(first, first + a, first + a + b, first + a + b + c);
        carry += piece;
        __syncthreads();
    }

    // probability sums of this expert: thread-wise over ascending pieces, then lanes, then wavefronts
    float acc = 0.f;
    const float* mrow = m_part + (size_t)e * n_blocks;
    for (int q0 = 0; q0 < n_blocks; q0 += 4 * kExpertThreads) {
        const int q = q0 + 4 * tid;
        // rows of n_blocks floats are not 16-byte aligned in general
        const float x0 = q < n_blocks ? mrow[q] : 0.f, x1 = q + 1 < n_blocks ? mrow[q + 1] : 0.f;
        const float x2 = q + 2 < n_blocks ? mrow[q + 2] : 0.f, x3 = q + 3 < n_blocks ? mrow[q + 3] : 0.f;
        acc += (x0 + x1) + (x2 + x3);
    }
#pragma unroll
    for (int sft = 32; sft > 0; sft >>= 1) acc += __shfl_xor(acc, sft);
    if (lane == 0) wave_sum[wave] = acc;
    __syncthreads();

    if (tid == 0) {
        const float sum = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
        const int32_t lim = cap[e] < 0 ? 0 : cap[e];
        publish(&m[e], S > 0 ? sum / (float)S : 0.f);
        publish(&c_expert[e], carry);
        publish(&kept_expert[e], carry < lim ? carry : lim);
        __threadfence();                                      // the three numbers before the ticket
        const uint32_t ticket = atomicAdd(done_counter, 1u);
        is_last = ticket == (uint32_t)N - 1u;
    }
    __syncthreads();
    if (!is_last) return;

    // ---- the last workgroup: what needs every expert ----
    __threadfence();                                          // the ticket before the others' numbers
    if (tid < TAMOE_MAX_EXPERTS) {
        int32_t c = 0, kp = 0;
        float t = 0.f;
        if (tid < N) {
            c = observe(&c_expert[tid]);
            kp = observe(&kept_expert[tid]);
            t = observe(&m[tid]) * (float)c * (penalty != nullptr ? penalty[tid] : 1.f);
        }
        total[tid] = c;
        kept[tid] = kp;
        term[tid] = t;
    }
    __syncthreads();
    // sizes (Section 4.3: what the size exchange carries), counts per device, the loss
    exclusive_scan_128(kept, off, tmp, N);
    if (tid <= N) expert_offset[tid] = off[tid];
    if (tid < P) {
        const int E = N / P;
        send_count_dev[tid] = off[(tid + 1) * E] - off[tid * E];
        int32_t c = 0;
        for (int q = 0; q < E; ++q) c += total[tid * E + q];
        c_device[tid] = c;
    }
    for (int stride = TAMOE_MAX_EXPERTS / 2; stride > 0; stride >>= 1) {
        if (tid < stride) term[tid] += term[tid + stride];
        __syncthreads();
    }
    if (tid == 0 && loss != nullptr) loss[0] = term[0] * loss_scale;
}

// No tokens: every size, count and sum is zero (the gate kernel, which resets the ticket counter of
// route_expert_kernel, does not run then).
__global__ __launch_bounds__(kExpertThreads) void route_empty_kernel(int N, int P, float* __restrict__ m,
                                                                    int32_t* __restrict__ c_expert,
                                                                    int32_t* __restrict__ c_device,
                                                                    float* __restrict__ loss,
                                                                    int32_t* __restrict__ kept_expert,
                                                                    int32_t* __restrict__ expert_offset,
                                                                    int32_t* __restrict__ send_count_dev) {
    const int tid = threadIdx.x;
    if (tid < N) {
        m[tid] = 0.f;
        c_expert[tid] = 0;
        kept_expert[tid] = 0;
    }
    if (tid <= N) expert_offset[tid] = 0;
    if (tid < P) {
        c_device[tid] = 0;
        send_count_dev[tid] = 0;
    }
    if (tid == 0 && loss != nullptr) loss[0] = 0.f;
}

// The scatter with the slot assignment folded in.  Layout of the work as in dispatch_copy_kernel: one
// 16-byte chunk per thread (two for k = 1), a wavefront inside one row when ROWU.  Only launched for
// batches whose send buffer fits the last-level cache, so the rows are written with ordinary stores.
template <int KK, int U, bool ROWU>
__global__ __launch_bounds__(kCopyThreads) void route_copy_kernel(
    const vec16* __restrict__ x, const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ local_pos,
    const int32_t* __restrict__ tile_base, const int32_t* __restrict__ cap,
    const int32_t* __restrict__ expert_offset, int64_t total_chunks, int k_arg, int cpr, int shift, int N,
    int n_blocks, int pitch, int tile_shift, int32_t* __restrict__ slot, vec16* __restrict__ send) {
    constexpr int KM = KK > 0 ? KK : TAMOE_MAX_K;
    const int k = KK > 0 ? KK : k_arg;
    const int64_t base = (int64_t)blockIdx.x * (kCopyThreads * U) + threadIdx.x;
    vec16 v[U];
    int32_t sl[U][KM];
    int col[U];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + (int64_t)u * kCopyThreads;
        live[u] = false;
        col[u] = 0;
        if (c < total_chunks) {
            int t;
            split_chunk(c, total_chunks, cpr, shift, t, col[u]);
            if (ROWU) t = __builtin_amdgcn_readfirstlane(t);
            const int blk = t >> tile_shift;
            int32_t e[KM], lp[KM];
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                e[j] = j < k ? topk_idx[(int64_t)t * k + j] : -1;
                lp[j] = j < k ? local_pos[(int64_t)t * k + j] : 0;
            }
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                sl[u][j] = -1;
                if (j < k && e[j] >= 0 && e[j] < N) {
                    const int32_t pos = tile_base[(size_t)e[j] * pitch + (size_t)j * n_blocks + blk] + lp[j];
                    const int32_t lim = cap[e[j]];
                    if (pos < lim) sl[u][j] = expert_offset[e[j]] + pos;
                }
                live[u] |= sl[u][j] >= 0;
            }
            if (live[u]) v[u] = __builtin_nontemporal_load(x + c);
            if (col[u] == 0) {
#pragma unroll
                for (int j = 0; j < KM; ++j)
                    if (j < k) slot[(int64_t)t * k + j] = sl[u][j];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!live[u]) continue;
#pragma unroll
        for (int j = 0; j < KM; ++j)
            if (sl[u][j] >= 0) send[(size_t)sl[u][j] * cpr + col[u]] = v[u];
    }
}

// The slot of every pair by itself: one thread per pair.  For batches whose scatter is bound by
// bandwidth, where the extra table lookups in front of every wavefront's copy would cost more than a
// launch.
__global__ __launch_bounds__(kCopyThreads) void route_slot_kernel(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ local_pos,
    const int32_t* __restrict__ tile_base, const int32_t* __restrict__ cap,
    const int32_t* __restrict__ expert_offset, int64_t pairs, int k, int N, int n_blocks, int pitch, int tile_shift,
    int32_t* __restrict__ slot) {
    const int64_t p = (int64_t)blockIdx.x * kCopyThreads + threadIdx.x;
    if (p >= pairs) return;
    const int e = topk_idx[p];
    const int32_t lp = local_pos[p];
    const int64_t t = p / k;
    const int j = (int)(p - t * k);
    int32_t sl = -1;
    if (e >= 0 && e < N) {
        const int32_t pos = tile_base[(size_t)e * pitch + (size_t)j * n_blocks + (t >> tile_shift)] + lp;
        if (pos < cap[e]) sl = expert_offset[e] + pos;
    }
    slot[p] = sl;
}

struct CopyArgs {
    const void* x;
    const int32_t* topk_idx;
    const int32_t* cap;
    const int32_t* expert_offset;
    int64_t S;
    int k, cpr, N, tile_shift;
    GateStats stats;
    int32_t* slot;
    void* send;
    hipStream_t st;
};

template <int KK, int U>
static void launch_route_copy(const CopyArgs& a) {
    const int64_t total = a.S * (int64_t)a.cpr;
    const dim3 grid((unsigned)ceil_div(total, kCopyThreads * U)), block(kCopyThreads);
    const vec16* src = static_cast<const vec16*>(a.x);
    vec16* dst = static_cast<vec16*>(a.send);
    const int shift = pow2_shift(a.cpr);
    if (a.cpr % 64 == 0)
        route_copy_kernel<KK, U, true><<<grid, block, 0, a.st>>>(
            src, a.topk_idx, a.stats.local_pos, a.stats.tile_pairs, a.cap, a.expert_offset, total, a.k, a.cpr, shift,
            a.N, a.stats.n_blocks, a.stats.pitch, a.tile_shift, a.slot, dst);
    else
        route_copy_kernel<KK, U, false><<<grid, block, 0, a.st>>>(
            src, a.topk_idx, a.stats.local_pos, a.stats.tile_pairs, a.cap, a.expert_offset, total, a.k, a.cpr, shift,
            a.N, a.stats.n_blocks, a.stats.pitch, a.tile_shift, a.slot, dst);
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_gate_dispatch(const void* x, const void* w, int dtype, int64_t S, int d, int N, int P, int k,
                                   const float* penalty, const int32_t* cap, float* logits, int32_t* topk_idx,
                                   float* topk_w, float* m, int32_t* c_expert, int32_t* c_device, float* loss,
                                   void* send, int32_t* slot, int32_t* kept_expert, int32_t* expert_offset,
                                   int32_t* send_count_dev, void* ws, size_t ws_bytes, void* stream) {
    const char* fn = "tamoe_gate_dispatch";
    clear_error();
    int rc;
    if ((rc = check_shape(fn, S, N, P, k)) != TAMOE_OK) return rc;
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if (S > 0) {
        if ((rc = check_ptr(fn, "x", x, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "w", w, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "send", send, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "slot", slot, 4)) != TAMOE_OK) return rc;
    }
    if ((rc = check_ptr(fn, "cap", cap, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "kept_expert", kept_expert, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "expert_offset", expert_offset, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "send_count_dev", send_count_dev, 4)) != TAMOE_OK) return rc;
    if (penalty != nullptr && (rc = check_ptr(fn, "penalty", penalty, 4)) != TAMOE_OK) return rc;
    if (loss != nullptr && (rc = check_ptr(fn, "loss", loss, 4)) != TAMOE_OK) return rc;
    const Workspace lay = workspace_layout(S, N, k, dtype);
    if ((rc = check_select_outputs(fn, S, topk_idx, topk_w, m, c_expert, c_device, ws, ws_bytes, lay)) != TAMOE_OK)
        return rc;
    const int cpr = d * elem_bytes(dtype) / 16;  // 16-byte chunks per row
    if (S > 0 && ceil_div(S * (int64_t)cpr, kCopyThreads) > 0x7fffffff)
        return fail(TAMOE_UNSUPPORTED, "%s: x is too large for one launch", fn);
    hipStream_t st = static_cast<hipStream_t>(stream);

    GateRun run{};
    if ((rc = run_gate_stage(fn, x, w, dtype, S, d, N, k, logits, topk_idx, topk_w, ws, lay, st, &run)) != TAMOE_OK)
        return rc;

    // scale in double on the host, one rounding to fp32 (as tamoe_aux_loss); S = 0 has no loss
    const float scale = S > 0 ? (float)((penalty != nullptr ? (double)N * (double)P : 1.0) / (double)S) : 0.f;
    if (S == 0) {
        route_empty_kernel<<<dim3(1), dim3(kExpertThreads), 0, st>>>(N, P, m, c_expert, c_device, loss, kept_expert,
                                                                      expert_offset, send_count_dev);
        return check_launch(fn, "route_empty_kernel");
    }
    {
        TraceScope tr("route_expert_kernel", st);
        route_expert_kernel<<<dim3(N), dim3(kExpertThreads), 0, st>>>(
            run.stats.m_part, run.stats.tile_pairs, run.stats.n_blocks, k * run.stats.n_blocks, run.stats.pitch, N, P, S,
            penalty, scale, cap, m, c_expert, c_device, loss, kept_expert, expert_offset, send_count_dev,
            run.stats.done);
    }
    if ((rc = check_launch(fn, "route_expert_kernel")) != TAMOE_OK) return rc;

    CopyArgs a{};
    a.x = x;
    a.topk_idx = topk_idx;
    a.cap = cap;
    a.expert_offset = expert_offset;
    a.S = S;
    a.k = k;
    a.cpr = cpr;
    a.N = N;
    a.tile_shift = pow2_shift(run.tile_tokens);
    a.stats = run.stats;
    a.slot = slot;
    a.send = send;
    a.st = st;
    // Slots in the scatter itself save a launch, but put two dependent table look-ups in front of every
    // wavefront's copy: that pays while the scatter is short (large configuration, 1 GiB of rows to
    // write: 270 us against 257 + 4 us for the two kernels; GPT-MoE layer, 64 MiB: a step of 61 against
    // 63 us).  The line is drawn where the send buffer stops fitting the last-level cache.
    if (!send_stays_in_cache(S, k, cpr)) {
        {
            TraceScope tr("route_slot_kernel", st);
            const int64_t pairs = S * k;
            route_slot_kernel<<<dim3((unsigned)ceil_div(pairs, kCopyThreads)), dim3(kCopyThreads), 0, st>>>(
                topk_idx, run.stats.local_pos, run.stats.tile_pairs, cap, expert_offset, pairs, k, N, run.stats.n_blocks,
                run.stats.pitch, a.tile_shift, slot);
        }
        if ((rc = check_launch(fn, "route_slot_kernel")) != TAMOE_OK) return rc;
        launch_dispatch_copy(x, slot, S, k, cpr, send, st);
        return check_launch(fn, "dispatch_copy_kernel");
    }
    {
        TraceScope tr("route_copy_kernel", st);
        if (k == 1)
            launch_route_copy<1, 2>(a);
        else if (k == 2)
            launch_route_copy<2, 1>(a);
        else
            launch_route_copy<0, 1>(a);
    }
    return check_launch(fn, "route_copy_kernel");
}
