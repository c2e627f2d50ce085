// tamoe_gate_dispatch: the forward path up to the send buffer in three launches (paper Section 3.1:
// gate, softmax, top-k, l_aux and local capacity; Section 4.1: one merged delivery per device;
// Section 4.3: l_topo, variable chunk sizes).  Same results as tamoe_gate + tamoe_aux_loss +
// tamoe_dispatch, which take seven.
//
//   1. the gate kernel (gate_tile.h) leaves, besides the selection, per gate workgroup b the number of
//      pairs per (expert e, choice j) and for every pair its position among the pairs of (b, e, j);
//   2. route_expert_kernel, one workgroup per expert: mean probability, count, the exclusive prefix of
//      the expert's pair counts in priority order (choice-major, then token order), kept rows;
//   3. route_copy_kernel: the scatter.  A pair's slot is offset[e] + prefix[e][j][b] + position, kept
//      iff prefix + position < cap[e]; offset[e] is the sum of the kept rows of the experts before e,
//      which every wavefront takes from the N kept counts by a scan of its own (two loads and a dozen
//      lane shifts: cheaper than one more pass over the experts in front of the scatter); every
//      thread derives the slots of its token on the way to moving its 16-byte chunk, and the thread
//      with the row's first chunk writes them to slot[].  The first workgroup also writes what
//      describes the layer as a whole: expert offsets, rows per destination device, the loss.
//      Rows are written with ordinary stores while the send buffer is small enough to stay in the
//      last-level cache, with streaming stores beyond that (as in the scatter of tamoe_dispatch).
#include "internal.h"

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
// Nothing here needs another expert: what does (offsets, rows per device, the loss) is left to the
// kernel that follows, which has to wait for this one anyway.
constexpr int kExpertThreads = 256;

__global__ __launch_bounds__(kExpertThreads) void route_expert_kernel(
    const float* __restrict__ m_part, int32_t* __restrict__ tile_pairs, int n_blocks, int entries, int pitch,
    int64_t S, const int32_t* __restrict__ cap, float* __restrict__ m, int32_t* __restrict__ c_expert,
    int32_t* __restrict__ kept_expert) {
    constexpr int kWaves = kExpertThreads / 64;
    __shared__ int32_t wave_cnt[kWaves];
    __shared__ float wave_sum[kWaves];

    const int e = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    // probability sums of this expert: thread-wise over ascending pieces, then lanes, then wavefronts
    // (requested first: they need nothing from the scan below)
    float acc = 0.f;
    const float* mrow = m_part + (size_t)e * n_blocks;
    for (int q0 = 0; q0 < n_blocks; q0 += 4 * kExpertThreads) {
        const int q = q0 + 4 * tid;
        // rows of n_blocks floats are not 16-byte aligned in general
        const float x0 = q < n_blocks ? mrow[q] : 0.f, x1 = q + 1 < n_blocks ? mrow[q + 1] : 0.f;
        const float x2 = q + 2 < n_blocks ? mrow[q + 2] : 0.f, x3 = q + 3 < n_blocks ? mrow[q + 3] : 0.f;
        acc += (x0 + x1) + (x2 + x3);
    }

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

#pragma unroll
    for (int sft = 32; sft > 0; sft >>= 1) acc += __shfl_xor(acc, sft);
    if (lane == 0) wave_sum[wave] = acc;
    __syncthreads();

    if (tid == 0) {
        const float sum = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
        const int32_t lim = cap[e] < 0 ? 0 : cap[e];
        m[e] = S > 0 ? sum / (float)S : 0.f;
        c_expert[e] = carry;
        kept_expert[e] = carry < lim ? carry : lim;
    }
}

// offset[e] = kept rows of the experts before e, for the (at most two) experts a lane is asked about:
// every wavefront scans the N <= 128 kept counts by itself.  Called by all 64 lanes.
struct WaveOffsets {
    int32_t ex0, ex1;   // exclusive prefix at expert lane, lane + 64
};
// The lane's two kept counts: requested at the top of a kernel, scanned (wave_offsets) only where the
// first offset is needed, so that the round trip runs beside the kernel's other loads.
struct KeptPair {
    int32_t k0, k1;
};
__device__ __forceinline__ KeptPair load_kept(const int32_t* __restrict__ kept_expert, int N) {
    static_assert(TAMOE_MAX_EXPERTS <= 128, "two experts per lane");
    const int lane = threadIdx.x & 63;
    return KeptPair{lane < N ? kept_expert[lane] : 0, lane + 64 < N ? kept_expert[lane + 64] : 0};
}
__device__ __forceinline__ WaveOffsets wave_offsets(const KeptPair& kp) {
    const int32_t i0 = wave_inclusive_scan(kp.k0);
    const int32_t i1 = wave_inclusive_scan(kp.k1) + __builtin_amdgcn_readlane(i0, 63);
    return WaveOffsets{i0 - kp.k0, i1 - kp.k1};
}
// e in [0, 128).  UNIFORM: e is the same in every lane (read through the scalar unit, no lane exchange);
// otherwise any value per lane, and all 64 lanes must take part.
template <bool UNIFORM>
__device__ __forceinline__ int32_t offset_of(const WaveOffsets& o, int e) {
    if constexpr (UNIFORM) {
        const int eu = __builtin_amdgcn_readfirstlane(e);
        const int32_t lo = __builtin_amdgcn_readlane(o.ex0, eu & 63), hi = __builtin_amdgcn_readlane(o.ex1, eu & 63);
        return eu < 64 ? lo : hi;
    } else {
        const int32_t lo = __shfl(o.ex0, e & 63), hi = __shfl(o.ex1, e & 63);
        return e < 64 ? lo : hi;
    }
}

// What describes the layer as a whole, by one workgroup of kCopyThreads threads that does nothing else
// (every thread calls): expert offsets (Section 4.3: what the size exchange carries), rows and pairs per
// destination device, the loss.  N <= 128 values: the first wavefront holds two experts per lane, scans
// and sums them with lane operations (fixed order), and hands offsets and counts to the threads that
// write the per-device numbers through LDS.
__device__ __forceinline__ void route_layer_outputs(const float* __restrict__ m, const int32_t* __restrict__ c_expert,
                                                    const int32_t* __restrict__ kept_expert,
                                                    const float* __restrict__ penalty, float loss_scale, int N, int P,
                                                    int32_t* __restrict__ c_device, float* __restrict__ loss,
                                                    int32_t* __restrict__ expert_offset,
                                                    int32_t* __restrict__ send_count_dev) {
    __shared__ int32_t total[TAMOE_MAX_EXPERTS];
    __shared__ int32_t off[TAMOE_MAX_EXPERTS + 1];
    const int tid = threadIdx.x;
    if (tid < 64) {
        const int e0 = tid, e1 = tid + 64;
        const int32_t c0 = e0 < N ? c_expert[e0] : 0, c1 = e1 < N ? c_expert[e1] : 0;
        const int32_t k0 = e0 < N ? kept_expert[e0] : 0, k1 = e1 < N ? kept_expert[e1] : 0;
        float t0 = 0.f, t1 = 0.f;
        if (e0 < N) t0 = m[e0] * (float)c0 * (penalty != nullptr ? penalty[e0] : 1.f);
        if (e1 < N) t1 = m[e1] * (float)c1 * (penalty != nullptr ? penalty[e1] : 1.f);
        const int32_t i0 = wave_inclusive_scan(k0);
        const int32_t i1 = wave_inclusive_scan(k1) + __builtin_amdgcn_readlane(i0, 63);
        total[e0] = c0;
        total[e1] = c1;
        off[e0] = i0 - k0;
        off[e1] = i1 - k1;
        if (e0 == N - 1) off[N] = i0;
        if (e1 == N - 1) off[N] = i1;
        float term = t0 + t1;
#pragma unroll
        for (int sft = 32; sft > 0; sft >>= 1) term += __shfl_xor(term, sft);
        if (tid == 0 && loss != nullptr) loss[0] = term * loss_scale;
    }
    __syncthreads();
    if (tid <= N) expert_offset[tid] = off[tid];
    if (tid < P) {
        const int E = N / P;
        send_count_dev[tid] = off[(tid + 1) * E] - off[tid * E];
        int32_t c = 0;
        for (int q = 0; q < E; ++q) c += total[tid * E + q];
        c_device[tid] = c;
    }
}

// Arguments of route_layer_outputs, handed through the kernels whose first workgroup calls it.
struct LayerOutputs {
    const float* m;
    const int32_t* c_expert;
    const int32_t* kept_expert;
    const float* penalty;
    float loss_scale;
    int P;
    int32_t* c_device;
    float* loss;
    int32_t* expert_offset;
    int32_t* send_count_dev;
};

// No tokens: every size, count and sum is zero.
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
// 16-byte chunk per thread (two for k = 1), a wavefront inside one row when ROWU (its token's experts,
// positions and table entries then go through the scalar unit).  STREAM: the rows are written with
// streaming stores (send buffers too large to stay in the last-level cache).  Workgroup 0 writes the
// layer's outputs and moves no rows: as part of a copying workgroup that tail would end after every
// other workgroup of a short launch.
template <int KK, int U, bool ROWU, bool STREAM>
__global__ __launch_bounds__(kCopyThreads) void route_copy_kernel(
    const vec16* __restrict__ x, const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ local_pos,
    const int32_t* __restrict__ tile_base, const int32_t* __restrict__ cap, int64_t total_chunks, int k_arg, int cpr,
    int shift, int N, int n_blocks, int pitch, int tile_shift, int32_t* __restrict__ slot, vec16* __restrict__ send,
    const LayerOutputs lo) {
    if (blockIdx.x == 0) {
        route_layer_outputs(lo.m, lo.c_expert, lo.kept_expert, lo.penalty, lo.loss_scale, N, lo.P, lo.c_device, lo.loss,
                            lo.expert_offset, lo.send_count_dev);
        return;
    }
    constexpr int KM = KK > 0 ? KK : TAMOE_MAX_K;
    const int k = KK > 0 ? KK : k_arg;
    const int64_t base = (int64_t)(blockIdx.x - 1) * (kCopyThreads * U) + threadIdx.x;
    const KeptPair kp = load_kept(lo.kept_expert, N);
    vec16 v[U];
    int32_t e[U][KM], pos[U][KM];   // pos < 0: the pair is not kept
    int col[U], tok[U];
    bool live[U], inside[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + (int64_t)u * kCopyThreads;
        inside[u] = c < total_chunks;
        live[u] = false;
        col[u] = 0;
        tok[u] = 0;
#pragma unroll
        for (int j = 0; j < KM; ++j) {
            e[u][j] = 0;
            pos[u][j] = -1;
        }
        if constexpr (ROWU) {   // the wavefront is inside or outside as a whole
            inside[u] = __builtin_amdgcn_readfirstlane((int)inside[u]) != 0;
            if (!inside[u]) continue;
            inside[u] = true;
        }
        if (inside[u]) {
            split_chunk(c, total_chunks, cpr, shift, tok[u], col[u]);
            if (ROWU) tok[u] = __builtin_amdgcn_readfirstlane(tok[u]);
        }
        const int t = tok[u];
        const int blk = t >> tile_shift;
        int32_t lp[KM], first[KM], lim[KM];
        bool valid[KM];
#pragma unroll
        for (int j = 0; j < KM; ++j) {
            e[u][j] = (inside[u] && j < k) ? topk_idx[(int64_t)t * k + j] : -1;
            lp[j] = (inside[u] && j < k) ? local_pos[(int64_t)t * k + j] : 0;
        }
        // the table entries of all choices are requested together and unconditionally (expert 0 stands
        // in for a missing one): behind a test each would be a memory round trip of its own
#pragma unroll
        for (int j = 0; j < KM; ++j) {
            valid[j] = e[u][j] >= 0 && e[u][j] < N;
            e[u][j] = valid[j] ? e[u][j] : 0;
            first[j] = 0;
            lim[j] = 0;
            if (j < k) {
                first[j] = tile_base[(size_t)e[u][j] * pitch + (size_t)j * n_blocks + blk];
                lim[j] = cap[e[u][j]];
            }
        }
#pragma unroll
        for (int j = 0; j < KM; ++j) {
            const int32_t p = first[j] + lp[j];
            if (valid[j] && p < lim[j]) pos[u][j] = p;
            live[u] |= pos[u][j] >= 0;
        }
        if (live[u]) v[u] = __builtin_nontemporal_load(x + c);
    }
    // every lane is back here: the scan and, without ROWU, the lane exchange of offset_of need them all
    const WaveOffsets wo = wave_offsets(kp);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        int32_t sl[KM];
#pragma unroll
        for (int j = 0; j < KM; ++j) {
            sl[j] = -1;
            if (j < k) {
                const int32_t off = offset_of<ROWU>(wo, e[u][j]);
                if (pos[u][j] >= 0) sl[j] = off + pos[u][j];
            }
        }
        if (inside[u] && col[u] == 0) {
#pragma unroll
            for (int j = 0; j < KM; ++j)
                if (j < k) slot[(int64_t)tok[u] * k + j] = sl[j];
        }
        if (live[u]) {
#pragma unroll
            for (int j = 0; j < KM; ++j)
                if (sl[j] >= 0) {
                    vec16* dst = send + (size_t)sl[j] * cpr + col[u];
                    if (STREAM)
                        __builtin_nontemporal_store(v[u], dst);
                    else
                        *dst = v[u];
                }
        }
    }
}

struct CopyArgs {
    const void* x;
    const int32_t* topk_idx;
    const int32_t* cap;
    int64_t S;
    int k, cpr, N, tile_shift;
    GateStats stats;
    int32_t* slot;
    void* send;
    LayerOutputs lo;
    hipStream_t st;
};

template <int KK, int U>
static void launch_route_copy(const CopyArgs& a) {
    const int64_t total = a.S * (int64_t)a.cpr;
    const dim3 grid((unsigned)ceil_div(total, kCopyThreads * U) + 1u), block(kCopyThreads);   // + workgroup 0
    const vec16* src = static_cast<const vec16*>(a.x);
    vec16* dst = static_cast<vec16*>(a.send);
    const int shift = pow2_shift(a.cpr);
    const bool rowu = a.cpr % 64 == 0;
    const bool stream = !send_stays_in_cache(a.S, a.k, a.cpr);
#define TAMOE_ROUTE_COPY(RU, ST)                                                                                   \
    route_copy_kernel<KK, U, RU, ST><<<grid, block, 0, a.st>>>(                                                    \
        src, a.topk_idx, a.stats.local_pos, a.stats.tile_pairs, a.cap, total, a.k, a.cpr, shift, a.N,             \
        a.stats.n_blocks, a.stats.pitch, a.tile_shift, a.slot, dst, a.lo)
    if (rowu) {
        if (stream) TAMOE_ROUTE_COPY(true, true); else TAMOE_ROUTE_COPY(true, false);
    } else {
        if (stream) TAMOE_ROUTE_COPY(false, true); else TAMOE_ROUTE_COPY(false, false);
    }
#undef TAMOE_ROUTE_COPY
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
    if (S > 0 && ceil_div(S * (int64_t)cpr, kCopyThreads) >= 0x7fffffff)   // one more workgroup is added
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
            run.stats.m_part, run.stats.tile_pairs, run.stats.n_blocks, k * run.stats.n_blocks, run.stats.pitch, S, cap,
            m, c_expert, kept_expert);
    }
    if ((rc = check_launch(fn, "route_expert_kernel")) != TAMOE_OK) return rc;

    CopyArgs a{};
    a.x = x;
    a.topk_idx = topk_idx;
    a.cap = cap;
    a.S = S;
    a.k = k;
    a.cpr = cpr;
    a.N = N;
    a.tile_shift = pow2_shift(run.tile_tokens);
    a.stats = run.stats;
    a.slot = slot;
    a.send = send;
    a.lo = LayerOutputs{m, c_expert, kept_expert, penalty, scale, P, c_device, loss, expert_offset, send_count_dev};
    a.st = st;
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
