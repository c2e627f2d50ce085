// tamoe_gate / tamoe_select: gate scores, softmax, top-k and the load statistics
// (paper Section 3.1: gate network G with softmax, top-k experts per token, c_ie, m_i;
// Section 4.1: per-destination-device volume).
//
// gate_bf16_kernel / gate_f16_kernel / gate_f32_kernel (one tile code, three element types): the one
// dense contraction of the path, on the matrix cores.  v_mfma_f32_32x32x16_bf16 (or _f16, or four
// v_mfma_f32_32x32x2_f32 for fp32 storage) with A = a 32-expert block of W and B = 32 tokens of x,
// both from LDS tiles filled by coalesced loads of 128-byte K chunks, so the
// accumulator tile is [expert][token]: lane l holds, for token (l & 31), the 16 experts
//     e(v, l) = 8*(v>>2) + 4*(l>>5) + (v&3),   v = 0..15          (+32 per expert block)
// and the lane pair (l, l^32) holds a token's whole score vector.  Softmax, top-k and the
// selected weights are therefore computed inside a lane with one cross-lane exchange per step;
// only the per-expert probability sums need a reduction over the 32 token lanes.
// The kernel is bound by the HBM read of x (intensity ~N flop/byte), not by the MFMA rate.
//
// tamoe_select runs the same selection code on a score matrix in memory (select_kernel).
//
// Determinism: probability sums are reduced in a fixed tree (lanes, wavefronts, workgroups);
// counts are integers.  A second small kernel folds the per-workgroup partials.
#include "gate_tile.h"

namespace tamoe {

// Selection stage on a score matrix in memory: 4 wavefronts x 32 tokens per workgroup.  The scores
// may arrive as n_parts partial matrices (the K shares of a split gate, part_stride floats apart),
// which are added in ascending order; logits_out (may be NULL) then receives the sums.
template <int NB>
__global__ __launch_bounds__(256) void select_kernel(const float* __restrict__ logits, int n_parts, size_t part_stride,
                                                     float* __restrict__ logits_out, int64_t S, int N, int k,
                                                     int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                     const GateStats gs) {
    constexpr int ROWS = NB * 32;
    __shared__ float m_w[4][ROWS];
    __shared__ int32_t pairs[4][TAMOE_MAX_K * ROWS];
    __shared__ __attribute__((aligned(16))) float out_tile[4][32 * kTileRow];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t token = ((int64_t)blockIdx.x * 4 + wave) * 32 + (lane & 31);
    const bool token_ok = token < S;
    for (int q = tid; q < 4 * ROWS; q += 256) (&m_w[0][0])[q] = 0.f;
    __syncthreads();
    float sc[NB][16];
    load_logits_tile<NB>(sc, lane, token, N, logits, n_parts, part_stride, out_tile[wave], S);
    TokenPairs tp;
    select_tile<NB>(sc, lane, token, token_ok, N, k, logits_out, topk_idx, topk_w, m_w[wave], pairs[wave],
                    out_tile[wave], S, tp);
    finish_block<NB, 4>(m_w, &pairs[0][0], TAMOE_MAX_K * ROWS, tp, lane, wave, token, token_ok, N, k, gs);
}

// One workgroup per expert: fixed-order sums of the per-workgroup partials.  entries = k * n_blocks.
__global__ __launch_bounds__(256) void gate_finalize_kernel(const float* __restrict__ m_part,
                                                            const int32_t* __restrict__ tile_pairs, int n_blocks,
                                                            int entries, int pitch, int N, int P, int64_t S,
                                                            float* __restrict__ m, int32_t* __restrict__ c_expert,
                                                            int32_t* __restrict__ c_device) {
    __shared__ float fs[256];
    __shared__ int32_t cs[256];
    const int e0 = blockIdx.x;
    const int E = N / P;
    const int span = (e0 % E == 0) ? E : 1;  // the first expert of a device also sums the device
    int32_t dev_total = 0;
    for (int de = 0; de < span; ++de) {
        const int e = e0 + de;
        float s = 0.f;
        int32_t c = 0;
        for (int i = threadIdx.x; i < n_blocks; i += 256) s += m_part[(size_t)e * n_blocks + i];
        for (int i = threadIdx.x; i < entries; i += 256) c += tile_pairs[(size_t)e * pitch + i];
        fs[threadIdx.x] = s;
        cs[threadIdx.x] = c;
        __syncthreads();
        for (int stride = 128; stride > 0; stride >>= 1) {
            if ((int)threadIdx.x < stride) {
                fs[threadIdx.x] += fs[threadIdx.x + stride];
                cs[threadIdx.x] += cs[threadIdx.x + stride];
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            if (de == 0) {
                m[e] = S > 0 ? fs[0] / (float)S : 0.f;
                c_expert[e] = cs[0];
            }
            dev_total += cs[0];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0 && e0 % E == 0) c_device[e0 / E] = dev_total;
}

// ---- host side ------------------------------------------------------------------------------

static void launch_select(int64_t blocks, hipStream_t st, const float* logits, int n_parts, size_t part_stride,
                          float* logits_out, int64_t S, int N, int k, int32_t* topk_idx, float* topk_w,
                          const GateStats& gs) {
    const dim3 grid((unsigned)blocks), block(256);
    TraceScope tr("select_kernel", st);
    if (N <= 32)
        select_kernel<1><<<grid, block, 0, st>>>(logits, n_parts, part_stride, logits_out, S, N, k, topk_idx, topk_w, gs);
    else if (N <= 64)
        select_kernel<2><<<grid, block, 0, st>>>(logits, n_parts, part_stride, logits_out, S, N, k, topk_idx, topk_w, gs);
    else
        select_kernel<4><<<grid, block, 0, st>>>(logits, n_parts, part_stride, logits_out, S, N, k, topk_idx, topk_w, gs);
}

int check_select_outputs(const char* fn, int64_t S, int32_t* topk_idx, float* topk_w, float* m, int32_t* c_expert,
                         int32_t* c_device, void* ws, size_t ws_bytes, const Workspace& lay) {
    int rc;
    if (S > 0) {
        if ((rc = check_ptr(fn, "topk_idx", topk_idx, 4)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "topk_w", topk_w, 4)) != TAMOE_OK) return rc;
    }
    if ((rc = check_ptr(fn, "m", m, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "c_expert", c_expert, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "c_device", c_device, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "ws", ws, 256)) != TAMOE_OK) return rc;
    if (ws_bytes < lay.total)
        return fail(TAMOE_WORKSPACE_TOO_SMALL, "%s: workspace has %zu bytes, %zu needed", fn, ws_bytes, lay.total);
    return TAMOE_OK;
}

static GateStats stats_in(void* ws, const Workspace& lay, int k, int64_t blocks) {
    GateStats gs{};
    gs.m_part = reinterpret_cast<float*>(static_cast<char*>(ws) + lay.m_part);
    gs.tile_pairs = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + lay.tile_pairs);
    gs.local_pos = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + lay.local_pos);
    gs.n_blocks = (int)blocks;
    gs.pitch = (int)pair_pitch(k, blocks);
    return gs;
}

int run_select_stage(const char* fn, const float* logits, int64_t S, int N, int k, int32_t* topk_idx, float* topk_w,
                     void* ws, const Workspace& lay, hipStream_t st, GateRun* run) {
    const int64_t blocks = ceil_div(S, 128);
    if ((int64_t)k * blocks > 0x3fffffff) return fail(TAMOE_UNSUPPORTED, "%s: too many token tiles", fn);
    run->stats = stats_in(ws, lay, k, blocks);
    run->tile_tokens = 128;
    if (blocks > 0) {
        launch_select(blocks, st, logits, 1, 0, nullptr, S, N, k, topk_idx, topk_w, run->stats);
        return check_launch(fn, "select_kernel");
    }
    return TAMOE_OK;
}

int run_gate_stage(const char* fn, const void* x, const void* w, int dtype, int64_t S, int d, int N, int k,
                   float* logits, int32_t* topk_idx, float* topk_w, void* ws, const Workspace& lay, hipStream_t st,
                   GateRun* run) {
    int rc;
    run->stats = stats_in(ws, lay, k, 0);
    run->tile_tokens = 32;
    if (S <= 0) return TAMOE_OK;
    const int waves = gate_waves(S, N);
    int64_t blocks = ceil_div(S, 32 * (int64_t)waves);
    if ((int64_t)k * blocks > 0x3fffffff) return fail(TAMOE_UNSUPPORTED, "%s: too many token tiles", fn);
    // the tile code addresses rows in 2-byte units: an fp32 row of d values is a row of 2*d units
    if (dtype == TAMOE_F32 && d > 0x3fffffff) return fail(TAMOE_UNSUPPORTED, "%s: d = %d is too large", fn, d);
    const int d_units = dtype == TAMOE_F32 ? 2 * d : d;
    GateLaunch g{};
    g.waves = waves;
    g.splits = gate_k_splits(dtype, S, d_units, waves);
    g.blocks = blocks;
    g.st = st;
    g.x = static_cast<const uint16_t*>(x);
    g.w = static_cast<const uint16_t*>(w);
    g.S = S;
    g.d_units = d_units;
    g.N = N;
    g.k = k;
    g.logits = logits;
    g.topk_idx = topk_idx;
    g.topk_w = topk_w;
    if (g.splits > 1) {
        // fp32, few token tiles: K shares on grid rows, partial scores in the workspace, then the
        // selection kernel adds them
        float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + lay.part_logits);
        g.logits = part;
        launch_gate_f32_split(g);
        if ((rc = check_launch(fn, "gate_f32_split_kernel")) != TAMOE_OK) return rc;
        blocks = ceil_div(S, 128);
        run->stats = stats_in(ws, lay, k, blocks);
        run->tile_tokens = 128;
        launch_select(blocks, st, part, g.splits, (size_t)S * N, logits, S, N, k, topk_idx, topk_w, run->stats);
        return check_launch(fn, "select_kernel");
    }
    run->stats = stats_in(ws, lay, k, blocks);
    run->tile_tokens = 32 * waves;
    g.stats = run->stats;
    if (dtype == TAMOE_F32)
        launch_gate_f32(g);
    else if (dtype == TAMOE_F16)
        launch_gate_f16(g);
    else
        launch_gate_bf16(g);
    return check_launch(fn, gate_kernel_name(dtype));
}

static int finalize(const char* fn, const GateRun& run, int N, int P, int k, int64_t S, float* m, int32_t* c_expert,
                    int32_t* c_device, hipStream_t st) {
    {
        TraceScope tr("gate_finalize_kernel", st);
        gate_finalize_kernel<<<dim3(N), dim3(256), 0, st>>>(run.stats.m_part, run.stats.tile_pairs, run.stats.n_blocks,
                                                            k * run.stats.n_blocks, run.stats.pitch, N, P, S, m,
                                                            c_expert, c_device);
    }
    return check_launch(fn, "gate_finalize_kernel");
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_select(const float* logits, int64_t S, int N, int P, int k, int32_t* topk_idx, float* topk_w,
                            float* m, int32_t* c_expert, int32_t* c_device, void* ws, size_t ws_bytes, void* stream) {
    const char* fn = "tamoe_select";
    clear_error();
    int rc;
    if ((rc = check_shape(fn, S, N, P, k)) != TAMOE_OK) return rc;
    if (S > 0 && (rc = check_ptr(fn, "logits", logits, 4)) != TAMOE_OK) return rc;
    const Workspace lay = workspace_layout(S, N, k);
    if ((rc = check_select_outputs(fn, S, topk_idx, topk_w, m, c_expert, c_device, ws, ws_bytes, lay)) != TAMOE_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    GateRun run{};
    if ((rc = run_select_stage(fn, logits, S, N, k, topk_idx, topk_w, ws, lay, st, &run)) != TAMOE_OK) return rc;
    return finalize(fn, run, N, P, k, S, m, c_expert, c_device, st);
}

extern "C" int tamoe_gate(const void* x, const void* w, int dtype, int64_t S, int d, int N, int P, int k,
                          float* logits, int32_t* topk_idx, float* topk_w, float* m, int32_t* c_expert,
                          int32_t* c_device, void* ws, size_t ws_bytes, void* stream) {
    const char* fn = "tamoe_gate";
    clear_error();
    int rc;
    if ((rc = check_shape(fn, S, N, P, k)) != TAMOE_OK) return rc;
    if ((rc = check_rows(fn, dtype, d)) != TAMOE_OK) return rc;
    if (S > 0) {
        if ((rc = check_ptr(fn, "x", x, 16)) != TAMOE_OK) return rc;
        if ((rc = check_ptr(fn, "w", w, 16)) != TAMOE_OK) return rc;
    }
    const Workspace lay = workspace_layout(S, N, k, dtype);
    if ((rc = check_select_outputs(fn, S, topk_idx, topk_w, m, c_expert, c_device, ws, ws_bytes, lay)) != TAMOE_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    GateRun run{};
    if ((rc = run_gate_stage(fn, x, w, dtype, S, d, N, k, logits, topk_idx, topk_w, ws, lay, st, &run)) != TAMOE_OK)
        return rc;
    return finalize(fn, run, N, P, k, S, m, c_expert, c_device, st);
}
