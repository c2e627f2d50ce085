// Internal declarations shared by the translation units of libtamoe (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstddef>
#include <cstdint>

#include "tamoe.h"

namespace tamoe {

// 16 bytes as a native vector, the unit of every row copy (global_load/store_dwordx4).
typedef uint32_t vec16 __attribute__((ext_vector_type(4)));

// Records the message returned by tamoe_last_error() and passes `code` through.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int elem_bytes(int dtype) { return dtype == TAMOE_F32 ? 4 : 2; }

// ---- launch geometry (host side; the kernels receive what they need as arguments) ----------

// Gate: a workgroup of 64*waves threads scores 32*waves tokens (one 32-token MFMA column block
// per wavefront).  More wavefronts per workgroup share one LDS copy of the W tile; fewer give
// more workgroups when S is small.
int gate_waves(int64_t S, int N);
// K-split gate (fp32 storage, one-wavefront workgroups, fewer token tiles than half the SIMDs): the
// number of K shares, 1 = no split.  d_units: row length in 2-byte units.
constexpr int kMaxKSplits = 8;
constexpr int64_t kSplitMaxTokens = 16384;  // above this the token tiles alone fill the device
int gate_k_splits(int dtype, int64_t S, int d_units, int waves);
// Upper bound of the number of gate workgroups over every choice of waves.
inline int64_t gate_blocks_max(int64_t S) { return ceil_div(S, 32); }

// Dispatch: pairs are counted per "count tile" of kCountTile tokens.
constexpr int kCountTile = 1024;
inline int64_t count_tiles(int64_t S) { return ceil_div(S, kCountTile); }

// ---- workspace layout -----------------------------------------------------------------------
// Row pitch of the gate's pair-count table for `blocks` gate workgroups: a multiple of 64 entries, so
// that every expert's row starts on a 256-byte boundary and can be read in 16-byte pieces.
inline int64_t pair_pitch(int k, int64_t blocks) { return (int64_t)align_up((size_t)((int64_t)k * blocks), 64); }

struct Workspace {
    size_t m_part;      // float  [N][gate blocks]        per-workgroup sums of gate probabilities
    size_t tile_pairs;  // int32  [N][pair_pitch]         gate: pairs per (expert; choice, workgroup), then their
                        //                                exclusive prefix in priority order
    size_t local_pos;   // int32  [S][k]                  gate: position of a pair among those of its workgroup
    size_t tile_count;  // int32  [k][count_tiles][N]     dispatch on given routing: pair counts, then their prefix
    size_t part_logits; // float  [kMaxKSplits][S][N]     partial scores of a K-split gate (small S only)
    size_t total;
};
// dtype: only fp32 storage adds the partial-score region (the gate's K split); every other region sits
// at the same offset for every storage type.
Workspace workspace_layout(int64_t S, int N, int k, int dtype = TAMOE_BF16);

// Where the block-wide results of the selection go (device memory, the caller's workspace).
struct GateStats {
    float* m_part;        // [N][n_blocks]      sums of gate probabilities per workgroup
    int32_t* tile_pairs;  // [N][pitch]         pairs per (expert; choice j, workgroup b) at [e*pitch + j*n_blocks + b]
    int32_t* local_pos;   // [S][k]             earlier pairs of the same workgroup with the same expert and choice
    int n_blocks;
    int pitch;
};

// What the gate stage left in the workspace for the stages behind it.
struct GateRun {
    GateStats stats;
    int tile_tokens;      // tokens per gate workgroup: token t belongs to workgroup t / tile_tokens
};
// The gate's kernels up to the per-workgroup partial results (no finalize).  Arguments are those of
// tamoe_gate / tamoe_select, already checked.
int run_gate_stage(const char* fn, const void* x, const void* w, int dtype, int64_t S, int d, int N, int k,
                   float* logits, int32_t* topk_idx, float* topk_w, void* ws, const Workspace& lay, hipStream_t st,
                   GateRun* run);
int run_select_stage(const char* fn, const float* logits, int64_t S, int N, int k, int32_t* topk_idx, float* topk_w,
                     void* ws, const Workspace& lay, hipStream_t st, GateRun* run);
int check_select_outputs(const char* fn, int64_t S, int32_t* topk_idx, float* topk_w, float* m, int32_t* c_expert,
                         int32_t* c_device, void* ws, size_t ws_bytes, const Workspace& lay);

// Rows written by the scatter stay in the last-level cache (ordinary stores) when the whole send buffer
// fits well inside its 256 MB, so that whoever reads them next (the exchange, a local expert, the
// combine of an identity layer) finds them there; larger buffers are written with streaming stores,
// which do not push the token matrix out of that cache while the scatter still reads it.  Measured:
// GPT-MoE layer (64 MiB of rows) 62.2 -> 60.6 us per step, skewed 59.8 -> 55.9, large (1 GiB) 648 -> 661.
constexpr int64_t kCacheResidentSendBytes = (int64_t)96 << 20;
inline bool send_stays_in_cache(int64_t S, int k, int cpr) { return S * k * (int64_t)cpr * 16 <= kCacheResidentSendBytes; }

// log2(v) if v is a power of two, else -1.
inline int pow2_shift(int v) {
    if (v <= 0 || (v & (v - 1)) != 0) return -1;
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

// Chunk index -> (row, column) for a matrix of `cpr` 16-byte chunks per row.
__device__ __forceinline__ void split_chunk(int64_t c, int64_t total, int cpr, int shift, int& row, int& col) {
    if (shift >= 0) {
        row = (int)(c >> shift);
        col = (int)c & (cpr - 1);
    } else if (total <= 0xffffffffll) {
        const uint32_t r = (uint32_t)c / (uint32_t)cpr;
        row = (int)r;
        col = (int)((uint32_t)c - r * (uint32_t)cpr);
    } else {
        const int64_t r = c / cpr;
        row = (int)r;
        col = (int)(c - r * cpr);
    }
}

// Common argument checks.  Return TAMOE_OK or a failure already recorded with fail().
int check_shape(const char* fn, int64_t S, int N, int P, int k);
int check_rows(const char* fn, int dtype, int d);
int check_ptr(const char* fn, const char* name, const void* p, size_t align);
int check_launch(const char* fn, const char* kernel);

// Brackets one kernel launch with a pair of events while a trace is running (tamoe_trace_start);
// a single branch otherwise.
extern std::atomic<bool> g_trace_on;
bool trace_begin(const char* kernel, hipStream_t st);
void trace_end(hipStream_t st);
struct TraceScope {
    hipStream_t st;
    bool on;
    TraceScope(const char* kernel, hipStream_t s) : st(s), on(false) {
        if (g_trace_on.load(std::memory_order_relaxed)) on = trace_begin(kernel, st);
    }
    ~TraceScope() {
        if (on) trace_end(st);
    }
};

}  // namespace tamoe
