// Host side of libtamoe: error reporting, argument checks, workspace layout and the setup-time
// derivation of the target dispatch pattern.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <map>
#include <mutex>
#include <vector>

#include "internal.h"

namespace tamoe {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

int gate_waves(int64_t S, int N) {
    // eight wavefronts (one workgroup per compute unit, 256 CUs) halve the traffic of W once
    // there are enough tokens; otherwise aim for two workgroups per compute unit, except that two
    // wavefronts sharing a W tile beat single-wavefront workgroups as soon as every compute unit
    // gets one (16384 tokens: 15.2 -> 13.3 us at d = 1024, 21.4 -> 18.6 us at d = 2048)
    if (N > 32 && ceil_div(S, 256) >= 256) return 8;
    if (ceil_div(S, 128) >= 512) return 4;
    if (ceil_div(S, 64) >= 256) return 2;
    return 1;
}

int gate_k_splits(int dtype, int64_t S, int d_units, int waves) {
    if (dtype != TAMOE_F32 || waves != 1 || S <= 0 || S >= kSplitMaxTokens) return 1;
    const int64_t tiles = ceil_div(S, 32);
    const int64_t room = 1024 / tiles;                    // wavefronts the device still has room for, per tile
    const int64_t by_chunks = ceil_div(d_units, 64) / 8;  // at least eight 128-byte chunks per share
    const int64_t s = room < by_chunks ? room : by_chunks;
    return (int)(s < 1 ? 1 : (s > kMaxKSplits ? kMaxKSplits : s));
}

Workspace workspace_layout(int64_t S, int N, int k, int dtype) {
    Workspace w{};
    size_t off = 0;
    const size_t gb = (size_t)gate_blocks_max(S);
    w.m_part = off;
    off = align_up(off + gb * N * sizeof(float), 256);
    w.tile_pairs = off;
    off = align_up(off + (size_t)pair_pitch(k, (int64_t)gb) * N * sizeof(int32_t), 256);
    w.local_pos = off;
    off = align_up(off + (size_t)S * k * sizeof(int32_t), 256);
    w.tile_count = off;
    off = align_up(off + (size_t)k * count_tiles(S) * N * sizeof(int32_t), 256);
    // last, so that the other offsets do not depend on the storage type; sized for the largest batch
    // that can be split, so that the total grows with S
    w.part_logits = off;
    if (dtype == TAMOE_F32) {
        const int64_t rows = S < kSplitMaxTokens ? S : kSplitMaxTokens;
        off = align_up(off + (size_t)kMaxKSplits * rows * N * sizeof(float), 256);
    }
    w.total = off < 4096 ? 4096 : off;  // never less than the offset tables of tamoe_regroup
    return w;
}

int check_shape(const char* fn, int64_t S, int N, int P, int k) {
    if (S < 0) return fail(TAMOE_INVALID_ARG, "%s: S = %lld is negative", fn, (long long)S);
    if (N <= 0 || P <= 0 || k <= 0)
        return fail(TAMOE_INVALID_ARG, "%s: N = %d, P = %d, k = %d must all be positive", fn, N, P, k);
    if (k > N) return fail(TAMOE_INVALID_ARG, "%s: k = %d exceeds N = %d", fn, k, N);
    if (N % P != 0) return fail(TAMOE_INVALID_ARG, "%s: N = %d is not a multiple of P = %d", fn, N, P);
    if (N > TAMOE_MAX_EXPERTS)
        return fail(TAMOE_UNSUPPORTED, "%s: N = %d exceeds the limit of %d experts", fn, N, TAMOE_MAX_EXPERTS);
    if (k > TAMOE_MAX_K) return fail(TAMOE_UNSUPPORTED, "%s: k = %d exceeds the limit of %d", fn, k, TAMOE_MAX_K);
    if (S * (int64_t)k >= (int64_t)1 << 31)
        return fail(TAMOE_UNSUPPORTED, "%s: S*k = %lld does not fit int32 slots", fn, (long long)(S * k));
    return TAMOE_OK;
}

int check_rows(const char* fn, int dtype, int d) {
    if (dtype != TAMOE_F32 && dtype != TAMOE_BF16 && dtype != TAMOE_F16)
        return fail(TAMOE_UNSUPPORTED, "%s: dtype %d is none of TAMOE_F32, TAMOE_BF16, TAMOE_F16", fn, dtype);
    if (d <= 0) return fail(TAMOE_INVALID_ARG, "%s: d = %d must be positive", fn, d);
    if (((int64_t)d * elem_bytes(dtype)) % 16 != 0)
        return fail(TAMOE_UNSUPPORTED, "%s: a row of d = %d elements is not a multiple of 16 bytes", fn, d);
    return TAMOE_OK;
}

int check_ptr(const char* fn, const char* name, const void* p, size_t align) {
    if (p == nullptr) return fail(TAMOE_INVALID_ARG, "%s: %s is NULL", fn, name);
    if (align > 1 && (reinterpret_cast<uintptr_t>(p) % align) != 0)
        return fail(TAMOE_INVALID_ARG, "%s: %s is not %zu-byte aligned", fn, name, align);
    return TAMOE_OK;
}

int check_launch(const char* fn, const char* kernel) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(TAMOE_HIP_ERROR, "%s: launch of %s failed: %s", fn, kernel, hipGetErrorString(e));
    return TAMOE_OK;
}

// ---- kernel timing aid --------------------------------------------------------------------
std::atomic<bool> g_trace_on{false};
namespace {
std::mutex g_trace_lock;              // guards everything below
struct TraceRecord {
    const char* kernel;
    hipEvent_t begin, end;
};
std::vector<TraceRecord> g_records;   // capacity fixed by tamoe_trace_start
size_t g_used = 0;
bool g_open = false;                  // a begin without its end
char g_filter[64] = "";               // "" = every kernel
}  // namespace

// Opens a record for this launch and returns true, or returns false (filtered out, table full, or a
// launch of another thread is being bracketed: records never nest).
bool trace_begin(const char* kernel, hipStream_t st) {
    std::lock_guard<std::mutex> hold(g_trace_lock);
    if (g_open) return false;
    if (g_filter[0] != '\0' && std::strcmp(kernel, g_filter) != 0) return false;
    if (g_used >= g_records.size()) {
        g_trace_on = false;
        return false;
    }
    g_records[g_used].kernel = kernel;
    g_open = hipEventRecord(g_records[g_used].begin, st) == hipSuccess;
    return g_open;
}

// Closes the record that the caller's trace_begin opened.
void trace_end(hipStream_t st) {
    std::lock_guard<std::mutex> hold(g_trace_lock);
    if (!g_open) return;              // cleared in between
    g_open = false;
    if (hipEventRecord(g_records[g_used].end, st) == hipSuccess) ++g_used;
    if (g_used >= g_records.size()) g_trace_on = false;
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_trace_clear(void) {
    std::lock_guard<std::mutex> hold(g_trace_lock);
    g_trace_on = false;
    for (auto& r : g_records) {
        (void)hipEventDestroy(r.begin);
        (void)hipEventDestroy(r.end);
    }
    g_records.clear();
    g_used = 0;
    g_open = false;
    return TAMOE_OK;
}

extern "C" int tamoe_trace_start(int max_launches) {
    clear_error();
    if (max_launches <= 0 || max_launches > (1 << 20))
        return fail(TAMOE_INVALID_ARG, "tamoe_trace_start: max_launches = %d outside (0, 2^20]", max_launches);
    tamoe_trace_clear();
    std::lock_guard<std::mutex> hold(g_trace_lock);
    g_records.reserve((size_t)max_launches);
    for (int i = 0; i < max_launches; ++i) {
        TraceRecord r{nullptr, nullptr, nullptr};
        if (hipEventCreate(&r.begin) != hipSuccess || hipEventCreate(&r.end) != hipSuccess) {
            for (auto& q : g_records) {
                (void)hipEventDestroy(q.begin);
                (void)hipEventDestroy(q.end);
            }
            g_records.clear();
            return fail(TAMOE_HIP_ERROR, "tamoe_trace_start: hipEventCreate failed");
        }
        g_records.push_back(r);
    }
    g_trace_on = true;
    return TAMOE_OK;
}

extern "C" int tamoe_trace_filter(const char* kernel_name) {
    clear_error();
    std::lock_guard<std::mutex> hold(g_trace_lock);
    if (kernel_name == nullptr) {
        g_filter[0] = '\0';
        return TAMOE_OK;
    }
    if (std::strlen(kernel_name) >= sizeof(g_filter))
        return fail(TAMOE_INVALID_ARG, "tamoe_trace_filter: kernel name longer than %zu characters", sizeof(g_filter) - 1);
    std::strcpy(g_filter, kernel_name);
    return TAMOE_OK;
}

extern "C" int tamoe_trace_stop(void) {
    clear_error();
    g_trace_on = false;
    std::lock_guard<std::mutex> hold(g_trace_lock);
    if (g_used > 0 && hipEventSynchronize(g_records[g_used - 1].end) != hipSuccess)
        return -fail(TAMOE_HIP_ERROR, "tamoe_trace_stop: hipEventSynchronize failed");
    return (int)g_used;
}

extern "C" int tamoe_trace_get(int i, char* name, size_t name_len, float* ms) {
    clear_error();
    std::lock_guard<std::mutex> hold(g_trace_lock);
    if (i < 0 || (size_t)i >= g_used) return fail(TAMOE_INVALID_ARG, "tamoe_trace_get: record %d does not exist", i);
    if (name != nullptr && name_len > 0) {
        std::snprintf(name, name_len, "%s", g_records[i].kernel);
    }
    if (ms != nullptr && hipEventElapsedTime(ms, g_records[i].begin, g_records[i].end) != hipSuccess)
        return fail(TAMOE_HIP_ERROR, "tamoe_trace_get: hipEventElapsedTime failed");
    return TAMOE_OK;
}

extern "C" int tamoe_version(void) { return TAMOE_VERSION; }

extern "C" const char* tamoe_last_error(void) { return g_err; }

extern "C" size_t tamoe_workspace_bytes(int64_t S, int d, int N, int P, int k, int dtype) {
    (void)d; (void)P;
    if (S < 0 || N <= 0 || k <= 0) return 0;
    return workspace_layout(S, N, k, dtype).total;
}

// Setup stage.  Per-level means of the profiled inverse bandwidths, then the closed-form target
// pattern of Section 4.2 (volume sent over a link inversely proportional to its inverse
// bandwidth, scaled so that the row sums to k*S), the L1-normalised reciprocal as penalty
// (Section 4.3) and the local capacities.
extern "C" int tamoe_topo_pattern(const double* beta, const int32_t* level, int P, int N, int rank,
                                  int k, int64_t S, double capacity_factor, int cap_mode,
                                  double* c_hat, float* penalty, int32_t* cap) {
    const char* fn = "tamoe_topo_pattern";
    clear_error();
    if (beta == nullptr) return fail(TAMOE_INVALID_ARG, "%s: beta is NULL", fn);
    if (N <= 0 || P <= 0 || k <= 0 || S <= 0)
        return fail(TAMOE_INVALID_ARG, "%s: N = %d, P = %d, k = %d, S = %lld must all be positive", fn, N, P, k,
                    (long long)S);
    if (N % P != 0) return fail(TAMOE_INVALID_ARG, "%s: N = %d is not a multiple of P = %d", fn, N, P);
    if (k > N) return fail(TAMOE_INVALID_ARG, "%s: k = %d exceeds N = %d", fn, k, N);
    if (rank < 0 || rank >= P) return fail(TAMOE_INVALID_ARG, "%s: rank = %d outside [0, %d)", fn, rank, P);
    if (cap_mode != TAMOE_CAP_UNIFORM && cap_mode != TAMOE_CAP_PROPORTIONAL)
        return fail(TAMOE_INVALID_ARG, "%s: unknown cap_mode %d", fn, cap_mode);
    if (!(capacity_factor > 0.0) || !std::isfinite(capacity_factor))
        return fail(TAMOE_INVALID_ARG, "%s: capacity_factor must be positive and finite", fn);
    for (int q = 0; q < P * P; ++q) {
        if (!(beta[q] > 0.0) || !std::isfinite(beta[q]))
            return fail(TAMOE_INVALID_ARG, "%s: beta[%d][%d] = %g is not a positive finite number", fn, q / P, q % P,
                        beta[q]);
        if (level != nullptr && level[q] < 0)
            return fail(TAMOE_INVALID_ARG, "%s: level[%d][%d] = %d is negative", fn, q / P, q % P, level[q]);
    }

    // Row `rank` of the hierarchical matrix.
    std::vector<double> row(beta + (size_t)rank * P, beta + (size_t)(rank + 1) * P);
    if (level != nullptr) {
        // labels are arbitrary non-negative integers: sums are kept per label that occurs
        struct LevelSum {
            double pair_sum = 0.0, self_sum = 0.0;
            int64_t pair_cnt = 0, self_cnt = 0;
        };
        std::map<int32_t, LevelSum> by_level;
        for (int a = 0; a < P; ++a) {
            for (int b = a; b < P; ++b) {
                LevelSum& s = by_level[level[a * P + b]];
                if (a == b) { s.self_sum += beta[a * P + b]; s.self_cnt += 1; }
                else        { s.pair_sum += beta[a * P + b]; s.pair_cnt += 1; }
            }
        }
        for (int j = 0; j < P; ++j) {
            // level[rank][j] and level[j][rank] may differ in a table that is not symmetric; the
            // upper triangle was summed, the label of the row is looked up
            const auto it = by_level.find(level[rank * P + j]);
            if (it == by_level.end() || (it->second.pair_cnt == 0 && it->second.self_cnt == 0))
                return fail(TAMOE_INVALID_ARG, "%s: level[%d][%d] = %d labels no pair i <= j", fn, rank, j,
                            level[rank * P + j]);
            const LevelSum& s = it->second;
            row[j] = s.pair_cnt > 0 ? s.pair_sum / (double)s.pair_cnt : s.self_sum / (double)s.self_cnt;
        }
    }

    const int E = N / P;
    double inv_sum = 0.0;
    for (int j = 0; j < P; ++j) inv_sum += 1.0 / row[j];
    const double share_unit = (double)k * (double)S / ((double)E * inv_sum);  // rows * beta per expert
    std::vector<double> target(N);
    double recip_sum = 0.0;
    for (int e = 0; e < N; ++e) {
        target[e] = share_unit / row[e / E];
        recip_sum += 1.0 / target[e];
    }
    for (int e = 0; e < N; ++e) {
        if (c_hat) c_hat[e] = target[e];
        if (penalty) penalty[e] = (float)((1.0 / target[e]) / recip_sum);
        if (cap) {
            const double v = cap_mode == TAMOE_CAP_UNIFORM ? capacity_factor * (double)k * (double)S / (double)N
                                                           : capacity_factor * target[e];
            const double c = std::ceil(v - 1e-9);
            if (c > 2147483647.0) return fail(TAMOE_UNSUPPORTED, "%s: capacity %g does not fit int32", fn, c);
            cap[e] = (int32_t)c;
        }
    }
    return TAMOE_OK;
}

// Norm variants of the penalty (Section 4.3).  The softmax form works on the reciprocal pattern
// in units of its own mean, so that `temperature` has the same meaning for every N and S; the
// largest argument is subtracted before exponentiation.
extern "C" int tamoe_penalty(const double* c_hat, int N, int norm, double temperature, float* penalty) {
    const char* fn = "tamoe_penalty";
    clear_error();
    if (c_hat == nullptr || penalty == nullptr) return fail(TAMOE_INVALID_ARG, "%s: NULL pointer", fn);
    if (N <= 0) return fail(TAMOE_INVALID_ARG, "%s: N = %d must be positive", fn, N);
    if (norm != TAMOE_NORM_L1 && norm != TAMOE_NORM_SOFTMAX)
        return fail(TAMOE_INVALID_ARG, "%s: unknown norm %d", fn, norm);
    if (norm == TAMOE_NORM_SOFTMAX && (!(temperature >= 0.0) || !std::isfinite(temperature)))
        return fail(TAMOE_INVALID_ARG, "%s: temperature must be finite and >= 0", fn);
    double recip_sum = 0.0;
    for (int e = 0; e < N; ++e) {
        if (!(c_hat[e] > 0.0) || !std::isfinite(c_hat[e]))
            return fail(TAMOE_INVALID_ARG, "%s: c_hat[%d] = %g is not a positive finite number", fn, e, c_hat[e]);
        recip_sum += 1.0 / c_hat[e];
    }
    if (norm == TAMOE_NORM_L1) {
        for (int e = 0; e < N; ++e) penalty[e] = (float)((1.0 / c_hat[e]) / recip_sum);
        return TAMOE_OK;
    }
    const double scale = temperature * (double)N / recip_sum;  // temperature / mean of the reciprocals
    std::vector<double> z(N);
    double top = 0.0;
    for (int e = 0; e < N; ++e) {
        z[e] = scale / c_hat[e];
        top = e == 0 || z[e] > top ? z[e] : top;
    }
    double denom = 0.0;
    for (int e = 0; e < N; ++e) {
        z[e] = std::exp(z[e] - top);
        denom += z[e];
    }
    for (int e = 0; e < N; ++e) penalty[e] = (float)(z[e] / denom);
    return TAMOE_OK;
}
