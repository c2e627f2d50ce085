// Bandwidth yardsticks for the benchmark (libtamoe_bench.so; not part of the product library):
// tamoe_copy_probe, a plain 16-byte-per-lane device copy (the HBM bandwidth a simple streaming kernel
// reaches on this machine, and the kernel of known size against which hardware byte counters are
// calibrated), and tamoe_mix_probe, the bare memory operations of the scatter and of the combine on
// given row tables.  Self-contained: no code shared with the library's kernels.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "tamoe_bench.h"

namespace {

typedef uint32_t vec16 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 4;

__global__ __launch_bounds__(kProbeThreads) void copy_probe_kernel(const vec16* __restrict__ src,
                                                                   vec16* __restrict__ dst, size_t n_vec) {
    const size_t base = (size_t)blockIdx.x * (kProbeThreads * kProbeUnroll) + threadIdx.x;
    vec16 v[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
        const size_t i = base + (size_t)u * kProbeThreads;
        if (i < n_vec) v[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
        const size_t i = base + (size_t)u * kProbeThreads;
        if (i < n_vec) __builtin_nontemporal_store(v[u], dst + i);
    }
}

// Row-mix yardsticks: the memory operations of the scatter (one row read, two row writes) and of
// the combine (two row reads, one row write) on given row tables, with nothing else around them.
// One 16-byte chunk per thread; a row is a multiple of 1 KiB, so a wavefront stays inside one row
// and reads its two row numbers through the scalar unit.  Negative or out-of-range rows are skipped.
template <int MODE>
__global__ __launch_bounds__(kProbeThreads) void mix_probe_kernel(const vec16* __restrict__ a, vec16* __restrict__ b,
                                                                  const int32_t* __restrict__ row0,
                                                                  const int32_t* __restrict__ row1, int64_t total,
                                                                  int cpr, int64_t other_rows) {
    const int64_t c = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
    if (c >= total) return;
    const int t = __builtin_amdgcn_readfirstlane((int)(c / cpr));
    const int col = (int)(c - (int64_t)t * cpr);
    const int32_t r0 = row0[t], r1 = row1[t];
    const bool ok0 = r0 >= 0 && r0 < other_rows, ok1 = r1 >= 0 && r1 < other_rows;
    if (MODE == 1) {
        if (!ok0 && !ok1) return;
        const vec16 v = __builtin_nontemporal_load(a + c);
        if (ok0) __builtin_nontemporal_store(v, b + (size_t)r0 * cpr + col);
        if (ok1) __builtin_nontemporal_store(v, b + (size_t)r1 * cpr + col);
    } else {
        vec16 v = {0u, 0u, 0u, 0u};
        if (ok0) v = __builtin_nontemporal_load(a + (size_t)r0 * cpr + col);
        if (ok1) v ^= __builtin_nontemporal_load(a + (size_t)r1 * cpr + col);
        __builtin_nontemporal_store(v, b + c);
    }
}

}  // namespace

static bool aligned16(const void* p) { return p != nullptr && reinterpret_cast<uintptr_t>(p) % 16 == 0; }

extern "C" int tamoe_mix_probe(const void* a, void* b, const int32_t* row0, const int32_t* row1, int64_t rows,
                               int64_t other_rows, int row_bytes, int mode, void* stream) {
    if (mode != 1 && mode != 2) return TAMOE_BENCH_BAD_ARG;
    if (rows < 0 || other_rows < 0) return TAMOE_BENCH_BAD_ARG;
    if (row_bytes <= 0 || row_bytes % 1024 != 0) return TAMOE_BENCH_BAD_ARG;
    if (rows == 0) return TAMOE_BENCH_OK;
    if (!aligned16(a) || !aligned16(b) || row0 == nullptr || row1 == nullptr) return TAMOE_BENCH_BAD_ARG;
    const int cpr = row_bytes / 16;
    const int64_t total = rows * cpr;
    const int64_t blocks = (total + kProbeThreads - 1) / kProbeThreads;
    if (rows >= ((int64_t)1 << 31) || blocks > 0x7fffffff) return TAMOE_BENCH_BAD_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    {
        if (mode == 1)
            mix_probe_kernel<1><<<dim3((unsigned)blocks), dim3(kProbeThreads), 0, st>>>(
                static_cast<const vec16*>(a), static_cast<vec16*>(b), row0, row1, total, cpr, other_rows);
        else
            mix_probe_kernel<2><<<dim3((unsigned)blocks), dim3(kProbeThreads), 0, st>>>(
                static_cast<const vec16*>(a), static_cast<vec16*>(b), row0, row1, total, cpr, other_rows);
    }
    return hipGetLastError() == hipSuccess ? TAMOE_BENCH_OK : TAMOE_BENCH_HIP_ERROR;
}

extern "C" int tamoe_copy_probe(const void* src, void* dst, size_t bytes, void* stream) {
    if (bytes == 0) return TAMOE_BENCH_OK;
    if (bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return TAMOE_BENCH_BAD_ARG;
    const size_t n_vec = bytes / 16;
    const size_t blocks = (n_vec + kProbeThreads * kProbeUnroll - 1) / (kProbeThreads * kProbeUnroll);
    if (blocks > 0x7fffffffu) return TAMOE_BENCH_BAD_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    {
        copy_probe_kernel<<<dim3((unsigned)blocks), dim3(kProbeThreads), 0, st>>>(static_cast<const vec16*>(src),
                                                                                   static_cast<vec16*>(dst), n_vec);
    }
    return hipGetLastError() == hipSuccess ? TAMOE_BENCH_OK : TAMOE_BENCH_HIP_ERROR;
}
