// tamoe_copy_probe: a plain 16-byte-per-lane device copy.  Not a step of the path: it is the
// yardstick the benchmark uses for the HBM bandwidth a simple streaming kernel reaches on this
// machine, and the kernel of known size against which hardware byte counters are calibrated.
#include "internal.h"

namespace tamoe {

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

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_copy_probe(const void* src, void* dst, size_t bytes, void* stream) {
    const char* fn = "tamoe_copy_probe";
    clear_error();
    int rc;
    if (bytes == 0) return TAMOE_OK;
    if (bytes % 16 != 0) return fail(TAMOE_INVALID_ARG, "%s: bytes = %zu is not a multiple of 16", fn, bytes);
    if ((rc = check_ptr(fn, "src", src, 16)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "dst", dst, 16)) != TAMOE_OK) return rc;
    const size_t n_vec = bytes / 16;
    const size_t blocks = (n_vec + kProbeThreads * kProbeUnroll - 1) / (kProbeThreads * kProbeUnroll);
    if (blocks > 0x7fffffffu) return fail(TAMOE_UNSUPPORTED, "%s: more than 2^31 blocks", fn);
    hipStream_t st = static_cast<hipStream_t>(stream);
    {
        TraceScope tr("copy_probe_kernel", st);
        copy_probe_kernel<<<dim3((unsigned)blocks), dim3(kProbeThreads), 0, st>>>(static_cast<const vec16*>(src),
                                                                                   static_cast<vec16*>(dst), n_vec);
    }
    return check_launch(fn, "copy_probe_kernel");
}
