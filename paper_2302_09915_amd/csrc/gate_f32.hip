// The gate's tile kernels for fp32 storage: whole-K tiles and the K-split variant for small batches
// (instantiations only; the code is in gate_tile.h).
#include "gate_tile.h"

namespace tamoe {

void launch_gate_f32(const GateLaunch& g) { launch_gate_typed<TAMOE_F32>(g); }

void launch_gate_f32_split(const GateLaunch& g) {
    const dim3 grid((unsigned)g.blocks, (unsigned)g.splits);
    const bool ktail = g.d_units % kKC != 0;
    TraceScope tr("gate_f32_split_kernel", g.st);
#define TAMOE_SPLIT(NBV)                                                                                          \
    do {                                                                                                          \
        if (ktail)                                                                                                \
            gate_f32_split_kernel<NBV, true><<<grid, dim3(64), 0, g.st>>>(g.x, g.w, g.S, g.d_units, g.N, g.k,     \
                                                                           g.logits, g.topk_idx, g.topk_w,         \
                                                                           g.stats);                               \
        else                                                                                                      \
            gate_f32_split_kernel<NBV, false><<<grid, dim3(64), 0, g.st>>>(g.x, g.w, g.S, g.d_units, g.N, g.k,    \
                                                                            g.logits, g.topk_idx, g.topk_w,        \
                                                                            g.stats);                              \
    } while (0)
    if (g.N <= 32)
        TAMOE_SPLIT(1);
    else if (g.N <= 64)
        TAMOE_SPLIT(2);
    else
        TAMOE_SPLIT(4);
#undef TAMOE_SPLIT
}

}  // namespace tamoe
