// The gate's tile kernels for bfloat16 storage (instantiations only; the code is in gate_tile.h).
#include "gate_tile.h"

namespace tamoe {

void launch_gate_bf16(const GateLaunch& g) { launch_gate_typed<TAMOE_BF16>(g); }

}  // namespace tamoe
