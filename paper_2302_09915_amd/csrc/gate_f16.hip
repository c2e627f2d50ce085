// The gate's tile kernels for half-precision storage (instantiations only; the code is in gate_tile.h).
#include "gate_tile.h"

namespace tamoe {

void launch_gate_f16(const GateLaunch& g) { launch_gate_typed<TAMOE_F16>(g); }

}  // namespace tamoe
