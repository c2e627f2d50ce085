// tamoe_aux_loss: the topology-aware auxiliary loss of paper Section 4.3,
//   l_topo = N*P * sum_e p[e] * m[e] * c[e] / S,
// or, without a penalty vector, the load-balance loss of Section 3.1, l_aux = sum_e m[e]*c[e]/S.
// N <= 128 terms: one workgroup, one term per thread, fixed-order tree sum in fp32.
#include "internal.h"

namespace tamoe {

__global__ __launch_bounds__(TAMOE_MAX_EXPERTS) void aux_loss_kernel(const float* __restrict__ m,
                                                                     const int32_t* __restrict__ c,
                                                                     const float* __restrict__ penalty, int N,
                                                                     float scale, float* __restrict__ loss) {
    __shared__ float term[TAMOE_MAX_EXPERTS];
    const int e = threadIdx.x;
    float v = 0.f;
    if (e < N) {
        v = m[e] * (float)c[e];
        if (penalty != nullptr) v *= penalty[e];
    }
    term[e] = v;
    __syncthreads();
    for (int stride = TAMOE_MAX_EXPERTS / 2; stride > 0; stride >>= 1) {
        if (e < stride) term[e] += term[e + stride];
        __syncthreads();
    }
    if (e == 0) loss[0] = term[0] * scale;
}

}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_aux_loss(const float* m, const int32_t* c_expert, const float* penalty, int N, int P, int64_t S,
                              float* loss, void* stream) {
    const char* fn = "tamoe_aux_loss";
    clear_error();
    int rc;
    if (N <= 0 || P <= 0) return fail(TAMOE_INVALID_ARG, "%s: N = %d and P = %d must be positive", fn, N, P);
    if (S <= 0) return fail(TAMOE_INVALID_ARG, "%s: S = %lld must be positive", fn, (long long)S);
    if (N % P != 0) return fail(TAMOE_INVALID_ARG, "%s: N = %d is not a multiple of P = %d", fn, N, P);
    if (N > TAMOE_MAX_EXPERTS)
        return fail(TAMOE_UNSUPPORTED, "%s: N = %d exceeds the limit of %d experts", fn, N, TAMOE_MAX_EXPERTS);
    if ((rc = check_ptr(fn, "m", m, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "c_expert", c_expert, 4)) != TAMOE_OK) return rc;
    if ((rc = check_ptr(fn, "loss", loss, 4)) != TAMOE_OK) return rc;
    if (penalty != nullptr && (rc = check_ptr(fn, "penalty", penalty, 4)) != TAMOE_OK) return rc;
    // scale in double on the host, one rounding to fp32
    const float scale = (float)((penalty != nullptr ? (double)N * (double)P : 1.0) / (double)S);
    hipStream_t st = static_cast<hipStream_t>(stream);
    {
        TraceScope tr("aux_loss_kernel", st);
        aux_loss_kernel<<<dim3(1), dim3(TAMOE_MAX_EXPERTS), 0, st>>>(m, c_expert, penalty, N, scale, loss);
    }
    return check_launch(fn, "aux_loss_kernel");
}
