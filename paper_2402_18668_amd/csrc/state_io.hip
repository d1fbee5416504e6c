// Copies between the library's state buffer and the canonical dense arrays S [U][D][d_v], z [U][D].
#include "common.h"

namespace based {

__global__ void state_copy_kernel(float *state, float *S, float *z, int D, int dv, size_t stride,
                                  int to_state)
{
    const int u = blockIdx.x;
    float *su = state + (size_t)u * stride;
    const int nS = D * dv;
    if (S) {
        float *Su = S + (size_t)u * nS;
        for (int i = threadIdx.x; i < nS; i += blockDim.x) {
            if (to_state) su[i] = Su[i]; else Su[i] = su[i];
        }
    }
    if (z) {
        float *zu = z + (size_t)u * D;
        for (int i = threadIdx.x; i < D; i += blockDim.x) {
            if (to_state) su[nS + i] = zu[i]; else zu[i] = su[nS + i];
        }
    }
}

hipError_t launch_state_copy(float *state, float *S, float *z, int U, int dp, int dv, int to_state,
                             hipStream_t s)
{
    hipLaunchKernelGGL(state_copy_kernel, dim3(U), dim3(256), 0, s, state, S, z, feature_dim(dp), dv,
                       state_stride(dp, dv), to_state);
    return hipGetLastError();
}

}  // namespace based
