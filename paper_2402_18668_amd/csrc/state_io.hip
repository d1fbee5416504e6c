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

// Packed <-> canonical.  Packing takes the symmetric part of the pair rows (the mean of rows (a, b)
// and (b, a)), which is all a readout can see; unpacking writes both rows of a pair.
__global__ void state_repack_kernel(float *state, float *packed, int dp, int dv, size_t stride,
                                    size_t pstride, int to_packed)
{
    const int u = blockIdx.x;
    const int D = feature_dim(dp), Dp = packed_feature_dim(dp);
    float *su = state + (size_t)u * stride, *pu = packed + (size_t)u * pstride;
    float *sz = su + (size_t)D * dv, *pz = pu + (size_t)Dp * dv;
    // rows are walked as (packed row, canonical row 1, canonical row 2)
    for (int r = 0; r < Dp; ++r) {
        int r1, r2;
        if (r <= dp) { r1 = r2 = r; }
        else {
            int t = r - 1 - dp, a = 0;
            while (t >= dp - a) { t -= dp - a; ++a; }
            const int b = a + t;
            r1 = 1 + dp + a * dp + b; r2 = 1 + dp + b * dp + a;
        }
        for (int c = threadIdx.x; c < dv; c += blockDim.x) {
            if (to_packed) pu[(size_t)r * dv + c] = 0.5f * (su[(size_t)r1 * dv + c] + su[(size_t)r2 * dv + c]);
            else { const float x = pu[(size_t)r * dv + c]; su[(size_t)r1 * dv + c] = x; su[(size_t)r2 * dv + c] = x; }
        }
        if (threadIdx.x == 0) {
            if (to_packed) pz[r] = 0.5f * (sz[r1] + sz[r2]);
            else { sz[r1] = pz[r]; sz[r2] = pz[r]; }
        }
    }
}

hipError_t launch_state_repack(float *state, float *packed, int U, int dp, int dv, int to_packed,
                               hipStream_t s)
{
    hipLaunchKernelGGL(state_repack_kernel, dim3(U), dim3(128), 0, s, state, packed, dp, dv,
                       state_stride(dp, dv), packed_state_stride(dp, dv), to_packed);
    return hipGetLastError();
}

__global__ void positions_advance_kernel(int *__restrict__ pos, int B)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) {
        const int p = pos[b];
        if (p >= 1) pos[b] = p + 1;
    }
}

hipError_t launch_positions_advance(int *pos, int B, hipStream_t s)
{
    hipLaunchKernelGGL(positions_advance_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, s, pos, B);
    return hipGetLastError();
}

}  // namespace based
