// Rotary position encoding for the sliding-window layers (the training-settings table names it as
// their positional encoding; the definition is the published one of that encoding): the head dimension
// is d_h / 2 adjacent pairs, pair i of the token at position p is rotated by p * base^(-2i / d_h).
//
// The angles depend on the position and the pair only, not on the batch, the head or the data, so their
// cosines and sines are tabulated once ([position][pair] -> (cos, sin), fp32, computed in fp64) and every
// kernel that stages q or k rows rotates them on the way in, reading its rows of the table (which all
// units share, so it stays in the caches).  The rotated rows never exist in global memory, except for the
// keys a prefill leaves in the decode ring.
#include "common.h"

namespace based {

namespace {

__global__ void rotary_table_kernel(float2 *__restrict__ table, int pos0, int N, int half, double log2_base,
                                    double inv_dh)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)N * half) return;
    const int t = (int)(idx / half), i = (int)(idx % half);
    const double theta = exp2(-2.0 * (double)i * inv_dh * log2_base);
    double s, c;
    sincos((double)(pos0 + t) * theta, &s, &c);
    table[idx] = make_float2((float)c, (float)s);
}

}  // namespace

hipError_t launch_rotary_table(float *table, int pos0, int N, int dh, float base, hipStream_t s)
{
    const int half = dh / 2;
    const size_t total = (size_t)N * half;
    hipLaunchKernelGGL(rotary_table_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<float2 *>(table), pos0, N, half, log2((double)base), 1.0 / (double)dh);
    return hipGetLastError();
}

}  // namespace based
