// The gate of a BaseConv layer (appendix on the gated convolution; training-settings table: filter
// size 3, SiLU): between the layer's two input projections a = u W1, c = u W2 and its output projection,
//     g[t] = (a[t] + b1) * silu(h[0] c[t] + h[1] c[t - 1] + h[2] c[t - 2] + b2),
// every product per channel.  Pure streaming work: each element of a and c is read once and each element
// of g written once, so the kernel is laid out for the memory system and nothing else (loads and stores
// carry the streaming hint: nothing is touched twice; 306 -> 290 us on the 1.3B shape).
//
// Work split.  A thread owns 16 bytes of channels (8 bf16 or 4 fp32) and walks a run of kRun tokens with
// the two previous rows of c in registers, so c is read once (plus a two-row halo per run).  The threads
// of a wave cover 1 KB of consecutive channels of one token: every load and store is a whole-row segment.
// The last two rows of c of every sequence can be written out as the state from which a later call (the
// next part of the sequence, or a decode step, which is the N = 1 case) continues.
#include "common.h"

namespace based {

namespace {

constexpr int kRun = 32;        // tokens per thread
constexpr int kThreads = 128;

template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int CE = 4;
    float4 raw;
    __device__ __forceinline__ float get(int i) const { return (&raw.x)[i]; }
    __device__ __forceinline__ void set(const float *v) { raw = make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct Vec16<bf16_t> {
    static constexpr int CE = 8;
    uint4 raw;
    __device__ __forceinline__ float get(int i) const
    {
        const uint32_t w = (&raw.x)[i >> 1];
        return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    __device__ __forceinline__ void set(const float *v)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            (&raw.x)[i] = (uint32_t)f32_to_bf16_bits(v[2 * i]) | ((uint32_t)f32_to_bf16_bits(v[2 * i + 1]) << 16);
    }
};

// grid: (channel chunks / kThreads, runs of kRun tokens, B)
template <typename T>
__global__ __launch_bounds__(kThreads) void short_conv_gate_kernel(
    const T *__restrict__ a, const T *__restrict__ c, const float *__restrict__ h, const float *__restrict__ b1,
    const float *__restrict__ b2, const T *c_prev, T *__restrict__ out, T *c_last, int N, int Dc)
{
    using V = Vec16<T>;
    constexpr int CE = V::CE;
    const int chunk = blockIdx.x * kThreads + threadIdx.x;
    if (chunk * CE >= Dc) return;
    const int ch0 = chunk * CE;
    const int b = blockIdx.z;
    const int t0 = blockIdx.y * kRun, t1 = min(N, t0 + kRun);
    const size_t seq = (size_t)b * N * Dc;
    using Raw = decltype(V::raw);
    typedef uint32_t nt16 __attribute__((ext_vector_type(4)));   // 16 bytes, the type the streaming hints take

    float h0[CE], h1[CE], h2[CE], bb1[CE], bb2[CE];
#pragma unroll
    for (int i = 0; i < CE; ++i) {
        h0[i] = h[ch0 + i]; h1[i] = h[Dc + ch0 + i]; h2[i] = h[2 * Dc + ch0 + i];
        bb1[i] = b1[ch0 + i]; bb2[i] = b2[ch0 + i];
    }
    // row t of the sequence extended to the left by the two rows of the earlier part (or zeros)
    auto row_c = [&](int t) -> V {
        V r;
        if (t >= 0) r.raw = *reinterpret_cast<const Raw *>(c + seq + (size_t)t * Dc + ch0);
        else if (c_prev) r.raw = *reinterpret_cast<const Raw *>(c_prev + ((size_t)b * 2 + (2 + t)) * Dc + ch0);
        else r.raw = Raw{};
        return r;
    };
    V p2 = row_c(t0 - 2), p1 = row_c(t0 - 1);
    // The state a later call continues from: the last two rows of the extended sequence (with N = 1 the
    // older of the two is a row of the earlier part), written by the thread that owns the end of the
    // sequence.  When the sequence is a single run that thread is also the only reader of c_prev for its
    // channels and has read it by then, so c_last may be the same buffer.
    const bool owns_end = c_last && t1 == N;

#pragma unroll 4
    for (int t = t0; t < t1; ++t) {
        V av, cv, o;
        av.raw = __builtin_bit_cast(Raw, __builtin_nontemporal_load(reinterpret_cast<const nt16 *>(a + seq + (size_t)t * Dc + ch0)));
        cv.raw = __builtin_bit_cast(Raw, __builtin_nontemporal_load(reinterpret_cast<const nt16 *>(c + seq + (size_t)t * Dc + ch0)));
        float g[CE];
#pragma unroll
        for (int i = 0; i < CE; ++i) {
            const float pre = fmaf(h0[i], cv.get(i), fmaf(h1[i], p1.get(i), fmaf(h2[i], p2.get(i), bb2[i])));
            const float sg = pre / (1.f + __expf(-pre));
            g[i] = (av.get(i) + bb1[i]) * sg;
        }
        o.set(g);
        __builtin_nontemporal_store(__builtin_bit_cast(nt16, o.raw), reinterpret_cast<nt16 *>(out + seq + (size_t)t * Dc + ch0));
        p2 = p1; p1 = cv;
    }
    if (owns_end) {
        *reinterpret_cast<Raw *>(c_last + ((size_t)b * 2 + 0) * Dc + ch0) = p2.raw;
        *reinterpret_cast<Raw *>(c_last + ((size_t)b * 2 + 1) * Dc + ch0) = p1.raw;
    }
}

}  // namespace

bool short_conv_gate_supported(int Dc, int dtype)
{
    return Dc >= 8 && Dc % (dtype == BASED_F32 ? 4 : 8) == 0;
}
int short_conv_gate_run() { return kRun; }

hipError_t launch_short_conv_gate(const void *a, const void *c, const float *h, const float *b1, const float *b2,
                                  const void *c_prev, void *out, void *c_last, int B, int N, int Dc, int dtype,
                                  hipStream_t s)
{
    const int ce = dtype == BASED_F32 ? 4 : 8;
    const int chunks = Dc / ce;
    const dim3 grid((unsigned)((chunks + kThreads - 1) / kThreads), (unsigned)((N + kRun - 1) / kRun), (unsigned)B);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    if (dtype == BASED_F32)
        hipLaunchKernelGGL(short_conv_gate_kernel<float>, grid, dim3(kThreads), 0, s, (const float *)a,
                           (const float *)c, h, b1, b2, (const float *)c_prev, (float *)out, (float *)c_last, N, Dc);
    else
        hipLaunchKernelGGL(short_conv_gate_kernel<bf16_t>, grid, dim3(kThreads), 0, s, (const bf16_t *)a,
                           (const bf16_t *)c, h, b1, b2, (const bf16_t *)c_prev, (bf16_t *)out, (bf16_t *)c_last, N,
                           Dc);
    return hipGetLastError();
}

}  // namespace based
