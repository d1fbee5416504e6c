// Sliding-window causal softmax attention over whole sequences (Sec. 3.2 restricting Eq. 1),
// fp32 vector-ALU kernel: the exact-arithmetic path for fp32 inputs and the fallback for every
// supported size.  One workgroup per (unit, block of QB consecutive queries); the K rows the
// block can see (at most w + QB - 1) are staged in LDS once and reused by all QB queries.
#include "common.h"

namespace based {

template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int CE = 4;
    float4 raw;
    __device__ __forceinline__ float get(int i) const { return (&raw.x)[i]; }
    __device__ __forceinline__ void set(const float *a) { raw = make_float4(a[0], a[1], a[2], a[3]); }
};
template <> struct Vec16<bf16_t> {
    static constexpr int CE = 8;
    uint4 raw;
    __device__ __forceinline__ float get(int i) const
    {
        const uint32_t w = (&raw.x)[i >> 1];
        return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    __device__ __forceinline__ void set(const float *a)
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = (uint32_t)f32_to_bf16_bits(a[2 * i]) | ((uint32_t)f32_to_bf16_bits(a[2 * i + 1]) << 16);
        raw = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

constexpr int kSwaQB = 16;       // queries per workgroup
constexpr int kSwaThreads = 256;

template <int DH, int W, typename T> struct SwaRefCfg {
    static constexpr int CE = Vec16<T>::CE;
    static constexpr int ROWS = W + kSwaQB - 1;
    static constexpr int STRIDE = DH + CE;  // elements; one 16-byte pad per row spreads LDS banks
    static constexpr size_t lds_bytes = (size_t)ROWS * STRIDE * sizeof(T) +
                                        (size_t)kSwaQB * DH * 4 + (size_t)(kSwaThreads / 64) * W * 4;
};

template <int DH, int W, typename T>
__global__ __launch_bounds__(kSwaThreads) void swa_prefill_ref_kernel(const T *__restrict__ q,
                                                                      const T *__restrict__ k,
                                                                      const T *__restrict__ v,
                                                                      T *__restrict__ y,
                                                                      const float2 *__restrict__ rot, int N,
                                                                      float scale)
{
    using Cfg = SwaRefCfg<DH, W, T>;
    using V16 = Vec16<T>;
    constexpr int CE = Cfg::CE, STRIDE = Cfg::STRIDE, QB = kSwaQB;
    constexpr int LPR = DH / CE;   // lanes per row
    constexpr int KG = 64 / LPR;   // key groups working in parallel in the value phase
    constexpr int KPL = (W + 63) / 64;   // keys per lane in the score phase (a window below 64 leaves lanes idle)

    extern __shared__ __align__(16) unsigned char lds_raw[];
    T *Ks = reinterpret_cast<T *>(lds_raw);
    float *qs = reinterpret_cast<float *>(lds_raw + (size_t)Cfg::ROWS * STRIDE * sizeof(T));
    float *pl = qs + QB * DH;

    const int nblk = (N + QB - 1) / QB;
    const int u = blockIdx.x / nblk, i0 = (blockIdx.x % nblk) * QB;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const size_t base = (size_t)u * N * DH;
    const int j_lo = max(0, i0 - W + 1), j_hi = min(N - 1, i0 + QB - 1);
    const int rows = j_hi - j_lo + 1;

    for (int idx = tid; idx < rows * LPR; idx += kSwaThreads) {
        const int r = idx / LPR, c = idx % LPR;
        V16 kc;
        kc.raw = *reinterpret_cast<const decltype(V16::raw) *>(k + base + (size_t)(j_lo + r) * DH + c * CE);
        if (rot) rotate_chunk(kc, rot + (size_t)(j_lo + r) * (DH / 2) + c * (CE / 2));
        *reinterpret_cast<decltype(V16::raw) *>(Ks + (size_t)r * STRIDE + c * CE) = kc.raw;
    }
    for (int idx = tid; idx < QB * DH / 2; idx += kSwaThreads) {
        const int qi = idx / (DH / 2), pr = idx % (DH / 2);
        float x0 = 0.f, x1 = 0.f;
        if (i0 + qi < N) {
            x0 = to_f32(q[base + (size_t)(i0 + qi) * DH + 2 * pr]);
            x1 = to_f32(q[base + (size_t)(i0 + qi) * DH + 2 * pr + 1]);
            if (rot) {
                const float2 cs = rot[(size_t)(i0 + qi) * (DH / 2) + pr];
                const float r0 = fmaf(x0, cs.x, -x1 * cs.y), r1 = fmaf(x0, cs.y, x1 * cs.x);
                x0 = r0; x1 = r1;
            }
        }
        qs[qi * DH + 2 * pr] = x0 * scale;
        qs[qi * DH + 2 * pr + 1] = x1 * scale;
    }
    __syncthreads();

    for (int qi = wv; qi < QB; qi += kSwaThreads / 64) {   // same trip count in every wave
        const int i = i0 + qi;
        const bool live = i < N;
        const int lo = max(0, i - W + 1);
        // scores: lane handles keys lo + lane (+ 64)
        float sc[KPL];
        float m = -INFINITY;
#pragma unroll
        for (int t = 0; t < KPL; ++t) {
            const int j = lo + lane + 64 * t;
            float d = -INFINITY;
            if (live && j <= i) {
                d = 0.f;
                const T *kr = Ks + (size_t)(j - j_lo) * STRIDE;
                const float *qr = qs + qi * DH;
#pragma unroll
                for (int c = 0; c < LPR; ++c) {
                    V16 kc;
                    kc.raw = *reinterpret_cast<const decltype(V16::raw) *>(kr + c * CE);
#pragma unroll
                    for (int e = 0; e < CE; ++e) d = fmaf(qr[c * CE + e], kc.get(e), d);
                }
            }
            sc[t] = d;
            m = fmaxf(m, d);
        }
        m = wave_max(m);
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < KPL; ++t) {
            const float p = (sc[t] == -INFINITY) ? 0.f : __expf(sc[t] - m);
            sum += p;
            if (lane + 64 * t < W) pl[wv * W + lane + 64 * t] = p;
        }
        sum = wave_sum(sum);
        __syncthreads();
        // values: lane = (key group kg, 16-byte column chunk); V rows stream from global / L2
        const int chunk = lane % LPR, kg = lane / LPR;
        float acc[CE];
#pragma unroll
        for (int e = 0; e < CE; ++e) acc[e] = 0.f;
        if (live) {
            const int cnt = i - lo + 1;
            for (int jj = kg; jj < cnt; jj += KG) {
                V16 vc;
                vc.raw = *reinterpret_cast<const decltype(V16::raw) *>(
                    v + base + (size_t)(lo + jj) * DH + chunk * CE);
                const float p = pl[wv * W + jj];
#pragma unroll
                for (int e = 0; e < CE; ++e) acc[e] = fmaf(p, vc.get(e), acc[e]);
            }
        }
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
            for (int e = 0; e < CE; ++e) acc[e] += __shfl_xor(acc[e], o, 64);
        }
        if (live && kg == 0) {
            const float inv = 1.f / sum;
#pragma unroll
            for (int e = 0; e < CE; ++e) acc[e] *= inv;
            V16 out;
            out.set(acc);
            *reinterpret_cast<decltype(V16::raw) *>(y + base + (size_t)i * DH + chunk * CE) = out.raw;
        }
        __syncthreads();
    }
}

// Copies the last min(N, w) rows of k (rotated, if a table is given) and v into ring slots j mod w.
template <typename T>
__global__ void swa_ring_fill_kernel(const T *__restrict__ k, const T *__restrict__ v,
                                     T *__restrict__ ring, const float2 *__restrict__ rot, int N, int dh, int w)
{
    const int u = blockIdx.x;
    const int first = N > w ? N - w : 0;
    const int total = (N - first) * (dh / 2);
    T *Kr = ring + (size_t)u * 2 * w * dh, *Vr = Kr + (size_t)w * dh;
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {   // one adjacent pair of columns at a time
        const int j = first + idx / (dh / 2), pr = idx % (dh / 2);
        const size_t src = ((size_t)u * N + j) * dh + 2 * pr, dst = (size_t)(j % w) * dh + 2 * pr;
        if (rot) {
            const float2 cs = rot[(size_t)j * (dh / 2) + pr];
            const float x0 = to_f32(k[src]), x1 = to_f32(k[src + 1]);
            Kr[dst] = from_f32<T>(fmaf(x0, cs.x, -x1 * cs.y));
            Kr[dst + 1] = from_f32<T>(fmaf(x0, cs.y, x1 * cs.x));
        } else {
            Kr[dst] = k[src];
            Kr[dst + 1] = k[src + 1];
        }
        Vr[dst] = v[src];
        Vr[dst + 1] = v[src + 1];
    }
}

template <int DH, int W, typename T>
static hipError_t launch_swa_ref(const void *q, const void *k, const void *v, void *y, const float *rot, int U,
                                 int N, float scale, hipStream_t s)
{
    using Cfg = SwaRefCfg<DH, W, T>;
    auto kern = swa_prefill_ref_kernel<DH, W, T>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)Cfg::lds_bytes);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((size_t)((N + kSwaQB - 1) / kSwaQB) * U));
    hipLaunchKernelGGL(kern, grid, dim3(kSwaThreads), Cfg::lds_bytes, s, (const T *)q, (const T *)k,
                       (const T *)v, (T *)y, reinterpret_cast<const float2 *>(rot), N, scale);
    return hipGetLastError();
}

hipError_t launch_swa_prefill_ref(const void *q, const void *k, const void *v, void *y, const float *rot, int U,
                                  int N, int dh, int w, float scale, int dtype, hipStream_t s)
{
#define SWA_CASE(DH_, W_)                                                                    \
    if (dh == DH_ && w == W_)                                                                \
        return dtype == BASED_F32 ? launch_swa_ref<DH_, W_, float>(q, k, v, y, rot, U, N, scale, s) \
                                  : launch_swa_ref<DH_, W_, bf16_t>(q, k, v, y, rot, U, N, scale, s)
    SWA_CASE(64, 16);
    SWA_CASE(64, 32);
    SWA_CASE(128, 16);
    SWA_CASE(128, 32);
    SWA_CASE(64, 64);
    SWA_CASE(64, 128);
    SWA_CASE(128, 64);
    SWA_CASE(128, 128);
#undef SWA_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_swa_ring_fill(const void *k, const void *v, void *ring, const float *rot, int U, int N, int dh,
                                int w, int dtype, hipStream_t s)
{
    if (dtype == BASED_F32)
        hipLaunchKernelGGL(swa_ring_fill_kernel<float>, dim3(U), dim3(256), 0, s, (const float *)k,
                           (const float *)v, (float *)ring, reinterpret_cast<const float2 *>(rot), N, dh, w);
    else
        hipLaunchKernelGGL(swa_ring_fill_kernel<bf16_t>, dim3(U), dim3(256), 0, s, (const bf16_t *)k,
                           (const bf16_t *)v, (bf16_t *)ring, reinterpret_cast<const float2 *>(rot), N, dh, w);
    return hipGetLastError();
}

}  // namespace based
