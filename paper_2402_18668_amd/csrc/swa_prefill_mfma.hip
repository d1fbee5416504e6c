// Sliding-window causal softmax attention over whole sequences (Sec. 3.2 restricting Eq. 1) on
// the gfx950 matrix cores: bf16 in, fp32 scores / softmax / accumulation.
//
// One workgroup of four waves per (unit, block of 128 consecutive queries).  The w + 128 key and
// value rows the block can see are staged in LDS once (K row-major, V transposed) and reused by
// the four waves; each wave owns one tile of 32 queries and walks the w / 32 + 1 key tiles that
// overlap its window.  Scores are computed transposed (S^T = K Q^T: lane = query, registers =
// keys), so the row maximum and row sum of the softmax are lane-local plus one cross-lane add,
// and the probabilities become the operand of Y^T = V^T P^T with a register-local conversion:
// with k-slot 8g + 4jj + i of slab s mapped to key 16 s + 8 jj + 4 g + i of the tile, accumulator
// registers 8s .. 8s+7 of a lane are exactly its k-slots (MFMA 32x32x16; lane = 32 g + n).
#include "common.h"

namespace based {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BQ = 128;   // queries per workgroup
constexpr int NT = 256;

template <int DH, int W> struct SwaCfg {
    static constexpr int NK = W + BQ;          // staged key rows
    static constexpr int K_LD = DH + 8;        // bf16 elements per staged K row (16-byte pad)
    static constexpr int VT_LD = NK + 4;       // bf16 elements per staged V^T row (8-byte aligned)
    static constexpr int NKT = W / 32 + 1;     // key tiles per query tile
    static constexpr size_t lds_bytes = ((size_t)NK * K_LD + (size_t)DH * VT_LD) * 2;
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 w) { return __builtin_bit_cast(bf16x8, w); }

}  // namespace

template <int DH, int W>
__global__ __launch_bounds__(NT) void swa_prefill_mfma_kernel(const uint16_t *__restrict__ q,
                                                              const uint16_t *__restrict__ k,
                                                              const uint16_t *__restrict__ v,
                                                              uint16_t *__restrict__ y,
                                                              uint16_t *__restrict__ ring, int N,
                                                              float scale_log2e)
{
    using Cfg = SwaCfg<DH, W>;
    constexpr int NK = Cfg::NK, K_LD = Cfg::K_LD, VT_LD = Cfg::VT_LD, NKT = Cfg::NKT;
    constexpr int SLABS = DH / 16;   // k-slabs of the score contraction
    constexpr int CT = DH / 32;      // column tiles of the output

    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint16_t *Ks = reinterpret_cast<uint16_t *>(lds_raw);      // [NK][K_LD]
    uint16_t *Vt = Ks + (size_t)NK * K_LD;                     // [DH][VT_LD]

    const int tid = threadIdx.x;
    // wave index as a scalar, so that branches on it are scalar branches (MFMA ignores EXEC)
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, g = lane >> 5, n = lane & 31;
    const int nblk = (N + BQ - 1) / BQ;
    const int u = blockIdx.x / nblk, i0 = (blockIdx.x % nblk) * BQ;
    const size_t base = (size_t)u * N * DH;
    const int key0 = i0 - W;   // sequence position of staged row 0 (may be negative)

    // ---- stage K (row-major) and V (transposed); rows outside the sequence are zero ------------
    // A wave instruction handles 64 consecutive rows of one 16-byte column chunk: the transposed
    // 2-byte V writes of its lanes are then contiguous in LDS (no bank conflicts).
    constexpr int CPR = DH / 8;   // 16-byte chunks per row
    static_assert(NK % 64 == 0, "staged rows must be a multiple of the wave size");
    for (int idx = tid; idx < NK * CPR; idx += NT) {
        const int c = (idx >> 6) % CPR, r = (idx & 63) + 64 * (idx / (64 * CPR));
        const int key = key0 + r;
        u32x4 kv = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
        if (key >= 0 && key < N) {
            kv = *reinterpret_cast<const u32x4 *>(k + base + (size_t)key * DH + c * 8);
            vv = *reinterpret_cast<const u32x4 *>(v + base + (size_t)key * DH + c * 8);
        }
        *reinterpret_cast<u32x4 *>(Ks + (size_t)r * K_LD + c * 8) = kv;
        // the w-slot ring receives the last min(N, w) rows (slot = position mod w); each row is
        // written by the block that owns it as a query row (staged rows W .. W + BQ - 1)
        if (ring && r >= W && key < N && key >= N - W) {
            uint16_t *rk = ring + (size_t)u * 2 * W * DH + (size_t)(key % W) * DH + c * 8;
            *reinterpret_cast<u32x4 *>(rk) = kv;
            *reinterpret_cast<u32x4 *>(rk + (size_t)W * DH) = vv;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            Vt[(size_t)(c * 8 + 2 * i) * VT_LD + r] = (uint16_t)(vv[i] & 0xffffu);
            Vt[(size_t)(c * 8 + 2 * i + 1) * VT_LD + r] = (uint16_t)(vv[i] >> 16);
        }
    }

    // ---- this wave's query tile: Q operand straight from global memory ---------------------------
    const int qbase = i0 + 32 * wv;          // first query of the tile
    const int query = qbase + n;
    const bool q_ok = query < N;
    u32x4 qop[SLABS];
#pragma unroll
    for (int s = 0; s < SLABS; ++s) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        qop[s] = q_ok ? *reinterpret_cast<const u32x4 *>(q + base + (size_t)query * DH + 16 * s + 8 * g) : zero;
    }
    __syncthreads();
    if (qbase >= N) return;   // whole tile past the end (no barrier follows)

    // ---- scores: S^T tile t covers staged rows 32 wv + 32 t .. +31 --------------------------------
    f32x16 P[NKT];
#pragma unroll
    for (int t = 0; t < NKT; ++t) {
#pragma unroll
        for (int r = 0; r < 16; ++r) P[t][r] = 0.f;
        const uint16_t *krow = Ks + (size_t)(32 * wv + 32 * t + n) * K_LD + 8 * g;
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            const u32x4 kop = *reinterpret_cast<const u32x4 *>(krow + 16 * s);
            P[t] = mfma(as_bf16x8(kop), as_bf16x8(qop[s]), P[t]);
        }
    }

    // ---- mask, softmax statistics (lane = query; its keys sit in registers and in lane ^ 32) ------
    float m = -INFINITY;
#pragma unroll
    for (int t = 0; t < NKT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int local = 8 * (r >> 2) + 4 * g + (r & 3);
            const int key = qbase - W + 32 * t + local;
            bool ok = key >= 0;
            if (t == 0) ok = ok && local > n;          // key > query - w
            if (t == NKT - 1) ok = ok && local <= n;   // key <= query
            const float x = ok ? P[t][r] * scale_log2e : -INFINITY;
            P[t][r] = x;
            m = fmaxf(m, x);
        }
    m = fmaxf(m, __shfl_xor(m, 32, 64));
    // the query's own key is always visible, so m is finite for every query inside the sequence
    const float mm = q_ok ? m : 0.f;
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < NKT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(P[t][r] - mm);   // exp2(-inf) = 0 for masked keys
            P[t][r] = p;
            sum += p;
        }
    sum += __shfl_xor(sum, 32, 64);

    // ---- Y^T = V^T P^T ----------------------------------------------------------------------------
    f32x16 Y[CT];
#pragma unroll
    for (int c2 = 0; c2 < CT; ++c2)
#pragma unroll
        for (int r = 0; r < 16; ++r) Y[c2][r] = 0.f;
#pragma unroll
    for (int t = 0; t < NKT; ++t)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            f32x8 f;
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = P[t][8 * s + e];
            const bf16x8 pb = __builtin_convertvector(f, bf16x8);
            const int rowk = 32 * wv + 32 * t + 16 * s + 4 * g;   // first staged key of this lane's k-slots
#pragma unroll
            for (int c2 = 0; c2 < CT; ++c2) {
                const uint16_t *p = Vt + (size_t)(32 * c2 + n) * VT_LD + rowk;
                const u32x2 a = *reinterpret_cast<const u32x2 *>(p);
                const u32x2 b = *reinterpret_cast<const u32x2 *>(p + 8);
                u32x4 o; o[0] = a[0]; o[1] = a[1]; o[2] = b[0]; o[3] = b[1];
                Y[c2] = mfma(as_bf16x8(o), pb, Y[c2]);
            }
        }

    // ---- normalise and store: lane = query, register r = column 8 (r / 4) + 4 g + r % 4 ----------
    if (q_ok) {
        const float inv = 1.f / sum;
        uint16_t *yrow = y + base + (size_t)query * DH + 4 * g;
#pragma unroll
        for (int c2 = 0; c2 < CT; ++c2)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = Y[c2][4 * j + i] * inv;
                const bf16x4 hv = __builtin_convertvector(o, bf16x4);
                *reinterpret_cast<u32x2 *>(yrow + 32 * c2 + 8 * j) = __builtin_bit_cast(u32x2, hv);
            }
    }
}

template <int DH, int W>
static hipError_t launch_swa_mfma(const void *q, const void *k, const void *v, void *y, void *ring, int U,
                                  int N, float scale, hipStream_t s)
{
    using Cfg = SwaCfg<DH, W>;
    auto kern = swa_prefill_mfma_kernel<DH, W>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::lds_bytes);
    if (e != hipSuccess) return e;
    const size_t nblk = (size_t)(N + BQ - 1) / BQ;
    hipLaunchKernelGGL(kern, dim3((unsigned)(nblk * U)), dim3(NT), Cfg::lds_bytes, s, (const uint16_t *)q,
                       (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)y, (uint16_t *)ring, N,
                       scale * 1.44269504088896340736f);
    return hipGetLastError();
}

bool swa_prefill_mfma_supported(int dh, int w, int dtype)
{
    return dtype == BASED_BF16 && (dh == 64 || dh == 128) && (w == 64 || w == 128);
}

hipError_t launch_swa_prefill_mfma(const void *q, const void *k, const void *v, void *y, void *ring, int U,
                                   int N, int dh, int w, float scale, hipStream_t s)
{
    if (dh == 64 && w == 64) return launch_swa_mfma<64, 64>(q, k, v, y, ring, U, N, scale, s);
    if (dh == 64 && w == 128) return launch_swa_mfma<64, 128>(q, k, v, y, ring, U, N, scale, s);
    if (dh == 128 && w == 64) return launch_swa_mfma<128, 64>(q, k, v, y, ring, U, N, scale, s);
    if (dh == 128 && w == 128) return launch_swa_mfma<128, 128>(q, k, v, y, ring, U, N, scale, s);
    return hipErrorInvalidValue;
}

}  // namespace based
