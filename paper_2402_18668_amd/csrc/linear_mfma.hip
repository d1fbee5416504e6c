// Bias-free linear projection y = x W^T on the gfx950 matrix cores (bf16 in, fp32 accumulate, bf16
// out): the q / k / v and output projections that surround the sequence mixers in a Based block
// (architecture of Sec. 3: projections of the d_model-wide input to H d' features for q and k and
// H d_v for v, and of the H d_v mixer output back to d_model; all without bias).
//
// x [M][K] and W [N][K] are both contiguous along K, so both MFMA operands are 16 contiguous bytes
// of a row per lane.  One workgroup of four waves computes a 256 x 128 tile of y (tokens x
// features); each wave a 128 x 64 quarter as 4 x 2 MFMA tiles of 32 x 32 (computed transposed: rows
// = output features, columns = tokens, so that a lane holds runs of 4 consecutive features of one
// token): 6 operand reads of 16 bytes per lane feed 8 MFMAs, which keeps the LDS pipe below the
// matrix pipe.  The K dimension is walked in steps of 64: the rows of the next step are fetched into
// registers while the current one is multiplied and written to LDS between two barriers.  The
// finished tile is turned through LDS and leaves as 128-byte row segments.
//
// Layouts.  The mixers read and write head-major tensors [B][H][N][d], the projections' natural output is
// token-major [B N][H d].  Rather than a transposing pass in between (one more read and write of q, k,
// v and of the mixer output through HBM), the kernel addresses head-major tensors directly:
//   SPLIT_OUT  the output features are three groups of heads (q, k, v: H d' + H d' + H d_v rows of W in
//              that order) and go to three head-major tensors; x is read once for all three;
//   HEADS_IN   the A operand is a head-major tensor (the mixer output): a K step of 64 lies inside one head.
//
// Workgroups that share rows of x run back to back on the same XCD (its L2 then serves x once per
// row of tiles): block b belongs to XCD b % 8, which walks its own rows of tiles one after another.
#include "common.h"

namespace based {

namespace lin {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BM = 256;        // tokens per workgroup tile
constexpr int BN = 128;        // output features per workgroup tile
constexpr int BK = 64;         // K step
constexpr int NT = 256;
constexpr int LD = BK + 8;     // bf16 elements per staged row (144-byte stride: 16-byte reads of 8 rows hit 32 banks)
constexpr int OUT_LD = 64 + 8; // bf16 elements per row of a wave's output staging tile
constexpr int kXcds = 8;

constexpr int TI = BM / 2 / 32;   // MFMA tiles along the tokens per wave
struct Lds {
    uint16_t a[BM][LD];        // rows of x
    uint16_t b[BN][LD];        // rows of W
};
static_assert(sizeof(Lds) <= 80 * 1024, "two workgroups per CU");
static_assert(4 * 64 * OUT_LD * 2 <= (int)sizeof(Lds), "the output staging reuses the operand buffers");

__device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
}

// Head-major addressing: seq_len tokens per sequence, H heads; d[0..2] the head dims of the (up to) three
// output groups, y1 / y2 the second and third output tensor; d_in the head dim of a head-major input.
struct HeadLayout {
    int seq_len, H;
    int d[3];
    uint16_t *y1, *y2;
    int d_in;
};

// K % 64 == 0, N % 128 == 0 (checked by the launcher); any M >= 1.
template <bool SPLIT_OUT, bool HEADS_IN>
__global__ __launch_bounds__(NT, 2) void linear_kernel(const uint16_t *__restrict__ x,
                                                       const uint16_t *__restrict__ W,
                                                       uint16_t *__restrict__ y, int M, int K, int N,
                                                       int tiles_m, int tiles_n, HeadLayout hl)
{
    __shared__ __align__(16) Lds lds;

    // block -> tile: XCD (b % 8) owns the rows of tiles xcd, xcd + 8, ... and walks each along N
    const int b = blockIdx.x;
    const int xcd = b % kXcds, local = b / kXcds;
    const int tm = (local / tiles_n) * kXcds + xcd, tn = local % tiles_n;
    if (tm >= tiles_m) return;   // uniform: the grid is padded to a multiple of 8 rows of tiles

    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63, g = lane >> 5, n = lane & 31;
    const int wm = w >> 1, wn = w & 1;   // this wave's quarter: tokens 128 wm .., features 64 wn ..
    const int row0 = tm * BM, col0 = tn * BN;

    // staging: thread t moves 16-byte chunk (t % 8) of rows t / 8 + 32 it of the two tiles
    constexpr int AIT = BM / 32, BIT = BN / 32;
    const int s_chunk = tid & 7, s_row = tid >> 3;
    const uint16_t *xa[AIT], *wb[BIT];
#pragma unroll
    for (int it = 0; it < AIT; ++it) {   // rows past M re-read the last one
        const int row = min(row0 + s_row + 32 * it, M - 1);
        if (HEADS_IN)   // token t of sequence b, head 0: [b][h][t][d_in]
            xa[it] = x + ((size_t)(row / hl.seq_len) * hl.H * hl.seq_len + row % hl.seq_len) * hl.d_in + 8 * s_chunk;
        else
            xa[it] = x + (size_t)row * K + 8 * s_chunk;
    }
#pragma unroll
    for (int it = 0; it < BIT; ++it) wb[it] = W + (size_t)(col0 + s_row + 32 * it) * K + 8 * s_chunk;
    u32x4 ra[AIT], rb[BIT];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int it = 0; it < AIT; ++it) {
            // head-major input: feature k0 is column k0 % d_in of head k0 / d_in, one head = seq_len rows on
            const size_t off = HEADS_IN ? (size_t)(k0 / hl.d_in) * hl.seq_len * hl.d_in + k0 % hl.d_in : (size_t)k0;
            ra[it] = *reinterpret_cast<const u32x4 *>(xa[it] + off);
        }
#pragma unroll
        for (int it = 0; it < BIT; ++it) rb[it] = *reinterpret_cast<const u32x4 *>(wb[it] + k0);
    };
    auto stage = [&]() {
#pragma unroll
        for (int it = 0; it < AIT; ++it) *reinterpret_cast<u32x4 *>(&lds.a[s_row + 32 * it][8 * s_chunk]) = ra[it];
#pragma unroll
        for (int it = 0; it < BIT; ++it) *reinterpret_cast<u32x4 *>(&lds.b[s_row + 32 * it][8 * s_chunk]) = rb[it];
    };

    // acc[j][i]: features 64 wn + 32 j .. (rows of the MFMA tile) x tokens 128 wm + 32 i .. (columns)
    f32x16 acc[2][TI];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    fetch(0);
    stage();
    __syncthreads();
    const int steps = K / BK;
    for (int kt = 0; kt < steps; ++kt) {
        const bool more = kt + 1 < steps;
        if (more) fetch((kt + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            u32x4 fw[2], fx[TI];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fw[j] = *reinterpret_cast<const u32x4 *>(&lds.b[64 * wn + 32 * j + n][16 * ks + 8 * g]);
#pragma unroll
            for (int i = 0; i < TI; ++i)
                fx[i] = *reinterpret_cast<const u32x4 *>(&lds.a[(BM / 2) * wm + 32 * i + n][16 * ks + 8 * g]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < TI; ++i) acc[j][i] = mfma(fw[j], fx[i], acc[j][i]);
        }
        __syncthreads();   // every wave is done reading this step's rows
        if (more) {
            stage();
            __syncthreads();
        }
    }

    // epilogue: lane (g, n) of tile (j, i) holds token 128 wm + 32 i + n, features 64 wn + 32 j + 8 (r / 4) +
    // 4 g + r % 4.  64 tokens at a time through this wave's staging rows [64 tokens][64 features], then
    // 128-byte row segments.
    uint16_t *out = reinterpret_cast<uint16_t *>(&lds) + (size_t)w * 64 * OUT_LD;
#pragma unroll
    for (int half = 0; half < TI / 2; ++half) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[j][2 * half + i2][4 * q4 + e];
                    const bf16x4 hv = __builtin_convertvector(o, bf16x4);
                    *reinterpret_cast<u32x2 *>(out + (size_t)(32 * i2 + n) * OUT_LD + 32 * j + 8 * q4 + 4 * g) =
                        __builtin_bit_cast(u32x2, hv);
                }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's own 64 x 64 piece is complete in LDS
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int r = 8 * it + (lane >> 3), c = lane & 7;
            const u32x4 val = *reinterpret_cast<const u32x4 *>(out + (size_t)r * OUT_LD + 8 * c);
            const int row = row0 + (BM / 2) * wm + 64 * half + r;
            if (row < M) {
                const int f = col0 + 64 * wn + 8 * c;   // first of this lane's 8 features
                if (SPLIT_OUT) {
                    // group of the feature (boundaries are multiples of 8: a chunk lies inside one head)
                    const int n0 = hl.H * hl.d[0], n1 = n0 + hl.H * hl.d[1];
                    uint16_t *dst = f < n0 ? y : (f < n1 ? hl.y1 : hl.y2);
                    const int dh = f < n0 ? hl.d[0] : (f < n1 ? hl.d[1] : hl.d[2]);
                    const int ff = f < n0 ? f : (f < n1 ? f - n0 : f - n1);
                    const size_t o = (((size_t)(row / hl.seq_len) * hl.H + ff / dh) * hl.seq_len + row % hl.seq_len) * dh + ff % dh;
                    *reinterpret_cast<u32x4 *>(dst + o) = val;
                } else {
                    *reinterpret_cast<u32x4 *>(y + (size_t)row * N + f) = val;
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // read back before the next piece overwrites it
    }
}

}  // namespace lin

bool linear_supported(int M, int K, int N, int dtype)
{
    return dtype == BASED_BF16 && M >= 1 && K >= lin::BK && K % lin::BK == 0 && N >= lin::BN && N % lin::BN == 0;
}

hipError_t launch_linear(const void *x, const void *W, void *y, int M, int K, int N, hipStream_t s)
{
    using namespace lin;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    const int rows_padded = (tiles_m + kXcds - 1) / kXcds * kXcds;
    hipLaunchKernelGGL((linear_kernel<false, false>), dim3((unsigned)((size_t)rows_padded * tiles_n)), dim3(NT), 0, s,
                       (const uint16_t *)x, (const uint16_t *)W, (uint16_t *)y, M, K, N, tiles_m, tiles_n, HeadLayout{});
    return hipGetLastError();
}

bool project_qkv_supported(int K, int H, int d_feat, int d_v, int dtype)
{
    return dtype == BASED_BF16 && K >= lin::BK && K % lin::BK == 0 && H >= 1 && d_feat >= 8 && d_feat % 8 == 0 &&
           d_v >= 8 && d_v % 8 == 0 && (H * (2 * d_feat + d_v)) % lin::BN == 0;
}

hipError_t launch_project_qkv(const void *x, const void *W, void *q, void *k, void *v, int B, int seq_len, int K,
                              int H, int d_feat, int d_v, hipStream_t s)
{
    using namespace lin;
    const int M = B * seq_len, N = H * (2 * d_feat + d_v);
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    const int rows_padded = (tiles_m + kXcds - 1) / kXcds * kXcds;
    HeadLayout hl{seq_len, H, {d_feat, d_feat, d_v}, (uint16_t *)k, (uint16_t *)v, 0};
    hipLaunchKernelGGL((linear_kernel<true, false>), dim3((unsigned)((size_t)rows_padded * tiles_n)), dim3(NT), 0, s,
                       (const uint16_t *)x, (const uint16_t *)W, (uint16_t *)q, M, K, N, tiles_m, tiles_n, hl);
    return hipGetLastError();
}

bool project_out_supported(int H, int d_v, int N, int dtype)
{
    return dtype == BASED_BF16 && H >= 1 && d_v >= lin::BK && d_v % lin::BK == 0 && N >= lin::BN && N % lin::BN == 0;
}

hipError_t launch_project_out(const void *y_heads, const void *W, void *out, int B, int seq_len, int H, int d_v,
                              int N, hipStream_t s)
{
    using namespace lin;
    const int M = B * seq_len, K = H * d_v;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    const int rows_padded = (tiles_m + kXcds - 1) / kXcds * kXcds;
    HeadLayout hl{seq_len, H, {0, 0, 0}, nullptr, nullptr, d_v};
    hipLaunchKernelGGL((linear_kernel<false, true>), dim3((unsigned)((size_t)rows_padded * tiles_n)), dim3(NT), 0, s,
                       (const uint16_t *)y_heads, (const uint16_t *)W, (uint16_t *)out, M, K, N, tiles_m, tiles_n, hl);
    return hipGetLastError();
}

}  // namespace based
