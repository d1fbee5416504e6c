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

// Where the 8 output features starting at f go in the head-major outputs: the tensor, its head dim, and the
// part of the element offset that does not depend on the token.  Offset of token t of sequence b:
// b * batch_stride + fixed + t * dh.  (Computed once per lane: the divisions are not cheap, and done per
// store they were most of the epilogue.)
struct FeatDst {
    uint16_t *dst;
    int dh;
    size_t fixed, batch_stride;
};
__device__ __forceinline__ FeatDst feat_dst(const HeadLayout &hl, uint16_t *y, int f)
{
    // group of the feature (boundaries are multiples of 8: a chunk lies inside one head)
    const int n0 = hl.H * hl.d[0], n1 = n0 + hl.H * hl.d[1];
    FeatDst r;
    r.dst = f < n0 ? y : (f < n1 ? hl.y1 : hl.y2);
    r.dh = f < n0 ? hl.d[0] : (f < n1 ? hl.d[1] : hl.d[2]);
    const int ff = f < n0 ? f : (f < n1 ? f - n0 : f - n1);
    r.fixed = (size_t)(ff / r.dh) * hl.seq_len * r.dh + ff % r.dh;
    r.batch_stride = (size_t)hl.H * hl.seq_len * r.dh;
    return r;
}
// (sequence, token) of a row, and of the rows after it
struct RowPos { int b, t; };
__device__ __forceinline__ RowPos row_pos(int row, int seq_len) { return {row / seq_len, row % seq_len}; }
__device__ __forceinline__ RowPos row_after(RowPos p, int delta, int seq_len)
{
    p.t += delta;
    while (p.t >= seq_len) { p.t -= seq_len; ++p.b; }
    return p;
}

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
    const int f_lane = col0 + 64 * wn + 8 * (lane & 7);   // first of this lane's 8 features
    FeatDst fd{};
    RowPos rp0{};
    if (SPLIT_OUT) {
        fd = feat_dst(hl, y, f_lane);
        rp0 = row_pos(row0 + (BM / 2) * wm + (lane >> 3), hl.seq_len);
    }
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
                if (SPLIT_OUT) {
                    const RowPos rp = row_after(rp0, 64 * half + 8 * it, hl.seq_len);
                    *reinterpret_cast<u32x4 *>(fd.dst + (size_t)rp.b * fd.batch_stride + fd.fixed + (size_t)rp.t * fd.dh) = val;
                } else {
                    *reinterpret_cast<u32x4 *>(y + (size_t)row * N + f_lane) = val;
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // read back before the next piece overwrites it
    }
}

// ---- the wide tiling: 256 x 256 outputs per workgroup ------------------------------------------------------
// For large projections with N a multiple of 256.  Four waves, each a 128 x 128 quarter as 4 x 4 MFMA tiles:
// 8 operand reads of 16 bytes per lane feed 16 MFMAs (half the LDS traffic per matrix instruction of the
// 4 x 2 tiling), with the 256 accumulator registers a wave then needs: one workgroup per CU, one wave per
// SIMD, the whole register file to a wave.  The LDS holds two generations of the 256 + 256 staged rows and
// one barrier per step separates them.  The global loads run two K steps ahead and are dealt out between the
// matrix instructions, one after every four: with the sixteen loads of a thread issued in one burst a wave
// stood 1,500 of a step's 5,500 clock counts just getting them accepted by the memory pipeline, and another
// 850 writing them to LDS, all of it with the matrix pipe idle.  During step kt a thread writes the piece it
// fetched a step ago (rows of step kt + 1) into the other generation and refills the same register with the
// same piece of step kt + 2, sixteen times, so sixteen loads stay in flight and each is a step old when it is
// needed.  Inside a step the operands of the next 16-deep slab are read while the matrix instructions of the
// current one run.
constexpr int WBM = 256, WBN = 256;
struct LdsWide {
    uint16_t a[2][WBM][LD];    // rows of x, two generations
    uint16_t b[2][WBN][LD];    // rows of W
};
static_assert(sizeof(LdsWide) <= 160 * 1024, "one workgroup per CU");

template <bool SPLIT_OUT, bool HEADS_IN>
__global__ __launch_bounds__(NT, 1) void linear_wide_kernel(const uint16_t *__restrict__ x,
                                                            const uint16_t *__restrict__ W,
                                                            uint16_t *__restrict__ y, int M, int K, int N,
                                                            int tiles_m, int tiles_n, HeadLayout hl)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    LdsWide &lds = *reinterpret_cast<LdsWide *>(lds_raw);

    const int b = blockIdx.x;
    const int xcd = b % kXcds, local = b / kXcds;
    const int tm = (local / tiles_n) * kXcds + xcd, tn = local % tiles_n;
    if (tm >= tiles_m) return;   // uniform: the grid is padded to a multiple of 8 rows of tiles

    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63, g = lane >> 5, n = lane & 31;
    const int wm = w >> 1, wn = w & 1;   // this wave's quarter: tokens 128 wm .., features 128 wn ..
    const int row0 = tm * WBM, col0 = tn * WBN;

    // staging: thread t moves 16-byte chunk (t % 8) of rows t / 8 + 32 it of the two tiles
    constexpr int AIT = WBM / 32, BIT = WBN / 32;
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
    // piece p of a thread: p < AIT a row chunk of x, else of W
    u32x4 rp[AIT + BIT];
    auto fetch_piece = [&](int p, int k0) {
        if (p < AIT) {
            const size_t off = HEADS_IN ? (size_t)(k0 / hl.d_in) * hl.seq_len * hl.d_in + k0 % hl.d_in : (size_t)k0;
            rp[p] = *reinterpret_cast<const u32x4 *>(xa[p] + off);
        } else {
            rp[p] = *reinterpret_cast<const u32x4 *>(wb[p - AIT] + k0);
        }
    };
    auto stage_piece = [&](int p, int gen) {
        if (p < AIT) *reinterpret_cast<u32x4 *>(&lds.a[gen][s_row + 32 * p][8 * s_chunk]) = rp[p];
        else *reinterpret_cast<u32x4 *>(&lds.b[gen][s_row + 32 * (p - AIT)][8 * s_chunk]) = rp[p];
    };

    // acc[j][i]: features 128 wn + 32 j .. (rows of the MFMA tile) x tokens 128 wm + 32 i .. (columns)
    f32x16 acc[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    const int steps = K / BK;
    // K steps past the end re-read the last one (the loads are unconditional so that the number in flight is
    // known; what they fetch is staged into a generation nobody reads any more)
    auto k_of = [&](int step) { return min(step, steps - 1) * BK; };
#pragma unroll
    for (int p = 0; p < AIT + BIT; ++p) fetch_piece(p, 0);
#pragma unroll
    for (int p = 0; p < AIT + BIT; ++p) {
        stage_piece(p, 0);
        fetch_piece(p, k_of(1));
    }
    __syncthreads();
    for (int kt = 0; kt < steps; ++kt) {
        const int cur = kt & 1;
        const int k_next2 = k_of(kt + 2);
        const uint16_t *pb = &lds.b[cur][128 * wn + n][8 * g];
        const uint16_t *pa = &lds.a[cur][128 * wm + n][8 * g];
        u32x4 fw[2][4], fx[2][4];
        auto read_ops = [&](int ks, int set) {
#pragma unroll
            for (int j = 0; j < 4; ++j) fw[set][j] = *reinterpret_cast<const u32x4 *>(pb + (size_t)32 * j * LD + 16 * ks);
#pragma unroll
            for (int i = 0; i < 4; ++i) fx[set][i] = *reinterpret_cast<const u32x4 *>(pa + (size_t)32 * i * LD + 16 * ks);
        };
        read_ops(0, 0);
        static_assert((BK / 16) * 4 == AIT + BIT, "one staged piece per group of four matrix instructions");
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) read_ops(ks + 1, (ks + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[j][i] = mfma(fw[ks & 1][j], fx[ks & 1][i], acc[j][i]);
                // the piece fetched a step ago goes to the other generation (every wave left it at the last
                // barrier), and its register takes the same piece of the step after the next
                const int p = 4 * ks + j;
                stage_piece(p, cur ^ 1);
                fetch_piece(p, k_next2);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    }
    // (the loads of the two steps past the end are still in flight: their registers are dead)

    // epilogue: lane (g, n) of tile (j, i) holds token 128 wm + 32 i + n, features 128 wn + 32 j + 8 (r / 4) +
    // 4 g + r % 4.  64 tokens x 64 features at a time through this wave's staging rows, then 128-byte row
    // segments.  (The last barrier of the loop has passed: nobody reads the operand buffers any more.)
    uint16_t *out = reinterpret_cast<uint16_t *>(lds_raw) + (size_t)w * 64 * OUT_LD;
    const int f_lane = col0 + 128 * wn + 8 * (lane & 7);   // first of this lane's 8 features of the piece jh = 0
    FeatDst fd[2] = {};
    RowPos rp0{};
    if (SPLIT_OUT) {
        fd[0] = feat_dst(hl, y, f_lane);
        fd[1] = feat_dst(hl, y, f_lane + 64);
        rp0 = row_pos(row0 + 128 * wm + (lane >> 3), hl.seq_len);
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int jh = 0; jh < 2; ++jh) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        f32x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = acc[2 * jh + j][2 * half + i2][4 * q4 + e];
                        const bf16x4 hv = __builtin_convertvector(o, bf16x4);
                        *reinterpret_cast<u32x2 *>(out + (size_t)(32 * i2 + n) * OUT_LD + 32 * j + 8 * q4 + 4 * g) =
                            __builtin_bit_cast(u32x2, hv);
                    }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's own 64 x 64 piece is complete in LDS
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int r = 8 * it + (lane >> 3), c = lane & 7;
                const u32x4 val = *reinterpret_cast<const u32x4 *>(out + (size_t)r * OUT_LD + 8 * c);
                const int row = row0 + 128 * wm + 64 * half + r;
                if (row < M) {
                    if (SPLIT_OUT) {
                        const RowPos rp = row_after(rp0, 64 * half + 8 * it, hl.seq_len);
                        *reinterpret_cast<u32x4 *>(fd[jh].dst + (size_t)rp.b * fd[jh].batch_stride + fd[jh].fixed +
                                                   (size_t)rp.t * fd[jh].dh) = val;
                    } else {
                        *reinterpret_cast<u32x4 *>(y + (size_t)row * N + f_lane + 64 * jh) = val;
                    }
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // read back before the next piece overwrites it
        }
    }
}

// The wide tiling pays when its tiles, one per CU at a time, come in nearly whole rounds of the chip: measured
// at 256, 512, 1280 tiles it is 6-16 % faster than the narrow one (4096^3: 1032 against 894 TFLOP/s), at 384
// tiles (a round and a half) 4 % slower.
__host__ inline bool use_wide(int M, int N)
{
    if (N % WBN != 0) return false;
    const long tiles = (long)((M + WBM - 1) / WBM) * (N / WBN);
    const long rounds = (tiles + 255) / 256;
    return tiles * 5 >= rounds * 256 * 4;   // the last round at least 80 % of the way to full, on average
}

template <bool SPLIT_OUT, bool HEADS_IN>
hipError_t launch_any(const uint16_t *x, const uint16_t *W, uint16_t *y, int M, int K, int N, const HeadLayout &hl,
                      hipStream_t s)
{
    if (use_wide(M, N)) {
        const int tiles_m = (M + WBM - 1) / WBM, tiles_n = N / WBN;
        const int rows_padded = (tiles_m + kXcds - 1) / kXcds * kXcds;
        const void *kern = reinterpret_cast<const void *>(linear_wide_kernel<SPLIT_OUT, HEADS_IN>);
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(LdsWide));
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((linear_wide_kernel<SPLIT_OUT, HEADS_IN>), dim3((unsigned)((size_t)rows_padded * tiles_n)),
                           dim3(NT), sizeof(LdsWide), s, x, W, y, M, K, N, tiles_m, tiles_n, hl);
        return hipGetLastError();
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    const int rows_padded = (tiles_m + kXcds - 1) / kXcds * kXcds;
    hipLaunchKernelGGL((linear_kernel<SPLIT_OUT, HEADS_IN>), dim3((unsigned)((size_t)rows_padded * tiles_n)), dim3(NT), 0,
                       s, x, W, y, M, K, N, tiles_m, tiles_n, hl);
    return hipGetLastError();
}

}  // namespace lin

bool linear_supported(int M, int K, int N, int dtype)
{
    return dtype == BASED_BF16 && M >= 1 && K >= lin::BK && K % lin::BK == 0 && N >= lin::BN && N % lin::BN == 0;
}

hipError_t launch_linear(const void *x, const void *W, void *y, int M, int K, int N, hipStream_t s)
{
    return lin::launch_any<false, false>((const uint16_t *)x, (const uint16_t *)W, (uint16_t *)y, M, K, N,
                                         lin::HeadLayout{}, s);
}

bool project_qkv_supported(int K, int H, int d_feat, int d_v, int dtype)
{
    return dtype == BASED_BF16 && K >= lin::BK && K % lin::BK == 0 && H >= 1 && d_feat >= 8 && d_feat % 8 == 0 &&
           d_v >= 8 && d_v % 8 == 0 && (H * (2 * d_feat + d_v)) % lin::BN == 0;
}

hipError_t launch_project_qkv(const void *x, const void *W, void *q, void *k, void *v, int B, int seq_len, int K,
                              int H, int d_feat, int d_v, hipStream_t s)
{
    const int M = B * seq_len, N = H * (2 * d_feat + d_v);
    lin::HeadLayout hl{seq_len, H, {d_feat, d_feat, d_v}, (uint16_t *)k, (uint16_t *)v, 0};
    return lin::launch_any<true, false>((const uint16_t *)x, (const uint16_t *)W, (uint16_t *)q, M, K, N, hl, s);
}

bool project_out_supported(int H, int d_v, int N, int dtype)
{
    return dtype == BASED_BF16 && H >= 1 && d_v >= lin::BK && d_v % lin::BK == 0 && N >= lin::BN && N % lin::BN == 0;
}

hipError_t launch_project_out(const void *y_heads, const void *W, void *out, int B, int seq_len, int H, int d_v,
                              int N, hipStream_t s)
{
    const int M = B * seq_len, K = H * d_v;
    lin::HeadLayout hl{seq_len, H, {0, 0, 0}, nullptr, nullptr, d_v};
    return lin::launch_any<false, true>((const uint16_t *)y_heads, (const uint16_t *)W, (uint16_t *)out, M, K, N, hl, s);
}

}  // namespace based
