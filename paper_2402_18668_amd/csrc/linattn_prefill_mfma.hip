// Causal Taylor linear attention, chunked prefill on the gfx950 matrix cores (bf16 in, fp32
// accumulate), d' = 16.
//
// Chunked form of Sec. 4: inside a chunk of C = 64 tokens the masked quadratic product
// (1 + A + A^2/2 with A = Q K^T, exact closed form of Eq. 4), across chunks the running
// KV-state S (Eq. 3) read out with phi(Q) and updated with phi(K)^T V.  The expanded features
// are produced in registers straight into MFMA operand layout and never stored anywhere.
//
// Work split.  One workgroup of two waves per (unit, 64-column slice of d_v, sequence segment).
// The 2nd-order feature rows (a, b) -> x_a x_b / sqrt(2) are cut into 8 tiles of 32 rows
// (tile t holds a in {2t, 2t+1}, all b); wave w owns tiles 4w .. 4w+3, whose 32x32 fp32 state
// tiles stay in its accumulator registers for the whole segment.  Wave 0 also owns the tile of
// the 1st/0th-order rows [x_0..x_15, 1]; wave 1 also does the intra-chunk block and the
// denominator.  Per chunk each wave produces a partial Y^T over its feature rows; the two
// partials are exchanged through LDS (each wave finishes 32 of the 64 tokens).
//
// MFMA 32x32x16 register layouts used throughout (lane = 32 g + n):
//   A operand: row n, k-slots 8g .. 8g+7;  B operand: column n, k-slots 8g .. 8g+7;
//   accumulator register r: row 8 (r / 4) + 4 g + r % 4, column n.
// Because a contraction may visit its index in any order, k-slot 8g + 4jj + i of "slab" s is
// mapped to index 16 s + 8 jj + 4 g + i: then accumulator registers 8s .. 8s+7 of a lane are
// exactly its 8 k-slots of slab s, and a state tile (or the masked intra-chunk block) becomes
// an MFMA operand with a register-local fp32 -> bf16 conversion and no data movement.
//
// Denominator.  z is kept as moments: M' = K'^T K' with K' = [k, 1] (17 x 17 inside one
// accumulator tile), i.e. sum k_a k_b, sum k_a and the token count; phi(q).z =
// count + q.z1 + q^T M q / 2 is evaluated with two small MFMAs (M' split into bf16 hi + lo).
//
// Long sequences / few units: the sequence is cut into G segments; a first launch computes each
// segment's state increment (update GEMMs only), and the main launch starts each segment from
// the sum of the increments before it.
#include "common.h"

namespace based {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int DP = 16;            // d'
constexpr int C = 64;             // chunk length (tokens)
constexpr int NW = 2;             // waves per workgroup
constexpr int NT = NW * 64;
constexpr int DVS = 64;           // d_v columns per workgroup
constexpr float kC4 = 0.84089641525371454303f;   // 2^(-1/4): (x_a c)(x_b c) = x_a x_b / sqrt(2)
constexpr float kHalfInvC4 = 0.59460355750136053336f;  // 0.5 * 2^(1/4)

// LDS strides (elements)
constexpr int KTS_LD = C + 4;     // fp32 K^T rows
constexpr int KTB_LD = C + 4;     // bf16 [K^T; ones; 0] rows (8-byte aligned reads)
constexpr int VT_LD = C + 4;      // bf16 V^T rows
constexpr int QS_LD = DP + 4;     // fp32 Q rows

// accumulator slots per wave: 4 main tiles x 2 column tiles, then the 1st/0th-order tile (2 column
// tiles) and the moment tile (both only used by wave 0)
constexpr int SLOTS = 11;
constexpr size_t kWsEntryFloats = (size_t)NW * SLOTS * 16 * 64;

struct Stage {
    float kts[DP][KTS_LD];        // c * K^T
    uint16_t ktb[32][KTB_LD];     // rows 0..15 K^T (bf16), row 16 token-valid ones, rest zero
    uint16_t vt[DVS][VT_LD];      // V^T (bf16)
    float qs[C][QS_LD];           // c * Q
};

struct Lds {
    Stage st[2];
    float xbuf[NW][8][64][4];     // partial Y^T exchange: [writer][c2 * 4 + r / 4][lane][r % 4]
    float den_inter[C];           // count + phi(q).z over earlier chunks (wave 0)
    float den_intra[C];           // row sums of the masked intra-chunk block (wave 1)
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 pack8(const float *v)
{
    f32x8 f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = v[e];
    return __builtin_convertvector(f, bf16x8);
}

__device__ __forceinline__ bf16x8 pack8_acc(const f32x16 &acc, int s)   // registers 8s .. 8s+7
{
    f32x8 f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = acc[8 * s + e];
    return __builtin_convertvector(f, bf16x8);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 w) { return __builtin_bit_cast(bf16x8, w); }

// Workgroup barrier that orders LDS traffic only: this wave's LDS operations have completed
// (lgkmcnt) before it arrives, and the compiler moves no memory access across it.  Global loads
// and stores stay in flight (the waves exchange data through LDS only), which is what lets the
// next chunk's rows stream in underneath the current chunk's arithmetic.
__device__ __forceinline__ void wg_sync()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// MFMA instructions ignore the EXEC mask.  A branch on the wave's role is uniform across the wave
// but the compiler lowers it to lane masking and may drop the jump over a short masked block, in
// which case the other waves would execute the MFMAs inside it.  An inline-asm statement in the
// block makes the compiler keep the jump (it never runs inline asm with an empty EXEC mask).
__device__ __forceinline__ void role_guard() { asm volatile("; wave-role block: keep the execz branch" ::: "memory"); }

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Workspace entry layout: [wave][slot][r / 4][lane][r % 4] floats, so that one 16-byte access per
// lane is contiguous across the wave.
__device__ __forceinline__ size_t ws_off(int w, int slot, int j, int lane)
{
    return ((((size_t)w * SLOTS + slot) * 4 + j) * 64 + lane) * 4;
}

// Loads one workspace entry (this wave's 11 accumulator tiles = 44 x 16 bytes per lane) with all
// loads in flight at once and the wait inside the same statement, so that every output register is
// valid as far as the compiler can tell.  Left to itself the compiler, short of registers in this
// kernel, issues these loads one memory latency apiece.
__device__ __forceinline__ void load_entry(const float *wave_base, int lane, f32x4 (&t)[SLOTS * 4])
{
    static_assert(SLOTS == 11, "the load sequence below is written out for 11 slots");
    const float *p0 = wave_base + ws_off(0, 0, 0, lane);
    const float *p1 = wave_base + ws_off(0, 1, 0, lane);
    const float *p2 = wave_base + ws_off(0, 2, 0, lane);
    const float *p3 = wave_base + ws_off(0, 3, 0, lane);
    const float *p4 = wave_base + ws_off(0, 4, 0, lane);
    const float *p5 = wave_base + ws_off(0, 5, 0, lane);
    const float *p6 = wave_base + ws_off(0, 6, 0, lane);
    const float *p7 = wave_base + ws_off(0, 7, 0, lane);
    const float *p8 = wave_base + ws_off(0, 8, 0, lane);
    const float *p9 = wave_base + ws_off(0, 9, 0, lane);
    const float *p10 = wave_base + ws_off(0, 10, 0, lane);
    asm volatile(
        "global_load_dwordx4 %0, %44, off offset:0\n\t"
        "global_load_dwordx4 %1, %44, off offset:1024\n\t"
        "global_load_dwordx4 %2, %44, off offset:2048\n\t"
        "global_load_dwordx4 %3, %44, off offset:3072\n\t"
        "global_load_dwordx4 %4, %45, off offset:0\n\t"
        "global_load_dwordx4 %5, %45, off offset:1024\n\t"
        "global_load_dwordx4 %6, %45, off offset:2048\n\t"
        "global_load_dwordx4 %7, %45, off offset:3072\n\t"
        "global_load_dwordx4 %8, %46, off offset:0\n\t"
        "global_load_dwordx4 %9, %46, off offset:1024\n\t"
        "global_load_dwordx4 %10, %46, off offset:2048\n\t"
        "global_load_dwordx4 %11, %46, off offset:3072\n\t"
        "global_load_dwordx4 %12, %47, off offset:0\n\t"
        "global_load_dwordx4 %13, %47, off offset:1024\n\t"
        "global_load_dwordx4 %14, %47, off offset:2048\n\t"
        "global_load_dwordx4 %15, %47, off offset:3072\n\t"
        "global_load_dwordx4 %16, %48, off offset:0\n\t"
        "global_load_dwordx4 %17, %48, off offset:1024\n\t"
        "global_load_dwordx4 %18, %48, off offset:2048\n\t"
        "global_load_dwordx4 %19, %48, off offset:3072\n\t"
        "global_load_dwordx4 %20, %49, off offset:0\n\t"
        "global_load_dwordx4 %21, %49, off offset:1024\n\t"
        "global_load_dwordx4 %22, %49, off offset:2048\n\t"
        "global_load_dwordx4 %23, %49, off offset:3072\n\t"
        "global_load_dwordx4 %24, %50, off offset:0\n\t"
        "global_load_dwordx4 %25, %50, off offset:1024\n\t"
        "global_load_dwordx4 %26, %50, off offset:2048\n\t"
        "global_load_dwordx4 %27, %50, off offset:3072\n\t"
        "global_load_dwordx4 %28, %51, off offset:0\n\t"
        "global_load_dwordx4 %29, %51, off offset:1024\n\t"
        "global_load_dwordx4 %30, %51, off offset:2048\n\t"
        "global_load_dwordx4 %31, %51, off offset:3072\n\t"
        "global_load_dwordx4 %32, %52, off offset:0\n\t"
        "global_load_dwordx4 %33, %52, off offset:1024\n\t"
        "global_load_dwordx4 %34, %52, off offset:2048\n\t"
        "global_load_dwordx4 %35, %52, off offset:3072\n\t"
        "global_load_dwordx4 %36, %53, off offset:0\n\t"
        "global_load_dwordx4 %37, %53, off offset:1024\n\t"
        "global_load_dwordx4 %38, %53, off offset:2048\n\t"
        "global_load_dwordx4 %39, %53, off offset:3072\n\t"
        "global_load_dwordx4 %40, %54, off offset:0\n\t"
        "global_load_dwordx4 %41, %54, off offset:1024\n\t"
        "global_load_dwordx4 %42, %54, off offset:2048\n\t"
        "global_load_dwordx4 %43, %54, off offset:3072\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]), "=&v"(t[7]), "=&v"(t[8]), "=&v"(t[9]), "=&v"(t[10]), "=&v"(t[11]), "=&v"(t[12]), "=&v"(t[13]), "=&v"(t[14]), "=&v"(t[15]), "=&v"(t[16]), "=&v"(t[17]), "=&v"(t[18]), "=&v"(t[19]), "=&v"(t[20]), "=&v"(t[21]), "=&v"(t[22]), "=&v"(t[23]), "=&v"(t[24]), "=&v"(t[25]), "=&v"(t[26]), "=&v"(t[27]), "=&v"(t[28]), "=&v"(t[29]), "=&v"(t[30]), "=&v"(t[31]), "=&v"(t[32]), "=&v"(t[33]), "=&v"(t[34]), "=&v"(t[35]), "=&v"(t[36]), "=&v"(t[37]), "=&v"(t[38]), "=&v"(t[39]), "=&v"(t[40]), "=&v"(t[41]), "=&v"(t[42]), "=&v"(t[43])
        : "v"(p0), "v"(p1), "v"(p2), "v"(p3), "v"(p4), "v"(p5), "v"(p6), "v"(p7), "v"(p8), "v"(p9), "v"(p10)
        : "memory");
}

// canonical state row of local feature row fl of main tile t / of the extra (1st/0th order) tile
__device__ __forceinline__ int canon_row_main(int t, int fl) { return 1 + DP + 32 * t + fl; }
__device__ __forceinline__ int canon_row_extra(int fl) { return fl < DP ? 1 + fl : (fl == DP ? 0 : -1); }

}  // namespace

// MODE 0: full prefill of the segment (readout + update); starts from the sum of workspace entries.
// MODE 1: state increment of the segment only (update GEMMs), written to workspace entry 1 + seg.
// MODE 2: the caller's initial state, converted to accumulator layout, written to entry 0.
// The main launch never reads the caller's state buffer, so writing the final state back into it
// cannot race with another workgroup still starting up.
template <int MODE>
__global__ __launch_bounds__(NT) void prefill_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ y, float *__restrict__ state, int has_init, float *__restrict__ ws, int N,
    int dv, int seg_len, int G)
{
    __shared__ __align__(16) Lds lds;

    const int tid = threadIdx.x;
    const int w = tid >> 6;              // wave: owns main tiles 4w .. 4w+3
    const int lane = tid & 63;
    const int g = lane >> 5, n = lane & 31;

    const int slices = dv / DVS;
    const int gseg = MODE == 1 ? G - 1 : (MODE == 2 ? 1 : G);   // segments this launch covers
    int bid = blockIdx.x;
    const int seg = bid % gseg; bid /= gseg;
    const int slice = bid % slices;
    const int u = bid / slices;
    const int col0 = slice * DVS;

    const int tok_begin = seg * seg_len;
    const int tok_end = min(N, tok_begin + seg_len);

    const uint16_t *qu = q + (size_t)u * N * DP;
    const uint16_t *ku = k + (size_t)u * N * DP;
    const uint16_t *vu = v + (size_t)u * N * dv + col0;
    uint16_t *yu = y + (size_t)u * N * dv + col0;
    float *Su = state ? state + (size_t)u * state_stride(DP, dv) : nullptr;
    float *zu = Su ? Su + (size_t)feature_dim(DP) * dv : nullptr;
    float *ws_unit = ws ? ws + ((size_t)(u * slices + slice) * G) * kWsEntryFloats : nullptr;

    // ---- accumulators -------------------------------------------------------------------------
    f32x16 S[4][2];        // main tiles [tt][c2]
    f32x16 X[2];           // wave 0: 1st/0th-order tile [c2]
    f32x16 M;              // wave 0: moment tile M' = [k, 1]^T [k, 1]
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
            for (int r = 0; r < 16; ++r) S[tt][c2][r] = 0.f;
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
        for (int r = 0; r < 16; ++r) X[c2][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) M[r] = 0.f;

    if (MODE == 0) {
        // start of segment: initial state (entry 0, if any) plus the increments of earlier segments
        for (int p = has_init ? 0 : 1; p <= seg; ++p) {
            f32x4 t[SLOTS * 4];
            load_entry(ws_unit + (size_t)p * kWsEntryFloats + ws_off(w, 0, 0, 0), lane, t);
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                    for (int r = 0; r < 16; ++r) S[tt][c2][r] += t[(tt * 2 + c2) * 4 + (r >> 2)][r & 3];
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int r = 0; r < 16; ++r) X[c2][r] += t[(8 + c2) * 4 + (r >> 2)][r & 3];
#pragma unroll
            for (int r = 0; r < 16; ++r) M[r] += t[10 * 4 + (r >> 2)][r & 3];
        }
    }
    if (MODE == 2) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2)
                    S[tt][c2][r] = Su[(size_t)canon_row_main(4 * w + tt, fl) * dv + col0 + 32 * c2 + n];
            if (w == 0) {
                const int row = canon_row_extra(fl);
                if (row >= 0) {
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2) X[c2][r] = Su[(size_t)row * dv + col0 + 32 * c2 + n];
                }
                float m = 0.f;   // M'[fl][n]
                if (fl < DP && n < DP) m = zu[1 + DP + fl * DP + n] * 1.41421356237309504880f;
                else if (fl == DP && n < DP) m = zu[1 + n];
                else if (fl < DP && n == DP) m = zu[1 + fl];
                else if (fl == DP && n == DP) m = zu[0];
                M[r] = m;
            }
        }
    }

    // zero rows 17..31 of both K'^T staging buffers once
    for (int i = tid; i < 2 * 15 * KTB_LD; i += NT) {
        const int b = i / (15 * KTB_LD), rem = i % (15 * KTB_LD);
        lds.st[b].ktb[17 + rem / KTB_LD][rem % KTB_LD] = 0;
    }

    // ---- staging: global -> registers -> LDS ----------------------------------------------------
    const int s_tok = tid & 63, s_half = tid >> 6;
    u32x4 raw_k, raw_q, raw_v[4];
    auto load_raw = [&](int tok0) {
        const int tok = tok0 + s_tok;
        const bool ok = tok < tok_end;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        raw_k = ok ? *reinterpret_cast<const u32x4 *>(ku + (size_t)tok * DP + 8 * s_half) : zero;
        if (MODE == 0) raw_q = ok ? *reinterpret_cast<const u32x4 *>(qu + (size_t)tok * DP + 8 * s_half) : zero;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            raw_v[j] = ok ? *reinterpret_cast<const u32x4 *>(vu + (size_t)tok * dv + 32 * s_half + 8 * j) : zero;
    };
    auto stage = [&](Stage &st, int tok0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t wd = raw_k[i];
            st.kts[8 * s_half + 2 * i][s_tok] = bf16lo(wd) * kC4;
            st.kts[8 * s_half + 2 * i + 1][s_tok] = bf16hi(wd) * kC4;
            st.ktb[8 * s_half + 2 * i][s_tok] = (uint16_t)(wd & 0xffffu);
            st.ktb[8 * s_half + 2 * i + 1][s_tok] = (uint16_t)(wd >> 16);
        }
        if (s_half == 0) st.ktb[16][s_tok] = (tok0 + s_tok < tok_end) ? (uint16_t)0x3F80u : (uint16_t)0u;
        if (MODE == 0) {
            f32x4 lo, hi;
            lo[0] = bf16lo(raw_q[0]) * kC4; lo[1] = bf16hi(raw_q[0]) * kC4;
            lo[2] = bf16lo(raw_q[1]) * kC4; lo[3] = bf16hi(raw_q[1]) * kC4;
            hi[0] = bf16lo(raw_q[2]) * kC4; hi[1] = bf16hi(raw_q[2]) * kC4;
            hi[2] = bf16lo(raw_q[3]) * kC4; hi[3] = bf16hi(raw_q[3]) * kC4;
            *reinterpret_cast<f32x4 *>(&st.qs[s_tok][8 * s_half]) = lo;
            *reinterpret_cast<f32x4 *>(&st.qs[s_tok][8 * s_half + 4]) = hi;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t wd = raw_v[j][i];
                st.vt[32 * s_half + 8 * j + 2 * i][s_tok] = (uint16_t)(wd & 0xffffu);
                st.vt[32 * s_half + 8 * j + 2 * i + 1][s_tok] = (uint16_t)(wd >> 16);
            }
    };

    // operand whose only non-zero entry is k-slot 0 (the constant feature, local row 16)
    u32x4 const_op = {0u, 0u, 0u, 0u};
    if (g == 0) const_op[0] = 0x3F80u;

    // operands that come straight from global memory: q (two 8-byte pieces per lane) for the
    // 1st-order rows and the moments; K and Q tiles of the intra-chunk block (wave 1)
    u32x4 kop[2], qop[2], qbop[2];
    auto load_ops = [&](int tok0) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
            const int tok = tok0 + 32 * t2 + n;
            const bool ok = tok < tok_end;
            qbop[t2] = zero;
            if (ok) {
                const u32x2 a = *reinterpret_cast<const u32x2 *>(qu + (size_t)tok * DP + 4 * g);
                const u32x2 b = *reinterpret_cast<const u32x2 *>(qu + (size_t)tok * DP + 8 + 4 * g);
                qbop[t2][0] = a[0]; qbop[t2][1] = a[1]; qbop[t2][2] = b[0]; qbop[t2][3] = b[1];
            }
            if (w == 1) {
                kop[t2] = ok ? *reinterpret_cast<const u32x4 *>(ku + (size_t)tok * DP + 8 * g) : zero;
                qop[t2] = ok ? *reinterpret_cast<const u32x4 *>(qu + (size_t)tok * DP + 8 * g) : zero;
            }
        }
    };
    // V^T operands of a chunk: [kt][s][c2]; lane (g, n): column 32 c2 + n, tokens of the slab
    auto load_vop = [&](const Stage &st, bf16x8 (&vop)[2][2][2]) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) {
                    const uint16_t *p = &st.vt[32 * c2 + n][32 * kt + 16 * s + 4 * g];
                    const u32x2 a = *reinterpret_cast<const u32x2 *>(p);
                    const u32x2 b = *reinterpret_cast<const u32x2 *>(p + 8);
                    u32x4 o; o[0] = a[0]; o[1] = a[1]; o[2] = b[0]; o[3] = b[1];
                    vop[kt][s][c2] = as_bf16x8(o);
                }
    };

    // Pipeline: chunk c+1 is fetched from global memory and staged into the other LDS buffer
    // during the update phase of chunk c, so its latency hides under the update MFMAs.
    if (MODE != 2) {
        load_raw(tok_begin);
        stage(lds.st[0], tok_begin);
        if (MODE == 0) load_ops(tok_begin);
    }
    int buf = 0;
    for (int tok0 = tok_begin; MODE != 2 && tok0 < tok_end; tok0 += C, buf ^= 1) {
        Stage &st = lds.st[buf];
        wg_sync();   // this chunk's staging is visible; the other buffer is free

        if (MODE == 0) {
            // =============================== readout ============================================
            f32x16 Y[2][2];   // Y^T [qt][c2]: lane (g, n) = query 32 qt + n, register r = column
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                    for (int r = 0; r < 16; ++r) Y[qt][c2][r] = 0.f;

            float qa[2][8], qb[2][8];   // c*q_a for a = 8w .. 8w+7; c*q_b for b = 8 jj + 4 g + i
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                const float *row = st.qs[32 * qt + n];
                const f32x4 a0 = *reinterpret_cast<const f32x4 *>(row + 8 * w);
                const f32x4 a1 = *reinterpret_cast<const f32x4 *>(row + 8 * w + 4);
                const f32x4 b0 = *reinterpret_cast<const f32x4 *>(row + 4 * g);
                const f32x4 b1 = *reinterpret_cast<const f32x4 *>(row + 8 + 4 * g);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    qa[qt][i] = a0[i]; qa[qt][4 + i] = a1[i];
                    qb[qt][i] = b0[i]; qb[qt][4 + i] = b1[i];
                }
            }

            // inter-chunk: Y^T += S^T phi(Q)^T over this wave's feature rows
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    bf16x8 phiq[2];
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt) {
                        float pr[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) pr[e] = qa[qt][2 * tt + s] * qb[qt][e];
                        phiq[qt] = pack8(pr);
                    }
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2) {
                        const bf16x8 sb = pack8_acc(S[tt][c2], s);
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt) Y[qt][c2] = mfma(sb, phiq[qt], Y[qt][c2]);
                    }
                }

            if (w == 0) {
                role_guard();
                // 1st-order rows (slab 0: operand is q itself) and the constant row (slab 1)
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) {
                    const bf16x8 s0 = pack8_acc(X[c2], 0), s1 = pack8_acc(X[c2], 1);
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt) {
                        Y[qt][c2] = mfma(s0, as_bf16x8(qbop[qt]), Y[qt][c2]);
                        Y[qt][c2] = mfma(s1, as_bf16x8(const_op), Y[qt][c2]);
                    }
                }
                // ---- inter-chunk denominator from the moments: count + q.z1 + q^T M q / 2 --------
                float mres[8];
                const bf16x8 mhi = pack8_acc(M, 0);
                {
                    const u32x4 hb = __builtin_bit_cast(u32x4, mhi);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        mres[2 * i] = M[2 * i] - bf16lo(hb[i]);
                        mres[2 * i + 1] = M[2 * i + 1] - bf16hi(hb[i]);
                    }
                }
                const bf16x8 mlo = pack8(mres);
                const float cnt_prev = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(M[8]), 16));
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    f32x16 T;
#pragma unroll
                    for (int r = 0; r < 16; ++r) T[r] = 0.f;
                    T = mfma(mhi, as_bf16x8(qbop[qt]), T);
                    T = mfma(mlo, as_bf16x8(qbop[qt]), T);
                    float d2 = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) d2 = fmaf(T[e], qb[qt][e], d2);
                    const float d = fmaf(d2, kHalfInvC4, T[8]);   // T[8]: row 16 = q.z1 on g = 0, zero on g = 1
                    const float tot = d + __shfl_xor(d, 32, 64) + cnt_prev;
                    if (g == 0) lds.den_inter[32 * qt + n] = tot;
                }
            } else {
                role_guard();
                // ---- intra-chunk block: P^T = mask(1 + A^T + A^T^2 / 2), Y^T += V^T P^T ----------
                bf16x8 vop[2][2][2];
                load_vop(st, vop);
                float den[2] = {0.f, 0.f};
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int kt = 0; kt <= qt; ++kt) {
                        f32x16 P;
#pragma unroll
                        for (int r = 0; r < 16; ++r) P[r] = 0.f;
                        P = mfma(as_bf16x8(kop[kt]), as_bf16x8(qop[qt]), P);   // rows keys, columns queries
                        float dsum = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float x = P[r];
                            float p = fmaf(x, fmaf(x, 0.5f, 1.f), 1.f);
                            if (kt == qt) {
                                const int key = 8 * (r >> 2) + 4 * g + (r & 3);
                                p = key <= n ? p : 0.f;
                            }
                            P[r] = p;
                            dsum += p;
                        }
                        den[qt] += dsum;
#pragma unroll
                        for (int s = 0; s < 2; ++s) {
                            const bf16x8 pb = pack8_acc(P, s);
#pragma unroll
                            for (int c2 = 0; c2 < 2; ++c2) Y[qt][c2] = mfma(vop[kt][s][c2], pb, Y[qt][c2]);
                        }
                    }
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    const float tot = den[qt] + __shfl_xor(den[qt], 32, 64);
                    if (g == 0) lds.den_intra[32 * qt + n] = tot;
                }
            }

            // ---- exchange partials: wave w finishes query tile qt = w ----------------------------
            auto put_partial = [&](const f32x16 (&Yo)[2]) {
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        f32x4 o;
#pragma unroll
                        for (int i = 0; i < 4; ++i) o[i] = Yo[c2][4 * j + i];
                        *reinterpret_cast<f32x4 *>(&lds.xbuf[w][c2 * 4 + j][lane][0]) = o;
                    }
            };
            auto finish = [&](const f32x16 (&Ym)[2]) {
                const int tok = tok0 + 32 * w + n;
                const float inv = 1.f / (lds.den_inter[32 * w + n] + lds.den_intra[32 * w + n]);
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const f32x4 o = *reinterpret_cast<const f32x4 *>(&lds.xbuf[1 - w][c2 * 4 + j][lane][0]);
                        float r4[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) r4[i] = (Ym[c2][4 * j + i] + o[i]) * inv;
                        if (tok < tok_end) {
                            f32x4 rv;
#pragma unroll
                            for (int i = 0; i < 4; ++i) rv[i] = r4[i];
                            const bf16x4 hv = __builtin_convertvector(rv, bf16x4);
                            *reinterpret_cast<u32x2 *>(yu + (size_t)tok * dv + 32 * c2 + 8 * j + 4 * g) =
                                __builtin_bit_cast(u32x2, hv);
                        }
                    }
            };
            if (w == 0) put_partial(Y[1]); else put_partial(Y[0]);
            wg_sync();
            if (w == 0) finish(Y[0]); else finish(Y[1]);
        }

        // =================================== update =============================================
        // S += phi(K)^T V over this wave's feature rows; lane (g, n): feature row n of the tile
        {
            const bool more = tok0 + C < tok_end;
            if (more) load_raw(tok0 + C);
            bf16x8 vop[2][2][2];
            load_vop(st, vop);
            const int brow = n & 15, ahalf = n >> 4;
            float kb[2][2][8];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const float *p = &st.kts[brow][32 * kt + 16 * s + 4 * g];
                    const f32x4 a = *reinterpret_cast<const f32x4 *>(p);
                    const f32x4 b = *reinterpret_cast<const f32x4 *>(p + 8);
#pragma unroll
                    for (int i = 0; i < 4; ++i) { kb[kt][s][i] = a[i]; kb[kt][s][4 + i] = b[i]; }
                }
            // rows a of c K^T for one tile: [kt * 2 + s][jj], fetched one tile ahead of its use so the
            // LDS latency hides under the previous tile's MFMAs
            f32x4 ka[2][4][2];
            auto load_ka = [&](int tt, f32x4 (&dst)[4][2]) {
                const int arow = 8 * w + 2 * tt + ahalf;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const float *p = &st.kts[arow][32 * kt + 16 * s + 4 * g];
                        dst[kt * 2 + s][0] = *reinterpret_cast<const f32x4 *>(p);
                        dst[kt * 2 + s][1] = *reinterpret_cast<const f32x4 *>(p + 8);
                    }
            };
            load_ka(0, ka[0]);
            // Software pipeline over the 16 (tile, slab) steps: the feature products of step i + 1 are
            // computed (into a second operand register set) while the MFMAs of step i run.  With a
            // single operand register set the vector ALU would have to wait for each MFMA to finish
            // reading it before overwriting it, and the two pipes would take turns instead of overlapping.
            auto gen = [&](int step) {
                const int tt = step >> 2, ks = step & 3;   // ks = kt * 2 + s
                float pr[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pr[i] = ka[tt & 1][ks][0][i] * kb[ks >> 1][ks & 1][i];
                    pr[4 + i] = ka[tt & 1][ks][1][i] * kb[ks >> 1][ks & 1][4 + i];
                }
                return pack8(pr);
            };
            bf16x8 phik[2];
            phik[0] = gen(0);
#pragma unroll
            for (int step = 0; step < 16; ++step) {
                const int tt = step >> 2, ks = step & 3;
                if (ks == 0 && tt + 1 < 4) load_ka(tt + 1, ka[(tt + 1) & 1]);
                if (step + 1 < 16) phik[(step + 1) & 1] = gen(step + 1);
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2)
                    S[tt][c2] = mfma(phik[step & 1], vop[ks >> 1][ks & 1][c2], S[tt][c2]);
            }
            // [k_0..k_15, 1, 0..]^T operand: the 1st/0th-order feature rows and the moment operand
            if (w == 0)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    role_guard();
                    const uint16_t *p = &st.ktb[n][32 * kt + 16 * s + 4 * g];
                    const u32x2 a = *reinterpret_cast<const u32x2 *>(p);
                    const u32x2 b = *reinterpret_cast<const u32x2 *>(p + 8);
                    u32x4 o; o[0] = a[0]; o[1] = a[1]; o[2] = b[0]; o[3] = b[1];
                    const bf16x8 kk = as_bf16x8(o);
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2) X[c2] = mfma(kk, vop[kt][s][c2], X[c2]);
                    M = mfma(kk, kk, M);
                }
            if (more) {
                stage(lds.st[buf ^ 1], tok0 + C);
                if (MODE == 0) load_ops(tok0 + C);
            }
        }
    }

    // ---- end of segment -----------------------------------------------------------------------
    if (MODE != 0) {
        float *e = ws_unit + (size_t)(MODE == 1 ? 1 + seg : 0) * kWsEntryFloats;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4 o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = S[tt][c2][4 * j + i];
                    *reinterpret_cast<f32x4 *>(e + ws_off(w, tt * 2 + c2, j, lane)) = o;
                }
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = X[c2][4 * j + i];
                *reinterpret_cast<f32x4 *>(e + ws_off(w, 8 + c2, j, lane)) = o;
            }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f32x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = M[4 * j + i];
            *reinterpret_cast<f32x4 *>(e + ws_off(w, 10, j, lane)) = o;
        }
    } else if (Su && seg == G - 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2)
                    Su[(size_t)canon_row_main(4 * w + tt, fl) * dv + col0 + 32 * c2 + n] = S[tt][c2][r];
            if (w == 0) {
                const int row = canon_row_extra(fl);
                if (row >= 0) {
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2) Su[(size_t)row * dv + col0 + 32 * c2 + n] = X[c2][r];
                }
                if (slice == 0) {
                    const float m = M[r];
                    if (fl < DP && n < DP) zu[1 + DP + fl * DP + n] = m * kRsqrt2;
                    else if (fl == DP && n < DP) zu[1 + n] = m;
                    else if (fl == DP && n == DP) zu[0] = m;
                }
            }
        }
    }
}

// ---- host side ----------------------------------------------------------------------------------
namespace {

// Segments per sequence: enough workgroups to put a wave on every SIMD of the chip, but segments
// of at least 512 tokens so that the state increments stay small next to q, k, v, y.
int pick_segments(int U, int N, int dv)
{
    const long groups = (long)U * (dv / DVS);
    const long want = 512;   // workgroups of two waves
    int G = (int)((want + groups - 1) / groups);
    const int max_by_len = N / 512;
    if (G > max_by_len) G = max_by_len;
    if (G > 8) G = 8;
    if (G < 1) G = 1;
    return G;
}

int segment_len(int N, int G)
{
    const int per = (N + G - 1) / G;
    return (per + C - 1) / C * C;
}

}  // namespace

bool prefill_mfma_supported(int dp, int dv, int dtype)
{
    return dtype == BASED_BF16 && dp == DP && (dv == 64 || dv == 128);
}

size_t prefill_mfma_workspace_bytes(int U, int N, int dp, int dv)
{
    (void)dp;
    const int G = pick_segments(U, N, dv);
    return (size_t)U * (dv / DVS) * G * kWsEntryFloats * sizeof(float);
}

hipError_t launch_prefill_mfma(const void *q, const void *k, const void *v, void *y, float *state,
                               int has_init, void *workspace, int U, int N, int dp, int dv,
                               hipStream_t s)
{
    (void)dp;
    const int slices = dv / DVS;
    int G = pick_segments(U, N, dv);
    const int seg_len = segment_len(N, G);
    // rounding the segment length up to whole chunks can leave trailing segments empty; a smaller
    // G only uses a prefix of the workspace that was sized for pick_segments()
    while (G > 1 && (G - 1) * seg_len >= N) --G;
    const uint16_t *q16 = (const uint16_t *)q, *k16 = (const uint16_t *)k, *v16 = (const uint16_t *)v;
    hipError_t e;
    if (has_init) {
        hipLaunchKernelGGL((prefill_mfma_kernel<2>), dim3((unsigned)(U * slices)), dim3(NT), 0, s, q16, k16,
                           v16, (uint16_t *)y, state, 1, (float *)workspace, N, dv, seg_len, G);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (G > 1) {
        hipLaunchKernelGGL((prefill_mfma_kernel<1>), dim3((unsigned)(U * slices * (G - 1))), dim3(NT), 0, s,
                           q16, k16, v16, (uint16_t *)y, state, has_init, (float *)workspace, N, dv,
                           seg_len, G);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    hipLaunchKernelGGL((prefill_mfma_kernel<0>), dim3((unsigned)(U * slices * G)), dim3(NT), 0, s, q16, k16,
                       v16, (uint16_t *)y, state, has_init, (float *)workspace, N, dv, seg_len, G);
    return hipGetLastError();
}

}  // namespace based
