// Causal Taylor linear attention, chunked prefill on the gfx950 matrix cores (bf16 in, fp32
// accumulate), d' = 32.
//
// Same method as the d' = 16 kernel (chunked form of Sec. 4: masked quadratic product inside a
// chunk of 64 tokens, running KV-state across chunks, features of Eq. 4 built in registers in
// MFMA operand layout, k-slots mapped onto the rows a lane holds in its accumulators), laid out
// for the larger state:
//
// Symmetric packing.  One state row per unordered pair {a, b}: row (a, delta) stands for the
// pair {a, (a + delta) mod 32}, delta = 0 .. 15 for every a (16 tiles of exactly 32 rows, one
// delta per tile) and delta = 16 for a < 16.  The k side builds x_a x_b / sqrt(2), the q side
// sqrt(2) x_a x_b (delta != 0) or x_a^2 / sqrt(2) (delta = 0).  528 pair rows instead of 1024.
//
// Work split.  One workgroup of four waves per (unit, 32-column slice of d_v, sequence segment);
// wave w owns the four main tiles delta = 4w .. 4w+3.  Two extra tiles: E1 = the 32 linear rows
// (wave 2), E2 = [1, 0 x 15, the 16 rows of delta = 16] (wave 0); wave 3 has the K-state.  The
// three blocks of the intra-chunk product go to waves 0 (keys 0, queries 0), 1 (keys 1, queries 1)
// and 2 (keys 0, queries 1).  Per chunk each wave produces a partial Y^T over its feature rows for
// both query tiles; wave 0 finishes query tile 0, wave 1 tile 1.  (Roles are spread so that the
// waves reach the two barriers of a chunk at about the same time.)
//
// Denominator.  Wave 3 carries the K-state as moments: M[a][b] = sum_t k_a k_b (one tile, an MFMA
// of the K rows with themselves), z1[a] = sum_t k_a (vector adds) and the token count.  Per query
// phi(q).z = z0 + sum_a q_a (z1[a] + (M q)[a] / 2); the part from inside the chunk is the column
// sum of the masked block P the intra-chunk waves hold anyway.
//
// Long sequences / few units: G segments; a first launch computes each segment's state increment
// (update GEMMs only), the later launches start each segment from the sum of the entries before it.
#include "common.h"

namespace based {

namespace dp32 {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int DP = 32;            // d'
constexpr int C = 64;             // chunk length (tokens)
constexpr int NW = 4;             // waves per workgroup
constexpr int NT = NW * 64;
constexpr int DVS = 32;           // d_v columns per workgroup
constexpr int TPW = 4;            // main tiles per wave
constexpr float kCK = 0.84089641525371454303f;   // 2^(-1/4): (c k_a)(c k_b) = k_a k_b / sqrt(2)
constexpr float kCQ = 1.18920711500272106672f;   // 2^(+1/4): (c q_a)(c q_b) = sqrt(2) q_a q_b

// LDS strides (elements)
constexpr int KTS_LD = C + 4;     // fp32 K^T rows
constexpr int VR_LD = DVS + 16;   // bf16 V rows (96-byte stride)
constexpr int QS_LD = DP + 4;     // fp32 Q rows
constexpr int QR_LD = DP + 8;     // bf16 Q rows as given (80-byte stride)
constexpr int KR_LD = 64 + 16;    // bf16 extended K rows (160-byte stride)
constexpr int YT_LD = 32 + 8;     // bf16 rows of a finished output tile on its way out

// Workspace entry (one segment's state in accumulator layout): 20 slots of 16 registers x 64 lanes:
// slot 4w + tt = main tile tt of wave w; 16 = E1; 17 = E2; 18 = M; 19 = [z1, z0] in the first two
// registers.  Within a slot: [r / 4][lane][r % 4].
constexpr int WS_SLOTS = 20;
constexpr size_t kWsEntryFloats = (size_t)WS_SLOTS * 16 * 64;

struct Stage {
    float kts[DP][KTS_LD];        // c_k * K^T
    uint16_t krow[C][KR_LD];      // extended K rows: [k_0..k_31 as given, 1 (0 past the end), 0 x 15,
                                  // k_a k_(a+16) / sqrt(2) for a < 16]
    uint16_t vrow[C][VR_LD];      // V rows of the slice, bf16 as given
    float qs[C][QS_LD];           // c_q * Q
    uint16_t qrow[C][QR_LD];      // Q rows, bf16 as given
};

struct Lds {
    Stage st;
    float xbuf[2][3][4][64][4];   // partial Y^T tiles: [query tile][sender slot][r / 4][lane][r % 4]
    float z1s[DP];                // z1, for wave 3's own broadcast reads
    float dint[2][32];            // denominators: the part from before the chunk, [query tile][query]
    float dsum[3][32];            // ... and from inside it: column sums of the blocks (k0,q0), (k0,q1), (k1,q1)
                                  // (written by waves 0, 2, 1)
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

__device__ __forceinline__ void zero16(f32x16 &a)
{
#pragma unroll
    for (int r = 0; r < 16; ++r) a[r] = 0.f;
}

// Workgroup barrier that orders LDS traffic only (global loads and stores stay in flight).
__device__ __forceinline__ void wg_sync()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// MFMA instructions ignore the EXEC mask; an inline-asm statement in a wave-role block makes the
// compiler keep the jump over it (it never runs inline asm with an empty EXEC mask).
__device__ __forceinline__ void role_guard() { asm volatile("; wave-role block: keep the execz branch"); }

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ size_t ws_slot_off(int slot, int j, int lane)
{
    return (((size_t)slot * 4 + j) * 64 + lane) * 4;
}

// Canonical state rows (Eq. 4 order) of a packed row; a pair row has two (equal for delta = 0).
// With packed_state the buffer is the packed layout (one row per unordered pair: a single row).
struct CanonRows { int r1, r2; };   // r1 < 0: padding
__device__ __forceinline__ CanonRows canon_pair(int a, int b, bool packed_state)
{
    if (packed_state) {
        const int r = packed_pair_row(DP, min(a, b), max(a, b));
        return {r, r};
    }
    return {1 + DP + a * DP + b, 1 + DP + b * DP + a};
}
__device__ __forceinline__ CanonRows canon_rows_main(int delta, int fl, bool packed_state)
{
    return canon_pair(fl, (fl + delta) & (DP - 1), packed_state);
}
__device__ __forceinline__ CanonRows canon_rows_e1(int fl) { return {1 + fl, 1 + fl}; }
__device__ __forceinline__ CanonRows canon_rows_e2(int fl, bool packed_state)
{
    if (fl == 0) return {0, 0};
    if (fl >= 16) return canon_pair(fl - 16, fl, packed_state);
    return {-1, -1};
}

constexpr int kMaxSegments = 16;
struct SegTable { int begin[kMaxSegments + 1]; };

// MODE 0: full prefill of the segment; MODE 1: state increment only, to workspace entry 1 + seg;
// MODE 2: the caller's initial state, converted, to entry 0.
// Slice: columns [32 slice, 32 slice + 32) of v / y.
template <int MODE>
__global__ __launch_bounds__(NT, 2) void prefill_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ y, float *__restrict__ state, int has_init, float *__restrict__ ws,
    int N, int dv, SegTable segs, int G)
{
    __shared__ __align__(16) Lds lds;

    // has_init carries three flags: bit 0 an initial state is given, bit 1 the state buffer is packed,
    // bit 2 the outputs are the numerators alone (no division by the denominator)
    const bool packed_state = (has_init & 2) != 0;
    const bool numerator_only = (has_init & 4) != 0;
    has_init &= 1;
    const int tid = threadIdx.x;
    const int w = tid >> 6;
    const int lane = tid & 63;
    const int g = lane >> 5, n = lane & 31;

    const int slices = dv / DVS;
    const int gseg = MODE == 1 ? G - 1 : (MODE == 2 ? 1 : G);
    int bid = blockIdx.x;
    const int seg = bid % gseg; bid /= gseg;
    const int slice = bid % slices;
    const int u = bid / slices;
    const int col0 = slice * DVS;

    const int tok_begin = segs.begin[seg];
    const int tok_end = min(N, segs.begin[seg + 1]);

    const uint16_t *qu = q + (size_t)u * N * DP;
    const uint16_t *ku = k + (size_t)u * N * DP;
    const uint16_t *vu = v + (size_t)u * N * dv + col0;
    uint16_t *yu = y + (size_t)u * N * dv + col0;
    float *Su = state ? state + (size_t)u * (packed_state ? packed_state_stride(DP, dv) : state_stride(DP, dv))
                      : nullptr;
    float *zu = Su ? Su + (size_t)(packed_state ? packed_feature_dim(DP) : feature_dim(DP)) * dv : nullptr;
    float *ws_unit = ws + ((size_t)(u * slices + slice) * G) * kWsEntryFloats;

    // ---- accumulators -------------------------------------------------------------------------
    f32x16 S[TPW];         // main tiles delta = 4w + tt
    f32x16 X;              // wave 0: E2; wave 2: E1; wave 3: M; unused by wave 1
    float z1 = 0.f, z0 = 0.f;   // wave 3: z1[n] (both halves of the wave), tokens before this call's first
#pragma unroll
    for (int tt = 0; tt < TPW; ++tt) zero16(S[tt]);
    zero16(X);

    if (MODE == 0) {
        // start of segment: entry 0 (the initial state, if any) plus the increments before it
        const int xs = w == 0 ? 17 : (w == 2 ? 16 : 18);
        for (int p = has_init ? 0 : 1; p <= seg; ++p) {
            const float *e = ws_unit + (size_t)p * kWsEntryFloats;
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const f32x4 t = *reinterpret_cast<const f32x4 *>(e + ws_slot_off(4 * w + tt, j, lane));
#pragma unroll
                    for (int i = 0; i < 4; ++i) S[tt][4 * j + i] += t[i];
                }
            if (w != 1) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const f32x4 t = *reinterpret_cast<const f32x4 *>(e + ws_slot_off(xs, j, lane));
#pragma unroll
                    for (int i = 0; i < 4; ++i) X[4 * j + i] += t[i];
                }
            }
            if (w == 3) {
                const f32x4 t = *reinterpret_cast<const f32x4 *>(e + ws_slot_off(19, 0, lane));
                z1 += t[0];
                z0 += t[1];
            }
        }
    }
    if (MODE == 2) {
        // canonical rows -> accumulator layout (the symmetric part of a pair's two rows)
        auto fetch = [&](CanonRows cr) -> float {
            if (cr.r1 < 0) return 0.f;
            const size_t col = (size_t)col0 + n;
            return 0.5f * (Su[(size_t)cr.r1 * dv + col] + Su[(size_t)cr.r2 * dv + col]);
        };
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt) S[tt][r] = fetch(canon_rows_main(4 * w + tt, fl, packed_state));
            if (w == 2) X[r] = fetch(canon_rows_e1(fl));
            else if (w == 0) X[r] = fetch(canon_rows_e2(fl, packed_state));
            else if (w == 3) {   // M[a][b] = sqrt(2) x the symmetric part of z's pair rows, a = fl, b = n
                const CanonRows cr = canon_pair(fl, n, packed_state);
                X[r] = kRsqrt2 * (zu[cr.r1] + zu[cr.r2]);
            }
        }
        if (w == 3) { z1 = zu[1 + n]; z0 = zu[0]; }
    }

    // ---- staging: global -> registers -> LDS ----------------------------------------------------
    // Thread (s_tok, s_q) stages, of token s_tok: elements 8h .. 8h+7 and 16+8h .. 16+8h+7 (h = s_q % 2)
    // of the K row (waves 0, 1) or of the Q row (waves 2, 3), and a quarter of the slice's V row.
    const int s_tok = tid & 63, s_q = tid >> 6, s_h = s_q & 1;
    u32x4 raw_x[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    u32x4 raw_v;
    auto load_raw = [&](int tok0) {
        const int tok = min(tok0 + s_tok, tok_end - 1);
        const uint16_t *xc = (s_q < 2 ? ku : qu) + (size_t)tok * DP + 8 * s_h;
        if (MODE == 0 || s_q < 2) {
#pragma unroll
            for (int j = 0; j < 2; ++j) raw_x[j] = *reinterpret_cast<const u32x4 *>(xc + 16 * j);
        }
        raw_v = *reinterpret_cast<const u32x4 *>(vu + (size_t)tok * dv + 8 * s_q);
    };
    auto stage = [&](int tok0) {
        Stage &st = lds.st;
        const bool valid = tok0 + s_tok < tok_end;
        const u32x4 zero4 = {0u, 0u, 0u, 0u};
        if (!valid) { raw_x[0] = zero4; raw_x[1] = zero4; raw_v = zero4; }
        if (s_q < 2) {
            float kf[2][8];   // c_k * k: [j][i] = element 16 j + 8 h + i
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t wd = raw_x[j][i];
                    const int a = 16 * j + 8 * s_h + 2 * i;
                    kf[j][2 * i] = bf16lo(wd) * kCK;
                    kf[j][2 * i + 1] = bf16hi(wd) * kCK;
                    st.kts[a][s_tok] = kf[j][2 * i];
                    st.kts[a + 1][s_tok] = kf[j][2 * i + 1];
                }
                *reinterpret_cast<u32x4 *>(&st.krow[s_tok][16 * j + 8 * s_h]) = raw_x[j];
            }
            f32x8 pr;
#pragma unroll
            for (int i = 0; i < 8; ++i) pr[i] = kf[0][i] * kf[1][i];
            *reinterpret_cast<u32x4 *>(&st.krow[s_tok][48 + 8 * s_h]) =
                __builtin_bit_cast(u32x4, __builtin_convertvector(pr, bf16x8));
            // columns 32 .. 47: the constant feature, then zeros
            u32x4 c = zero4;
            if (s_h == 0 && valid) c[0] = 0x3F80u;
            if (s_q == s_h) *reinterpret_cast<u32x4 *>(&st.krow[s_tok][32 + 8 * s_h]) = c;
        } else if (MODE == 0) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    f32x4 qv;
                    qv[0] = bf16lo(raw_x[j][2 * hh]) * kCQ; qv[1] = bf16hi(raw_x[j][2 * hh]) * kCQ;
                    qv[2] = bf16lo(raw_x[j][2 * hh + 1]) * kCQ; qv[3] = bf16hi(raw_x[j][2 * hh + 1]) * kCQ;
                    *reinterpret_cast<f32x4 *>(&st.qs[s_tok][16 * j + 8 * s_h + 4 * hh]) = qv;
                }
                *reinterpret_cast<u32x4 *>(&st.qrow[s_tok][16 * j + 8 * s_h]) = raw_x[j];
            }
        }
        *reinterpret_cast<u32x4 *>(&st.vrow[s_tok][8 * s_q]) = raw_v;
    };

    // V^T operand (lane (g, n): column n at the 8 tokens of its k-slots, two runs of 4 tokens
    // starting at tok4 and tok4 + 8) from row-major rows, by the transposing LDS read: in each group
    // of 16 lanes, lane k supplies the address of 4 consecutive columns (4 (k % 4) ..) of row k / 4 of
    // the group's 16-column block and receives column k of that block at the 4 rows.
    const int tr_kk = lane & 15, tr_grp = (lane >> 4) & 1;
    const uint16_t *tr_vbase = &lds.st.vrow[tr_kk >> 2][16 * tr_grp + 4 * (tr_kk & 3)];
    const uint16_t *tr_kbase = &lds.st.krow[tr_kk >> 2][16 * tr_grp + 4 * (tr_kk & 3)];
    auto tr_read = [&](const uint16_t *p, int stride, s16x4 &a, s16x4 &b) {
        a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
        b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p + 8 * stride));
    };
    auto join = [](s16x4 a, s16x4 b) {
        s16x8 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[i] = a[i]; o[4 + i] = b[i]; }
        return __builtin_bit_cast(bf16x8, o);
    };

    if (MODE != 2) {
        load_raw(tok_begin);
        stage(tok_begin);
        if (w == 3 && g == 0) lds.z1s[n] = z1;
    }
    for (int tok0 = tok_begin; MODE != 2 && tok0 < tok_end; tok0 += C) {
        const Stage &st = lds.st;
        wg_sync();   // this chunk's staging is visible
        const bool more = tok0 + C < tok_end;
        if (more) load_raw(tok0 + C);   // a whole chunk ahead: consumed by stage() at the bottom

        f32x4 acc[4];     // the output tile this wave finishes (waves 0, 1)
        float inv = 1.f;
        if (MODE == 0) {
            // =============================== readout ============================================
            f32x16 Yown;
            zero16(Yown);
#pragma unroll 1
            for (int qt = 0; qt < 2; ++qt) {
                f32x16 Y;
                zero16(Y);
                // This lane's query row: qa[4m + i] = c_q q[4g + 8m + i] (m = 0..3: the "a side", k-slot
                // (s, jj, i) is a = 16 s + 8 jj + 4 g + i = element 4m + i with m = 2s + jj) and
                // qr[j] = c_q q[(4g + 4w + j) % 32] (the "b side" of delta = 4w + tt is
                // qr[(16 s + 8 jj + i + tt) % 32]).
                float qa[16], qr[32];
                {
                    const float *row = st.qs[32 * qt + n];
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        const f32x4 t = *reinterpret_cast<const f32x4 *>(row + 4 * g + 8 * m);
#pragma unroll
                        for (int i = 0; i < 4; ++i) qa[4 * m + i] = t[i];
                    }
#pragma unroll
                    for (int m = 0; m < 8; ++m) {
                        const f32x4 t = *reinterpret_cast<const f32x4 *>(row + ((4 * g + 4 * w + 4 * m) & 31));
#pragma unroll
                        for (int i = 0; i < 4; ++i) qr[4 * m + i] = t[i];
                    }
                }
                // inter-chunk: Y^T += S^T phi(Q)^T over this wave's feature rows.  (The empty asm keeps the
                // bf16 copies of the state from being made once per chunk and held in 32 registers.)
#pragma unroll
                for (int tt = 0; tt < TPW; ++tt) {
                    asm volatile("" : "+v"(S[tt]));
                    const float dw = (w == 0 && tt == 0) ? 0.5f : 1.f;   // delta = 0: x_a^2 / sqrt(2)
#pragma unroll
                    for (int sl = 0; sl < 2; ++sl) {
                        float pr[8];
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                pr[4 * jj + i] = qa[4 * (2 * sl + jj) + i] * dw * qr[(16 * sl + 8 * jj + i + tt) & 31];
                        Y = mfma(pack8_acc(S[tt], sl), pack8(pr), Y);
                    }
                }
                if (w == 0 || w == 2) {
                    role_guard();
                    const bf16x8 xlo = pack8_acc(X, 0), xhi = pack8_acc(X, 1);
                    if (w == 2) {
                        role_guard();
                        // E1: the linear rows; the operand is q itself (k-slot (s, jj, i) = element
                        // 16 s + 8 jj + 4 g + i)
                        const uint16_t *p = &st.qrow[32 * qt + n][4 * g];
#pragma unroll
                        for (int sl = 0; sl < 2; ++sl) {
                            const u32x2 a = *reinterpret_cast<const u32x2 *>(p + 16 * sl);
                            const u32x2 b = *reinterpret_cast<const u32x2 *>(p + 16 * sl + 8);
                            u32x4 o; o[0] = a[0]; o[1] = a[1]; o[2] = b[0]; o[3] = b[1];
                            Y = mfma(sl == 0 ? xlo : xhi, as_bf16x8(o), Y);
                        }
                    } else {
                        role_guard();
                        // E2: row 0 constant (slab 0, k-slot 0 of g = 0); rows 16 + a, a = 8 jj + 4 g + i:
                        // sqrt(2) q_a q_(a+16)
                        float c0[8], c1[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) c0[e] = 0.f;
                        c0[0] = g == 0 ? 1.f : 0.f;
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                            for (int i = 0; i < 4; ++i) c1[4 * jj + i] = qa[4 * jj + i] * qa[4 * (2 + jj) + i];
                        Y = mfma(xlo, pack8(c0), Y);
                        Y = mfma(xhi, pack8(c1), Y);
                    }
                }
                if (w == 3) {
                    role_guard();
                    // denominator from before the chunk: T[b][query] = sum_a M[a][b] q_a, then
                    // z0 + sum_b q_b (z1[b] + T[b] / 2) over this lane's 16 rows b and the other half's
                    f32x16 T;
                    zero16(T);
                    const uint16_t *p = &st.qrow[32 * qt + n][4 * g];
#pragma unroll
                    for (int sl = 0; sl < 2; ++sl) {
                        const u32x2 a = *reinterpret_cast<const u32x2 *>(p + 16 * sl);
                        const u32x2 b = *reinterpret_cast<const u32x2 *>(p + 16 * sl + 8);
                        u32x4 o; o[0] = a[0]; o[1] = a[1]; o[2] = b[0]; o[3] = b[1];
                        T = mfma(pack8_acc(X, sl), as_bf16x8(o), T);
                    }
                    float d = 0.f;
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        const f32x4 zv = *reinterpret_cast<const f32x4 *>(&lds.z1s[8 * m + 4 * g]);
#pragma unroll
                        for (int i = 0; i < 4; ++i) d = fmaf(qa[4 * m + i], fmaf(0.5f, T[4 * m + i], zv[i]), d);
                    }
                    d *= 1.f / kCQ;
                    d += __shfl_xor(d, 32, 64);
                    if (g == 0) lds.dint[qt][n] = z0 + (float)(tok0) + d;
                }
                // ---- intra-chunk block: P^T = mask(1 + A^T + A^T^2 / 2), Y^T += V^T P^T ----------
                // wave 0: key tile 0 against query tile 0; wave 1: keys 1, queries 1; wave 2: keys 0, queries 1
                if ((w == 0 && qt == 0) || ((w == 1 || w == 2) && qt == 1)) {
                    role_guard();
                    const int kt = w == 1 ? 1 : 0;
                    const bool diag = kt == qt;
                    f32x16 P;
                    zero16(P);
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {   // contraction over d' = 32 in two steps of 16
                        const u32x4 kop = *reinterpret_cast<const u32x4 *>(&st.krow[32 * kt + n][16 * ks + 8 * g]);
                        const u32x4 qop = *reinterpret_cast<const u32x4 *>(&st.qrow[32 * qt + n][16 * ks + 8 * g]);
                        P = mfma(as_bf16x8(kop), as_bf16x8(qop), P);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float x = P[r];
                        const float pv = fmaf(x, fmaf(x, 0.5f, 1.f), 1.f);
                        const int key = 8 * (r >> 2) + 4 * g + (r & 3);
                        P[r] = (!diag || key <= n) ? pv : 0.f;
                    }
                    {   // this block's share of the denominators: sum over its keys
                        float cs = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) cs += P[r];
                        cs += __shfl_xor(cs, 32, 64);
                        if (g == 0) lds.dsum[w == 0 ? 0 : (w == 2 ? 1 : 2)][n] = cs;
                    }
#pragma unroll
                    for (int sl = 0; sl < 2; ++sl) {
                        s16x4 a, b;
                        tr_read(tr_vbase + (32 * kt + 16 * sl + 4 * g) * VR_LD, VR_LD, a, b);
                        Y = mfma(join(a, b), pack8_acc(P, sl), Y);
                    }
                }
                // the partial tile goes to the wave that finishes this query tile
                if (qt == w) {
                    Yown = Y;
                } else {
                    const int slot = ((w - qt) & 3) - 1;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        f32x4 o;
#pragma unroll
                        for (int i = 0; i < 4; ++i) o[i] = Y[4 * j + i];
                        *reinterpret_cast<f32x4 *>(&lds.xbuf[qt][slot][j][lane][0]) = o;
                    }
                }
            }
            wg_sync();
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[j][i] = Yown[4 * j + i];
            if (w < 2) inv = lds.dint[w][n] + lds.dsum[w][n] + (w == 1 ? lds.dsum[2][n] : 0.f);
        }

        // =================================== update =============================================
        {
            const int arow = n;
            float z1c = 0.f;   // wave 3: this chunk's share of z1[n] from this half's tokens
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int tcol = 16 * i4 + 4 * g;   // first token of this lane's k-slots
                s16x4 va, vb;
                tr_read(tr_vbase + tcol * VR_LD, VR_LD, va, vb);
                const bf16x8 vk = join(va, vb);
                const f32x4 ka0 = *reinterpret_cast<const f32x4 *>(&st.kts[arow][tcol]);
                const f32x4 ka1 = *reinterpret_cast<const f32x4 *>(&st.kts[arow][tcol + 8]);
#pragma unroll
                for (int tt = 0; tt < TPW; ++tt) {
                    const int brow = (n + 4 * w + tt) & 31;
                    const f32x4 kb0 = *reinterpret_cast<const f32x4 *>(&st.kts[brow][tcol]);
                    const f32x4 kb1 = *reinterpret_cast<const f32x4 *>(&st.kts[brow][tcol + 8]);
                    float pr[8];
#pragma unroll
                    for (int i = 0; i < 4; ++i) { pr[i] = ka0[i] * kb0[i]; pr[4 + i] = ka1[i] * kb1[i]; }
                    S[tt] = mfma(pack8(pr), vk, S[tt]);
                }
                if (w == 0 || w == 2) {
                    role_guard();
                    s16x4 ea, eb;
                    tr_read(tr_kbase + tcol * KR_LD + (w == 0 ? 32 : 0), KR_LD, ea, eb);
                    X = mfma(join(ea, eb), vk, X);
                }
                if (w == 3) {
                    role_guard();
                    // the K rows against themselves: lane (g, n) holds k_n at its 8 tokens, which is both
                    // the row n of K^T and the column n of K
                    s16x4 ea, eb;
                    tr_read(tr_kbase + tcol * KR_LD, KR_LD, ea, eb);
                    const bf16x8 ek = join(ea, eb);
                    X = mfma(ek, ek, X);
                    const u32x4 kw = __builtin_bit_cast(u32x4, ek);
#pragma unroll
                    for (int i = 0; i < 4; ++i) z1c += bf16lo(kw[i]) + bf16hi(kw[i]);
                }
                if (MODE == 0 && w < 2) {
                    // collect a quarter of the other waves' partial tiles under this step's MFMAs
#pragma unroll
                    for (int sl = 0; sl < 3; ++sl) {
                        const f32x4 o = *reinterpret_cast<const f32x4 *>(&lds.xbuf[w][sl][i4][lane][0]);
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[i4][i] += o[i];
                    }
                }
            }
            if (w == 3) {
                z1 += z1c + __shfl_xor(z1c, 32, 64);
                if (g == 0) lds.z1s[n] = z1;
            }
        }
        if (MODE == 0 && w < 2) {
            const int qt = w;
            {
                // normalise and turn the tile through LDS (this wave's own exchange slots, which it has
                // finished reading): the tile leaves as 64-byte row segments, 16 rows a store
                const float rinv = numerator_only ? 1.f : 1.f / inv;
                uint16_t *yt = reinterpret_cast<uint16_t *>(&lds.xbuf[w][0][0][0][0]);   // [32][YT_LD] bf16
#pragma unroll
                for (int j = 0; j < 4; ++j) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[j][i] *= rinv;
                    const bf16x4 hv = __builtin_convertvector(acc[j], bf16x4);
                    *reinterpret_cast<u32x2 *>(yt + n * YT_LD + 8 * j + 4 * g) = __builtin_bit_cast(u32x2, hv);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                uint16_t *yc = yu + (size_t)tok0 * dv;
                u32x4 val[2];
                uint32_t yoff[2];
#pragma unroll
                for (int it = 0; it < 2; ++it) {
                    const int row = 16 * it + (lane >> 2), c = lane & 3;
                    val[it] = *reinterpret_cast<const u32x4 *>(yt + row * YT_LD + 8 * c);
                    yoff[it] = (uint32_t)(32 * qt + row) * (uint32_t)dv + (uint32_t)(8 * c);
                }
                if (tok0 + C <= tok_end) {
#pragma unroll
                    for (int it = 0; it < 2; ++it) *reinterpret_cast<u32x4 *>(yc + yoff[it]) = val[it];
                } else {
#pragma unroll
                    for (int it = 0; it < 2; ++it)
                        if (tok0 + 32 * qt + 16 * it + (lane >> 2) < tok_end) *reinterpret_cast<u32x4 *>(yc + yoff[it]) = val[it];
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                }
            }
        }
        if (more) {
            wg_sync();   // every wave is done reading this chunk's staging
            stage(tok0 + C);
        }
    }

    // ---- end of segment -----------------------------------------------------------------------
    if (MODE != 0) {
        float *e = ws_unit + (size_t)(MODE == 1 ? 1 + seg : 0) * kWsEntryFloats;
        auto put = [&](int slot, const f32x16 &a) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = a[4 * j + i];
                *reinterpret_cast<f32x4 *>(e + ws_slot_off(slot, j, lane)) = o;
            }
        };
#pragma unroll
        for (int tt = 0; tt < TPW; ++tt) put(4 * w + tt, S[tt]);
        if (w == 0) put(17, X);
        if (w == 2) put(16, X);
        if (w == 3) {
            put(18, X);
            const f32x4 o = {z1, MODE == 2 ? z0 : 0.f, 0.f, 0.f};
            *reinterpret_cast<f32x4 *>(e + ws_slot_off(19, 0, lane)) = o;
        }
    } else if (Su && seg == G - 1) {
        // final state in the canonical layout (both rows of a pair); slice 0 writes z
        auto emit = [&](CanonRows cr, float val) {
            if (cr.r1 < 0) return;
            const size_t col = (size_t)col0 + n;
            Su[(size_t)cr.r1 * dv + col] = val;
            if (cr.r2 != cr.r1) Su[(size_t)cr.r2 * dv + col] = val;
        };
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt) emit(canon_rows_main(4 * w + tt, fl, packed_state), S[tt][r]);
            if (w == 2) emit(canon_rows_e1(fl), X[r]);
            else if (w == 0) emit(canon_rows_e2(fl, packed_state), X[r]);
            else if (w == 3 && slice == 0 && (!packed_state || fl <= n))
                zu[canon_pair(fl, n, packed_state).r1] = kRsqrt2 * X[r];
        }
        if (w == 3 && slice == 0 && g == 0) {
            zu[1 + n] = z1;
            if (n == 0) zu[0] = z0 + (float)N;
        }
    }
}

// Segments: enough workgroups for two per CU, segments of at least 512 tokens.
static int pick_segments(int U, int N, int dv)
{
    const long groups = (long)U * (dv / DVS);
    int G = (int)((512 + groups - 1) / groups);
    if (G > N / 512) G = N / 512;
    if (G > kMaxSegments) G = kMaxSegments;
    return G < 1 ? 1 : G;
}

static int make_segments(int N, int G, SegTable &t)
{
    const int T = (N + C - 1) / C;
    if (G > T) G = T;
    int pos = 0;
    for (int g = 0; g < G; ++g) {
        t.begin[g] = pos * C;
        pos += T / G + (g < T % G ? 1 : 0);
    }
    for (int g = G; g <= kMaxSegments; ++g) t.begin[g] = pos * C;
    return G;
}

static size_t entry_bytes(int U, int N, int dv)
{
    return (size_t)U * (dv / DVS) * pick_segments(U, N, dv) * kWsEntryFloats * sizeof(float);
}

}  // namespace dp32

bool prefill_mfma32_supported(int dp, int dv, int dtype)
{
    return dtype == BASED_BF16 && dp == dp32::DP && (dv == 64 || dv == 128);
}

// Workspace: one entry per (unit, slice, segment).
size_t prefill_mfma32_workspace_bytes(int U, int N, int dp, int dv)
{
    (void)dp;
    return (dp32::entry_bytes(U, N, dv) + 255) / 256 * 256;
}

hipError_t launch_prefill_mfma32(const void *q, const void *k, const void *v, void *y, float *state,
                                 int has_init, int packed_state, void *workspace, int U, int N, int dp, int dv,
                                 hipStream_t s)
{
    // the kernels' flag word (has_init arrives with bit 2 set for numerator-only outputs)
    has_init = (has_init & 1) | (packed_state ? 2 : 0) | (has_init & 4);
    using namespace dp32;
    (void)dp;
    const int slices = dv / DVS;
    SegTable segs;
    const int G = make_segments(N, pick_segments(U, N, dv), segs);
    const uint16_t *q16 = (const uint16_t *)q, *k16 = (const uint16_t *)k, *v16 = (const uint16_t *)v;
    float *ws = static_cast<float *>(workspace);
    hipError_t e;
    if (has_init & 1) {
        hipLaunchKernelGGL((prefill_kernel<2>), dim3((unsigned)(U * slices)), dim3(NT), 0, s, q16, k16, v16,
                           (uint16_t *)y, state, has_init, ws, N, dv, segs, G);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (G > 1) {
        hipLaunchKernelGGL((prefill_kernel<1>), dim3((unsigned)(U * slices * (G - 1))), dim3(NT), 0, s, q16, k16,
                           v16, (uint16_t *)y, state, has_init, ws, N, dv, segs, G);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    hipLaunchKernelGGL((prefill_kernel<0>), dim3((unsigned)(U * slices * G)), dim3(NT), 0, s, q16, k16, v16,
                       (uint16_t *)y, state, has_init, ws, N, dv, segs, G);
    return hipGetLastError();
}

}  // namespace based
