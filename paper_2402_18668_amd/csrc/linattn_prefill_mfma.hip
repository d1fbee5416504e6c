// Causal Taylor linear attention, chunked prefill on the gfx950 matrix cores (bf16 in, fp32
// accumulate), d' = 16.
//
// Chunked form of Sec. 4: inside a chunk of C = 64 tokens the masked quadratic product
// (1 + A + A^2/2 with A = Q K^T, exact closed form of Eq. 4), across chunks the running
// KV-state S (Eq. 3) read out with phi(Q) and updated with phi(K)^T V.  The expanded features
// are produced in registers straight into MFMA operand layout and never stored anywhere.
//
// Symmetric packing of the 2nd-order block.  The state rows (a, b) and (b, a) of Eq. 4 are equal
// (x_a x_b = x_b x_a), so only one row per unordered pair is carried: row (a, delta) stands for
// the pair {a, (a + delta) mod 16} with delta = 0 .. 7 for every a (128 rows) and delta = 8 for
// a < 8 (8 rows), 136 rows instead of 256.  The k side builds x_a x_b / sqrt(2) (the canonical
// state row); the q side builds sqrt(2) x_a x_b for delta != 0 (the pair counts twice in the sum
// over ordered pairs) and x_a^2 / sqrt(2) for delta = 0.  The cyclic enumeration keeps the
// operand construction regular: for a fixed delta the 16 features are x (.) rotate(x, delta).
// The final state is written in the canonical layout (both rows of a pair); an initial state is
// read as its symmetric part, which is all the readout can see.
//
// Work split.  One workgroup of four waves per (unit, 64-column slice of d_v, sequence segment).
// Wave w owns the 32 rows delta in {2w, 2w+1} (its "main tile"), whose 32x32 fp32 state tiles
// stay in its registers for the whole segment.  The remaining work is spread over the waves:
// the "extra tile" [x_0..x_15, 1, 0 x 7, the 8 rows of delta = 8] is split by column tile between
// waves 0 and 1; wave 2 owns the moments that give the denominator; the three blocks of the
// intra-chunk product go to waves 0, 1 (the two cut by the diagonal) and 3.  Per chunk each wave produces a
// partial Y^T over its feature rows; the partials are exchanged through LDS and wave w finishes
// the 32x32 output tile (query tile w / 2, column tile w % 2).  Two workgroups (eight waves)
// share a CU, so one wave's vector-ALU work (feature products, conversions) overlaps another's
// MFMAs.
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
// Long sequences / few units: the sequence is cut into G segments.  Update-only workgroups compute
// each segment's state increment, and the main-pass workgroup of a segment starts from the sum of
// the increments before it.  Both kinds run in one launch: the increment workgroups come first in
// the grid, the main-pass workgroups wait (bounded) on per-entry ready flags in the workspace.
#include "common.h"

#include <atomic>

namespace based {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int DP = 16;            // d'
constexpr int C = 64;             // chunk length (tokens)
constexpr int NW = 4;             // waves per workgroup
constexpr int NT = NW * 64;
constexpr int DVS = 64;           // d_v columns per workgroup
constexpr float kCK = 0.84089641525371454303f;   // 2^(-1/4): (c k_a)(c k_b) = k_a k_b / sqrt(2)
constexpr float kCQ = 1.18920711500272106672f;   // 2^(+1/4): (c q_a)(c q_b) = sqrt(2) q_a q_b
constexpr float kHalfInvCQ = 0.42044820762685725f;   // 0.5 / kCQ

// LDS strides (elements)
constexpr int KTS_LD = C + 4;     // fp32 K^T rows
constexpr int VR_LD = DVS + 16;   // bf16 V rows (160-byte stride: the transposing reads below are conflict-free)
constexpr int QS_LD = DP + 4;     // fp32 Q rows
constexpr int RB_LD = DP + 8;     // bf16 row-major Q rows (48-byte stride)
constexpr int KR_LD = 32 + 16;    // bf16 row-major extended K rows (96-byte stride)
constexpr int YT_LD = 32 + 8;     // bf16 rows of a finished output tile on its way out (80-byte stride)

// Workspace entry (one segment's state in accumulator layout): 11 slots of 16 registers x 64
// lanes: slot 2w + c2 = main tile of wave w, column tile c2; slots 8, 9 = extra tile (column
// tiles 0, 1); slot 10 = moment tile.  Within a slot: [r / 4][lane][r % 4], so that one 16-byte
// access per lane is contiguous across the wave.
constexpr int WS_SLOTS = 11;
constexpr size_t kWsEntryFloats = (size_t)WS_SLOTS * 16 * 64;

struct Stage {
    float kts[DP][KTS_LD];        // c_k * K^T
    uint16_t vrow[C][VR_LD];      // V rows, bf16 as given (operands are read transposed)
    float qs[C][QS_LD];           // c_q * Q
    uint16_t qrow[C][RB_LD];      // Q rows, bf16 as given
    uint16_t krow[C][KR_LD];      // extended K rows: [k_0..k_15 as given, 1 (0 past the end), 0 x 7,
                                  // k_a k_(a+8) / sqrt(2) for a < 8]: read row-wise by the intra-chunk
                                  // block and transposed as the operand of the extra tile and the moments
};

struct Lds {
    Stage st;
    float xbuf[NW][3][4][64][4];  // partial Y^T tiles: [destination wave][sender slot][r / 4][lane][r % 4]
    float den_inter[C];           // count + phi(q).z over earlier chunks (wave 1)
    float den_intra[2][C];        // row sums of the masked intra-chunk block (waves 2 and 3)
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
__device__ __forceinline__ void role_guard() { asm volatile("; wave-role block: keep the execz branch"); }

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ size_t ws_slot_off(int slot, int j, int lane)
{
    return (((size_t)slot * 4 + j) * 64 + lane) * 4;
}

// Canonical state rows (Eq. 4 order: row 0 constant, 1 + a linear, 1 + d' + a d' + b the pair
// (a, b)) of a packed row.  A pair row has two canonical rows (equal for delta = 0).
// With packed_state the buffer is the packed layout (one row per unordered pair), where a pair has a
// single row and the constant and linear rows sit at the same indices.
struct CanonRows { int r1, r2; };   // r1 < 0: the packed row is padding
__device__ __forceinline__ CanonRows canon_pair(int a, int b, bool packed_state)
{
    if (packed_state) {
        const int r = packed_pair_row(DP, min(a, b), max(a, b));
        return {r, r};
    }
    return {1 + DP + a * DP + b, 1 + DP + b * DP + a};
}
// local row fl of the main tile of wave w: delta = 2w + fl / 16, a = fl % 16
__device__ __forceinline__ CanonRows canon_rows_main(int w, int fl, bool packed_state)
{
    const int a = fl & 15;
    return canon_pair(a, (a + 2 * w + (fl >> 4)) & 15, packed_state);
}
// local row fl of the extra tile: 0..15 linear, 16 constant, 24..31 the delta = 8 pairs
__device__ __forceinline__ CanonRows canon_rows_extra(int fl, bool packed_state)
{
    if (fl < DP) return {1 + fl, 1 + fl};
    if (fl == DP) return {0, 0};
    if (fl >= 24) return canon_pair(fl - 24, fl - 16, packed_state);
    return {-1, -1};
}

// Workspace accesses that cross workgroups inside one launch.  Each XCD has its own L2, and memory
// written by a workgroup on one XCD is only guaranteed to be seen by another XCD's workgroups at a
// kernel boundary, unless the accesses are marked system-coherent (sc0 sc1: written through to, and
// read from, the memory side of the L2s).  All loads of an entry are in flight at once and the wait
// sits in the same statement, so that every output register is valid as far as the compiler can tell.
__device__ __forceinline__ void store16_coherent(float *p, const f32x4 &v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void load_entry_coherent(const float *p0, const float *p1, const float *p2,
                                                    f32x4 (&t)[12])
{
    asm volatile(
        "global_load_dwordx4 %0, %12, off offset:0 sc0 sc1\n\t"
        "global_load_dwordx4 %1, %12, off offset:1024 sc0 sc1\n\t"
        "global_load_dwordx4 %2, %12, off offset:2048 sc0 sc1\n\t"
        "global_load_dwordx4 %3, %12, off offset:3072 sc0 sc1\n\t"
        "global_load_dwordx4 %4, %13, off offset:0 sc0 sc1\n\t"
        "global_load_dwordx4 %5, %13, off offset:1024 sc0 sc1\n\t"
        "global_load_dwordx4 %6, %13, off offset:2048 sc0 sc1\n\t"
        "global_load_dwordx4 %7, %13, off offset:3072 sc0 sc1\n\t"
        "global_load_dwordx4 %8, %14, off offset:0 sc0 sc1\n\t"
        "global_load_dwordx4 %9, %14, off offset:1024 sc0 sc1\n\t"
        "global_load_dwordx4 %10, %14, off offset:2048 sc0 sc1\n\t"
        "global_load_dwordx4 %11, %14, off offset:3072 sc0 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]),
          "=&v"(t[7]), "=&v"(t[8]), "=&v"(t[9]), "=&v"(t[10]), "=&v"(t[11])
        : "v"(p0), "v"(p1), "v"(p2)
        : "memory");
}

// Default upper bound on the polls of a segment-ready flag (each poll sleeps ~0.25 us): a workgroup
// never waits forever, whatever happens to the workgroup it waits for.  A workgroup that gives up
// stores the call's epoch into the workspace's status word (a plain vector store) and carries on, so
// that every workgroup of the launch exits normally; its outputs are then wrong, and
// based_prefill_status reports the launch as failed.
constexpr int kMaxFlagPolls = 1 << 20;
std::atomic<int> g_flag_poll_limit{kMaxFlagPolls};

constexpr int kMaxSegments = 16;
// first token of each segment (multiples of the chunk length), and the end of the last one
struct SegTable { int begin[kMaxSegments + 1]; };

}  // namespace

// MODE 0: full prefill of the segment (readout + update); starts from the sum of workspace entries.
// MODE 1: state increment of the segment only (update GEMMs), written to workspace entry 1 + seg.
// MODE 2: the caller's initial state, converted to accumulator layout, written to entry 0.
// The main pass never reads the caller's state buffer, so writing the final state back into it
// cannot race with another workgroup still starting up.
// FUSED: the increments and the main pass run in ONE launch.  Increment workgroups come first in the
// grid and wait for nothing; a main-pass workgroup of segment g > 0 waits (bounded) for the flags
// of the increments before it.  Flag word F[unit slice][p][g] == epoch tells the main-pass workgroup
// of segment g that entry p of this call is complete: every word has one writer and one reader, and
// the reader zeroes it once it has seen it, so the words are clear again when the launch ends (a
// replay of a captured launch, which repeats the same epoch, starts from cleared flags).
template <int MODE, bool FUSED>
__device__ __forceinline__ void prefill_body(
    Lds &lds, const uint16_t *__restrict__ q, const uint16_t *__restrict__ k,
    const uint16_t *__restrict__ v, uint16_t *__restrict__ y, float *__restrict__ state, int has_init,
    float *__restrict__ ws, unsigned *__restrict__ flags, unsigned *__restrict__ status, int max_polls,
    unsigned epoch, int N, int dv, const SegTable &segs, int G, int seg, int slice, int u)
{
    // has_init carries two flags: bit 0 an initial state is given, bit 1 the state buffer is packed
    const bool packed_state = (has_init & 2) != 0;
    has_init &= 1;
    const int tid = threadIdx.x;
    const int w = tid >> 6;   // wave index: owns the main tile delta in {2w, 2w+1}
    const int lane = tid & 63;
    const int g = lane >> 5, n = lane & 31;

    const int slices = dv / DVS;
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
    float *ws_unit = ws ? ws + ((size_t)(u * slices + slice) * G) * kWsEntryFloats : nullptr;
    unsigned *flags_unit = flags ? flags + (size_t)(u * slices + slice) * G * G : nullptr;

    // ---- accumulators -------------------------------------------------------------------------
    f32x16 S[2];           // main tile [c2]
    f32x16 X;              // waves 0, 1: column tile w of the extra tile; wave 2: the moment tile
                           // M' = [k, 1]^T [k, 1]; unused by wave 3
    zero16(S[0]); zero16(S[1]);
    zero16(X);

    if (MODE == 0) {
        // start of segment: initial state (entry 0, if any) plus the increments of earlier segments.
        // Slots 2w, 2w+1, and for waves 0 .. 2 their extra tile (wave 3 re-reads a main slot).
        // The loads of entry p + 1 are issued before entry p is added up (they are unconditional:
        // past the last entry the last one is fetched again and dropped), so the entries stream in
        // back to back instead of costing one trip to memory each.
        const int x0 = w < 3 ? 8 + w : 2 * w;
        const size_t so[3] = {ws_slot_off(2 * w + 0, 0, lane), ws_slot_off(2 * w + 1, 0, lane),
                              ws_slot_off(x0, 0, lane)};
        auto add_in = [&](const f32x4 (&t)[12]) {
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[c2][r] += t[c2 * 4 + (r >> 2)][r & 3];
            if (w < 3) {
#pragma unroll
                for (int r = 0; r < 16; ++r) X[r] += t[2 * 4 + (r >> 2)][r & 3];
            }
        };
        const int p0 = has_init ? 0 : 1;
        if (FUSED) {
            // wait for the increments of this call (entry 0 comes from an earlier launch)
            if (tid == 0) {
                bool gave_up = false;
                for (int p = 1; p <= seg; ++p) {
                    unsigned *f = flags_unit + p * G + seg;
                    int polls = 0;
                    while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != epoch) {
                        if (polls++ >= max_polls) { gave_up = true; break; }
                        __builtin_amdgcn_s_sleep(8);
                    }
                    __hip_atomic_store(f, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                }
                // sticky: stays set until based_prefill_status has reported it
                if (gave_up) __hip_atomic_store(status, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            __syncthreads();
            for (int p = p0; p <= seg; ++p) {
                const float *e = ws_unit + (size_t)p * kWsEntryFloats;
                f32x4 t[12];
                load_entry_coherent(e + so[0], e + so[1], e + so[2], t);
                add_in(t);
            }
        } else {
            auto fetch = [&](int p, f32x4 (&t)[12]) {
                const float *e = ws_unit + (size_t)min(p, seg) * kWsEntryFloats;
#pragma unroll
                for (int sl = 0; sl < 3; ++sl)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        t[sl * 4 + j] = *reinterpret_cast<const f32x4 *>(e + so[sl] + (size_t)j * 256);
            };
            if (p0 <= seg) {
                f32x4 ta[12], tb[12];
                fetch(p0, ta);
                for (int p = p0; p <= seg; p += 2) {
                    fetch(p + 1, tb);
                    add_in(ta);
                    fetch(p + 2, ta);
                    if (p + 1 <= seg) add_in(tb);
                }
            }
        }
    }
    if (MODE == 2) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
            const CanonRows cm = canon_rows_main(w, fl, packed_state);
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2) {
                const size_t col = (size_t)col0 + 32 * c2 + n;
                S[c2][r] = 0.5f * (Su[(size_t)cm.r1 * dv + col] + Su[(size_t)cm.r2 * dv + col]);
            }
            if (w < 2) {
                const CanonRows cx = canon_rows_extra(fl, packed_state);
                if (cx.r1 >= 0) {
                    const size_t col = (size_t)col0 + 32 * w + n;
                    X[r] = 0.5f * (Su[(size_t)cx.r1 * dv + col] + Su[(size_t)cx.r2 * dv + col]);
                }
            } else if (w == 2) {
                float m = 0.f;   // M'[fl][n]
                if (fl < DP && n < DP) m = zu[canon_pair(fl, n, packed_state).r1] * 1.41421356237309504880f;
                else if (fl == DP && n < DP) m = zu[1 + n];
                else if (fl < DP && n == DP) m = zu[1 + fl];
                else if (fl == DP && n == DP) m = zu[0];
                X[r] = m;
            }
        }
    }

    // zero the unused half of den_intra[1] once
    if (tid < C) lds.den_intra[1][tid] = 0.f;

    // ---- staging: global -> registers -> LDS ----------------------------------------------------
    // Thread (s_tok, s_q) stages, of token s_tok: elements 4h .. 4h+3 and 8+4h .. 8+4h+3 (h = s_q % 2)
    // of the K row (waves 0, 1) or of the Q row (waves 2, 3), and a quarter of the V row.  Holding
    // elements a and a + 8 together lets the K threads build the delta = 8 feature rows here.
    const int s_tok = tid & 63, s_q = tid >> 6, s_h = s_q & 1;
    u32x2 raw_x[2];        // the two 8-byte pieces of the K or Q row
    u32x4 raw_v[2];
    // Loads are unconditional (rows past the end of the segment re-read its last row and are zeroed
    // when staged): a conditional load would have the compiler pre-zero its destination registers,
    // and before that write it waits for every memory operation still in flight, stores included.
    auto load_raw = [&](int tok0) {
        const int tok = min(tok0 + s_tok, tok_end - 1);
        const uint16_t *xc = (s_q < 2 ? ku : qu) + (size_t)tok * DP + 4 * s_h;
        const uint16_t *vc = vu + (size_t)tok * dv + 16 * s_q;
        if (MODE == 0 || s_q < 2) {
#pragma unroll
            for (int j = 0; j < 2; ++j) raw_x[j] = *reinterpret_cast<const u32x2 *>(xc + 8 * j);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) raw_v[j] = *reinterpret_cast<const u32x4 *>(vc + 8 * j);
    };
    auto stage = [&](int tok0) {
        Stage &st = lds.st;
        if (tok0 + s_tok >= tok_end) {
            const u32x2 zero2 = {0u, 0u};
            const u32x4 zero4 = {0u, 0u, 0u, 0u};
            raw_x[0] = zero2; raw_x[1] = zero2; raw_v[0] = zero4; raw_v[1] = zero4;
        }
        if (s_q < 2) {
            float kf[2][4];   // c_k * k: [j][i] = element 8 j + 4 h + i
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const uint32_t wd = raw_x[j][i];
                    const int a = 8 * j + 4 * s_h + 2 * i;
                    kf[j][2 * i] = bf16lo(wd) * kCK;
                    kf[j][2 * i + 1] = bf16hi(wd) * kCK;
                    st.kts[a][s_tok] = kf[j][2 * i];
                    st.kts[a + 1][s_tok] = kf[j][2 * i + 1];
                }
                *reinterpret_cast<u32x2 *>(&st.krow[s_tok][8 * j + 4 * s_h]) = raw_x[j];
            }
            f32x4 pr;
#pragma unroll
            for (int i = 0; i < 4; ++i) pr[i] = kf[0][i] * kf[1][i];
            const u32x2 pb = __builtin_bit_cast(u32x2, __builtin_convertvector(pr, bf16x4));
            *reinterpret_cast<u32x2 *>(&st.krow[s_tok][24 + 4 * s_h]) = pb;
            if (s_q == 0) {
                u32x4 one = {0u, 0u, 0u, 0u};
                if (tok0 + s_tok < tok_end) one[0] = 0x3F80u;
                *reinterpret_cast<u32x4 *>(&st.krow[s_tok][16]) = one;
            }
        } else if (MODE == 0) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                f32x4 qv;
                qv[0] = bf16lo(raw_x[j][0]) * kCQ; qv[1] = bf16hi(raw_x[j][0]) * kCQ;
                qv[2] = bf16lo(raw_x[j][1]) * kCQ; qv[3] = bf16hi(raw_x[j][1]) * kCQ;
                *reinterpret_cast<f32x4 *>(&st.qs[s_tok][8 * j + 4 * s_h]) = qv;
                *reinterpret_cast<u32x2 *>(&st.qrow[s_tok][8 * j + 4 * s_h]) = raw_x[j];
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) *reinterpret_cast<u32x4 *>(&st.vrow[s_tok][16 * s_q + 8 * j]) = raw_v[j];
    };

    // V^T operand of an MFMA (lane (g, n): column 32 c2 + n at the 8 tokens of its k-slots, two runs
    // of 4 consecutive tokens starting at tok4 and tok4 + 8) from the row-major V rows: the
    // transposing LDS read.  In each group of 16 lanes, lane k supplies the address of 4 consecutive
    // columns (4 (k % 4) ..) of row k / 4 of the group's 16-column block and receives column k of
    // that block at the 4 rows.
    const int tr_kk = lane & 15, tr_grp = (lane >> 4) & 1;
    const uint16_t *tr_base = &lds.st.vrow[tr_kk >> 2][16 * tr_grp + 4 * (tr_kk & 3)];
    const uint16_t *tr_kbase = &lds.st.krow[tr_kk >> 2][16 * tr_grp + 4 * (tr_kk & 3)];
    auto load_vt = [&](int tok4, int c2, s16x4 &a, s16x4 &b) {
        const uint16_t *p = tr_base + tok4 * VR_LD + 32 * c2;
        a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
        b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p + 8 * VR_LD));
    };
    auto join_vt = [](s16x4 a, s16x4 b) {
        s16x8 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[i] = a[i]; o[4 + i] = b[i]; }
        return __builtin_bit_cast(bf16x8, o);
    };

    // Pipeline: the rows of chunk c+1 are fetched from global memory into registers at the top of
    // chunk c and written to LDS at its bottom, so their latency hides under the whole chunk.
    if (MODE != 2) {
        load_raw(tok_begin);
        stage(tok_begin);
    }
    for (int tok0 = tok_begin; MODE != 2 && tok0 < tok_end; tok0 += C) {
        const Stage &st = lds.st;
        wg_sync();   // this chunk's staging is visible
        const bool more = tok0 + C < tok_end;
        if (more) load_raw(tok0 + C);   // a whole chunk ahead: consumed by stage() at the bottom

        // The finished tile of this wave, (query tile w / 2, column tile w % 2): its own partial, to
        // which the other waves' partials are added while the update phase runs.
        f32x4 acc[4];
        float inv = 0.f;
        if (MODE == 0) {
            // =============================== readout ============================================
            // One query tile (32 tokens) at a time, so that only two partial output tiles are live:
            // Y^T [c2]: lane (g, n) = query 32 qt + n, register r = column within column tile c2.
            f32x16 Yown;      // this wave's partial of the tile it finishes (query tile w / 2, column tile w % 2)
            zero16(Yown);
            // bf16 copies of the state tiles: operands of the readout, [slab][c2]
            bf16x8 Sb[2][2];
#pragma unroll
            for (int sl = 0; sl < 2; ++sl)
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) Sb[sl][c2] = pack8_acc(S[c2], sl);
            const float diag_w = w == 0 ? 0.5f : 1.f;   // delta = 0 (wave 0, slab 0): x_a^2 / sqrt(2)
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                f32x16 Y[2];
                zero16(Y[0]); zero16(Y[1]);

                // This lane's query row, rotated: qa[j] = c_q q[(4g + j) % 16] for j = 0..3, 8..11 (the
                // "a side": k-slot (jj, i) is a = 8 jj + 4 g + i) and qr[j] = c_q q[(4g + 2w + j) % 16]
                // (the "b side" of delta = 2w + s: b = a + delta is qr[(8 jj + i + s) % 16]).
                float qa[8], qr[16];
                {
                    const float *row = st.qs[32 * qt + n];
                    const f32x4 a0 = *reinterpret_cast<const f32x4 *>(row + 4 * g);
                    const f32x4 a1 = *reinterpret_cast<const f32x4 *>(row + 8 + 4 * g);
#pragma unroll
                    for (int i = 0; i < 4; ++i) { qa[i] = a0[i]; qa[4 + i] = a1[i]; }
                    const int rot = 4 * g + 2 * w;
#pragma unroll
                    for (int m = 0; m < 8; ++m) {
                        if (m == 3 || m == 7) continue;   // qr[6], qr[7], qr[14], qr[15] are never used
                        const f32x2 pp = *reinterpret_cast<const f32x2 *>(row + ((rot + 2 * m) & 15));
                        qr[2 * m] = pp[0];
                        qr[2 * m + 1] = pp[1];
                    }
                }

                // inter-chunk: Y^T += S^T phi(Q)^T over this wave's feature rows
#pragma unroll
                for (int sl = 0; sl < 2; ++sl) {
                    float pr[8];
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float av = sl == 0 ? qa[4 * jj + i] * diag_w : qa[4 * jj + i];
                            pr[4 * jj + i] = av * qr[(8 * jj + i + sl) & 15];
                        }
                    const bf16x8 phiq = pack8(pr);
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2) Y[c2] = mfma(Sb[sl][c2], phiq, Y[c2]);
                }

                // q pieces of this lane's query: elements 4g .. 4g+3 and 8+4g .. 8+4g+3 (bf16, as given)
                auto load_qb = [&]() {
                    const uint16_t *p = &st.qrow[32 * qt + n][4 * g];
                    const u32x2 a = *reinterpret_cast<const u32x2 *>(p);
                    const u32x2 b = *reinterpret_cast<const u32x2 *>(p + 8);
                    u32x4 o; o[0] = a[0]; o[1] = a[1]; o[2] = b[0]; o[3] = b[1];
                    return as_bf16x8(o);
                };
                if (w < 2) {
                    role_guard();
                    // extra tile, column tile w.  Slab 0: the 1st-order rows (the operand is q itself).
                    // Slab 1: the constant row (k-slot 0 of g = 0 = local row 16) and the delta = 8 rows
                    // (k-slots 4 + i = local row 24 + 4g + i: sqrt(2) q_a q_(a+8), a = 4g + i)
                    const bf16x8 qbo = load_qb();
                    float pr[8];
                    pr[0] = g == 0 ? 1.f : 0.f; pr[1] = 0.f; pr[2] = 0.f; pr[3] = 0.f;
#pragma unroll
                    for (int i = 0; i < 4; ++i) pr[4 + i] = qa[i] * qa[4 + i];
                    const bf16x8 hi = pack8(pr);
                    const bf16x8 xlo = pack8_acc(X, 0), xhi = pack8_acc(X, 1);
                    if (w == 0) {
                        role_guard();
                        Y[0] = mfma(xlo, qbo, Y[0]);
                        Y[0] = mfma(xhi, hi, Y[0]);
                    } else {
                        role_guard();
                        Y[1] = mfma(xlo, qbo, Y[1]);
                        Y[1] = mfma(xhi, hi, Y[1]);
                    }
                } else if (w == 2) {
                    role_guard();
                    const bf16x8 qbo = load_qb();
                    // ---- inter-chunk denominator from the moments: count + q.z1 + q^T M q / 2 ----
                    float mres[8];
                    const bf16x8 mhi = pack8_acc(X, 0);
                    {
                        const u32x4 hb = __builtin_bit_cast(u32x4, mhi);
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            mres[2 * i] = X[2 * i] - bf16lo(hb[i]);
                            mres[2 * i + 1] = X[2 * i + 1] - bf16hi(hb[i]);
                        }
                    }
                    const bf16x8 mlo = pack8(mres);
                    const float cnt_prev = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(X[8]), 16));
                    f32x16 T;
                    zero16(T);
                    T = mfma(mhi, qbo, T);
                    T = mfma(mlo, qbo, T);
                    float d2 = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) d2 = fmaf(T[e], qa[e], d2);   // row of T[e] = 8 (e / 4) + 4 g + e % 4
                    const float d = fmaf(d2, kHalfInvCQ, T[8]);   // T[8]: row 16 = q.z1 on g = 0, zero on g = 1
                    const float tot = d + __shfl_xor(d, 32, 64) + cnt_prev;
                    if (g == 0) lds.den_inter[32 * qt + n] = tot;
                }
                // ---- intra-chunk block: P^T = mask(1 + A^T + A^T^2 / 2), Y^T += V^T P^T ----------
                // wave 0: key tile 0 against query tile 0; wave 1: key tile 1 against query tile 1 (both
                // cut by the diagonal); wave 3: key tile 0 against query tile 1
                if (qt == 0 ? w == 0 : (w == 1 || w == 3)) {
                    role_guard();
                    const int kt = w == 1 ? 1 : 0;
                    const bool diag = w != 3;
                    bf16x8 vk[2][2];   // V^T operands of key tile kt: [s][c2]
#pragma unroll
                    for (int s = 0; s < 2; ++s)
#pragma unroll
                        for (int c2 = 0; c2 < 2; ++c2) {
                            s16x4 a, b;
                            load_vt(32 * kt + 16 * s + 4 * g, c2, a, b);
                            vk[s][c2] = join_vt(a, b);
                        }
                    f32x16 P;
                    zero16(P);
                    {   // rows keys (K tile kt), columns queries (Q tile qt), contraction over d'
                        const u32x4 kop = *reinterpret_cast<const u32x4 *>(&st.krow[32 * kt + n][8 * g]);
                        const u32x4 qop = *reinterpret_cast<const u32x4 *>(&st.qrow[32 * qt + n][8 * g]);
                        P = mfma(as_bf16x8(kop), as_bf16x8(qop), P);
                    }
                    float dsum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float x = P[r];
                        float pv = fmaf(x, fmaf(x, 0.5f, 1.f), 1.f);
                        const int key = 8 * (r >> 2) + 4 * g + (r & 3);
                        pv = (!diag || key <= n) ? pv : 0.f;
                        P[r] = pv;
                        dsum += pv;
                    }
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const bf16x8 pb = pack8_acc(P, s);
#pragma unroll
                        for (int c2 = 0; c2 < 2; ++c2) Y[c2] = mfma(vk[s][c2], pb, Y[c2]);
                    }
                    dsum += __shfl_xor(dsum, 32, 64);
                    if (g == 0) lds.den_intra[kt][32 * qt + n] = dsum;
                }

                // partial tiles of this query tile go to the waves that finish them
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) {
                    const int d = 2 * qt + c2;
                    if (d == w) {
                        Yown = Y[c2];
                    } else {
                        const int slot = ((w - d) & 3) - 1;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            f32x4 o;
#pragma unroll
                            for (int i = 0; i < 4; ++i) o[i] = Y[c2][4 * j + i];
                            *reinterpret_cast<f32x4 *>(&lds.xbuf[d][slot][j][lane][0]) = o;
                        }
                    }
                }
            }
            wg_sync();
            {
                const int qi = 32 * (w >> 1) + n;
                inv = 1.f / (lds.den_inter[qi] + lds.den_intra[0][qi] + lds.den_intra[1][qi]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[j][i] = Yown[4 * j + i];
            }
        }

        // =================================== update =============================================
        // S += phi(K)^T V over this wave's feature rows; lane (g, n): feature row n of the tile
        {
            // main tile: row n is the pair a = n % 16, b = (a + 2w + n / 16) % 16
            const int arow = n & 15, brow = (arow + 2 * w + (n >> 4)) & 15;
            // LDS operands of one step (16 tokens: slab s of key tile kt).  The operands of step i + 1
            // are requested before step i is worked on, so their latency hides under its arithmetic.
            struct StepOps {
                s16x4 va[2], vb[2];   // V^T operands [c2]: column 32 c2 + n, the two runs of 4 tokens
                f32x4 ka0, ka1, kb0, kb1;
                s16x4 ea, eb;         // [k_0..k_15, 1, 0 x 7, delta = 8 rows]^T operand (extra tile, moments)
            };
            auto load_step = [&](int i, StepOps &o) {
                const int tcol = 16 * i + 4 * g;   // first token of this lane's k-slots
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) load_vt(tcol, c2, o.va[c2], o.vb[c2]);
                o.ka0 = *reinterpret_cast<const f32x4 *>(&st.kts[arow][tcol]);
                o.ka1 = *reinterpret_cast<const f32x4 *>(&st.kts[arow][tcol + 8]);
                o.kb0 = *reinterpret_cast<const f32x4 *>(&st.kts[brow][tcol]);
                o.kb1 = *reinterpret_cast<const f32x4 *>(&st.kts[brow][tcol + 8]);
                const uint16_t *pe = tr_kbase + tcol * KR_LD;
                o.ea = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)pe);
                o.eb = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(pe + 8 * KR_LD));
            };
            auto work_step = [&](const StepOps &o) {
                bf16x8 vk[2];
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) vk[c2] = join_vt(o.va[c2], o.vb[c2]);
                float pr[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) { pr[i] = o.ka0[i] * o.kb0[i]; pr[4 + i] = o.ka1[i] * o.kb1[i]; }
                const bf16x8 phik = pack8(pr);
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) S[c2] = mfma(phik, vk[c2], S[c2]);
                if (w < 3) {
                    role_guard();
                    const bf16x8 kk = join_vt(o.ea, o.eb);
                    if (w == 0) {
                        role_guard();
                        X = mfma(kk, vk[0], X);
                    } else if (w == 1) {
                        role_guard();
                        X = mfma(kk, vk[1], X);
                    } else {
                        role_guard();
                        X = mfma(kk, kk, X);
                    }
                }
            };
            // The other waves' partial output tiles are collected a quarter per step, so that these
            // LDS reads (the largest block of LDS traffic in a chunk) run underneath the MFMAs
            // instead of in a burst of all waves at once after the barrier.
            f32x4 xr[3];
            auto fetch_partials = [&](int j) {
                if (MODE == 0) {
#pragma unroll
                    for (int sl = 0; sl < 3; ++sl)
                        xr[sl] = *reinterpret_cast<const f32x4 *>(&lds.xbuf[w][sl][j][lane][0]);
                }
            };
            auto add_partials = [&](int j) {
                if (MODE == 0) {
#pragma unroll
                    for (int sl = 0; sl < 3; ++sl)
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[j][i] += xr[sl][i];
                }
            };
            StepOps oa, ob;
            load_step(0, oa);
            load_step(1, ob);
            fetch_partials(0);
            work_step(oa);
            add_partials(0);
            load_step(2, oa);
            fetch_partials(1);
            work_step(ob);
            add_partials(1);
            load_step(3, ob);
            fetch_partials(2);
            work_step(oa);
            add_partials(2);
            fetch_partials(3);
            work_step(ob);
            add_partials(3);
        }
        if (MODE == 0) {
            // Normalise and turn the tile through LDS (the wave's own exchange slot, which it has
            // finished reading): a lane holds 8-byte pieces of its token's row, and stored directly
            // those become 16-byte write requests that stall the memory pipeline; from LDS the tile
            // leaves as 64-byte row segments, 16 rows a store.
            const int qt = w >> 1, c2 = w & 1;
            uint16_t *yt = reinterpret_cast<uint16_t *>(&lds.xbuf[w][0][0][0][0]);   // [32][YT_LD] bf16
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[j][i] *= inv;
                const bf16x4 hv = __builtin_convertvector(acc[j], bf16x4);
                *reinterpret_cast<u32x2 *>(yt + n * YT_LD + 8 * j + 4 * g) = __builtin_bit_cast(u32x2, hv);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            uint16_t *yc = yu + (size_t)tok0 * dv;
            // A full chunk stores without a per-lane condition: stores that are certain to be
            // issued can be counted, so the later wait for the prefetched rows (issued before
            // them; the counter retires in order) does not have to wait for the stores as well.
            u32x4 val[2];
            uint32_t yoff[2];
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = 16 * it + (lane >> 2), c = lane & 3;
                val[it] = *reinterpret_cast<const u32x4 *>(yt + row * YT_LD + 8 * c);
                yoff[it] = (uint32_t)(32 * qt + row) * (uint32_t)dv + (uint32_t)(32 * c2 + 8 * c);
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
                if (FUSED) store16_coherent(e + ws_slot_off(slot, j, lane), o);
                else *reinterpret_cast<f32x4 *>(e + ws_slot_off(slot, j, lane)) = o;
            }
        };
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) put(2 * w + c2, S[c2]);
        if (w < 3) put(8 + w, X);
        if (FUSED) {
            // the entry has reached memory (the stores are written through) before the flag is raised
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            // entry 1 + seg is read by the main-pass workgroups of segments 1 + seg .. G - 1
            if (tid >= 1 + seg && tid < G)
                __hip_atomic_store(flags_unit + (1 + seg) * G + tid, epoch, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_SYSTEM);
        }
    } else if (Su && seg == G - 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
            const CanonRows cm = canon_rows_main(w, fl, packed_state);
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2) {
                const size_t col = (size_t)col0 + 32 * c2 + n;
                Su[(size_t)cm.r1 * dv + col] = S[c2][r];
                if (cm.r2 != cm.r1) Su[(size_t)cm.r2 * dv + col] = S[c2][r];
            }
            if (w < 2) {
                const CanonRows cx = canon_rows_extra(fl, packed_state);
                if (cx.r1 >= 0) {
                    const size_t col = (size_t)col0 + 32 * w + n;
                    Su[(size_t)cx.r1 * dv + col] = X[r];
                    if (cx.r2 != cx.r1) Su[(size_t)cx.r2 * dv + col] = X[r];
                }
            } else if (w == 2 && slice == 0) {
                const float m = X[r];
                if (fl < DP && n < DP) {
                    if (!packed_state || fl <= n) zu[canon_pair(fl, n, packed_state).r1] = m * kRsqrt2;
                }
                else if (fl == DP && n < DP) zu[1 + n] = m;
                else if (fl == DP && n == DP) zu[0] = m;
            }
        }
    }
}

template <int MODE>
__global__ __launch_bounds__(NT, 2) void prefill_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ y, float *__restrict__ state, int has_init, float *__restrict__ ws, int N,
    int dv, SegTable segs, int G)
{
    __shared__ __align__(16) Lds lds;
    const int slices = dv / DVS;
    const int gseg = MODE == 1 ? G - 1 : (MODE == 2 ? 1 : G);   // segments this launch covers
    int bid = blockIdx.x;
    const int seg = bid % gseg; bid /= gseg;
    prefill_body<MODE, false>(lds, q, k, v, y, state, has_init, ws, nullptr, nullptr, 0, 0u, N, dv, segs, G,
                              seg, bid % slices, bid / slices);
}

// Increments and main pass in one launch.  Grid: first the (G - 1) increments of every unit slice,
// then the main-pass workgroups segment by segment (all segment-0 workgroups first: they depend
// on nothing and fill the slots the increment workgroups leave free).
__global__ __launch_bounds__(NT, 2) void prefill_mfma_fused_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ y, float *__restrict__ state, int has_init, float *__restrict__ ws,
    unsigned *__restrict__ flags, unsigned *__restrict__ status, int max_polls, unsigned epoch, int N, int dv,
    SegTable segs, int G, int groups)
{
    __shared__ __align__(16) Lds lds;
    const int slices = dv / DVS;
    const int n_inc = groups * (G - 1);
    int bid = blockIdx.x;
    if (bid < n_inc) {
        const int seg = bid % (G - 1); bid /= (G - 1);
        prefill_body<1, true>(lds, q, k, v, y, state, has_init, ws, flags, status, max_polls, epoch, N, dv,
                              segs, G, seg, bid % slices, bid / slices);
    } else {
        bid -= n_inc;
        const int seg = bid / groups; bid %= groups;
        prefill_body<0, true>(lds, q, k, v, y, state, has_init, ws, flags, status, max_polls, epoch, N, dv,
                              segs, G, seg, bid % slices, bid / slices);
    }
}

// ---- host side ----------------------------------------------------------------------------------
namespace {

// Segments per sequence: enough workgroups to put two on every CU of the chip, but segments
// of at least 512 tokens so that the state increments stay small next to q, k, v, y.
int pick_segments(int U, int N, int dv)
{
    const long groups = (long)U * (dv / DVS);
    const long want = 512;
    int G = (int)((want + groups - 1) / groups);
    const int max_by_len = N / 512;
    if (G > max_by_len) G = max_by_len;
    if (G > kMaxSegments) G = kMaxSegments;
    if (G < 1) G = 1;
    return G;
}

// Segment boundaries.  The main pass starts segment g by summing g workspace entries (about 0.6
// of a chunk's time each) and the last segment also writes the final state, so later segments
// get fewer chunks, so that the main-pass workgroups, which run side by side, end close together.
// Returns the number of segments actually used (a short sequence may leave trailing ones empty).
int make_segments(int N, int G, SegTable &t)
{
    const int T = (N + C - 1) / C;   // chunks
    if (G > T) G = T;
    int len[kMaxSegments];
    int sum = 0;
    for (int g = 0; g < G; ++g) {
        float off = 0.6f * (0.5f * (G - 1) - g);
        if (g == G - 1 && G > 1) off -= 0.5f;
        len[g] = T / G + (int)(off >= 0.f ? off + 0.5f : off - 0.5f);
        if (len[g] < 1) len[g] = 1;
        sum += len[g];
    }
    // hand the rounding remainder to (or take it from) the early segments, one chunk at a time
    for (int g = 0; sum != T; g = (g + 1) % G) {
        if (sum < T) { ++len[g]; ++sum; }
        else if (len[g] > 1) { --len[g]; --sum; }
    }
    int pos = 0;
    for (int g = 0; g < G; ++g) { t.begin[g] = pos * C; pos += len[g]; }
    for (int g = G; g <= kMaxSegments; ++g) t.begin[g] = pos * C;
    return G;
}

}  // namespace

bool prefill_mfma_supported(int dp, int dv, int dtype)
{
    return dtype == BASED_BF16 && dp == DP && (dv == 64 || dv == 128);
}

// Workspace: G entries per unit slice, then G x G ready-flag words per unit slice (256-byte aligned).
static size_t ws_entry_bytes(int U, int N, int dv)
{
    return (size_t)U * (dv / DVS) * pick_segments(U, N, dv) * kWsEntryFloats * sizeof(float);
}
static size_t ws_flag_bytes(int U, int N, int dv)
{
    const size_t Gmax = (size_t)pick_segments(U, N, dv);
    const size_t flags = (size_t)U * (dv / DVS) * Gmax * Gmax * sizeof(unsigned);
    return (flags + 255) / 256 * 256;
}

size_t prefill_mfma_workspace_bytes(int U, int N, int dp, int dv)
{
    (void)dp;
    return ws_entry_bytes(U, N, dv) + ws_flag_bytes(U, N, dv);
}

void prefill_mfma_flags_region(int U, int N, int dp, int dv, size_t *offset, size_t *bytes)
{
    (void)dp;
    *offset = ws_entry_bytes(U, N, dv);
    *bytes = ws_flag_bytes(U, N, dv);
}

void prefill_mfma_set_poll_limit(int polls) { g_flag_poll_limit.store(polls < 0 ? kMaxFlagPolls : polls); }

hipError_t launch_prefill_mfma(const void *q, const void *k, const void *v, void *y, float *state,
                               int has_init, int packed_state, void *workspace, unsigned *status, int U, int N,
                               int dp, int dv, hipStream_t s)
{
    has_init = (has_init ? 1 : 0) | (packed_state ? 2 : 0);   // the kernels' flag word
    (void)dp;
    const int slices = dv / DVS;
    SegTable segs;
    // a smaller G only uses a prefix of the workspace that was sized for pick_segments()
    const int G = make_segments(N, pick_segments(U, N, dv), segs);
    const uint16_t *q16 = (const uint16_t *)q, *k16 = (const uint16_t *)k, *v16 = (const uint16_t *)v;
    hipError_t e;
    if (has_init & 1) {
        hipLaunchKernelGGL((prefill_mfma_kernel<2>), dim3((unsigned)(U * slices)), dim3(NT), 0, s, q16, k16,
                           v16, (uint16_t *)y, state, has_init, (float *)workspace, N, dv, segs, G);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (G > 1) {
        // Every call raises its flags to a value no earlier call used: the flag words of a workspace
        // that has never been used hold whatever was in that memory.
        static std::atomic<unsigned> calls{0};
        const unsigned epoch = 0x5EED0000u + calls.fetch_add(1u) + 1u;
        unsigned *flags = reinterpret_cast<unsigned *>((char *)workspace + ws_entry_bytes(U, N, dv));
        const int groups = U * slices;
        hipLaunchKernelGGL(prefill_mfma_fused_kernel, dim3((unsigned)(groups * (2 * G - 1))), dim3(NT), 0, s,
                           q16, k16, v16, (uint16_t *)y, state, has_init, (float *)workspace, flags, status,
                           g_flag_poll_limit.load(), epoch, N, dv, segs, G, groups);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((prefill_mfma_kernel<0>), dim3((unsigned)(U * slices * G)), dim3(NT), 0, s, q16, k16,
                       v16, (uint16_t *)y, state, has_init, (float *)workspace, N, dv, segs, G);
    return hipGetLastError();
}

}  // namespace based
