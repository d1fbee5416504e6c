// Causal Taylor linear attention, chunked prefill on the gfx950 matrix cores (bf16 in, fp32
// accumulate), d' = 16.
//
// Chunked form of Sec. 4: inside a chunk of C = 64 tokens the masked quadratic product
// (1 + A + A^2/2 with A = Q K^T, exact closed form of Eq. 4), across chunks the running
// KV-state S (Eq. 3) read out with phi(Q) and updated with phi(K)^T V.  The expanded features
// are produced in registers in MFMA operand layout, pass through LDS once, and never reach HBM.
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
// The 153 rows are laid out as five tiles of 32 (160 rows): tile T < 4 holds delta = 2T (local rows
// 0..15, a = row) and delta = 2T + 1 (rows 16..31); tile 4 holds the 16 linear rows, the constant
// row (16), seven rows of padding and the eight rows of delta = 8 (24..31).
//
// Work split.  One workgroup per (unit, sequence segment): one CONSUMER wave per 32 columns of d_v
// (two at d_v = 64, four at 128) and four PRODUCER waves.  A consumer owns ALL 160 state rows of its
// 32 columns: five 32x32 fp32 accumulator tiles that stay in its registers for the whole segment (the
// paper keeps its 2nd-order state in registers for the same reason), and issues every matrix
// instruction for those columns: readout Y^T = S^T phi(Q)^T, intra-chunk Y^T += V^T P^T, update
// S += phi(K)^T V; then it normalises and stores its piece of y.  With the columns split this way
// nothing of one consumer's accumulators is needed by another: no partial outputs are exchanged.
// What the waves share is the operands, which do not depend on the column: each operand (32 x 16
// bf16, one kilobyte) is built ONCE per chunk by a producer, written to LDS in MFMA operand layout
// (16 bytes per lane), and read by every consumer with one 16-byte LDS load per lane, so that the
// vector-ALU cost of the feature map is paid once per workgroup.  The masked intra-chunk blocks P
// and the denominators are shared the same way.
//
// Pipeline.  The producers run one chunk ahead of the consumers: while the consumers multiply the
// operands of chunk t (LDS generation t % 2), the producers stage the rows of chunk t + 1 (fetched
// into registers during chunk t - 1), and build its operands into the other generation.  Per chunk
// there is one workgroup barrier (chunk t + 1's operands are visible, chunk t's are free) and one
// counter in LDS that the producer waves bump when their rows are staged and that only the waves
// building from those rows poll.
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
#include <type_traits>

namespace based {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int DP = 16;            // d'
constexpr int C = 64;             // chunk length (tokens)
constexpr int NTILE = 5;          // state tiles of 32 rows
constexpr int NSLAB = 2 * NTILE;  // feature slabs of 16 rows
constexpr float kCK = 0.84089641525371454303f;   // 2^(-1/4): (c k_a)(c k_b) = k_a k_b / sqrt(2)
constexpr float kCQ = 1.18920711500272106672f;   // 2^(+1/4): (c q_a)(c q_b) = sqrt(2) q_a q_b
constexpr float kHalfInvCQ = 0.42044820762685725f;   // 0.5 / kCQ

// LDS strides (elements)
constexpr int KTS_LD = C + 4;     // fp32 K^T rows
constexpr int KT_ROWS = DP + 3;   // c_k k_a (16 rows); valid / c_k; valid * c_k; zeros
constexpr int QS_LD = DP + 4;     // fp32 Q rows
constexpr int RB_LD = DP + 8;     // bf16 row-major Q and K rows as given (48-byte stride)
constexpr int YT_LD = 32 + 8;     // bf16 rows of a finished output tile on its way out (80-byte stride)

// Workspace entry (one segment's state in accumulator layout): six slots of 16 registers x 64 lanes
// per wave: slot 6c + T = tile T of the wave that owns columns 32c .. 32c+31, slot 6c + 5 = the
// moment tile (kept by wave 0 only; the others' sixth slot is never written and its contents are
// never used).  Within a slot: [r / 4][lane][r % 4], so one 16-byte access per lane is contiguous
// across the wave.
constexpr int WS_WAVE_SLOTS = 6;
constexpr size_t kSlotFloats = 16 * 64;
__host__ __device__ constexpr size_t entry_floats(int nc) { return (size_t)nc * WS_WAVE_SLOTS * kSlotFloats; }

template <int NC>
struct Lds {
    // the producers' own staging of the q and k rows of the chunk they are preparing
    float kts[KT_ROWS][KTS_LD];         // c_k * K^T, then the rows [valid / c_k], [valid * c_k], [0]
    float qs[C][QS_LD];                 // c_q * Q
    uint16_t qrow[C][RB_LD];            // Q rows, bf16 as given
    uint16_t krow[C][RB_LD];            // K rows, bf16 as given
    // everything the consumers read exists twice, indexed by the parity of the chunk: the producers fill
    // one generation while the consumers work on the other
    uint16_t vrow[2][C][32 * NC + 16];  // V rows, bf16 as given (operands are read transposed; the stride
                                        // leaves those reads free of bank conflicts)
    u32x4 phiq[2][2][NSLAB][64];        // phi(Q)^T operands: [parity][query tile][slab][lane]
    u32x4 phik[2][NTILE][4][64];        // phi(K)^T operands: [parity][state tile][16-token slab][lane]
    u32x4 pop[2][3][2][64];             // masked intra-chunk blocks as operands: [parity][block][slab][lane]
    float den[2][3][C];                 // per query: inter-chunk part; row sums of the blocks of key tile 0, 1
    uint16_t yt[NC][32][YT_LD];         // per consumer wave: a finished output tile on its way out
    unsigned staged;                    // producer waves that have staged their part, summed over the chunks so far
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
__device__ __forceinline__ u32x4 as_u32x4(bf16x8 w) { return __builtin_bit_cast(u32x4, w); }

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

// The rows of a chunk are staged by the producer waves only, and read by every wave that builds an
// operand from them.  That hand-over does not stop the whole workgroup: a producer wave that has finished
// its LDS writes adds one to a counter in LDS, and whoever needs the rows waits until the counter has
// reached the number of producer waves times the number of chunks staged so far.  (LDS operations of a
// wave complete in order, and the add is issued after the wave's own writes have completed.)
__device__ __forceinline__ void signal_staged(unsigned *counter, int lane)
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (lane == 0) __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void wait_staged(unsigned *counter, unsigned target)
{
    while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target)
        __builtin_amdgcn_s_sleep(1);
    asm volatile("" ::: "memory");
}

// MFMA instructions ignore the EXEC mask.  A branch on the wave's role is uniform across the wave
// but the compiler lowers it to lane masking and may drop the jump over a short masked block, in
// which case the other waves would execute the MFMAs inside it.  An inline-asm statement in the
// block makes the compiler keep the jump (it never runs inline asm with an empty EXEC mask).
__device__ __forceinline__ void role_guard() { asm volatile("; wave-role block: keep the execz branch"); }

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

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
// local row fl of tile T: T < 4: delta = 2T + fl / 16, a = fl % 16; T = 4: 0..15 linear, 16 constant,
// 24..31 the delta = 8 pairs
__device__ __forceinline__ CanonRows canon_rows(int T, int fl, bool packed_state)
{
    if (T < 4) {
        const int a = fl & 15;
        return canon_pair(a, (a + 2 * T + (fl >> 4)) & 15, packed_state);
    }
    if (fl < DP) return {1 + fl, 1 + fl};
    if (fl == DP) return {0, 0};
    if (fl >= 24) return canon_pair(fl - 24, fl - 16, packed_state);
    return {-1, -1};
}

// Workspace accesses that cross workgroups inside one launch.  Each XCD has its own L2, and memory
// written by a workgroup on one XCD is only guaranteed to be seen by another XCD's workgroups at a
// kernel boundary, unless the accesses are marked system-coherent (sc0 sc1: written through to, and
// read from, the memory side of the L2s).
// (A store of more than 64 bits reads its data registers a few cycles after it issues, and whatever
// overwrites them in the next two cycles corrupts the stored data.  The compiler keeps that distance for
// stores it emits itself but cannot see inside an asm statement, so the wait states are part of it.)
__device__ __forceinline__ void store16_coherent(float *p, const f32x4 &v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 2" : : "v"(p), "v"(v) : "memory");
}
// The six slots of one wave in one entry: all 24 loads are in flight at once and the wait sits in the
// same statement, so that every output register is valid as far as the compiler can tell.  p1, p3, p5
// point at the lane's 16 bytes of slots 1, 3, 5; the slot before each is reached with negative offsets.
__device__ __forceinline__ void load_wave_slots_coherent(const float *p1, const float *p3, const float *p5,
                                                         f32x4 (&t)[24])
{
    asm volatile(
        "global_load_dwordx4 %0, %24, off offset:-4096 sc0 sc1\n\t"
        "global_load_dwordx4 %1, %24, off offset:-3072 sc0 sc1\n\t"
        "global_load_dwordx4 %2, %24, off offset:-2048 sc0 sc1\n\t"
        "global_load_dwordx4 %3, %24, off offset:-1024 sc0 sc1\n\t"
        "global_load_dwordx4 %4, %24, off offset:0 sc0 sc1\n\t"
        "global_load_dwordx4 %5, %24, off offset:1024 sc0 sc1\n\t"
        "global_load_dwordx4 %6, %24, off offset:2048 sc0 sc1\n\t"
        "global_load_dwordx4 %7, %24, off offset:3072 sc0 sc1\n\t"
        "global_load_dwordx4 %8, %25, off offset:-4096 sc0 sc1\n\t"
        "global_load_dwordx4 %9, %25, off offset:-3072 sc0 sc1\n\t"
        "global_load_dwordx4 %10, %25, off offset:-2048 sc0 sc1\n\t"
        "global_load_dwordx4 %11, %25, off offset:-1024 sc0 sc1\n\t"
        "global_load_dwordx4 %12, %25, off offset:0 sc0 sc1\n\t"
        "global_load_dwordx4 %13, %25, off offset:1024 sc0 sc1\n\t"
        "global_load_dwordx4 %14, %25, off offset:2048 sc0 sc1\n\t"
        "global_load_dwordx4 %15, %25, off offset:3072 sc0 sc1\n\t"
        "global_load_dwordx4 %16, %26, off offset:-4096 sc0 sc1\n\t"
        "global_load_dwordx4 %17, %26, off offset:-3072 sc0 sc1\n\t"
        "global_load_dwordx4 %18, %26, off offset:-2048 sc0 sc1\n\t"
        "global_load_dwordx4 %19, %26, off offset:-1024 sc0 sc1\n\t"
        "global_load_dwordx4 %20, %26, off offset:0 sc0 sc1\n\t"
        "global_load_dwordx4 %21, %26, off offset:1024 sc0 sc1\n\t"
        "global_load_dwordx4 %22, %26, off offset:2048 sc0 sc1\n\t"
        "global_load_dwordx4 %23, %26, off offset:3072 sc0 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]),
          "=&v"(t[7]), "=&v"(t[8]), "=&v"(t[9]), "=&v"(t[10]), "=&v"(t[11]), "=&v"(t[12]), "=&v"(t[13]),
          "=&v"(t[14]), "=&v"(t[15]), "=&v"(t[16]), "=&v"(t[17]), "=&v"(t[18]), "=&v"(t[19]), "=&v"(t[20]),
          "=&v"(t[21]), "=&v"(t[22]), "=&v"(t[23])
        : "v"(p1), "v"(p3), "v"(p5)
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
// Increments and main pass run in ONE launch.  A main-pass workgroup of segment g > 0 waits (bounded)
// for the flags of the increments before it.  Flag word F[unit][p][g] == epoch tells the main-pass
// workgroup of segment g that entry p of this call is complete: every word has one writer and one
// reader, and the reader zeroes it once it has seen it, so the words are clear again when the launch
// ends (a replay of a captured launch, which repeats the same epoch, starts from cleared flags).
template <int NC, int MODE>
__device__ __forceinline__ void prefill_body(
    Lds<NC> &lds, const uint16_t *__restrict__ q, const uint16_t *__restrict__ k,
    const uint16_t *__restrict__ v, uint16_t *__restrict__ y, float *__restrict__ state, int has_init,
    float *__restrict__ ws, unsigned *__restrict__ flags, unsigned *__restrict__ status, int max_polls,
    unsigned epoch, int N, const SegTable &segs, int G, int seg, int u)
{
    constexpr int NPW = 4;            // producer waves
    constexpr int NP = 64 * NPW;      // producer threads
    constexpr int DV = 32 * NC;       // d_v
    constexpr int VR_LD = DV + 16;
    // has_init carries three flags: bit 0 an initial state is given, bit 1 the state buffer is packed,
    // bit 2 the outputs are the numerators alone (no division by the denominator)
    const bool packed_state = (has_init & 2) != 0;
    const bool numerator_only = (has_init & 4) != 0;
    has_init &= 1;
    const int tid = threadIdx.x;
    const int w = tid >> 6;
    const bool is_p = w >= NC;            // producer wave; else consumer wave (owns the state tiles)
    const int c = is_p ? w - NC : w;      // consumer: column tile (columns 32c .. 32c+31); producer: its role
    const int lane = tid & 63;
    const int g = lane >> 5, n = lane & 31;

    const int tok_begin = segs.begin[seg];
    const int tok_end = min(N, segs.begin[seg + 1]);
    const int n_chunks = (tok_end - tok_begin + C - 1) / C;

    const uint16_t *qu = q + (size_t)u * N * DP;
    const uint16_t *ku = k + (size_t)u * N * DP;
    const uint16_t *vu = v + (size_t)u * N * DV;
    uint16_t *yu = y + (size_t)u * N * DV;
    float *Su = state ? state + (size_t)u * (packed_state ? packed_state_stride(DP, DV) : state_stride(DP, DV))
                      : nullptr;
    float *zu = Su ? Su + (size_t)(packed_state ? packed_feature_dim(DP) : feature_dim(DP)) * DV : nullptr;
    float *ws_unit = ws ? ws + (size_t)u * G * entry_floats(NC) : nullptr;
    unsigned *flags_unit = flags ? flags + (size_t)u * G * G : nullptr;
    // this lane's 16 bytes of register group 0 of slot 0 of column tile c (producer 0 keeps the moment
    // tile, which travels in the sixth slot of column tile 0), inside an entry
    const size_t lane_off = (size_t)(is_p ? 0 : c) * WS_WAVE_SLOTS * kSlotFloats + (size_t)lane * 4;
    const bool holds_x = is_p && c == 0;

    if (MODE == 0 && G > 1 && seg > 0) {
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
    }

    // Intra-chunk block bb of the chunk whose rows are staged, into generation b: 0 = key tile 0 against
    // query tile 0, 1 = key tile 0 against query tile 1, 2 = key tile 1 against query tile 1 (0 and 2 are
    // cut by the diagonal).  P^T = mask(1 + A^T + A^T^2 / 2), A^T = K Q^T: lane (g, n) is query 32 qt + n,
    // register r is key 32 kt + 8 (r / 4) + 4 g + r % 4.  Keys past the end of the segment come after every
    // valid query and fall to the causal mask.  Built by the consumer waves (one block each), which wait
    // for the producers otherwise.
    auto build_block = [&](const int b, const int bb) {
        const int kt = bb == 2 ? 1 : 0, qt = bb == 0 ? 0 : 1;
        const bool diag = bb != 1;
        f32x16 P;
        zero16(P);
        const u32x4 kop = *reinterpret_cast<const u32x4 *>(&lds.krow[32 * kt + n][8 * g]);
        const u32x4 qop = *reinterpret_cast<const u32x4 *>(&lds.qrow[32 * qt + n][8 * g]);
        P = mfma(as_bf16x8(kop), as_bf16x8(qop), P);
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
        lds.pop[b][bb][0][lane] = as_u32x4(pack8_acc(P, 0));
        lds.pop[b][bb][1][lane] = as_u32x4(pack8_acc(P, 1));
        dsum += __shfl_xor(dsum, 32, 64);
        if (g == 0) lds.den[b][1 + kt][32 * qt + n] = dsum;
    };
    // which blocks a consumer builds: four consumers: c = 0..2 one each; two: 0 -> blocks 0 and 1, 1 -> block 2
    auto build_my_blocks = [&](const int b) {
        if (NC == 4) {
#pragma unroll
            for (int bb = 0; bb < 3; ++bb)
                if (c == bb) build_block(b, bb);
        }
    };

    if (MODE != 2 && tid == 0) lds.staged = 0u;   // ordered before its first use by the prologue's barriers
    if (!is_p) {
        // =================================== consumer waves =========================================
        f32x16 S[NTILE];       // the five state tiles of this wave's 32 columns
#pragma unroll
        for (int T = 0; T < NTILE; ++T) zero16(S[T]);

        if (MODE == 0) {
            // start of segment: initial state (entry 0, if any) plus the increments of earlier segments
            for (int p = has_init ? 0 : 1; p <= seg; ++p) {
                const float *e = ws_unit + (size_t)p * entry_floats(NC) + lane_off;
                f32x4 t[24];
                load_wave_slots_coherent(e + 1 * kSlotFloats, e + 3 * kSlotFloats, e + 5 * kSlotFloats, t);
#pragma unroll
                for (int T = 0; T < NTILE; ++T)
#pragma unroll
                    for (int r = 0; r < 16; ++r) S[T][r] += t[T * 4 + (r >> 2)][r & 3];
            }
        }
        if (MODE == 2) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
                const size_t col = (size_t)32 * c + n;
#pragma unroll
                for (int T = 0; T < NTILE; ++T) {
                    const CanonRows cr = canon_rows(T, fl, packed_state);
                    if (cr.r1 >= 0) S[T][r] = 0.5f * (Su[(size_t)cr.r1 * DV + col] + Su[(size_t)cr.r2 * DV + col]);
                }
            }
        }

        if (MODE != 2) {
            // V operand of an MFMA (lane (g, n): column 32 c + n at the 8 tokens of its k-slots, two runs of
            // 4 consecutive tokens starting at tok4 and tok4 + 8) from the row-major V rows: the transposing
            // LDS read.  In each group of 16 lanes, lane k supplies the address of 4 consecutive columns
            // (4 (k % 4) ..) of row k / 4 of the group's 16-column block and receives column k of that
            // block at the 4 rows.  The same registers serve as A operand (V^T, output product) and as B
            // operand (update).
            const int tr_kk = lane & 15, tr_grp = (lane >> 4) & 1;
            const uint16_t *tr_base = &lds.vrow[0][(tr_kk >> 2) + 4 * g][32 * c + 16 * tr_grp + 4 * (tr_kk & 3)];
            auto load_v = [&](int b, int ts) {   // tokens 16 ts + 4 g + {0..3, 8..11}
                const uint16_t *p = tr_base + (b * C + 16 * ts) * VR_LD;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p + 8 * VR_LD));
                s16x8 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) { o[i] = lo[i]; o[4 + i] = hi[i]; }
                return __builtin_bit_cast(bf16x8, o);
            };

            wg_sync();   // the producers have staged the first chunk
            if (MODE == 0) build_my_blocks(0);
            wg_sync();   // the operands of the first chunk are visible
            for (int t = 0; t < n_chunks; ++t) {
                const int b = t & 1;
                const int tok0 = tok_begin + C * t;
                bf16x8 vop[4];
#pragma unroll
                for (int ts = 0; ts < 4; ++ts) vop[ts] = load_v(b, ts);
                f32x16 Y[2];
                float dn[2][3];
                if (MODE == 0) {
                    // ---- readout: Y^T of query tile qt: lane (g, n) = query 32 qt + n, register r = column
                    // 32 c + 8 (r / 4) + 4 g + r % 4.  The bf16 copy of a state tile (a register-local
                    // conversion: accumulator registers 8 sl .. 8 sl + 7 are the k-slots of slab 2T + sl) is the
                    // A operand.  The LDS loads go out in groups, into registers of their own, ahead of the
                    // matrix instructions that consume them.
                    u32x4 oa[2][5], ob[2][5];
#pragma unroll
                    for (int sl = 0; sl < 5; ++sl)
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt) oa[qt][sl] = lds.phiq[b][qt][sl][lane];
#pragma unroll
                    for (int sl = 0; sl < 5; ++sl)
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt) ob[qt][sl] = lds.phiq[b][qt][5 + sl][lane];
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                        for (int d = 0; d < 3; ++d) dn[qt][d] = lds.den[b][d][32 * qt + n];
                    __builtin_amdgcn_sched_barrier(0);
                    zero16(Y[0]); zero16(Y[1]);
#pragma unroll
                    for (int sl = 0; sl < 5; ++sl) {
                        const bf16x8 sb = pack8_acc(S[sl >> 1], sl & 1);
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt) Y[qt] = mfma(sb, as_bf16x8(oa[qt][sl]), Y[qt]);
                    }
                    // the intra-chunk blocks, into the registers the first group has left
                    u32x4 op[3][2];
#pragma unroll
                    for (int bb = 0; bb < 3; ++bb)
#pragma unroll
                        for (int sl = 0; sl < 2; ++sl) op[bb][sl] = lds.pop[b][bb][sl][lane];
#pragma unroll
                    for (int sl = 5; sl < NSLAB; ++sl) {
                        const bf16x8 sb = pack8_acc(S[sl >> 1], sl & 1);
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt) Y[qt] = mfma(sb, as_bf16x8(ob[qt][sl - 5]), Y[qt]);
                    }
                    // intra-chunk: Y^T += V^T P^T over the key tiles at or before the query tile
#pragma unroll
                    for (int sl = 0; sl < 2; ++sl) {
                        Y[0] = mfma(vop[sl], as_bf16x8(op[0][sl]), Y[0]);
                        Y[1] = mfma(vop[sl], as_bf16x8(op[1][sl]), Y[1]);
                    }
#pragma unroll
                    for (int sl = 0; sl < 2; ++sl) Y[1] = mfma(vop[2 + sl], as_bf16x8(op[2][sl]), Y[1]);
                }
                if (MODE == 0 && NC == 4 && t + 1 < n_chunks) {
                    wait_staged(&lds.staged, (unsigned)(NPW * (t + 1)));   // the next chunk's rows are staged
                    build_my_blocks(b ^ 1);
                }

                // ---- update: S += phi(K)^T V over all 160 rows, with the normalisation and the store of
                // the outputs placed between the matrix instructions
                u32x4 ok[4][NTILE];
#pragma unroll
                for (int ts = 0; ts < 4; ++ts)
#pragma unroll
                    for (int T = 0; T < NTILE; ++T) ok[ts][T] = lds.phik[b][T][ts][lane];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
#pragma unroll
                    for (int ts = 2 * half; ts < 2 * half + 2; ++ts)
#pragma unroll
                        for (int T = 0; T < NTILE; ++T) S[T] = mfma(as_bf16x8(ok[ts][T]), vop[ts], S[T]);
                    if (MODE == 0) {
                        const int qt = half;
                        // normalise and turn the tile through LDS: a lane holds 8-byte pieces of its token's
                        // row, and stored directly those become 16-byte write requests that stall the memory
                        // pipeline; from LDS the tile leaves as 64-byte row segments, 16 rows a store.
                        const float inv = numerator_only ? 1.f : __builtin_amdgcn_rcpf(dn[qt][0] + dn[qt][1] + dn[qt][2]);
                        uint16_t *yt = &lds.yt[c][0][0];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            f32x4 o;
#pragma unroll
                            for (int i = 0; i < 4; ++i) o[i] = Y[qt][4 * j + i] * inv;
                            const bf16x4 hv = __builtin_convertvector(o, bf16x4);
                            *reinterpret_cast<u32x2 *>(yt + n * YT_LD + 8 * j + 4 * g) = __builtin_bit_cast(u32x2, hv);
                        }
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        uint16_t *yc = yu + (size_t)tok0 * DV;
                        u32x4 val[2];
                        uint32_t yoff[2];
#pragma unroll
                        for (int it = 0; it < 2; ++it) {
                            const int row = 16 * it + (lane >> 2), cc = lane & 3;
                            val[it] = *reinterpret_cast<const u32x4 *>(yt + row * YT_LD + 8 * cc);
                            yoff[it] = (uint32_t)(32 * qt + row) * (uint32_t)DV + (uint32_t)(32 * c + 8 * cc);
                        }
                        if (tok0 + C <= tok_end) {
#pragma unroll
                            for (int it = 0; it < 2; ++it) *reinterpret_cast<u32x4 *>(yc + yoff[it]) = val[it];
                        } else {
#pragma unroll
                            for (int it = 0; it < 2; ++it)
                                if (tok0 + 32 * qt + 16 * it + (lane >> 2) < tok_end) *reinterpret_cast<u32x4 *>(yc + yoff[it]) = val[it];
                        }
                        // the next tile overwrites this wave's staging only after these reads: LDS
                        // operations of one wave execute in order
                    }
                }
                wg_sync();   // the next chunk's operands are visible; this chunk's are free
            }
        }

        // ---- end of segment --------------------------------------------------------------------
        if (MODE != 0) {
            float *e = ws_unit + (size_t)(MODE == 1 ? 1 + seg : 0) * entry_floats(NC) + lane_off;
#pragma unroll
            for (int T = 0; T < NTILE; ++T)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4 o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = S[T][4 * j + i];
                    store16_coherent(e + (size_t)T * kSlotFloats + (size_t)j * 256, o);
                }
        } else if (Su && seg == G - 1) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
                const size_t col = (size_t)32 * c + n;
#pragma unroll
                for (int T = 0; T < NTILE; ++T) {
                    const CanonRows cr = canon_rows(T, fl, packed_state);
                    if (cr.r1 >= 0) {
                        Su[(size_t)cr.r1 * DV + col] = S[T][r];
                        if (cr.r2 != cr.r1) Su[(size_t)cr.r2 * DV + col] = S[T][r];
                    }
                }
            }
        }
    } else {
        // =================================== producer waves =========================================
        const int ptid = tid - 64 * NC;   // thread index among the producers
        f32x16 X;                      // producer 0: the moment tile M' = [k, 1]^T [k, 1]
        zero16(X);
        if (MODE == 0 && holds_x) {
            for (int p = has_init ? 0 : 1; p <= seg; ++p) {
                const float *e = ws_unit + (size_t)p * entry_floats(NC) + lane_off;
                f32x4 t[24];
                load_wave_slots_coherent(e + 1 * kSlotFloats, e + 3 * kSlotFloats, e + 5 * kSlotFloats, t);
#pragma unroll
                for (int r = 0; r < 16; ++r) X[r] += t[20 + (r >> 2)][r & 3];
            }
        }
        if (MODE == 2 && holds_x) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
                float m = 0.f;   // M'[fl][n]
                if (fl < DP && n < DP) m = zu[canon_pair(fl, n, packed_state).r1] * 1.41421356237309504880f;
                else if (fl == DP && n < DP) m = zu[1 + n];
                else if (fl < DP && n == DP) m = zu[1 + fl];
                else if (fl == DP && n == DP) m = zu[0];
                X[r] = m;
            }
        }

        if (MODE != 2) {
            // once: the zero row of K^T, and the row sums of a block that does not exist (key tile 1
            // against query tile 0)
            // (only the first 32 queries of den[.][2]: the other half belongs to block 2, whose builder does
            // not wait for this wave)
            if (ptid < C) lds.kts[DP + 2][ptid] = 0.f;
            if (ptid < 32) {
                lds.den[0][2][ptid] = 0.f;
                lds.den[1][2][ptid] = 0.f;
            }

            // ---- staging: global -> registers -> LDS --------------------------------------------
            // A chunk of V is one contiguous block of 64 rows x DV columns: 16-byte piece p = ptid + NP j
            // (j = 0..3) is row p / (DV / 8), columns 8 (p % (DV / 8)) ...  A chunk of K (and of Q) is 128
            // pieces: piece p holds elements 8 (p % 2) .. of token p / 2.  With four producer waves the
            // first two stage K and the other two Q; with two every thread stages one piece of each.
            constexpr int VPR = DV / 8;   // pieces per V row
            constexpr bool kBoth = false;
            constexpr int NVP = VPR * C / NP;   // V pieces per producer thread
            const int xp = ptid & 127;
            const bool is_k = kBoth || ptid < 128;
            const int x_tok = xp >> 1, x_h = xp & 1;
            u32x4 raw_k = {0u, 0u, 0u, 0u}, raw_q = {0u, 0u, 0u, 0u};   // four waves: raw_k is the thread's one piece
            u32x4 raw_v[NVP];
            // Loads are unconditional (rows past the end of the segment re-read its last row and are
            // zeroed when staged): a conditional load would have the compiler pre-zero its destination
            // registers, and before that write it waits for every memory operation still in flight.
            auto load_raw = [&](int tok0) {
                const int tok = min(tok0 + x_tok, tok_end - 1);
                if (kBoth) {
                    raw_k = *reinterpret_cast<const u32x4 *>(ku + (size_t)tok * DP + 8 * x_h);
                    if (MODE == 0) raw_q = *reinterpret_cast<const u32x4 *>(qu + (size_t)tok * DP + 8 * x_h);
                } else {
                    const uint16_t *src = (is_k || MODE != 0) ? ku : qu;   // increment pass: q is not needed
                    raw_k = *reinterpret_cast<const u32x4 *>(src + (size_t)tok * DP + 8 * x_h);
                }
#pragma unroll
                for (int j = 0; j < NVP; ++j) {
                    const int p = ptid + NP * j;
                    const int row = min(tok0 + p / VPR, tok_end - 1);
                    raw_v[j] = *reinterpret_cast<const u32x4 *>(vu + (size_t)row * DV + 8 * (p % VPR));
                }
            };
            auto stage_k = [&](u32x4 raw, bool valid) {
                const u32x4 zero4 = {0u, 0u, 0u, 0u};
                if (!valid) raw = zero4;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    lds.kts[8 * x_h + 2 * i][x_tok] = bf16lo(raw[i]) * kCK;
                    lds.kts[8 * x_h + 2 * i + 1][x_tok] = bf16hi(raw[i]) * kCK;
                }
                *reinterpret_cast<u32x4 *>(&lds.krow[x_tok][8 * x_h]) = raw;
                if (x_h == 0) {
                    lds.kts[DP][x_tok] = valid ? 1.f / kCK : 0.f;
                    lds.kts[DP + 1][x_tok] = valid ? kCK : 0.f;
                }
            };
            auto stage_q = [&](u32x4 raw) {
                f32x4 lo, hi;
                lo[0] = bf16lo(raw[0]) * kCQ; lo[1] = bf16hi(raw[0]) * kCQ;
                lo[2] = bf16lo(raw[1]) * kCQ; lo[3] = bf16hi(raw[1]) * kCQ;
                hi[0] = bf16lo(raw[2]) * kCQ; hi[1] = bf16hi(raw[2]) * kCQ;
                hi[2] = bf16lo(raw[3]) * kCQ; hi[3] = bf16hi(raw[3]) * kCQ;
                *reinterpret_cast<f32x4 *>(&lds.qs[x_tok][8 * x_h]) = lo;
                *reinterpret_cast<f32x4 *>(&lds.qs[x_tok][8 * x_h + 4]) = hi;
                *reinterpret_cast<u32x4 *>(&lds.qrow[x_tok][8 * x_h]) = raw;
            };
            auto stage = [&](int tok0, int b) {
                const bool valid = tok0 + x_tok < tok_end;
                if (kBoth) {
                    stage_k(raw_k, valid);
                    if (MODE == 0) stage_q(raw_q);
                } else if (is_k) {
                    stage_k(raw_k, valid);
                } else if (MODE == 0) {
                    stage_q(raw_k);
                }
                const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int j = 0; j < NVP; ++j) {
                    const int p = ptid + NP * j;
                    const int row = p / VPR;
                    *reinterpret_cast<u32x4 *>(&lds.vrow[b][row][8 * (p % VPR)]) = tok0 + row < tok_end ? raw_v[j] : zero4;
                }
            };

            // ---- builders of the shared operands (b: the generation they write) ------------------
            // phi(Q)^T operands of query tile qt, all ten slabs: lane (g, n) is query 32 qt + n; k-slot
            // (jj, i) of slab s is feature row 16 s + 8 jj + 4 g + i.  xr[j] = c_q q[(4g + j) % 16] is the
            // lane's query row rotated by 4g, so that the "a side" of k-slot (jj, i) is xr[8 jj + i] and the
            // "b side" of delta is xr[(8 jj + i + delta) % 16]: every product is between two registers known
            // at compile time.
            auto build_phiq = [&](const int b, const int qt) {
                float xr[16];
                const float *row = lds.qs[32 * qt + n];
                f32x4 t[4];
#pragma unroll
                for (int m = 0; m < 4; ++m) t[m] = *reinterpret_cast<const f32x4 *>(row + ((4 * g + 4 * m) & 15));
                // slab 8: the linear rows; the operand is q itself, as given
                const uint16_t *p = &lds.qrow[32 * qt + n][4 * g];
                const u32x2 ra = *reinterpret_cast<const u32x2 *>(p);
                const u32x2 rb = *reinterpret_cast<const u32x2 *>(p + 8);
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int i = 0; i < 4; ++i) xr[4 * m + i] = t[m][i];
#pragma unroll
                for (int s = 0; s < 8; ++s) {   // pair slabs: delta = s
                    float pr[8];
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int a = 8 * jj + i;
                            const float av = s == 0 ? xr[a] * 0.5f : xr[a];   // delta = 0: x_a^2 / sqrt(2)
                            pr[4 * jj + i] = av * xr[(a + s) & 15];
                        }
                    lds.phiq[b][qt][s][lane] = as_u32x4(pack8(pr));
                }
                {
                    u32x4 o; o[0] = ra[0]; o[1] = ra[1]; o[2] = rb[0]; o[3] = rb[1];
                    lds.phiq[b][qt][8][lane] = o;
                }
                {   // slab 9: the constant row (k-slot 0 of g = 0 = row 16 of the tile), padding, and the
                    // delta = 8 rows (k-slots 4 + i = row 24 + 4g + i: sqrt(2) q_a q_(a+8), a = 4g + i)
                    float pr[8];
                    pr[0] = g == 0 ? 1.f : 0.f; pr[1] = 0.f; pr[2] = 0.f; pr[3] = 0.f;
#pragma unroll
                    for (int i = 0; i < 4; ++i) pr[4 + i] = xr[i] * xr[8 + i];
                    lds.phiq[b][qt][9][lane] = as_u32x4(pack8(pr));
                }
            };
            // phi(K)^T operands of token slab ts, all five state tiles: lane (g, n) is feature row n of a
            // tile, its k-slots are the tokens 16 ts + 4 g + {0..3, 8..11}.  Every row is a product of two
            // rows of the staged K^T: pair rows k_a k_b / sqrt(2); linear rows (c_k k_a)(valid / c_k); the
            // constant row (valid c_k)(valid / c_k); padding rows 0 * 0.  (c_k k_a / c_k differs from k_a by
            // fp32 rounding only, far below half a bf16 step, so the conversion returns k_a exactly.)  The
            // "a" row of the four pair tiles is the same (a = n % 16), so a slab costs 14 LDS loads, all
            // issued before the products.
            const float *kt_a03 = &lds.kts[n & 15][4 * g];
            const float *kt_a4 = &lds.kts[n < DP ? n : (n == DP ? DP + 1 : (n < 24 ? DP + 2 : n - 24))][4 * g];
            const float *kt_b[NTILE];
#pragma unroll
            for (int T = 0; T < 4; ++T) kt_b[T] = &lds.kts[((n & 15) + 2 * T + (n >> 4)) & 15][4 * g];
            kt_b[4] = &lds.kts[n < DP ? DP : (n == DP ? DP : (n < 24 ? DP + 2 : n - 16))][4 * g];
            // (NTS token slabs at a time: all their LDS loads go out before the first product)
            auto build_phik_n = [&](const int b, const int ts0, auto nts_tag) {
                constexpr int NTS = decltype(nts_tag)::value;
                f32x4 a03[NTS][2], a4[NTS][2], kb[NTS][NTILE][2];
#pragma unroll
                for (int s2 = 0; s2 < NTS; ++s2)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int off = 16 * (ts0 + s2) + 8 * h;
                        a03[s2][h] = *reinterpret_cast<const f32x4 *>(kt_a03 + off);
                        a4[s2][h] = *reinterpret_cast<const f32x4 *>(kt_a4 + off);
#pragma unroll
                        for (int T = 0; T < NTILE; ++T) kb[s2][T][h] = *reinterpret_cast<const f32x4 *>(kt_b[T] + off);
                    }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s2 = 0; s2 < NTS; ++s2)
#pragma unroll
                    for (int T = 0; T < NTILE; ++T) {
                        float pr[8];
#pragma unroll
                        for (int h = 0; h < 2; ++h)
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                pr[4 * h + i] = (T < 4 ? a03[s2][h][i] : a4[s2][h][i]) * kb[s2][T][h][i];
                        lds.phik[b][T][ts0 + s2][lane] = as_u32x4(pack8(pr));
                    }
            };
            auto build_phik = [&](const int b, const int ts) { build_phik_n(b, ts, std::integral_constant<int, 1>{}); };
            auto build_phik2 = [&](const int b, const int ts) { build_phik_n(b, ts, std::integral_constant<int, 2>{}); };
            // Inter-chunk denominators of both query tiles from the moments: count + q.z1 + q^T M q / 2.
            auto build_den = [&](const int b) {
                f32x4 a0[2], a1[2];
                u32x2 ra[2], rb[2];
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    const float *row = lds.qs[32 * qt + n];
                    a0[qt] = *reinterpret_cast<const f32x4 *>(row + 4 * g);
                    a1[qt] = *reinterpret_cast<const f32x4 *>(row + 8 + 4 * g);
                    const uint16_t *p = &lds.qrow[32 * qt + n][4 * g];
                    ra[qt] = *reinterpret_cast<const u32x2 *>(p);
                    rb[qt] = *reinterpret_cast<const u32x2 *>(p + 8);
                }
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
                f32x16 T[2];
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    u32x4 o; o[0] = ra[qt][0]; o[1] = ra[qt][1]; o[2] = rb[qt][0]; o[3] = rb[qt][1];
                    zero16(T[qt]);
                    T[qt] = mfma(mhi, as_bf16x8(o), T[qt]);
                    T[qt] = mfma(mlo, as_bf16x8(o), T[qt]);
                }
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    float d2 = 0.f;
                    // row of T[e] = 8 (e / 4) + 4 g + e % 4
#pragma unroll
                    for (int e = 0; e < 4; ++e) d2 = fmaf(T[qt][e], a0[qt][e], d2);
#pragma unroll
                    for (int e = 0; e < 4; ++e) d2 = fmaf(T[qt][4 + e], a1[qt][e], d2);
                    const float d = fmaf(d2, kHalfInvCQ, T[qt][8]);   // T[8]: row 16 = q.z1 on g = 0, zero on g = 1
                    const float tot = d + __shfl_xor(d, 32, 64) + cnt_prev;
                    if (g == 0) lds.den[b][0][32 * qt + n] = tot;
                }
            };
            // The producers' share of the operands of one chunk, into generation b (the intra-chunk blocks
            // are built by the consumers, which have the time).  Four producer waves: 0 = denominators; 1 =
            // phi(Q) of both query tiles; 2 = phi(K) of token slabs 0, 1; 3 = phi(K) of token slabs 2, 3.
            // Two: 0 = denominators, phi(Q); 1 = phi(K).  Increment pass: phi(K) only.
            auto build = [&](const int b) {
                if (MODE == 0) {
                    if (c == 0) {
                        role_guard();
                        build_den(b);
                        build_phiq(b, 0);
                    } else if (c == 1) {
                        build_phiq(b, 1);
                        if (NC == 2) build_block(b, 1);
                    } else if (c == 2) {
                        build_phik2(b, 0);
                        if (NC == 2) build_block(b, 0);
                    } else {
                        build_phik2(b, 2);
                        if (NC == 2) build_block(b, 2);
                    }
                } else {
#pragma unroll
                    for (int ts = 0; ts < 4; ++ts)
                        if (c == ts) build_phik(b, ts);
                }
            };

            // ---- the producers' loop: one chunk ahead of the consumers -----------------------------
            load_raw(tok_begin);
            stage(tok_begin, 0);
            if (n_chunks > 1) load_raw(tok_begin + C);
            wg_sync();   // the first chunk's rows are staged
            build(0);
            wg_sync();   // the first chunk's operands are visible
            for (int t = 0; t < n_chunks; ++t) {
                const int b = t & 1;
                const int tok_next = tok_begin + C * (t + 1);
                const bool has_next = t + 1 < n_chunks;
                if (has_next) {
                    stage(tok_next, b ^ 1);
                    signal_staged(&lds.staged, lane);
                }
                if (t + 2 < n_chunks) load_raw(tok_next + C);   // two chunks ahead of the consumers
                if (has_next) wait_staged(&lds.staged, (unsigned)(NPW * (t + 1)));   // all of the next chunk's rows
                if (holds_x) {
                    // M' += K'^T K' of the chunk the consumers are working on (the operand of tile 4 carries k
                    // as given in rows 0..15 and the valid flag in row 16); the denominators of the next chunk
                    // need it
                    role_guard();
#pragma unroll
                    for (int ts = 0; ts < 4; ++ts) {
                        const bf16x8 e = as_bf16x8(lds.phik[b][NTILE - 1][ts][lane]);
                        X = mfma(e, e, X);
                    }
                }
                if (has_next) build(b ^ 1);
                wg_sync();   // the next chunk's operands are visible
            }
        }

        // ---- end of segment: the moments ----------------------------------------------------------
        if (holds_x) {
            if (MODE != 0) {
                float *e = ws_unit + (size_t)(MODE == 1 ? 1 + seg : 0) * entry_floats(NC) + lane_off;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4 o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = X[4 * j + i];
                    store16_coherent(e + (size_t)5 * kSlotFloats + (size_t)j * 256, o);
                }
            } else if (Su && seg == G - 1) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int fl = 8 * (r >> 2) + 4 * g + (r & 3);
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
    if (MODE == 1) {
        // the entry has reached memory (the stores are written through) before the flag is raised
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        // entry 1 + seg is read by the main-pass workgroups of segments 1 + seg .. G - 1
        if (tid >= 1 + seg && tid < G)
            __hip_atomic_store(flags_unit + (1 + seg) * G + tid, epoch, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// Grid: first the (G - 1) increments of every unit, then the main-pass workgroups segment by segment
// (all segment-0 workgroups first: they depend on nothing and fill the slots the increment
// workgroups leave free).
template <int NC>
__global__ __launch_bounds__(64 * (NC + 4), 2) void prefill_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ y, float *__restrict__ state, int has_init, float *__restrict__ ws,
    unsigned *__restrict__ flags, unsigned *__restrict__ status, int max_polls, unsigned epoch, int N,
    SegTable segs, int G, int U)
{
    __shared__ __align__(16) Lds<NC> lds;
    const int n_inc = U * (G - 1);
    int bid = blockIdx.x;
    if (bid < n_inc) {
        prefill_body<NC, 1>(lds, q, k, v, y, state, has_init, ws, flags, status, max_polls, epoch, N, segs, G,
                            bid % (G - 1), bid / (G - 1));
    } else {
        bid -= n_inc;
        prefill_body<NC, 0>(lds, q, k, v, y, state, has_init, ws, flags, status, max_polls, epoch, N, segs, G,
                            bid / U, bid % U);
    }
}

// The caller's initial state into entry 0 of every unit.
template <int NC>
__global__ __launch_bounds__(64 * (NC + 4), 2) void prefill_mfma_import_kernel(
    float *__restrict__ state, int has_init, float *__restrict__ ws, int N, SegTable segs, int G)
{
    __shared__ __align__(16) Lds<NC> lds;
    prefill_body<NC, 2>(lds, nullptr, nullptr, nullptr, nullptr, state, has_init, ws, nullptr, nullptr, 0, 0u, N,
                        segs, G, 0, blockIdx.x);
}

// ---- host side ----------------------------------------------------------------------------------
namespace {

// Segments per sequence: enough main-pass workgroups to fill the chip once (one workgroup per CU fits),
// but segments of at least 512 tokens so that the state increments stay small next to q, k, v, y.
// More segments than that only add increment work and workspace traffic (360M-shaped prefill, 128 units:
// 4 segments 72 us, 3 segments 71 us, 2 segments 60.5 us).
int pick_segments(int U, int N, int dv)
{
    const long want = 256;
    int G = (int)((want + U - 1) / U);
    const int max_by_len = N / 512;
    if (G > max_by_len) G = max_by_len;
    if (G > kMaxSegments) G = kMaxSegments;
    if (G < 1) G = 1;
    return G;
}

// Segment boundaries.  The main pass starts segment g by summing g workspace entries and the last
// segment also writes the final state, so later segments get fewer chunks, so that the main-pass
// workgroups, which run side by side, end close together.
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

// Workspace: G entries per unit, then G x G ready-flag words per unit (256-byte aligned).
size_t ws_entry_bytes(int U, int N, int dv)
{
    return (size_t)U * pick_segments(U, N, dv) * entry_floats(dv / 32) * sizeof(float);
}
size_t ws_flag_bytes(int U, int N, int dv)
{
    const size_t Gmax = (size_t)pick_segments(U, N, dv);
    const size_t flags = (size_t)U * Gmax * Gmax * sizeof(unsigned);
    return (flags + 255) / 256 * 256;
}

template <int NC>
hipError_t launch(const uint16_t *q, const uint16_t *k, const uint16_t *v, uint16_t *y, float *state, int flags_word,
                  void *workspace, unsigned *status, int U, int N, hipStream_t s)
{
    constexpr int dv = 32 * NC;
    SegTable segs;
    // a smaller G only uses a prefix of the workspace that was sized for pick_segments()
    const int Gmax = pick_segments(U, N, dv);
    const int G = make_segments(N, Gmax, segs);
    // what the kernels index must lie inside what the workspace was sized for
    if (G < 1 || G > Gmax || segs.begin[G] < N) return hipErrorInvalidValue;
    if ((long long)U * (2 * G - 1) >= (1ll << 31)) return hipErrorInvalidValue;
    float *ws = static_cast<float *>(workspace);
    unsigned *flags = reinterpret_cast<unsigned *>((char *)workspace + ws_entry_bytes(U, N, dv));
    hipError_t e;
    if (flags_word & 1) {
        hipLaunchKernelGGL((prefill_mfma_import_kernel<NC>), dim3((unsigned)U), dim3(64 * (NC + 4)), 0, s, state,
                           flags_word, ws, N, segs, G);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    // Every call raises its flags to a value no earlier call used: the flag words of a workspace
    // that has never been used hold whatever was in that memory.
    static std::atomic<unsigned> calls{0};
    const unsigned epoch = 0x5EED0000u + calls.fetch_add(1u) + 1u;
    hipLaunchKernelGGL((prefill_mfma_kernel<NC>), dim3((unsigned)(U * (2 * G - 1))), dim3(64 * (NC + 4)), 0, s, q, k, v,
                       y, state, flags_word, ws, flags, status, g_flag_poll_limit.load(), epoch, N, segs, G, U);
    return hipGetLastError();
}

}  // namespace

bool prefill_mfma_supported(int dp, int dv, int dtype)
{
    return dtype == BASED_BF16 && dp == DP && (dv == 64 || dv == 128);
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
    (void)dp;
    // the kernels' flag word (has_init arrives with bit 2 set for numerator-only outputs)
    const int flags_word = (has_init & 1) | (packed_state ? 2 : 0) | (has_init & 4);
    const uint16_t *q16 = (const uint16_t *)q, *k16 = (const uint16_t *)k, *v16 = (const uint16_t *)v;
    if (dv == 128)
        return launch<4>(q16, k16, v16, (uint16_t *)y, state, flags_word, workspace, status, U, N, s);
    return launch<2>(q16, k16, v16, (uint16_t *)y, state, flags_word, workspace, status, U, N, s);
}

}  // namespace based
