// Sliding-window causal softmax attention over whole sequences (Sec. 3.2 restricting Eq. 1) on
// the gfx950 matrix cores: bf16 in, fp32 scores / softmax / accumulation.
//
// Work split.  One workgroup of four waves per (unit, segment of the sequence) walks its segment
// in steps of 128 queries; each wave owns one tile of 32 queries of the step and walks the
// w / 32 + 1 key tiles that overlap its window.
//
// Staging.  The w + 128 key and value rows a step can see sit in an LDS ring.  Each step
// overwrites the 128 oldest rows with its 128 new ones, which were fetched into registers during
// the previous step, so every row is read from global memory once per segment, with fully
// coalesced row-major loads, and its latency hides under the arithmetic.  (Fetching K per query
// tile instead multiplies the L2 traffic by w / 32 + 1.)  The Q tile of the next step is
// prefetched the same way.
//
// Operands.  K and Q tiles are MFMA operands exactly as they lie in memory: a lane's 8 k-slots
// are 16 contiguous bytes of its row.  The operand of P.V needs 8 keys of one column per lane,
// which the transposing LDS read (ds_read_b64_tr_b16) delivers from the row-major V rows.
//
// Softmax.  Scores are computed transposed (S^T = K Q^T: lane = query, registers = keys), so the
// row maximum and row sum are lane-local plus one cross-lane exchange, and the probabilities
// become the operand of Y^T = V^T P^T with a register-local conversion: with k-slot 8g + 4jj + i
// of slab s mapped to key 16 s + 8 jj + 4 g + i of the tile, accumulator registers 8s .. 8s+7 of
// a lane are exactly its k-slots (MFMA 32x32x16; lane = 32 g + n).
//
// Output.  Y^T leaves a lane holding scattered 8-byte pieces of its query's row; the tile is
// turned through a per-wave LDS staging area so that it is stored as whole 128-byte segments.
// The last w rows of K and V of a sequence are also written to the decode ring buffer by the
// workgroup that owns the last segment.
//
// Rotary encoding (ROT).  Query and key rows are rotated between their arrival in registers and their
// use: keys before they are written to the LDS ring (and to the decode ring, which therefore holds
// rotated keys), queries before they become the score operand.  A 16-byte chunk of a row is four
// adjacent pairs, so the rotation is local to the registers that hold the chunk; the (cos, sin) values
// come from a table indexed by [token][pair] that all units share.  Reading the table entry of every
// chunk would double what the kernel pulls through the memory system (8 bytes of cos / sin per 4 bytes of
// bf16 pair; measured + 57 % time).  Instead: (a) the new query rows of a step are the same tokens as its
// new key rows, so the queries are fetched with the same thread-to-chunk mapping as the keys, rotated with
// the same values and handed to the waves through LDS (in the space the output tiles use later in the
// step); (b) a thread's chunks are the same four pairs of rows a fixed distance apart, so it reads the
// table entry of its first row only (requested with that row, a step ahead) and advances it by a constant
// rotation, the ratio of two table rows, for each further row.  The table traffic drops to 1 / 16 (1 / 8
// at d_h = 64).
#include "common.h"

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

constexpr int BQ = 128;   // queries per workgroup
constexpr int NT = 256;

// WIN is the attention window; the key tiles are laid out for W = max(WIN, 32) (a window below one
// tile of 32 keys walks two tiles and masks the rest).
template <int DH, int WIN> struct SwaCfg {
    static constexpr int W = WIN < 32 ? 32 : WIN;
    static constexpr int NK = W + BQ;          // staged key rows
    static constexpr int V_LD = DH + 16;       // bf16 elements per staged V row (row stride = 8 banks mod 32)
    static constexpr int K_LD = DH + 8;        // bf16 elements per staged K row (16-byte pad)
    static constexpr int NKT = W / 32 + 1;     // key tiles per query tile
    static constexpr int Y_LD = 64 + 8;        // bf16 elements per row of a wave's output staging tile (64 columns a pass)
    static constexpr size_t lds_bytes = ((size_t)NK * (V_LD + K_LD) + (size_t)4 * 32 * Y_LD) * 2;
    // rotary variant: the per-wave region holds either the wave's 32 rotated query rows or its output tile
    static constexpr int Q_LD = DH + 8;
    static constexpr int WREG = 32 * (Q_LD > Y_LD ? Q_LD : Y_LD);   // elements of a wave's region
    static constexpr size_t lds_bytes_rotary = ((size_t)NK * (V_LD + K_LD) + (size_t)4 * WREG) * 2;
};

// (cos, sin) of four adjacent pairs
struct Rot4 { f32x4 t01, t23; };

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 w) { return __builtin_bit_cast(bf16x8, w); }

// Eight bf16 elements (four adjacent pairs) rotated by the table entries t[0..3] = (cos, sin) of their
// position and pairs; results rounded to bf16 (nearest even).
__device__ __forceinline__ Rot4 load_rot4(const float2 *__restrict__ t)
{
    Rot4 r;
    r.t01 = *reinterpret_cast<const f32x4 *>(t);
    r.t23 = *reinterpret_cast<const f32x4 *>(t + 2);
    return r;
}
__device__ __forceinline__ u32x4 rotate8(u32x4 x, const Rot4 &r)
{
    const f32x4 t01 = r.t01, t23 = r.t23;
    const float cs[8] = {t01[0], t01[1], t01[2], t01[3], t23[0], t23[1], t23[2], t23[3]};
    u32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float x0 = __uint_as_float(x[j] << 16), x1 = __uint_as_float(x[j] & 0xffff0000u);
        const float c = cs[2 * j], s = cs[2 * j + 1];
        const float r0 = fmaf(x0, c, -x1 * s), r1 = fmaf(x0, s, x1 * c);
        o[j] = (uint32_t)f32_to_bf16_bits(r0) | ((uint32_t)f32_to_bf16_bits(r1) << 16);
    }
    return o;
}
// a * b as rotations (complex products pair by pair); conj_b: a * conj(b)
__device__ __forceinline__ Rot4 rot_mul(const Rot4 &a, const Rot4 &b, bool conj_b = false)
{
    Rot4 o;
    const float sg = conj_b ? -1.f : 1.f;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const f32x4 x = h ? a.t23 : a.t01, y = h ? b.t23 : b.t01;
        f32x4 z;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float ac = x[2 * j], as = x[2 * j + 1], bc = y[2 * j], bs = sg * y[2 * j + 1];
            z[2 * j] = fmaf(ac, bc, -as * bs);
            z[2 * j + 1] = fmaf(as, bc, ac * bs);
        }
        if (h) o.t23 = z; else o.t01 = z;
    }
    return o;
}

}  // namespace

template <int DH, int WIN, bool ROT>
__device__ __forceinline__ void swa_prefill_mfma_body(const uint16_t *__restrict__ q,
                                                      const uint16_t *__restrict__ k,
                                                      const uint16_t *__restrict__ v,
                                                      uint16_t *__restrict__ y,
                                                      uint16_t *__restrict__ ring,
                                                      const float2 *__restrict__ rot, int N,
                                                      int seg_len, int nseg, float scale_log2e)
{
    using Cfg = SwaCfg<DH, WIN>;
    constexpr int W = Cfg::W;
    constexpr int NK = Cfg::NK, V_LD = Cfg::V_LD, K_LD = Cfg::K_LD, NKT = Cfg::NKT;
    constexpr int SLABS = DH / 16;   // k-slabs of the score contraction
    constexpr int CT = DH / 32;      // column tiles of the output
    constexpr int CPR = DH / 8;      // 16-byte chunks per row
    constexpr int NEWIT = BQ * CPR / NT;   // 16-byte chunks per thread for the BQ new rows of a step

    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint16_t *Vs = reinterpret_cast<uint16_t *>(lds_raw);      // [NK][V_LD]: ring of staged V rows
    uint16_t *Ks = Vs + (size_t)NK * V_LD;                     // [NK][K_LD]: ring of staged K rows
    constexpr int Y_LD = Cfg::Y_LD;
    // [4 waves][32][Y_LD]: output tiles on their way out.  Rotary: a wave's region is WREG elements and
    // starts the step as its 32 rotated query rows [32][Q_LD].
    uint16_t *Ysh = Ks + (size_t)NK * K_LD;
    constexpr int Q_LD = Cfg::Q_LD;
    constexpr int WREG = ROT ? Cfg::WREG : 32 * Y_LD;

    const int tid = threadIdx.x;
    // wave index as a scalar, so that branches on it are scalar branches (MFMA ignores EXEC)
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, g = lane >> 5, n = lane & 31;
    const int u = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const int q0 = seg * seg_len;                       // first query of this workgroup's segment
    const int q_end = min(N, q0 + seg_len);
    const size_t base = (size_t)u * N * DH;
    uint16_t *ring_u = ring ? ring + (size_t)u * 2 * WIN * DH : nullptr;

    // Staged row of key position p lives in LDS row (p - (q0 - W)) mod NK: a ring of W + BQ rows.
    // A step handles BQ queries; going to the next step overwrites the BQ oldest rows with the BQ
    // new keys, every K / V row of the segment is staged exactly once (plus the W-row halo at the
    // segment start), and the next step's rows are fetched into registers while this step computes.
    {   // initial fill: keys q0 - W .. q0 + BQ - 1 into ring rows 0 .. NK - 1, every load in flight at once
        constexpr int FILLIT = NK * CPR / NT;
        static_assert(NK * CPR % NT == 0, "the initial fill is a whole number of passes");
        u32x4 fk[FILLIT], fv[FILLIT];
#pragma unroll
        for (int it = 0; it < FILLIT; ++it) {
            const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
            const int key = min(max(q0 - W + r, 0), N - 1);
            fk[it] = *reinterpret_cast<const u32x4 *>(k + base + (size_t)key * DH + c * 8);
            fv[it] = *reinterpret_cast<const u32x4 *>(v + base + (size_t)key * DH + c * 8);
        }
#pragma unroll
        for (int it = 0; it < FILLIT; ++it) {
            const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
            const int key = q0 - W + r;
            if (key < 0 || key >= N) {
                const u32x4 zero = {0u, 0u, 0u, 0u};
                fk[it] = zero; fv[it] = zero;
            } else if (ROT) {
                // (once per segment: every chunk reads its own table entry)
                fk[it] = rotate8(fk[it], load_rot4(rot + (size_t)key * (DH / 2) + 4 * c));
            }
            *reinterpret_cast<u32x4 *>(Vs + (size_t)r * V_LD + c * 8) = fv[it];
            *reinterpret_cast<u32x4 *>(Ks + (size_t)r * K_LD + c * 8) = fk[it];
            // the w-slot ring receives the last min(N, w) rows (slot = position mod w), written
            // by the segment that owns the row as a query row
            if (ring_u && key >= q0 && key < N && key >= N - WIN) {
                uint16_t *rk = ring_u + (size_t)(key % WIN) * DH + c * 8;
                *reinterpret_cast<u32x4 *>(rk) = fk[it];
                *reinterpret_cast<u32x4 *>(rk + (size_t)WIN * DH) = fv[it];
            }
        }
    }

    u32x4 nk[NEWIT], nv[NEWIT];   // next step's new rows, in flight during this step
    u32x4 qop[SLABS], qnext[SLABS];   // rotary: qnext holds the new query rows in the key rows' chunk mapping
    static_assert(NEWIT == SLABS, "a thread stages as many query chunks as a lane holds operand slabs");
    Rot4 tk0;        // rotary: the table entry of the thread's first new row
    Rot4 rot_step;   // rotary: rotation by the NT / CPR rows between a thread's consecutive chunks
    // where row r (of the BQ rows of a step) of the rotated queries sits: wave r / 32's region
    auto q_stage = [&](int r) { return Ysh + (size_t)(r >> 5) * WREG + (size_t)(r & 31) * Q_LD; };
    auto read_qop = [&]() {
        const uint16_t *row = Ysh + (size_t)wv * WREG + (size_t)n * Q_LD + 8 * g;
#pragma unroll
        for (int s = 0; s < SLABS; ++s) qop[s] = *reinterpret_cast<const u32x4 *>(row + 16 * s);
    };
    if constexpr (ROT) {
        const int c = tid % CPR;
        const int dl = min(NT / CPR, N - 1);   // (a sequence shorter than that has a single step and no use for it)
        rot_step = rot_mul(load_rot4(rot + (size_t)dl * (DH / 2) + 4 * c), load_rot4(rot + 4 * c), true);
        // the first step's queries: fetched and rotated chunk by chunk, each with its own table entry
#pragma unroll
        for (int it = 0; it < NEWIT; ++it) {
            const int idx = tid + it * NT, r = idx / CPR;
            const int row = min(q0 + r, N - 1);
            const u32x4 x = *reinterpret_cast<const u32x4 *>(q + base + (size_t)row * DH + c * 8);
            *reinterpret_cast<u32x4 *>(q_stage(r) + c * 8) = rotate8(x, load_rot4(rot + (size_t)row * (DH / 2) + 4 * c));
        }
    }
    // Loads of the pipeline are unconditional (a row past the end of the sequence re-reads the last
    // row; it is zeroed when staged, or belongs to a query that is never stored).  With a conditional
    // load the compiler cannot tell how many memory operations are in flight, waits for all of them
    // wherever it needs one, and the prefetch below would be waited for as soon as it is issued.
    auto load_q = [&](int step_q0, u32x4 (&dst)[SLABS]) {
        const int query = min(step_q0 + 32 * wv + n, N - 1);
#pragma unroll
        for (int s = 0; s < SLABS; ++s)
            dst[s] = *reinterpret_cast<const u32x4 *>(q + base + (size_t)query * DH + 16 * s + 8 * g);
    };
    if constexpr (!ROT) {
        load_q(q0, qop);
        // The first queries have arrived before the pipeline starts (an asm statement that takes them as
        // operands): otherwise every step would wait for "loads that may still be in flight from before
        // the loop", which at that point means waiting for the prefetch it has just issued.
#pragma unroll
        for (int s = 0; s < SLABS; ++s) asm volatile("" : "+v"(qop[s]));
    }
    __syncthreads();
    if constexpr (ROT) read_qop();

    // One step of BQ queries.  Steps that have a successor are instantiated apart from the last one
    // of the segment, so that inside them every prefetch and every store is unconditional code and
    // the number of memory operations in flight is known exactly wherever one has to be waited for.
    auto step = [&](const int sq0, auto more_c) {
        constexpr bool more = decltype(more_c)::value;
        // The BQ rows of the next step and its queries are requested in three portions, before the
        // scores, the softmax and the P.V product: all waves of a CU asking for everything at once
        // would queue behind each other at the memory pipeline with nothing else to issue.
        auto prefetch_k = [&]() {
            if constexpr (more) {
#pragma unroll
                for (int it = 0; it < NEWIT; ++it) {
                    const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
                    const int key = min(sq0 + BQ + r, N - 1);
                    nk[it] = *reinterpret_cast<const u32x4 *>(k + base + (size_t)key * DH + c * 8);
                    if constexpr (ROT) {
                        if (it == 0) tk0 = load_rot4(rot + (size_t)key * (DH / 2) + 4 * c);
                    }
                }
            }
        };
        auto prefetch_v = [&]() {
            if constexpr (more) {
#pragma unroll
                for (int it = 0; it < NEWIT; ++it) {
                    const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
                    const int key = min(sq0 + BQ + r, N - 1);
                    nv[it] = *reinterpret_cast<const u32x4 *>(v + base + (size_t)key * DH + c * 8);
                }
            }
        };
        auto prefetch_q = [&]() {
            if constexpr (more) {
                if constexpr (ROT) {
#pragma unroll
                    for (int it = 0; it < NEWIT; ++it) {
                        const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
                        const int row = min(sq0 + BQ + r, N - 1);
                        qnext[it] = *reinterpret_cast<const u32x4 *>(q + base + (size_t)row * DH + c * 8);
                    }
                } else {
                    load_q(sq0 + BQ, qnext);
                }
            }
        };
        prefetch_q();

        const int qbase = sq0 + 32 * wv;          // first query of this wave's tile
        const int query = qbase + n;
        const bool q_ok = query < q_end;
        {   // every wave computes (a tile past the end of the segment works on staged rows like any
            // other and stores nothing): no wave-dependent branch around the stores below
            // row of key position p in the LDS ring
            const int rel0 = qbase - W - (q0 - W);   // ring position of the oldest key tile of this query tile

            // ---- scores: S^T tile t holds keys qbase - W + 32 t .. +31 (rows) against the 32 queries --
            f32x16 P[NKT];
#pragma unroll
            for (int t = 0; t < NKT; ++t) {
#pragma unroll
                for (int r = 0; r < 16; ++r) P[t][r] = 0.f;
                const int slot0 = (rel0 + 32 * t) % NK;   // tiles never wrap inside (NK is a multiple of 32)
                const uint16_t *krow = Ks + (size_t)(slot0 + n) * K_LD + 8 * g;
#pragma unroll
                for (int s = 0; s < SLABS; ++s) {
                    const u32x4 kop = *reinterpret_cast<const u32x4 *>(krow + 16 * s);
                    P[t] = mfma(as_bf16x8(kop), as_bf16x8(qop[s]), P[t]);
                }
            }

            prefetch_k();

            // ---- mask, softmax statistics (lane = query; its keys sit in registers and in lane ^ 32) --
            // Raw scores are masked and their maximum taken; the scale (times log2 e) is applied inside
            // the exponential, exp2(scale * (x - m)), which is one fused multiply-add per element.
            // Key 32 t - W + local of the tile row against query n: visible iff -WIN < 32 t - W + local - n <= 0.
            // Only the tiles whose rows can fall outside get the comparisons (for WIN >= 32 the first
            // and the last one); keys before the start of the sequence exist only for the first W
            // queries (a uniform branch).
            float m = -INFINITY;
            auto mask_and_max = [&](auto head_c) {
                constexpr bool HEAD = decltype(head_c)::value;
#pragma unroll
                for (int t = 0; t < NKT; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int local = 8 * (r >> 2) + 4 * g + (r & 3);
                        const bool cut_low = 32 * t <= W - WIN + 31, cut_high = t == NKT - 1;   // folded when unrolled
                        if (HEAD || cut_low || cut_high) {
                            bool ok = true;
                            if (HEAD) ok = qbase - W + 32 * t + local >= 0;
                            if (cut_low) ok = ok && 32 * t - W + local - n > -WIN;   // key > query - w
                            if (cut_high) ok = ok && local <= n;                      // key <= query
                            P[t][r] = ok ? P[t][r] : -INFINITY;
                        }
                        m = fmaxf(m, P[t][r]);
                    }
            };
            if (qbase < W) mask_and_max(std::true_type{});
            else mask_and_max(std::false_type{});
            m = fmaxf(m, __shfl_xor(m, 32, 64));
            // the query's own key is always visible, so m is finite for every query inside the sequence
            const float neg_ms = q_ok ? -m * scale_log2e : 0.f;
            float sum = 0.f;
#pragma unroll
            for (int t = 0; t < NKT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(P[t][r], scale_log2e, neg_ms));   // exp2(-inf) = 0: masked keys
                    P[t][r] = pe;
                    sum += pe;
                }
            sum += __shfl_xor(sum, 32, 64);

            prefetch_v();

            // ---- Y^T = V^T P^T ----------------------------------------------------------------------------
            f32x16 Y[CT];
#pragma unroll
            for (int c2 = 0; c2 < CT; ++c2)
#pragma unroll
                for (int r = 0; r < 16; ++r) Y[c2][r] = 0.f;
#pragma unroll
            for (int t = 0; t < NKT; ++t) {
                const int slot0 = (rel0 + 32 * t) % NK;
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    f32x8 f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[e] = P[t][8 * s + e];
                    const bf16x8 pb = __builtin_convertvector(f, bf16x8);
                    // V^T operand: lane (g, n) needs column 32 c2 + n at the 8 keys of its k-slots (two runs
                    // of 4 consecutive staged rows).  Transposing read: in each group of 16 lanes, lane k
                    // supplies the address of 4 consecutive columns of row (k / 4), columns 4 (k % 4) .. of the
                    // group's 16-column block, and receives column k of that block at the 4 rows.
                    const int rowk = slot0 + 16 * s + 4 * g;   // first staged row of this lane's k-slots
                    const int kk = lane & 15, grp = (lane >> 4) & 1;
                    const uint16_t *pv = Vs + (size_t)(rowk + (kk >> 2)) * V_LD + 16 * grp + 4 * (kk & 3);
#pragma unroll
                    for (int c2 = 0; c2 < CT; ++c2) {
                        const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4 *)(pv + 32 * c2));
                        const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4 *)(pv + 32 * c2 + 8 * V_LD));
                        s16x8 o;
#pragma unroll
                        for (int i = 0; i < 4; ++i) { o[i] = a[i]; o[4 + i] = b[i]; }
                        Y[c2] = mfma(__builtin_bit_cast(bf16x8, o), pb, Y[c2]);
                    }
                }
            }

            // ---- normalise and store ---------------------------------------------------------------------
            // lane = query, register r = column 8 (r / 4) + 4 g + r % 4: stored directly, a lane would
            // write 8-byte pieces of its own row (16-byte write requests, which stall the memory
            // pipeline).  The tile goes through this wave's LDS staging rows instead and leaves as
            // whole 128-byte row segments, 64 columns a pass: lane l writes 16 bytes of row l / 8.
            {
                const float inv = q_ok ? 1.f / sum : 0.f;
                uint16_t *yt = Ysh + (size_t)wv * WREG;
#pragma unroll
                for (int cp = 0; cp < DH / 64; ++cp) {
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            f32x4 o;
#pragma unroll
                            for (int i = 0; i < 4; ++i) o[i] = Y[2 * cp + c2][4 * j + i] * inv;
                            const bf16x4 hv = __builtin_convertvector(o, bf16x4);
                            *reinterpret_cast<u32x2 *>(yt + (size_t)n * Y_LD + 32 * c2 + 8 * j + 4 * g) =
                                __builtin_bit_cast(u32x2, hv);
                        }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's tile is complete in LDS
                    u32x4 val[4];
                    uint16_t *dst[4];
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const int row = it * 8 + lane / 8, c = lane % 8;
                        val[it] = *reinterpret_cast<const u32x4 *>(yt + (size_t)row * Y_LD + c * 8);
                        dst[it] = y + base + (size_t)(qbase + row) * DH + 64 * cp + c * 8;
                    }
                    // A full step stores without a per-lane condition, so that the stores can be
                    // counted and the wait for the prefetched rows (older, retired in order) is not
                    // also a wait for these stores.
                    if (more || sq0 + BQ <= q_end) {
#pragma unroll
                        for (int it = 0; it < 4; ++it) *reinterpret_cast<u32x4 *>(dst[it]) = val[it];
                    } else {
#pragma unroll
                        for (int it = 0; it < 4; ++it)
                            if (qbase + it * 8 + lane / 8 < q_end) *reinterpret_cast<u32x4 *>(dst[it]) = val[it];
                        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
                    }
                }
            }
        }

        if constexpr (more) {
            if constexpr (ROT) {
                // The rotations happen in registers, ahead of the barrier: a wave that is early does them
                // while the others finish the step.  rcur: the entry of the chunk at hand; a row past the
                // end of the sequence got the last row's entry, and so do all rows after it, which are
                // not used.
                Rot4 rcur = tk0;
#pragma unroll
                for (int it = 0; it < NEWIT; ++it) {
                    if (it > 0) rcur = rot_mul(rcur, rot_step);
                    nk[it] = rotate8(nk[it], rcur);
                    qnext[it] = rotate8(qnext[it], rcur);
                }
            }
            __syncthreads();   // every wave is done with the rows that are overwritten now
            const int rel_new = (sq0 + BQ) - (q0 - W);   // ring position of the first new key
#pragma unroll
            for (int it = 0; it < NEWIT; ++it) {
                const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
                const int key = sq0 + BQ + r;
                const int slot = (rel_new + r) % NK;
                if constexpr (ROT) *reinterpret_cast<u32x4 *>(q_stage(r) + c * 8) = qnext[it];
                if (key >= N) {
                    const u32x4 zero = {0u, 0u, 0u, 0u};
                    nk[it] = zero; nv[it] = zero;
                }
                *reinterpret_cast<u32x4 *>(Vs + (size_t)slot * V_LD + c * 8) = nv[it];
                *reinterpret_cast<u32x4 *>(Ks + (size_t)slot * K_LD + c * 8) = nk[it];
                if (ring_u && key < N && key >= N - WIN && key < q_end) {
                    uint16_t *rk = ring_u + (size_t)(key % WIN) * DH + c * 8;
                    *reinterpret_cast<u32x4 *>(rk) = nk[it];
                    *reinterpret_cast<u32x4 *>(rk + (size_t)WIN * DH) = nv[it];
                }
            }
#pragma unroll
            for (int s = 0; s < SLABS; ++s)
                if constexpr (!ROT) qop[s] = qnext[s];
            __syncthreads();
            if constexpr (ROT) read_qop();
        }
    };
    int sq0 = q0;
    for (; sq0 + BQ < q_end; sq0 += BQ) step(sq0, std::true_type{});
    step(sq0, std::false_type{});
}

template <int DH, int WIN>
__global__ __launch_bounds__(NT) void swa_prefill_mfma_kernel(const uint16_t *__restrict__ q,
                                                              const uint16_t *__restrict__ k,
                                                              const uint16_t *__restrict__ v,
                                                              uint16_t *__restrict__ y,
                                                              uint16_t *__restrict__ ring, int N,
                                                              int seg_len, int nseg, float scale_log2e)
{
    swa_prefill_mfma_body<DH, WIN, false>(q, k, v, y, ring, nullptr, N, seg_len, nseg, scale_log2e);
}

// The rotary variant keeps the table entries of the rows in flight in registers: where the LDS ring
// leaves room for one workgroup per CU only, a wave may have the whole register file of its SIMD.
template <int DH, int WIN>
__global__ __launch_bounds__(NT, (SwaCfg<DH, WIN>::lds_bytes_rotary > 80u * 1024u ? 1 : 2)) void swa_prefill_mfma_rotary_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ y, uint16_t *__restrict__ ring, const float2 *__restrict__ rot, int N, int seg_len,
    int nseg, float scale_log2e)
{
    swa_prefill_mfma_body<DH, WIN, true>(q, k, v, y, ring, rot, N, seg_len, nseg, scale_log2e);
}

template <int DH, int WIN, bool ROT>
static hipError_t launch_swa_mfma_rot(const void *q, const void *k, const void *v, void *y, void *ring,
                                      const float *rot, int U, int N, float scale, hipStream_t s)
{
    using Cfg = SwaCfg<DH, WIN>;
    constexpr size_t lds_bytes = ROT ? Cfg::lds_bytes_rotary : Cfg::lds_bytes;
    if (lds_bytes > 160u * 1024u) return hipErrorInvalidValue;   // callers ask swa_prefill_mfma_supported first
    const void *kern = ROT ? reinterpret_cast<const void *>(swa_prefill_mfma_rotary_kernel<DH, WIN>)
                           : reinterpret_cast<const void *>(swa_prefill_mfma_kernel<DH, WIN>);
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    // Segments per sequence.  The launch should be whole rounds of resident workgroups (256 CUs x as
    // many workgroups as the LDS ring lets a CU hold: a partial last round costs as much as a full
    // one), with segments long next to the W-row halo and the ring fill every segment starts with.
    // Score of a candidate: fill of its rounds / (1 + (W + 64) / tokens per segment).
    const int steps = (N + BQ - 1) / BQ;
    const int per_cu = (int)((160u * 1024u) / lds_bytes) < 1 ? 1 : (int)((160u * 1024u) / lds_bytes);
    const long slots = 256L * per_cu;
    int nseg = 1;
    double best = -1.0;
    for (int c = 1; c <= steps && c <= 64; ++c) {
        const int seg_steps = (steps + c - 1) / c;
        const int segs = (steps + seg_steps - 1) / seg_steps;   // segments this candidate really makes
        const long wgs = (long)segs * U;
        const double fill = (double)wgs / (double)(((wgs + slots - 1) / slots) * slots);
        const double score = fill / (1.0 + (double)(Cfg::W + 64) / ((double)seg_steps * BQ));
        if (score > best * 1.0001) { best = score; nseg = segs; }
    }
    const int seg_len = ((steps + nseg - 1) / nseg) * BQ;
    nseg = (N + seg_len - 1) / seg_len;
    const dim3 grid((unsigned)((size_t)nseg * U));
    const float scale_log2e = scale * 1.44269504088896340736f;
    if (ROT)
        hipLaunchKernelGGL((swa_prefill_mfma_rotary_kernel<DH, WIN>), grid, dim3(NT), lds_bytes, s,
                           (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)y,
                           (uint16_t *)ring, reinterpret_cast<const float2 *>(rot), N, seg_len, nseg, scale_log2e);
    else
        hipLaunchKernelGGL((swa_prefill_mfma_kernel<DH, WIN>), grid, dim3(NT), Cfg::lds_bytes, s,
                           (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)y,
                           (uint16_t *)ring, N, seg_len, nseg, scale_log2e);
    return hipGetLastError();
}

template <int DH, int WIN>
static hipError_t launch_swa_mfma(const void *q, const void *k, const void *v, void *y, void *ring,
                                  const float *rot, int U, int N, float scale, hipStream_t s)
{
    return rot ? launch_swa_mfma_rot<DH, WIN, true>(q, k, v, y, ring, rot, U, N, scale, s)
               : launch_swa_mfma_rot<DH, WIN, false>(q, k, v, y, ring, nullptr, U, N, scale, s);
}

bool swa_prefill_mfma_supported(int dh, int w, int dtype, int rotary)
{
    // the rotary variant stages the queries in LDS as well, which the largest ring leaves no room for
    if (rotary && dh == 128 && w == 128) return false;
    return dtype == BASED_BF16 && (dh == 64 || dh == 128) && (w == 16 || w == 32 || w == 64 || w == 128);
}

hipError_t launch_swa_prefill_mfma(const void *q, const void *k, const void *v, void *y, void *ring,
                                   const float *rot, int U, int N, int dh, int w, float scale, hipStream_t s)
{
    if (dh == 64 && w == 16) return launch_swa_mfma<64, 16>(q, k, v, y, ring, rot, U, N, scale, s);
    if (dh == 64 && w == 32) return launch_swa_mfma<64, 32>(q, k, v, y, ring, rot, U, N, scale, s);
    if (dh == 128 && w == 16) return launch_swa_mfma<128, 16>(q, k, v, y, ring, rot, U, N, scale, s);
    if (dh == 128 && w == 32) return launch_swa_mfma<128, 32>(q, k, v, y, ring, rot, U, N, scale, s);
    if (dh == 64 && w == 64) return launch_swa_mfma<64, 64>(q, k, v, y, ring, rot, U, N, scale, s);
    if (dh == 64 && w == 128) return launch_swa_mfma<64, 128>(q, k, v, y, ring, rot, U, N, scale, s);
    if (dh == 128 && w == 64) return launch_swa_mfma<128, 64>(q, k, v, y, ring, rot, U, N, scale, s);
    if (dh == 128 && w == 128) return launch_swa_mfma<128, 128>(q, k, v, y, ring, rot, U, N, scale, s);
    return hipErrorInvalidValue;
}

}  // namespace based
