// Sliding-window causal softmax attention over whole sequences (Sec. 3.2 restricting Eq. 1) on the gfx950
// matrix cores, tiled 16 queries to a wave: bf16 in, fp32 scores / softmax / accumulation.
//
// Why a second tiling.  With 32-query tiles a workgroup's LDS ring (window + 128 rows of K and V) leaves room
// for one workgroup of four waves per CU, one wave per SIMD, and a wave alone on its SIMD cannot hide its own
// latencies: the matrix instructions wait for their LDS operands, the softmax is a chain of dependent vector
// instructions, and measured per phase about 70 % of a step was this arithmetic, not the wait for memory.
// A wave that owns 16 queries works on w + 16 keys instead of w + 32, a step of four waves is 64 queries, the
// ring is window + 64 rows, and two workgroups fit a CU: two waves per SIMD that fill each other's gaps, and
// two workgroups that are in different phases, so one of them usually has memory requests in flight.
//
// Work split.  One workgroup of four waves per (unit, segment of the sequence) walks its segment in steps of
// 64 queries; each wave owns one tile of 16 queries of the step and the w / 16 + 1 tiles of 16 keys it can see.
//
// Staging.  As in the 32-query kernel: the w + 64 key and value rows a step can see sit in an LDS ring, every
// step overwrites the 64 oldest rows with its 64 new ones, fetched into registers during the step before.
//
// Operands (MFMA 16x16x32 bf16; lane = 16 g + n).  Scores are computed transposed, S^T = K Q^T: a lane's 8
// k-slots of slab s are the 16 bytes at columns 32 s + 8 g of its row, for K (from LDS) and Q (from global
// memory) alike.  The result leaves lane (g, n) with keys 4 g .. 4 g + 3 of the tile for query n, so row
// maximum and row sum are lane-local plus two cross-lane exchanges.  For Y^T = V^T P^T two key tiles form one
// slab of 32 keys: k-slot 8 g + j is key 4 g + j of the first tile (j < 4) or key 4 g + j - 4 of the second,
// which is what the lane holds; V^T comes from two transposing LDS reads (ds_read_b64_tr_b16), one per tile.
// The number of key tiles is odd; the last one goes through the 16x16x16 instruction, whose k-slots 4 g + j
// are the tile's keys as they lie.
#include "common.h"

#include <type_traits>

namespace based {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int BQ = 64;    // queries per step
constexpr int NT = 256;   // four waves

template <int DH, int WIN> struct Swa16Cfg {
    static constexpr int NK = WIN + BQ;        // staged key rows
    static constexpr int V_LD = DH + 16;       // bf16 elements per staged V row (row stride = 8 banks mod 32)
    static constexpr int K_LD = DH + 8;        // bf16 elements per staged K row (16-byte pad)
    static constexpr int NKT = WIN / 16 + 1;   // key tiles per query tile
    static constexpr int Y_LD = 64 + 8;        // bf16 elements per row of a wave's output staging tile
    static constexpr size_t lds_bytes = ((size_t)NK * (V_LD + K_LD) + (size_t)4 * 16 * Y_LD) * 2;
};

__device__ __forceinline__ f32x4 mfma32(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16(s16x4 a, s16x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 w) { return __builtin_bit_cast(bf16x8, w); }

}  // namespace

template <int DH, int WIN>
__global__ __launch_bounds__(NT, 2) void swa_prefill_mfma16_kernel(const uint16_t *__restrict__ q,
                                                                   const uint16_t *__restrict__ k,
                                                                   const uint16_t *__restrict__ v,
                                                                   uint16_t *__restrict__ y,
                                                                   uint16_t *__restrict__ ring, int N,
                                                                   int seg_len, int nseg, float scale_log2e)
{
    using Cfg = Swa16Cfg<DH, WIN>;
    constexpr int NK = Cfg::NK, V_LD = Cfg::V_LD, K_LD = Cfg::K_LD, NKT = Cfg::NKT, Y_LD = Cfg::Y_LD;
    constexpr int SLABS = DH / 32;   // k-slabs of the score contraction
    constexpr int CT = DH / 16;      // column tiles of the output
    constexpr int CPR = DH / 8;      // 16-byte chunks per row
    constexpr int NEWIT = BQ * CPR / NT;   // 16-byte chunks per thread for the BQ new rows of a step
    static_assert(WIN % 16 == 0 && NKT % 2 == 1, "an even number of key tiles plus the diagonal one");
    static_assert(BQ * CPR % NT == 0 && NK * CPR % NT == 0, "staging passes are whole");

    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint16_t *Vs = reinterpret_cast<uint16_t *>(lds_raw);      // [NK][V_LD]: ring of staged V rows
    uint16_t *Ks = Vs + (size_t)NK * V_LD;                     // [NK][K_LD]: ring of staged K rows
    uint16_t *Ysh = Ks + (size_t)NK * K_LD;                    // [4 waves][16][Y_LD]: output tiles on their way out

    const int tid = threadIdx.x;
    // wave index as a scalar, so that branches on it are scalar branches (MFMA ignores EXEC)
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, g = lane >> 4, n = lane & 15;
    const int u = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const int q0 = seg * seg_len;                       // first query of this workgroup's segment
    const int q_end = min(N, q0 + seg_len);
    const size_t base = (size_t)u * N * DH;
    uint16_t *ring_u = ring ? ring + (size_t)u * 2 * WIN * DH : nullptr;

    // Staged row of key position p lives in LDS row (p - (q0 - WIN)) mod NK.
    {   // initial fill: keys q0 - WIN .. q0 + BQ - 1 into ring rows 0 .. NK - 1, every load in flight at once
        constexpr int FILLIT = NK * CPR / NT;
        u32x4 fk[FILLIT], fv[FILLIT];
#pragma unroll
        for (int it = 0; it < FILLIT; ++it) {
            const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
            const int key = min(max(q0 - WIN + r, 0), N - 1);
            fk[it] = *reinterpret_cast<const u32x4 *>(k + base + (size_t)key * DH + c * 8);
            fv[it] = *reinterpret_cast<const u32x4 *>(v + base + (size_t)key * DH + c * 8);
        }
#pragma unroll
        for (int it = 0; it < FILLIT; ++it) {
            const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
            const int key = q0 - WIN + r;
            if (key < 0 || key >= N) {
                const u32x4 zero = {0u, 0u, 0u, 0u};
                fk[it] = zero; fv[it] = zero;
            }
            *reinterpret_cast<u32x4 *>(Vs + (size_t)r * V_LD + c * 8) = fv[it];
            *reinterpret_cast<u32x4 *>(Ks + (size_t)r * K_LD + c * 8) = fk[it];
            // the w-slot ring receives the last min(N, w) rows (slot = position mod w), written by the
            // segment that owns the row as a query row
            if (ring_u && key >= q0 && key < N && key >= N - WIN) {
                uint16_t *rk = ring_u + (size_t)(key % WIN) * DH + c * 8;
                *reinterpret_cast<u32x4 *>(rk) = fk[it];
                *reinterpret_cast<u32x4 *>(rk + (size_t)WIN * DH) = fv[it];
            }
        }
    }

    u32x4 nk[NEWIT], nv[NEWIT];       // next step's new rows, in flight during this step
    u32x4 qop[SLABS], qnext[SLABS];   // score operand of this step's queries and of the next step's
    // Loads of the pipeline are unconditional (a row past the end of the sequence re-reads the last row; it
    // is zeroed when staged, or belongs to a query that is never stored), so that the number of memory
    // operations in flight is known wherever one has to be waited for.
    auto load_q = [&](int step_q0, u32x4 (&dst)[SLABS]) {
        const int query = min(step_q0 + 16 * wv + n, N - 1);
#pragma unroll
        for (int s = 0; s < SLABS; ++s)
            dst[s] = *reinterpret_cast<const u32x4 *>(q + base + (size_t)query * DH + 32 * s + 8 * g);
    };
    load_q(q0, qop);
    // the first queries have arrived before the pipeline starts, so that no step waits for "loads that may
    // still be in flight from before the loop"
#pragma unroll
    for (int s = 0; s < SLABS; ++s) asm volatile("" : "+v"(qop[s]));
    __syncthreads();

    // One step of BQ queries.  Steps that have a successor are instantiated apart from the last one of the
    // segment, so that inside them every prefetch and every store is unconditional code.
    auto step = [&](const int sq0, auto more_c) {
        constexpr bool more = decltype(more_c)::value;
        // the BQ rows of the next step and its queries are requested in three portions, before the scores,
        // the softmax and the P.V product
        if constexpr (more) load_q(sq0 + BQ, qnext);

        const int qbase = sq0 + 16 * wv;          // first query of this wave's tile
        const int query = qbase + n;
        const bool q_ok = query < q_end;
        const int rel0 = qbase - q0;              // ring position of the oldest key tile of this query tile

        // ---- scores: S^T tile t holds keys qbase - WIN + 16 t .. + 15 (rows) against the 16 queries ----
        f32x4 P[NKT];
#pragma unroll
        for (int t = 0; t < NKT; ++t) {
#pragma unroll
            for (int r = 0; r < 4; ++r) P[t][r] = 0.f;
            const int slot0 = (rel0 + 16 * t) % NK;   // tiles never wrap inside (NK is a multiple of 16)
            const uint16_t *krow = Ks + (size_t)(slot0 + n) * K_LD + 8 * g;
#pragma unroll
            for (int s = 0; s < SLABS; ++s) {
                const u32x4 kop = *reinterpret_cast<const u32x4 *>(krow + 32 * s);
                P[t] = mfma32(as_bf16x8(kop), as_bf16x8(qop[s]), P[t]);
            }
        }

        if constexpr (more) {
#pragma unroll
            for (int it = 0; it < NEWIT; ++it) {
                const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
                const int key = min(sq0 + BQ + r, N - 1);
                nk[it] = *reinterpret_cast<const u32x4 *>(k + base + (size_t)key * DH + c * 8);
            }
        }

        // ---- mask, softmax statistics (lane = query; its keys sit in registers and in the lanes n + 16 g') --
        // Key 16 t - WIN + local of tile t against query n is visible iff -WIN < 16 t - WIN + local - n <= 0:
        // the first tile needs local > n, the last one local <= n, the ones between are visible whole.  Keys
        // before the start of the sequence exist only for the first WIN queries (a uniform branch).
        float m = -INFINITY;
        auto mask_and_max = [&](auto head_c) {
            constexpr bool HEAD = decltype(head_c)::value;
#pragma unroll
            for (int t = 0; t < NKT; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int local = 4 * g + r;
                    const bool cut_low = t == 0, cut_high = t == NKT - 1;   // folded when unrolled
                    if (HEAD || cut_low || cut_high) {
                        bool ok = true;
                        if (HEAD) ok = qbase - WIN + 16 * t + local >= 0;
                        if (cut_low) ok = ok && local > n;      // key > query - w
                        if (cut_high) ok = ok && local <= n;    // key <= query
                        P[t][r] = ok ? P[t][r] : -INFINITY;
                    }
                    m = fmaxf(m, P[t][r]);
                }
        };
        if (qbase < WIN) mask_and_max(std::true_type{});
        else mask_and_max(std::false_type{});
        m = fmaxf(m, __shfl_xor(m, 16, 64));
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        // the query's own key is always visible, so m is finite for every query inside the sequence
        const float neg_ms = q_ok ? -m * scale_log2e : 0.f;
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < NKT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float pe = __builtin_amdgcn_exp2f(fmaf(P[t][r], scale_log2e, neg_ms));   // exp2(-inf) = 0: masked keys
                P[t][r] = pe;
                sum += pe;
            }
        sum += __shfl_xor(sum, 16, 64);
        sum += __shfl_xor(sum, 32, 64);

        if constexpr (more) {
#pragma unroll
            for (int it = 0; it < NEWIT; ++it) {
                const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
                const int key = min(sq0 + BQ + r, N - 1);
                nv[it] = *reinterpret_cast<const u32x4 *>(v + base + (size_t)key * DH + c * 8);
            }
        }

        // ---- Y^T = V^T P^T ----------------------------------------------------------------------------------
        f32x4 Y[CT];
#pragma unroll
        for (int c2 = 0; c2 < CT; ++c2)
#pragma unroll
            for (int r = 0; r < 4; ++r) Y[c2][r] = 0.f;
        // Transposing read: in each group of 16 lanes, lane kk supplies the address of 4 consecutive columns
        // (4 (kk % 4) ..) of row kk / 4 of a 4 x 16 block and receives column kk of the block at its 4 rows.
        // Group g reads rows 4 g .. 4 g + 3 of the key tile: the keys of the lane's k-slots.
        const int kk_row = 4 * g + (n >> 2), kk_col = 4 * (n & 3);
#pragma unroll
        for (int s = 0; s < NKT / 2; ++s) {
            const int slot_a = (rel0 + 32 * s) % NK, slot_b = (rel0 + 32 * s + 16) % NK;
            f32x4 fa = P[2 * s], fb = P[2 * s + 1];
            const bf16x4 ha = __builtin_convertvector(fa, bf16x4), hb = __builtin_convertvector(fb, bf16x4);
            bf16x8 pb;
#pragma unroll
            for (int i = 0; i < 4; ++i) { pb[i] = ha[i]; pb[4 + i] = hb[i]; }
            const uint16_t *pa = Vs + (size_t)(slot_a + kk_row) * V_LD + kk_col;
            const uint16_t *pbv = Vs + (size_t)(slot_b + kk_row) * V_LD + kk_col;
#pragma unroll
            for (int c2 = 0; c2 < CT; ++c2) {
                const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(pa + 16 * c2));
                const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(pbv + 16 * c2));
                s16x8 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) { o[i] = a[i]; o[4 + i] = b[i]; }
                Y[c2] = mfma32(__builtin_bit_cast(bf16x8, o), pb, Y[c2]);
            }
        }
        {   // the diagonal tile on its own
            const int slot_a = (rel0 + 16 * (NKT - 1)) % NK;
            f32x4 fa = P[NKT - 1];
            const s16x4 pb = __builtin_bit_cast(s16x4, __builtin_convertvector(fa, bf16x4));
            const uint16_t *pa = Vs + (size_t)(slot_a + kk_row) * V_LD + kk_col;
#pragma unroll
            for (int c2 = 0; c2 < CT; ++c2) {
                const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(pa + 16 * c2));
                Y[c2] = mfma16(a, pb, Y[c2]);
            }
        }

        // ---- normalise and store ---------------------------------------------------------------------------
        // lane = query, register r of column tile c2 = column 16 c2 + 4 g + r: the tile goes through this
        // wave's LDS staging rows and leaves as whole 128-byte row segments, 64 columns a pass.
        {
            const float inv = q_ok ? 1.f / sum : 0.f;
            uint16_t *yt = Ysh + (size_t)wv * 16 * Y_LD;
#pragma unroll
            for (int cp = 0; cp < DH / 64; ++cp) {
#pragma unroll
                for (int c2 = 0; c2 < 4; ++c2) {
                    f32x4 o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = Y[4 * cp + c2][i] * inv;
                    const bf16x4 hv = __builtin_convertvector(o, bf16x4);
                    *reinterpret_cast<u32x2 *>(yt + (size_t)n * Y_LD + 16 * c2 + 4 * g) = __builtin_bit_cast(u32x2, hv);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's tile is complete in LDS
                u32x4 val[2];
                uint16_t *dst[2];
#pragma unroll
                for (int it = 0; it < 2; ++it) {
                    const int row = it * 8 + lane / 8, c = lane % 8;
                    val[it] = *reinterpret_cast<const u32x4 *>(yt + (size_t)row * Y_LD + c * 8);
                    dst[it] = y + base + (size_t)(qbase + row) * DH + 64 * cp + c * 8;
                }
                // a full step stores without a per-lane condition, so that the stores can be counted
                if (more || sq0 + BQ <= q_end) {
#pragma unroll
                    for (int it = 0; it < 2; ++it) *reinterpret_cast<u32x4 *>(dst[it]) = val[it];
                } else {
#pragma unroll
                    for (int it = 0; it < 2; ++it)
                        if (qbase + it * 8 + lane / 8 < q_end) *reinterpret_cast<u32x4 *>(dst[it]) = val[it];
                    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
                }
                if (cp + 1 < DH / 64) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // staging rows are read before they are rewritten
            }
        }

        if constexpr (more) {
            __syncthreads();   // every wave is done with the rows that are overwritten now
            const int rel_new = (sq0 + BQ) - (q0 - WIN);   // ring position of the first new key
#pragma unroll
            for (int it = 0; it < NEWIT; ++it) {
                const int idx = tid + it * NT, r = idx / CPR, c = idx % CPR;
                const int key = sq0 + BQ + r;
                const int slot = (rel_new + r) % NK;
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
            for (int s = 0; s < SLABS; ++s) qop[s] = qnext[s];
            __syncthreads();
        }
    };
    int sq0 = q0;
    for (; sq0 + BQ < q_end; sq0 += BQ) step(sq0, std::true_type{});
    step(sq0, std::false_type{});
}

template <int DH, int WIN>
static hipError_t launch_swa_mfma16(const void *q, const void *k, const void *v, void *y, void *ring, int U, int N,
                                    float scale, hipStream_t s)
{
    using Cfg = Swa16Cfg<DH, WIN>;
    constexpr size_t lds_bytes = Cfg::lds_bytes;
    static_assert(lds_bytes <= 160u * 1024u, "the ring fits a CU");
    const void *kern = reinterpret_cast<const void *>(swa_prefill_mfma16_kernel<DH, WIN>);
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    // Segments per sequence: whole rounds of resident workgroups (256 CUs x as many workgroups as the LDS
    // ring and the wave slots let a CU hold), with segments long next to the window-sized halo and the ring
    // fill every segment starts with.  Score of a candidate: fill of its rounds / (1 + halo / tokens per segment).
    const int steps = (N + BQ - 1) / BQ;
    static int per_cu = 0;   // (the same value whichever thread writes it)
    if (per_cu == 0) {
        int nb = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, NT, lds_bytes);
        if (e != hipSuccess) return e;
        per_cu = nb < 1 ? 1 : nb;
    }
    const long slots = 256L * per_cu;
    int nseg = 1;
    double best = -1.0;
    for (int c = 1; c <= steps && c <= 64; ++c) {
        const int seg_steps = (steps + c - 1) / c;
        const int segs = (steps + seg_steps - 1) / seg_steps;   // segments this candidate really makes
        const long wgs = (long)segs * U;
        const double fill = (double)wgs / (double)(((wgs + slots - 1) / slots) * slots);
        const double score = fill / (1.0 + (double)(WIN + 64) / ((double)seg_steps * BQ));
        if (score > best * 1.0001) { best = score; nseg = segs; }
    }
    const int seg_len = ((steps + nseg - 1) / nseg) * BQ;
    nseg = (N + seg_len - 1) / seg_len;
    const dim3 grid((unsigned)((size_t)nseg * U));
    const float scale_log2e = scale * 1.44269504088896340736f;
    hipLaunchKernelGGL((swa_prefill_mfma16_kernel<DH, WIN>), grid, dim3(NT), lds_bytes, s, (const uint16_t *)q,
                       (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)y, (uint16_t *)ring, N, seg_len, nseg,
                       scale_log2e);
    return hipGetLastError();
}

bool swa_prefill_mfma16_supported(int dh, int w, int dtype)
{
    // the sizes where this tiling was measured to be the faster one: d_h = 128 with a ring that then fits a CU
    // twice (with d_h = 64 the 32-query kernel already holds two workgroups per CU and the two run alike; with
    // window 128 this one holds a single workgroup as well and is slower)
    return dtype == BASED_BF16 && dh == 128 && (w == 32 || w == 64);
}

hipError_t launch_swa_prefill_mfma16(const void *q, const void *k, const void *v, void *y, void *ring, int U, int N,
                                     int dh, int w, float scale, hipStream_t s)
{
    if (dh == 128 && w == 32) return launch_swa_mfma16<128, 32>(q, k, v, y, ring, U, N, scale, s);
    if (dh == 128 && w == 64) return launch_swa_mfma16<128, 64>(q, k, v, y, ring, U, N, scale, s);
    return hipErrorInvalidValue;
}

}  // namespace based
