// Per-token decode kernels: the recurrent Taylor linear-attention step (Eq. 3; the operation of
// Alg. 2 plus the K-state and the division), the sliding-window attention step over the w-slot
// ring (the operation of Alg. 3 plus the cache update), and both in one launch.
//
// Both steps are HBM-bandwidth bound: every state / ring element is read once (and the state
// written once) per token, with 16-byte accesses that are contiguous across lanes.  Nothing is
// reused within a step, so rows go HBM -> registers directly; LDS only carries the expanded
// features, the softmax scores and the cross-wave partial sums.
#include "common.h"

#include <atomic>

namespace based {

constexpr int kDecodeThreads = 256;

__device__ __forceinline__ int resolve_pos(const PosArg &p, int u)
{
    return p.per_seq ? p.per_seq[u / p.H] : p.pos;
}

// y of a sequence that does not take part in the step
template <typename T>
__device__ __forceinline__ void zero_row(T *y, int n)
{
    for (int i = threadIdx.x; i < n; i += kDecodeThreads) y[i] = from_f32<T>(0.f);
}

// ---------------------------------------------------------------------------------------------
// Linear attention: z += phi(k); S += phi(k) v^T; y = phi(q) S / (phi(q).z)      one unit / block
// ---------------------------------------------------------------------------------------------
// PACKED: the state holds one row per unordered feature pair (packed_feature_dim rows); the k side
// of a pair row is k_a k_b / sqrt(2) (the canonical row), the q side sqrt(2) q_a q_b for a < b (the
// pair occurs twice in the sum over ordered pairs) and q_a^2 / sqrt(2) for a = b.
template <int DP, int DV, typename T, bool PACKED>
__device__ __forceinline__ void decode_step_body(const T *__restrict__ q, const T *__restrict__ k,
                                                 const T *__restrict__ v, T *__restrict__ y,
                                                 float *__restrict__ state, int u,
                                                 bool numerator_only = false, float gm = 1.f, float gate = 1.f)
{
    constexpr int D = PACKED ? packed_feature_dim(DP) : feature_dim(DP);
    constexpr int NT = kDecodeThreads;
    constexpr int LPR = DV / 4;      // lanes per state row (float4 each)
    constexpr int RPS = NT / LPR;    // rows per sweep step
    constexpr int STEPS = (D + RPS - 1) / RPS;
    constexpr int DPAD = STEPS * RPS;
    // State rows in flight per lane.  A narrow state (d_v = 64: 18 rows per lane) is fetched in one
    // round, so that a small batch, which cannot hide latency behind other workgroups, pays one trip
    // to memory; a wide one goes in rounds of 8 rows, each round fetched while the one before it is
    // worked on.
    constexpr int UNR = STEPS <= 20 ? STEPS : 8;
    constexpr int ROUNDS = (STEPS + UNR - 1) / UNR;
    constexpr int ZPT = (D + NT - 1) / NT;   // K-state features per thread

    __shared__ float pk[DPAD], pq[DPAD];
    __shared__ float qs[DP], ks[DP];
    __shared__ float yred[NT / 64][DV];
    __shared__ float dred[NT / 64];

    const int tid = threadIdx.x;
    float *Su = state + (size_t)u * (PACKED ? packed_state_stride(DP, DV) : state_stride(DP, DV));
    float *zu = Su + (size_t)D * DV;

    if (tid < DP) {
        qs[tid] = to_f32(q[(size_t)u * DP + tid]);
        ks[tid] = to_f32(k[(size_t)u * DP + tid]);
    }
    const int col4 = (tid % LPR) * 4, row = tid / LPR;
    float4 v4;
    {
        const T *vp = v + (size_t)u * DV + col4;
        v4 = make_float4(to_f32(vp[0]), to_f32(vp[1]), to_f32(vp[2]), to_f32(vp[3]));
    }
    // The state does not depend on the token: its first round and the K-state are requested now and
    // arrive while the features are expanded.  Rows past D re-read row D - 1 and are not used.
    float4 *Srow = reinterpret_cast<float4 *>(Su + col4);
    auto load_round = [&](int st0, float4 (&dst)[UNR]) {
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            const int f = min((st0 + j) * RPS + row, D - 1);
            dst[j] = Srow[(size_t)f * (DV / 4)];
        }
    };
    float4 sv[UNR];
    load_round(0, sv);
    float zv[ZPT];
#pragma unroll
    for (int i = 0; i < ZPT; ++i) zv[i] = zu[min(tid + i * NT, D - 1)];
    __syncthreads();
    // feature expansion (Eq. 4) in LDS; rows past D are zero so the tail of the sweep is inert
    for (int f = tid; f < DPAD; f += NT) {
        float a, b;
        if (f == 0) { a = 1.f; b = 1.f; }
        else if (f <= DP) { a = qs[f - 1]; b = ks[f - 1]; }
        else if (f < D) {
            int i, j;
            if (PACKED) {
                int t = f - 1 - DP;   // row i of the triangle holds the DP - i pairs (i, i .. DP - 1)
                i = 0;
                while (t >= DP - i) { t -= DP - i; ++i; }
                j = i + t;
            } else {
                i = (f - 1 - DP) / DP; j = (f - 1 - DP) % DP;
            }
            b = ks[i] * ks[j] * kRsqrt2;
            a = qs[i] * qs[j] * ((PACKED && i != j) ? 1.41421356237309504880f : kRsqrt2);
        } else { a = 0.f; b = 0.f; }
        pq[f] = a; pk[f] = b;
    }
    __syncthreads();

    // K-state: each feature handled by one thread
    float dpart = 0.f;
#pragma unroll
    for (int i = 0; i < ZPT; ++i) {
        const int f = tid + i * NT;
        if (f < D) {
            const float zn = fmaf(gm, zv[i], pk[f]);   // gm: the decay rate (1 without decay: exact)
            zu[f] = zn;
            dpart = fmaf(pq[f], zn, dpart);
        }
    }

    // one read-modify-write sweep over the KV-state, readout fused in
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    // A round whose rows all exist stores without a per-lane condition: stores that are certain to
    // be issued can be counted, so waiting for the next round's rows (requested before them) is not
    // also a wait for these stores to complete.
    auto work_round = [&](int st0, float4 (&cur)[UNR]) {
        const bool full = (st0 + UNR) * RPS <= D;
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            const int f = min((st0 + j) * RPS + row, DPAD - 1);   // features D .. DPAD - 1 are zero
            const float a = pk[f], b = pq[f];
            cur[j].x = fmaf(a, v4.x, gm * cur[j].x); cur[j].y = fmaf(a, v4.y, gm * cur[j].y);
            cur[j].z = fmaf(a, v4.z, gm * cur[j].z); cur[j].w = fmaf(a, v4.w, gm * cur[j].w);
            acc.x = fmaf(b, cur[j].x, acc.x); acc.y = fmaf(b, cur[j].y, acc.y);
            acc.z = fmaf(b, cur[j].z, acc.z); acc.w = fmaf(b, cur[j].w, acc.w);
        }
        if (full) {
#pragma unroll
            for (int j = 0; j < UNR; ++j) Srow[(size_t)((st0 + j) * RPS + row) * (DV / 4)] = cur[j];
        } else {
#pragma unroll
            for (int j = 0; j < UNR; ++j) {
                const int f = (st0 + j) * RPS + row;
                if (st0 + j < STEPS && f < D) Srow[(size_t)f * (DV / 4)] = cur[j];
            }
        }
    };
    if (ROUNDS == 1) {
        work_round(0, sv);
    } else {
        float4 sn[UNR];
#pragma unroll 1
        for (int r = 0; r < ROUNDS; r += 2) {
            if (r + 1 < ROUNDS) load_round((r + 1) * UNR, sn);
            work_round(r * UNR, sv);
            if (r + 1 < ROUNDS) {
                if (r + 2 < ROUNDS) load_round((r + 2) * UNR, sv);
                work_round((r + 1) * UNR, sn);
            }
        }
    }

    // rows are spread over the lanes above LPR within a wave, and over the waves
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
        acc.x += __shfl_xor(acc.x, o, 64); acc.y += __shfl_xor(acc.y, o, 64);
        acc.z += __shfl_xor(acc.z, o, 64); acc.w += __shfl_xor(acc.w, o, 64);
    }
    dpart = wave_sum(dpart);
    const int wv = tid >> 6, lane = tid & 63;
    if (lane < LPR) {
        yred[wv][col4 + 0] = acc.x; yred[wv][col4 + 1] = acc.y;
        yred[wv][col4 + 2] = acc.z; yred[wv][col4 + 3] = acc.w;
    }
    if (lane == 0) dred[wv] = dpart;
    __syncthreads();
    if (tid < DV) {
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) { num += yred[w][tid]; den += dred[w]; }
        y[(size_t)u * DV + tid] = from_f32<T>((numerator_only ? num : num / den) * gate);
    }
}

// ---------------------------------------------------------------------------------------------
// Sliding-window attention, one query against the ring                           one unit / block
// ---------------------------------------------------------------------------------------------
template <typename T> struct Chunk;  // 16 bytes of elements
template <> struct Chunk<float> {
    static constexpr int CE = 4;
    float4 raw;
    __device__ __forceinline__ float get(int i) const { return (&raw.x)[i]; }
    __device__ __forceinline__ void set(const float *a) { raw = make_float4(a[0], a[1], a[2], a[3]); }
};
template <> struct Chunk<bf16_t> {
    static constexpr int CE = 8;
    uint4 raw;
    __device__ __forceinline__ float get(int i) const
    {
        const uint32_t w = (&raw.x)[i >> 1];
        return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    __device__ __forceinline__ void set(const float *a)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            (&raw.x)[i] = (uint32_t)f32_to_bf16_bits(a[2 * i]) | ((uint32_t)f32_to_bf16_bits(a[2 * i + 1]) << 16);
    }
};

template <int DH, int W, typename T>
__device__ __forceinline__ void swa_decode_body(const T *__restrict__ q, const T *__restrict__ k,
                                                const T *__restrict__ v, T *__restrict__ y,
                                                T *__restrict__ ring, int pos, float scale, int u,
                                                bool ring_stream, const float2 *__restrict__ rot = nullptr,
                                                int rot_rows = 0)
{
    using Ch = Chunk<T>;
    constexpr int NT = kDecodeThreads;
    constexpr int CE = Ch::CE;
    constexpr int LPR = DH / CE;    // lanes per ring row
    constexpr int RPP = NT / LPR;   // ring rows per pass
    constexpr int PASSES = (W + RPP - 1) / RPP;   // a window below one pass leaves row groups idle
    static_assert(W % RPP == 0 || W < RPP, "window must be a multiple of the rows per pass, or below it");

    __shared__ float sc[PASSES * RPP];
    __shared__ float part[RPP][DH];

    const int tid = threadIdx.x;
    const int chunk = tid % LPR, rg = tid / LPR;
    const int slot = (pos - 1) % W;
    const int valid = pos < W ? pos : W;

    T *Kr = ring + (size_t)u * 2 * W * DH;
    T *Vr = Kr + (size_t)W * DH;

    // Every load is unconditional and issued up front (none depends on the scores): the token's own
    // q, k, v chunks, then the ring rows.  Rows the window does not hold yet re-read row 0 and are
    // zeroed, the row of this token's slot is replaced by the new k, v once the data is here.  (A
    // conditional load of the new row inside the sweep would wait for every ring row requested before it.)
    using Raw = decltype(Ch::raw);
    Ch qc, kc[PASSES], vc[PASSES], knew, vnew;
    qc.raw = *reinterpret_cast<const Raw *>(q + (size_t)u * DH + chunk * CE);
    knew.raw = *reinterpret_cast<const Raw *>(k + (size_t)u * DH + chunk * CE);
    vnew.raw = *reinterpret_cast<const Raw *>(v + (size_t)u * DH + chunk * CE);
    // rotary: the token sits at position pos - 1; its (cos, sin) pairs are requested with the rest
    float2 cs[CE / 2];
    if (rot) {
        const float2 *t = rot + (size_t)min(pos - 1, rot_rows - 1) * (DH / 2) + chunk * (CE / 2);
#pragma unroll
        for (int j = 0; j < CE / 2; ++j) cs[j] = t[j];
    }
    if (ring_stream) {
        // non-temporal: the ring is read once per step and should not push the state, which the next
        // step reads again, out of the last-level cache
        typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
        // (Two empty asm statements fence this branch: the compiler would otherwise hoist or sink these
        // loads together with the cached ones of the other branch into one sequence, which drops the
        // hint.  The first hides an offset of zero, the second names the last loaded value, which the
        // replacement of the token's own row needs next anyway.)
        int hidden_zero = 0;
        asm volatile("" : "+s"(hidden_zero));
        const T *Kn = Kr + hidden_zero, *Vn = Vr + hidden_zero;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int j = p * RPP + rg;
            const int jr = j < valid ? j : 0;
            kc[p].raw = __builtin_bit_cast(Raw, __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt *>(
                                                    Kn + (size_t)jr * DH + chunk * CE)));
            vc[p].raw = __builtin_bit_cast(Raw, __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt *>(
                                                    Vn + (size_t)jr * DH + chunk * CE)));
        }
        asm volatile("" : "+v"(vc[PASSES - 1].raw.x));
    } else {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int j = p * RPP + rg;
            const int jr = j < valid ? j : 0;
            kc[p].raw = *reinterpret_cast<const Raw *>(Kr + (size_t)jr * DH + chunk * CE);
            vc[p].raw = *reinterpret_cast<const Raw *>(Vr + (size_t)jr * DH + chunk * CE);
        }
    }
    if (rot) {
        // the ring holds rotated keys: the new key is rotated (and rounded to the ring's type) before it
        // is scored and stored
        rotate_chunk(qc, cs);
        rotate_chunk(knew, cs);
    }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int j = p * RPP + rg;
        if (j == slot) { kc[p].raw = knew.raw; vc[p].raw = vnew.raw; }
        else if (j >= valid) { kc[p].raw = Raw{}; vc[p].raw = Raw{}; }
    }
    // scores
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < CE; ++i) d = fmaf(qc.get(i), kc[p].get(i), d);
#pragma unroll
        for (int o = 1; o < LPR; o <<= 1) d += __shfl_xor(d, o, 64);
        if (chunk == 0) sc[p * RPP + rg] = d * scale;
    }
    __syncthreads();
    // softmax statistics (every wave computes the same numbers)
    const int lane = tid & 63;
    float m = -INFINITY;
    for (int j = lane; j < valid; j += 64) m = fmaxf(m, sc[j]);
    m = wave_max(m);
    float sum = 0.f;
    for (int j = lane; j < valid; j += 64) sum += __expf(sc[j] - m);
    sum = wave_sum(sum);
    // weighted sum of the value rows
    float acc[CE];
#pragma unroll
    for (int i = 0; i < CE; ++i) acc[i] = 0.f;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int j = p * RPP + rg;
        const float pj = j < valid ? __expf(sc[j] - m) : 0.f;
#pragma unroll
        for (int i = 0; i < CE; ++i) acc[i] = fmaf(pj, vc[p].get(i), acc[i]);
    }
#pragma unroll
    for (int i = 0; i < CE; ++i) part[rg][chunk * CE + i] = acc[i];
    __syncthreads();
    if (tid < DH) {
        float num = 0.f;
#pragma unroll
        for (int r = 0; r < RPP; ++r) num += part[r][tid];
        y[(size_t)u * DH + tid] = from_f32<T>(num / sum);
    }
    // cache update: the new row goes into its slot (the threads of that row group hold it)
    if (rg == slot % RPP) {
        *reinterpret_cast<Raw *>(Kr + (size_t)slot * DH + chunk * CE) = knew.raw;
        *reinterpret_cast<Raw *>(Vr + (size_t)slot * DH + chunk * CE) = vnew.raw;
    }
}

// ---------------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------------
template <int DP, int DV, typename T, bool PACKED>
__global__ __launch_bounds__(kDecodeThreads) void decode_step_kernel(const T *q, const T *k,
                                                                     const T *v, T *y, float *state,
                                                                     int reverse, int numerator_only,
                                                                     const float *gamma, const T *gate, int H)
{
    const int u = reverse ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
    // decay variant: a rate per head, an optional gate per (sequence, head)
    decode_step_body<DP, DV, T, PACKED>(q, k, v, y, state, u, numerator_only != 0, gamma ? gamma[u % H] : 1.f,
                                        gate ? to_f32(gate[u]) : 1.f);
}

template <int DH, int W, typename T>
__global__ __launch_bounds__(kDecodeThreads) void swa_decode_kernel(const T *q, const T *k,
                                                                    const T *v, T *y, T *ring,
                                                                    PosArg pa, float scale)
{
    const int u = blockIdx.x, pos = resolve_pos(pa, u);
    if (pos < 1) { zero_row(y + (size_t)u * DH, DH); return; }
    swa_decode_body<DH, W, T>(q, k, v, y, ring, pos, scale, u, pa.ring_stream != 0,
                              reinterpret_cast<const float2 *>(pa.rot), pa.rot_rows);
}

// Blocks [0, U) run the linear-attention step (the heavy one, scheduled first), blocks [U, 2U)
// the window attention step.  (Interleaving the two kinds block by block measured 15 % slower.)
// reverse: the units are walked from the last to the first.  Consecutive decode steps alternate the
// direction, so that a step starts with the state the step before it touched last, which is what
// the last-level cache still holds when the whole state does not fit (batch 192, d_v 128, 433 MB of
// state: 188 -> 149 us per fused step; neutral when it fits).
template <int DP, int DV, int DH, int W, typename T, bool PACKED>
__global__ __launch_bounds__(kDecodeThreads) void decode_fused_kernel(
    const T *q, const T *k, const T *v, T *y_lin, float *state, const T *sq, const T *sk,
    const T *sv, T *y_swa, T *ring, PosArg pa, float scale, int U, int reverse)
{
    const bool lin = (int)blockIdx.x < U;
    const int ub = lin ? blockIdx.x : blockIdx.x - U;
    const int u = reverse ? U - 1 - ub : ub;
    const int pos = resolve_pos(pa, u);
    if (pos < 1) {
        if (lin) zero_row(y_lin + (size_t)u * DV, DV);
        else zero_row(y_swa + (size_t)u * DH, DH);
        return;
    }
    if (lin)
        decode_step_body<DP, DV, T, PACKED>(q, k, v, y_lin, state, u);
    else
        swa_decode_body<DH, W, T>(sq, sk, sv, y_swa, ring, pos, scale, u, pa.ring_stream != 0,
                                  reinterpret_cast<const float2 *>(pa.rot), pa.rot_rows);
}

// ---------------------------------------------------------------------------------------------
// dispatch
// ---------------------------------------------------------------------------------------------
// head dim (64, 128) x window (16, 32, 64, 128)
#define BASED_PICK_SWA(DH, W, CALL)                               \
    do {                                                          \
        if (DH == 64) {                                           \
            if (W == 16) { CALL(64, 16); }                        \
            else if (W == 32) { CALL(64, 32); }                   \
            else if (W == 64) { CALL(64, 64); }                   \
            else { CALL(64, 128); }                               \
        } else {                                                  \
            if (W == 16) { CALL(128, 16); }                       \
            else if (W == 32) { CALL(128, 32); }                  \
            else if (W == 64) { CALL(128, 64); }                  \
            else { CALL(128, 128); }                              \
        }                                                         \
    } while (0)
#define BASED_PICK2(A, a0, a1, B, b0, b1, CALL)                  \
    do {                                                          \
        if (A == a0 && B == b0) { CALL(a0, b0); }                 \
        else if (A == a0 && B == b1) { CALL(a0, b1); }            \
        else if (A == a1 && B == b0) { CALL(a1, b0); }            \
        else { CALL(a1, b1); }                                    \
    } while (0)

// Direction of the sweep over the units.  For a state well beyond the 256 MB last-level cache it
// alternates from one launch of the process to the next; a state that fits, or nearly fits (batch 128,
// d_v 128: 288 MB), is served better by the cache as it is (85.3 against 90.6 us per state update).
static int next_direction(size_t state_bytes)
{
    static std::atomic<unsigned> calls{0};
    if (state_bytes <= ((size_t)340 << 20)) return 0;
    return (int)(calls.fetch_add(1, std::memory_order_relaxed) & 1u);
}
template <int DP, int DV> static size_t state_bytes_of(int U, int packed)
{
    return (size_t)U * (packed ? packed_state_stride(DP, DV) : state_stride(DP, DV)) * sizeof(float);
}

template <int DP, int DV, typename T>
static void step_pick(const void *q, const void *k, const void *v, void *y, float *state, int U,
                      int packed, int numer, const float *gamma, const void *gate, int H, hipStream_t s)
{
    const int reverse = next_direction(state_bytes_of<DP, DV>(U, packed));
    if (packed)
        hipLaunchKernelGGL((decode_step_kernel<DP, DV, T, true>), dim3(U), dim3(kDecodeThreads), 0, s,
                           (const T *)q, (const T *)k, (const T *)v, (T *)y, state, reverse, numer, gamma,
                           (const T *)gate, H);
    else
        hipLaunchKernelGGL((decode_step_kernel<DP, DV, T, false>), dim3(U), dim3(kDecodeThreads), 0, s,
                           (const T *)q, (const T *)k, (const T *)v, (T *)y, state, reverse, numer, gamma,
                           (const T *)gate, H);
}

hipError_t launch_decode_step(const void *q, const void *k, const void *v, void *y, float *state,
                              int U, int dp, int dv, int dtype, int packed, int numerator_only,
                              const float *gamma, const void *gate, int H, hipStream_t s)
{
#define CALL_LIN(DP_, DV_)                                                                        \
    if (dtype == BASED_F32) step_pick<DP_, DV_, float>(q, k, v, y, state, U, packed, numerator_only, gamma, gate, H, s); \
    else step_pick<DP_, DV_, bf16_t>(q, k, v, y, state, U, packed, numerator_only, gamma, gate, H, s)
    if (dp == 8 || dp == 24) BASED_PICK2(dp, 8, 24, dv, 64, 128, CALL_LIN);
    else BASED_PICK2(dp, 16, 32, dv, 64, 128, CALL_LIN);
#undef CALL_LIN
    return hipGetLastError();
}

hipError_t launch_swa_decode(const void *q, const void *k, const void *v, void *y, void *ring,
                             PosArg pos, int U, int dh, int w, float scale, int dtype, hipStream_t s)
{
#define CALL_SWA(DH_, W_)                                                                         \
    if (dtype == BASED_F32)                                                                       \
        hipLaunchKernelGGL((swa_decode_kernel<DH_, W_, float>), dim3(U), dim3(kDecodeThreads), 0, \
                           s, (const float *)q, (const float *)k, (const float *)v, (float *)y,   \
                           (float *)ring, pos, scale);                                            \
    else                                                                                          \
        hipLaunchKernelGGL((swa_decode_kernel<DH_, W_, bf16_t>), dim3(U), dim3(kDecodeThreads),   \
                           0, s, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,         \
                           (bf16_t *)y, (bf16_t *)ring, pos, scale)
    BASED_PICK_SWA(dh, w, CALL_SWA);
#undef CALL_SWA
    return hipGetLastError();
}

template <int DP, int DV, typename T, bool PACKED>
static void fused_pick(const void *q, const void *k, const void *v, void *y_lin, float *state,
                       const void *sq, const void *sk, const void *sv, void *y_swa, void *ring,
                       PosArg pos, int dh, int w, float scale, int U, hipStream_t s)
{
    const int reverse = next_direction(state_bytes_of<DP, DV>(U, PACKED ? 1 : 0));
#define CALL_F(DH_, W_)                                                                           \
    hipLaunchKernelGGL((decode_fused_kernel<DP, DV, DH_, W_, T, PACKED>), dim3(2 * U),            \
                       dim3(kDecodeThreads), 0, s, (const T *)q, (const T *)k, (const T *)v,      \
                       (T *)y_lin, state, (const T *)sq, (const T *)sk, (const T *)sv,            \
                       (T *)y_swa, (T *)ring, pos, scale, U, reverse)
    BASED_PICK_SWA(dh, w, CALL_F);
#undef CALL_F
}

hipError_t launch_decode_fused(const void *q, const void *k, const void *v, void *y_lin,
                               float *state, int dp, int dv, const void *sq, const void *sk,
                               const void *sv, void *y_swa, void *ring, PosArg pos, int dh, int w,
                               float scale, int U, int dtype, int packed, hipStream_t s)
{
    // A state that is re-read every step stays in the 256 MB last-level cache only as far as it fits.
    // When state and ring together exceed it, the ring (read once per step) is streamed past the cache
    // with non-temporal loads so that it does not evict state rows (batch 128, d_v 128: 111.8 -> 96.0 us
    // per step); when both fit (the packed state of that batch: 229 MB), cached ring reads are faster
    // (60.1 against 61.8 us).
    {
        const size_t esz = dtype == BASED_F32 ? 4 : 2;
        const size_t st = packed ? packed_state_stride(dp, dv) : state_stride(dp, dv);
        const size_t bytes = (size_t)U * (st * sizeof(float) + (size_t)2 * w * dh * esz);
        pos.ring_stream = bytes > ((size_t)256 << 20) ? 1 : 0;
    }
#define FUSED_ARGS q, k, v, y_lin, state, sq, sk, sv, y_swa, ring, pos, dh, w, scale, U, s
#define CALL_L(DP_, DV_)                                                                          \
    if (dtype == BASED_F32) {                                                                     \
        if (packed) fused_pick<DP_, DV_, float, true>(FUSED_ARGS);                                \
        else fused_pick<DP_, DV_, float, false>(FUSED_ARGS);                                      \
    } else {                                                                                      \
        if (packed) fused_pick<DP_, DV_, bf16_t, true>(FUSED_ARGS);                               \
        else fused_pick<DP_, DV_, bf16_t, false>(FUSED_ARGS);                                     \
    }
    BASED_PICK2(dp, 16, 32, dv, 64, 128, CALL_L);
#undef FUSED_ARGS
#undef CALL_L
    return hipGetLastError();
}

}  // namespace based
