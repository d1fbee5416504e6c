// Causal Taylor linear attention, prefill, all-fp32 vector-ALU kernel.
//
// Computes Eq. 2 (with the feature map of Eq. 4) through the recurrent view of Eq. 3, a few
// tokens at a time: the expanded features phi(q), phi(k) of a small token batch are built in
// LDS (never in HBM), the KV-state lives in registers spread over the workgroup, and each
// token's numerator and denominator are reduced across the workgroup through LDS.
//
// This is the exact-arithmetic path: it serves fp32 inputs (1e-4 class accuracy) and every
// supported size; the bf16 MFMA kernel takes over where it applies.
//
// Work split: one workgroup per (unit, 64-column slice of d_v, sequence segment).  Thread
// (c = tid % 64, r = tid / 64) owns column c of the slice and the feature rows
// [r * FPT, (r + 1) * FPT).  The K-state z is spread over all threads by feature (f = tid + NT * i).
//
// Long sequences on few units are cut into G segments that run side by side: a first launch
// computes each segment's state increment (the same loop without the readout), a small launch
// turns the increments into the state at the start of every segment (running sum, on top of the
// caller's initial state), and the main launch starts every segment from its entry.
#include "common.h"

namespace based {

template <int DP, int NT> struct RefCfg {
    static constexpr int D = feature_dim(DP);
    static constexpr int RG = NT / 64;                          // row groups (= waves)
    static constexpr int FPT = ((D + RG - 1) / RG + 3) / 4 * 4; // features per thread, mult of 4
    static constexpr int DPAD = RG * FPT;
    static constexpr int TB = DP <= 16 ? 8 : 4;                 // tokens per batch
    static constexpr int ZPT = (DPAD + NT - 1) / NT;
};

// Workspace entry of one (unit, slice, segment): S[D][64] then z[D], rounded up to 64 floats.
__host__ __device__ constexpr size_t ref_entry_floats(int dp)
{
    return ((size_t)feature_dim(dp) * 65 + 63) / 64 * 64;
}

// Decay variant (appendix paragraph on decay): a fixed rate per head multiplies the state at every token,
// S_i = gamma S_{i-1} + phi(k_i) v_i^T, z likewise; an optional gate [B][N][H] scales row i of y.
struct DecayArg {
    const float *gamma;   // [H], device; null: no decay
    const void *gate;     // [B][N][H] in the dtype of y, device; null: none
    int H;
};

// INCREMENT: state increment of the segment only (no readout), written to workspace entry 1 + seg.
// Otherwise: the full pass over the segment; with G > 1 it starts from workspace entry seg.
template <int DP, int NT, typename T, bool INCREMENT, bool DECAY>
__global__ __launch_bounds__(NT) void prefill_ref_kernel(const T *__restrict__ q,
                                                         const T *__restrict__ k,
                                                         const T *__restrict__ v,
                                                         T *__restrict__ y, float *state,
                                                         int has_init, int N, int dv, float *ws,
                                                         int seg_len, int G, DecayArg dk)
{
    using C = RefCfg<DP, NT>;
    constexpr int D = C::D, RG = C::RG, FPT = C::FPT, DPAD = C::DPAD, TB = C::TB, ZPT = C::ZPT;

    __shared__ __align__(16) float phiq[TB][DPAD];
    __shared__ __align__(16) float phik[TB][DPAD];
    __shared__ float qs[TB][DP], ks[TB][DP], vs[TB][64];
    __shared__ float red[TB][RG][64];
    __shared__ float redd[TB][RG];

    // has_init: bit 0 an initial state is given, bit 2 the outputs are the numerators alone
    const bool numerator_only = (has_init & 4) != 0;
    has_init &= 1;
    const int slices = dv / 64;
    const int gseg = INCREMENT ? G - 1 : G;
    const int seg = blockIdx.x % gseg, us = blockIdx.x / gseg;   // us = unit * slices + slice
    const int u = us / slices, col0 = (us % slices) * 64;
    const int tid = threadIdx.x, c = tid & 63, r = tid >> 6;
    const int tok_begin = seg * seg_len, tok_end = min(N, tok_begin + seg_len);
    float *ws_us = ws ? ws + (size_t)us * G * ref_entry_floats(DP) : nullptr;

    const T *qu = q + (size_t)u * N * DP, *ku = k + (size_t)u * N * DP;
    const T *vu = v + (size_t)u * N * dv + col0;
    T *yu = y + (size_t)u * N * dv + col0;
    float *Su = state ? state + (size_t)u * state_stride(DP, dv) : nullptr;
    float *zu = Su ? Su + (size_t)D * dv : nullptr;

    const float gm = DECAY ? dk.gamma[u % dk.H] : 1.f;
    const T *gate = DECAY && dk.gate ? static_cast<const T *>(dk.gate) + (size_t)(u / dk.H) * N * dk.H + (u % dk.H)
                                     : nullptr;
    float s[FPT], zreg[ZPT];
    if (!INCREMENT && G > 1) {
        // state at the start of this segment, prepared by the scan launch
        const float *e = ws_us + (size_t)seg * ref_entry_floats(DP);
#pragma unroll
        for (int i = 0; i < FPT; ++i) {
            const int f = r * FPT + i;
            s[i] = f < D ? e[(size_t)f * 64 + c] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < ZPT; ++i) {
            const int f = tid + NT * i;
            zreg[i] = f < D ? e[(size_t)D * 64 + f] : 0.f;
        }
    } else {
        const bool init = !INCREMENT && has_init;
#pragma unroll
        for (int i = 0; i < FPT; ++i) {
            const int f = r * FPT + i;
            s[i] = (init && f < D) ? Su[(size_t)f * dv + col0 + c] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < ZPT; ++i) {
            const int f = tid + NT * i;
            zreg[i] = (init && f < D) ? zu[f] : 0.f;
        }
    }

    for (int tok0 = tok_begin; tok0 < tok_end; tok0 += TB) {
        // (a) stage the token batch
        for (int idx = tid; idx < TB * DP; idx += NT) {
            const int t = idx / DP, a = idx % DP;
            const bool ok = tok0 + t < tok_end;
            qs[t][a] = ok ? to_f32(qu[(size_t)(tok0 + t) * DP + a]) : 0.f;
            ks[t][a] = ok ? to_f32(ku[(size_t)(tok0 + t) * DP + a]) : 0.f;
        }
        for (int idx = tid; idx < TB * 64; idx += NT) {
            const int t = idx >> 6, cc = idx & 63;
            vs[t][cc] = (tok0 + t < tok_end) ? to_f32(vu[(size_t)(tok0 + t) * dv + cc]) : 0.f;
        }
        __syncthreads();
        // (b) feature expansion, Eq. 4, into LDS
        for (int idx = tid; idx < TB * DPAD; idx += NT) {
            const int t = idx / DPAD, f = idx % DPAD;
            const bool ok = tok0 + t < tok_end;
            float pq, pk;
            if (f == 0) {
                pq = 1.f; pk = 1.f;
            } else if (f <= DP) {
                pq = qs[t][f - 1]; pk = ks[t][f - 1];
            } else if (f < D) {
                const int a = (f - 1 - DP) / DP, b = (f - 1 - DP) % DP;
                pq = qs[t][a] * qs[t][b] * kRsqrt2;
                pk = ks[t][a] * ks[t][b] * kRsqrt2;
            } else {
                pq = 0.f; pk = 0.f;
            }
            phiq[t][f] = pq;
            phik[t][f] = ok ? pk : 0.f;  // tokens past the end must not touch the state
        }
        __syncthreads();
        // (c) state update fused with readout, token by token (Eq. 3)
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            const float vt = vs[t][c];
            // (a token past the end of the segment must leave the state as it is: no decay for it either)
            const float gt = (DECAY && tok0 + t < tok_end) ? gm : 1.f;
            const float4 *pk4 = reinterpret_cast<const float4 *>(&phik[t][r * FPT]);
            const float4 *pq4 = reinterpret_cast<const float4 *>(&phiq[t][r * FPT]);
            float num = 0.f;
#pragma unroll
            for (int i = 0; i < FPT / 4; ++i) {
                const float4 a = pk4[i], b = pq4[i];
                if (DECAY) {
                    s[4 * i + 0] *= gt; s[4 * i + 1] *= gt; s[4 * i + 2] *= gt; s[4 * i + 3] *= gt;
                }
                s[4 * i + 0] = fmaf(a.x, vt, s[4 * i + 0]); num = fmaf(b.x, s[4 * i + 0], num);
                s[4 * i + 1] = fmaf(a.y, vt, s[4 * i + 1]); num = fmaf(b.y, s[4 * i + 1], num);
                s[4 * i + 2] = fmaf(a.z, vt, s[4 * i + 2]); num = fmaf(b.z, s[4 * i + 2], num);
                s[4 * i + 3] = fmaf(a.w, vt, s[4 * i + 3]); num = fmaf(b.w, s[4 * i + 3], num);
            }
            if (INCREMENT) {
                // Update only.  The readout sum above is kept alive (and thrown away): without it the
                // compiler fetches whole feature rows ahead of the updates and spills the state.
                asm volatile("" : : "v"(num));
#pragma unroll
                for (int i = 0; i < ZPT; ++i) {
                    const int f = tid + NT * i;
                    if (f < DPAD) zreg[i] = (DECAY ? gt * zreg[i] : zreg[i]) + phik[t][f];
                }
                continue;
            }
            red[t][r][c] = num;
            float dpart = 0.f;
#pragma unroll
            for (int i = 0; i < ZPT; ++i) {
                const int f = tid + NT * i;
                if (f < DPAD) {
                    zreg[i] = (DECAY ? gt * zreg[i] : zreg[i]) + phik[t][f];
                    dpart = fmaf(phiq[t][f], zreg[i], dpart);
                }
            }
            dpart = wave_sum(dpart);
            if (c == 0) redd[t][r] = dpart;
        }
        __syncthreads();
        // (d) reduce over row groups, normalise, store
        for (int idx = tid; !INCREMENT && idx < TB * 64; idx += NT) {
            const int t = idx >> 6, cc = idx & 63;
            if (tok0 + t < tok_end) {
                float num = 0.f, den = 0.f;
#pragma unroll
                for (int g = 0; g < RG; ++g) { num += red[t][g][cc]; den += redd[t][g]; }
                float o = numerator_only ? num : num / den;
                if (DECAY && gate) o *= to_f32(gate[(size_t)(tok0 + t) * dk.H]);
                yu[(size_t)(tok0 + t) * dv + cc] = from_f32<T>(o);
            }
        }
        __syncthreads();
    }

    if (INCREMENT) {
        float *e = ws_us + (size_t)(1 + seg) * ref_entry_floats(DP);
#pragma unroll
        for (int i = 0; i < FPT; ++i) {
            const int f = r * FPT + i;
            if (f < D) e[(size_t)f * 64 + c] = s[i];
        }
#pragma unroll
        for (int i = 0; i < ZPT; ++i) {
            const int f = tid + NT * i;
            if (f < D) e[(size_t)D * 64 + f] = zreg[i];
        }
    } else if (Su && seg == G - 1) {
#pragma unroll
        for (int i = 0; i < FPT; ++i) {
            const int f = r * FPT + i;
            if (f < D) Su[(size_t)f * dv + col0 + c] = s[i];
        }
        if (col0 == 0) {
#pragma unroll
            for (int i = 0; i < ZPT; ++i) {
                const int f = tid + NT * i;
                if (f < D) zu[f] = zreg[i];
            }
        }
    }
}

// Entry 0 <- the caller's initial state (or zero); entry g <- gamma^(tokens of segment g - 1) x entry g - 1 +
// increment g - 1 (gamma = 1 without decay).
// grid: (unit slices, blocks over the elements of an entry)
__global__ void prefill_ref_scan_kernel(float *ws, const float *state, int has_init, int dp, int dv,
                                        int G, int seg_len, DecayArg dk)
{
    const int D = feature_dim(dp), slices = dv / 64;
    const int us = blockIdx.x, u = us / slices, col0 = (us % slices) * 64;
    const size_t E = ref_entry_floats(dp);
    float *e = ws + (size_t)us * G * E;
    const float *Su = state ? state + (size_t)u * state_stride(dp, dv) : nullptr;
    const int nS = D * 64;
    const float gseg = dk.gamma ? powf(dk.gamma[u % dk.H], (float)seg_len) : 1.f;   // every segment but the last is seg_len long
    for (int i = blockIdx.y * blockDim.x + threadIdx.x; i < nS + D; i += gridDim.y * blockDim.x) {
        float acc = 0.f;
        if (has_init) acc = i < nS ? Su[(size_t)(i / 64) * dv + col0 + (i % 64)] : Su[(size_t)D * dv + (i - nS)];
        e[i] = acc;
        for (int g = 1; g < G; ++g) {
            acc = fmaf(acc, gseg, e[(size_t)g * E + i]);
            e[(size_t)g * E + i] = acc;
        }
    }
}

namespace {

// Segments: enough workgroups for four per CU, segments of at least 256 tokens, at most 32.
int ref_segments(int U, int N, int dv)
{
    const long groups = (long)U * (dv / 64);
    int G = (int)((1024 + groups - 1) / groups);
    if (G > N / 256) G = N / 256;
    if (G > 32) G = 32;
    return G < 1 ? 1 : G;
}

int ref_segment_len(int N, int G) { return ((N + G - 1) / G + 63) / 64 * 64; }

}  // namespace

size_t prefill_ref_workspace_bytes(int U, int N, int dp, int dv)
{
    const int G = ref_segments(U, N, dv);
    return G > 1 ? (size_t)U * (dv / 64) * G * ref_entry_floats(dp) * sizeof(float) : 0;
}

template <int DP, int NT, typename T, bool DECAY>
static hipError_t launch_ref(const void *q, const void *k, const void *v, void *y, float *state,
                             int has_init, void *workspace, int U, int N, int dv, DecayArg dk, hipStream_t s)
{
    const int groups = U * (dv / 64);
    int G = ref_segments(U, N, dv);
    const int seg_len = ref_segment_len(N, G);
    while (G > 1 && (G - 1) * seg_len >= N) --G;   // rounding the length up can empty trailing segments
    float *ws = static_cast<float *>(workspace);
    hipError_t e;
    if (G > 1) {
        hipLaunchKernelGGL((prefill_ref_kernel<DP, NT, T, true, DECAY>), dim3((unsigned)(groups * (G - 1))), dim3(NT),
                           0, s, (const T *)q, (const T *)k, (const T *)v, (T *)y, state, has_init, N, dv, ws,
                           seg_len, G, dk);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(prefill_ref_scan_kernel, dim3((unsigned)groups, 32), dim3(256), 0, s, ws, state, has_init & 1,
                           DP, dv, G, seg_len, dk);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    hipLaunchKernelGGL((prefill_ref_kernel<DP, NT, T, false, DECAY>), dim3((unsigned)(groups * G)), dim3(NT), 0, s,
                       (const T *)q, (const T *)k, (const T *)v, (T *)y, state, has_init, N, dv, ws, seg_len, G, dk);
    return hipGetLastError();
}

template <bool DECAY>
static hipError_t launch_ref_any(const void *q, const void *k, const void *v, void *y, float *state, int has_init,
                                 void *workspace, int U, int N, int dp, int dv, int dtype, DecayArg dk,
                                 hipStream_t s)
{
#define REF_CASE(DP_, NT_)                                                                                      \
    if (dp == DP_)                                                                                              \
        return dtype == BASED_F32                                                                               \
                   ? launch_ref<DP_, NT_, float, DECAY>(q, k, v, y, state, has_init, workspace, U, N, dv, dk, s) \
                   : launch_ref<DP_, NT_, bf16_t, DECAY>(q, k, v, y, state, has_init, workspace, U, N, dv, dk, s)
    REF_CASE(8, 256);
    REF_CASE(16, 256);
    REF_CASE(24, 512);
    REF_CASE(32, 512);
#undef REF_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_prefill_ref(const void *q, const void *k, const void *v, void *y, float *state,
                              int has_init, void *workspace, int U, int N, int dp, int dv, int dtype,
                              hipStream_t s)
{
    return launch_ref_any<false>(q, k, v, y, state, has_init, workspace, U, N, dp, dv, dtype, DecayArg{nullptr, nullptr, 1}, s);
}

hipError_t launch_prefill_ref_decay(const void *q, const void *k, const void *v, void *y, float *state,
                                    int has_init, void *workspace, const float *gamma, const void *gate, int H,
                                    int U, int N, int dp, int dv, int dtype, hipStream_t s)
{
    return launch_ref_any<true>(q, k, v, y, state, has_init, workspace, U, N, dp, dv, dtype, DecayArg{gamma, gate, H}, s);
}

}  // namespace based
