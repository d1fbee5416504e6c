// Shared device helpers for the Based HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/based.h"

namespace based {

constexpr float kRsqrt2 = 0.70710678118654752440f;

// Element types of q/k/v/y.  bf16 is carried as raw 16-bit patterns.
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }

// fp32 -> bf16 with the hardware conversion (v_cvt_pk_bf16_f32: round to nearest even, NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x)
{
    bf16_t r;
    r.bits = f32_to_bf16_bits(x);
    return r;
}

__host__ __device__ constexpr int feature_dim(int dp) { return 1 + dp + dp * dp; }
__host__ __device__ constexpr size_t state_stride(int dp, int dv)
{
    return ((size_t)feature_dim(dp) * dv + feature_dim(dp) + 63) / 64 * 64;
}

// Packed state variant: one row per unordered feature pair (the rows (a, b) and (b, a) of Eq. 4 are
// equal).  Row 0 constant, 1 + a linear, 1 + d' + tri(a, b) for a <= b with
// tri(a, b) = a d' - a (a - 1) / 2 + (b - a); the stored value is the canonical row (a, b).
__host__ __device__ constexpr int packed_feature_dim(int dp) { return 1 + dp + dp * (dp + 1) / 2; }
__host__ __device__ constexpr size_t packed_state_stride(int dp, int dv)
{
    return ((size_t)packed_feature_dim(dp) * dv + packed_feature_dim(dp) + 63) / 64 * 64;
}
__host__ __device__ constexpr int packed_pair_row(int dp, int a, int b)   // a <= b
{
    return 1 + dp + a * dp - a * (a - 1) / 2 + (b - a);
}

// Sum over the 64 lanes of a wave; every lane gets the total.
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

// Rotary encoding of one 16-byte chunk of a q or k row (CE / 2 adjacent pairs): pair j becomes
// (x0 cos - x1 sin, x0 sin + x1 cos) with (cos, sin) = t[j], the table entries of the row's position and of
// the chunk's pairs.  Chunk: get(i), set(float[CE]), CE.
template <typename Chunk> __device__ __forceinline__ void rotate_chunk(Chunk &c, const float2 *t)
{
    float o[Chunk::CE];
#pragma unroll
    for (int j = 0; j < Chunk::CE / 2; ++j) {
        const float2 cs = t[j];
        const float x0 = c.get(2 * j), x1 = c.get(2 * j + 1);
        o[2 * j] = fmaf(x0, cs.x, -x1 * cs.y);
        o[2 * j + 1] = fmaf(x0, cs.y, x1 * cs.x);
    }
    c.set(o);
}

// ---- launchers implemented in the kernel translation units ---------------------------------
// Each returns a hipError_t from the launch (hipGetLastError), never synchronises.
hipError_t launch_prefill_ref(const void *q, const void *k, const void *v, void *y, float *state,
                              int has_init, void *workspace, int U, int N, int dp, int dv, int dtype,
                              hipStream_t s);
size_t prefill_ref_workspace_bytes(int U, int N, int dp, int dv);
bool prefill_mfma_supported(int dp, int dv, int dtype);
size_t prefill_mfma_workspace_bytes(int U, int N, int dp, int dv);
// packed_state != 0: the state buffer is the packed layout (one row per unordered feature pair);
// status: the sticky word a workgroup sets when it gives up waiting for a segment's ready flag
hipError_t launch_prefill_mfma(const void *q, const void *k, const void *v, void *y, float *state,
                               int has_init, int packed_state, void *workspace, unsigned *status, int U, int N,
                               int dp, int dv, hipStream_t s);
// where the ready flags sit inside a workspace of prefill_mfma_workspace_bytes
void prefill_mfma_flags_region(int U, int N, int dp, int dv, size_t *offset, size_t *bytes);
// bound on the polls of one flag for later launches (negative: the default); a testing hook
void prefill_mfma_set_poll_limit(int polls);
bool prefill_mfma32_supported(int dp, int dv, int dtype);
size_t prefill_mfma32_workspace_bytes(int U, int N, int dp, int dv);
hipError_t launch_prefill_mfma32(const void *q, const void *k, const void *v, void *y, float *state,
                                 int has_init, int packed_state, void *workspace, int U, int N, int dp, int dv,
                                 hipStream_t s);
// numerator_only != 0: y is phi(q) S without the division by phi(q).z
// gamma [H] (device, or null): per-head decay of the state; gate [U] in the dtype of y (or null): scales y
hipError_t launch_decode_step(const void *q, const void *k, const void *v, void *y, float *state,
                              int U, int dp, int dv, int dtype, int packed, int numerator_only,
                              const float *gamma, const void *gate, int H, hipStream_t s);
// the fp32 vector kernel with a per-head decay gamma [H] and an optional gate [B][N][H] in the dtype of y
hipError_t launch_prefill_ref_decay(const void *q, const void *k, const void *v, void *y, float *state,
                                    int has_init, void *workspace, const float *gamma, const void *gate, int H,
                                    int U, int N, int dp, int dv, int dtype, hipStream_t s);
// rot (everywhere below): the rotary table, (cos, sin) per [position][pair], row 0 = the first token of
// the call (prefill) or position 0 of the sequence (decode); null = no rotation
hipError_t launch_rotary_table(float *table, int pos0, int N, int dh, float base, hipStream_t s);
hipError_t launch_swa_prefill_ref(const void *q, const void *k, const void *v, void *y, const float *rot, int U,
                                  int N, int dh, int w, float scale, int dtype, hipStream_t s);
bool swa_prefill_mfma_supported(int dh, int w, int dtype, int rotary);
hipError_t launch_swa_prefill_mfma(const void *q, const void *k, const void *v, void *y, void *ring,
                                   const float *rot, int U, int N, int dh, int w, float scale, hipStream_t s);
// the same with 16 queries to a wave (two workgroups per CU); no rotary variant
bool swa_prefill_mfma16_supported(int dh, int w, int dtype);
hipError_t launch_swa_prefill_mfma16(const void *q, const void *k, const void *v, void *y, void *ring, int U, int N,
                                     int dh, int w, float scale, hipStream_t s);
hipError_t launch_swa_ring_fill(const void *k, const void *v, void *ring, const float *rot, int U, int N, int dh,
                                int w, int dtype, hipStream_t s);
// Position of the decoded token: one value for every sequence, or (per_seq != NULL) one per batch
// element in device memory, where a value < 1 marks a sequence that does not take part in the step.
struct PosArg {
    int pos;
    const int *per_seq;
    int H;
    int ring_stream;   // set by the fused launcher: read the ring with non-temporal loads (see there)
    const float *rot;  // rotary table from position 0 (null: none); the token at position pos - 1 uses row pos - 1
    int rot_rows;      // rows in it (a position beyond the table uses its last row)
};
hipError_t launch_swa_decode(const void *q, const void *k, const void *v, void *y, void *ring,
                             PosArg pos, int U, int dh, int w, float scale, int dtype, hipStream_t s);
hipError_t launch_decode_fused(const void *q, const void *k, const void *v, void *y_lin,
                               float *state, int dp, int dv, const void *sq, const void *sk,
                               const void *sv, void *y_swa, void *ring, PosArg pos, int dh, int w,
                               float scale, int U, int dtype, int packed, hipStream_t s);
hipError_t launch_state_copy(float *state, float *S, float *z, int U, int dp, int dv, int to_state,
                             hipStream_t s);
// canonical state buffer <-> packed state buffer (to_packed: symmetric part; else both rows of a pair)
hipError_t launch_state_repack(float *state, float *packed, int U, int dp, int dv, int to_packed,
                               hipStream_t s);
hipError_t launch_positions_advance(int *pos, int B, hipStream_t s);
// BaseConv gate: out = (a + b1) * silu(causal 3-tap conv of c + b2); c_prev / c_last: the two rows before /
// at the end of the sequence (either may be null)
bool short_conv_gate_supported(int Dc, int dtype);
int short_conv_gate_run();   // tokens one thread walks: c_last may alias c_prev only for N up to this
hipError_t launch_short_conv_gate(const void *a, const void *c, const float *h, const float *b1, const float *b2,
                                  const void *c_prev, void *out, void *c_last, int B, int N, int Dc, int dtype,
                                  hipStream_t s);
bool linear_supported(int M, int K, int N, int dtype);
hipError_t launch_linear(const void *x, const void *W, void *y, int M, int K, int N, hipStream_t s);
// x [B seq_len][K] times W [H (2 d' + d_v)][K] (rows: q heads, k heads, v heads) into head-major q, k, v
bool project_qkv_supported(int K, int H, int d_feat, int d_v, int dtype);
hipError_t launch_project_qkv(const void *x, const void *W, void *q, void *k, void *v, int B, int seq_len, int K,
                              int H, int d_feat, int d_v, hipStream_t s);
// head-major mixer output [B][H][seq_len][d_v] times W [N][H d_v] into token-major [B seq_len][N]
bool project_out_supported(int H, int d_v, int N, int dtype);
hipError_t launch_project_out(const void *y_heads, const void *W, void *out, int B, int seq_len, int H, int d_v,
                              int N, hipStream_t s);

}  // namespace based
