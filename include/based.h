/*
 * based.h -- C ABI of the MI355X (gfx950) hot path of the Based sequence mixer
 * (arXiv 2402.18668): causal linear attention with the 2nd-order Taylor feature map,
 * and small-window causal softmax attention, for prefill and for per-token decode.
 *
 * General contract (all entry points)
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or keeps device memory.  Its only process-wide state is two launch
 *     counters (one of segmented prefill calls, used to tag the ready flags it keeps in the
 *     caller's workspace, and one of decode launches on states far larger than the last-level
 *     cache, which alternates the order in which such a launch walks the units; results do
 *     not depend on either) and the poll limit of based_debug_set_poll_limit.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on it and never synchronise; buffers must stay alive until the work
 *     has run.
 *   - Return value: BASED_OK or an error code.  BASED_ERR_INVALID_ARG and BASED_ERR_UNSUPPORTED are
 *     decided on the host before anything is launched.  BASED_ERR_LAUNCH means the HIP runtime
 *     refused a launch; a call that consists of several launches (based_prefill can be up to
 *     three) may then have enqueued the earlier ones, and its outputs are unspecified.
 *     Nothing aborts or throws.
 *   - Tensors are contiguous, last index fastest, base pointers 16-byte aligned.
 *     A "unit" is one (batch, head) pair; units are independent, u = b * H + h.
 *   - dtype selects the element type of q, k, v, y (and of the window ring):
 *     BASED_F32 or BASED_BF16.  All accumulation and the recurrent state are fp32.
 *     Outputs are rounded to dtype with round-to-nearest-even.
 *   - Supported sizes: d_feat in {8, 16, 24, 32} (the feature dimensions of the ablation table;
 *     16 and 32 have matrix-core prefill kernels for bf16, 8 and 24 run on the fp32 vector kernel
 *     for both dtypes; the packed-state prefill and the fused decode step exist for 16 and 32
 *     only); d_v, d_h in {64, 128}; w in {16, 32, 64, 128}; any B, H, N >= 1 with
 *     B * H * N < 2^31.  Anything else: BASED_ERR_UNSUPPORTED.
 *
 * Notation follows the paper: d' = d_feat is the projected feature dimension of q and k,
 * D = 1 + d' + d'^2 the expanded feature dimension (Sec. 4), d_v the value dimension.
 * Feature order (Eq. 4): phi(x) = [1, x_0..x_{d'-1}, x_a x_b / sqrt(2) at 1 + d' + a d' + b].
 * No temperature is applied inside the linear-attention calls: the kernel evaluated is
 * exactly 1 + q.k + (q.k)^2 / 2; a caller who wants exp(q.k / sqrt(d')) approximated
 * scales q and k by d'^(-1/4) beforehand.
 */
#ifndef BASED_H
#define BASED_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    BASED_OK = 0,
    BASED_ERR_INVALID_ARG = 1, /* null / misaligned pointer, non-positive size, bad pos */
    BASED_ERR_UNSUPPORTED = 2, /* size or dtype outside the supported set               */
    BASED_ERR_TOO_LARGE = 4,   /* based_prefill_static: needs more than the static scratch   */
    BASED_ERR_LAUNCH = 3       /* the HIP runtime refused the launch, or (based_prefill_status)
                                  a launch gave up a bounded wait and its outputs are invalid */
};

enum { BASED_F32 = 0, BASED_BF16 = 1 };

/* Human-readable text for a status code (static storage, never NULL). */
const char *based_strerror(int status);

/* Library version, major * 100 + minor. */
int based_version(void);

/* D = 1 + d' + d'^2 (Sec. 4), or 0 if d_feat < 1. */
int based_feature_dim(int d_feat);

/*
 * Recurrent state of linear attention (Sec. 3.1, Eq. 3): the KV-state s = sum_j phi(k_j) v_j^T
 * and the K-state z = sum_j phi(k_j), fp32.
 *
 * Device layout of a state buffer: for each unit u, at float offset u * stride,
 *   S[D][d_v] (row f = feature, in the feature order above) followed by z[D];
 *   stride = D * d_v + D rounded up to a multiple of 64 floats (the tail is padding).
 * based_state_bytes returns B * H * stride * 4, or 0 for unsupported sizes.
 * based_state_stride_floats returns stride.
 */
size_t based_state_bytes(int B, int H, int d_feat, int d_v);
size_t based_state_stride_floats(int d_feat, int d_v);

/*
 * Copy between a state buffer and the canonical dense arrays S [B][H][D][d_v] and
 * z [B][H][D] (fp32, device).  Either of S, z may be NULL to skip it.
 */
int based_state_export(const void *state, float *S, float *z, int B, int H, int d_feat, int d_v,
                       void *stream);
int based_state_import(void *state, const float *S, const float *z, int B, int H, int d_feat,
                       int d_v, void *stream);

/*
 * based_prefill -- causal Taylor linear attention over whole sequences (Eq. 2 with the feature
 * map of Eq. 4), computed in the chunked form of Sec. 4: inside a chunk of tokens the masked
 * quadratic product, across chunks the running state (Eq. 3).
 *
 *   y_i = sum_{j<=i} kappa(q_i, k_j) v_j / sum_{j<=i} kappa(q_i, k_j),
 *   kappa(q, k) = phi(q).phi(k) = 1 + q.k + (q.k)^2 / 2,
 * plus, with an initial state (S0, z0): numerator + phi(q_i) S0, denominator + phi(q_i).z0.
 *
 *   q, k   [B][H][N][d_feat]   in,  dtype
 *   v      [B][H][N][d_v]      in,  dtype
 *   y      [B][H][N][d_v]      out, dtype
 *   state  state buffer (layout above) or NULL.  has_init != 0: read as (S0, z0) (must be
 *          non-NULL).  If non-NULL it receives the state after the last token.
 *          A state of this recurrence has equal rows for the feature pairs (a, b) and (b, a)
 *          (x_a x_b = x_b x_a in Eq. 4), and y depends only on their sum.  The bf16 paths
 *          carry one row per unordered pair: it reads an initial state as the mean of
 *          the two rows and writes both rows equal.  For a state produced by this library, or
 *          imported from the canonical arrays of such a state, that changes nothing.
 *   workspace  scratch of at least based_prefill_workspace_bytes(...) bytes, 256-byte aligned;
 *          may be NULL when that size is 0 (it never is for bf16).  It must be zero-filled ONCE
 *          after it is allocated; after that the library maintains it, and calls may reuse it
 *          without clearing.  For few units and long sequences the sequence is cut into segments
 *          that run side by side; state increments of the segments travel through the workspace.
 *          At d' = 16 (bf16) that is one launch, in which a workgroup waits for the increments of
 *          the segments before its own with a bounded number of polls (about a quarter of a
 *          second per increment).  A launch therefore always terminates; a workgroup that gives
 *          up sets a sticky status word in the workspace and carries on with incomplete data:
 *          y and the final state of that call are then INVALID although based_prefill itself
 *          returned BASED_OK (it returns when the work is enqueued).  based_prefill_status
 *          reports it.  The wait cannot time out as long as the device starts the workgroups of
 *          a launch in grid order (the workgroups waited for come first in the grid and wait for
 *          nothing), which is how the hardware dispatcher works but is not a documented promise.
 *
 * Calls sharing a workspace or a state buffer must be ordered on one stream.
 *
 * based_prefill_status -- did a based_prefill / based_prefill_packed call that used this workspace
 * give up a bounded wait?  Same size arguments as the call it asks about.  It waits for `stream`
 * (hipStreamSynchronize) and reads the status word back, so it is a host-synchronous call and
 * must not be made while the stream is being captured.  BASED_OK: no launch since the last query
 * gave up.  BASED_ERR_LAUNCH: at least one did (outputs of those calls are invalid); the query
 * also clears the status word and the ready flags, after which the workspace can be used again.
 * Without a query, eager calls after a failed one are still correct (every call tags its flags
 * with a new epoch); a replayed graph repeats its epoch and needs the query's clean-up first.
 * Configurations whose prefill has no such waits (fp32, d' = 32) always give BASED_OK.
 *
 * based_debug_set_poll_limit -- testing hook: the bound on the polls of one ready flag for later
 * calls in this process (negative: back to the default).  With 0 a waiting workgroup gives up at
 * once, which lets a test drive the error path while every workgroup still exits normally.
 */
size_t based_prefill_workspace_bytes(int B, int H, int N, int d_feat, int d_v, int dtype);
int based_prefill(const void *q, const void *k, const void *v, void *y, void *state, int has_init,
                  void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype,
                  void *stream);
int based_prefill_status(void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype,
                         void *stream);
void based_debug_set_poll_limit(int polls);

/*
 * based_prefill_static -- based_prefill for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as based_prefill without the workspace: the scratch is a device array of
 * BASED_STATIC_SCRATCH_BYTES that lives inside the library (one copy per GPU, held from the
 * moment the library's code is loaded on that GPU until the process ends).  The call allocates
 * and frees nothing, on the host or on the device.
 *   Errors: as based_prefill; BASED_ERR_TOO_LARGE when based_prefill_workspace_bytes(...) of the
 *   sizes exceeds BASED_STATIC_SCRATCH_BYTES (nothing is launched); BASED_ERR_LAUNCH also when
 *   the address of the scratch cannot be obtained.
 *   All calls on one GPU share that GPU's scratch, whatever their stream: calls that may overlap
 *   in time race on it and give wrong results; order them on one stream (or with events).  The
 *   scratch keeps the last call's contents; nothing in it needs clearing between calls.
 *   based_prefill_status with workspace = NULL asks about the calls made through this entry point
 *   on the current device.
 */
#define BASED_STATIC_SCRATCH_BYTES (64u << 20)
int based_prefill_static(const void *q, const void *k, const void *v, void *y, void *state,
                         int has_init, int B, int H, int N, int d_feat, int d_v, int dtype,
                         void *stream);

/*
 * based_decode_step -- one token of the recurrent view (Eq. 3), state update fused with
 * readout (the operation of Alg. 2, here including the K-state and the division):
 *   z += phi(k);  S += phi(k) v^T;  y = phi(q) S / (phi(q).z)
 * The token is added to the state before it is read (it attends to itself).
 *
 *   q, k   [B][H][d_feat]  in, dtype        v  [B][H][d_v]  in, dtype
 *   y      [B][H][d_v]     out, dtype       state  in-out (layout above)
 */
int based_decode_step(const void *q, const void *k, const void *v, void *y, void *state, int B,
                      int H, int d_feat, int d_v, int dtype, void *stream);

/*
 * Numerator-only variants: what Alg. 1 (prefill) and Alg. 2 (recurrent update) compute as printed,
 * and what the paper's kernel micro-benchmarks time (the captions of the two timing figures say
 * they cover the numerator of the linear attention).  Same arguments, layouts, state handling and
 * error behaviour as based_prefill / based_decode_step; the only difference is the output:
 *   y_i = sum_{j<=i} kappa(q_i, k_j) v_j  (+ phi(q_i) S0 with an initial state),
 * without the division by sum_{j<=i} kappa(q_i, k_j).  The K-state z is still maintained, so a
 * state can be handed between the two kinds of call.  The magnitude of y grows with the number of
 * tokens seen; in bf16 it is rounded like any other output.
 */
int based_prefill_numerator(const void *q, const void *k, const void *v, void *y, void *state, int has_init,
                            void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype,
                            void *stream);
int based_decode_step_numerator(const void *q, const void *k, const void *v, void *y, void *state, int B,
                                int H, int d_feat, int d_v, int dtype, void *stream);

/*
 * Decay variant (appendix paragraph on decay; the main experiments use none, the ablation table has a
 * row for it).  That paragraph describes a fixed decay rate per head and a learned projection of the
 * layer input to one scalar per (token, head) that weights the heads when they are combined; it gives
 * no formula, so the recurrence is the customary one of the works it cites:
 *   S_i = gamma_h S_{i-1} + phi(k_i) v_i^T,   z_i = gamma_h z_{i-1} + phi(k_i),
 *   y_i = gate_i,h * phi(q_i) S_i / (phi(q_i).z_i)
 * i.e. key j enters row i with weight gamma_h^(i-j) kappa(q_i, k_j), in numerator and denominator alike.
 *
 *   gamma  [H]        in, fp32, device: the rate of every head (1 = no decay)
 *   gate   [B][N][H]  in, dtype, device, or NULL (based_decode_step_decay: [B][H]): scales the rows of y
 * Everything else as based_prefill / based_decode_step (canonical state).  Both dtypes run on the fp32
 * vector kernels (there is no matrix-core kernel for this variant), so based_prefill_decay needs a
 * workspace of based_prefill_decay_workspace_bytes, which differs from based_prefill's for bf16.
 */
size_t based_prefill_decay_workspace_bytes(int B, int H, int N, int d_feat, int d_v, int dtype);
int based_prefill_decay(const void *q, const void *k, const void *v, void *y, void *state, int has_init,
                        void *workspace, const float *gamma, const void *gate, int B, int H, int N, int d_feat,
                        int d_v, int dtype, void *stream);
int based_decode_step_decay(const void *q, const void *k, const void *v, void *y, void *state, const float *gamma,
                            const void *gate, int B, int H, int d_feat, int d_v, int dtype, void *stream);

/*
 * Sliding-window attention (Sec. 3.2): causal softmax attention (Eq. 1) in which query i sees
 * the w keys i-w+1 .. i (fewer at the start of the sequence), logits scale * q_i.k_j.
 *
 * Ring buffer (the w-sized KV cache): for each unit, K[w][d_h] then V[w][d_h] in dtype;
 * token j (0-based position in the sequence) lives in slot j mod w.
 * based_swa_ring_bytes returns B * H * 2 * w * d_h * sizeof(dtype), or 0 if unsupported.
 */
size_t based_swa_ring_bytes(int B, int H, int w, int d_h, int dtype);

/*
 * based_swa_prefill -- all rows of a sequence.
 *   q, k, v [B][H][N][d_h] in;  y [B][H][N][d_h] out;  ring: NULL or ring buffer that receives
 *   the last min(N, w) rows of k and v (other slots are left untouched).
 */
int based_swa_prefill(const void *q, const void *k, const void *v, void *y, void *ring, int B,
                      int H, int N, int d_h, int w, float scale, int dtype, void *stream);

/*
 * based_swa_decode -- one token (the operation of Alg. 3, with the cache update included):
 * writes (k, v) into slot (pos - 1) mod w, then attends q over the last min(pos, w) tokens.
 *   q, k, v [B][H][d_h] in;  y [B][H][d_h] out;  ring in-out;
 *   pos = number of tokens seen including this one, >= 1 (same for every unit).
 */
int based_swa_decode(const void *q, const void *k, const void *v, void *y, void *ring, int pos,
                     int B, int H, int d_h, int w, float scale, int dtype, void *stream);

/*
 * Rotary position encoding for the sliding-window layers (the training-settings table lists it as the
 * positional encoding of those layers and of no others; the paper prints no formula, so the definition
 * is the published one of the encoding it names): the head dimension is d_h / 2 adjacent pairs
 * (x_2i, x_2i+1), and pair i of the q and k rows of the token at position p is rotated by the angle
 * p * base^(-2i / d_h) before the scores are taken.  v is not touched.
 *
 * based_rotary_table -- the cosines and sines, computed once in fp64 and stored as fp32:
 *   table  [N][d_h / 2][2]  out, fp32: (cos, sin) of (pos0 + t) * base^(-2i / d_h) at [t][i]
 * base > 1 (10000 is the customary value), pos0 >= 0, pos0 + N <= 2^30.
 *
 * based_swa_prefill_rotary -- based_swa_prefill on rotated q and k, rotated while the rows are staged
 * (the rotated rows are never written to global memory).  Row t of `table` belongs to token t of the
 * call, so a call that continues a sequence passes a table built with pos0 = the number of tokens
 * before it.  The ring, if given, receives ROTATED keys.  Everything else as based_swa_prefill.
 *
 * based_swa_decode_rotary -- based_swa_decode / based_swa_decode_ragged on a ring of rotated keys: the
 * new q and k are rotated by the table row of the token's position pos - 1 (`table` built with
 * pos0 = 0, table_rows rows); the rotated k, rounded to dtype, goes into the ring.  pos_per_seq == NULL:
 * every sequence is at `pos`, 1 <= pos <= table_rows (else BASED_ERR_INVALID_ARG).  Otherwise `pos` is
 * ignored and pos_per_seq [B] (device, int32) gives each sequence's position as in
 * based_swa_decode_ragged; the host cannot see those values, and a position beyond the table uses the
 * table's last row.
 */
int based_rotary_table(float *table, int pos0, int N, int d_h, float base, void *stream);
int based_swa_prefill_rotary(const void *q, const void *k, const void *v, void *y, void *ring, const float *table,
                             int B, int H, int N, int d_h, int w, float scale, int dtype, void *stream);
int based_swa_decode_rotary(const void *q, const void *k, const void *v, void *y, void *ring, const float *table,
                            int table_rows, int pos, const int *pos_per_seq, int B, int H, int d_h, int w,
                            float scale, int dtype, void *stream);
/*
 * based_decode_fused_rotary -- based_decode_fused / _packed / _ragged with the window half of the step on
 * rotary-encoded q and k, as in based_swa_decode_rotary (same `table`, `table_rows`, `pos`,
 * `pos_per_seq` rules); `packed` != 0 selects the packed linear-attention state.  The linear-attention
 * half is unchanged (those layers carry no positional encoding).
 */
int based_decode_fused_rotary(const void *q, const void *k, const void *v, void *y_lin, void *state, int packed,
                              int d_feat, int d_v, const void *swa_q, const void *swa_k, const void *swa_v,
                              void *y_swa, void *ring, const float *table, int table_rows, int pos,
                              const int *pos_per_seq, int d_h, int w, float scale, int B, int H, int dtype,
                              void *stream);

/*
 * based_decode_fused -- based_decode_step and based_swa_decode for the same token in ONE
 * kernel launch.  The two mixers belong to different layers of the model, so their outputs
 * stay separate (y_lin, y_swa).  Arguments as in the two calls above.
 */
int based_decode_fused(const void *q, const void *k, const void *v, void *y_lin, void *state,
                       int d_feat, int d_v, const void *swa_q, const void *swa_k,
                       const void *swa_v, void *y_swa, void *ring, int pos, int d_h, int w,
                       float scale, int B, int H, int dtype, void *stream);

/*
 * Packed state (variant).  The rows (a, b) and (b, a) of the 2nd-order block of a state of this
 * recurrence are equal (x_a x_b = x_b x_a in Eq. 4; the paper's own state-size count uses one row
 * per unordered pair), so a decode step that carries one row per pair moves 44 % fewer bytes at
 * d' = 16.  D_packed = 1 + d' + d'(d'+1)/2 (153 at d' = 16, 561 at d' = 32).
 *
 * Packed layout, per unit at float offset u * stride: Sp[D_packed][d_v] then zp[D_packed];
 * row 0 constant, 1 + a linear, 1 + d' + a d' - a(a-1)/2 + (b - a) the pair a <= b, holding the
 * value of the canonical row (a, b).  stride = D_packed * d_v + D_packed rounded up to 64 floats.
 *
 * based_state_pack reads a state buffer (layout at the top of this file) and writes the packed
 * one, taking the mean of the two rows of a pair; based_state_unpack writes both rows of a pair.
 * based_decode_step_packed and based_decode_fused_packed are based_decode_step and
 * based_decode_fused on a packed state (same y up to rounding order).
 * based_prefill_packed is based_prefill with the packed layout for the initial and the final state
 * (same arguments, same workspace size, same y): the prefill hands its state to the packed decode
 * without a conversion.  Served by the matrix-core kernels only: dtype BASED_BF16, else
 * BASED_ERR_UNSUPPORTED (use based_prefill and based_state_pack there).
 */
int based_packed_feature_dim(int d_feat);
size_t based_packed_state_stride_floats(int d_feat, int d_v);
size_t based_packed_state_bytes(int B, int H, int d_feat, int d_v);
int based_state_pack(const void *state, void *packed, int B, int H, int d_feat, int d_v, void *stream);
int based_state_unpack(const void *packed, void *state, int B, int H, int d_feat, int d_v, void *stream);
int based_prefill_packed(const void *q, const void *k, const void *v, void *y, void *packed, int has_init,
                         void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype,
                         void *stream);
int based_decode_step_packed(const void *q, const void *k, const void *v, void *y, void *packed, int B,
                             int H, int d_feat, int d_v, int dtype, void *stream);
int based_decode_fused_packed(const void *q, const void *k, const void *v, void *y_lin, void *packed,
                              int d_feat, int d_v, const void *swa_q, const void *swa_k,
                              const void *swa_v, void *y_swa, void *ring, int pos, int d_h, int w,
                              float scale, int B, int H, int dtype, void *stream);

/*
 * Ragged batches: the position of the decoded token is read per batch element from DEVICE memory
 * (pos[b] for all heads of sequence b; int32).  pos[b] >= 1 as in based_swa_decode; pos[b] < 1
 * marks a sequence that does not take part in the step: its ring and state are left untouched and
 * its y rows are written as zeros.  Because the positions live in device memory, a captured launch
 * (HIP graph) can be replayed for token after token while another kernel advances pos.
 * based_decode_fused_ragged: packed != 0 selects the packed state layout.
 *
 * based_positions_advance is that other kernel: pos[b] += 1 for every b with pos[b] >= 1 (sequences
 * that sit out stay out).  pos: device, B int32 values.  A loop of [decode launch, advance] can be
 * captured once and replayed for every token (the cache position bookkeeping of Alg. 3 kept on the
 * device).  Errors: BASED_ERR_INVALID_ARG for a null pointer or B < 1.
 */
int based_positions_advance(int *pos, int B, void *stream);

/*
 * based_linear -- a bias-free linear projection, y = x W^T: the q / k / v projections that feed the
 * mixers and the output projection after them (the block of Sec. 3; the architecture listing in the
 * appendix gives all four as linear layers without bias).  A plain dense product on the matrix
 * cores, bf16 in and out, fp32 accumulation; not part of the mixers' hot path.
 *   x [M][K] in,  W [N][K] in (one row per output feature),  y [M][N] out; all BASED_BF16, device.
 *   Supported: K a multiple of 64, N a multiple of 128, any M >= 1; dtype BASED_BF16.
 *   Errors: BASED_ERR_UNSUPPORTED for other sizes or dtype, BASED_ERR_INVALID_ARG for null or
 *   misaligned pointers or non-positive sizes.
 */
int based_linear(const void *x, const void *W, void *y, int M, int K, int N, int dtype, void *stream);

/*
 * The projections of a linear-attention layer, reading and writing the mixer's own layout (architecture
 * of Sec. 3 and the appendix's layer listing: bias-free projections of the d_model-wide input to H heads
 * of d' features for q and k and of d_v for v, and of the concatenated heads back to d_model).  The
 * mixers work on head-major tensors [B][H][N][d]; a plain GEMM produces token-major [B][N][H d] and
 * would need a transposing pass (one more trip of q, k, v and of the mixer output through HBM) on either
 * side.  These two calls are the GEMM of based_linear with that addressing folded into their stores
 * and loads, and with q, k, v produced from one pass over x:
 *
 * based_project_qkv    q = x Wq^T, k = x Wk^T, v = x Wv^T
 *   x  [B][N][d_model]            in, bf16
 *   W  [H (2 d' + d_v)][d_model]  in, bf16: the rows of Wq (head-major: row h d' + j), then Wk, then Wv
 *   q, k  [B][H][N][d']           out, bf16        v  [B][H][N][d_v]  out, bf16
 *   d_model % 64 == 0; d', d_v multiples of 8; H (2 d' + d_v) % 128 == 0.
 * based_project_out    out = concat_heads(y) Wo^T
 *   y_heads  [B][H][N][d_v]  in, bf16      W  [d_model][H d_v]  in, bf16      out  [B][N][d_model]  out, bf16
 *   d_v % 64 == 0; d_model % 128 == 0.
 * bf16 only (BASED_ERR_UNSUPPORTED otherwise); fp32 accumulation, outputs rounded to nearest even.
 */
int based_project_qkv(const void *x, const void *W, void *q, void *k, void *v, int B, int N, int d_model, int H,
                      int d_feat, int d_v, int dtype, void *stream);
int based_project_out(const void *y_heads, const void *W, void *out, int B, int N, int H, int d_v, int d_model,
                      int dtype, void *stream);

/*
 * based_short_conv_gate -- the gate of a BaseConv layer (appendix on the gated convolution layers;
 * training-settings table: filter size 3, SiLU activation), i.e. everything of that layer between its
 * two input projections and its output projection (which are based_linear calls):
 *   out[t] = (a[t] + b1) * silu(h[0] c[t] + h[1] c[t-1] + h[2] c[t-2] + b2),  silu(x) = x / (1 + e^-x),
 * per channel; the convolution is causal and runs along the sequence.
 *
 *   a, c    [B][N][Dc]  in, dtype   the two projections u W1 and u W2 (Dc = expansion factor x d_model)
 *   h       [3][Dc]     in, fp32    filter taps, tap j looks j tokens back
 *   b1, b2  [Dc]        in, fp32
 *   c_prev  [B][2][Dc]  in, dtype, or NULL: the two rows of c before the first token (older first);
 *                       NULL = the sequence starts here (zeros)
 *   out     [B][N][Dc]  out, dtype
 *   c_last  [B][2][Dc]  out, dtype, or NULL: the last two rows of c, the state a later call passes as
 *                       c_prev.  A decode step is the N = 1 call.  c_last may be the same buffer as
 *                       c_prev when N <= 32 (else BASED_ERR_INVALID_ARG).
 * Dc must be a multiple of 8 (bf16) or 4 (fp32), and at least 8; B <= 65535.
 */
int based_short_conv_gate(const void *a, const void *c, const float *h, const float *b1, const float *b2,
                          const void *c_prev, void *out, void *c_last, int B, int N, int Dc, int dtype,
                          void *stream);
int based_swa_decode_ragged(const void *q, const void *k, const void *v, void *y, void *ring,
                            const int *pos, int B, int H, int d_h, int w, float scale, int dtype,
                            void *stream);
int based_decode_fused_ragged(const void *q, const void *k, const void *v, void *y_lin, void *state,
                              int packed, int d_feat, int d_v, const void *swa_q, const void *swa_k,
                              const void *swa_v, void *y_swa, void *ring, const int *pos, int d_h, int w,
                              float scale, int B, int H, int dtype, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BASED_H */
