// C ABI of the library: argument validation and dispatch only; see include/based.h for the
// contract of every entry point.
#include "common.h"

#include <mutex>

using namespace based;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool ok_ptr(const void *p) { return p != nullptr && aligned16(p); }
bool ok_dtype(int dtype) { return dtype == BASED_F32 || dtype == BASED_BF16; }
bool ok_lin_dims(int dp, int dv)
{
    return (dp == 8 || dp == 16 || dp == 24 || dp == 32) && (dv == 64 || dv == 128);
}
// the fused decode step is built for the feature dimensions of the trained models only
bool ok_fused_lin_dims(int dp, int dv) { return (dp == 16 || dp == 32) && (dv == 64 || dv == 128); }
bool ok_swa_dims(int dh, int w)
{
    return (dh == 64 || dh == 128) && (w == 16 || w == 32 || w == 64 || w == 128);
}
bool ok_counts(int B, int H, int N)
{
    if (B < 1 || H < 1 || N < 1) return false;
    const unsigned long long t = (unsigned long long)B * (unsigned long long)H * (unsigned long long)N;
    return t < (1ull << 31);
}
int status_of(hipError_t e) { return e == hipSuccess ? BASED_OK : BASED_ERR_LAUNCH; }

// ---- scratch of based_prefill_static ------------------------------------------------------------
// A file-scope device array: every GPU this library runs on holds its own copy, at its own address,
// from the moment the code object is loaded there until the process ends (zero-filled at load).
// In host code the array's name is only a handle; the device address comes from
// hipGetSymbolAddress, asked once per device with that device current, and only that pointer is
// ever handed to kernels or memory calls.
constexpr size_t kStaticScratchBytes = BASED_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device, or nullptr (err says why)
void *static_scratch(hipError_t *err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !p) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

const char *based_strerror(int status)
{
    switch (status) {
    case BASED_OK: return "ok";
    case BASED_ERR_INVALID_ARG: return "invalid argument (null or misaligned pointer, non-positive size, bad pos)";
    case BASED_ERR_UNSUPPORTED: return "unsupported size or dtype";
    case BASED_ERR_TOO_LARGE: return "the call needs more scratch memory than the library's static scratch holds";
    case BASED_ERR_LAUNCH: return "HIP launch failed, or a launch gave up waiting for one of its own workgroups";
    default: return "unknown status";
    }
}

int based_version(void) { return 100; }

int based_feature_dim(int d_feat) { return d_feat < 1 ? 0 : feature_dim(d_feat); }

size_t based_state_stride_floats(int d_feat, int d_v)
{
    return ok_lin_dims(d_feat, d_v) ? state_stride(d_feat, d_v) : 0;
}

size_t based_state_bytes(int B, int H, int d_feat, int d_v)
{
    if (!ok_lin_dims(d_feat, d_v) || !ok_counts(B, H, 1)) return 0;
    return (size_t)B * H * state_stride(d_feat, d_v) * sizeof(float);
}

int based_state_export(const void *state, float *S, float *z, int B, int H, int d_feat, int d_v,
                       void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(state) || (S && !aligned16(S)) || (z && !aligned16(z))) return BASED_ERR_INVALID_ARG;
    return status_of(launch_state_copy(const_cast<float *>(static_cast<const float *>(state)), S, z,
                                       B * H, d_feat, d_v, 0, (hipStream_t)stream));
}

int based_state_import(void *state, const float *S, const float *z, int B, int H, int d_feat,
                       int d_v, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(state) || (S && !aligned16(S)) || (z && !aligned16(z))) return BASED_ERR_INVALID_ARG;
    return status_of(launch_state_copy(static_cast<float *>(state), const_cast<float *>(S),
                                       const_cast<float *>(z), B * H, d_feat, d_v, 1,
                                       (hipStream_t)stream));
}

// A prefill workspace is a 256-byte header followed by the scratch of the kernel family that serves
// the call.  The header's first word is the sticky status of the bounded waits; it sits at offset 0
// whatever the sizes, so a workspace can be reused for calls of any shape.
constexpr size_t kWsHeader = 256;

static size_t prefill_scratch_bytes(int U, int N, int d_feat, int d_v, int dtype)
{
    if (prefill_mfma32_supported(d_feat, d_v, dtype)) return prefill_mfma32_workspace_bytes(U, N, d_feat, d_v);
    if (prefill_mfma_supported(d_feat, d_v, dtype)) return prefill_mfma_workspace_bytes(U, N, d_feat, d_v);
    return prefill_ref_workspace_bytes(U, N, d_feat, d_v);
}

size_t based_prefill_workspace_bytes(int B, int H, int N, int d_feat, int d_v, int dtype)
{
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype) || !ok_counts(B, H, N)) return 0;
    const size_t scratch_bytes = prefill_scratch_bytes(B * H, N, d_feat, d_v, dtype);
    return scratch_bytes ? kWsHeader + scratch_bytes : 0;
}

static int prefill_any(const void *q, const void *k, const void *v, void *y, void *state, int has_init,
                       int packed, int numerator_only, void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype,
                       void *stream)
{
    if (!ok_counts(B, H, N)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    const bool m32 = prefill_mfma32_supported(d_feat, d_v, dtype);
    const bool m16 = prefill_mfma_supported(d_feat, d_v, dtype);
    // only the matrix-core kernels carry the state packed
    if (packed && !m32 && !m16) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y)) return BASED_ERR_INVALID_ARG;
    if (state && !aligned16(state)) return BASED_ERR_INVALID_ARG;
    if (has_init && !state) return BASED_ERR_INVALID_ARG;
    const int U = B * H;
    const size_t need = prefill_scratch_bytes(U, N, d_feat, d_v, dtype);
    if (need && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))) return BASED_ERR_INVALID_ARG;
    void *inner = workspace ? static_cast<char *>(workspace) + kWsHeader : nullptr;
    float *st = static_cast<float *>(state);
    hipStream_t s = (hipStream_t)stream;
    // the launchers' flag word: bit 0 an initial state is given, bit 2 numerators only
    const int fl = (has_init ? 1 : 0) | (numerator_only ? 4 : 0);
    if (m32)
        return status_of(launch_prefill_mfma32(q, k, v, y, st, fl, packed, inner, U, N, d_feat, d_v, s));
    if (m16)
        return status_of(launch_prefill_mfma(q, k, v, y, st, fl, packed, inner,
                                             static_cast<unsigned *>(workspace), U, N, d_feat, d_v, s));
    return status_of(launch_prefill_ref(q, k, v, y, st, fl, inner, U, N, d_feat, d_v, dtype, s));
}

int based_prefill(const void *q, const void *k, const void *v, void *y, void *state, int has_init,
                  void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype, void *stream)
{
    return prefill_any(q, k, v, y, state, has_init, 0, 0, workspace, B, H, N, d_feat, d_v, dtype, stream);
}

int based_prefill_numerator(const void *q, const void *k, const void *v, void *y, void *state, int has_init,
                            void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype, void *stream)
{
    return prefill_any(q, k, v, y, state, has_init, 0, 1, workspace, B, H, N, d_feat, d_v, dtype, stream);
}

int based_prefill_packed(const void *q, const void *k, const void *v, void *y, void *packed, int has_init,
                         void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype, void *stream)
{
    return prefill_any(q, k, v, y, packed, has_init, 1, 0, workspace, B, H, N, d_feat, d_v, dtype, stream);
}

int based_prefill_static(const void *q, const void *k, const void *v, void *y, void *state, int has_init,
                         int B, int H, int N, int d_feat, int d_v, int dtype, void *stream)
{
    if (!ok_counts(B, H, N)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y)) return BASED_ERR_INVALID_ARG;
    if (state && !aligned16(state)) return BASED_ERR_INVALID_ARG;
    if (has_init && !state) return BASED_ERR_INVALID_ARG;
    const size_t need = based_prefill_workspace_bytes(B, H, N, d_feat, d_v, dtype);
    if (need > kStaticScratchBytes) return BASED_ERR_TOO_LARGE;
    void *ws = nullptr;
    if (need) {
        hipError_t e;
        ws = static_scratch(&e);
        if (!ws) return BASED_ERR_LAUNCH;
    }
    // Nothing in the scratch has to start at zero for a new call: workspace entries are written
    // before they are read, ready flags carry a per-call epoch and are cleared by their readers, and
    // the status word (zero when the array is created) is meant to persist until
    // based_prefill_status has seen it.
    return prefill_any(q, k, v, y, state, has_init, 0, 0, ws, B, H, N, d_feat, d_v, dtype, stream);
}

int based_prefill_status(void *workspace, int B, int H, int N, int d_feat, int d_v, int dtype, void *stream)
{
    if (!ok_counts(B, H, N)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    // only the single-launch segmented prefill (bf16, d' = 16) has workgroups that wait for each other
    if (!prefill_mfma_supported(d_feat, d_v, dtype)) return BASED_OK;
    if (!workspace) {
        // the calls asked about went through based_prefill_static
        if (based_prefill_workspace_bytes(B, H, N, d_feat, d_v, dtype) > kStaticScratchBytes) return BASED_ERR_TOO_LARGE;
        hipError_t e;
        workspace = static_scratch(&e);
        if (!workspace) return BASED_ERR_LAUNCH;
    }
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return BASED_ERR_INVALID_ARG;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return BASED_ERR_LAUNCH;
    unsigned word = 0;
    char *base = static_cast<char *>(workspace);
    if (hipMemcpy(&word, base, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess) return BASED_ERR_LAUNCH;
    if (word == 0) return BASED_OK;
    // a workgroup gave up: report it once; clear the status word, and the ready flags of this shape (a
    // late writer may have left one raised), so that the workspace can be used again
    size_t flags_off = 0, flags_bytes = 0;
    prefill_mfma_flags_region(B * H, N, d_feat, d_v, &flags_off, &flags_bytes);
    if (hipMemset(base, 0, kWsHeader) != hipSuccess) return BASED_ERR_LAUNCH;
    if (flags_bytes && hipMemset(base + kWsHeader + flags_off, 0, flags_bytes) != hipSuccess) return BASED_ERR_LAUNCH;
    return BASED_ERR_LAUNCH;
}

void based_debug_set_poll_limit(int polls) { prefill_mfma_set_poll_limit(polls); }

int based_decode_step(const void *q, const void *k, const void *v, void *y, void *state, int B,
                      int H, int d_feat, int d_v, int dtype, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y) || !ok_ptr(state))
        return BASED_ERR_INVALID_ARG;
    return status_of(launch_decode_step(q, k, v, y, static_cast<float *>(state), B * H, d_feat, d_v,
                                        dtype, 0, 0, nullptr, nullptr, 1, (hipStream_t)stream));
}

int based_decode_step_numerator(const void *q, const void *k, const void *v, void *y, void *state, int B,
                                int H, int d_feat, int d_v, int dtype, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y) || !ok_ptr(state))
        return BASED_ERR_INVALID_ARG;
    return status_of(launch_decode_step(q, k, v, y, static_cast<float *>(state), B * H, d_feat, d_v,
                                        dtype, 0, 1, nullptr, nullptr, 1, (hipStream_t)stream));
}

size_t based_prefill_decay_workspace_bytes(int B, int H, int N, int d_feat, int d_v, int dtype)
{
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype) || !ok_counts(B, H, N)) return 0;
    const size_t scratch_bytes = prefill_ref_workspace_bytes(B * H, N, d_feat, d_v);
    return scratch_bytes ? kWsHeader + scratch_bytes : 0;
}

int based_prefill_decay(const void *q, const void *k, const void *v, void *y, void *state, int has_init,
                        void *workspace, const float *gamma, const void *gate, int B, int H, int N, int d_feat,
                        int d_v, int dtype, void *stream)
{
    if (!ok_counts(B, H, N)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y)) return BASED_ERR_INVALID_ARG;
    if (!gamma || (reinterpret_cast<uintptr_t>(gamma) & 3u)) return BASED_ERR_INVALID_ARG;
    if (gate && (reinterpret_cast<uintptr_t>(gate) & 3u)) return BASED_ERR_INVALID_ARG;
    if (state && !aligned16(state)) return BASED_ERR_INVALID_ARG;
    if (has_init && !state) return BASED_ERR_INVALID_ARG;
    const int U = B * H;
    const size_t need = prefill_ref_workspace_bytes(U, N, d_feat, d_v);
    if (need && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))) return BASED_ERR_INVALID_ARG;
    void *inner = workspace ? static_cast<char *>(workspace) + kWsHeader : nullptr;
    return status_of(launch_prefill_ref_decay(q, k, v, y, static_cast<float *>(state), has_init ? 1 : 0, inner, gamma,
                                              gate, H, U, N, d_feat, d_v, dtype, (hipStream_t)stream));
}

int based_decode_step_decay(const void *q, const void *k, const void *v, void *y, void *state, const float *gamma,
                            const void *gate, int B, int H, int d_feat, int d_v, int dtype, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y) || !ok_ptr(state)) return BASED_ERR_INVALID_ARG;
    if (!gamma || (reinterpret_cast<uintptr_t>(gamma) & 3u)) return BASED_ERR_INVALID_ARG;
    if (gate && (reinterpret_cast<uintptr_t>(gate) & 3u)) return BASED_ERR_INVALID_ARG;
    return status_of(launch_decode_step(q, k, v, y, static_cast<float *>(state), B * H, d_feat, d_v, dtype, 0, 0,
                                        gamma, gate, H, (hipStream_t)stream));
}

int based_packed_feature_dim(int d_feat) { return d_feat >= 1 ? packed_feature_dim(d_feat) : 0; }

size_t based_packed_state_stride_floats(int d_feat, int d_v)
{
    return ok_lin_dims(d_feat, d_v) ? packed_state_stride(d_feat, d_v) : 0;
}

size_t based_packed_state_bytes(int B, int H, int d_feat, int d_v)
{
    if (!ok_lin_dims(d_feat, d_v) || !ok_counts(B, H, 1)) return 0;
    return (size_t)B * H * packed_state_stride(d_feat, d_v) * sizeof(float);
}

int based_state_pack(const void *state, void *packed, int B, int H, int d_feat, int d_v, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(state) || !ok_ptr(packed)) return BASED_ERR_INVALID_ARG;
    return status_of(launch_state_repack(const_cast<float *>(static_cast<const float *>(state)),
                                         static_cast<float *>(packed), B * H, d_feat, d_v, 1,
                                         (hipStream_t)stream));
}

int based_state_unpack(const void *packed, void *state, int B, int H, int d_feat, int d_v, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(state) || !ok_ptr(packed)) return BASED_ERR_INVALID_ARG;
    return status_of(launch_state_repack(static_cast<float *>(state),
                                         const_cast<float *>(static_cast<const float *>(packed)), B * H,
                                         d_feat, d_v, 0, (hipStream_t)stream));
}

int based_decode_step_packed(const void *q, const void *k, const void *v, void *y, void *packed, int B,
                             int H, int d_feat, int d_v, int dtype, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_lin_dims(d_feat, d_v) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y) || !ok_ptr(packed))
        return BASED_ERR_INVALID_ARG;
    return status_of(launch_decode_step(q, k, v, y, static_cast<float *>(packed), B * H, d_feat, d_v,
                                        dtype, 1, 0, nullptr, nullptr, 1, (hipStream_t)stream));
}

size_t based_swa_ring_bytes(int B, int H, int w, int d_h, int dtype)
{
    if (!ok_swa_dims(d_h, w) || !ok_dtype(dtype) || !ok_counts(B, H, 1)) return 0;
    return (size_t)B * H * 2 * w * d_h * (dtype == BASED_F32 ? 4 : 2);
}

static int swa_prefill_any(const void *q, const void *k, const void *v, void *y, void *ring, const float *rot,
                           int B, int H, int N, int d_h, int w, float scale, int dtype, void *stream)
{
    if (!ok_counts(B, H, N)) return BASED_ERR_INVALID_ARG;
    if (!ok_swa_dims(d_h, w) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y)) return BASED_ERR_INVALID_ARG;
    if (ring && !aligned16(ring)) return BASED_ERR_INVALID_ARG;
    const int U = B * H;
    hipError_t e;
    // the matrix-core kernel takes the row maximum of the unscaled scores, which is the maximum of
    // the scaled ones only for a positive scale; anything else goes to the vector-ALU kernel
    if (!rot && swa_prefill_mfma16_supported(d_h, w, dtype) && scale > 0.f) {
        // (the tiling of 16 queries to a wave, for the sizes where it is the faster one; fills the ring too)
        e = launch_swa_prefill_mfma16(q, k, v, y, ring, U, N, d_h, w, scale, (hipStream_t)stream);
    } else if (swa_prefill_mfma_supported(d_h, w, dtype, rot != nullptr) && scale > 0.f) {
        // this kernel also fills the ring
        e = launch_swa_prefill_mfma(q, k, v, y, ring, rot, U, N, d_h, w, scale, (hipStream_t)stream);
    } else {
        e = launch_swa_prefill_ref(q, k, v, y, rot, U, N, d_h, w, scale, dtype, (hipStream_t)stream);
        if (e == hipSuccess && ring)
            e = launch_swa_ring_fill(k, v, ring, rot, U, N, d_h, w, dtype, (hipStream_t)stream);
    }
    return status_of(e);
}

int based_swa_prefill(const void *q, const void *k, const void *v, void *y, void *ring, int B, int H,
                      int N, int d_h, int w, float scale, int dtype, void *stream)
{
    return swa_prefill_any(q, k, v, y, ring, nullptr, B, H, N, d_h, w, scale, dtype, stream);
}

int based_rotary_table(float *table, int pos0, int N, int d_h, float base, void *stream)
{
    if (N < 1 || pos0 < 0 || (long long)pos0 + N > (1ll << 30)) return BASED_ERR_INVALID_ARG;
    if (!(base > 1.f)) return BASED_ERR_INVALID_ARG;
    if (d_h != 64 && d_h != 128) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(table)) return BASED_ERR_INVALID_ARG;
    return status_of(launch_rotary_table(table, pos0, N, d_h, base, (hipStream_t)stream));
}

int based_swa_prefill_rotary(const void *q, const void *k, const void *v, void *y, void *ring, const float *table,
                             int B, int H, int N, int d_h, int w, float scale, int dtype, void *stream)
{
    if (!ok_ptr(table)) return BASED_ERR_INVALID_ARG;
    return swa_prefill_any(q, k, v, y, ring, table, B, H, N, d_h, w, scale, dtype, stream);
}

static int swa_decode_any(const void *q, const void *k, const void *v, void *y, void *ring, PosArg pos,
                          int B, int H, int d_h, int w, float scale, int dtype, void *stream);

int based_swa_decode_rotary(const void *q, const void *k, const void *v, void *y, void *ring, const float *table,
                            int table_rows, int pos, const int *pos_per_seq, int B, int H, int d_h, int w,
                            float scale, int dtype, void *stream)
{
    if (!ok_ptr(table) || table_rows < 1) return BASED_ERR_INVALID_ARG;
    if (pos_per_seq) {
        if (reinterpret_cast<uintptr_t>(pos_per_seq) & 3u) return BASED_ERR_INVALID_ARG;
        return swa_decode_any(q, k, v, y, ring, PosArg{0, pos_per_seq, H, 0, table, table_rows}, B, H, d_h, w, scale,
                              dtype, stream);
    }
    if (pos < 1 || pos > table_rows) return BASED_ERR_INVALID_ARG;
    return swa_decode_any(q, k, v, y, ring, PosArg{pos, nullptr, H, 0, table, table_rows}, B, H, d_h, w, scale, dtype,
                          stream);
}

static int swa_decode_any(const void *q, const void *k, const void *v, void *y, void *ring, PosArg pos,
                          int B, int H, int d_h, int w, float scale, int dtype, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_swa_dims(d_h, w) || !ok_dtype(dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y) || !ok_ptr(ring))
        return BASED_ERR_INVALID_ARG;
    return status_of(launch_swa_decode(q, k, v, y, ring, pos, B * H, d_h, w, scale, dtype,
                                       (hipStream_t)stream));
}

int based_swa_decode(const void *q, const void *k, const void *v, void *y, void *ring, int pos, int B,
                     int H, int d_h, int w, float scale, int dtype, void *stream)
{
    if (pos < 1) return BASED_ERR_INVALID_ARG;
    return swa_decode_any(q, k, v, y, ring, PosArg{pos, nullptr, H, 0}, B, H, d_h, w, scale, dtype, stream);
}

int based_linear(const void *x, const void *W, void *y, int M, int K, int N, int dtype, void *stream)
{
    if (M < 1 || K < 1 || N < 1) return BASED_ERR_INVALID_ARG;
    if ((unsigned long long)M * (unsigned long long)(K > N ? K : N) >= (1ull << 40)) return BASED_ERR_INVALID_ARG;
    if (!linear_supported(M, K, N, dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(x) || !ok_ptr(W) || !ok_ptr(y)) return BASED_ERR_INVALID_ARG;
    return status_of(launch_linear(x, W, y, M, K, N, (hipStream_t)stream));
}

int based_project_qkv(const void *x, const void *W, void *q, void *k, void *v, int B, int N, int d_model, int H,
                      int d_feat, int d_v, int dtype, void *stream)
{
    if (!ok_counts(B, H, N) || d_model < 1 || d_feat < 1 || d_v < 1) return BASED_ERR_INVALID_ARG;
    if ((unsigned long long)B * N * (unsigned long long)(d_model > H * (2 * d_feat + d_v) ? d_model : H * (2 * d_feat + d_v)) >=
        (1ull << 40))
        return BASED_ERR_INVALID_ARG;
    if (!project_qkv_supported(d_model, H, d_feat, d_v, dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(x) || !ok_ptr(W) || !ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v)) return BASED_ERR_INVALID_ARG;
    return status_of(launch_project_qkv(x, W, q, k, v, B, N, d_model, H, d_feat, d_v, (hipStream_t)stream));
}

int based_project_out(const void *y_heads, const void *W, void *out, int B, int N, int H, int d_v, int d_model,
                      int dtype, void *stream)
{
    if (!ok_counts(B, H, N) || d_model < 1 || d_v < 1) return BASED_ERR_INVALID_ARG;
    if ((unsigned long long)B * N * (unsigned long long)(d_model > H * d_v ? d_model : H * d_v) >= (1ull << 40))
        return BASED_ERR_INVALID_ARG;
    if (!project_out_supported(H, d_v, d_model, dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(y_heads) || !ok_ptr(W) || !ok_ptr(out)) return BASED_ERR_INVALID_ARG;
    return status_of(launch_project_out(y_heads, W, out, B, N, H, d_v, d_model, (hipStream_t)stream));
}

int based_short_conv_gate(const void *a, const void *c, const float *h, const float *b1, const float *b2,
                          const void *c_prev, void *out, void *c_last, int B, int N, int Dc, int dtype, void *stream)
{
    if (B < 1 || N < 1 || Dc < 1 || B > 65535) return BASED_ERR_INVALID_ARG;
    if ((unsigned long long)B * (unsigned long long)N * (unsigned long long)Dc >= (1ull << 40)) return BASED_ERR_INVALID_ARG;
    if (!ok_dtype(dtype) || !short_conv_gate_supported(Dc, dtype)) return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(a) || !ok_ptr(c) || !ok_ptr(h) || !ok_ptr(b1) || !ok_ptr(b2) || !ok_ptr(out)) return BASED_ERR_INVALID_ARG;
    if ((c_prev && !aligned16(c_prev)) || (c_last && !aligned16(c_last))) return BASED_ERR_INVALID_ARG;
    // in place only when one thread both reads and writes the state rows of its channels
    if (c_last && c_last == c_prev && N > short_conv_gate_run()) return BASED_ERR_INVALID_ARG;
    if ((N + short_conv_gate_run() - 1) / short_conv_gate_run() > 65535) return BASED_ERR_INVALID_ARG;
    return status_of(launch_short_conv_gate(a, c, h, b1, b2, c_prev, out, c_last, B, N, Dc, dtype, (hipStream_t)stream));
}

int based_positions_advance(int *pos, int B, void *stream)
{
    if (!pos || B < 1) return BASED_ERR_INVALID_ARG;
    return status_of(launch_positions_advance(pos, B, (hipStream_t)stream));
}

int based_swa_decode_ragged(const void *q, const void *k, const void *v, void *y, void *ring,
                            const int *pos, int B, int H, int d_h, int w, float scale, int dtype,
                            void *stream)
{
    if (!pos || (reinterpret_cast<uintptr_t>(pos) & 3u)) return BASED_ERR_INVALID_ARG;
    return swa_decode_any(q, k, v, y, ring, PosArg{0, pos, H, 0}, B, H, d_h, w, scale, dtype, stream);
}

static int decode_fused_any(const void *q, const void *k, const void *v, void *y_lin, void *state,
                            int d_feat, int d_v, const void *swa_q, const void *swa_k, const void *swa_v,
                            void *y_swa, void *ring, PosArg pos, int d_h, int w, float scale, int B, int H,
                            int dtype, int packed, void *stream)
{
    if (!ok_counts(B, H, 1)) return BASED_ERR_INVALID_ARG;
    if (!ok_fused_lin_dims(d_feat, d_v) || !ok_swa_dims(d_h, w) || !ok_dtype(dtype))
        return BASED_ERR_UNSUPPORTED;
    if (!ok_ptr(q) || !ok_ptr(k) || !ok_ptr(v) || !ok_ptr(y_lin) || !ok_ptr(state) || !ok_ptr(swa_q) ||
        !ok_ptr(swa_k) || !ok_ptr(swa_v) || !ok_ptr(y_swa) || !ok_ptr(ring))
        return BASED_ERR_INVALID_ARG;
    if ((unsigned long long)B * H * 2ull >= (1ull << 31)) return BASED_ERR_INVALID_ARG;
    return status_of(launch_decode_fused(q, k, v, y_lin, static_cast<float *>(state), d_feat, d_v,
                                         swa_q, swa_k, swa_v, y_swa, ring, pos, d_h, w, scale, B * H,
                                         dtype, packed, (hipStream_t)stream));
}

int based_decode_fused(const void *q, const void *k, const void *v, void *y_lin, void *state,
                       int d_feat, int d_v, const void *swa_q, const void *swa_k, const void *swa_v,
                       void *y_swa, void *ring, int pos, int d_h, int w, float scale, int B, int H,
                       int dtype, void *stream)
{
    if (pos < 1) return BASED_ERR_INVALID_ARG;
    return decode_fused_any(q, k, v, y_lin, state, d_feat, d_v, swa_q, swa_k, swa_v, y_swa, ring,
                            PosArg{pos, nullptr, H, 0}, d_h, w, scale, B, H, dtype, 0, stream);
}

int based_decode_fused_packed(const void *q, const void *k, const void *v, void *y_lin, void *packed,
                              int d_feat, int d_v, const void *swa_q, const void *swa_k,
                              const void *swa_v, void *y_swa, void *ring, int pos, int d_h, int w,
                              float scale, int B, int H, int dtype, void *stream)
{
    if (pos < 1) return BASED_ERR_INVALID_ARG;
    return decode_fused_any(q, k, v, y_lin, packed, d_feat, d_v, swa_q, swa_k, swa_v, y_swa, ring,
                            PosArg{pos, nullptr, H, 0}, d_h, w, scale, B, H, dtype, 1, stream);
}

int based_decode_fused_rotary(const void *q, const void *k, const void *v, void *y_lin, void *state, int packed,
                              int d_feat, int d_v, const void *swa_q, const void *swa_k, const void *swa_v,
                              void *y_swa, void *ring, const float *table, int table_rows, int pos,
                              const int *pos_per_seq, int d_h, int w, float scale, int B, int H, int dtype,
                              void *stream)
{
    if (!ok_ptr(table) || table_rows < 1) return BASED_ERR_INVALID_ARG;
    if (pos_per_seq) {
        if (reinterpret_cast<uintptr_t>(pos_per_seq) & 3u) return BASED_ERR_INVALID_ARG;
        return decode_fused_any(q, k, v, y_lin, state, d_feat, d_v, swa_q, swa_k, swa_v, y_swa, ring,
                                PosArg{0, pos_per_seq, H, 0, table, table_rows}, d_h, w, scale, B, H, dtype,
                                packed ? 1 : 0, stream);
    }
    if (pos < 1 || pos > table_rows) return BASED_ERR_INVALID_ARG;
    return decode_fused_any(q, k, v, y_lin, state, d_feat, d_v, swa_q, swa_k, swa_v, y_swa, ring,
                            PosArg{pos, nullptr, H, 0, table, table_rows}, d_h, w, scale, B, H, dtype, packed ? 1 : 0,
                            stream);
}

int based_decode_fused_ragged(const void *q, const void *k, const void *v, void *y_lin, void *state,
                              int packed, int d_feat, int d_v, const void *swa_q, const void *swa_k,
                              const void *swa_v, void *y_swa, void *ring, const int *pos, int d_h, int w,
                              float scale, int B, int H, int dtype, void *stream)
{
    if (!pos || (reinterpret_cast<uintptr_t>(pos) & 3u)) return BASED_ERR_INVALID_ARG;
    return decode_fused_any(q, k, v, y_lin, state, d_feat, d_v, swa_q, swa_k, swa_v, y_swa, ring,
                            PosArg{0, pos, H, 0}, d_h, w, scale, B, H, dtype, packed ? 1 : 0, stream);
}

}  // extern "C"
