#include "common.h"
namespace based {
bool prefill_mfma_supported(int, int, int) { return false; }
size_t prefill_mfma_workspace_bytes(int, int, int, int) { return 0; }
hipError_t launch_prefill_mfma(const void *, const void *, const void *, void *, float *, int, void *,
                               int, int, int, int, hipStream_t) { return hipErrorNotSupported; }
}
