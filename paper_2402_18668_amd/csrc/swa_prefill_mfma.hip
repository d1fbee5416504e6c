#include "common.h"
namespace based {
bool swa_prefill_mfma_supported(int, int, int) { return false; }
hipError_t launch_swa_prefill_mfma(const void *, const void *, const void *, void *, int, int, int, int,
                                   float, hipStream_t) { return hipErrorNotSupported; }
}
