// placeholder until the matrix-core kernel lands
#include "qc_device.h"
namespace qc {
hipError_t launch_prefill_mfma_bf16_d128(const PrefillArgs&, hipStream_t) { return hipErrorNotSupported; }
}
