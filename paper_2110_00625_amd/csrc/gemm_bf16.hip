#include "kavg_internal.h"
namespace kavg {
hipError_t bf16_forward(const LayerCall&, hipStream_t) { return hipErrorNotSupported; }
hipError_t bf16_backward_data(const LayerCall&, hipStream_t) { return hipErrorNotSupported; }
hipError_t bf16_update(const LayerCall&, hipStream_t) { return hipErrorNotSupported; }
}
