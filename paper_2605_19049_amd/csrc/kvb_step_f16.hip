// kvb_step_kernel for fp16 inputs, fp32 records.
#include "kvb_step_kernel.h"

namespace kvb_impl {

template int launch_step_typed<f16_t, float>(int dk, const StepArgs &a, int blocks, hipStream_t stream);

}  // namespace kvb_impl
