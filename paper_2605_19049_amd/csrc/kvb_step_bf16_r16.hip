// kvb_step_kernel for bf16 inputs, bf16 records.
#include "kvb_step_kernel.h"

namespace kvb_impl {

template int launch_step_typed<bf16_t, bf16_t>(int dk, const StepArgs &a, int blocks, hipStream_t stream);

}  // namespace kvb_impl
