// kvb_step_kernel for fp32 inputs (fp32 records).
#include "kvb_step_kernel.h"

namespace kvb_impl {

template int launch_step_typed<float, float>(int dk, const StepArgs &a, int blocks, hipStream_t stream);

}  // namespace kvb_impl
