// kvb_step_kernel for fp32 inputs.
#include "kvb_step_kernel.h"

namespace kvb_impl {

int launch_step_f32(int dk, const StepArgs &a, int blocks, hipStream_t stream)
{
    return launch_step_typed<float>(dk, a, blocks, stream);
}

}  // namespace kvb_impl
