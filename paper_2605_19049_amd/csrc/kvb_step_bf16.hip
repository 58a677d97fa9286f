// kvb_step_kernel for bf16 inputs.
#include "kvb_step_kernel.h"

namespace kvb_impl {

int launch_step_bf16(int dk, const StepArgs &a, int blocks, hipStream_t stream)
{
    return launch_step_typed<bf16_t>(dk, a, blocks, stream);
}

}  // namespace kvb_impl
