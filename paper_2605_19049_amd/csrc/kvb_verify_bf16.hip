// kvb_verify_mfma_kernel for bf16 inputs (fp32 and 16-bit records).
#include "kvb_verify_kernel.h"

namespace kvb_impl {

template void launch_verify_typed<bf16_t, float>(const StepArgs &a, int blocks, hipStream_t stream);
template void launch_verify_typed<bf16_t, bf16_t>(const StepArgs &a, int blocks, hipStream_t stream);

}  // namespace kvb_impl
