// Schedule "chain" (placeholder until the on-chip kernel lands): reports unsupported.
#include "specgbv_internal.hpp"

namespace specgbv {

bool chain_supported(const Problem &) { return false; }

hipError_t launch_chain_main(const Problem &) { return hipErrorNotSupported; }

}  // namespace specgbv
