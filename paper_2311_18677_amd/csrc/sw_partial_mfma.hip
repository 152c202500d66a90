// Partial decode attention on the matrix cores (placeholder until the MFMA
// kernel lands: reports that no shape is covered, so the dispatcher uses the
// vector-ALU kernel).
#include "sw_internal.h"

bool sw_partial_mfma_supported(const SwArgs &) { return false; }

hipError_t sw_launch_partial_mfma(const SwArgs &, hipStream_t, const SwLaunchEvents *)
{
    return hipErrorNotSupported;
}
