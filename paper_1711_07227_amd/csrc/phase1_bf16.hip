// bf16-in / fp32-accumulate variant of the first phase.  Placeholder translation unit: the packed copy
// and the kernel are added next; until then the bf16 path reports that it is not supported.
#include "lcrwmd_internal.h"

namespace lcrwmd {

int32_t bf16_pitch(int32_t m) { return ((m + 15) / 16) * 16 + 16; }
size_t pack_bf16_bytes(int64_t v, int32_t m) { return (size_t)v * (size_t)bf16_pitch(m) * 2; }

hipError_t launch_pack_bf16(const void*, lcrwmd_dtype, int64_t, int32_t, int64_t, void*, float*, hipStream_t)
{
    return hipErrorNotSupported;
}

hipError_t launch_phase1_bf16(const Phase1Args&, const TokenPlan&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace lcrwmd
