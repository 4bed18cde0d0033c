// Streaming scoring kernels for bf16 keys (placeholder until the streaming pass lands).
#include "nkv_device.h"

namespace nkv {

bool fast_score_supported(int, int, int, const PromptTab &) { return false; }
size_t fast_score_ws_floats(int, int, const PromptTab &) { return 0; }
hipError_t launch_score_fast(const void *, int, int, const PromptTab &, float *, float *, float *, const Prof &,
                             hipStream_t)
{
    return hipErrorNotSupported;
}

}  // namespace nkv
