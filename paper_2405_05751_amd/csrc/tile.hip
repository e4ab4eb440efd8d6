// Matrix-core variant for large M (placeholder until the kernel lands).
#include "common.hpp"

namespace rmsnl {

hipError_t launch_tile(const Problem&, hipStream_t, const char** why)
{
    if (why) *why = "tile variant not built yet";
    return hipErrorInvalidValue;
}

}  // namespace rmsnl
