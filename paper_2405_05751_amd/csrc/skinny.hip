// Matrix-core variant for small M (placeholder until the kernel lands).
#include "common.hpp"

namespace rmsnl {

size_t skinny_workspace_bytes(const Problem&) { return 0; }

hipError_t launch_skinny(const Problem&, hipStream_t, const char** why)
{
    if (why) *why = "skinny variant not built yet";
    return hipErrorInvalidValue;
}

}  // namespace rmsnl
