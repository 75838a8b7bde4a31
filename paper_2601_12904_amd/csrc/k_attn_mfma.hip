#include "fr_internal.hpp"
namespace fr {
bool attn_mfma_supported(const Shape&) { return false; }
hipError_t launch_attn_mfma(const Shape&, const void*, const int32_t*, int, const void*, const void*, int64_t,
                            const void*, const void*, const int32_t*, void*, float*, const Workspace&, hipStream_t) {
    return hipErrorNotSupported;
}
}  // namespace fr
