#include "fr_internal.hpp"
namespace fr {
bool score_mfma_supported(const Shape&) { return false; }
hipError_t launch_score_mfma(const Shape&, const void*, int, const void*, const ChunkTable&, int, const Workspace&,
                             float*, hipStream_t) { return hipErrorNotSupported; }
}  // namespace fr
