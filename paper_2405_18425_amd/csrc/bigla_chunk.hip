// placeholder until the chunkwise MFMA kernels land
#include "vig_kernels.hpp"
namespace vig {
bool bigla_chunk_supported(int, int, bool) { return false; }
size_t bigla_chunk_workspace_bytes(long, int) { return 0; }
hipError_t bigla_chunk_launch(const void *, const void *, const void *, const void *, const void *, void *, long, int,
                              void *, hipStream_t)
{
    return hipErrorNotSupported;
}
}  // namespace vig
