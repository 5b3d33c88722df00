// placeholder until the matrix-core kernel lands
#include "lpq_internal.h"
namespace lpq {
bool mfma_supported(int, int) { return false; }
size_t mfma_list_scratch_bytes(int64_t, int, int) { return 0; }
hipError_t launch_search_mfma(const SearchArgs &, int64_t, int64_t, int, const cand_t *, cand_t *, void *, hipStream_t)
{
    return hipErrorNotSupported;
}
}  // namespace lpq
