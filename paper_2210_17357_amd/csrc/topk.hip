// Top-K (stub, replaced below in the build order): radix-histogram threshold search.
#include "internal.h"

namespace lgreco {

hipError_t topk_scratch_create(TopkScratch*, int64_t, int, int) { return hipSuccess; }
void topk_scratch_destroy(TopkScratch*) {}
hipError_t topk_profile_begin(TopkScratch*, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t topk_profile_finish(TopkScratch*, const float*, const float*, const DevLayer*, const DevLayer*,
                               const Tile*, int, int, const double*, const int*, int, double*, int, double*,
                               Timing*, hipStream_t) {
    return hipErrorNotSupported;
}
hipError_t topk_compress(TopkScratch*, const float*, float*, const DevLayer*, const DevLayer*, const Tile*,
                         const Tile*, int, int, uint8_t*, Timing*, hipStream_t) {
    return hipErrorNotSupported;
}

}  // namespace lgreco
