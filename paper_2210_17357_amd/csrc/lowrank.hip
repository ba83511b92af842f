// Low rank (stub, replaced below in the build order).
#include "internal.h"

namespace lgreco {

hipError_t lowrank_scratch_create(LowrankScratch*, int64_t, int, int) { return hipSuccess; }
void lowrank_scratch_destroy(LowrankScratch*) {}
hipError_t lowrank_profile(LowrankScratch*, const float*, const float*, const DevLayer*, const DevLayer*, int,
                           const float*, int, const int*, const int*, int, double*, int, Timing*, hipStream_t) {
    return hipErrorNotSupported;
}
hipError_t lowrank_compress(LowrankScratch*, const float*, float*, const DevLayer*, const DevLayer*, int, float*,
                            int, uint8_t*, Timing*, hipStream_t) {
    return hipErrorNotSupported;
}

}  // namespace lgreco
