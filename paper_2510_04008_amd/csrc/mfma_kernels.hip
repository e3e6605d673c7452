// placeholder until the MFMA family lands
#include "internal.h"
namespace race {
bool mfma_supported(int, int, int) { return false; }
size_t mfma_projection_bytes(const Plan &) { return 0; }
void mfma_pack_projection(const Plan &, const float *, void *) {}
hipError_t mfma_fwd(const Plan &, const void *, const void *, const void *, void *, float *, char *, hipStream_t) { return hipErrorNotSupported; }
hipError_t mfma_bwd(const Plan &, const void *, const void *, const void *, const void *, const float *, const void *, void *, void *, void *, char *, hipStream_t) { return hipErrorNotSupported; }
hipError_t mfma_hash(const Plan &, const void *, uint8_t *, float *, char *, hipStream_t) { return hipErrorNotSupported; }
hipError_t mfma_buckets(const Plan &, const void *, const void *, float *, float *, char *, hipStream_t) { return hipErrorNotSupported; }
}
