// Stand-ins for the kernel launchers of libwkv, so that the host half of the library (argument
// validation, derived sizes, launch planning) links and runs on a machine without a GPU, under
// AddressSanitizer and UndefinedBehaviorSanitizer.  Each stub counts its calls and launches nothing.
#include "wkv_internal.h"

extern "C" int wkv_stub_launches = 0;

namespace wkv {
hipError_t launch_score(const Shape &, const BatchParams &, const ScorePlan &, const GroupPtrs &, int32_t, bool, float2 *,
                        float *, float *, float *, hipStream_t, hipEvent_t, const uint32_t *) { ++wkv_stub_launches; return hipSuccess; }
hipError_t launch_resident(const Shape &, const BatchParams &, const ResidentPlan &, const GroupPtrs &, int32_t,
                           unsigned long long *, float *, uint32_t *, float *, float *, hipStream_t) { ++wkv_stub_launches; return hipSuccess; }
hipError_t launch_pool(const Shape &, const BatchParams &, int32_t, const float *, float *, hipStream_t) { ++wkv_stub_launches; return hipSuccess; }
hipError_t launch_topk(const Shape &, const BatchParams &, const GroupK &, int32_t, const float *, int32_t *, int32_t *,
                       int32_t *, hipStream_t) { ++wkv_stub_launches; return hipSuccess; }
hipError_t launch_select(const Shape &, const BatchParams &, const GroupK &, int32_t, const float *, int32_t *, int32_t *,
                         int32_t *, hipStream_t) { ++wkv_stub_launches; return hipSuccess; }
hipError_t launch_gather(const Shape &, const LayerPtrs &, int32_t, int32_t, const int32_t *, const int32_t *, hipStream_t) {
  ++wkv_stub_launches; return hipSuccess;
}
hipError_t launch_jaccard(const Shape &, int32_t, const int32_t *, const int32_t *, float *, hipStream_t) { ++wkv_stub_launches; return hipSuccess; }
hipError_t launch_decode(const DecodeShape &, const void *, const void *, const void *, void *, void *, int32_t *, float *,
                         float *, hipStream_t) { ++wkv_stub_launches; return hipSuccess; }
hipError_t launch_decode_static(const DecodeShape &, const void *, const void *, const void *, void *, void *, int32_t *,
                                float *, hipStream_t) { ++wkv_stub_launches; return hipSuccess; }
}  // namespace wkv
