// Stand-ins for the kernel launchers of libhkv, so that the host planner (csrc/hkv_api.hip) links into a
// CPU-only program built with AddressSanitizer and UndefinedBehaviorSanitizer.  The fuzz driver never reaches
// them: it calls only entry points that plan on the host.
#include "hkv_internal.h"

#include <cstdlib>

namespace hkv {
static hipError_t never() { std::abort(); }
hipError_t launch_chunk_score_sum(const CacheView&, int, int, int, int, int, const void*, hipStream_t, hipEvent_t, hipEvent_t) {
  return never();
}
hipError_t launch_chunk_score_max(const CacheView&, int, int, int, int, const void*, int, hipStream_t) { return never(); }
hipError_t launch_decode(const CacheView&, int, int, int, int, int, int, int, const void*, const void*, const void*, float*,
                         float*, void*, int, int, int, int, hipStream_t, hipEvent_t, hipEvent_t) { return never(); }
hipError_t launch_dynamic_tiles(const CacheView&, int, int, int, int, int, int, int, const void*, const void*, const void*,
                                float*, float*, void*, int, int, int, int, void*, int, hipStream_t, hipEvent_t, hipEvent_t) {
  return never();
}
hipError_t launch_units(const CacheView&, int, int, int, int, int, int, const void*, const void*, const void*, void*, int, int,
                        hipStream_t, hipEvent_t, hipEvent_t) { return never(); }
hipError_t launch_attn_merge(const CacheView&, int, const UnitDesc*, int, int, int, int, float*, float*, void*, int, int,
                             hipStream_t, hipEvent_t, hipEvent_t) { return never(); }
hipError_t launch_stream(const CacheView&, int, const StreamBound*, int, int, int, const void*, const void*, const void*,
                         float*, float*, void*, int, int, hipStream_t, hipEvent_t, hipEvent_t) { return never(); }
hipError_t launch_stream_merge(const CacheView&, int, const StreamMulti*, int, int, int, int, float*, float*, void*, int,
                               hipStream_t, hipEvent_t, hipEvent_t) { return never(); }
hipError_t launch_rewind(const CacheView&, int, int, hipStream_t) { return never(); }
hipError_t launch_full_attn(const FullView&, int, const void*, const void*, const void*, float*, float*, void*, hipStream_t) { return never(); }
hipError_t launch_score(const CacheView&, int, int, int, int, int, const void*, const void*, int64_t, float2*, float2*,
                        int, hipStream_t) { return never(); }
hipError_t launch_select(const CacheView&, int, int, hipStream_t) { return never(); }
hipError_t launch_compact(const CacheView&, int, int, int, int, int, const void*, const void*, int64_t, hipStream_t) { return never(); }
hipError_t launch_adopt(const CacheView&, int, int, int, int, int, int, const void*, const void*, int64_t, hipStream_t) { return never(); }
}  // namespace hkv
