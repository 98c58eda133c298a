// Host-only build of libkvp's state machine: the kernel launchers are replaced by stubs (a dry-run
// cache never calls them), everything else -- validation, layout, the per-layer state machine,
// the launch planning of plan.cpp -- is the real code, compiled with -fsanitize=address,undefined.
#include "kvp_internal.h"

namespace kvp {

hipError_t launch_attention(const AttnArgs&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_colsum(const ColsumArgs&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_select(const SelectArgs&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_merge(const CompactArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_move(const CompactArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_init(int32_t*, float*, size_t, const Seg*, int, Seg*, unsigned long long*, hipStream_t) {
  return hipErrorNotSupported;
}
hipError_t launch_rowstat(RowstatArgs, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_keydiff(KeydiffArgs, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_decode(const DecodeArgs&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t decode_static_scratch(float** ptr, size_t* n_floats) {
  *ptr = nullptr;
  *n_floats = 0;
  return hipErrorNotSupported;
}
hipError_t prepare_attention() { return hipErrorNotSupported; }
hipError_t prepare_select() { return hipErrorNotSupported; }

}  // namespace kvp

// the HIP runtime calls kvp.cpp makes (events, stream waits): never reached by a dry-run cache
extern "C" {
hipError_t hipEventCreate(hipEvent_t*) { return hipErrorNotSupported; }
hipError_t hipEventCreateWithFlags(hipEvent_t*, unsigned) { return hipErrorNotSupported; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipErrorNotSupported; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipErrorNotSupported; }
hipError_t hipEventElapsedTime(float*, hipEvent_t, hipEvent_t) { return hipErrorNotSupported; }
hipError_t hipEventDestroy(hipEvent_t) { return hipErrorNotSupported; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipErrorNotSupported; }
}
