// Error text, version and the profiling-event helpers of the C ABI.
#include "common.h"

namespace roll {
char* error_buffer() {
    static thread_local char buf[kErrorBufferBytes] = {0};
    return buf;
}
}  // namespace roll

extern "C" const char* roll_last_error(void) { return roll::error_buffer(); }
extern "C" const char* roll_version(void) { return "0.5"; }

extern "C" int roll_prof_event_create(void** event) {
    if (!event) return roll::fail(ROLL_ERR_INVALID_ARG, "event is NULL");
    hipEvent_t e;
    ROLL_HIP_CHECK(hipEventCreate(&e));
    *event = (void*)e;
    return ROLL_OK;
}

extern "C" int roll_prof_event_destroy(void* event) {
    if (!event) return roll::fail(ROLL_ERR_INVALID_ARG, "event is NULL");
    ROLL_HIP_CHECK(hipEventDestroy((hipEvent_t)event));
    return ROLL_OK;
}

extern "C" int roll_prof_event_record(void* event, void* stream) {
    if (!event) return roll::fail(ROLL_ERR_INVALID_ARG, "event is NULL");
    ROLL_HIP_CHECK(hipEventRecord((hipEvent_t)event, (hipStream_t)stream));
    return ROLL_OK;
}

extern "C" int roll_prof_event_elapsed_ms(void* begin, void* end, float* ms) {
    if (!begin || !end || !ms) return roll::fail(ROLL_ERR_INVALID_ARG, "NULL argument");
    ROLL_HIP_CHECK(hipEventSynchronize((hipEvent_t)end));
    ROLL_HIP_CHECK(hipEventElapsedTime(ms, (hipEvent_t)begin, (hipEvent_t)end));
    return ROLL_OK;
}
