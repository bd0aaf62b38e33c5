// The four HIP runtime calls surgeon_host.cpp references (its kernel timing aid), as inert stand-ins: the sanitizer run
// exercises host arithmetic only and must not load the GPU runtime.
#include <hip/hip_runtime_api.h>

extern "C" {
hipError_t hipEventCreate(hipEvent_t* e) { *e = nullptr; return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
}
