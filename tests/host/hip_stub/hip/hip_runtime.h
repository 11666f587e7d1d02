// Host-only stand-in for the few HIP runtime calls the swap engine makes, so that its host logic (state machine, arena,
// planner, error paths) can be built with g++ and the address / undefined-behaviour sanitizers and run without a GPU.
// "Device" memory is host memory, copies run at once, streams are in order by construction.  Events either fire at
// once or, while hipstub_hold_events is set, stay pending until hipstub_fire_events() (to reach the code paths that
// deal with copies still in flight).
#pragma once
#include <cstdlib>
#include <cstring>
#include <set>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __restrict__
#define __launch_bounds__(...)

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorNotReady = 600, hipErrorInvalidValue = 1 };
typedef struct hipstub_stream* hipStream_t;
struct hipstub_event { bool recorded = false; bool fired = false; };
typedef hipstub_event* hipEvent_t;
enum { hipHostMallocDefault = 0, hipStreamNonBlocking = 1, hipEventDefault = 0, hipEventDisableTiming = 2 };
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 };

inline bool& hipstub_hold_events() { static bool hold = false; return hold; }
inline std::set<hipstub_event*>& hipstub_pending() { static std::set<hipstub_event*> p; return p; }
inline void hipstub_fire_events() {
    for (hipstub_event* e : hipstub_pending()) e->fired = true;
    hipstub_pending().clear();
}
inline int& hipstub_live_objects() { static int n = 0; return n; }   // streams + events + host allocations not yet destroyed

inline unsigned __float_as_uint(float f) { unsigned u; std::memcpy(&u, &f, 4); return u; }
inline float __uint_as_float(unsigned u) { float f; std::memcpy(&f, &u, 4); return f; }

inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipDeviceSynchronize() { hipstub_fire_events(); return hipSuccess; }
inline hipError_t hipHostMalloc(void** p, size_t n, unsigned) { *p = std::malloc(n); ++hipstub_live_objects(); return *p ? hipSuccess : hipErrorInvalidValue; }
inline hipError_t hipHostFree(void* p) { std::free(p); --hipstub_live_objects(); return hipSuccess; }
inline hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) { *s = (hipStream_t)std::malloc(1); ++hipstub_live_objects(); return hipSuccess; }
inline hipError_t hipStreamDestroy(hipStream_t s) { std::free(s); --hipstub_live_objects(); return hipSuccess; }
inline hipError_t hipStreamSynchronize(hipStream_t) { hipstub_fire_events(); return hipSuccess; }
inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
inline hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { *e = new hipstub_event(); ++hipstub_live_objects(); return hipSuccess; }
inline hipError_t hipEventCreate(hipEvent_t* e) { return hipEventCreateWithFlags(e, 0); }
inline hipError_t hipEventDestroy(hipEvent_t e) { hipstub_pending().erase(e); delete e; --hipstub_live_objects(); return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t e, hipStream_t) {
    e->recorded = true;
    e->fired = !hipstub_hold_events();
    if (!e->fired) hipstub_pending().insert(e);
    else hipstub_pending().erase(e);
    return hipSuccess;
}
inline hipError_t hipEventQuery(hipEvent_t e) { return (!e->recorded || e->fired) ? hipSuccess : hipErrorNotReady; }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
inline hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t) { std::memcpy(dst, src, n); return hipSuccess; }
