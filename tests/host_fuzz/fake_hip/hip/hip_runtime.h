// CPU stand-in for the few HIP runtime calls that the staging pool (csrc/sdl_offload.cpp) makes, so that its
// host logic can run under sanitizers without a GPU: "device" memory is host memory, copies are done at once
// (in issue order, which is the order a single copy stream would give them), events and waits do nothing.
// Used only by tests/test_host_sanitizers.py.
#pragma once
#include <cstddef>
#include <cstring>
typedef int hipError_t;
typedef struct fake_stream* hipStream_t;
typedef struct fake_event* hipEvent_t;
enum { hipSuccess = 0 };
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 };
enum { hipEventDisableTiming = 2 };
extern long fake_hip_copies, fake_hip_bytes;
inline hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind, hipStream_t)
{
    std::memcpy(dst, src, bytes);
    ++fake_hip_copies; fake_hip_bytes += (long)bytes;
    return hipSuccess;
}
inline hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { *e = reinterpret_cast<hipEvent_t>(new char); return hipSuccess; }
inline hipError_t hipEventDestroy(hipEvent_t e) { delete reinterpret_cast<char*>(e); return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
