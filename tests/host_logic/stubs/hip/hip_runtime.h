// Minimal stand-in for the HIP runtime header: just enough for the library's host-only file path to compile and run
// on a machine without a GPU (tests only).
#pragma once
#include <stdint.h>
#include <stddef.h>
typedef int hipError_t;
#define hipSuccess 0
typedef struct ihipStream_t* hipStream_t;
typedef struct ihipEvent_t* hipEvent_t;
inline const char* hipGetErrorString(hipError_t) { return "stub"; }
inline hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t e);   // defined by the harness
