/* Stand-in for <hip/hip_runtime.h> when the host side of the library (argument checks, plan,
 * launch geometry, workspace layout) is built with a plain C++ compiler for the sanitizer run.
 * Only what that code names; nothing here touches a GPU. */
#pragma once
#include <stddef.h>
#include <stdint.h>

#define __host__
#define __device__
#define __global__
#define __forceinline__ inline
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))

typedef void* hipStream_t;
typedef enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorNoDevice = 100, hipErrorLaunchFailure = 719 } hipError_t;

/* no device in this build: the one call that asks for one says so */
static inline hipError_t hipGetDevice(int* dev) { *dev = -1; return hipErrorNoDevice; }
static inline hipError_t hipGetSymbolAddress(void** ptr, const void* symbol) { *ptr = (void*)symbol; return hipSuccess; }
static inline hipError_t hipGetLastError(void) { return hipSuccess; }
