/* Stand-in for the HIP runtime header, for the host-only sanitizer build of the library's argument checks: every
 * runtime call fails, so only the code in front of the first HIP call is exercised (it must reject bad arguments on
 * a machine without a GPU). */
#ifndef KSA_TEST_HIP_STUB_H_
#define KSA_TEST_HIP_STUB_H_
#include <stddef.h>
typedef int hipError_t;
enum { hipSuccess = 0, hipErrorNoDevice = 100 };
enum hipMemcpyKind { hipMemcpyHostToDevice = 1 };
static inline hipError_t hipGetDevice(int *dev) { *dev = -1; return hipErrorNoDevice; }
static inline hipError_t hipMalloc(void **p, size_t) { *p = 0; return hipErrorNoDevice; }
static inline hipError_t hipFree(void *) { return hipSuccess; }
static inline hipError_t hipMemcpy(void *, const void *, size_t, hipMemcpyKind) { return hipErrorNoDevice; }
#endif
