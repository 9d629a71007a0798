// A stand-in for the HIP runtime, linked in its place under the host-side objects of libqnn when they are
// built for the sanitizer run (tests/test_sanitized_host.py).  Registration of device code is a no-op (there is
// none: the objects are compiled host-only), and every call that would touch a device counts itself, so the
// driver can assert that an entry point rejected its arguments before making any HIP call.
//
// The HIP headers are deliberately not included: the functions below are defined with C linkage and
// ABI-compatible parameter types of their own (an enum return is an int, dim3 is three 32-bit unsigned).
#include <stddef.h>

typedef int hipError_t;
typedef void *hipStream_t;
typedef int hipDeviceAttribute_t;
struct dim3 {
    unsigned x, y, z;
};
enum { hipSuccess = 0, hipErrorNoDevice = 100 };

static int g_device_calls = 0;

extern "C" int hipstub_device_calls(void) { return g_device_calls; }

extern "C" {
void **__hipRegisterFatBinary(const void *) { static void *handle = nullptr; return &handle; }
void __hipUnregisterFatBinary(void **) {}
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
void __hipRegisterVar(void **, void *, char *, const char *, int, size_t, int, int) {}
hipError_t __hipPushCallConfiguration(dim3, dim3, size_t, hipStream_t) { ++g_device_calls; return hipSuccess; }
hipError_t __hipPopCallConfiguration(dim3 *, dim3 *, size_t *, hipStream_t *) { ++g_device_calls; return hipSuccess; }
hipError_t hipLaunchKernel(const void *, dim3, dim3, void **, size_t, hipStream_t) { ++g_device_calls; return hipErrorNoDevice; }
hipError_t hipGetLastError(void) { ++g_device_calls; return hipErrorNoDevice; }
hipError_t hipGetDevice(int *) { ++g_device_calls; return hipErrorNoDevice; }
hipError_t hipDeviceGetAttribute(int *, hipDeviceAttribute_t, int) { ++g_device_calls; return hipErrorNoDevice; }
hipError_t hipGetSymbolAddress(void **, const void *) { ++g_device_calls; return hipErrorNoDevice; }
hipError_t hipOccupancyMaxActiveBlocksPerMultiprocessor(int *, const void *, int, size_t) { ++g_device_calls; return hipErrorNoDevice; }
const char *hipGetErrorString(hipError_t) { return "no device (stub runtime)"; }
}
