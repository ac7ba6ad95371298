// Test-only stand-ins for the four HIP runtime calls the shard-plan code makes, backed by host memory, so
// that plan construction (counting sort, tile lists, their copies) can run on a machine without a GPU under
// AddressSanitizer / UndefinedBehaviorSanitizer.  "Device" arrays are then heap blocks the sanitizer guards.
// Linked into the sanitizer test executable only; the library itself always links the real runtime.
#include <hip/hip_runtime.h>
#include <cstdlib>
#include <cstring>

extern "C" {
hipError_t hipMalloc(void **p, size_t n) {
    *p = malloc(n ? n : 1);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *p) {
    free(p);
    return hipSuccess;
}
hipError_t hipMemcpy(void *dst, const void *src, size_t n, hipMemcpyKind) {
    memcpy(dst, src, n);
    return hipSuccess;
}
hipError_t hipGetDevice(int *d) {
    *d = 0;
    return hipSuccess;
}
}
