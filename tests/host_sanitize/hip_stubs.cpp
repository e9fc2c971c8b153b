// Stand-ins for the HIP runtime, for the host-only sanitizer build of the library (tests/test_host_sanitizers.py).
// The checker only exercises paths that end before any device work; should one of them reach the runtime after
// all, these report "no device" (or do nothing, for the start-up registration of kernels) instead of touching a
// driver.  C linkage: the real declarations' parameter lists do not matter to the linker.
#include <cstddef>
extern "C" {
enum { kNoDevice = 100 };  // hipErrorNoDevice
void** __hipRegisterFatBinary(const void*) { static void* handle; return &handle; }
void __hipUnregisterFatBinary(void**) {}
void __hipRegisterFunction(void**, const void*, char*, const char*, unsigned, void*, void*, void*, void*, int*) {}
void __hipRegisterVar(void**, void*, char*, char*, int, size_t, int, int) {}
int __hipPushCallConfiguration(...) { return kNoDevice; }
int __hipPopCallConfiguration(...) { return kNoDevice; }
int hipLaunchKernel(...) { return kNoDevice; }
int hipGetLastError() { return kNoDevice; }
int hipStreamWaitEvent(...) { return kNoDevice; }
int hipStreamIsCapturing(...) { return kNoDevice; }
int hipFuncSetAttribute(...) { return kNoDevice; }
int hipEventRecord(...) { return kNoDevice; }
int hipEventCreate(...) { return kNoDevice; }
int hipEventCreateWithFlags(...) { return kNoDevice; }
int hipEventSynchronize(...) { return kNoDevice; }
int hipEventElapsedTime(...) { return kNoDevice; }
int hipEventDestroy(...) { return kNoDevice; }
int hipStreamSynchronize(...) { return kNoDevice; }
int hipStreamDestroy(...) { return kNoDevice; }
int hipStreamCreateWithFlags(...) { return kNoDevice; }
int hipGetSymbolAddress(...) { return kNoDevice; }
int hipGetDevice(...) { return kNoDevice; }
int hipMemsetAsync(...) { return kNoDevice; }
int hipMemcpyAsync(...) { return kNoDevice; }
}
