// A stand-in for the HIP runtime, for running the HOST side of libmoonwalk on a machine without a GPU under
// AddressSanitizer / UBSan. "Device" memory is zeroed host memory (so the sanitizer sees every host-side
// copy to and from it), kernel launches only have their launch configuration checked and are otherwise
// ignored, and every device-side flag the library reads back is therefore 0. Test infrastructure only.
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>

namespace {
std::mutex g_lock;
std::map<const void*, void*> g_symbols;  // host handle of a __device__ variable -> its fake device copy
struct FreeSymbolsAtExit {
  ~FreeSymbolsAtExit() {
    for (auto& kv : g_symbols) free(kv.second);
    g_symbols.clear();
  }
} g_free_symbols;
thread_local hipError_t g_last = hipSuccess;
unsigned long long g_launches = 0, g_bad_launches = 0;
struct CallConfig {
  dim3 grid, block;
  size_t shmem;
  hipStream_t stream;
};
thread_local CallConfig g_cfg[8];
thread_local int g_cfg_depth = 0;
}  // namespace

extern "C" {

unsigned long long fake_hip_launches() { return g_launches; }
unsigned long long fake_hip_bad_launches() { return g_bad_launches; }
// launch configurations pushed by the calling thread that no launch has taken up (must be 0 between calls)
int fake_hip_pending_configurations() { return g_cfg_depth; }

hipError_t hipMalloc(void** ptr, size_t size) {
  if (!ptr) return hipErrorInvalidValue;
  *ptr = calloc(size ? size : 1, 1);
  return *ptr ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void* p) {
  free(p);
  return hipSuccess;
}
hipError_t hipMemcpy(void* dst, const void* src, size_t bytes, hipMemcpyKind) {
  if (bytes && (!dst || !src)) return hipErrorInvalidValue;
  memmove(dst, src, bytes);
  return hipSuccess;
}
// streams and events are tokens: everything "runs" at once, in program order
hipError_t hipStreamCreateWithFlags(hipStream_t* stream, unsigned) {
  if (!stream) return hipErrorInvalidValue;
  *stream = reinterpret_cast<hipStream_t>(malloc(8));
  return *stream ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipStreamDestroy(hipStream_t stream) {
  free(stream);
  return hipSuccess;
}
hipError_t hipEventCreateWithFlags(hipEvent_t* event, unsigned) {
  if (!event) return hipErrorInvalidValue;
  *event = reinterpret_cast<hipEvent_t>(malloc(8));
  return *event ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipEventDestroy(hipEvent_t event) {
  free(event);
  return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t event, hipStream_t) { return event ? hipSuccess : hipErrorInvalidHandle; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t event, unsigned) { return event ? hipSuccess : hipErrorInvalidHandle; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipDeviceSynchronize() { return hipSuccess; }
hipError_t hipGetLastError() {
  hipError_t e = g_last;
  g_last = hipSuccess;
  return e;
}
const char* hipGetErrorString(hipError_t e) { return e == hipSuccess ? "no error" : "fake HIP runtime error"; }
hipError_t hipGetDevice(int* dev) {
  if (!dev) return hipErrorInvalidValue;
  *dev = 0;
  return hipSuccess;
}
hipError_t hipFuncSetAttribute(const void* func, hipFuncAttribute, int value) {
  return (func && value >= 0 && value <= 160 * 1024) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t hipGetSymbolAddress(void** devPtr, const void* symbol) {
  std::lock_guard<std::mutex> guard(g_lock);
  auto it = g_symbols.find(symbol);
  if (!devPtr || it == g_symbols.end()) return hipErrorInvalidSymbol;
  *devPtr = it->second;
  return hipSuccess;
}

// What a launch must satisfy on the real machine: a non-empty grid, at most 1024 threads per
// workgroup, at most 160 KiB of LDS, grid dimensions within the hardware's limits.
hipError_t hipLaunchKernel(const void* func, dim3 grid, dim3 block, void** args, size_t shmem, hipStream_t) {
  ++g_launches;
  const unsigned long long threads = (unsigned long long)block.x * block.y * block.z;
  const bool ok = func && args && grid.x >= 1 && grid.y >= 1 && grid.z >= 1 && grid.y <= 65535 && grid.z <= 65535 &&
                  grid.x <= 0x7FFFFFFFu && threads >= 1 && threads <= 1024 && shmem <= 160 * 1024;
  if (!ok) {
    ++g_bad_launches;
    fprintf(stderr, "fake HIP: invalid launch grid (%u,%u,%u) block (%u,%u,%u) lds %zu\n", grid.x, grid.y, grid.z, block.x,
            block.y, block.z, shmem);
    g_last = hipErrorInvalidConfiguration;
    return g_last;
  }
  return hipSuccess;
}
hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t shmem, hipStream_t stream) {
  if (g_cfg_depth >= 8) return hipErrorInvalidValue;
  g_cfg[g_cfg_depth++] = CallConfig{grid, block, shmem, stream};
  return hipSuccess;
}
hipError_t __hipPopCallConfiguration(dim3* grid, dim3* block, size_t* shmem, hipStream_t* stream) {
  if (g_cfg_depth <= 0) return hipErrorInvalidValue;
  const CallConfig& c = g_cfg[--g_cfg_depth];
  *grid = c.grid;
  *block = c.block;
  *shmem = c.shmem;
  *stream = c.stream;
  return hipSuccess;
}

static void* g_module_token[1];
void** __hipRegisterFatBinary(const void*) { return g_module_token; }
void __hipUnregisterFatBinary(void**) {}
void __hipRegisterFunction(void**, const void*, char*, const char*, unsigned, void*, void*, void*, void*, int*) {}
void __hipRegisterVar(void**, void* var, char*, char*, int, size_t size, int, int) {
  std::lock_guard<std::mutex> guard(g_lock);
  if (!g_symbols.count(var)) {
    g_symbols[var] = calloc(size ? size : 1, 1);
  }
}
void __hipRegisterManagedVar(void*, void**, void*, const char*, size_t, unsigned) {}
}
