// A stand-in for the HIP runtime, for running the library's HOST code on a machine without a
// GPU under AddressSanitizer / UBSan. Test infrastructure only: nothing in the product links it.
//
// Device memory is host memory (hipMalloc = malloc, copies = memcpy, so the sanitizer checks
// every upload against both the host vector and the "device" allocation); kernel launches do
// nothing; streams, events, graphs and graph executables are counted handles whose life the
// stub tracks. Any misuse the real runtime would answer with undefined behaviour (use after
// destroy, double destroy, freeing a pointer that was never allocated, elapsed time between
// events that were never recorded, synchronising a capturing stream, a capture that records a
// memset) is reported on stderr and ends the process with abort(), so a test sees it.
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>

namespace {

enum Kind { kStream, kEvent, kGraph, kExec, kAlloc, kKinds };
const char* const kKindName[kKinds] = {"stream", "event", "graph", "graph exec", "allocation"};

struct Handle {
  Kind kind;
  bool alive = true;
  bool recorded = false;   // event
  bool capturing = false;  // stream
  const void* on = nullptr; // event: the stream it was last recorded on
  size_t bytes = 0;        // allocation
};

std::mutex g_mu;
std::map<const void*, Handle> g_handles;  // every handle ever handed out (addresses are not reused:
                                          // handle objects are leaked on purpose, allocations are
                                          // quarantined by the sanitizer)
std::map<const void*, size_t> g_pinned;   // host ranges registered as mapped pinned memory
long g_launches = 0, g_created[kKinds] = {0}, g_live[kKinds] = {0};

[[noreturn]] void die(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  std::fprintf(stderr, "hipstub: MISUSE: ");
  std::vfprintf(stderr, fmt, ap);
  std::fprintf(stderr, "\n");
  va_end(ap);
  std::abort();
}

void* make(Kind k, void* at = nullptr, size_t bytes = 0) {
  if (!at) at = std::malloc(16);  // a unique address; never freed, so never handed out twice
  Handle h;
  h.kind = k;
  h.bytes = bytes;
  g_handles[at] = h;
  ++g_created[k];
  ++g_live[k];
  return at;
}

Handle& use(const void* p, Kind k, const char* what) {
  auto it = g_handles.find(p);
  if (it == g_handles.end() || it->second.kind != k) die("%s: %p is not a %s", what, p, kKindName[k]);
  if (!it->second.alive) die("%s: %s %p was already destroyed", what, kKindName[k], p);
  return it->second;
}

void kill(const void* p, Kind k, const char* what) {
  Handle& h = use(p, k, what);
  h.alive = false;
  --g_live[k];
}

// nullptr is the null stream
Handle* use_stream(hipStream_t s, const char* what) {
  return s ? &use(s, kStream, what) : nullptr;
}

thread_local struct { dim3 grid, block; size_t shmem; hipStream_t stream; } t_cfg;

}  // namespace

extern "C" {

// ---- test hooks
void hipstub_pin(void* p, size_t bytes) { std::lock_guard<std::mutex> l(g_mu); g_pinned[p] = bytes; }
void hipstub_unpin(void* p) { std::lock_guard<std::mutex> l(g_mu); g_pinned.erase(p); }
long hipstub_live(int kind) { std::lock_guard<std::mutex> l(g_mu); return kind >= 0 && kind < kKinds ? g_live[kind] : -1; }
long hipstub_created(int kind) { std::lock_guard<std::mutex> l(g_mu); return kind >= 0 && kind < kKinds ? g_created[kind] : -1; }
long hipstub_launches(void) { std::lock_guard<std::mutex> l(g_mu); return g_launches; }

// ---- what hipcc's host code calls around a kernel launch
void** __hipRegisterFatBinary(const void*) { static void* h = nullptr; return &h; }
void __hipUnregisterFatBinary(void**) {}
void __hipRegisterFunction(void**, const void*, char*, const char*, unsigned, void*, void*, void*, void*, int*) {}
void __hipRegisterVar(void**, void*, char*, const char*, int, size_t, int, int) {}
hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t shmem, hipStream_t stream) {
  t_cfg = {grid, block, shmem, stream};
  return hipSuccess;
}
hipError_t __hipPopCallConfiguration(dim3* grid, dim3* block, size_t* shmem, hipStream_t* stream) {
  *grid = t_cfg.grid; *block = t_cfg.block; *shmem = t_cfg.shmem; *stream = t_cfg.stream;
  return hipSuccess;
}

static hipError_t launch(const void* fn, dim3 grid, dim3 block, hipStream_t s, const char* what) {
  std::lock_guard<std::mutex> l(g_mu);
  if (!fn) die("%s: null kernel", what);
  use_stream(s, what);
  if (!grid.x || !grid.y || !grid.z || !block.x || !block.y || !block.z) die("%s: empty grid or block", what);
  if ((size_t)block.x * block.y * block.z > 1024) die("%s: block of more than 1024 threads", what);
  if (grid.y > 65535 || grid.z > 65535) die("%s: grid.y or grid.z above 65535", what);
  ++g_launches;
  return hipSuccess;
}
hipError_t hipLaunchKernel(const void* fn, dim3 grid, dim3 block, void**, size_t, hipStream_t s) {
  return launch(fn, grid, block, s, "hipLaunchKernel");
}
hipError_t hipExtLaunchKernel(const void* fn, dim3 grid, dim3 block, void**, size_t, hipStream_t s,
                              hipEvent_t start, hipEvent_t stop, int) {
  const hipError_t e = launch(fn, grid, block, s, "hipExtLaunchKernel");
  std::lock_guard<std::mutex> l(g_mu);
  if (start) use(start, kEvent, "hipExtLaunchKernel start").recorded = true;
  if (stop) use(stop, kEvent, "hipExtLaunchKernel stop").recorded = true;
  return e;
}

// ---- device
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipSetDevice(int d) { return d == 0 ? hipSuccess : hipErrorInvalidDevice; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipDeviceSynchronize(void) {
  std::lock_guard<std::mutex> l(g_mu);
  for (auto& kv : g_handles)
    if (kv.second.kind == kStream && kv.second.alive && kv.second.capturing)
      die("hipDeviceSynchronize while stream %p is capturing", kv.first);
  return hipSuccess;
}
hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t attr, int) {
  *v = attr == hipDeviceAttributeMultiprocessorCount ? 256 : 1;
  return hipSuccess;
}

// ---- memory
hipError_t hipMalloc(void** p, size_t bytes) {
  void* m = std::malloc(bytes ? bytes : 1);
  if (!m) return hipErrorOutOfMemory;
  std::memset(m, 0xA5, bytes);
  std::lock_guard<std::mutex> l(g_mu);
  make(kAlloc, m, bytes);
  *p = m;
  return hipSuccess;
}
hipError_t hipFree(void* p) {
  if (!p) return hipSuccess;
  {
    std::lock_guard<std::mutex> l(g_mu);
    kill(p, kAlloc, "hipFree");
    g_handles.erase(p);  // malloc may hand the address out again
  }
  std::free(p);
  return hipSuccess;
}
hipError_t hipMemcpy(void* dst, const void* src, size_t n, hipMemcpyKind) {
  std::memmove(dst, src, n);
  return hipSuccess;
}
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t s) {
  { std::lock_guard<std::mutex> l(g_mu); use_stream(s, "hipMemcpyAsync"); }
  std::memmove(dst, src, n);
  return hipSuccess;
}
hipError_t hipMemcpy2DAsync(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width,
                            size_t height, hipMemcpyKind, hipStream_t s) {
  { std::lock_guard<std::mutex> l(g_mu); use_stream(s, "hipMemcpy2DAsync"); }
  if (width > dpitch || width > spitch) die("hipMemcpy2DAsync: width above a pitch");
  for (size_t r = 0; r < height; ++r) std::memmove((char*)dst + r * dpitch, (const char*)src + r * spitch, width);
  return hipSuccess;
}
hipError_t hipMemset(void* p, int v, size_t n) { std::memset(p, v, n); return hipSuccess; }
hipError_t hipMemsetAsync(void* p, int v, size_t n, hipStream_t s) {
  {
    std::lock_guard<std::mutex> l(g_mu);
    Handle* h = use_stream(s, "hipMemsetAsync");
    if (h && h->capturing) die("hipMemsetAsync recorded into a capture");
  }
  std::memset(p, v, n);
  return hipSuccess;
}
hipError_t hipPointerGetAttributes(hipPointerAttribute_t* a, const void* p) {
  std::lock_guard<std::mutex> l(g_mu);
  std::memset(a, 0, sizeof(*a));
  for (const auto& kv : g_pinned)
    if ((const char*)p >= (const char*)kv.first && (const char*)p < (const char*)kv.first + kv.second) {
      a->type = hipMemoryTypeHost;
      a->hostPointer = const_cast<void*>(p);
      a->devicePointer = const_cast<void*>(p);
      return hipSuccess;
    }
  for (const auto& kv : g_handles)
    if (kv.second.kind == kAlloc && kv.second.alive && (const char*)p >= (const char*)kv.first &&
        (const char*)p < (const char*)kv.first + kv.second.bytes) {
      a->type = hipMemoryTypeDevice;
      a->devicePointer = const_cast<void*>(p);
      return hipSuccess;
    }
  return hipErrorInvalidValue;  // pageable host memory
}

// ---- streams
hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) {
  std::lock_guard<std::mutex> l(g_mu);
  *s = (hipStream_t)make(kStream);
  return hipSuccess;
}
hipError_t hipStreamDestroy(hipStream_t s) {
  std::lock_guard<std::mutex> l(g_mu);
  if (use(s, kStream, "hipStreamDestroy").capturing) die("hipStreamDestroy of capturing stream %p", (void*)s);
  // house rule of the library (stricter than the API): an event is released before the stream
  // it was recorded on, so that no live event ever refers to a stream that is gone
  for (const auto& kv : g_handles)
    if (kv.second.kind == kEvent && kv.second.alive && kv.second.on == (const void*)s)
      die("hipStreamDestroy of stream %p while event %p recorded on it is alive", (void*)s, kv.first);
  kill(s, kStream, "hipStreamDestroy");
  return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t s) {
  std::lock_guard<std::mutex> l(g_mu);
  Handle* h = use_stream(s, "hipStreamSynchronize");
  if (h && h->capturing) die("hipStreamSynchronize of capturing stream %p", (void*)s);
  return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned) {
  std::lock_guard<std::mutex> l(g_mu);
  use_stream(s, "hipStreamWaitEvent");
  use(e, kEvent, "hipStreamWaitEvent");
  return hipSuccess;
}
hipError_t hipStreamBeginCapture(hipStream_t s, hipStreamCaptureMode) {
  std::lock_guard<std::mutex> l(g_mu);
  Handle& h = use(s, kStream, "hipStreamBeginCapture");
  if (h.capturing) die("hipStreamBeginCapture: %p is capturing already", (void*)s);
  h.capturing = true;
  return hipSuccess;
}
hipError_t hipStreamEndCapture(hipStream_t s, hipGraph_t* g) {
  std::lock_guard<std::mutex> l(g_mu);
  Handle& h = use(s, kStream, "hipStreamEndCapture");
  if (!h.capturing) die("hipStreamEndCapture: %p is not capturing", (void*)s);
  h.capturing = false;
  *g = (hipGraph_t)make(kGraph);
  return hipSuccess;
}

// ---- events
hipError_t hipEventCreate(hipEvent_t* e) {
  std::lock_guard<std::mutex> l(g_mu);
  *e = (hipEvent_t)make(kEvent);
  return hipSuccess;
}
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { return hipEventCreate(e); }
hipError_t hipEventDestroy(hipEvent_t e) {
  std::lock_guard<std::mutex> l(g_mu);
  kill(e, kEvent, "hipEventDestroy");
  return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s) {
  std::lock_guard<std::mutex> l(g_mu);
  use_stream(s, "hipEventRecord");
  Handle& h = use(e, kEvent, "hipEventRecord");
  h.recorded = true;
  h.on = s;
  return hipSuccess;
}
hipError_t hipEventSynchronize(hipEvent_t e) {
  std::lock_guard<std::mutex> l(g_mu);
  use(e, kEvent, "hipEventSynchronize");
  return hipSuccess;
}
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b) {
  std::lock_guard<std::mutex> l(g_mu);
  if (!use(a, kEvent, "hipEventElapsedTime").recorded || !use(b, kEvent, "hipEventElapsedTime").recorded)
    die("hipEventElapsedTime between events that were never recorded");
  *ms = 0.01f;
  return hipSuccess;
}

// ---- graphs
hipError_t hipGraphInstantiate(hipGraphExec_t* x, hipGraph_t g, hipGraphNode_t*, char*, size_t) {
  std::lock_guard<std::mutex> l(g_mu);
  use(g, kGraph, "hipGraphInstantiate");
  *x = (hipGraphExec_t)make(kExec);
  return hipSuccess;
}
hipError_t hipGraphLaunch(hipGraphExec_t x, hipStream_t s) {
  std::lock_guard<std::mutex> l(g_mu);
  use(x, kExec, "hipGraphLaunch");
  use_stream(s, "hipGraphLaunch");
  return hipSuccess;
}
hipError_t hipGraphDestroy(hipGraph_t g) {
  std::lock_guard<std::mutex> l(g_mu);
  kill(g, kGraph, "hipGraphDestroy");
  return hipSuccess;
}
hipError_t hipGraphExecDestroy(hipGraphExec_t x) {
  std::lock_guard<std::mutex> l(g_mu);
  kill(x, kExec, "hipGraphExecDestroy");
  return hipSuccess;
}

hipError_t hipGetSymbolAddress(void** p, const void* symbol) {
  // a __device__ array's host-side stand-in is a host object of the same size: use it
  *p = const_cast<void*>(symbol);
  return hipSuccess;
}

}  // extern "C"
