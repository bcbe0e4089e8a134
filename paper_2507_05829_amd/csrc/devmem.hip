// Device allocations with optional guard zones (see devmem.hpp).
#include "devmem.hpp"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>

#include "lop.h"

namespace lop {
namespace {

constexpr unsigned char kPattern = 0xC3;

struct Guarded {
  void* base;
  size_t bytes;
};

std::mutex g_mu;
std::map<void*, Guarded> g_live;  // user pointer -> allocation
int g_violations = 0;

size_t guard_bytes() {
  static const size_t n = [] {
    const char* e = std::getenv("LOP_GUARD_BYTES");
    const long v = e ? std::atol(e) : 0;
    return v > 0 ? (size_t)((v + 255) / 256 * 256) : (size_t)0;
  }();
  return n;
}

// Number of guard bytes around `user` that no longer hold the pattern (0: intact).
size_t damaged(void* user, const Guarded& g) {
  const size_t n = guard_bytes();
  const size_t slack = (g.bytes + 255) / 256 * 256 - g.bytes;  // the rounding behind the body is guarded too
  std::vector<unsigned char> host(n + slack);
  size_t bad = 0;
  for (int side = 0; side < 2; ++side) {
    const char* src = side == 0 ? (const char*)g.base : (const char*)user + g.bytes;
    const size_t len = side == 0 ? n : n + slack;
    if (hipMemcpy(host.data(), src, len, hipMemcpyDeviceToHost) != hipSuccess) return (size_t)-1;
    for (size_t i = 0; i < len; ++i) bad += host[i] != kPattern;
    if (bad) {
      size_t first = 0;
      while (first < len && host[first] == kPattern) ++first;
      std::fprintf(stderr, "lop: guard %s an allocation of %zu bytes was overwritten (%zu bytes, first at offset %zu)\n",
                   side == 0 ? "in front of" : "behind", g.bytes, bad, first);
    }
  }
  return bad;
}

}  // namespace

hipError_t dev_alloc(void** p, size_t bytes) {
  const size_t n = guard_bytes();
  if (!n) return hipMalloc(p, bytes);
  const size_t body = (bytes + 255) / 256 * 256;
  void* base = nullptr;
  hipError_t e = hipMalloc(&base, body + 2 * n);
  if (e != hipSuccess) return e;
  e = hipMemset(base, kPattern, n);
  if (e == hipSuccess) e = hipMemset((char*)base + n + bytes, kPattern, body - bytes + n);
  if (e != hipSuccess) {
    (void)hipFree(base);
    return e;
  }
  *p = (char*)base + n;
  std::lock_guard<std::mutex> lock(g_mu);
  g_live[*p] = Guarded{base, bytes};
  return hipSuccess;
}

hipError_t dev_free(void* p) {
  if (!p) return hipSuccess;
  if (!guard_bytes()) return hipFree(p);
  Guarded g{};
  {
    std::lock_guard<std::mutex> lock(g_mu);
    auto it = g_live.find(p);
    if (it == g_live.end()) return hipErrorInvalidValue;
    g = it->second;
    g_live.erase(it);
  }
  if (damaged(p, g)) {
    std::lock_guard<std::mutex> lock(g_mu);
    ++g_violations;
  }
  return hipFree(g.base);
}

}  // namespace lop

extern "C" int lop_debug_guard_check(void) {
  if (!lop::guard_bytes()) return 0;
  if (hipDeviceSynchronize() != hipSuccess) return LOP_ERR_HIP;
  std::lock_guard<std::mutex> lock(lop::g_mu);
  int bad = lop::g_violations;
  for (auto& kv : lop::g_live) bad += lop::damaged(kv.first, kv.second) ? 1 : 0;
  return bad;
}
