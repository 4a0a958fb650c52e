// A stand-in for the HIP virtual-memory driver calls, used ONLY by tests/test_vmm_host_logic.py: mosaic_vmm.hip is
// linked against this file instead of the runtime, so that its book-keeping -- growth in place, the fall-back when the
// driver refuses, shrinking, clean-up -- runs on the CPU, under the sanitizers, with refusals forced from the test.
// The fake checks what a driver would: ranges inside the reservation, aligned, mapped once, unmapped exactly as they
// were mapped, handles released once and only when nothing maps them.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <string>
#include <vector>

namespace {
constexpr size_t kGranularity = 2u << 20;
struct Handle {
  size_t bytes;
  bool mapped;
  bool released;
};
struct State {
  char* base = nullptr;
  size_t reserved = 0;
  std::vector<Handle> handles;                 // handle value = index + 1
  std::map<size_t, std::pair<size_t, size_t>> maps;   // offset -> (bytes, handle index)
  std::map<size_t, size_t> open;               // offset -> bytes with access set
  std::vector<std::string> log;
  int refuse_access_whole = 0, refuse_access_part = 0, refuse_create_after = -1, creates = 0, syncs = 0;
  int violations = 0;
  hipError_t last = hipSuccess;
} g;

hipError_t fail(hipError_t e) {
  g.last = e;
  return e;
}
void violation(const char* what) {
  ++g.violations;
  g.log.push_back(std::string("VIOLATION ") + what);
}
}  // namespace

extern "C" {
// ---- control surface for the test
void fake_reset() { g = State(); }
void fake_refuse(int access_whole, int access_part, int create_after) {
  g.refuse_access_whole = access_whole;
  g.refuse_access_part = access_part;
  g.refuse_create_after = create_after;
}
int fake_violations() { return g.violations; }
int fake_syncs() { return g.syncs; }
int fake_live_handles() {
  int n = 0;
  for (const Handle& h : g.handles) n += !h.released;
  return n;
}
int fake_mappings() { return (int)g.maps.size(); }
long long fake_mapped_bytes() {
  long long n = 0;
  for (const auto& m : g.maps) n += (long long)m.second.first;
  return n;
}
// 1 if every mapped byte of [0, bytes) has had access set
int fake_open_prefix(long long bytes) {
  size_t at = 0;
  while (at < (size_t)bytes) {
    bool found = false;
    for (const auto& o : g.open)
      if (o.first <= at && at < o.first + o.second) {
        at = o.first + o.second;
        found = true;
        break;
      }
    if (!found) return 0;
  }
  return 1;
}
int fake_log(char* out, int cap) {
  std::string all;
  for (const std::string& s : g.log) all += s + "\n";
  std::snprintf(out, cap, "%s", all.c_str());
  return (int)g.log.size();
}
}

// ---- the driver calls mosaic_vmm.hip makes
hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int) {
  *v = 1;
  return hipSuccess;
}
hipError_t hipGetDevice(int* d) {
  *d = 0;
  return hipSuccess;
}
hipError_t hipDeviceSynchronize() {
  ++g.syncs;
  g.log.push_back("sync");
  return hipSuccess;
}
hipError_t hipGetLastError() {
  const hipError_t e = g.last;
  g.last = hipSuccess;
  return e;
}
hipError_t hipMemGetAllocationGranularity(size_t* out, const hipMemAllocationProp*, hipMemAllocationGranularity_flags) {
  *out = kGranularity;
  return hipSuccess;
}
hipError_t hipMemAddressReserve(void** ptr, size_t size, size_t, void*, unsigned long long) {
  if (g.base != nullptr || size % kGranularity) return fail(hipErrorInvalidValue);
  g.base = reinterpret_cast<char*>(uintptr_t(1) << 40);   // never dereferenced
  g.reserved = size;
  *ptr = g.base;
  g.log.push_back("reserve " + std::to_string(size));
  return hipSuccess;
}
hipError_t hipMemAddressFree(void* ptr, size_t size) {
  if (ptr != g.base || size != g.reserved) violation("free of something that was not reserved");
  if (!g.maps.empty()) violation("reservation freed with pages still mapped");
  g.base = nullptr;
  g.log.push_back("free");
  return hipSuccess;
}
hipError_t hipMemCreate(hipMemGenericAllocationHandle_t* h, size_t size, const hipMemAllocationProp*, unsigned long long) {
  if (size == 0 || size % kGranularity) {
    violation("create of a size that is not a multiple of the granularity");
    return fail(hipErrorInvalidValue);
  }
  if (g.refuse_create_after >= 0 && g.creates >= g.refuse_create_after) return fail(hipErrorOutOfMemory);
  ++g.creates;
  g.handles.push_back({size, false, false});
  *h = reinterpret_cast<hipMemGenericAllocationHandle_t>(uintptr_t(g.handles.size()));
  g.log.push_back("create " + std::to_string(size));
  return hipSuccess;
}
hipError_t hipMemRelease(hipMemGenericAllocationHandle_t h) {
  const size_t i = size_t(reinterpret_cast<uintptr_t>(h)) - 1;
  if (i >= g.handles.size() || g.handles[i].released) {
    violation("release of a handle that is not live");
    return fail(hipErrorInvalidValue);
  }
  if (g.handles[i].mapped) violation("release of a handle that is still mapped");
  g.handles[i].released = true;
  g.log.push_back("release " + std::to_string(g.handles[i].bytes));
  return hipSuccess;
}
hipError_t hipMemMap(void* ptr, size_t size, size_t offset, hipMemGenericAllocationHandle_t h, unsigned long long) {
  const size_t i = size_t(reinterpret_cast<uintptr_t>(h)) - 1;
  const size_t at = size_t(static_cast<char*>(ptr) - g.base);
  if (i >= g.handles.size() || g.handles[i].released || g.handles[i].mapped || g.handles[i].bytes != size || offset != 0 ||
      at % kGranularity || at + size > g.reserved) {
    violation("map with arguments a driver rejects");
    return fail(hipErrorInvalidValue);
  }
  for (const auto& m : g.maps)
    if (at < m.first + m.second.first && m.first < at + size) {
      violation("map over pages that are already mapped");
      return fail(hipErrorInvalidValue);
    }
  g.maps[at] = {size, i};
  g.handles[i].mapped = true;
  g.log.push_back("map " + std::to_string(at) + " " + std::to_string(size));
  return hipSuccess;
}
hipError_t hipMemUnmap(void* ptr, size_t size) {
  const size_t at = size_t(static_cast<char*>(ptr) - g.base);
  auto it = g.maps.find(at);
  if (it == g.maps.end() || it->second.first != size) {
    violation("unmap of a range that was not mapped as one piece");
    return fail(hipErrorInvalidValue);
  }
  g.handles[it->second.second].mapped = false;
  g.maps.erase(it);
  for (auto o = g.open.begin(); o != g.open.end();)
    o = (o->first < at + size && at < o->first + o->second) ? g.open.erase(o) : std::next(o);
  g.log.push_back("unmap " + std::to_string(at) + " " + std::to_string(size));
  return hipSuccess;
}
hipError_t hipMemSetAccess(void* ptr, size_t size, const hipMemAccessDesc* desc, size_t count) {
  const size_t at = size_t(static_cast<char*>(ptr) - g.base);
  const bool whole = at == 0 && g.maps.size() > 1;
  g.log.push_back(std::string("access ") + std::to_string(at) + " " + std::to_string(size));
  if (count != 1 || desc == nullptr || desc->flags != hipMemAccessFlagsProtReadWrite) {
    violation("access descriptor");
    return fail(hipErrorInvalidValue);
  }
  if (whole && g.refuse_access_whole) return fail(hipErrorInvalidValue);
  if (at != 0 && g.refuse_access_part) return fail(hipErrorInvalidValue);
  size_t covered = at;   // the range has to be mapped from end to end
  while (covered < at + size) {
    auto it = g.maps.find(covered);
    if (it == g.maps.end()) {
      violation("access set over pages that are not mapped");
      return fail(hipErrorInvalidValue);
    }
    covered += it->second.first;
  }
  g.open[at] = size;
  return hipSuccess;
}
