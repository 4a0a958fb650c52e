// Workspace on virtual memory management (paper section 4.5, VMM-based allocator): one large contiguous range of
// virtual addresses is reserved once and costs no memory; physical pages are mapped behind its start up to the
// planned peak of the current request, so the kernels see one contiguous buffer while the memory actually
// taken follows the plan.  Host code only: hipMemAddressReserve / hipMemCreate / hipMemMap / hipMemSetAccess.
//
// Growth maps one more allocation handle behind the pages already there (paper section 4.5: pages are mapped up to
// the planned peak as it rises), leaves the existing mapping alone and needs no wait; access is then set for the
// whole mapped prefix from the range's start.  On this driver hipMemSetAccess on a later sub-range has returned
// hipErrorInvalidValue in about one run out of four, so growth is an attempt: if the driver refuses to map or to
// open the new piece, the piece is taken back and the resize falls back to the plain path, which is also the path
// of a shrink and of a first mapping: wait for the device, drop every piece, map ONE handle of the new size at the
// range's start.  Contents survive the first path and not the second; mosaic_vmm_kept_contents() tells which one
// the last resize took (the workspace holds a step's transients, so nothing depends on it).
#include <new>
#include <vector>

#include "mosaic_internal.h"

struct mosaic_vmm {
  int device = 0;
  char* base = nullptr;
  size_t reserved = 0;
  size_t granularity = 0;
  size_t committed = 0;
  hipMemAllocationProp prop{};
  struct Piece {
    hipMemGenericAllocationHandle_t handle;
    size_t bytes;
  };
  std::vector<Piece> pieces;   // mapped back to back from `base`; their sizes add up to `committed`
  int kept_contents = 0;       // the last resize that changed the size only added a piece: 1 = access was set over
                               // the whole prefix, 2 = the driver refused that and accepted the new piece alone
  int last_hip_error = 0;      // hipError_t of the most recent failing driver call
  const char* last_call = "";  // and its name
};

namespace {

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr size_t kMaxPieces = 32;   // beyond this a growth takes the plain path, which leaves one piece

// Unmaps and releases every piece, last first.  Returns false if a driver call failed (the pieces not yet dropped
// stay recorded).
bool drop_mapping(mosaic_vmm* v) {
  while (!v->pieces.empty()) {
    const mosaic_vmm::Piece piece = v->pieces.back();
    hipError_t e = hipMemUnmap(v->base + (v->committed - piece.bytes), piece.bytes);
    if (e != hipSuccess) {
      v->last_hip_error = (int)e;
      v->last_call = "hipMemUnmap";
      return false;
    }
    v->pieces.pop_back();
    v->committed -= piece.bytes;
    e = hipMemRelease(piece.handle);
    if (e != hipSuccess) {
      v->last_hip_error = (int)e;
      v->last_call = "hipMemRelease";
      return false;
    }
  }
  return true;
}

hipMemAccessDesc read_write(const mosaic_vmm* v) {
  hipMemAccessDesc access{};
  access.location = v->prop.location;
  access.flags = hipMemAccessFlagsProtReadWrite;
  return access;
}

// Tries to map `more` further bytes behind the committed prefix.  1 or 2: done (which of the two access calls the
// driver accepted).  0: nothing changed (what was mapped before is still mapped and usable) and *out_of_memory says
// whether the driver had no memory to give.
int try_grow(mosaic_vmm* v, size_t more, bool* out_of_memory) {
  *out_of_memory = false;
  hipMemGenericAllocationHandle_t handle{};
  hipError_t e = hipMemCreate(&handle, more, &v->prop, 0);
  if (e != hipSuccess) {
    v->last_hip_error = (int)e;
    v->last_call = "hipMemCreate";
    *out_of_memory = true;
    (void)hipGetLastError();
    return 0;
  }
  e = hipMemMap(v->base + v->committed, more, 0, handle, 0);
  if (e == hipSuccess) {
    const hipMemAccessDesc access = read_write(v);
    int how = 1;
    e = hipMemSetAccess(v->base, v->committed + more, &access, 1);            // the whole prefix, from the start
    if (e != hipSuccess) {
      how = 2;
      e = hipMemSetAccess(v->base + v->committed, more, &access, 1);          // else the new piece alone
    }
    if (e == hipSuccess) {
      if (how == 2) (void)hipGetLastError();
      v->pieces.push_back({handle, more});
      v->committed += more;
      return how;
    }
    (void)hipMemUnmap(v->base + v->committed, more);
  }
  (void)hipMemRelease(handle);
  (void)hipGetLastError();   // the refusal is handled here: it must not surface in the caller's next launch check
  return 0;
}

}  // namespace

extern "C" {

int mosaic_vmm_create(int device, int64_t reserve_bytes, mosaic_vmm** out) {
  if (out == nullptr) return MOSAIC_ERR_INVALID_ARG;
  *out = nullptr;
  if (device < 0 || reserve_bytes <= 0) return MOSAIC_ERR_INVALID_ARG;
  int supported = 0;
  if (hipDeviceGetAttribute(&supported, hipDeviceAttributeVirtualMemoryManagementSupported, device) != hipSuccess)
    return MOSAIC_ERR_HIP;
  if (!supported) return MOSAIC_ERR_UNSUPPORTED_SHAPE;
  mosaic_vmm* v = new (std::nothrow) mosaic_vmm();
  if (v == nullptr) return MOSAIC_ERR_HIP;
  v->device = device;
  v->prop.type = hipMemAllocationTypePinned;
  v->prop.location.type = hipMemLocationTypeDevice;
  v->prop.location.id = device;
  if (hipMemGetAllocationGranularity(&v->granularity, &v->prop, hipMemAllocationGranularityRecommended) != hipSuccess ||
      v->granularity == 0) {
    delete v;
    return MOSAIC_ERR_HIP;
  }
  v->reserved = round_up((size_t)reserve_bytes, v->granularity);
  void* p = nullptr;
  if (hipMemAddressReserve(&p, v->reserved, v->granularity, nullptr, 0) != hipSuccess || p == nullptr) {
    delete v;
    return MOSAIC_ERR_HIP;
  }
  v->base = static_cast<char*>(p);
  *out = v;
  return MOSAIC_OK;
}

int mosaic_vmm_resize(mosaic_vmm* v, int64_t bytes) {
  if (v == nullptr || bytes < 0) return MOSAIC_ERR_INVALID_ARG;
  int current = -1;   // the synchronisation below acts on the current device: it must be the object's
  if (hipGetDevice(&current) != hipSuccess) return MOSAIC_ERR_HIP;
  if (current != v->device) return MOSAIC_ERR_INVALID_ARG;
  const size_t want = round_up((size_t)bytes, v->granularity);
  if (want > v->reserved) return MOSAIC_ERR_WORKSPACE_TOO_SMALL;
  if (want == v->committed) return MOSAIC_OK;
  if (want > v->committed && v->committed > 0 && v->pieces.size() < kMaxPieces) {
    bool out_of_memory = false;
    const int how = try_grow(v, want - v->committed, &out_of_memory);
    if (how != 0) {
      v->kept_contents = how;
      return MOSAIC_OK;
    }
    if (out_of_memory) return MOSAIC_ERR_HIP;   // the pages mapped so far stay
  }
  v->kept_contents = 0;
  if (v->committed > 0) {
    // Pages are about to leave the range: nothing may still be running on them.
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      v->last_hip_error = (int)e;
      v->last_call = "hipDeviceSynchronize";
      return MOSAIC_ERR_HIP;
    }
    if (!drop_mapping(v)) return MOSAIC_ERR_HIP;
  }
  if (want == 0) return MOSAIC_OK;
  hipMemGenericAllocationHandle_t handle{};
  hipError_t e = hipMemCreate(&handle, want, &v->prop, 0);   // fails when the device is out of memory
  if (e != hipSuccess) {
    v->last_hip_error = (int)e;
    v->last_call = "hipMemCreate";
    return MOSAIC_ERR_HIP;
  }
  e = hipMemMap(v->base, want, 0, handle, 0);
  if (e != hipSuccess) {
    v->last_hip_error = (int)e;
    v->last_call = "hipMemMap";
    (void)hipMemRelease(handle);
    return MOSAIC_ERR_HIP;
  }
  const hipMemAccessDesc access = read_write(v);
  e = hipMemSetAccess(v->base, want, &access, 1);
  if (e != hipSuccess) {
    v->last_hip_error = (int)e;
    v->last_call = "hipMemSetAccess";
    (void)hipMemUnmap(v->base, want);
    (void)hipMemRelease(handle);
    return MOSAIC_ERR_HIP;
  }
  v->pieces.push_back({handle, want});
  v->committed = want;
  return MOSAIC_OK;
}

void* mosaic_vmm_ptr(const mosaic_vmm* v) { return v == nullptr ? nullptr : v->base; }
int64_t mosaic_vmm_committed_bytes(const mosaic_vmm* v) { return v == nullptr ? 0 : (int64_t)v->committed; }
int64_t mosaic_vmm_reserved_bytes(const mosaic_vmm* v) { return v == nullptr ? 0 : (int64_t)v->reserved; }
int64_t mosaic_vmm_granularity(const mosaic_vmm* v) { return v == nullptr ? 0 : (int64_t)v->granularity; }
int mosaic_vmm_kept_contents(const mosaic_vmm* v) { return v == nullptr ? 0 : v->kept_contents; }
const char* mosaic_vmm_last_error(const mosaic_vmm* v, int* hip_error) {
  if (hip_error != nullptr) *hip_error = v == nullptr ? 0 : v->last_hip_error;
  return v == nullptr ? "" : v->last_call;
}

int mosaic_vmm_destroy(mosaic_vmm* v) {
  if (v == nullptr) return MOSAIC_OK;
  int rc = MOSAIC_OK;
  int current = -1;
  if (v->committed > 0 && (hipGetDevice(&current) != hipSuccess || current != v->device)) rc = MOSAIC_ERR_INVALID_ARG;
  if (rc == MOSAIC_OK && v->committed > 0 && hipDeviceSynchronize() != hipSuccess) rc = MOSAIC_ERR_HIP;
  if (rc == MOSAIC_OK && !drop_mapping(v)) rc = MOSAIC_ERR_HIP;
  if (rc == MOSAIC_OK && v->base != nullptr && hipMemAddressFree(v->base, v->reserved) != hipSuccess) rc = MOSAIC_ERR_HIP;
  delete v;   // on an error the mappings are abandoned to the process's end rather than touched again
  return rc;
}

}  // extern "C"
