// Workspace on virtual memory management (paper section 4.5, VMM-based allocator): one large contiguous range of
// virtual addresses is reserved once and costs no memory; physical pages are mapped behind its start up to the
// planned peak of the current request, so the kernels see one contiguous buffer while the memory actually
// taken follows the plan.  Host code only: hipMemAddressReserve / hipMemCreate / hipMemMap / hipMemSetAccess.
//
// Physical memory is ONE allocation handle mapped at the start of the range.  A resize that changes the size waits
// for the device, drops the old mapping and maps a new handle of the new size at the same address, so contents do
// not survive it (the workspace holds a step's transients, nothing that outlives a request).  Mapping further
// handles behind the first one was tried first: on this driver hipMemSetAccess on such a later sub-range returned
// hipErrorInvalidValue in about one run out of four, so every driver call here works on the range's start only.
#include <new>

#include "mosaic_internal.h"

struct mosaic_vmm {
  int device = 0;
  char* base = nullptr;
  size_t reserved = 0;
  size_t granularity = 0;
  size_t committed = 0;
  hipMemAllocationProp prop{};
  hipMemGenericAllocationHandle_t handle{};   // valid while committed > 0
  int last_hip_error = 0;      // hipError_t of the most recent failing driver call
  const char* last_call = "";  // and its name
};

namespace {

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Unmaps and releases the current mapping, if any.  Returns false if a driver call failed.
bool drop_mapping(mosaic_vmm* v) {
  if (v->committed == 0) return true;
  hipError_t e = hipMemUnmap(v->base, v->committed);
  if (e != hipSuccess) {
    v->last_hip_error = (int)e;
    v->last_call = "hipMemUnmap";
    return false;
  }
  e = hipMemRelease(v->handle);
  v->committed = 0;
  if (e != hipSuccess) {
    v->last_hip_error = (int)e;
    v->last_call = "hipMemRelease";
    return false;
  }
  return true;
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
  hipMemAccessDesc access{};
  access.location = v->prop.location;
  access.flags = hipMemAccessFlagsProtReadWrite;
  e = hipMemSetAccess(v->base, want, &access, 1);
  if (e != hipSuccess) {
    v->last_hip_error = (int)e;
    v->last_call = "hipMemSetAccess";
    (void)hipMemUnmap(v->base, want);
    (void)hipMemRelease(handle);
    return MOSAIC_ERR_HIP;
  }
  v->handle = handle;
  v->committed = want;
  return MOSAIC_OK;
}

void* mosaic_vmm_ptr(const mosaic_vmm* v) { return v == nullptr ? nullptr : v->base; }
int64_t mosaic_vmm_committed_bytes(const mosaic_vmm* v) { return v == nullptr ? 0 : (int64_t)v->committed; }
int64_t mosaic_vmm_reserved_bytes(const mosaic_vmm* v) { return v == nullptr ? 0 : (int64_t)v->reserved; }
int64_t mosaic_vmm_granularity(const mosaic_vmm* v) { return v == nullptr ? 0 : (int64_t)v->granularity; }
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
