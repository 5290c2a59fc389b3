// Independently allocated KV blocks (paper Sec. 5.1) on HIP's virtual memory
// management calls: one reserved address range, single blocks of it backed by
// physical memory on demand and returned to the device on release.  Host code
// only; the kernels see ordinary device addresses.
#include "internal.h"

#include <set>
#include <vector>

struct pipelive_vmm_pool {
  int device = 0;
  size_t block_bytes = 0;
  int64_t max_blocks = 0;
  char *base = nullptr;
  std::vector<hipMemGenericAllocationHandle_t> handle;  // per position; valid where used[i]
  std::vector<uint8_t> used;
  std::set<int64_t> free_pos;  // ascending: allocation takes the lowest positions
  int64_t allocated = 0;
  hipMemAllocationProp prop = {};
};

namespace {

constexpr size_t kBackingUnit = (size_t)2 << 20;

// undo a partial allocation: positions pos[0 .. mapped) are mapped, handles of pos[0 .. created) exist
void rollback(pipelive_vmm_pool *p, const std::vector<int64_t> &pos, size_t created, size_t mapped) {
  for (size_t i = 0; i < created; ++i) {
    if (i < mapped) (void)hipMemUnmap(p->base + (size_t)pos[i] * p->block_bytes, p->block_bytes);
    (void)hipMemRelease(p->handle[pos[i]]);
  }
}

}  // namespace

extern "C" {

size_t pipelive_vmm_backing_bytes(size_t block_bytes) {
  return (block_bytes + kBackingUnit - 1) / kBackingUnit * kBackingUnit;
}

int32_t pipelive_vmm_pool_create(size_t block_bytes, int64_t max_blocks, pipelive_vmm_pool_t **out) {
  if (!out || block_bytes == 0 || max_blocks <= 0 || max_blocks >= (1ll << 31)) return PIPELIVE_E_INVAL;
  *out = nullptr;
  int dev = 0, ok = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&ok, hipDeviceAttributeVirtualMemoryManagementSupported, dev));
  if (!ok) {
    pipelive::set_hip_error("device has no virtual memory management");
    return PIPELIVE_E_HIP;
  }
  pipelive_vmm_pool *p = new (std::nothrow) pipelive_vmm_pool;
  if (!p) return PIPELIVE_E_NOSPACE;
  p->device = dev;
  p->prop.type = hipMemAllocationTypePinned;
  p->prop.location.type = hipMemLocationTypeDevice;
  p->prop.location.id = dev;
  size_t gran = 0;
  hipError_t e = hipMemGetAllocationGranularity(&gran, &p->prop, hipMemAllocationGranularityMinimum);
  if (e != hipSuccess || gran == 0 || block_bytes % gran || block_bytes % 256) {
    delete p;
    if (e != hipSuccess) {
      pipelive::set_hip_error(hipGetErrorString(e));
      return PIPELIVE_E_HIP;
    }
    return PIPELIVE_E_INVAL;
  }
  void *va = nullptr;
  e = hipMemAddressReserve(&va, block_bytes * (size_t)max_blocks, 0, nullptr, 0);
  if (e != hipSuccess) {
    delete p;
    pipelive::set_hip_error(hipGetErrorString(e));
    return PIPELIVE_E_HIP;
  }
  p->base = (char *)va;
  p->block_bytes = block_bytes;
  p->max_blocks = max_blocks;
  p->handle.resize((size_t)max_blocks);
  p->used.assign((size_t)max_blocks, 0);
  for (int64_t i = 0; i < max_blocks; ++i) p->free_pos.insert(p->free_pos.end(), i);
  *out = p;
  return PIPELIVE_OK;
}

void pipelive_vmm_pool_destroy(pipelive_vmm_pool_t *p) {
  if (!p) return;
  for (int64_t i = 0; i < p->max_blocks; ++i)
    if (p->used[i]) {
      (void)hipMemUnmap(p->base + (size_t)i * p->block_bytes, p->block_bytes);
      (void)hipMemRelease(p->handle[i]);
    }
  (void)hipMemAddressFree(p->base, p->block_bytes * (size_t)p->max_blocks);
  delete p;
}

int32_t pipelive_vmm_pool_alloc(pipelive_vmm_pool_t *p, int64_t n, uint64_t *addrs) {
  if (!p || n < 0 || (n > 0 && !addrs)) return PIPELIVE_E_INVAL;
  if (n == 0) return PIPELIVE_OK;
  if ((int64_t)p->free_pos.size() < n) return PIPELIVE_E_NOSPACE;
  std::vector<int64_t> pos;
  pos.reserve((size_t)n);
  for (auto it = p->free_pos.begin(); (int64_t)pos.size() < n; ++it) pos.push_back(*it);
  size_t created = 0, mapped = 0;
  hipError_t e = hipSuccess;
  for (size_t i = 0; i < (size_t)n && e == hipSuccess; ++i) {
    e = hipMemCreate(&p->handle[pos[i]], p->block_bytes, &p->prop, 0);
    if (e != hipSuccess) break;
    ++created;
    e = hipMemMap(p->base + (size_t)pos[i] * p->block_bytes, p->block_bytes, 0, p->handle[pos[i]], 0);
    if (e == hipSuccess) ++mapped;
  }
  // enable access, one call per run of adjacent positions
  hipMemAccessDesc ad = {};
  ad.location = p->prop.location;
  ad.flags = hipMemAccessFlagsProtReadWrite;
  for (size_t i = 0; i < (size_t)n && e == hipSuccess;) {
    size_t j = i + 1;
    while (j < (size_t)n && pos[j] == pos[j - 1] + 1) ++j;
    e = hipMemSetAccess(p->base + (size_t)pos[i] * p->block_bytes, (j - i) * p->block_bytes, &ad, 1);
    i = j;
  }
  if (e != hipSuccess) {
    pipelive::set_hip_error(hipGetErrorString(e));
    rollback(p, pos, created, mapped);
    (void)hipGetLastError();
    return PIPELIVE_E_HIP;
  }
  for (size_t i = 0; i < (size_t)n; ++i) {
    p->used[pos[i]] = 1;
    p->free_pos.erase(pos[i]);
    addrs[i] = (uint64_t)(p->base + (size_t)pos[i] * p->block_bytes);
  }
  p->allocated += n;
  return PIPELIVE_OK;
}

int32_t pipelive_vmm_pool_free(pipelive_vmm_pool_t *p, int64_t n, const uint64_t *addrs) {
  if (!p || n < 0 || (n > 0 && !addrs)) return PIPELIVE_E_INVAL;
  std::vector<int64_t> pos((size_t)n);
  {
    std::set<int64_t> seen;
    for (int64_t i = 0; i < n; ++i) {
      const uint64_t a = addrs[i], b = (uint64_t)p->base;
      if (a < b || (a - b) % p->block_bytes) return PIPELIVE_E_INVAL;
      const uint64_t k = (a - b) / p->block_bytes;
      if (k >= (uint64_t)p->max_blocks || !p->used[k] || !seen.insert((int64_t)k).second)
        return PIPELIVE_E_INVAL;
      pos[i] = (int64_t)k;
    }
  }
  int32_t rc = PIPELIVE_OK;
  for (int64_t i = 0; i < n; ++i) {
    hipError_t e = hipMemUnmap(p->base + (size_t)pos[i] * p->block_bytes, p->block_bytes);
    if (e == hipSuccess) e = hipMemRelease(p->handle[pos[i]]);
    if (e != hipSuccess) {  // keep going: the position stays unusable rather than half released
      pipelive::set_hip_error(hipGetErrorString(e));
      rc = PIPELIVE_E_HIP;
      p->used[pos[i]] = 0;
      --p->allocated;
      continue;
    }
    p->used[pos[i]] = 0;
    p->free_pos.insert(pos[i]);
    --p->allocated;
  }
  return rc;
}

int64_t pipelive_vmm_pool_allocated(const pipelive_vmm_pool_t *p) { return p ? p->allocated : -1; }
uint64_t pipelive_vmm_pool_base(const pipelive_vmm_pool_t *p) { return p ? (uint64_t)p->base : 0; }

}  // extern "C"
