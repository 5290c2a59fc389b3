// Region-aware device arena (placement for MI355X; see the header).  One
// virtually contiguous range of large physical pieces.  A timing probe at
// creation finds out which pieces share a region of the device memory (a copy
// that runs inside two pieces at once is slow when both lie in the same
// region).  The range is then laid out in zones: a spread zone whose pieces
// alternate between the regions, and one zone per region.  Host code and one
// probe kernel; everything carved out of the range is an ordinary device
// address to the other kernels.
#include "internal.h"

#include <algorithm>
#include <vector>

struct pipelive_arena {
  char *base = nullptr;
  size_t bytes = 0, piece_bytes = 0;
  size_t probe_bytes = 0;  // size of the unit the probe times: a whole number of pieces
  int32_t device = 0;
  std::vector<hipMemGenericAllocationHandle_t> handle;  // physical pieces in the order they were created
  std::vector<uint8_t> created;
  std::vector<int32_t> cls;    // class of each physical piece
  std::vector<int32_t> order;  // virtual piece j is physical piece order[j]
  bool mapped = false;
  pipelive_arena_info_t info = {};
  uint64_t zone_off[PIPELIVE_ARENA_MAX_CLASSES + 1] = {};    // zone 0: spread; zone 1 + c: class c
  uint64_t zone_bytes[PIPELIVE_ARENA_MAX_CLASSES + 1] = {};
};

namespace {

constexpr size_t kBackingUnit = (size_t)2 << 20;
constexpr size_t kChunk = 32768;  // bytes one workgroup moves per pass
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Copies the lower half of stretch a into its upper half and the same inside stretch b, both at once (chunks of
// 32 KiB, nontemporal like the library's copy kernels), `passes` times over, so that a launch on short stretches
// still runs long enough to time.
__global__ __launch_bounds__(256) void arena_probe_kernel(char *a, char *b, int32_t chunks_per_piece, size_t half,
                                                          int32_t passes) {
  const int32_t n = 2 * chunks_per_piece;
  for (int32_t it = blockIdx.x; it < n * passes; it += gridDim.x) {
    const int32_t c = it % n;
    char *base = c < chunks_per_piece ? a : b;
    const size_t off = (size_t)(c < chunks_per_piece ? c : c - chunks_per_piece) * kChunk;
    const u32x4 *s = (const u32x4 *)(base + off);
    u32x4 *d = (u32x4 *)(base + half + off);
    u32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = __builtin_nontemporal_load(s + threadIdx.x + 256 * i);
#pragma unroll
    for (int i = 0; i < 8; ++i) __builtin_nontemporal_store(v[i], d + threadIdx.x + 256 * i);
  }
}

hipError_t map_in_order(pipelive_arena *r, const std::vector<int32_t> &order) {
  hipMemAccessDesc ad = {};
  ad.location.type = hipMemLocationTypeDevice;
  ad.location.id = r->device;
  ad.flags = hipMemAccessFlagsProtReadWrite;
  const size_t np = r->handle.size();
  for (size_t j = 0; j < np; ++j) {
    hipError_t e = hipMemMap(r->base + j * r->piece_bytes, r->piece_bytes, 0, r->handle[order[j]], 0);
    if (e != hipSuccess) {
      for (size_t k = 0; k < j; ++k) (void)hipMemUnmap(r->base + k * r->piece_bytes, r->piece_bytes);
      return e;
    }
  }
  hipError_t e = hipMemSetAccess(r->base, r->bytes, &ad, 1);
  if (e != hipSuccess) {
    (void)hipMemUnmap(r->base, r->bytes);
    return e;
  }
  r->mapped = true;
  r->order = order;
  return hipSuccess;
}

// rate of the pair copy in bytes per second (read + written, both units); one launch to warm, one timed.
// Units are consecutive stretches of probe_bytes of the range as first mapped (pieces in creation order).
hipError_t pair_rate(pipelive_arena *r, hipEvent_t e0, hipEvent_t e1, size_t a, size_t b, double *rate) {
  const size_t half = r->probe_bytes / 2;
  const int32_t chunks = (int32_t)(half / kChunk);
  const int32_t passes = (int32_t)std::max<size_t>(1, ((size_t)1 << 29) / r->probe_bytes);  // at least 512 MiB moved per stretch
  float best = 0.f;
  for (int rep = 0; rep < 2; ++rep) {
    hipError_t e = hipEventRecord(e0, nullptr);
    if (e != hipSuccess) return e;
    arena_probe_kernel<<<dim3(4096), dim3(256), 0, nullptr>>>(r->base + a * r->probe_bytes, r->base + b * r->probe_bytes,
                                                            chunks, half, passes);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = hipEventRecord(e1, nullptr)) != hipSuccess) return e;
    if ((e = hipEventSynchronize(e1)) != hipSuccess) return e;
    float ms = 0.f;
    if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) return e;
    if (rep > 0 && (best == 0.f || ms < best)) best = ms;
  }
  *rate = 4.0 * (double)half * passes / ((double)best * 1e-3);
  return hipSuccess;
}

// Classes by reference units.  The first reference is unit 0 (or, if nothing contrasts beside it, one of a few
// others); the unit that copies fastest beside it is the second; a unit that is clearly fast beside every reference so far (in the upper quarter of the span between the
// slowest and the fastest rate seen beside the first: a unit that straddles two regions is not) becomes the next one,
// up to PIPELIVE_ARENA_MAX_CLASSES.  Every unit then joins the reference beside which its pair copy is slowest.
// Without contrast (spread under 6 %) beside any of the tried first references there is one class.
hipError_t classify(pipelive_arena *r) {
  const size_t ppu = r->probe_bytes / r->piece_bytes;  // pieces per unit
  const size_t nu = r->handle.size() / ppu;            // whole units; pieces behind them take the last unit's class
  hipEvent_t e0 = nullptr, e1 = nullptr, t0 = nullptr, t1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) e = hipEventCreate(&t0);
  if (e == hipSuccess) e = hipEventCreate(&t1);
  if (e == hipSuccess) e = hipEventRecord(t0, nullptr);
  std::vector<size_t> ref;
  std::vector<std::vector<double>> rate;  // rate[k][i]: unit i beside reference k (0 for the reference itself)
  auto add_ref = [&](size_t u) {
    ref.push_back(u);
    rate.emplace_back(nu, 0.0);
    for (size_t i = 0; i < nu && e == hipSuccess; ++i)
      if (i != u) e = pair_rate(r, e0, e1, u, i, &rate.back()[i]);
  };
  // The first reference has to lie inside one region: a unit that straddles two shows no contrast.  Unit 0 is
  // tried first, then a few others; if none shows contrast there is one class.
  double thr = 0;
  const size_t candidates[5] = {0, nu / 2, nu - 1, nu / 4, (3 * nu) / 4};
  bool contrast = false;
  size_t fastest = 0;
  for (int c = 0; c < 5 && e == hipSuccess && !contrast; ++c) {
    const size_t u = candidates[c];
    bool tried = false;
    for (int k = 0; k < c; ++k) tried |= candidates[k] == u;
    if (tried) continue;
    ref.clear();
    rate.clear();
    add_ref(u);
    if (e != hipSuccess) break;
    double lo = 0, hi = 0;
    bool any = false;
    for (size_t i = 0; i < nu; ++i) {
      if (i == u) continue;
      if (!any || rate[0][i] < lo) lo = rate[0][i];
      if (!any || rate[0][i] > hi) hi = rate[0][i], fastest = i;
      any = true;
    }
    thr = lo + 0.75 * (hi - lo);
    contrast = hi - lo >= 0.06 * hi;
  }
  if (e == hipSuccess && contrast) {
    add_ref(fastest);
    while (e == hipSuccess && (int32_t)ref.size() < PIPELIVE_ARENA_MAX_CLASSES) {
      size_t best = 0;
      double best_min = 0;
      for (size_t i = 0; i < nu; ++i) {
        double m = rate[0][i];
        for (size_t k = 1; k < ref.size(); ++k) m = std::min(m, rate[k][i]);
        if (m > best_min) best_min = m, best = i;  // a reference has rate 0 beside itself and is never picked
      }
      if (best_min <= thr) break;
      add_ref(best);
    }
  }
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventRecord(t1, nullptr);
  if (e == hipSuccess) e = hipEventSynchronize(t1);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
  for (hipEvent_t ev : {e0, e1, t0, t1})
    if (ev) (void)hipEventDestroy(ev);
  if (e != hipSuccess) return e;
  const size_t nk = ref.size();
  std::vector<int32_t> ucls(nu, 0);
  double same_sum = 0, other_sum = 0;
  size_t same_n = 0, other_n = 0;
  for (size_t i = 0; i < nu; ++i) {
    size_t k_min = 0;
    for (size_t k = 1; k < nk; ++k)
      if (rate[k][i] < rate[k_min][i]) k_min = k;
    ucls[i] = (int32_t)k_min;
    for (size_t k = 0; k < nk; ++k) {
      if (i == ref[k]) continue;
      if (k == k_min) same_sum += rate[k][i], ++same_n;
      else other_sum += rate[k][i], ++other_n;
    }
  }
  r->cls.assign(r->handle.size(), 0);
  for (size_t i = 0; i < r->handle.size(); ++i) r->cls[i] = ucls[std::min(i / ppu, nu - 1)];
  r->info.n_classes = (int32_t)nk;
  r->info.probe_ms = ms;
  r->info.rate_same_GBps = same_n ? (float)(same_sum / same_n / 1e9) : 0.f;
  r->info.rate_other_GBps = other_n ? (float)(other_sum / other_n / 1e9) : 0.f;
  return hipSuccess;
}

void release_all(pipelive_arena *r) {
  if (r->mapped) (void)hipMemUnmap(r->base, r->bytes);
  for (size_t i = 0; i < r->handle.size(); ++i)
    if (r->created[i]) (void)hipMemRelease(r->handle[i]);
  if (r->base) (void)hipMemAddressFree(r->base, r->bytes);
  delete r;
}

}  // namespace

extern "C" {

int32_t pipelive_arena_create(size_t bytes, size_t piece_bytes, size_t probe_bytes, pipelive_arena_t **out) {
  if (!out || bytes == 0 || piece_bytes == 0 || piece_bytes % kBackingUnit || probe_bytes % piece_bytes)
    return PIPELIVE_E_INVAL;
  *out = nullptr;
  const size_t np = (bytes + piece_bytes - 1) / piece_bytes;
  if (np >= ((size_t)1 << 20)) return PIPELIVE_E_INVAL;
  int dev = 0, ok = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&ok, hipDeviceAttributeVirtualMemoryManagementSupported, dev));
  if (!ok) {
    pipelive::set_hip_error("device has no virtual memory management");
    return PIPELIVE_E_HIP;
  }
  pipelive_arena *r = new (std::nothrow) pipelive_arena;
  if (!r) return PIPELIVE_E_NOSPACE;
  r->bytes = np * piece_bytes;
  r->piece_bytes = piece_bytes;
  r->probe_bytes = probe_bytes;
  r->device = dev;
  r->handle.resize(np);
  r->created.assign(np, 0);
  r->info.n_pieces = (int32_t)np;
  auto fail = [&](hipError_t e) {
    const bool oom = e == hipErrorOutOfMemory;
    pipelive::set_hip_error(hipGetErrorString(e));
    release_all(r);
    (void)hipGetLastError();
    return oom ? PIPELIVE_E_NOSPACE : PIPELIVE_E_HIP;
  };
  void *va = nullptr;
  hipError_t e = hipMemAddressReserve(&va, r->bytes, 0, nullptr, 0);
  if (e != hipSuccess) return fail(e);
  r->base = (char *)va;
  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = dev;
  for (size_t i = 0; i < np; ++i) {
    e = hipMemCreate(&r->handle[i], piece_bytes, &prop, 0);
    if (e != hipSuccess) return fail(e);
    r->created[i] = 1;
  }
  std::vector<int32_t> order(np);
  for (size_t i = 0; i < np; ++i) order[i] = (int32_t)i;
  e = map_in_order(r, order);
  if (e != hipSuccess) return fail(e);
  r->cls.assign(np, 0);
  r->info.n_classes = 1;
  if (probe_bytes && np >= 2 * (probe_bytes / piece_bytes)) {
    e = classify(r);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail(e);
  }
  for (int32_t c = 0; c < PIPELIVE_ARENA_MAX_CLASSES; ++c) r->info.class_pieces[c] = 0;
  for (size_t i = 0; i < np; ++i) r->info.class_pieces[r->cls[i]]++;
  r->info.n_runs = 1;
  for (size_t i = 1; i < np; ++i) r->info.n_runs += r->cls[i] != r->cls[i - 1];
  const int32_t rc = pipelive_arena_layout(r, r->bytes);  // everything in the spread zone to begin with
  if (rc != PIPELIVE_OK) {
    release_all(r);
    return rc;
  }
  *out = r;
  return PIPELIVE_OK;
}

int32_t pipelive_arena_layout(pipelive_arena_t *r, size_t spread_bytes) {
  if (!r) return PIPELIVE_E_INVAL;
  const size_t np = r->handle.size();
  const int32_t nc = r->info.n_classes;
  size_t n_spread = (spread_bytes + r->piece_bytes - 1) / r->piece_bytes;
  if (n_spread > np) n_spread = np;
  std::vector<std::vector<int32_t>> by((size_t)nc);
  for (size_t i = 0; i < np; ++i) by[(size_t)r->cls[i]].push_back((int32_t)i);
  std::vector<size_t> taken((size_t)nc, 0);
  std::vector<int32_t> order(np);
  // spread zone: the classes in turn, each in proportion to its size, so that every stretch of the zone holds
  // the same mix
  for (size_t j = 0; j < n_spread; ++j) {
    int32_t pick = -1;
    double most = -1.0;
    for (int32_t c = 0; c < nc; ++c) {
      const size_t n = by[(size_t)c].size();
      if (taken[(size_t)c] >= n) continue;
      const double left = (double)(n - taken[(size_t)c]) / (double)n;  // share of the class not yet placed
      if (left > most + 1e-12) most = left, pick = c;
    }
    order[j] = by[(size_t)pick][taken[(size_t)pick]++];
  }
  // class zones: what is left of each class, in the order the driver handed the pieces out
  size_t j = n_spread;
  r->zone_off[0] = 0;
  r->zone_bytes[0] = (uint64_t)n_spread * r->piece_bytes;
  for (int32_t c = 0; c < PIPELIVE_ARENA_MAX_CLASSES; ++c) {
    r->zone_off[1 + c] = (uint64_t)j * r->piece_bytes;
    if (c < nc)
      while (taken[(size_t)c] < by[(size_t)c].size()) order[j++] = by[(size_t)c][taken[(size_t)c]++];
    r->zone_bytes[1 + c] = (uint64_t)j * r->piece_bytes - r->zone_off[1 + c];
  }
  if (r->mapped && order == r->order) return PIPELIVE_OK;
  HIP_TRY(hipDeviceSynchronize());
  if (r->mapped) {
    HIP_TRY(hipMemUnmap(r->base, r->bytes));
    r->mapped = false;
  }
  hipError_t e = map_in_order(r, order);
  if (e != hipSuccess) {  // the range is unmapped now: the arena can only be destroyed
    pipelive::set_hip_error(hipGetErrorString(e));
    return PIPELIVE_E_HIP;
  }
  return PIPELIVE_OK;
}

int32_t pipelive_arena_zone(const pipelive_arena_t *r, int32_t zone, uint64_t *offset, uint64_t *bytes) {
  if (!r || !offset || !bytes || zone < 0 || zone > r->info.n_classes) return PIPELIVE_E_INVAL;
  *offset = r->zone_off[zone];
  *bytes = r->zone_bytes[zone];
  return PIPELIVE_OK;
}

void pipelive_arena_destroy(pipelive_arena_t *r) {
  if (r) release_all(r);
}

uint64_t pipelive_arena_base(const pipelive_arena_t *r) { return r ? (uint64_t)r->base : 0; }
size_t pipelive_arena_bytes(const pipelive_arena_t *r) { return r ? r->bytes : 0; }

int32_t pipelive_arena_info(const pipelive_arena_t *r, pipelive_arena_info_t *out) {
  if (!r || !out) return PIPELIVE_E_INVAL;
  *out = r->info;
  return PIPELIVE_OK;
}

int32_t pipelive_arena_piece_class(const pipelive_arena_t *r, int64_t piece) {
  if (!r || piece < 0 || piece >= (int64_t)r->order.size()) return PIPELIVE_E_INVAL;
  return r->cls[(size_t)r->order[(size_t)piece]];
}

}  // extern "C"
