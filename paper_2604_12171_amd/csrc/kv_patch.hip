// Incremental KV patching (paper Sec. 6.1 "KV Migration with KV Patch"):
// dirty bitmap, atomic drain, gather of the dirty blocks into a contiguous
// patch, scatter-apply on the target, and the n_acc / T_applied counters.
//
// mark    : atomicOr of one bit per written block; n_acc += n_tokens.
// drain   : one workgroup swaps every bitmap word with zero (atomicExch, so a
//           concurrent mark is either in this snapshot or stays for the next
//           drain), prefix-sums the popcounts, writes the ascending id list
//           and the header, and ORs back the bits beyond the patch capacity.
// gather  : persistent workgroups copy (block, layer) chunks into the payload;
//           the number of blocks is read from the header on the device, so
//           the host never waits for it.
// scatter : the same loop in the other direction, with optional id remapping.
#include "internal.h"
#include "kv_copy.h"
#include "scan.h"

namespace pipelive {
namespace {

typedef unsigned long long u64;

__global__ void mark_kernel(u64 *dirty, int64_t B, const int32_t *ids, int32_t n, u64 n_tokens,
                            DevState *st) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0 && n_tokens) atomicAdd(&st->n_acc, n_tokens);
  if (i < n) {
    const int32_t id = ids[i];
    if (id < 0 || id >= B) {
      atomicCAS(&st->status, 0, PIPELIVE_E_RANGE);
    } else {
      atomicOr(&dirty[id >> 6], 1ull << (id & 63));
    }
  }
}

__global__ __launch_bounds__(kScanThreads) void drain_kernel(u64 *dirty, int64_t B, u64 *snap,
                                                             DevState *st, uint8_t *patch,
                                                             uint32_t max_blocks, uint32_t n_layers,
                                                             u64 block_bytes, u64 payload_offset) {
  __shared__ uint32_t sh[17];
  const int64_t nwords = (B + 63) / 64;
  const int64_t per = (nwords + kScanThreads - 1) / kScanThreads;
  const int64_t w0 = (int64_t)threadIdx.x * per;
  const int64_t w1 = w0 + per < nwords ? w0 + per : nwords;
  uint32_t cnt = 0;
  for (int64_t w = w0; w < w1; ++w) {
    u64 v = dirty[w];
    if (v) v = atomicExch(&dirty[w], 0ull);
    snap[w] = v;
    cnt += __popcll(v);
  }
  uint32_t total;
  uint32_t rank = wg_exclusive_scan(cnt, sh, &total);
  const uint32_t n_take = total < max_blocks ? total : max_blocks;
  int32_t *ids = (int32_t *)(patch + 64);
  for (int64_t w = w0; w < w1; ++w) {
    u64 v = snap[w];
    u64 back = 0;
    while (v) {
      const int b = __ffsll((long long)v) - 1;
      if (rank < n_take) ids[rank] = (int32_t)(w * 64 + b);
      else back |= 1ull << b;
      ++rank;
      v &= v - 1;
    }
    if (back) atomicOr(&dirty[w], back);
  }
  if (threadIdx.x == 0) {
    pipelive_patch_hdr_t h;
    h.magic = PIPELIVE_PATCH_MAGIC;
    h.version = PIPELIVE_PATCH_VERSION;
    h.n_blocks = n_take;
    h.n_layers = n_layers;
    h.block_bytes = block_bytes;
    h.more_pending = total > max_blocks ? 1u : 0u;
    h.n_acc_tokens = h.more_pending ? 0ull : atomicExch(&st->n_acc, 0ull);
    h.payload_offset = payload_offset;
    h.max_blocks = max_blocks;
    for (int i = 0; i < 16; ++i) h.pad[i] = 0;
    *(pipelive_patch_hdr_t *)patch = h;
  }
}

struct XferArgs {
  const uint64_t *block_list;
  int64_t capacity, num_blocks;
  uint32_t stack_k, blk_bytes, sub_bytes, subs_per_block;
  LayerList layers;
  const int32_t *dst_map;
  DevState *st;
};

// payload[(r * n_layers + i) * blk] <- block ids[r] of layer layers[i]
__global__ __launch_bounds__(kCopyThreads) void gather_kernel(XferArgs a, uint8_t *patch) {
  const pipelive_patch_hdr_t *h = (const pipelive_patch_hdr_t *)patch;
  const uint32_t n_blocks = h->n_blocks;
  const int32_t *ids = (const int32_t *)(patch + 64);
  char *payload = (char *)patch + h->payload_offset;
  const uint32_t nl = a.layers.n;
  const int64_t n_items = (int64_t)n_blocks * nl * a.subs_per_block;
  for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const uint32_t sub = (uint32_t)(item % a.subs_per_block);
    const int64_t e = item / a.subs_per_block;
    const uint32_t i = (uint32_t)(e % nl);
    const int64_t r = e / nl;
    const int32_t layer = a.layers.layer[i];
    const int32_t id = ids[r];
    const char *src = (const char *)a.block_list[(int64_t)(layer / a.stack_k) * a.capacity + id] +
                      (uint64_t)(layer % a.stack_k) * a.blk_bytes;
    const uint32_t off = sub * a.sub_bytes;
    const uint32_t len = a.blk_bytes - off < a.sub_bytes ? a.blk_bytes - off : a.sub_bytes;
    wg_copy(payload + (uint64_t)e * a.blk_bytes + off, src + off, len);
  }
}

// block dst_map[ids[r]] of layer layers[i] <- payload[(r * n_layers + i) * blk]
__global__ __launch_bounds__(kCopyThreads) void scatter_kernel(XferArgs a, const uint8_t *patch) {
  const pipelive_patch_hdr_t *h = (const pipelive_patch_hdr_t *)patch;
  const uint32_t nl = a.layers.n;
  if (h->magic != PIPELIVE_PATCH_MAGIC || h->version != PIPELIVE_PATCH_VERSION ||
      h->n_layers != nl || h->block_bytes != a.blk_bytes) {
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicCAS(&a.st->status, 0, PIPELIVE_E_INVAL);
    return;
  }
  const uint32_t n_blocks = h->n_blocks;
  const int32_t *ids = (const int32_t *)(patch + 64);
  const char *payload = (const char *)patch + h->payload_offset;
  if (blockIdx.x == 0 && threadIdx.x == 0 && h->n_acc_tokens)
    atomicAdd(&a.st->t_applied, (u64)h->n_acc_tokens);
  const int64_t n_items = (int64_t)n_blocks * nl * a.subs_per_block;
  for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const uint32_t sub = (uint32_t)(item % a.subs_per_block);
    const int64_t e = item / a.subs_per_block;
    const uint32_t i = (uint32_t)(e % nl);
    const int64_t r = e / nl;
    const int32_t layer = a.layers.layer[i];
    int64_t id = ids[r];
    if (a.dst_map) id = a.dst_map[id];
    if (id < 0 || id >= a.num_blocks) {  // uniform over the workgroup
      if (threadIdx.x == 0) atomicCAS(&a.st->status, 0, PIPELIVE_E_RANGE);
      continue;
    }
    char *dst = (char *)a.block_list[(int64_t)(layer / a.stack_k) * a.capacity + id] +
                (uint64_t)(layer % a.stack_k) * a.blk_bytes;
    const uint32_t off = sub * a.sub_bytes;
    const uint32_t len = a.blk_bytes - off < a.sub_bytes ? a.blk_bytes - off : a.sub_bytes;
    wg_copy(dst + off, payload + (uint64_t)e * a.blk_bytes + off, len);
  }
}

__global__ void clear_status_kernel(DevState *st) { st->status = 0; }

XferArgs make_xfer(const pipelive_kv *kv, const LayerList &layers, const int32_t *dst_map) {
  XferArgs a;
  a.block_list = kv->d.block_list;
  a.capacity = kv->d.capacity_blocks;
  a.num_blocks = kv->d.num_blocks;
  a.stack_k = (uint32_t)kv->d.stack_k;
  a.blk_bytes = (uint32_t)kv->blk_bytes;
  a.sub_bytes = kCopyChunk;
  a.subs_per_block = (a.blk_bytes + a.sub_bytes - 1) / a.sub_bytes;
  a.layers = layers;
  a.dst_map = dst_map;
  a.st = dev_state(kv);
  return a;
}

}  // namespace

hipError_t launch_mark(const pipelive_kv *kv, const int32_t *ids, int32_t n, int64_t n_tokens,
                       hipStream_t st) {
  const int threads = 256;
  const int grid = n > 0 ? (n + threads - 1) / threads : 1;
  hipLaunchKernelGGL(mark_kernel, dim3(grid), dim3(threads), 0, st, (u64 *)kv->d.dirty_bitmap,
                     kv->d.num_blocks, ids, n, (u64)n_tokens, dev_state(kv));
  return hipGetLastError();
}

hipError_t launch_collect(const pipelive_kv *kv, const LayerList &layers, uint8_t *patch,
                          uint32_t max_blocks, uint64_t payload_offset, hipStream_t st) {
  hipLaunchKernelGGL(drain_kernel, dim3(1), dim3(kScanThreads), 0, st, (u64 *)kv->d.dirty_bitmap,
                     kv->d.num_blocks, snap_words(kv), dev_state(kv), patch, max_blocks,
                     (uint32_t)layers.n, (u64)kv->blk_bytes, (u64)payload_offset);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  XferArgs a = make_xfer(kv, layers, nullptr);
  const int64_t max_items = (int64_t)max_blocks * layers.n * a.subs_per_block;
  const int64_t max_grid = (int64_t)device_cu_count() * copy_wgs_per_cu();
  const int grid = (int)(max_items < max_grid ? max_items : max_grid);
  hipLaunchKernelGGL(gather_kernel, dim3(grid), dim3(kCopyThreads), 0, st, a, patch);
  return hipGetLastError();
}

hipError_t launch_apply(const pipelive_kv *kv, const LayerList &layers, const uint8_t *patch,
                        const int32_t *dst_map, hipStream_t st) {
  XferArgs a = make_xfer(kv, layers, dst_map);
  const int grid = device_cu_count() * copy_wgs_per_cu();
  hipLaunchKernelGGL(scatter_kernel, dim3(grid), dim3(kCopyThreads), 0, st, a, patch);
  return hipGetLastError();
}

hipError_t launch_clear_status(const pipelive_kv *kv, hipStream_t st) {
  hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, dev_state(kv));
  return hipGetLastError();
}

}  // namespace pipelive
