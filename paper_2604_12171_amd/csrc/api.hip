// Host side of the C ABI: argument validation, launch heuristics, and the one
// wait (on the plan, not on the commit) that ResizeKV needs to return its verdict.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>

#include "internal.h"

using namespace pipelive;

namespace {

thread_local char g_hip_err[256] = "";

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int g_cu_count = 0;

// Scratch memory built into the library for pipelive_paged_attn_decode_noalloc: the partial records
// of a decode launch.  Every device the library runs on holds its own copy of the array at its own
// address; host code never uses the array's name for that memory, only the address looked up below.
constexpr size_t kNoallocScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
__device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (looked up once per device)
int32_t noalloc_scratch(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return pipelive::hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return PIPELIVE_E_INVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return pipelive::hip_fail(e);
    if (!ptr) return PIPELIVE_E_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return PIPELIVE_OK;
}

}  // namespace

namespace pipelive {
void set_hip_error(const char *text) { snprintf(g_hip_err, sizeof g_hip_err, "%s", text); }
int32_t hip_fail(hipError_t e) {
  set_hip_error(hipGetErrorString(e));
  return PIPELIVE_E_HIP;
}
int device_cu_count() {
  if (g_cu_count == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      g_cu_count = n;
    else
      g_cu_count = 256;
  }
  return g_cu_count;
}
// persistent copy kernels: 16 workgroups per CU, the setting the launch-shape sweeps of the copies settled on
int copy_wgs_per_cu() { return 16; }
}  // namespace pipelive

extern "C" {

size_t pipelive_bitmap_bytes(int64_t n_bits) {
  return n_bits <= 0 ? 8 : (size_t)((n_bits + 63) / 64 * 8);
}

int64_t pipelive_kv_dirty_units(int64_t capacity_blocks, int32_t block_tokens, int32_t granularity) {
  return granularity == PIPELIVE_DIRTY_SLOT ? capacity_blocks * block_tokens : capacity_blocks;
}

size_t pipelive_kv_state_bytes(int64_t dirty_units) {
  // counters | drain snapshot words | per-workgroup counts of the multi-kernel drain
  const size_t words = pipelive_bitmap_bytes(dirty_units) / 8;
  return kSnapOffset + round_up(words * 8 + (words / 256 + 2) * 4, 256);
}

int32_t pipelive_kv_create(const pipelive_kv_desc_t *d, pipelive_kv_t **out) {
  if (!d || !out) return PIPELIVE_E_INVAL;
  *out = nullptr;
  if (d->num_layers <= 0 || d->num_kv_heads <= 0 || d->num_q_heads <= 0) return PIPELIVE_E_INVAL;
  if (d->num_q_heads % d->num_kv_heads) return PIPELIVE_E_INVAL;
  if (d->num_q_heads / d->num_kv_heads > 16) return PIPELIVE_E_INVAL;
  if (d->head_dim != 64 && d->head_dim != 128) return PIPELIVE_E_INVAL;
  if (d->block_tokens != 16 && d->block_tokens != 32 && d->block_tokens != 64 && d->block_tokens != 128)
    return PIPELIVE_E_INVAL;
  if (d->block_backing != PIPELIVE_BACKING_ARENA && d->block_backing != PIPELIVE_BACKING_PER_BLOCK)
    return PIPELIVE_E_INVAL;
  if (d->stack_k < 1 || d->dtype != PIPELIVE_DTYPE_BF16) return PIPELIVE_E_INVAL;
  if (d->in_block_layout != PIPELIVE_LAYOUT_D8) return PIPELIVE_E_INVAL;
  if (d->dirty_granularity != PIPELIVE_DIRTY_BLOCK && d->dirty_granularity != PIPELIVE_DIRTY_SLOT)
    return PIPELIVE_E_INVAL;
  if (pipelive_kv_dirty_units(d->capacity_blocks, d->block_tokens, d->dirty_granularity) >= (1ll << 31))
    return PIPELIVE_E_INVAL;
  if (d->num_blocks < 0 || d->capacity_blocks < d->num_blocks) return PIPELIVE_E_INVAL;
  if (d->capacity_blocks >= (1ll << 31)) return PIPELIVE_E_INVAL;
  if (!d->block_list || !d->live_bitmap || !d->dirty_bitmap || !d->dev_state)
    return PIPELIVE_E_INVAL;
  if (!aligned(d->live_bitmap, 8) || !aligned(d->dirty_bitmap, 8) || !aligned(d->dev_state, 256) ||
      !aligned(d->block_list, 8))
    return PIPELIVE_E_INVAL;
  pipelive_kv *kv = new (std::nothrow) pipelive_kv;
  if (!kv) return PIPELIVE_E_NOSPACE;
  kv->d = *d;
  kv->groups = (d->num_layers + d->stack_k - 1) / d->stack_k;
  kv->blk_bytes = (uint64_t)2 * d->num_kv_heads * d->block_tokens * d->head_dim * 2;
  kv->phys_bytes = kv->blk_bytes * (uint64_t)d->stack_k;
  kv->units_per_block = d->dirty_granularity == PIPELIVE_DIRTY_SLOT ? d->block_tokens : 1;
  kv->unit_bytes = d->dirty_granularity == PIPELIVE_DIRTY_SLOT
                       ? (uint64_t)2 * d->num_kv_heads * d->head_dim * 2
                       : kv->blk_bytes;
  kv->pinned = nullptr;
  hipError_t e = hipHostMalloc((void **)&kv->pinned, sizeof(HostPinned), hipHostMallocDefault);
  if (e != hipSuccess) {
    delete kv;
    return hip_fail(e);
  }
  memset(kv->pinned, 0, sizeof(HostPinned));
  e = hipEventCreateWithFlags(&kv->plan_ready, hipEventDisableTiming);
  if (e != hipSuccess) {
    (void)hipHostFree(kv->pinned);
    delete kv;
    return hip_fail(e);
  }
  *out = kv;
  return PIPELIVE_OK;
}

void pipelive_kv_destroy(pipelive_kv_t *kv) {
  if (!kv) return;
  if (kv->pinned) (void)hipHostFree(kv->pinned);
  (void)hipEventDestroy(kv->plan_ready);
  delete kv;
}

int64_t pipelive_kv_num_blocks(const pipelive_kv_t *kv) { return kv ? kv->d.num_blocks : -1; }

/* ------------------------------------------------------------ attention */

// launch shape: number of waves and share size for a decode call
struct AttnShape {
  int32_t num_waves, tiles_per_wave;
};

static bool attn_shape(const pipelive_kv_t *kv, int32_t num_seqs, int32_t max_ctx,
                       int32_t split_tokens, AttnShape *out) {
  if (split_tokens < 0 || split_tokens % 32) return false;
  const int64_t upper = (int64_t)num_seqs * kv->d.num_kv_heads * ((max_ctx + 31) / 32);
  if (upper >= (1ll << 31)) return false;  // the kernels' share arithmetic is 32-bit
  if (split_tokens == 0) {
    // equal shares over exactly the waves the device keeps resident
    // One wave per SIMD: measured on MI355X, 768-1024 waves with one 16 KiB tile in
    // flight and one being computed (24-32 MB outstanding) saturate HBM; more waves
    // only lengthen the queues that every dependent access (block table, block
    // list, partial records) then has to wait in.
    int wpc = attn_waves_per_cu(kv->d.head_dim, kv->d.block_tokens);
    if (wpc > 4) wpc = 4;
    const int64_t resident = (int64_t)device_cu_count() * wpc;
    int64_t nw = upper < resident ? upper : resident;
    out->num_waves = (int32_t)(nw < 1 ? 1 : nw);
    out->tiles_per_wave = 0;
  } else {
    const int64_t q = split_tokens / 32;
    const int64_t nw = (upper + q - 1) / q;
    if (nw > (1ll << 30)) return false;
    out->num_waves = (int32_t)(nw < 1 ? 1 : nw);
    out->tiles_per_wave = (int32_t)q;
  }
  return true;
}

static int32_t effective_max_ctx(const pipelive_kv_t *kv, int32_t table_stride, int32_t max_ctx) {
  const int64_t table_cap = (int64_t)table_stride * kv->d.block_tokens;
  if (max_ctx <= 0 || max_ctx > table_cap) return (int32_t)(table_cap > 0x7FFFFF00 ? 0x7FFFFF00 : table_cap);
  return max_ctx;
}

size_t pipelive_paged_attn_workspace_bytes(const pipelive_kv_t *kv, int32_t num_seqs,
                                           int32_t max_ctx, int32_t split_tokens) {
  if (!kv || num_seqs <= 0 || max_ctx <= 0) return 256;
  AttnShape sh;
  if (!attn_shape(kv, num_seqs, max_ctx, split_tokens, &sh)) return 0;
  const int G = kv->d.num_q_heads / kv->d.num_kv_heads;
  size_t bytes = (size_t)2 * sh.num_waves * attn_record_floats(G, kv->d.head_dim) * 4;
  return round_up(bytes, 256);
}

int32_t pipelive_paged_attn_decode(const pipelive_kv_t *kv, int32_t layer, const void *q, void *out,
                                   int32_t out_dtype, const int32_t *block_table,
                                   int32_t table_stride, const int32_t *ctx_lens, int32_t num_seqs,
                                   int32_t max_ctx, float scale, int32_t split_tokens,
                                   void *workspace, size_t workspace_bytes, void *stream) {
  if (!kv || !q || !out || !block_table || !ctx_lens) return PIPELIVE_E_INVAL;
  if (layer < 0 || layer >= kv->d.num_layers) return PIPELIVE_E_RANGE;
  if (num_seqs < 0 || num_seqs > 65535 || table_stride <= 0) return PIPELIVE_E_INVAL;
  if (out_dtype != PIPELIVE_OUT_F32 && out_dtype != PIPELIVE_OUT_BF16) return PIPELIVE_E_INVAL;
  if (!aligned(q, 16) || !aligned(out, 16)) return PIPELIVE_E_INVAL;
  if (num_seqs == 0) return PIPELIVE_OK;
  max_ctx = effective_max_ctx(kv, table_stride, max_ctx);
  AttnShape sh;
  if (!attn_shape(kv, num_seqs, max_ctx, split_tokens, &sh)) return PIPELIVE_E_INVAL;
  const size_t need = pipelive_paged_attn_workspace_bytes(kv, num_seqs, max_ctx, split_tokens);
  if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return PIPELIVE_E_NOSPACE;

  AttnParams p;
  p.block_list = kv->d.block_list + (int64_t)(layer / kv->d.stack_k) * kv->d.capacity_blocks;
  p.layer_off = (uint32_t)((layer % kv->d.stack_k) * kv->blk_bytes);
  p.q = (const uint16_t *)q;
  p.out = out;
  p.out_dtype = out_dtype;
  p.table = block_table;
  p.table_stride = table_stride;
  p.ctx = ctx_lens;
  p.num_seqs = num_seqs;
  p.max_ctx = max_ctx;
  p.Hq = kv->d.num_q_heads;
  p.Hkv = kv->d.num_kv_heads;
  p.G = p.Hq / p.Hkv;
  const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)kv->d.head_dim);
  p.scale_log2 = sc * 1.4426950408889634f;
  p.num_waves = sh.num_waves;
  p.tiles_per_wave = sh.tiles_per_wave;
  p.ws = (float *)workspace;
  p.num_blocks = kv->d.num_blocks;
  p.status = &dev_state(kv)->status;
  if (p.Hq > 65535) return PIPELIVE_E_INVAL;
  HIP_TRY(launch_attn_decode(p, kv->d.head_dim, kv->d.block_tokens, (hipStream_t)stream));
  return PIPELIVE_OK;
}

size_t pipelive_noalloc_scratch_bytes(void) { return kNoallocScratchBytes; }

int32_t pipelive_paged_attn_decode_noalloc(const pipelive_kv_t *kv, int32_t layer, const void *q, void *out,
                                           int32_t out_dtype, const int32_t *block_table,
                                           int32_t table_stride, const int32_t *ctx_lens,
                                           int32_t num_seqs, int32_t max_ctx, float scale,
                                           int32_t split_tokens, void *stream) {
  if (!kv || table_stride <= 0) return PIPELIVE_E_INVAL;
  if (num_seqs > 0) {
    const size_t need = pipelive_paged_attn_workspace_bytes(kv, num_seqs, effective_max_ctx(kv, table_stride, max_ctx),
                                                            split_tokens);
    if (need == 0) return PIPELIVE_E_INVAL;
    if (need > kNoallocScratchBytes) return PIPELIVE_E_NOSPACE;  // this launch shape needs a caller's workspace
  }
  void *ptr = nullptr;
  const int32_t rc = noalloc_scratch(&ptr);
  if (rc != PIPELIVE_OK) return rc;
  return pipelive_paged_attn_decode(kv, layer, q, out, out_dtype, block_table, table_stride, ctx_lens, num_seqs,
                                    max_ctx, scale, split_tokens, ptr, kNoallocScratchBytes, stream);
}

int32_t pipelive_paged_attn_prefill(const pipelive_kv_t *kv, int32_t layer, const void *q, void *out,
                                    int32_t out_dtype, const int32_t *block_table,
                                    int32_t table_stride, const int32_t *ctx_lens,
                                    const int32_t *q_offsets, int32_t num_seqs, int32_t total_q,
                                    int32_t max_ctx, float scale, void *stream) {
  if (!kv || !q || !out || !block_table || !ctx_lens || !q_offsets) return PIPELIVE_E_INVAL;
  if (layer < 0 || layer >= kv->d.num_layers) return PIPELIVE_E_RANGE;
  if (num_seqs < 0 || total_q < 0 || table_stride <= 0) return PIPELIVE_E_INVAL;
  if (out_dtype != PIPELIVE_OUT_F32 && out_dtype != PIPELIVE_OUT_BF16) return PIPELIVE_E_INVAL;
  if (!aligned(q, 16) || !aligned(out, 16)) return PIPELIVE_E_INVAL;
  if (num_seqs == 0 || total_q == 0) return PIPELIVE_OK;
  PrefillParams p;
  p.block_list = kv->d.block_list + (int64_t)(layer / kv->d.stack_k) * kv->d.capacity_blocks;
  p.layer_off = (uint32_t)((layer % kv->d.stack_k) * kv->blk_bytes);
  p.q = (const uint16_t *)q;
  p.out = out;
  p.out_dtype = out_dtype;
  p.table = block_table;
  p.table_stride = table_stride;
  p.ctx = ctx_lens;
  p.q_offsets = q_offsets;
  p.num_seqs = num_seqs;
  p.max_ctx = effective_max_ctx(kv, table_stride, max_ctx);
  p.Hq = kv->d.num_q_heads;
  p.Hkv = kv->d.num_kv_heads;
  p.G = p.Hq / p.Hkv;
  const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)kv->d.head_dim);
  p.scale_log2 = sc * 1.4426950408889634f;
  // units = (sequence, KV head, block of 4 * QB query tokens); the ragged split is only known on the
  // device, so the kernel gets an upper bound and stops at the first ticket that names no unit
  const int wb = 4 * ((kPrefillNQ * 16) / p.G);
  const int64_t units = (int64_t)p.Hkv * ((total_q + wb - 1) / wb + num_seqs);
  if (units > (1ll << 30)) return PIPELIVE_E_INVAL;
  p.num_units = (int32_t)units;
  p.num_blocks = kv->d.num_blocks;
  p.status = &dev_state(kv)->status;
  p.ticket = prefill_tickets(kv);
  p.n_lists = 1;
  p.finished = &dev_state(kv)->prefill_finished;
  HIP_TRY(launch_attn_prefill(p, kv->d.head_dim, kv->d.block_tokens, (hipStream_t)stream));
  return PIPELIVE_OK;
}

/* --------------------------------------------------------------- resize */

size_t pipelive_kv_resize_workspace_bytes(const pipelive_kv_t *kv) {
  if (!kv) return 0;
  const size_t cap = (size_t)(kv->d.capacity_blocks > 0 ? kv->d.capacity_blocks : 1);
  return 256 + 3 * round_up(cap * 4, 256);
}

int64_t pipelive_max_blocks(double mem_bytes, double util, int64_t layers,
                            double weight_bytes_per_layer, double block_bytes_per_layer) {
  if (layers <= 0 || block_bytes_per_layer <= 0) return 0;
  const double v = (mem_bytes * util - (double)layers * weight_bytes_per_layer) /
                   ((double)layers * block_bytes_per_layer);
  return v < 0 ? 0 : (int64_t)floor(v);
}

int32_t pipelive_kv_resize(pipelive_kv_t *kv, int64_t new_num_blocks, int32_t *const *block_tables,
                           const int32_t *table_rows, const int32_t *table_strides,
                           const int32_t *const *table_used, int32_t num_tables,
                           int32_t *remap_out, pipelive_resize_result_t *result, void *workspace,
                           size_t workspace_bytes, void *stream) {
  if (!kv || new_num_blocks < 0 || num_tables < 0 || num_tables > PIPELIVE_MAX_TABLES)
    return PIPELIVE_E_INVAL;
  if (num_tables > 0 && (!block_tables || !table_rows || !table_strides || !table_used))
    return PIPELIVE_E_INVAL;
  TableRef tabs[PIPELIVE_MAX_TABLES];
  for (int t = 0; t < num_tables; ++t) {
    if (!block_tables[t] || !table_used[t] || table_rows[t] < 0 || table_strides[t] <= 0)
      return PIPELIVE_E_INVAL;
    tabs[t].table = block_tables[t];
    tabs[t].used = table_used[t];
    tabs[t].rows = table_rows[t];
    tabs[t].stride = table_strides[t];
  }
  if (!workspace || !aligned(workspace, 256) ||
      workspace_bytes < pipelive_kv_resize_workspace_bytes(kv))
    return PIPELIVE_E_NOSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int64_t B = kv->d.num_blocks;
  const size_t cap = (size_t)(kv->d.capacity_blocks > 0 ? kv->d.capacity_blocks : 1);
  ResizePlanOut *plan = (ResizePlanOut *)workspace;
  int32_t *move_src = (int32_t *)((char *)workspace + 256);
  int32_t *move_dst = (int32_t *)((char *)move_src + round_up(cap * 4, 256));
  int32_t *remap = remap_out ? remap_out : (int32_t *)((char *)move_dst + round_up(cap * 4, 256));

  pipelive_resize_result_t res;
  memset(&res, 0, sizeof res);
  res.old_num_blocks = B;
  res.new_num_blocks = B;
  int32_t rc = PIPELIVE_OK;

  HIP_TRY(launch_resize_plan(kv, B, new_num_blocks, plan, move_src, move_dst, st));
  for (int t = 0; t < num_tables; ++t) HIP_TRY(launch_table_check(kv, B, tabs[t], plan, st));
  HIP_TRY(hipMemcpyAsync(kv->pinned->plan, plan, sizeof(ResizePlanOut), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipEventRecord(kv->plan_ready, st));
  // The commit is queued behind the plan without waiting for it: its kernels take the verdict from
  // the plan in device memory and leave everything untouched when it refuses. Only a size beyond
  // the capacity is a host decision (the device verdict does not know the capacity).
  const bool fits = new_num_blocks <= kv->d.capacity_blocks;
  if (fits && new_num_blocks < B)
    HIP_TRY(launch_resize_commit(kv, B, new_num_blocks, plan, move_src, move_dst, remap, tabs,
                                 num_tables, st));
  else if (fits)
    HIP_TRY(launch_grow(kv, B, new_num_blocks, remap, plan, st));
  HIP_TRY(hipEventSynchronize(kv->plan_ready));
  const int64_t n_live = kv->pinned->plan[0], n_moved = kv->pinned->plan[1];
  const bool any_dirty = kv->pinned->plan[2] != 0, bad_table = kv->pinned->plan[3] != 0;
  res.n_live = n_live;
  if (!fits) rc = PIPELIVE_E_NOSPACE;
  else if (any_dirty) rc = PIPELIVE_E_BUSY;
  else if (n_live > new_num_blocks) rc = PIPELIVE_E_INFEASIBLE;
  else if (bad_table) rc = PIPELIVE_E_RANGE;

  if (rc == PIPELIVE_OK) {
    if (new_num_blocks < B) res.n_moved = n_moved;
    kv->d.num_blocks = new_num_blocks;
    res.new_num_blocks = new_num_blocks;
  }
  res.status = rc;
  if (result) *result = res;
  return rc;
}

/* ---------------------------------------------------------------- patch */

int32_t pipelive_kv_mark_dirty(pipelive_kv_t *kv, const int32_t *block_ids, int32_t n,
                               int64_t n_tokens, void *stream) {
  if (!kv || n < 0 || n_tokens < 0 || (n > 0 && !block_ids)) return PIPELIVE_E_INVAL;
  if (n == 0 && n_tokens == 0) return PIPELIVE_OK;
  HIP_TRY(launch_mark(kv, block_ids, n, n_tokens, (hipStream_t)stream));
  return PIPELIVE_OK;
}

int32_t pipelive_kv_append(pipelive_kv_t *kv, int32_t layer, const void *k_new, const void *v_new,
                           const int32_t *block_table, int32_t table_stride,
                           const int32_t *positions, int32_t num_seqs, int32_t mark,
                           int32_t count_tokens, void *stream) {
  if (!kv || !k_new || !v_new || !block_table || !positions) return PIPELIVE_E_INVAL;
  if (layer < 0 || layer >= kv->d.num_layers) return PIPELIVE_E_RANGE;
  if (num_seqs < 0 || table_stride <= 0 || !aligned(k_new, 16) || !aligned(v_new, 16))
    return PIPELIVE_E_INVAL;
  if (num_seqs == 0) return PIPELIVE_OK;
  HIP_TRY(launch_append(kv, layer, (const uint16_t *)k_new, (const uint16_t *)v_new, block_table,
                        table_stride, positions, num_seqs, mark, count_tokens, (hipStream_t)stream));
  return PIPELIVE_OK;
}

int32_t pipelive_kv_append_chunk(pipelive_kv_t *kv, int32_t layer, const void *k_new, const void *v_new,
                                 const int32_t *block_table, int32_t table_stride,
                                 const int32_t *ctx_lens, const int32_t *q_offsets, int32_t num_seqs,
                                 int32_t total_q, int32_t mark, int32_t count_tokens, void *stream) {
  if (!kv || !k_new || !v_new || !block_table || !ctx_lens || !q_offsets) return PIPELIVE_E_INVAL;
  if (layer < 0 || layer >= kv->d.num_layers) return PIPELIVE_E_RANGE;
  if (num_seqs < 0 || total_q < 0 || table_stride <= 0 || !aligned(k_new, 16) || !aligned(v_new, 16))
    return PIPELIVE_E_INVAL;
  if (num_seqs == 0 || total_q == 0) return PIPELIVE_OK;
  HIP_TRY(launch_append_chunk(kv, layer, (const uint16_t *)k_new, (const uint16_t *)v_new, block_table,
                              table_stride, ctx_lens, q_offsets, num_seqs, total_q, mark, count_tokens,
                              (hipStream_t)stream));
  return PIPELIVE_OK;
}

int64_t pipelive_patch_max_blocks(const pipelive_kv_t *kv, int32_t n_layers, size_t capacity) {
  if (!kv || n_layers <= 0 || capacity < 64 + 256) return 0;
  const uint64_t per = 4 + (uint64_t)n_layers * kv->unit_bytes;
  uint64_t mb = (capacity - 64 - 256) / per;
  const uint64_t units = (uint64_t)(kv->d.num_blocks * kv->units_per_block);
  if (mb > units) mb = units;
  return (int64_t)mb;
}

static int32_t fill_layers(const pipelive_kv_t *kv, const int32_t *layers, int32_t n, LayerList *ll) {
  if (!layers || n <= 0 || n > PIPELIVE_MAX_PATCH_LAYERS) return PIPELIVE_E_INVAL;
  ll->n = n;
  for (int i = 0; i < n; ++i) {
    if (layers[i] < 0 || layers[i] >= kv->d.num_layers) return PIPELIVE_E_RANGE;
    ll->layer[i] = layers[i];
  }
  for (int i = n; i < PIPELIVE_MAX_PATCH_LAYERS; ++i) ll->layer[i] = 0;
  return PIPELIVE_OK;
}

int32_t pipelive_kv_patch_collect(pipelive_kv_t *src, const int32_t *layers, int32_t n_layers,
                                  void *patch_buf, size_t patch_capacity_bytes,
                                  pipelive_patch_hdr_t *hdr_host_copy, void *stream) {
  if (!src || !patch_buf || !aligned(patch_buf, 256)) return PIPELIVE_E_INVAL;
  LayerList ll;
  int32_t rc = fill_layers(src, layers, n_layers, &ll);
  if (rc != PIPELIVE_OK) return rc;
  const int64_t mb = pipelive_patch_max_blocks(src, n_layers, patch_capacity_bytes);
  if (mb <= 0) return PIPELIVE_E_NOSPACE;
  const uint64_t payload_offset = round_up(64 + 4 * (uint64_t)mb, 256);
  hipStream_t st = (hipStream_t)stream;
  HIP_TRY(launch_collect(src, ll, (uint8_t *)patch_buf, (uint32_t)mb, payload_offset, st));
  if (hdr_host_copy)
    HIP_TRY(hipMemcpyAsync(hdr_host_copy, patch_buf, sizeof(pipelive_patch_hdr_t),
                           hipMemcpyDeviceToHost, st));
  return PIPELIVE_OK;
}

int32_t pipelive_kv_patch_apply(pipelive_kv_t *dst, const int32_t *dst_layers, int32_t n_layers,
                                const void *patch_buf, size_t patch_bytes,
                                const int32_t *dst_block_map, int64_t map_entries, void *stream) {
  if (!dst || !patch_buf || !aligned(patch_buf, 256)) return PIPELIVE_E_INVAL;
  if (patch_bytes < 64 + 256 || (dst_block_map && map_entries < 0)) return PIPELIVE_E_INVAL;
  LayerList ll;
  int32_t rc = fill_layers(dst, dst_layers, n_layers, &ll);
  if (rc != PIPELIVE_OK) return rc;
  HIP_TRY(launch_apply(dst, ll, (const uint8_t *)patch_buf, (uint64_t)patch_bytes, dst_block_map,
                       map_entries, (hipStream_t)stream));
  return PIPELIVE_OK;
}

int64_t pipelive_kv_tokens_applied(const pipelive_kv_t *dst) {
  if (!dst) return PIPELIVE_E_INVAL;
  unsigned long long t = 0;
  hipError_t e = hipMemcpy(&t, &dev_state(dst)->t_applied, sizeof t, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(e);
  return (int64_t)t;
}

int32_t pipelive_kv_read_state(pipelive_kv_t *kv, pipelive_kv_state_t *out, void *stream) {
  if (!kv || !out) return PIPELIVE_E_INVAL;
  hipStream_t st = (hipStream_t)stream;
  HIP_TRY(hipMemcpyAsync(&kv->pinned->state, dev_state(kv), sizeof(DevState), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  out->n_acc = kv->pinned->state.n_acc;
  out->t_applied = kv->pinned->state.t_applied;
  out->status = kv->pinned->state.status;
  out->reserved = 0;
  return PIPELIVE_OK;
}

int32_t pipelive_kv_clear_status(pipelive_kv_t *kv, void *stream) {
  if (!kv) return PIPELIVE_E_INVAL;
  HIP_TRY(launch_clear_status(kv, (hipStream_t)stream));
  return PIPELIVE_OK;
}

const char *pipelive_strerror(int32_t code) {
  switch (code) {
    case PIPELIVE_OK: return "ok";
    case PIPELIVE_E_INVAL: return "invalid argument";
    case PIPELIVE_E_INFEASIBLE: return "infeasible: more live blocks than the requested pool size";
    case PIPELIVE_E_NOSPACE: return "no space: capacity, workspace or patch buffer too small";
    case PIPELIVE_E_BUSY: return "busy: dirty blocks pending";
    case PIPELIVE_E_RANGE: return "block id or layer out of range";
    case PIPELIVE_E_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

const char *pipelive_last_hip_error(void) { return g_hip_err; }

int32_t pipelive_device_ok(void) {
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
  return strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 0;
}

}  // extern "C"
