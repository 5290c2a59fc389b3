// Incremental KV patching (paper Sec. 6.1 "KV Migration with KV Patch"):
// dirty bitmap, atomic drain, gather of the dirty blocks into a contiguous
// patch, scatter-apply on the target, and the n_acc / T_applied counters.
//
// A dirty-tracking unit is a block or, at slot granularity, one token slot
// (unit id = block id * bs + slot); a slot's patch entry is the token's
// K[Hkv][D] then V[Hkv][D], gathered out of the in-block layout.
//
// append  : write one new token per sequence into its slot (K as 16-byte
//           d-slices, V element-wise), mark the written unit, count tokens.
// mark    : atomicOr of one bit per written unit; n_acc += n_tokens once every
//           bit of the call is set.
// drain   : takes n_acc, then one workgroup swaps every bitmap word with zero
//           (atomicExch, so a concurrent mark is either in this snapshot or
//           stays for the next drain), prefix-sums the popcounts, writes the
//           ascending id list and the header, and ORs back the bits beyond the
//           patch capacity.  Order of the two sides (writers: data, then bit,
//           then count; drain: count, then bits): a patch never acknowledges a
//           token whose slot it, or an earlier patch, does not carry.
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

// Ordering between a writer (slot bytes, then dirty bit, then token count) and a drain that runs beside it
// on another stream (count, then bits, then bytes).  Every access that takes part is a device-scope
// operation that bypasses the per-XCD L2 (atomics, write-through stores, device-scope loads), so "earlier"
// only has to mean "acknowledged before the next one is issued": order_point() waits for the wave's
// outstanding memory operations and nothing else.  It writes back or invalidates no cache, unlike a
// device-scope fence, which costs several microseconds per launch on this chip.
__device__ __forceinline__ void order_point() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // keeps the compiler from moving accesses across
  __builtin_amdgcn_s_waitcnt(0x0F70);                     // s_waitcnt vmcnt(0): stores and atomics acknowledged
}

template <typename T>
__device__ __forceinline__ void store_through(T *p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ u64 load_through(const u64 *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int64_t kDrainOneWgWords = 4096;  // bitmaps up to this many words are drained by one workgroup
constexpr int kDrainWordsPerLane = (int)(kDrainOneWgWords / kScanThreads);

__global__ void mark_kernel(u64 *dirty, int64_t B, const int32_t *ids, int32_t n, u64 n_tokens,
                            DevState *st) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const int32_t id = ids[i];
    if (id < 0 || id >= B) {
      atomicCAS(&st->status, 0, PIPELIVE_E_RANGE);
    } else {
      atomicOr(&dirty[id >> 6], 1ull << (id & 63));
    }
  }
  if (n_tokens == 0) return;  // uniform over the launch
  // the tokens are counted once every bit of this call is set: the last workgroup to get here adds them
  order_point();
  __syncthreads();
  if (threadIdx.x == 0) {
    bool last = gridDim.x == 1;
    if (!last && atomicAdd(&st->mark_blocks_done, 1) == (int)gridDim.x - 1) {
      atomicExch(&st->mark_blocks_done, 0);
      last = true;
    }
    if (last) atomicAdd(&st->n_acc, n_tokens);
  }
}

__global__ __launch_bounds__(kScanThreads) void drain_kernel(u64 *dirty, int64_t B, u64 *snap,
                                                             DevState *st, uint8_t *patch,
                                                             uint32_t max_blocks, uint32_t n_layers,
                                                             u64 block_bytes, u64 payload_offset,
                                                             uint32_t unit_tokens) {
  __shared__ uint32_t sh[17];
  __shared__ u64 sh_acc;
  const int64_t nwords = (B + 63) / 64;
  const int64_t per = (nwords + kScanThreads - 1) / kScanThreads;  // <= kDrainOneWgWords / kScanThreads
  const int64_t w0 = (int64_t)threadIdx.x * per;
  const int64_t w1 = w0 + per < nwords ? w0 + per : nwords;
  // n_acc is taken before the first word is looked at (it goes back below if bits stay behind): a count
  // taken here belongs to bits that were set before it, and the reads below come after it
  if (threadIdx.x == 0) sh_acc = atomicExch(&st->n_acc, 0ull);
  __syncthreads();
  // which words need an exchange at all
  u64 seen[kDrainWordsPerLane];
#pragma unroll
  for (int k = 0; k < kDrainWordsPerLane; ++k) seen[k] = (w0 + k < w1) ? load_through(&dirty[w0 + k]) : 0ull;
  uint32_t cnt = 0;
#pragma unroll
  for (int k = 0; k < kDrainWordsPerLane; ++k) {
    const int64_t w = w0 + k;
    if (w >= w1) break;
    const u64 v = seen[k] ? atomicExch(&dirty[w], 0ull) : 0ull;
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
    h.n_acc_tokens = h.more_pending ? 0ull : sh_acc;
    if (h.more_pending && sh_acc) atomicAdd(&st->n_acc, sh_acc);
    h.payload_offset = payload_offset;
    h.max_blocks = max_blocks;
    h.unit_tokens = unit_tokens;
    for (int i = 0; i < 12; ++i) h.pad[i] = 0;
    *(pipelive_patch_hdr_t *)patch = h;
  }
}

// ---- drain of a large bitmap in three small kernels (used above kDrainOneWgWords
// words, e.g. slot granularity on a big pool): count per workgroup, scan the
// workgroup counts, emit.  Same result as drain_kernel.
constexpr int kDrainThreads = 256;

// first kernel of the large-bitmap drain: n_acc is taken before any word is exchanged
__global__ void drain_begin_kernel(DevState *st) { st->n_acc_taken = atomicExch(&st->n_acc, 0ull); }

__global__ __launch_bounds__(kDrainThreads) void drain_count_kernel(u64 *dirty, int64_t nwords, u64 *snap,
                                                                    uint32_t *wg_count) {
  __shared__ uint32_t sh[kDrainThreads / 64];
  const int64_t w = (int64_t)blockIdx.x * kDrainThreads + threadIdx.x;
  u64 v = 0;
  if (w < nwords) {
    v = load_through(&dirty[w]);
    if (v) v = atomicExch(&dirty[w], 0ull);
    snap[w] = v;
  }
  uint32_t c = __popcll(v);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
    for (int i = 0; i < kDrainThreads / 64; ++i) t += sh[i];
    wg_count[blockIdx.x] = t;
  }
}

// exclusive scan of the workgroup counts (in place) and the patch header
__global__ __launch_bounds__(kScanThreads) void drain_scan_kernel(uint32_t *wg_count, int64_t n_wg, DevState *st,
                                                                  uint8_t *patch, uint32_t max_blocks,
                                                                  uint32_t n_layers, u64 block_bytes,
                                                                  u64 payload_offset, uint32_t unit_tokens) {
  __shared__ uint32_t sh[17];
  uint32_t carry = 0;
  for (int64_t base = 0; base < n_wg; base += kScanThreads) {
    const int64_t i = base + threadIdx.x;
    const uint32_t c = i < n_wg ? wg_count[i] : 0;
    uint32_t tot;
    const uint32_t ex = wg_exclusive_scan(c, sh, &tot);
    if (i < n_wg) wg_count[i] = carry + ex;
    carry += tot;
  }
  if (threadIdx.x == 0) {
    const uint32_t total = carry;
    pipelive_patch_hdr_t h;
    h.magic = PIPELIVE_PATCH_MAGIC;
    h.version = PIPELIVE_PATCH_VERSION;
    h.n_blocks = total < max_blocks ? total : max_blocks;
    h.n_layers = n_layers;
    h.block_bytes = block_bytes;
    h.more_pending = total > max_blocks ? 1u : 0u;
    const u64 taken = st->n_acc_taken;  // by drain_begin_kernel, before the words were exchanged
    st->n_acc_taken = 0;
    h.n_acc_tokens = h.more_pending ? 0ull : taken;
    if (h.more_pending && taken) atomicAdd(&st->n_acc, taken);
    h.payload_offset = payload_offset;
    h.max_blocks = max_blocks;
    h.unit_tokens = unit_tokens;
    for (int i = 0; i < 12; ++i) h.pad[i] = 0;
    *(pipelive_patch_hdr_t *)patch = h;
  }
}

__global__ __launch_bounds__(kDrainThreads) void drain_emit_kernel(u64 *dirty, int64_t nwords, const u64 *snap,
                                                                   const uint32_t *wg_offset, uint8_t *patch,
                                                                   uint32_t max_blocks) {
  __shared__ uint32_t sh[kDrainThreads / 64];
  const int64_t w = (int64_t)blockIdx.x * kDrainThreads + threadIdx.x;
  u64 v = w < nwords ? snap[w] : 0;
  const uint32_t c = __popcll(v);
  // exclusive prefix inside the workgroup: wave scan, then the 4 wave totals
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  uint32_t inc = c;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  if (lane == 63) sh[wv] = inc;
  __syncthreads();
  uint32_t rank = wg_offset[blockIdx.x] + inc - c;
  for (int i = 0; i < wv; ++i) rank += sh[i];
  int32_t *ids = (int32_t *)(patch + 64);
  u64 back = 0;
  while (v) {
    const int b = __ffsll((long long)v) - 1;
    if (rank < max_blocks) ids[rank] = (int32_t)(w * 64 + b);
    else back |= 1ull << b;
    ++rank;
    v &= v - 1;
  }
  if (back) atomicOr(&dirty[w], back);
}

struct XferArgs {
  const uint64_t *block_list;
  int64_t capacity, num_blocks;
  uint32_t stack_k, blk_bytes, sub_bytes, subs_per_block;
  uint32_t Hkv, D, bs, unit_tokens;
  LayerList layers;
  const int32_t *dst_map;
  int64_t map_entries;   // source block ids a patch may name: entries of dst_map, or num_blocks without a map
  uint64_t patch_bytes;  // size of the buffer an incoming patch lies in
  DevState *st;
};

// The receiver's check of an incoming patch (it may come from another sender): header fields against the
// target region and the buffer size, every id against the id space, every mapped id against the target.
// One workgroup; the verdict goes to the region's device state and the scatter kernel behind it obeys
// it: a patch that fails is refused as a whole (no byte written, T_applied unchanged, status set).
__global__ __launch_bounds__(kScanThreads) void apply_check_kernel(XferArgs a, const uint8_t *patch) {
  __shared__ int sh_bad;
  const pipelive_patch_hdr_t *h = (const pipelive_patch_hdr_t *)patch;
  if (threadIdx.x == 0) sh_bad = 0;
  __syncthreads();
  int verdict = PIPELIVE_OK;
  const uint64_t ids_end = 64 + 4 * (uint64_t)h->max_blocks;
  if (a.patch_bytes < 64 || h->magic != PIPELIVE_PATCH_MAGIC || h->version != PIPELIVE_PATCH_VERSION ||
      h->n_layers != (uint32_t)a.layers.n || h->block_bytes != a.blk_bytes || h->unit_tokens != a.unit_tokens) {
    verdict = PIPELIVE_E_INVAL;
  } else if (h->n_blocks > h->max_blocks || h->payload_offset != (ids_end + 255) / 256 * 256 ||
             h->payload_offset > a.patch_bytes ||
             (uint64_t)h->n_blocks * a.layers.n * a.blk_bytes > a.patch_bytes - h->payload_offset) {
    verdict = PIPELIVE_E_INVAL;
  } else {
    const int32_t *ids = (const int32_t *)(patch + 64);
    const int64_t upb = a.unit_tokens == 1 ? (int64_t)a.bs : 1;  // units per block
    const uint32_t n = h->n_blocks;
    bool bad = false;
    for (uint32_t r = threadIdx.x; r < n; r += kScanThreads) {
      const int64_t u = ids[r];
      int64_t blk = u / upb;
      if (u < 0 || blk >= a.map_entries) {
        bad = true;
      } else {
        if (a.dst_map) blk = a.dst_map[blk];
        if (blk < 0 || blk >= a.num_blocks) bad = true;
      }
    }
    if (bad) sh_bad = 1;
    __syncthreads();
    if (sh_bad) verdict = PIPELIVE_E_RANGE;
  }
  if (threadIdx.x == 0) {
    a.st->apply_verdict = verdict;
    if (verdict != PIPELIVE_OK) atomicCAS(&a.st->status, 0, verdict);
    else if (h->n_acc_tokens) atomicAdd(&a.st->t_applied, (u64)h->n_acc_tokens);
  }
}

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
  if (a.st->apply_verdict != PIPELIVE_OK) return;  // refused by apply_check_kernel: nothing is written
  const pipelive_patch_hdr_t *h = (const pipelive_patch_hdr_t *)patch;
  const uint32_t nl = a.layers.n;
  const uint32_t n_blocks = h->n_blocks;
  const int32_t *ids = (const int32_t *)(patch + 64);
  const char *payload = (const char *)patch + h->payload_offset;
  const int64_t n_items = (int64_t)n_blocks * nl * a.subs_per_block;
  for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const uint32_t sub = (uint32_t)(item % a.subs_per_block);
    const int64_t e = item / a.subs_per_block;
    const uint32_t i = (uint32_t)(e % nl);
    const int64_t r = e / nl;
    const int32_t layer = a.layers.layer[i];
    int64_t id = ids[r];  // checked by apply_check_kernel, as is the mapped id
    if (a.dst_map) id = a.dst_map[id];
    char *dst = (char *)a.block_list[(int64_t)(layer / a.stack_k) * a.capacity + id] +
                (uint64_t)(layer % a.stack_k) * a.blk_bytes;
    const uint32_t off = sub * a.sub_bytes;
    const uint32_t len = a.blk_bytes - off < a.sub_bytes ? a.blk_bytes - off : a.sub_bytes;
    wg_copy(dst + off, payload + (uint64_t)e * a.blk_bytes + off, len);
  }
}

// ---- slot granularity: one token per unit -------------------------------------
// In-block layout: sub-blocks of sb = min(bs, 32) tokens, each K[Hkv][D/8][sb][8]
// then V[Hkv][D][sb].  Returns the sub-block holding token t of the block and
// leaves t's position inside it in `tt`.
__device__ __forceinline__ char *token_sub_block(char *blk, uint32_t t, uint32_t Hkv, uint32_t D,
                                                 uint32_t bs, uint32_t &sb, uint32_t &tt) {
  sb = bs < 32u ? bs : 32u;
  tt = t % sb;
  return blk + (uint64_t)(t / sb) * ((uint64_t)2 * Hkv * sb * D * 2);
}

// Copy token `t` of a layer's block between the in-block layout and a
// token-major record K[Hkv][D] | V[Hkv][D].
// to_record = true gathers block -> record, false scatters record -> block.
template <bool to_record>
__device__ __forceinline__ void wg_copy_token(char *blk, char *rec, uint32_t t, uint32_t Hkv,
                                              uint32_t D, uint32_t bs_block) {
  uint32_t bs;
  blk = token_sub_block(blk, t, Hkv, D, bs_block, bs, t);
  const uint32_t n_chunks = Hkv * D / 8;  // K: 16-byte d-slices
  for (uint32_t c = threadIdx.x; c < n_chunks; c += blockDim.x) {
    u32x4 *in_blk = (u32x4 *)(blk + ((uint64_t)c * bs + t) * 16);
    u32x4 *in_rec = (u32x4 *)(rec + (uint64_t)c * 16);
    if (to_record) *in_rec = *in_blk;
    else *in_blk = *in_rec;
  }
  const uint32_t n_el = Hkv * D;  // V: one bf16 per (head, d), bs apart in the block
  uint16_t *vblk = (uint16_t *)(blk + (uint64_t)Hkv * bs * D * 2);
  uint16_t *vrec = (uint16_t *)(rec + (uint64_t)n_el * 2);
  for (uint32_t e = threadIdx.x; e < n_el; e += blockDim.x) {
    if (to_record) vrec[e] = vblk[(uint64_t)e * bs + t];
    else vblk[(uint64_t)e * bs + t] = vrec[e];
  }
}

__global__ __launch_bounds__(kCopyThreads) void gather_slots_kernel(XferArgs a, uint8_t *patch) {
  const pipelive_patch_hdr_t *h = (const pipelive_patch_hdr_t *)patch;
  const int32_t *ids = (const int32_t *)(patch + 64);
  char *payload = (char *)patch + h->payload_offset;
  const uint32_t nl = a.layers.n;
  const int64_t n_items = (int64_t)h->n_blocks * nl;
  for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const uint32_t i = (uint32_t)(item % nl);
    const int64_t r = item / nl;
    const int32_t layer = a.layers.layer[i];
    const int32_t u = ids[r];
    char *blk = (char *)a.block_list[(int64_t)(layer / a.stack_k) * a.capacity + u / a.bs] +
                (uint64_t)(layer % a.stack_k) * ((uint64_t)2 * a.Hkv * a.bs * a.D * 2);
    wg_copy_token<true>(blk, payload + (uint64_t)item * a.blk_bytes, u % a.bs, a.Hkv, a.D, a.bs);
  }
}

__global__ __launch_bounds__(kCopyThreads) void scatter_slots_kernel(XferArgs a, const uint8_t *patch) {
  if (a.st->apply_verdict != PIPELIVE_OK) return;  // refused by apply_check_kernel: nothing is written
  const pipelive_patch_hdr_t *h = (const pipelive_patch_hdr_t *)patch;
  const uint32_t nl = a.layers.n;
  const int32_t *ids = (const int32_t *)(patch + 64);
  const char *payload = (const char *)patch + h->payload_offset;
  const int64_t n_items = (int64_t)h->n_blocks * nl;
  for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const uint32_t i = (uint32_t)(item % nl);
    const int64_t r = item / nl;
    const int32_t layer = a.layers.layer[i];
    const int32_t u = ids[r];
    int64_t id = u / a.bs;  // checked by apply_check_kernel, as is the mapped id
    if (a.dst_map) id = a.dst_map[id];
    char *blk = (char *)a.block_list[(int64_t)(layer / a.stack_k) * a.capacity + id] +
                (uint64_t)(layer % a.stack_k) * ((uint64_t)2 * a.Hkv * a.bs * a.D * 2);
    wg_copy_token<false>(blk, (char *)payload + (uint64_t)item * a.blk_bytes, u % a.bs, a.Hkv, a.D, a.bs);
  }
}

struct AppendArgs {
  const uint64_t *block_list;  // the layer's group row
  uint64_t layer_off;
  int64_t num_blocks;
  const uint16_t *k_new, *v_new;
  const int32_t *table, *positions;
  int32_t table_stride;
  uint32_t Hkv, D, bs, units_per_block;
  int32_t mark, count_tokens;
  u64 *dirty;
  DevState *st;
};

// ---- the write side of a prefill chunk: up to 32 consecutive tokens of one (sequence, KV head)
// per workgroup.  The token-major input rows are read coalesced into LDS and written out in the
// in-block layout with the token index fastest, so K leaves as 512-byte runs and V^T as 64-byte
// rows instead of 16-byte and 2-byte pieces.
struct AppendChunkArgs {
  const uint64_t *block_list;  // the layer's group row
  uint64_t layer_off;
  int64_t num_blocks;
  const uint16_t *k_new, *v_new;  // [total_q][Hkv][D]
  const int32_t *table, *ctx, *q_offsets;
  int32_t table_stride, num_seqs;
  uint32_t Hkv, D, bs, units_per_block;
  int32_t mark, count_tokens;
  u64 *dirty;
  DevState *st;
};

template <int D>
__global__ __launch_bounds__(256) void append_chunk_kernel(AppendChunkArgs a) {
  constexpr int ROW = D * 2 + 16;  // LDS row of one token and head, padded against bank conflicts
  constexpr int CH = D / 8;        // 16-byte pieces of a row
  __shared__ __attribute__((aligned(16))) char lk[32 * ROW];
  __shared__ __attribute__((aligned(16))) char lv[32 * ROW];
  const int tid = threadIdx.x, lane = tid & 63;
  const int Hkv = (int)a.Hkv, S = a.num_seqs, bs = (int)a.bs;
  const int g = blockIdx.x % Hkv;
  const int unit = blockIdx.x / Hkv;

  // ---- locate the unit: sequence s owns one unit per 32-token window that its chunk touches
  int s = -1, wi = 0;
  {
    int carry = 0;
    // workgroup 0 looks at every sequence (it is the one that flags over-long chunks)
    for (int base = 0; base < S && (s < 0 || blockIdx.x == 0); base += 64) {
      const bool in = base + lane < S;
      int nwin = 0;
      if (in) {
        const int ql = a.q_offsets[base + lane + 1] - a.q_offsets[base + lane];
        const int hi = a.ctx[base + lane], lo = hi - ql;
        if (ql > 0 && lo >= 0) nwin = (hi - 1) / 32 - lo / 32 + 1;
        // a chunk longer than its context has no place in the cache: flag it (once) and skip it
        if (ql > hi && blockIdx.x == 0 && tid < 64) atomicCAS(&a.st->status, 0, PIPELIVE_E_INVAL);
      }
      const int inc = wave_inclusive_scan(nwin, lane);
      const uint64_t bal = s < 0 ? __ballot(in && carry + inc > unit) : 0ull;
      if (bal) {
        const int k = __ffsll((long long)bal) - 1;
        s = base + k;
        wi = unit - (carry + __builtin_amdgcn_readlane(inc, k) - __builtin_amdgcn_readlane(nwin, k));
      }
      carry += __builtin_amdgcn_readlane(inc, 63);
    }
  }
  if (s < 0) return;  // beyond the last unit; the same decision in every wave
  const int q0 = a.q_offsets[s], ql = a.q_offsets[s + 1] - q0;
  const int pos_hi = a.ctx[s], pos_lo = pos_hi - ql;
  const int w = pos_lo / 32 + wi;                    // window [32w, 32w + 32)
  const int j_lo = max(32 * w, pos_lo), j_hi = min(32 * w + 32, pos_hi);
  const int tt_lo = j_lo - 32 * w, tt_hi = j_hi - 32 * w;  // valid token offsets inside the window

  // ---- the blocks of the window: one, or two 16-token blocks
  const int sb = bs < 32 ? bs : 32;
  const int halves = 32 / sb;
  char *base_h[2] = {nullptr, nullptr};
  int32_t id_h[2] = {-1, -1};
  bool ok = true;
  for (int h = 0; h < halves; ++h) {
    const int first = 32 * w + h * sb;  // first token position of this half
    if (first + sb <= j_lo || first >= j_hi) continue;  // no token of the chunk in it
    const int bi = first / bs;
    if (bi >= a.table_stride) {
      if (tid == 0) atomicCAS(&a.st->status, 0, PIPELIVE_E_INVAL);
      ok = false;
      continue;
    }
    const int32_t id = a.table[(int64_t)s * a.table_stride + bi];
    if (id < 0 || id >= a.num_blocks) {
      if (tid == 0) atomicCAS(&a.st->status, 0, PIPELIVE_E_RANGE);
      ok = false;
      continue;
    }
    id_h[h] = id;
    // the sub-block that holds this half: blocks above 32 tokens are runs of 32-token sub-blocks
    base_h[h] = (char *)a.block_list[id] + a.layer_off +
                (uint64_t)((first % bs) / sb) * ((uint64_t)2 * Hkv * sb * D * 2);
  }
  if (!ok) return;  // uniform: nothing of a window with a bad table entry is written

  // ---- token-major rows -> LDS (coalesced: a row of one head is D * 2 contiguous bytes)
  for (int e = tid; e < 32 * CH; e += 256) {
    const int tt = e / CH, c = e % CH;
    if (tt < tt_lo || tt >= tt_hi) continue;
    const int64_t row = (int64_t)q0 + (32 * w + tt - pos_lo);
    const uint64_t off = ((uint64_t)row * Hkv + g) * D + 8 * c;
    *(u32x4 *)(lk + tt * ROW + c * 16) = *(const u32x4 *)(a.k_new + off);
    *(u32x4 *)(lv + tt * ROW + c * 16) = *(const u32x4 *)(a.v_new + off);
  }
  __syncthreads();

  // ---- K[D/8][sb][8]: 16-byte pieces, token index fastest
  const uint32_t khead = (uint32_t)(sb * D * 2);
  for (int e = tid; e < 32 * CH; e += 256) {
    const int c = e / 32, tt = e % 32;
    if (tt < tt_lo || tt >= tt_hi) continue;
    char *dst = base_h[tt / sb] + (uint64_t)g * khead + (uint32_t)((c * sb + tt % sb) * 16);
    *(u32x4 *)dst = *(const u32x4 *)(lk + tt * ROW + c * 16);
  }
  // ---- V[D][sb]: a thread owns row d and a run of 32 * D / 256 consecutive tokens
  {
    constexpr int TPT = 32 * D / 256;  // tokens per thread: 16 (D 128) or 8 (D 64)
    const int d = tid % D, t0 = (tid / D) * TPT;
    uint16_t vals[TPT];
#pragma unroll
    for (int i = 0; i < TPT; ++i) vals[i] = *(const uint16_t *)(lv + (t0 + i) * ROW + d * 2);
    if (t0 < tt_hi && t0 + TPT > tt_lo) {
      uint16_t *dst = (uint16_t *)(base_h[t0 / sb] + (uint64_t)(Hkv + g) * khead) + (uint32_t)(d * sb + t0 % sb);
      if (t0 >= tt_lo && t0 + TPT <= tt_hi) {  // whole run inside the chunk: 16-byte stores
#pragma unroll
        for (int i = 0; i < TPT; i += 8) {
          u32x4 pk;
          pk.x = vals[i] | ((uint32_t)vals[i + 1] << 16);
          pk.y = vals[i + 2] | ((uint32_t)vals[i + 3] << 16);
          pk.z = vals[i + 4] | ((uint32_t)vals[i + 5] << 16);
          pk.w = vals[i + 6] | ((uint32_t)vals[i + 7] << 16);
          *(u32x4 *)(dst + i) = pk;
        }
      } else {  // the chunk begins or ends inside the run: tokens outside it keep their bytes
#pragma unroll
        for (int i = 0; i < TPT; ++i)
          if (t0 + i >= tt_lo && t0 + i < tt_hi) dst[i] = vals[i];
      }
    }
  }
  // ---- dirty marks after this head's bytes (every head's workgroup sets them: a drain that runs
  // beside the chunk's writes must find the bit again after the last of them); the tokens are
  // counted once per window, by the workgroup of KV head 0
  if (!a.mark && !(a.count_tokens && g == 0)) return;
  __threadfence();  // this window's bytes are plain 16-byte stores: written back before the bits are set
  __syncthreads();
  if (a.mark && tid >= tt_lo && tid < tt_hi) {
    const int j = 32 * w + tid;
    const int32_t id = id_h[tid / sb];
    const int64_t u = a.units_per_block > 1 ? (int64_t)id * bs + j % bs : id;
    atomicOr(&a.dirty[u >> 6], 1ull << (u & 63));
  }
  if (a.count_tokens && g == 0) {
    order_point();
    __syncthreads();
    if (tid == 0) atomicAdd(&a.st->n_acc, (unsigned long long)(tt_hi - tt_lo));
  }
}

// one workgroup per sequence: the new token's K and V of one layer
__global__ __launch_bounds__(kCopyThreads) void append_kernel(AppendArgs a) {
  const int s = blockIdx.x;
  const int pos = a.positions[s];
  if (pos < 0) return;
  if (pos / (int)a.bs >= a.table_stride) {
    if (threadIdx.x == 0) atomicCAS(&a.st->status, 0, PIPELIVE_E_INVAL);
    return;
  }
  const int32_t id = a.table[(int64_t)s * a.table_stride + pos / (int)a.bs];
  if (id < 0 || id >= a.num_blocks) {
    if (threadIdx.x == 0) atomicCAS(&a.st->status, 0, PIPELIVE_E_RANGE);
    return;
  }
  const uint32_t t = (uint32_t)pos % a.bs;
  uint32_t sb, tt;
  char *blk = token_sub_block((char *)a.block_list[id] + a.layer_off, t, a.Hkv, a.D, a.bs, sb, tt);
  const uint32_t n_el = a.Hkv * a.D;
  const uint16_t *k = a.k_new + (int64_t)s * n_el, *v = a.v_new + (int64_t)s * n_el;
  // the slot's bytes go through to memory (a drain on another stream may read them as soon as it finds
  // the bit), then the dirty bit, then the token count
  for (uint32_t c = threadIdx.x; c < n_el / 8; c += blockDim.x) {
    const u32x4 piece = *(const u32x4 *)(k + (uint64_t)c * 8);
    uint32_t *dst = (uint32_t *)(blk + ((uint64_t)c * sb + tt) * 16);
    store_through(dst + 0, piece.x);
    store_through(dst + 1, piece.y);
    store_through(dst + 2, piece.z);
    store_through(dst + 3, piece.w);
  }
  uint16_t *vblk = (uint16_t *)(blk + (uint64_t)a.Hkv * sb * a.D * 2);
  for (uint32_t e = threadIdx.x; e < n_el; e += blockDim.x) store_through(&vblk[(uint64_t)e * sb + tt], v[e]);
  if (!a.mark && !a.count_tokens) return;
  order_point();
  __syncthreads();
  if (threadIdx.x == 0) {
    if (a.mark) {
      const int64_t u = a.units_per_block > 1 ? (int64_t)id * a.bs + t : id;
      atomicOr(&a.dirty[u >> 6], 1ull << (u & 63));
    }
    if (a.count_tokens) {
      order_point();
      atomicAdd(&a.st->n_acc, 1ull);
    }
  }
}

// also re-arms the prefill kernel's work counters (they are zero already unless a launch was cut short)
__global__ void clear_status_kernel(DevState *st) {
  st->status = 0;
  st->prefill_finished = 0;
  int32_t *tickets = (int32_t *)((char *)st + kListOffset);
  for (int i = 0; i < kPrefillLists; ++i) tickets[i] = 0;
}

XferArgs make_xfer(const pipelive_kv *kv, const LayerList &layers, const int32_t *dst_map) {
  XferArgs a;
  a.block_list = kv->d.block_list;
  a.capacity = kv->d.capacity_blocks;
  a.num_blocks = kv->d.num_blocks;
  a.stack_k = (uint32_t)kv->d.stack_k;
  a.blk_bytes = (uint32_t)kv->unit_bytes;  // bytes of one patch entry
  a.Hkv = (uint32_t)kv->d.num_kv_heads;
  a.D = (uint32_t)kv->d.head_dim;
  a.bs = (uint32_t)kv->d.block_tokens;
  a.unit_tokens = kv->units_per_block > 1 ? 1u : a.bs;
  a.sub_bytes = kCopyChunk;
  a.subs_per_block = (a.blk_bytes + a.sub_bytes - 1) / a.sub_bytes;
  a.layers = layers;
  a.dst_map = dst_map;
  a.map_entries = kv->d.num_blocks;
  a.patch_bytes = 0;
  a.st = dev_state(kv);
  return a;
}

}  // namespace

hipError_t launch_mark(const pipelive_kv *kv, const int32_t *ids, int32_t n, int64_t n_tokens,
                       hipStream_t st) {
  const int threads = 256;
  const int grid = n > 0 ? (n + threads - 1) / threads : 1;
  hipLaunchKernelGGL(mark_kernel, dim3(grid), dim3(threads), 0, st, (u64 *)kv->d.dirty_bitmap,
                     kv->d.num_blocks * kv->units_per_block, ids, n, (u64)n_tokens, dev_state(kv));
  return hipGetLastError();
}

hipError_t launch_append(const pipelive_kv *kv, int32_t layer, const uint16_t *k_new,
                         const uint16_t *v_new, const int32_t *table, int32_t table_stride,
                         const int32_t *positions, int32_t num_seqs, int32_t mark,
                         int32_t count_tokens, hipStream_t st) {
  AppendArgs a;
  a.block_list = kv->d.block_list + (int64_t)(layer / kv->d.stack_k) * kv->d.capacity_blocks;
  a.layer_off = (uint64_t)(layer % kv->d.stack_k) * kv->blk_bytes;
  a.num_blocks = kv->d.num_blocks;
  a.k_new = k_new;
  a.v_new = v_new;
  a.table = table;
  a.positions = positions;
  a.table_stride = table_stride;
  a.Hkv = (uint32_t)kv->d.num_kv_heads;
  a.D = (uint32_t)kv->d.head_dim;
  a.bs = (uint32_t)kv->d.block_tokens;
  a.units_per_block = (uint32_t)kv->units_per_block;
  a.mark = mark;
  a.count_tokens = count_tokens;
  a.dirty = (u64 *)kv->d.dirty_bitmap;
  a.st = dev_state(kv);
  hipLaunchKernelGGL(append_kernel, dim3(num_seqs), dim3(kCopyThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_append_chunk(const pipelive_kv *kv, int32_t layer, const uint16_t *k_new,
                               const uint16_t *v_new, const int32_t *table, int32_t table_stride,
                               const int32_t *ctx, const int32_t *q_offsets, int32_t num_seqs,
                               int32_t total_q, int32_t mark, int32_t count_tokens, hipStream_t st) {
  AppendChunkArgs a;
  a.block_list = kv->d.block_list + (int64_t)(layer / kv->d.stack_k) * kv->d.capacity_blocks;
  a.layer_off = (uint64_t)(layer % kv->d.stack_k) * kv->blk_bytes;
  a.num_blocks = kv->d.num_blocks;
  a.k_new = k_new;
  a.v_new = v_new;
  a.table = table;
  a.ctx = ctx;
  a.q_offsets = q_offsets;
  a.table_stride = table_stride;
  a.num_seqs = num_seqs;
  a.Hkv = (uint32_t)kv->d.num_kv_heads;
  a.D = (uint32_t)kv->d.head_dim;
  a.bs = (uint32_t)kv->d.block_tokens;
  a.units_per_block = (uint32_t)kv->units_per_block;
  a.mark = mark;
  a.count_tokens = count_tokens;
  a.dirty = (u64 *)kv->d.dirty_bitmap;
  a.st = dev_state(kv);
  // a chunk of q tokens touches at most q / 32 + 2 windows; the surplus workgroups exit
  const int64_t units = ((int64_t)total_q / 32 + 2 * (int64_t)num_seqs) * kv->d.num_kv_heads;
  if (units > 0x7FFFFFFF) return hipErrorInvalidValue;
  if (kv->d.head_dim == 128)
    hipLaunchKernelGGL(append_chunk_kernel<128>, dim3((unsigned)units), dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(append_chunk_kernel<64>, dim3((unsigned)units), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_collect(const pipelive_kv *kv, const LayerList &layers, uint8_t *patch,
                          uint32_t max_blocks, uint64_t payload_offset, hipStream_t st) {
  const bool slots = kv->units_per_block > 1;
  const int64_t n_units = kv->d.num_blocks * kv->units_per_block;
  const int64_t nwords = (n_units + 63) / 64;
  const uint32_t unit_tokens = slots ? 1u : (uint32_t)kv->d.block_tokens;
  hipError_t e;
  if (nwords <= kDrainOneWgWords) {
    hipLaunchKernelGGL(drain_kernel, dim3(1), dim3(kScanThreads), 0, st, (u64 *)kv->d.dirty_bitmap,
                       n_units, snap_words(kv), dev_state(kv), patch, max_blocks, (uint32_t)layers.n,
                       (u64)kv->unit_bytes, (u64)payload_offset, unit_tokens);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  } else {
    const int64_t n_wg = (nwords + kDrainThreads - 1) / kDrainThreads;
    uint32_t *wg_count = (uint32_t *)(snap_words(kv) + nwords);  // behind the snapshot words
    hipLaunchKernelGGL(drain_begin_kernel, dim3(1), dim3(1), 0, st, dev_state(kv));
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(drain_count_kernel, dim3((unsigned)n_wg), dim3(kDrainThreads), 0, st,
                       (u64 *)kv->d.dirty_bitmap, nwords, snap_words(kv), wg_count);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(drain_scan_kernel, dim3(1), dim3(kScanThreads), 0, st, wg_count, n_wg,
                       dev_state(kv), patch, max_blocks, (uint32_t)layers.n, (u64)kv->unit_bytes,
                       (u64)payload_offset, unit_tokens);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(drain_emit_kernel, dim3((unsigned)n_wg), dim3(kDrainThreads), 0, st,
                       (u64 *)kv->d.dirty_bitmap, nwords, (const u64 *)snap_words(kv),
                       (const uint32_t *)wg_count, patch, max_blocks);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  XferArgs a = make_xfer(kv, layers, nullptr);
  const int64_t max_items = (int64_t)max_blocks * layers.n * (slots ? 1 : a.subs_per_block);
  const int64_t max_grid = (int64_t)device_cu_count() * copy_wgs_per_cu();
  const int grid = (int)(max_items < max_grid ? max_items : max_grid);
  if (slots) hipLaunchKernelGGL(gather_slots_kernel, dim3(grid), dim3(kCopyThreads), 0, st, a, patch);
  else hipLaunchKernelGGL(gather_kernel, dim3(grid), dim3(kCopyThreads), 0, st, a, patch);
  return hipGetLastError();
}

hipError_t launch_apply(const pipelive_kv *kv, const LayerList &layers, const uint8_t *patch,
                        uint64_t patch_bytes, const int32_t *dst_map, int64_t map_entries,
                        hipStream_t st) {
  XferArgs a = make_xfer(kv, layers, dst_map);
  a.patch_bytes = patch_bytes;
  a.map_entries = dst_map ? map_entries : kv->d.num_blocks;
  hipLaunchKernelGGL(apply_check_kernel, dim3(1), dim3(kScanThreads), 0, st, a, patch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int grid = device_cu_count() * copy_wgs_per_cu();
  if (kv->units_per_block > 1)
    hipLaunchKernelGGL(scatter_slots_kernel, dim3(grid), dim3(kCopyThreads), 0, st, a, patch);
  else
    hipLaunchKernelGGL(scatter_kernel, dim3(grid), dim3(kCopyThreads), 0, st, a, patch);
  return hipGetLastError();
}

hipError_t launch_clear_status(const pipelive_kv *kv, hipStream_t st) {
  hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, dev_state(kv));
  return hipGetLastError();
}

}  // namespace pipelive
