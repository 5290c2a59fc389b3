// ResizeKV with compaction for a block-list KV region (paper Sec. 4.2
// primitive ResizeKV(B), Alg. 1 phases 1, 2 and 5, Sec. 5.1).
//
// plan    : one workgroup scans the live bitmap: n_live, the ascending list T
//           of live ids in the tail [B_new, B) and the ascending list F of
//           free ids in the head [0, B_new) (prefix sums of popcounts), and
//           whether any dirty bit is pending.  It changes nothing.
// check   : every used table entry must be a live id below B.
// commit  : two launches: copy block T[k] -> F[k] in every layer group and
//           build remap[]; then rewrite the tables and move the live bits.  Sources and destinations
//           are disjoint id sets, so the copy needs no ordering.  The commit
//           kernels are queued right behind the plan and read its verdict on
//           the device: a refused resize changes nothing.
#include <string.h>

#include "internal.h"
#include "kv_copy.h"
#include "scan.h"

namespace pipelive {
namespace {

typedef unsigned long long u64;

__device__ __forceinline__ u64 range_mask(int64_t word, int64_t lo, int64_t hi) {
  // bits of 64-bit word `word` whose id lies in [lo, hi)
  const int64_t base = word * 64;
  int64_t a = lo - base, b = hi - base;
  if (a < 0) a = 0;
  if (b > 64) b = 64;
  if (a >= b) return 0;
  const u64 upto_b = b == 64 ? ~0ull : ((1ull << b) - 1ull);
  const u64 upto_a = (1ull << a) - 1ull;  // a < 64 here
  return upto_b & ~upto_a;
}

// The verdict of the plan, evaluated on the device by every commit kernel: they are queued before the
// host has seen it (no idle gap on the stream) and do nothing when the resize is refused.
__device__ __forceinline__ bool plan_ok(const ResizePlanOut *plan, int64_t B_new) {
  return plan->any_dirty == 0 && plan->bad_table == 0 && plan->n_live <= B_new;
}

__global__ __launch_bounds__(kScanThreads) void resize_plan_kernel(
    const u64 *live, const u64 *dirty, int64_t n_dirty_units, int64_t B, int64_t B_new,
    ResizePlanOut *plan, int32_t *move_src, int32_t *move_dst) {
  __shared__ uint32_t sh[17];
  __shared__ uint32_t sh_live[kScanThreads / 64], sh_dirty[kScanThreads / 64];
  const int64_t nwords = (B + 63) / 64;
  const int64_t per = (nwords + kScanThreads - 1) / kScanThreads;
  const int64_t w0 = (int64_t)threadIdx.x * per;
  const int64_t w1 = w0 + per < nwords ? w0 + per : nwords;
  uint32_t cT = 0, cF = 0, cL = 0, anyd = 0;
  for (int64_t w = w0; w < w1; ++w) {
    const u64 in = range_mask(w, 0, B);
    const u64 lv = live[w] & in;
    cL += __popcll(lv);
    cT += __popcll(lv & range_mask(w, B_new, B));
    cF += __popcll(~lv & range_mask(w, 0, B_new < B ? B_new : B));
  }
  for (int64_t w = threadIdx.x; w < (n_dirty_units + 63) / 64; w += kScanThreads)
    anyd |= (dirty[w] & range_mask(w, 0, n_dirty_units)) != 0;
  uint32_t totT, totF;
  const uint32_t exT = wg_exclusive_scan(cT, sh, &totT);
  const uint32_t exF = wg_exclusive_scan(cF, sh, &totF);
  // n_live and any_dirty: wave reduce then LDS
  uint32_t rl = cL;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) rl += __shfl_xor(rl, o);
  const uint32_t rd = __any(anyd) ? 1u : 0u;
  if ((threadIdx.x & 63) == 0) {
    sh_live[threadIdx.x >> 6] = rl;
    sh_dirty[threadIdx.x >> 6] = rd;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long nl = 0, ad = 0;
    for (int i = 0; i < kScanThreads / 64; ++i) {
      nl += sh_live[i];
      ad |= sh_dirty[i];
    }
    plan->n_live = nl;
    plan->n_moved = totT;
    plan->any_dirty = ad;
    plan->bad_table = 0;
  }
  // expand the lists (only meaningful when the shrink is feasible: then |F| >= |T|)
  uint32_t rT = exT, rF = exF;
  for (int64_t w = w0; w < w1; ++w) {
    const u64 lv = live[w] & range_mask(w, 0, B);
    u64 t = lv & range_mask(w, B_new, B);
    while (t) {
      const int b = __ffsll((long long)t) - 1;
      move_src[rT++] = (int32_t)(w * 64 + b);
      t &= t - 1;
    }
    u64 f = ~lv & range_mask(w, 0, B_new < B ? B_new : B);
    while (f && rF < totT) {
      const int b = __ffsll((long long)f) - 1;
      move_dst[rF++] = (int32_t)(w * 64 + b);
      f &= f - 1;
    }
  }
}

__global__ void table_check_kernel(const u64 *live, int64_t B, TableRef t, ResizePlanOut *plan) {
  const int row = blockIdx.x;
  const int used = t.used[row];
  bool bad = used < 0 || used > t.stride;
  if (!bad)
    for (int i = threadIdx.x; i < used; i += blockDim.x) {
      const int32_t e = t.table[(int64_t)row * t.stride + i];
      if (e < 0 || e >= B || !((live[e >> 6] >> (e & 63)) & 1ull)) bad = true;
    }
  if (bad) atomicOr((u64 *)&plan->bad_table, 1ull);
}

// remap[b] for b in [0,B): identity if live and kept, -1 if not live; moved ids are written from the
// move list (disjoint from the first set).  Index i runs over [0, B + n_moved).  Reads the live bitmap
// as it was before the resize: the kernels that call this run before the one that moves the live bits.
struct RemapArgs {
  const u64 *live;
  int64_t B, B_new;
  const int32_t *move_src, *move_dst;
  int32_t *remap;
};
__device__ __forceinline__ void remap_all(const RemapArgs &r, int64_t n_moved) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < r.B + n_moved; i += stride) {
    if (i < r.B) {
      const bool lv = (r.live[i >> 6] >> (i & 63)) & 1ull;
      if (!lv) r.remap[i] = -1;
      else if (i < r.B_new) r.remap[i] = (int32_t)i;
    } else {
      const int64_t k = i - r.B;
      r.remap[r.move_src[k]] = r.move_dst[k];
    }
  }
}

struct MoveArgs {
  const uint64_t *block_list;
  int64_t capacity;
  int32_t groups;
  uint32_t phys_bytes, sub_bytes, subs_per_block;
  const int32_t *move_src, *move_dst;
  const ResizePlanOut *plan;  // n_moved and the verdict
  int64_t B_new;
  RemapArgs remap;
};

// The copies of a shrink; the same launch also writes remap[] (a megabyte next to gigabytes).
__global__ __launch_bounds__(kCopyThreads) void move_kernel(MoveArgs a) {
  if (!plan_ok(a.plan, a.B_new)) return;
  remap_all(a.remap, a.plan->n_moved);
  const int64_t n_items = a.plan->n_moved * a.groups * a.subs_per_block;
  for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const uint32_t sub = (uint32_t)(item % a.subs_per_block);
    const int64_t e = item / a.subs_per_block;
    const int32_t grp = (int32_t)(e % a.groups);
    const int64_t k = e / a.groups;
    const uint64_t *bl = a.block_list + (int64_t)grp * a.capacity;
    const char *src = (const char *)bl[a.move_src[k]];
    char *dst = (char *)bl[a.move_dst[k]];
    const uint32_t off = sub * a.sub_bytes;
    const uint32_t len = a.phys_bytes - off < a.sub_bytes ? a.phys_bytes - off : a.sub_bytes;
    wg_copy(dst + off, src + off, len);
  }
}

// Per-block backing: a move exchanges the two block_list entries of every
// group instead of copying bytes (the sets of sources and targets are
// disjoint, so the exchanges are independent).  Writes remap[] as well.
__global__ void swap_kernel(uint64_t *block_list, int64_t capacity, int32_t groups,
                            const ResizePlanOut *plan, RemapArgs r) {
  if (!plan_ok(plan, r.B_new)) return;
  const int64_t n_moved = plan->n_moved;
  remap_all(r, n_moved);
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n_moved * groups; i += stride) {
    uint64_t *bl = block_list + (i % groups) * capacity;
    const int64_t k = i / groups;
    const uint64_t a = bl[r.move_src[k]], b = bl[r.move_dst[k]];
    bl[r.move_src[k]] = b;
    bl[r.move_dst[k]] = a;
  }
}

// Last kernel of a shrink: every used table entry follows remap[] (one workgroup per table row, all
// tables in one launch), and the workgroups behind them move the live bits of the moved ids.
struct FinishArgs {
  TableRef t[PIPELIVE_MAX_TABLES];
  int32_t row_end[PIPELIVE_MAX_TABLES];  // running sum of the tables' rows
  int32_t n_tables, total_rows;
  const int32_t *remap;
  const ResizePlanOut *plan;
  int64_t B_new;
  u64 *live;
  const int32_t *move_src, *move_dst;
};
__global__ __launch_bounds__(256) void finish_kernel(FinishArgs a) {
  if (!plan_ok(a.plan, a.B_new)) return;
  if ((int)blockIdx.x < a.total_rows) {
    int ti = 0;
    while (ti + 1 < a.n_tables && (int)blockIdx.x >= a.row_end[ti]) ++ti;
    const TableRef &t = a.t[ti];
    const int row = (int)blockIdx.x - (ti ? a.row_end[ti - 1] : 0);
    const int used = t.used[row];
    for (int i = threadIdx.x; i < used; i += blockDim.x) {
      int32_t *e = &t.table[(int64_t)row * t.stride + i];
      *e = a.remap[*e];
    }
  } else {
    const int64_t k = (int64_t)((int)blockIdx.x - a.total_rows) * blockDim.x + threadIdx.x;
    if (k < a.plan->n_moved) {
      const int32_t s = a.move_src[k], d = a.move_dst[k];
      atomicAnd(&a.live[s >> 6], ~(1ull << (s & 63)));
      atomicOr(&a.live[d >> 6], 1ull << (d & 63));
    }
  }
}

// grow: ids [B, B_new) become valid and are neither live nor dirty
__global__ void grow_kernel(u64 *live, u64 *dirty, int64_t B, int64_t B_new, int64_t upb,
                            int32_t *remap, const ResizePlanOut *plan) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (!plan_ok(plan, B_new)) return;
  const int64_t w_lo = B / 64, w_hi = (B_new + 63) / 64;
  if (i < w_hi - w_lo) atomicAnd(&live[w_lo + i], ~range_mask(w_lo + i, B, B_new));
  const int64_t d_lo = B * upb / 64, d_hi = (B_new * upb + 63) / 64;  // dirty units of the new ids
  if (i < d_hi - d_lo) atomicAnd(&dirty[d_lo + i], ~range_mask(d_lo + i, B * upb, B_new * upb));
  if (remap && i < B) remap[i] = ((live[i >> 6] >> (i & 63)) & 1ull) ? (int32_t)i : -1;
}

}  // namespace

hipError_t launch_resize_plan(const pipelive_kv *kv, int64_t B, int64_t B_new, ResizePlanOut *plan,
                              int32_t *move_src, int32_t *move_dst, hipStream_t st) {
  hipLaunchKernelGGL(resize_plan_kernel, dim3(1), dim3(kScanThreads), 0, st,
                     (const u64 *)kv->d.live_bitmap, (const u64 *)kv->d.dirty_bitmap,
                     B * kv->units_per_block, B, B_new, plan, move_src, move_dst);
  return hipGetLastError();
}

hipError_t launch_table_check(const pipelive_kv *kv, int64_t B, const TableRef &t,
                              ResizePlanOut *plan, hipStream_t st) {
  if (t.rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(table_check_kernel, dim3(t.rows), dim3(256), 0, st,
                     (const u64 *)kv->d.live_bitmap, B, t, plan);
  return hipGetLastError();
}

hipError_t launch_resize_commit(const pipelive_kv *kv, int64_t B, int64_t B_new,
                                const ResizePlanOut *plan, const int32_t *move_src,
                                const int32_t *move_dst, int32_t *remap, const TableRef *tables,
                                int n_tables, hipStream_t st) {
  // Two launches, sized for the most a shrink can move (B - B_new blocks; the count itself is read
  // from the plan on the device): the moves with remap[], then the tables with the live bits.
  hipError_t e;
  const int64_t max_moved = B - B_new;
  if (max_moved <= 0) return hipSuccess;
  RemapArgs r;
  r.live = (const u64 *)kv->d.live_bitmap;
  r.B = B;
  r.B_new = B_new;
  r.move_src = move_src;
  r.move_dst = move_dst;
  r.remap = remap;
  if (kv->d.block_backing == PIPELIVE_BACKING_PER_BLOCK) {
    const int64_t n = B + max_moved;  // remap entries: the larger of the two index spaces
    hipLaunchKernelGGL(swap_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       const_cast<uint64_t *>(kv->d.block_list), kv->d.capacity_blocks,
                       (int32_t)kv->groups, plan, r);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  } else {
    MoveArgs a;
    a.block_list = kv->d.block_list;
    a.capacity = kv->d.capacity_blocks;
    a.groups = (int32_t)kv->groups;
    a.phys_bytes = (uint32_t)kv->phys_bytes;
    a.sub_bytes = kCopyChunk;
    a.subs_per_block = (a.phys_bytes + a.sub_bytes - 1) / a.sub_bytes;
    a.move_src = move_src;
    a.move_dst = move_dst;
    a.plan = plan;
    a.B_new = B_new;
    a.remap = r;
    const int64_t max_items = max_moved * kv->groups * a.subs_per_block;
    const int64_t max_grid = (int64_t)device_cu_count() * copy_wgs_per_cu();
    const int grid = (int)(max_items < max_grid ? max_items : max_grid);
    hipLaunchKernelGGL(move_kernel, dim3(grid), dim3(kCopyThreads), 0, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  FinishArgs f;
  memset(&f, 0, sizeof f);
  int rows = 0;
  for (int t = 0; t < n_tables; ++t) {
    if (tables[t].rows <= 0) continue;
    f.t[f.n_tables] = tables[t];
    rows += tables[t].rows;
    f.row_end[f.n_tables] = rows;
    ++f.n_tables;
  }
  f.total_rows = rows;
  f.remap = remap;
  f.plan = plan;
  f.B_new = B_new;
  f.live = (u64 *)kv->d.live_bitmap;
  f.move_src = move_src;
  f.move_dst = move_dst;
  const int64_t grid = rows + (max_moved + 255) / 256;
  hipLaunchKernelGGL(finish_kernel, dim3((unsigned)grid), dim3(256), 0, st, f);
  return hipGetLastError();
}

hipError_t launch_grow(const pipelive_kv *kv, int64_t B, int64_t B_new, int32_t *remap,
                       const ResizePlanOut *plan, hipStream_t st) {
  const int64_t upb = kv->units_per_block;
  const int64_t words = (B_new * upb + 63) / 64 - B * upb / 64 + 1;
  const int64_t n = words > B ? words : B;
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(grow_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     (u64 *)kv->d.live_bitmap, (u64 *)kv->d.dirty_bitmap, B, B_new, upb, remap, plan);
  return hipGetLastError();
}

}  // namespace pipelive
