/*
 * CPU oracle for the PipeLive single-GPU hot path.  TEST INFRASTRUCTURE ONLY:
 * it is imported by the tests, the smoke check and the bench's cpu_baseline
 * leg, never by the product path, and it shares no code with the HIP library.
 *
 * Plain C, double precision, one obvious loop per definition:
 *   - paged decode attention == softmax attention over the KV gathered through
 *     the block table (paper Sec. 2 "LLM Inference": decode reads the cached
 *     keys/values; Sec. 5.1: blocks are reached through a block list of
 *     independently placed blocks and a block table);
 *   - ResizeKV / compaction as a state transformation (Sec. 4.2 primitive
 *     ResizeKV(B), Alg. 1 phase 1 feasibility test and phase 2, Sec. 5.1);
 *   - dirty bitmap, atomic drain, gather into a KV patch, apply on the target,
 *     token counters (Sec. 6.1 "KV Migration with KV Patch"; the n_acc counter
 *     follows the appendix remark on bitmap de-duplication).
 *
 * The only concurrency is an optional OpenMP "parallel for" over independent
 * outer iterations (sequence x head, or block); the arithmetic per output is
 * untouched by it.
 *
 * Pins (tests/test_oracle_*.py, all CPU): attention against textbook dense
 * softmax attention on KV scattered by a test-local routine, closed forms
 * (n=1, equal keys, constant values, dominant key), brute-force resize on all
 * subsets of an 8-block pool, patch invariants (popcount, ascending ids,
 * idempotent apply, conservation of marks and of n_acc, final equality).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum {
  ORC_OK = 0,
  ORC_E_INVAL = -1,
  ORC_E_INFEASIBLE = -2,
  ORC_E_NOSPACE = -3,
  ORC_E_BUSY = -4,
  ORC_E_RANGE = -5
};

/* A KV region on the host.  block_list holds HOST addresses. */
typedef struct {
  int32_t num_layers, num_q_heads, num_kv_heads, head_dim;
  int32_t block_tokens, stack_k, layout;
  int32_t dirty_gran;    /* dirty-tracking unit: 0 = block, 1 = token slot */
  int64_t num_blocks, capacity_blocks;
  uint64_t *block_list;  /* [ceil(L/stack_k)][capacity_blocks] */
  uint8_t *live_bitmap;  /* bit i: byte i>>3, bit i&7 */
  uint8_t *dirty_bitmap;
  uint64_t n_acc;        /* tokens marked since the last complete drain */
  uint64_t t_applied;    /* tokens acknowledged by applied patches */
  int32_t per_block;     /* 1: every physical block is an allocation of its own, so a shrink
                            exchanges block-list entries instead of copying (Sec. 5.1) */
  int32_t pad_;
} orc_kv_t;

typedef struct {
  uint32_t magic, version, n_blocks, n_layers;
  uint64_t block_bytes, n_acc_tokens, payload_offset;
  uint32_t max_blocks, more_pending;
  uint32_t unit_tokens; /* tokens per patch unit: block_tokens, or 1 for slot granularity */
  uint8_t pad[12];
} orc_patch_hdr_t;

#define ORC_PATCH_MAGIC 0x564B4C50u /* bytes 'P','L','K','V' */
#define ORC_PATCH_VERSION 1u

static int get_bit(const uint8_t *bm, int64_t i) { return (bm[i >> 3] >> (i & 7)) & 1; }
static void set_bit(uint8_t *bm, int64_t i) { bm[i >> 3] |= (uint8_t)(1u << (i & 7)); }
static void clr_bit(uint8_t *bm, int64_t i) { bm[i >> 3] &= (uint8_t)~(1u << (i & 7)); }

static double bf16_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* bytes of one (layer, block): K and V, all KV heads, bf16 */
static uint64_t blk_bytes(const orc_kv_t *kv) {
  return (uint64_t)2 * kv->num_kv_heads * kv->block_tokens * kv->head_dim * 2;
}

/* dirty-tracking units: one per block, or one per token slot (the granularity
 * of the paper's bitmap, Sec. 6.1) */
static int64_t unit_tokens(const orc_kv_t *kv) { return kv->dirty_gran ? 1 : kv->block_tokens; }
static int64_t num_units(const orc_kv_t *kv) {
  return kv->num_blocks * (kv->dirty_gran ? kv->block_tokens : 1);
}
/* bytes one unit contributes to a patch, per layer */
static uint64_t unit_bytes(const orc_kv_t *kv) {
  return kv->dirty_gran ? (uint64_t)2 * kv->num_kv_heads * kv->head_dim * 2 : blk_bytes(kv);
}

static int64_t num_groups(const orc_kv_t *kv) {
  return (kv->num_layers + kv->stack_k - 1) / kv->stack_k;
}

/* address of layer `layer`'s part of physical block `id` */
static uint8_t *layer_block(const orc_kv_t *kv, int layer, int64_t id) {
  uint64_t base = kv->block_list[(int64_t)(layer / kv->stack_k) * kv->capacity_blocks + id];
  return (uint8_t *)(uintptr_t)base + (uint64_t)(layer % kv->stack_k) * blk_bytes(kv);
}

/* element index (in bf16 units from the start of the layer's block) of
 * K[g][t][d] and V[g][t][d], for the two in-block layouts:
 *   layout 0: the block is a sequence of sub-blocks of sb = min(bs, 32)
 *             tokens; sub-block u holds tokens u*sb .. u*sb+sb-1 as
 *             K[Hkv][D/8][sb][8] then V[Hkv][D][sb]
 *   layout 1: K[Hkv][bs][D] then V[Hkv][bs][D]                          */
static int64_t k_elem(const orc_kv_t *kv, int g, int t, int d) {
  int64_t bs = kv->block_tokens, D = kv->head_dim;
  if (kv->layout == 0) {
    int64_t sb = bs < 32 ? bs : 32, u = t / sb, tt = t % sb;
    int64_t sub = u * (2 * (int64_t)kv->num_kv_heads * sb * D);
    return sub + (((int64_t)g * (D / 8) + d / 8) * sb + tt) * 8 + d % 8;
  }
  return ((int64_t)g * bs + t) * D + d;
}
static int64_t v_elem(const orc_kv_t *kv, int g, int t, int d) {
  int64_t bs = kv->block_tokens, D = kv->head_dim;
  if (kv->layout == 0) {
    int64_t sb = bs < 32 ? bs : 32, u = t / sb, tt = t % sb;
    int64_t sub = u * (2 * (int64_t)kv->num_kv_heads * sb * D);
    return sub + (int64_t)kv->num_kv_heads * sb * D + ((int64_t)g * D + d) * sb + tt;
  }
  return (int64_t)kv->num_kv_heads * bs * D + ((int64_t)g * bs + t) * D + d;
}

int32_t orc_struct_bytes(void) { return (int32_t)sizeof(orc_kv_t); }

/* ---------------------------------------------------------------- attention
 * For sequence s with n cached tokens and query head h (KV head g = h / G):
 *   x_j = scale * <q_h, K_j>,  p_j = exp(x_j - max x),  out = sum p_j V_j / sum p_j
 * over j = 0..n-1 where token j lives in block table[s][j / bs], slot j % bs.
 * No mask: the decode token attends to every cached token.  n == 0 -> zeros. */
int32_t orc_paged_attn_decode(const orc_kv_t *kv, int32_t layer, const uint16_t *q, float *out,
                              const int32_t *table, int32_t table_stride, const int32_t *ctx_lens,
                              int32_t num_seqs, double scale, int32_t nthreads) {
  if (!kv || layer < 0 || layer >= kv->num_layers || num_seqs < 0) return ORC_E_INVAL;
  const int Hq = kv->num_q_heads, Hkv = kv->num_kv_heads, D = kv->head_dim, bs = kv->block_tokens;
  const int G = Hq / Hkv;
  if (scale <= 0) scale = 1.0 / sqrt((double)D);
  int rc = ORC_OK;
  /* validate ids first so the parallel loop never dereferences a bad one */
  for (int s = 0; s < num_seqs; ++s) {
    int n = ctx_lens[s];
    if (n < 0 || (int64_t)(n + bs - 1) / bs > table_stride) return ORC_E_INVAL;
    for (int b = 0; b < (n + bs - 1) / bs; ++b) {
      int32_t id = table[(int64_t)s * table_stride + b];
      if (id < 0 || id >= kv->num_blocks) return ORC_E_RANGE;
    }
  }
#ifdef _OPENMP
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
#endif
  for (int sh = 0; sh < num_seqs * Hq; ++sh) {
    int s = sh / Hq, h = sh % Hq, g = h / G;
    int n = ctx_lens[s];
    float *o = out + ((int64_t)s * Hq + h) * D;
    if (n == 0) {
      for (int d = 0; d < D; ++d) o[d] = 0.0f;
      continue;
    }
    const uint16_t *qh = q + ((int64_t)s * Hq + h) * D;
    double *x = (double *)malloc(sizeof(double) * (size_t)n);
    double *num = (double *)calloc((size_t)D, sizeof(double));
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
      const uint16_t *blk =
          (const uint16_t *)layer_block(kv, layer, table[(int64_t)s * table_stride + j / bs]);
      int t = j % bs;
      double acc = 0.0;
      for (int d = 0; d < D; ++d) acc += bf16_to_double(qh[d]) * bf16_to_double(blk[k_elem(kv, g, t, d)]);
      x[j] = scale * acc;
      if (x[j] > m) m = x[j];
    }
    double den = 0.0;
    for (int j = 0; j < n; ++j) {
      const uint16_t *blk =
          (const uint16_t *)layer_block(kv, layer, table[(int64_t)s * table_stride + j / bs]);
      int t = j % bs;
      double p = exp(x[j] - m);
      den += p;
      for (int d = 0; d < D; ++d) num[d] += p * bf16_to_double(blk[v_elem(kv, g, t, d)]);
    }
    for (int d = 0; d < D; ++d) o[d] = (float)(num[d] / den);
    free(x);
    free(num);
  }
  return rc;
}

/* ------------------------------------------------------------------- resize
 * Shrink to B_new < B:
 *   n_live > B_new            -> INFEASIBLE, nothing changes (Alg. 1 phase 1)
 *   any dirty bit set         -> BUSY, nothing changes (primitives are issued
 *                                sequentially: resize precedes migration and
 *                                follows the commit)
 *   T = ascending live ids in [B_new, B); F = ascending free ids in [0, B_new);
 *   block T[k] moves to F[k] in every layer; remap[T[k]] = F[k]; other live
 *   ids map to themselves; non-live ids map to -1; every used table entry e
 *   becomes remap[e]; live bits follow the blocks; B <- B_new.
 * With independently allocated blocks (per_block) the move of T[k] to F[k]
 * is the exchange of the two block-list entries in every layer group: id
 * F[k] then names the physical block T[k] named, no byte is copied, and the
 * free physical blocks collect at the ids >= B_new (Sec. 5.1: compaction
 * moves the unallocated blocks to the end of the list by pointer updates).
 * Grow to B_new > B (<= capacity): B <- B_new, new ids not live, no data
 * moves (Sec. 5.1: expansion appends blocks to the block list).
 * result[0..3] = n_live, n_moved, old B, new B. */
int32_t orc_kv_resize(orc_kv_t *kv, int64_t new_num_blocks, int32_t **tables,
                      const int32_t *table_rows, const int32_t *table_strides,
                      const int32_t **table_used, int32_t num_tables, int32_t *remap_out,
                      int64_t *result) {
  if (!kv || new_num_blocks < 0) return ORC_E_INVAL;
  const int64_t B = kv->num_blocks;
  int64_t n_live = 0;
  for (int64_t b = 0; b < B; ++b) n_live += get_bit(kv->live_bitmap, b);
  if (result) {
    result[0] = n_live; result[1] = 0; result[2] = B; result[3] = B;
  }
  if (new_num_blocks > kv->capacity_blocks) return ORC_E_NOSPACE;
  for (int64_t u = 0; u < num_units(kv); ++u)
    if (get_bit(kv->dirty_bitmap, u)) return ORC_E_BUSY;
  if (n_live > new_num_blocks) return ORC_E_INFEASIBLE;
  for (int t = 0; t < num_tables; ++t)
    for (int r = 0; r < table_rows[t]; ++r)
      for (int i = 0; i < table_used[t][r]; ++i) {
        int32_t e = tables[t][(int64_t)r * table_strides[t] + i];
        if (e < 0 || e >= B || !get_bit(kv->live_bitmap, e)) return ORC_E_RANGE;
      }

  int32_t *remap = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B > 0 ? B : 1));
  for (int64_t b = 0; b < B; ++b) remap[b] = get_bit(kv->live_bitmap, b) ? (int32_t)b : -1;
  int64_t n_moved = 0;
  if (new_num_blocks < B) {
    const uint64_t bytes = blk_bytes(kv) * (uint64_t)kv->stack_k; /* a physical block */
    int64_t f = 0; /* next candidate hole in the head */
    for (int64_t t = new_num_blocks; t < B; ++t) {
      if (!get_bit(kv->live_bitmap, t)) continue;
      while (get_bit(kv->live_bitmap, f)) ++f; /* f < new_num_blocks since n_live <= B_new */
      for (int64_t grp = 0; grp < num_groups(kv); ++grp) {
        uint64_t *et = &kv->block_list[grp * kv->capacity_blocks + t];
        uint64_t *ef = &kv->block_list[grp * kv->capacity_blocks + f];
        if (kv->per_block) {
          uint64_t tmp = *et;
          *et = *ef;
          *ef = tmp;
        } else {
          memcpy((uint8_t *)(uintptr_t)*ef, (const uint8_t *)(uintptr_t)*et, bytes);
        }
      }
      remap[t] = (int32_t)f;
      set_bit(kv->live_bitmap, f);
      clr_bit(kv->live_bitmap, t);
      ++n_moved;
    }
  } else {
    const int64_t ut = kv->dirty_gran ? kv->block_tokens : 1;
    for (int64_t b = B; b < new_num_blocks; ++b) clr_bit(kv->live_bitmap, b);
    for (int64_t u = B * ut; u < new_num_blocks * ut; ++u) clr_bit(kv->dirty_bitmap, u);
  }
  for (int t = 0; t < num_tables; ++t)
    for (int r = 0; r < table_rows[t]; ++r)
      for (int i = 0; i < table_used[t][r]; ++i) {
        int32_t *e = &tables[t][(int64_t)r * table_strides[t] + i];
        *e = remap[*e];
      }
  if (remap_out) memcpy(remap_out, remap, sizeof(int32_t) * (size_t)B);
  free(remap);
  kv->num_blocks = new_num_blocks;
  if (result) { result[1] = n_moved; result[3] = new_num_blocks; }
  return ORC_OK;
}

/* ----------------------------------------------------------------- patching
 * mark: B[s] <- 1 for every written block; n_acc += n_tokens. */
int32_t orc_kv_mark_dirty(orc_kv_t *kv, const int32_t *ids, int32_t n, int64_t n_tokens) {
  if (!kv || n < 0 || n_tokens < 0) return ORC_E_INVAL;
  for (int i = 0; i < n; ++i)
    if (ids[i] < 0 || ids[i] >= num_units(kv)) return ORC_E_RANGE;
  for (int i = 0; i < n; ++i) set_bit(kv->dirty_bitmap, ids[i]);
  kv->n_acc += (uint64_t)n_tokens;
  return ORC_OK;
}

static uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

/* largest number of blocks a patch buffer of `capacity` bytes can carry */
int64_t orc_patch_max_blocks(const orc_kv_t *kv, int32_t n_layers, uint64_t capacity) {
  if (capacity < 64 + 256) return 0;
  uint64_t per = 4 + (uint64_t)n_layers * unit_bytes(kv);
  uint64_t mb = (capacity - 64 - 256) / per;
  if (mb > (uint64_t)num_units(kv)) mb = (uint64_t)num_units(kv);
  return (int64_t)mb;
}

/* drain + gather: D = ascending ids with the bit set, clipped to max_blocks;
 * exactly those bits are cleared; patch = header | ids[max_blocks] | pad to
 * 256 | payload[r][i] = bytes of block D[r] in layer layers[i].
 * n_acc travels (and is reset) only when the drain empties the bitmap. */
int32_t orc_kv_patch_collect(orc_kv_t *kv, const int32_t *layers, int32_t n_layers,
                             uint8_t *patch, uint64_t capacity) {
  if (!kv || n_layers <= 0 || !patch) return ORC_E_INVAL;
  for (int i = 0; i < n_layers; ++i)
    if (layers[i] < 0 || layers[i] >= kv->num_layers) return ORC_E_RANGE;
  int64_t max_blocks = orc_patch_max_blocks(kv, n_layers, capacity);
  if (max_blocks <= 0) return ORC_E_NOSPACE;
  const uint64_t bb = unit_bytes(kv);
  orc_patch_hdr_t h;
  memset(&h, 0, sizeof h);
  h.magic = ORC_PATCH_MAGIC;
  h.version = ORC_PATCH_VERSION;
  h.n_layers = (uint32_t)n_layers;
  h.block_bytes = bb;
  h.unit_tokens = (uint32_t)unit_tokens(kv);
  h.max_blocks = (uint32_t)max_blocks;
  h.payload_offset = round_up(64 + 4 * (uint64_t)max_blocks, 256);
  int32_t *ids = (int32_t *)(patch + 64);
  uint8_t *payload = patch + h.payload_offset;
  uint32_t n = 0;
  int more = 0;
  for (int64_t u = 0; u < num_units(kv); ++u) {
    if (!get_bit(kv->dirty_bitmap, u)) continue;
    if ((int64_t)n == max_blocks) { more = 1; break; }
    clr_bit(kv->dirty_bitmap, u);
    ids[n] = (int32_t)u;
    for (int i = 0; i < n_layers; ++i) {
      uint8_t *dst = payload + ((uint64_t)n * n_layers + i) * bb;
      if (!kv->dirty_gran) {
        memcpy(dst, layer_block(kv, layers[i], u), bb);
      } else { /* one token: K[Hkv][D] then V[Hkv][D], gathered out of the block layout */
        const uint16_t *blk = (const uint16_t *)layer_block(kv, layers[i], u / kv->block_tokens);
        uint16_t *o = (uint16_t *)dst;
        const int t = (int)(u % kv->block_tokens), Hkv = kv->num_kv_heads, D = kv->head_dim;
        for (int g = 0; g < Hkv; ++g)
          for (int d = 0; d < D; ++d) {
            o[g * D + d] = blk[k_elem(kv, g, t, d)];
            o[Hkv * D + g * D + d] = blk[v_elem(kv, g, t, d)];
          }
      }
    }
    ++n;
  }
  h.n_blocks = n;
  h.more_pending = (uint32_t)more;
  if (!more) { h.n_acc_tokens = kv->n_acc; kv->n_acc = 0; }
  memcpy(patch, &h, sizeof h);
  return ORC_OK;
}

/* receiver: write every patch entry into block dst_map[id] (identity when
 * dst_map is NULL) of layer dst_layers[i]; T_applied += n_acc. */
int32_t orc_kv_patch_apply(orc_kv_t *dst, const int32_t *dst_layers, int32_t n_layers,
                           const uint8_t *patch, const int32_t *dst_map) {
  if (!dst || !patch || n_layers <= 0) return ORC_E_INVAL;
  orc_patch_hdr_t h;
  memcpy(&h, patch, sizeof h);
  if (h.magic != ORC_PATCH_MAGIC || h.version != ORC_PATCH_VERSION) return ORC_E_INVAL;
  if (h.n_layers != (uint32_t)n_layers || h.block_bytes != unit_bytes(dst)) return ORC_E_INVAL;
  if (h.unit_tokens != (uint32_t)unit_tokens(dst)) return ORC_E_INVAL;
  for (int i = 0; i < n_layers; ++i)
    if (dst_layers[i] < 0 || dst_layers[i] >= dst->num_layers) return ORC_E_RANGE;
  const int32_t *ids = (const int32_t *)(patch + 64);
  const int64_t upb = dst->dirty_gran ? dst->block_tokens : 1; /* units per block */
  for (uint32_t r = 0; r < h.n_blocks; ++r) {
    int64_t blk_id = ids[r] / upb;
    if (dst_map) blk_id = dst_map[blk_id];
    if (blk_id < 0 || blk_id >= dst->num_blocks) return ORC_E_RANGE;
  }
  const uint8_t *payload = patch + h.payload_offset;
  for (uint32_t r = 0; r < h.n_blocks; ++r) {
    int64_t blk_id = ids[r] / upb;
    if (dst_map) blk_id = dst_map[blk_id];
    for (int i = 0; i < n_layers; ++i) {
      const uint8_t *src = payload + ((uint64_t)r * n_layers + i) * h.block_bytes;
      if (!dst->dirty_gran) {
        memcpy(layer_block(dst, dst_layers[i], blk_id), src, h.block_bytes);
      } else {
        uint16_t *blk = (uint16_t *)layer_block(dst, dst_layers[i], blk_id);
        const uint16_t *o = (const uint16_t *)src;
        const int t = (int)(ids[r] % upb), Hkv = dst->num_kv_heads, D = dst->head_dim;
        for (int g = 0; g < Hkv; ++g)
          for (int d = 0; d < D; ++d) {
            blk[k_elem(dst, g, t, d)] = o[g * D + d];
            blk[v_elem(dst, g, t, d)] = o[Hkv * D + g * D + d];
          }
      }
    }
  }
  dst->t_applied += h.n_acc_tokens;
  return ORC_OK;
}

/* -------------------------------------------------------------------- append
 * The write side of a decode step for one layer (Sec. 6.1: the inference side
 * flags the slots a step wrote): token `positions[s]`
 * of sequence s gets K/V k_new[s], v_new[s] ([Hkv][D] each) in block
 * table[s][pos / bs], slot pos % bs.  positions[s] < 0 skips the sequence.
 * mark != 0 sets the dirty bit of the written unit; count_tokens != 0 adds the
 * number of written tokens to n_acc (done for one layer per step: n^(t) counts
 * tokens, not layer writes). */
int32_t orc_kv_append(orc_kv_t *kv, int32_t layer, const uint16_t *k_new, const uint16_t *v_new,
                      const int32_t *table, int32_t table_stride, const int32_t *positions,
                      int32_t num_seqs, int32_t mark, int32_t count_tokens) {
  if (!kv || layer < 0 || layer >= kv->num_layers) return ORC_E_INVAL;
  const int Hkv = kv->num_kv_heads, D = kv->head_dim, bs = kv->block_tokens;
  for (int s = 0; s < num_seqs; ++s) {
    if (positions[s] < 0) continue;
    if (positions[s] / bs >= table_stride) return ORC_E_INVAL;
    int32_t id = table[(int64_t)s * table_stride + positions[s] / bs];
    if (id < 0 || id >= kv->num_blocks) return ORC_E_RANGE;
  }
  uint64_t written = 0;
  for (int s = 0; s < num_seqs; ++s) {
    const int pos = positions[s];
    if (pos < 0) continue;
    const int32_t id = table[(int64_t)s * table_stride + pos / bs];
    const int t = pos % bs;
    uint16_t *blk = (uint16_t *)layer_block(kv, layer, id);
    for (int g = 0; g < Hkv; ++g)
      for (int d = 0; d < D; ++d) {
        blk[k_elem(kv, g, t, d)] = k_new[((int64_t)s * Hkv + g) * D + d];
        blk[v_elem(kv, g, t, d)] = v_new[((int64_t)s * Hkv + g) * D + d];
      }
    if (mark) set_bit(kv->dirty_bitmap, kv->dirty_gran ? (int64_t)id * bs + t : id);
    ++written;
  }
  if (count_tokens) kv->n_acc += written;
  return ORC_OK;
}

/* The write side of a prefill chunk for one layer: sequence s holds ctx[s]
 * tokens including the chunk; its q_len = q_offsets[s+1] - q_offsets[s] new
 * tokens (rows q_offsets[s] .. of k_new / v_new, each [Hkv][D]) take the
 * positions ctx[s] - q_len .. ctx[s] - 1, one after the other, exactly as
 * q_len single-token appends would place them.  A chunk longer than its
 * context, a position beyond the table row or a bad block id is an error and
 * nothing is written. */
int32_t orc_kv_append_chunk(orc_kv_t *kv, int32_t layer, const uint16_t *k_new, const uint16_t *v_new,
                            const int32_t *table, int32_t table_stride, const int32_t *ctx,
                            const int32_t *q_offsets, int32_t num_seqs, int32_t mark,
                            int32_t count_tokens) {
  if (!kv || layer < 0 || layer >= kv->num_layers) return ORC_E_INVAL;
  const int Hkv = kv->num_kv_heads, D = kv->head_dim, bs = kv->block_tokens;
  for (int s = 0; s < num_seqs; ++s) {
    const int ql = q_offsets[s + 1] - q_offsets[s];
    if (ql < 0 || ql > ctx[s]) return ORC_E_INVAL;
    for (int i = 0; i < ql; ++i) {
      const int pos = ctx[s] - ql + i;
      if (pos / bs >= table_stride) return ORC_E_INVAL;
      int32_t id = table[(int64_t)s * table_stride + pos / bs];
      if (id < 0 || id >= kv->num_blocks) return ORC_E_RANGE;
    }
  }
  uint64_t written = 0;
  for (int s = 0; s < num_seqs; ++s) {
    const int ql = q_offsets[s + 1] - q_offsets[s];
    for (int i = 0; i < ql; ++i) {
      const int pos = ctx[s] - ql + i;
      const int64_t row = (int64_t)q_offsets[s] + i;
      const int32_t id = table[(int64_t)s * table_stride + pos / bs];
      const int t = pos % bs;
      uint16_t *blk = (uint16_t *)layer_block(kv, layer, id);
      for (int g = 0; g < Hkv; ++g)
        for (int d = 0; d < D; ++d) {
          blk[k_elem(kv, g, t, d)] = k_new[(row * Hkv + g) * D + d];
          blk[v_elem(kv, g, t, d)] = v_new[(row * Hkv + g) * D + d];
        }
      if (mark) set_bit(kv->dirty_bitmap, kv->dirty_gran ? (int64_t)id * bs + t : id);
      ++written;
    }
  }
  if (count_tokens) kv->n_acc += written;
  return ORC_OK;
}

/* MaxBlocks(i, L) = floor((M_i * u - L * W) / (L * P))  (Alg. 1, function MaxBlocks) */
int64_t orc_max_blocks(double mem_bytes, double util, int64_t layers, double weight_bytes_per_layer,
                       double block_bytes_per_layer) {
  if (layers <= 0 || block_bytes_per_layer <= 0) return 0;
  double v = (mem_bytes * util - (double)layers * weight_bytes_per_layer) /
             ((double)layers * block_bytes_per_layer);
  return v < 0 ? 0 : (int64_t)floor(v);
}

/* Effective KV utilisation (Sec. 7.5): tokens held / token slots of the blocks
 * the sequences occupy, a sequence of n tokens occupying ceil(n / bs) blocks. */
double orc_kv_utilization(const int32_t *ctx_lens, int64_t n, int32_t block_tokens) {
  double tokens = 0.0, slots = 0.0;
  for (int64_t s = 0; s < n; ++s) {
    if (ctx_lens[s] <= 0) continue;
    int64_t blocks = 0;
    while (blocks * block_tokens < ctx_lens[s]) ++blocks;
    tokens += (double)ctx_lens[s];
    slots += (double)(blocks * block_tokens);
  }
  return slots > 0.0 ? tokens / slots : 1.0;
}

/* Tokens per layer in a physical block of `phys_bytes` shared by k layers (Sec. 5.2: C / k). */
int64_t orc_stacked_block_tokens(uint64_t phys_bytes, int32_t k, uint64_t token_bytes_per_layer) {
  int64_t t = 0;
  while ((uint64_t)(t + 1) * (uint64_t)k * token_bytes_per_layer <= phys_bytes) ++t;
  return t;
}

/* ------------------------------------------------------------------ planner
 * Alg. 1, written with explicit layer sets (one byte per layer per GPU):
 *   C_tmp[i] = C_cur[i] U C_tgt[i]; B_shrink = min_i MaxBlocks(i, |C_tmp[i]|);
 *   feasible iff B_used <= B_shrink; M_add(i) = C_tgt[i] \ C_cur[i];
 *   M_mig[src][dst] gets every layer of M_add(dst) from its owner in C_cur;
 *   M_del(i) = C_tmp[i] \ C_tgt[i]; B_new = min_i MaxBlocks(i, |C_tgt[i]|).
 * cur/tgt: [num_gpus][num_layers] membership flags (layer ids 0..num_layers-1).
 * Outputs: tmp [N][L] flags; mig [N][N][L] flags; del [N][L] flags;
 * scalars[0..3] = feasible, need_shrink, B_shrink, B_new.  Returns 0, or
 * ORC_E_RANGE when a target layer has no current owner. */
int32_t orc_plan_reconfig(int32_t num_gpus, int32_t num_layers, const uint8_t *cur, const uint8_t *tgt,
                          const double *mem_bytes, double util, double weight_bytes_per_layer,
                          double block_bytes_per_layer, int64_t blocks_in_use, int64_t cur_blocks,
                          uint8_t *tmp, uint8_t *mig, uint8_t *del, int64_t *scalars) {
  const int N = num_gpus, L = num_layers;
  int64_t b_shrink = -1, b_new = -1;
  memset(mig, 0, (size_t)N * N * L);
  for (int i = 0; i < N; ++i) {
    int n_tmp = 0, n_tgt = 0;
    for (int l = 0; l < L; ++l) {
      tmp[i * L + l] = (uint8_t)(cur[i * L + l] || tgt[i * L + l]);
      del[i * L + l] = (uint8_t)(tmp[i * L + l] && !tgt[i * L + l]);
      n_tmp += tmp[i * L + l];
      n_tgt += tgt[i * L + l];
    }
    if (n_tmp > 0) {
      int64_t b = orc_max_blocks(mem_bytes[i], util, n_tmp, weight_bytes_per_layer, block_bytes_per_layer);
      if (b_shrink < 0 || b < b_shrink) b_shrink = b;
    }
    if (n_tgt > 0) {
      int64_t b = orc_max_blocks(mem_bytes[i], util, n_tgt, weight_bytes_per_layer, block_bytes_per_layer);
      if (b_new < 0 || b < b_new) b_new = b;
    }
  }
  if (b_shrink < 0) b_shrink = 0;
  if (b_new < 0) b_new = 0;
  for (int dst = 0; dst < N; ++dst)
    for (int l = 0; l < L; ++l) {
      if (!tgt[dst * L + l] || cur[dst * L + l]) continue; /* not in M_add(dst) */
      int src = -1;
      for (int j = 0; j < N; ++j)
        if (cur[j * L + l]) src = j;
      if (src < 0) return ORC_E_RANGE;
      mig[((size_t)src * N + dst) * L + l] = 1;
    }
  scalars[0] = blocks_in_use <= b_shrink;
  scalars[1] = b_shrink < cur_blocks;
  scalars[2] = b_shrink;
  scalars[3] = b_new;
  return ORC_OK;
}

/* ------------------------------------------------------- prefill attention
 * Chunked prefill over the same paged layout (the compute-bound stage of
 * Sec. 2 "LLM Inference": the prompt's tokens are processed in parallel).
 * Sequence s has ctx_lens[s] tokens in the cache, the last
 * q_len = q_offsets[s+1] - q_offsets[s] of them are the new chunk; query row
 * q_offsets[s] + i sits at position p = ctx - q_len + i and attends to the
 * cached tokens 0..p (causal).  Decode is the case q_len = 1.
 *   q   bf16 [total_q][Hq][D],  out fp32 [total_q][Hq][D]                  */
int32_t orc_paged_attn_prefill(const orc_kv_t *kv, int32_t layer, const uint16_t *q, float *out,
                               const int32_t *table, int32_t table_stride, const int32_t *ctx_lens,
                               const int32_t *q_offsets, int32_t num_seqs, double scale,
                               int32_t nthreads) {
  if (!kv || layer < 0 || layer >= kv->num_layers || num_seqs < 0) return ORC_E_INVAL;
  const int Hq = kv->num_q_heads, Hkv = kv->num_kv_heads, D = kv->head_dim, bs = kv->block_tokens;
  const int G = Hq / Hkv;
  if (scale <= 0) scale = 1.0 / sqrt((double)D);
  for (int s = 0; s < num_seqs; ++s) {
    const int n = ctx_lens[s], ql = q_offsets[s + 1] - q_offsets[s];
    if (n < 0 || ql < 0 || ql > n || (int64_t)(n + bs - 1) / bs > table_stride) return ORC_E_INVAL;
    for (int b = 0; b < (n + bs - 1) / bs; ++b) {
      int32_t id = table[(int64_t)s * table_stride + b];
      if (id < 0 || id >= kv->num_blocks) return ORC_E_RANGE;
    }
  }
  const int total_q = num_seqs > 0 ? q_offsets[num_seqs] : 0;
  /* sequence of every query row */
  int32_t *seq_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total_q > 0 ? total_q : 1));
  for (int s = 0; s < num_seqs; ++s)
    for (int r = q_offsets[s]; r < q_offsets[s + 1]; ++r) seq_of[r] = s;
#ifdef _OPENMP
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 4)
#endif
  for (int rh = 0; rh < total_q * Hq; ++rh) {
    const int row = rh / Hq, h = rh % Hq, g = h / G;
    const int s = seq_of[row];
    const int ql = q_offsets[s + 1] - q_offsets[s];
    const int p = ctx_lens[s] - ql + (row - q_offsets[s]); /* position of this query */
    const uint16_t *qh = q + ((int64_t)row * Hq + h) * D;
    float *o = out + ((int64_t)row * Hq + h) * D;
    double *x = (double *)malloc(sizeof(double) * (size_t)(p + 1));
    double *num = (double *)calloc((size_t)D, sizeof(double));
    double m = -INFINITY;
    for (int j = 0; j <= p; ++j) {
      const uint16_t *blk =
          (const uint16_t *)layer_block(kv, layer, table[(int64_t)s * table_stride + j / bs]);
      double acc = 0.0;
      for (int d = 0; d < D; ++d)
        acc += bf16_to_double(qh[d]) * bf16_to_double(blk[k_elem(kv, g, j % bs, d)]);
      x[j] = scale * acc;
      if (x[j] > m) m = x[j];
    }
    double den = 0.0;
    for (int j = 0; j <= p; ++j) {
      const uint16_t *blk =
          (const uint16_t *)layer_block(kv, layer, table[(int64_t)s * table_stride + j / bs]);
      const double w = exp(x[j] - m);
      den += w;
      for (int d = 0; d < D; ++d) num[d] += w * bf16_to_double(blk[v_elem(kv, g, j % bs, d)]);
    }
    for (int d = 0; d < D; ++d) o[d] = (float)(num[d] / den);
    free(x);
    free(num);
  }
  free(seq_of);
  return ORC_OK;
}
