/*
 * pipelive.h - C ABI of the MI355X (gfx950) hot path of PipeLive:
 * paged-attention decode over a resizable, block-list-indirected KV cache,
 * in-place KV resize/compaction, and incremental KV patching.
 *
 * Conventions
 *  - Plain C, every call returns int32_t: PIPELIVE_OK (0) or a negative
 *    PIPELIVE_E_* code.  Nothing throws.
 *  - "DEVICE" pointers are HIP device addresses on the current device,
 *    "HOST" pointers are ordinary host memory.  The caller owns every device
 *    buffer; the library never allocates or frees device memory (it keeps one
 *    small pinned host buffer per handle).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on it unless the text says they synchronise.
 *  - Faults found on the device (a block id out of range in a table or a
 *    patch) never touch memory: the access is skipped and a sticky status
 *    word in the region's device state is set; pipelive_kv_read_state
 *    returns it.
 *  - A handle is not re-entrant; distinct handles are independent.  Calls on
 *    one handle must be issued in stream order on one stream, with one
 *    exception that Sec. 6.1 needs (the sender drains while inference keeps
 *    writing): pipelive_kv_patch_collect may run on a second stream beside
 *    pipelive_kv_mark_dirty / pipelive_kv_append / pipelive_kv_append_chunk
 *    calls that are issued, among themselves, in order on one stream.
 *
 * KV region layout (paper Sec. 5.1 "KV Cache Resizing", Sec. 5.2 "Layer
 * Stacking"): the cache is a *block list* of independently placed physical
 * blocks; nothing assumes address = base + id * stride.  Physical block `id`
 * of layer group `g = layer / stack_k` is at block_list[g * capacity + id];
 * layer `l` occupies bytes [(l % stack_k) * blk, +blk) of it, where
 *     blk = 2 (K,V) * num_kv_heads * block_tokens * head_dim * 2 bytes (bf16).
 * In-block layout 0 (PIPELIVE_LAYOUT_D8): a layer's block is a sequence of
 * sub-blocks of sb = min(block_tokens, 32) tokens; token t lies in sub-block
 * u = t / sb at position tt = t % sb.  Element offsets in bf16 units:
 *     K[g][t][d] at u * (2*Hkv*sb*D) + ((g * (D/8) + d/8) * sb + tt) * 8 + d % 8
 *     V[g][t][d] at u * (2*Hkv*sb*D) + Hkv*sb*D + (g * D + d) * sb + tt
 * i.e. inside a sub-block K is stored as [Hkv][D/8][sb][8] (16-byte token
 * vectors, token-major inside a d-slice) and V as [Hkv][D][sb]
 * (token-contiguous), so that both MFMA operands of a 32-token tile are
 * fetched with fully coalesced loads from two contiguous runs per KV head,
 * whatever the block size.
 */
#ifndef PIPELIVE_H
#define PIPELIVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PIPELIVE_OK 0
#define PIPELIVE_E_INVAL (-1)      /* bad argument, shape or alignment */
#define PIPELIVE_E_INFEASIBLE (-2) /* shrink below the number of live blocks (Alg. 1, phase 1) */
#define PIPELIVE_E_NOSPACE (-3)    /* grow beyond capacity, workspace or patch buffer too small */
#define PIPELIVE_E_BUSY (-4)       /* resize while dirty bits are pending */
#define PIPELIVE_E_RANGE (-5)      /* block id or layer out of range / table entry not live */
#define PIPELIVE_E_HIP (-6)        /* HIP runtime error, see pipelive_last_hip_error() */

#define PIPELIVE_LAYOUT_D8 0
#define PIPELIVE_DIRTY_BLOCK 0
#define PIPELIVE_DIRTY_SLOT 1
#define PIPELIVE_DTYPE_BF16 0
#define PIPELIVE_OUT_F32 0
#define PIPELIVE_OUT_BF16 1
#define PIPELIVE_MAX_PATCH_LAYERS 128
#define PIPELIVE_BACKING_ARENA 0
#define PIPELIVE_BACKING_PER_BLOCK 1
#define PIPELIVE_MAX_TABLES 8
#define PIPELIVE_PATCH_MAGIC 0x564B4C50u /* bytes 'P','L','K','V' */
#define PIPELIVE_PATCH_VERSION 1u

typedef struct pipelive_kv pipelive_kv_t;

/* Description of one KV region (HOST struct, copied by pipelive_kv_create). */
typedef struct {
  int32_t num_layers;      /* L: layers resident in this region */
  int32_t num_q_heads;     /* Hq */
  int32_t num_kv_heads;    /* Hkv, divides Hq; query head h reads KV head h / (Hq/Hkv) */
  int32_t head_dim;        /* D: 64 or 128 */
  int32_t block_tokens;    /* bs: 16, 32, 64 or 128 tokens per block */
  int32_t stack_k;         /* layers per physical block (Sec. 5.2); 1 = one pool per layer */
  int32_t dtype;           /* PIPELIVE_DTYPE_BF16 */
  int32_t in_block_layout; /* PIPELIVE_LAYOUT_D8, the only layout of the device library (the CPU
                              oracle used by the tests also reads a plain row-major layout) */
  int32_t dirty_granularity; /* PIPELIVE_DIRTY_BLOCK: one dirty bit per block id;
                                PIPELIVE_DIRTY_SLOT: one per token slot (unit id = block id * bs + slot),
                                the paper's own granularity (Sec. 6.1) */
  int32_t block_backing;   /* PIPELIVE_BACKING_ARENA: blocks lie inside larger allocations, a shrink
                              vacates ids >= B_new by copying (block_list is only read);
                              PIPELIVE_BACKING_PER_BLOCK: every physical block is an allocation of its
                              own (Sec. 5.1), a shrink permutes block_list in place (pointer updates
                              only) and the caller releases the blocks left at ids >= B_new */
  int64_t num_blocks;      /* B: valid ids are 0 .. B-1 */
  int64_t capacity_blocks; /* entries per group in block_list, B <= capacity < 2^31 */
  const uint64_t *block_list; /* DEVICE [ceil(L/stack_k)][capacity]: block addresses, 256-B aligned;
                                 written by pipelive_kv_resize when block_backing is PER_BLOCK */
  uint8_t *live_bitmap;    /* DEVICE, pipelive_bitmap_bytes(capacity): bit i = byte i>>3, bit i&7;
                              maintained by the caller's block manager, updated by resize */
  uint8_t *dirty_bitmap;   /* DEVICE, pipelive_bitmap_bytes(U) with U = pipelive_kv_dirty_units(capacity, bs,
                              granularity), same bit order; maintained by the library; zeroed by the caller at start */
  void *dev_state;         /* DEVICE, pipelive_kv_state_bytes(U) bytes, 256-B aligned,
                              zeroed by the caller before pipelive_kv_create */
} pipelive_kv_desc_t;

/* bytes of one bitmap of `n_bits` bits (a whole number of 64-bit words) */
size_t pipelive_bitmap_bytes(int64_t n_bits);
/* dirty-tracking units of a region: capacity (block granularity) or capacity * block_tokens */
int64_t pipelive_kv_dirty_units(int64_t capacity_blocks, int32_t block_tokens, int32_t granularity);
/* bytes of the per-region device state (counters, status, drain snapshot) for `dirty_units` units */
size_t pipelive_kv_state_bytes(int64_t dirty_units);

/* Create / destroy the host-side handle.  No device work. */
int32_t pipelive_kv_create(const pipelive_kv_desc_t *desc, pipelive_kv_t **out);
void pipelive_kv_destroy(pipelive_kv_t *kv);
/* current B of the region */
int64_t pipelive_kv_num_blocks(const pipelive_kv_t *kv);

/* -------------------------------------------------------------------------
 * 1. Decode attention of ONE layer (Sec. 2 "LLM Inference": a decode step
 * reads the whole cached K/V of every running sequence; Sec. 5.1: blocks are
 * resolved through the block table and the block list at kernel time).
 *
 *   out[s][h][:] = sum_j softmax_j(scale * <q[s][h], K_j>) V_j ,  j < ctx_lens[s]
 * with token j in block block_table[s][j / bs], slot j % bs, KV head
 * h / (Hq/Hkv); bf16 inputs, fp32 accumulation.  No mask.  ctx_lens[s] == 0
 * gives a zero row.  Slots >= ctx_lens[s] and free blocks are never read into
 * the result (they may hold NaN).
 *
 * q            DEVICE bf16 [num_seqs][Hq][D], 16-B aligned
 * out          DEVICE [num_seqs][Hq][D], fp32 (PIPELIVE_OUT_F32) or bf16, 16-B aligned
 * block_table  DEVICE int32 [num_seqs][table_stride] of block ids; only the
 *              first ceil(ctx/bs) entries of a row are read
 * ctx_lens     DEVICE int32 [num_seqs]
 * max_ctx      HOST upper bound on ctx_lens (sizes the launch; sequences
 *              longer than it are truncated to it and flagged E_RANGE)
 * scale        <= 0 selects 1/sqrt(D)
 * split_tokens tokens of (sequence, KV head) work per wavefront, a multiple of
 *              32; 0 = cut the whole batch into equal shares, one per
 *              wavefront the device keeps resident (best throughput).  The
 *              partition depends only on ctx_lens, max_ctx and this value, so
 *              for equal arguments the result is bit-identical whatever the
 *              physical placement of the blocks.
 * workspace    DEVICE, >= pipelive_paged_attn_workspace_bytes(...), 256-B
 *              aligned; holds the partial results of (sequence, head) pairs
 *              that are cut by a share boundary.  Two calls that may run
 *              concurrently need two workspaces.
 * Asynchronous on `stream`.
 */
int32_t pipelive_paged_attn_decode(const pipelive_kv_t *kv, int32_t layer, const void *q, void *out,
                                   int32_t out_dtype, const int32_t *block_table,
                                   int32_t table_stride, const int32_t *ctx_lens, int32_t num_seqs,
                                   int32_t max_ctx, float scale, int32_t split_tokens,
                                   void *workspace, size_t workspace_bytes, void *stream);
size_t pipelive_paged_attn_workspace_bytes(const pipelive_kv_t *kv, int32_t num_seqs,
                                           int32_t max_ctx, int32_t split_tokens);

/* For callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * operation, kernels and result (bit for bit) as pipelive_paged_attn_decode,
 * with the partial records kept in a scratch buffer that is built into the
 * library (a __device__ array of pipelive_noalloc_scratch_bytes() = 16 MiB
 * which every GPU the library runs on holds until the process ends).  The call
 * allocates nothing and frees nothing.  A launch shape whose records do not fit
 * (pipelive_paged_attn_workspace_bytes(...) above that size; only explicit
 * split_tokens on very large batches get there) returns PIPELIVE_E_NOSPACE and
 * launches nothing.  All calls on one GPU share the one buffer, whatever the
 * region or stream: calls that may overlap in time on a GPU race on it and must
 * use pipelive_paged_attn_decode with workspaces of their own instead.  Nothing
 * in the buffer has to survive between calls and nothing has to be zero at the
 * start of one.  Other arguments and errors as for pipelive_paged_attn_decode. */
int32_t pipelive_paged_attn_decode_noalloc(const pipelive_kv_t *kv, int32_t layer, const void *q, void *out,
                                           int32_t out_dtype, const int32_t *block_table,
                                           int32_t table_stride, const int32_t *ctx_lens,
                                           int32_t num_seqs, int32_t max_ctx, float scale,
                                           int32_t split_tokens, void *stream);
size_t pipelive_noalloc_scratch_bytes(void);

/* Chunked-prefill attention of ONE layer over the same KV layout (Sec. 2 "LLM
 * Inference": the prompt's tokens are processed in parallel; compute-bound).
 * The new chunk's K/V is already in the cache (pipelive_kv_append_chunk or
 * the caller's own writes).  Sequence s holds ctx_lens[s] cached tokens, of which
 * the last q_len = q_offsets[s+1] - q_offsets[s] are the chunk; query row
 * q_offsets[s] + i sits at position ctx_lens[s] - q_len + i and attends to the
 * cached tokens 0 .. that position (causal).  q_len = 1 is a decode step.
 *
 * q          DEVICE bf16 [total_q][Hq][D], rows packed sequence after sequence
 * out        DEVICE [total_q][Hq][D], fp32 or bf16, 16-B aligned.  The
 *            precision of the softmax weights in the PV product follows it:
 *            16 significant bits for fp32 output, one rounded bf16 (the
 *            output's own precision, a third fewer matrix instructions)
 *            for bf16 output.
 * q_offsets  DEVICE int32 [num_seqs + 1], q_offsets[0] = 0, non-decreasing
 * total_q    HOST: q_offsets[num_seqs] (sizes the launch)
 * other arguments as for pipelive_paged_attn_decode; no workspace is needed.
 * A sequence with more queries than cached tokens sets the status word
 * (PIPELIVE_E_INVAL) and its rows are not written; so does a context longer
 * than max_ctx (PIPELIVE_E_RANGE: unlike in decode it cannot be truncated, the
 * query positions depend on it).  Asynchronous.
 * The kernel hands out its work through a few counters in the region's
 * dev_state (zero between launches; the last workgroup re-arms them, so
 * replaying a captured launch is fine): two prefill calls on the same region
 * must not run at the same time (e.g. on two streams).  After a launch that
 * was cut short, pipelive_kv_clear_status() re-arms the counters.
 */
int32_t pipelive_paged_attn_prefill(const pipelive_kv_t *kv, int32_t layer, const void *q, void *out,
                                    int32_t out_dtype, const int32_t *block_table,
                                    int32_t table_stride, const int32_t *ctx_lens,
                                    const int32_t *q_offsets, int32_t num_seqs, int32_t total_q,
                                    int32_t max_ctx, float scale, void *stream);

/* -------------------------------------------------------------------------
 * 2. ResizeKV(B) with compaction (Sec. 4.2 primitive ResizeKV; Alg. 1 phases
 * 1-2 and 5; Sec. 5.1).
 *
 * Shrink (new_num_blocks < B): if more than new_num_blocks blocks are live
 * the call returns PIPELIVE_E_INFEASIBLE; if a dirty bit is pending,
 * PIPELIVE_E_BUSY; if a used table entry is out of range or not live,
 * PIPELIVE_E_RANGE - in all three cases no byte of pool, tables or bitmaps
 * changes.  Otherwise the live blocks with id >= new_num_blocks, in
 * ascending order, move into the free ids below new_num_blocks, in ascending
 * order (every layer's bytes are copied), the live bitmap and every used
 * table entry follow, and B becomes new_num_blocks.  Blocks that stay keep
 * their ids; bytes below new_num_blocks that no move targets are untouched.
 * With PIPELIVE_BACKING_PER_BLOCK no byte is copied: for every move the two
 * block_list entries (of every layer group) are exchanged, so the moved id
 * names the same physical block as before under its new id - the same
 * logical result - and the physical blocks that were free end up at ids >=
 * new_num_blocks, ready to be released once `stream` has been synchronised
 * (the exchange may still be queued when the call returns).
 * Grow (new_num_blocks > B, <= capacity; the caller has filled the new
 * block_list entries): B becomes new_num_blocks, the new ids are not live, no
 * data moves.
 *
 * block_tables  HOST array of num_tables DEVICE pointers, int32 [rows][stride]
 * table_rows, table_strides  HOST int32 [num_tables]
 * table_used    HOST array of num_tables DEVICE pointers, int32 [rows]: number
 *               of valid leading entries of each row (e.g. ceil(ctx/bs))
 * remap_out     DEVICE int32 [old B] or NULL: new id of every old id
 *               (identity if it stayed, -1 if it was not live)
 * result        HOST; filled before returning
 * workspace     DEVICE >= pipelive_kv_resize_workspace_bytes(kv), 256-B aligned
 * The call waits until the plan (the feasibility verdict) has been computed on
 * `stream`; the commit is queued behind it and may still be running when the
 * call returns, ordered on `stream` like any asynchronous call.  A refused
 * resize modifies nothing.
 */
typedef struct {
  int64_t n_live, n_moved, old_num_blocks, new_num_blocks;
  int32_t status; /* same as the return value */
  int32_t reserved;
} pipelive_resize_result_t;

int32_t pipelive_kv_resize(pipelive_kv_t *kv, int64_t new_num_blocks, int32_t *const *block_tables,
                           const int32_t *table_rows, const int32_t *table_strides,
                           const int32_t *const *table_used, int32_t num_tables,
                           int32_t *remap_out, pipelive_resize_result_t *result, void *workspace,
                           size_t workspace_bytes, void *stream);
size_t pipelive_kv_resize_workspace_bytes(const pipelive_kv_t *kv);

/* -------------------------------------------------------------------------
 * Independently allocated blocks (Sec. 5.1: the KV cache is a list of GPU
 * blocks that are allocated and freed on demand; Sec. 5.2: such allocations
 * come in units of the virtual-memory allocation granularity).
 *
 * A pool reserves one virtual address range of max_blocks * block_bytes and
 * backs single blocks of it with physical memory through HIP's virtual memory
 * management calls.  pipelive_vmm_pool_alloc / _free are the only calls of
 * this library that allocate or release device memory; they are host-side
 * driver calls (tens to hundreds of microseconds per block) and belong
 * outside the serving loop.  A pool is bound to the device that was current
 * at creation and is not thread-safe.
 *
 * Together with PIPELIVE_BACKING_PER_BLOCK a shrink is:
 *   pipelive_kv_resize(kv, B_new, ...)         permutes block_list, remaps tables
 *   read block_list[g][B_new .. B_old) back    the blocks no id refers to any more
 *   pipelive_vmm_pool_free(pool, n, addrs)     returns their memory to the device
 * and a grow is pipelive_vmm_pool_alloc, write the addresses to
 * block_list[g][B_old .. B_new), pipelive_kv_resize(kv, B_new, ...).
 */
typedef struct pipelive_vmm_pool pipelive_vmm_pool_t;

/* Physical memory one block of `block_bytes` consumes: block_bytes rounded up
 * to the 2 MiB unit in which MI355X backs such allocations (measured: the
 * runtime reports a 4 KiB granularity, free memory drops by 2 MiB per handle). */
size_t pipelive_vmm_backing_bytes(size_t block_bytes);

/* block_bytes: a multiple of the granularity the runtime reports (E_INVAL
 * otherwise); max_blocks: size of the address range, in blocks.  No physical
 * memory is taken.  E_HIP if the device has no virtual memory management. */
int32_t pipelive_vmm_pool_create(size_t block_bytes, int64_t max_blocks, pipelive_vmm_pool_t **out);
/* unmaps and releases every block still allocated, frees the address range */
void pipelive_vmm_pool_destroy(pipelive_vmm_pool_t *pool);
/* Back n more blocks (lowest free positions of the range first) and return
 * their device addresses in addrs (HOST, n entries).  E_NOSPACE if fewer than n
 * positions are free, E_HIP if the device is out of memory; in both cases
 * nothing stays allocated from this call. */
int32_t pipelive_vmm_pool_alloc(pipelive_vmm_pool_t *pool, int64_t n, uint64_t *addrs);
/* Release the blocks at addrs (HOST, n entries, each returned by _alloc and not
 * yet freed; E_INVAL otherwise, checked before anything is released).  No
 * kernel may be using them: the caller synchronises first. */
int32_t pipelive_vmm_pool_free(pipelive_vmm_pool_t *pool, int64_t n, const uint64_t *addrs);
/* blocks currently backed by physical memory; -1 for a null pool */
int64_t pipelive_vmm_pool_allocated(const pipelive_vmm_pool_t *pool);
/* first address of the pool's range (position i lies at base + i * block_bytes); 0 for a null pool */
uint64_t pipelive_vmm_pool_base(const pipelive_vmm_pool_t *pool);

/* -------------------------------------------------------------------------
 * Region-aware device arena: memory placement for MI355X (not from the paper;
 * for callers that allocate KV pools and patch buffers).  The 288 GB of this
 * part behave as three regions of 96 GB.  A copy whose reads and writes all
 * fall into one region runs at 0.64-0.70 of the HBM peak, one whose traffic is
 * spread over the regions at 0.78-0.80; a kernel that only reads (decode
 * attention) is fastest, 0.80 against 0.73, when all it reads in one launch
 * lies in ONE region; and which region an allocation lands in depends on what
 * the process, and the one before it, allocated earlier.
 * An arena is one virtually contiguous range made of physical pieces of
 * piece_bytes.  With probe_bytes > 0 the call times, for pairs of stretches
 * of probe_bytes (consecutive pieces as the driver handed them out), a copy
 * that runs inside both at once (slow: same region) and sorts the pieces into
 * classes that way.  The range is laid out in zones:
 *   zone 0, the spread zone: consecutive pieces come from the classes in turn
 *           (each class in proportion to its size) - for buffers a copy
 *           streams through, such as patch buffers;
 *   zone 1 + c: the remaining pieces of class c - for what one launch reads
 *           alone, such as the KV blocks of one layer.  A pool whose layers
 *           take the class zones in turn gives decode its one region per
 *           launch and the copies, which work on all layers at once, all
 *           regions per launch.
 * pipelive_arena_layout sets the size of the spread zone (create leaves the
 * whole range in it) and remaps the pieces accordingly; the caller carves its
 * buffers out of the zones.  The kernels see ordinary device addresses; the
 * result of every library call is the same with or without an arena.
 *
 * bytes        rounded up to a multiple of piece_bytes; all of it is backed
 *              by physical memory when create returns
 * piece_bytes  a multiple of 2 MiB (E_INVAL otherwise): the grain at which the
 *              spread zone alternates between the classes; 64 MiB in the bench
 * probe_bytes  0: no probe, one class.  Otherwise a multiple of piece_bytes
 *              (E_INVAL otherwise): 1 GiB in the bench.  Shorter stretches
 *              resolve a finer mix of regions but are harder to time (the
 *              probe's launches go over a stretch until 512 MiB have moved;
 *              256 MiB still classifies cleanly on an idle device, not under
 *              a tracing profiler; below 64 MiB the classes found are noise,
 *              which is harmless: only the order of the pieces depends on
 *              them).  About 2 ms per GiB of the range at 1 GiB, 4 ms at
 *              256 MiB: device work on the null stream, the call returns when
 *              it is done; the device should be idle otherwise.  A range
 *              shorter than two such stretches is not probed
 * spread_bytes rounded up to whole pieces, at most the range
 * E_NOSPACE if the device is out of memory, E_HIP for any other runtime error;
 * nothing of a failing create stays allocated (after a failing layout the
 * arena can only be destroyed).  At start-up or between workloads, not in the
 * serving loop: create and layout wait for the device and are host-side driver
 * calls of the order of a millisecond per piece.  The contents of the range
 * are undefined after either; no kernel may be using the range during layout
 * or destroy, which unmaps and releases everything.
 * For some seconds after a process has released a few hundred GB the driver
 * hands memory out with the regions mixed at a grain no probe resolves; n_runs
 * in the info shows it (dozens to hundreds instead of n_classes).  A caller
 * that sees it can destroy the arena, wait about ten seconds and create it
 * again. */
#define PIPELIVE_ARENA_MAX_CLASSES 4
typedef struct pipelive_arena pipelive_arena_t;
typedef struct {
  int32_t n_pieces, n_classes;
  int32_t class_pieces[PIPELIVE_ARENA_MAX_CLASSES]; /* pieces per class */
  int32_t n_runs;        /* runs of equal class among the pieces in the order the driver handed them out: equal to
                            n_classes when each region came in one stretch, large when the hand-out was mixed */
  float probe_ms;        /* time the probe took (0 without probe) */
  float rate_same_GBps;  /* mean rate (read + written) of the pair copies judged "same region" ... */
  float rate_other_GBps; /* ... and of those judged "different regions"; 0 if there was no contrast */
} pipelive_arena_info_t;
int32_t pipelive_arena_create(size_t bytes, size_t piece_bytes, size_t probe_bytes, pipelive_arena_t **out);
int32_t pipelive_arena_layout(pipelive_arena_t *arena, size_t spread_bytes);
void pipelive_arena_destroy(pipelive_arena_t *arena);
/* first address and size of the range; 0 for a null arena */
uint64_t pipelive_arena_base(const pipelive_arena_t *arena);
size_t pipelive_arena_bytes(const pipelive_arena_t *arena);
int32_t pipelive_arena_info(const pipelive_arena_t *arena, pipelive_arena_info_t *out);
/* byte offset from base and size of zone 0 .. n_classes (a zone may be empty); E_INVAL for any other zone */
int32_t pipelive_arena_zone(const pipelive_arena_t *arena, int32_t zone, uint64_t *offset, uint64_t *bytes);
/* class (0 .. n_classes-1) of the piece at [base + piece * piece_bytes, ...); E_INVAL outside the range */
int32_t pipelive_arena_piece_class(const pipelive_arena_t *arena, int64_t piece);

/* Effective KV utilisation (Sec. 7.5, effects of layer stacking): tokens held
 * divided by token slots of the blocks the sequences occupy,
 *   sum_s n_s / sum_s ceil(n_s / block_tokens) * block_tokens ;  1.0 when no
 * sequence holds a token.  ctx_lens HOST int32 [n].  Host arithmetic only. */
double pipelive_kv_utilization(const int32_t *ctx_lens, int64_t n, int32_t block_tokens);
/* Tokens per layer in one physical block of `phys_block_bytes` shared by
 * stack_k layers (Sec. 5.2: C / k): floor(phys_block_bytes / (stack_k * token_bytes_per_layer)). */
int64_t pipelive_stacked_block_tokens(size_t phys_block_bytes, int32_t stack_k,
                                      size_t token_bytes_per_layer);

/* MaxBlocks(i, L) = floor((M_i * u - L * W) / (L * P))  (Alg. 1); host arithmetic only. */
int64_t pipelive_max_blocks(double mem_bytes, double util, int64_t layers,
                            double weight_bytes_per_layer, double block_bytes_per_layer);

/* Planning arithmetic of the reconfiguration algorithm (Alg. 1; worked example
 * in Sec. 4.1).  Host only.  GPU i holds the inclusive layer range
 * [cur_first[i], cur_last[i]] and shall hold [tgt_first[i], tgt_last[i]]
 * (last < first = no layers).
 *   phase 1: C_tmp[i] = C_cur[i] U C_tgt[i];  b_shrink = min_i MaxBlocks(i, |C_tmp[i]|);
 *            feasible = blocks_in_use <= b_shrink;  need_shrink = b_shrink < cur_blocks
 *   phase 3: mig[k] = (src GPU, dst GPU, layer) for every layer of C_tgt[dst] \ C_cur[dst],
 *            src = the GPU that owns the layer in C_cur (ascending dst, then layer)
 *   phase 5: del[k] = (GPU, layer) for every layer of C_tmp[i] \ C_tgt[i];
 *            b_new = min_i MaxBlocks(i, |C_tgt[i]|)
 * mig holds 3*max_mig int32, del 2*max_del int32; n_mig / n_del report the
 * full counts (PIPELIVE_E_NOSPACE if a list did not fit, PIPELIVE_E_RANGE if
 * the target names a layer that no GPU currently holds). */
typedef struct {
  int32_t feasible, need_shrink;
  int64_t b_shrink, b_new;
  int32_t n_mig, n_del;
} pipelive_reconfig_plan_t;
int32_t pipelive_plan_reconfig(int32_t num_gpus, const int32_t *cur_first, const int32_t *cur_last,
                               const int32_t *tgt_first, const int32_t *tgt_last,
                               const double *mem_bytes, double util, double weight_bytes_per_layer,
                               double block_bytes_per_layer, int64_t blocks_in_use,
                               int64_t cur_blocks, pipelive_reconfig_plan_t *plan, int32_t *mig,
                               int32_t max_mig, int32_t *del, int32_t max_del);
/* phase 4: 1 when T_sched - T_applied[i] < tau for every destination, else 0 */
int32_t pipelive_converged(int64_t t_sched, const int64_t *t_applied, int32_t n, int64_t tau);

/* -------------------------------------------------------------------------
 * 3. Incremental KV patching (Sec. 6.1 "KV Migration with KV Patch").
 * One dirty bit per *unit*, shared by all layers of the region (a decode step
 * writes the same slot in every layer).  A unit is a block
 * (PIPELIVE_DIRTY_BLOCK) or one token slot (PIPELIVE_DIRTY_SLOT, unit id =
 * block id * bs + slot); a unit's patch entry is the block's bytes verbatim,
 * or the token's K[Hkv][D] followed by its V[Hkv][D] (bf16, gathered out of
 * the in-block layout).
 *
 * append: the write side of a decode step for one layer.  Token
 * positions[s] (>= 0; < 0 skips the sequence) of sequence s receives
 * k_new[s], v_new[s] (DEVICE bf16 [num_seqs][Hkv][D], 16-B aligned) in block
 * block_table[s][pos / bs], slot pos % bs.  mark != 0 sets the dirty bit of
 * the written unit; count_tokens != 0 adds the number of written tokens to
 * n_acc (pass it for one layer per step: n(t) counts tokens, not layer
 * writes).  A bad block id or a position beyond the table row sets the status
 * word and writes nothing for that sequence.  Asynchronous.
 */
int32_t pipelive_kv_append(pipelive_kv_t *kv, int32_t layer, const void *k_new, const void *v_new,
                           const int32_t *block_table, int32_t table_stride,
                           const int32_t *positions, int32_t num_seqs, int32_t mark,
                           int32_t count_tokens, void *stream);

/* append_chunk: the write side of a prefill chunk for one layer (Sec. 2 "LLM
 * Inference": the prompt's tokens are processed together and their K/V enter
 * the cache; Sec. 6.1: what a step writes is flagged).  Same convention as
 * pipelive_paged_attn_prefill: sequence s holds ctx_lens[s] tokens *including*
 * the chunk, whose q_len = q_offsets[s+1] - q_offsets[s] tokens are rows
 * q_offsets[s] .. of k_new / v_new (DEVICE bf16 [total_q][Hkv][D], 16-B
 * aligned); row q_offsets[s] + i goes to position ctx_lens[s] - q_len + i.
 * mark and count_tokens as for append (count_tokens adds total_q's written
 * tokens).  A chunk longer than its context is skipped; a 32-token window with
 * a block id out of range or a position beyond the table row sets the status
 * word and is not written.  total_q is a HOST value (sizes the launch).
 * Asynchronous. */
int32_t pipelive_kv_append_chunk(pipelive_kv_t *kv, int32_t layer, const void *k_new, const void *v_new,
                                 const int32_t *block_table, int32_t table_stride,
                                 const int32_t *ctx_lens, const int32_t *q_offsets, int32_t num_seqs,
                                 int32_t total_q, int32_t mark, int32_t count_tokens, void *stream);

/* mark_dirty: B[id] <- 1 for the n unit ids in ids (DEVICE int32), and
 * n_acc += n_tokens (the tokens scheduled in that step).  Asynchronous. */
int32_t pipelive_kv_mark_dirty(pipelive_kv_t *kv, const int32_t *block_ids, int32_t n,
                               int64_t n_tokens, void *stream);

/* 64-byte header at patch_buf[0] (little endian). */
typedef struct {
  uint32_t magic, version;
  uint32_t n_blocks; /* ids carried by this patch */
  uint32_t n_layers;
  uint64_t block_bytes;    /* blk */
  uint64_t n_acc_tokens;   /* tokens this patch acknowledges */
  uint64_t payload_offset; /* round_up(64 + 4 * max_blocks, 256) */
  uint32_t max_blocks;     /* capacity of the id list */
  uint32_t more_pending;   /* 1 if dirty bits were left behind */
  uint32_t unit_tokens;    /* tokens per unit: bs (block granularity) or 1 (slot granularity) */
  uint8_t pad[12];
} pipelive_patch_hdr_t;

/* number of units a patch buffer of `capacity` bytes can carry:
 * min(units of the region, floor((capacity - 320) / (4 + n_layers * unit_bytes))) */
int64_t pipelive_patch_max_blocks(const pipelive_kv_t *kv, int32_t n_layers, size_t capacity);

/* collect: atomically take the dirty set D (ascending ids, at most
 * max_blocks of them - the lowest; the others stay set and more_pending = 1),
 * clear exactly those bits, and gather into patch_buf
 *     header | int32 ids[max_blocks] | pad to 256 B | payload[r][i][blk]
 * where payload[r][i] is the verbatim K-then-V bytes of block ids[r] in layer
 * layers[i].  n_acc travels in the header (and restarts from 0) only when the
 * drain empties the bitmap.  A write that races with the drain (mark or append
 * on another stream) lands in this patch or in the next one, never nowhere:
 * writers store the slot, then set its bit, then count its tokens, and the
 * drain takes the count before it takes the bits, so a patch never
 * acknowledges tokens that neither it nor an earlier patch carries.
 *
 * layers         HOST int32 [n_layers] (region-local layer indices, patch order)
 * patch_buf      DEVICE, 256-B aligned, patch_capacity_bytes
 * hdr_host_copy  HOST (pinned) or NULL; filled by an async copy on `stream`
 * Asynchronous; no host round trip (the number of dirty blocks stays on the device).
 */
int32_t pipelive_kv_patch_collect(pipelive_kv_t *src, const int32_t *layers, int32_t n_layers,
                                  void *patch_buf, size_t patch_capacity_bytes,
                                  pipelive_patch_hdr_t *hdr_host_copy, void *stream);

/* apply: write every entry of the patch into block dst_block_map[id]
 * (identity when NULL) of layer dst_layers[i] of `dst`, then
 * T_applied += n_acc_tokens.  The patch may come from another sender, so it is
 * checked on the device before anything is written: a header that does not
 * match the target (magic, version, n_layers, block_bytes, unit_tokens) or the
 * buffer (n_blocks <= max_blocks, payload_offset = round_up(64 + 4 max_blocks,
 * 256), payload inside patch_bytes) sets the status word to PIPELIVE_E_INVAL;
 * a source id outside [0, map_entries) (without a map: outside dst), or one
 * that the map sends outside dst, sets it to PIPELIVE_E_RANGE.  A refused
 * patch is refused as a whole: no byte of dst changes and T_applied stays.
 * Asynchronous.
 *
 * dst_layers     HOST int32 [n_layers]
 * patch_bytes    HOST size of the buffer at patch_buf (what may be read)
 * dst_block_map  DEVICE int32 [map_entries] indexed by source *block* id, or NULL
 *                (a slot keeps its position inside the mapped block); source and
 *                target must have the same dirty granularity
 * map_entries    HOST number of entries of dst_block_map (ignored when it is NULL)
 */
int32_t pipelive_kv_patch_apply(pipelive_kv_t *dst, const int32_t *dst_layers, int32_t n_layers,
                                const void *patch_buf, size_t patch_bytes,
                                const int32_t *dst_block_map, int64_t map_entries, void *stream);

/* T_applied of `dst` (Sec. 6.1: tokens acknowledged by the patches applied so
 * far), read back with a blocking copy: the caller has synchronised the stream
 * the applies were issued on.  Negative PIPELIVE_E_* on failure. */
int64_t pipelive_kv_tokens_applied(const pipelive_kv_t *dst);

/* Counters and status of a region; synchronises `stream`. */
typedef struct {
  uint64_t n_acc;     /* tokens marked since the last complete drain */
  uint64_t t_applied; /* tokens acknowledged by applied patches (T_applied) */
  int32_t status;     /* sticky device status: PIPELIVE_OK or the first PIPELIVE_E_* seen */
  int32_t reserved;
} pipelive_kv_state_t;
int32_t pipelive_kv_read_state(pipelive_kv_t *kv, pipelive_kv_state_t *out, void *stream);
/* clear the sticky status (asynchronous) */
int32_t pipelive_kv_clear_status(pipelive_kv_t *kv, void *stream);

const char *pipelive_strerror(int32_t code);
/* text of the last HIP error seen by the calling thread ("" if none) */
const char *pipelive_last_hip_error(void);
/* 1 if the current device is a gfx950, else 0 */
int32_t pipelive_device_ok(void);

#ifdef __cplusplus
}
#endif
#endif /* PIPELIVE_H */
