// Internal declarations shared by the host API and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pipelive.h"

namespace pipelive {

// Per-region device state (at desc.dev_state).  The drain snapshot words
// follow at byte offset kSnapOffset.
struct DevState {
  unsigned long long n_acc;      // tokens marked since the last complete drain
  unsigned long long t_applied;  // T_applied
  int32_t status;                // sticky: first PIPELIVE_E_* seen on the device
  int32_t unused_;
  int32_t prefill_finished;      // prefill kernel: workgroups that have left; zero whenever no launch is running
  int32_t mark_blocks_done;      // workgroups of the running mark launch that have set their bits
  unsigned long long n_acc_taken;  // drain: n_acc as taken before the first bitmap word was exchanged
  int32_t apply_verdict;         // apply: PIPELIVE_OK or why the patch at hand is refused as a whole
  int32_t pad_[5];
};
static_assert(sizeof(DevState) == 64, "DevState layout");
constexpr size_t kSnapOffset = 256;
// The prefill kernel's work lists draw their tickets from kPrefillLists counters at byte offset kListOffset of the
// state (one list per XCD of the part); like prefill_finished they are zero whenever no prefill launch of the
// region is running.
constexpr int kPrefillLists = 8;
constexpr size_t kListOffset = 64;
static_assert(kListOffset + kPrefillLists * sizeof(int32_t) <= kSnapOffset, "list counters fit before the snapshot");

struct HostPinned {  // small pinned mailbox per handle
  int64_t plan[8];
  DevState state;
};

}  // namespace pipelive

struct pipelive_kv {
  pipelive_kv_desc_t d;
  int64_t groups;
  uint64_t blk_bytes;   // one (layer, block)
  uint64_t phys_bytes;  // one physical block = stack_k * blk_bytes
  int64_t units_per_block;  // dirty-tracking units per block: 1 or block_tokens
  uint64_t unit_bytes;      // patch bytes of one unit per layer
  pipelive::HostPinned *pinned;
  hipEvent_t plan_ready;  // recorded after the copy of a resize plan into `pinned`
};

namespace pipelive {

inline DevState *dev_state(const pipelive_kv *kv) { return (DevState *)kv->d.dev_state; }
inline int32_t *prefill_tickets(const pipelive_kv *kv) { return (int32_t *)((char *)kv->d.dev_state + kListOffset); }
inline unsigned long long *snap_words(const pipelive_kv *kv) {
  return (unsigned long long *)((char *)kv->d.dev_state + kSnapOffset);
}

// ---- attention
struct AttnParams {
  const uint64_t *block_list;  // this layer's group row
  uint32_t layer_off;          // byte offset of the layer inside a physical block
  const uint16_t *q;
  void *out;
  int32_t out_dtype;
  const int32_t *table;
  int32_t table_stride;
  const int32_t *ctx;
  int32_t num_seqs, max_ctx;
  int32_t Hq, Hkv, G;
  float scale_log2;  // scale * log2(e)
  int32_t num_waves;       // waves launched
  int32_t tiles_per_wave;  // share size in 32-token tiles; 0 = total / num_waves
  float *ws;               // partial records: [2 * num_waves][attn_record_floats(G, D)]
  int64_t num_blocks;
  int32_t *status;
};
// floats of one partial record: O[G][D], m[G], l[G], padded to 16 bytes
__host__ __device__ inline int64_t attn_record_floats(int G, int D) {
  return (int64_t)G * D + ((2 * G + 3) & ~3);
}
hipError_t launch_attn_decode(const AttnParams &p, int D, int BS, hipStream_t st);
int attn_waves_per_cu(int D, int BS);

// ---- prefill attention
constexpr int kPrefillNQ = 2;  // 16-column score blocks per wave: 32 (token, head) columns
struct PrefillParams {
  const uint64_t *block_list;
  uint32_t layer_off;
  const uint16_t *q;
  void *out;
  int32_t out_dtype;
  const int32_t *table;
  int32_t table_stride;
  const int32_t *ctx;
  const int32_t *q_offsets;
  int32_t num_seqs, max_ctx;
  int32_t Hq, Hkv, G;
  float scale_log2;
  int32_t num_units;  // an upper bound on the units of one list (the ragged split is only known on the device)
  int32_t n_lists;    // work lists (set by the launch)
  int64_t num_blocks;
  int32_t *status;
  int32_t *ticket;    // per list: units drawn beyond the first one of every workgroup; zero between launches
  int32_t *finished;  // workgroups that have left; the last one zeroes both
};
hipError_t launch_attn_prefill(const PrefillParams &p, int D, int BS, hipStream_t st);

// ---- resize
struct TableRef {
  int32_t *table;
  const int32_t *used;
  int32_t rows, stride;
};
struct ResizePlanOut {  // in the workspace
  long long n_live, n_moved, any_dirty, bad_table;
};
hipError_t launch_resize_plan(const pipelive_kv *kv, int64_t B, int64_t B_new, ResizePlanOut *plan,
                              int32_t *move_src, int32_t *move_dst, hipStream_t st);
hipError_t launch_table_check(const pipelive_kv *kv, int64_t B, const TableRef &t,
                              ResizePlanOut *plan, hipStream_t st);
// Both read the verdict (and the number of moves) from `plan` on the device and do nothing when
// the plan refuses the resize, so they can be queued before the host has seen it.
hipError_t launch_resize_commit(const pipelive_kv *kv, int64_t B, int64_t B_new,
                                const ResizePlanOut *plan, const int32_t *move_src,
                                const int32_t *move_dst, int32_t *remap, const TableRef *tables,
                                int n_tables, hipStream_t st);
hipError_t launch_grow(const pipelive_kv *kv, int64_t B, int64_t B_new, int32_t *remap,
                       const ResizePlanOut *plan, hipStream_t st);

// ---- patch
struct LayerList {
  int32_t n;
  int32_t layer[PIPELIVE_MAX_PATCH_LAYERS];
};
hipError_t launch_mark(const pipelive_kv *kv, const int32_t *ids, int32_t n, int64_t n_tokens,
                       hipStream_t st);
hipError_t launch_append(const pipelive_kv *kv, int32_t layer, const uint16_t *k_new,
                         const uint16_t *v_new, const int32_t *table, int32_t table_stride,
                         const int32_t *positions, int32_t num_seqs, int32_t mark,
                         int32_t count_tokens, hipStream_t st);
hipError_t launch_append_chunk(const pipelive_kv *kv, int32_t layer, const uint16_t *k_new,
                               const uint16_t *v_new, const int32_t *table, int32_t table_stride,
                               const int32_t *ctx, const int32_t *q_offsets, int32_t num_seqs,
                               int32_t total_q, int32_t mark, int32_t count_tokens, hipStream_t st);
hipError_t launch_collect(const pipelive_kv *kv, const LayerList &layers, uint8_t *patch,
                          uint32_t max_blocks, uint64_t payload_offset, hipStream_t st);
hipError_t launch_apply(const pipelive_kv *kv, const LayerList &layers, const uint8_t *patch,
                        uint64_t patch_bytes, const int32_t *dst_map, int64_t map_entries,
                        hipStream_t st);
hipError_t launch_clear_status(const pipelive_kv *kv, hipStream_t st);

int device_cu_count();
int copy_wgs_per_cu();  // persistent copy workgroups launched per CU

// the calling thread's last HIP error text (what pipelive_last_hip_error returns)
void set_hip_error(const char *text);
int32_t hip_fail(hipError_t e);  // records the text, returns PIPELIVE_E_HIP

}  // namespace pipelive

#define HIP_TRY(expr)                                    \
  do {                                                   \
    hipError_t e_ = (expr);                              \
    if (e_ != hipSuccess) return pipelive::hip_fail(e_); \
  } while (0)
