// Chunked-prefill paged attention for gfx950 (CDNA4, wave64, MFMA): the
// compute-bound stage (paper Sec. 2 "LLM Inference": prompt tokens are
// processed in parallel) over the same block-list KV layout as decode.
//
// Work unit = (sequence, KV head, block of 4*QB consecutive query tokens), one
// per workgroup; wave w of it owns the QB tokens [w*QB, (w+1)*QB) of the block.
// A wave's NQ*16 score columns are its QB tokens x the G query heads of the KV
// head (column = token * G + head).  The workgroup walks the 32-token KV tiles
// that its last query may see; each tile's K and V of the KV head (two
// contiguous runs of the in-block layout) are copied once from global memory
// into a ring of three LDS stages by LDS-direct loads (global_load_lds_dwordx4:
// no staging registers), issued two tiles ahead of the arithmetic, and all
// four waves take their MFMA operands from there.  Per tile a wave computes
// S^T = K Q^T for its columns, applies the causal mask by predicate, runs the
// online softmax per column and accumulates O^T += V^T P^T with P split into
// two bf16 terms.  A wave whose queries cannot see a tile, or that has no
// queries at all, still takes part in the copies and barriers.
#include <type_traits>

#include "attn_common.h"

namespace pipelive {
namespace {

// LDS image of one tile: the K runs as in global memory, then the V runs with the 16-byte pieces of
// every row permuted (piece k of row d sits at position k ^ swizzle(d)), so that a wave's 8-byte
// reads, 16 rows apart by lane, fall into distinct banks.  The image has no holes: the copies are
// LDS-direct loads, which write 64 consecutive pieces per wave instruction.
template <int D, int BS>
struct Stage {
  static constexpr int SB = SubBlock<BS>::SB;           // tokens per contiguous run: 16 or 32
  static constexpr int HALVES = kTile / SB;             // runs per tile: 2 or 1
  static constexpr int KRUN = SB * D * 2;               // bytes of one K run (= one V run)
  static constexpr int VROW = SB * 2;                   // bytes of one V row in global memory
  static constexpr int CPR = VROW / 16;                 // 16-byte pieces per V row: 4 or 2
  static constexpr int VRUN = D * VROW;                 // bytes of one V run (= KRUN)
  // rows d and d + 4 (SB 32) or d + 8 (SB 16) would share banks: their pieces are rotated apart
  __device__ static int swizzle(int d) { return SB == 32 ? (d >> 2) & 3 : (d >> 3) & 1; }
  static constexpr int KBYTES = HALVES * KRUN;          // K of the tile
  static constexpr int BYTES = KBYTES + HALVES * VRUN;  // whole stage
  static constexpr int CHUNKS = 2 * HALVES * KRUN / 16; // 16-byte pieces copied per tile
  static constexpr int PER_THREAD = CHUNKS / 256;       // 4 (D 128) or 2 (D 64)
};

#ifdef PIPELIVE_PREFILL_TRACE
// development builds: shader-clock totals per phase, summed over the tiles of wave 0 of workgroup 0
__device__ long long g_prefill_trace[16];
#define PTRACE_DECL long long tr_t0 = 0; long long tr_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}; const bool tr_on = blockIdx.x == 0 && tid < 64; const long long tr_c0 = clock64(), tr_w0 = wall_clock64()
#define PTRACE_START() do { __builtin_amdgcn_sched_barrier(0); tr_t0 = clock64(); __builtin_amdgcn_sched_barrier(0); } while (0)
#define PTRACE(k) do { __builtin_amdgcn_sched_barrier(0); const long long n_ = clock64(); tr_acc[k] += n_ - tr_t0; tr_t0 = n_; __builtin_amdgcn_sched_barrier(0); } while (0)
#define PTRACE_FLUSH(ntiles) do { if (tr_on && lane == 0) { for (int i_ = 0; i_ < 8; ++i_) g_prefill_trace[i_] = tr_acc[i_]; g_prefill_trace[8] = (ntiles); g_prefill_trace[9] = clock64() - tr_c0; g_prefill_trace[10] = wall_clock64() - tr_w0; } } while (0)
#else
#define PTRACE_DECL do {} while (0)
#define PTRACE_START() do {} while (0)
#define PTRACE(k) do {} while (0)
#define PTRACE_FLUSH(n) do {} while (0)
#endif

constexpr int kStages = 3;
constexpr float kLazyMaxStep = 8.0f;  // log2 of the growth of a column's maximum that triggers a rescale
typedef u32x4 __attribute__((address_space(3))) *lds_u4;
typedef char __attribute__((address_space(3))) *lds_ptr;

// PAIR: the softmax weights enter the PV product as a pair of bf16 numbers (16 significant bits, for
// the fp32 output); without it as one rounded bf16, the precision of the bf16 output itself, which
// saves a third of the matrix instructions and the splitting arithmetic.
template <int D, int BS, int NQ, bool PAIR>
__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(PrefillParams p) {
  using St = Stage<D, BS>;
  constexpr int NC = D / 32, ND = D / 16, SB = St::SB;
  __shared__ __attribute__((aligned(16))) char lds[kStages * St::BYTES];

  const int tid = threadIdx.x;
  PTRACE_DECL;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, qg = lane >> 4;
  const int G = p.G, Hkv = p.Hkv, S = p.num_seqs;
  const int QB = (NQ * 16) / G;  // query tokens per wave
  const int WB = 4 * QB;         // query tokens per workgroup
  const int unit = blockIdx.x;

  // ---- locate the unit: units of sequence s = Hkv * ceil(q_len / WB), ordered (s, head, block)
  // (the lanes that scan the sequences also fetch what the unit needs of its sequence, so that no
  // second round trip to memory follows the search)
  int s = -1, nwb = 0, q0 = 0, qlen = 0, n = 0;
  int64_t rem = 0;
  {
    int64_t carry = 0;
    for (int base = 0; base < S && s < 0; base += 64) {
      const bool in = base + lane < S;
      int qa = 0, ql = 0, cx = 0;
      if (in) {
        qa = p.q_offsets[base + lane];
        ql = p.q_offsets[base + lane + 1] - qa;
        cx = p.ctx[base + lane];
      }
      const int nb = ql > 0 ? (ql + WB - 1) / WB : 0;
      const int units = nb * Hkv;
      const int inc = wave_inclusive_scan(units, lane);
      const uint64_t bal = __ballot(in && carry + inc > unit);  // first sequence whose range holds it
      if (bal) {
        const int k = __ffsll((long long)bal) - 1;
        s = base + k;
        nwb = __builtin_amdgcn_readlane(nb, k);
        q0 = __builtin_amdgcn_readlane(qa, k);
        qlen = __builtin_amdgcn_readlane(ql, k);
        n = __builtin_amdgcn_readlane(cx, k);
        rem = unit - (carry + __builtin_amdgcn_readlane(inc, k) - __builtin_amdgcn_readlane(units, k));
      }
      carry += __builtin_amdgcn_readlane(inc, 63);
    }
  }
  if (s < 0) return;  // beyond the last unit (whole workgroup: the decision is the same in every wave)
  // later query blocks attend to more tokens: hand them out first so the launch ends evenly
  const int g = (int)(rem / nwb), wb = nwb - 1 - (int)(rem % nwb);
  if (n > p.max_ctx) n = p.max_ctx;
  if (qlen > n) {  // more queries than cached tokens: flag and skip
    if (tid == 0) atomicCAS(p.status, 0, PIPELIVE_E_INVAL);
    return;
  }
  // workgroup: the tiles its last query may see
  const int wg_tok0 = wb * WB;
  const int wg_ntok = min(WB, qlen - wg_tok0);
  const int wg_pmax = n - qlen + wg_tok0 + wg_ntok - 1;
  const int nt_wg = (wg_pmax + kTile) / kTile;
  const int wg_nkv = wg_pmax + 1;
  // wave: its own queries
  const int tok0 = wg_tok0 + w * QB;
  const int ntok = max(min(QB, qlen - tok0), 0);
  const int pos0 = n - qlen + tok0;         // position of the wave's first query
  const int p_max = pos0 + ntok - 1;        // last position any of its columns attends to
  const int nt_w = ntok > 0 ? (p_max + kTile) / kTile : 0;
  const int n_kv = p_max + 1;

  // per column block: validity, causal limit, Q^T operand
  int p_col[NQ];
  bool col_ok[NQ];
  bf16x8 qreg[NQ][NC];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int col = nq * 16 + r;
    const int ti = col / G, hh = col % G;
    col_ok[nq] = ti < ntok;
    p_col[nq] = col_ok[nq] ? pos0 + ti : p_max;  // idle columns behave like the last query (finite, never stored)
    const uint16_t *qp = p.q + ((int64_t)(q0 + tok0 + ti) * p.Hq + (int64_t)g * G + hh) * D + 8 * qg;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      u32x4 v = {0, 0, 0, 0};
      if (col_ok[nq]) v = *(const u32x4 *)(qp + 32 * c);
      qreg[nq][c] = as_bf16x8(v);
    }
  }

  f32x4 acc[ND][NQ];
  f32x4 lacc[NQ];  // every element: the column's running denominator
  float m[NQ];
  // kept opaque so that it stays in registers instead of being rebuilt from scalars in every tile
  u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  asm volatile("" : "+v"(ones_bits));
  const bf16x8 ones = as_bf16x8(ones_bits);
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    m[nq] = -INFINITY;
    lacc[nq] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < ND; ++c) acc[c][nq] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  // ---- block addresses, resolved 32 tiles at a time, one block per lane; the batch after the
  // current one is resolved early so that the copies never wait for it
  constexpr int TPB = BS >= kTile ? BS / kTile : 1;  // tiles per block (a 16-token block is half a tile)
  const int n_blocks_seq = (wg_nkv + BS - 1) / BS;
  const uint32_t sub_bytes = SubBlock<BS>::bytes(Hkv, D);
  uint64_t addr_a = 0, addr_b = 0;  // this lane's block address in the batches held (even, odd)
  uint32_t bad_bits = 0;            // bit 0 / 1: the even / odd batch has an invalid table entry
  struct Resolved {
    uint64_t addr;
    uint32_t bad;
  };
  auto resolve = [&](int batch) -> Resolved {
    Resolved out = {0, 0};
    const int t_lo = batch * kSubTiles;
    if (t_lo >= nt_wg) return out;
    const int t_hi = min(t_lo + kSubTiles, nt_wg);  // exclusive
    const int first_blk = BS < kTile ? t_lo * 2 : t_lo / TPB;
    const int last_blk = BS < kTile ? t_hi * 2 - 1 : (t_hi - 1) / TPB;
    const int nblk = min(last_blk + 1, n_blocks_seq) - first_blk;
    bool bad = false;
    if (lane < nblk) {
      const int id = p.table[(int64_t)s * p.table_stride + first_blk + lane];
      if ((uint32_t)id < (uint64_t)p.num_blocks) out.addr = p.block_list[id] + p.layer_off;
      else bad = true;
    }
    if (__any(bad)) {  // never dereference a bad id: flag it and leave the batch's tokens out
      if (bad) atomicCAS(p.status, 0, PIPELIVE_E_RANGE);
      out.bad = 1;
    }
    return out;
  };
  auto resolve_into_slot = [&](int batch) {
    Resolved rv = resolve(batch);
    // use the address here, so that the wait for its load is placed here (once per 32 tiles) and not
    // in front of every later read of it, where it would also wait for the tile copies in flight
    asm volatile("" : "+v"(rv.addr));
    // the flags are wave-uniform: kept in a scalar register, their tests cost no vector instruction
    if (batch & 1) {
      addr_b = rv.addr;
      bad_bits = __builtin_amdgcn_readfirstlane((bad_bits & 1u) | (rv.bad << 1));
    } else {
      addr_a = rv.addr;
      bad_bits = __builtin_amdgcn_readfirstlane((bad_bits & 2u) | rv.bad);
    }
  };
  // addresses of the two runs' sub-blocks of tile t (the same sub-block twice when SB = 32)
  auto tile_addr = [&](int t, uint64_t &a0, uint64_t &a1, bool &bad) {
    const int batch = t / kSubTiles, i = t % kSubTiles;
    const uint64_t my = (batch & 1) ? addr_b : addr_a;
    bad = (bad_bits >> (batch & 1)) & 1u;
    if (BS < kTile) {
      const int nblk = min((batch * kSubTiles + kSubTiles) * 2, n_blocks_seq) - batch * kSubTiles * 2;
      a0 = readlane64(my, 2 * i);
      a1 = (2 * i + 1 < nblk) ? readlane64(my, 2 * i + 1) : a0;
    } else {
      const int first_blk = batch * kSubTiles / TPB;
      a0 = a1 = readlane64(my, t / TPB - first_blk) + (uint64_t)((t % TPB) * sub_bytes);
    }
  };

  // ---- global -> LDS copy of one tile: PER_THREAD LDS-direct loads per wave, each writing the 64
  // consecutive 16-byte pieces [256 j + 64 w, +64) of the stage.  Which global piece a lane fetches
  // for its position (the run, the byte inside it, for V the un-permuted piece) is fixed per thread.
  constexpr int RC = St::KRUN / 16;  // 16-byte pieces per run
  uint32_t src_off[St::PER_THREAD];  // byte offset from the run's sub-block address (head included)
  bool second_half[St::PER_THREAD];  // the run belongs to the tile's second 16-token half (SB = 16 only)
#pragma unroll
  for (int j = 0; j < St::PER_THREAD; ++j) {
    const int ci = tid + 256 * j;  // position in the stage
    const int run = ci / RC, q = ci % RC;
    const int is_v = run / St::HALVES, half = run % St::HALVES;
    second_half[j] = half != 0;
    int off = q * 16;
    if (is_v) {
      const int d = q / St::CPR, pos = q % St::CPR;
      off = d * St::VROW + ((pos ^ St::swizzle(d)) * 16);
    }
    src_off[j] = (uint32_t)((is_v ? Hkv + g : g) * St::KRUN + off);
  }
  auto stage_load = [&](int t) {
    uint64_t a0, a1;
    bool bad;
    tile_addr(t, a0, a1, bad);
    if (__builtin_expect(bad, 0)) return;  // the batch is skipped by every wave: whatever the stage holds is never used
    lds_ptr st = (lds_ptr)lds + (t % kStages) * St::BYTES + w * 1024;
#pragma unroll
    for (int j = 0; j < St::PER_THREAD; ++j) {
      uint64_t base = a0;
      if (St::HALVES == 2) {
        // with RC >= 256 the half is a constant of j; otherwise it is a constant of the thread
        if (RC >= 256) base = ((256 * j / RC) % 2) ? a1 : a0;
        else base = second_half[j] ? a1 : a0;
      }
      __builtin_amdgcn_global_load_lds((global_u4)(base + src_off[j]), (lds_u4)(st + 4096 * j), 16, 0, 0);
    }
  };
  // The barrier that ends a tile: this wave's copies of the next tile have landed and its LDS reads of
  // the current one are done; the copies of the tile after next, issued a moment ago, may still be
  // in flight (a plain __syncthreads() would wait for them too and halve the prefetch distance).
  auto tile_barrier = [&](bool newest_tile_in_flight) {
    asm volatile("" ::: "memory");
    if (__builtin_expect(newest_tile_in_flight, 1)) {
      if (St::PER_THREAD == 4) __builtin_amdgcn_s_waitcnt(0x0074);  // vmcnt(4) lgkmcnt(0)
      else __builtin_amdgcn_s_waitcnt(0x0072);                      // vmcnt(2) lgkmcnt(0)
    } else {
      __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // MASK = false: every column sees the whole tile and every token of it is readable, so neither
  // the causal predicate nor the clearing of unreadable V is needed (all tiles below the diagonal).
  auto compute = [&](int tile, auto mask_tag) {
    constexpr bool MASK = decltype(mask_tag)::value;
    lds_ptr st = (lds_ptr)lds + (tile % kStages) * St::BYTES;
    const int j0 = tile * kTile;
    // The two 16-row score tiles of a 32-token KV tile take interleaved tokens: row m of tile T is
    // token 8 (m / 4) + 4 T + m % 4.  The accumulator rows a lane holds (4 qg + i of each tile) are then
    // the eight consecutive tokens 8 qg .. 8 qg + 7, so the V^T operand of the PV product is one
    // 16-byte LDS read per lane.
    // K operand: lane (row r of tile T, k-group qg) holds K[token][32c + 8qg .. +7]
    u32x4 kreg[2][NC];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      const int tok = 8 * (r >> 2) + 4 * T + (r & 3);
      const int hb = (SB == kTile) ? 0 : (tok / 16) * St::KRUN;
#pragma unroll
      for (int c = 0; c < NC; ++c)
        kreg[T][c] = *(lds_u4)(st + hb + ((qg + 4 * c) * SB + tok % SB) * 16);
    }
    // QK^T: the 2 NQ score tiles are independent accumulator chains, issued round-robin so that a
    // chain's next product never waits for its previous one
    f32x4 sc[NQ][2];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int T = 0; T < 2; ++T) sc[nq][T] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
        for (int T = 0; T < 2; ++T)
          sc[nq][T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kreg[T][c]), qreg[nq][c], sc[nq][T], 0, 0, 0);
    // V^T operand: lane (row d = 16c + r, k-group qg) holds V[d][tokens 8qg .. 8qg+7], one 16-byte
    // piece of the row.  All row blocks are requested here, behind the QK products, so that they
    // arrive while the softmax runs and the PV products can be issued back to back.
    const int vhalf = (SB == kTile) ? 0 : qg / 2;
    const int vpiece = (SB == kTile) ? qg : qg % 2;
    // swizzle(16 c + r) depends on r alone: the piece's position is a lane constant
    const int vlane = St::KBYTES + vhalf * St::VRUN + r * St::VROW + ((vpiece ^ St::swizzle(r)) * 16);
    u32x4 vreg[ND];
#pragma unroll
    for (int c = 0; c < ND; ++c) vreg[c] = *(lds_u4)(st + vlane + 16 * c * St::VROW);
    __builtin_amdgcn_sched_barrier(0);
    PTRACE(1);  // K read, QK, V requests

    // raw scores; the scale (positive) is applied inside the exponent: exp2(s * c - m)
    float x[NQ][8];
    float m_seen[NQ], mloc[NQ];
    bool grow = false;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      mloc[nq] = -INFINITY;
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v = sc[nq][T][i];
          if (MASK) {  // by predicate: unused slots may hold NaN
            const int j = j0 + 8 * qg + 4 * T + i;
            v = j <= p_col[nq] ? v : -INFINITY;
          }
          x[nq][4 * T + i] = v;
          mloc[nq] = fmaxf(mloc[nq], v);
        }
    }
    // column maxima across the four 16-lane rows (the scores that reach here are never NaN)
    if (NQ == 2) {
      rows_max_pair(mloc[0], mloc[1], mloc[0], mloc[1]);
    } else {
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) mloc[nq] = xor32_max(xor16_max(mloc[nq]));
    }
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      m_seen[nq] = max_no_nan(m[nq], mloc[nq] * p.scale_log2);
      grow |= m_seen[nq] - m[nq] > kLazyMaxStep;
    }
    // m is kept in the scaled domain and only follows the running maximum when that has grown by
    // more than 2^8: until then the weights are taken against the older reference (they stay below
    // 2^8, harmless in fp32 sums and in the bf16 pair) and the accumulators need no rescaling.  The
    // common factor cancels in O / l, so the result is the same softmax.
    if (__builtin_expect(__any(grow), 0)) {  // rare after the first tiles; -inf -> finite counts as growth
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        const float m_new = (m_seen[nq] - m[nq] > kLazyMaxStep) ? m_seen[nq] : m[nq];
        // a column that has seen nothing yet (m_new still -inf, masked tiles only) keeps its state
        const float alpha = (m_new == -INFINITY) ? 1.0f : fast_exp2(m[nq] - m_new);
        m[nq] = m_new;
        lacc[nq] *= alpha;
#pragma unroll
        for (int c = 0; c < ND; ++c) acc[c][nq] *= alpha;
      }
    }
    u32x4 ph[NQ], pl[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      const float neg_m = (MASK && m[nq] == -INFINITY) ? 0.f : -m[nq];
      float pv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        pv[i] = fast_exp2(__builtin_fmaf(x[nq][i], p.scale_log2, neg_m));  // exp2(-inf) = 0 for masked scores
      if (PAIR) {
        split_weights(pv, ph[nq], pl[nq]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) ph[nq][i] = pack_bf16_rne(pv[2 * i], pv[2 * i + 1]);
      }
    }
    PTRACE(2);  // softmax
    // V of tokens past the wave's readable range must be zero (0 * NaN is NaN)
    if (MASK) {
      u32x4 vmask;
      const int keep = min(max(n_kv - j0 - 8 * qg, 0), 8);  // readable tokens among the lane's eight
#pragma unroll
      for (int wd = 0; wd < 4; ++wd)
        vmask[wd] = keep >= 2 * wd + 2 ? ~0u : (keep == 2 * wd + 1 ? 0xFFFFu : 0u);
#pragma unroll
      for (int c = 0; c < ND; ++c) vreg[c] &= vmask;
    }
    // the denominators: sum over the tile's tokens of the same bf16 weights, as one more row of V^T
    // that holds ones (every row of the 16 x 16 result is that sum: no cross-lane reduction later)
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      lacc[nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, as_bf16x8(ph[nq]), lacc[nq], 0, 0, 0);
      if (PAIR) lacc[nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, as_bf16x8(pl[nq]), lacc[nq], 0, 0, 0);
    }
    // two row blocks at a time, first all products with the high halves of the weights, then all with
    // the low halves: an accumulator's two MFMAs are then four MFMAs apart and never wait for each other
#pragma unroll
    for (int c = 0; c < ND; c += 2) {
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
          acc[c + u][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vreg[c + u]), as_bf16x8(ph[nq]), acc[c + u][nq], 0, 0, 0);
      if (PAIR) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq)
            acc[c + u][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vreg[c + u]), as_bf16x8(pl[nq]), acc[c + u][nq], 0, 0, 0);
      }
    }
    PTRACE(5);  // V read + PV
  };

  // ---- the tile loop: copies are issued two tiles ahead of the arithmetic and need to have landed
  // one tile ahead, one barrier per tile.  Stage (t+2) % 3 was last read for tile t-1, which every
  // wave left before the barrier that ended iteration t-1.
  resolve_into_slot(0);
  resolve_into_slot(1);
  stage_load(0);
  if (nt_wg > 1) stage_load(1);
  tile_barrier(false);
  auto step = [&](int t, auto mask_tag) {
    PTRACE_START();
    const bool more = t + 2 < nt_wg;
    if (__builtin_expect(more, 1)) stage_load(t + 2);
    const int batch = t / kSubTiles;
    const bool bad = (bad_bits >> (batch & 1)) & 1u;
    // a quarter into a batch the slot of the batch before it is free: resolve the batch after it
    if (__builtin_expect(t % kSubTiles == 8 && batch >= 1, 0)) resolve_into_slot(batch + 1);
    PTRACE(0);  // issue of the copies
    if (__builtin_expect(t < nt_w && !bad, 1)) compute(t, mask_tag);
    PTRACE(6);
    tile_barrier(more);  // tile t+1 must be in LDS past the barrier; the copies of tile t+2 may still fly
    PTRACE(7);           // wait for the copies + barrier
  };
  // tiles wholly below the workgroup's first query need no mask in any wave; the few tiles on the
  // diagonal take the masked form (two loops, so that each form is generated once)
  const int nt_plain = min((n - qlen + wg_tok0 + 1) / kTile, nt_wg);
#pragma unroll 1
  for (int t = 0; t < nt_plain; ++t) step(t, std::false_type{});
#pragma unroll 1
  for (int t = nt_plain; t < nt_wg; ++t) step(t, std::true_type{});

  PTRACE_FLUSH(nt_wg);

  // ---- normalise and store: lane (qg, r) holds O[column r of block nq][16c + 4qg + i]
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const float lt = lacc[nq][0];
    if (!col_ok[nq]) continue;
    const int col = nq * 16 + r;
    const int ti = col / G, hh = col % G;
    const float inv = lt > 0.f ? 1.0f / lt : 0.f;
    const int64_t row = (int64_t)(q0 + tok0 + ti) * p.Hq + (int64_t)g * G + hh;
    if (PAIR) {  // fp32 output
      float *dst = (float *)p.out + row * D + 4 * qg;
#pragma unroll
      for (int c = 0; c < ND; ++c)
        *(float4 *)(dst + 16 * c) = make_float4(acc[c][nq][0] * inv, acc[c][nq][1] * inv, acc[c][nq][2] * inv,
                                                acc[c][nq][3] * inv);
    } else {
      uint16_t *dst = (uint16_t *)p.out + row * D + 4 * qg;
#pragma unroll
      for (int c = 0; c < ND; ++c) {
        const uint32_t w0 = f32_to_bf16_rne(acc[c][nq][0] * inv) | ((uint32_t)f32_to_bf16_rne(acc[c][nq][1] * inv) << 16);
        const uint32_t w1 = f32_to_bf16_rne(acc[c][nq][2] * inv) | ((uint32_t)f32_to_bf16_rne(acc[c][nq][3] * inv) << 16);
        *(uint2 *)(dst + 16 * c) = make_uint2(w0, w1);
      }
    }
  }
}

template <int D, int BS>
hipError_t launch_t(const PrefillParams &p, hipStream_t st) {
  if (p.out_dtype == PIPELIVE_OUT_F32)
    hipLaunchKernelGGL((attn_prefill_kernel<D, BS, kPrefillNQ, true>), dim3((unsigned)p.num_units), dim3(256), 0, st, p);
  else
    hipLaunchKernelGGL((attn_prefill_kernel<D, BS, kPrefillNQ, false>), dim3((unsigned)p.num_units), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace

#ifdef PIPELIVE_PREFILL_TRACE
extern "C" int pipelive_dev_prefill_trace(long long *out16) {
  return (int)hipMemcpyFromSymbol(out16, HIP_SYMBOL(g_prefill_trace), 16 * sizeof(long long));
}
#endif

hipError_t launch_attn_prefill(const PrefillParams &p, int D, int BS, hipStream_t st) {
#define X(d, b) \
  if (D == d && BS == b) return launch_t<d, b>(p, st);
  X(128, 16) X(128, 32) X(128, 64) X(128, 128) X(64, 16) X(64, 32) X(64, 64) X(64, 128)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace pipelive
