// Chunked-prefill paged attention for gfx950 (CDNA4, wave64, MFMA): the
// compute-bound stage (paper Sec. 2 "LLM Inference": prompt tokens are
// processed in parallel) over the same block-list KV layout as decode.
//
// Work unit = (sequence, KV head, block of 4*QB consecutive query tokens); wave
// w of the workgroup that takes it owns the QB tokens [w*QB, (w+1)*QB) of the
// block.  A wave's NQ*16 score columns are its QB tokens x the G query heads of
// the KV head (column = token * G + head).  The kernel is persistent: as many
// workgroups as the device holds at once.  The units are dealt to work lists
// by KV head, one list per XCD, so that the query blocks of a (sequence, KV
// head) pair share one L2; a workgroup takes a unit of its XCD's list first
// and then draws units from that list's ticket counter (from the next list's
// once its own is used up), and while it works on one unit it already draws,
// searches and resolves the next (one step per tile, the loads going straight
// into a few LDS rows), so that a unit starts with its block addresses in hand.  For a unit the workgroup walks the 32-token KV
// tiles that its last query may see; each tile's K and V of the KV head (two
// contiguous runs of the in-block layout) are copied once from global memory
// into a ring of three LDS stages by LDS-direct loads (global_load_lds_dwordx4:
// no staging registers), issued two tiles ahead of the arithmetic, and all
// four waves take their MFMA operands from there.  Per tile a wave computes
// S^T = K Q^T for its columns, applies the causal mask by predicate, runs the
// online softmax per column and accumulates O^T += V^T P^T (P as a pair of bf16
// terms for fp32 output, as one for bf16 output).  A wave whose queries cannot
// see a tile, or that has no queries at all, still takes part in the copies and
// barriers.
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
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, qg = lane >> 4;
  const int G = p.G, Hkv = p.Hkv, S = p.num_seqs;
  const int QB = (NQ * 16) / G;  // query tokens per wave
  const int WB = 4 * QB;         // query tokens per workgroup
  const int grid = gridDim.x;
  // Work lists: the units are dealt to NL lists by KV head (list x holds heads x, x + NL, ...), each with a ticket
  // counter of its own.  A workgroup starts on list blockIdx.x mod NL - with NL = 8 that is the XCD the hardware
  // places it on (workgroups go to the XCDs in turn) - so the query blocks of one (sequence, KV head) pair run
  // on one XCD and its L2 fetches the pair's K and V once; when its list is used up a workgroup moves on to
  // the next one.  Every list holds the same sequences, so the lists are equally long.
  const int NL = p.n_lists, HPL = Hkv / NL;
  const int gpl = grid / NL;  // workgroups per list (the host makes the grid a multiple of NL)
  __shared__ int mailbox;  // the ticket that thread 0 drew, for the other waves

  // ---- work units of a list: units of sequence s = (Hkv / NL) * ceil(q_len / WB), ordered (s, head, block); the
  // later query blocks of a sequence attend to more tokens and come first.  The lanes that scan the
  // sequences also fetch what the unit needs of its sequence (no second round trip after the search).
  struct Unit {
    int s, g, wb, q0, qlen, n;  // s < 0: no such unit
  };
  struct Scan {
    int qa, ql, cx;  // q_offsets[i], q_len and context length of sequence base + lane
  };
  auto scan_issue = [&](int base) -> Scan {
    Scan sc = {0, 0, 0};
    if (base + lane < S) {
      sc.qa = p.q_offsets[base + lane];
      sc.ql = p.q_offsets[base + lane + 1] - sc.qa;
      sc.cx = p.ctx[base + lane];
    }
    return sc;
  };
  auto locate = [&](int unit, Scan first, int list) -> Unit {
    Unit u = {-1, 0, 0, 0, 0, 0};
    int carry = 0;  // the host keeps the number of units below 2^30
    for (int base = 0; base < S && u.s < 0; base += 64) {
      const Scan sc = base == 0 ? first : scan_issue(base);
      const int nb = sc.ql > 0 ? (sc.ql + WB - 1) / WB : 0;
      const int units = nb * HPL;
      const int inc = wave_inclusive_scan(units, lane);
      const uint64_t bal = __ballot(carry + inc > unit);  // first sequence whose range holds it
      if (bal) {
        const int k = __ffsll((long long)bal) - 1;
        const uint32_t nwb = (uint32_t)__builtin_amdgcn_readlane(nb, k);
        const uint32_t rem =
            (uint32_t)(unit - (carry + __builtin_amdgcn_readlane(inc, k) - __builtin_amdgcn_readlane(units, k)));
        u.s = base + k;
        u.g = list + NL * (int)(rem / nwb);
        u.wb = (int)(nwb - 1 - rem % nwb);
        u.q0 = __builtin_amdgcn_readlane(sc.qa, k);
        u.qlen = __builtin_amdgcn_readlane(sc.ql, k);
        // a context beyond max_ctx cannot be truncated here (the queries' positions hang on it): the
        // unit is marked invalid (n = -1 < q_len) and skipped with PIPELIVE_E_RANGE
        const int cx = __builtin_amdgcn_readlane(sc.cx, k);
        u.n = cx > p.max_ctx ? -1 : cx;
      }
      carry += __builtin_amdgcn_readlane(inc, 63);
    }
    return u;
  };
  // tiles and blocks that the workgroup of a unit walks
  auto unit_tiles = [&](const Unit &u) { return (u.n - u.qlen + min((u.wb + 1) * WB, u.qlen) - 1 + kTile) / kTile; };
  auto unit_blocks = [&](const Unit &u) { return (u.n - u.qlen + min((u.wb + 1) * WB, u.qlen) + BS - 1) / BS; };

  // ---- block addresses of a unit's first 32 tiles (one block per lane), in two dependent loads
  constexpr int TPB = BS >= kTile ? BS / kTile : 1;  // tiles per block (a 16-token block is half a tile)
  auto batch_blocks = [&](int batch, int nt, int nblocks) {  // blocks of the batch that exist: [first, first + count)
    const int t_lo = batch * kSubTiles, t_hi = min(t_lo + kSubTiles, nt);
    const int first = BS < kTile ? t_lo * 2 : t_lo / TPB;
    const int last = BS < kTile ? t_hi * 2 - 1 : (t_hi - 1) / TPB;
    return min(last + 1, nblocks) - first;
  };
  auto table_issue = [&](const Unit &u) -> int {  // block id of this lane's block in batch 0, -1: none
    const int nblk = batch_blocks(0, unit_tiles(u), unit_blocks(u));
    return lane < nblk ? p.table[(int64_t)u.s * p.table_stride + lane] : -1;
  };
  auto list_issue = [&](const Unit &u, int id, uint32_t &bad) -> uint64_t {
    const int nblk = batch_blocks(0, unit_tiles(u), unit_blocks(u));
    const bool have = lane < nblk;
    const bool ok = have && (uint32_t)id < (uint64_t)p.num_blocks;
    const bool lane_bad = have && !ok;
    bad = __any(lane_bad) ? 1u : 0u;  // never dereference a bad id: flag it and leave the batch's tokens out
    if (lane_bad) atomicCAS(p.status, 0, PIPELIVE_E_RANGE);
    return ok ? p.block_list[id] : 0;
  };

  // ---- the next unit is drawn, searched and resolved one step per tile of the current unit, so
  // that its memory round trips (ticket, sequence scan, table, block list) hide behind arithmetic.
  // The steps' loads are LDS-direct loads into a few rows of LDS per wave: nothing is pending in a
  // vector register while the tile loop runs (the compiler guards every reuse of a register with a
  // pending load by a wait for ALL memory operations, the tile copies in flight included).  They are
  // older than the tile copies issued after them, so the wait of the tile's barrier covers them and
  // the next iteration reads the rows.  Only the ticket comes back in a register; thread 0 passes it
  // on at the end of the same iteration.  Every wave runs the same steps; `cs` is uniform over the
  // workgroup.
  constexpr int kChainReady = 5, kChainEnd = 6;
  constexpr int kRows = 6;  // q_offsets[i], q_offsets[i + 1], ctx[i], table entry, block list entry (two halves)
  __shared__ uint32_t chain_rows[4 * kRows * 64];
  typedef uint32_t __attribute__((address_space(3))) *lds_u1;
  typedef const uint32_t __attribute__((address_space(1))) *global_u1;
  auto row = [&](int k) { return chain_rows + (w * kRows + k) * 64; };
  auto row_fetch = [&](int k, const void *lane_src) {  // lane i: 4 bytes from its address -> row k, word i
    __builtin_amdgcn_global_load_lds((global_u1)lane_src, (lds_u1)row(k), 4, 0, 0);
  };
  int cs = kChainEnd;
  int c_ticket = 0;  // thread 0: the ticket it drew
  int c_unit = -1;
  int c_list = __builtin_amdgcn_readfirstlane((int)(blockIdx.x % (unsigned)NL));  // the list tickets are drawn from
  int c_spent = 0;                                                                   // lists found used up
  Unit nxt = {-1, 0, 0, 0, 0, 0};
  uint64_t nxt_addr = 0;
  uint32_t nxt_bad = 0;
  // what is uniform goes through readfirstlane, so that it provably lives in scalar registers
  auto uniform_unit = [&](const Unit &u) -> Unit {
    Unit o;
    o.s = __builtin_amdgcn_readfirstlane(u.s);
    o.g = __builtin_amdgcn_readfirstlane(u.g);
    o.wb = __builtin_amdgcn_readfirstlane(u.wb);
    o.q0 = __builtin_amdgcn_readfirstlane(u.q0);
    o.qlen = __builtin_amdgcn_readfirstlane(u.qlen);
    o.n = __builtin_amdgcn_readfirstlane(u.n);
    return o;
  };
  // the list at hand is used up: on to the next one (step 0 draws again), or the end after the last
  auto list_spent = [&]() -> int {
    c_spent = __builtin_amdgcn_readfirstlane(c_spent + 1);
    c_list = __builtin_amdgcn_readfirstlane(c_list + 1 == NL ? 0 : c_list + 1);
    return c_spent < NL ? 0 : kChainEnd;
  };
  // Before the tile's arithmetic: take up what the step before fetched, fetch for the next one.
  auto chain_step = [&]() {
    int next_cs = cs;
    switch (cs) {
      case 0:  // draw a ticket
        if (tid == 0) c_ticket = atomicAdd(p.ticket + c_list, 1);
        break;  // chain_pass_on() moves on
      case 1:  // the ticket is in the mailbox: fetch the first 64 sequences' offsets and lengths
        c_unit = gpl + __builtin_amdgcn_readfirstlane(mailbox);
        if (c_unit >= p.num_units) {
          next_cs = list_spent();
        } else {
          if (lane < S) {
            row_fetch(0, p.q_offsets + lane);
            row_fetch(1, p.q_offsets + lane + 1);
            row_fetch(2, p.ctx + lane);
          }
          next_cs = 2;
        }
        break;
      case 2: {  // search the unit, fetch the table entries of its first batch (one block per lane)
        Scan sc = {0, 0, 0};
        if (lane < S) {
          sc.qa = (int)row(0)[lane];
          sc.ql = (int)row(1)[lane] - sc.qa;
          sc.cx = (int)row(2)[lane];
        }
        nxt = uniform_unit(locate(c_unit, sc, c_list));
        if (nxt.s < 0) {
          next_cs = list_spent();  // beyond the list's last unit: so is every later ticket of it
        } else if (nxt.qlen > nxt.n) {
          next_cs = kChainReady;  // invalid unit: nothing to resolve
        } else {
          if (lane < batch_blocks(0, unit_tiles(nxt), unit_blocks(nxt)))
            row_fetch(3, p.table + (int64_t)nxt.s * p.table_stride + lane);
          next_cs = 3;
        }
        break;
      }
      case 3: {  // check the entries, fetch their block list entries
        const bool have = lane < batch_blocks(0, unit_tiles(nxt), unit_blocks(nxt));
        const uint32_t id = have ? row(3)[lane] : 0u;
        const bool lane_bad = have && !(id < (uint64_t)p.num_blocks);
        nxt_bad = __builtin_amdgcn_readfirstlane(__any(lane_bad) ? 1u : 0u);
        if (lane_bad) atomicCAS(p.status, 0, PIPELIVE_E_RANGE);  // never dereferenced: the batch's tokens are left out
        if (have && !lane_bad) {
          row_fetch(4, (const uint32_t *)(p.block_list + id));
          row_fetch(5, (const uint32_t *)(p.block_list + id) + 1);
        }
        next_cs = 4;
        break;
      }
      case 4: {
        const bool have = lane < batch_blocks(0, unit_tiles(nxt), unit_blocks(nxt));
        const bool ok = have && row(3)[lane] < (uint64_t)p.num_blocks;
        nxt_addr = ok ? (((uint64_t)row(5)[lane] << 32) | row(4)[lane]) + p.layer_off : 0;
        next_cs = kChainReady;
        break;
      }
      default:
        break;
    }
    cs = __builtin_amdgcn_readfirstlane(next_cs);
  };
  // After the tile's arithmetic, before its barrier (which publishes the mailbox).
  auto chain_pass_on = [&]() {
    if (cs == 0) {
      if (tid == 0) mailbox = c_ticket;
      cs = __builtin_amdgcn_readfirstlane(1);
    }
  };

  // the first unit is the workgroup's own index; its search and addresses are waited for
  Unit cur = uniform_unit(locate((int)blockIdx.x / NL, scan_issue(0), c_list));
  uint64_t cur_addr = 0;
  uint32_t cur_bad = 0;
  if (cur.s >= 0 && cur.qlen <= cur.n) {
    const uint64_t e = list_issue(cur, table_issue(cur), cur_bad);
    cur_addr = e ? e + p.layer_off : 0;
    cur_bad = __builtin_amdgcn_readfirstlane(cur_bad);
  }

  // kept opaque so that it stays in registers instead of being rebuilt from scalars in every tile
  u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  asm volatile("" : "+v"(ones_bits));
  const bf16x8 ones = as_bf16x8(ones_bits);

  // ---- global -> LDS copy of one tile: PER_THREAD LDS-direct loads per wave, each writing the 64
  // consecutive 16-byte pieces [256 j + 64 w, +64) of the stage.  Which global piece a lane fetches
  // for its position (the run, the byte inside it, for V the un-permuted piece) is fixed per thread;
  // the KV head's offset joins the (scalar) sub-block address.
  constexpr int RC = St::KRUN / 16;  // 16-byte pieces per run
  uint32_t src_off[St::PER_THREAD];  // byte offset from the sub-block address of head 0's K run
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
    src_off[j] = (uint32_t)((is_v ? Hkv : 0) * St::KRUN + off);
  }

  while (cur.s >= 0) {
  // (uniform by construction; said again so that everything derived from them is scalar)
  const int s = __builtin_amdgcn_readfirstlane(cur.s), g = __builtin_amdgcn_readfirstlane(cur.g);
  const int wb = __builtin_amdgcn_readfirstlane(cur.wb), q0 = __builtin_amdgcn_readfirstlane(cur.q0);
  const int qlen = __builtin_amdgcn_readfirstlane(cur.qlen), n = __builtin_amdgcn_readfirstlane(cur.n);
  cs = 0;  // start drawing the unit after this one
  if (qlen > n) {  // more queries than cached tokens, or a context beyond max_ctx (n = -1): flag and skip
    if (tid == 0) atomicCAS(p.status, 0, n < 0 ? PIPELIVE_E_RANGE : PIPELIVE_E_INVAL);
  } else {
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
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    m[nq] = -INFINITY;
    lacc[nq] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < ND; ++c) acc[c][nq] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  // ---- block addresses, resolved 32 tiles at a time, one block per lane; batch 0 came with the unit,
  // each later batch is resolved early so that the copies never wait for it
  const int n_blocks_seq = (wg_nkv + BS - 1) / BS;
  const uint32_t sub_bytes = SubBlock<BS>::bytes(Hkv, D);
  const uint64_t head_off = (uint64_t)g * St::KRUN;  // the KV head's K run inside a sub-block
  uint64_t addr_a = cur_addr, addr_b = 0;  // this lane's block address in the batches held (even, odd)
  // bit 0 / 1: the even / odd batch has an invalid table entry (wave-uniform: kept in a scalar
  // register, the tests cost no vector instruction)
  uint32_t bad_bits = __builtin_amdgcn_readfirstlane(cur_bad);
  struct Resolved {
    uint64_t addr;
    uint32_t bad;
  };
  auto resolve = [&](int batch) -> Resolved {
    Resolved out = {0, 0};
    if (batch * kSubTiles >= nt_wg) return out;
    const int first_blk = BS < kTile ? batch * kSubTiles * 2 : batch * kSubTiles / TPB;
    const int nblk = batch_blocks(batch, nt_wg, n_blocks_seq);
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
      a0 = readlane64(my, 2 * i) + head_off;
      a1 = (2 * i + 1 < nblk) ? readlane64(my, 2 * i + 1) + head_off : a0;
    } else {
      const int first_blk = batch * kSubTiles / TPB;
      a0 = a1 = readlane64(my, t / TPB - first_blk) + (uint64_t)((t % TPB) * sub_bytes) + head_off;
    }
  };

  auto stage_load = [&](int t) -> bool {  // false: nothing was issued
    uint64_t a0, a1;
    bool bad;
    tile_addr(t, a0, a1, bad);
    if (__builtin_expect(bad, 0)) return false;  // the batch is skipped by every wave: whatever the stage holds is never used
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
    return true;
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
    // the wave asks for issue priority while it feeds the MFMA pipe (QK products here, PV products
    // below) and gives it back for the softmax: the CU's other workgroup then fills the gaps with its
    // vector instructions instead of delaying these (measured: 2-3 % on long chunks)
    __builtin_amdgcn_s_setprio(2);
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
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);

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
    __builtin_amdgcn_s_setprio(2);
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
    __builtin_amdgcn_s_setprio(0);
  };

  // ---- the tile loop: copies are issued two tiles ahead of the arithmetic and need to have landed
  // one tile ahead, one barrier per tile.  Stage (t+2) % 3 was last read for tile t-1, which every
  // wave left before the barrier that ended iteration t-1.
  resolve_into_slot(1);
  stage_load(0);
  if (nt_wg > 1) stage_load(1);
  tile_barrier(false);
  auto step = [&](int t, auto mask_tag) {
    // (its loads are older than this tile's copies: the barrier's count still holds; the test keeps
    // the chain's code and its waits off the path of the tiles that have nothing left to step)
    const bool stepping = __builtin_amdgcn_readfirstlane(cs) < kChainReady;
    if (__builtin_expect(stepping, 0)) chain_step();
    bool more = t + 2 < nt_wg;
    if (__builtin_expect(more, 1)) more = stage_load(t + 2);
    const int batch = t / kSubTiles;
    const bool bad = (bad_bits >> (batch & 1)) & 1u;
    // a quarter into a batch the slot of the batch before it is free: resolve the batch after it
    if (__builtin_expect(t % kSubTiles == 8 && batch >= 1, 0)) resolve_into_slot(batch + 1);
    if (__builtin_expect(t < nt_w && !bad, 1)) compute(t, mask_tag);
    if (__builtin_expect(stepping, 0)) chain_pass_on();
    tile_barrier(more);  // tile t+1 must be in LDS past the barrier; the copies of tile t+2 may still fly
  };
  // tiles wholly below the workgroup's first query need no mask in any wave; the few tiles on the
  // diagonal take the masked form (two loops, so that each form is generated once)
  const int nt_plain = min((n - qlen + wg_tok0 + 1) / kTile, nt_wg);
#pragma unroll 1
  for (int t = 0; t < nt_plain; ++t) step(t, std::false_type{});
#pragma unroll 1
  for (int t = nt_plain; t < nt_wg; ++t) step(t, std::true_type{});


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
        const uint32_t w0 = pack_bf16_rne(acc[c][nq][0] * inv, acc[c][nq][1] * inv);  // one conversion per pair
        const uint32_t w1 = pack_bf16_rne(acc[c][nq][2] * inv, acc[c][nq][3] * inv);
        *(uint2 *)(dst + 16 * c) = make_uint2(w0, w1);
      }
    }
  }
  }  // a valid unit

  // whatever is left of the next unit's steps (short units): now with their latency in the open
  while (cs < kChainReady) {
    chain_step();
    chain_pass_on();
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): the rows have landed, the mailbox is written
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  if (cs == kChainReady) {
    cur = nxt;
    cur_addr = nxt_addr;
    cur_bad = nxt_bad;
  } else {
    cur.s = -1;
  }
  }  // units of this workgroup

  // the last workgroup to leave re-arms both counters for the next launch
  if (tid == 0) {
    const int done = atomicAdd(p.finished, 1);
    if (done == grid - 1) {
      for (int i = 0; i < NL; ++i) atomicExch(p.ticket + i, 0);
      atomicExch(p.finished, 0);
    }
  }
}

// Persistent launch: as many workgroups as the device holds at once (never more than there are
// units); each takes a unit of its list first and draws the following ones from the lists' ticket
// counters.
template <int D, int BS, bool PAIR>
int resident_workgroups() {
  static int cached = 0;
  if (cached == 0) {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, attn_prefill_kernel<D, BS, kPrefillNQ, PAIR>, 256, 0) !=
            hipSuccess ||
        nb < 1)
      nb = 1;
    cached = nb * device_cu_count();
  }
  return cached;
}

// One list per XCD when the KV heads and the grid divide by the XCD count, else one list for all.  num_units
// comes in as the bound over all heads and leaves as the bound of one list.
PrefillParams with_lists(PrefillParams p, int grid) {
  p.n_lists = (p.Hkv % kPrefillLists == 0 && grid % kPrefillLists == 0) ? kPrefillLists : 1;
  p.num_units /= p.n_lists;
  return p;
}

template <int D, int BS>
hipError_t launch_t(const PrefillParams &p, hipStream_t st) {
  if (p.out_dtype == PIPELIVE_OUT_F32) {
    const int grid = p.num_units < resident_workgroups<D, BS, true>() ? p.num_units : resident_workgroups<D, BS, true>();
    hipLaunchKernelGGL((attn_prefill_kernel<D, BS, kPrefillNQ, true>), dim3((unsigned)grid), dim3(256), 0, st,
                       with_lists(p, grid));
  } else {
    const int grid = p.num_units < resident_workgroups<D, BS, false>() ? p.num_units : resident_workgroups<D, BS, false>();
    hipLaunchKernelGGL((attn_prefill_kernel<D, BS, kPrefillNQ, false>), dim3((unsigned)grid), dim3(256), 0, st,
                       with_lists(p, grid));
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_prefill(const PrefillParams &p, int D, int BS, hipStream_t st) {
#define X(d, b) \
  if (D == d && BS == b) return launch_t<d, b>(p, st);
  X(128, 16) X(128, 32) X(128, 64) X(128, 128) X(64, 16) X(64, 32) X(64, 64) X(64, 128)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace pipelive
