// Chunked-prefill paged attention for gfx950 (CDNA4, wave64, MFMA): the
// compute-bound stage (paper Sec. 2 "LLM Inference": prompt tokens are
// processed in parallel) over the same block-list KV layout as decode.
//
// Work unit = (sequence, KV head, block of QB consecutive query tokens), one
// per wave; the 4 waves of a workgroup take consecutive query blocks of the
// same (sequence, KV head), so they stream the same K/V tiles at about the
// same time and share them through the CU's cache.  A unit's NQ*16 score
// columns are its QB tokens x the G query heads of the KV head (column =
// token * G + head).  Per 32-token KV tile the wave computes S^T = K Q^T for
// all columns with the K operand fetched once, applies the causal mask by
// predicate, runs the online softmax per column and accumulates
// O^T += V^T P^T with P split into two bf16 terms, the V operand again fetched
// once for all columns.  The K operand of the next tile is in flight while the
// current one is computed; V is loaded at the top of its own tile and lands
// during the score/softmax phase.  NQ = 2 keeps the kernel at 250 VGPRs, so
// two waves share a SIMD and one's softmax overlaps the other's MFMAs.
#include "attn_common.h"

namespace pipelive {
namespace {

template <int D, int BS, int NQ>
__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(PrefillParams p) {
  constexpr int NC = D / 32, ND = D / 16;
  const int lane = threadIdx.x & 63;
  const int gw = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int r = lane & 15, qg = lane >> 4;
  const int G = p.G, Hkv = p.Hkv, S = p.num_seqs;
  const int QB = (NQ * 16) / G;  // query tokens per unit

  // ---- locate unit gw: units of sequence s = Hkv * ceil(q_len / QB), ordered (s, head, block)
  int s = -1, nqb = 0;
  int64_t rem = 0;
  {
    int64_t carry = 0;
    for (int base = 0; base < S && s < 0; base += 64) {
      const bool in = base + lane < S;
      int ql = 0;
      if (in) ql = p.q_offsets[base + lane + 1] - p.q_offsets[base + lane];
      const int nb = ql > 0 ? (ql + QB - 1) / QB : 0;
      const int units = nb * Hkv;
      const int inc = wave_inclusive_scan(units, lane);
      const uint64_t bal = __ballot(in && carry + inc > gw);  // first sequence whose range holds gw
      if (bal) {
        const int k = __ffsll((long long)bal) - 1;
        s = base + k;
        nqb = __builtin_amdgcn_readlane(nb, k);
        rem = gw - (carry + __builtin_amdgcn_readlane(inc, k) - __builtin_amdgcn_readlane(units, k));
      }
      carry += __builtin_amdgcn_readlane(inc, 63);
    }
  }
  if (s < 0) return;  // beyond the last unit
  // later query blocks attend to more tokens: hand them out first so the launch ends evenly
  const int g = (int)(rem / nqb), qb = nqb - 1 - (int)(rem % nqb);
  const int q0 = p.q_offsets[s], qlen = p.q_offsets[s + 1] - q0;
  int n = p.ctx[s];
  if (n > p.max_ctx) n = p.max_ctx;
  if (qlen > n) {  // more queries than cached tokens: flag and skip
    if (lane == 0) atomicCAS(p.status, 0, PIPELIVE_E_INVAL);
    return;
  }
  const int tok0 = qb * QB;                                // first query token of the unit
  const int ntok = min(QB, qlen - tok0);                   // query tokens in this unit
  const int pos0 = n - qlen + tok0;                        // position of the first query token
  const int p_max = pos0 + ntok - 1;                       // last position any column attends to

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
  const int p_min = pos0;  // smallest causal limit over the unit's columns (wave-uniform)

  f32x4 acc[ND][NQ];
  float m[NQ], l[NQ];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    m[nq] = -INFINITY;
    l[nq] = 0.f;
#pragma unroll
    for (int c = 0; c < ND; ++c) acc[c][nq] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  const int nt_all = (p_max + kTile) / kTile;  // KV tiles 0 .. nt_all-1 cover positions 0 .. p_max
  const int n_kv = p_max + 1;                  // tokens this unit may read

  auto compute = [&](KRegs<D> &kc, VRegs<D> &vc, int tile) {
    const int j0 = tile * kTile;
    const bool need_mask = j0 + kTile - 1 > p_min;  // some column cannot see the whole tile
    u32x4 ph[NQ], pl[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      f32x4 sc[2];
#pragma unroll
      for (int T = 0; T < 2; ++T) {
        sc[T] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NC; ++c)
          sc[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kc.k[T][c]), qreg[nq][c], sc[T], 0, 0, 0);
      }
      float x[8];
      float mloc = -INFINITY;
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = j0 + 16 * T + 4 * qg + i;
          const bool ok = !need_mask || j <= p_col[nq];  // by predicate: unused slots may hold NaN
          const float v = ok ? sc[T][i] * p.scale_log2 : -INFINITY;
          x[4 * T + i] = v;
          mloc = fmaxf(mloc, v);
        }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
      const float m_new = fmaxf(m[nq], mloc);
      // a column that sees nothing of this tile keeps its state (m_new may still be -inf only before
      // its first visible token, which is in tile 0 for every column)
      const float alpha = (m_new == -INFINITY) ? 1.0f : fast_exp2(m[nq] - m_new);
      float pv[8], psum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        pv[i] = (x[i] == -INFINITY) ? 0.f : fast_exp2(x[i] - m_new);
        psum += pv[i];
      }
      l[nq] = l[nq] * alpha + psum;
      m[nq] = m_new;
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int c = 0; c < ND; ++c) acc[c][nq] *= alpha;
      }
      split_weights(pv, ph[nq], pl[nq]);
    }
    // V of tokens past the readable range must be zero (0 * NaN is NaN)
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      const int nv = kc.nvalid[T];
      if (nv < 16) {
        const int keep = min(max(nv - 4 * qg, 0), 4);
        const uint64_t mask = keep >= 4 ? ~0ull : ((1ull << (16 * keep)) - 1ull);
#pragma unroll
        for (int c = 0; c < ND; ++c) {
          vc.v[c][T].x &= (uint32_t)mask;
          vc.v[c][T].y &= (uint32_t)(mask >> 32);
        }
      }
    }
#pragma unroll
    for (int c = 0; c < ND; ++c) {
      const bf16x8 va = as_bf16x8((u32x4){vc.v[c][0].x, vc.v[c][0].y, vc.v[c][1].x, vc.v[c][1].y});
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        acc[c][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, as_bf16x8(ph[nq]), acc[c][nq], 0, 0, 0);
        acc[c][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, as_bf16x8(pl[nq]), acc[c][nq], 0, 0, 0);
      }
    }
  };

  for (int sub = 0; sub < nt_all; sub += kSubTiles) {
    const int nt = min(nt_all - sub, kSubTiles);
    constexpr int TPB = BS >= kTile ? BS / kTile : 1;  // tiles per block (a 16-token block is half a tile)
    const int first_blk = BS < kTile ? sub * 2 : sub / TPB;
    const int last_blk = BS < kTile ? (sub + nt) * 2 - 1 : (sub + nt - 1) / TPB;
    const int nblk = min(last_blk + 1, (n_kv + BS - 1) / BS) - first_blk;
    uint64_t my_addr = 0;
    bool bad = false;
    if (lane < nblk) {
      const int id = p.table[(int64_t)s * p.table_stride + first_blk + lane];
      if ((uint32_t)id < (uint64_t)p.num_blocks) my_addr = p.block_list[id] + p.layer_off;
      else bad = true;
    }
    if (__any(bad)) {
      if (bad) atomicCAS(p.status, 0, PIPELIVE_E_RANGE);
      continue;
    }
    const uint32_t sub_bytes = SubBlock<BS>::bytes(Hkv, D);
    auto addr_of = [&](int i, uint64_t &a0, uint64_t &a1, int &nv0, int &nv1) {
      const int t0 = (sub + i) * kTile;
      if (BS < kTile) {
        a0 = readlane64(my_addr, 2 * i);
        a1 = (2 * i + 1 < nblk) ? readlane64(my_addr, 2 * i + 1) : a0;
      } else {  // the tile's 32-token sub-block inside its block
        a0 = a1 = readlane64(my_addr, (sub + i) / TPB - first_blk) +
                  (uint64_t)(((sub + i) % TPB) * sub_bytes);
      }
      nv0 = min(n_kv - t0, 16);
      nv1 = min(n_kv - t0 - 16, 16);
    };
    // Two waves per SIMD overlap each other's loads and arithmetic; K of the next tile is
    // requested before the current tile is computed, V is fetched tile by tile.
    KRegs<D> kc, kn;
    VRegs<D> vc;
    uint64_t a0, a1;
    int nv0, nv1;
    addr_of(0, a0, a1, nv0, nv1);
    load_k<D, BS>(kc, a0, a1, nv0, nv1, g, r, qg);
#pragma unroll 1
    for (int i = 0; i < nt; ++i) {
      load_v<D, BS>(vc, a0, a1, g, Hkv, r, qg);
      if (i + 1 < nt) {
        addr_of(i + 1, a0, a1, nv0, nv1);
        load_k<D, BS>(kn, a0, a1, nv0, nv1, g, r, qg);
      }
      compute(kc, vc, sub + i);
      kc = kn;
    }
  }

  // ---- normalise and store: lane (qg, r) holds O[column r of block nq][16c + 4qg + i]
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    float lt = l[nq];
    lt += __shfl_xor(lt, 16);
    lt += __shfl_xor(lt, 32);
    if (!col_ok[nq]) continue;
    const int col = nq * 16 + r;
    const int ti = col / G, hh = col % G;
    const float inv = lt > 0.f ? 1.0f / lt : 0.f;
    const int64_t row = (int64_t)(q0 + tok0 + ti) * p.Hq + (int64_t)g * G + hh;
    if (p.out_dtype == PIPELIVE_OUT_F32) {
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
  const unsigned grid = (unsigned)((p.num_waves + 3) / 4);
  hipLaunchKernelGGL((attn_prefill_kernel<D, BS, kPrefillNQ>), dim3(grid), dim3(256), 0, st, p);
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
