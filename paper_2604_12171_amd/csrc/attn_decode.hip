// Paged-attention decode for gfx950 (CDNA4, wave64, MFMA).
//
// Work partition.  The unit of work is a *tile*: 32 consecutive tokens of one
// (sequence, KV head).  All tiles of the batch, ordered by (sequence, KV head,
// position), form one flat range that is cut into equal shares, one per wave,
// so every wave streams the same number of KV bytes whatever the mix of
// context lengths.  A share may cross (sequence, head) boundaries; a pair that
// lies entirely inside one share is finished by that wave; a pair cut by a
// share boundary leaves partial (m, l, O) records (at most two per wave) that
// a small merge kernel combines in share order.  The partition and the merge
// order are pure functions of the context lengths and of the share size, never
// of addresses or of timing.
//
// Data path.  Per tile a wave fetches two 16-token K tiles and the matching
// V^T tiles straight from HBM into MFMA operand registers (the in-block layout
// makes every load instruction cover whole contiguous cache lines), double
// buffered: the loads of tile i+1 are in flight while tile i is computed.
// S^T = K Q^T uses v_mfma_f32_16x16x32_bf16 (rows = tokens, columns = the G
// query heads sharing the KV head, padded to 16); the online softmax runs on
// the accumulator layout; O^T += V^T P^T uses the same MFMA with P split into
// two bf16 terms so nothing is lost against fp32 weights.  The S^T
// accumulator layout (a lane holds 4 consecutive tokens of one head) is
// exactly the B-operand layout of the PV product, so scores never cross lanes
// except for the running max.
//
// Paper: Sec. 2 "LLM Inference" (decode re-reads the cached K/V: memory
// bound), Sec. 5.1 (block addresses are resolved through the block table and
// the block list at kernel time; blocks are not contiguous).
#include "attn_common.h"

namespace pipelive {

namespace {


__device__ __forceinline__ int tiles_of(int n, int max_ctx) {
  if (n > max_ctx) n = max_ctx;
  return n <= 0 ? 0 : (n + kTile - 1) / kTile;
}

// S^T = K Q^T, online softmax update; returns the P^T operand as two bf16 terms.
template <int D>
__device__ __forceinline__ void qk_softmax(const KRegs<D> &t, const bf16x8 (&qreg)[D / 32],
                                           f32x4 (&acc)[D / 16], float &m, float &l, float scale_log2,
                                           int qg, u32x4 &ph, u32x4 &pl) {
  constexpr int NC = D / 32, ND = D / 16;
  f32x4 sc[2];
#pragma unroll
  for (int T = 0; T < 2; ++T) {
    sc[T] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < NC; ++c)
      sc[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(t.k[T][c]), qreg[c], sc[T], 0, 0, 0);
  }
  // scale; mask by predicate, never by arithmetic: unused slots may hold NaN
  float x[8];
  float mloc = -INFINITY;
#pragma unroll
  for (int T = 0; T < 2; ++T)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = (4 * qg + i) < t.nvalid[T];
      const float v = ok ? sc[T][i] * scale_log2 : -INFINITY;
      x[4 * T + i] = v;
      mloc = fmaxf(mloc, v);
    }
  mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
  mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
  const float m_new = fmaxf(m, mloc);  // finite: the tile holds at least one valid token
  const float alpha = fast_exp2(m - m_new);
  float pv[8], psum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pv[i] = fast_exp2(x[i] - m_new);
    psum += pv[i];
  }
  l = l * alpha + psum;
  m = m_new;
  if (__any(alpha != 1.0f)) {
#pragma unroll
    for (int c = 0; c < ND; ++c) acc[c] *= alpha;
  }
  // P^T operand: slots 0..3 = half 0 tokens 4qg+i, slots 4..7 = half 1; two bf16 terms
  split_weights(pv, ph, pl);
}

// O^T += V^T P^T.  nv0/nv1: valid tokens of the two halves (as recorded by load_k).
template <int D>
__device__ __forceinline__ void pv_accumulate(VRegs<D> &t, int nv0, int nv1, u32x4 ph, u32x4 pl,
                                              f32x4 (&acc)[D / 16], int qg) {
  constexpr int ND = D / 16;
  // V of masked tokens must be zero (0 * NaN is NaN): partial halves only
#pragma unroll
  for (int T = 0; T < 2; ++T) {
    const int nv = T ? nv1 : nv0;
    if (nv < 16) {
      const int keep = min(max(nv - 4 * qg, 0), 4);
      const uint64_t mask = keep >= 4 ? ~0ull : ((1ull << (16 * keep)) - 1ull);
#pragma unroll
      for (int c = 0; c < ND; ++c) {
        t.v[c][T].x &= (uint32_t)mask;
        t.v[c][T].y &= (uint32_t)(mask >> 32);
      }
    }
  }
#pragma unroll
  for (int c = 0; c < ND; ++c) {
    const bf16x8 va = as_bf16x8((u32x4){t.v[c][0].x, t.v[c][0].y, t.v[c][1].x, t.v[c][1].y});
    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, as_bf16x8(ph), acc[c], 0, 0, 0);
    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, as_bf16x8(pl), acc[c], 0, 0, 0);
  }
}

// ---- the partition of the flat tile range [0, total) into per-wave shares.
// Fixed mode (tiles_per_wave > 0): wave w owns [w*Q, (w+1)*Q).
// Balanced mode: total = nw*Qf + rem; the first `rem` waves own Qf+1 tiles, the
// others Qf, so no wave carries more than one tile above the mean.
// The host admits only launches whose tile count is below 2^31, so every
// quotient here is a 32-bit division (a 64-bit one is a long emulated sequence
// that sits in front of a wave's first load).
__device__ __forceinline__ uint32_t div32(int64_t a, int64_t b) { return (uint32_t)a / (uint32_t)b; }
__device__ __forceinline__ int64_t share_start(const AttnParams &p, int64_t total, int64_t w) {
  if (p.tiles_per_wave > 0) return w * p.tiles_per_wave;
  const int64_t qf = div32(total, p.num_waves), rem = total - qf * p.num_waves;
  return w * qf + (w < rem ? w : rem);
}
__device__ __forceinline__ int64_t share_wave(const AttnParams &p, int64_t total, int64_t t) {
  if (p.tiles_per_wave > 0) return div32(t, p.tiles_per_wave);
  const int64_t qf = div32(total, p.num_waves), rem = total - qf * p.num_waves;
  const int64_t big = rem * (qf + 1);
  if (t < big) return div32(t, qf + 1);
  return rem + div32(t - big, qf);  // qf > 0 here because t < total
}

template <int D, int BS>
__global__ __launch_bounds__(256, 2) void attn_decode_kernel(AttnParams p) {
  constexpr int NC = D / 32, ND = D / 16;
  const int lane = threadIdx.x & 63;
  const int gw = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int r = lane & 15, qg = lane >> 4;
  const int G = p.G, Hkv = p.Hkv, S = p.num_seqs;
  if (gw >= p.num_waves) return;

  // ---- total number of tiles; rows of sequences without tokens are zeroed here
  int64_t carry = 0;
  for (int base = 0; base < S; base += 64) {
    const int n_raw = (base + lane < S) ? p.ctx[base + lane] : 0;
    if (gw == 0 && n_raw > p.max_ctx) atomicCAS(p.status, 0, PIPELIVE_E_RANGE);
    const int ti = tiles_of(n_raw, p.max_ctx);
    const int inc = wave_inclusive_scan(ti, lane);
    carry += __builtin_amdgcn_readlane(inc, 63);
  }
  const int64_t total = carry * Hkv;
  for (int s0 = gw; s0 < S; s0 += p.num_waves) {
    if (tiles_of(p.ctx[s0], p.max_ctx) == 0) {
      for (int e = lane; e < p.Hq * D; e += 64) {
        if (p.out_dtype == PIPELIVE_OUT_F32) ((float *)p.out)[(int64_t)s0 * p.Hq * D + e] = 0.f;
        else ((uint16_t *)p.out)[(int64_t)s0 * p.Hq * D + e] = 0;
      }
    }
  }
  const int64_t a = share_start(p, total, gw);
  const int64_t b0 = share_start(p, total, (int64_t)gw + 1);
  const int64_t b = b0 < total ? b0 : total;
  if (a >= b) return;

  // first sequence whose flat start is <= a (sequences without tokens never match last)
  int s = 0;
  int64_t P_s = 0;  // tiles of all sequences before s
  carry = 0;
  for (int base = 0; base < S; base += 64) {
    const bool in = base + lane < S;
    const int ti = in ? tiles_of(p.ctx[base + lane], p.max_ctx) : 0;
    const int inc = wave_inclusive_scan(ti, lane);
    const int64_t excl = carry + inc - ti;
    const uint64_t bal = __ballot(in && excl * Hkv <= a);
    const int cnt = __popcll(bal);
    if (cnt > 0) {
      s = base + cnt - 1;
      P_s = carry + (__builtin_amdgcn_readlane(inc, cnt - 1) - __builtin_amdgcn_readlane(ti, cnt - 1));
    }
    carry += __builtin_amdgcn_readlane(inc, 63);
  }

  const int64_t rec_sz = attn_record_floats(G, D);

  int64_t t = a;
  while (t < b) {
    // (s, g, j): sequence, KV head, tile inside the sequence of flat position t
    int n = p.ctx[s];
    if (n > p.max_ctx) n = p.max_ctx;
    const int ts = tiles_of(n, p.max_ctx);
    const int64_t rem = t - P_s * Hkv;
    if (ts == 0 || rem >= (int64_t)ts * Hkv) {  // step to the next sequence
      P_s += ts;
      ++s;
      continue;
    }
    const int g = (int)div32(rem, ts);
    const int j0 = (int)(rem - (int64_t)g * ts);
    const int cnt = (int)min((int64_t)(ts - j0), b - t);  // tiles of this pair inside the share
    const int64_t T0 = t - j0;                            // flat start of the pair

    // Q^T operand: lane (head = r, k-group qg) holds q[head][32c + 8qg .. +7]
    bf16x8 qreg[NC];
    {
      const uint16_t *qp = p.q + ((int64_t)s * p.Hq + (int64_t)g * G + r) * D + 8 * qg;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        u32x4 v = {0, 0, 0, 0};
        if (r < G) v = *(const u32x4 *)(qp + 32 * c);
        qreg[c] = as_bf16x8(v);
      }
    }
    f32x4 acc[ND];
#pragma unroll
    for (int c = 0; c < ND; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    for (int sub = 0; sub < cnt; sub += kSubTiles) {
      const int jb = j0 + sub;                        // first tile of this batch
      const int nt = min(cnt - sub, kSubTiles);       // tiles in this batch
      // resolve the batch's blocks: one block per lane (a block holds half a tile,
      // one tile, or TPB tiles)
      constexpr int TPB = BS >= kTile ? BS / kTile : 1;
      const int first_blk = BS < kTile ? jb * 2 : jb / TPB;
      const int last_blk = BS < kTile ? (jb + nt) * 2 - 1 : (jb + nt - 1) / TPB;
      const int nblk = min(last_blk + 1, (n + BS - 1) / BS) - first_blk;
      uint64_t my_addr = 0;
      bool bad = false;
      if (lane < nblk) {
        const int id = p.table[(int64_t)s * p.table_stride + first_blk + lane];
        if ((uint32_t)id < (uint64_t)p.num_blocks) my_addr = p.block_list[id] + p.layer_off;
        else bad = true;
      }
      if (__any(bad)) {  // never dereference a bad id: flag it and leave these tokens out
        if (bad) atomicCAS(p.status, 0, PIPELIVE_E_RANGE);
        continue;
      }
      // tile i of the batch: addresses of the sub-blocks of its two halves and
      // the valid-token counts of the halves
      const uint32_t sub_bytes = SubBlock<BS>::bytes(Hkv, D);
      auto addr_of = [&](int i, uint64_t &a0, uint64_t &a1, int &nv0, int &nv1) {
        const int tok0 = (jb + i) * kTile;
        if (BS < kTile) {
          a0 = readlane64(my_addr, 2 * i);
          a1 = (2 * i + 1 < nblk) ? readlane64(my_addr, 2 * i + 1) : a0;
        } else {
          a0 = a1 = readlane64(my_addr, (jb + i) / TPB - first_blk) +
                    (uint64_t)(((jb + i) % TPB) * sub_bytes);
        }
        nv0 = min(n - tok0, 16);
        nv1 = min(n - tok0 - 16, 16);
      };
      // Software pipeline: K and V of tile i+1 are requested before the QK^T of tile i
      // (V as early as K: on long launches the extra bytes in flight are worth 2 %).
      KRegs<D> kc, kn;
      VRegs<D> vc, vn;
      uint64_t a0, a1;
      int nv0, nv1;
      addr_of(0, a0, a1, nv0, nv1);
      load_k<D, BS>(kc, a0, a1, nv0, nv1, g, r, qg);
      load_v<D, BS>(vc, a0, a1, g, Hkv, r, qg);
#pragma unroll 1
      for (int i = 0; i + 1 < nt; ++i) {
        addr_of(i + 1, a0, a1, nv0, nv1);
        load_k<D, BS>(kn, a0, a1, nv0, nv1, g, r, qg);
        load_v<D, BS>(vn, a0, a1, g, Hkv, r, qg);
        u32x4 ph, pl;
        qk_softmax<D>(kc, qreg, acc, m, l, p.scale_log2, qg, ph, pl);
        pv_accumulate<D>(vc, kc.nvalid[0], kc.nvalid[1], ph, pl, acc, qg);
        kc = kn;
        vc = vn;
      }
      {  // last tile of the batch: nothing left to prefetch
        u32x4 ph, pl;
        qk_softmax<D>(kc, qreg, acc, m, l, p.scale_log2, qg, ph, pl);
        pv_accumulate<D>(vc, kc.nvalid[0], kc.nvalid[1], ph, pl, acc, qg);
      }
    }
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const int64_t row = (int64_t)s * p.Hq + (int64_t)g * G + r;
    // lane (qg, r) holds O[head r][16c + 4qg + i]
    auto store_out = [&](const f32x4 (&o)[ND], float inv) {
      if (r >= G) return;
      if (p.out_dtype == PIPELIVE_OUT_F32) {
        float *dst = (float *)p.out + row * D + 4 * qg;
#pragma unroll
        for (int c = 0; c < ND; ++c)
          *(float4 *)(dst + 16 * c) = make_float4(o[c][0] * inv, o[c][1] * inv, o[c][2] * inv, o[c][3] * inv);
      } else {
        uint16_t *dst = (uint16_t *)p.out + row * D + 4 * qg;
#pragma unroll
        for (int c = 0; c < ND; ++c) {
          const uint32_t w0 = f32_to_bf16_rne(o[c][0] * inv) | ((uint32_t)f32_to_bf16_rne(o[c][1] * inv) << 16);
          const uint32_t w1 = f32_to_bf16_rne(o[c][2] * inv) | ((uint32_t)f32_to_bf16_rne(o[c][3] * inv) << 16);
          *(uint2 *)(dst + 16 * c) = make_uint2(w0, w1);
        }
      }
    };
    const bool complete = (j0 == 0) && (j0 + cnt == ts);
    if (complete) {
      store_out(acc, l > 0.f ? 1.0f / l : 0.f);  // l == 0 only after a bad block id
    } else {
      // The pair is cut by a share boundary.  Leave a partial record O[G][D], m[G],
      // l[G] for the merge kernel: the pair that began before this share uses slot
      // 2*gw, a pair that runs past its end uses slot 2*gw+1.
      const int64_t slot = 2 * (int64_t)gw + (T0 <= a ? 0 : 1);
      float *rec = p.ws + slot * rec_sz;
      if (r < G) {
        float *o = rec + (int64_t)r * D + 4 * qg;
#pragma unroll
        for (int c = 0; c < ND; ++c)
          *(float4 *)(o + 16 * c) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
        if (qg == 0) {
          rec[(int64_t)G * D + r] = m;
          rec[(int64_t)G * D + G + r] = l;
        }
      }
    }
    t += cnt;
  }
}

// Merge kernel: one wave per (sequence, KV head) pair that was cut by share
// boundaries.  Records are merged in share order, so the result does not depend
// on which wave finished first.  Lane e handles the float4 at element
// 4*lane + 256*j of the pair's [G][D] output.
template <int D, int NJ>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnParams p) {
  const int lane = threadIdx.x & 63;
  const int pair = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int G = p.G, Hkv = p.Hkv, S = p.num_seqs;
  if (pair >= S * Hkv) return;
  const int s = pair / Hkv, g = pair % Hkv;
  // tiles before sequence s and in total
  int64_t carry = 0, before = 0;
  int ts = 0;
  for (int base = 0; base < S; base += 64) {
    const int ti = (base + lane < S) ? tiles_of(p.ctx[base + lane], p.max_ctx) : 0;
    const int inc = wave_inclusive_scan(ti, lane);
    if (s >= base && s < base + 64) {
      const int k = s - base;
      ts = __builtin_amdgcn_readlane(ti, k);
      before = carry + (__builtin_amdgcn_readlane(inc, k) - ts);
    }
    carry += __builtin_amdgcn_readlane(inc, 63);
  }
  const int64_t total = carry * Hkv;
  if (ts == 0) return;  // zero row, written by the main kernel
  const int64_t T0 = before * Hkv + (int64_t)g * ts;
  const int64_t w_first = share_wave(p, total, T0), w_last = share_wave(p, total, T0 + ts - 1);
  if (w_first == w_last) return;  // finished by the wave that owns it
  const int64_t rec_sz = attn_record_floats(G, D);
  const int GD = G * D;
  float M[NJ], L[NJ];
  float4 O[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    M[j] = -INFINITY;
    L[j] = 0.f;
    O[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  constexpr int kChunk = NJ <= 2 ? 8 : 4;  // records fetched together, merged in order
  for (int64_t w0 = w_first; w0 <= w_last; w0 += kChunk) {
    float mw[kChunk][NJ], lw[kChunk][NJ];
    float4 ow[kChunk][NJ];
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
      const int64_t w = w0 + u < w_last ? w0 + u : w_last;  // clamp: re-reads the last record, unused
      const float *rw = p.ws + (2 * w + (T0 <= share_start(p, total, w) ? 0 : 1)) * rec_sz;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int e = 4 * lane + 256 * j;
        const int ec = e < GD ? e : 0;
        mw[u][j] = rw[GD + ec / D];
        lw[u][j] = rw[GD + G + ec / D];
        ow[u][j] = *(const float4 *)(rw + ec);
      }
    }
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
      if (w0 + u > w_last) break;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const float Mn = fmaxf(M[j], mw[u][j]);
        const float fa = (M[j] == -INFINITY) ? 0.f : fast_exp2(M[j] - Mn);
        const float fb = (mw[u][j] == -INFINITY) ? 0.f : fast_exp2(mw[u][j] - Mn);
        L[j] = L[j] * fa + lw[u][j] * fb;
        O[j] = make_float4(O[j].x * fa + ow[u][j].x * fb, O[j].y * fa + ow[u][j].y * fb,
                           O[j].z * fa + ow[u][j].z * fb, O[j].w * fa + ow[u][j].w * fb);
        M[j] = Mn;
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int e = 4 * lane + 256 * j;
    if (e < GD) {
      const float inv = L[j] > 0.f ? 1.0f / L[j] : 0.f;
      const int64_t idx = ((int64_t)s * p.Hq + (int64_t)g * G) * D + e;
      if (p.out_dtype == PIPELIVE_OUT_F32) {
        *(float4 *)((float *)p.out + idx) = make_float4(O[j].x * inv, O[j].y * inv, O[j].z * inv, O[j].w * inv);
      } else {
        const uint32_t w0 = f32_to_bf16_rne(O[j].x * inv) | ((uint32_t)f32_to_bf16_rne(O[j].y * inv) << 16);
        const uint32_t w1 = f32_to_bf16_rne(O[j].z * inv) | ((uint32_t)f32_to_bf16_rne(O[j].w * inv) << 16);
        *(uint2 *)((uint16_t *)p.out + idx) = make_uint2(w0, w1);
      }
    }
  }
}

template <int D>
hipError_t launch_merge(const AttnParams &p, hipStream_t st) {
  const unsigned mgrid = (unsigned)(((int64_t)p.num_seqs * p.Hkv + 3) / 4);
  const int nj = (p.G * D + 255) / 256;
  if (nj <= 1) hipLaunchKernelGGL((attn_merge_kernel<D, 1>), dim3(mgrid), dim3(256), 0, st, p);
  else if (nj <= 2) hipLaunchKernelGGL((attn_merge_kernel<D, 2>), dim3(mgrid), dim3(256), 0, st, p);
  else if (nj <= 4) hipLaunchKernelGGL((attn_merge_kernel<D, 4>), dim3(mgrid), dim3(256), 0, st, p);
  else hipLaunchKernelGGL((attn_merge_kernel<D, 8>), dim3(mgrid), dim3(256), 0, st, p);
  return hipGetLastError();
}

template <int D, int BS>
hipError_t launch_t(const AttnParams &p, hipStream_t st) {
  const unsigned grid = (unsigned)((p.num_waves + 3) / 4);
  hipLaunchKernelGGL((attn_decode_kernel<D, BS>), dim3(grid), dim3(256), 0, st, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_merge<D>(p, st);
}

template <int D, int BS>
int occupancy_t() {
  int nb = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, attn_decode_kernel<D, BS>, 256, 0) != hipSuccess || nb < 1)
    nb = 2;
  return nb * 4;  // waves per CU
}

}  // namespace

// one instantiation per (head_dim, block_tokens) the interface admits
#define PIPELIVE_ATTN_SHAPES(X) \
  X(128, 16) X(128, 32) X(128, 64) X(128, 128) X(64, 16) X(64, 32) X(64, 64) X(64, 128)

hipError_t launch_attn_decode(const AttnParams &p, int D, int BS, hipStream_t st) {
#define X(d, b) \
  if (D == d && BS == b) return launch_t<d, b>(p, st);
  PIPELIVE_ATTN_SHAPES(X)
#undef X
  return hipErrorInvalidValue;
}

int attn_waves_per_cu(int D, int BS) {
#define X(d, b)                                   \
  if (D == d && BS == b) {                        \
    static int cached = 0;                        \
    if (cached == 0) cached = occupancy_t<d, b>(); \
    return cached;                                \
  }
  PIPELIVE_ATTN_SHAPES(X)
#undef X
  return 4;
}

}  // namespace pipelive
