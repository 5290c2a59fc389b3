// Paged-attention decode for gfx950 (CDNA4, wave64, MFMA).
//
// One workgroup of 4 waves per (split, KV head, sequence).  A wave walks its
// share of the split in steps of 32 tokens.  Per step it fetches two 16-token
// K tiles and the matching V^T tiles straight from HBM into the MFMA operand
// registers (the in-block layout makes every load instruction cover whole
// contiguous cache lines), computes S^T = K Q^T with v_mfma_f32_16x16x32_bf16
// (rows = tokens, columns = the G query heads that share this KV head, padded
// to 16), runs the online softmax on the accumulator layout, and accumulates
// O^T += V^T P^T with P split into two bf16 terms so that no precision is
// lost against fp32 weights.  The S^T accumulator layout (lane holds 4
// consecutive tokens of one head) is exactly the B-operand layout of the PV
// product, so scores never cross lanes except for the running max.
//
// Paper: Sec. 2 "LLM Inference" (decode re-reads the cached K/V: memory
// bound), Sec. 5.1 (block addresses are resolved through the block table and
// the block list at kernel time; blocks are not contiguous).
#include "internal.h"

namespace pipelive {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint64_t readlane64(uint64_t v, int lane) {
  uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, lane);
  uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
  return ((uint64_t)hi << 32) | lo;
}

// top 16 bits of two floats packed into one dword: [hi16(a) | hi16(b) << 16]
__device__ __forceinline__ uint32_t pack_hi16(float a, float b) {
  return (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xFFFF0000u);
}

constexpr int kWaves = 4;
constexpr int kMaxG = 16;

template <int D, int BS>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnParams p) {
  constexpr int NC = D / 32;  // QK^T: 32 head-dim elements per MFMA
  constexpr int ND = D / 16;  // PV: 16 output dims per MFMA
  constexpr int KHEAD = BS * D * 2;  // bytes of one head's K (or V) in a block

  const int sp = blockIdx.x, g = blockIdx.y, s = blockIdx.z;
  int n = p.ctx[s];
  if (n > p.max_ctx) n = p.max_ctx;
  const int ST = p.split_tokens;
  const int c0 = sp * ST;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + ST);
  const int nsplit = (n + ST - 1) / ST;

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform
  const int r = lane & 15, qg = lane >> 4;
  const int G = p.G;

  // resolve this split's blocks: one block per lane (ST <= 64 * BS)
  const int nblk = (c1 - c0 + BS - 1) / BS;
  uint64_t my_addr = 0;
  if (lane < nblk) {
    int id = p.table[(int64_t)s * p.table_stride + c0 / BS + lane];
    if ((uint32_t)id < (uint64_t)p.num_blocks) {
      my_addr = p.block_list[id] + p.layer_off;
    } else {
      atomicCAS(p.status, 0, PIPELIVE_E_RANGE);
    }
  }

  // Q^T operand: lane (head = r, k-group qg) holds q[head][32c + 8qg .. +7]
  bf16x8 qreg[NC];
  {
    const uint16_t *qp = p.q + ((int64_t)s * p.Hq + (int64_t)g * G + r) * D + 8 * qg;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (r < G) v = *(const uint4 *)(qp + 32 * c);
      qreg[c] = as_bf16x8(v);
    }
  }

  f32x4 acc[ND];
#pragma unroll
  for (int c = 0; c < ND; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;

  const int nsteps = (c1 - c0 + 31) / 32;
  for (int st = w; st < nsteps; st += kWaves) {
    const int t0 = c0 + 32 * st;
    uint4 kreg[2][NC];
    uint2 vreg[ND][2];
    int nvalid[2];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      const int tile_start = t0 + 16 * T;
      nvalid[T] = c1 - tile_start;  // > 0: tile holds valid tokens
      const int bidx = (BS == 16) ? (2 * st + T) : st;
      const uint64_t addr = readlane64(my_addr, bidx);
      const bool on = nvalid[T] > 0 && addr != 0;
      if (!on) nvalid[T] = 0;
      const int toff = (BS == 32) ? 16 * T : 0;
      const char *kb = (const char *)addr + (int64_t)g * KHEAD;
      const char *vb = (const char *)addr + (int64_t)p.Hkv * KHEAD + (int64_t)g * KHEAD;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        kreg[T][c] = make_uint4(0, 0, 0, 0);
        if (on) kreg[T][c] = *(const uint4 *)(kb + (((4 * c + qg) * BS + toff + r) * 16));
      }
#pragma unroll
      for (int c = 0; c < ND; ++c) {
        vreg[c][T] = make_uint2(0, 0);
        if (on) vreg[c][T] = *(const uint2 *)(vb + (((16 * c + r) * BS + toff + 4 * qg) * 2));
      }
    }

    if (nvalid[0] <= 0 && nvalid[1] <= 0) continue;  // only after a bad block id

    // S^T tiles: rows = tokens, columns = heads
    f32x4 sc[2];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      sc[T] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < NC; ++c)
        sc[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kreg[T][c]), qreg[c], sc[T], 0, 0, 0);
    }

    // scale, mask by predicate (never by arithmetic: unused slots may hold NaN)
    float x[8];
    float mloc = -INFINITY;
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ok = (4 * qg + i) < nvalid[T];
        float v = ok ? sc[T][i] * p.scale_log2 : -INFINITY;
        x[4 * T + i] = v;
        mloc = fmaxf(mloc, v);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float m_new = fmaxf(m, mloc);  // finite: the step holds at least one valid token
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

    // P^T operand: slots 0..3 = tile 0 tokens 4qg+i, slots 4..7 = tile 1; two bf16 terms
    uint4 ph, pl;
    {
      float lo[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) lo[i] = pv[i] - __uint_as_float(__float_as_uint(pv[i]) & 0xFFFF0000u);
      ph = make_uint4(pack_hi16(pv[0], pv[1]), pack_hi16(pv[2], pv[3]), pack_hi16(pv[4], pv[5]),
                      pack_hi16(pv[6], pv[7]));
      pl = make_uint4(pack_hi16(lo[0], lo[1]), pack_hi16(lo[2], lo[3]), pack_hi16(lo[4], lo[5]),
                      pack_hi16(lo[6], lo[7]));
    }

    // V of masked tokens must be zero (0 * NaN is NaN): partial tiles only
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      if (nvalid[T] > 0 && nvalid[T] < 16) {
        const int keep = min(max(nvalid[T] - 4 * qg, 0), 4);
        const uint64_t mask = keep >= 4 ? ~0ull : ((1ull << (16 * keep)) - 1ull);
#pragma unroll
        for (int c = 0; c < ND; ++c) {
          vreg[c][T].x &= (uint32_t)mask;
          vreg[c][T].y &= (uint32_t)(mask >> 32);
        }
      }
    }

#pragma unroll
    for (int c = 0; c < ND; ++c) {
      const bf16x8 va = as_bf16x8(make_uint4(vreg[c][0].x, vreg[c][0].y, vreg[c][1].x, vreg[c][1].y));
      acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, as_bf16x8(ph), acc[c], 0, 0, 0);
      acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, as_bf16x8(pl), acc[c], 0, 0, 0);
    }
  }

  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  // merge the 4 waves through LDS
  __shared__ float sh_o[kWaves][kMaxG][D];
  __shared__ float sh_m[kWaves][kMaxG];
  __shared__ float sh_l[kWaves][kMaxG];
  if (r < G) {
#pragma unroll
    for (int c = 0; c < ND; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) sh_o[w][r][16 * c + 4 * qg + i] = acc[c][i];
    if (qg == 0) {
      sh_m[w][r] = m;
      sh_l[w][r] = l;
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += 256) {
    const int hh = idx / D, d = idx % D;
    float M = sh_m[0][hh];
#pragma unroll
    for (int k = 1; k < kWaves; ++k) M = fmaxf(M, sh_m[k][hh]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int k = 0; k < kWaves; ++k) {
      const float wk = fast_exp2(sh_m[k][hh] - M);  // -inf (idle wave) -> 0
      L += wk * sh_l[k][hh];
      O += wk * sh_o[k][hh][d];
    }
    const int64_t row = (int64_t)s * p.Hq + (int64_t)g * G + hh;
    if (nsplit == 1) {
      const float o = O / L;
      if (p.out_dtype == PIPELIVE_OUT_F32) {
        ((float *)p.out)[row * D + d] = o;
      } else {
        uint32_t u = __float_as_uint(o);
        u += 0x7FFFu + ((u >> 16) & 1u);
        ((uint16_t *)p.out)[row * D + d] = (uint16_t)(u >> 16);
      }
    } else {
      p.ws_o[(row * p.max_splits + sp) * D + d] = O;
      if (d == 0) {
        p.ws_ml[(row * p.max_splits + sp) * 2 + 0] = M;
        p.ws_ml[(row * p.max_splits + sp) * 2 + 1] = L;
      }
    }
  }
}

// Merge the per-split partial results of one (sequence, head): fixed order, so
// the result does not depend on which workgroup finished first.
template <int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(AttnParams p) {
  const int h = blockIdx.x, s = blockIdx.y, d = threadIdx.x;
  int n = p.ctx[s];
  if (n > p.max_ctx) {
    n = p.max_ctx;
    if (d == 0 && h == 0) atomicCAS(p.status, 0, PIPELIVE_E_RANGE);
  }
  const int nsplit = (n + p.split_tokens - 1) / p.split_tokens;
  if (nsplit == 1) return;  // written by the main kernel
  const int64_t row = (int64_t)s * p.Hq + h;
  float o = 0.f;
  if (nsplit > 1) {
    const float *ml = p.ws_ml + row * p.max_splits * 2;
    const float *wo = p.ws_o + row * p.max_splits * D;
    float M = -INFINITY;
    for (int k = 0; k < nsplit; ++k) M = fmaxf(M, ml[2 * k]);
    float L = 0.f, O = 0.f;
    for (int k = 0; k < nsplit; ++k) {
      const float wk = fast_exp2(ml[2 * k] - M);
      L += wk * ml[2 * k + 1];
      O += wk * wo[(int64_t)k * D + d];
    }
    o = O / L;
  }
  if (p.out_dtype == PIPELIVE_OUT_F32) {
    ((float *)p.out)[row * D + d] = o;
  } else {
    uint32_t u = __float_as_uint(o);
    u += 0x7FFFu + ((u >> 16) & 1u);
    ((uint16_t *)p.out)[row * D + d] = (uint16_t)(u >> 16);
  }
}

template <int D, int BS>
hipError_t launch_t(const AttnParams &p, hipStream_t st) {
  dim3 grid(p.max_splits, p.Hkv, p.num_seqs);
  hipLaunchKernelGGL((attn_decode_kernel<D, BS>), grid, dim3(256), 0, st, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_combine_kernel<D>), dim3(p.Hq, p.num_seqs), dim3(D), 0, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_decode(const AttnParams &p, int D, int BS, hipStream_t st) {
  if (D == 128 && BS == 16) return launch_t<128, 16>(p, st);
  if (D == 128 && BS == 32) return launch_t<128, 32>(p, st);
  if (D == 64 && BS == 16) return launch_t<64, 16>(p, st);
  if (D == 64 && BS == 32) return launch_t<64, 32>(p, st);
  return hipErrorInvalidValue;
}

}  // namespace pipelive
