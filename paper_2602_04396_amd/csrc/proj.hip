// Projection GEMMs of the local step on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
//   down:  g = Q^T (s G)      (Sec. 2; Alg. 1 "low-rank gradient signal")   contraction over the p rows
//   up:    W <- W - eta Q N   (Sec. 2; Alg. 1 parameter update)             contraction over the rank
//
// fp32 operands the library owns (Q, N) are kept as two bf16 planes hi + lo (x = hi + lo up to
// 2^-17 relative), already in the lane order of the MFMA operand fragment, so a fragment is one
// 16-byte load per lane.  The bf16 gradient is exact; an fp32 gradient is split on the fly.
//   down:  acc += Qhi^T G + Qlo^T G                      (+ Qhi^T Glo for fp32 G)
//   up:    acc += Qhi Nhi + Qhi Nlo + Qlo Nhi
// Accumulation is fp32 in the matrix core.
#include "common.h"

namespace lordo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 as_bf(uint4 x) { return __builtin_bit_cast(bf16x8, x); }

__device__ __forceinline__ uint32_t f2bf_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

constexpr int DBK = 32;        // rows of G per pipeline stage
constexpr int DBN = 128;       // columns of G per workgroup

// ---------------------------------------------------------------------------------------
// Down-projection.  Workgroup = 4 waves; output tile = (32*MB rank indices) x 128 columns.
// Wave w owns rank block w % MB and MB column blocks starting at (w / MB) * MB.
// The G tile (32 rows x 128 columns) is transposed in registers and staged in LDS in fragment
// order: slot (nblk, kgrp, n) is the 16-byte vector G[k0 + 8*kgrp + 0..7][n0 + 32*nblk + n].
// ---------------------------------------------------------------------------------------
template <bool GF32>
struct GStage {
  uint32_t x[GF32 ? 16 : 8];   // bf16: row i -> two columns packed; fp32: row i -> two floats
};

template <bool GF32>
__device__ __forceinline__ void load_gstage(GStage<GF32>& st, const void* Gp, int q, int krow, int klim, int col,
                                            bool vec_ok) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int row = krow + i;
    if constexpr (!GF32) {
      const uint16_t* G = reinterpret_cast<const uint16_t*>(Gp);
      uint32_t val = 0;
      if (row < klim) {
        int64_t o = (int64_t)row * q + col;
        if (vec_ok && col + 1 < q) val = *reinterpret_cast<const uint32_t*>(G + o);
        else {
          if (col < q) val = G[o];
          if (col + 1 < q) val |= (uint32_t)G[o + 1] << 16;
        }
      }
      st.x[i] = val;
    } else {
      const float* G = reinterpret_cast<const float*>(Gp);
      float a = 0.f, b = 0.f;
      if (row < klim) {
        int64_t o = (int64_t)row * q + col;
        if (vec_ok && col + 1 < q) { float2 t = *reinterpret_cast<const float2*>(G + o); a = t.x; b = t.y; }
        else {
          if (col < q) a = G[o];
          if (col + 1 < q) b = G[o + 1];
        }
      }
      st.x[2 * i] = __float_as_uint(a);
      st.x[2 * i + 1] = __float_as_uint(b);
    }
  }
}

// 8 rows x 2 columns -> two 16-byte vectors (one per column, 8 consecutive k each)
template <bool GF32>
__device__ __forceinline__ void store_gstage(const GStage<GF32>& st, uint4* lds_hi, uint4* lds_lo, int slot) {
  if constexpr (!GF32) {
    uint4 c0, c1;
    c0.x = (st.x[0] & 0xffffu) | (st.x[1] << 16);  c1.x = (st.x[0] >> 16) | (st.x[1] & 0xffff0000u);
    c0.y = (st.x[2] & 0xffffu) | (st.x[3] << 16);  c1.y = (st.x[2] >> 16) | (st.x[3] & 0xffff0000u);
    c0.z = (st.x[4] & 0xffffu) | (st.x[5] << 16);  c1.z = (st.x[4] >> 16) | (st.x[5] & 0xffff0000u);
    c0.w = (st.x[6] & 0xffffu) | (st.x[7] << 16);  c1.w = (st.x[6] >> 16) | (st.x[7] & 0xffff0000u);
    lds_hi[slot] = c0;
    lds_hi[slot + 1] = c1;
  } else {
    uint32_t h0[8], l0[8], h1[8], l1[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float a = __uint_as_float(st.x[2 * i]), b = __uint_as_float(st.x[2 * i + 1]);
      h0[i] = f2bf_rne(a); l0[i] = f2bf_rne(a - __uint_as_float(h0[i] << 16));
      h1[i] = f2bf_rne(b); l1[i] = f2bf_rne(b - __uint_as_float(h1[i] << 16));
    }
    lds_hi[slot] = make_uint4(h0[0] | (h0[1] << 16), h0[2] | (h0[3] << 16), h0[4] | (h0[5] << 16), h0[6] | (h0[7] << 16));
    lds_hi[slot + 1] = make_uint4(h1[0] | (h1[1] << 16), h1[2] | (h1[3] << 16), h1[4] | (h1[5] << 16), h1[6] | (h1[7] << 16));
    lds_lo[slot] = make_uint4(l0[0] | (l0[1] << 16), l0[2] | (l0[3] << 16), l0[4] | (l0[5] << 16), l0[6] | (l0[7] << 16));
    lds_lo[slot + 1] = make_uint4(l1[0] | (l1[1] << 16), l1[2] | (l1[3] << 16), l1[4] | (l1[5] << 16), l1[6] | (l1[7] << 16));
  }
}

template <int MB, bool GF32>
__global__ __launch_bounds__(256) void k_proj_down(DevCtx d, const ProjTile* __restrict__ tiles, float* __restrict__ glow,
                                                   int64_t split_stride, float grad_scale) {
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0) return;
  const MatDev& m = d.mats[t.mat];
  const void* Gp = d.ext[EXT_G * d.n + t.mat];
  const uint4* qt_hi = reinterpret_cast<const uint4*>(d.arena + m.qt_hi);
  const uint4* qt_lo = reinterpret_cast<const uint4*>(d.arena + m.qt_lo);

  constexpr int STAGE_SLOTS = 4 * 4 * 32;                    // (nblk, kgrp, n) 16-byte slots
  __shared__ uint4 lds_hi[2 * STAGE_SLOTS];
  __shared__ uint4 lds_lo[GF32 ? 2 * STAGE_SLOTS : 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mbg = t.m0 / 32 + wave % MB;                      // global rank block of this wave
  const int nb_first = (wave / MB) * MB;                      // first column block (0..3) of this wave
  const bool active = mbg < m.rp / 32;

  const int q = m.q;
  const int col = t.n0 + 2 * lane;                            // first of the two columns this lane stages
  const bool vec_ok = GF32 ? ((q & 1) == 0 && (reinterpret_cast<uintptr_t>(Gp) & 7) == 0)
                           : ((q & 1) == 0 && (reinterpret_cast<uintptr_t>(Gp) & 3) == 0);
  const int klim = t.k1 < m.p ? t.k1 : m.p;
  const int wslot = ((lane >> 4) * 4 + wave) * 32 + 2 * (lane & 15);   // nblk = lane/16, kgrp = wave

  f32x16 acc[MB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;

  const int nstages = (t.k1 - t.k0 + DBK - 1) / DBK;
  GStage<GF32> st;
  load_gstage<GF32>(st, Gp, q, t.k0 + 8 * wave, klim, col, vec_ok);
  store_gstage<GF32>(st, lds_hi, lds_lo, wslot);
  __syncthreads();

  const int64_t kgroups = m.pp / 8;
  for (int s = 0; s < nstages; ++s) {
    const int kr = t.k0 + s * DBK;
    if (s + 1 < nstages) load_gstage<GF32>(st, Gp, q, kr + DBK + 8 * wave, klim, col, vec_ok);
    if (active) {
      const uint4* bh = lds_hi + (s & 1) * STAGE_SLOTS;
      const uint4* bl = lds_lo + (GF32 ? (s & 1) * STAGE_SLOTS : 0);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        int64_t ag = ((int64_t)mbg * kgroups + (kr / 8 + 2 * ks + (lane >> 5))) * 32 + (lane & 31);
        bf16x8 a_hi = as_bf(qt_hi[ag]);
        bf16x8 a_lo = as_bf(qt_lo[ag]);
#pragma unroll
        for (int a = 0; a < MB; ++a) {
          int bslot = ((nb_first + a) * 4 + 2 * ks + (lane >> 5)) * 32 + (lane & 31);
          bf16x8 b = as_bf(bh[bslot]);
          acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, b, acc[a], 0, 0, 0);
          acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, b, acc[a], 0, 0, 0);
          if constexpr (GF32) {
            bf16x8 b2 = as_bf(bl[bslot]);
            acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, b2, acc[a], 0, 0, 0);
          }
        }
      }
    }
    if (s + 1 < nstages) store_gstage<GF32>(st, lds_hi + ((s + 1) & 1) * STAGE_SLOTS,
                                            lds_lo + (GF32 ? ((s + 1) & 1) * STAGE_SLOTS : 0), wslot);
    __syncthreads();
  }

  if (!active) return;
  // accumulator register v of lane l: rank index 32*mbg + 8*(v/4) + 4*(l/32) + v%4, column 32*nbg + l%32
  float* out = glow + (int64_t)t.split * split_stride + m.lr_off;
  const int64_t rgroups = m.rp / 8;
#pragma unroll
  for (int a = 0; a < MB; ++a) {
    int nbg = t.n0 / 32 + nb_first + a;
    if (nbg >= m.qp / 32) continue;
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      int64_t o = (((int64_t)nbg * rgroups + 4 * mbg + vq) * 32 + (lane & 31)) * 8 + 4 * (lane >> 5);
      float4 val = make_float4(grad_scale * acc[a][4 * vq], grad_scale * acc[a][4 * vq + 1],
                               grad_scale * acc[a][4 * vq + 2], grad_scale * acc[a][4 * vq + 3]);
      *reinterpret_cast<float4*>(out + o) = val;
    }
  }
}

hipError_t launch_proj_down(const DevCtx& d, const ProjTile* tiles, int ntiles, int mb, float* glow, int64_t split_stride,
                            float grad_scale, bool g_is_f32, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  dim3 grid(ntiles), block(256);
#define LORDO_DOWN(MBV)                                                                                            \
  if (g_is_f32) hipLaunchKernelGGL((k_proj_down<MBV, true>), grid, block, 0, s, d, tiles, glow, split_stride, grad_scale); \
  else hipLaunchKernelGGL((k_proj_down<MBV, false>), grid, block, 0, s, d, tiles, glow, split_stride, grad_scale);
  if (mb == 4) { LORDO_DOWN(4) } else if (mb == 2) { LORDO_DOWN(2) } else { LORDO_DOWN(1) }
#undef LORDO_DOWN
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Up-projection with the weight update fused.  Workgroup tile 128 x 128 of W, 4 waves in a
// 2 x 2 grid, each wave 64 x 64 = 2 x 2 accumulator blocks.  Operand fragments come straight
// from the packed planes (one coalesced 1 KiB read per wave and fragment).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_proj_up(DevCtx d, const ProjTile* __restrict__ tiles,
                                                 const uint16_t* __restrict__ n_hi, const uint16_t* __restrict__ n_lo, float lr) {
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0) return;
  const MatDev& m = d.mats[t.mat];
  float* W = reinterpret_cast<float*>(d.ext[EXT_W * d.n + t.mat]);
  const uint4* qa_hi = reinterpret_cast<const uint4*>(d.arena + m.qa_hi);
  const uint4* qa_lo = reinterpret_cast<const uint4*>(d.arena + m.qa_lo);
  const uint4* nh = reinterpret_cast<const uint4*>(n_hi + m.lr_off);
  const uint4* nl = reinterpret_cast<const uint4*>(n_lo + m.lr_off);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int mb0 = t.m0 / 32 + 2 * (wave & 1);
  const int nb0 = t.n0 / 32 + 2 * (wave >> 1);
  const int mblocks = m.pp / 32, nblocks = m.qp / 32;
  if (mb0 >= mblocks || nb0 >= nblocks) return;
  const int64_t rgroups = m.rp / 8;
  int mbc[2], nbc[2];          // clamped block indices: loads stay inside the planes, stores are masked
  mbc[0] = mb0; mbc[1] = mb0 + 1 < mblocks ? mb0 + 1 : mb0;
  nbc[0] = nb0; nbc[1] = nb0 + 1 < nblocks ? nb0 + 1 : nb0;

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  const int ksteps = m.rp / 16;
  const int sub = (lane >> 5) * 32 + (lane & 31);
  for (int ks = 0; ks < ksteps; ++ks) {
    bf16x8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      int64_t g = ((int64_t)mbc[a] * rgroups + 2 * ks) * 32 + sub;
      ah[a] = as_bf(qa_hi[g]);
      al[a] = as_bf(qa_lo[g]);
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      int64_t g = ((int64_t)nbc[b] * rgroups + 2 * ks) * 32 + sub;
      bh[b] = as_bf(nh[g]);
      bl[b] = as_bf(nl[g]);
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[a], bh[b], acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[a], bl[b], acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[a], bh[b], acc[a][b], 0, 0, 0);
      }
  }

#pragma unroll
  for (int a = 0; a < 2; ++a) {
    if (mb0 + a >= mblocks) continue;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if (nb0 + b >= nblocks) continue;
      int colw = 32 * (nb0 + b) + (lane & 31);
      if (colw >= m.q) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int row = 32 * (mb0 + a) + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < m.p) {
          int64_t o = (int64_t)row * m.q + colw;
          W[o] = fmaf(-lr, acc[a][b][v], W[o]);
        }
      }
    }
  }
}

hipError_t launch_proj_up(const DevCtx& d, const ProjTile* tiles, int ntiles, const uint16_t* n_hi,
                          const uint16_t* n_lo, float lr, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_proj_up, dim3(ntiles), dim3(256), 0, s, d, tiles, n_hi, n_lo, lr);
  return hipGetLastError();
}

}  // namespace lordo
