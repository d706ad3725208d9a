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
//
// Caller matrices (G, W) are reached through buffer resources: the hardware range check returns
// zero for reads past the end (rows beyond the matrix or beyond this workgroup's slice of the
// contraction) and drops such writes, and a lane whose column is outside the matrix is given an
// offset beyond the range.  No access is guarded by a branch.  Pointers into the arena are cast
// to the global address space so that no access is a flat one.
#include "common.h"

namespace lordo {

#define GAS __attribute__((address_space(1)))
// generic -> global address space (a C-style cast; reinterpret_cast may not change address spaces)
#define TO_GLOBAL(T, ptr) ((GAS T*)(ptr))

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// native vectors: the only vector types that can be read through address-space pointers
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf(u32x4 x) { return __builtin_bit_cast(bf16x8, x); }
__device__ __forceinline__ u32x4 mk4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  u32x4 r;
  r.x = a; r.y = b; r.z = c; r.w = d;
  return r;
}

__device__ __forceinline__ uint32_t f2bf_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}


typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// Compiler-level fence: keeps the loads issued before it from being sunk to their first use
// (prefetches must be in flight while the matrix cores work); it emits no instruction.
#define ISSUE_FENCE() asm volatile("" ::: "memory")
constexpr uint32_t OOB = 0x80000000u;        // byte offset beyond any resource (sizes are < 2 GiB)
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// ---------------------------------------------------------------------------------------
// Down-projection.  Workgroup = 4 waves; output tile = (32*MB rank indices) x 128 columns.
// Wave w owns rank block w % MB and MB column blocks starting at (w / MB) * MB.
// The G tile (32 rows x 128 columns) is transposed in registers and staged in LDS in fragment
// order: slot (nblk, kgrp, n) is the 16-byte vector G[k0 + 8*kgrp + 0..7][n0 + 32*nblk + n].
// Each lane stages two adjacent columns of 8 consecutive rows.
// ---------------------------------------------------------------------------------------
template <bool GF32>
struct GStage {
  uint32_t x[GF32 ? 16 : 8];   // bf16: row i -> two columns packed; fp32: row i -> two floats
};

// Column handling of one lane, fixed for the whole kernel: byte offsets of its two columns
// inside a row (OOB if the column is outside the matrix).
struct GCol {
  uint32_t off0, off1;
  bool vec;           // both columns with one aligned access
};

// Rows krow .. krow+7 (krow uniform over the wave) of the lane's two columns.
template <bool GF32>
__device__ __forceinline__ void load_gstage(GStage<GF32>& st, rsrc_t rs, uint32_t row_bytes, int krow, const GCol& gc) {
  if (gc.vec) {                     // uniform branch, taken once per stage
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t soff = (uint32_t)(krow + i) * row_bytes;       // scalar
      if constexpr (!GF32) {
        st.x[i] = __builtin_amdgcn_raw_buffer_load_b32(rs, gc.off0, soff, 0);
      } else {
        u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rs, gc.off0, soff, 0);
        st.x[2 * i] = t.x;
        st.x[2 * i + 1] = t.y;
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t soff = (uint32_t)(krow + i) * row_bytes;
      if constexpr (!GF32) {
        uint32_t lo = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, gc.off0, soff, 0);
        uint32_t hi = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, gc.off1, soff, 0);
        st.x[i] = lo | (hi << 16);
      } else {
        st.x[2 * i] = __builtin_amdgcn_raw_buffer_load_b32(rs, gc.off0, soff, 0);
        st.x[2 * i + 1] = __builtin_amdgcn_raw_buffer_load_b32(rs, gc.off1, soff, 0);
      }
    }
  }
}

// 8 rows x 2 columns -> two 16-byte vectors (one per column, 8 consecutive k each)
template <bool GF32>
__device__ __forceinline__ void store_gstage(const GStage<GF32>& st, u32x4* lds_hi, u32x4* lds_lo, int slot) {
  if constexpr (!GF32) {
    u32x4 c0, c1;
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
    lds_hi[slot] = mk4(h0[0] | (h0[1] << 16), h0[2] | (h0[3] << 16), h0[4] | (h0[5] << 16), h0[6] | (h0[7] << 16));
    lds_hi[slot + 1] = mk4(h1[0] | (h1[1] << 16), h1[2] | (h1[3] << 16), h1[4] | (h1[5] << 16), h1[6] | (h1[7] << 16));
    lds_lo[slot] = mk4(l0[0] | (l0[1] << 16), l0[2] | (l0[3] << 16), l0[4] | (l0[5] << 16), l0[6] | (l0[7] << 16));
    lds_lo[slot + 1] = mk4(l1[0] | (l1[1] << 16), l1[2] | (l1[3] << 16), l1[4] | (l1[5] << 16), l1[6] | (l1[7] << 16));
  }
}

template <int MB, bool GF32, int KG>
__global__ __launch_bounds__(256) void k_proj_down(DevCtx d, const ProjTile* __restrict__ tiles, float* __restrict__ glow,
                                                   int64_t split_stride, float grad_scale) {
  constexpr int BK = 32 * KG;                                 // rows of G per pipeline stage
  constexpr int KGRPS = 4 * KG;                               // 8-row groups per stage
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0) return;
  const MatDev m = d.mats[t.mat];
  const GAS u32x4* qt_hi = TO_GLOBAL(const u32x4, d.arena + m.qt_hi);
  const GAS u32x4* qt_lo = TO_GLOBAL(const u32x4, d.arena + m.qt_lo);

  constexpr int STAGE_SLOTS = 4 * KGRPS * 32;                 // (nblk, kgrp, n) 16-byte slots
  __shared__ u32x4 lds_hi[2 * STAGE_SLOTS];
  __shared__ u32x4 lds_lo[GF32 ? 2 * STAGE_SLOTS : 1];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps row offsets scalar
  const int mbg = t.m0 / 32 + wave % MB;                      // global rank block of this wave
  const int nb_first = (wave / MB) * MB;                      // first column block (0..3) of this wave
  const bool active = mbg < m.rp / 32;

  // G as a buffer that ends after the last row of this workgroup's slice: rows past it read as zero
  constexpr uint32_t ES = GF32 ? 4 : 2;
  const int klim = t.k1 < m.p ? t.k1 : m.p;
  const void* Gbase = ext_ptr(d, EXT_G, t.mat);
  const uint32_t row_bytes = (uint32_t)m.q * ES;
  const rsrc_t rs = make_rsrc(Gbase, (uint32_t)klim * row_bytes);
  const int col = t.n0 + 2 * lane;                            // first of the two columns this lane stages
  GCol gc;
  gc.vec = (m.q & 1) == 0 && (reinterpret_cast<uintptr_t>(Gbase) & (2 * ES - 1)) == 0;
  gc.off0 = col < m.q ? (uint32_t)col * ES : OOB;
  gc.off1 = col + 1 < m.q ? (uint32_t)(col + 1) * ES : OOB;
  // this wave stages the 8-row groups h*4 + wave, h < KG; nblk = lane/16
  const int wslot = ((lane >> 4) * KGRPS + wave) * 32 + 2 * (lane & 15);

  f32x16 acc[MB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;

  const int nstages = (t.k1 - t.k0 + BK - 1) / BK;
  const int64_t kgroups = m.pp / 8;
  // A fragments of one stage: [k-step][hi, lo]
  const GAS u32x4* pa_hi = qt_hi + (int64_t)(active ? mbg : 0) * kgroups * 32;     // uniform over the wave
  const GAS u32x4* pa_lo = qt_lo + (int64_t)(active ? mbg : 0) * kgroups * 32;
  const uint32_t agmax = (uint32_t)kgroups * 32u - 64u;                           // last k-step of the plane row block
  u32x4 a_cur[4 * KG], a_nxt[4 * KG];
  auto load_a = [&](u32x4* dst, int kr) {
#pragma unroll
    for (int ks = 0; ks < 2 * KG; ++ks) {
      uint32_t ag = (uint32_t)(kr / 8 + 2 * ks) * 32u;
      ag = (ag < agmax ? ag : agmax) + (uint32_t)lane;        // a stage may reach past the padded height
      dst[2 * ks] = pa_hi[ag];
      dst[2 * ks + 1] = pa_lo[ag];
    }
  };
  GStage<GF32> st[KG];
#pragma unroll
  for (int h = 0; h < KG; ++h) load_gstage<GF32>(st[h], rs, row_bytes, t.k0 + 8 * (h * 4 + wave), gc);
  load_a(a_cur, t.k0);
#pragma unroll
  for (int h = 0; h < KG; ++h) store_gstage<GF32>(st[h], lds_hi, lds_lo, wslot + h * 4 * 32);
  __syncthreads();

  for (int s = 0; s < nstages; ++s) {
    const int kr = t.k0 + s * BK;
    if (s + 1 < nstages) {
#pragma unroll
      for (int h = 0; h < KG; ++h) load_gstage<GF32>(st[h], rs, row_bytes, kr + BK + 8 * (h * 4 + wave), gc);
      load_a(a_nxt, kr + BK);
    }
    ISSUE_FENCE();
    if (active) {
      const u32x4* bh = lds_hi + (s & 1) * STAGE_SLOTS;
      const u32x4* bl = lds_lo + (GF32 ? (s & 1) * STAGE_SLOTS : 0);
#pragma unroll
      for (int ks = 0; ks < 2 * KG; ++ks) {
        bf16x8 a_hi = as_bf(a_cur[2 * ks]);
        bf16x8 a_lo = as_bf(a_cur[2 * ks + 1]);
#pragma unroll
        for (int a = 0; a < MB; ++a) {
          int bslot = ((nb_first + a) * KGRPS + 2 * ks + (lane >> 5)) * 32 + (lane & 31);
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
    ISSUE_FENCE();
    if (s + 1 < nstages) {
#pragma unroll
      for (int h = 0; h < KG; ++h)
        store_gstage<GF32>(st[h], lds_hi + ((s + 1) & 1) * STAGE_SLOTS, lds_lo + (GF32 ? ((s + 1) & 1) * STAGE_SLOTS : 0),
                           wslot + h * 4 * 32);
#pragma unroll
      for (int i = 0; i < 4 * KG; ++i) a_cur[i] = a_nxt[i];
    }
    __syncthreads();
  }

  if (!active) return;
  // accumulator register v of lane l: rank index 32*mbg + 8*(v/4) + 4*(l/32) + v%4, column 32*nbg + l%32
  GAS float* out = TO_GLOBAL(float, glow) + (int64_t)t.split * split_stride + m.lr_off;
  const int64_t rgroups = m.rp / 8;
#pragma unroll
  for (int a = 0; a < MB; ++a) {
    int nbg = t.n0 / 32 + nb_first + a;
    if (nbg >= m.qp / 32) continue;
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      int64_t o = (((int64_t)nbg * rgroups + 4 * mbg + vq) * 32 + (lane & 31)) * 8 + 4 * (lane >> 5);
      f32x4 val;
      val.x = grad_scale * acc[a][4 * vq];     val.y = grad_scale * acc[a][4 * vq + 1];
      val.z = grad_scale * acc[a][4 * vq + 2]; val.w = grad_scale * acc[a][4 * vq + 3];
      *reinterpret_cast<GAS f32x4*>(out + o) = val;
    }
  }
}

hipError_t launch_proj_down(const DevCtx& d, const ProjTile* tiles, int ntiles, int mb, float* glow, int64_t split_stride,
                            float grad_scale, bool g_is_f32, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  dim3 grid(ntiles), block(256);
#define LORDO_DOWN(MBV)                                                                                            \
  if (g_is_f32) hipLaunchKernelGGL((k_proj_down<MBV, true, 1>), grid, block, 0, s, d, tiles, glow, split_stride, grad_scale); \
  else hipLaunchKernelGGL((k_proj_down<MBV, false, 2>), grid, block, 0, s, d, tiles, glow, split_stride, grad_scale);
  if (mb == 4) { LORDO_DOWN(4) } else if (mb == 2) { LORDO_DOWN(2) } else { LORDO_DOWN(1) }
#undef LORDO_DOWN
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Up-projection with the weight update fused.  Workgroup tile 128 x 128 of W, 4 waves in a
// 2 x 2 grid, each wave 64 x 64 = 2 x 2 accumulator blocks.  Operand fragments come straight
// from the packed planes (one coalesced 1 KiB read per wave and fragment), double-buffered in
// registers; the W tile is fetched before the contraction so its latency hides behind it.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_proj_up(DevCtx d, const ProjTile* __restrict__ tiles,
                                                 const uint16_t* __restrict__ n_hi, const uint16_t* __restrict__ n_lo, float lr) {
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0) return;
  const MatDev m = d.mats[t.mat];
  const GAS u32x4* qa_hi = TO_GLOBAL(const u32x4, d.arena + m.qa_hi);
  const GAS u32x4* qa_lo = TO_GLOBAL(const u32x4, d.arena + m.qa_lo);
  const GAS u32x4* nh = TO_GLOBAL(const u32x4, n_hi + m.lr_off);
  const GAS u32x4* nl = TO_GLOBAL(const u32x4, n_lo + m.lr_off);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps row offsets scalar
  const int mb0 = t.m0 / 32 + 2 * (wave & 1);
  const int nb0 = t.n0 / 32 + 2 * (wave >> 1);
  const int mblocks = m.pp / 32, nblocks = m.qp / 32;
  if (mb0 >= mblocks || nb0 >= nblocks) return;
  const int p = m.p, q = m.q;
  const int64_t rgroups = m.rp / 8;
  int mbc[2], nbc[2];          // clamped block indices: loads stay inside the planes, stores are masked
  mbc[0] = mb0; mbc[1] = mb0 + 1 < mblocks ? mb0 + 1 : mb0;
  nbc[0] = nb0; nbc[1] = nb0 + 1 < nblocks ? nb0 + 1 : nb0;

  // accumulator register v of block (a, b): row 32*(mb0+a) + 8*(v/4) + 4*(lane/32) + v%4,
  // column 32*(nb0+b) + lane%32.  W is a buffer of p*q floats: the lane supplies the byte offset
  // of (row 4*(lane/32), its column) or an out-of-range offset if the column is outside the
  // matrix; the row of (a, v) is a scalar offset; rows past p fall outside the buffer.
  const uint32_t row_bytes = (uint32_t)q * 4u;
  const rsrc_t rw = make_rsrc(ext_ptr(d, EXT_W, t.mat), (uint32_t)p * row_bytes);
  uint32_t voff[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    int colw = 32 * (nb0 + b) + (lane & 31);
    voff[b] = colw < q ? (uint32_t)(4 * (lane >> 5)) * row_bytes + (uint32_t)colw * 4u : OOB;
  }
  float wv[2][2][16];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const uint32_t soff = (uint32_t)(32 * (mb0 + a) + 8 * (v >> 2) + (v & 3)) * row_bytes;
#pragma unroll
      for (int b = 0; b < 2; ++b)
        wv[a][b][v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rw, voff[b], soff, 0));
    }
  ISSUE_FENCE();

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  const int ksteps = m.rp / 16;                    // even: rp is a multiple of 32
  // uniform plane pointers of the two row blocks and two column blocks; the lane adds its index
  const GAS u32x4* pah0 = qa_hi + (int64_t)mbc[0] * rgroups * 32;
  const GAS u32x4* pah1 = qa_hi + (int64_t)mbc[1] * rgroups * 32;
  const GAS u32x4* pal0 = qa_lo + (int64_t)mbc[0] * rgroups * 32;
  const GAS u32x4* pal1 = qa_lo + (int64_t)mbc[1] * rgroups * 32;
  const GAS u32x4* pbh0 = nh + (int64_t)nbc[0] * rgroups * 32;
  const GAS u32x4* pbh1 = nh + (int64_t)nbc[1] * rgroups * 32;
  const GAS u32x4* pbl0 = nl + (int64_t)nbc[0] * rgroups * 32;
  const GAS u32x4* pbl1 = nl + (int64_t)nbc[1] * rgroups * 32;
  struct Frags { u32x4 ah[2], al[2], bh[2], bl[2]; };
  auto load_frags = [&](Frags& f, int ks) {
    const uint32_t o = (uint32_t)ks * 64u + (uint32_t)lane;
    f.ah[0] = pah0[o]; f.al[0] = pal0[o];
    f.ah[1] = pah1[o]; f.al[1] = pal1[o];
    f.bh[0] = pbh0[o]; f.bl[0] = pbl0[o];
    f.bh[1] = pbh1[o]; f.bl[1] = pbl1[o];
  };
  auto compute = [&](const Frags& f) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.ah[a]), as_bf(f.bh[b]), acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.ah[a]), as_bf(f.bl[b]), acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.al[a]), as_bf(f.bh[b]), acc[a][b], 0, 0, 0);
      }
  };
  Frags f0, f1;
  load_frags(f0, 0);
  for (int ks = 0; ks < ksteps; ks += 2) {
    load_frags(f1, ks + 1);
    ISSUE_FENCE();
    compute(f0);
    if (ks + 2 < ksteps) load_frags(f0, ks + 2);
    ISSUE_FENCE();
    compute(f1);
  }
  ISSUE_FENCE();

#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const uint32_t soff = (uint32_t)(32 * (mb0 + a) + 8 * (v >> 2) + (v & 3)) * row_bytes;
#pragma unroll
      for (int b = 0; b < 2; ++b)
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(fmaf(-lr, acc[a][b][v], wv[a][b][v])), rw, voff[b], soff, 0);
    }
}

hipError_t launch_proj_up(const DevCtx& d, const ProjTile* tiles, int ntiles, const uint16_t* n_hi,
                          const uint16_t* n_lo, float lr, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_proj_up, dim3(ntiles), dim3(256), 0, s, d, tiles, n_hi, n_lo, lr);
  return hipGetLastError();
}

}  // namespace lordo
