// Projection GEMMs of the local step on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
//   down:  g = Q^T (s G)      (Sec. 2; Alg. 1 "low-rank gradient signal")   contraction over the p rows
//   up:    W <- W - eta Q N   (Sec. 2; Alg. 1 parameter update)             contraction over the rank
// with their variants (error feedback, full-rank QHM term, residual update, outer step from the up-link
// buffers), and the range-finder products of the refresh that have the same shapes: Z = Src^T Y runs on the
// down-projection kernel, Y = Src B on k_src_times_block (contraction over the q columns).
//
// fp32 operands the library owns (Q, N) are kept as two bf16 planes hi + lo (x = hi + lo up to
// 2^-17 relative), already in the lane order of the MFMA operand fragment, so a fragment is one
// 16-byte load per lane.  The bf16 gradient is exact; the fp32 sum s G + E of the error feedback is split on the fly
// (fp32 gradients do not come here: their products run in the grouped GEMM with three-term operands).
//   down:  acc += Qhi^T G + Qlo^T G                      (+ Qhi^T Alo for a staged fp32 sum A)
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


__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {       // the hardware's packed round-to-nearest-even conversion
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2_ __attribute__((ext_vector_type(2)));
  const f32x2_ v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// two fp32 values -> packed bf16 hi parts (nearest-even) and packed bf16 parts of what is left: x = hi + lo to 2^-17
__device__ __forceinline__ void split2_bf(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  hi = pack_bf16_rne(x0, x1);
  lo = pack_bf16_rne(x0 - __uint_as_float(hi << 16), x1 - __uint_as_float(hi & 0xffff0000u));
}

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// Compiler-level fence: keeps the loads issued before it from being sunk to their first use
// (prefetches must be in flight while the matrix cores work); it emits no instruction.
#define ISSUE_FENCE() asm volatile("" ::: "memory")
// Byte offset given to a lane whose column lies outside the matrix: beyond the range of any resource smaller than 2 GiB.
// lordo_init admits larger matrices only with sides that are multiples of 256, where no such lane exists.
constexpr uint32_t OOB = 0x80000000u;
// Cache policy of the caller's matrices.  G is read once and W is read once and written once per
// step, hundreds of megabytes each: they are marked non-temporal so that they pass through L2 and
// the last-level cache as streaming lines and leave both to the operands that are reused (the Q and
// N planes, the low-rank state).  Measured on the c2 set: one local step 0.272 -> 0.232 ms.
constexpr int STREAM = 2;                    // "nt" bit of the buffer instructions' cache policy
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// Direct global-to-LDS load of one 1 KiB operand fragment: lane i's 16 bytes land at
// lds_dst_wave_base + i (checked on the hardware); the LDS address must be uniform over the wave.
#define LDS_AS __attribute__((address_space(3)))
__device__ __forceinline__ void dma16(const GAS u32x4* src, u32x4* lds_dst_wave_base) {
  __builtin_amdgcn_global_load_lds((const GAS void*)src, (LDS_AS void*)lds_dst_wave_base, 16, 0, 0);
}

// ---------------------------------------------------------------------------------------
// Staging of gradient rows for the register-staged down-projection kernel: the G tile of a stage is transposed
// in registers and written to LDS in fragment order, slot (nblk, kgrp, n) = the 16-byte vector
// G[k0 + 8*kgrp + 0..7][n0 + 32*nblk + n].  Each lane stages two adjacent columns of 8 consecutive rows.
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

// Rows krow .. krow+7 (krow uniform over the wave) of the lane's two columns.  The resource ends
// after row `rows`; a row at or beyond it is clamped to `rows`, which puts the scalar offset exactly
// at the end of the resource, so every lane of that access is out of range and reads zero.
template <bool GF32, int AUX>     // AUX: cache policy of the loads (STREAM where G is read once, 0 where rank tiles re-read it)
__device__ __forceinline__ void load_gstage(GStage<GF32>& st, rsrc_t rs, uint32_t row_bytes, int krow, int rows, const GCol& gc) {
  if (gc.vec) {                     // uniform branch, taken once per stage
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t soff = (uint32_t)(krow + i < rows ? krow + i : rows) * row_bytes;       // scalar
      if constexpr (!GF32) {
        st.x[i] = __builtin_amdgcn_raw_buffer_load_b32(rs, gc.off0, soff, AUX);
      } else {
        u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rs, gc.off0, soff, AUX);
        st.x[2 * i] = t.x;
        st.x[2 * i + 1] = t.y;
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t soff = (uint32_t)(krow + i < rows ? krow + i : rows) * row_bytes;
      if constexpr (!GF32) {
        uint32_t lo = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, gc.off0, soff, AUX);
        uint32_t hi = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, gc.off1, soff, AUX);
        st.x[i] = lo | (hi << 16);
      } else {
        st.x[2 * i] = __builtin_amdgcn_raw_buffer_load_b32(rs, gc.off0, soff, AUX);
        st.x[2 * i + 1] = __builtin_amdgcn_raw_buffer_load_b32(rs, gc.off1, soff, AUX);
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
    // column 0 of the lane: floats st.x[0], st.x[2], ...; column 1: st.x[1], st.x[3], ...; rows pair up into packed words
    uint32_t h0[4], l0[4], h1[4], l1[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      split2_bf(__uint_as_float(st.x[4 * i]), __uint_as_float(st.x[4 * i + 2]), h0[i], l0[i]);
      split2_bf(__uint_as_float(st.x[4 * i + 1]), __uint_as_float(st.x[4 * i + 3]), h1[i], l1[i]);
    }
    lds_hi[slot] = mk4(h0[0], h0[1], h0[2], h0[3]);
    lds_hi[slot + 1] = mk4(h1[0], h1[1], h1[2], h1[3]);
    lds_lo[slot] = mk4(l0[0], l0[1], l0[2], l0[3]);
    lds_lo[slot + 1] = mk4(l1[0], l1[1], l1[2], l1[3]);
  }
}

// grad_scale * G + E of one stage (error feedback, Alg. 1: the projected matrix is the gradient plus the residual)
template <bool GF32, bool EF32>     // EF32: the residual is stored in fp32 (else bf16: widened exactly)
__device__ __forceinline__ void add_residual(GStage<true>& out, const GStage<GF32>& g, const GStage<EF32>& e, float scale) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float g0, g1, e0, e1;
    if constexpr (GF32) { g0 = __uint_as_float(g.x[2 * i]); g1 = __uint_as_float(g.x[2 * i + 1]); }
    else { g0 = __uint_as_float(g.x[i] << 16); g1 = __uint_as_float(g.x[i] & 0xffff0000u); }
    if constexpr (EF32) { e0 = __uint_as_float(e.x[2 * i]); e1 = __uint_as_float(e.x[2 * i + 1]); }
    else { e0 = __uint_as_float(e.x[i] << 16); e1 = __uint_as_float(e.x[i] & 0xffff0000u); }
    out.x[2 * i] = __float_as_uint(fmaf(scale, g0, e0));
    out.x[2 * i + 1] = __float_as_uint(fmaf(scale, g1, e1));
  }
}

// ---------------------------------------------------------------------------------------
// Down-projection, main path (rank tile of 128, bf16 G): 8 waves, output tile 128 rank indices x
// 256 columns.  Wave w owns rank block w % 4 and the four column blocks of half w / 4.
// Per stage of 32 rows of G: the G tile (32 x 256) is read once, transposed in registers and staged
// in LDS in fragment order (wave w stages the 8-row group w / 2 of column half w % 2); the Q
// fragments of the stage (16 KiB) come in ONCE per workgroup by direct global-to-LDS loads.
//
// Software pipeline.  In iteration s the workgroup multiplies stage s (in LDS) while the Q
// fragments of stage s+1 and the G rows of stage s+2 are in flight; the G rows of stage s+1, read
// one iteration earlier, wait in registers and go to LDS at the end of the iteration.  The
// global-to-LDS loads are issued from inline assembly: the compiler would otherwise make every LDS
// access that follows such a load wait for it, which serialises memory latency and arithmetic.
// The waits are therefore explicit: vector-memory operations complete in issue order, the
// Q fragments of stage s+1 are issued BEFORE the G loads of stage s+2, so "at most one stage of G
// loads outstanding" implies that the fragments have landed.
// ---------------------------------------------------------------------------------------
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// Lane i's 16 bytes land at lds_dst_wave_base + i.  M0 carries the LDS address; one wait state is
// required between the write of M0 and the load that uses it.
__device__ __forceinline__ void dma16_async(const GAS u32x4* src, u32x4* lds_dst_wave_base) {
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(LDS_AS void*)lds_dst_wave_base;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr) : "memory", "m0");
}
// The same with the non-temporal bit: for data that is read once (streaming lines in L2 and the last-level cache).
__device__ __forceinline__ void dma16_async_nt(const GAS u32x4* src, u32x4* lds_dst_wave_base) {
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(LDS_AS void*)lds_dst_wave_base;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(src), "s"(lds_addr) : "memory", "m0");
}
#pragma clang diagnostic pop

// Wait until at most N vector-memory operations are outstanding and all LDS operations are done,
// then the workgroup barrier (no wait for the N youngest loads, unlike __syncthreads()).
#define WAIT_VM_BARRIER(N) asm volatile("s_waitcnt vmcnt(" #N ") lgkmcnt(0)\n\ts_barrier" ::: "memory")

// Low-rank Adam on four consecutive state elements (Alg. 1, moment and direction lines; the same
// arithmetic, in the same order, as the stand-alone Adam kernel).
struct FusedAdam {
  float* u;
  float* v;
  uint16_t* n_hi;
  uint16_t* n_lo;
  float b1, omb1, b2, omb2, eps;
  const StepDev* step;        // bias corrections of the current step (device memory: a replayed graph sees its own step)
  float qw, qg;               // update bracket (qw u_hat + qg g) / den: 1, 0 for "No QHM"; omega, 1 - omega for low-rank QHM
  // 256-rank tiles only (the 128-rank kernel has no registers to spare):
  uint16_t* g_hi;             // error feedback: the bf16 hi / lo operand planes of g for the residual update (else null)
  uint16_t* g_lo;
  float* colpart;             // full-rank QHM: per column and rank block of 32, the sum of sqrt(v_hat) + eps (else null)
};

// Returns the sum of the four denominators sqrt(v_hat) + eps (the full-rank QHM scale is their mean over the rank).
template <bool EXTRA>
__device__ __forceinline__ float adam4(const FusedAdam& f, int64_t at, f32x4 g, f32x4 uu, f32x4 vv) {
  float nn[4];
  float dsum = 0.f;
  const float inv_c1 = f.step->inv_c1, inv_c2 = f.step->inv_c2;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float un = fmaf(f.b1, uu[e], f.omb1 * g[e]);
    const float vn = fmaf(f.b2, vv[e], f.omb2 * (g[e] * g[e]));
    uu[e] = un;
    vv[e] = vn;
    const float den = sqrtf(vn * inv_c2) + f.eps;
    dsum += den;
    // with qw = 1, qg = 0 bit-identical to u_hat / den; eps == 0 and no gradient yet (e.g. the padding): zero, not 0 / 0
    nn[e] = den == 0.f ? 0.f : fmaf(f.qg, g[e], f.qw * (un * inv_c1)) / den;
  }
  __builtin_nontemporal_store(uu, TO_GLOBAL(f32x4, f.u + at));       // next use is a whole step away
  __builtin_nontemporal_store(vv, TO_GLOBAL(f32x4, f.v + at));
  uint32_t h0, l0, h1, l1;
  split2_bf(nn[0], nn[1], h0, l0);
  split2_bf(nn[2], nn[3], h1, l1);
  u32x2 ph = {h0, h1}, pl = {l0, l1};
  *TO_GLOBAL(u32x2, f.n_hi + at) = ph;
  *TO_GLOBAL(u32x2, f.n_lo + at) = pl;
  if constexpr (EXTRA) {
    if (f.g_hi) {
      split2_bf(g[0], g[1], h0, l0);
      split2_bf(g[2], g[3], h1, l1);
      ph = u32x2{h0, h1}; pl = u32x2{l0, l1};
      *TO_GLOBAL(u32x2, f.g_hi + at) = ph;
      *TO_GLOBAL(u32x2, f.g_lo + at) = pl;
    }
  }
  return dsum;
}
// Full-rank QHM scale from inside a fused epilogue: `dsum` holds the lane's sixteen denominators of one accumulator
// block (rank indices 8 vq + 4 (lane / 32) + e of column lane % 32); the other sixteen rank indices of the block sit
// in lane ^ 32.  Fixed order of additions.
__device__ __forceinline__ void store_colpart(const FusedAdam& f, const MatDev& m, int nbg, int mbg, int lane, float dsum) {
  const float other = __shfl_xor(dsum, 32);
  const float total = (lane < 32) ? dsum + other : other + dsum;
  if (lane < 32) f.colpart[m.lr_off / 32 + ((int64_t)nbg * (m.rp / 32) + mbg) * 32 + lane] = total;
}

// 8 waves, 256-column tiles: wave w owns column half w / 4 (four column blocks) and RB rank blocks,
// w % 4 + 4*rb: the tile spans 128*RB rank indices.  RB = 2 (ranks from 256 up) halves the number of
// passes over G and the LDS reads per MFMA (each G fragment feeds two rank blocks); its 96 KiB of
// LDS admit one workgroup per compute unit.
// VEC: every G row is read with aligned 4-byte accesses (8 loads per stage, else 16).
// GONCE: one rank tile per column block, G is read once (streaming loads).
// A tile marked `fuse` holds the whole contraction (no split-K): its epilogue applies Adam to its
// elements of the low-rank state instead of leaving that to a separate pass over g.
// EF: error feedback (Alg. 1): the contraction runs over A = grad_scale * G + E, E the fp32 residual in the
// arena.  E rows travel with the G rows of their stage; the sum is formed in registers when the stage
// goes to LDS, as bf16 hi and lo planes (one more 16 KiB plane per stage and a third MFMA pass), and
// the result is not scaled again.
// EFM = 2: the projected matrix is an fp32 matrix alone (no G): the fp32 source of a subspace refresh, taken
// from the caller's source table -- the product Z = Src^T Y of the power iteration has the shape of g = Q^T G.
// EFM = 3: error feedback with the residual stored in bf16 (widened exactly; the sum is formed in fp32 as before).
template <int RB, bool VEC, bool GONCE, int EFM>
__global__ __launch_bounds__(512) void k_proj_down_pipe(DevCtx d, const ProjTile* __restrict__ tiles, float* __restrict__ glow,
                                                        int64_t split_stride, float grad_scale, FusedAdam fa) {
  constexpr bool EF = EFM != 0;                                // an fp32 operand is staged: hi and lo planes, three passes
  constexpr bool SRC32 = EFM == 2;                             // ... and it is the whole operand
  constexpr bool E32 = EFM != 3;                               // storage type of the second operand (residual or source)
  constexpr uint32_t EES = E32 ? 4u : 2u;
  constexpr int BK = 32;
  constexpr int NW = 8;
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0 || mat_skipped(d, t.mat)) return;
  const MatDev m = d.mats[t.mat];
  const GAS u32x4* qt_hi = TO_GLOBAL(const u32x4, d.arena + m.qt_hi);
  const GAS u32x4* qt_lo = TO_GLOBAL(const u32x4, d.arena + m.qt_lo);

  constexpr int GSLOTS = 8 * 4 * 32;                           // (nblk, kgrp, n) 16-byte slots of one stage: 16 KiB
  constexpr int ASLOTS = 4 * RB * 2 * 2 * 64;                  // (mblk, kstep, plane, lane): 16 KiB per 128 rank indices
  extern __shared__ u32x4 lds_dyn[];                           // 2 stages of each: 64 KiB (RB = 1) or 96 KiB (RB = 2), + 32 KiB with EF
  u32x4* gfrag = lds_dyn;
  u32x4* glo = lds_dyn + 2 * GSLOTS;                           // EF: lo plane of the staged sum
  u32x4* afrag = lds_dyn + (EF ? 4 : 2) * GSLOTS;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mb = wave & 3, nh = wave >> 2;                     // compute role
  const int kgrp = wave >> 1, half = wave & 1;                 // G staging role: 8-row group, column half
  const int rblocks = m.rp / 32;
  int mbg[RB];
  bool active[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    mbg[rb] = t.m0 / 32 + mb + 4 * rb;
    active[rb] = mbg[rb] < rblocks;
  }

  const int klim = t.k1 < m.p ? t.k1 : m.p;
  const void* Gbase = ext_ptr(d, EXT_G, t.mat);
  const uint32_t row_bytes = (uint32_t)m.q * 2u;
  const rsrc_t rs = make_rsrc(Gbase, (uint32_t)klim * row_bytes);
  const int col = t.n0 + 128 * half + 2 * lane;
  GCol gc;
  gc.vec = VEC;
  gc.off0 = col < m.q ? (uint32_t)col * 2u : OOB;
  gc.off1 = col + 1 < m.q ? (uint32_t)(col + 1) * 2u : OOB;
  const int wslot = ((4 * half + (lane >> 4)) * 4 + kgrp) * 32 + 2 * (lane & 15);
  // residual E: fp32 p x q in the arena, same rows and columns (8-byte accesses need an even q: VEC)
  const uint32_t erow_bytes = (uint32_t)m.q * EES;
  const rsrc_t re = SRC32 ? make_rsrc(ext_ptr(d, EXT_SRC, t.mat), (uint32_t)klim * erow_bytes)
                          : (EF ? make_rsrc(d.arena + m.err, (uint32_t)klim * erow_bytes) : rs);
  GCol ge;
  ge.vec = VEC;
  ge.off0 = col < m.q ? (uint32_t)col * EES : OOB;
  ge.off1 = col + 1 < m.q ? (uint32_t)(col + 1) * EES : OOB;

  // Q fragments of a stage: (mblk, kstep) pairs, both planes each; 8*RB pairs, RB per wave
  const int64_t kgroups = m.pp / 8;
  const int kgmax = (int)kgroups - 2;
  auto issue_a = [&](int kr, int sbuf) {
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      const int pair = wave * RB + j;                          // 0 .. 8*RB-1
      const int fmb = pair >> 1, fks = pair & 1;
      const int fmbg = t.m0 / 32 + fmb < rblocks ? t.m0 / 32 + fmb : rblocks - 1;
      int kg = kr / 8 + 2 * fks;
      kg = kg < kgmax ? kg : kgmax;                            // a stage may reach past the padded height
      const int64_t src = ((int64_t)fmbg * kgroups + kg) * 32 + lane;
      u32x4* dst = afrag + sbuf * ASLOTS + pair * 2 * 64;
      dma16_async(qt_hi + src, dst);
      dma16_async(qt_lo + src, dst + 64);
    }
  };

  f32x16 acc[RB][4];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][a][i] = 0.f;

  // Operand fragments of one k-step of 16: RB pairs of Q planes and the four G column blocks.
  struct Frags { u32x4 ah[RB], al[RB], b[4], bl[EF ? 4 : 1]; };
  auto load_frags = [&](Frags& f, int sbuf, int ks) {
    const u32x4* gb = gfrag + sbuf * GSLOTS;
    const u32x4* ab = afrag + sbuf * ASLOTS;
    if constexpr (EF) {
#pragma unroll
      for (int a = 0; a < 4; ++a) f.bl[a] = glo[sbuf * GSLOTS + ((4 * nh + a) * 4 + 2 * ks + (lane >> 5)) * 32 + (lane & 31)];
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      f.ah[rb] = ab[(((mb + 4 * rb) * 2 + ks) * 2 + 0) * 64 + lane];
      f.al[rb] = ab[(((mb + 4 * rb) * 2 + ks) * 2 + 1) * 64 + lane];
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) f.b[a] = gb[((4 * nh + a) * 4 + 2 * ks + (lane >> 5)) * 32 + (lane & 31)];
  };
  auto mfma_frags = [&](const Frags& f) {
    // an absent second rank block (rank not a multiple of 256) is multiplied anyway: its Q fragments
    // repeat the last block and its accumulators are never stored; no branch splits the MFMA run
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        acc[rb][a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.ah[rb]), as_bf(f.b[a]), acc[rb][a], 0, 0, 0);
        acc[rb][a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.al[rb]), as_bf(f.b[a]), acc[rb][a], 0, 0, 0);
        if constexpr (EF)
          acc[rb][a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.ah[rb]), as_bf(f.bl[a]), acc[rb][a], 0, 0, 0);
      }
  };
  auto compute = [&](int sbuf) {
    if (!active[0]) return;                                    // rank blocks are filled from the lowest: nothing to do
    if constexpr (RB == 2) {
      // both k-steps' fragments are requested before the first MFMA: the second set lands while the
      // sixteen MFMAs of the first run
      Frags f0, f1;
      load_frags(f0, sbuf, 0);
      load_frags(f1, sbuf, 1);
      mfma_frags(f0);
      mfma_frags(f1);
    } else {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        Frags f;
        load_frags(f, sbuf, ks);
        mfma_frags(f);
      }
    }
  };

  const int nstages = (t.k1 - t.k0 + BK - 1) / BK;
  const int krow0 = t.k0 + 8 * kgrp;
  // Rows at or beyond the end of the slice are read as zero (the loader clamps the row to the size of
  // the resource), so the loads of stages past the last one are issued unconditionally: the number of
  // outstanding loads is then the same in every iteration, which the explicit waits rely on.
  GStage<false> st0, st1;
  GStage<E32> se0, se1;                                        // EF: rows of E of the same stages
  constexpr int GAUX = GONCE ? STREAM : 0;
  // outstanding loads of one stage: 8 (or 16 two-byte ones) of G, as many again of E
  constexpr int NLOADS = ((SRC32 ? 0 : 1) + (EF ? 1 : 0)) * (VEC ? 8 : 16);
  auto wait_one_stage = [&]() {
    if constexpr (NLOADS == 8) WAIT_VM_BARRIER(8);
    else if constexpr (NLOADS == 16) WAIT_VM_BARRIER(16);
    else WAIT_VM_BARRIER(32);
  };
  auto stage_out = [&](const GStage<false>& g, const GStage<E32>& e, int sbuf) {
    if constexpr (SRC32) {
      store_gstage<true>(e, gfrag + sbuf * GSLOTS, glo + sbuf * GSLOTS, wslot);
    } else if constexpr (EF) {
      GStage<true> sa;
      add_residual<false, E32>(sa, g, e, grad_scale);
      store_gstage<true>(sa, gfrag + sbuf * GSLOTS, glo + sbuf * GSLOTS, wslot);
    } else {
      store_gstage<false>(g, gfrag + sbuf * GSLOTS, nullptr, wslot);
    }
  };
  issue_a(t.k0, 0);
  if constexpr (!SRC32) load_gstage<false, GAUX>(st0, rs, row_bytes, krow0, klim, gc);                  // stage 0
  if constexpr (EF) load_gstage<E32, GAUX>(se0, re, erow_bytes, krow0, klim, ge);
  if constexpr (!SRC32) load_gstage<false, GAUX>(st1, rs, row_bytes, krow0 + BK, klim, gc);             // stage 1
  if constexpr (EF) load_gstage<E32, GAUX>(se1, re, erow_bytes, krow0 + BK, klim, ge);
  stage_out(st0, se0, 0);
  wait_one_stage();

  // one iteration; NEXT holds stage s+1 (read one iteration ago), LOAD receives stage s+2
#define LORDO_DOWN_ITER(S, NEXT, LOAD, NEXTE, LOADE)                                              \
  {                                                                                               \
    const int kr = t.k0 + (S) * BK;                                                               \
    if ((S) + 1 < nstages) issue_a(kr + BK, ((S) + 1) & 1);                                       \
    if constexpr (!SRC32) load_gstage<false, GAUX>(LOAD, rs, row_bytes, krow0 + ((S) + 2) * BK, klim, gc); \
    if constexpr (EF) load_gstage<E32, GAUX>(LOADE, re, erow_bytes, krow0 + ((S) + 2) * BK, klim, ge); \
    ISSUE_FENCE();                                                                                \
    compute((S) & 1);                                                                             \
    ISSUE_FENCE();                                                                                \
    stage_out(NEXT, NEXTE, ((S) + 1) & 1);                                                        \
    wait_one_stage();                                                                             \
  }
  // two stages per trip so that the two register sets alternate statically; the odd last stage is
  // peeled (an exit in the middle of the trip would make the compiler treat loads as outstanding
  // at the loop head that are not)
  int s = 0;
  for (; s + 1 < nstages; s += 2) {
    LORDO_DOWN_ITER(s, st1, st0, se1, se0)
    LORDO_DOWN_ITER(s + 1, st0, st1, se0, se1)
  }
  if (s < nstages) LORDO_DOWN_ITER(s, st1, st0, se1, se0)
#undef LORDO_DOWN_ITER

  const int64_t base = m.lr_off;
  GAS float* out = TO_GLOBAL(float, glow) + (int64_t)t.split * split_stride + base;
  const bool fuse = t.fuse != 0 && fa.u != nullptr;            // uniform over the workgroup
  const int64_t rgroups = m.rp / 8;
  const float osc = EF ? 1.f : grad_scale;                     // with error feedback the scale went into the staged sum
  // accumulator block idx = 4 rb + a: rank block mbg[rb], column block t.n0 / 32 + 4 nh + a
  auto live = [&](int idx) { return active[idx >> 2] && t.n0 / 32 + 4 * nh + (idx & 3) < m.qp / 32; };
  // offset of the lane's four consecutive rank indices of that block's column block, rank group 4*mbg + vq
  auto offset_of = [&](int idx, int vq) {
    const int nbg = t.n0 / 32 + 4 * nh + (idx & 3);
    return (((int64_t)nbg * rgroups + 4 * mbg[idx >> 2] + vq) * 32 + (lane & 31)) * 8 + 4 * (lane >> 5);
  };
  if (!fuse) {
#pragma unroll
    for (int idx = 0; idx < 4 * RB; ++idx) {
      if (!live(idx)) continue;
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        f32x4 val;
        val.x = osc * acc[idx >> 2][idx & 3][4 * vq];     val.y = osc * acc[idx >> 2][idx & 3][4 * vq + 1];
        val.z = osc * acc[idx >> 2][idx & 3][4 * vq + 2]; val.w = osc * acc[idx >> 2][idx & 3][4 * vq + 3];
        *reinterpret_cast<GAS f32x4*>(out + offset_of(idx, vq)) = val;
      }
    }
    return;
  }
  // fused Adam.  With 256-rank tiles (one workgroup per compute unit, nothing else to run while it waits) the moments of
  // the next block are requested before this one is worked on; the 128-rank tile has no registers to spare for that
  // without giving up its second workgroup per compute unit
  constexpr int PF = RB == 2 ? 1 : 0;
  f32x4 uu[1 + PF][4], vv[1 + PF][4];
  auto fetch = [&](int idx, int buf) {
    if (!live(idx)) return;
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int64_t at = base + offset_of(idx, vq);
      uu[buf][vq] = __builtin_nontemporal_load(TO_GLOBAL(const f32x4, fa.u + at));
      vv[buf][vq] = __builtin_nontemporal_load(TO_GLOBAL(const f32x4, fa.v + at));
    }
  };
  if (PF) fetch(0, 0);
#pragma unroll
  for (int idx = 0; idx < 4 * RB; ++idx) {
    if (!PF) fetch(idx, 0);
    else if (idx + 1 < 4 * RB) fetch(idx + 1, (idx + 1) & 1);
    ISSUE_FENCE();
    if (!live(idx)) continue;
    const int rb = idx >> 2, a = idx & 3;
    float dsum = 0.f;
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int64_t o = offset_of(idx, vq);
      f32x4 val;
      val.x = osc * acc[rb][a][4 * vq];     val.y = osc * acc[rb][a][4 * vq + 1];
      val.z = osc * acc[rb][a][4 * vq + 2]; val.w = osc * acc[rb][a][4 * vq + 3];
      *reinterpret_cast<GAS f32x4*>(out + o) = val;
      dsum += adam4<RB == 2>(fa, base + o, val, uu[idx & PF][vq], vv[idx & PF][vq]);
    }
    if constexpr (RB == 2) {
      if (fa.colpart) store_colpart(fa, m, t.n0 / 32 + 4 * nh + a, mbg[rb], lane, dsum);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Down-projection with the gradient moved by global-to-LDS loads only (bf16 G, q % 8 == 0, G 16-byte aligned).
// The matrix-core operand wants, per lane, 8 consecutive ROWS of one column of G, which is row-major: in the
// kernel above the rows pass through registers, are transposed there and written to LDS in fragment order.
// gfx950 can do that transposition while READING LDS (ds_read_b64_tr_b16: sixteen lanes each fetch 8 bytes,
// i.e. 4 consecutive columns of one row; the 4 x 16 block they cover -- lanes 4e .. 4e+3 hold row e -- comes
// back with lane i holding column i, one element per row e; layout checked on the hardware).  So the G tile of
// a stage (32 rows x 256 columns, 16 KiB) goes to LDS untouched, row-major, two rows per 1 KiB load, and a
// fragment is two such reads (rows 0..3 and 4..7 of the lane's 8).  No vector ALU work and no LDS write per
// stage is left, and with registers out of the path the ring can be deeper: NS stages of G and of the Q
// fragments, NS - 1 of them in flight.
// Bank spreading: a row is 512 bytes, so the 4 rows of one transposing read would meet in the same banks; the
// 16-byte unit u of row k is therefore stored at unit u ^ 4 (k % 4) of the row (the per-lane global address
// of the load picks the columns that land at each position).
// Rows past the matrix are read from its last row: the operand planes of Q are zero there.  Column segments
// past the last column are read from the last full segment (the results of such columns are never stored
// beyond the padding of the low-rank state, which nothing reads).
// ---------------------------------------------------------------------------------------
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x2 lds_read_tr16(const u32x4* lds_base, uint32_t byte_off) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (LDS_AS s16x4*)((LDS_AS char*)(LDS_AS void*)lds_base + byte_off));
  return __builtin_bit_cast(u32x2, v);
}

template <int RB, bool GONCE>
__global__ __launch_bounds__(512) void k_proj_down_tr(DevCtx d, const ProjTile* __restrict__ tiles, float* __restrict__ glow,
                                                      int64_t split_stride, float grad_scale, FusedAdam fa) {
  constexpr int BK = 32;
  constexpr int NS = RB == 2 ? 3 : 4;                          // ring depth: 4 x 32 KiB or 3 x 48 KiB
  constexpr int GSLOTS = 32 * 32;                              // 16-byte units of the raw G tile of a stage
  constexpr int ASLOTS = 4 * RB * 2 * 2 * 64;                  // (mblk, kstep, plane, lane)
  constexpr int SSLOTS = GSLOTS + ASLOTS;
  constexpr int NDMA = 2 + 2 * RB;                             // loads per wave and stage
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0 || mat_skipped(d, t.mat)) return;
  const MatDev m = d.mats[t.mat];
  const GAS u32x4* qt_hi = TO_GLOBAL(const u32x4, d.arena + m.qt_hi);
  const GAS u32x4* qt_lo = TO_GLOBAL(const u32x4, d.arena + m.qt_lo);
  extern __shared__ u32x4 lds_dyn[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mb = wave & 3, nh = wave >> 2;
  const int rblocks = m.rp / 32;
  int mbg[RB];
  bool active[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    mbg[rb] = t.m0 / 32 + mb + 4 * rb;
    active[rb] = mbg[rb] < rblocks;
  }

  // G loads of this wave: chunks 2*wave and 2*wave + 1 of a stage = rows 4*wave .. 4*wave + 3
  const GAS uint16_t* G = TO_GLOBAL(const uint16_t, ext_ptr(d, EXT_G, t.mat));
  const int p = m.p, q = m.q;
  const int last_seg = q / 8 - 1;
  int grow[2];                                                 // row inside the stage
  int64_t gcol[2];                                             // first column of the 16-byte segment this lane fetches
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    grow[j] = 4 * wave + 2 * j + (lane >> 5);
    int seg = t.n0 / 8 + ((lane & 31) ^ (4 * (grow[j] & 3)));
    seg = seg < last_seg ? seg : last_seg;
    gcol[j] = (int64_t)seg * 8;
  }
  const int64_t kgroups = m.pp / 8;
  const int kgmax = (int)kgroups - 2;
  auto issue_stage = [&](int sidx, int sbuf) {                 // NDMA loads
    const int kr = t.k0 + sidx * BK;
    u32x4* gdst = lds_dyn + sbuf * SSLOTS;
    u32x4* adst = gdst + GSLOTS;
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      const int pair = wave * RB + j;
      const int fmb = pair >> 1, fks = pair & 1;
      const int fmbg = t.m0 / 32 + fmb < rblocks ? t.m0 / 32 + fmb : rblocks - 1;
      int kg = kr / 8 + 2 * fks;
      kg = kg < kgmax ? kg : kgmax;
      const int64_t src = ((int64_t)fmbg * kgroups + kg) * 32 + lane;
      dma16_async(qt_hi + src, adst + pair * 2 * 64);
      dma16_async(qt_lo + src, adst + pair * 2 * 64 + 64);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int row = kr + grow[j];
      row = row < p ? row : p - 1;
      const GAS u32x4* gsrc = reinterpret_cast<const GAS u32x4*>(G + (int64_t)row * q + gcol[j]);
      if constexpr (GONCE) dma16_async_nt(gsrc, gdst + (2 * wave + j) * 64);
      else dma16_async(gsrc, gdst + (2 * wave + j) * 64);
    }
  };

  // transposing reads: lane = (g, i), g = lane / 16, i = lane % 16; as a source it fetches row 8 (g / 2) + i / 4
  // (+ 4 for the second read) of the k-step, columns 16 (g % 2) + 4 (i % 4) .. + 3 of the column block
  const int tg = lane >> 4, ti = lane & 15;
  uint32_t toff[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int unit = (16 * nh + 4 * (a ^ (ti >> 2)) + 2 * (tg & 1) + ((ti >> 1) & 1));    // u ^ 4 (k % 4), k % 4 = i / 4
    toff[a] = (uint32_t)((8 * (tg >> 1) + (ti >> 2)) * 512 + unit * 16 + (ti & 1) * 8);
  }

  f32x16 acc[RB][4];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][a][i] = 0.f;

  auto compute = [&](int sbuf) {
    if (!active[0]) return;
    const u32x4* gb = lds_dyn + sbuf * SSLOTS;
    const u32x4* ab = gb + GSLOTS;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      u32x4 ah[RB], al[RB], b[4];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        ah[rb] = ab[(((mb + 4 * rb) * 2 + ks) * 2 + 0) * 64 + lane];
        al[rb] = ab[(((mb + 4 * rb) * 2 + ks) * 2 + 1) * 64 + lane];
      }
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const u32x2 lo = lds_read_tr16(gb, toff[a] + (16 * ks) * 512);
        const u32x2 hi = lds_read_tr16(gb, toff[a] + (16 * ks + 4) * 512);
        b[a] = u32x4{lo.x, lo.y, hi.x, hi.y};
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          acc[rb][a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(ah[rb]), as_bf(b[a]), acc[rb][a], 0, 0, 0);
          acc[rb][a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(al[rb]), as_bf(b[a]), acc[rb][a], 0, 0, 0);
        }
    }
  };

  const int nstages = (t.k1 - t.k0 + BK - 1) / BK;
  // stages past the last one are loaded all the same (rows clamped, fragments clamped): the number of loads in
  // flight is then the same in every iteration, which the explicit waits count on
#pragma unroll
  for (int s0 = 0; s0 < NS - 1; ++s0) issue_stage(s0, s0);
  int sbuf = 0;
  for (int s = 0; s < nstages; ++s) {
    // at most NS - 2 younger stages outstanding: stage s has landed; barrier: visible to all, stage s-1 consumed by all
    if constexpr ((NS - 2) * NDMA == 8) WAIT_VM_BARRIER(8);
    else WAIT_VM_BARRIER(6);
    static_assert((NS - 2) * NDMA == 8 || (NS - 2) * NDMA == 6, "wait count");
    int nbuf = sbuf + NS - 1;
    nbuf = nbuf >= NS ? nbuf - NS : nbuf;
    issue_stage(s + NS - 1, nbuf);                              // into the buffer of stage s-1
    ISSUE_FENCE();
    compute(sbuf);
    sbuf = sbuf + 1 == NS ? 0 : sbuf + 1;
  }
  WAIT_VM_BARRIER(0);             // the loads past the last stage must land before this workgroup's LDS is released

  const int64_t base = m.lr_off;
  GAS float* out = TO_GLOBAL(float, glow) + (int64_t)t.split * split_stride + base;
  const bool fuse = t.fuse != 0 && fa.u != nullptr;
  const int64_t rgroups = m.rp / 8;
  // accumulator block idx = 4 rb + a: rank block mbg[rb], column block t.n0 / 32 + 4 nh + a
  auto live = [&](int idx) { return active[idx >> 2] && t.n0 / 32 + 4 * nh + (idx & 3) < m.qp / 32; };
  auto offset_of = [&](int idx, int vq) {
    const int nbg = t.n0 / 32 + 4 * nh + (idx & 3);
    return (((int64_t)nbg * rgroups + 4 * mbg[idx >> 2] + vq) * 32 + (lane & 31)) * 8 + 4 * (lane >> 5);
  };
  // fused Adam: the moments of the NEXT block are requested before this one is worked on, so that the epilogue of a
  // tile exposes one memory latency and not one per block (this workgroup has the compute unit to itself: nothing
  // else runs while it waits)
  f32x4 uu[2][4], vv[2][4];
  auto fetch = [&](int idx, int buf) {
    if (!live(idx)) return;
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int64_t at = base + offset_of(idx, vq);
      uu[buf][vq] = __builtin_nontemporal_load(TO_GLOBAL(const f32x4, fa.u + at));
      vv[buf][vq] = __builtin_nontemporal_load(TO_GLOBAL(const f32x4, fa.v + at));
    }
  };
  if (fuse) fetch(0, 0);
#pragma unroll
  for (int idx = 0; idx < 4 * RB; ++idx) {
    if (fuse && idx + 1 < 4 * RB) fetch(idx + 1, (idx + 1) & 1);
    ISSUE_FENCE();
    if (!live(idx)) continue;
    const int rb = idx >> 2, a = idx & 3;
    float dsum = 0.f;
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int64_t o = offset_of(idx, vq);
      f32x4 val;
      val.x = grad_scale * acc[rb][a][4 * vq];     val.y = grad_scale * acc[rb][a][4 * vq + 1];
      val.z = grad_scale * acc[rb][a][4 * vq + 2]; val.w = grad_scale * acc[rb][a][4 * vq + 3];
      *reinterpret_cast<GAS f32x4*>(out + o) = val;
      if (fuse) dsum += adam4<RB == 2>(fa, base + o, val, uu[idx & 1][vq], vv[idx & 1][vq]);
    }
    if constexpr (RB == 2) {
      if (fuse && fa.colpart) store_colpart(fa, m, t.n0 / 32 + 4 * nh + a, mbg[rb], lane, dsum);
    }
  }
}

template <int RB, bool GONCE>
static hipError_t launch_down_tr(dim3 grid, const DevCtx& d, const ProjTile* tiles, float* glow, int64_t split_stride,
                                 float grad_scale, const FusedAdam& fa, hipStream_t s) {
  constexpr int LDS_BYTES = (RB == 2 ? 3 * 48 : 4 * 32) * 1024;
  static LdsRaised raised;
  if (hipError_t e = raise_lds(reinterpret_cast<const void*>(k_proj_down_tr<RB, GONCE>), LDS_BYTES, raised); e != hipSuccess) return e;
  hipLaunchKernelGGL((k_proj_down_tr<RB, GONCE>), grid, dim3(512), LDS_BYTES, s, d, tiles, glow, split_stride, grad_scale, fa);
  return hipGetLastError();
}

// One instantiation of the pipelined kernel; its dynamic LDS (64 KiB for 128-rank tiles, 96 KiB for
// 256-rank tiles, 32 KiB more with error feedback) is raised above the default limit at first use.
template <int RB, bool VEC, bool GONCE, int EF>
static hipError_t launch_pipe(dim3 grid, const DevCtx& d, const ProjTile* tiles, float* glow, int64_t split_stride,
                              float grad_scale, const FusedAdam& fa, hipStream_t s) {
  constexpr int LDS_BYTES = (RB == 2 ? 98304 : 65536) + (EF != 0 ? 32768 : 0);
  static LdsRaised raised;
  if constexpr (LDS_BYTES > 65536)
    if (hipError_t e = raise_lds(reinterpret_cast<const void*>(k_proj_down_pipe<RB, VEC, GONCE, EF>), LDS_BYTES, raised); e != hipSuccess) return e;
  hipLaunchKernelGGL((k_proj_down_pipe<RB, VEC, GONCE, EF>), grid, dim3(512), LDS_BYTES, s, d, tiles, glow, split_stride, grad_scale, fa);
  return hipGetLastError();
}
template <int RB, int EF>
static hipError_t launch_pipe_vo(bool g_vec, bool g_once, dim3 grid, const DevCtx& d, const ProjTile* tiles, float* glow,
                                 int64_t split_stride, float grad_scale, const FusedAdam& fa, hipStream_t s) {
  if (g_once) return g_vec ? launch_pipe<RB, true, true, EF>(grid, d, tiles, glow, split_stride, grad_scale, fa, s)
                           : launch_pipe<RB, false, true, EF>(grid, d, tiles, glow, split_stride, grad_scale, fa, s);
  return g_vec ? launch_pipe<RB, true, false, EF>(grid, d, tiles, glow, split_stride, grad_scale, fa, s)
               : launch_pipe<RB, false, false, EF>(grid, d, tiles, glow, split_stride, grad_scale, fa, s);
}
static hipError_t launch_pipe_select(int rb, bool g_vec, bool g_once, int ef, dim3 grid, const DevCtx& d, const ProjTile* tiles,
                                     float* glow, int64_t split_stride, float grad_scale, const FusedAdam& fa, hipStream_t s) {
#define LORDO_PIPE_RB(RBV)                                                                                               \
  (ef == 3 ? launch_pipe_vo<RBV, 3>(g_vec, g_once, grid, d, tiles, glow, split_stride, grad_scale, fa, s)                \
   : ef == 2 ? launch_pipe_vo<RBV, 2>(g_vec, g_once, grid, d, tiles, glow, split_stride, grad_scale, fa, s)              \
   : ef == 1 ? launch_pipe_vo<RBV, 1>(g_vec, g_once, grid, d, tiles, glow, split_stride, grad_scale, fa, s)              \
             : launch_pipe_vo<RBV, 0>(g_vec, g_once, grid, d, tiles, glow, split_stride, grad_scale, fa, s))
  return rb == 2 ? LORDO_PIPE_RB(2) : LORDO_PIPE_RB(1);
#undef LORDO_PIPE_RB
}

hipError_t launch_proj_down(const DevCtx& d, const ProjTile* tiles, int ntiles, int mb, int pipe_rb, bool g_vec, bool g_tr, bool g_once, float* glow,
                            int64_t split_stride, float grad_scale, bool g_is_f32, int ef, const DownFuse* fuse, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  dim3 grid(ntiles), block(256);
  if (pipe_rb) {       // pipelined kernel: 128 * pipe_rb rank indices per tile
    FusedAdam fa{};
    if (fuse) {
      fa.u = fuse->u; fa.v = fuse->v; fa.n_hi = fuse->n_hi; fa.n_lo = fuse->n_lo;
      fa.b1 = fuse->a.b1; fa.omb1 = fuse->a.omb1; fa.b2 = fuse->a.b2; fa.omb2 = fuse->a.omb2;
      fa.step = fuse->a.step; fa.eps = fuse->a.eps;
      fa.qw = fuse->a.qw; fa.qg = fuse->a.qg;
      fa.g_hi = fuse->a.g_hi; fa.g_lo = fuse->a.g_lo; fa.colpart = fuse->a.colpart;
    }
    // 256-rank tiles (ranks from 256 up, where the matrix cores bound the kernel): gradient by global-to-LDS loads,
    // transposed while it is read from LDS -- 8 to 11 % faster there than staging through registers; with 128-rank
    // tiles (memory-bound, two workgroups per compute unit) the register-staged kernel is as fast or faster
    if (g_tr && ef == 0 && pipe_rb == 2)
      return g_once ? launch_down_tr<2, true>(grid, d, tiles, glow, split_stride, grad_scale, fa, s)
                    : launch_down_tr<2, false>(grid, d, tiles, glow, split_stride, grad_scale, fa, s);
    return launch_pipe_select(pipe_rb, g_vec, g_once, ef, grid, d, tiles, glow, split_stride, grad_scale, fa, s);
  }
  // fp32 gradients do not come here: their products run in the grouped GEMM with three-term operands
  (void)mb; (void)g_is_f32; (void)block;
  return hipErrorInvalidValue;
}

// Element type of the caller's weights: fp32, or bf16 storage (the update is formed in fp32 from the stored value and
// rounded to nearest-even once when it is written back).  Four consecutive columns of a row per lane.
template <bool WBF> struct WAcc;
template <> struct WAcc<false> {
  static constexpr uint32_t ES = 4;
  typedef u32x4 raw_t;
  static __device__ __forceinline__ raw_t load(rsrc_t r, uint32_t voff, uint32_t soff) { return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, STREAM); }
  static __device__ __forceinline__ f32x4 unpack(raw_t w) {
    return f32x4{__uint_as_float(w.x), __uint_as_float(w.y), __uint_as_float(w.z), __uint_as_float(w.w)};
  }
  static __device__ __forceinline__ void store(f32x4 x, rsrc_t r, uint32_t voff, uint32_t soff) {
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{__float_as_uint(x.x), __float_as_uint(x.y), __float_as_uint(x.z), __float_as_uint(x.w)}, r, voff, soff, STREAM);
  }
};
template <> struct WAcc<true> {
  static constexpr uint32_t ES = 2;
  typedef u32x2 raw_t;
  static __device__ __forceinline__ raw_t load(rsrc_t r, uint32_t voff, uint32_t soff) { return __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, STREAM); }
  static __device__ __forceinline__ f32x4 unpack(raw_t w) {
    return f32x4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xffff0000u)};
  }
  static __device__ __forceinline__ void store(f32x4 x, rsrc_t r, uint32_t voff, uint32_t soff) {
    __builtin_amdgcn_raw_buffer_store_b64(u32x2{pack_bf16_rne(x.x, x.y), pack_bf16_rne(x.z, x.w)}, r, voff, soff, STREAM);
  }
};

// ---------------------------------------------------------------------------------------
// Up-projection with the weight update fused, fallback for any q and any alignment of W (the main
// path below needs q % 4 == 0 and 16-byte aligned W).  Workgroup tile 128 x 128 of W, 4 waves in a
// 2 x 2 grid, each wave 64 x 64 = 2 x 2 accumulator blocks.  Operand fragments come straight from
// the packed planes (one coalesced 1 KiB read per wave and fragment), double-buffered in registers;
// the W tile is fetched through a buffer resource, one dword per access, before the contraction so
// that its latency hides behind it.
// ---------------------------------------------------------------------------------------
template <bool WBF>       // WBF: the caller's W is bf16 (never together with to_mom: the momentum is fp32)
__global__ __launch_bounds__(256) void k_proj_up(DevCtx d, const ProjTile* __restrict__ tiles,
                                                 const uint16_t* __restrict__ n_hi, const uint16_t* __restrict__ n_lo, float lr, int to_mom) {
  constexpr uint32_t ES = WBF ? 2u : 4u;
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0 || mat_skipped(d, t.mat)) return;
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

  // W is a buffer of p*q floats: a lane whose column or row is outside the matrix gets an offset
  // outside the buffer (reads give 0, writes are dropped).  Register v of block (a, b) is row
  // 8*(v/4) + 4*(lane/32) + v%4, column lane%32: the lane supplies its part of the offset, the
  // block / register part is scalar, and a row at or past p gets the size of the resource.
  const uint32_t row_bytes = (uint32_t)q * ES;
  const rsrc_t rw = make_rsrc(to_mom ? static_cast<void*>(d.arena + m.mom) : ext_ptr(d, EXT_W, t.mat), (uint32_t)p * row_bytes);
  uint32_t voff[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    int col = 32 * (nb0 + b) + (lane & 31);
    voff[b] = col < q ? (uint32_t)(4 * (lane >> 5)) * row_bytes + (uint32_t)(lane & 31) * ES : OOB;
  }
  auto w_soff = [&](int a, int b, int v) -> uint32_t {
    const int row = 32 * (mb0 + a) + 8 * (v >> 2) + (v & 3);
    return row < p ? (uint32_t)row * row_bytes + (uint32_t)(32 * (nb0 + b)) * ES : (uint32_t)p * row_bytes;
  };
  float wv[2][2][16];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if constexpr (WBF) wv[a][b][v] = __uint_as_float((uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rw, voff[b], w_soff(a, b, v), STREAM) << 16);
        else wv[a][b][v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rw, voff[b], w_soff(a, b, v), STREAM));
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
  // uniform plane pointers of the row blocks and column blocks (clamped into the planes: loads of
  // blocks past the edge stay inside, their stores fall outside the buffer); the lane adds its index
  const GAS u32x4* pqh[2]; const GAS u32x4* pql[2];
  const GAS u32x4* pnh[2]; const GAS u32x4* pnl[2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    int mbc = mb0 + a < mblocks ? mb0 + a : mblocks - 1;
    pqh[a] = qa_hi + (int64_t)mbc * rgroups * 32;
    pql[a] = qa_lo + (int64_t)mbc * rgroups * 32;
  }
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    int nbc = nb0 + b < nblocks ? nb0 + b : nblocks - 1;
    pnh[b] = nh + (int64_t)nbc * rgroups * 32;
    pnl[b] = nl + (int64_t)nbc * rgroups * 32;
  }
  struct Frags { u32x4 qh[2], ql[2], nh[2], nl[2]; };
  auto load_frags = [&](Frags& f, int ks) {
    const uint32_t o = (uint32_t)ks * 64u + (uint32_t)lane;
#pragma unroll
    for (int a = 0; a < 2; ++a) { f.qh[a] = pqh[a][o]; f.ql[a] = pql[a][o]; }
#pragma unroll
    for (int b = 0; b < 2; ++b) { f.nh[b] = pnh[b][o]; f.nl[b] = pnl[b][o]; }
  };
  auto compute = [&](const Frags& f) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.qh[a]), as_bf(f.nh[b]), acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.qh[a]), as_bf(f.nl[b]), acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f.ql[a]), as_bf(f.nh[b]), acc[a][b], 0, 0, 0);
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
    for (int v = 0; v < 16; ++v)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const float val = fmaf(-lr, acc[a][b][v], wv[a][b][v]);
        if constexpr (WBF) __builtin_amdgcn_raw_buffer_store_b16((short)f2bf_rne(val), rw, voff[b], w_soff(a, b, v), STREAM);
        else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val), rw, voff[b], w_soff(a, b, v), STREAM);
      }
}

// ---------------------------------------------------------------------------------------
// Up-projection, main path (q % 4 == 0, W 16-byte aligned).  Same tile and wave layout as the
// fallback above.
// W access.  The vector-memory front end costs about 16 cycles per instruction whatever its width
// and one tag look-up per cache line touched, so W is moved with 16-byte accesses that cover whole
// 128-byte lines: the matrix core computes the transposed block (Q N)^T = N^T Q^T, which puts four
// consecutive COLUMNS of a row in a lane's four consecutive accumulator registers; each 32 x 32
// block then goes through a per-wave LDS buffer (16-byte writes, 16-byte reads) into row order,
// where 8 lanes cover one 128-byte line of a row, and is combined with the W values that were
// fetched in that same order.
// Operands.  The fragments are brought in ONCE per workgroup by direct global-to-LDS loads (each
// 1 KiB fragment is one 16-byte-per-lane load that lands in lane order, so no registers and no
// transposition are involved) and every wave then reads its fragments from LDS.  This halves the
// bytes that pass through the vector L1 (each fragment is needed by two of the four waves), which
// is what bounds a register-fed variant.  Chunks of 32 of the contraction (2 MFMA k-steps, 32 KiB
// of fragments) are double-buffered; one barrier per chunk.
// ---------------------------------------------------------------------------------------

// WITH_G adds a gradient term to the epilogue: target <- target + coef_acc * (Q B) + coef_g * G * c_j, with
//   full-rank quasi-hyperbolic update (Alg. 1, "Full-Rank QHM"; Sec. 3.2): target W, B = N, coef_acc = -eta*omega,
//     coef_g = -eta*(1-omega)*grad_scale, c_j = 1 / mean_i(sqrt(v_hat_ij) + eps);
//   error-feedback residual (Alg. 1 error-feedback lines): target E, B = g, coef_acc = -1, coef_g = grad_scale, c_j = 1
//     (E <- grad_scale*G + E - Q g).
// EPI = 2 is the outer step fed from the averaged up-link buffers (App. A.5.1; Alg. 1 OuterOpt): B = mean of the buffers,
//   Delta = Q B stays in the accumulators, the tile that is read is the anchor, and the epilogue does
//   b <- mu b + Delta;  x <- anchor - eta_s (Delta + mu b) (Nesterov), anchor - eta_s b (heavy ball) or anchor - eta_s Delta
//   (no momentum);  W <- x, anchor <- x.
template <int NW, int EPI, bool WBF>   // NW waves per workgroup: 4 (wave tile 64 x 64) or 8 (wave tile 32 x 64); EPI 0 plain, 1 gradient term, 2 outer step;
                                       // WBF: the target (the caller's W, or the residual E) is stored in bf16
__global__ __launch_bounds__(64 * NW) void k_proj_up_dma(DevCtx d, const ProjTile* __restrict__ tiles,
                                                         const uint16_t* __restrict__ n_hi, const uint16_t* __restrict__ n_lo, UpArgs ua) {
  constexpr bool WITH_G = EPI == 1;
  constexpr bool OUTER = EPI == 2;
  static_assert(!WBF || EPI != 2, "bf16 targets: plain update and gradient-term epilogue");
  typedef WAcc<WBF> WA;
  constexpr uint32_t WES = WA::ES;
  const float lr = -ua.coef_acc;
  constexpr int AM = NW == 4 ? 2 : 1;                      // row blocks per wave
  constexpr int WM = 4 / AM;                               // wave rows
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0 || mat_skipped(d, t.mat)) return;
  const MatDev m = d.mats[t.mat];
  const GAS u32x4* qa_hi = TO_GLOBAL(const u32x4, d.arena + m.qa_hi);
  const GAS u32x4* qa_lo = TO_GLOBAL(const u32x4, d.arena + m.qa_lo);
  const GAS u32x4* nh = TO_GLOBAL(const u32x4, n_hi + m.lr_off);
  const GAS u32x4* nl = TO_GLOBAL(const u32x4, n_lo + m.lr_off);

  // fragment slot (64 x 16 bytes) of chunk buffer s: ((s*2 + kind)*4 + blk)*4 + ks*2 + plane,
  // kind 0 = Q rows, 1 = N columns; the epilogue staging blocks reuse the same memory
  constexpr int TP = 68;                                   // pitch of the 32 x 64 staging tile of a wave
  constexpr int SLOTS = 2 * 2 * 4 * 4;
  __shared__ u32x4 frag[SLOTS * 64];                       // 64 KiB
  static_assert(sizeof(u32x4) * SLOTS * 64 >= sizeof(float) * NW * 32 * TP, "staging blocks must fit");

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave % WM, wn = wave / WM;
  const int mblocks = m.pp / 32, nblocks = m.qp / 32;
  const int mb0 = t.m0 / 32 + AM * wm, nb0 = t.n0 / 32 + 2 * wn;    // this wave's first row / column block
  const int p = m.p, q = m.q;
  const int64_t rgroups = m.rp / 8;
  const int nchunks = m.rp / 32;

  // feeding role: 32 fragments per chunk = (kind, blk) x (k-step, plane); NW = 4: wave w feeds block w of
  // both kinds; NW = 8: wave w feeds block w % 4 of kind w / 4
  const int fblk = wave & 3;
  const int mbf = t.m0 / 32 + fblk < mblocks ? t.m0 / 32 + fblk : mblocks - 1;
  const int nbf = t.n0 / 32 + fblk < nblocks ? t.n0 / 32 + fblk : nblocks - 1;
  const GAS u32x4* src[4] = {qa_hi + (int64_t)mbf * rgroups * 32 + lane, qa_lo + (int64_t)mbf * rgroups * 32 + lane,
                             nh + (int64_t)nbf * rgroups * 32 + lane, nl + (int64_t)nbf * rgroups * 32 + lane};
  auto issue_chunk = [&](int c, int s) {
#pragma unroll
    for (int kind = 0; kind < 2; ++kind) {
      if (NW == 8 && kind != (wave >> 2)) continue;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int pl = 0; pl < 2; ++pl)
          dma16(src[kind * 2 + pl] + (int64_t)(2 * c + ks) * 64, frag + ((((s * 2 + kind) * 4 + fblk) * 4) + ks * 2 + pl) * 64);
    }
  };

  // W tile in row order: lane = (rr, c16): row rr + 4j of a row block, columns 4*c16 .. 4*c16+3 of the wave's two
  // column blocks, so that one access of the wave covers four rows of 256 contiguous bytes
  const uint32_t row_bytes = (uint32_t)q * WES;
  const void* target = ua.target_err == 1 ? static_cast<const void*>(d.arena + m.err)
                       : ua.target_err == 2 ? static_cast<const void*>(d.arena + m.mom) : ext_ptr(d, EXT_W, t.mat);
  const rsrc_t rw_out = make_rsrc(target, (uint32_t)p * row_bytes);
  // outer step: the tile read before the contraction is the anchor; the momentum tile is read in the epilogue
  const rsrc_t ranchor = make_rsrc(d.arena + m.anchor, (uint32_t)p * row_bytes);
  const rsrc_t rmom = make_rsrc(d.arena + (OUTER && ua.has_mom ? m.mom : m.anchor), (uint32_t)p * row_bytes);
  const rsrc_t rw = OUTER ? ranchor : rw_out;
  const int rr = lane >> 4, c16 = lane & 15;
  const int bsel = c16 >> 3;                                 // which of the two column blocks the lane's columns lie in
  const int lcol = 32 * nb0 + 4 * c16;                       // first of the lane's four columns
  const uint32_t voff = lcol < q ? (uint32_t)rr * row_bytes + (uint32_t)c16 * (4u * WES) : OOB;
  // a group of four rows that starts at or past the last row gets the size of the resource as its
  // scalar offset, which puts every lane of the access out of range
  auto w_soff = [&](int a, int j) -> uint32_t {
    const int row = 32 * (mb0 + a) + 4 * j;
    return row < p ? (uint32_t)row * row_bytes + (uint32_t)(32 * nb0) * WES : (uint32_t)p * row_bytes;
  };

  issue_chunk(0, 0);
  typename WA::raw_t wv[AM][8];
#pragma unroll
  for (int a = 0; a < AM; ++a)
#pragma unroll
    for (int j = 0; j < 8; ++j) wv[a][j] = WA::load(rw, voff, w_soff(a, j));
  // gradient term (WITH_G): four consecutive columns per lane, same rows as the W accesses; a bf16 G tile is
  // requested here, with the W tile, so that it arrives during the contraction
  const uint32_t ges = ua.g_is_f32 ? 4u : 2u;
  const uint32_t grow_bytes = (uint32_t)q * ges;
  const rsrc_t rg = WITH_G ? make_rsrc(ext_ptr(d, EXT_G, t.mat), (uint32_t)p * grow_bytes) : rw;
  auto g_soff = [&](int a, int j) -> uint32_t {
    const int row = 32 * (mb0 + a) + 4 * j;
    return row < p ? (uint32_t)row * grow_bytes + (uint32_t)(32 * nb0) * ges : (uint32_t)p * grow_bytes;
  };
  const uint32_t gvoff = lcol < q ? (uint32_t)rr * grow_bytes + (uint32_t)c16 * 4u * ges : OOB;
  u32x2 gpre[WITH_G ? AM : 1][8];
  if constexpr (WITH_G) {
    if (!ua.g_is_f32) {
#pragma unroll
      for (int a = 0; a < AM; ++a)
#pragma unroll
        for (int j = 0; j < 8; ++j) gpre[a][j] = __builtin_amdgcn_raw_buffer_load_b64(rg, gvoff, g_soff(a, j), STREAM);
    }
  }
  ISSUE_FENCE();

  f32x16 acc[AM][2];
#pragma unroll
  for (int a = 0; a < AM; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  for (int c = 0; c < nchunks; ++c) {
    __builtin_amdgcn_s_waitcnt(0x0f70);                            // vmcnt(0): this wave's part of chunk c has landed
    __syncthreads();              // chunk c visible to all waves; every wave is done with chunk c-1
    if (c + 1 < nchunks) issue_chunk(c + 1, (c + 1) & 1);
    ISSUE_FENCE();
    const u32x4* fb = frag + (c & 1) * (2 * 4 * 4 * 64);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      u32x4 qh[AM], ql[AM], xh[2], xl[2];
#pragma unroll
      for (int a = 0; a < AM; ++a) {
        qh[a] = fb[((0 * 4 + AM * wm + a) * 4 + ks * 2 + 0) * 64 + lane];
        ql[a] = fb[((0 * 4 + AM * wm + a) * 4 + ks * 2 + 1) * 64 + lane];
      }
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        xh[b] = fb[((1 * 4 + 2 * wn + b) * 4 + ks * 2 + 0) * 64 + lane];
        xl[b] = fb[((1 * 4 + 2 * wn + b) * 4 + ks * 2 + 1) * 64 + lane];
      }
#pragma unroll
      for (int a = 0; a < AM; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {      // transposed block: N fragment first
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(xh[b]), as_bf(qh[a]), acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(xl[b]), as_bf(qh[a]), acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(xh[b]), as_bf(ql[a]), acc[a][b], 0, 0, 0);
        }
    }
  }
  __syncthreads();                // all waves are done reading fragments: reuse the memory for staging

  if (mb0 >= mblocks || nb0 >= nblocks) return;
  f32x4 cscale = {1.f, 1.f, 1.f, 1.f};
  if constexpr (WITH_G) {
    if (ua.colscale == 1 && nb0 + bsel < nblocks) {
      const GAS float* cp = TO_GLOBAL(const float, ua.colpart) + m.lr_off / 32;
      const int rblocks = m.rp / 32;
      const float pad = (float)(m.rp - m.r) * ua.eps;          // padded rank indices hold v = 0: eps each
      const float inv_r = 1.f / (float)m.r;
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
      for (int rb = 0; rb < rblocks; ++rb)                      // fixed order
        sum += *reinterpret_cast<const GAS f32x4*>(cp + ((int64_t)(nb0 + bsel) * rblocks + rb) * 32 + 4 * (c16 & 7));
#pragma unroll
      for (int e = 0; e < 4; ++e) cscale[e] = 1.f / ((sum[e] - pad) * inv_r);
    }
  }
  auto g_term = [&](int a, int j) -> f32x4 {
    f32x4 gv;
    if (ua.g_is_f32) {
      u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rg, gvoff, g_soff(a, j), STREAM);
      gv.x = __uint_as_float(w.x); gv.y = __uint_as_float(w.y); gv.z = __uint_as_float(w.z); gv.w = __uint_as_float(w.w);
    } else {
      const u32x2 w = gpre[WITH_G ? a : 0][j];
      gv.x = __uint_as_float(w.x << 16); gv.y = __uint_as_float(w.x & 0xffff0000u);
      gv.z = __uint_as_float(w.y << 16); gv.w = __uint_as_float(w.y & 0xffff0000u);
    }
    return gv * cscale * ua.coef_g;
  };
  // colscale == 2: the scale belongs to the ROWS of this tile -- a right-projected matrix, whose low-rank state has one
  // column per row of W (Sec. 3.2 on the transposed problem): 1 / mean over the rank of sqrt(v_hat) + eps of that row.
  // The shadow record of such a matrix keeps the matrix's place in the flat low-rank arrays in `qt_hi`.
  auto row_scales = [&](int a, float (&rs)[8]) {
    const GAS float* cp = TO_GLOBAL(const float, ua.colpart) + m.qt_hi / 32;
    const int rblocks = m.rp / 32;
    const float pad = (float)(m.rp - m.r) * ua.eps;
    const float inv_r = 1.f / (float)m.r;
    const int cb = mb0 + a < mblocks ? mb0 + a : mblocks - 1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float sum = 0.f;
      for (int rb = 0; rb < rblocks; ++rb) sum += cp[((int64_t)cb * rblocks + rb) * 32 + rr + 4 * j];      // fixed order
      const float den = (sum - pad) * inv_r;
      rs[j] = den > 0.f ? 1.f / den : 0.f;                      // (rows of the padding: nothing is stored there)
    }
  };
  // transposed accumulator: register 4*vq+e of lane l is row l%32, column 8*vq + 4*(l/32) + e of its block; both
  // column blocks of a row block go into one 32 x 64 staging tile
  float* T = reinterpret_cast<float*>(frag) + wave * 32 * TP;
#pragma unroll
  for (int a = 0; a < AM; ++a) {
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        f32x4 x;
        x.x = acc[a][b][4 * vq]; x.y = acc[a][b][4 * vq + 1]; x.z = acc[a][b][4 * vq + 2]; x.w = acc[a][b][4 * vq + 3];
        *reinterpret_cast<f32x4*>(T + (lane & 31) * TP + 32 * b + 8 * vq + 4 * (lane >> 5)) = x;
      }
    // LDS operations of one wave complete in order: the reads below see the writes above
    f32x4 gt[8];
    if constexpr (WITH_G) {
#pragma unroll
      for (int j = 0; j < 8; ++j) gt[j] = g_term(a, j);
      if (ua.colscale == 2) {
        float rs[8];
        row_scales(a, rs);
#pragma unroll
        for (int j = 0; j < 8; ++j) gt[j] *= rs[j];
      }
    }
    u32x4 mv[8];
    if constexpr (OUTER) {
      if (ua.has_mom) {
#pragma unroll
        for (int j = 0; j < 8; ++j) mv[j] = __builtin_amdgcn_raw_buffer_load_b128(rmom, voff, w_soff(a, j), STREAM);
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      f32x4 x = *reinterpret_cast<const f32x4*>(T + (rr + 4 * j) * TP + 4 * c16);
      const f32x4 wf = WA::unpack(wv[a][j]);
      if constexpr (WBF) {       // bf16 target: the new value is formed in fp32 and rounded once
        f32x4 val = {fmaf(-lr, x.x, wf.x), fmaf(-lr, x.y, wf.y), fmaf(-lr, x.z, wf.z), fmaf(-lr, x.w, wf.w)};
        if constexpr (WITH_G) val += gt[j];
        WA::store(val, rw_out, voff, w_soff(a, j));
        continue;
      }
      u32x4 o;
      o.x = __float_as_uint(fmaf(-lr, x.x, wf.x));
      o.y = __float_as_uint(fmaf(-lr, x.y, wf.y));
      o.z = __float_as_uint(fmaf(-lr, x.z, wf.z));
      o.w = __float_as_uint(fmaf(-lr, x.w, wf.w));
      if constexpr (WITH_G) {
        o.x = __float_as_uint(__uint_as_float(o.x) + gt[j].x); o.y = __float_as_uint(__uint_as_float(o.y) + gt[j].y);
        o.z = __float_as_uint(__uint_as_float(o.z) + gt[j].z); o.w = __float_as_uint(__uint_as_float(o.w) + gt[j].w);
      }
      if constexpr (OUTER) {
        f32x4 step = x;                                    // Delta
        if (ua.has_mom) {
          const f32x4 bo = {__uint_as_float(mv[j].x), __uint_as_float(mv[j].y), __uint_as_float(mv[j].z), __uint_as_float(mv[j].w)};
          f32x4 bn;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            bn[e] = fmaf(ua.mu, bo[e], x[e]);
            step[e] = ua.nesterov ? fmaf(ua.mu, bn[e], x[e]) : bn[e];
          }
          u32x4 bs = {__float_as_uint(bn.x), __float_as_uint(bn.y), __float_as_uint(bn.z), __float_as_uint(bn.w)};
          __builtin_amdgcn_raw_buffer_store_b128(bs, rmom, voff, w_soff(a, j), STREAM);
        }
        o.x = __float_as_uint(fmaf(-lr, step.x, wf.x));
        o.y = __float_as_uint(fmaf(-lr, step.y, wf.y));
        o.z = __float_as_uint(fmaf(-lr, step.z, wf.z));
        o.w = __float_as_uint(fmaf(-lr, step.w, wf.w));
        __builtin_amdgcn_raw_buffer_store_b128(o, ranchor, voff, w_soff(a, j), STREAM);
      }
      __builtin_amdgcn_raw_buffer_store_b128(o, rw_out, voff, w_soff(a, j), STREAM);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Up-projection for ranks from 256 up (q % 4 == 0, target aligned to four of its elements): workgroup tile 256 rows x 128
// columns of W, 4 waves in a 2 x 2 grid, wave tile 128 x 64 = 4 x 2 accumulator blocks.  With the 128 x 128 tile
// above every wave reads 16 KiB of fragments from LDS per 24 MFMAs and
// the workgroup pulls 1 byte of operand planes through L2 per output element and k-step; here a wave reads 12 KiB per
// 24 MFMAs and the tile pulls 0.75 bytes.  The operand fragments of one k-step of 16 (24 KiB: eight row blocks of Q,
// four column blocks of N, two planes each) arrive by global-to-LDS loads through a ring of three buffers, two
// k-steps in flight, with explicit waits as in the pipelined down-projection; 72 KiB of LDS and 128 accumulator
// registers admit two workgroups per compute unit, so that the epilogue of one (read, update, write of its W tile)
// runs under the contraction of the other.  Inside a wave the fragments of the next k-step are read from LDS into a
// second register set while the matrix cores work on the current one; the registers then leave no room for W during
// the contraction: its row blocks are requested when the contraction ends, three in flight (two when the epilogue
// also reads a gradient tile: the full-rank QHM update, the residual of the error feedback).
// ---------------------------------------------------------------------------------------
template <bool WBF, bool WITH_G>     // WITH_G: gradient-term epilogue (bf16 G): the full-rank QHM update, or the residual E as target
__global__ __launch_bounds__(256) void k_proj_up_wide(DevCtx d, const ProjTile* __restrict__ tiles,
                                                      const uint16_t* __restrict__ n_hi, const uint16_t* __restrict__ n_lo, UpArgs ua) {
  typedef WAcc<WBF> WA;
  constexpr uint32_t WES = WA::ES;
  const float lr = -ua.coef_acc;
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0) return;
  const MatDev m = d.mats[t.mat];
  const GAS u32x4* qa_hi = TO_GLOBAL(const u32x4, d.arena + m.qa_hi);
  const GAS u32x4* qa_lo = TO_GLOBAL(const u32x4, d.arena + m.qa_lo);
  const GAS u32x4* nh = TO_GLOBAL(const u32x4, n_hi + m.lr_off);
  const GAS u32x4* nl = TO_GLOBAL(const u32x4, n_lo + m.lr_off);

  // fragment slot (64 x 16 bytes) of ring buffer s: s*24 + [Q: blk*2 + plane | 16 + blk*2 + plane : N]
  constexpr int TP = 68;                                   // pitch of the 32 x 64 staging tile of a wave
  constexpr int SLOTS = 24;
  constexpr int NS = 3;
  extern __shared__ u32x4 lds_dyn[];                       // 3 x 24 KiB
  u32x4* frag = lds_dyn;
  static_assert(sizeof(u32x4) * NS * SLOTS * 64 >= sizeof(float) * 4 * 32 * TP, "staging blocks must fit");

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave & 1, wn = wave >> 1;
  const int mblocks = m.pp / 32, nblocks = m.qp / 32;
  const int mb0 = t.m0 / 32 + 4 * wm, nb0 = t.n0 / 32 + 2 * wn;    // this wave's first row / column block
  const int p = m.p, q = m.q;
  const int64_t rgroups = m.rp / 8;
  const int nchunks = m.rp / 16;

  // feeding role: wave w brings in row blocks 2w, 2w + 1 of Q and column block w of N, both planes: six loads per k-step
  const GAS u32x4* fsrc[6];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int mbf = t.m0 / 32 + 2 * wave + j < mblocks ? t.m0 / 32 + 2 * wave + j : mblocks - 1;
    fsrc[2 * j] = qa_hi + (int64_t)mbf * rgroups * 32 + lane;
    fsrc[2 * j + 1] = qa_lo + (int64_t)mbf * rgroups * 32 + lane;
  }
  {
    const int nbf = t.n0 / 32 + wave < nblocks ? t.n0 / 32 + wave : nblocks - 1;
    fsrc[4] = nh + (int64_t)nbf * rgroups * 32 + lane;
    fsrc[5] = nl + (int64_t)nbf * rgroups * 32 + lane;
  }
  auto issue_chunk = [&](int c, int s) {
    c = c < nchunks ? c : nchunks - 1;                     // past the end the last k-step is loaded again: same count every iteration
    u32x4* base = frag + s * SLOTS * 64;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int pl = 0; pl < 2; ++pl) dma16_async(fsrc[2 * j + pl] + (int64_t)c * 64, base + ((2 * wave + j) * 2 + pl) * 64);
#pragma unroll
    for (int pl = 0; pl < 2; ++pl) dma16_async(fsrc[4 + pl] + (int64_t)c * 64, base + (16 + wave * 2 + pl) * 64);
  };

  // W tile in row order: lane = (rr, c16): row rr + 4j of a row block, columns 4*c16 .. 4*c16+3 of the wave's two
  // column blocks, so that one access of the wave covers four rows of 256 contiguous bytes
  const uint32_t row_bytes = (uint32_t)q * WES;
  const void* target = WITH_G && ua.target_err == 1 ? static_cast<const void*>(d.arena + m.err) : ext_ptr(d, EXT_W, t.mat);
  const rsrc_t rw = make_rsrc(target, (uint32_t)p * row_bytes);
  const int rr = lane >> 4, c16 = lane & 15;
  const int lcol = 32 * nb0 + 4 * c16;                       // first of the lane's four columns
  const uint32_t voff = lcol < q ? (uint32_t)rr * row_bytes + (uint32_t)c16 * (4u * WES) : OOB;
  auto w_soff = [&](int a, int j) -> uint32_t {
    const int row = 32 * (mb0 + a) + 4 * j;
    return row < p ? (uint32_t)row * row_bytes + (uint32_t)(32 * nb0) * WES : (uint32_t)p * row_bytes;
  };

  issue_chunk(0, 0);
  issue_chunk(1, 1);

  f32x16 acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  // Fragments of a k-step in registers: [0..3] Q hi, [4..7] Q lo of the wave's four row blocks, [8..9] N hi, [10..11] N lo
  // of its two column blocks.  The fragments of k-step c+1 are read from LDS while the matrix cores work on k-step c.
  auto read_frags = [&](u32x4 (&f)[12], int s) {
    const u32x4* fb = frag + s * SLOTS * 64;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      f[8 + b] = fb[(16 + (2 * wn + b) * 2 + 0) * 64 + lane];
      f[10 + b] = fb[(16 + (2 * wn + b) * 2 + 1) * 64 + lane];
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      f[a] = fb[((4 * wm + a) * 2 + 0) * 64 + lane];
      f[4 + a] = fb[((4 * wm + a) * 2 + 1) * 64 + lane];
    }
  };
  auto multiply = [&](const u32x4 (&f)[12]) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {      // transposed block: N fragment first
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f[8 + b]), as_bf(f[a]), acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f[10 + b]), as_bf(f[a]), acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(f[8 + b]), as_bf(f[4 + a]), acc[a][b], 0, 0, 0);
      }
  };
  // one k-step: on entry `cur` holds the fragments of k-step c; k-steps c+1 and c+2 are in flight
  int sbuf = 0;                                              // ring buffer of k-step c
  auto step = [&](const u32x4 (&cur)[12], u32x4 (&nxt)[12], int c) {
    WAIT_VM_BARRIER(6);                                      // k-step c+1 has landed; every wave holds k-step c in registers
    issue_chunk(c + 3, sbuf);                                // into the buffer of k-step c
    sbuf = sbuf == 2 ? 0 : sbuf + 1;
    read_frags(nxt, sbuf);
    ISSUE_FENCE();
    multiply(cur);
  };
  u32x4 fa[12], fb2[12];
  WAIT_VM_BARRIER(6);                                        // k-step 0 has landed
  issue_chunk(2, 2);
  read_frags(fa, 0);
  ISSUE_FENCE();
  for (int c = 0; c < nchunks; c += 2) {                     // (the padded rank is a multiple of 32: an even number of k-steps)
    step(fa, fb2, c);
    step(fb2, fa, c + 1);
  }
  WAIT_VM_BARRIER(0);             // the repeated loads of the last k-step have landed, all waves are done reading fragments

  if (mb0 >= mblocks || nb0 >= nblocks) return;
  float* T = reinterpret_cast<float*>(frag) + wave * 32 * TP;
  // gradient term: coef_g * G * c_j on the lane's four columns, c_j the column scale of the full-rank QHM update
  // (1 / mean over the rank of sqrt(v_hat) + eps, from the sums the Adam kernel left) or 1
  const uint32_t grow_bytes = (uint32_t)q * 2u;
  const rsrc_t rg = WITH_G ? make_rsrc(ext_ptr(d, EXT_G, t.mat), (uint32_t)p * grow_bytes) : rw;
  const uint32_t gvoff = lcol < q ? (uint32_t)rr * grow_bytes + (uint32_t)c16 * 8u : OOB;
  auto g_soff = [&](int a, int j) -> uint32_t {
    const int row = 32 * (mb0 + a) + 4 * j;
    return row < p ? (uint32_t)row * grow_bytes + (uint32_t)(32 * nb0) * 2u : (uint32_t)p * grow_bytes;
  };
  f32x4 cscale = {1.f, 1.f, 1.f, 1.f};
  if constexpr (WITH_G) {
    const int bsel = c16 >> 3;
    if (ua.colscale == 1 && nb0 + bsel < nblocks) {
      const GAS float* cp = TO_GLOBAL(const float, ua.colpart) + m.lr_off / 32;
      const int rblocks = m.rp / 32;
      const float pad = (float)(m.rp - m.r) * ua.eps;          // padded rank indices hold v = 0: eps each
      const float inv_r = 1.f / (float)m.r;
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
      for (int rb = 0; rb < rblocks; ++rb)                      // fixed order
        sum += *reinterpret_cast<const GAS f32x4*>(cp + ((int64_t)(nb0 + bsel) * rblocks + rb) * 32 + 4 * (c16 & 7));
#pragma unroll
      for (int e = 0; e < 4; ++e) cscale[e] = ua.coef_g / ((sum[e] - pad) * inv_r);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) cscale[e] = ua.coef_g;
    }
  }
  struct GRows { u32x2 g[WITH_G ? 8 : 1]; };
  auto combine = [&](int a, const typename WA::raw_t (&wv)[8], const GRows& gr) {
    // transposed accumulator: register 4*vq+e of lane l is row l%32, column 8*vq + 4*(l/32) + e of its block
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        f32x4 x;
        x.x = acc[a][b][4 * vq]; x.y = acc[a][b][4 * vq + 1]; x.z = acc[a][b][4 * vq + 2]; x.w = acc[a][b][4 * vq + 3];
        *reinterpret_cast<f32x4*>(T + (lane & 31) * TP + 32 * b + 8 * vq + 4 * (lane >> 5)) = x;
      }
    // LDS operations of one wave complete in order: the reads below see the writes above
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const f32x4 x = *reinterpret_cast<const f32x4*>(T + (rr + 4 * j) * TP + 4 * c16);
      const f32x4 wf = WA::unpack(wv[j]);
      f32x4 val = {fmaf(-lr, x.x, wf.x), fmaf(-lr, x.y, wf.y), fmaf(-lr, x.z, wf.z), fmaf(-lr, x.w, wf.w)};
      if constexpr (WITH_G) {
        const u32x2 w = gr.g[j];
        val.x = fmaf(cscale.x, __uint_as_float(w.x << 16), val.x); val.y = fmaf(cscale.y, __uint_as_float(w.x & 0xffff0000u), val.y);
        val.z = fmaf(cscale.z, __uint_as_float(w.y << 16), val.z); val.w = fmaf(cscale.w, __uint_as_float(w.y & 0xffff0000u), val.w);
      }
      WA::store(val, rw, voff, w_soff(a, j));
    }
  };
  auto fetch = [&](int a, typename WA::raw_t (&wv)[8], GRows& gr) {
#pragma unroll
    for (int j = 0; j < 8; ++j) wv[j] = WA::load(rw, voff, w_soff(a, j));
    if constexpr (WITH_G) {
#pragma unroll
      for (int j = 0; j < 8; ++j) gr.g[j] = __builtin_amdgcn_raw_buffer_load_b64(rg, gvoff, g_soff(a, j), STREAM);
    }
  };
  // the fragment registers are free now: two further row blocks are requested at once, the last one as soon as
  // the first has been combined, so that only one memory latency is left exposed per tile
  // (fp32 target with a gradient tile: 48 registers per row block, two in flight keep the kernel at two waves per SIMD)
  constexpr bool THREE = !(WITH_G && !WBF);
  typename WA::raw_t wv0[8], wv1[8], wv2[THREE ? 8 : 1];
  GRows g0, g1, g2;
  fetch(0, wv0, g0);
  fetch(1, wv1, g1);
  if constexpr (THREE) {
    fetch(2, wv2, g2);
    ISSUE_FENCE();
    combine(0, wv0, g0);
    fetch(3, wv0, g0);
    ISSUE_FENCE();
    combine(1, wv1, g1);
    combine(2, wv2, g2);
    combine(3, wv0, g0);
  } else {
    ISSUE_FENCE();
    combine(0, wv0, g0);
    fetch(2, wv0, g0);
    ISSUE_FENCE();
    combine(1, wv1, g1);
    fetch(3, wv1, g1);
    ISSUE_FENCE();
    combine(2, wv0, g0);
    combine(3, wv1, g1);
  }
}

hipError_t launch_proj_up_wide(const DevCtx& d, const ProjTile* tiles, int ntiles, const uint16_t* b_hi, const uint16_t* b_lo,
                               const UpArgs& ua, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  constexpr int LDS_BYTES = 3 * 24 * 1024;
  static LdsRaised raised[4];
  const void* kernels[4] = {reinterpret_cast<const void*>(k_proj_up_wide<false, false>), reinterpret_cast<const void*>(k_proj_up_wide<true, false>),
                            reinterpret_cast<const void*>(k_proj_up_wide<false, true>), reinterpret_cast<const void*>(k_proj_up_wide<true, true>)};
  for (int k = 0; k < 4; ++k)
    if (hipError_t e = raise_lds(kernels[k], LDS_BYTES, raised[k]); e != hipSuccess) return e;
  const bool with_g = ua.coef_g != 0.f || ua.target_err == 1;
  if (with_g && ua.g_is_f32) return hipErrorInvalidValue;      // the gradient-term epilogue here reads bf16 gradients
  if (ua.target_err == 2 || ua.outer || ua.colscale == 2) return hipErrorInvalidValue;
#define LORDO_WIDE(WBFV, GV) hipLaunchKernelGGL((k_proj_up_wide<WBFV, GV>), dim3(ntiles), dim3(256), LDS_BYTES, s, d, tiles, b_hi, b_lo, ua)
  if (ua.w_bf16) { if (with_g) LORDO_WIDE(true, true); else LORDO_WIDE(true, false); }
  else { if (with_g) LORDO_WIDE(false, true); else LORDO_WIDE(false, false); }
#undef LORDO_WIDE
  return hipGetLastError();
}

// Epilogue of the Y = Src B kernels: the 2 x 2 accumulator blocks of a wave (register 4*vq+e of lane l: row l%32
// of the row block, rank 8*vq + 4*(l/32) + e of the rank block) go through a per-wave LDS tile into row order
// and out to buffer 0 of the Y pair with 16-byte stores along the rows.
__device__ __forceinline__ void store_y_tile(const DevCtx& d, const MatDev& m, const ProjTile& t, const f32x16 (&acc)[2][2],
                                             float* lds_stage, int wave, int lane, int wm, int wn) {
  constexpr int TP = 36;
  const int p = m.p, r = m.r;
  const uint32_t yrow_bytes = (uint32_t)r * 4u;
  const rsrc_t ry = make_rsrc(d.arena + m.y[0], (uint32_t)p * yrow_bytes);
  const int rr = lane >> 3, c4 = lane & 7;
  float* T = lds_stage + wave * 32 * TP;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int rank0 = t.n0 + 32 * (2 * wn + a), row0 = t.m0 + 32 * (2 * wm + b);
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        f32x4 x;
        x.x = acc[a][b][4 * vq]; x.y = acc[a][b][4 * vq + 1]; x.z = acc[a][b][4 * vq + 2]; x.w = acc[a][b][4 * vq + 3];
        *reinterpret_cast<f32x4*>(T + (lane & 31) * TP + 8 * vq + 4 * (lane >> 5)) = x;
      }
      // LDS operations of one wave complete in order: the reads below see the writes above
      const uint32_t voff = rank0 + 4 * c4 < r ? (uint32_t)rr * yrow_bytes + (uint32_t)(rank0 + 4 * c4) * 4u : OOB;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4 x = *reinterpret_cast<const f32x4*>(T + (rr + 8 * j) * TP + 4 * c4);
        const int row = row0 + 8 * j;                       // first of the eight rows this access covers
        const uint32_t soff = row < p ? (uint32_t)row * yrow_bytes : (uint32_t)p * yrow_bytes;
        u32x4 o = {__float_as_uint(x.x), __float_as_uint(x.y), __float_as_uint(x.z), __float_as_uint(x.w)};
        __builtin_amdgcn_raw_buffer_store_b128(o, ry, voff, soff, 0);
      }
    }
}

// ---------------------------------------------------------------------------------------
// Range-finder products with the contraction over the columns of the source: Y = Src B, B = Omega or the
// orthonormalised block Z (q x r), Src bf16 p x q (Sec. 2 ComputeProjection; sketch and second half of a power
// iteration).  Tile = 128 rows of Src x 128 rank indices, 4 waves in a 2 x 2 grid, wave tile 64 x 64.
// The matrix core computes D[rank][row] = B^T(rank, j) Src^T(j, row):
//   A operand  the planes of B in operand layout (m = rank, k = column j), bf16 hi + lo, two passes;
//   B operand  Src itself: the fragment of a k-step wants, per lane, 8 consecutive j of one row -- 16
//              contiguous bytes of the row-major source -- so the source goes from global memory straight into
//              LDS in fragment order (one 16-byte global-to-LDS load per lane and fragment), untransposed and
//              unconverted.
// Fragments arrive once per workgroup in chunks of 32 columns (24 KiB) through a ring of three LDS buffers:
// while chunk c is multiplied, chunks c+1 and c+2 are in flight (the tiles with the longest contraction run
// alone at the end of the launch, one workgroup per compute unit, and are bound by memory latency).  The
// loads are issued from inline assembly with explicit waits, as in the pipelined down-projection kernel;
// past the last chunk the last one is loaded again, so that the number of outstanding loads is the same in
// every iteration.  The epilogue is the row-order store of the up-projection kernel (per-wave LDS tile,
// 16-byte stores along the rows of Y).
// Needs q % 32 == 0, r % 4 == 0 and a 16-byte aligned source; rows past p are read from row p-1 and not stored.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_src_times_block(DevCtx d, const ProjTile* __restrict__ tiles,
                                                         const uint16_t* __restrict__ b_hi, const uint16_t* __restrict__ b_lo) {
  const ProjTile t = tiles[blockIdx.x];
  if (t.mat < 0 || mat_skipped(d, t.mat)) return;
  const MatDev m = d.mats[t.mat];
  const GAS u32x4* bh = TO_GLOBAL(const u32x4, b_hi + m.lr_off);
  const GAS u32x4* bl = TO_GLOBAL(const u32x4, b_lo + m.lr_off);
  const GAS uint16_t* src = TO_GLOBAL(const uint16_t, ext_ptr(d, EXT_SRC, t.mat));

  // fragment slot (64 x 16 bytes) of chunk buffer s: s*24 + [B planes: (blk*2 + ks)*2 + plane | 16 + blk*2 + ks : Src]
  constexpr int TP = 36;
  constexpr int SLOTS = 24;
  extern __shared__ u32x4 lds_dyn[];                       // 3 x 24 KiB
  u32x4* frag = lds_dyn;
  static_assert(sizeof(u32x4) * 3 * SLOTS * 64 >= sizeof(float) * 4 * 32 * TP, "staging blocks must fit");

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave & 1, wn = wave >> 1;                 // row-block pair, rank-block pair of this wave
  const int p = m.p, q = m.q, r = m.r;
  const int rblocks = m.rp / 32;
  const int64_t kgroups = m.qp / 8;
  const int nchunks = q / 32;

  // feeding role: wave w brings in rank block w of B (2 k-steps x 2 planes) and row block w of Src (2 k-steps)
  const int rbf = t.n0 / 32 + wave < rblocks ? t.n0 / 32 + wave : rblocks - 1;
  const GAS u32x4* bsrc[2] = {bh + (int64_t)rbf * kgroups * 32 + lane, bl + (int64_t)rbf * kgroups * 32 + lane};
  int frow = t.m0 + 32 * wave + (lane & 31);
  frow = frow < p ? frow : p - 1;
  const GAS uint16_t* srow = src + (int64_t)frow * q + 8 * (lane >> 5);
  auto issue_chunk = [&](int c, int s) {                   // six loads per wave
    c = c < nchunks ? c : nchunks - 1;
    u32x4* base = frag + s * SLOTS * 64;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int pl = 0; pl < 2; ++pl) dma16_async(bsrc[pl] + (int64_t)(2 * c + ks) * 64, base + ((wave * 2 + ks) * 2 + pl) * 64);
      dma16_async(reinterpret_cast<const GAS u32x4*>(srow + 32 * c + 16 * ks), base + (16 + wave * 2 + ks) * 64);
    }
  };

  f32x16 acc[2][2];                                        // [rank block][row block]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  issue_chunk(0, 0);
  issue_chunk(1, 1);
  int sbuf = 0;                                            // c % 3
  for (int c = 0; c < nchunks; ++c) {
    WAIT_VM_BARRIER(6);           // only chunk c+1 may be outstanding: this wave's part of chunk c has landed;
                                  // barrier: chunk c visible to all waves, every wave is done with chunk c-1
    issue_chunk(c + 2, sbuf == 0 ? 2 : sbuf - 1);          // into the buffer of chunk c-1
    ISSUE_FENCE();
    const u32x4* fb = frag + sbuf * SLOTS * 64;
    sbuf = sbuf == 2 ? 0 : sbuf + 1;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      u32x4 zh[2], zl[2], sv[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        zh[a] = fb[(((2 * wn + a) * 2 + ks) * 2 + 0) * 64 + lane];
        zl[a] = fb[(((2 * wn + a) * 2 + ks) * 2 + 1) * 64 + lane];
      }
#pragma unroll
      for (int b = 0; b < 2; ++b) sv[b] = fb[(16 + (2 * wm + b) * 2 + ks) * 64 + lane];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(zh[a]), as_bf(sv[b]), acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(zl[a]), as_bf(sv[b]), acc[a][b], 0, 0, 0);
        }
    }
  }
  WAIT_VM_BARRIER(0);             // the repeated loads of the last chunk have landed and all waves are done reading
                                  // fragments: reuse the memory for staging

  store_y_tile(d, m, t, acc, reinterpret_cast<float*>(frag), wave, lane, wm, wn);
}

hipError_t launch_src_times_block(const DevCtx& d, const ProjTile* tiles, int ntiles, const uint16_t* b_hi, const uint16_t* b_lo,
                                  hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  constexpr int LDS_BYTES = 3 * 24 * 1024;
  static LdsRaised raised;
  if (hipError_t e = raise_lds(reinterpret_cast<const void*>(k_src_times_block), LDS_BYTES, raised); e != hipSuccess) return e;
  hipLaunchKernelGGL(k_src_times_block, dim3(ntiles), dim3(256), LDS_BYTES, s, d, tiles, b_hi, b_lo);
  return hipGetLastError();
}

hipError_t launch_proj_up(const DevCtx& d, const ProjTile* tiles, int ntiles, bool vec, const uint16_t* b_hi,
                          const uint16_t* b_lo, const UpArgs& ua, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  dim3 grid(ntiles), block(256);
  const bool with_g = ua.coef_g != 0.f || ua.target_err == 1;
  const bool w_bf16 = ua.w_bf16 != 0 && ua.target_err != 2;     // element type of the target as the caller of this launch states it (the momentum is always fp32)
  if (ua.outer) {
    if (!vec || w_bf16) return hipErrorInvalidValue;       // the outer-step epilogue exists for 16-byte row accesses of fp32 weights only
    hipLaunchKernelGGL((k_proj_up_dma<4, 2, false>), grid, block, 0, s, d, tiles, b_hi, b_lo, ua);
  } else if (with_g) {
    if (!vec) return hipErrorInvalidValue;                 // the gradient-term epilogue exists for four-column row accesses only
    if (w_bf16) hipLaunchKernelGGL((k_proj_up_dma<4, 1, true>), grid, block, 0, s, d, tiles, b_hi, b_lo, ua);
    else hipLaunchKernelGGL((k_proj_up_dma<4, 1, false>), grid, block, 0, s, d, tiles, b_hi, b_lo, ua);
  } else if (vec) {
    if (w_bf16) hipLaunchKernelGGL((k_proj_up_dma<4, 0, true>), grid, block, 0, s, d, tiles, b_hi, b_lo, ua);
    else hipLaunchKernelGGL((k_proj_up_dma<4, 0, false>), grid, block, 0, s, d, tiles, b_hi, b_lo, ua);
  } else {
    if (w_bf16) hipLaunchKernelGGL(k_proj_up<true>, grid, block, 0, s, d, tiles, b_hi, b_lo, -ua.coef_acc, 0);
    else hipLaunchKernelGGL(k_proj_up<false>, grid, block, 0, s, d, tiles, b_hi, b_lo, -ua.coef_acc, ua.target_err == 2 ? 1 : 0);
  }
  return hipGetLastError();
}

}  // namespace lordo
