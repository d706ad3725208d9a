// Grouped GEMM for the subspace refresh: range-finder products (any shape and alignment), Gram matrices,
// blocked Cholesky panels, the inverse of the factor and its application, and the moment rotation.
// One launch runs a list of independent problems (one per weight matrix); a tile table maps each
// workgroup to (problem, tile, K slice).  Operands are addressed by element strides, so any transpose
// and the bf16 gradient type are handled by the loader; accumulation is fp32.  Arithmetic: operands that
// can be read with 16-byte accesses are split into bf16 terms (three per fp32 operand: as exact as fp32)
// and multiplied on v_mfma_f32_32x32x16_bf16; anything else runs on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32).
#include "common.h"

namespace lordo {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TK = 32;

#define GAS __attribute__((address_space(1)))

__device__ __forceinline__ const char* resolve(const DevCtx& d, const OpRef& r, int mat) {
  if (r.ext >= 0) return reinterpret_cast<const char*>(ext_ptr(d, r.ext, mat)) + r.off;
  return d.arena + r.off;
}

// One operand of a workgroup tile: X(i, k), i < LIM (the M or N side), k < kend, at base + i*s_i + k*s_k.
// The tile is TMN x TK; a thread fetches NV vectors of four elements along the unit-stride direction
// (scalar accesses at ragged edges and for unaligned operands) and later writes them to LDS as
// S[k][i], the order the matrix-core operands are read in.
template <int TMN, int NV>
struct Operand {
  const char* base;
  int64_t s_i, s_k;
  int is_bf16, lim, kend, i0;
  bool kfast, vec_ok;

  __device__ __forceinline__ void setup(const char* b, int64_t si, int64_t sk, int bf, int lim_, int kend_, int i0_, int kbeg) {
    base = b; s_i = si; s_k = sk; is_bf16 = bf; lim = lim_; kend = kend_; i0 = i0_;
    kfast = sk == 1 && si != 1;
    const int64_t s_fast = kfast ? sk : si, s_slow = kfast ? si : sk;
    const int n_fast = kfast ? kend_ : lim_;
    const uintptr_t align = is_bf16 ? 7 : 15;
    // whole vectors only: every vector then lies entirely inside or entirely outside the operand
    vec_ok = s_fast == 1 && (s_slow & 3) == 0 && (n_fast & 3) == 0 && (reinterpret_cast<uintptr_t>(b) & align) == 0 && (kbeg & 3) == 0;
  }
  __device__ __forceinline__ void coords(int v, int& ii, int& kk) const {
    if (kfast) { kk = (v % (TK / 4)) * 4; ii = v / (TK / 4); }
    else { ii = (v % (TMN / 4)) * 4; kk = v / (TMN / 4); }
  }
  // Branch-free: an element outside the operand is read from element 0 (always valid) and replaced
  // by zero when the tile is written to LDS.  fetch_raw only issues the loads and leaves the loaded
  // bits untouched, so nothing waits for them until stash() runs one K step later.
  template <bool BF16, bool VEC>
  __device__ __forceinline__ void fetch_raw(u32x4 (&raw)[NV], int k0, int tid) const {
    const int64_t e_step = kfast ? s_k : s_i;                        // from one element of a vector to the next
    const int d_i = kfast ? 0 : 1, d_k = kfast ? 1 : 0;
#pragma unroll
    for (int n = 0; n < NV; ++n) {
      int ii, kk;
      coords(tid + n * 256, ii, kk);
      const int gi = i0 + ii, gk = k0 + kk;
      const int64_t idx = (int64_t)gi * s_i + (int64_t)gk * s_k;
      if constexpr (VEC) {
        const int64_t at = (gi < lim && gk < kend) ? idx : 0;
        if constexpr (BF16) {
          u32x2 w = *reinterpret_cast<const GAS u32x2*>((const GAS char*)base + at * 2);
          raw[n].x = w.x; raw[n].y = w.y;
        } else {
          raw[n] = *reinterpret_cast<const GAS u32x4*>((const GAS char*)base + at * 4);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool ok = gi + e * d_i < lim && gk + e * d_k < kend;
          const int64_t at = ok ? idx + e * e_step : 0;
          if constexpr (BF16) raw[n][e] = *reinterpret_cast<const GAS uint16_t*>((const GAS char*)base + at * 2);
          else raw[n][e] = *reinterpret_cast<const GAS uint32_t*>((const GAS char*)base + at * 4);
        }
      }
    }
  }
  // Converts the raw bits of the tile starting at k0, zeroes what lies outside the operand and writes S[k][i].
  template <bool BF16, bool VEC>
  __device__ __forceinline__ void stash(const u32x4 (&raw)[NV], float (*S)[TMN + 4], int k0, int tid) const {
    const int d_i = kfast ? 0 : 1, d_k = kfast ? 1 : 0;
#pragma unroll
    for (int n = 0; n < NV; ++n) {
      int ii, kk;
      coords(tid + n * 256, ii, kk);
      const int gi = i0 + ii, gk = k0 + kk;
      f32x4 r;
      if constexpr (VEC && BF16) {
        r.x = __uint_as_float(raw[n].x << 16); r.y = __uint_as_float(raw[n].x & 0xffff0000u);
        r.z = __uint_as_float(raw[n].y << 16); r.w = __uint_as_float(raw[n].y & 0xffff0000u);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = __uint_as_float(BF16 ? raw[n][e] << 16 : raw[n][e]);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (!(gi + e * d_i < lim && gk + e * d_k < kend)) r[e] = 0.f;
      if (kfast) {
#pragma unroll
        for (int e = 0; e < 4; ++e) S[kk + e][ii] = r[e];
      } else {
        *reinterpret_cast<f32x4*>(&S[kk][ii]) = r;
      }
    }
  }
};

// K loop of one workgroup tile, specialised on the element type of A and on whole-vector access.
template <int WB, bool A_BF16, bool VEC, int TM, int NV>
__device__ __forceinline__ void gemm_loop(f32x16 (&acc)[WB][WB], const Operand<TM, NV>& opA, const Operand<TM, NV>& opB,
                                          float (*As)[TM + 4], float (*Bs)[TM + 4], int kbeg, int K, int tid, int lane, int wm, int wn) {
  u32x4 ra[NV], rb[NV];
  opA.template fetch_raw<A_BF16, VEC>(ra, kbeg, tid);
  opB.template fetch_raw<false, VEC>(rb, kbeg, tid);
  for (int k0 = kbeg; k0 < K; k0 += TK) {
    __syncthreads();                           // previous tile fully consumed
    opA.template stash<A_BF16, VEC>(ra, As, k0, tid);
    opB.template stash<false, VEC>(rb, Bs, k0, tid);
    __syncthreads();
    if (k0 + TK < K) {
      opA.template fetch_raw<A_BF16, VEC>(ra, k0 + TK, tid);
      opB.template fetch_raw<false, VEC>(rb, k0 + TK, tid);
    }
    asm volatile("" ::: "memory");             // keep the loads above the arithmetic: they must be in flight during it
#pragma unroll
    for (int kk = 0; kk < TK; kk += 2) {
      float av[WB], bv[WB];
#pragma unroll
      for (int a = 0; a < WB; ++a) av[a] = As[kk + (lane >> 5)][wm + 32 * a + (lane & 31)];
#pragma unroll
      for (int b = 0; b < WB; ++b) bv[b] = Bs[kk + (lane >> 5)][wn + 32 * b + (lane & 31)];
#pragma unroll
      for (int a = 0; a < WB; ++a)
#pragma unroll
        for (int b = 0; b < WB; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a], bv[b], acc[a][b], 0, 0, 0);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Split-bf16 variant of the K loop for the range-finder products (Alg. 2 sketch and power
// iteration).  Operands go to LDS as bf16 planes in matrix-core fragment order -- a bf16 source is
// exact, an fp32 operand becomes hi + mid + lo, each rounded to nearest (2^-26 relative, as exact as fp32) -- and the
// products run on v_mfma_f32_32x32x16_bf16: three passes for a bf16 source, six for an fp32 one
// (all products of terms down to 2^-24).  Two terms (2^-16) are not enough: the trailing directions
// of the range finder's block sit in the noise of the source, where gaps between singular values are
// of the order of a percent, and a 2^-16 perturbation moved the subspace by up to 9e-4 in Frobenius
// norm of the projector, against 3e-5 for fp32 arithmetic.
// Plane element (i, k) of a TMN x 32 tile: ((i/32)*4 + k/8) * 264 + (i%32)*8 + k%8 (eight elements
// of padding per 32 x 8 group spread the groups over the LDS banks).
// ---------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int frag_index(int i, int k) { return ((i >> 5) * 4 + (k >> 3)) * 264 + (i & 31) * 8 + (k & 7); }

// Operand tile of the split-bf16 loop; whole-vector access only (the caller falls back to the fp32
// loop otherwise).  A thread owns up to four vectors of four elements; along k they pack directly,
// along i the thread owns a 4 x 4 patch (four i, four consecutive k) and transposes it in registers.
template <int TMN>
struct OperandBF {
  const char* base;
  int64_t s_i, s_k;
  int lim, kend, i0;
  bool kfast;
  static constexpr int NVK = TMN / 32;          // vectors per thread when k is the unit-stride direction

  __device__ __forceinline__ void setup(const char* b, int64_t si, int64_t sk, int lim_, int kend_, int i0_) {
    base = b; s_i = si; s_k = sk; lim = lim_; kend = kend_; i0 = i0_;
    kfast = sk == 1 && si != 1;
  }
  // vector n of thread tid: first element (ii, kk); false if the thread has no such vector
  __device__ __forceinline__ bool coords(int tid, int n, int& ii, int& kk) const {
    if (kfast) {
      if (n >= NVK) return false;
      const int v = tid + n * 256;
      kk = (v & 7) * 4; ii = v >> 3;
      return true;
    }
    if (tid >= TMN * 2) return false;           // TMN/4 i-quads x 8 k-quads patches
    ii = (tid % (TMN / 4)) * 4;
    kk = (tid / (TMN / 4)) * 4 + n;
    return true;
  }
  template <bool BF16>
  __device__ __forceinline__ void fetch_raw(u32x4 (&raw)[4], int k0, int tid) const {
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      int ii = 0, kk = 0;
      const bool have = coords(tid, n, ii, kk);
      const int gi = i0 + ii, gk = k0 + kk;
      const int64_t at = (have && gi < lim && gk < kend) ? (int64_t)gi * s_i + (int64_t)gk * s_k : 0;
      if constexpr (BF16) {
        u32x2 w = *reinterpret_cast<const GAS u32x2*>((const GAS char*)base + at * 2);
        raw[n].x = w.x; raw[n].y = w.y;
      } else {
        raw[n] = *reinterpret_cast<const GAS u32x4*>((const GAS char*)base + at * 4);
      }
    }
  }
  // Two fp32 values -> three packed bf16 pairs whose sum is the values to 2^-26: hi is the value rounded to nearest,
  // mid the (exactly representable) remainder rounded to nearest, lo the rounded rest; the conversion is the
  // hardware's packed round-to-nearest-even instruction, about five vector operations per element.
  // Rounding to nearest, not truncation: truncated terms all carry the sign of the value, so on the diagonal of a
  // Gram matrix X^T X every cross product hi * lo is positive; those below half an ulp of the running sum are
  // rounded away one k-step after the other, and the diagonal came out too small by up to 2e-5 relative (growing
  // with the length of the contraction), i.e. the columns of the orthonormalised block too long by 1e-5.  With
  // terms of random sign the same loss has zero mean.
  static __device__ __forceinline__ uint32_t pack_rne(float x0, float x1) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {x0, x1};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  }
  static __device__ __forceinline__ void split3(uint32_t x0, uint32_t x1, uint32_t (&t)[3]) {
    const float f0 = __uint_as_float(x0), f1 = __uint_as_float(x1);
    t[0] = pack_rne(f0, f1);
    const float r0 = f0 - __uint_as_float(t[0] << 16);
    const float r1 = f1 - __uint_as_float(t[0] & 0xffff0000u);
    t[1] = pack_rne(r0, r1);
    const float s0 = r0 - __uint_as_float(t[1] << 16);
    const float s1 = r1 - __uint_as_float(t[1] & 0xffff0000u);
    t[2] = pack_rne(s0, s1);
  }
  // P: the operand's planes (one for an exact bf16 operand, three for an fp32 one), PLANE elements apart
  template <bool BF16>
  __device__ __forceinline__ void stash(const u32x4 (&raw)[4], uint16_t* P, int plane, int k0, int tid) const {
    if (kfast) {
#pragma unroll
      for (int n = 0; n < NVK; ++n) {
        int ii = 0, kk = 0;
        coords(tid, n, ii, kk);
        const bool ok = i0 + ii < lim && k0 + kk < kend;
        const int at = frag_index(ii, kk);                    // four consecutive k: 8 contiguous bytes
        if constexpr (BF16) {
          *reinterpret_cast<u32x2*>(P + at) = ok ? u32x2{raw[n].x, raw[n].y} : u32x2{0u, 0u};
        } else {
          uint32_t ta[3], tb[3];
          split3(raw[n].x, raw[n].y, ta);
          split3(raw[n].z, raw[n].w, tb);
#pragma unroll
          for (int c = 0; c < 3; ++c) *reinterpret_cast<u32x2*>(P + c * plane + at) = ok ? u32x2{ta[c], tb[c]} : u32x2{0u, 0u};
        }
      }
    } else if (tid < TMN * 2) {
      // 4 x 4 patch: vector n holds i = ii .. ii+3 at k = kfirst + n; row ii + e of the plane gets k = kfirst .. kfirst+3
      int ii = 0, kfirst = 0;
      coords(tid, 0, ii, kfirst);
      const bool i_ok = i0 + ii < lim;
      u32x4 r[4];
#pragma unroll
      for (int n = 0; n < 4; ++n) r[n] = (i_ok && k0 + kfirst + n < kend) ? raw[n] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int at = frag_index(ii + e, kfirst);
        if constexpr (BF16) {                                 // element e of vector n: half (e & 1) of word e / 2
          const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
          u32x2 h;
          h.x = __builtin_amdgcn_perm(r[1][e >> 1], r[0][e >> 1], sel);
          h.y = __builtin_amdgcn_perm(r[3][e >> 1], r[2][e >> 1], sel);
          *reinterpret_cast<u32x2*>(P + at) = h;
        } else {
          uint32_t ta[3], tb[3];
          split3(r[0][e], r[1][e], ta);
          split3(r[2][e], r[3][e], tb);
#pragma unroll
          for (int c = 0; c < 3; ++c) *reinterpret_cast<u32x2*>(P + c * plane + at) = u32x2{ta[c], tb[c]};
        }
      }
    }
  }
};

// same_ab (uniform): the tile of B is the tile of A (a diagonal tile of a Gram matrix X^T X): it is fetched and
// split once and the B fragments are read from the planes of A.
template <int WB, bool A_BF16, int TM>
__device__ __forceinline__ void gemm_loop_bf(f32x16 (&acc)[WB][WB], const OperandBF<TM>& opA, const OperandBF<TM>& opB,
                                             uint16_t* lds, int kbeg, int K, int tid, int lane, int wm, int wn, bool same_ab) {
  constexpr int PLANE = (TM / 32) * 4 * 264;                   // elements
  constexpr int NA = A_BF16 ? 1 : 3;                           // planes of A; B always has three
  uint16_t* PA = lds;
  uint16_t* PB = (!A_BF16 && same_ab) ? lds : lds + NA * PLANE;
  const bool own_b = A_BF16 || !same_ab;
  u32x4 ra[4], rb[4];
  opA.template fetch_raw<A_BF16>(ra, kbeg, tid);
  if (own_b) opB.template fetch_raw<false>(rb, kbeg, tid);
  for (int k0 = kbeg; k0 < K; k0 += TK) {
    __syncthreads();                           // previous tile fully consumed
    opA.template stash<A_BF16>(ra, PA, PLANE, k0, tid);
    if (own_b) opB.template stash<false>(rb, PB, PLANE, k0, tid);
    __syncthreads();
    if (k0 + TK < K) {
      opA.template fetch_raw<A_BF16>(ra, k0 + TK, tid);
      if (own_b) opB.template fetch_raw<false>(rb, k0 + TK, tid);
    }
    asm volatile("" ::: "memory");             // keep the loads above the arithmetic: they must be in flight during it
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      bf16x8 fa[NA][WB], fb[3][WB];
      const int kg = 16 * ks + 8 * (lane >> 5);
#pragma unroll
      for (int a = 0; a < WB; ++a) {
        const int at = frag_index(wm + 32 * a + (lane & 31), kg);
#pragma unroll
        for (int c = 0; c < NA; ++c) fa[c][a] = *reinterpret_cast<const bf16x8*>(PA + c * PLANE + at);
      }
#pragma unroll
      for (int b = 0; b < WB; ++b) {
        const int at = frag_index(wn + 32 * b + (lane & 31), kg);
#pragma unroll
        for (int c = 0; c < 3; ++c) fb[c][b] = *reinterpret_cast<const bf16x8*>(PB + c * PLANE + at);
      }
      // every product of terms down to 2^-24: (a0, b0..b2) for an exact A; plus (a1, b0), (a1, b1), (a2, b0)
#pragma unroll
      for (int ca = 0; ca < NA; ++ca)
#pragma unroll
        for (int cb = 0; cb + ca < 3; ++cb)
#pragma unroll
          for (int a = 0; a < WB; ++a)
#pragma unroll
            for (int b = 0; b < WB; ++b)
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ca][a], fb[cb][b], acc[a][b], 0, 0, 0);
    }
  }
}

// 256 threads = 4 waves in a 2 x 2 grid; each wave WB x WB accumulator blocks of 32 x 32, so the
// workgroup tile is 64*WB square (64 for small problems, 128 for large launches).  The next K tile
// is fetched into registers while the matrix cores work on the one in LDS.
template <int WB>
__global__ __launch_bounds__(256) void k_gemm32(DevCtx d, const GemmDesc* __restrict__ descs,
                                                const GemmTile* __restrict__ tiles, int src_is_bf16, float alpha_mul) {
  constexpr int TM = 64 * WB, TN = 64 * WB;
  constexpr int PITCH = TM + 4;
  constexpr int NV = TM * TK / 4 / 256;
  const GemmTile t = tiles[blockIdx.x];
  const GemmDesc g = descs[t.desc];
  if (mat_skipped(d, g.mat)) return;
  const int M = g.M, N = g.N;
  const int kbeg = g.ksplit > 1 ? t.ks * g.klen : 0;
  int K = g.ksplit > 1 ? (kbeg + g.klen < g.K ? kbeg + g.klen : g.K) : g.K;           // end of this slice
  const int m0 = t.tm * TM, n0 = t.tn * TN;
  if (g.tri && n0 + TN < K) K = n0 + TN;            // B is zero below this tile's last column
  const int a_bf16 = g.a_bf16 == 2 ? src_is_bf16 : g.a_bf16;
  float* C = reinterpret_cast<float*>(const_cast<char*>(resolve(d, g.C, g.mat)));
  float* C2 = g.C2.off >= 0 ? reinterpret_cast<float*>(const_cast<char*>(resolve(d, g.C2, g.mat))) : nullptr;

  // As | Bs of the fp32 loop, or up to six bf16 planes of the split loop
  constexpr int LDS_FLOATS = 2 * TK * PITCH > 3 * (TM / 32) * 4 * 264 ? 2 * TK * PITCH : 3 * (TM / 32) * 4 * 264;
  __shared__ __attribute__((aligned(16))) float lds_raw[LDS_FLOATS];
  float (*As)[PITCH] = reinterpret_cast<float (*)[PITCH]>(lds_raw);
  float (*Bs)[PITCH] = reinterpret_cast<float (*)[PITCH]>(lds_raw + TK * PITCH);
  static_assert(sizeof(lds_raw) >= sizeof(uint16_t) * 6 * (TM / 32) * 4 * 264, "six bf16 planes must fit");

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = (wave & 1) * 32 * WB, wn = (wave >> 1) * 32 * WB;

  Operand<TM, NV> opA, opB;
  opA.setup(resolve(d, g.A, g.mat), g.sAm, g.sAk, a_bf16, M, K, m0, kbeg);
  opB.setup(resolve(d, g.B, g.mat), g.sBn, g.sBk, 0, N, K, n0, kbeg);

  f32x16 acc[WB][WB];
#pragma unroll
  for (int a = 0; a < WB; ++a)
#pragma unroll
    for (int b = 0; b < WB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  if (kbeg < K && g.prec == 1 && opA.vec_ok && opB.vec_ok) {
    OperandBF<TM> pa, pb;
    pa.setup(opA.base, g.sAm, g.sAk, M, K, m0);
    pb.setup(opB.base, g.sBn, g.sBk, N, K, n0);
    uint16_t* planes = reinterpret_cast<uint16_t*>(lds_raw);
    // same matrix, same strides with the roles of the two indices swapped, same tile: A(m, k) = B(k, n = m)
    const bool same_ab = g.A.off == g.B.off && g.A.ext == g.B.ext && g.sAm == g.sBn && g.sAk == g.sBk && m0 == n0 && M == N;
    if (a_bf16) gemm_loop_bf<WB, true>(acc, pa, pb, planes, kbeg, K, tid, lane, wm, wn, false);
    else gemm_loop_bf<WB, false>(acc, pa, pb, planes, kbeg, K, tid, lane, wm, wn, same_ab);
  } else if (kbeg < K) {
    const bool vec = opA.vec_ok && opB.vec_ok;
    if (a_bf16) {
      if (vec) gemm_loop<WB, true, true>(acc, opA, opB, As, Bs, kbeg, K, tid, lane, wm, wn);
      else gemm_loop<WB, true, false>(acc, opA, opB, As, Bs, kbeg, K, tid, lane, wm, wn);
    } else {
      if (vec) gemm_loop<WB, false, true>(acc, opA, opB, As, Bs, kbeg, K, tid, lane, wm, wn);
      else gemm_loop<WB, false, false>(acc, opA, opB, As, Bs, kbeg, K, tid, lane, wm, wn);
    }
  }

  float* Pp = g.ksplit > 1 ? reinterpret_cast<float*>(const_cast<char*>(resolve(d, g.P, g.mat))) + (int64_t)t.ks * M * N : nullptr;
  // accumulator register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the block
#pragma unroll
  for (int a = 0; a < WB; ++a)
#pragma unroll
    for (int b = 0; b < WB; ++b) {
      const int col = n0 + wn + 32 * b + (lane & 31);
      if (col >= N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int row = m0 + wm + 32 * a + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < M && Pp) {
          Pp[(int64_t)row * N + col] = acc[a][b][v];
        } else if (row < M) {
          int64_t o = (int64_t)row * g.ldc + col;
          float val = g.alpha * alpha_mul * acc[a][b][v];
          if (g.beta != 0.f) val = fmaf(g.beta, C[o], val);
          C[o] = val;
          if (C2) C2[o] = val * val;
        }
      }
    }
}

// Sum of the split-K slices in slice order (deterministic), then alpha, beta and the optional square.
__global__ __launch_bounds__(256) void k_gemm_reduce(DevCtx d, const GemmDesc* __restrict__ descs) {
  const GemmDesc g = descs[blockIdx.y];
  if (g.ksplit <= 1 || mat_skipped(d, g.mat)) return;
  const float* Pp = reinterpret_cast<const float*>(resolve(d, g.P, g.mat));
  float* C = reinterpret_cast<float*>(const_cast<char*>(resolve(d, g.C, g.mat)));
  float* C2 = g.C2.off >= 0 ? reinterpret_cast<float*>(const_cast<char*>(resolve(d, g.C2, g.mat))) : nullptr;
  const int64_t total = (int64_t)g.M * g.N;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    float acc = 0.f;
    for (int sl = 0; sl < g.ksplit; ++sl) acc += Pp[(int64_t)sl * total + e];
    int64_t o = (e / g.N) * g.ldc + e % g.N;
    float val = g.alpha * acc;
    if (g.beta != 0.f) val = fmaf(g.beta, C[o], val);
    C[o] = val;
    if (C2) C2[o] = val * val;
  }
}
hipError_t launch_gemm_reduce(const DevCtx& d, const GemmDesc* descs, int ndescs, hipStream_t s) {
  if (ndescs <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_gemm_reduce, dim3(64, ndescs), dim3(256), 0, s, d, descs);
  return hipGetLastError();
}

hipError_t launch_gemm32(const DevCtx& d, const GemmDesc* descs, const GemmTile* tiles, int ntiles, int tile, int src_is_bf16,
                         hipStream_t s, float alpha_mul) {
  if (ntiles <= 0) return hipSuccess;
  if (tile == 128) hipLaunchKernelGGL((k_gemm32<2>), dim3(ntiles), dim3(256), 0, s, d, descs, tiles, src_is_bf16, alpha_mul);
  else hipLaunchKernelGGL((k_gemm32<1>), dim3(ntiles), dim3(256), 0, s, d, descs, tiles, src_is_bf16, alpha_mul);
  return hipGetLastError();
}

}  // namespace lordo
