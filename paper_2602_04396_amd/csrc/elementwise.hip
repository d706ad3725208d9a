// Elementwise, packing and small dense kernels of the LoRDO library (gfx950).
//   k_adam4           fused low-rank Adam update on the flat low-rank arena (Sec. 2; Alg. 1 moment lines), with the
//                     low-rank QHM bracket, the column sums of the full-rank QHM scale (Sec. 3.2), the planes of g
//                     for the error-feedback residual and the up-link buffer (App. A.5.1) as options
//   k_pq<MODE>        p x q family: outer step (Alg. 1 OuterOpt; App. A.2, D.4), pseudo-gradient anchor - W
//                     (App. A.1), anchor copy, and the part of the outer step that does not depend on Delta
//   k_fold_grad       E <- E + s G, the projection source of the local variant (Alg. 2)
//   k_pack_q / k_pack_y / k_pack_block / k_split_planes   fp32 -> bf16 hi/lo operand planes in matrix-core order
//   k_glow_to_z, k_lr_to_plain, k_plain_to_lr, k_lr_exchange, k_tr_exchange   between the operand layout of the low-rank state and plain buffers
//   k_gram_shift, k_potf2, k_diag_inverses   CholeskyQR: diagonal shift, Cholesky of a diagonal block and its inverse
//   k_jacobi_svd      singular vectors of the Cholesky factor of the r x r Ritz matrix (Rayleigh-Ritz step: basis ordered as in Sec. 2's SVD projection)
//   k_frob2_chunks / k_frob2_sum / k_stable_rank   squared Frobenius norm of the refresh source and its stable rank (Sec. 5.1)
//   k_rot_pre / k_rot_post, k_mssv   elementwise parts of the moment rotation (Alg. 1 rotation lines); similarity diagnostic (Sec. 5.1)
//   k_step            step count and bias corrections 1 - beta^t (Sec. 2) in device memory, advanced once per local step
//   k_gauss_block     Gaussian start blocks of the range finder and of the random initial projection (Alg. 1 Require)
//   k_gram_diag_part / k_gram_diag_sum   exact diagonal of the Gram matrices of CholeskyQR
//   k_bf16_to_f32 / k_f32_to_bf16   a bf16-stored residual through the fp32 state interface
#include "common.h"

namespace lordo {

// ---------------------------------------------------------------------------------------
// bf16 helpers: round-to-nearest-even split of an fp32 value into hi + lo
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t f2bf(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf2f(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ void split_bf(float x, uint32_t& hi, uint32_t& lo) {
  hi = f2bf(x);
  lo = f2bf(x - bf2f(hi));
}

// ---------------------------------------------------------------------------------------
// fused low-rank Adam: one thread per 4 consecutive elements of the flat arena
// ---------------------------------------------------------------------------------------
typedef float f32x4n __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2n __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4n __attribute__((ext_vector_type(4)));

// g is read for the last time here and the moments are not touched again before the next step, a
// gigabyte of traffic later: their accesses are non-temporal (streaming lines in L2 and the
// last-level cache).  N is consumed by the up-projection right away and stays cacheable.
__device__ __forceinline__ f32x4n ld_stream(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4n*>(p)); }
__device__ __forceinline__ void st_stream(float* p, f32x4n x) { __builtin_nontemporal_store(x, reinterpret_cast<f32x4n*>(p)); }
// COLSUM: also leave, per column and block of 32 rank indices, the sum of the denominators
// sqrt(v_hat) + eps (the column scale of the full-rank quasi-hyperbolic update, Sec. 3.2, is their
// mean over the rank).  Eight threads of a workgroup hold the four octets of such a block: their
// sums meet in LDS and are added in fixed order.  Padded rank indices contribute eps each; the
// consumer subtracts that.
// Four elements per thread: every load and store instruction of a wave covers one dense kilobyte (16 bytes per lane,
// consecutive lanes consecutive addresses).  With eight elements per thread, as two 16-byte accesses per lane and array,
// a wave instruction touched every other 16 bytes of two kilobytes and the pass took 15 % longer.
template <bool COLSUM>
__global__ __launch_bounds__(256) void k_adam4(const float* __restrict__ glow, float* __restrict__ u,
                                               float* __restrict__ v, uint16_t* __restrict__ n_hi,
                                               uint16_t* __restrict__ n_lo, int64_t nquads, AdamArgs a) {
  __shared__ float part[COLSUM ? 256 : 1];
  const int64_t qidx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const bool live = qidx < nquads;
  if (!COLSUM && !live) return;
  const int64_t base = a.first + qidx * 4;
  float dsum = 0.f;
  const float inv_c1 = a.step->inv_c1, inv_c2 = a.step->inv_c2;      // uniform: scalar loads
  if (live) {
  f32x4n g = __builtin_nontemporal_load(reinterpret_cast<const f32x4n*>(glow + base));
  int nsplit = a.grp_nsplit[0];
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (base >= a.grp_start[i]) nsplit = a.grp_nsplit[i];
  for (int sidx = 1; sidx < nsplit; ++sidx)               // deterministic split-K reduction, fixed order
    g += __builtin_nontemporal_load(reinterpret_cast<const f32x4n*>(glow + sidx * a.split_stride + base));
  f32x4n uu = ld_stream(u + base), vv = ld_stream(v + base);
  uint32_t hi[4], lo[4];
  f32x4n nv;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float un = fmaf(a.b1, uu[e], a.omb1 * g[e]);
    const float vn = fmaf(a.b2, vv[e], a.omb2 * (g[e] * g[e]));
    uu[e] = un;
    vv[e] = vn;
    const float den = sqrtf(vn * inv_c2) + a.eps;
    dsum += den;
    // Alg. 1 update bracket: u_hat / den, or (omega u_hat + (1 - omega) g) / den for the low-rank
    // quasi-hyperbolic case; with qw = 1, qg = 0 the value is bit-identical to u_hat / den
    // den == 0 needs eps == 0 and a second moment of exactly zero, i.e. every gradient so far was zero there (always
    // true in the zero padding of the arena): the update is then zero, not 0 / 0
    const float nn = den == 0.f ? 0.f : fmaf(a.qg, g[e], a.qw * (un * inv_c1)) / den;
    split_bf(nn, hi[e], lo[e]);
    nv[e] = nn;
  }
  if (a.acc) {
    f32x4n c0 = ld_stream(a.acc + base);
#pragma unroll
    for (int e = 0; e < 4; ++e) c0[e] = fmaf(a.lr, nv[e], c0[e]);
    st_stream(a.acc + base, c0);
  }
  st_stream(u + base, uu);
  st_stream(v + base, vv);
  u32x2n ph, pl;
  ph.x = hi[0] | (hi[1] << 16); ph.y = hi[2] | (hi[3] << 16);
  pl.x = lo[0] | (lo[1] << 16); pl.y = lo[2] | (lo[3] << 16);
  *reinterpret_cast<u32x2n*>(n_hi + base) = ph;
  *reinterpret_cast<u32x2n*>(n_lo + base) = pl;
  if (a.g_hi) {
#pragma unroll
    for (int e = 0; e < 4; ++e) split_bf(g[e], hi[e], lo[e]);
    ph.x = hi[0] | (hi[1] << 16); ph.y = hi[2] | (hi[3] << 16);
    pl.x = lo[0] | (lo[1] << 16); pl.y = lo[2] | (lo[3] << 16);
    *reinterpret_cast<u32x2n*>(a.g_hi + base) = ph;
    *reinterpret_cast<u32x2n*>(a.g_lo + base) = pl;
  }
  }
  if constexpr (COLSUM) {
    // Full-rank QHM scale (Sec. 3.2): per column and block of 32 rank indices, the sum of sqrt(v_hat) + eps.  A group
    // of eight elements has index (column block * (rp/8) + octet) * 32 + column and is held by two threads; a.first/8
    // and the group count of every matrix are multiples of 128, so threadIdx = ((octet % 4) * 32 + column) * 2 + half.
    part[threadIdx.x] = dsum;
    __syncthreads();
    if (live && threadIdx.x < 64 && (threadIdx.x & 1) == 0) {
      const int t0 = threadIdx.x;                    // octet % 4 = 0, half = 0 of its column
      float sum = 0.f;
#pragma unroll
      for (int o = 0; o < 4; ++o) sum += part[t0 + 64 * o] + part[t0 + 64 * o + 1];      // fixed order
      // this thread's group is (cb*(rp/8) + 4*rb)*32 + column; the sum goes to (cb*(rp/32) + rb)*32 + column
      const int64_t grp = base >> 3;
      a.colpart[((grp & ~int64_t(31)) >> 2) + (grp & 31)] = sum;
    }
  }
}

// fp32 array in operand layout -> bf16 hi / lo planes (the low-rank pseudo-gradient as B operand of the up-projection)
__global__ __launch_bounds__(256) void k_split_planes(const float* __restrict__ src, uint16_t* __restrict__ p_hi,
                                                      uint16_t* __restrict__ p_lo, int64_t ngroups) {
  const int64_t gidx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gidx >= ngroups) return;
  const int64_t base = gidx * 8;
  const f32x4n a0 = *reinterpret_cast<const f32x4n*>(src + base), a1 = *reinterpret_cast<const f32x4n*>(src + base + 4);
  const float x[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
  uint32_t hi[8], lo[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) split_bf(x[e], hi[e], lo[e]);
  u32x4n ph, pl;
  ph.x = hi[0] | (hi[1] << 16); ph.y = hi[2] | (hi[3] << 16); ph.z = hi[4] | (hi[5] << 16); ph.w = hi[6] | (hi[7] << 16);
  pl.x = lo[0] | (lo[1] << 16); pl.y = lo[2] | (lo[3] << 16); pl.z = lo[4] | (lo[5] << 16); pl.w = lo[6] | (lo[7] << 16);
  *reinterpret_cast<u32x4n*>(p_hi + base) = ph;
  *reinterpret_cast<u32x4n*>(p_lo + base) = pl;
}
hipError_t launch_split_planes(const float* src, uint16_t* p_hi, uint16_t* p_lo, int64_t nelem, hipStream_t s) {
  const int64_t ngroups = nelem / 8;                  // nelem is a multiple of 8
  if (ngroups <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_split_planes, dim3((unsigned)((ngroups + 255) / 256)), dim3(256), 0, s, src, p_hi, p_lo, ngroups);
  return hipGetLastError();
}

hipError_t launch_adam(const float* glow, float* u, float* v, uint16_t* n_hi, uint16_t* n_lo, int64_t nelem,
                       const AdamArgs& a, hipStream_t s) {
  int64_t ngroups = (nelem - a.first) / 8;            // a.first and nelem are multiples of 8
  if (ngroups <= 0) return hipSuccess;
  unsigned blocks = (unsigned)((ngroups + 255) / 256);
  if (a.colpart) hipLaunchKernelGGL(k_adam4<true>, dim3(2 * blocks), dim3(256), 0, s, glow, u, v, n_hi, n_lo, 2 * ngroups, a);
  else hipLaunchKernelGGL(k_adam4<false>, dim3(2 * blocks), dim3(256), 0, s, glow, u, v, n_hi, n_lo, 2 * ngroups, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// step counter on the device: t <- t + 1 (set_to < 0) or t <- set_to, and the bias corrections of the new t
// (Sec. 2: u_hat = u / (1 - beta1^t), v_hat = v / (1 - beta2^t)), formed in double and rounded to fp32 once
// ---------------------------------------------------------------------------------------
__global__ void k_step(StepDev* sd, double beta1, double beta2, int bias_correction, int64_t set_to) {
  const int64_t t = set_to < 0 ? sd->t + 1 : set_to;
  double c1 = 1.0, c2 = 1.0;
  if (bias_correction && t > 0) {
    c1 = 1.0 - pow(beta1, (double)t);
    c2 = 1.0 - pow(beta2, (double)t);
  }
  sd->t = t;
  sd->c1 = (float)c1; sd->c2 = (float)c2;
  sd->inv_c1 = (float)(1.0 / c1); sd->inv_c2 = (float)(1.0 / c2);
}
hipError_t launch_step(StepDev* sd, double beta1, double beta2, int bias_correction, int64_t set_to, hipStream_t s) {
  hipLaunchKernelGGL(k_step, dim3(1), dim3(1), 0, s, sd, beta1, beta2, bias_correction, set_to);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// caller pointer tables: the pointers travel in the kernel arguments, so no host buffer has
// to outlive the call
// ---------------------------------------------------------------------------------------
struct PtrPack { void* p[256]; };
__global__ void k_store_ptrs(PtrPack pack, void** dst, int count) {
  int i = threadIdx.x;
  if (i < count) dst[i] = pack.p[i];
}
hipError_t launch_store_ptrs(void** dst, void* const* host_src, int count, hipStream_t s) {
  for (int done = 0; done < count; done += 256) {
    PtrPack pack;
    int c = count - done < 256 ? count - done : 256;
    for (int i = 0; i < 256; ++i) pack.p[i] = i < c ? host_src[done + i] : nullptr;
    hipLaunchKernelGGL(k_store_ptrs, dim3(1), dim3(256), 0, s, pack, dst + done, c);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------
// fill / copy
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_fill_zero(uint4* dst, int64_t n16) {
  int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = make_uint4(0, 0, 0, 0);
}
hipError_t launch_fill_zero(void* dst, int64_t bytes, hipStream_t s) {
  int64_t n16 = bytes / 16;      // regions are 256-byte multiples
  if (n16 == 0) return hipSuccess;
  int64_t blocks = (n16 + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<uint4*>(dst), n16);
  return hipGetLastError();
}
__global__ __launch_bounds__(256) void k_copy_f32(float* dst, const float* src, int64_t n) {
  int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}
hipError_t launch_copy_f32(float* dst, const float* src, int64_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(k_copy_f32, dim3((unsigned)blocks), dim3(256), 0, s, dst, src, n);
  return hipGetLastError();
}

// a bf16-stored state array read and written through the fp32 state interface
__global__ __launch_bounds__(256) void k_bf16_to_f32(float* dst, const uint16_t* src, int64_t n) {
  int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = __uint_as_float((uint32_t)src[i] << 16);
}
__global__ __launch_bounds__(256) void k_f32_to_bf16(uint16_t* dst, const float* src, int64_t n) {
  int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    uint32_t hi, lo;
    split_bf(src[i], hi, lo);          // hi: the nearest-even bf16 of the value
    dst[i] = (uint16_t)hi;
  }
}
hipError_t launch_bf16_to_f32(float* dst, const uint16_t* src, int64_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(k_bf16_to_f32, dim3((unsigned)blocks), dim3(256), 0, s, dst, src, n);
  return hipGetLastError();
}
hipError_t launch_f32_to_bf16(uint16_t* dst, const float* src, int64_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(k_f32_to_bf16, dim3((unsigned)blocks), dim3(256), 0, s, dst, src, n);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// projection packing
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_identity_q(DevCtx d) {
  const MatDev& m = d.mats[blockIdx.y];
  float* q32 = reinterpret_cast<float*>(d.arena + m.q32);
  int64_t total = (int64_t)m.p * m.r;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int64_t row = i / m.r, col = i % m.r;
    q32[i] = row == col ? 1.0f : 0.0f;
  }
}
hipError_t launch_identity_q(const DevCtx& d, hipStream_t s) {
  hipLaunchKernelGGL(k_identity_q, dim3(64, d.n), dim3(256), 0, s, d);
  return hipGetLastError();
}

// One thread writes one 8-element group of the up-projection planes and one of the
// down-projection planes (both have pp*rp/8 groups).
__global__ __launch_bounds__(256) void k_pack_q(DevCtx d, int mat_first) {
  if (mat_skipped(d, mat_first + blockIdx.y)) return;
  const MatDev& m = d.mats[mat_first + blockIdx.y];
  const float* q32 = reinterpret_cast<const float*>(d.arena + m.q32);
  uint16_t* qa_hi = reinterpret_cast<uint16_t*>(d.arena + m.qa_hi);
  uint16_t* qa_lo = reinterpret_cast<uint16_t*>(d.arena + m.qa_lo);
  uint16_t* qt_hi = reinterpret_cast<uint16_t*>(d.arena + m.qt_hi);
  uint16_t* qt_lo = reinterpret_cast<uint16_t*>(d.arena + m.qt_lo);
  int64_t ngroups = (int64_t)m.pp * m.rp / 8;
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < ngroups; g += (int64_t)gridDim.x * 256) {
    uint32_t hi[8], lo[8];
    {   // up-projection plane: group = (row block, rank octet, row in block)
      int64_t per_mb = (int64_t)(m.rp / 8) * 32;
      int64_t mb = g / per_mb, rem = g % per_mb;
      int64_t k8 = rem / 32, m32 = rem % 32;
      int64_t row = mb * 32 + m32;
      for (int e = 0; e < 8; ++e) {
        int64_t k = k8 * 8 + e;
        float x = (row < m.p && k < m.r) ? q32[row * m.r + k] : 0.0f;
        split_bf(x, hi[e], lo[e]);
      }
      uint4 ph = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
      uint4 pl = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
      *reinterpret_cast<uint4*>(qa_hi + g * 8) = ph;
      *reinterpret_cast<uint4*>(qa_lo + g * 8) = pl;
    }
    {   // down-projection plane: group = (rank block, row octet, rank in block)
      int64_t per_ib = (int64_t)(m.pp / 8) * 32;
      int64_t ib = g / per_ib, rem = g % per_ib;
      int64_t k8 = rem / 32, i32 = rem % 32;
      int64_t i = ib * 32 + i32;
      for (int e = 0; e < 8; ++e) {
        int64_t row = k8 * 8 + e;
        float x = (row < m.p && i < m.r) ? q32[row * m.r + i] : 0.0f;
        split_bf(x, hi[e], lo[e]);
      }
      uint4 ph = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
      uint4 pl = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
      *reinterpret_cast<uint4*>(qt_hi + g * 8) = ph;
      *reinterpret_cast<uint4*>(qt_lo + g * 8) = pl;
    }
  }
}
hipError_t launch_pack_q(const DevCtx& d, int mat_first, int mat_count, hipStream_t s) {
  if (mat_count <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_pack_q, dim3(128, mat_count), dim3(256), 0, s, d, mat_first);
  return hipGetLastError();
}

// Does nothing while a numerical breakdown is latched: a refresh (or an initial projection) whose factorisation met a
// non-positive pivot leaves the projection as it was.
__global__ __launch_bounds__(256) void k_q_from_y(DevCtx d, int ybuf) {
  if (*d.flag != 0 || mat_skipped(d, blockIdx.y)) return;
  const MatDev& m = d.mats[blockIdx.y];
  float* q32 = reinterpret_cast<float*>(d.arena + m.q32);
  const float* y = reinterpret_cast<const float*>(d.arena + m.y[ybuf]);
  int64_t total = (int64_t)m.p * m.r;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) q32[i] = y[i];
}
// Range-finder product Z = Src^T Y on the down-projection kernel (Alg. 2 of the refresh: the product has the
// shape of g = Q^T G with Y in the place of Q): Y (plain p x r, buffer ybuf) -> the down-projection operand
// planes.  The planes hold Q between refreshes; the refresh repacks them from the new Q when it ends.
__global__ __launch_bounds__(256) void k_pack_y(DevCtx d, int ybuf) {
  if (mat_skipped(d, blockIdx.y)) return;
  const MatDev& m = d.mats[blockIdx.y];
  const float* y = reinterpret_cast<const float*>(d.arena + m.y[ybuf]);
  uint16_t* qt_hi = reinterpret_cast<uint16_t*>(d.arena + m.qt_hi);
  uint16_t* qt_lo = reinterpret_cast<uint16_t*>(d.arena + m.qt_lo);
  const int64_t ngroups = (int64_t)m.pp * m.rp / 8;
  const int64_t per_ib = (int64_t)(m.pp / 8) * 32;
  // thread -> (rank block, row octet, rank in block) with the rank fastest: reads of one row are contiguous
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < ngroups; g += (int64_t)gridDim.x * 256) {
    const int64_t ib = g / per_ib, rem = g % per_ib;
    const int64_t k8 = rem / 32, i = ib * 32 + rem % 32;
    uint32_t hi[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int64_t row = k8 * 8 + e;
      const float x = (row < m.p && i < m.r) ? y[row * m.r + i] : 0.0f;
      split_bf(x, hi[e], lo[e]);
    }
    *reinterpret_cast<uint4*>(qt_hi + g * 8) = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
    *reinterpret_cast<uint4*>(qt_lo + g * 8) = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
  }
}
hipError_t launch_pack_y(const DevCtx& d, int ybuf, hipStream_t s) {
  hipLaunchKernelGGL(k_pack_y, dim3(128, d.n), dim3(256), 0, s, d, ybuf);
  return hipGetLastError();
}
// The result of that product, left by the down-projection kernel in the layout of g (split-K slices
// included), as the plain q x r block Z: Z[j][i] = sum over slices of g(i, j), slices added in order.
__global__ __launch_bounds__(256) void k_glow_to_z(DevCtx d, const float* __restrict__ glow, int zbuf, AdamArgs a) {
  if (mat_skipped(d, blockIdx.y)) return;
  const MatDev& m = d.mats[blockIdx.y];
  float* z = reinterpret_cast<float*>(d.arena + m.zw[zbuf]);
  int nsplit = a.grp_nsplit[0];
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (m.lr_off >= a.grp_start[i]) nsplit = a.grp_nsplit[i];
  const int64_t total = (int64_t)m.q * m.r;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t j = t / m.r, i = t % m.r;
    const int64_t src = m.lr_off + bl_index(j, i, m.rp);
    float acc = glow[src];
    for (int sp = 1; sp < nsplit; ++sp) acc += glow[src + sp * a.split_stride];
    z[t] = acc;
  }
}
hipError_t launch_glow_to_z(const DevCtx& d, const float* glow, int zbuf, const AdamArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_glow_to_z, dim3(64, d.n), dim3(256), 0, s, d, glow, zbuf, a);
  return hipGetLastError();
}
// The q x r block of the products Y = Src B (B = Omega from the caller's table when zbuf < 0, else the
// orthonormalised Z in buffer zbuf) as bf16 hi / lo planes in operand layout (m = rank, k = column j),
// at this matrix's place in the flat plane arrays.
__global__ __launch_bounds__(256) void k_pack_block(DevCtx d, int zbuf, uint16_t* __restrict__ p_hi, uint16_t* __restrict__ p_lo) {
  if (mat_skipped(d, blockIdx.y)) return;
  const MatDev& m = d.mats[blockIdx.y];
  const float* z = zbuf < 0 ? reinterpret_cast<const float*>(ext_ptr(d, EXT_OMEGA, blockIdx.y))
                            : reinterpret_cast<const float*>(d.arena + m.zw[zbuf]);
  uint16_t* hi_p = p_hi + m.lr_off;
  uint16_t* lo_p = p_lo + m.lr_off;
  const int64_t ngroups = (int64_t)m.qp * m.rp / 8;
  const int64_t per_ib = (int64_t)(m.qp / 8) * 32;
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < ngroups; g += (int64_t)gridDim.x * 256) {
    const int64_t ib = g / per_ib, rem = g % per_ib;
    const int64_t k8 = rem / 32, i = ib * 32 + rem % 32;       // rank fastest over the threads: reads of one row of Z are contiguous
    uint32_t hi[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int64_t j = k8 * 8 + e;
      const float x = (j < m.q && i < m.r) ? z[j * m.r + i] : 0.0f;
      split_bf(x, hi[e], lo[e]);
    }
    *reinterpret_cast<uint4*>(hi_p + g * 8) = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
    *reinterpret_cast<uint4*>(lo_p + g * 8) = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
  }
}
hipError_t launch_pack_block(const DevCtx& d, int zbuf, uint16_t* p_hi, uint16_t* p_lo, hipStream_t s) {
  hipLaunchKernelGGL(k_pack_block, dim3(128, d.n), dim3(256), 0, s, d, zbuf, p_hi, p_lo);
  return hipGetLastError();
}
// buffer 0 of the Y pair <- the caller's p x r block (table EXT_DIN): start of the initial projection
__global__ __launch_bounds__(256) void k_y_from_ext(DevCtx d) {
  const MatDev& m = d.mats[blockIdx.y];
  float* y = reinterpret_cast<float*>(d.arena + m.y[0]);
  const float* src = reinterpret_cast<const float*>(ext_ptr(d, EXT_DIN, blockIdx.y));
  const int64_t total = (int64_t)m.p * m.r;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) y[i] = src[i];
}
hipError_t launch_y_from_ext(const DevCtx& d, hipStream_t s) {
  hipLaunchKernelGGL(k_y_from_ext, dim3(128, d.n), dim3(256), 0, s, d);
  return hipGetLastError();
}
hipError_t launch_q_from_y(const DevCtx& d, int ybuf, hipStream_t s) {
  hipLaunchKernelGGL(k_q_from_y, dim3(128, d.n), dim3(256), 0, s, d, ybuf);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// p x q elementwise family (outer step, pseudo-gradient, anchor copy)
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int find_mat(const int64_t* chunk_start, int n, int64_t b) {
  int lo = 0, hi = n;             // invariant: chunk_start[lo] <= b < chunk_start[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (chunk_start[mid] <= b) lo = mid; else hi = mid;
  }
  return lo;
}

// Four consecutive weights at W + i0: fp32, or bf16 storage (values widened exactly on the way in, rounded to
// nearest-even once on the way out; the value an outer step leaves in the anchor is the rounded one, i.e. the stored model).
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2n __attribute__((ext_vector_type(2)));
  const f32x2n v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
template <bool WBF>
__device__ __forceinline__ void load_w4(const void* W, int64_t i0, float (&w)[4]) {
  if constexpr (WBF) {
    const u32x2n t = __builtin_nontemporal_load(reinterpret_cast<const u32x2n*>(reinterpret_cast<const uint16_t*>(W) + i0));
    w[0] = __uint_as_float(t.x << 16); w[1] = __uint_as_float(t.x & 0xffff0000u);
    w[2] = __uint_as_float(t.y << 16); w[3] = __uint_as_float(t.y & 0xffff0000u);
  } else {
    const f32x4n t = ld_stream(reinterpret_cast<const float*>(W) + i0);
    w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
  }
}
// returns the values as stored (rounded for bf16 weights); `cached`: an ordinary store (the consumer reads it right away)
template <bool WBF>
__device__ __forceinline__ f32x4n store_w4(void* W, int64_t i0, f32x4n x, bool cached) {
  if constexpr (WBF) {
    const u32x2n t = {pack2_bf16(x.x, x.y), pack2_bf16(x.z, x.w)};
    u32x2n* dst = reinterpret_cast<u32x2n*>(reinterpret_cast<uint16_t*>(W) + i0);
    if (cached) *dst = t; else __builtin_nontemporal_store(t, dst);
    return f32x4n{__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xffff0000u), __uint_as_float(t.y << 16), __uint_as_float(t.y & 0xffff0000u)};
  } else {
    float* dst = reinterpret_cast<float*>(W) + i0;
    if (cached) *reinterpret_cast<f32x4n*>(dst) = x; else st_stream(dst, x);
    return x;
  }
}
template <bool WBF>
__device__ __forceinline__ float load_w1(const void* W, int64_t i) {
  if constexpr (WBF) return bf2f(reinterpret_cast<const uint16_t*>(W)[i]);
  else return reinterpret_cast<const float*>(W)[i];
}
template <bool WBF>
__device__ __forceinline__ float store_w1(void* W, int64_t i, float x) {
  if constexpr (WBF) {
    const uint32_t h = f2bf(x);
    reinterpret_cast<uint16_t*>(W)[i] = (uint16_t)h;
    return bf2f(h);
  } else {
    reinterpret_cast<float*>(W)[i] = x;
    return x;
  }
}

template <int MODE, bool WBF>   // 0 outer step, 1 export delta, 2 anchor <- W, 3 part of the outer step that does not depend on Delta; WBF: bf16 weights
__global__ __launch_bounds__(256) void k_pq(DevCtx d, const int64_t* __restrict__ chunk_start, OuterArgs a) {
  int64_t b = blockIdx.x;
  int mat = find_mat(chunk_start, d.n, b);
  const MatDev& m = d.mats[mat];
  int64_t total = (int64_t)m.p * m.q;
  int64_t off = (b - chunk_start[mat]) * CHUNK;
  void* W = ext_ptr(d, EXT_W, mat);
  float* anchor = reinterpret_cast<float*>(d.arena + m.anchor);
  float* mom = a.has_mom ? reinterpret_cast<float*>(d.arena + m.mom) : nullptr;
  const float* din = (MODE == 0 && !a.own_delta) ? reinterpret_cast<const float*>(ext_ptr(d, EXT_DIN, mat)) : nullptr;
  float* dout = MODE == 1 ? reinterpret_cast<float*>(ext_ptr(d, EXT_DOUT, mat)) : nullptr;
  bool vec = (total % 4 == 0) && ((reinterpret_cast<uintptr_t>(W) & (WBF ? 7 : 15)) == 0) &&
             (din == nullptr || (reinterpret_cast<uintptr_t>(din) & 15) == 0) &&
             (dout == nullptr || (reinterpret_cast<uintptr_t>(dout) & 15) == 0);
#pragma unroll
  for (int rep = 0; rep < 2; ++rep) {
    int64_t i0 = off + rep * 1024 + threadIdx.x * 4;
    if (i0 >= total) continue;
    float w[4], an[4], dl[4], bb[4];
    int cnt = total - i0 < 4 ? (int)(total - i0) : 4;
    if (vec) {       // every array here is touched once per call and is far larger than the caches: streaming accesses
      f32x4n t;
      if ((MODE != 0 && MODE != 3) || (MODE == 0 && a.own_delta)) load_w4<WBF>(W, i0, w);
      if (MODE != 2) { t = ld_stream(anchor + i0); an[0] = t.x; an[1] = t.y; an[2] = t.z; an[3] = t.w; }
      if (din) { t = ld_stream(din + i0); dl[0] = t.x; dl[1] = t.y; dl[2] = t.z; dl[3] = t.w; }
      if ((MODE == 0 || MODE == 3) && mom) { t = ld_stream(mom + i0); bb[0] = t.x; bb[1] = t.y; bb[2] = t.z; bb[3] = t.w; }
    } else {
      for (int e = 0; e < cnt; ++e) {
        if ((MODE != 0 && MODE != 3) || (MODE == 0 && a.own_delta)) w[e] = load_w1<WBF>(W, i0 + e);
        if (MODE != 2) an[e] = anchor[i0 + e];
        if (din) dl[e] = din[i0 + e];
        if ((MODE == 0 || MODE == 3) && mom) bb[e] = mom[i0 + e];
      }
    }
    float o0[4], o1[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (MODE == 0) {
        float dd = a.own_delta ? an[e] - w[e] : dl[e];
        float step = dd;
        if (mom) {
          float bn = fmaf(a.mu, bb[e], dd);
          o1[e] = bn;
          step = a.nesterov ? fmaf(a.mu, bn, dd) : bn;
        }
        o0[e] = fmaf(-a.lr, step, an[e]);
      } else if (MODE == 1) {
        o0[e] = an[e] - w[e];
      } else if (MODE == 2) {
        o0[e] = w[e];
      } else {
        // outer step with Delta = Q A still to be added by the up-projection kernel:
        // b' = mu b + Delta;  W' = anchor - lr (Delta + mu b') (Nesterov) or anchor - lr b' (heavy ball)
        // => b <- mu b,  W <- anchor - lr mu (mu b)  or  anchor - lr (mu b)
        o0[e] = an[e];
        if (mom) {
          const float bn = a.mu * bb[e];
          o1[e] = bn;
          o0[e] = fmaf(-a.lr, a.nesterov ? a.mu * bn : bn, an[e]);
        }
      }
    }
    if (vec) {
      f32x4n t0 = {o0[0], o0[1], o0[2], o0[3]};
      if (MODE == 0) {
        const f32x4n kept = store_w4<WBF>(W, i0, t0, false);
        st_stream(anchor + i0, kept);                          // the anchor is the model as it is stored
        if (mom) st_stream(mom + i0, f32x4n{o1[0], o1[1], o1[2], o1[3]});
      } else if (MODE == 1) {
        st_stream(dout + i0, t0);
      } else if (MODE == 2) {
        st_stream(anchor + i0, t0);
      } else {             // the up-projection kernel reads both again right away: cacheable stores
        store_w4<WBF>(W, i0, t0, true);
        if (mom) *reinterpret_cast<f32x4n*>(mom + i0) = f32x4n{o1[0], o1[1], o1[2], o1[3]};
      }
    } else {
      for (int e = 0; e < cnt; ++e) {
        if (MODE == 0) { anchor[i0 + e] = store_w1<WBF>(W, i0 + e, o0[e]); if (mom) mom[i0 + e] = o1[e]; }
        else if (MODE == 1) dout[i0 + e] = o0[e];
        else if (MODE == 2) anchor[i0 + e] = o0[e];
        else { store_w1<WBF>(W, i0 + e, o0[e]); if (mom) mom[i0 + e] = o1[e]; }
      }
    }
  }
}

hipError_t launch_outer(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, const OuterArgs& a, hipStream_t s) {
  if (a.w_bf16) hipLaunchKernelGGL((k_pq<0, true>), dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, a);
  else hipLaunchKernelGGL((k_pq<0, false>), dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, a);
  return hipGetLastError();
}
hipError_t launch_outer_base(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, const OuterArgs& a, hipStream_t s) {
  if (a.w_bf16) return hipErrorInvalidValue;       // (the outer step from the up-link buffers is built for fp32 weights)
  hipLaunchKernelGGL((k_pq<3, false>), dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, a);
  return hipGetLastError();
}
hipError_t launch_export_delta(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, bool w_bf16, hipStream_t s) {
  OuterArgs a{};
  if (w_bf16) hipLaunchKernelGGL((k_pq<1, true>), dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, a);
  else hipLaunchKernelGGL((k_pq<1, false>), dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, a);
  return hipGetLastError();
}
hipError_t launch_anchor_from_w(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, bool w_bf16, hipStream_t s) {
  OuterArgs a{};
  if (w_bf16) hipLaunchKernelGGL((k_pq<2, true>), dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, a);
  else hipLaunchKernelGGL((k_pq<2, false>), dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, a);
  return hipGetLastError();
}

// E <- E + scale * G for every matrix (Alg. 2: the projection of the local variant is computed from
// the gradient plus the error buffer; the sum is formed in place in the buffer).
template <bool GF32>
__global__ __launch_bounds__(256) void k_fold_grad(DevCtx d, const int64_t* __restrict__ chunk_start, float scale, int only_tr) {
  const int64_t b = blockIdx.x;
  const int mat = find_mat(chunk_start, d.n, b);
  const MatDev& m = d.mats[mat];
  if (only_tr && !m.tr) return;       // the local step folds for the right-projected matrices only (the others add E in their kernel)
  const int64_t total = (int64_t)m.p * m.q;
  const int64_t off = (b - chunk_start[mat]) * CHUNK;
  float* E = reinterpret_cast<float*>(d.arena + m.err);
  const void* G = ext_ptr(d, EXT_G, mat);
  const bool vec = (total % 4 == 0) && (reinterpret_cast<uintptr_t>(G) & (GF32 ? 15 : 7)) == 0;
#pragma unroll
  for (int rep = 0; rep < 2; ++rep) {
    const int64_t i0 = off + rep * 1024 + threadIdx.x * 4;
    if (i0 >= total) continue;
    if (vec) {
      float g[4];
      if constexpr (GF32) {
        f32x4n t = ld_stream(reinterpret_cast<const float*>(G) + i0);
        g[0] = t.x; g[1] = t.y; g[2] = t.z; g[3] = t.w;
      } else {
        const u32x2n t = __builtin_nontemporal_load(reinterpret_cast<const u32x2n*>(reinterpret_cast<const uint16_t*>(G) + i0));
        g[0] = __uint_as_float(t.x << 16); g[1] = __uint_as_float(t.x & 0xffff0000u);
        g[2] = __uint_as_float(t.y << 16); g[3] = __uint_as_float(t.y & 0xffff0000u);
      }
      f32x4n e = ld_stream(E + i0);
      e.x = fmaf(scale, g[0], e.x); e.y = fmaf(scale, g[1], e.y); e.z = fmaf(scale, g[2], e.z); e.w = fmaf(scale, g[3], e.w);
      st_stream(E + i0, e);
    } else {
      const int cnt = total - i0 < 4 ? (int)(total - i0) : 4;
      for (int e = 0; e < cnt; ++e) {
        float g;
        if constexpr (GF32) g = reinterpret_cast<const float*>(G)[i0 + e];
        else g = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(G)[i0 + e] << 16);
        E[i0 + e] = fmaf(scale, g, E[i0 + e]);
      }
    }
  }
}
hipError_t launch_fold_grad(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, float scale, bool g_is_f32, hipStream_t s, bool only_tr) {
  if (g_is_f32) hipLaunchKernelGGL(k_fold_grad<true>, dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, scale, only_tr ? 1 : 0);
  else hipLaunchKernelGGL(k_fold_grad<false>, dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, scale, only_tr ? 1 : 0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// CholeskyQR helpers
// ---------------------------------------------------------------------------------------
// S_ii += coef * trace(S): keeps the first factorisation positive definite in fp32.
// store: also keep the shift behind the Ritz values (the Rayleigh-Ritz step subtracts it from the eigenvalues).
__global__ __launch_bounds__(256) void k_gram_shift(DevCtx d, float coef, int store) {
  if (mat_skipped(d, blockIdx.x)) return;
  const MatDev& m = d.mats[blockIdx.x];
  float* S = reinterpret_cast<float*>(d.arena + m.gram);
  __shared__ float red[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < m.r; i += 256) acc += S[(int64_t)i * m.r + i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  float shift = coef * red[0];
  for (int i = threadIdx.x; i < m.r; i += 256) S[(int64_t)i * m.r + i] += shift;
  if (store && m.ritz >= 0 && threadIdx.x == 0) reinterpret_cast<float*>(d.arena + m.ritz)[m.r + 2] = shift;
}
// Diagonal of the Gram matrix S = X^T X of a tall block X (rows x r, row-major), summed in double from the fp32
// entries: S_kk = sum_i X_ik^2.  The grouped GEMM forms S from three-term bf16 operands; on the diagonal the product
// of the two middle terms is a square, always positive and about 2^-18 of the entry, and in a long contraction it
// falls below half an ulp of the running sum and is rounded away step after step: the diagonal came out 2e-6 to
// 3e-6 too small at p >= 4096 and the columns of the orthonormalised block that much too long -- 7e-5 in
// || Q^T Q - I ||_F at r = 512.  The diagonal carries the column norms, so it alone is recomputed exactly.
// Two stages, both in a fixed order: workgroup (64 columns, row chunk, matrix) sums its rows (4 row lanes x 64
// columns, eight loads in flight per thread) into the split-K partial-sum buffer of the matrix, which the Gram
// product has just released; one thread per column then adds the chunks and writes the diagonal entry.
// which: 0, 1 = buffers of the Y pair (rows = p); 2, 3 = zw[0], zw[1] (rows = q).
constexpr int GD_CHUNKS = 64;
__device__ __forceinline__ int gram_diag_chunks(const MatDev& m, int part_slices) {
  const int cap = (m.r * part_slices) / 2;              // doubles per column that fit into part_slices * r * r floats
  return cap < 1 ? 1 : (cap < GD_CHUNKS ? cap : GD_CHUNKS);
}
__global__ __launch_bounds__(256) void k_gram_diag_part(DevCtx d, int which, int part_slices) {
  const int mat = blockIdx.z;
  if (mat_skipped(d, mat)) return;
  const MatDev& m = d.mats[mat];
  if ((int)blockIdx.x * 64 >= m.r) return;
  const int nch = gram_diag_chunks(m, part_slices);
  if ((int)blockIdx.y >= nch) return;
  const int k = blockIdx.x * 64 + (threadIdx.x & 63);
  const float* X = reinterpret_cast<const float*>(d.arena + (which < 2 ? m.y[which] : m.zw[which - 2]));
  const int rows = which < 2 ? m.p : m.q;
  const int per = ((rows + nch - 1) / nch + 3) & ~3;
  const int r0 = blockIdx.y * per, r1 = r0 + per < rows ? r0 + per : rows;
  const int lane_row = threadIdx.x >> 6;
  double acc = 0.0;
  if (k < m.r) {
    int i = r0 + lane_row;
    for (; i + 28 < r1; i += 32) {
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = X[(int64_t)(i + 4 * e) * m.r + k];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fma((double)x[e], (double)x[e], acc);
    }
    for (; i < r1; i += 4) {
      const double x = (double)X[(int64_t)i * m.r + k];
      acc = fma(x, x, acc);
    }
  }
  __shared__ double part[4][64];
  part[lane_row][threadIdx.x & 63] = acc;
  __syncthreads();
  if (lane_row == 0 && k < m.r) {
    const int c = threadIdx.x & 63;
    reinterpret_cast<double*>(d.arena + m.part)[(int64_t)blockIdx.y * m.r + k] = (part[0][c] + part[1][c]) + (part[2][c] + part[3][c]);
  }
}
__global__ __launch_bounds__(64) void k_gram_diag_sum(DevCtx d, int part_slices) {
  const int mat = blockIdx.y;
  if (mat_skipped(d, mat)) return;
  const MatDev& m = d.mats[mat];
  const int k = blockIdx.x * 64 + threadIdx.x;
  if (k >= m.r) return;
  const int nch = gram_diag_chunks(m, part_slices);
  const double* part = reinterpret_cast<const double*>(d.arena + m.part);
  double acc = 0.0;
  for (int c = 0; c < nch; ++c) acc += part[(int64_t)c * m.r + k];
  reinterpret_cast<float*>(d.arena + m.gram)[(int64_t)k * m.r + k] = (float)acc;
}
hipError_t launch_gram_diag(const DevCtx& d, int which, int rmax, int part_slices, hipStream_t s) {
  hipLaunchKernelGGL(k_gram_diag_part, dim3((rmax + 63) / 64, GD_CHUNKS, d.n), dim3(256), 0, s, d, which, part_slices);
  hipLaunchKernelGGL(k_gram_diag_sum, dim3((rmax + 63) / 64, d.n), dim3(64), 0, s, d, part_slices);
  return hipGetLastError();
}

// Mean squared singular value of R = Q_new^T Q_old of the last refresh (Sec. 5.1, Metrics):
// (1/r) sum_i sigma_i^2 = ||R||_F^2 / r, from the elementwise square the rotation already keeps.
__global__ __launch_bounds__(256) void k_mssv(DevCtx d, float* __restrict__ out) {
  const MatDev& m = d.mats[blockIdx.x];
  const float* R2 = reinterpret_cast<const float*>(d.arena + m.rot2);
  __shared__ float red[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < m.r * m.r; i += 256) acc += R2[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = red[0] / (float)m.r;
}
hipError_t launch_mssv(const DevCtx& d, float* out, hipStream_t s) {
  hipLaunchKernelGGL(k_mssv, dim3(d.n), dim3(256), 0, s, d, out);
  return hipGetLastError();
}

// Stable rank of the refresh source (Sec. 5.1, Metrics): sr = ||Src||_F^2 / ||Src||_2^2.  The squared Frobenius norm is
// summed here, per workgroup over CHUNK elements and then per matrix over its workgroups, both in a fixed order; the
// spectral norm is the leading Ritz value of the Rayleigh-Ritz step.
template <bool SF32>
__global__ __launch_bounds__(256) void k_frob2_chunks(DevCtx d, const int64_t* __restrict__ chunk_start, float* __restrict__ partial) {
  const int64_t b = blockIdx.x;
  const int mat = find_mat(chunk_start, d.n, b);
  if (mat_skipped(d, mat)) return;
  const MatDev& m = d.mats[mat];
  const int64_t total = (int64_t)m.p * m.q;
  const int64_t off = (b - chunk_start[mat]) * CHUNK;
  const void* S = ext_ptr(d, EXT_SRC, mat);
  float acc = 0.f;
#pragma unroll
  for (int rep = 0; rep < CHUNK / 256; ++rep) {
    const int64_t i = off + rep * 256 + threadIdx.x;
    if (i < total) {
      float x;
      if constexpr (SF32) x = reinterpret_cast<const float*>(S)[i];
      else x = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(S)[i] << 16);
      acc = fmaf(x, x, acc);
    }
  }
  __shared__ float red[256];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[b] = red[0];
}
// one workgroup per matrix: sum of its partial sums in double, stored behind the r Ritz values
__global__ __launch_bounds__(256) void k_frob2_sum(DevCtx d, const int64_t* __restrict__ chunk_start, const float* __restrict__ partial) {
  const MatDev& m = d.mats[blockIdx.x];
  if (m.ritz < 0 || mat_skipped(d, blockIdx.x)) return;
  __shared__ double red[256];
  double acc = 0.0;
  for (int64_t b = chunk_start[blockIdx.x] + threadIdx.x; b < chunk_start[blockIdx.x + 1]; b += 256) acc += (double)partial[b];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) reinterpret_cast<float*>(d.arena + m.ritz)[m.r] = (float)red[0];
}
// which = 0: stable rank ||Src||_F^2 / sigma_1^2;  1: spectral gap sigma_r - sigma_{r+1} (estimates of both)
__global__ void k_stable_rank(DevCtx d, float* __restrict__ out, int which) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d.n) return;
  const MatDev& m = d.mats[i];
  const float* rz = reinterpret_cast<const float*>(d.arena + m.ritz);
  out[i] = which == 0 ? rz[m.r] / (rz[0] * rz[0]) : rz[m.r - 1] - rz[m.r + 1];
}
hipError_t launch_frob2(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, float* partial, bool src_f32, hipStream_t s) {
  if (src_f32) hipLaunchKernelGGL(k_frob2_chunks<true>, dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, partial);
  else hipLaunchKernelGGL(k_frob2_chunks<false>, dim3((unsigned)nchunks), dim3(256), 0, s, d, chunk_start, partial);
  hipLaunchKernelGGL(k_frob2_sum, dim3(d.n), dim3(256), 0, s, d, chunk_start, partial);
  return hipGetLastError();
}
hipError_t launch_stable_rank(const DevCtx& d, float* out, int which, hipStream_t s) {
  hipLaunchKernelGGL(k_stable_rank, dim3((d.n + 63) / 64), dim3(64), 0, s, d, out, which);
  return hipGetLastError();
}

hipError_t launch_gram_shift(const DevCtx& d, float coef, bool store, hipStream_t s) {
  hipLaunchKernelGGL(k_gram_shift, dim3(d.n), dim3(256), 0, s, d, coef, store ? 1 : 0);
  return hipGetLastError();
}

// Diagonal block jb of the Gram matrix: L = chol(S_jj) (lower), X = L^{-1}; writes L into the
// factor and X into the block-inverse array.  One workgroup per matrix.
__device__ __forceinline__ float lane_value(float x, int lane) {      // value of x in lane `lane` (a constant), as a scalar
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane));
}

// One wave per matrix; lane i keeps row i of the 64 x 64 block in 64 registers, so the 64 column
// steps of the factorisation and of the inversion need no barrier and no LDS round trip: a column
// is broadcast lane by lane through scalar registers (v_readlane) and applied with one FMA per
// element.  Everything is unrolled, every register index is a constant.
__global__ __launch_bounds__(256) void k_potf2(DevCtx d, int jb) {
  if (mat_skipped(d, blockIdx.x)) return;
  const MatDev& m = d.mats[blockIdx.x];
  const int o = jb * NB;
  int nbk = m.r - o;
  if (nbk <= 0) return;
  if (nbk > NB) nbk = NB;
  const float* S = reinterpret_cast<const float*>(d.arena + m.gram);
  float* L = reinterpret_cast<float*>(d.arena + m.lfac);
  float* X = reinterpret_cast<float*>(d.arena + m.dinv) + (int64_t)jb * NB * NB;
  static_assert(NB == 64, "four waves of sixteen columns each");
  __shared__ float tile[NB][NB + 1];
  __shared__ __align__(16) float lrow[NB][NB];       // the factor, rows 16-byte aligned: operand of the inversion
  __shared__ __align__(16) float ccol[2][NB];        // column k of the factor with entries <= k zeroed (multipliers of step k)
  __shared__ float crow[2][NB];                      // column k of the factor (every row's own factor)
  __shared__ float red[4];
  __shared__ int bad_s;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  // rows are read coalesced and handed to their lanes through LDS; identity outside the block
  for (int rr = w; rr < NB; rr += 4) {
    float val;
    if (rr < nbk && lane < nbk) val = lane <= rr ? S[(int64_t)(o + rr) * m.r + (o + lane)] : 0.f;
    else val = rr == lane ? 1.f : 0.f;
    tile[rr][lane] = val;
  }
  if (tid == 0) bad_s = 0;
  __syncthreads();
  // lane = row, wave w holds columns 16 w .. 16 w + 15 of it
  float a[16];
#pragma unroll
  for (int jc = 0; jc < 16; ++jc) a[jc] = tile[lane][16 * w + jc];
  float dmax = lane < nbk ? tile[lane][lane] : 0.f;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) dmax = fmaxf(dmax, __shfl_xor(dmax, off));
  const float floor_piv = 1e-12f * dmax + 1e-37f;
  // right-looking Cholesky, one barrier per column: the wave that holds column k scales it and leaves it in LDS (two
  // buffers alternate, so the next column can be written while this one is still being read); every wave then updates
  // its sixteen columns, a[j] -= L[i][k] L[j][k], with the multipliers L[j][k] read as broadcasts (zero for j <= k, which
  // leaves the finished columns alone)
#pragma clang loop unroll(full)
  for (int k = 0; k < NB; ++k) {
    const int buf = k & 1;
    if (w == k / 16) {
      float piv = lane_value(a[k % 16], k);
      if (!(piv > floor_piv)) {
        if (lane == 0) bad_s = 1;
        piv = floor_piv;
      }
      const float dd = sqrtf(piv);
      const float lk = lane == k ? dd : (lane > k ? a[k % 16] / dd : 0.f);
      a[k % 16] = lk;
      crow[buf][lane] = lk;
      ccol[buf][lane] = lane > k ? lk : 0.f;
    }
    __syncthreads();
    if (16 * w + 15 > k) {                           // this wave still has columns to the right of k
      const float mine = crow[buf][lane];
      const f32x4n* cp = reinterpret_cast<const f32x4n*>(&ccol[buf][16 * w]);
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x4n cv = cp[g4];
#pragma unroll
        for (int e = 0; e < 4; ++e) a[4 * g4 + e] = fmaf(-mine, cv[e], a[4 * g4 + e]);
      }
    }
  }
  // the factor to LDS (zeros above the diagonal): for the inversion and for the coalesced store
#pragma unroll
  for (int jc = 0; jc < 16; ++jc) {
    const int j = 16 * w + jc;
    const float v = j <= lane ? a[jc] : 0.f;
    lrow[lane][j] = v;
    tile[lane][j] = v;
  }
  __syncthreads();
  if (w == 0) {
    // X = L^{-1} by forward substitution: lane j builds column j, x[i] = X[i][j]; row i of L is read as broadcasts
    float x[NB];
#pragma clang loop unroll(full)
    for (int i = 0; i < NB; ++i) {
      // four partial sums: the FMA chain of a row is split so that consecutive terms overlap
      float acc[4] = {lane == i ? 1.f : 0.f, 0.f, 0.f, 0.f};
      const f32x4n* lp = reinterpret_cast<const f32x4n*>(&lrow[i][0]);
#pragma clang loop unroll(full)
      for (int g4 = 0; g4 < NB / 4; ++g4) {
        if (4 * g4 < i) {
          const f32x4n lv = lp[g4];
#pragma clang loop unroll(full)
          for (int e = 0; e < 4; ++e)
            if (4 * g4 + e < i) acc[e] = fmaf(-lv[e], x[4 * g4 + e], acc[e]);
        }
      }
      x[i] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) / lrow[i][i];
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) X[i * NB + lane] = lane <= i ? x[i] : 0.f;
  }
  if (tid == 0 && bad_s) *d.flag = 1;
  for (int rr = w; rr < nbk; rr += 4)
    if (lane < nbk) L[(int64_t)(o + rr) * m.r + (o + lane)] = tile[rr][lane];
}
// The inverses of the diagonal blocks, copied to their places on the diagonal of the r x r inverse of the
// whole factor (the rows below are then built from them by products).
__global__ __launch_bounds__(256) void k_diag_inverses(DevCtx d) {
  if (mat_skipped(d, blockIdx.x)) return;
  const MatDev& m = d.mats[blockIdx.x];
  const float* X = reinterpret_cast<const float*>(d.arena + m.dinv);
  float* M = reinterpret_cast<float*>(d.arena + m.minv);
  const int nblocks = (m.r + NB - 1) / NB;
  for (int t = threadIdx.x; t < nblocks * NB * NB; t += 256) {
    const int jb = t / (NB * NB), i = (t / NB) % NB, j = t % NB;
    const int row = jb * NB + i, col = jb * NB + j;
    if (row < m.r && col < m.r) M[(int64_t)row * m.r + col] = X[t];
  }
}
hipError_t launch_diag_inverses(const DevCtx& d, hipStream_t s) {
  hipLaunchKernelGGL(k_diag_inverses, dim3(d.n), dim3(256), 0, s, d);
  return hipGetLastError();
}
hipError_t launch_potf2(const DevCtx& d, int jb, hipStream_t s) {
  hipLaunchKernelGGL(k_potf2, dim3(d.n), dim3(256), 0, s, d, jb);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Rayleigh-Ritz step of the refresh (Sec. 2 ComputeProjection wants Q = the first r columns of U, largest
// singular value first): eigenvectors of the r x r matrix T = (Q^T Src)(Q^T Src)^T, r <= 128, from its Cholesky
// factor: T + shift I = L L^T (the factorisation of the orthonormalisation, with its diagonal shift), and the left
// singular vectors of L are the eigenvectors of T, its singular values s_i give the eigenvalues s_i^2 - shift.
// One-sided Jacobi on the columns of X = L, one workgroup per matrix: a plane rotation of two columns makes them
// orthogonal; at convergence X = U diag(s).  The columns stay in registers for the whole iteration: a group of
// sixteen lanes holds the two columns at positions 2k and 2k + 1 (eight rows of each per lane; n = r rounded up to
// even, the added column is zero and never rotated).  The pairs follow the odd-even transposition order: even steps
// pair positions (2k, 2k + 1) inside a group, odd steps pair (2k + 1, 2k + 2) -- the left column of the next group
// comes over through LDS and the rotated right column goes back -- and every step ends with the two columns of a
// pair changing places, so that in n steps every column has met every other exactly once (one sweep).  Half the
// steps touch no LDS and need no barrier; the other half move one column per group each way.  The three inner
// products of a pair are summed over its sixteen lanes by a butterfly of lane exchanges (both partners of an exchange
// add the same two numbers, so all lanes hold the same bits and take the same decision).  A pair is left alone when
// |x_p . x_q| <= 3e-7 |x_p| |x_q|; the iteration ends with the first sweep that rotates nothing (at most 20).
// Working on the factor instead of T keeps the small singular values accurate relative to themselves (the
// factor has the square root of T's condition number).
// Output: column k of `rot` (r x r row-major) = singular vector of the k-th largest singular value, signed so
// that its entry of largest magnitude is positive; ritz[k] = sqrt(max(s_k^2 - shift, 0)), the Ritz values of Src.
// top_value_only: nothing but the largest Ritz value, to ritz[r + 1] (spectral-gap estimate).
// Reads the lower triangle of `lfac` and the shift the factorisation stored at ritz[r + 2].
// ---------------------------------------------------------------------------------------
__global__ void k_fill_zero_i32(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Sum over the sixteen lanes of a DPP row, the same bits in every lane: four exchange steps (lanes 1 and 2 apart
// inside a quad, then the mirror image inside eight and inside sixteen lanes, which pairs quads and halves whose
// lanes already agree); both partners of an exchange add the same two numbers.
template <int CTRL>
__device__ __forceinline__ float dpp_get(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float sum16(float v) {
  v += dpp_get<0xB1>(v);      // quad_perm [1, 0, 3, 2]
  v += dpp_get<0x4E>(v);      // quad_perm [2, 3, 0, 1]
  v += dpp_get<0x141>(v);     // row_half_mirror
  v += dpp_get<0x140>(v);     // row_mirror
  return v;
}

// Rotation of two columns held in registers (eight rows per lane, sixteen lanes): returns the columns swapped, as the
// odd-even order wants them (p <- rotated q, q <- rotated p), and whether a rotation was applied.
__device__ __forceinline__ bool rotate_swap(float (&p)[8], float (&q)[8]) {
  float a = 0.f, b = 0.f, c = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a = fmaf(p[j], p[j], a);
    b = fmaf(q[j], q[j], b);
    c = fmaf(p[j], q[j], c);
  }
  a = sum16(a);
  b = sum16(b);
  c = sum16(c);
  float cs = 1.f, sn = 0.f;
  const bool rot = fabsf(c) > 3e-7f * __builtin_amdgcn_sqrtf(a * b);            // the same in all sixteen lanes
  if (rot) {
    const float zeta = (b - a) * 0.5f * __builtin_amdgcn_rcpf(c);
    const float t = copysignf(1.f, zeta) * __builtin_amdgcn_rcpf(fabsf(zeta) + __builtin_amdgcn_sqrtf(1.f + zeta * zeta));
    cs = __builtin_amdgcn_rsqf(1.f + t * t);
    sn = t * cs;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float pn = cs * p[j] - sn * q[j], qn = sn * p[j] + cs * q[j];      // cs = 1, sn = 0 leave both as they are
    p[j] = qn;
    q[j] = pn;
  }
  return rot;
}

__global__ __launch_bounds__(1024) void k_jacobi_svd(DevCtx d, int top_value_only) {
  const MatDev m = d.mats[blockIdx.x];
  const int r = m.r;
  if (r > 128 || m.ritz < 0 || mat_skipped(d, blockIdx.x)) return;
  const int n = (r + 1) & ~1;
  const int ld = n + 1;
  const int half = n / 2;
  extern __shared__ float jsm[];
  float* X = jsm;                         // n x ld: the columns at the end, for the ordering and the output
  float* nrm2 = X + n * ld;               // n
  float* ex = nrm2 + n;                   // half x EXLD: the column that crosses to the neighbouring group
  constexpr int EXLD = 129;               // all 128 register rows of a column are exchanged, whatever n is
  __shared__ int rotated;
  const int tid = threadIdx.x, nt = blockDim.x;
  const float* L = reinterpret_cast<const float*>(d.arena + m.lfac);
  float* rz = reinterpret_cast<float*>(d.arena + m.ritz);

  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k = wave * 4 + (lane >> 4);              // this group of sixteen lanes holds positions 2k and 2k + 1
  const int gl = lane & 15;
  const bool act = k < half;
  constexpr int ROWS = 8;                            // 16 lanes x 8 rows = 128 >= n
  float pl[ROWS], pr[ROWS];                          // the columns at positions 2k (left) and 2k + 1 (right)
#pragma unroll
  for (int j = 0; j < ROWS; ++j) {
    const int row = gl + 16 * j, c0 = 2 * k, c1 = 2 * k + 1;
    pl[j] = (act && row < r && c0 <= row) ? L[(int64_t)row * r + c0] : 0.f;      // lower triangle; c0 <= row < r
    pr[j] = (act && row < r && c1 <= row) ? L[(int64_t)row * r + c1] : 0.f;
  }
  if (tid == 0) rotated = 0;
  __syncthreads();

  for (int sweep = 0; sweep < 20; ++sweep) {
    for (int step = 0; step < n; ++step) {
      if ((step & 1) == 0) {
        // positions (2k, 2k + 1): both columns are here
        if (act && rotate_swap(pl, pr) && gl == 0) rotated = 1;                  // benign race: every writer stores 1
      } else {
        // positions (2k + 1, 2k + 2): the left column of the next group comes over, the rotated right column goes back
        if (act && k >= 1) {
#pragma unroll
          for (int j = 0; j < ROWS; ++j) ex[k * EXLD + gl + 16 * j] = pl[j];
        }
        __syncthreads();
        if (act && k + 1 < half) {
          float t[ROWS];
#pragma unroll
          for (int j = 0; j < ROWS; ++j) t[j] = ex[(k + 1) * EXLD + gl + 16 * j];
          if (rotate_swap(pr, t) && gl == 0) rotated = 1;
#pragma unroll
          for (int j = 0; j < ROWS; ++j) ex[(k + 1) * EXLD + gl + 16 * j] = t[j];
        }
        __syncthreads();
        if (act && k >= 1) {
#pragma unroll
          for (int j = 0; j < ROWS; ++j) pl[j] = ex[k * EXLD + gl + 16 * j];
        }
      }
    }
    __syncthreads();                                 // n is even: the last step of a sweep ends with a barrier anyway
    const int any = rotated;
    __syncthreads();
    if (tid == 0) rotated = 0;
    __syncthreads();
    if (!any) break;
  }
  if (act) {
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
      const int row = gl + 16 * j;
      if (row < n) {
        X[row * ld + 2 * k] = pl[j];
        X[row * ld + 2 * k + 1] = pr[j];
      }
    }
  }
  __syncthreads();

  // squared column norms = squared singular values; the columns have travelled, the zero column added for an odd rank
  // is wherever it ended up and has norm zero (the shift keeps every other norm positive)
  for (int i = tid; i < n; i += nt) {
    float acc = 0.f;
    for (int row = 0; row < n; ++row) acc = fmaf(X[row * ld + i], X[row * ld + i], acc);
    nrm2[i] = acc;
  }
  __syncthreads();
  const float shift = rz[r + 2];
  if (top_value_only) {
    if (tid == 0) {
      float mx = 0.f;
      for (int i = 0; i < n; ++i) mx = fmaxf(mx, nrm2[i]);
      rz[r + 1] = sqrtf(fmaxf(mx - shift, 0.f));
      if (!(mx <= 3.0e38f)) *d.flag = 1;
    }
    return;
  }
  // descending order (ties by position); one thread per singular vector writes its column
  for (int i = tid; i < n; i += nt) {
    const float li = nrm2[i];
    if (!(li <= 3.0e38f)) *d.flag = 1;               // NaN or infinity in the factor
    if (!(li > 0.f)) continue;                       // the added zero column
    int rank = 0;
    for (int j = 0; j < n; ++j) rank += (nrm2[j] > li || (nrm2[j] == li && j < i)) ? 1 : 0;
    if (rank >= r) continue;
    float best = 0.f, bestv = 1.f;
    for (int row = 0; row < r; ++row) {
      const float v = X[row * ld + i];
      if (fabsf(v) > best) { best = fabsf(v); bestv = v; }
    }
    const float scale = (bestv < 0.f ? -1.f : 1.f) / sqrtf(li);
    float* U = reinterpret_cast<float*>(d.arena + m.rot);
    for (int row = 0; row < r; ++row) U[(int64_t)row * r + rank] = scale * X[row * ld + i];
    rz[rank] = sqrtf(fmaxf(li - shift, 0.f));
  }
}
size_t jacobi_lds_bytes(int rmax) {
  const int n = (rmax + 1) & ~1;
  return sizeof(float) * ((size_t)n * (n + 1) + n + (size_t)(n / 2) * 129);
}
hipError_t launch_jacobi_svd(const DevCtx& d, int rmax, bool top_value_only, hipStream_t s) {
  if (rmax > 128) return hipErrorInvalidValue;
  const size_t lds = jacobi_lds_bytes(rmax);
  static LdsRaised raised;
  if (hipError_t e = raise_lds(reinterpret_cast<const void*>(k_jacobi_svd), (int)jacobi_lds_bytes(128), raised); e != hipSuccess) return e;
  const int threads = rmax > 64 ? 1024 : (rmax > 32 ? 512 : 256);
  hipLaunchKernelGGL(k_jacobi_svd, dim3(d.n), dim3(threads), lds, s, d, top_value_only ? 1 : 0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// The same one-sided Jacobi for ranks above 128 (up to 1024), where the factor does not fit into LDS, in blocked
// form: the columns of L live as contiguous rows of an r x r buffer in device memory (the Gram buffer, which the
// factorisation has consumed) and are cut into blocks of BW columns; the round-robin order runs over pairs of blocks,
// one kernel launch is one outer round, one workgroup takes one pair of blocks of one matrix and sweeps once over all
// pairs of its 2 BW columns in LDS.  The barrier between outer rounds is the kernel boundary.  Convergence is tracked
// on the device: the rotations of outer sweep s are counted in flag[s]; the launches of sweep s + 1 return at once when
// that count is below a small allowance, so the host enqueues a fixed number of sweeps without reading anything back.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_jsvd_init(DevCtx d) {
  const MatDev& m = d.mats[blockIdx.y];
  if (m.ritz < 0 || mat_skipped(d, blockIdx.y)) return;
  const int r = m.r;
  const float* L = reinterpret_cast<const float*>(d.arena + m.lfac);
  float* Xt = reinterpret_cast<float*>(d.arena + m.gram);
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < (int64_t)r * r; idx += (int64_t)gridDim.x * 256) {
    const int c = (int)(idx / r), row = (int)(idx - (int64_t)c * r);
    Xt[idx] = row >= c ? L[(int64_t)row * r + c] : 0.f;       // column c of L
  }
}
// One outer round: workgroup (kb, matrix) takes the pair of column blocks (bi, bj) that the round-robin order gives
// for block-pair slot kb, brings their 2 BW columns into LDS (one column contiguous, so a pair's lanes read
// consecutive addresses), runs one full cyclic sweep over all pairs of these columns there (2 BW - 1 rounds of BW
// pairs, 32 lanes per pair, one barrier per round) and writes the columns back.
// CH: 16-byte chunks per lane and column, i.e. the LDS pitch of a column is 128 CH rows for every matrix of the launch
// (rows past a matrix's rank are zero); a compile-time count lets all loads of a pair be issued before the first wait.
template <int BW, int CH>
__global__ __launch_bounds__(BW * 32) void k_jsvd_block(DevCtx d, int oround, int sweep, int* __restrict__ flags, int allow) {
  if (sweep > 0 && flags[sweep - 1] <= allow) return;         // the previous sweep rotated (next to) nothing: converged
  const MatDev& m = d.mats[blockIdx.y];
  if (m.ritz < 0 || mat_skipped(d, blockIdx.y)) return;
  const int r = m.r;
  const int nb = (r + BW - 1) / BW, nbe = (nb + 1) & ~1, mmb = nbe - 1;
  const int kb = blockIdx.x;
  if (kb >= nbe / 2 || oround >= mmb) return;
  int bi, bj;
  {
    const int a0 = (oround + kb) % mmb, b0 = kb == 0 ? mmb : (oround + mmb - kb) % mmb;
    bi = a0 < b0 ? a0 : b0; bj = a0 < b0 ? b0 : a0;
  }
  if (bi >= nb) return;                                       // (bj may be the added empty block)
  constexpr int NL = 2 * BW;                                  // local columns
  constexpr int pitch = 128 * CH;                             // a lane takes four consecutive rows with one 16-byte access
  extern __shared__ f32x4n jsm16[];                           // 16-byte aligned, also behind the static variable below
  float* Xl = reinterpret_cast<float*>(jsm16);                // NL x pitch
  float* Xt = reinterpret_cast<float*>(d.arena + m.gram);
  const int tid = threadIdx.x, nt = BW * 32;
  auto gcol = [&](int lc) { return lc < BW ? bi * BW + lc : bj * BW + (lc - BW); };
  for (int idx = tid; idx < NL * pitch; idx += nt) {
    const int lc = idx / pitch, row = idx - lc * pitch;
    const int gc = gcol(lc);
    Xl[idx] = (gc < r && row < r) ? Xt[(int64_t)gc * r + row] : 0.f;
  }
  __syncthreads();
  const int slot = tid >> 5, l32 = tid & 31;                  // local pair slot, lane within the pair
  int nrot = 0;
  // rounding of an inner product of r terms grows with sqrt(r): so does the level below which a pair counts as orthogonal
  const float tol = 3e-7f * fmaxf(1.f, __builtin_amdgcn_sqrtf((float)r * (1.f / 128.f)));
  __shared__ int wg_rot;
  if (tid == 0) wg_rot = 0;
  for (int inner = 0; inner < NL - 1; ++inner) {
    const int a0 = (inner + slot) % (NL - 1), b0 = slot == 0 ? NL - 1 : (inner + NL - 1 - slot) % (NL - 1);
    f32x4n* xpp = reinterpret_cast<f32x4n*>(Xl + (a0 < b0 ? a0 : b0) * pitch) + l32;
    f32x4n* xqq = reinterpret_cast<f32x4n*>(Xl + (a0 < b0 ? b0 : a0) * pitch) + l32;
    f32x4n xp[CH], xq[CH];
    float a = 0.f, b = 0.f, c = 0.f;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      xp[j] = xpp[32 * j];
      xq[j] = xqq[32 * j];
    }
#pragma unroll
    for (int j = 0; j < CH; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        a = fmaf(xp[j][e], xp[j][e], a);
        b = fmaf(xq[j][e], xq[j][e], b);
        c = fmaf(xp[j][e], xq[j][e], c);
      }
    a = sum16(a); b = sum16(b); c = sum16(c);
    a += __shfl_xor(a, 16); b += __shfl_xor(b, 16); c += __shfl_xor(c, 16);      // same bits in all 32 lanes
    if (fabsf(c) > tol * __builtin_amdgcn_sqrtf(a * b)) {
      const float zeta = (b - a) * 0.5f * __builtin_amdgcn_rcpf(c);
      const float t = copysignf(1.f, zeta) * __builtin_amdgcn_rcpf(fabsf(zeta) + __builtin_amdgcn_sqrtf(1.f + zeta * zeta));
      const float cs = __builtin_amdgcn_rsqf(1.f + t * t);
      const float sn = t * cs;
#pragma unroll
      for (int j = 0; j < CH; ++j) {
        xpp[32 * j] = cs * xp[j] - sn * xq[j];
        xqq[32 * j] = sn * xp[j] + cs * xq[j];
      }
      ++nrot;
    }
    __syncthreads();                                          // the pairs of the next round take other columns
  }
  for (int idx = tid; idx < NL * pitch; idx += nt) {
    const int lc = idx / pitch, row = idx - lc * pitch;
    const int gc = gcol(lc);
    if (gc < r && row < r) Xt[(int64_t)gc * r + row] = Xl[idx];
  }
  // rotations of the sweep, counted over all matrices (integer sums: the order of the additions does not matter)
  if (l32 == 0 && nrot) atomicAdd(&wg_rot, nrot);
  __syncthreads();
  if (tid == 0 && wg_rot) atomicAdd(&flags[sweep], wg_rot);
}
// squared column norms, order, signs, output: one workgroup per matrix (as the tail of k_jacobi_svd)
__global__ __launch_bounds__(256) void k_jsvd_finish(DevCtx d, int top_value_only) {
  const MatDev& m = d.mats[blockIdx.x];
  if (m.ritz < 0 || mat_skipped(d, blockIdx.x)) return;
  const int r = m.r;
  const float* Xt = reinterpret_cast<const float*>(d.arena + m.gram);
  float* rz = reinterpret_cast<float*>(d.arena + m.ritz);
  __shared__ float nrm2[1024];
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  for (int cidx = wave; cidx < r; cidx += 4) {                // one wave per column: fixed order of the sum
    float acc = 0.f;
    for (int e = lane; e < r; e += 64) acc = fmaf(Xt[(int64_t)cidx * r + e], Xt[(int64_t)cidx * r + e], acc);
    acc = sum16(acc);
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if (lane == 0) nrm2[cidx] = acc;
  }
  __syncthreads();
  const float shift = rz[r + 2];
  if (top_value_only) {
    if (tid == 0) {
      float mx = 0.f;
      for (int i = 0; i < r; ++i) mx = fmaxf(mx, nrm2[i]);
      rz[r + 1] = sqrtf(fmaxf(mx - shift, 0.f));
      if (!(mx <= 3.0e38f)) *d.flag = 1;
    }
    return;
  }
  float* U = reinterpret_cast<float*>(d.arena + m.rot);
  for (int i = tid; i < r; i += 256) {
    const float li = nrm2[i];
    int rank = 0;
    for (int j = 0; j < r; ++j) rank += (nrm2[j] > li || (nrm2[j] == li && j < i)) ? 1 : 0;
    float best = 0.f, bestv = 1.f;
    for (int row = 0; row < r; ++row) {
      const float v = Xt[(int64_t)i * r + row];
      if (fabsf(v) > best) { best = fabsf(v); bestv = v; }
    }
    const float scale = (bestv < 0.f ? -1.f : 1.f) * (li > 0.f ? 1.f / sqrtf(li) : 0.f);
    for (int row = 0; row < r; ++row) U[(int64_t)row * r + rank] = scale * Xt[(int64_t)i * r + row];
    rz[rank] = sqrtf(fmaxf(li - shift, 0.f));
    if (!(li <= 3.0e38f)) *d.flag = 1;
  }
}
template <int BW, int CH>
static hipError_t jsvd_block_sweeps(const DevCtx& d, int rmax, int* flags, int sweeps, int allow, hipStream_t s) {
  constexpr size_t lds = sizeof(float) * 2 * BW * 128 * CH;
  static_assert(lds <= 147456, "two blocks of columns must fit into LDS");
  static LdsRaised raised;
  if (hipError_t e = raise_lds(reinterpret_cast<const void*>(k_jsvd_block<BW, CH>), (int)lds, raised); e != hipSuccess) return e;
  if (rmax > 128 * CH) return hipErrorInvalidValue;
  const int nb = (rmax + BW - 1) / BW, nbe = (nb + 1) & ~1;
  for (int sweep = 0; sweep < sweeps; ++sweep)
    for (int oround = 0; oround < nbe - 1; ++oround)
      hipLaunchKernelGGL((k_jsvd_block<BW, CH>), dim3(nbe / 2, d.n), dim3(BW * 32), lds, s, d, oround, sweep, flags, allow);
  return hipGetLastError();
}
hipError_t launch_jacobi_svd_blocked(const DevCtx& d, int rmax, int64_t rank_sq_sum, bool top_value_only, int* flags, hipStream_t s) {
  if (rmax > 1024) return hipErrorInvalidValue;
  constexpr int SWEEPS = 14;                                  // flags holds 16 ints
  hipLaunchKernelGGL(k_fill_zero_i32, dim3(1), dim3(64), 0, s, flags, 16);
  hipLaunchKernelGGL(k_jsvd_init, dim3(64, d.n), dim3(256), 0, s, d);
  // two blocks of columns must fit into LDS: 32 columns each up to rank 512, 16 beyond; column pitch 256, 512 or 1024 rows
  // a sweep visits about r^2 / 2 pairs per matrix (more: pairs inside a block come up again with every partner block);
  // it counts as converged when fewer than one in 8192 of them still rotates (by angles of the size of the rounding)
  const int allow = (int)std::min<int64_t>(rank_sq_sum >> 14, 1 << 30);
  hipError_t e = rmax <= 256 ? jsvd_block_sweeps<32, 2>(d, rmax, flags, SWEEPS, allow, s)
               : rmax <= 512 ? jsvd_block_sweeps<32, 4>(d, rmax, flags, SWEEPS, allow, s)
                             : jsvd_block_sweeps<16, 8>(d, rmax, flags, SWEEPS, allow, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_jsvd_finish, dim3(d.n), dim3(256), 0, s, d, top_value_only ? 1 : 0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// moment rotation, elementwise parts.  Plain temporaries are q x r row-major (the transposes of
// the paper's r x q arrays): zw[2] = u_hat^T, zw[3] = (v_hat - u_hat^2)^T; the two GEMMs leave
// zw[0] = (R u_hat)^T and zw[1] = ((R o R)(v_hat - u_hat^2))^T.
// ---------------------------------------------------------------------------------------
// Both kernels move eight consecutive rank indices of one column per thread, as two 16-byte accesses
// where r % 4 == 0.  k_rot_pre numbers its threads so that eight neighbours hold eight consecutive
// octets of one column: their writes to the plain temporaries form one 256-byte run (the blocked
// side is then read in 32-byte pieces, which costs far less than scattered partial-line writes).
// k_rot_post keeps the flat numbering: its writes go to the blocked arrays, contiguous over threads.
__global__ __launch_bounds__(256) void k_rot_pre(DevCtx d, const float* __restrict__ u, const float* __restrict__ v,
                                                 const StepDev* __restrict__ step) {
  if (mat_skipped(d, blockIdx.y)) return;
  const float inv_c1 = step->inv_c1, inv_c2 = step->inv_c2;
  const MatDev& m = d.mats[blockIdx.y];
  float* uh = reinterpret_cast<float*>(d.arena + m.zw[2]);
  float* var = reinterpret_cast<float*>(d.arena + m.zw[3]);
  const int64_t octets = m.rp / 8;                     // rank octets per column; a multiple of 4
  const int64_t ngroups = (int64_t)m.qp * octets;
  const bool vec = (m.r & 3) == 0;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < ngroups; t += (int64_t)gridDim.x * 256) {
    // t = (column * octets/4 + octet quad) * 4 + octet in quad: four neighbours share a column
    const int64_t j = t / octets, i8 = t % octets;
    if (j >= m.q || i8 * 8 >= m.r) continue;
    const int64_t src = m.lr_off + (((j >> 5) * octets + i8) * 32 + (j & 31)) * 8;
    const f32x4n u0 = *reinterpret_cast<const f32x4n*>(u + src), u1 = *reinterpret_cast<const f32x4n*>(u + src + 4);
    const f32x4n v0 = *reinterpret_cast<const f32x4n*>(v + src), v1 = *reinterpret_cast<const f32x4n*>(v + src + 4);
    const f32x4n a0 = u0 * inv_c1, a1 = u1 * inv_c1;
    const f32x4n b0 = v0 * inv_c2 - a0 * a0, b1 = v1 * inv_c2 - a1 * a1;
    const int64_t dst = j * m.r + i8 * 8;
    if (vec && i8 * 8 + 8 <= m.r) {
      *reinterpret_cast<f32x4n*>(uh + dst) = a0;  *reinterpret_cast<f32x4n*>(uh + dst + 4) = a1;
      *reinterpret_cast<f32x4n*>(var + dst) = b0; *reinterpret_cast<f32x4n*>(var + dst + 4) = b1;
    } else {
      for (int e = 0; e < 8 && i8 * 8 + e < m.r; ++e) {
        uh[dst + e] = e < 4 ? a0[e] : a1[e - 4];
        var[dst + e] = e < 4 ? b0[e] : b1[e - 4];
      }
    }
  }
}
hipError_t launch_rot_pre(const DevCtx& d, const float* u, const float* v, const StepDev* step, hipStream_t s) {
  hipLaunchKernelGGL(k_rot_pre, dim3(256, d.n), dim3(256), 0, s, d, u, v, step);
  return hipGetLastError();
}
__global__ __launch_bounds__(256) void k_rot_post(DevCtx d, float* __restrict__ u, float* __restrict__ v, const StepDev* __restrict__ step) {
  const float c1 = step->c1, c2 = step->c2;
  if (*d.flag != 0 || mat_skipped(d, blockIdx.y)) return;       // a breakdown is latched: the moments stay in the coordinates of the projection that stays
  const MatDev& m = d.mats[blockIdx.y];
  const float* a1 = reinterpret_cast<const float*>(d.arena + m.zw[0]);
  const float* a2 = reinterpret_cast<const float*>(d.arena + m.zw[1]);
  int64_t ngroups = (int64_t)m.qp * m.rp / 8;
  int64_t per_jb = (int64_t)(m.rp / 8) * 32;
  const bool vec = (m.r & 3) == 0;
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < ngroups; g += (int64_t)gridDim.x * 256) {
    int64_t jb = g / per_jb, rem = g % per_jb;
    int64_t i8 = rem / 32, j = jb * 32 + rem % 32;
    f32x4n ru[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, rv[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    if (j < m.q && i8 * 8 < m.r) {
      const int64_t src = j * m.r + i8 * 8;
      if (vec && i8 * 8 + 8 <= m.r) {
        ru[0] = *reinterpret_cast<const f32x4n*>(a1 + src); ru[1] = *reinterpret_cast<const f32x4n*>(a1 + src + 4);
        rv[0] = *reinterpret_cast<const f32x4n*>(a2 + src); rv[1] = *reinterpret_cast<const f32x4n*>(a2 + src + 4);
      } else {
        for (int e = 0; e < 8 && i8 * 8 + e < m.r; ++e) { ru[e >> 2][e & 3] = a1[src + e]; rv[e >> 2][e & 3] = a2[src + e]; }
      }
    }
    // R u = c1 * R u_hat;  v = c2 | (R o R)(v_hat - u_hat^2) + (R u_hat)^2 |; zero in the padding
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      f32x4n un = ru[h] * c1, vn;
#pragma unroll
      for (int e = 0; e < 4; ++e) vn[e] = c2 * fabsf(rv[h][e] + ru[h][e] * ru[h][e]);
      *reinterpret_cast<f32x4n*>(u + m.lr_off + g * 8 + 4 * h) = un;
      *reinterpret_cast<f32x4n*>(v + m.lr_off + g * 8 + 4 * h) = vn;
    }
  }
}
hipError_t launch_rot_post(const DevCtx& d, float* u, float* v, const StepDev* step, hipStream_t s) {
  hipLaunchKernelGGL(k_rot_post, dim3(256, d.n), dim3(256), 0, s, d, u, v, step);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// state exchange: blocked low-rank arrays <-> plain r x q row-major
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_lr_to_plain(DevCtx d, int mat, const float* lr_arr, const uint16_t* n_hi,
                                                     const uint16_t* n_lo, float* dst, int nsplit, int64_t stride) {
  const MatDev& m = d.mats[mat];
  int64_t total = (int64_t)m.r * m.q;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    int64_t i = t / m.q, j = t % m.q;
    int64_t src = m.lr_off + bl_index(j, i, m.rp);
    if (lr_arr) {
      float acc = lr_arr[src];
      for (int sp = 1; sp < nsplit; ++sp) acc += lr_arr[src + sp * stride];   // same order as the Adam kernel
      dst[t] = acc;
    } else {
      dst[t] = bf2f(n_hi[src]) + bf2f(n_lo[src]);
    }
  }
}
hipError_t launch_lr_to_plain(const DevCtx& d, int mat, const float* lr_arr, const uint16_t* n_hi, const uint16_t* n_lo,
                              float* dst, int nsplit, int64_t stride, hipStream_t s) {
  hipLaunchKernelGGL(k_lr_to_plain, dim3(256), dim3(256), 0, s, d, mat, lr_arr, n_hi, n_lo, dst, nsplit, stride);
  return hipGetLastError();
}
__global__ __launch_bounds__(256) void k_plain_to_lr(DevCtx d, int mat, float* lr_arr, const float* src) {
  const MatDev& m = d.mats[mat];
  int64_t total = (int64_t)m.r * m.q;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    int64_t i = t / m.q, j = t % m.q;
    lr_arr[m.lr_off + bl_index(j, i, m.rp)] = src[t];
  }
}
hipError_t launch_plain_to_lr(const DevCtx& d, int mat, float* lr_arr, const float* src, hipStream_t s) {
  hipLaunchKernelGGL(k_plain_to_lr, dim3(256), dim3(256), 0, s, d, mat, lr_arr, src);
  return hipGetLastError();
}

// All matrices at once, plain r x q buffers from the caller's pointer tables (up-link buffer exchange):
// TO_PLAIN: table EXT_DOUT <- lr_arr;  else lr_arr <- table EXT_DIN.  Padded positions are not touched.
template <bool TO_PLAIN>
__global__ __launch_bounds__(256) void k_lr_exchange(DevCtx d, float* lr_arr) {
  const int mat = blockIdx.y;
  const MatDev& m = d.mats[mat];
  float* ext = reinterpret_cast<float*>(ext_ptr(d, TO_PLAIN ? EXT_DOUT : EXT_DIN, mat));
  const int64_t total = (int64_t)m.r * m.q;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t i = t / m.q, j = t % m.q;
    const int64_t at = m.lr_off + bl_index(j, i, m.rp);
    if (TO_PLAIN) ext[t] = lr_arr[at];
    else lr_arr[at] = ext[t];
  }
}
hipError_t launch_lr_exchange(const DevCtx& d, float* lr_arr, bool to_plain, hipStream_t s) {
  if (to_plain) hipLaunchKernelGGL(k_lr_exchange<true>, dim3(64, d.n), dim3(256), 0, s, d, lr_arr);
  else hipLaunchKernelGGL(k_lr_exchange<false>, dim3(64, d.n), dim3(256), 0, s, d, lr_arr);
  return hipGetLastError();
}

// Right-projected matrices (m.tr): their down-projection leaves g^T as the plain q x r block zw[0] (q = rows of the caller's
// matrix); the Adam kernel reads slice 0 of the blocked array g.  `scale` is the caller's gradient scale where the product
// was formed from the raw gradient.
__global__ __launch_bounds__(256) void k_tr_exchange(DevCtx d, float* glow, float scale, int all) {
  const int mat = blockIdx.y;
  const MatDev& m = d.mats[mat];
  if (!m.tr && !all) return;      // all: the product of every matrix was formed as a plain block (fp32 gradients)
  const float* plain = reinterpret_cast<const float*>(d.arena + m.zw[0]);
  // in the order of the blocked array (contiguous writes; the reads are 32-byte pieces of rows that neighbouring threads
  // complete); padded columns and ranks are written as zeros
  const int64_t total = (int64_t)m.qp * m.rp;
  const int64_t per_jb = (int64_t)m.rp * 32;
  for (int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (int64_t)gridDim.x * 256) {
    const int64_t jb = o / per_jb, rem = o % per_jb;
    const int64_t j = jb * 32 + ((rem >> 3) & 31), i = (rem >> 8) * 8 + (rem & 7);      // column j of the low-rank state, rank index i
    glow[m.lr_off + o] = (j < m.q && i < m.r) ? scale * plain[j * m.r + i] : 0.f;
  }
}
// ---------------------------------------------------------------------------------------
// Gaussian start blocks drawn on the device (Alg. 1 Require: a random initial projection; the start block of the
// range finder when the caller supplies none).  Counter-based: element e (row-major index in the block) of matrix
// `mat` in draw number `draw` of a context seeded with `seed` is output e % 4 of
//   Philox-4x32-10(counter = (e / 4 low, e / 4 high, mat, draw), key = (seed low, seed high))      (Salmon et al., SC 2011)
// turned into standard normals two at a time by the Box-Muller transform: u = (x >> 8 + 0.5) 2^-24 in (0, 1),
// (z0, z1) = sqrt(-2 ln u0) (cos 2 pi u1, sin 2 pi u1) from outputs (0, 1), (z2, z3) likewise from outputs (2, 3).
// A float64 reference of the same generator reproduces the block to fp32 rounding of ln / cos / sin.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c[0]), lo0 = 0xD2511F53u * c[0];
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c[2]), lo1 = 0xCD9E8D57u * c[2];
    const uint32_t n0 = hi1 ^ c[1] ^ k0, n2 = hi0 ^ c[3] ^ k1;
    c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
}
// which = 0: buffer 0 of the Y pair (p x r: the block of an initial projection); 1: zw[3] (q x r: a start block Omega)
__global__ __launch_bounds__(256) void k_gauss_block(DevCtx d, int which, uint64_t seed, uint32_t draw) {
  const int mat = blockIdx.y;
  if (mat_skipped(d, mat)) return;
  const MatDev& m = d.mats[mat];
  float* dst = reinterpret_cast<float*>(d.arena + (which == 0 ? m.y[0] : m.zw[3]));
  const int64_t total = (int64_t)(which == 0 ? m.p : m.q) * m.r;
  const int64_t nquads = (total + 3) / 4;
  for (int64_t qd = (int64_t)blockIdx.x * 256 + threadIdx.x; qd < nquads; qd += (int64_t)gridDim.x * 256) {
    uint32_t c[4] = {(uint32_t)qd, (uint32_t)((uint64_t)qd >> 32), (uint32_t)mat, draw};
    philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
    float z[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const float u0 = ((float)(c[2 * h] >> 8) + 0.5f) * 5.9604644775390625e-8f;
      const float u1 = ((float)(c[2 * h + 1] >> 8) + 0.5f) * 5.9604644775390625e-8f;
      const float rad = sqrtf(-2.f * logf(u0));
      const float ang = 6.283185307179586f * u1;
      z[2 * h] = rad * cosf(ang);
      z[2 * h + 1] = rad * sinf(ang);
    }
    for (int e = 0; e < 4 && qd * 4 + e < total; ++e) dst[qd * 4 + e] = z[e];
  }
}
hipError_t launch_gauss_block(const DevCtx& d, int which, uint64_t seed, uint32_t draw, hipStream_t s) {
  hipLaunchKernelGGL(k_gauss_block, dim3(128, d.n), dim3(256), 0, s, d, which, seed, draw);
  return hipGetLastError();
}

hipError_t launch_tr_exchange(const DevCtx& d, float* glow, float scale, bool all, hipStream_t s) {
  hipLaunchKernelGGL(k_tr_exchange, dim3(64, d.n), dim3(256), 0, s, d, glow, scale, all ? 1 : 0);
  return hipGetLastError();
}

}  // namespace lordo
