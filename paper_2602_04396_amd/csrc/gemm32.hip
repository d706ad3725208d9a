// Grouped fp32 GEMM on the fp32 matrix cores (v_mfma_f32_32x32x2_f32) for the subspace refresh:
// range-finder products, Gram matrices, blocked Cholesky / triangular solves and the moment
// rotation.  One launch runs a list of independent problems (one per weight matrix); a tile
// table maps each workgroup to (problem, tile).  Operands are addressed by element strides, so
// any transpose and the bf16 gradient type are handled by the loader; accumulation is fp32.
#include "common.h"

namespace lordo {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int TK = 16;

__device__ __forceinline__ float load_elem(const char* base, int64_t idx, int is_bf16) {
  if (is_bf16) {
    uint32_t h = reinterpret_cast<const uint16_t*>(base)[idx];
    return __uint_as_float(h << 16);
  }
  return reinterpret_cast<const float*>(base)[idx];
}

__device__ __forceinline__ const char* resolve(const DevCtx& d, const OpRef& r, int mat) {
  if (r.ext >= 0) return reinterpret_cast<const char*>(ext_ptr(d, r.ext, mat)) + r.off;
  return d.arena + r.off;
}

// 256 threads = 4 waves in a 2 x 2 grid; each wave WB x WB accumulator blocks of 32 x 32, so the
// workgroup tile is 64*WB square (64 for small problems, 128 where both output sides reach 128).
template <int WB>
__global__ __launch_bounds__(256) void k_gemm32(DevCtx d, const GemmDesc* __restrict__ descs,
                                                const GemmTile* __restrict__ tiles, int src_is_bf16) {
  constexpr int TM = 64 * WB, TN = 64 * WB;
  constexpr int PITCH = TM + 4;
  constexpr int PER_THREAD = TM * TK / 256;
  const GemmTile t = tiles[blockIdx.x];
  const GemmDesc g = descs[t.desc];
  const int M = g.M, N = g.N;
  const int kbeg = g.ksplit > 1 ? t.ks * g.klen : 0;
  const int K = g.ksplit > 1 ? (kbeg + g.klen < g.K ? kbeg + g.klen : g.K) : g.K;     // end of this slice
  const int m0 = t.tm * TM, n0 = t.tn * TN;
  const int a_bf16 = g.a_bf16 == 2 ? src_is_bf16 : g.a_bf16;
  const char* A = resolve(d, g.A, g.mat);
  const char* B = resolve(d, g.B, g.mat);
  float* C = reinterpret_cast<float*>(const_cast<char*>(resolve(d, g.C, g.mat)));
  float* C2 = g.C2.off >= 0 ? reinterpret_cast<float*>(const_cast<char*>(resolve(d, g.C2, g.mat))) : nullptr;

  __shared__ float As[TK][PITCH];
  __shared__ float Bs[TK][PITCH];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = (wave & 1) * 32 * WB, wn = (wave >> 1) * 32 * WB;

  // loader mapping: the unit-stride direction of each operand varies fastest across threads
  const bool a_kfast = g.sAk == 1 && g.sAm != 1;
  const bool b_kfast = g.sBk == 1 && g.sBn != 1;

  f32x16 acc[WB][WB];
#pragma unroll
  for (int a = 0; a < WB; ++a)
#pragma unroll
    for (int b = 0; b < WB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  for (int k0 = kbeg; k0 < K; k0 += TK) {
    float ra[PER_THREAD], rb[PER_THREAD];
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      int idx = tid + i * 256;                 // 0 .. TM*TK-1
      int mm, kk;
      if (a_kfast) { kk = idx % TK; mm = idx / TK; } else { mm = idx % TM; kk = idx / TM; }
      int gm = m0 + mm, gk = k0 + kk;
      ra[i] = (gm < M && gk < K) ? load_elem(A, (int64_t)gm * g.sAm + (int64_t)gk * g.sAk, a_bf16) : 0.f;
      int nn, kb;
      if (b_kfast) { kb = idx % TK; nn = idx / TK; } else { nn = idx % TN; kb = idx / TN; }
      int gn = n0 + nn, gkb = k0 + kb;
      rb[i] = (gn < N && gkb < K) ? load_elem(B, (int64_t)gkb * g.sBk + (int64_t)gn * g.sBn, g.b_bf16) : 0.f;
    }
    __syncthreads();                           // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      int idx = tid + i * 256;
      int mm, kk;
      if (a_kfast) { kk = idx % TK; mm = idx / TK; } else { mm = idx % TM; kk = idx / TM; }
      As[kk][mm] = ra[i];
      int nn, kb;
      if (b_kfast) { kb = idx % TK; nn = idx / TK; } else { nn = idx % TN; kb = idx / TN; }
      Bs[kb][nn] = rb[i];
    }
    __syncthreads();
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
          float val = g.alpha * acc[a][b][v];
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
  if (g.ksplit <= 1) return;
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
                         hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  if (tile == 128) hipLaunchKernelGGL((k_gemm32<2>), dim3(ntiles), dim3(256), 0, s, d, descs, tiles, src_is_bf16);
  else hipLaunchKernelGGL((k_gemm32<1>), dim3(ntiles), dim3(256), 0, s, d, descs, tiles, src_is_bf16);
  return hipGetLastError();
}

}  // namespace lordo
