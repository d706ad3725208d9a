// Shared host/device definitions of the LoRDO gfx950 library: packed layouts, per-matrix
// device records, GEMM descriptors and the launchers each translation unit exports.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lordo {

// ---------------------------------------------------------------------------------------
// Blocked operand layout ("BL").  A logical matrix X[m][k], m < Mp, k < Kp (both padded to a
// multiple of 32 with zeros) is stored so that the 32 x 16 operand fragment of one
// v_mfma_f32_32x32x16_bf16 -- lane l holds X[32*mb + l%32][16*ks + 8*(l/32) + 0..7] -- is one
// contiguous run in lane order:
//     index(m, k) = (((m/32) * (Kp/8) + k/8) * 32 + m%32) * 8 + k%8
// The same indexing holds the fp32 low-rank state (g, u, v) with m = column j of the weight
// matrix and k = rank index i, so that the flat position of a state element equals the flat
// position of its entry in the bf16 operand planes of N.
// ---------------------------------------------------------------------------------------
__host__ __device__ inline int64_t bl_index(int64_t m, int64_t k, int64_t Kp) {
  return (((m >> 5) * (Kp >> 3) + (k >> 3)) * 32 + (m & 31)) * 8 + (k & 7);
}
__host__ __device__ inline int64_t pad32(int64_t x) { return (x + 31) & ~int64_t(31); }

enum ExtTable : int32_t {       // per-call tables of caller pointers, one entry per matrix
  EXT_NONE = -1, EXT_W = 0, EXT_G = 1, EXT_SRC = 2, EXT_OMEGA = 3, EXT_DIN = 4, EXT_DOUT = 5, EXT_COUNT = 6
};

// Per-matrix record in device memory.  Offsets are in BYTES from the arena base unless noted.
struct MatDev {
  int32_t p, q, r, pp, qp, rp;
  int32_t tr, pad_;       // tr = 1: projection on the right (Sec. 2 projects the rows; the short side is the usual choice for tall matrices):
                          // p, q are the dimensions of the TRANSPOSE of the caller's row-major matrix, on which the method runs unchanged
  int64_t q32;            // fp32 p x r plain projection
  int64_t qa_hi, qa_lo;   // bf16 BL(m = row of W, k = rank)      : A operand of the up-projection
  int64_t qt_hi, qt_lo;   // bf16 BL(m = rank, k = row of W)      : A operand of the down-projection
  int64_t lr_off;         // ELEMENT offset of this matrix in the flat low-rank arrays (g, u, v, N)
  int64_t anchor, mom;    // fp32 p x q plain (mom = -1 if no outer momentum)
  // refresh workspace
  int64_t y[2];           // fp32 p x r, ping-pong of the orthonormalisation
  int64_t zw[4];          // fp32 q x r; zw[0], zw[1] ping-pong of the q-side block, all four rotation temporaries
  int64_t gram, lfac;     // fp32 r x r : Gram matrix (consumed by the factorisation) and its Cholesky factor
  int64_t dinv;           // fp32 ceil(r/NB) blocks of NB x NB : inverses of the diagonal blocks of the factor
  int64_t minv;           // fp32 r x r : inverse of the whole factor, lower triangular (zeros above the diagonal are never written)
  int64_t rot, rot2;      // fp32 r x r : R = Q_new^T Q_old and its elementwise square
  int64_t part;           // fp32 split-K partial sums of the r x r products (Gram, R): slices x r x r
  int64_t err;            // fp32 p x q error-feedback residual E (-1 without error feedback)
  int64_t ritz;           // fp32 r + 3 : Ritz values of the last refresh, ||Src||_F^2, estimate of sigma_{r+1}, shift of the
                          // last factorisation of a Ritz matrix (-1 without the Rayleigh-Ritz step)
};

// Work item of the projection kernels.
struct ProjTile {
  int32_t mat;
  int32_t m0;             // first row of the output tile (down: rank index; up: row of W)
  int32_t n0;             // first column of the tile (column of W)
  int32_t k0, k1;         // contraction range (down: rows of W; up: unused)
  int32_t split;          // split-K slice index of the output (down)
  int32_t fuse;           // down: the tile holds the whole contraction and applies Adam to its state elements
  int32_t pad1;
};

// Operand reference of the generic GEMM: arena offset, or caller pointer from table `ext`.
struct OpRef {
  int64_t off;            // bytes (added to the arena base, or to the caller pointer)
  int32_t ext;            // ExtTable
  int32_t pad;
};

// C[M x N] = alpha * A[M x K] * B[K x N] + beta * C, fp32 accumulate.
// A(m, k) at A + m*sAm + k*sAk, B(k, n) at B + k*sBk + n*sBn (element strides), C row-major ldc.
struct GemmDesc {
  OpRef A, B, C, C2;      // C2 (off < 0 = none) receives the elementwise square of the result
  int32_t M, N, K, mat;
  int64_t sAm, sAk, sBk, sBn;
  int32_t ldc, a_bf16, b_bf16;        // a_bf16: 0 fp32, 1 bf16, 2 = element type given at launch (refresh source)
  int32_t prec;                       // 0: fp32 matrix cores; 1: operands split into bf16 hi + lo (range-finder products)
  float alpha, beta;
  // split-K (ksplit > 1): slice s covers k in [s*klen, (s+1)*klen) and writes its raw M x N sum to
  // P + s*M*N; a reduction kernel then adds the slices in order and applies alpha, beta, C2
  int32_t ksplit, klen;
  OpRef P;
  int32_t tri, pad_;      // tri = 1: B(k, n) = 0 for k > n (transposed lower-triangular factor): the contraction of a column tile ends at its last column
};

struct GemmTile { int32_t desc; int16_t tm, tn; int16_t ks, pad; };

// Device-side view handed to kernels.
constexpr int EXT_SLOTS = 8;     // cached pointer tables per kind (e.g. alternating gradient buffers)

struct DevCtx {
  char* arena;
  const MatDev* mats;
  void* const* ext;       // EXT_COUNT * EXT_SLOTS tables of n pointers each
  int32_t n;
  int32_t* flag;          // numerical breakdown latch
  int32_t slot[EXT_COUNT];  // table (absolute index) each kind uses in this launch
  int32_t skip_null;        // 1: the source table of this refresh has NULL entries; those matrices are left as they are
};

__device__ __forceinline__ void* ext_ptr(const DevCtx& d, int table, int mat) {
  return d.ext[(int64_t)d.slot[table] * d.n + mat];
}

// A refresh may leave matrices out (NULL entry in the caller's source table): every kernel of the refresh program
// returns at once for such a matrix, so its projection, moments and scratch are not touched.  Uniform per workgroup.
__device__ __forceinline__ bool mat_skipped(const DevCtx& d, int mat) {
  return d.skip_null != 0 && ext_ptr(d, EXT_SRC, mat) == nullptr;
}

constexpr int CHUNK = 2048;       // elements per workgroup of the p x q elementwise kernels
constexpr int NB = 64;            // Cholesky / triangular-solve block size

// ---------------------------------------------------------------------------------------
// launchers (each defined in one .hip file)
// ---------------------------------------------------------------------------------------
// proj.hip
struct DownFuse;     // below: state arrays and coefficients of the Adam update fused into the down-projection
hipError_t launch_proj_down(const DevCtx& d, const ProjTile* tiles, int ntiles, int mb, int pipe_rb, bool g_vec, bool g_tr, bool g_once, float* glow,
                            int64_t split_stride, float grad_scale, bool g_is_f32, int ef, const DownFuse* fuse, hipStream_t s);
// Epilogue of the up-projection: target <- target + coef_acc * (Q B) + coef_g * G * c_j
struct UpArgs {
  float coef_acc;         // -eta (plain), -eta*omega (full-rank QHM), -1 (error-feedback residual)
  float coef_g;           // 0 (plain), -eta*(1-omega)*grad_scale (full-rank QHM), grad_scale (residual)
  int32_t target_err;     // 0: the caller's W; 1: the residual E kept in the arena; 2: the outer momentum b
  int32_t colscale;       // 1: c_j = 1 / mean over the rank of sqrt(v_hat) + eps (full-rank QHM); 0: c_j = 1
  int32_t g_is_f32;       // element type of G
  float eps;
  const float* colpart;   // column sums left by the Adam kernel (colscale == 1)
  // outer step from the up-link buffers: target W, coef_acc = -eta_s, B = averaged buffer; the epilogue reads the
  // anchor instead of W and also writes the anchor and the momentum b
  int32_t outer, nesterov, has_mom;
  float mu;
  int32_t w_bf16;         // the caller's W is bf16 storage (target W only; the plain update)
};
hipError_t launch_proj_up(const DevCtx& d, const ProjTile* tiles, int ntiles, bool vec, const uint16_t* b_hi,
                          const uint16_t* b_lo, const UpArgs& ua, hipStream_t s);
// plain update with 256 x 128 tiles (ranks from 256 up, 16-byte row accesses); `tiles` hold m0 in steps of 256
hipError_t launch_proj_up_wide(const DevCtx& d, const ProjTile* tiles, int ntiles, const uint16_t* b_hi, const uint16_t* b_lo,
                               const UpArgs& ua, hipStream_t s);
// gemm32.hip
hipError_t launch_gemm32(const DevCtx& d, const GemmDesc* descs, const GemmTile* tiles, int ntiles, int tile, int src_is_bf16,
                         hipStream_t s, float alpha_mul = 1.f);   // alpha_mul scales every product of the launch (per-call coefficients)
hipError_t launch_gemm_reduce(const DevCtx& d, const GemmDesc* descs, int ndescs, hipStream_t s);
// elementwise.hip
// Elements at flat position >= grp_start[i] are the sum of grp_nsplit[i] split-K slices of g.
// Step count and the bias corrections 1 - beta^t derived from it (Sec. 2), kept in device memory and advanced by a
// kernel at the head of every local step: a local step recorded into a HIP graph then counts its REPLAYS, which
// values passed as kernel arguments could not.
struct StepDev {
  int64_t t;
  float inv_c1, inv_c2;   // 1 / (1 - beta1^t), 1 / (1 - beta2^t); 1 without bias correction
  float c1, c2;
};
hipError_t launch_step(StepDev* sd, double beta1, double beta2, int bias_correction, int64_t set_to, hipStream_t s);

struct AdamArgs {
  float b1, omb1, b2, omb2, eps;
  const StepDev* step;    // bias corrections of the current step
  int32_t grp_nsplit[4];
  int64_t grp_start[4];
  int64_t split_stride;
  int64_t first;          // flat position of the first element the stand-alone kernel updates
  float qw, qg;           // update bracket (qw * u_hat + qg * g) / den: 1, 0 without low-rank QHM; omega, 1 - omega with it
  float* colpart;         // full-rank QHM: per column and rank block of 32, sum of sqrt(v_hat) + eps (else null)
  uint16_t* g_hi;         // error feedback: bf16 hi / lo operand planes of the summed g (else null)
  uint16_t* g_lo;
  float* acc;             // up-link buffer (App. A.5.1): acc += lr * N every step (else null)
  float lr;
};
struct DownFuse {
  float* u;
  float* v;
  uint16_t* n_hi;
  uint16_t* n_lo;
  AdamArgs a;
};
hipError_t launch_adam(const float* glow, float* u, float* v, uint16_t* n_hi, uint16_t* n_lo, int64_t nelem,
                       const AdamArgs& a, hipStream_t s);
hipError_t launch_store_ptrs(void** dst, void* const* host_src, int count, hipStream_t s);
hipError_t launch_pack_q(const DevCtx& d, int mat_first, int mat_count, hipStream_t s);
hipError_t launch_identity_q(const DevCtx& d, hipStream_t s);
hipError_t launch_fill_zero(void* dst, int64_t bytes, hipStream_t s);
hipError_t launch_bf16_to_f32(float* dst, const uint16_t* src, int64_t n, hipStream_t s);      // exact widening
hipError_t launch_f32_to_bf16(uint16_t* dst, const float* src, int64_t n, hipStream_t s);      // round to nearest-even
hipError_t launch_copy_f32(float* dst, const float* src, int64_t n, hipStream_t s);
// p x q elementwise family: chunk_start (device) has n+1 entries, prefix sums of per-matrix chunk counts
struct OuterArgs { float lr, mu; int32_t nesterov, has_mom, own_delta, w_bf16; };
hipError_t launch_outer(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, const OuterArgs& a, hipStream_t s);
hipError_t launch_outer_base(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, const OuterArgs& a, hipStream_t s);
hipError_t launch_split_planes(const float* src, uint16_t* p_hi, uint16_t* p_lo, int64_t nelem, hipStream_t s);
hipError_t launch_export_delta(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, bool w_bf16, hipStream_t s);
hipError_t launch_anchor_from_w(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, bool w_bf16, hipStream_t s);
hipError_t launch_fold_grad(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, float scale, bool g_is_f32, hipStream_t s, bool only_tr = false);
// refresh helpers (grouped over all matrices)
hipError_t launch_gram_shift(const DevCtx& d, float coef, bool store, hipStream_t s);
// exact diagonal of the Gram matrix of block `which` (0, 1: Y pair; 2, 3: zw[0], zw[1]) written over the one the GEMM left
hipError_t launch_gram_diag(const DevCtx& d, int which, int rmax, int part_slices, hipStream_t s);
hipError_t launch_mssv(const DevCtx& d, float* out, hipStream_t s);
hipError_t launch_potf2(const DevCtx& d, int jb, hipStream_t s);
hipError_t launch_frob2(const DevCtx& d, const int64_t* chunk_start, int64_t nchunks, float* partial, bool src_f32, hipStream_t s);
hipError_t launch_stable_rank(const DevCtx& d, float* out, int which, hipStream_t s);
hipError_t launch_jacobi_svd(const DevCtx& d, int rmax, bool top_value_only, hipStream_t s);
hipError_t launch_jacobi_svd_blocked(const DevCtx& d, int rmax, int64_t rank_sq_sum, bool top_value_only, int* flags, hipStream_t s);
hipError_t launch_diag_inverses(const DevCtx& d, hipStream_t s);
hipError_t launch_rot_pre(const DevCtx& d, const float* u, const float* v, const StepDev* step, hipStream_t s);
hipError_t launch_rot_post(const DevCtx& d, float* u, float* v, const StepDev* step, hipStream_t s);
hipError_t launch_q_from_y(const DevCtx& d, int ybuf, hipStream_t s);
hipError_t launch_y_from_ext(const DevCtx& d, hipStream_t s);
hipError_t launch_pack_y(const DevCtx& d, int ybuf, hipStream_t s);
hipError_t launch_pack_block(const DevCtx& d, int zbuf, uint16_t* p_hi, uint16_t* p_lo, hipStream_t s);
hipError_t launch_src_times_block(const DevCtx& d, const ProjTile* tiles, int ntiles, const uint16_t* b_hi, const uint16_t* b_lo,
                                  hipStream_t s);
hipError_t launch_glow_to_z(const DevCtx& d, const float* glow, int zbuf, const AdamArgs& a, hipStream_t s);
// state exchange with plain row-major buffers (one matrix)
hipError_t launch_lr_to_plain(const DevCtx& d, int mat, const float* lr_arr, const uint16_t* n_hi, const uint16_t* n_lo,
                              float* dst, int nsplit, int64_t stride, hipStream_t s);
hipError_t launch_plain_to_lr(const DevCtx& d, int mat, float* lr_arr, const float* src, hipStream_t s);
hipError_t launch_lr_exchange(const DevCtx& d, float* lr_arr, bool to_plain, hipStream_t s);
// right-projected matrices only: slice 0 of the blocked array g <- scale * (plain rows x r block in zw[0])
hipError_t launch_tr_exchange(const DevCtx& d, float* glow, float scale, bool all, hipStream_t s);
// Gaussian block of every matrix from the counter-based generator: which = 0 into y[0] (p x r), 1 into zw[3] (q x r)
hipError_t launch_gauss_block(const DevCtx& d, int which, uint64_t seed, uint32_t draw, hipStream_t s);

// Dynamic LDS beyond 64 KiB has to be allowed per kernel, and the permission belongs to the device the kernel is loaded
// on: asked for once per (kernel, device), on the first launch there.
constexpr int MAX_LDS_DEVICES = 64;
struct LdsRaised { bool done[MAX_LDS_DEVICES] = {}; };
inline hipError_t raise_lds(const void* kernel, int bytes, LdsRaised& st) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < MAX_LDS_DEVICES;
  if (tracked && st.done[dev]) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return e;
  if (tracked) st.done[dev] = true;
  return hipSuccess;
}

}  // namespace lordo
