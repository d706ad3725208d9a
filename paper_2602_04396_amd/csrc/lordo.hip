// C ABI of the LoRDO library: arena planning, static launch plans and the entry points.
// Everything that depends only on the shapes (tile tables, GEMM descriptors of the refresh,
// per-matrix records) is built once in lordo_init and kept in the caller's arena; the entry
// points then only enqueue kernels.
#include "../../include/lordo.h"
#include "common.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

using namespace lordo;

namespace {

#define HIPCHK(expr)                                                                              \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) {                                                                       \
      fprintf(stderr, "lordo: %s failed: %s (%s:%d)\n", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return LORDO_EHIP;                                                                          \
    }                                                                                             \
  } while (0)

enum OpKind : int { OP_GEMM, OP_SHIFT, OP_POTF2, OP_DIAG_INV, OP_ROT_PRE, OP_ROT_POST, OP_Q_FROM_Y, OP_PACK, OP_Y_FROM_EXT, OP_JSVD, OP_FROB, OP_GRAM_DIAG };

struct Op {
  int kind;
  int tile_first = 0, ntiles = 0;   // OP_GEMM
  int tile = 64;                    // OP_GEMM: workgroup tile edge (64 or 128)
  int desc_first = 0, ndescs = 0;   // OP_GEMM: descriptors of this launch
  bool split = false;               // OP_GEMM: split-K launch, followed by the slice reduction
  int iarg = 0;                     // OP_POTF2: block index; OP_Q_FROM_Y: y buffer
  float farg = 0.f;                 // OP_SHIFT: coefficient
  bool rot_only = false;            // part of the moment rotation (skipped while t == 0)
  int fast = 0;                     // OP_GEMM: 1 = the product Z = Src^T Y, which the down-projection kernel can take over (iarg: y buffer);
                                    // 2 = a product Y = Src B for the source-streaming kernel (iarg: z buffer of B, -1 = Omega)
};

struct Plan {
  int part_slices = 1;              // K slices the split-K partial buffers are sized for
  size_t bytes = 0;
  int64_t lr_total = 0;             // elements of one flat low-rank array
  int64_t nchunks = 0;
  int mb = 4;
  int up_waves = 4;                 // waves per workgroup of the up-projection (4: 64 x 64 wave tiles, 8: 32 x 64)
  int r_max = 0;                    // largest rank of any matrix
  int64_t rank_sq_sum = 0;          // sum of r^2 over the matrices
  int64_t frob_part = -1;           // per-chunk partial sums of ||Src||_F^2 (Rayleigh-Ritz option)
  int64_t jflags = -1;              // per-sweep "something rotated" flags of the multi-launch Jacobi solver
  int down_pipe = 0;                // pipelined down-projection: rank blocks per wave (1: 128-rank tiles, 2: 256-rank), 0: plain kernel
  int rank_tile = 128;              // rank indices per down-projection tile
  bool g_once = true;               // every matrix has one rank tile of the down-projection: G is read exactly once
  int64_t colpart = -1, g_hi = -1, g_lo = -1;   // full-rank QHM column sums; error-feedback planes of g
  int64_t acc = -1;                 // up-link buffer: flat low-rank array, sum over the window of lr * N
  int64_t adam_first = 0;           // flat position from which the stand-alone Adam kernel runs (elements before it are fused)
  int nsplit = 1;                   // largest split-K factor of the down-projection
  std::vector<int> splits;          // split-K factor per matrix (1, 2, 4 or 8)
  int32_t grp_nsplit[4] = {1, 1, 1, 1};
  int64_t grp_start[4] = {0, INT64_MAX, INT64_MAX, INT64_MAX};
  // global regions (byte offsets)
  int64_t flag, step, mats, ext, chunk_start, down_tiles, up_tiles, descs, gtiles, glow, u, v, n_hi, n_lo;
  std::vector<MatDev> mat;
  std::vector<int64_t> chunk_start_h;
  std::vector<ProjTile> down_h, up_h, ytile_h;       // ytile: 128 rows x 128 ranks tiles of the products Y = Src B
  std::vector<ProjTile> up_wide_h;                   // 256 x 128 tiles of the plain update (every left-projected rank >= 256)
  int64_t up_wide_tiles = -1;
  int64_t ytiles = 0;
  bool y_fast_shapes = false;       // every matrix has q % 32 == 0 and r % 4 == 0
  std::vector<GemmDesc> desc_h;
  std::vector<GemmTile> gtile_h;
  std::vector<Op> ops;              // the refresh
  std::vector<Op> init_ops;         // Q_0 from a caller-supplied block: copy, orthonormalise, pack
  std::vector<Op> gap_ops;          // estimate of sigma_{r+1} of a source (Rayleigh-Ritz option)
  bool any_tr = false;              // some matrix is projected on the right
  bool down_generic = false;        // fp32 gradients: the down-projection of EVERY matrix runs in the grouped GEMM (three-term operands)
  std::vector<Op> tr_down_ops;      // their product g^T = G Q by the generic GEMM (fp32 gradients, shapes the streaming kernel does not take)
  // Right-projected matrices in the kernels of the left projection: the products of the step are those of the caller's
  // p x q matrix with the operand planes in exchanged roles (see build_plan), described by two shadow tables of MatDev.
  std::vector<MatDev> mat_up, mat_stb, mat_up_ef;    // mat_up_ef: the planes of g in the place of N (error-feedback residual)
  std::vector<Op> tr_down_ef_ops;                    // g^T = (s G + E) Q from the folded residual, by the generic GEMM
  int64_t mats_up = -1, mats_stb = -1, mats_up_ef = -1, up_tr_tiles = -1, ytile_tr = -1;
  std::vector<ProjTile> up_tr_h, ytile_tr_h;
  int64_t tr_plane_gap = 0;         // bytes from a hi plane of such a matrix to its lo plane (the same for all of them)
  bool tr_stream_shapes = false;    // every right-projected matrix has cols % 32 == 0 and r % 4 == 0
};

constexpr int MAX_KSPLIT = 16;

// Launch shape of the r x r products with a long contraction, taken over all matrices: workgroup
// tile edge and the number of K slices that brings the launch to about 1024 workgroups.
static int small_out_split(const MatDev* mats, int n, int* tile_out) {
  int64_t t128 = 0, t64 = 0;
  bool big_ok = true;
  for (int i = 0; i < n; ++i) {
    const int r = mats[i].r;
    if (r < 128) big_ok = false;
    t128 += (int64_t)((r + 127) / 128) * ((r + 127) / 128);
    t64 += (int64_t)((r + 63) / 64) * ((r + 63) / 64);
  }
  const bool big = big_ok;           // r x r outputs with r >= 128: 128-wide tiles read the tall operand half as often
  if (tile_out) *tile_out = big ? 128 : 64;
  const int64_t tiles = big ? t128 : t64;
  if (tiles <= 0 || tiles >= 1024) return 1;
  return (int)std::min<int64_t>(MAX_KSPLIT, (1024 + tiles - 1) / tiles);
}

struct Alloc {
  size_t cur = 0;
  int64_t take(size_t bytes) {
    size_t o = cur;
    cur += (bytes + 255) & ~size_t(255);
    return (int64_t)o;
  }
};

OpRef ref_arena(int64_t off) { return OpRef{off, EXT_NONE, 0}; }
OpRef ref_ext(int table, int64_t off = 0) { return OpRef{off, table, 0}; }
OpRef ref_none() { return OpRef{-1, EXT_NONE, 0}; }

// Workgroups are handed to the 8 XCDs round-robin by index.  Placing logical tile
// (b % 8) * ceil(T/8) + b / 8 at index b gives each XCD, and so each L2, a contiguous run of
// logical tiles, which share operand planes.  Holes are marked mat = -1.
std::vector<ProjTile> xcd_order(const std::vector<ProjTile>& logical) {
  size_t T = logical.size();
  size_t per = (T + 7) / 8;
  std::vector<ProjTile> out(per * 8);
  for (size_t b = 0; b < per * 8; ++b) {
    size_t l = (b % 8) * per + b / 8;
    if (l < T) out[b] = logical[l];
    else { ProjTile h{}; h.mat = -1; out[b] = h; }
  }
  return out;
}

struct ProgramBuilder {
  Plan& P;
  int n;
  explicit ProgramBuilder(Plan& p, int n_) : P(p), n(n_) {}

  // One grouped GEMM launch.  `small_out` marks r x r products with a long contraction (Gram matrix,
  // rotation matrix): with few output tiles they are split along K so that the chip is filled.
  template <class F>
  void gemm(F make, bool rot_only = false, bool small_out = false, bool lower_only = false) {   // make(i, desc) -> false to skip matrix i
    Op op;
    op.kind = OP_GEMM;
    op.tile_first = (int)P.gtile_h.size();
    op.rot_only = rot_only;
    std::vector<GemmDesc> made;
    int64_t tiles128 = 0, tiles64 = 0;
    bool big_ok = true;
    for (int i = 0; i < n; ++i) {
      GemmDesc g{};
      g.C2 = ref_none();
      g.P = ref_none();
      g.alpha = 1.f;
      g.beta = 0.f;
      g.mat = i;
      g.ksplit = 1;
      // every product of the program runs on the bf16 matrix cores with operands split into three terms
      // (as exact as fp32, and faster than the fp32 matrix-core path from r = 256 up); the kernel falls back
      // to fp32 matrix cores for operands it cannot read with 16-byte accesses
      g.prec = 1;
      if (!make(i, g)) continue;
      if (g.M <= 0 || g.N <= 0 || g.K <= 0) continue;
      if (g.M < 128 || g.N < 128) big_ok = false;
      tiles128 += (int64_t)((g.M + 127) / 128) * ((g.N + 127) / 128);
      tiles64 += (int64_t)((g.M + 63) / 64) * ((g.N + 63) / 64);
      made.push_back(g);
    }
    op.tile = (big_ok && (tiles128 >= 512 || small_out)) ? 128 : 64;
    const int64_t tiles = op.tile == 128 ? tiles128 : tiles64;
    int ksplit = 1;
    if (small_out && tiles > 0 && tiles < 1024)
      ksplit = (int)std::min<int64_t>(P.part_slices, (1024 + tiles - 1) / tiles);     // never more slices than allocated
    op.desc_first = (int)P.desc_h.size();
    for (GemmDesc g : made) {
      int ks = ksplit;
      int klen = ((g.K + ks - 1) / ks + 31) / 32 * 32;
      ks = (g.K + klen - 1) / klen;
      if (ks > 1) {
        g.ksplit = ks;
        g.klen = klen;
        g.P = ref_arena(P.mat[g.mat].part);
        op.split = true;
      }
      int di = (int)P.desc_h.size();
      P.desc_h.push_back(g);
      for (int sl = 0; sl < g.ksplit; ++sl)
        for (int tm = 0; tm < (g.M + op.tile - 1) / op.tile; ++tm)
          for (int tn = 0; tn < (g.N + op.tile - 1) / op.tile; ++tn) {
            if (lower_only && tn > tm) continue;      // symmetric result of which only the lower triangle is read
            P.gtile_h.push_back(GemmTile{di, (int16_t)tm, (int16_t)tn, (int16_t)sl, 0});
          }
    }
    op.ndescs = (int)P.desc_h.size() - op.desc_first;
    op.ntiles = (int)P.gtile_h.size() - op.tile_first;
    P.ops.push_back(op);
  }
  // A operand = the source (transposed: its transpose).  The source of a right-projected matrix is the caller's
  // row-major array read as its transpose: element (i, j) of the p x q matrix at j * p + i.
  static void src_operand(GemmDesc& g, const MatDev& m, bool transposed) {
    g.A = ref_ext(EXT_SRC); g.a_bf16 = 2; g.prec = 1;
    const int64_t s_row = m.tr ? 1 : m.q, s_col = m.tr ? m.p : 1;
    g.sAm = transposed ? s_col : s_row;
    g.sAk = transposed ? s_row : s_col;
  }
  void simple(int kind, int iarg = 0, float farg = 0.f, bool rot_only = false) {
    Op op;
    op.kind = kind;
    op.iarg = iarg;
    op.farg = farg;
    op.rot_only = rot_only;
    P.ops.push_back(op);
  }

  // Cholesky factor of the Gram matrix of every matrix, block column by block column (NB-wide: diagonal block by
  // k_potf2, two grouped GEMMs for the panel and the trailing update); the Gram buffer is consumed, the factor
  // goes to its own buffer, the inverses of the diagonal blocks to theirs.
  int max_blocks_all() const {
    int mb = 0;
    for (int i = 0; i < n; ++i) mb = std::max(mb, (P.mat[i].r + NB - 1) / NB);
    return mb;
  }
  void factor(int max_blocks) {
    for (int jb = 0; jb < max_blocks; ++jb) {
      simple(OP_POTF2, jb);
      // L_21 = S_21 L_11^{-T}
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        int rest = m.r - (jb + 1) * NB;
        if (rest <= 0) return false;
        int64_t o = ((int64_t)(jb + 1) * NB * m.r + (int64_t)jb * NB) * 4;
        g.A = ref_arena(m.gram + o); g.sAm = m.r; g.sAk = 1;
        g.B = ref_arena(m.dinv + (int64_t)jb * NB * NB * 4); g.sBk = 1; g.sBn = NB;
        g.C = ref_arena(m.lfac + o); g.ldc = m.r;
        g.M = rest; g.N = NB; g.K = NB;
        return true;
      });
      // S_22 -= L_21 L_21^T
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        int rest = m.r - (jb + 1) * NB;
        if (rest <= 0) return false;
        int64_t o = ((int64_t)(jb + 1) * NB * m.r + (int64_t)jb * NB) * 4;
        g.A = ref_arena(m.lfac + o); g.sAm = m.r; g.sAk = 1;
        g.B = ref_arena(m.lfac + o); g.sBk = 1; g.sBn = m.r;
        g.C = ref_arena(m.gram + ((int64_t)(jb + 1) * NB * m.r + (int64_t)(jb + 1) * NB) * 4); g.ldc = m.r;
        g.M = rest; g.N = rest; g.K = NB;
        g.alpha = -1.f; g.beta = 1.f;
        return true;
      });
    }
  }

  // Thin QR of the block held in buffer `cur` of the pair selected by `buf` (rows = p or q),
  // by `passes` rounds of CholeskyQR; returns the buffer index that holds the result.
  // The first `nshift` passes add the diagonal shift to their Gram matrix: such a pass cannot break down and divides the
  // condition number of the block by about 700; a pass without the shift needs a condition number below about 2000.
  int orth(bool y_side, int cur, int passes, int nshift = 1) {
    auto buf_of = [&](int i, int which) { return y_side ? P.mat[i].y[which] : P.mat[i].zw[which]; };
    auto rows_of = [&](int i) { return y_side ? P.mat[i].p : P.mat[i].q; };
    int max_blocks = 0;
    for (int i = 0; i < n; ++i) max_blocks = std::max(max_blocks, (P.mat[i].r + NB - 1) / NB);
    for (int pass = 0; pass < passes; ++pass) {
      // S = X^T X
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        g.A = ref_arena(buf_of(i, cur)); g.sAm = 1; g.sAk = m.r;
        g.B = ref_arena(buf_of(i, cur)); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.gram); g.ldc = m.r;
        g.M = m.r; g.N = m.r; g.K = rows_of(i);
        return true;
      }, false, true, true);      // the factorisation reads the lower triangle only
      simple(OP_GRAM_DIAG, (y_side ? 0 : 2) + cur);      // the diagonal (the column norms) exactly
      if (pass < nshift) simple(OP_SHIFT, 0, 32.f * 5.9604645e-8f);
      factor(max_blocks);
      simple(OP_DIAG_INV);
      // M = L^{-1}, row block by row block from the inverses of the diagonal blocks:
      // M[i, <i] = -M_ii (L[i, <i] M[<i, <i]); the Gram buffer, consumed by the factorisation, holds the inner product
      for (int ib = 1; ib < max_blocks; ++ib) {
        gemm([&](int i, GemmDesc& g) {
          const MatDev& m = P.mat[i];
          const int nbk = std::min(NB, m.r - ib * NB);
          if (nbk <= 0) return false;
          const int64_t row = (int64_t)ib * NB * m.r * 4;
          g.A = ref_arena(m.lfac + row); g.sAm = m.r; g.sAk = 1;
          g.B = ref_arena(m.minv); g.sBk = m.r; g.sBn = 1;
          g.C = ref_arena(m.gram + row); g.ldc = m.r;
          g.M = nbk; g.N = ib * NB; g.K = ib * NB;
          return true;
        });
        gemm([&](int i, GemmDesc& g) {
          const MatDev& m = P.mat[i];
          const int nbk = std::min(NB, m.r - ib * NB);
          if (nbk <= 0) return false;
          const int64_t row = (int64_t)ib * NB * m.r * 4;
          g.A = ref_arena(m.minv + row + (int64_t)ib * NB * 4); g.sAm = m.r; g.sAk = 1;
          g.B = ref_arena(m.gram + row); g.sBk = m.r; g.sBn = 1;
          g.C = ref_arena(m.minv + row); g.ldc = m.r;
          g.M = nbk; g.N = ib * NB; g.K = nbk;
          g.alpha = -1.f;
          return true;
        });
      }
      // Q = X M^T in one product over the full rank (the contraction of a column tile stops at its last column)
      int dst = 1 - cur;
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        g.A = ref_arena(buf_of(i, cur)); g.sAm = m.r; g.sAk = 1;
        g.B = ref_arena(m.minv); g.sBk = 1; g.sBn = m.r;
        g.C = ref_arena(buf_of(i, dst)); g.ldc = m.r;
        g.M = rows_of(i); g.N = m.r; g.K = m.r;
        g.tri = 1;
        return true;
      });
      cur = dst;
    }
    return cur;
  }

  // Q_0 = orth(block supplied by the caller) (Alg. 1 Require: a random initial projection)
  void build_init(int passes) {
    std::vector<Op> saved;
    saved.swap(P.ops);
    simple(OP_Y_FROM_EXT);
    const int ycur = orth(true, 0, passes, passes >= 3 ? 2 : 1);
    simple(OP_Q_FROM_Y, ycur);
    simple(OP_PACK);
    P.init_ops.swap(P.ops);
    P.ops.swap(saved);
  }

  // Estimate of sigma_{r+1} of the source for the r-th spectral gap (Sec. 5.1, Metrics): block power iteration on the
  // source deflated by the current basis, (I - Q Q^T) Src, then the largest Ritz value of the block.
  void build_gap(int iters, int passes) {
    const int inner = passes >= 3 ? 2 : 1;
    std::vector<Op> saved;
    saved.swap(P.ops);
    auto deflate = [&](int ycur) {      // Y <- Y - Q (Q^T Y); the r x r product goes through the buffer of the Cholesky factor
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        g.A = ref_arena(m.q32); g.sAm = 1; g.sAk = m.r;
        g.B = ref_arena(m.y[ycur]); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.lfac); g.ldc = m.r;
        g.M = m.r; g.N = m.r; g.K = m.p;
        return true;
      }, false, true);
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        g.A = ref_arena(m.q32); g.sAm = m.r; g.sAk = 1;
        g.B = ref_arena(m.lfac); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.y[ycur]); g.ldc = m.r;
        g.M = m.p; g.N = m.r; g.K = m.r;
        g.alpha = -1.f; g.beta = 1.f;
        return true;
      });
    };
    auto z_product = [&](int ycur) {    // Z = Src^T Y
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        src_operand(g, m, true);
        g.B = ref_arena(m.y[ycur]); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.zw[0]); g.ldc = m.r;
        g.M = m.q; g.N = m.r; g.K = m.p;
        return true;
      });
      P.ops.back().fast = 1;
      P.ops.back().iarg = ycur;
    };
    auto y_product = [&](int ext_or_z) {   // Y = Src B, B = Omega (-1) or the block in zw[ext_or_z]
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        src_operand(g, m, false);
        g.B = ext_or_z < 0 ? ref_ext(EXT_OMEGA) : ref_arena(m.zw[ext_or_z]); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.y[0]); g.ldc = m.r;
        g.M = m.p; g.N = m.r; g.K = m.q;
        return true;
      });
      P.ops.back().fast = 2;
      P.ops.back().iarg = ext_or_z;
    };
    y_product(-1);
    deflate(0);
    int ycur = orth(true, 0, inner, inner);
    for (int it = 0; it < iters; ++it) {
      z_product(ycur);                  // Src^T (I - Q Q^T) Y = Src^T Y for a block orthogonal to Q
      const int zcur = orth(false, 0, inner, inner);
      y_product(zcur);
      deflate(0);
      ycur = it + 1 < iters ? orth(true, 0, inner, inner) : orth(true, 0, inner + 1, inner);
    }
    // with 2r > min(p, q) the deflated source has fewer than r directions and the orthonormalisation completes the
    // block arbitrarily: deflated once more, the block keeps the estimate below the norm of the deflated source
    deflate(ycur);
    z_product(ycur);
    gemm([&](int i, GemmDesc& g) {
      const MatDev& m = P.mat[i];
      g.A = ref_arena(m.zw[0]); g.sAm = 1; g.sAk = m.r;
      g.B = ref_arena(m.zw[0]); g.sBk = m.r; g.sBn = 1;
      g.C = ref_arena(m.gram); g.ldc = m.r;
      g.M = m.r; g.N = m.r; g.K = m.q;
      return true;
    }, false, true, true);
    simple(OP_SHIFT, 1, 32.f * 5.9604645e-8f);
    factor(max_blocks_all());
    simple(OP_JSVD, 1);                 // largest singular value only
    simple(OP_PACK);                    // the Z products borrowed the operand planes of Q
    P.gap_ops.swap(P.ops);
    P.ops.swap(saved);
  }

  // Down-projection of the right-projected matrices (Sec. 2 with the roles of rows and columns exchanged) on the
  // caller's row-major arrays by the generic GEMM: g^T = (s G) Q into zw[0]; the scale s multiplies the launch (it
  // changes per call).  Taken for fp32 gradients and for shapes or pointers the streaming kernel does not read.
  void build_tr_step(bool g_bf16, bool ef, bool all_mats) {
    // g^T (columns of the low-rank state x r, plain, into zw[0]) = (caller's matrix, read in the orientation of the
    // matrix's problem) x Q.  Right-projected matrix: rows of the caller's array are the columns of the state,
    // element (row i, column j) at i * m.p + j.  Left-projected matrix (all_mats: fp32 gradients, whose products run
    // here with three-term operands, as exact as fp32): the columns of the caller's array are the columns of the
    // state, element (row i, column j) at i * m.q + j, contracted over the rows.
    auto a_strides = [](GemmDesc& g, const MatDev& m) {
      if (m.tr) { g.sAm = m.p; g.sAk = 1; }
      else { g.sAm = 1; g.sAk = m.q; }
    };
    std::vector<Op> keep;
    keep.swap(P.ops);
    gemm([&](int i, GemmDesc& g) {
      const MatDev& m = P.mat[i];
      if (!m.tr && !all_mats) return false;
      g.A = ref_ext(EXT_G); a_strides(g, m); g.a_bf16 = g_bf16 ? 1 : 0;
      g.B = ref_arena(m.q32); g.sBk = m.r; g.sBn = 1;
      g.C = ref_arena(m.zw[0]); g.ldc = m.r;
      g.M = m.q; g.N = m.r; g.K = m.p;
      return true;
    });
    P.tr_down_ops.swap(P.ops);
    if (ef) {           // source: the residual after E <- s G + E (fp32, in the arena, the caller's layout)
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        if (!m.tr && !all_mats) return false;
        g.A = ref_arena(m.err); a_strides(g, m);
        g.B = ref_arena(m.q32); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.zw[0]); g.ldc = m.r;
        g.M = m.q; g.N = m.r; g.K = m.p;
        return true;
      });
      P.tr_down_ef_ops.swap(P.ops);
    }
    keep.swap(P.ops);
  }

  // The refresh (Sec. 2 ComputeProjection by a randomised range finder, then the rotation of the moments).
  // passes = 3 is the robust variant: two shifted passes after every product of the power iteration (the conditioning
  // of the source then does not compound from product to product) and shifted, shifted, plain at the end.
  void build(int power_iters, int passes, bool rayleigh_ritz) {
    const int inner = passes >= 3 ? 2 : 1, nshift = passes >= 3 ? 2 : 1;
    // Y = Src Omega
    gemm([&](int i, GemmDesc& g) {
      const MatDev& m = P.mat[i];
      src_operand(g, m, false);
      g.B = ref_ext(EXT_OMEGA); g.sBk = m.r; g.sBn = 1;
      g.C = ref_arena(m.y[0]); g.ldc = m.r;
      g.M = m.p; g.N = m.r; g.K = m.q;
      return true;
    });
    P.ops.back().fast = 2;
    P.ops.back().iarg = -1;
    // Inside the power iteration the blocks only have to stay well conditioned (any basis of the
    // same span serves the next product), so one shifted CholeskyQR pass is enough there; the basis
    // that becomes Q gets the full number of passes.
    int ycur = power_iters > 0 ? orth(true, 0, inner, inner) : orth(true, 0, passes, nshift);
    for (int it = 0; it < power_iters; ++it) {
      // Z = Src^T Y
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        src_operand(g, m, true);
        g.B = ref_arena(m.y[ycur]); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.zw[0]); g.ldc = m.r;
        g.M = m.q; g.N = m.r; g.K = m.p;
        return true;
      });
      P.ops.back().fast = 1;
      P.ops.back().iarg = ycur;
      int zcur = orth(false, 0, inner, inner);
      // Y = Src Z
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        src_operand(g, m, false);
        g.B = ref_arena(m.zw[zcur]); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.y[0]); g.ldc = m.r;
        g.M = m.p; g.N = m.r; g.K = m.q;
        return true;
      });
      P.ops.back().fast = 2;
      P.ops.back().iarg = zcur;
      ycur = it + 1 < power_iters ? orth(true, 0, inner, inner) : orth(true, 0, passes, nshift);
    }
    if (rayleigh_ritz) {
      // Rayleigh-Ritz step (Sec. 2: Q = the first r columns of U, largest singular value first):
      // Z = Src^T Y (= B^T, B the source restricted to the subspace), T = Z^T Z = B B^T, T = U diag U^T, Y <- Y U
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        src_operand(g, m, true);
        g.B = ref_arena(m.y[ycur]); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.zw[0]); g.ldc = m.r;
        g.M = m.q; g.N = m.r; g.K = m.p;
        return true;
      });
      P.ops.back().fast = 1;
      P.ops.back().iarg = ycur;
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        g.A = ref_arena(m.zw[0]); g.sAm = 1; g.sAk = m.r;
        g.B = ref_arena(m.zw[0]); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.gram); g.ldc = m.r;
        g.M = m.r; g.N = m.r; g.K = m.q;
        return true;
      }, false, true, true);      // the factorisation reads the lower triangle only
      // T + shift I = L L^T, then the singular vectors of L (= eigenvectors of T) by one-sided Jacobi on its columns
      simple(OP_SHIFT, 1, 32.f * 5.9604645e-8f);
      factor(max_blocks_all());
      // left singular vectors, by descending singular value, into the buffer the rotation matrix R takes later
      // (not the buffer of the factor's inverse: its upper triangle has to stay zero)
      simple(OP_JSVD);
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        g.A = ref_arena(m.y[ycur]); g.sAm = m.r; g.sAk = 1;
        g.B = ref_arena(m.rot); g.sBk = m.r; g.sBn = 1;
        g.C = ref_arena(m.y[1 - ycur]); g.ldc = m.r;
        g.M = m.p; g.N = m.r; g.K = m.r;
        return true;
      });
      // the columns found are orthogonal to about 1e-6 per pair only: one CholeskyQR pass (unshifted: the block is
      // orthonormal to 1e-4 already) brings them back to working precision without changing their order or,
      // visibly, their directions
      ycur = orth(true, 1 - ycur, 1, 0);
      simple(OP_FROB);            // ||Src||_F^2 for the stable rank (Sec. 5.1)
    }
    // rotation: R = Q_new^T Q_old (and R o R)
    gemm([&](int i, GemmDesc& g) {
      const MatDev& m = P.mat[i];
      g.A = ref_arena(m.y[ycur]); g.sAm = 1; g.sAk = m.r;
      g.B = ref_arena(m.q32); g.sBk = m.r; g.sBn = 1;
      g.C = ref_arena(m.rot); g.C2 = ref_arena(m.rot2); g.ldc = m.r;
      g.M = m.r; g.N = m.r; g.K = m.p;
      return true;
    }, false, true);          // always: the similarity diagnostic (Sec. 5.1, MSSV) reads R o R even when nothing is rotated
    simple(OP_ROT_PRE, 0, 0.f, true);
    for (int which = 0; which < 2; ++which)
      gemm([&](int i, GemmDesc& g) {
        const MatDev& m = P.mat[i];
        g.A = ref_arena(m.zw[2 + which]); g.sAm = m.r; g.sAk = 1;
        g.B = ref_arena(which == 0 ? m.rot : m.rot2); g.sBk = 1; g.sBn = m.r;
        g.C = ref_arena(m.zw[which]); g.ldc = m.r;
        g.M = m.q; g.N = m.r; g.K = m.r;
        return true;
      }, true);
    simple(OP_ROT_POST, 0, 0.f, true);
    simple(OP_Q_FROM_Y, ycur);
    simple(OP_PACK);
  }
};

int validate(const lordo_shape* shapes, int32_t n, const lordo_hparams* hp) {
  if (!shapes || !hp || n <= 0) return LORDO_EINVAL;
  for (int i = 0; i < n; ++i) {
    const lordo_shape& s = shapes[i];
    if (s.rows <= 0 || s.cols <= 0 || s.rank <= 0 || (s.side != 0 && s.side != 1)) return LORDO_EINVAL;
    if (s.rank > (s.side ? s.cols : s.rows)) return LORDO_EINVAL;
    // (tile coordinates of the grouped GEMM are 16-bit: at most 32767 tiles of 64 rows)
    if (s.rows > (1 << 20) || s.cols > (1 << 20) || s.rank > 4096) return LORDO_EINVAL;
    // The kernels address a matrix through buffer descriptors with 32-bit byte offsets: the fp32 array and one tile
    // (256 rows or columns) beyond it must stay below 4 GiB, so that no sum of offsets wraps.
    const int64_t with_tile = std::max((s.rows + 256) * s.cols, s.rows * (s.cols + 256));
    if (with_tile >= (int64_t(1) << 30)) return LORDO_EINVAL;
    // A lane whose column lies outside the matrix is given the byte offset 2^31, and a row outside it the offset of the
    // array's end: both are out of the descriptor's range only while the array (with that tile) is below 2 GiB.  From
    // there on the sides must be multiples of the largest tile, 256, so that no such lane or row exists; the
    // right-projected path is verified below 2 GiB only.
    if (with_tile >= (int64_t(1) << 29) && ((s.rows & 255) != 0 || (s.cols & 255) != 0 || s.side != 0)) return LORDO_EINVAL;
    // the low-rank arrays of the matrix (p x r, r x q in fp32) are addressed the same way and stay below 2 GiB
    if (std::max(s.rows, s.cols) * (int64_t)s.rank >= (int64_t(1) << 29)) return LORDO_EINVAL;
  }
  if (!(hp->beta1 >= 0 && hp->beta1 < 1) || !(hp->beta2 >= 0 && hp->beta2 < 1) || !(hp->eps >= 0)) return LORDO_EINVAL;
  if (hp->qhm_mode < 0 || hp->qhm_mode > 2 || (hp->error_feedback != 0 && hp->error_feedback != 1)) return LORDO_EINVAL;
  // the up-link buffer holds the update in low-rank form; the full-rank QHM update has no such form (App. A.5.1)
  if ((hp->uplink_buffer != 0 && hp->uplink_buffer != 1) || (hp->uplink_buffer && hp->qhm_mode == 2)) return LORDO_EINVAL;
  if (hp->qhm_mode != 0 && !(hp->omega >= 0.0 && hp->omega <= 1.0)) return LORDO_EINVAL;
  if (hp->power_iters < 0 || hp->power_iters > 8) return LORDO_EINVAL;
  if (hp->rayleigh_ritz != 0 && hp->rayleigh_ritz != 1) return LORDO_EINVAL;
  if (hp->param_dtype != LORDO_F32 && hp->param_dtype != LORDO_BF16) return LORDO_EINVAL;
  // bf16 weights: every update case; the fused outer step from the up-link buffers writes fp32 weights only
  if (hp->param_dtype == LORDO_BF16 && hp->uplink_buffer) return LORDO_EINVAL;
  // bf16 residual: the pipelined down-projection of bf16 gradients widens it on the way in and the residual launch of
  // the up-projection rounds it once on the way out; the paths that form s G + E inside the buffer (fp32 gradients,
  // right-projected matrices, the refresh of the local variant) keep an fp32 buffer
  if ((hp->err_dtype != LORDO_F32 && hp->err_dtype != LORDO_BF16) || hp->reserved != 0) return LORDO_EINVAL;
  if (hp->err_dtype == LORDO_BF16) {
    if (!hp->error_feedback || hp->grad_dtype != LORDO_BF16) return LORDO_EINVAL;
    for (int i = 0; i < n; ++i)
      if (shapes[i].side) return LORDO_EINVAL;
  }
  if (hp->rayleigh_ritz)          // a wave of the multi-launch Jacobi solver keeps two columns of r elements in registers
    for (int i = 0; i < n; ++i)
      if (shapes[i].rank > 1024) return LORDO_EINVAL;
  if (hp->orth_passes != 0 && hp->orth_passes != 2 && hp->orth_passes != 3) return LORDO_EINVAL;
  if (hp->grad_dtype != LORDO_BF16 && hp->grad_dtype != LORDO_F32) return LORDO_EINVAL;
  if (!std::isfinite(hp->outer_lr) || !std::isfinite(hp->outer_momentum)) return LORDO_EINVAL;
  return LORDO_OK;
}

void build_plan(const lordo_shape* shapes, int n, const lordo_hparams& hp, Plan& P) {
  Alloc A;
  P.flag = A.take(256);
  P.step = A.take(256);
  P.mats = A.take(sizeof(MatDev) * n);
  P.ext = A.take(sizeof(void*) * EXT_COUNT * EXT_SLOTS * n);
  P.chunk_start = A.take(sizeof(int64_t) * (n + 1));
  P.mat.resize(n);
  P.chunk_start_h.resize(n + 1);
  int64_t lr = 0, chunks = 0;
  int rp_max = 0, pp_min = 1 << 30;
  const bool has_mom = hp.outer_momentum != 0.0;
  for (int i = 0; i < n; ++i) {
    MatDev& m = P.mat[i];
    m.tr = shapes[i].side;
    m.p = (int)(m.tr ? shapes[i].cols : shapes[i].rows); m.q = (int)(m.tr ? shapes[i].rows : shapes[i].cols); m.r = shapes[i].rank;
    if (m.tr) P.any_tr = true;
    m.pp = (int)pad32(m.p); m.qp = (int)pad32(m.q); m.rp = (int)pad32(m.r);
    rp_max = std::max(rp_max, m.rp);
    P.r_max = std::max(P.r_max, (int)m.r);
    P.rank_sq_sum += (int64_t)m.r * m.r;
    if (!m.tr) pp_min = std::min(pp_min, m.pp);
    P.chunk_start_h[i] = chunks;
    chunks += ((int64_t)m.p * m.q + CHUNK - 1) / CHUNK;
  }
  P.chunk_start_h[n] = chunks;
  P.nchunks = chunks;
  if (hp.rayleigh_ritz) { P.frob_part = A.take(sizeof(float) * (size_t)chunks); P.jflags = A.take(256); }
  // rank blocks of 32 per down-projection tile: the pipelined kernel (bf16 G) always takes four and
  // leaves the waves of absent blocks idle; the plain kernel is instantiated for 1, 2 and 4
  P.down_generic = hp.grad_dtype == LORDO_F32;
  P.mb = 4;
  // Down-projection launch shape: the pipelined kernel (rank tiles of 128, bf16 G, 256-column
  // tiles) where it applies, else the plain kernel with 128-column tiles.
  P.down_pipe = (P.mb == 4 && hp.grad_dtype == LORDO_BF16) ? (rp_max >= 256 ? 2 : 1) : 0;
  P.rank_tile = P.down_pipe ? 128 * P.down_pipe : 32 * P.mb;
  P.g_once = rp_max <= P.rank_tile;
  const int down_bn = P.down_pipe ? 256 : 128;
  P.up_waves = 4;

  // Split-K of the down-projection.  With few output tiles (small models) the long contraction
  // over p is cut into slices of about the shortest matrix's height, so that every workgroup
  // has the same amount of work and the chip is filled; slices are summed, in fixed order, by
  // the Adam kernel.  Factors are powers of two up to 8.
  int64_t tiles0 = 0;
  for (int i = 0; i < n; ++i)
    if (!P.mat[i].tr) tiles0 += (int64_t)((P.mat[i].qp + down_bn - 1) / down_bn) * ((P.mat[i].rp + P.rank_tile - 1) / P.rank_tile);
  P.splits.assign(n, 1);
  P.nsplit = 1;
  if (tiles0 > 0 && tiles0 < 1536 && !P.down_generic) {
    // slices of about the shortest matrix's height; halved while the launch would still have fewer
    // than about 1.5 workgroups per compute unit (a single tall matrix, for instance)
    int chunk = std::max(256, pp_min);
    for (;;) {
      int64_t tiles = 0;
      bool can_grow = false;
      P.nsplit = 1;
      for (int i = 0; i < n; ++i) {
        if (P.mat[i].tr) continue;       // right-projected matrices take the generic GEMM: one slice
        int want = (P.mat[i].pp + chunk - 1) / chunk;
        int f = 1;
        while (f * 2 <= want && f < 8) f *= 2;
        if (f < 8 && P.mat[i].pp / (2 * f) >= 256) can_grow = true;
        P.splits[i] = f;
        P.nsplit = std::max(P.nsplit, f);
        tiles += (int64_t)f * ((P.mat[i].qp + down_bn - 1) / down_bn) * ((P.mat[i].rp + P.rank_tile - 1) / P.rank_tile);
      }
      if (tiles >= 400 || !can_grow || chunk <= 256) break;
      chunk = std::max(256, chunk / 2);
    }
  }
  // flat low-rank layout: matrices ordered by split factor, so that the Adam kernel knows the
  // number of slices to sum from the flat position alone
  {
    int g = 0;
    for (int f = 1; f <= 8; f *= 2) {
      bool any = false;
      for (int i = 0; i < n; ++i) {
        if (P.splits[i] != f) continue;
        if (!any) {
          any = true;
          P.grp_nsplit[g] = f;
          P.grp_start[g] = g == 0 ? 0 : lr;
        }
        P.mat[i].lr_off = lr;
        lr += (int64_t)P.mat[i].qp * P.mat[i].rp;
      }
      if (any) ++g;
    }
  }
  P.lr_total = lr;
  // Adam rides in the epilogue of the pipelined down-projection when no matrix is split, i.e. when
  // the launch has several rounds of workgroups and the epilogue of one overlaps the main loop of
  // another; a launch that needs split-K is a single round of workgroups in lock step, where the
  // stand-alone kernel is as fast and leaves the down-projection shorter.
  // The 256-rank tiles also write what the full-rank QHM update and the error feedback need from that pass (column
  // sums of the denominators, operand planes of g); the 128-rank kernel has no registers to spare for them.
  const bool fuse_adam = P.down_pipe && P.nsplit == 1 && !hp.uplink_buffer && !P.any_tr &&
                         (P.down_pipe == 2 || (hp.qhm_mode != 2 && !hp.error_feedback));
  P.adam_first = fuse_adam ? lr : 0;
  P.glow = A.take(sizeof(float) * lr * P.nsplit);
  P.u = A.take(sizeof(float) * lr);
  P.v = A.take(sizeof(float) * lr);
  if (hp.uplink_buffer) P.acc = A.take(sizeof(float) * lr);   // directly behind u and v: [u | v | A] is the packed payload
  P.n_hi = A.take(sizeof(uint16_t) * lr);
  P.n_lo = A.take(sizeof(uint16_t) * lr);
  if (hp.qhm_mode == 2) P.colpart = A.take(sizeof(float) * (lr / 32));
  if (hp.error_feedback) { P.g_hi = A.take(sizeof(uint16_t) * lr); P.g_lo = A.take(sizeof(uint16_t) * lr); }
  P.part_slices = small_out_split(P.mat.data(), n, nullptr);
  for (int i = 0; i < n; ++i) {
    MatDev& m = P.mat[i];
    size_t pr = (size_t)m.p * m.r, pq = (size_t)m.p * m.q, qr = (size_t)m.q * m.r, rr = (size_t)m.r * m.r;
    size_t planes = (size_t)m.pp * m.rp * 2;
    m.q32 = A.take(pr * 4);
    if (!m.tr) {
      m.qa_hi = A.take(planes); m.qa_lo = A.take(planes);
      m.qt_hi = A.take(planes); m.qt_lo = A.take(planes);
    }
    m.anchor = A.take(pq * 4);
    m.mom = has_mom ? A.take(pq * 4) : -1;
    m.err = hp.error_feedback ? A.take(pq * (hp.err_dtype == LORDO_BF16 ? 2 : 4)) : -1;
    m.y[0] = A.take(pr * 4); m.y[1] = A.take(pr * 4);
    for (int k = 0; k < 4; ++k) m.zw[k] = A.take(qr * 4);
    m.gram = A.take(rr * 4); m.lfac = A.take(rr * 4);
    m.dinv = A.take((size_t)((m.r + NB - 1) / NB) * NB * NB * 4);
    m.minv = A.take(rr * 4);
    m.rot = A.take(rr * 4); m.rot2 = A.take(rr * 4);
    m.part = A.take(rr * 4 * P.part_slices);
    m.ritz = hp.rayleigh_ritz ? A.take((size_t)(m.r + 3) * 4) : -1;
  }
  if (P.any_tr) {
    // operand planes of the right-projected matrices: all hi planes of a kind, then all lo planes in the same order,
    // so that one pair of base pointers (hi, hi + gap) serves every such matrix in a launch
    for (int kind = 0; kind < 4; ++kind)          // qa hi, qa lo, qt hi, qt lo
      for (int i = 0; i < n; ++i) {
        MatDev& m = P.mat[i];
        if (!m.tr) continue;
        const int64_t at = A.take((size_t)m.pp * m.rp * 2);
        (kind == 0 ? m.qa_hi : kind == 1 ? m.qa_lo : kind == 2 ? m.qt_hi : m.qt_lo) = at;
      }
    for (int i = 0; i < n; ++i)
      if (P.mat[i].tr) { P.tr_plane_gap = P.mat[i].qa_lo - P.mat[i].qa_hi; break; }
    // Shadow records: the caller's matrix W (rows x cols) as a left-projected problem.
    //   up-projection  W -= eta N^T Q^T: its A planes (row of W, rank) are the planes of N (column of the low-rank
    //     state = row of W, rank), its B planes (column of W, rank) the up-projection planes of Q (row of Q = column of W);
    //   streaming product  g^T = G Q: its B planes (rank, column of W) are the down-projection planes of Q (rank, row of Q),
    //     its result goes to zw[0] as the plain rows x r block.
    // The kernels add lr_off (in 2-byte elements) to the plane base pointers they are given: with the arena base as hi
    // pointer and arena + gap as lo pointer, lr_off = (offset of the hi plane) / 2 selects the planes of Q.
    P.mat_up = P.mat;
    P.mat_stb = P.mat;
    P.mat_up_ef = P.mat;
    P.tr_stream_shapes = hp.grad_dtype == LORDO_BF16;
    for (int i = 0; i < n; ++i) {
      const MatDev& m = P.mat[i];
      if (!m.tr) continue;
      MatDev sdw = m;
      sdw.tr = 0;
      sdw.p = m.q; sdw.q = m.p; sdw.pp = m.qp; sdw.qp = m.pp;
      MatDev up = sdw, stb = sdw;
      up.qa_hi = P.n_hi + 2 * m.lr_off; up.qa_lo = P.n_lo + 2 * m.lr_off;
      up.lr_off = m.qa_hi / 2;
      up.qt_hi = m.lr_off;          // (unused by the up-projection otherwise) the matrix's place in the flat low-rank arrays: row scales of the full-rank QHM term
      stb.lr_off = m.qt_hi / 2;
      stb.y[0] = m.zw[0];
      P.mat_up[i] = up;
      P.mat_stb[i] = stb;
      if (hp.error_feedback) {
        up.qa_hi = P.g_hi + 2 * m.lr_off; up.qa_lo = P.g_lo + 2 * m.lr_off;
        P.mat_up_ef[i] = up;
      }
      if ((sdw.q & 31) != 0 || (sdw.r & 3) != 0) P.tr_stream_shapes = false;
      constexpr int SB = 8 * 128;
      for (int ms = 0; ms < sdw.pp; ms += SB)
        for (int ns = 0; ns < sdw.qp; ns += SB)
          for (int m0 = ms; m0 < std::min(ms + SB, (int)sdw.pp); m0 += 128)
            for (int n0 = ns; n0 < std::min(ns + SB, (int)sdw.qp); n0 += 128) {
              ProjTile t{};
              t.mat = i; t.m0 = m0; t.n0 = n0;
              P.up_tr_h.push_back(t);
            }
      for (int m0 = 0; m0 < sdw.pp; m0 += 128)
        for (int n0 = 0; n0 < sdw.rp; n0 += 128) {
          ProjTile t{};
          t.mat = i; t.m0 = m0; t.n0 = n0;
          P.ytile_tr_h.push_back(t);
        }
    }
    P.up_tr_h = xcd_order(P.up_tr_h);
  }
  // projection tile tables
  std::vector<ProjTile> down, up;
  for (int i = 0; i < n; ++i) {
    const MatDev& m = P.mat[i];
    if (m.tr) continue;               // no tiles of the projection kernels
    const int f = P.splits[i];
    const int klen = ((m.pp + f - 1) / f + 31) / 32 * 32;
    for (int n0 = 0; n0 < (P.down_generic ? 0 : m.qp); n0 += down_bn)
      for (int m0 = 0; m0 < m.rp; m0 += P.rank_tile)
        for (int sp = 0; sp < f; ++sp) {
          ProjTile t{};
          t.mat = i; t.m0 = m0; t.n0 = n0; t.split = sp;
          t.k0 = std::min(sp * klen, m.pp); t.k1 = std::min(t.k0 + klen, m.pp);
          t.fuse = fuse_adam ? 1 : 0;
          down.push_back(t);
        }
    // Up-projection tiles in super-blocks of 8 x 8: the 64 workgroups an XCD runs at a time then share
    // eight row blocks of Q and eight column blocks of N (4 MiB at r = 512, the size of its L2) instead
    // of one row block and 64 column blocks, so the operand planes are re-read from L2 and not from HBM
    constexpr int SB = 8 * 128;
    for (int ms = 0; ms < m.pp; ms += SB)
      for (int ns = 0; ns < m.qp; ns += SB)
        for (int m0 = ms; m0 < std::min(ms + SB, m.pp); m0 += 128)
          for (int n0 = ns; n0 < std::min(ns + SB, m.qp); n0 += 128) {
            ProjTile t{};
            t.mat = i; t.m0 = m0; t.n0 = n0;
            up.push_back(t);
          }
  }
  P.down_h = xcd_order(down);
  P.up_h = xcd_order(up);
  P.down_tiles = A.take(sizeof(ProjTile) * P.down_h.size());
  P.up_tiles = A.take(sizeof(ProjTile) * P.up_h.size());
  {   // ranks from 256 up: the plain update runs on 256 x 128 tiles (fewer operand bytes per output through LDS and L2)
    bool wide = !up.empty();
    for (int i = 0; i < n; ++i)
      if (!P.mat[i].tr && P.mat[i].rp < 256) wide = false;
    if (wide) {
      std::vector<ProjTile> uw;
      constexpr int SBM = 8 * 256, SBN = 8 * 128;     // super-blocks of 8 x 8 tiles: what one XCD runs at a time
      for (int i = 0; i < n; ++i) {
        const MatDev& m = P.mat[i];
        if (m.tr) continue;
        for (int ms = 0; ms < m.pp; ms += SBM)
          for (int ns = 0; ns < m.qp; ns += SBN)
            for (int m0 = ms; m0 < std::min(ms + SBM, m.pp); m0 += 256)
              for (int n0 = ns; n0 < std::min(ns + SBN, m.qp); n0 += 128) {
                ProjTile t{};
                t.mat = i; t.m0 = m0; t.n0 = n0;
                uw.push_back(t);
              }
      }
      P.up_wide_h = xcd_order(uw);
      P.up_wide_tiles = A.take(sizeof(ProjTile) * P.up_wide_h.size());
    }
  }
  if (P.any_tr) {     // tables, like the two above: behind the state that lordo_init clears after the tables are uploaded
    P.mats_up = A.take(sizeof(MatDev) * n);
    P.mats_stb = A.take(sizeof(MatDev) * n);
    P.mats_up_ef = A.take(sizeof(MatDev) * n);
    P.up_tr_tiles = A.take(sizeof(ProjTile) * P.up_tr_h.size());
    P.ytile_tr = A.take(sizeof(ProjTile) * P.ytile_tr_h.size());
  }
  {   // products Y = Src B of the refresh: tiles of 128 rows x 128 rank indices, matrices with a long contraction first
    std::vector<ProjTile> yt;
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return P.mat[a].q > P.mat[b].q; });
    P.y_fast_shapes = true;
    for (int i : order) {
      const MatDev& m = P.mat[i];
      if ((m.q & 31) != 0 || (m.r & 3) != 0 || m.tr) P.y_fast_shapes = false;
      for (int m0 = 0; m0 < m.pp; m0 += 128)
        for (int n0 = 0; n0 < m.rp; n0 += 128) {
          ProjTile t{};
          t.mat = i; t.m0 = m0; t.n0 = n0;
          yt.push_back(t);
        }
    }
    P.ytile_h = yt;            // launch order = list order: workgroups with the longest contraction start first
    P.ytiles = A.take(sizeof(ProjTile) * P.ytile_h.size());
  }
  // refresh program
  ProgramBuilder pb(P, n);
  pb.build(hp.power_iters, hp.orth_passes == 0 ? 2 : hp.orth_passes, hp.rayleigh_ritz != 0);
  if (hp.rayleigh_ritz) pb.build_gap(2, hp.orth_passes == 0 ? 2 : hp.orth_passes);
  pb.build_init(hp.orth_passes == 0 ? 2 : hp.orth_passes);
  if (P.any_tr || P.down_generic) pb.build_tr_step(hp.grad_dtype == LORDO_BF16, hp.error_feedback != 0, P.down_generic);
  P.descs = A.take(sizeof(GemmDesc) * P.desc_h.size());
  P.gtiles = A.take(sizeof(GemmTile) * P.gtile_h.size());
  P.bytes = A.cur;
}

}  // namespace

constexpr int NUM_KCLASS = 8;

struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> pool;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> spans[NUM_KCLASS];
  bool open[NUM_KCLASS] = {};         // begin() recorded, end() not yet
  double sum_ms[NUM_KCLASS] = {};     // spans already read: their events went back to the pool
  int64_t count[NUM_KCLASS] = {};
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  void begin(int k, hipStream_t s) {
    if (!on) return;
    hipEvent_t a = get(), b = get();
    if (!a || !b) return;
    (void)hipEventRecord(a, s);
    spans[k].push_back({a, b});
    open[k] = true;
  }
  void end(int k, hipStream_t s) {
    if (!on || !open[k]) return;
    (void)hipEventRecord(spans[k].back().second, s);
    open[k] = false;
  }
  // a call that fails between begin() and end() drops its span: the closing event was never recorded
  void abandon(int k) {
    if (!open[k]) return;
    pool.push_back(spans[k].back().first);
    pool.push_back(spans[k].back().second);
    spans[k].pop_back();
    open[k] = false;
  }
  void clear() {
    for (int k = 0; k < NUM_KCLASS; ++k) {
      for (auto& pr : spans[k]) { pool.push_back(pr.first); pool.push_back(pr.second); }
      spans[k].clear();
      open[k] = false;
      sum_ms[k] = 0.0;
      count[k] = 0;
    }
  }
  ~Profiler() {
    clear();
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
  }
};

struct lordo_ctx {
  Profiler prof;
  int n = 0;
  lordo_hparams hp{};
  Plan plan;
  DevCtx dev{};
  int64_t t = 0;
  bool refreshed = false;        // a subspace refresh has run: R = Q_new^T Q_old of the last one is in the arena
  bool step_dirty = false;       // the step count on the device has to be set from `t` (after lordo_set_step)
  int sync_step(hipStream_t s) {
    if (!step_dirty) return LORDO_OK;
    if (launch_step(at<StepDev>(plan.step), hp.beta1, hp.beta2, hp.bias_correction, t, s) != hipSuccess) return LORDO_EHIP;
    step_dirty = false;
    return LORDO_OK;
  }
  // lordo_refresh_subspace_local left grad_scale * G + E in the error buffer; the next local step must
  // come with the same gradient pointers and takes its projected matrix from the buffer alone
  bool grad_folded = false;
  int64_t window_steps = 0;      // local steps since the last outer step: what the up-link buffer holds
  uint32_t draws = 0;            // Gaussian blocks drawn from the internal generator so far (the `draw` word of its counter)
  bool gauss_init = false;       // lordo_init_projection without a block: the program's first op draws it
  std::vector<const void*> folded_g;
  int device = 0;
  int static_device = -1;        // >= 0: the context lives in the library's static workspace of that device (lordo_init_static)
  // cached caller pointer tables: EXT_SLOTS per kind, replaced round-robin
  std::vector<void*> shadow[EXT_COUNT][EXT_SLOTS];
  int next_slot[EXT_COUNT] = {0, 0, 0, 0, 0, 0};

  template <class T>
  T* at(int64_t off) const { return reinterpret_cast<T*>(dev.arena + off); }

  // the arena, the tables in it and the caller's matrices live on the GPU that was current at lordo_init: a call with
  // another GPU current would launch kernels there on addresses of this one
  bool on_its_device() const {
    int cur = -1;
    return hipGetDevice(&cur) == hipSuccess && cur == device;
  }

  static bool has_null(const void* const* host, int n) {
    for (int i = 0; i < n; ++i)
      if (!host[i]) return true;
    return false;
  }
  int set_ext(int table, void* const* host, hipStream_t s, bool allow_null = false) {
    if (!host) return LORDO_EINVAL;
    if (!allow_null && has_null(host, n)) return LORDO_EINVAL;
    for (int k = 0; k < EXT_SLOTS; ++k) {
      const std::vector<void*>& sh = shadow[table][k];
      if (!sh.empty() && std::memcmp(sh.data(), host, sizeof(void*) * n) == 0) {
        dev.slot[table] = table * EXT_SLOTS + k;
        return LORDO_OK;
      }
    }
    int k = next_slot[table];
    next_slot[table] = (k + 1) % EXT_SLOTS;
    void** dst = const_cast<void**>(dev.ext) + (size_t)(table * EXT_SLOTS + k) * n;
    HIPCHK(launch_store_ptrs(dst, host, n, s));
    shadow[table][k].assign(host, host + n);
    dev.slot[table] = table * EXT_SLOTS + k;
    return LORDO_OK;
  }
};

extern "C" {

int lordo_workspace_bytes(const lordo_shape* shapes, int32_t n, const lordo_hparams* hp, size_t* out_bytes) {
  if (!out_bytes) return LORDO_EINVAL;
  int rc = validate(shapes, n, hp);
  if (rc != LORDO_OK) return rc;
  Plan P;
  build_plan(shapes, n, *hp, P);
  *out_bytes = P.bytes;
  return LORDO_OK;
}

}  // extern "C"

// Workspace for callers that cannot allocate device memory (see lordo_init_static): a fixed array in the code object,
// one copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle of the
// symbol: the device address of each GPU's copy is looked up once per device (hipGetSymbolAddress) and only that
// address is ever handed to kernels, fills and copies.
static __device__ __align__(256) unsigned char scratch[LORDO_STATIC_WORKSPACE_BYTES];
namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_static_mutex;
void* g_static_ptr[MAX_DEVICES] = {};       // device address of this GPU's copy of `scratch`
bool g_static_busy[MAX_DEVICES] = {};       // a context created by lordo_init_static on this GPU is alive
}  // namespace

static int init_context(lordo_ctx** out, const lordo_shape* shapes, int32_t n, const lordo_hparams* hp, void* arena,
                        size_t arena_bytes, void* const* W, void* stream) {
  if (!out) return LORDO_EINVAL;
  *out = nullptr;
  int rc = validate(shapes, n, hp);
  if (rc != LORDO_OK) return rc;
  if (!arena || !W || (reinterpret_cast<uintptr_t>(arena) & 255) != 0) return LORDO_EINVAL;
  for (int i = 0; i < n; ++i)
    if (!W[i]) return LORDO_EINVAL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
    fprintf(stderr, "lordo: no HIP device available\n");
    return LORDO_EHIP;
  }
  lordo_ctx* c = new lordo_ctx();
  c->n = n;
  c->hp = *hp;
  build_plan(shapes, n, *hp, c->plan);
  Plan& P = c->plan;
  if (arena_bytes < P.bytes) { delete c; return LORDO_ENOMEM; }
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  auto fail = [&](int code) { delete c; return code; };
  if (hipGetDevice(&c->device) != hipSuccess) return fail(LORDO_EHIP);
  c->dev.arena = reinterpret_cast<char*>(arena);
  c->dev.mats = c->at<MatDev>(P.mats);
  c->dev.ext = c->at<void*>(P.ext);
  c->dev.n = n;
  c->dev.flag = c->at<int32_t>(P.flag);
  for (int k = 0; k < EXT_COUNT; ++k) c->dev.slot[k] = k * EXT_SLOTS;
#define INITCHK(expr)                                                                             \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) {                                                                       \
      fprintf(stderr, "lordo: %s failed: %s\n", #expr, hipGetErrorString(e_));                    \
      return fail(LORDO_EHIP);                                                                    \
    }                                                                                             \
  } while (0)
  INITCHK(hipStreamSynchronize(s));
  INITCHK(hipMemcpy(c->at<void>(P.mats), P.mat.data(), sizeof(MatDev) * n, hipMemcpyHostToDevice));
  if (P.any_tr) {
    INITCHK(hipMemcpy(c->at<void>(P.mats_up), P.mat_up.data(), sizeof(MatDev) * n, hipMemcpyHostToDevice));
    INITCHK(hipMemcpy(c->at<void>(P.mats_stb), P.mat_stb.data(), sizeof(MatDev) * n, hipMemcpyHostToDevice));
    INITCHK(hipMemcpy(c->at<void>(P.mats_up_ef), P.mat_up_ef.data(), sizeof(MatDev) * n, hipMemcpyHostToDevice));
    INITCHK(hipMemcpy(c->at<void>(P.up_tr_tiles), P.up_tr_h.data(), sizeof(ProjTile) * P.up_tr_h.size(), hipMemcpyHostToDevice));
    INITCHK(hipMemcpy(c->at<void>(P.ytile_tr), P.ytile_tr_h.data(), sizeof(ProjTile) * P.ytile_tr_h.size(), hipMemcpyHostToDevice));
  }
  INITCHK(hipMemcpy(c->at<void>(P.chunk_start), P.chunk_start_h.data(), sizeof(int64_t) * (n + 1), hipMemcpyHostToDevice));
  if (!P.down_h.empty()) INITCHK(hipMemcpy(c->at<void>(P.down_tiles), P.down_h.data(), sizeof(ProjTile) * P.down_h.size(), hipMemcpyHostToDevice));
  if (!P.up_h.empty()) INITCHK(hipMemcpy(c->at<void>(P.up_tiles), P.up_h.data(), sizeof(ProjTile) * P.up_h.size(), hipMemcpyHostToDevice));
  if (!P.up_wide_h.empty())
    INITCHK(hipMemcpy(c->at<void>(P.up_wide_tiles), P.up_wide_h.data(), sizeof(ProjTile) * P.up_wide_h.size(), hipMemcpyHostToDevice));
  INITCHK(hipMemcpy(c->at<void>(P.ytiles), P.ytile_h.data(), sizeof(ProjTile) * P.ytile_h.size(), hipMemcpyHostToDevice));
  if (!P.desc_h.empty())
    INITCHK(hipMemcpy(c->at<void>(P.descs), P.desc_h.data(), sizeof(GemmDesc) * P.desc_h.size(), hipMemcpyHostToDevice));
  if (!P.gtile_h.empty())
    INITCHK(hipMemcpy(c->at<void>(P.gtiles), P.gtile_h.data(), sizeof(GemmTile) * P.gtile_h.size(), hipMemcpyHostToDevice));
  // zero everything from the flat low-rank arrays to the end of the per-matrix regions except
  // the tables written above: state (u, v, g, N), momentum and scratch all start at zero
  INITCHK(launch_fill_zero(c->at<void>(P.flag), 256, s));
  INITCHK(launch_fill_zero(c->at<void>(P.ext), ((sizeof(void*) * EXT_COUNT * EXT_SLOTS * n + 255) & ~size_t(255)), s));
  INITCHK(launch_fill_zero(c->at<void>(P.glow), (int64_t)(P.down_tiles - P.glow), s));
  INITCHK(launch_step(c->at<StepDev>(P.step), hp->beta1, hp->beta2, hp->bias_correction, 0, s));      // t = 0
  c->step_dirty = false;
  INITCHK(launch_identity_q(c->dev, s));
  INITCHK(launch_pack_q(c->dev, 0, n, s));
  {
    int r2 = c->set_ext(EXT_W, W, s);
    if (r2 != LORDO_OK) return fail(r2);
  }
  INITCHK(launch_anchor_from_w(c->dev, c->at<int64_t>(P.chunk_start), P.nchunks, hp->param_dtype == LORDO_BF16, s));
  INITCHK(hipStreamSynchronize(s));
#undef INITCHK
  *out = c;
  return LORDO_OK;
}

extern "C" {

int lordo_init(lordo_ctx** out, const lordo_shape* shapes, int32_t n, const lordo_hparams* hp, void* arena,
               size_t arena_bytes, void* const* W, void* stream) {
  return init_context(out, shapes, n, hp, arena, arena_bytes, W, stream);
}

int lordo_init_static(lordo_ctx** out, const lordo_shape* shapes, int32_t n, const lordo_hparams* hp, void* const* W, void* stream) {
  if (!out) return LORDO_EINVAL;
  *out = nullptr;
  int rc = validate(shapes, n, hp);
  if (rc != LORDO_OK) return rc;
  {
    Plan P;
    build_plan(shapes, n, *hp, P);
    if (P.bytes > (size_t)LORDO_STATIC_WORKSPACE_BYTES) {
      fprintf(stderr, "lordo_init_static: these shapes need %zu bytes of workspace, the static workspace holds %zu\n", P.bytes,
              (size_t)LORDO_STATIC_WORKSPACE_BYTES);
      return LORDO_ENOMEM;
    }
  }
  int dev = 0;
  HIPCHK(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return LORDO_EINVAL;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (g_static_busy[dev]) return LORDO_ESTATE;         // one context at a time per GPU: a second one would share the array
  if (!g_static_ptr[dev]) {                            // once per device, with that device current
    void* ptr = nullptr;
    HIPCHK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255) != 0) return LORDO_EHIP;
    g_static_ptr[dev] = ptr;
  }
  // the array keeps what the last context left in it: init_context overwrites every table and clears the flag, the
  // pointer tables, the state and the scratch regions, exactly as it does for a caller's uninitialised arena
  rc = init_context(out, shapes, n, hp, g_static_ptr[dev], LORDO_STATIC_WORKSPACE_BYTES, W, stream);
  if (rc != LORDO_OK) return rc;
  (*out)->static_device = dev;
  g_static_busy[dev] = true;
  return LORDO_OK;
}

int lordo_local_step(lordo_ctx* c, void* const* W, const void* const* G, double lr, double grad_scale, void* stream) {
  if (!c || !W || !G || !std::isfinite(lr) || !std::isfinite(grad_scale)) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  Plan& P = c->plan;
  if (lordo_ctx::has_null(reinterpret_cast<const void* const*>(W), c->n) || lordo_ctx::has_null(G, c->n)) return LORDO_EINVAL;
  // after lordo_refresh_subspace_local the error buffer already holds grad_scale * G + E of this step
  const bool folded = c->grad_folded;
  if (folded && std::memcmp(c->folded_g.data(), G, sizeof(void*) * c->n) != 0) return LORDO_ESTATE;
  // fp32 gradients with error feedback: the sum s G + E of every matrix is formed in the residual buffer before the
  // product (as it is for right-projected matrices), so the residual update adds no gradient term of its own
  const bool generic = P.down_generic;
  const double proj_scale = (folded || (generic && c->hp.error_feedback)) ? 0.0 : grad_scale;
  const int64_t t = c->t + 1;
  AdamArgs a;
  a.b1 = (float)c->hp.beta1; a.omb1 = (float)(1.0 - c->hp.beta1);
  a.b2 = (float)c->hp.beta2; a.omb2 = (float)(1.0 - c->hp.beta2);
  a.step = c->at<StepDev>(P.step);        // the step count and 1 - beta^t live on the device: advanced below, by a kernel
  a.eps = (float)c->hp.eps;
  for (int i = 0; i < 4; ++i) { a.grp_nsplit[i] = P.grp_nsplit[i]; a.grp_start[i] = P.grp_start[i]; }
  a.split_stride = P.lr_total;
  a.first = P.adam_first;
  const bool qhm_low = c->hp.qhm_mode == 1, qhm_full = c->hp.qhm_mode == 2, ef = c->hp.error_feedback != 0;
  a.qw = qhm_low ? (float)c->hp.omega : 1.f;
  a.qg = qhm_low ? (float)(1.0 - c->hp.omega) : 0.f;
  a.colpart = qhm_full ? c->at<float>(P.colpart) : nullptr;
  a.g_hi = ef ? c->at<uint16_t>(P.g_hi) : nullptr;
  a.g_lo = ef ? c->at<uint16_t>(P.g_lo) : nullptr;
  a.acc = c->hp.uplink_buffer ? c->at<float>(P.acc) : nullptr;
  a.lr = (float)lr;
  const bool g_f32 = c->hp.grad_dtype == LORDO_F32;
  bool g_vec = true;            // 4-byte accesses to a bf16 G need an even q and 4-byte aligned pointers
  for (int i = 0; i < c->n; ++i)      // (right-projected matrices do not pass through the projection kernels)
    if (!P.mat[i].tr && ((P.mat[i].q & 1) != 0 || (reinterpret_cast<uintptr_t>(G[i]) & 3) != 0)) { g_vec = false; break; }
  const bool w_bf16 = c->hp.param_dtype == LORDO_BF16, e_bf16 = c->hp.err_dtype == LORDO_BF16;
  const uintptr_t w_mask = w_bf16 ? 7 : 15;     // four weights with one access: 16 bytes of fp32, 8 bytes of bf16
  bool w_vec = true;            // four-column accesses to W need q % 4 == 0 and pointers aligned to them
  for (int i = 0; i < c->n; ++i)
    if (!P.mat[i].tr && ((P.mat[i].q & 3) != 0 || (reinterpret_cast<uintptr_t>(W[i]) & w_mask) != 0)) { w_vec = false; break; }
  if (qhm_full || ef) {         // the gradient-term epilogue reads four columns of G per lane
    if (!w_vec) return LORDO_EINVAL;
    for (int i = 0; i < c->n; ++i)
      if (P.mat[i].tr && ((P.mat[i].p & 3) != 0 || (reinterpret_cast<uintptr_t>(W[i]) & w_mask) != 0)) return LORDO_EINVAL;
    for (int i = 0; i < c->n; ++i)
      if ((reinterpret_cast<uintptr_t>(G[i]) & (g_f32 ? 15 : 7)) != 0) return LORDO_EINVAL;
  }
  // every argument and state check has passed: from here on kernels are enqueued
  int rc = c->sync_step(s);
  if (rc != LORDO_OK) return rc;
  HIPCHK(launch_step(c->at<StepDev>(P.step), c->hp.beta1, c->hp.beta2, c->hp.bias_correction, -1, s));      // t <- t + 1
  c->step_dirty = true;         // until the whole step is enqueued: a call that fails below leaves the device count to be set back from `t`
  rc = c->set_ext(EXT_W, W, s);
  if (rc != LORDO_OK) return rc;
  rc = c->set_ext(EXT_G, const_cast<void* const*>(reinterpret_cast<const void* const*>(G)), s);
  if (rc != LORDO_OK) return rc;
  DownFuse fuse;
  fuse.u = c->at<float>(P.u); fuse.v = c->at<float>(P.v);
  fuse.n_hi = c->at<uint16_t>(P.n_hi); fuse.n_lo = c->at<uint16_t>(P.n_lo);
  fuse.a = a;
  c->prof.begin(LORDO_K_DOWN, s);
  bool g_tr = true;             // 16-byte global-to-LDS loads of G need q % 8 == 0 and 16-byte aligned pointers
  for (int i = 0; i < c->n && g_tr; ++i)
    if (!P.mat[i].tr && ((P.mat[i].q & 7) != 0 || (reinterpret_cast<uintptr_t>(G[i]) & 15) != 0)) g_tr = false;
  if (!P.down_h.empty())
    HIPCHK(launch_proj_down(c->dev, c->at<ProjTile>(P.down_tiles), (int)P.down_h.size(), P.mb, P.down_pipe, g_vec, g_tr, P.g_once, c->at<float>(P.glow),
                            P.lr_total, (float)proj_scale, g_f32, ef ? (e_bf16 ? 3 : 1) : 0, &fuse, s));
  if (P.any_tr || generic) {    // g^T = (s G) Q into the plain block zw[0], then into the blocked array the Adam kernel reads
    bool stream = P.tr_stream_shapes && !ef && !generic;
    if (ef) {                   // A = s G + E is formed in the residual buffer first (unless a refresh of the local variant has done it)
      if (!folded)
        HIPCHK(launch_fold_grad(c->dev, c->at<int64_t>(P.chunk_start), P.nchunks, (float)grad_scale, g_f32, s, !generic));
      for (const Op& op : P.tr_down_ef_ops)
        HIPCHK(launch_gemm32(c->dev, c->at<GemmDesc>(P.descs), c->at<GemmTile>(P.gtiles) + op.tile_first, op.ntiles, op.tile, 0, s, 1.f));
    }
    for (int i = 0; i < c->n && stream; ++i)
      if (P.mat[i].tr && (reinterpret_cast<uintptr_t>(G[i]) & 15) != 0) stream = false;
    uint16_t* planes_hi = reinterpret_cast<uint16_t*>(c->dev.arena);
    uint16_t* planes_lo = reinterpret_cast<uint16_t*>(c->dev.arena + P.tr_plane_gap);
    if (stream) {               // the kernel of the refresh products Y = Src B, with G as source and the planes of Q as B
      DevCtx dv = c->dev;
      dv.mats = c->at<MatDev>(P.mats_stb);
      dv.slot[EXT_SRC] = dv.slot[EXT_G];
      HIPCHK(launch_src_times_block(dv, c->at<ProjTile>(P.ytile_tr), (int)P.ytile_tr_h.size(), planes_hi, planes_lo, s));
    } else if (!ef) {
      for (const Op& op : P.tr_down_ops)
        HIPCHK(launch_gemm32(c->dev, c->at<GemmDesc>(P.descs), c->at<GemmTile>(P.gtiles) + op.tile_first, op.ntiles, op.tile, 0, s, (float)grad_scale));
    }
    HIPCHK(launch_tr_exchange(c->dev, c->at<float>(P.glow), stream ? (float)grad_scale : 1.f, generic, s));
  }
  c->prof.end(LORDO_K_DOWN, s);
  c->prof.begin(LORDO_K_ADAM, s);
  if (P.adam_first < P.lr_total)
    HIPCHK(launch_adam(c->at<float>(P.glow), c->at<float>(P.u), c->at<float>(P.v), c->at<uint16_t>(P.n_hi),
                       c->at<uint16_t>(P.n_lo), P.lr_total, a, s));
  c->prof.end(LORDO_K_ADAM, s);
  c->prof.begin(LORDO_K_UP, s);
  UpArgs ua{};
  ua.g_is_f32 = g_f32 ? 1 : 0;
  ua.eps = (float)c->hp.eps;
  ua.w_bf16 = w_bf16 ? 1 : 0;
  if (ef) {                     // E <- grad_scale*G + E - Q g (Alg. 1 error-feedback lines); reads the E the down-projection used
    ua.coef_acc = -1.f; ua.coef_g = (float)proj_scale; ua.target_err = 1; ua.colscale = 0; ua.colpart = nullptr;
    ua.w_bf16 = e_bf16 ? 1 : 0;         // element type of this launch's target: the residual
    if (!P.up_wide_h.empty() && w_vec && !g_f32)
      HIPCHK(launch_proj_up_wide(c->dev, c->at<ProjTile>(P.up_wide_tiles), (int)P.up_wide_h.size(), c->at<uint16_t>(P.g_hi),
                                 c->at<uint16_t>(P.g_lo), ua, s));
    else if (!P.up_h.empty())
      HIPCHK(launch_proj_up(c->dev, c->at<ProjTile>(P.up_tiles), (int)P.up_h.size(), w_vec, c->at<uint16_t>(P.g_hi),
                            c->at<uint16_t>(P.g_lo), ua, s));
    if (P.any_tr) {             // right-projected matrices: E already holds s G + E; E <- E - g^T Q^T on the shadow records (planes of g as A)
      UpArgs ue = ua;
      ue.coef_g = 0.f;
      DevCtx du = c->dev;
      du.mats = c->at<MatDev>(P.mats_up_ef);
      HIPCHK(launch_proj_up(du, c->at<ProjTile>(P.up_tr_tiles), (int)P.up_tr_h.size(), true, reinterpret_cast<uint16_t*>(c->dev.arena),
                            reinterpret_cast<uint16_t*>(c->dev.arena + P.tr_plane_gap), ue, s));
    }
  }
  ua.target_err = 0;
  ua.w_bf16 = w_bf16 ? 1 : 0;
  if (qhm_full) {               // W <- W - eta [ (1-omega) G_hat diag(1/s) + omega Q N ]  (Alg. 1 "Full-Rank QHM")
    ua.coef_acc = (float)(-lr * c->hp.omega);
    ua.coef_g = (float)(-lr * (1.0 - c->hp.omega) * grad_scale);
    ua.colscale = 1; ua.colpart = c->at<float>(P.colpart);
  } else {
    ua.coef_acc = (float)-lr; ua.coef_g = 0.f; ua.colscale = 0; ua.colpart = nullptr;
  }
  if (!P.up_wide_h.empty() && w_vec && !(qhm_full && g_f32))   // (the wide kernel's gradient-term epilogue reads bf16 gradients)
    HIPCHK(launch_proj_up_wide(c->dev, c->at<ProjTile>(P.up_wide_tiles), (int)P.up_wide_h.size(), c->at<uint16_t>(P.n_hi),
                               c->at<uint16_t>(P.n_lo), ua, s));
  else if (!P.up_h.empty())
    HIPCHK(launch_proj_up(c->dev, c->at<ProjTile>(P.up_tiles), (int)P.up_h.size(), w_vec, c->at<uint16_t>(P.n_hi),
                          c->at<uint16_t>(P.n_lo), ua, s));
  if (P.any_tr) {               // W <- W - eta N^T Q^T: the up-projection kernel on the shadow records (planes of N as A, of Q as B)
    bool w_vec_tr = true;
    for (int i = 0; i < c->n && w_vec_tr; ++i)
      if (P.mat[i].tr && ((P.mat[i].p & 3) != 0 || (reinterpret_cast<uintptr_t>(W[i]) & w_mask) != 0)) w_vec_tr = false;
    DevCtx du = c->dev;
    du.mats = c->at<MatDev>(P.mats_up);
    UpArgs ut = ua;
    if (qhm_full) ut.colscale = 2;      // the scale of the gradient term runs over the rows of W: the columns of the low-rank state
    HIPCHK(launch_proj_up(du, c->at<ProjTile>(P.up_tr_tiles), (int)P.up_tr_h.size(), w_vec_tr, reinterpret_cast<uint16_t*>(c->dev.arena),
                          reinterpret_cast<uint16_t*>(c->dev.arena + P.tr_plane_gap), ut, s));
  }
  c->prof.end(LORDO_K_UP, s);
  c->t = t;
  c->step_dirty = false;
  c->grad_folded = false;
  ++c->window_steps;
  return LORDO_OK;
}

static int run_ops(lordo_ctx* c, const std::vector<Op>& ops, int32_t src_dtype, hipStream_t s, bool rotate, double c1, double c2,
                   bool proj_kernels, bool stream_kernel, bool proj_tr = false);

// Runs the refresh program on the source table currently selected in EXT_SRC; with `fold` the error
// buffer first takes E <- fold_scale * G + E (Alg. 2, argument of ComputeProjection).
static int run_refresh(lordo_ctx* c, int32_t src_dtype, hipStream_t s, bool fold = false, double fold_scale = 0.0,
                       bool proj_kernels = false, bool stream_kernel = false, bool proj_tr = false) {
  Plan& P = c->plan;
  const bool rotate = c->t > 0;
  const double c1 = 1.0, c2 = 1.0;       // (the rotation passes read the bias corrections of the current step from the device)
  int rc = c->sync_step(s);
  if (rc != LORDO_OK) return rc;
  c->prof.begin(LORDO_K_REFRESH, s);
  if (fold && launch_fold_grad(c->dev, c->at<int64_t>(P.chunk_start), P.nchunks, (float)fold_scale, c->hp.grad_dtype == LORDO_F32, s) != hipSuccess)
    rc = LORDO_EHIP;
  if (rc == LORDO_OK) rc = run_ops(c, P.ops, src_dtype, s, rotate, c1, c2, proj_kernels, stream_kernel, proj_tr);
  if (rc != LORDO_OK) { c->prof.abandon(LORDO_K_REFRESH); return rc; }
  c->prof.end(LORDO_K_REFRESH, s);
  c->refreshed = true;
  return LORDO_OK;
}

// Enqueues one static program (the refresh, or the initial projection).
static int run_ops(lordo_ctx* c, const std::vector<Op>& ops, int32_t src_dtype, hipStream_t s, bool rotate, double c1, double c2,
                   bool proj_kernels, bool stream_kernel, bool proj_tr) {
  Plan& P = c->plan;
  const GemmDesc* descs = c->at<GemmDesc>(P.descs);
  const GemmTile* tiles = c->at<GemmTile>(P.gtiles);
  for (const Op& op : ops) {
    if (op.rot_only && !rotate) continue;
    switch (op.kind) {
      case OP_GEMM:
        if (op.fast == 1 && proj_kernels) {
          // Z = Src^T Y has the shape of the down-projection g = Q^T G: Y goes into the operand planes of Q
          // (the refresh repacks them at its end), the source takes the place of the gradient, and the
          // result comes back from the layout of g as the plain q x r block
          AdamArgs a{};
          for (int i = 0; i < 4; ++i) { a.grp_nsplit[i] = P.grp_nsplit[i]; a.grp_start[i] = P.grp_start[i]; }
          a.split_stride = P.lr_total;
          HIPCHK(launch_pack_y(c->dev, op.iarg, s));
          HIPCHK(launch_proj_down(c->dev, c->at<ProjTile>(P.down_tiles), (int)P.down_h.size(), P.mb, P.down_pipe, true, proj_tr, P.g_once,
                                  c->at<float>(P.glow), P.lr_total, 1.f, false, src_dtype == LORDO_F32 ? 2 : 0, nullptr, s));
          HIPCHK(launch_glow_to_z(c->dev, c->at<float>(P.glow), 0, a, s));
          break;
        }
        if (op.fast == 2 && stream_kernel) {
          // Y = Src B: B (Omega or Z) goes, as bf16 hi / lo planes, where the planes of N live between steps
          HIPCHK(launch_pack_block(c->dev, op.iarg, c->at<uint16_t>(P.n_hi), c->at<uint16_t>(P.n_lo), s));
          HIPCHK(launch_src_times_block(c->dev, c->at<ProjTile>(P.ytiles), (int)P.ytile_h.size(), c->at<uint16_t>(P.n_hi),
                                        c->at<uint16_t>(P.n_lo), s));
          break;
        }
        HIPCHK(launch_gemm32(c->dev, descs, tiles + op.tile_first, op.ntiles, op.tile, src_dtype == LORDO_BF16, s));
        if (op.split) HIPCHK(launch_gemm_reduce(c->dev, descs + op.desc_first, op.ndescs, s));
        break;
      case OP_SHIFT: HIPCHK(launch_gram_shift(c->dev, op.farg, op.iarg != 0, s)); break;
      case OP_GRAM_DIAG: HIPCHK(launch_gram_diag(c->dev, op.iarg, P.r_max, P.part_slices, s)); break;
      case OP_POTF2: HIPCHK(launch_potf2(c->dev, op.iarg, s)); break;
      case OP_DIAG_INV: HIPCHK(launch_diag_inverses(c->dev, s)); break;
      case OP_JSVD:
        if (P.r_max <= 128) HIPCHK(launch_jacobi_svd(c->dev, P.r_max, op.iarg != 0, s));
        else HIPCHK(launch_jacobi_svd_blocked(c->dev, P.r_max, P.rank_sq_sum, op.iarg != 0, c->at<int>(P.jflags), s));
        break;
      case OP_FROB:
        HIPCHK(launch_frob2(c->dev, c->at<int64_t>(P.chunk_start), P.nchunks, c->at<float>(P.frob_part), src_dtype == LORDO_F32, s));
        break;
      case OP_ROT_PRE:
        HIPCHK(launch_rot_pre(c->dev, c->at<float>(P.u), c->at<float>(P.v), c->at<StepDev>(P.step), s));
        break;
      case OP_ROT_POST:
        HIPCHK(launch_rot_post(c->dev, c->at<float>(P.u), c->at<float>(P.v), c->at<StepDev>(P.step), s));
        break;
      case OP_Q_FROM_Y: HIPCHK(launch_q_from_y(c->dev, op.iarg, s)); break;
      case OP_PACK: HIPCHK(launch_pack_q(c->dev, 0, c->n, s)); break;
      case OP_Y_FROM_EXT:
        if (c->gauss_init) HIPCHK(launch_gauss_block(c->dev, 0, c->hp.seed, c->draws, s));
        else HIPCHK(launch_y_from_ext(c->dev, s));
        break;
      default: return LORDO_ESTATE;
    }
  }
  return LORDO_OK;
}

// Which of the projection-type kernels can take the products of a program whose source is Src.
struct SrcPaths { bool proj_kernels, stream_kernel, proj_tr; };
static int source_paths(lordo_ctx* c, const void* const* Src, int32_t src_dtype, hipStream_t s, SrcPaths& out) {
  // a bf16 source with the alignment the pipelined down-projection kernel reads gradients with lets that
  // kernel take the products of the power iteration that have its shape
  // (an fp32 source too: that kernel then stages it as bf16 hi + lo planes, as it does the error-feedback sum)
  bool proj_kernels = c->plan.down_pipe != 0 && !c->plan.any_tr;      // a right-projected matrix: the generic products for all
  const uintptr_t pair_mask = src_dtype == LORDO_BF16 ? 3 : 7;       // two adjacent columns with one access
  for (int i = 0; i < c->n && proj_kernels; ++i)
    if ((c->plan.mat[i].q & 1) != 0 || (reinterpret_cast<uintptr_t>(Src[i]) & pair_mask) != 0) proj_kernels = false;
  if (proj_kernels && src_dtype == LORDO_BF16) {
    int rc = c->set_ext(EXT_G, const_cast<void* const*>(reinterpret_cast<const void* const*>(Src)), s, true);
    if (rc != LORDO_OK) return rc;
  }
  // the products contracted over the columns stream a bf16 source straight into matrix-core fragment order
  // (bf16 only: an fp32 source would have to be cut to bf16 hi + lo, 2^-18, on the way, which moved the projector by
  // 3e-4 .. 4e-4 on the parity shapes; it keeps the three-term GEMM for these products.  In the products of the
  // other orientation, above, the same cut costs 1e-4 and is taken.)
  bool stream_kernel = src_dtype == LORDO_BF16 && c->plan.y_fast_shapes;
  for (int i = 0; i < c->n && stream_kernel; ++i)
    if ((reinterpret_cast<uintptr_t>(Src[i]) & 15) != 0) stream_kernel = false;
  // global-to-LDS loads of a bf16 source in the down-projection kernel: q % 8 == 0, 16-byte aligned
  bool proj_tr = proj_kernels && src_dtype == LORDO_BF16;
  for (int i = 0; i < c->n && proj_tr; ++i)
    if ((c->plan.mat[i].q & 7) != 0 || (reinterpret_cast<uintptr_t>(Src[i]) & 15) != 0) proj_tr = false;
  out = SrcPaths{proj_kernels, stream_kernel, proj_tr};
  return LORDO_OK;
}

// Start blocks of the range finder: the caller's table, or (Omega == NULL) blocks drawn by the library's generator
// into the fourth q x r scratch block of every matrix, which nothing touches before the first product has read it.
static int select_omega(lordo_ctx* c, const void* const* Omega, hipStream_t s) {
  if (Omega) return c->set_ext(EXT_OMEGA, const_cast<void* const*>(reinterpret_cast<const void* const*>(Omega)), s, c->dev.skip_null != 0);
  HIPCHK(launch_gauss_block(c->dev, 1, c->hp.seed, c->draws, s));
  ++c->draws;
  std::vector<void*> own(c->n);
  for (int i = 0; i < c->n; ++i) own[i] = c->dev.arena + c->plan.mat[i].zw[3];
  return c->set_ext(EXT_OMEGA, own.data(), s);
}

int lordo_refresh_subspace(lordo_ctx* c, const void* const* Src, int32_t src_dtype, const void* const* Omega, void* stream) {
  if (!c || !Src) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (src_dtype != LORDO_BF16 && src_dtype != LORDO_F32) return LORDO_EINVAL;
  for (int i = 0; i < c->n; ++i)
    if (Omega && Src[i] && !Omega[i]) return LORDO_EINVAL;      // (a matrix that is left out needs no start block)
  if (c->grad_folded) return LORDO_ESTATE;          // the error buffer holds a folded gradient: a local step must consume it first
  if (c->hp.uplink_buffer && c->window_steps > 0) return LORDO_ESTATE;   // the buffer is in coordinates of the current Q
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  // a NULL source leaves that matrix out: its projection, moments and similarity value stay as they are
  int live = 0;
  for (int i = 0; i < c->n; ++i) live += Src[i] != nullptr;
  if (live == 0) return LORDO_OK;
  const bool some_null = live < c->n;
  int rc = c->set_ext(EXT_SRC, const_cast<void* const*>(reinterpret_cast<const void* const*>(Src)), s, true);
  if (rc != LORDO_OK) return rc;
  c->dev.skip_null = some_null ? 1 : 0;             // (before the start blocks are drawn: none for a matrix left out)
  rc = select_omega(c, Omega, s);
  SrcPaths sp{};
  if (rc == LORDO_OK) rc = source_paths(c, Src, src_dtype, s, sp);
  if (rc == LORDO_OK) rc = run_refresh(c, src_dtype, s, false, 0.0, sp.proj_kernels, sp.stream_kernel, sp.proj_tr);
  c->dev.skip_null = 0;
  return rc;
}

int lordo_spectral_gap(lordo_ctx* c, const void* const* Src, int32_t src_dtype, const void* const* Omega, float* dev_out, void* stream) {
  if (!c || !Src || !Omega || !dev_out) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (src_dtype != LORDO_BF16 && src_dtype != LORDO_F32) return LORDO_EINVAL;
  if (!c->hp.rayleigh_ritz || !c->refreshed || c->grad_folded) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  int rc = c->set_ext(EXT_SRC, const_cast<void* const*>(reinterpret_cast<const void* const*>(Src)), s);
  if (rc != LORDO_OK) return rc;
  rc = c->set_ext(EXT_OMEGA, const_cast<void* const*>(reinterpret_cast<const void* const*>(Omega)), s);
  if (rc != LORDO_OK) return rc;
  SrcPaths sp;
  rc = source_paths(c, Src, src_dtype, s, sp);
  if (rc != LORDO_OK) return rc;
  c->prof.begin(LORDO_K_REFRESH, s);
  rc = run_ops(c, c->plan.gap_ops, src_dtype, s, false, 1.0, 1.0, sp.proj_kernels, sp.stream_kernel, sp.proj_tr);
  if (rc == LORDO_OK && launch_stable_rank(c->dev, dev_out, 1, s) != hipSuccess) rc = LORDO_EHIP;
  if (rc != LORDO_OK) { c->prof.abandon(LORDO_K_REFRESH); return rc; }
  c->prof.end(LORDO_K_REFRESH, s);
  return LORDO_OK;
}

int lordo_refresh_subspace_local(lordo_ctx* c, const void* const* G, double grad_scale, const void* const* Omega, void* stream) {
  if (!c || !G || !std::isfinite(grad_scale)) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (lordo_ctx::has_null(G, c->n) || (Omega && lordo_ctx::has_null(Omega, c->n))) return LORDO_EINVAL;
  if (c->hp.err_dtype == LORDO_BF16) return LORDO_EINVAL;      // the sum s G + E is formed inside the residual buffer: fp32 only
  if (!c->hp.error_feedback || c->grad_folded) return LORDO_ESTATE;
  if (c->hp.uplink_buffer && c->window_steps > 0) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  Plan& P = c->plan;
  int rc = c->set_ext(EXT_G, const_cast<void* const*>(reinterpret_cast<const void* const*>(G)), s);
  if (rc != LORDO_OK) return rc;
  rc = select_omega(c, Omega, s);
  if (rc != LORDO_OK) return rc;
  std::vector<void*> src(c->n);
  for (int i = 0; i < c->n; ++i) src[i] = c->dev.arena + P.mat[i].err;
  rc = c->set_ext(EXT_SRC, src.data(), s);
  if (rc != LORDO_OK) return rc;
  bool proj_kernels = P.down_pipe != 0 && !P.any_tr;   // the residual is 256-byte aligned; pairs of columns need an even q
  for (int i = 0; i < c->n && proj_kernels; ++i)
    if ((P.mat[i].q & 1) != 0) proj_kernels = false;
  rc = run_refresh(c, LORDO_F32, s, true, grad_scale, proj_kernels, false);
  if (rc != LORDO_OK) return rc;
  // only a refresh that was enqueued in full commits the context to the step that consumes the folded buffer
  c->grad_folded = true;
  c->folded_g.assign(G, G + c->n);
  return LORDO_OK;
}

int lordo_init_projection(lordo_ctx* c, const void* const* Block, void* stream) {
  if (!c) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (Block && lordo_ctx::has_null(Block, c->n)) return LORDO_EINVAL;
  if (c->t != 0 || c->grad_folded) return LORDO_ESTATE;      // the moments would have to be rotated: that is what a refresh does
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (Block) {
    int rc = c->set_ext(EXT_DIN, const_cast<void* const*>(reinterpret_cast<const void* const*>(Block)), s);
    if (rc != LORDO_OK) return rc;
  }
  c->gauss_init = Block == nullptr;              // no block: the program's first op draws a Gaussian one from hp.seed
  const int rc = run_ops(c, c->plan.init_ops, LORDO_F32, s, false, 1.0, 1.0, false, false);
  if (c->gauss_init) ++c->draws;
  c->gauss_init = false;
  return rc;
}

int lordo_export_pseudograd(lordo_ctx* c, const void* const* W, void* const* DeltaOut, void* stream) {
  if (!c || !W || !DeltaOut) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  int rc = c->set_ext(EXT_W, const_cast<void* const*>(reinterpret_cast<const void* const*>(W)), s);
  if (rc != LORDO_OK) return rc;
  rc = c->set_ext(EXT_DOUT, DeltaOut, s);
  if (rc != LORDO_OK) return rc;
  c->prof.begin(LORDO_K_EXPORT, s);
  HIPCHK(launch_export_delta(c->dev, c->at<int64_t>(c->plan.chunk_start), c->plan.nchunks, c->hp.param_dtype == LORDO_BF16, s));
  c->prof.end(LORDO_K_EXPORT, s);
  return LORDO_OK;
}

int lordo_outer_step(lordo_ctx* c, void* const* W, const void* const* AvgDelta, void* stream) {
  if (!c || !W) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (lordo_ctx::has_null(reinterpret_cast<const void* const*>(W), c->n) || (AvgDelta && lordo_ctx::has_null(AvgDelta, c->n))) return LORDO_EINVAL;
  // this worker's own pseudo-gradient exists only after local steps: none since the last outer step is a caller error
  if (!AvgDelta && c->window_steps == 0) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  int rc = c->set_ext(EXT_W, W, s);
  if (rc != LORDO_OK) return rc;
  OuterArgs a;
  a.lr = (float)c->hp.outer_lr;
  a.mu = (float)c->hp.outer_momentum;
  a.nesterov = c->hp.outer_nesterov ? 1 : 0;
  a.has_mom = c->hp.outer_momentum != 0.0 ? 1 : 0;
  a.own_delta = AvgDelta ? 0 : 1;
  a.w_bf16 = c->hp.param_dtype == LORDO_BF16 ? 1 : 0;
  if (AvgDelta) {
    rc = c->set_ext(EXT_DIN, const_cast<void* const*>(reinterpret_cast<const void* const*>(AvgDelta)), s);
    if (rc != LORDO_OK) return rc;
  }
  c->prof.begin(LORDO_K_OUTER, s);
  HIPCHK(launch_outer(c->dev, c->at<int64_t>(c->plan.chunk_start), c->plan.nchunks, a, s));
  if (c->hp.uplink_buffer) HIPCHK(launch_fill_zero(c->at<void>(c->plan.acc), sizeof(float) * c->plan.lr_total, s));
  c->prof.end(LORDO_K_OUTER, s);
  c->window_steps = 0;
  return LORDO_OK;
}

int lordo_export_uplink(lordo_ctx* c, void* const* AccOut, void* stream) {
  if (!c || !AccOut) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (!c->hp.uplink_buffer) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  int rc = c->set_ext(EXT_DOUT, AccOut, s);
  if (rc != LORDO_OK) return rc;
  c->prof.begin(LORDO_K_EXPORT, s);
  HIPCHK(launch_lr_exchange(c->dev, c->at<float>(c->plan.acc), true, s));
  c->prof.end(LORDO_K_EXPORT, s);
  return LORDO_OK;
}

int lordo_sync_payload(lordo_ctx* c, void** dev_ptr, size_t* count, size_t* moments_count) {
  if (!c || !dev_ptr || !count) return LORDO_EINVAL;
  const Plan& P = c->plan;
  const size_t lr = (size_t)P.lr_total;
  // the three flat arrays were taken from the arena back to back (their sizes are multiples of the arena's granule)
  if (P.v != P.u + (int64_t)(sizeof(float) * lr) || (c->hp.uplink_buffer && P.acc != P.v + (int64_t)(sizeof(float) * lr)))
    return LORDO_ESTATE;
  *dev_ptr = c->at<void>(P.u);
  *count = lr * (c->hp.uplink_buffer ? 3 : 2);
  if (moments_count) *moments_count = lr * 2;
  return LORDO_OK;
}

int lordo_outer_step_lowrank(lordo_ctx* c, void* const* W, const void* const* AvgAcc, void* stream) {
  if (!c || !W) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (!c->hp.uplink_buffer) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  Plan& P = c->plan;
  int rc = c->set_ext(EXT_W, W, s);
  if (rc != LORDO_OK) return rc;
  if (AvgAcc) {
    rc = c->set_ext(EXT_DIN, const_cast<void* const*>(reinterpret_cast<const void* const*>(AvgAcc)), s);
    if (rc != LORDO_OK) return rc;
  }
  bool w_vec = true;            // rows of W of a multiple of 4 floats (a right-projected matrix: its p is the row length)
  for (int i = 0; i < c->n; ++i)
    if (((P.mat[i].tr ? P.mat[i].p : P.mat[i].q) & 3) != 0 || (reinterpret_cast<uintptr_t>(W[i]) & 15) != 0) { w_vec = false; break; }
  // Delta = Q A through the up-projection kernel: the left-projected matrices, then the right-projected ones on their
  // shadow records (planes of A in the place of N as A operand, planes of Q as B operand)
  auto up_all = [&](const UpArgs& ua) -> hipError_t {
    hipError_t e = hipSuccess;
    if (!P.up_h.empty())
      e = launch_proj_up(c->dev, c->at<ProjTile>(P.up_tiles), (int)P.up_h.size(), w_vec, c->at<uint16_t>(P.n_hi), c->at<uint16_t>(P.n_lo), ua, s);
    if (e == hipSuccess && P.any_tr) {
      DevCtx du = c->dev;
      du.mats = c->at<MatDev>(P.mats_up);
      e = launch_proj_up(du, c->at<ProjTile>(P.up_tr_tiles), (int)P.up_tr_h.size(), w_vec, reinterpret_cast<uint16_t*>(c->dev.arena),
                         reinterpret_cast<uint16_t*>(c->dev.arena + P.tr_plane_gap), ua, s);
    }
    return e;
  };
  OuterArgs a;
  a.lr = (float)c->hp.outer_lr;
  a.mu = (float)c->hp.outer_momentum;
  a.nesterov = c->hp.outer_nesterov ? 1 : 0;
  a.has_mom = c->hp.outer_momentum != 0.0 ? 1 : 0;
  a.own_delta = 0;
  a.w_bf16 = 0;               // (the up-link buffer is refused with bf16 weights)
  const int64_t* chunks = c->at<int64_t>(P.chunk_start);
  c->prof.begin(LORDO_K_OUTER, s);
  // the averaged buffer replaces this worker's own (which the step clears anyway); its bf16 hi / lo planes
  // take the place of N as B operand of the up-projection kernel: Delta = Q A (App. A.5.1)
  if (AvgAcc) HIPCHK(launch_lr_exchange(c->dev, c->at<float>(P.acc), false, s));
  HIPCHK(launch_split_planes(c->at<float>(P.acc), c->at<uint16_t>(P.n_hi), c->at<uint16_t>(P.n_lo), P.lr_total, s));
  UpArgs ua{};
  ua.coef_g = 0.f; ua.colscale = 0; ua.colpart = nullptr; ua.g_is_f32 = 0; ua.eps = 0.f;
  ua.target_err = 0;
  if (w_vec) {
    // one pass: Delta = Q A stays in the accumulators of the up-projection kernel, whose epilogue reads the
    // anchor and the momentum and writes W, the anchor and the momentum
    ua.outer = 1; ua.nesterov = a.nesterov; ua.has_mom = a.has_mom; ua.mu = a.mu;
    ua.coef_acc = (float)-c->hp.outer_lr;
    HIPCHK(up_all(ua));
    HIPCHK(launch_fill_zero(c->at<void>(P.acc), sizeof(float) * P.lr_total, s));
    c->prof.end(LORDO_K_OUTER, s);
    c->window_steps = 0;
    return LORDO_OK;
  }
  // any q, any alignment of W: b' = mu b + Delta, W' = anchor - eta_s (Delta + mu b') or anchor - eta_s b' in
  // separate passes -- the part without Delta elementwise, then Delta through the fallback up-projection
  // kernel into W and into b, then anchor <- W
  HIPCHK(launch_outer_base(c->dev, chunks, P.nchunks, a, s));
  ua.coef_acc = (float)(-c->hp.outer_lr * ((a.has_mom && a.nesterov) ? 1.0 + c->hp.outer_momentum : 1.0));
  HIPCHK(up_all(ua));
  if (a.has_mom) {
    ua.target_err = 2;
    ua.coef_acc = 1.f;
    HIPCHK(up_all(ua));
  }
  HIPCHK(launch_anchor_from_w(c->dev, chunks, P.nchunks, false, s));
  HIPCHK(launch_fill_zero(c->at<void>(P.acc), sizeof(float) * P.lr_total, s));
  c->prof.end(LORDO_K_OUTER, s);
  c->window_steps = 0;
  return LORDO_OK;
}

int lordo_get_state(lordo_ctx* c, int32_t mat, int32_t which, void* dev_dst, void* stream) {
  if (!c || !dev_dst || mat < 0 || mat >= c->n) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const MatDev& m = c->plan.mat[mat];
  Plan& P = c->plan;
  float* dst = reinterpret_cast<float*>(dev_dst);
  switch (which) {
    case LORDO_STATE_Q: HIPCHK(launch_copy_f32(dst, c->at<float>(m.q32), (int64_t)m.p * m.r, s)); break;
    case LORDO_STATE_ANCHOR: HIPCHK(launch_copy_f32(dst, c->at<float>(m.anchor), (int64_t)m.p * m.q, s)); break;
    case LORDO_STATE_MOM:
      if (m.mom < 0) return LORDO_ESTATE;
      HIPCHK(launch_copy_f32(dst, c->at<float>(m.mom), (int64_t)m.p * m.q, s));
      break;
    case LORDO_STATE_ERR:
      if (m.err < 0 || c->grad_folded) return LORDO_ESTATE;      // folded: the buffer holds G + E until the next local step
      if (c->hp.err_dtype == LORDO_BF16) HIPCHK(launch_bf16_to_f32(dst, c->at<uint16_t>(m.err), (int64_t)m.p * m.q, s));
      else HIPCHK(launch_copy_f32(dst, c->at<float>(m.err), (int64_t)m.p * m.q, s));
      break;
    case LORDO_STATE_UPLINK:
      if (P.acc < 0) return LORDO_ESTATE;
      HIPCHK(launch_lr_to_plain(c->dev, mat, c->at<float>(P.acc), nullptr, nullptr, dst, 1, 0, s));
      break;
    case LORDO_STATE_RITZ:
      if (m.ritz < 0 || !c->refreshed) return LORDO_ESTATE;
      HIPCHK(launch_copy_f32(dst, c->at<float>(m.ritz), (int64_t)m.r, s));
      break;
    case LORDO_STATE_U: HIPCHK(launch_lr_to_plain(c->dev, mat, c->at<float>(P.u), nullptr, nullptr, dst, 1, 0, s)); break;
    case LORDO_STATE_V: HIPCHK(launch_lr_to_plain(c->dev, mat, c->at<float>(P.v), nullptr, nullptr, dst, 1, 0, s)); break;
    case LORDO_STATE_GLOW:
      HIPCHK(launch_lr_to_plain(c->dev, mat, c->at<float>(P.glow), nullptr, nullptr, dst, P.splits[mat], P.lr_total, s));
      break;
    case LORDO_STATE_NUPD:
      HIPCHK(launch_lr_to_plain(c->dev, mat, nullptr, c->at<uint16_t>(P.n_hi), c->at<uint16_t>(P.n_lo), dst, 1, 0, s));
      break;
    default: return LORDO_EINVAL;
  }
  return LORDO_OK;
}

int lordo_set_state(lordo_ctx* c, int32_t mat, int32_t which, const void* dev_src, void* stream) {
  if (!c || !dev_src || mat < 0 || mat >= c->n) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const MatDev& m = c->plan.mat[mat];
  Plan& P = c->plan;
  const float* src = reinterpret_cast<const float*>(dev_src);
  switch (which) {
    case LORDO_STATE_Q:
      HIPCHK(launch_copy_f32(c->at<float>(m.q32), src, (int64_t)m.p * m.r, s));
      HIPCHK(launch_pack_q(c->dev, mat, 1, s));
      break;
    case LORDO_STATE_ANCHOR: HIPCHK(launch_copy_f32(c->at<float>(m.anchor), src, (int64_t)m.p * m.q, s)); break;
    case LORDO_STATE_MOM:
      if (m.mom < 0) return LORDO_ESTATE;
      HIPCHK(launch_copy_f32(c->at<float>(m.mom), src, (int64_t)m.p * m.q, s));
      break;
    case LORDO_STATE_ERR:
      if (m.err < 0 || c->grad_folded) return LORDO_ESTATE;
      if (c->hp.err_dtype == LORDO_BF16) HIPCHK(launch_f32_to_bf16(c->at<uint16_t>(m.err), src, (int64_t)m.p * m.q, s));
      else HIPCHK(launch_copy_f32(c->at<float>(m.err), src, (int64_t)m.p * m.q, s));
      break;
    case LORDO_STATE_UPLINK:
      if (P.acc < 0) return LORDO_ESTATE;
      HIPCHK(launch_plain_to_lr(c->dev, mat, c->at<float>(P.acc), src, s));
      break;
    case LORDO_STATE_U: HIPCHK(launch_plain_to_lr(c->dev, mat, c->at<float>(P.u), src, s)); break;
    case LORDO_STATE_V: HIPCHK(launch_plain_to_lr(c->dev, mat, c->at<float>(P.v), src, s)); break;
    default: return LORDO_EINVAL;
  }
  return LORDO_OK;
}

int lordo_get_mssv(lordo_ctx* c, float* dev_out, void* stream) {
  if (!c || !dev_out) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (!c->refreshed) return LORDO_ESTATE;
  HIPCHK(launch_mssv(c->dev, dev_out, reinterpret_cast<hipStream_t>(stream)));
  return LORDO_OK;
}

int lordo_get_stable_rank(lordo_ctx* c, float* dev_out, void* stream) {
  if (!c || !dev_out) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  if (!c->refreshed || !c->hp.rayleigh_ritz) return LORDO_ESTATE;
  HIPCHK(launch_stable_rank(c->dev, dev_out, 0, reinterpret_cast<hipStream_t>(stream)));
  return LORDO_OK;
}

int lordo_get_step(lordo_ctx* c, int64_t* t) {
  if (!c || !t) return LORDO_EINVAL;
  *t = c->t;
  return LORDO_OK;
}

int lordo_set_step(lordo_ctx* c, int64_t t) {
  if (!c || t < 0) return LORDO_EINVAL;
  c->t = t;
  c->step_dirty = true;          // the device copy follows at the head of the next call that uses it
  return LORDO_OK;
}

int lordo_poll_status(lordo_ctx* c, void* stream) {
  if (!c) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  HIPCHK(hipStreamSynchronize(s));
  int32_t flag = 0;
  HIPCHK(hipMemcpy(&flag, c->dev.flag, sizeof(flag), hipMemcpyDeviceToHost));
  if (flag != 0) {
    HIPCHK(launch_fill_zero(c->dev.flag, 256, s));
    HIPCHK(hipStreamSynchronize(s));
    return LORDO_ENUMERIC;
  }
  return LORDO_OK;
}

int lordo_profile_enable(lordo_ctx* c, int32_t on) {
  if (!c) return LORDO_EINVAL;
  c->prof.clear();
  c->prof.on = on != 0;
  return LORDO_OK;
}

int lordo_profile_read(lordo_ctx* c, int32_t kernel_class, double* total_ms, int64_t* launches, void* stream) {
  if (!c || !total_ms || !launches || kernel_class < 0 || kernel_class >= NUM_KCLASS) return LORDO_EINVAL;
  if (!c->on_its_device()) return LORDO_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  HIPCHK(hipStreamSynchronize(s));
  Profiler& pf = c->prof;
  pf.abandon(kernel_class);                       // (only a failed call leaves a span open)
  // completed spans are folded into the running sums and their events reused, so a long profiled run holds a
  // bounded number of events
  for (auto& pr : pf.spans[kernel_class]) {
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, pr.first, pr.second));
    pf.sum_ms[kernel_class] += ms;
    ++pf.count[kernel_class];
    pf.pool.push_back(pr.first);
    pf.pool.push_back(pr.second);
  }
  pf.spans[kernel_class].clear();
  *total_ms = pf.sum_ms[kernel_class];
  *launches = pf.count[kernel_class];
  return LORDO_OK;
}

const char* lordo_strerror(int code) {
  switch (code) {
    case LORDO_OK: return "ok";
    case LORDO_EINVAL: return "invalid argument (null pointer, bad shape, rank > rows, unsupported option)";
    case LORDO_ENOMEM: return "arena smaller than lordo_workspace_bytes";
    case LORDO_EHIP: return "HIP runtime error or no GPU";
    case LORDO_ESTATE: return "call not valid in the current state";
    case LORDO_ENUMERIC: return "numerical breakdown in a kernel (non-positive Cholesky pivot)";
    default: return "unknown error";
  }
}

void lordo_destroy(lordo_ctx* c) {
  if (c && c->static_device >= 0) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    g_static_busy[c->static_device] = false;
  }
  delete c;
}

}  // extern "C"
