// Device-side data layout of the Fira step: per-matrix tables that live in the caller's slab,
// work-list entries, and small numeric helpers.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned short bf16_raw;  // storage of one bf16 value

// Pointers read out of the device tables are generic; the kernels cast them to the global address
// space so that loads and stores are global_* instructions (flat_* would also tick the LDS counter).
#define FIRA_GLOBAL __attribute__((address_space(1)))
template <typename T>
using gptr = FIRA_GLOBAL T*;
template <typename T>
__device__ __forceinline__ gptr<T> as_global(T* p) { return (gptr<T>)p; }
// vector types with element alignment only: rows of W and G start at any element (odd n, odd ld)
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 __attribute__((aligned(2))) u32x4_a2;
typedef f32x4 __attribute__((aligned(4))) f32x4_a4;

// K-expansion used for fp32 matrices: an fp32 value x is split as x = h + m + l with h, m, l bf16,
// and a product a*b is summed over the six (a-part, b-part) pairs below, which keeps ~2^-24
// relative accuracy on the bf16 MFMA pipe.  "Data" operands (G, R, N, Z) use sequence A,
// projector operands use sequence B; position p of A meets position p of B in the contraction.
//   A: h h m h l m        B: h m h l h m
#define FIRA_KX_SPLIT 6
#define FIRA_ZREADY_MAX_R 1024

// Immutable description of one weight matrix (device array, one element per matrix).
struct FiraMat {
  int m, n, r, left;   // left = (m <= n): P multiplies from the left, one factor per column
  long long ld;        // leading dimension of W and G, elements
  int L, S;            // long side max(m,n) (number of factors), short side min(m,n)
  int rp, Sp;          // rank and short side rounded up to 64 (zero padded operand rows)
  int kx, dtype;       // K-expansion (1: bf16, 6: fp32 split); dtype of W and G (0 f32, 1 bf16)
  long long gx_ld;     // leading dimension of the split copy of G (fp32 matrices only)
  // The library's own bf16 operand arrays are stored K-blocked, [K/32][rows][32]: the 32 k of one
  // row are 64 contiguous bytes and consecutive rows follow each other, so the 16 rows x 32 k that
  // one LDS-direct load instruction moves are 1 KB of contiguous memory (see kblk_index).  Row
  // counts are rounded up to 256, a whole tile, so tile loads need no clamping; padding is zero.
  int Lq;              // rows of Nb and Rb: L rounded up to 256
  int Sq;              // rows of Pn: S rounded up to 256
  int rq;              // rows of PT: r rounded up to 256
  // 1: the Adam kernel keeps a factor's row in registers and writes Z for c = 1 directly (bf16
  // matrices with r a multiple of 4, up to FIRA_ZREADY_MAX_R); the Z kernel then only corrects
  // the matrices whose limiter factor came out below 1.
  int zready;
  // low-rank arrays, all "long-side major": row i holds the r values of factor i
  float* M;            // [L][r]   first moment
  float* V;            // [L][r]   second moment
  float* Rt;           // [L][r]   low-rank gradient of this step (scratch)
  float* phi;          // [L]      scaling factors k_i of this step
  float* g2;           // [L]      ||G_i||^2 (Gram mode)
  float* q;            // [L]      k_i^2 (||G_i||^2 - ||R_i||^2), the terms of ||S||^2 (Gram mode)
  bf16_raw* Nb;        // [kx*rp/32][Lq][32] Z = N - c k_i R_i of this step (MFMA operand); bf16 matrices have room for a
                       // second plane of K blocks, Z's rounding remainder, used when FiraHp::zsplit is set
  bf16_raw* Rb;        // [kx*rp/32][Lq][32] R of this step as MFMA operand (residual route)
  bf16_raw* Pn;        // [kx*rp/32][Sq][32] projector, rank along K (operand of the back-projection)
  bf16_raw* PT;        // [kx*Sp/32][rq][32] projector transposed, short side along K (operand of R)
  bf16_raw* Gx;        // fp32 matrices: split copy of G ([kx*Sp][gx_ld] if left, [m][gx_ld] else)
};

// Element (row, k) of a K-blocked operand with `rows` (padded) rows.
__host__ __device__ __forceinline__ long long kblk_index(int rows, long long row, int k) {
  return ((long long)(k >> 5) * rows + row) * 32 + (k & 31);
}

// Mutable per-matrix scalars (device array).
struct FiraScal {
  double s_prev;   // ||S_{t-1}|| (after limiting)
  double s_pre;    // ||S_t|| before limiting, last step
  double s_post;   // ||S_t|| after limiting, last step
  float c;         // limiter factor of the current step
  int has_prev;    // 0 until the first step has recorded a norm
  int t;           // steps taken
  float ortho_err; // estimate of ||P^T P - I|| from the last fira_set_projector (first gate of the Gram route)
  // Second gate of the Gram route: relative error of its ||S||^2 against the residual route's, measured on
  // the first step after the projector was installed (that step takes the residual route and has both).
  // +inf until measured.  ||G_i||^2 - ||R_i||^2 cancels when the gradient lies almost entirely in the
  // subspace, and what is left is then the orthonormality defect of the rounded P and fp32 rounding.
  float gram_err;
  int gram_now;    // route of the last step for this matrix: 0 residual, 1 Gram with two kernels, 2 Gram with the fused kernel
  int pad;
};

// One entry of a step's work list.
struct FiraEnt {
  int mat;          // index into FiraMat / FiraScal
  int part0;        // first partial-sum slot of this entry
  int npart;        // number of partial-sum slots
  int row0;         // first row-block (elementwise kernels) of this entry
  int g2b0;         // first block of the ||G_i||^2 kernel of this entry
  int pad;
  void* W;
  const void* G;
};

// One GEMM tile of a grouped launch.
struct FiraTile {
  int ent;  // work-list entry
  int ta;   // tile index along the MFMA A side (long side for R; n for the back-projection)
  int tb;   // tile index along the MFMA B side (rank for R; m for the back-projection)
  int part; // partial-sum slot (residual-norm kernel)
};

struct FiraHp {     // hyper-parameters as the kernels take them
  double beta1, beta2, eps, gamma;
  float b1, b2, omb1, omb2, epsf;
  const float* lr_alpha;   // device address of lr * alpha (fira_set_hparams rewrites it in stream order, so a
                           // learning-rate schedule reaches a step that replays from a HIP graph)
  int scaling;      // 0 column, 1 matrix, 2 none
  int norm_mode;    // 0: ||S|| from the residual tiles; 1: from ||G_i||^2 - ||R_i||^2 where P passes the gate
  float ortho_tol;  // gate of the Gram mode on FiraScal::ortho_err
  float gram_tol;   // ... and on FiraScal::gram_err
  int mixed;        // 1: the fused kernel serves the matrices on the Gram route, the two-kernel path the others
  int zsplit;       // 1: Z of the register-resident Adam rows is stored as two bf16 planes, hi + lo (K = 2 rp)
  int variant;      // 0: Algorithm 1; 1: factors on the full gradient, no Adam term ("Fira-only-scaling")
  int fused;        // 1: this step's projection and Adam ran as one kernel (no copy of R exists)
};

// Whether matrix `sc` takes the Gram route to ||S||^2 in this step.
// (The only-scaling variant needs ||G diag(k)||^2 = sum_i k_i^2 ||G_i||^2, which is this route's data
// without any condition on P.)
__device__ __forceinline__ bool use_gram(const FiraHp& hp, const FiraScal& sc) {
  return hp.variant == 1 || (hp.norm_mode == 1 && sc.ortho_err <= hp.ortho_tol && sc.gram_err <= hp.gram_tol);
}
// Whether ||G_i||^2 is computed in this step (every listed matrix, whatever its route: the step that
// measures FiraScal::gram_err needs both routes' data).
__device__ __forceinline__ bool have_g2(const FiraHp& hp) { return hp.variant == 1 || hp.norm_mode == 1; }
// Whether this step measures FiraScal::gram_err for matrix `sc`: Gram mode, P passes the first gate, the
// step takes the residual route, and no measurement has been made since the projector was installed.
__device__ __forceinline__ bool calibrates_gram(const FiraHp& hp, const FiraScal& sc) {
  return hp.variant == 0 && hp.norm_mode == 1 && sc.ortho_err <= hp.ortho_tol && !(sc.gram_err < INFINITY);
}


// ---- tile geometry shared by the kernels and the host planner -----------------------------------
#define FIRA_PA 128          // projection: tile rows on the gradient (long) side
#define FIRA_PB 256          // projection: tile rows on the rank side
#define FIRA_PS 64           // projection at small ranks (r <= 64): rank columns of the tile
#define FIRA_BA 256          // rank-axis contractions (back-projection): tile rows on the A side (n)
#define FIRA_BB 128          // ... and on the B side (m)
#define FIRA_ROWS_PER_WG 16  // Adam pass: 4 wavefronts x 4 rows
#define FIRA_G2_ROWS_PER_WG 32   // ||G_i||^2 kernel, right orientation: rows per workgroup (8 per wavefront)
#define FIRA_FUSE_MAX_R 512  // largest rank of the fused projection/Adam kernel
#define FIRA_FUSE_MIN_R 128  // below half a rank tile its epilogue works mostly on padding; the two-kernel path is faster
#define FIRA_ORTHO_SPLITS 64 // workgroups of the orthonormality estimate's second phase
#define FIRA_SOLVE_JB 64     // projector refresh: column block of the triangular solve

// One list entry of the projector refresh (device array in the caller's workspace).
struct FiraRefreshEnt {
  int S, L, r, left;   // short side, long side, rank, orientation of the real matrix
  int Lp;              // L rounded up to 64: contraction length of the packed operand
  int rq;              // r rounded up to 256: rows of the packed operand
  int mat;
  int q_dtype;         // element type of Q when it is installed as the projector (0 fp32, 1 bf16: a caller's array)
  const float* T;      // [L][r]            the matrix's Rt
  bf16_raw* Top;       // [Lp/32][rq][32]   T transposed, K-blocked along the long side
  float* Y;            // [S][r]
  float* Q;            // [S][r]
  double* C;           // [r][r]            Gram matrix, then its Cholesky factor (lower triangle)
  float* inst;         // scratch: inverses of the solve's diagonal blocks ([r/64][64][64] fp64), later the
                       // orthonormality estimate's [S][4] and [FIRA_ORTHO_SPLITS][r][4]
  int* done;           // second orthonormalisation pass only (else null): set to 1 by the check of its Gram matrix when
                       // the basis it was given (Y) is orthonormal already; the pass's other kernels then leave, and
                       // the installation takes Y instead of Q
  float done_tol;      // ... when max |Y^T Y - I| is at most this
  int pad1;
};


// ---- bf16 helpers ---------------------------------------------------------------------------
// fp32 -> bf16, nearest even (v_cvt_pk_bf16_f32: one instruction for two values; NaN stays NaN)
__device__ __forceinline__ bf16_raw f32_to_bf16(float x) { return __builtin_bit_cast(bf16_raw, (__bf16)x); }
__device__ __forceinline__ float bf16_to_f32(bf16_raw b) { return __uint_as_float(((unsigned)b) << 16); }
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2_v __attribute__((ext_vector_type(2)));
  typedef float f32x2_v __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2_v{lo, hi}, bf16x2_v));
}
__device__ __forceinline__ void split3(float x, bf16_raw& h, bf16_raw& m, bf16_raw& l) {
  h = f32_to_bf16(x);
  float r1 = x - bf16_to_f32(h);
  m = f32_to_bf16(r1);
  float r2 = r1 - bf16_to_f32(m);
  l = f32_to_bf16(r2);
}

// XCD-aware mapping of a linear workgroup id onto a logical work index: consecutive workgroup
// ids are dispatched round-robin over the 8 XCDs (each with its own L2), so XCD x takes the
// contiguous chunk [x*per, (x+1)*per) of the logical order; neighbours in that order (which share
// operand panels) then share an L2.  Returns -1 for padding workgroups.
__device__ __forceinline__ int xcd_chunked_index(int bid, int total) {
  int per = (total + 7) >> 3;
  int idx = (bid & 7) * per + (bid >> 3);
  return (bid >> 3) < per && idx < total ? idx : -1;
}
