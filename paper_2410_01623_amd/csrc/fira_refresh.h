// Projector refresh on the device (Sec. 3.3, Eq. 7 and the "if t mod T = 0" branch of Algorithm 1: every
// T steps P is replaced by the leading r singular vectors of the current gradient, on the short side).
// The paper calls an SVD; only the subspace spanned by the leading vectors enters the step (the step is
// invariant to a rotation of P inside that subspace up to the Adam state's coordinates, which the paper
// resets to nothing: M and V carry over), so the basis is computed by subspace iteration:
//
//     Q <- orth( G G^T Q )   (m <= n),        Q <- orth( G^T G Q )   (m > n),
//
// a fixed number of times from a seeded random start.  The two big products are the projection
// kernel itself: T = (G applied along the short side) is exactly R for the projector Q, and the way
// back is the same kernel run on the other orientation of G with T packed as its K-blocked operand.
// The small dense algebra of the orthonormalisation (CholeskyQR: C = Y^T Y, C = L L^T, Q = Y L^-T by forward substitution) is
// done in fp64 so that it survives gradients with a steep spectrum; the kernels below are plain
// (no MFMA): r^2 S flops per matrix, every listed matrix in one grouped launch.
#pragma once
#include "fira_device.h"


// splitmix64 finaliser: one independent 64-bit value per counter
__device__ __forceinline__ unsigned long long refresh_mix64(unsigned long long z) {
  z += 0x9e3779b97f4a7c15ull;
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}

// Q0: uniform(-1, 1) entries, a function of (seed, matrix, element) only.
__global__ __launch_bounds__(256) void fira_refresh_init_kernel(const FiraRefreshEnt* __restrict__ ents, unsigned long long seed) {
  const FiraRefreshEnt e = ents[blockIdx.y];
  const long long total = (long long)e.S * e.r;
  gptr<float> Q = as_global(e.Q);
  const unsigned long long key = refresh_mix64(seed ^ ((unsigned long long)(unsigned)e.mat << 32));
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const unsigned long long h = refresh_mix64(key + (unsigned long long)i);
    Q[i] = (float)((double)(h >> 11) * (2.0 / 9007199254740992.0) - 1.0);
  }
}

// Top[a][i] = bf16(T[i][a]) in the K-blocked layout; k >= L is zero.  (Rows a >= r stay zero from the
// workspace clear.)  One workgroup per 32 (i) x 64 (a) tile.
__global__ __launch_bounds__(256) void fira_refresh_pack_kernel(const FiraRefreshEnt* __restrict__ ents) {
  __shared__ float tile[32][65];
  const FiraRefreshEnt e = ents[blockIdx.y];
  const int atiles = (e.r + 63) / 64;
  const int ib = blockIdx.x / atiles, ab = blockIdx.x % atiles;
  if (ib * 32 >= e.Lp) return;
  gptr<const float> T = as_global<const float>(e.T);
  const int t = threadIdx.x;
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int il = (t >> 6) + 4 * p, al = t & 63;
    const int i = ib * 32 + il, a = ab * 64 + al;
    tile[il][al] = (i < e.L && a < e.r) ? T[(long long)i * e.r + a] : 0.0f;
  }
  __syncthreads();
  const int al = t >> 2, i8 = (t & 3) * 8;
  const int a = ab * 64 + al;
  if (a < e.r) {
    unsigned w[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) w[d] = pack_bf16x2(tile[i8 + 2 * d][al], tile[i8 + 2 * d + 1][al]);
    gptr<bf16_raw> Top = as_global(e.Top);
    *reinterpret_cast<gptr<u32x4>>(Top + kblk_index(e.rq, a, ib * 32 + i8)) = u32x4{w[0], w[1], w[2], w[3]};
  }
}

// 64 x 64 tile of a product accumulated in fp64 on the matrix pipe (v_mfma_f64_16x16x4_f64): 256 threads, wave w
// owns the 32 x 32 block at rows 32 (w >> 1), columns 32 (w & 1), as 2 x 2 blocks of 16 x 16.  Operand layout of
// the instruction: lane l supplies A[m = l % 16][k = l / 16] and B[k = l / 16][n = l % 16]; of its four result
// values, number v is D[m = l / 16 + 4 v][n = l % 16] (checked on the device against a plain product).  The products are fp64 multiply-adds like the vector
// unit's; the matrix pipe has the same peak on this chip but takes one instruction for 2048 of them, which
// frees the issue slots that the vector form spends on conversions and LDS reads.
typedef double f64x4_t __attribute__((ext_vector_type(4)));
struct RefreshAcc { f64x4_t v[2][2]; };
__device__ __forceinline__ void refresh_acc_zero(RefreshAcc& acc) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc.v[i][j] = f64x4_t{0.0, 0.0, 0.0, 0.0};
}
// K steps [0, KN) of a staged pair of operands: A(k, m) = sa[k * ak + m * am], B(k, n) = sb[k * bk + n * bn],
// m and n counted inside the workgroup's 64 x 64 tile.
template <int KN, typename TA, typename TB>
__device__ __forceinline__ void refresh_acc_steps(RefreshAcc& acc, const TA* sa, int ak, int am, const TB* sb, int bk, int bn) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m0 = 32 * (wave >> 1) + (lane & 15), n0 = 32 * (wave & 1) + (lane & 15), kq = lane >> 4;
#pragma unroll
  for (int k4 = 0; k4 < KN; k4 += 4) {
    const int k = k4 + kq;
    const double a0 = (double)sa[k * ak + m0 * am], a1 = (double)sa[k * ak + (m0 + 16) * am];
    const double b0 = (double)sb[k * bk + n0 * bn], b1 = (double)sb[k * bk + (n0 + 16) * bn];
    acc.v[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc.v[0][0], 0, 0, 0);
    acc.v[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc.v[0][1], 0, 0, 0);
    acc.v[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc.v[1][0], 0, 0, 0);
    acc.v[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc.v[1][1], 0, 0, 0);
  }
}
// Calls f(row, col, value) for every element of the workgroup's tile that this lane holds.
template <typename F>
__device__ __forceinline__ void refresh_acc_foreach(const RefreshAcc& acc, F f) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        f(32 * (wave >> 1) + 16 * i + (lane >> 4) + 4 * v, 32 * (wave & 1) + 16 * j + (lane & 15), acc.v[i][j][v]);
}
#define FIRA_STAGE_LD 80   // floats per staged K row of 64: the four K rows that one load instruction touches fall on distinct banks

// Four consecutive floats of a row-major fp32 array (row `row`, columns col .. col + 3, leading dimension ld,
// `rows` x `cols` valid): one 16-byte load when ld is a multiple of 4 (col is), else element by element.
__device__ __forceinline__ f32x4 refresh_load4(gptr<const float> A, int row, int col, int rows, int cols, int ld) {
  if (row >= rows || col >= cols) return f32x4{0.f, 0.f, 0.f, 0.f};
  gptr<const float> p = A + (long long)row * ld + col;
  if ((ld & 3) == 0) return *reinterpret_cast<gptr<const f32x4>>(p);
  return f32x4{p[0], col + 1 < cols ? p[1] : 0.f, col + 2 < cols ? p[2] : 0.f, col + 3 < cols ? p[3] : 0.f};
}

// C = Y^T Y (lower triangle tiles only), fp64.  K stages of 32 rows; the next stage's rows are requested into
// registers before the current one is multiplied.
#define FIRA_GRAM_KS 32
__global__ __launch_bounds__(256) void fira_refresh_gram_kernel(const FiraRefreshEnt* __restrict__ ents) {
  __shared__ __attribute__((aligned(16))) float sa[FIRA_GRAM_KS * FIRA_STAGE_LD], sb[FIRA_GRAM_KS * FIRA_STAGE_LD];
  const FiraRefreshEnt e = ents[blockIdx.y];
  const int nt = (e.r + 63) / 64;
  // linear index -> (ta >= tb)
  int ta = 0, rem = blockIdx.x;
  while (ta < nt && rem > ta) { rem -= ta + 1; ++ta; }
  if (ta >= nt) return;
  const int tb = rem;
  gptr<const float> Y = as_global<const float>(e.Y);
  const int t = threadIdx.x;
  RefreshAcc acc;
  refresh_acc_zero(acc);
  f32x4 ra[2], rb[2];
  auto fetch = [&](int s0) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int x = t + 256 * p, sl = x >> 4, c4 = (x & 15) * 4;
      ra[p] = refresh_load4(Y, s0 + sl, ta * 64 + c4, e.S, e.r, e.r);
      rb[p] = refresh_load4(Y, s0 + sl, tb * 64 + c4, e.S, e.r, e.r);
    }
  };
  fetch(0);
  for (int s0 = 0; s0 < e.S; s0 += FIRA_GRAM_KS) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int x = t + 256 * p, sl = x >> 4, c4 = (x & 15) * 4;
      *reinterpret_cast<f32x4*>(&sa[sl * FIRA_STAGE_LD + c4]) = ra[p];
      *reinterpret_cast<f32x4*>(&sb[sl * FIRA_STAGE_LD + c4]) = rb[p];
    }
    __syncthreads();
    if (s0 + FIRA_GRAM_KS < e.S) fetch(s0 + FIRA_GRAM_KS);
    refresh_acc_steps<FIRA_GRAM_KS>(acc, sa, FIRA_STAGE_LD, 1, sb, FIRA_STAGE_LD, 1);
    __syncthreads();
  }
  gptr<double> C = as_global(e.C);
  refresh_acc_foreach(acc, [&](int row, int col, double v) {
    const int ra_ = ta * 64 + row, cb = tb * 64 + col;
    if (ra_ < e.r && cb < e.r && cb <= ra_) C[(long long)ra_ * e.r + cb] = v;
  });
}

// Second pass only: is the basis that the pass was given orthonormal already?  max |C - I| over the lower triangle
// of its Gram matrix (just computed) against the entry's tolerance; one workgroup per matrix.
__global__ __launch_bounds__(256) void fira_refresh_orthocheck_kernel(const FiraRefreshEnt* __restrict__ ents) {
  __shared__ double red[4];
  const FiraRefreshEnt e = ents[blockIdx.x];
  if (!e.done) return;
  gptr<const double> C = as_global<const double>(e.C);
  const int r = e.r, t = threadIdx.x;
  double worst = 0.0;
  for (long long x = t; x < (long long)r * r; x += 256) {
    const int i = (int)(x / r), k = (int)(x - (long long)i * r);
    if (k <= i) {
      const double d = fabs(C[x] - (i == k ? 1.0 : 0.0));
      worst = (d > worst || d != d) ? d : worst;      // a NaN stays
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double other = __shfl_xor(worst, o, 64);
    worst = (other > worst || other != other) ? other : worst;
  }
  if ((t & 63) == 0) red[t >> 6] = worst;
  __syncthreads();
  if (t == 0) {
    double w = red[0];
    for (int i = 1; i < 4; ++i) w = (red[i] > w || red[i] != red[i]) ? red[i] : w;
    *as_global(e.done) = (w <= (double)e.done_tol) ? 1 : 0;     // false for a NaN
  }
}
__device__ __forceinline__ bool refresh_pass_done(const FiraRefreshEnt& e) { return e.done && *as_global<const int>(e.done) != 0; }

// In-place Cholesky factorisation of the lower triangle of C (fp64), one workgroup per matrix,
// blocked by 32 columns: factor the diagonal block in LDS, solve the panel below it one row per
// thread, update the trailing triangle from the panel.  A pivot that is not safely positive (Y
// numerically rank deficient) is replaced by a small multiple of the largest diagonal entry, which
// keeps the factor finite; the directions it affects carry no energy of G.
#define FIRA_CHOL_THREADS 512
#define FIRA_CHOL_NB 32
#define FIRA_CHOL_PAN_ROWS 544   // panel rows kept in LDS: 544 x 33 doubles = 140 KB (every panel of a matrix with r <= 576)
__global__ __launch_bounds__(FIRA_CHOL_THREADS) void fira_refresh_chol_kernel(const FiraRefreshEnt* __restrict__ ents, int pan_rows) {
  __shared__ double D[FIRA_CHOL_NB][FIRA_CHOL_NB + 1];
  __shared__ double rinv_s[FIRA_CHOL_NB];
  __shared__ double dmax_s;
  // the panel below the diagonal block, [rows][FIRA_CHOL_NB + 1], while it fits (pan_rows rows of dynamic LDS):
  // the panel solve and the trailing update then read it from LDS instead of walking through memory
  extern __shared__ __attribute__((aligned(16))) double chol_pan[];
  constexpr int PP = FIRA_CHOL_NB + 1;
  const FiraRefreshEnt e = ents[blockIdx.x];
  if (refresh_pass_done(e)) return;
  const int r = e.r, t = threadIdx.x;
  gptr<double> C = as_global(e.C);
  if (t == 0) {
    double mx = 0.0;
    for (int i = 0; i < r; ++i) mx = fmax(mx, C[(long long)i * r + i]);
    dmax_s = mx;
  }
  __syncthreads();
  const double floor_piv = dmax_s * 1e-24 + 1e-300;
  for (int jb = 0; jb < r; jb += FIRA_CHOL_NB) {
    const int nb = min(FIRA_CHOL_NB, r - jb);
    // (1) diagonal block -> LDS, factor with the first 32 threads (column by column)
    for (int x = t; x < nb * nb; x += FIRA_CHOL_THREADS) {
      const int i = x / nb, k = x % nb;
      D[i][k] = (k <= i) ? C[(long long)(jb + i) * r + jb + k] : 0.0;
    }
    __syncthreads();
    if (t < 64) {
      for (int j = 0; j < nb; ++j) {
        // every lane computes the same pivot from LDS
        const double piv = sqrt(fmax(D[j][j], floor_piv));
        const double inv = 1.0 / piv;
        __builtin_amdgcn_wave_barrier();
        if (t == j) D[j][j] = piv;
        if (t > j && t < nb) D[t][j] *= inv;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // trailing update inside the block: row t, columns j+1..t
        if (t > j && t < nb) {
          const double lt = D[t][j];
          for (int k = j + 1; k <= t; ++k) D[t][k] -= lt * D[k][j];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
    __syncthreads();
    for (int x = t; x < nb * nb; x += FIRA_CHOL_THREADS) {
      const int i = x / nb, k = x % nb;
      if (k <= i) C[(long long)(jb + i) * r + jb + k] = D[i][k];
    }
    if (t < nb) rinv_s[t] = 1.0 / D[t][t];
    // (2) panel: rows below the block, X D^T = C_panel  (forward substitution along the block's columns)
    const int below = r - (jb + nb);
    const bool in_lds = below <= pan_rows;
    if (in_lds) {
      for (int x = t; x < below * nb; x += FIRA_CHOL_THREADS) {
        const int i = x / nb, k = x % nb;
        chol_pan[i * PP + k] = C[(long long)(jb + nb + i) * r + jb + k];
      }
      __syncthreads();
      for (int i = t; i < below; i += FIRA_CHOL_THREADS) {
        double* row = chol_pan + i * PP;
        for (int k = 0; k < nb; ++k) {
          double sacc = row[k];
          for (int p = 0; p < k; ++p) sacc -= row[p] * D[k][p];
          row[k] = sacc * rinv_s[k];
        }
      }
      __syncthreads();
      for (int x = t; x < below * nb; x += FIRA_CHOL_THREADS) {
        const int i = x / nb, k = x % nb;
        C[(long long)(jb + nb + i) * r + jb + k] = chol_pan[i * PP + k];
      }
    } else
    for (int i = t; i < below; i += FIRA_CHOL_THREADS) {
      gptr<double> row = C + (long long)(jb + nb + i) * r + jb;
      // the row's own earlier results are read back from memory (a thread sees its own stores)
      for (int k = 0; k < nb; ++k) {
        double sacc = row[k];
        for (int p = 0; p < k; ++p) sacc -= row[p] * D[k][p];
        row[k] = sacc / D[k][k];
      }
    }
    __syncthreads();   // (HIP's barrier also waits for this wave's global stores)
    // (3) trailing triangle: C[i][k] -= sum_p P[i][p] P[k][p],  jb+nb <= k <= i < r,  P = the panel
    if (in_lds && below > 0) {
      // on the matrix pipe: 32 x 32 blocks of the triangle dealt out to the wavefronts, operands from the panel in
      // LDS (rows past the end are clamped to the last row; what they produce is not stored)
      const int lane = t & 63, wave = t >> 6, nb32 = (below + 31) / 32;
      int cnt = 0;
      for (int bi = 0; bi < nb32; ++bi)
        for (int bk = 0; bk <= bi; ++bk, ++cnt) {
          if (cnt % (FIRA_CHOL_THREADS / 64) != wave) continue;
          const int m0 = min(32 * bi + (lane & 15), below - 1), m1 = min(32 * bi + 16 + (lane & 15), below - 1);
          const int n0 = min(32 * bk + (lane & 15), below - 1), n1 = min(32 * bk + 16 + (lane & 15), below - 1);
          RefreshAcc acc;
          refresh_acc_zero(acc);
#pragma unroll
          for (int k4 = 0; k4 < FIRA_CHOL_NB; k4 += 4) {
            const int k = k4 + (lane >> 4);
            const bool kin = k < nb;
            const double a0 = kin ? chol_pan[m0 * PP + k] : 0.0, a1 = kin ? chol_pan[m1 * PP + k] : 0.0;
            const double b0 = kin ? chol_pan[n0 * PP + k] : 0.0, b1 = kin ? chol_pan[n1 * PP + k] : 0.0;
            acc.v[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc.v[0][0], 0, 0, 0);
            acc.v[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc.v[0][1], 0, 0, 0);
            acc.v[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc.v[1][0], 0, 0, 0);
            acc.v[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc.v[1][1], 0, 0, 0);
          }
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int v = 0; v < 4; ++v) {
                const int ri = 32 * bi + 16 * i + (lane >> 4) + 4 * v, ck = 32 * bk + 16 * j + (lane & 15);
                if (ri < below && ck <= ri) C[(long long)(jb + nb + ri) * r + jb + nb + ck] -= acc.v[i][j][v];
              }
        }
    } else {
    const int nt4 = (below + 3) / 4;
    for (int x = t; x < nt4 * nt4; x += FIRA_CHOL_THREADS) {
      const int bi = x / nt4, bk = x % nt4;
      if (bk > bi) continue;
      const int i0 = jb + nb + 4 * bi, k0 = jb + nb + 4 * bk;
      double acc[4][4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[i][k] = 0.0;
      for (int p = 0; p < nb; ++p) {
        double a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a[i] = (i0 + i < r) ? C[(long long)(i0 + i) * r + jb + p] : 0.0;
          b[i] = (k0 + i < r) ? C[(long long)(k0 + i) * r + jb + p] : 0.0;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int k = 0; k < 4; ++k) acc[i][k] += a[i] * b[k];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (i0 + i < r && k0 + k <= i0 + i) C[(long long)(i0 + i) * r + k0 + k] -= acc[i][k];
    }
    }
    __syncthreads();
  }
}

// Q = Y L^-T, i.e. every row solves  q L^T = y  by forward substitution, done in column blocks of 64:
//     Q_J = (Y_J - Q_{<J} L_{J,<J}^T) inv(L_JJ)^T.
// Everything but the 64 x 64 inverses of the diagonal blocks is a dense product, so the work is tiled like
// the Gram kernel (64 x 64 output tile, fp64 on the matrix pipe, operands staged through LDS with the next
// stage's values requested into registers meanwhile): one launch per column block J, in order, each reading the blocks of Q written by the launches
// before it (fp32, as the result is stored).  The inverses of the diagonal blocks come from a small
// kernel of their own (one thread per column of an inverse) and live in the scratch of the installation,
// which is idle until the solves are done.  (Forms that kept a workgroup's rows in LDS and walked along
// the columns, one row per lane with L read from memory or staged in LDS, ran at a tenth of the fp64
// rate: bound by the latency, or the LDS bandwidth, of the operand every lane shares.)
#define FIRA_SOLVE_LDS (16 * 80 * 4 + 16 * 64 * 8 + 64 * 65 * 8 + 64 * 64 * 8)   // staged Q (rows of FIRA_STAGE_LD floats), staged L, T, inverse

// inv(L_JJ) for every diagonal block J of a matrix: inv[J][k][c], k >= c (zero above the diagonal).
// Rows and columns beyond r act as an identity.
__global__ __launch_bounds__(64) void fira_refresh_diaginv_kernel(const FiraRefreshEnt* __restrict__ ents) {
  __shared__ double Ld[64][65];
  const FiraRefreshEnt e = ents[blockIdx.y];
  const int r = e.r, j0 = blockIdx.x * FIRA_SOLVE_JB, c = threadIdx.x;
  if (j0 >= r || refresh_pass_done(e)) return;
  gptr<const double> Lm = as_global<const double>(e.C);
  for (int x = c; x < 64 * 64; x += 64) {
    const int i = x >> 6, k = x & 63;
    const bool in = j0 + i < r && j0 + k < r;
    Ld[i][k] = (in && k <= i) ? Lm[(long long)(j0 + i) * r + j0 + k] : (i == k ? 1.0 : 0.0);
  }
  __syncthreads();
  // column c of the inverse: L x = e_c
  double x[64];
#pragma unroll
  for (int i = 0; i < 64; ++i) {
    double v = (i == c) ? 1.0 : 0.0;
#pragma unroll
    for (int p = 0; p < 64; ++p)
      if (p < i) v -= Ld[i][p] * x[p];
    x[i] = (i < c) ? 0.0 : v / Ld[i][i];
  }
  gptr<double> inv = reinterpret_cast<gptr<double>>(as_global(e.inst)) + (size_t)blockIdx.x * 64 * 64;
#pragma unroll
  for (int i = 0; i < 64; ++i) inv[i * 64 + c] = x[i];
}

// Column block J of Q for 64 rows.
__global__ __launch_bounds__(256) void fira_refresh_solve_kernel(const FiraRefreshEnt* __restrict__ ents, int J) {
  extern __shared__ __attribute__((aligned(16))) char solve_lds[];
  float* sa = reinterpret_cast<float*>(solve_lds);                                   // [16][FIRA_STAGE_LD]  Q[s0 + i][k0 + kk]
  double* sb = reinterpret_cast<double*>(solve_lds + 16 * FIRA_STAGE_LD * 4);        // [16][64]  L[j0 + j][k0 + kk]
  double (*st)[65] = reinterpret_cast<double (*)[65]>(solve_lds + 16 * FIRA_STAGE_LD * 4 + 16 * 64 * 8);   // [64][65] Y_J - update
  double* invT = reinterpret_cast<double*>(solve_lds + 16 * FIRA_STAGE_LD * 4 + 16 * 64 * 8 + 64 * 65 * 8);   // [c][k]
  const FiraRefreshEnt e = ents[blockIdx.y];
  const int r = e.r, s0 = blockIdx.x * 64, j0 = J * FIRA_SOLVE_JB;
  if (s0 >= e.S || j0 >= r || refresh_pass_done(e)) return;
  gptr<const float> Y = as_global<const float>(e.Y);
  gptr<const double> Lm = as_global<const double>(e.C);
  gptr<float> Q = as_global(e.Q);
  gptr<const double> inv = reinterpret_cast<gptr<const double>>(as_global(e.inst)) + (size_t)J * 64 * 64;
  const int t = threadIdx.x;
  RefreshAcc acc;
  refresh_acc_zero(acc);
  const int lr = t >> 2, lk = (t & 3) * 4;      // staging: row (or column of the block) lr, four k from lk
  // (j0 is a multiple of 64: whole tiles along k, all inside the matrix.)  The next stage's values are requested
  // into registers before the current one is multiplied.
  f32x4 rq;
  double rl[4];
  auto fetch = [&](int k0) {
    rq = refresh_load4(Q, s0 + lr, k0 + lk, e.S, r, r);
    if (j0 + lr < r) {
      gptr<const double> pl = Lm + (long long)(j0 + lr) * r + k0 + lk;
      if ((r & 1) == 0) {
        typedef double f64x2_t __attribute__((ext_vector_type(2)));
        const f64x2_t u = *reinterpret_cast<gptr<const f64x2_t>>(pl), w = *reinterpret_cast<gptr<const f64x2_t>>(pl + 2);
        rl[0] = u.x; rl[1] = u.y; rl[2] = w.x; rl[3] = w.y;
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) rl[q] = pl[q];
      }
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) rl[q] = 0.0;
    }
  };
  if (j0 > 0) fetch(0);
  for (int k0 = 0; k0 < j0; k0 += 16) {
    const float qv[4] = {rq.x, rq.y, rq.z, rq.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      sa[(lk + q) * FIRA_STAGE_LD + lr] = qv[q];
      sb[(lk + q) * 64 + lr] = rl[q];
    }
    __syncthreads();
    if (k0 + 16 < j0) fetch(k0 + 16);
    refresh_acc_steps<16>(acc, sa, FIRA_STAGE_LD, 1, sb, 64, 1);   // sum_k Q[row][k] L[j0 + col][k]
    __syncthreads();
  }
  // T = Y_J - update, and the inverse of the diagonal block (transposed: invT[c][k] = inv[k][c])
  refresh_acc_foreach(acc, [&](int row, int col, double v) {
    const double y = (s0 + row < e.S && j0 + col < r) ? (double)Y[(long long)(s0 + row) * r + j0 + col] : 0.0;
    st[row][col] = y - v;
  });
  for (int x = t; x < 64 * 64; x += 256) {
    const int k = x >> 6, c = x & 63;
    invT[c * 64 + k] = inv[x];
  }
  __syncthreads();
  // Q_J = T inv^T:  q[row][k] = sum_{c <= k} T[row][c] inv[k][c]
  refresh_acc_zero(acc);
  refresh_acc_steps<64>(acc, &st[0][0], 1, 65, invT, 64, 1);
  refresh_acc_foreach(acc, [&](int row, int k, double v) {
    if (s0 + row < e.S && j0 + k < r) Q[(long long)(s0 + row) * r + j0 + k] = (float)v;
  });
}

// ------------------------------------------------------------------------------------------------
// Installation of the listed matrices' projectors from their Q buffers, one launch per phase for all
// of them (blockIdx.y = list entry) instead of four launches per matrix: the operand copies Pn / PT
// (fira_prep_projector_kernel) and the estimate of ||P^T P - I|| behind the Gram gate (the three
// fira_ortho_* kernels), each with its own scratch.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fira_refresh_prep_kernel(const FiraMat* __restrict__ mats, const FiraRefreshEnt* __restrict__ ents) {
  const FiraRefreshEnt e = ents[blockIdx.y];
  if (e.q_dtype == 1) prep_projector_body<bf16_raw>(mats[e.mat], reinterpret_cast<const bf16_raw*>(e.Q));
  else prep_projector_body<float>(mats[e.mat], refresh_pass_done(e) ? e.Y : e.Q);   // (a second pass that had nothing to do left its input as the result)
}
__global__ __launch_bounds__(256) void fira_refresh_ortho_y_kernel(const FiraMat* __restrict__ mats, const FiraRefreshEnt* __restrict__ ents) {
  const FiraRefreshEnt e = ents[blockIdx.y];
  if ((int)blockIdx.x * 4 >= e.S) return;
  ortho_y_body(mats[e.mat], e.inst);
}
__global__ __launch_bounds__(256) void fira_refresh_ortho_z_kernel(const FiraMat* __restrict__ mats, const FiraRefreshEnt* __restrict__ ents) {
  const FiraRefreshEnt e = ents[blockIdx.y];
  ortho_z_body(mats[e.mat], e.inst, e.inst + (size_t)e.S * 4);
}
__global__ __launch_bounds__(256) void fira_refresh_ortho_final_kernel(const FiraMat* __restrict__ mats, const FiraRefreshEnt* __restrict__ ents,
                                                                       FiraScal* __restrict__ scal) {
  __shared__ float red[4][4];
  const FiraRefreshEnt e = ents[blockIdx.x];
  ortho_final_body(mats[e.mat], e.inst + (size_t)e.S * 4, scal, e.mat, red);
}
