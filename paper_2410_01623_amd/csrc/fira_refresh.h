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

// 64 x 64 tile of a product accumulated in fp64, 256 threads, 4 x 4 outputs per thread.
// A[k][i] and B[k][j] come from row-major arrays with leading dimension r (k is the slow index).
struct RefreshAcc { double v[4][4]; };

// C = Y^T Y (lower triangle tiles only), fp64.
__global__ __launch_bounds__(256) void fira_refresh_gram_kernel(const FiraRefreshEnt* __restrict__ ents) {
  __shared__ float sa[16][64], sb[16][64];
  const FiraRefreshEnt e = ents[blockIdx.y];
  const int nt = (e.r + 63) / 64;
  // linear index -> (ta >= tb)
  int ta = 0, rem = blockIdx.x;
  while (ta < nt && rem > ta) { rem -= ta + 1; ++ta; }
  if (ta >= nt) return;
  const int tb = rem;
  gptr<const float> Y = as_global<const float>(e.Y);
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  RefreshAcc acc;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc.v[i][j] = 0.0;
  for (int s0 = 0; s0 < e.S; s0 += 16) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int sl = (t >> 6) + 4 * p, c = t & 63;
      const int s = s0 + sl;
      const int ca = ta * 64 + c, cb = tb * 64 + c;
      sa[sl][c] = (s < e.S && ca < e.r) ? Y[(long long)s * e.r + ca] : 0.0f;
      sb[sl][c] = (s < e.S && cb < e.r) ? Y[(long long)s * e.r + cb] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int sl = 0; sl < 16; ++sl) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = (double)sa[sl][4 * ty + i]; b[i] = (double)sb[sl][4 * tx + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc.v[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
  gptr<double> C = as_global(e.C);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int ra = ta * 64 + 4 * ty + i, cb = tb * 64 + 4 * tx + j;
      if (ra < e.r && cb < e.r && cb <= ra) C[(long long)ra * e.r + cb] = acc.v[i][j];
    }
}

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
          if (in_lds) {
            a[i] = (i0 + i < r) ? chol_pan[(4 * bi + i) * PP + p] : 0.0;
            b[i] = (k0 + i < r) ? chol_pan[(4 * bk + i) * PP + p] : 0.0;
          } else {
            a[i] = (i0 + i < r) ? C[(long long)(i0 + i) * r + jb + p] : 0.0;
            b[i] = (k0 + i < r) ? C[(long long)(k0 + i) * r + jb + p] : 0.0;
          }
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
    __syncthreads();
  }
}

// Q = Y L^-T, i.e. every row solves  q L^T = y  by forward substitution, done in column blocks of 64:
//     Q_J = (Y_J - Q_{<J} L_{J,<J}^T) inv(L_JJ)^T.
// Everything but the 64 x 64 inverses of the diagonal blocks is a dense product, so the work is tiled like
// the Gram kernel (64 x 64 output tile, fp64 accumulation, 4 x 4 outputs per thread, operands staged through
// LDS): one launch per column block J, in order, each reading the blocks of Q written by the launches
// before it (fp32, as the result is stored).  The inverses of the diagonal blocks come from a small
// kernel of their own (one thread per column of an inverse) and live in the scratch of the installation,
// which is idle until the solves are done.  (Forms that kept a workgroup's rows in LDS and walked along
// the columns, one row per lane with L read from memory or staged in LDS, ran at a tenth of the fp64
// rate: bound by the latency, or the LDS bandwidth, of the operand every lane shares.)
#define FIRA_SOLVE_LDS (16 * 64 * 4 + 16 * 64 * 8 + 64 * 65 * 8 + 64 * 64 * 8)

// inv(L_JJ) for every diagonal block J of a matrix: inv[J][k][c], k >= c (zero above the diagonal).
// Rows and columns beyond r act as an identity.
__global__ __launch_bounds__(64) void fira_refresh_diaginv_kernel(const FiraRefreshEnt* __restrict__ ents) {
  __shared__ double Ld[64][65];
  const FiraRefreshEnt e = ents[blockIdx.y];
  const int r = e.r, j0 = blockIdx.x * FIRA_SOLVE_JB, c = threadIdx.x;
  if (j0 >= r) return;
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
  float (*sa)[64] = reinterpret_cast<float (*)[64]>(solve_lds);                       // [16][64]  Q[s0 + i][k0 + kk]
  double (*sb)[64] = reinterpret_cast<double (*)[64]>(solve_lds + 16 * 64 * 4);        // [16][64]  L[j0 + j][k0 + kk]
  double (*st)[65] = reinterpret_cast<double (*)[65]>(solve_lds + 16 * 64 * 4 + 16 * 64 * 8);   // [64][65] Y_J - update
  double (*invT)[64] = reinterpret_cast<double (*)[64]>(solve_lds + 16 * 64 * 4 + 16 * 64 * 8 + 64 * 65 * 8);   // [c][k]
  const FiraRefreshEnt e = ents[blockIdx.y];
  const int r = e.r, s0 = blockIdx.x * 64, j0 = J * FIRA_SOLVE_JB;
  if (s0 >= e.S || j0 >= r) return;
  gptr<const float> Y = as_global<const float>(e.Y);
  gptr<const double> Lm = as_global<const double>(e.C);
  gptr<float> Q = as_global(e.Q);
  gptr<const double> inv = reinterpret_cast<gptr<const double>>(as_global(e.inst)) + (size_t)J * 64 * 64;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  RefreshAcc acc;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc.v[i][j] = 0.0;
  const int lr = t >> 2, lk = (t & 3) * 4;      // staging: row (or column of the block) lr, four k from lk
  for (int k0 = 0; k0 < j0; k0 += 16) {         // j0 is a multiple of 64: whole tiles, all inside the matrix
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      sa[lk + q][lr] = (s0 + lr < e.S) ? Q[(long long)(s0 + lr) * r + k0 + lk + q] : 0.0f;
      sb[lk + q][lr] = (j0 + lr < r) ? Lm[(long long)(j0 + lr) * r + k0 + lk + q] : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = (double)sa[kk][4 * ty + i]; b[i] = sb[kk][4 * tx + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc.v[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
  // T = Y_J - update, and the inverse of the diagonal block (transposed: invT[c][k] = inv[k][c])
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = 4 * ty + i, col = 4 * tx + j;
      const double y = (s0 + row < e.S && j0 + col < r) ? (double)Y[(long long)(s0 + row) * r + j0 + col] : 0.0;
      st[row][col] = y - acc.v[i][j];
    }
  for (int x = t; x < 64 * 64; x += 256) {
    const int k = x >> 6, c = x & 63;
    invT[c][k] = inv[x];
  }
  __syncthreads();
  // Q_J = T inv^T:  q[row][k] = sum_{c <= k} T[row][c] inv[k][c]
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc.v[i][j] = 0.0;
  for (int c = 0; c < 64; ++c) {
    double a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = st[4 * ty + i][c]; b[i] = invT[c][4 * tx + i]; }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc.v[i][j] += a[i] * b[j];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = 4 * ty + i, k = 4 * tx + j;
      if (s0 + row < e.S && j0 + k < r) Q[(long long)(s0 + row) * r + j0 + k] = (float)acc.v[i][j];
    }
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
  else prep_projector_body<float>(mats[e.mat], e.Q);
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
