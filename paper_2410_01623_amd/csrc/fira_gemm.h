// Grouped bf16 MFMA contractions of the Fira step for gfx950 (v_mfma_f32_32x32x16_bf16).
//
// One 256-thread workgroup (4 wavefronts, 2 x 2) computes a 256 x 128 tile
//     D[a][b] = sum_k A[a][k] * B[b][k]
// where "A" is the MFMA A operand (256 rows per tile) and "B" the MFMA B operand (128 rows).
// Both operands are staged through LDS as [row][64 k] bf16 tiles (128 B per row, 16-byte chunks
// XOR-swizzled by row so that fragment reads and tile writes spread over all banks).  An operand is
// either K-contiguous in memory (row pointer + k) or, for the gradient when P multiplies from the
// left, K-slow (element (a, k) at base[k*ld + a]); the K-slow loader reads 8 x 8 blocks with
// row-contiguous 16-byte loads and transposes them in registers before the LDS write.
//
// Accumulator layout of one 32 x 32 block (per lane, 16 floats v = 0..15):
//     b (B row) = lane % 32,   a (A row) = 8*(v/4) + 4*(lane/32) + v%4
// so a lane owns 4 consecutive A rows per group of 4 registers.  The kernels choose which side of
// each product plays A so that this run of 4 lies along the contiguous axis of what they touch.
#pragma once
#include "fira_device.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

#define FIRA_BK 64
#define FIRA_TA 256  // tile rows on the A side
#define FIRA_TB 128  // tile rows on the B side
#define FIRA_LDS_A (FIRA_TA * 128)
#define FIRA_LDS_B (FIRA_TB * 128)
#define FIRA_EPI_STRIDE 68   // floats per staged row: 64 + 4 (keeps 16-byte alignment, shifts banks)
#define FIRA_LDS_EPI (4 * 32 * FIRA_EPI_STRIDE * 4)
#define FIRA_LDS_BYTES (FIRA_LDS_EPI > (FIRA_LDS_A + FIRA_LDS_B) ? FIRA_LDS_EPI : (FIRA_LDS_A + FIRA_LDS_B))

__device__ __forceinline__ int lds_tile_off(int row, int chunk) {
  return row * 128 + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

// 8 consecutive bf16 of a row that has `limit` valid elements, starting at element idx; elements
// outside [0, limit) read as zero and are never touched in memory.  No alignment assumed.
__device__ __forceinline__ u32x4 load8_bf16(gptr<const bf16_raw> row, long long idx, long long limit) {
  u32x4 v = u32x4{0u, 0u, 0u, 0u};
  if (idx + 8 <= limit) {
    v = *reinterpret_cast<gptr<const u32x4_a2>>(row + idx);
  } else if (idx < limit) {
    unsigned w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (idx + e < limit) w[e >> 1] |= ((unsigned)row[idx + e]) << ((e & 1) * 16);
    v = u32x4{w[0], w[1], w[2], w[3]};
  }
  return v;
}

struct GemmOperands {
  gptr<const bf16_raw> A;  // A side
  long long lda;      // elements between consecutive A rows (K-contiguous) or K steps (K-slow)
  int a_row0, a_rows; // first A row of this tile, number of valid A rows
  int KA;             // valid contraction length on the A side (elements beyond read as zero)
  gptr<const bf16_raw> B;  // B side: always K-contiguous, rows zero-padded to a multiple of 64 in K
  long long ldb;
  int b_row0, b_rows;
  int KB;             // readable row length of B (>= KA rounded up to 64)
};

template <bool AKSLOW>
__device__ __forceinline__ void gemm_load_tiles(u32x4 (&ra)[8], u32x4 (&rb)[4], const GemmOperands& g, int k0) {
  const int t = threadIdx.x;
  if (AKSLOW) {
    const int ib = t & 31, kb = t >> 5;
    const long long a = (long long)g.a_row0 + 8 * ib;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = k0 + 8 * kb + j;
      ra[j] = (k < g.KA) ? load8_bf16(g.A + (long long)k * g.lda, a, g.a_rows) : u32x4{0u, 0u, 0u, 0u};
    }
  } else {
    const int cc = t & 7, rr = t >> 3;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = g.a_row0 + rr + 32 * i;
      ra[i] = (row < g.a_rows) ? load8_bf16(g.A + (long long)row * g.lda, k0 + 8 * cc, g.KA)
                               : u32x4{0u, 0u, 0u, 0u};
    }
  }
  {
    const int cc = t & 7, rr = t >> 3;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = g.b_row0 + rr + 32 * i;
      rb[i] = (row < g.b_rows) ? load8_bf16(g.B + (long long)row * g.ldb, k0 + 8 * cc, g.KB)
                               : u32x4{0u, 0u, 0u, 0u};
    }
  }
}

template <bool AKSLOW>
__device__ __forceinline__ void gemm_store_tiles(char* lds, const u32x4 (&ra)[8], const u32x4 (&rb)[4]) {
  const int t = threadIdx.x;
  char* la = lds;
  char* lb = lds + FIRA_LDS_A;
  if (AKSLOW) {
    // ra[j] holds row k = 8*kb + j of an 8(k) x 8(a) block; emit, for each a, the 8 k values.
    const int ib = t & 31, kb = t >> 5;
    const unsigned* in = reinterpret_cast<const unsigned*>(&ra[0]);  // in[4*j + d]: a = 2d, 2d+1
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
      unsigned w[4];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const unsigned x = in[4 * (2 * d) + (ii >> 1)];      // k = 2d
        const unsigned y = in[4 * (2 * d + 1) + (ii >> 1)];  // k = 2d + 1
        w[d] = (ii & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
      }
      const int row = 8 * ib + ii;
      *reinterpret_cast<u32x4*>(la + lds_tile_off(row, kb)) = u32x4{w[0], w[1], w[2], w[3]};
    }
  } else {
    const int cc = t & 7, rr = t >> 3;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<u32x4*>(la + lds_tile_off(rr + 32 * i, cc)) = ra[i];
  }
  {
    const int cc = t & 7, rr = t >> 3;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<u32x4*>(lb + lds_tile_off(rr + 32 * i, cc)) = rb[i];
  }
}

// acc[tm][tn]: wave (wm, wn) = (wave & 1, wave >> 1) owns A rows wm*128 + 32*tm + .., B rows wn*64 + 32*tn + ..
template <bool AKSLOW>
__device__ __forceinline__ void gemm_mainloop(f32x16_t (&acc)[4][2], char* lds, const GemmOperands& g) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave & 1, wn = wave >> 1;
#pragma unroll
  for (int tm = 0; tm < 4; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.0f;

  const int KT = (g.KA + FIRA_BK - 1) / FIRA_BK;
  u32x4 ra[8], rb[4];
  gemm_load_tiles<AKSLOW>(ra, rb, g, 0);
  const char* la = lds;
  const char* lb = lds + FIRA_LDS_A;
  for (int kt = 0; kt < KT; ++kt) {
    gemm_store_tiles<AKSLOW>(lds, ra, rb);
    __syncthreads();
    if (kt + 1 < KT) gemm_load_tiles<AKSLOW>(ra, rb, g, (kt + 1) * FIRA_BK);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int chunk = 2 * kk + (lane >> 5);
      bf16x8_t af[4], bfr[2];
#pragma unroll
      for (int tm = 0; tm < 4; ++tm)
        af[tm] = *reinterpret_cast<const bf16x8_t*>(la + lds_tile_off(wm * 128 + 32 * tm + (lane & 31), chunk));
#pragma unroll
      for (int tn = 0; tn < 2; ++tn)
        bfr[tn] = *reinterpret_cast<const bf16x8_t*>(lb + lds_tile_off(wn * 64 + 32 * tn + (lane & 31), chunk));
#pragma unroll
      for (int tm = 0; tm < 4; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[tm], bfr[tn], acc[tm][tn], 0, 0, 0);
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------
// Kernel 1: low-rank gradient, long-side major:  Rt[i][a] = sum_s G(s, i) P[s][a]
//   left  (m <= n): i = column of G, s = row of G      -> A side is G read K-slow
//   right (m >  n): i = row of G,    s = column of G   -> A side is G read K-contiguous
//   B side is PT[a][s] (rank rows, short-side contiguous).
// Also (Gram mode) g2[i] = sum_s G(s, i)^2 is not computed here; see fira_gram.h.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void fira_project_kernel(const FiraMat* __restrict__ mats,
                                                              const FiraEnt* __restrict__ ents,
                                                              const FiraTile* __restrict__ tiles, int ntiles) {
  __shared__ __attribute__((aligned(16))) char lds[FIRA_LDS_A + FIRA_LDS_B];
  const int ti = xcd_chunked_index(blockIdx.x, ntiles);
  if (ti < 0) return;
  const FiraTile tile = tiles[ti];
  const FiraEnt ent = ents[tile.ent];
  const FiraMat mt = mats[ent.mat];

  GemmOperands g;
  g.a_row0 = tile.ta * FIRA_TA;
  g.a_rows = mt.L;
  g.b_row0 = tile.tb * FIRA_TB;
  g.b_rows = mt.r;
  g.B = as_global<const bf16_raw>(mt.PT);
  g.ldb = (long long)mt.kx * mt.Sp;
  g.KB = mt.kx * mt.Sp;
  if (mt.kx == 1) {
    g.A = as_global(reinterpret_cast<const bf16_raw*>(ent.G));
    g.lda = mt.ld;
    g.KA = mt.S;
  } else {
    g.A = as_global<const bf16_raw>(mt.Gx);
    g.lda = mt.left ? mt.gx_ld : (long long)mt.kx * mt.Sp;
    g.KA = mt.kx * mt.Sp;
  }
  f32x16_t acc[4][2];
  if (mt.left)
    gemm_mainloop<true>(acc, lds, g);
  else
    gemm_mainloop<false>(acc, lds, g);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  gptr<float> Rt = as_global(mt.Rt);
#pragma unroll
  for (int tm = 0; tm < 4; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
      const int col = g.b_row0 + wn * 64 + 32 * tn + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = g.a_row0 + wm * 128 + 32 * tm + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < mt.L && col < mt.r) Rt[(long long)row * mt.r + col] = acc[tm][tn][v];
      }
    }
}

// ------------------------------------------------------------------------------------------------
// Kernels 2 and 3 share the contraction  U[i][j] = sum_a X[i][a] Y[j][a]  over the rank axis, with
// X = P (m x r) and Y = Z or R long-side major (n x r) when left, X = Z or R (m x r) and Y = Q (n x r)
// when right.  The A side is Y (so a lane owns 4 consecutive columns j), the B side is X.
// The accumulators are re-laid out through LDS, one 32(i) x 64(j) slab per wave at a time, so that
// G and W are touched with 16-byte, row-contiguous accesses.
//   MODE 0: partial[tile] = sum_ij (k (G - U))^2            with Y/X built from R      (Eq. 12's norm)
//   MODE 1: W -= lr*alpha*(U + c k G)                       with Y/X built from Z = N - c k R
// ------------------------------------------------------------------------------------------------
template <typename T>
struct Elem8;  // 8 consecutive elements of W or G as floats
template <>
struct Elem8<bf16_raw> {
  static __device__ __forceinline__ void load(float (&x)[8], gptr<const bf16_raw> row, long long idx, long long limit) {
    const u32x4 v = load8_bf16(row, idx, limit);
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      x[2 * d] = __uint_as_float(w[d] << 16);
      x[2 * d + 1] = __uint_as_float(w[d] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(const float (&x)[8], gptr<bf16_raw> row, long long idx, long long limit) {
    if (idx + 8 <= limit) {
      const u32x4 v = u32x4{pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]),
                                 pack_bf16x2(x[6], x[7])};
      *reinterpret_cast<gptr<u32x4_a2>>(row + idx) = v;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (idx + e < limit) row[idx + e] = f32_to_bf16(x[e]);
    }
  }
};
template <>
struct Elem8<float> {
  static __device__ __forceinline__ void load(float (&x)[8], gptr<const float> row, long long idx, long long limit) {
    if (idx + 8 <= limit) {
      const f32x4 a = *reinterpret_cast<gptr<const f32x4_a4>>(row + idx);
      const f32x4 b = *reinterpret_cast<gptr<const f32x4_a4>>(row + idx + 4);
      x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = (idx + e < limit) ? row[idx + e] : 0.0f;
    }
  }
  static __device__ __forceinline__ void store(const float (&x)[8], gptr<float> row, long long idx, long long limit) {
    if (idx + 8 <= limit) {
      *reinterpret_cast<gptr<f32x4_a4>>(row + idx) = f32x4{x[0], x[1], x[2], x[3]};
      *reinterpret_cast<gptr<f32x4_a4>>(row + idx + 4) = f32x4{x[4], x[5], x[6], x[7]};
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (idx + e < limit) row[idx + e] = x[e];
    }
  }
};

template <int MODE, typename T>
__device__ __forceinline__ float backproject_epilogue(f32x16_t (&acc)[4][2], char* lds, const FiraMat& mt,
                                                      const FiraEnt& ent, int i0, int j0, float c, float lr_alpha) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  float* buf = reinterpret_cast<float*>(lds) + wave * (32 * FIRA_EPI_STRIDE);
  gptr<const T> G = as_global(reinterpret_cast<const T*>(ent.G));
  gptr<T> W = as_global(reinterpret_cast<T*>(ent.W));
  gptr<const float> phi = as_global<const float>(mt.phi);
  const int jl = 8 * (lane & 7);              // this lane's 8 columns inside the staged 64
  float sum = 0.0f;
#pragma unroll
  for (int th = 0; th < 2; ++th) {            // halves of the wave's 128 columns (A-side blocks 2th, 2th+1)
    const long long j = (long long)j0 + wm * 128 + 64 * th + jl;
    float cphi[8];
    if (mt.left) {
#pragma unroll
      for (int e = 0; e < 8; ++e) cphi[e] = (j + e < mt.n) ? c * phi[j + e] : 0.0f;
    }
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
      __syncthreads();  // previous slab fully consumed (first time: the main loop's LDS reads are done)
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const f32x16_t& a = acc[2 * th + t2][tn];
          const f32x4 val = f32x4{a[4 * vg], a[4 * vg + 1], a[4 * vg + 2], a[4 * vg + 3]};
          *reinterpret_cast<f32x4*>(buf + (lane & 31) * FIRA_EPI_STRIDE + 32 * t2 + 8 * vg + 4 * (lane >> 5)) = val;
        }
      __syncthreads();
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int il = 8 * p + (lane >> 3);
        const long long i = (long long)i0 + wn * 64 + 32 * tn + il;
        if (i < mt.m && j < mt.n) {
          const f32x4 u0 = *reinterpret_cast<const f32x4*>(buf + il * FIRA_EPI_STRIDE + jl);
          const f32x4 u1 = *reinterpret_cast<const f32x4*>(buf + il * FIRA_EPI_STRIDE + jl + 4);
          const float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
          float g[8];
          Elem8<T>::load(g, G + i * mt.ld, j, mt.n);
          if (!mt.left) {
            const float f = c * phi[i];
#pragma unroll
            for (int e = 0; e < 8; ++e) cphi[e] = f;
          }
          if (MODE == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float s = cphi[e] * (g[e] - u[e]);   // c = 1 here: k_i (G - P R)
              sum += (j + e < mt.n) ? s * s : 0.0f;
            }
          } else {
            float w[8];
            Elem8<T>::load(w, W + i * mt.ld, j, mt.n);
#pragma unroll
            for (int e = 0; e < 8; ++e) w[e] = w[e] - lr_alpha * (u[e] + cphi[e] * g[e]);
            Elem8<T>::store(w, W + i * mt.ld, j, mt.n);
          }
        }
      }
    }
  }
  return sum;
}

template <int MODE>
__global__ __launch_bounds__(256, 2) void fira_backproject_kernel(const FiraMat* __restrict__ mats,
                                                                  const FiraScal* __restrict__ scal,
                                                                  const FiraEnt* __restrict__ ents,
                                                                  const FiraTile* __restrict__ tiles, int ntiles,
                                                                  float* __restrict__ partial, float lr_alpha) {
  __shared__ __attribute__((aligned(16))) char lds[FIRA_LDS_BYTES];
  __shared__ float red[4];
  const int ti = xcd_chunked_index(blockIdx.x, ntiles);
  if (ti < 0) return;
  const FiraTile tile = tiles[ti];
  const FiraEnt ent = ents[tile.ent];
  const FiraMat mt = mats[ent.mat];

  // Y (n side) is the A operand, X (m side) the B operand.
  gptr<const bf16_raw> lowrank = as_global<const bf16_raw>((MODE == 0) ? mt.Rb : mt.Nb);
  gptr<const bf16_raw> proj = as_global<const bf16_raw>(mt.Pn);
  GemmOperands g;
  g.a_row0 = tile.ta * FIRA_TA;
  g.a_rows = mt.n;
  g.b_row0 = tile.tb * FIRA_TB;
  g.b_rows = mt.m;
  g.lda = g.ldb = (long long)mt.kx * mt.rp;
  g.KA = g.KB = mt.kx * mt.rp;
  g.A = mt.left ? lowrank : proj;
  g.B = mt.left ? proj : lowrank;
  f32x16_t acc[4][2];
  gemm_mainloop<false>(acc, lds, g);

  const float c = (MODE == 0) ? 1.0f : scal[ent.mat].c;
  float sum;
  if (mt.dtype == 1)
    sum = backproject_epilogue<MODE, bf16_raw>(acc, lds, mt, ent, g.b_row0, g.a_row0, c, lr_alpha);
  else
    sum = backproject_epilogue<MODE, float>(acc, lds, mt, ent, g.b_row0, g.a_row0, c, lr_alpha);

  if (MODE == 0) {
    // deterministic workgroup reduction: xor-butterfly inside each wave, then waves in order
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) as_global(partial)[tile.part] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}
