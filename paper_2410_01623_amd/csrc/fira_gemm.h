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

// Unguarded tile loads for interior tiles (every row of the tile valid, KA a multiple of 64): one
// uniform base pointer per operand that advances along K, plus per-thread element offsets that are
// computed once.  Rows may start at any element (odd n / ld): the loads only assume 2-byte alignment.
template <bool AKSLOW>
struct FastLoader {
  gptr<const bf16_raw> pa, pb;
  unsigned offa[8], offb[4];
  long long stepa;
  __device__ __forceinline__ FastLoader(const GemmOperands& g) {
    const int t = threadIdx.x;
    const int cc = t & 7, rr = t >> 3;
    if (AKSLOW) {
      const int ib = t & 31, kb = t >> 5;
      pa = g.A + g.a_row0;
#pragma unroll
      for (int j = 0; j < 8; ++j) offa[j] = (unsigned)((8 * kb + j) * g.lda + 8 * ib);
      stepa = FIRA_BK * g.lda;
    } else {
      pa = g.A + (long long)g.a_row0 * g.lda;
#pragma unroll
      for (int i = 0; i < 8; ++i) offa[i] = (unsigned)((rr + 32 * i) * g.lda + 8 * cc);
      stepa = FIRA_BK;
    }
    pb = g.B + (long long)g.b_row0 * g.ldb;
#pragma unroll
    for (int i = 0; i < 4; ++i) offb[i] = (unsigned)((rr + 32 * i) * g.ldb + 8 * cc);
  }
  __device__ __forceinline__ void load(u32x4 (&ra)[8], u32x4 (&rb)[4]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) ra[i] = *reinterpret_cast<gptr<const u32x4_a2>>(pa + offa[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) rb[i] = *reinterpret_cast<gptr<const u32x4_a2>>(pb + offb[i]);
    pa += stepa;
    pb += FIRA_BK;
  }
};

__device__ __forceinline__ bool gemm_tile_is_interior(const GemmOperands& g) {
  return g.a_row0 + FIRA_TA <= g.a_rows && g.b_row0 + FIRA_TB <= g.b_rows && (g.KA % FIRA_BK) == 0;
}

__device__ __forceinline__ void gemm_compute_step(f32x16_t (&acc)[4][2], const char* la, const char* lb) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave & 1, wn = wave >> 1;
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
}

// acc[tm][tn]: wave (wm, wn) = (wave & 1, wave >> 1) owns A rows wm*128 + 32*tm + .., B rows wn*64 + 32*tn + ..
// Single LDS buffer, register prefetch: the global loads of step k+1 are in flight while step k is
// multiplied; two workgroups per CU overlap one another's barriers.
template <bool AKSLOW>
__device__ __forceinline__ void gemm_mainloop(f32x16_t (&acc)[4][2], char* lds, const GemmOperands& g) {
#pragma unroll
  for (int tm = 0; tm < 4; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.0f;

  const int KT = (g.KA + FIRA_BK - 1) / FIRA_BK;
  u32x4 ra[8], rb[4];
  const char* la = lds;
  const char* lb = lds + FIRA_LDS_A;
  if (gemm_tile_is_interior(g)) {
    FastLoader<AKSLOW> ld(g);
    ld.load(ra, rb);
    for (int kt = 0; kt < KT; ++kt) {
      gemm_store_tiles<AKSLOW>(lds, ra, rb);
      __syncthreads();
      if (kt + 1 < KT) ld.load(ra, rb);
      gemm_compute_step(acc, la, lb);
      __syncthreads();
    }
  } else {
    gemm_load_tiles<AKSLOW>(ra, rb, g, 0);
    for (int kt = 0; kt < KT; ++kt) {
      gemm_store_tiles<AKSLOW>(lds, ra, rb);
      __syncthreads();
      if (kt + 1 < KT) gemm_load_tiles<AKSLOW>(ra, rb, g, (kt + 1) * FIRA_BK);
      gemm_compute_step(acc, la, lb);
      __syncthreads();
    }
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
struct Elem8;  // 8 consecutive elements of W or G: raw registers, conversion to floats, store
template <>
struct Elem8<bf16_raw> {
  typedef u32x4 Raw;
  template <bool INTERIOR>
  static __device__ __forceinline__ Raw load_raw(gptr<const bf16_raw> row, long long idx, long long limit) {
    if (INTERIOR) return *reinterpret_cast<gptr<const u32x4_a2>>(row + idx);
    return load8_bf16(row, idx, limit);
  }
  static __device__ __forceinline__ Raw zero() { return u32x4{0u, 0u, 0u, 0u}; }
  static __device__ __forceinline__ void unpack(const Raw& v, float (&x)[8]) {
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      x[2 * d] = __uint_as_float(w[d] << 16);
      x[2 * d + 1] = __uint_as_float(w[d] & 0xffff0000u);
    }
  }
  template <bool INTERIOR>
  static __device__ __forceinline__ void store(const float (&x)[8], gptr<bf16_raw> row, long long idx, long long limit) {
    if (INTERIOR || idx + 8 <= limit) {
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
  struct Raw { f32x4 a, b; };
  template <bool INTERIOR>
  static __device__ __forceinline__ Raw load_raw(gptr<const float> row, long long idx, long long limit) {
    Raw r;
    if (INTERIOR || idx + 8 <= limit) {
      r.a = *reinterpret_cast<gptr<const f32x4_a4>>(row + idx);
      r.b = *reinterpret_cast<gptr<const f32x4_a4>>(row + idx + 4);
    } else {
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = (idx + e < limit) ? row[idx + e] : 0.0f;
      r.a = f32x4{x[0], x[1], x[2], x[3]};
      r.b = f32x4{x[4], x[5], x[6], x[7]};
    }
    return r;
  }
  static __device__ __forceinline__ Raw zero() { Raw r; r.a = f32x4{0.f, 0.f, 0.f, 0.f}; r.b = r.a; return r; }
  static __device__ __forceinline__ void unpack(const Raw& r, float (&x)[8]) {
    x[0] = r.a.x; x[1] = r.a.y; x[2] = r.a.z; x[3] = r.a.w; x[4] = r.b.x; x[5] = r.b.y; x[6] = r.b.z; x[7] = r.b.w;
  }
  template <bool INTERIOR>
  static __device__ __forceinline__ void store(const float (&x)[8], gptr<float> row, long long idx, long long limit) {
    if (INTERIOR || idx + 8 <= limit) {
      *reinterpret_cast<gptr<f32x4_a4>>(row + idx) = f32x4{x[0], x[1], x[2], x[3]};
      *reinterpret_cast<gptr<f32x4_a4>>(row + idx + 4) = f32x4{x[4], x[5], x[6], x[7]};
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (idx + e < limit) row[idx + e] = x[e];
    }
  }
};

// Epilogue of the rank-axis contractions.  The wave's 64(i) x 128(j) accumulators are processed as
// four 32 x 64 slabs; the G (and W) values of slab s+1 are requested from HBM before slab s is
// re-laid out through LDS and consumed, so their latency overlaps the LDS work.
template <int MODE, typename T, bool INTERIOR>
__device__ __forceinline__ float backproject_epilogue(f32x16_t (&acc)[4][2], char* lds, const FiraMat& mt,
                                                      const FiraEnt& ent, int i0, int j0, float c, float lr_alpha) {
  typedef typename Elem8<T>::Raw Raw;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  float* buf = reinterpret_cast<float*>(lds) + wave * (32 * FIRA_EPI_STRIDE);
  gptr<const T> G = as_global(reinterpret_cast<const T*>(ent.G));
  gptr<T> W = as_global(reinterpret_cast<T*>(ent.W));
  gptr<const float> phi = as_global<const float>(mt.phi);
  const int jl = 8 * (lane & 7);              // this lane's 8 columns inside the staged 64
  const int il0 = lane >> 3;                  // this lane's row inside each group of 8 staged rows
  Raw gbuf[sizeof(T) == 2 ? 2 : 1][4], wbuf[sizeof(T) == 2 ? 2 : 1][4];
  auto preload = [&](int s, Raw (&gr)[4], Raw (&wr)[4]) {
    const int th = s >> 1, tn = s & 1;
    const long long j = (long long)j0 + wm * 128 + 64 * th + jl;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const long long i = (long long)i0 + wn * 64 + 32 * tn + 8 * p + il0;
      const bool ok = INTERIOR || (i < mt.m && j < mt.n);
      gr[p] = ok ? Elem8<T>::template load_raw<INTERIOR>(G + i * mt.ld, j, mt.n) : Elem8<T>::zero();
      if (MODE == 1) wr[p] = ok ? Elem8<T>::template load_raw<INTERIOR>(W + i * mt.ld, j, mt.n) : Elem8<T>::zero();
    }
  };
  constexpr bool PIPE = sizeof(T) == 2;       // fp32 tiles would need 128 more registers: no prefetch
  if (PIPE) preload(0, gbuf[0], wbuf[0]);
  float sum = 0.0f;
  float cphi[8];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int th = s >> 1, tn = s & 1;
    const long long j = (long long)j0 + wm * 128 + 64 * th + jl;
    if (PIPE && s + 1 < 4) preload(s + 1, gbuf[PIPE ? ((s + 1) & 1) : 0], wbuf[PIPE ? ((s + 1) & 1) : 0]);
    if (!PIPE) preload(s, gbuf[0], wbuf[0]);
    if (mt.left && tn == 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) cphi[e] = (INTERIOR || j + e < mt.n) ? c * phi[j + e] : 0.0f;
    }
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
      const int il = 8 * p + il0;
      const long long i = (long long)i0 + wn * 64 + 32 * tn + il;
      if (INTERIOR || (i < mt.m && j < mt.n)) {
        const f32x4 u0 = *reinterpret_cast<const f32x4*>(buf + il * FIRA_EPI_STRIDE + jl);
        const f32x4 u1 = *reinterpret_cast<const f32x4*>(buf + il * FIRA_EPI_STRIDE + jl + 4);
        const float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
        float g[8];
        Elem8<T>::unpack(gbuf[PIPE ? (s & 1) : 0][p], g);
        if (!mt.left) {
          const float f = c * phi[i];
#pragma unroll
          for (int e = 0; e < 8; ++e) cphi[e] = f;
        }
        if (MODE == 0) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float sv = cphi[e] * (g[e] - u[e]);   // c = 1 here: k_i (G - P R)
            sum += (INTERIOR || j + e < mt.n) ? sv * sv : 0.0f;
          }
        } else {
          float w[8];
          Elem8<T>::unpack(wbuf[PIPE ? (s & 1) : 0][p], w);
#pragma unroll
          for (int e = 0; e < 8; ++e) w[e] = w[e] - lr_alpha * (u[e] + cphi[e] * g[e]);
          Elem8<T>::template store<INTERIOR>(w, W + i * mt.ld, j, mt.n);
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
  const bool interior = g.b_row0 + FIRA_TB <= mt.m && g.a_row0 + FIRA_TA <= mt.n;
  if (mt.dtype == 1) {
    if (interior) sum = backproject_epilogue<MODE, bf16_raw, true>(acc, lds, mt, ent, g.b_row0, g.a_row0, c, lr_alpha);
    else sum = backproject_epilogue<MODE, bf16_raw, false>(acc, lds, mt, ent, g.b_row0, g.a_row0, c, lr_alpha);
  } else {
    sum = backproject_epilogue<MODE, float, false>(acc, lds, mt, ent, g.b_row0, g.a_row0, c, lr_alpha);
  }

  if (MODE == 0) {
    // deterministic workgroup reduction: xor-butterfly inside each wave, then waves in order
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) as_global(partial)[tile.part] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}
