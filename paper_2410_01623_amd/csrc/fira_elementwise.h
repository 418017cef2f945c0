// Fused element-wise / reduction passes of the Fira step (HBM-bound): Adam on the low-rank gradient
// with the per-factor norms, the limiter scalar, the construction of the back-projection operand,
// and the operand conversions done when a projector is installed.
#pragma once
#include "fira_device.h"


// Work-list lookup for the row-blocked kernels: entry e covers row-blocks [ents[e].row0, ents[e+1].row0).
__device__ __forceinline__ int find_entry(const FiraEnt* __restrict__ ents, int count, int rowblock) {
  int lo = 0, hi = count - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (ents[mid].row0 <= rowblock) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// ||G_i - P R_i||^2 from ||G_i||^2 and ||R_i||^2 (Gram route), or ||G_i||^2 itself for the variant that
// scales the full gradient.
__device__ __forceinline__ float residual_sq(const FiraHp& hp, float g2, float rr) {
  return hp.variant == 1 ? g2 : fmaxf(g2 - rr, 0.0f);
}

// Adam's direction for one element (Eqs. 2-4), N = bias * m / (sqrt(v) + eps), bias = sqrt(1 - beta2^t) /
// (1 - beta1^t), from the hardware's square root and reciprocal (1 ulp each) rather than the correctly
// rounded library forms, which cost about five times the instructions: in the fused kernel that
// arithmetic is not hidden behind memory traffic.  The square-root instruction takes no subnormal
// input, so v is raised to the smallest normal number first: sqrt(v) then reads 1.1e-19 where it is
// smaller, which only an eps of that order could tell apart.  Otherwise the result is within a few
// ulp of the exact quotient.
__device__ __forceinline__ float adam_direction(float m1, float v1, float bias, float eps) {
  const float s = __builtin_amdgcn_sqrtf(fmaxf(v1, 0x1p-126f));
  return bias * m1 * __builtin_amdgcn_rcpf(s + eps);
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// store one low-rank value as an MFMA operand element (plain bf16, or the 6-plane split, sequence A)
// (`op` is a K-blocked array with `rows` padded rows; plane p of the split occupies k = p*rp + a.)
template <int KX>
__device__ __forceinline__ void store_operand(gptr<bf16_raw> op, int rows, long long row, int rp, int a, float x) {
  if (KX == 1) {
    op[kblk_index(rows, row, a)] = f32_to_bf16(x);
  } else {
    bf16_raw h, m, l;
    split3(x, h, m, l);
    const bf16_raw seq[6] = {h, h, m, h, l, m};
#pragma unroll
    for (int p = 0; p < 6; ++p) op[kblk_index(rows, row, p * rp + a)] = seq[p];
  }
}
template <int KX>
__device__ __forceinline__ float load_operand(gptr<const bf16_raw> op, int rows, long long row, int rp, int a) {
  if (KX == 1) return bf16_to_f32(op[kblk_index(rows, row, a)]);
  return (bf16_to_f32(op[kblk_index(rows, row, a)]) + bf16_to_f32(op[kblk_index(rows, row, 2 * rp + a)])) +
         bf16_to_f32(op[kblk_index(rows, row, 4 * rp + a)]);
}

// ------------------------------------------------------------------------------------------------
// Adam on R (Eqs. 2-4 applied to R, Algorithm 1's Adam block) fused with the two norms of every
// factor (Algorithm 1, "Norm-Based Scaling").  One wavefront per long-side row:
//   M <- b1 M + (1-b1) R;  V <- b2 V + (1-b2) R^2;  N = bias * M / (sqrt(V) + eps)
//   k_i = ||N_i|| / (||R_i|| + eps);  N and R are also written as bf16 MFMA operands.
// ------------------------------------------------------------------------------------------------
template <int KX, int VEC>
__device__ __forceinline__ void adam_row(const FiraMat& mt, const FiraHp& hp, float bias, long long row, bool gram) {
  const int lane = threadIdx.x & 63;
  const int r = mt.r;
  gptr<const float> R = as_global<const float>(mt.Rt) + row * r;
  gptr<float> M = as_global(mt.M) + row * r;
  gptr<float> V = as_global(mt.V) + row * r;
  gptr<bf16_raw> Nb = as_global(mt.Nb);
  gptr<bf16_raw> Rb = as_global(mt.Rb);
  float nn = 0.0f, rr = 0.0f;
  for (int a = lane * VEC; a < r; a += 64 * VEC) {
    float rv[VEC], mv[VEC], vv[VEC], nv[VEC];
    if (VEC == 4) {
      *reinterpret_cast<f32x4*>(rv) = *reinterpret_cast<gptr<const f32x4>>(R + a);
      *reinterpret_cast<f32x4*>(mv) = *reinterpret_cast<gptr<const f32x4>>(M + a);
      *reinterpret_cast<f32x4*>(vv) = *reinterpret_cast<gptr<const f32x4>>(V + a);
    } else {
      rv[0] = R[a]; mv[0] = M[a]; vv[0] = V[a];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      mv[e] = hp.b1 * mv[e] + hp.omb1 * rv[e];
      vv[e] = hp.b2 * vv[e] + hp.omb2 * (rv[e] * rv[e]);
      nv[e] = adam_direction(mv[e], vv[e], bias, hp.epsf);
      nn += nv[e] * nv[e];
      rr += rv[e] * rv[e];
    }
    if (VEC == 4) {
      *reinterpret_cast<gptr<f32x4>>(M + a) = *reinterpret_cast<const f32x4*>(mv);
      *reinterpret_cast<gptr<f32x4>>(V + a) = *reinterpret_cast<const f32x4*>(vv);
    } else {
      M[a] = mv[0]; V[a] = vv[0];
    }
    if (KX == 1 && VEC == 4) {
      const long long o = kblk_index(mt.Lq, row, a);
      *reinterpret_cast<gptr<u32x2>>(Nb + o) = u32x2{pack_bf16x2(nv[0], nv[1]), pack_bf16x2(nv[2], nv[3])};
      *reinterpret_cast<gptr<u32x2>>(Rb + o) = u32x2{pack_bf16x2(rv[0], rv[1]), pack_bf16x2(rv[2], rv[3])};
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        store_operand<KX>(Nb, mt.Lq, row, mt.rp, a + e, nv[e]);
        store_operand<KX>(Rb, mt.Lq, row, mt.rp, a + e, rv[e]);
      }
    }
  }
  nn = wave_sum(nn);
  rr = wave_sum(rr);
  if (lane == 0) {
    if (hp.scaling == 1) {
      // one factor per matrix: leave the row's ||N_i||^2 and ||R_i||^2 for the limiter kernel, which
      // sums them, forms the factor and writes it over phi
      as_global(mt.phi)[row] = nn;
      as_global(mt.q)[row] = rr;
    } else {
      const float k = (hp.scaling == 2) ? 1.0f : sqrtf(nn) / (sqrtf(rr) + hp.epsf);
      as_global(mt.phi)[row] = k;
      // Gram route: ||G_i - P R_i||^2 = ||G_i||^2 - ||R_i||^2 when P^T P = I (G_i^T P = R_i^T always)
      if (have_g2(hp)) as_global(mt.q)[row] = k * k * residual_sq(hp, as_global<const float>(mt.g2)[row], rr);
    }
  }
}

// Second bf16 plane of four values whose first plane (nearest-even bf16) is `hi`: bf16(z - hi), so that
// hi + lo carries 16 mantissa bits of z.
__device__ __forceinline__ u32x2 split_remainder(const f32x4& z, const u32x2& hi) {
  const float h0 = __uint_as_float(hi.x << 16), h1 = __uint_as_float(hi.x & 0xffff0000u);
  const float h2 = __uint_as_float(hi.y << 16), h3 = __uint_as_float(hi.y & 0xffff0000u);
  return u32x2{pack_bf16x2(z[0] - h0, z[1] - h1), pack_bf16x2(z[2] - h2, z[3] - h3)};
}

// Same update for bf16 matrices with r % 4 == 0 and r <= FIRA_ZREADY_MAX_R: the factor's N and R stay
// in registers until k_i is known, and the row is written once as the back-projection operand for
// an inactive limiter, Z_i = N_i - k_i R_i, rounded from fp32 a single time.  R is written as an
// operand only when the residual contraction will need it.  Z is K-blocked, 64 B per row and K
// block, so the workgroup's 16 rows are collected in LDS ([K block][16 rows][32]) and leave as
// 1 KB contiguous pieces (fira_adam_kernel).
template <int NIT>   // 256 * NIT >= r
__device__ __forceinline__ void adam_row_zready(const FiraMat& mt, const FiraHp& hp, float bias, long long row, bool gram,
                                                bf16_raw* zl, int rowlocal) {
  const int lane = threadIdx.x & 63;
  const int r = mt.r;
  gptr<const float> R = as_global<const float>(mt.Rt) + row * r;
  gptr<float> M = as_global(mt.M) + row * r;
  gptr<float> V = as_global(mt.V) + row * r;
  gptr<bf16_raw> Rb = as_global(mt.Rb);
  float nn = 0.0f, rr = 0.0f;
  f32x4 nv[NIT], rv[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int a = lane * 4 + 256 * it;
    if (a < r) {
      rv[it] = *reinterpret_cast<gptr<const f32x4>>(R + a);
      f32x4 mv = *reinterpret_cast<gptr<const f32x4>>(M + a);
      f32x4 vv = *reinterpret_cast<gptr<const f32x4>>(V + a);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        mv[e] = hp.b1 * mv[e] + hp.omb1 * rv[it][e];
        vv[e] = hp.b2 * vv[e] + hp.omb2 * (rv[it][e] * rv[it][e]);
        nv[it][e] = adam_direction(mv[e], vv[e], bias, hp.epsf);
        nn += nv[it][e] * nv[it][e];
        rr += rv[it][e] * rv[it][e];
      }
      *reinterpret_cast<gptr<f32x4>>(M + a) = mv;
      *reinterpret_cast<gptr<f32x4>>(V + a) = vv;
    }
  }
  nn = wave_sum(nn);
  rr = wave_sum(rr);
  const float k = (hp.scaling == 2) ? 1.0f : sqrtf(nn) / (sqrtf(rr) + hp.epsf);
  const int lo_off = (mt.rp >> 5) * (FIRA_ROWS_PER_WG * 32);   // second plane of the LDS image (hp.zsplit)
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int a = lane * 4 + 256 * it;
    if (a < mt.rp) {
      u32x2 zv = u32x2{0u, 0u}, zlo = u32x2{0u, 0u};
      if (a < r) {
        const f32x4 z = nv[it] - k * rv[it];
        zv = u32x2{pack_bf16x2(z[0], z[1]), pack_bf16x2(z[2], z[3])};
        if (hp.zsplit) zlo = split_remainder(z, zv);
        if (!gram)
          *reinterpret_cast<gptr<u32x2>>(Rb + kblk_index(mt.Lq, row, a)) =
              u32x2{pack_bf16x2(rv[it][0], rv[it][1]), pack_bf16x2(rv[it][2], rv[it][3])};
      }
      bf16_raw* dst = zl + (a >> 5) * (FIRA_ROWS_PER_WG * 32) + rowlocal * 32 + (a & 31);
      *reinterpret_cast<u32x2*>(dst) = zv;
      if (hp.zsplit) *reinterpret_cast<u32x2*>(dst + lo_off) = zlo;
    }
  }
  if (lane == 0) {
    as_global(mt.phi)[row] = k;
    if (have_g2(hp)) as_global(mt.q)[row] = k * k * residual_sq(hp, as_global<const float>(mt.g2)[row], rr);
  }
}

// Small ranks (r <= 64, e.g. the fine-tuning setting's r = 32): a factor's row is at most 256 bytes, so
// a wavefront takes its four rows at once, 16 lanes per row, instead of one after the other.
__device__ __forceinline__ void adam_rows4_small(const FiraMat& mt, const FiraHp& hp, float bias, long long row_base,
                                                 bool gram, bf16_raw* zl, int wave) {
  const int lane = threadIdx.x & 63;
  const int g = lane >> 4, a = (lane & 15) * 4;
  const int r = mt.r;
  const long long row = row_base + g;
  const bool live = row < mt.L && a < r;
  gptr<const float> R = as_global<const float>(mt.Rt) + row * r;
  gptr<float> M = as_global(mt.M) + row * r;
  gptr<float> V = as_global(mt.V) + row * r;
  f32x4 nv = f32x4{0.f, 0.f, 0.f, 0.f}, rv = nv;
  float nn = 0.0f, rr = 0.0f;
  if (live) {
    rv = *reinterpret_cast<gptr<const f32x4>>(R + a);
    f32x4 mv = *reinterpret_cast<gptr<const f32x4>>(M + a);
    f32x4 vv = *reinterpret_cast<gptr<const f32x4>>(V + a);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      mv[e] = hp.b1 * mv[e] + hp.omb1 * rv[e];
      vv[e] = hp.b2 * vv[e] + hp.omb2 * (rv[e] * rv[e]);
      nv[e] = adam_direction(mv[e], vv[e], bias, hp.epsf);
      nn += nv[e] * nv[e];
      rr += rv[e] * rv[e];
    }
    *reinterpret_cast<gptr<f32x4>>(M + a) = mv;
    *reinterpret_cast<gptr<f32x4>>(V + a) = vv;
  }
#pragma unroll
  for (int off = 8; off >= 1; off >>= 1) {   // sums within the 16 lanes of a row
    nn += __shfl_xor(nn, off, 64);
    rr += __shfl_xor(rr, off, 64);
  }
  const float k = (hp.scaling == 2) ? 1.0f : sqrtf(nn) / (sqrtf(rr) + hp.epsf);
  if (a < mt.rp) {
    u32x2 zv = u32x2{0u, 0u}, zlo = u32x2{0u, 0u};   // rows beyond L and columns beyond r: the operand's zero padding
    if (live) {
      const f32x4 z = nv - k * rv;
      zv = u32x2{pack_bf16x2(z[0], z[1]), pack_bf16x2(z[2], z[3])};
      if (hp.zsplit) zlo = split_remainder(z, zv);
      if (!gram)
        *reinterpret_cast<gptr<u32x2>>(as_global(mt.Rb) + kblk_index(mt.Lq, row, a)) =
            u32x2{pack_bf16x2(rv[0], rv[1]), pack_bf16x2(rv[2], rv[3])};
    }
    bf16_raw* dst = zl + (a >> 5) * (FIRA_ROWS_PER_WG * 32) + (wave * 4 + g) * 32 + (a & 31);
    *reinterpret_cast<u32x2*>(dst) = zv;
    if (hp.zsplit) *reinterpret_cast<u32x2*>(dst + (mt.rp >> 5) * (FIRA_ROWS_PER_WG * 32)) = zlo;
  }
  if ((lane & 15) == 0 && row < mt.L) {
    as_global(mt.phi)[row] = k;
    if (have_g2(hp)) as_global(mt.q)[row] = k * k * residual_sq(hp, as_global<const float>(mt.g2)[row], rr);
  }
}

__global__ __launch_bounds__(256, 4) void fira_adam_kernel(const FiraMat* __restrict__ mats,
                                                        const FiraScal* __restrict__ scal,
                                                        const FiraEnt* __restrict__ ents, int count,
                                                        int total_rowblocks, FiraHp hp) {
  extern __shared__ __attribute__((aligned(16))) char adam_lds[];   // zready matrices: 16 rows x rp bf16
  const int rb = blockIdx.x;
  if (rb >= total_rowblocks) return;
  const int e = find_entry(ents, count, rb);
  const FiraEnt ent = ents[e];
  const FiraMat mt = mats[ent.mat];
  bf16_raw* zl = reinterpret_cast<bf16_raw*>(adam_lds);
  const bool zready = mt.zready && hp.scaling != 1;   // the matrix-level factor is not known in this kernel
  // bias correction with the 1-based step count (Eq. 4), in double: 1 - beta2^t loses all
  // accuracy in fp32 at small t.
  const FiraScal sc = scal[ent.mat];
  const int t = sc.t + 1;
  const bool gram = use_gram(hp, sc);
  if (hp.mixed && gram) return;                // the fused kernel has served this matrix
  const float bias = (float)(sqrt(1.0 - pow(hp.beta2, (double)t)) / (1.0 - pow(hp.beta1, (double)t)));
  const int wave = threadIdx.x >> 6;
  const long long row_base = (long long)(rb - ent.row0) * FIRA_ROWS_PER_WG + wave * 4;
  if (zready && mt.r <= 64) adam_rows4_small(mt, hp, bias, row_base, gram, zl, wave);
  else for (int i = 0; i < 4; ++i) {
    const long long row = row_base + i;
    if (row >= mt.L) {
      if (zready)   // rows of the padding: zeros
        for (int a = (threadIdx.x & 63) * 4; a < (hp.zsplit ? 2 : 1) * mt.rp; a += 256)
          *reinterpret_cast<u32x2*>(zl + (a >> 5) * (FIRA_ROWS_PER_WG * 32) + (wave * 4 + i) * 32 + (a & 31)) = u32x2{0u, 0u};
      continue;
    }
    if (zready) {
      if (mt.r <= 256) adam_row_zready<1>(mt, hp, bias, row, gram, zl, wave * 4 + i);
      else if (mt.r <= 512) adam_row_zready<2>(mt, hp, bias, row, gram, zl, wave * 4 + i);
      else adam_row_zready<FIRA_ZREADY_MAX_R / 256>(mt, hp, bias, row, gram, zl, wave * 4 + i);
    } else if (mt.kx == 1) {
      if ((mt.r & 3) == 0) adam_row<1, 4>(mt, hp, bias, row, gram); else adam_row<1, 1>(mt, hp, bias, row, gram);
    } else {
      adam_row<FIRA_KX_SPLIT, 1>(mt, hp, bias, row, gram);
    }
  }
  if (zready) {
    __syncthreads();
    // the 16 rows of one K block are 1 KB of contiguous memory
    gptr<char> nb = reinterpret_cast<gptr<char>>(as_global(mt.Nb));
    const long long row0 = (long long)(rb - ent.row0) * FIRA_ROWS_PER_WG;
    const int nbytes = (hp.zsplit ? 2 : 1) * (mt.rp >> 5) * (FIRA_ROWS_PER_WG * 64);   // K blocks [rp/32, 2 rp/32): the lo plane
    for (int o = threadIdx.x * 16; o < nbytes; o += 256 * 16) {
      const int kb = o / (FIRA_ROWS_PER_WG * 64), w = o % (FIRA_ROWS_PER_WG * 64);
      *reinterpret_cast<gptr<u32x4>>(nb + ((long long)kb * mt.Lq + row0) * 64 + w) =
          *reinterpret_cast<const u32x4*>(adam_lds + o);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Norm-growth limiter (Eq. 12 in Algorithm 1's form): one workgroup per listed matrix sums the
// tile partials of ||S||^2 in a fixed order (fp64), derives the factor c, and advances the state.
// ------------------------------------------------------------------------------------------------
#define FIRA_LIMITER_THREADS 256
// Workgroup sum in a fixed order: butterfly inside each wavefront, then the four wavefronts in order.
__device__ __forceinline__ double limiter_block_sum(double x, double* red) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  __syncthreads();                       // red may still be read from the previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(FIRA_LIMITER_THREADS) void fira_limiter_kernel(const FiraMat* __restrict__ mats,
                                                                            FiraScal* __restrict__ scal,
                                                                            const FiraEnt* __restrict__ ents,
                                                                            const float* __restrict__ partial, FiraHp hp) {
  __shared__ double red[4];
  const FiraEnt ent = ents[blockIdx.x];
  const int tid = threadIdx.x;
  const FiraScal sc0 = scal[ent.mat];
  const bool gram = use_gram(hp, sc0);
  // On the residual route with the Gram data at hand (the first step after an install), also form the
  // Gram route's value and record how far it is from the exact one: the second gate of that route.
  const bool calibrate = !gram && calibrates_gram(hp, sc0);
  double acc = 0.0, accg = 0.0;
  if (hp.scaling == 1) {
    // Matrix-level factor (Eq. 9): k = ||N|| / (||R|| + eps) from the row sums the Adam kernel left in
    // phi and q; ||S||^2 = k^2 * (sum_i ||G_i - P R_i||^2), the sum taken with unit factors by either route.
    const FiraMat mt = mats[ent.mat];
    gptr<float> phi = as_global(mt.phi);
    gptr<const float> q = as_global<const float>(mt.q);
    gptr<const float> g2 = as_global<const float>(mt.g2);
    double nn = 0.0, rr = 0.0;
    for (int i = tid; i < mt.L; i += FIRA_LIMITER_THREADS) {
      nn += (double)phi[i];
      rr += (double)q[i];
      if (gram) acc += (double)residual_sq(hp, g2[i], q[i]);
      else if (calibrate) accg += (double)residual_sq(hp, g2[i], q[i]);
    }
    if (!gram)
      for (int i = tid; i < ent.npart; i += FIRA_LIMITER_THREADS) acc += (double)partial[ent.part0 + i];
    nn = limiter_block_sum(nn, red);     // (the barriers inside also order the reads of phi before its rewrite)
    rr = limiter_block_sum(rr, red);
    const float k = (float)(sqrt(nn) / (sqrt(rr) + hp.eps));
    acc *= (double)k * (double)k;
    accg *= (double)k * (double)k;
    for (int i = tid; i < mt.L; i += FIRA_LIMITER_THREADS) phi[i] = k;
  } else {
    if (gram || calibrate) {
      const FiraMat mt = mats[ent.mat];
      gptr<const float> q = as_global<const float>(mt.q);
      double a = 0.0;
      for (int i = tid; i < mt.L; i += FIRA_LIMITER_THREADS) a += (double)q[i];
      if (gram) acc = a; else accg = a;
    }
    if (!gram)
      for (int i = tid; i < ent.npart; i += FIRA_LIMITER_THREADS) acc += (double)partial[ent.part0 + i];
  }
  acc = limiter_block_sum(acc, red);
  if (calibrate) accg = limiter_block_sum(accg, red);   // (uniform over the workgroup)
  if (tid == 0) {
    FiraScal s = scal[ent.mat];
    const double sn = sqrt(acc);
    double c = 1.0;
    if (s.has_prev && !isinf(hp.gamma) && sn != 0.0) {
      const double den = s.s_prev + hp.eps;
      const double ratio = den > 0.0 ? sn / den : INFINITY;
      c = hp.gamma / fmax(ratio, hp.gamma);
    }
    if (calibrate) s.gram_err = (acc == accg) ? 0.0f : (float)fmin(fabs(accg - acc) / fmax(acc, 1e-300), 3.0e38);
    s.gram_now = gram ? (hp.fused ? 2 : 1) : 0;
    s.s_pre = sn;
    s.s_post = c * sn;
    s.s_prev = s.s_post;      // the remembered norm is the limited one
    s.has_prev = 1;
    s.c = (float)c;
    s.t += 1;
    scal[ent.mat] = s;
  }
}

// ------------------------------------------------------------------------------------------------
// Back-projection operand: Z_i = N_i - c k_i R_i, so that P N + c k (G - P R) = P Z + c k G.
// Overwrites N in place.  Matrices flagged zready skip this unless their limiter factor is below 1.
// ------------------------------------------------------------------------------------------------
template <int KX>
__device__ __forceinline__ void makez_row(const FiraMat& mt, float f, long long row) {
  const int lane = threadIdx.x & 63;
  gptr<bf16_raw> Nb = as_global(mt.Nb);
  gptr<const bf16_raw> Rb = as_global<const bf16_raw>(mt.Rb);
  if (KX == 1) {
    // rp is a multiple of 64 and padded entries are zero: whole 16-byte groups
    for (int a = lane * 8; a < mt.rp; a += 512) {
      const long long o = kblk_index(mt.Lq, row, a);
      const u32x4 nv = *reinterpret_cast<gptr<const u32x4>>(Nb + o);
      const u32x4 rv = *reinterpret_cast<gptr<const u32x4>>(Rb + o);
      const unsigned nw[4] = {nv.x, nv.y, nv.z, nv.w}, rw[4] = {rv.x, rv.y, rv.z, rv.w};
      unsigned zw[4];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        float z0 = __uint_as_float(nw[d] << 16) - f * __uint_as_float(rw[d] << 16);
        float z1 = __uint_as_float(nw[d] & 0xffff0000u) - f * __uint_as_float(rw[d] & 0xffff0000u);
        if (a + 2 * d >= mt.r) z0 = 0.0f;       // padding stays zero even for a non-finite factor
        if (a + 2 * d + 1 >= mt.r) z1 = 0.0f;
        zw[d] = pack_bf16x2(z0, z1);
      }
      *reinterpret_cast<gptr<u32x4>>(Nb + o) = u32x4{zw[0], zw[1], zw[2], zw[3]};
    }
  } else {
    for (int a = lane; a < mt.r; a += 64) {
      const float z = load_operand<KX>((gptr<const bf16_raw>)Nb, mt.Lq, row, mt.rp, a) -
                      f * load_operand<KX>(Rb, mt.Lq, row, mt.rp, a);
      store_operand<KX>(Nb, mt.Lq, row, mt.rp, a, z);
    }
  }
}

// Rows that already hold Z for c = 1 (N_i - k_i R_i): add back (1 - c) k_i R_i, with R in fp32.
__device__ __forceinline__ void fixz_row(const FiraMat& mt, float f, long long row, bool zsplit) {
  const int lane = threadIdx.x & 63;
  gptr<bf16_raw> Nb = as_global(mt.Nb);
  gptr<const float> R = as_global<const float>(mt.Rt) + row * mt.r;
  for (int a = lane * 4; a < mt.r; a += 256) {
    const long long o = kblk_index(mt.Lq, row, a), ol = kblk_index(mt.Lq, row, mt.rp + a);
    const u32x2 zv = *reinterpret_cast<gptr<const u32x2>>(Nb + o);
    const f32x4 rv = *reinterpret_cast<gptr<const f32x4>>(R + a);
    f32x4 z = f32x4{__uint_as_float(zv.x << 16), __uint_as_float(zv.x & 0xffff0000u), __uint_as_float(zv.y << 16),
                    __uint_as_float(zv.y & 0xffff0000u)};
    if (zsplit) {
      const u32x2 lv = *reinterpret_cast<gptr<const u32x2>>(Nb + ol);
      z += f32x4{__uint_as_float(lv.x << 16), __uint_as_float(lv.x & 0xffff0000u), __uint_as_float(lv.y << 16),
                 __uint_as_float(lv.y & 0xffff0000u)};
    }
    z += f * rv;
    const u32x2 hi = u32x2{pack_bf16x2(z[0], z[1]), pack_bf16x2(z[2], z[3])};
    *reinterpret_cast<gptr<u32x2>>(Nb + o) = hi;
    if (zsplit) *reinterpret_cast<gptr<u32x2>>(Nb + ol) = split_remainder(z, hi);
  }
}

// The same correction without R (after the fused kernel): Z = N - c k R = c (N - k R) + (1 - c) N, with N
// formed again from the updated M and V.  c Z_1 carries Z_1's bf16 rounding, so Z is rounded twice
// here; that happens only on the steps on which the limiter is active.
__device__ __forceinline__ void fixz_row_from_moments(const FiraMat& mt, const FiraHp& hp, float c, float bias, long long row) {
  const int lane = threadIdx.x & 63;
  gptr<bf16_raw> Nb = as_global(mt.Nb);
  gptr<const float> M = as_global<const float>(mt.M) + row * mt.r;
  gptr<const float> V = as_global<const float>(mt.V) + row * mt.r;
  for (int a = lane * 4; a < mt.r; a += 256) {
    const long long o = kblk_index(mt.Lq, row, a);
    const u32x2 zv = *reinterpret_cast<gptr<const u32x2>>(Nb + o);
    const f32x4 mv = *reinterpret_cast<gptr<const f32x4>>(M + a);
    const f32x4 vv = *reinterpret_cast<gptr<const f32x4>>(V + a);
    const float z1[4] = {__uint_as_float(zv.x << 16), __uint_as_float(zv.x & 0xffff0000u), __uint_as_float(zv.y << 16),
                         __uint_as_float(zv.y & 0xffff0000u)};
    float z[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) z[e] = c * z1[e] + (1.0f - c) * adam_direction(mv[e], vv[e], bias, hp.epsf);
    *reinterpret_cast<gptr<u32x2>>(Nb + o) = u32x2{pack_bf16x2(z[0], z[1]), pack_bf16x2(z[2], z[3])};
  }
}

#define FIRA_MAKEZ_PARTS 32   // workgroups per listed matrix
// One workgroup per (listed matrix, part): it reads the matrix's c once and, in the common case, exits;
// otherwise it takes every FIRA_MAKEZ_PARTS-th block of 16 rows.
__global__ __launch_bounds__(256) void fira_makez_kernel(const FiraMat* __restrict__ mats,
                                                         const FiraScal* __restrict__ scal,
                                                         const FiraEnt* __restrict__ ents, FiraHp hp) {
  const FiraEnt ent = ents[blockIdx.x / FIRA_MAKEZ_PARTS];
  const int part = blockIdx.x % FIRA_MAKEZ_PARTS;
  const float c = scal[ent.mat].c;
  const FiraMat mt = mats[ent.mat];
  const bool zready = mt.zready && hp.scaling != 1;
  if (zready && c == 1.0f) return;             // the Adam kernel already wrote Z for c = 1
  // whether the fused kernel served this matrix (then no copy of R exists)
  const bool fused_here = scal[ent.mat].gram_now == 2;
  const int wave = threadIdx.x >> 6;
  const int rowblocks = (mt.L + FIRA_ROWS_PER_WG - 1) / FIRA_ROWS_PER_WG;
  // the limiter has already advanced t: the bias correction of this step uses the count as it stands now
  const int t = scal[ent.mat].t;
  const float bias = fused_here ? (float)(sqrt(1.0 - pow(hp.beta2, (double)t)) / (1.0 - pow(hp.beta1, (double)t))) : 0.0f;
  for (int rb = part; rb < rowblocks; rb += FIRA_MAKEZ_PARTS) {
    const long long row_base = (long long)rb * FIRA_ROWS_PER_WG + wave * 4;
    for (int i = 0; i < 4; ++i) {
      const long long row = row_base + i;
      if (row >= mt.L) break;
      const float k = as_global<const float>(mt.phi)[row];
      if (zready && fused_here) fixz_row_from_moments(mt, hp, c, bias, row);
      else if (zready) fixz_row(mt, (1.0f - c) * k, row, hp.zsplit != 0);
      else if (mt.kx == 1) makez_row<1>(mt, c * k, row);
      else makez_row<FIRA_KX_SPLIT>(mt, c * k, row);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// "Fira-only-scaling" update: W -= lr*alpha * c * k_i * G over the tiles of the back-projection list
// (256 columns x 128 rows per workgroup), a pure stream: 16 bytes per lane, 512 contiguous bytes per
// row piece, factors per column (m <= n) or per row (m > n).
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void fira_scale_update_kernel(const FiraMat* __restrict__ mats,
                                                                const FiraScal* __restrict__ scal,
                                                                const FiraEnt* __restrict__ ents,
                                                                const FiraTile* __restrict__ tiles, int ntiles, FiraHp hp) {
  const int ti = xcd_chunked_index(blockIdx.x, ntiles);
  if (ti < 0) return;
  const FiraTile tile = tiles[ti];
  const FiraEnt ent = ents[tile.ent];
  const FiraMat mt = mats[ent.mat];
  const float f = *hp.lr_alpha * scal[ent.mat].c;
  gptr<const T> G = as_global(reinterpret_cast<const T*>(ent.G));
  gptr<T> W = as_global(reinterpret_cast<T*>(ent.W));
  gptr<const float> phi = as_global<const float>(mt.phi);
  const int t = threadIdx.x;
  const long long j = (long long)tile.ta * 256 + 8 * (t & 31);
  if (j >= mt.n) return;
  float kc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) kc[e] = (mt.left && j + e < mt.n) ? f * phi[j + e] : 0.0f;
  for (int p = 0; p < 16; ++p) {
    const long long i = (long long)tile.tb * 128 + (t >> 5) + 8 * p;
    if (i >= mt.m) break;
    if (!mt.left) {
      const float fr = f * phi[i];
#pragma unroll
      for (int e = 0; e < 8; ++e) kc[e] = fr;
    }
    if (sizeof(T) == 2) {
      gptr<const bf16_raw> gr = reinterpret_cast<gptr<const bf16_raw>>(G) + i * mt.ld + j;
      gptr<bf16_raw> wr = reinterpret_cast<gptr<bf16_raw>>(W) + i * mt.ld + j;
      if (j + 8 <= mt.n) {       // rows may start at any element: 2-byte alignment only
        const u32x4 gv = __builtin_nontemporal_load(reinterpret_cast<gptr<const u32x4_a2>>(gr));
        const u32x4 wv = __builtin_nontemporal_load(reinterpret_cast<gptr<const u32x4_a2>>(wr));
        const unsigned gw[4] = {gv.x, gv.y, gv.z, gv.w}, ww[4] = {wv.x, wv.y, wv.z, wv.w};
        unsigned o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const float w0 = __uint_as_float(ww[d] << 16) - kc[2 * d] * __uint_as_float(gw[d] << 16);
          const float w1 = __uint_as_float(ww[d] & 0xffff0000u) - kc[2 * d + 1] * __uint_as_float(gw[d] & 0xffff0000u);
          o[d] = pack_bf16x2(w0, w1);
        }
        __builtin_nontemporal_store(u32x4{o[0], o[1], o[2], o[3]}, reinterpret_cast<gptr<u32x4_a2>>(wr));
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (j + e < mt.n) wr[e] = f32_to_bf16(bf16_to_f32(wr[e]) - kc[e] * bf16_to_f32(gr[e]));
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (j + e < mt.n) {
          gptr<float> wp = reinterpret_cast<gptr<float>>(W) + i * mt.ld + j + e;
          *wp = *wp - kc[e] * reinterpret_cast<gptr<const float>>(G)[i * mt.ld + j + e];
        }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Operand preparation (outside the per-step hot loop)
// ------------------------------------------------------------------------------------------------

// Projector P[S][r] (fp32 or bf16) -> Pn[S][kx*rp] and PT[r][kx*Sp]; split planes follow sequence B.
template <typename TP>
__device__ __forceinline__ void prep_projector_body(const FiraMat& mt, const TP* __restrict__ P) {
  const long long total = (long long)mt.S * mt.r;
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const long long s = idx / mt.r;
    const int a = (int)(idx - s * mt.r);
    float x;
    if (sizeof(TP) == 2) x = bf16_to_f32(*reinterpret_cast<const bf16_raw*>(&P[idx]));
    else x = *reinterpret_cast<const float*>(&P[idx]);
    gptr<bf16_raw> pn = as_global(mt.Pn);
    gptr<bf16_raw> pt = as_global(mt.PT);
    if (mt.kx == 1) {
      const bf16_raw b = f32_to_bf16(x);
      pn[kblk_index(mt.Sq, s, a)] = b;
      pt[kblk_index(mt.rq, a, (int)s)] = b;
    } else {
      bf16_raw h, m, l;
      split3(x, h, m, l);
      const bf16_raw seq[6] = {h, m, h, l, h, m};
#pragma unroll
      for (int p = 0; p < 6; ++p) {
        pn[kblk_index(mt.Sq, s, p * mt.rp + a)] = seq[p];
        pt[kblk_index(mt.rq, a, p * mt.Sp + (int)s)] = seq[p];
      }
    }
  }
}
template <typename TP>
__global__ void fira_prep_projector_kernel(FiraMat mt, const TP* __restrict__ P) { prep_projector_body<TP>(mt, P); }

// fp32 gradient -> split bf16 planes (sequence A), stacked along the contraction axis.
__device__ __forceinline__ void split_gradient_body(const FiraMat& mt, const float* __restrict__ G) {
  const long long total = (long long)mt.m * mt.n;
  gptr<bf16_raw> Gx = as_global(mt.Gx);
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const long long i = idx / mt.n;
    const long long j = idx - i * mt.n;
    bf16_raw h, m, l;
    split3(G[i * mt.ld + j], h, m, l);
    const bf16_raw seq[6] = {h, h, m, h, l, m};
    if (mt.left) {   // contraction over rows i: plane p occupies rows [p*Sp, p*Sp + m)
#pragma unroll
      for (int p = 0; p < 6; ++p) Gx[((long long)p * mt.Sp + i) * mt.gx_ld + j] = seq[p];
    } else {         // contraction over columns j: plane p occupies columns [p*Sp, p*Sp + n)
#pragma unroll
      for (int p = 0; p < 6; ++p) Gx[i * mt.gx_ld + (long long)p * mt.Sp + j] = seq[p];
    }
  }
}
__global__ void fira_split_gradient_kernel(FiraMat mt, const float* __restrict__ G) { split_gradient_body(mt, G); }
// ... for every fp32 matrix of a step's work list in one launch (blockIdx.y = list entry; bf16 entries exit)
__global__ void fira_split_gradients_kernel(const FiraMat* __restrict__ mats, const FiraEnt* __restrict__ ents) {
  const FiraEnt ent = ents[blockIdx.y];
  const FiraMat mt = mats[ent.mat];
  if (mt.kx == 1) return;
  split_gradient_body(mt, reinterpret_cast<const float*>(ent.G));
}

// One float in device memory (the step size lr * alpha), written in stream order.
__global__ void fira_store_float_kernel(float* __restrict__ dst, float value) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *as_global(dst) = value;
}

// fp32 gradient -> its bf16 rounding (nearest even), rows of ldb elements (the projector refresh's way back).
__global__ void fira_round_gradient_kernel(const float* __restrict__ G, bf16_raw* __restrict__ Gb, int m, int n,
                                           long long ld, long long ldb) {
  const long long total = (long long)m * n;
  gptr<bf16_raw> out = as_global(Gb);
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const long long i = idx / n;
    const long long j = idx - i * n;
    out[i * ldb + j] = f32_to_bf16(G[i * ld + j]);
  }
}

// ------------------------------------------------------------------------------------------------
// Gram route to ||S||: g2[i] = sum over the short axis of G(s, i)^2 for every long index i.
//   left  (m <= n): column sums of squares; one workgroup per 256 columns walks all m rows with
//                   row-contiguous 16-byte loads (32 lanes = 512 B of one row), 8 row lanes.
//   right (m >  n): row sums of squares; one wavefront per row.
// Fixed summation order: deterministic.
// ------------------------------------------------------------------------------------------------

__device__ __forceinline__ int find_g2_entry(const FiraEnt* __restrict__ ents, int count, int blk) {
  int lo = 0, hi = count - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (ents[mid].g2b0 <= blk) lo = mid; else hi = mid - 1;
  }
  return lo;
}

template <typename T>
__device__ __forceinline__ void g2_load8(float (&x)[8], gptr<const T> row, long long idx, long long limit);
template <>
__device__ __forceinline__ void g2_load8<bf16_raw>(float (&x)[8], gptr<const bf16_raw> row, long long idx, long long limit) {
  unsigned w[4] = {0u, 0u, 0u, 0u};
  if (idx + 8 <= limit) {
    const u32x4 v = *reinterpret_cast<gptr<const u32x4_a2>>(row + idx);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (idx + e < limit) w[e >> 1] |= ((unsigned)row[idx + e]) << ((e & 1) * 16);
  }
#pragma unroll
  for (int d = 0; d < 4; ++d) { x[2 * d] = __uint_as_float(w[d] << 16); x[2 * d + 1] = __uint_as_float(w[d] & 0xffff0000u); }
}
template <>
__device__ __forceinline__ void g2_load8<float>(float (&x)[8], gptr<const float> row, long long idx, long long limit) {
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = (idx + e < limit) ? row[idx + e] : 0.0f;
}

template <typename T>
__device__ __forceinline__ void g2_block(const FiraMat& mt, const FiraEnt& ent, int blk, float* red) {
  gptr<const T> G = as_global(reinterpret_cast<const T*>(ent.G));
  gptr<float> g2 = as_global(mt.g2);
  const int t = threadIdx.x;
  if (mt.left) {
    const int cc = t & 31, rl = t >> 5;                 // 32 column chunks x 8 row lanes
    const long long j = (long long)blk * 256 + 8 * cc;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (j < mt.n) {
      for (int i = rl; i < mt.m; i += 8) {
        float x[8];
        g2_load8<T>(x, G + (long long)i * mt.ld, j, mt.n);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += x[e] * x[e];
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[(rl * 32 + cc) * 8 + e] = acc[e];
    __syncthreads();
    // thread t sums column t of the block over the 8 row lanes, in order
    const int c = t >> 3, e = t & 7;
    float s = 0.0f;
#pragma unroll
    for (int r8 = 0; r8 < 8; ++r8) s += red[(r8 * 32 + c) * 8 + e];
    const long long col = (long long)blk * 256 + t;
    if (col < mt.n) g2[col] = s;
  } else {
    const int lane = t & 63, wave = t >> 6;
    for (int rr = 0; rr < 8; ++rr) {
      const long long i = (long long)blk * FIRA_G2_ROWS_PER_WG + wave * 8 + rr;
      if (i >= mt.m) break;
      float s = 0.0f;
      for (long long j = 8 * lane; j < mt.n; j += 512) {
        float x[8];
        g2_load8<T>(x, G + i * mt.ld, j, mt.n);
#pragma unroll
        for (int e = 0; e < 8; ++e) s += x[e] * x[e];
      }
      s = wave_sum(s);
      if (lane == 0) g2[i] = s;
    }
  }
}

__global__ __launch_bounds__(256) void fira_gradnorm_kernel(const FiraMat* __restrict__ mats,
                                                            const FiraScal* __restrict__ scal,
                                                            const FiraEnt* __restrict__ ents, int count,
                                                            int total_blocks, FiraHp hp) {
  __shared__ float red[256 * 8];
  const int b = blockIdx.x;
  if (b >= total_blocks) return;
  const int e = find_g2_entry(ents, count, b);
  const FiraEnt ent = ents[e];
  if (!have_g2(hp)) return;
  const FiraMat mt = mats[ent.mat];
  if (mt.dtype == 1) return;   // bf16 matrices: the projection kernel accumulates ||G_i||^2 itself
  g2_block<float>(mt, ent, b - ent.g2b0, red);
}

// ------------------------------------------------------------------------------------------------
// Gate of the Gram route, evaluated when a projector is installed: a randomized estimate of
// ||P^T P - I|| from 4 sign vectors x (err = max_t ||P^T (P x_t) - x_t|| / ||x_t||), on the bf16
// operand copy of P that the contractions use.  Two small kernels: y_t = P x_t (one wavefront per
// row of P), then z_t = P^T y_t - x_t (one workgroup, threads along the rank axis).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float ortho_sign(int a, int trial) {
  const unsigned h = ((unsigned)a * 2654435761u) ^ ((unsigned)trial * 2246822519u + 374761393u);
  return ((h >> 15) & 1u) ? 1.0f : -1.0f;
}

__device__ __forceinline__ void ortho_y_body(const FiraMat& mt, float* __restrict__ y /* [S][4] */) {
  gptr<const bf16_raw> Pn = as_global<const bf16_raw>(mt.Pn);
  const int lane = threadIdx.x & 63;
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= mt.S) return;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int a = lane; a < mt.r; a += 64) {
    const float p = bf16_to_f32(Pn[kblk_index(mt.Sq, s, a)]);
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] += p * ortho_sign(a, t);
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = wave_sum(acc[t]);
  if (lane == 0) {
#pragma unroll
    for (int t = 0; t < 4; ++t) as_global(y)[(long long)s * 4 + t] = acc[t];
  }
}

__global__ __launch_bounds__(256) void fira_ortho_y_kernel(FiraMat mt, float* __restrict__ y) { ortho_y_body(mt, y); }

// z-partials: workgroup b sums rows [b*chunk, (b+1)*chunk) of P^T y for all four trials.
__device__ __forceinline__ void ortho_z_body(const FiraMat& mt, const float* __restrict__ y,
                                             float* __restrict__ zpart /* [splits][r][4] */) {
  gptr<const bf16_raw> Pn = as_global<const bf16_raw>(mt.Pn);
  gptr<const float> yy = as_global(y);
  const int chunk = (mt.S + FIRA_ORTHO_SPLITS - 1) / FIRA_ORTHO_SPLITS;
  const int s0 = blockIdx.x * chunk, s1 = min(mt.S, s0 + chunk);
  for (int a = threadIdx.x; a < mt.r; a += 256) {
    float z[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = s0; s < s1; ++s) {
      const float p = bf16_to_f32(Pn[kblk_index(mt.Sq, s, a)]);
#pragma unroll
      for (int k = 0; k < 4; ++k) z[k] += p * yy[(long long)s * 4 + k];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) as_global(zpart)[((long long)blockIdx.x * mt.r + a) * 4 + k] = z[k];
  }
}

__global__ __launch_bounds__(256) void fira_ortho_z_kernel(FiraMat mt, const float* __restrict__ y, float* __restrict__ zpart) {
  ortho_z_body(mt, y, zpart);
}

__device__ __forceinline__ void ortho_final_body(const FiraMat& mt, const float* __restrict__ zpart,
                                                 FiraScal* __restrict__ scal, int mat, float (&red)[4][4]) {
  gptr<const float> zp = as_global(zpart);
  const int t = threadIdx.x;
  float zz[4] = {0.f, 0.f, 0.f, 0.f};
  for (int a = t; a < mt.r; a += 256) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float z = 0.0f;
      for (int b = 0; b < FIRA_ORTHO_SPLITS; ++b) z += zp[((long long)b * mt.r + a) * 4 + k];
      const float d = z - ortho_sign(a, k);
      zz[k] += d * d;
    }
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) zz[k] = wave_sum(zz[k]);
  if ((t & 63) == 0) {
#pragma unroll
    for (int k = 0; k < 4; ++k) red[t >> 6][k] = zz[k];
  }
  __syncthreads();
  if (t == 0) {
    float worst = 0.0f;
    for (int k = 0; k < 4; ++k)
      worst = fmaxf(worst, sqrtf(((red[0][k] + red[1][k]) + (red[2][k] + red[3][k])) / (float)mt.r));
    as_global(scal)[mat].ortho_err = worst;
    as_global(scal)[mat].gram_err = INFINITY;   // to be measured on the next step
  }
}
__global__ __launch_bounds__(256) void fira_ortho_final_kernel(FiraMat mt, const float* __restrict__ zpart,
                                                               FiraScal* __restrict__ scal, int mat) {
  __shared__ float red[4][4];
  ortho_final_body(mt, zpart, scal, mat, red);
}
