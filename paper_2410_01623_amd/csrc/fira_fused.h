// Projection and Adam in one kernel (Algorithm 1: R = P^T G, the moment updates of Eqs. 2-4, the factor
// k_i of Eq. 11, and the back-projection operand Z_i = N_i - k_i R_i).
//
// When the rank fits one workgroup (r <= 512) the whole row R_i of a factor sits in the accumulators of
// the workgroup that projected it, so Adam can run on it there: R never goes to memory, and neither
// does a second launch read it back.  Per factor and rank component that leaves M and V read and
// written once (16 B) and Z written once (2 B), against 26 B for the two-kernel sequence.
//
// Tile: 128 factors x 256 RT rank components, 256 RT threads; wave w holds all 128 factors x rank
// components 64 w .. 64 w + 63 (RT = 1: r <= 256, two workgroups per CU; RT = 2: r <= 512, one per CU,
// the two rank tiles share one copy of the gradient tile, which is then read from memory once).
// The multiply phase is proj_pipeline.  The epilogue cannot keep many loads of M and V in flight from
// registers (the accumulators fill them), so M and V travel through LDS, which the multiply phase
// has left free: the tile is worked through in eight chunks of 16 factors, and while chunk c is
// processed the rows of M and V of chunk c + 1 arrive by LDS-direct loads (1 KB per instruction) in the
// other of two landing buffers.  Per chunk:
//   1. every lane updates M and V in place in the landing buffer for its 16 elements, forms N (kept in
//      registers) and sums N^2 and R^2 per factor; the sums are reduced over the 32 lanes that share a
//      factor (a reduce-scatter, fixed order) and left in LDS per wave;
//   2. one thread per factor adds the waves' sums in order, forms k_i, writes phi and q;
//   3. Z = N - k R is rounded to bf16 into an LDS image of the K-blocked operand;
//   4. the new M and V and Z leave LDS in 16-byte pieces, whole rows contiguous.
// Waits on the LDS-direct loads are explicit (see fira_gemm.h).  The wait for chunk c + 1 stands between
// steps 3 and 4 of chunk c, before the chunk's stores are issued, and waits for everything in flight: that
// is the loads of chunk c + 1 and the stores of chunk c - 1, which are a whole chunk old.  The stores of
// chunk c then stay in flight while chunk c + 1 is processed.  No count of instructions, and no
// assumption about the order in which loads and stores retire relative to each other, is involved.
//
// A step takes this kernel only if every listed matrix is bf16 with r % 4 == 0, 128 <= r <= 512, column
// factors, Algorithm 1 proper, and the Gram route to ||S|| (no operand copy of R is made here).
// The limiter runs after it; for a matrix whose factor c came out below 1, fira_makez_kernel turns the Z
// written here (for c = 1) into c Z + (1 - c) N, with N formed again from the updated M and V.
#pragma once
#include "fira_device.h"
#include "fira_elementwise.h"
#include "fira_gemm.h"

#define FIRA_FUSE_F 16   // factors per chunk of the epilogue
#define FIRA_FUSE_LDS_MAIN(RT) (FIRA_PROJ_LDS_A + FIRA_RING_STAGES * (RT) * FIRA_PROJ_RING_STAGE)
// two landing buffers (M and V of a chunk, fp32), the Z image (bf16), per-wave sums, ||G_i||^2 of the tile, k_i
#define FIRA_FUSE_LDS_EPI(RT) (2 * FIRA_FUSE_F * 256 * (RT) * 8 + FIRA_FUSE_F * 256 * (RT) * 2 + 4 * (RT) * FIRA_FUSE_F * 8 + 128 * 4 + FIRA_FUSE_F * 4)
#define FIRA_FUSE_LDS(RT) (FIRA_FUSE_LDS_MAIN(RT) > FIRA_FUSE_LDS_EPI(RT) ? FIRA_FUSE_LDS_MAIN(RT) : FIRA_FUSE_LDS_EPI(RT))

// Sum of x[v] over the 32 lanes of a half wave, for 8 values at once.  Afterwards every lane holds the
// total of value  v = 4*bit4(l) + 2*bit3(l) + bit2(l).
__device__ __forceinline__ float half_wave_reduce8(const float (&x)[8]) {
  const int lane = threadIdx.x & 63;
  float a[4], b[2];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float keep = (lane & 16) ? x[4 + j] : x[j], send = (lane & 16) ? x[j] : x[4 + j];
    a[j] = keep + __shfl_xor(send, 16, 64);
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const float keep = (lane & 8) ? a[2 + j] : a[j], send = (lane & 8) ? a[j] : a[2 + j];
    b[j] = keep + __shfl_xor(send, 8, 64);
  }
  const float keep = (lane & 4) ? b[1] : b[0], send = (lane & 4) ? b[0] : b[1];
  float d = keep + __shfl_xor(send, 4, 64);
  d += __shfl_xor(d, 2, 64);
  d += __shfl_xor(d, 1, 64);
  return d;
}

template <int RT, bool INTERIOR>
__device__ __forceinline__ void project_adam_epilogue(f32x16_t (&acc)[4][2], char* lds, const FiraMat& mt, const FiraHp& hp,
                                                      float bias, int a_row0, const float (&sq)[4]) {
  constexpr int NW = 4 * RT, THREADS = 256 * RT, C = 256 * RT, F = FIRA_FUSE_F;
  constexpr int ARR = F * C * 4;                                   // bytes of one array (M or V) of a chunk
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l32 = lane & 31, hi = lane >> 5;
  bf16_raw* zl = reinterpret_cast<bf16_raw*>(lds + 4 * ARR);       // [C / 32 K blocks][16 factors][32]
  float* part = reinterpret_cast<float*>(lds + 4 * ARR + F * C * 2);   // [NW][16 factors][2]
  float* g2s = part + NW * F * 2;                                  // [128]
  float* ks = g2s + 128;                                           // [16]
  const unsigned lds0 = (unsigned)(size_t)(lds_ptr)lds;
  const int r = mt.r, L = mt.L;
  const int kblocks = mt.rp >> 5;
  const char* Mg = reinterpret_cast<const char*>(mt.M);
  const char* Vg = reinterpret_cast<const char*>(mt.V);

  // Requests of chunk c: 16 rows x RT pieces of 256 floats for each of M and V, 8 instructions per wave.
  auto request = [&](int c) {
    const unsigned dst0 = lds0 + (unsigned)((c & 1) * 2 * ARR);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int q = wave * 8 + i;                                  // 0 .. 32 RT - 1
      const int arr = q / (F * RT), row = (q % (F * RT)) / RT, piece = q % RT;
      const long long grow = (long long)a_row0 + F * c + row;
      const char* src = (arr ? Vg : Mg) + (grow * r + piece * 256) * 4;
      const unsigned dst = dst0 + (unsigned)(arr * ARR + (row * C + piece * 256) * 4);
      if (INTERIOR) {
        lds_dma16(src, (unsigned)lane * 16u, dst);
      } else if (grow < L) {
        if (piece * 256 + lane * 4 < r) lds_dma16(src, (unsigned)lane * 16u, dst);
      }
    }
  };

  __syncthreads();                                                 // the multiply phase is done with LDS
  request(0);
  if (wave == 0) {
    gptr<float> g2 = as_global(mt.g2);
#pragma unroll
    for (int tm = 0; tm < 4; ++tm) {
      const float tot = sq[tm] + __shfl_xor(sq[tm], 32, 64);
      const int row = a_row0 + 32 * tm + l32;
      if (lane < 32) {
        g2s[32 * tm + l32] = tot;
        if (row < L) g2[row] = tot;
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // the factor (of a chunk of 16) whose sums this lane holds after half_wave_reduce8
  const int vown = (lane >> 2) & 7;
  const int rl_own = 8 * (vown >> 2) + 4 * hi + (vown & 3);
  // this lane's element (v', tn) of a chunk sits at float index (8*(v'>>2) + 4*hi + (v'&3)) * C + 64*wave + 32*tn + l32
  const int lane_idx = 4 * hi * C + 64 * wave + l32;

  // (one call per chunk with the chunk index as a type: the accumulators must be indexed statically)
  auto chunk = [&](auto c_c) {
    constexpr int c = decltype(c_c)::value, tm = c >> 1, h = c & 1;
    const int row_c = a_row0 + F * c;                              // first factor of the chunk
    float* landM = reinterpret_cast<float*>(lds + (c & 1) * 2 * ARR);
    float* landV = landM + F * C;
    if (c + 1 < 8) request(c + 1);
    float nv[2][8], nn[8], rr[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) nn[v] = rr[v] = 0.0f;
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
      const int col = 64 * wave + 32 * tn + l32;
#pragma unroll
      for (int v = 0; v < 8; ++v) {
        const int dr = 8 * (v >> 2) + (v & 3);
        const int idx = lane_idx + dr * C + 32 * tn;
        const bool ok = INTERIOR || (col < r && row_c + 4 * hi + dr < L);
        const float x = acc[tm][tn][8 * h + v];
        const float m0 = ok ? landM[idx] : 0.0f, v0 = ok ? landV[idx] : 0.0f;
        const float m1 = hp.b1 * m0 + hp.omb1 * x;
        const float v1 = hp.b2 * v0 + hp.omb2 * (x * x);
        float n = adam_direction(m1, v1, bias, hp.epsf);
        if (!ok) n = 0.0f;
        landM[idx] = m1;
        landV[idx] = v1;
        nv[tn][v] = n;
        nn[v] += n * n;
        rr[v] += x * x;
      }
    }
    {
      const float tn_ = half_wave_reduce8(nn), tr_ = half_wave_reduce8(rr);
      if ((lane & 3) == 0) *reinterpret_cast<float2*>(part + (wave * F + rl_own) * 2) = float2{tn_, tr_};
    }
    __syncthreads();
    if (threadIdx.x < F) {
      float snn = 0.0f, srr = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float2 p = *reinterpret_cast<const float2*>(part + (w * F + threadIdx.x) * 2);
        snn += p.x;
        srr += p.y;
      }
      const int row = row_c + threadIdx.x;
      float k = sqrtf(snn) / (sqrtf(srr) + hp.epsf);
      if (row < L) {
        as_global(mt.phi)[row] = k;
        as_global(mt.q)[row] = k * k * residual_sq(hp, g2s[F * c + threadIdx.x], srr);
      } else {
        k = 0.0f;
      }
      ks[threadIdx.x] = k;
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const f32x4 kq = *reinterpret_cast<const f32x4*>(ks + 8 * g + 4 * hi);
#pragma unroll
      for (int tn = 0; tn < 2; ++tn) {
        const int kb = 2 * wave + tn;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = 4 * g + e;
          const bool ok = INTERIOR || (64 * wave + 32 * tn + l32 < r && row_c + 8 * g + 4 * hi + e < L);
          const float z = ok ? nv[tn][v] - kq[e] * acc[tm][tn][8 * h + v] : 0.0f;
          zl[(kb * F + 8 * g + 4 * hi + e) * 32 + l32] = f32_to_bf16(z);
        }
      }
    }
    __syncthreads();
    // The next chunk has landed (this wave's share of it).  The wait stands before this chunk's stores are
    // issued, so that it can be "everything": the only other operations in flight are the previous chunk's
    // stores, which have had this whole chunk to complete.  (Placed after the stores, the wait would have
    // to let exactly their number stay in flight, which is right only if stores never retire before older
    // loads and the compiler emits exactly the instructions counted.)
    if (c + 1 < 8) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // M and V: 2 x 16 rows x C/4 pieces of 16 bytes, 8 per thread; Z: C/32 K blocks x 1 KB, 2 per thread
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int arr = i >> 2, rem = threadIdx.x + THREADS * (i & 3);
      const int row = rem / (C / 4), c4 = rem % (C / 4);
      const long long grow = (long long)row_c + row;
      if (INTERIOR || (grow < L && 4 * c4 < r)) {
        const u32x4 val = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(landM) + arr * ARR + (row * C + 4 * c4) * 4);
        gptr<char> dst = reinterpret_cast<gptr<char>>(as_global(arr ? mt.V : mt.M)) + (grow * r + 4 * c4) * 4;
        *reinterpret_cast<gptr<u32x4>>(dst) = val;
      }
    }
    {
      gptr<char> nb = reinterpret_cast<gptr<char>>(as_global(mt.Nb));
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int p = threadIdx.x + THREADS * i;                   // 16-byte piece: K block p / 64, piece p % 64 of its 1 KB
        const int kb = p >> 6;
        if (INTERIOR || kb < kblocks)
          *reinterpret_cast<gptr<u32x4>>(nb + ((long long)kb * mt.Lq + row_c) * 64 + (p & 63) * 16) =
              *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(zl) + p * 16);
      }
    }
    // everybody's share of the next chunk has landed, and all are done reading this chunk's LDS (the stores
    // above have read it into registers: the compiler waits for those LDS reads before the barrier)
    if (c + 1 < 8) __syncthreads();
  };
  chunk(std::integral_constant<int, 0>{});
  chunk(std::integral_constant<int, 1>{});
  chunk(std::integral_constant<int, 2>{});
  chunk(std::integral_constant<int, 3>{});
  chunk(std::integral_constant<int, 4>{});
  chunk(std::integral_constant<int, 5>{});
  chunk(std::integral_constant<int, 6>{});
  chunk(std::integral_constant<int, 7>{});
}

template <bool LEFT, int RT>
__device__ __forceinline__ void project_adam_tile(char* lds, const FiraMat* __restrict__ mats, const FiraScal* __restrict__ scal,
                                                  const FiraEnt* __restrict__ ents, const FiraTile& tile, const FiraHp& hp) {
  const FiraEnt ent = ents[tile.ent];
  if (!use_gram(hp, scal[ent.mat])) return;    // this matrix takes the residual route: the two-kernel path serves it
  const FiraMat mt = mats[ent.mat];

  GemmOperands g;
  g.a_row0 = tile.ta * FIRA_PA;
  g.a_rows = mt.L;
  g.b_row0 = 0;
  g.b_rows = mt.r;
  g.B = as_global<const bf16_raw>(mt.PT);
  g.ldb = mt.rq;
  g.KB = mt.Sp;
  g.A = as_global(reinterpret_cast<const bf16_raw*>(ent.G));
  g.lda = mt.ld;
  g.KA = mt.S;
  // bias correction with the 1-based step count (Eq. 4), in double as in fira_adam_kernel
  const int t = scal[ent.mat].t + 1;
  const float bias = (float)(sqrt(1.0 - pow(hp.beta2, (double)t)) / (1.0 - pow(hp.beta1, (double)t)));
  f32x16_t acc[4][2];
  float sq[4];
#pragma unroll
  for (int tm = 0; tm < 4; ++tm) {
    sq[tm] = 0.0f;
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.0f;
  }
  const int wave = threadIdx.x >> 6;
  const bool interior = g.a_row0 + FIRA_PA <= g.a_rows && g.KA == g.KB;
  if (interior) {
    if (wave == 0) proj_pipeline<LEFT, true, true, RT>(acc, lds, g, sq);
    else if (RT == 1 || wave < 4) proj_pipeline<LEFT, true, false, RT>(acc, lds, g, sq);
    else proj_pipeline<LEFT, true, false, 2, false>(acc, lds, g, sq);
  } else {
    if (wave == 0) proj_pipeline<LEFT, false, true, RT>(acc, lds, g, sq);
    else if (RT == 1 || wave < 4) proj_pipeline<LEFT, false, false, RT>(acc, lds, g, sq);
    else proj_pipeline<LEFT, false, false, 2, false>(acc, lds, g, sq);
  }
  if (g.a_row0 + FIRA_PA <= mt.L && mt.r == 256 * RT) project_adam_epilogue<RT, true>(acc, lds, mt, hp, bias, g.a_row0, sq);
  else project_adam_epilogue<RT, false>(acc, lds, mt, hp, bias, g.a_row0, sq);
}

// One grid for both orientations: workgroups [0, blocks_left) take the tiles of the matrices with
// m <= n, the rest those with m > n.  With one workgroup per CU (RT = 2) a launch ends in a round that is
// only partly filled; one launch instead of two has one such round.  blocks_left is a multiple of 8,
// which keeps the XCD-aware mapping of each part.
template <int RT>
__global__ __launch_bounds__(256 * RT, RT == 1 ? 2 : 1) void fira_project_adam_kernel(const FiraMat* __restrict__ mats,
                                                                                      const FiraScal* __restrict__ scal,
                                                                                      const FiraEnt* __restrict__ ents,
                                                                                      const FiraTile* __restrict__ tiles_left, int ntiles_left,
                                                                                      int blocks_left,
                                                                                      const FiraTile* __restrict__ tiles_right, int ntiles_right,
                                                                                      FiraHp hp) {
  extern __shared__ __attribute__((aligned(16))) char lds[];   // FIRA_FUSE_LDS(RT) bytes
  if ((int)blockIdx.x < blocks_left) {
    const int ti = xcd_chunked_index(blockIdx.x, ntiles_left);
    if (ti < 0) return;
    project_adam_tile<true, RT>(lds, mats, scal, ents, tiles_left[ti], hp);
  } else {
    const int ti = xcd_chunked_index((int)blockIdx.x - blocks_left, ntiles_right);
    if (ti < 0) return;
    project_adam_tile<false, RT>(lds, mats, scal, ents, tiles_right[ti], hp);
  }
}
