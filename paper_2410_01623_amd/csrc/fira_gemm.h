// Grouped bf16 MFMA contractions of the Fira step for gfx950 (v_mfma_f32_32x32x16_bf16).
//
// Every contraction has the form  D[a][b] = sum_k A[a][k] * B[b][k]  ("A" is the MFMA A operand,
// "B" the MFMA B operand) and runs in 256-thread workgroups, two per CU, each wavefront owning a
// 128 (A) x 64 (B) block of accumulators.  Two independent workgroups per CU matter more than a
// bigger tile: the phases of one (operand requests, LDS traffic, the HBM-bound epilogue) overlap the
// multiplies of the other, which a single workgroup in lockstep on its barriers cannot do.
//
// Operands that the library stores itself (P in both orientations, Z, R) are K-blocked
// ([K/32][rows][32], see kblk_index) and go from global memory straight into an LDS ring with
// LDS-direct loads.  The gradient is the caller's: its rows start at any 2-byte boundary and, when P
// multiplies from the left, it is K-slow (element (a, k) at base[k*ld + a]); it passes through
// registers (K-slow: 4(k) x 8(a) blocks, row-contiguous 16-byte loads, transposed in registers
// before the LDS write).
//
// Accumulator layout of one 32 x 32 block (per lane, 16 floats v = 0..15):
//     b (B row) = lane % 32,   a (A row) = 8*(v/4) + 4*(lane/32) + v%4
// so a lane owns 4 consecutive A rows per group of 4 registers.
#pragma once
#include <type_traits>
#include "fira_device.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;


// [row][64 k] bf16 tile, 128 B per row, 16-byte chunks XOR-swizzled by row so that fragment reads
// and tile writes spread over all banks.
__device__ __forceinline__ int lds_tile_off(int row, int chunk) {
  return row * 128 + (((chunk ^ row ^ (row >> 3) ^ (row >> 6)) & 7) << 4);
}

// 8 consecutive bf16 of a row that has `limit` valid elements, starting at element idx; elements
// outside [0, limit) read as zero and are never touched in memory.  No alignment assumed.
// Branch-free for limit >= 8: the 16-byte load is moved back so that it ends inside the row and the
// value is shifted down again, which also shifts zeros into the out-of-range positions.  (A ragged
// chunk handled with per-element loads costs a serialized memory round trip per element.)
__device__ __forceinline__ u32x4 load8_bf16(gptr<const bf16_raw> row, long long idx, long long limit) {
  if (limit >= 8) {
    long long start = idx < limit - 8 ? idx : limit - 8;
    if (start < 0) start = 0;
    const u32x4 v = *reinterpret_cast<gptr<const u32x4_a2>>(row + start);
    const long long d = idx - start;          // elements to shift out at the low end
    const unsigned sh = d < 8 ? (unsigned)d : 8u;
    // 128-bit logical shift right by 16*sh bits
    const unsigned long long lo = ((unsigned long long)v.y << 32) | v.x, hi = ((unsigned long long)v.w << 32) | v.z;
    const unsigned bits = 16u * sh;
    unsigned long long rlo, rhi;
    if (bits == 0) { rlo = lo; rhi = hi; }
    else if (bits < 64) { rlo = (lo >> bits) | (hi << (64 - bits)); rhi = hi >> bits; }
    else if (bits < 128) { rlo = hi >> (bits - 64); rhi = 0; }
    else { rlo = 0; rhi = 0; }
    return u32x4{(unsigned)rlo, (unsigned)(rlo >> 32), (unsigned)rhi, (unsigned)(rhi >> 32)};
  }
  unsigned w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e)
    if (idx + e >= 0 && idx + e < limit) w[e >> 1] |= ((unsigned)row[idx + e]) << ((e & 1) * 16);
  return u32x4{w[0], w[1], w[2], w[3]};
}

struct GemmOperands {
  gptr<const bf16_raw> A;  // A side
  long long lda;      // gradient operand: elements between consecutive A rows (K-contiguous) or K steps
                      // (K-slow); K-blocked operand: its padded row count
  int a_row0, a_rows; // first A row of this tile, number of valid A rows
  int KA;             // valid contraction length on the A side (elements beyond read as zero)
  gptr<const bf16_raw> B;  // B side: always K-blocked, zero padded to a multiple of 64 in K
  long long ldb;      // padded row count of B
  int b_row0, b_rows;
  int KB;             // stored contraction length of B (>= KA, a multiple of 64)
  int wrapA = 0, wrapB = 0;   // ring core only: K blocks of 32 after which the operand repeats (Z in two planes meets P twice); 0 = never
};

// Fragments of one k-slice (16) of a wave's 128 (A) x 64 (B) block and its 8 MFMAs.
struct Frags { bf16x8_t a[4], b[2]; };
__device__ __forceinline__ void gemm_mfma_slice(f32x16_t (&acc)[4][2], const Frags& f) {
#pragma unroll
  for (int tm = 0; tm < 4; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
      acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[tm], f.b[tn], acc[tm][tn], 0, 0, 0);
}
// Sum of squares of the A fragments (v_dot2c_f32_bf16: two bf16 products per instruction): with the
// gradient on the A side this accumulates ||G_i||^2 for the wave's A rows at no extra memory traffic.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void gemm_sumsq_slice(float (&sq)[4], const Frags& f) {
#pragma unroll
  for (int tm = 0; tm < 4; ++tm) {
    const u32x4 w = __builtin_bit_cast(u32x4, f.a[tm]);
    const unsigned d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bf16x2_t v = __builtin_bit_cast(bf16x2_t, d[e]);
      sq[tm] = __builtin_amdgcn_fdot2_f32_bf16(v, v, sq[tm], false);
    }
  }
}
// ------------------------------------------------------------------------------------------------
// Ring core for the rank-axis contractions (K = r is short, the epilogue is long): 256 threads,
// 256 (A) x 128 (B) tile, two workgroups per CU, so one runs its HBM-bound epilogue while the other
// multiplies.  Both operands are K-blocked, so they go from global memory straight into LDS
// (global_load_lds_dwordx4: lane l of a wave writes 16 bytes at M0 + 16*l) without passing through
// registers, and one load instruction (16 rows x 32 k) reads 1 KB of contiguous memory: row
// segments of 64 B spread over 16 separate rows reach only two thirds of that L2 bandwidth.
// LDS holds a ring of three K stages of 32
// ([row][32 k] bf16, 64 B per row, 24 KB per stage): while stage s is multiplied, stages s+1 and
// s+2 are in flight, and there is one barrier per stage.
//
// The loads are written as inline assembly because the compiler, which cannot tell the ring's
// buffers apart, would wait for every outstanding LDS-direct load before each fragment read.  The
// waits are explicit instead: loads retire in order, so vmcnt(6) (one stage = 6 loads per thread)
// means "everything but the newest stage has landed".  Other vector memory operations the compiler
// may have in flight only make that wait stricter.
//
// Slot layout of a stage: the 16-byte chunk c (8 k) of row r sits at  r*64 + 16*((c ^ f(r)) & 3),
// f(r) = bit2(r) | (bit3(r) ^ bit1(r)) << 1, which makes the fragment reads (32 consecutive rows,
// one chunk) hit distinct 16-byte bank groups within every aligned group of 8 and of 16 lanes.
// Since a lane may fetch any global address, the loader realises the permutation on the global
// side: lane l of a load covers row l/4 of a 16-row group and fetches chunk (l%4) ^ f(l/4).
// Operand rows are padded to whole tiles (zeros), so no row index needs clamping; what the padding
// rows produce lands in accumulators that are never stored.
// ------------------------------------------------------------------------------------------------
#define FIRA_BACK_THREADS 256
#define FIRA_RK 32
#define FIRA_RING_A (FIRA_BA * 64)
#define FIRA_RING_B (FIRA_BB * 64)
#define FIRA_RING_STAGE (FIRA_RING_A + FIRA_RING_B)
#define FIRA_RING_STAGES 3
#define FIRA_RING_LDS (FIRA_RING_STAGES * FIRA_RING_STAGE)

typedef __attribute__((address_space(3))) char* lds_ptr;

__device__ __forceinline__ int ring_swz(int row) { return ((row >> 2) & 1) | ((((row >> 3) ^ (row >> 1)) & 1) << 1); }
__device__ __forceinline__ int ring_tile_off(int row, int chunk) {
  return row * 64 + (((chunk ^ ring_swz(row)) & 3) << 4);
}

// 16 bytes per lane from base + voff (base wave-uniform) to LDS byte address lds_addr + 16*lane.
// M0 is not preserved; on this target the compiler loads M0 right before each of its own uses.
__device__ __forceinline__ void lds_dma16(const void* base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(base), "s"(lds_addr) : "memory");
}

__device__ __forceinline__ void ring_compute(f32x16_t (&acc)[4][2], const char* stage) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const char* la = stage;
  const char* lb = stage + FIRA_RING_A;
  Frags f[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const int chunk = 2 * kk + (lane >> 5);
#pragma unroll
    for (int t = 0; t < 4; ++t)
      f[kk].a[t] = *reinterpret_cast<const bf16x8_t*>(la + ring_tile_off(wm * 128 + 32 * t + (lane & 31), chunk));
#pragma unroll
    for (int t = 0; t < 2; ++t)
      f[kk].b[t] = *reinterpret_cast<const bf16x8_t*>(lb + ring_tile_off(wn * 64 + 32 * t + (lane & 31), chunk));
  }
  gemm_mfma_slice(acc, f[0]);
  gemm_mfma_slice(acc, f[1]);
}

// Both operands K-blocked with lda / ldb padded rows (multiples of 256) and KB stored k (a multiple
// of 64).
__device__ __forceinline__ void ring_mainloop(f32x16_t (&acc)[4][2], char* lds, const GemmOperands& g) {
#pragma unroll
  for (int tm = 0; tm < 4; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.0f;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned lds0 = (unsigned)(size_t)(lds_ptr)lds;
  const int KT = g.KB / FIRA_RK;
  const int lrow = lane >> 2;
  const int chunk = (lane & 3) ^ ring_swz(lrow);
  const unsigned off = (unsigned)(lrow * 64 + chunk * 16);   // inside a 16-row group (1 KB, contiguous)
  // this wave's first group of each operand in K block 0; a K block is rows * 64 bytes further
  const char* pa = reinterpret_cast<const char*>((const bf16_raw*)g.A) + ((long long)g.a_row0 + 64 * wave) * 64;
  const char* pb = reinterpret_cast<const char*>((const bf16_raw*)g.B) + ((long long)g.b_row0 + 32 * wave) * 64;
  auto issue = [&](int s) {
    const unsigned dst = lds0 + (unsigned)((s % FIRA_RING_STAGES) * FIRA_RING_STAGE);
    const int sa = (g.wrapA && s >= g.wrapA) ? s - g.wrapA : s, sb = (g.wrapB && s >= g.wrapB) ? s - g.wrapB : s;
    const char* ka = pa + (long long)sa * g.lda * 64;
    const char* kb = pb + (long long)sb * g.ldb * 64;
#pragma unroll
    for (int q = 0; q < 4; ++q) lds_dma16(ka + q * 1024, off, dst + (unsigned)((4 * wave + q) * 1024));
#pragma unroll
    for (int q = 0; q < 2; ++q) lds_dma16(kb + q * 1024, off, dst + (unsigned)(FIRA_RING_A + (2 * wave + q) * 1024));
  };
  issue(0);
  if (KT > 1) issue(1);
  for (int s = 0; s < KT; ++s) {
    // stage s has landed (this wave's share), then everybody's; everybody is also done with stage s-1
    if (s + 1 < KT) asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    if (s + 2 < KT) issue(s + 2);            // into the buffer of stage s-1
    ring_compute(acc, lds + (s % FIRA_RING_STAGES) * FIRA_RING_STAGE);
  }
}

// ------------------------------------------------------------------------------------------------
// Kernel 1 (pipelined form): low-rank gradient, long-side major:  Rt[i][a] = sum_s G(s, i) P[s][a]
//   LEFT  (m <= n): i = column of G, s = row of G      -> A side is G read K-slow
//   RIGHT (m >  n): i = row of G,    s = column of G   -> A side is G read K-contiguous
//   B side is PT (rank rows, short side along K, K-blocked).
// 256 threads, 128 (A: gradient side) x 256 (B: rank) tile, two independent workgroups per CU so
// that the load/store phases of one overlap the multiplies of the other.  Wave w owns all 128 A rows
// and B rows 64 w .. 64 w + 63.
//   B goes straight from global memory into a three-stage LDS ring (K stages of 32, as in the ring
//   core above).
//   A cannot: a gradient row starts at any 2-byte boundary and the left orientation needs a
//   transpose.  It passes through registers, one K stage of 64 per two ring stages, into a single
//   128-B-per-row LDS tile.
// Per K stage of 64 ("E" half, then "O" half; D(s) = ring stage s of B, A(S) = register stage):
//   E: wait A(S), D(2S); barrier; registers -> LDS A; request D(2S+2), A(S+1); barrier; multiply
//      k = 0..31 of the stage
//   O: wait D(2S+1); barrier; request D(2S+3); multiply k = 32..63
// All requests of the interior path are inline assembly, so the waits can be exact: loads retire in
// order, each request group is 4 instructions per thread, and the queue order is
// A(0) D(0) D(1) | D(2) A(1) | D(3) | D(4) A(2) | D(5) ...; E waits with vmcnt(4) (only the newest
// D may be in flight), O with vmcnt(8).  Edge tiles load A with ordinary guarded loads at the same
// points of the sequence; the compiler's own waits for those only wait longer.
// ------------------------------------------------------------------------------------------------
#define FIRA_PROJ_THREADS 256
#define FIRA_PROJ_LDS_A (FIRA_PA * 128)
#define FIRA_PROJ_RING_STAGE (FIRA_PB * 64)
#define FIRA_PROJ_LDS (FIRA_PROJ_LDS_A + FIRA_RING_STAGES * FIRA_PROJ_RING_STAGE)

// 16 bytes per lane from base + voff into registers; the result may only be read after a wait that
// names the registers (wait_loads below; the names also go into a comment on the instruction, which
// is what the static check of the compiled code keys on).
__device__ __forceinline__ void gload16_async(u32x4& dst, const void* base, unsigned voff) {
  asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads(u32x4 (&r)[4]) {
  static_assert(N == 4 || N == 1 || N == 0, "queue depths used by the projection pipelines");
  if (N == 4) asm volatile("s_waitcnt vmcnt(4) ; %0 %1 %2 %3" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) :: "memory");
  else if (N == 1) asm volatile("s_waitcnt vmcnt(1) ; %0 %1 %2 %3" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) :: "memory");
  else asm volatile("s_waitcnt vmcnt(0) ; %0 %1 %2 %3" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) :: "memory");
}

// Thread -> element mapping of the A loaders (256 threads, 64 k x 128 rows per stage):
//   K-contiguous: chunk cc = t & 7, rows rr + 32*q, rr = t >> 3, q = 0..3.
//   K-slow:       one 4(k) x 8(a) block per thread: a-block ib (16), k-quad kq (16).  Thread bits
//                 [0:3) -> ib low, bit 3 -> kq low, bit 4 -> ib high, bits [5:8) -> kq high: 8 lanes
//                 read 128 contiguous bytes of one gradient row, and any 16 consecutive lanes write
//                 16 distinct 8-byte LDS slots of a 128-byte bank window (8 chunk positions from the
//                 row swizzle x the two halves of a chunk from kq's low bit).
__device__ __forceinline__ int proj_kslow_ib(int t) { return (t & 7) | ((t >> 1) & 8); }
__device__ __forceinline__ int proj_kslow_kq(int t) { return ((t >> 3) & 1) | ((t >> 4) & ~1); }

template <bool LEFT, bool FAST>
struct ProjALoader {
  const GemmOperands& g;
  const char* base;       // wave-uniform, advances along K
  unsigned off[4];        // byte offsets of this thread's four 16-byte loads
  long long step;         // bytes per K stage of 64
  int k0;
  __device__ __forceinline__ ProjALoader(const GemmOperands& g_) : g(g_), k0(0) {
    const int t = threadIdx.x;
    if (LEFT) {
      const int ib = proj_kslow_ib(t), kq = proj_kslow_kq(t);
      base = reinterpret_cast<const char*>((const bf16_raw*)g.A + g.a_row0);
#pragma unroll
      for (int j = 0; j < 4; ++j) off[j] = (unsigned)(((4 * kq + j) * g.lda + 8 * ib) * 2);
      step = 64 * g.lda * 2;
    } else {
      const int cc = t & 7, rr = t >> 3;
      base = reinterpret_cast<const char*>((const bf16_raw*)g.A + (long long)g.a_row0 * g.lda);
#pragma unroll
      for (int q = 0; q < 4; ++q) off[q] = (unsigned)(((rr + 32 * q) * g.lda + 8 * cc) * 2);
      step = 64 * 2;
    }
  }
  // FAST only: request j of the four of a stage (the caller issues all four, in order, then advance())
  __device__ __forceinline__ void load_one(u32x4 (&ra)[4], int j) { gload16_async(ra[j], base, off[j]); }
  __device__ __forceinline__ void advance() { base += step; }
  __device__ __forceinline__ void load(u32x4 (&ra)[4]) {
    if (FAST) {
#pragma unroll
      for (int j = 0; j < 4; ++j) gload16_async(ra[j], base, off[j]);
      base += step;
    } else {
      const int t = threadIdx.x;
      const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
      if (LEFT) {
        const int ib = proj_kslow_ib(t), kq = proj_kslow_kq(t);
        const long long a = (long long)g.a_row0 + 8 * ib;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int k = k0 + 4 * kq + j;
          const int kc = k < g.KA ? k : g.KA - 1;
          const u32x4 v = load8_bf16(g.A + (long long)kc * g.lda, a, g.a_rows);
          ra[j] = k < g.KA ? v : zero;
        }
      } else {
        const int cc = t & 7, rr = t >> 3;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = g.a_row0 + rr + 32 * q;
          const int rc = row < g.a_rows ? row : g.a_rows - 1;
          ra[q] = load8_bf16(g.A + (long long)rc * g.lda, k0 + 8 * cc, g.KA);
        }
      }
      k0 += 64;
    }
  }
};

// Registers -> LDS tile of one K stage (128 rows x 64 k, lds_tile_off layout), written as eight parts.  t = the thread's place among the 256 loaders.
//   K-slow (LEFT): ra[j] holds row k = 4*kq + j of a 4(k) x 8(a) block, dword d of it the elements
//   a = 2d, 2d+1.  Part p emits output row a = p: its four k values, two byte permutes and one 8-byte
//   write.  The row's chunk position is (chunk ^ row ^ row>>3 ^ row>>6) & 7 with row = 8*ib + p, i.e.
//   a per-thread constant XOR p.
//   K-contiguous: part p is half p & 1 of the 16-byte piece q = p >> 1 (row rr + 32 q); the chunk
//   position is a per-thread constant XOR a constant of q.
template <bool LEFT>
__device__ __forceinline__ void proj_store_a_part(char* la, const u32x4 (&ra)[4], int p, int t) {
  if (LEFT) {
    const int ib = proj_kslow_ib(t), kq = proj_kslow_kq(t);
    const int bx = ((kq >> 1) ^ ib ^ (ib >> 3)) & 7;
    char* row0 = la + ib * 1024 + 8 * (kq & 1);
    const unsigned in[16] = {ra[0].x, ra[0].y, ra[0].z, ra[0].w, ra[1].x, ra[1].y, ra[1].z, ra[1].w,
                             ra[2].x, ra[2].y, ra[2].z, ra[2].w, ra[3].x, ra[3].y, ra[3].z, ra[3].w};  // in[4*j + d]
    const unsigned sel = (p & 1) ? 0x07060302u : 0x05040100u;   // the high or the low halves of (x, y)
    const unsigned w0 = __builtin_amdgcn_perm(in[4 + (p >> 1)], in[0 + (p >> 1)], sel);    // k = 0, 1
    const unsigned w1 = __builtin_amdgcn_perm(in[12 + (p >> 1)], in[8 + (p >> 1)], sel);   // k = 2, 3
    *reinterpret_cast<u32x2*>(row0 + p * 128 + ((bx ^ p) << 4)) = u32x2{w0, w1};
  } else {
    const int cc = t & 7, rr = t >> 3, q = p >> 1;
    const int bx = (cc ^ rr ^ (rr >> 3)) & 7;
    const int cq = (4 * (q & 1)) ^ (q >> 1);
    const u32x2 half = (p & 1) ? u32x2{ra[q].z, ra[q].w} : u32x2{ra[q].x, ra[q].y};
    *reinterpret_cast<u32x2*>(la + rr * 128 + q * 4096 + ((bx ^ cq) << 4) + 8 * (p & 1)) = half;
  }
}

template <bool LEFT>
__device__ __forceinline__ void proj_store_a(char* la, const u32x4 (&ra)[4], int t = threadIdx.x) {
#pragma unroll
  for (int p = 0; p < 8; ++p) proj_store_a_part<LEFT>(la, ra, p, t);
}

// 32 k of the wave's 128 x 64 sub-tile: A fragments from the 128-B-per-row tile (k-slices kk4, kk4+1
// of its 4), B fragments from a ring stage.
// A wavefront issues in order, and a multiply holds the matrix pipe for 32 cycles: sixteen multiplies
// in a row leave the wavefront unable to issue anything else for as long as they queue, and whatever
// else the half stage has to do (the second slice's fragment reads, the requests of the next ring stage
// and gradient tile) then runs with the matrix pipe idle.  So that work is dealt out between the
// multiplies of the first slice: `piece(j)`, j = 0..7, is called after the j-th of them, and scheduling
// barriers keep the compiler from gathering the multiplies again.
template <bool SUMSQ, typename Piece>
__device__ __forceinline__ void proj_compute(f32x16_t (&acc)[4][2], const char* la, const char* lb, int kk4,
                                             float (&sq)[4], Piece piece) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Frags f[2];
  auto read_a = [&](int kk, int t) {
    f[kk].a[t] = *reinterpret_cast<const bf16x8_t*>(la + lds_tile_off(32 * t + (lane & 31), 2 * (kk4 + kk) + (lane >> 5)));
  };
  auto read_b = [&](int kk, int t) {
    f[kk].b[t] = *reinterpret_cast<const bf16x8_t*>(lb + ring_tile_off(wave * 64 + 32 * t + (lane & 31), 2 * kk + (lane >> 5)));
  };
#pragma unroll
  for (int t = 0; t < 4; ++t) read_a(0, t);
#pragma unroll
  for (int t = 0; t < 2; ++t) read_b(0, t);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int tm = j >> 1, tn = j & 1;
    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[0].a[tm], f[0].b[tn], acc[tm][tn], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (j < 4) read_a(1, j);
    else if (j < 6) read_b(1, j - 4);
    piece(j);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (SUMSQ) gemm_sumsq_slice(sq, f[0]);
  gemm_mfma_slice(acc, f[1]);
  if (SUMSQ) gemm_sumsq_slice(sq, f[1]);
}

// RT = rank tiles of 256 that one workgroup covers (256*RT threads, wave w owns rank rows 64 w ..).
// With RT = 2 both tiles share the A tile, which only the first four wavefronts load and store
// (LOADER); the other four have no A requests in their queue, so their O-half wait is vmcnt(4) where a
// loading wavefront's is vmcnt(8).
// (LOADER is a template parameter rather than a test inside, so that each kind of wavefront runs
// straight-line code in which every request is followed by its own wait.)
template <bool LEFT, bool FAST, bool SUMSQ, int RT = 1, bool LOADER = true>
__device__ __forceinline__ void proj_pipeline(f32x16_t (&acc)[4][2], char* lds, const GemmOperands& g, float (&sq)[4]) {
  static_assert(LOADER || RT == 2, "only the second rank tile's wavefronts go without the gradient");
  constexpr int STAGE = RT * FIRA_PROJ_RING_STAGE;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  constexpr bool loader = LOADER;
  char* la = lds;
  char* ring = lds + FIRA_PROJ_LDS_A;
  const unsigned ring0 = (unsigned)(size_t)(lds_ptr)ring;
  const int SS = g.KB / 64;                    // K stages of 64; the ring runs 2*SS stages of 32
  const int lrow = lane >> 2;
  const int chunk = (lane & 3) ^ ring_swz(lrow);
  const unsigned offb = (unsigned)(lrow * 64 + chunk * 16);
  const char* pb = reinterpret_cast<const char*>((const bf16_raw*)g.B) + ((long long)g.b_row0 + 64 * wave) * 64;
  auto request_b = [&](int s) {
    const unsigned dst = ring0 + (unsigned)((s % FIRA_RING_STAGES) * STAGE);
    const char* kb = pb + (long long)s * g.ldb * 64;
#pragma unroll
    for (int q = 0; q < 4; ++q) lds_dma16(kb + q * 1024, offb, dst + (unsigned)((4 * wave + q) * 1024));
  };
  // request q (of 4) of ring stage s
  auto request_b1 = [&](int s, int q) {
    const unsigned dst = ring0 + (unsigned)((s % FIRA_RING_STAGES) * STAGE);
    const char* kb = pb + (long long)s * g.ldb * 64;
    lds_dma16(kb + q * 1024, offb, dst + (unsigned)((4 * wave + q) * 1024));
  };
  ProjALoader<LEFT, FAST> al(g);
  u32x4 ra[4];
  if (loader) al.load(ra);                     // A(0)
  request_b(0);
  request_b(1);
  // LAST: the final K stage requests nothing more.  It is written out separately rather than
  // guarded inside the loop, so that on every path a request is followed by the wait that covers it.
  auto stage = [&](auto last, int S) {
    constexpr bool LAST = decltype(last)::value;
    // E half
    if (loader) wait_loads<4>(ra);             // A(S) and D(2S) have landed; D(2S+1) may be in flight
    else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");    // everybody is done with the previous stage's A tile and ring slot
    if (loader) proj_store_a<LEFT>(la, ra);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // the requests of D(2S+2) (into the slot of D(2S-1), free since the first barrier) and of A(S+1)
    // (whose registers proj_store_a has just released) go out between the multiplies
    proj_compute<SUMSQ>(acc, la, ring + ((2 * S) % FIRA_RING_STAGES) * STAGE, 0, sq, [&](int j) {
      if (LAST) return;
      if (j < 4) request_b1(2 * S + 2, j);
      else if (loader) {
        if (FAST) {
          al.load_one(ra, j - 4);
          if (j == 7) al.advance();
        } else if (j == 4) {
          al.load(ra);
        }
      }
    });
    // O half
    // D(2S+1) has landed.  Guarded A loads are the compiler's and may be fewer than 4 instructions,
    // so the edge path only lets D(2S+2)'s four stay in flight.
    if (LAST) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    else if (FAST && loader) asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
    proj_compute<SUMSQ>(acc, la, ring + ((2 * S + 1) % FIRA_RING_STAGES) * STAGE, 2, sq, [&](int j) {
      if (!LAST && j < 4) request_b1(2 * S + 3, j);
    });
  };
  for (int S = 0; S + 1 < SS; ++S) stage(std::false_type{}, S);
  stage(std::true_type{}, SS - 1);
}

template <bool LEFT>
__device__ __forceinline__ void project_tile(char* lds, const FiraMat* __restrict__ mats, const FiraEnt* __restrict__ ents,
                                             const FiraTile& tile, int norm_mode, const FiraScal* __restrict__ scal, const FiraHp& hp) {
  const FiraEnt ent = ents[tile.ent];
  if (hp.mixed && use_gram(hp, scal[ent.mat])) return;   // the fused kernel serves this matrix
  const FiraMat mt = mats[ent.mat];

  GemmOperands g;
  g.a_row0 = tile.ta * FIRA_PA;
  g.a_rows = mt.L;
  g.b_row0 = tile.tb * FIRA_PB;
  g.b_rows = mt.r;
  g.B = as_global<const bf16_raw>(mt.PT);
  g.ldb = mt.rq;
  g.KB = mt.kx * mt.Sp;
  if (mt.kx == 1) {
    g.A = as_global(reinterpret_cast<const bf16_raw*>(ent.G));
    g.lda = mt.ld;
    g.KA = mt.S;
  } else {
    g.A = as_global<const bf16_raw>(mt.Gx);
    g.lda = mt.gx_ld;
    g.KA = mt.kx * mt.Sp;
  }
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
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Gram route: ||G_i||^2 of the tile's 128 factors falls out of the A fragments of wave 0 in the
  // first rank tile of each panel.  (fp32 matrices feed split planes through here; their norms
  // come from fira_gradnorm_kernel.)
  const bool sumsq = norm_mode == 1 && mt.kx == 1 && tile.tb == 0 && wave == 0;
  // LEFT: the k rows of G are whole rows of the matrix (any ld); RIGHT: a row of G holds KA values
  const bool interior = g.a_row0 + FIRA_PA <= g.a_rows && g.KA == g.KB;
  if (interior) {
    if (sumsq) proj_pipeline<LEFT, true, true>(acc, lds, g, sq);
    else proj_pipeline<LEFT, true, false>(acc, lds, g, sq);
  } else {
    if (sumsq) proj_pipeline<LEFT, false, true>(acc, lds, g, sq);
    else proj_pipeline<LEFT, false, false>(acc, lds, g, sq);
  }
  if (sumsq) {
    gptr<float> g2 = as_global(mt.g2);
#pragma unroll
    for (int tm = 0; tm < 4; ++tm) {
      const float tot = sq[tm] + __shfl_xor(sq[tm], 32, 64);
      const int row = g.a_row0 + 32 * tm + (lane & 31);
      if (lane < 32 && row < mt.L) g2[row] = tot;
    }
  }
  gptr<float> Rt = as_global(mt.Rt);
#pragma unroll
  for (int tm = 0; tm < 4; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
      const int col = g.b_row0 + wave * 64 + 32 * tn + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = g.a_row0 + 32 * tm + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < mt.L && col < mt.r) Rt[(long long)row * mt.r + col] = acc[tm][tn][v];
      }
    }
}

// One grid for both orientations: workgroups [0, blocks_left) take the tiles of the matrices with
// m <= n (gradient K-slow), the rest those with m > n, so that only one partly filled round of
// workgroups ends the launch.  blocks_left is a multiple of 8, which keeps the XCD-aware mapping of
// each part.  scal is read only when hp.mixed is set (a step in which the fused kernel serves the
// matrices on the Gram route and this kernel the others).
__global__ __launch_bounds__(FIRA_PROJ_THREADS, 2) void fira_project_kernel(const FiraMat* __restrict__ mats,
                                                                            const FiraEnt* __restrict__ ents,
                                                                            const FiraTile* __restrict__ tiles_left, int ntiles_left,
                                                                            int blocks_left,
                                                                            const FiraTile* __restrict__ tiles_right, int ntiles_right,
                                                                            int norm_mode, const FiraScal* __restrict__ scal, FiraHp hp) {
  extern __shared__ __attribute__((aligned(16))) char lds[];   // FIRA_PROJ_LDS bytes
  if ((int)blockIdx.x < blocks_left) {
    const int ti = xcd_chunked_index(blockIdx.x, ntiles_left);
    if (ti < 0) return;
    project_tile<true>(lds, mats, ents, tiles_left[ti], norm_mode, scal, hp);
  } else {
    const int ti = xcd_chunked_index((int)blockIdx.x - blocks_left, ntiles_right);
    if (ti < 0) return;
    project_tile<false>(lds, mats, ents, tiles_right[ti], norm_mode, scal, hp);
  }
}

// ------------------------------------------------------------------------------------------------
// Kernel 1 for small ranks (r <= 64, the fine-tuning setting's r = 32): with a 256-wide rank tile three
// quarters or more of the multiplies would work on padding.  Here the tile is 128 (gradient side) x 64
// (rank); wave w owns gradient rows 32 w .. 32 w + 31 and all 64 rank columns (two accumulator
// blocks), so the kernel needs few registers and 28 KB of LDS, several workgroups share a CU, and the
// gradient stream is what bounds it.  Same pipeline as above (single gradient tile, E and O halves);
// a ring stage is 64 rows x 32 k = 4 KB, one request instruction per wavefront, so the E-half wait is
// vmcnt(1) and the O-half wait vmcnt(5) (one ring request and the four of A(S+1) are younger).
// ------------------------------------------------------------------------------------------------
#define FIRA_PROJ_SMALL_STAGE (FIRA_PS * 64)
#define FIRA_PROJ_SMALL_LDS (FIRA_PROJ_LDS_A + FIRA_RING_STAGES * FIRA_PROJ_SMALL_STAGE)

template <bool SUMSQ>
__device__ __forceinline__ void proj_compute_small(f32x16_t (&acc)[2], const char* la, const char* lb, int kk4, float& sq) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bf16x8_t fa[2], fb[2][2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    fa[kk] = *reinterpret_cast<const bf16x8_t*>(la + lds_tile_off(32 * wave + (lane & 31), 2 * (kk4 + kk) + (lane >> 5)));
#pragma unroll
    for (int t = 0; t < 2; ++t)
      fb[kk][t] = *reinterpret_cast<const bf16x8_t*>(lb + ring_tile_off(32 * t + (lane & 31), 2 * kk + (lane >> 5)));
  }
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
    for (int t = 0; t < 2; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk], fb[kk][t], acc[t], 0, 0, 0);
    if (SUMSQ) {
      const u32x4 w = __builtin_bit_cast(u32x4, fa[kk]);
      const unsigned d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bf16x2_t v = __builtin_bit_cast(bf16x2_t, d[e]);
        sq = __builtin_amdgcn_fdot2_f32_bf16(v, v, sq, false);
      }
    }
  }
}

template <bool LEFT, bool FAST, bool SUMSQ>
__device__ __forceinline__ void proj_pipeline_small(f32x16_t (&acc)[2], char* lds, const GemmOperands& g, float& sq) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* la = lds;
  char* ring = lds + FIRA_PROJ_LDS_A;
  const unsigned ring0 = (unsigned)(size_t)(lds_ptr)ring;
  const int SS = g.KB / 64;
  const int lrow = lane >> 2;
  const int chunk = (lane & 3) ^ ring_swz(lrow);
  const unsigned offb = (unsigned)(lrow * 64 + chunk * 16);
  const char* pb = reinterpret_cast<const char*>((const bf16_raw*)g.B) + ((long long)g.b_row0 + 16 * wave) * 64;
  auto request_b = [&](int s) {   // this wave's 16 of the stage's 64 rows
    lds_dma16(pb + (long long)s * g.ldb * 64, offb, ring0 + (unsigned)((s % FIRA_RING_STAGES) * FIRA_PROJ_SMALL_STAGE + wave * 1024));
  };
  ProjALoader<LEFT, FAST> al(g);
  u32x4 ra[4];
  al.load(ra);                                 // A(0)
  request_b(0);
  request_b(1);
  auto stage = [&](auto last, int S) {
    constexpr bool LAST = decltype(last)::value;
    wait_loads<1>(ra);                         // A(S) and D(2S) have landed; D(2S+1) may be in flight
    asm volatile("s_barrier" ::: "memory");
    proj_store_a<LEFT>(la, ra);
    if (!LAST) {
      request_b(2 * S + 2);
      al.load(ra);                             // A(S+1)
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    proj_compute_small<SUMSQ>(acc, la, ring + ((2 * S) % FIRA_RING_STAGES) * FIRA_PROJ_SMALL_STAGE, 0, sq);
    // D(2S+1) has landed (guarded A loads may be fewer than 4 instructions: the edge path lets one stay)
    if (LAST) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    else if (FAST) asm volatile("s_waitcnt vmcnt(5)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(1)\n\ts_barrier" ::: "memory");
    if (!LAST) request_b(2 * S + 3);
    proj_compute_small<SUMSQ>(acc, la, ring + ((2 * S + 1) % FIRA_RING_STAGES) * FIRA_PROJ_SMALL_STAGE, 2, sq);
  };
  for (int S = 0; S + 1 < SS; ++S) stage(std::false_type{}, S);
  stage(std::true_type{}, SS - 1);
}

template <bool LEFT>
__device__ __forceinline__ void project_small_tile(char* lds, const FiraMat* __restrict__ mats, const FiraEnt* __restrict__ ents,
                                                   const FiraTile& tile, int norm_mode, const FiraScal* __restrict__ scal, const FiraHp& hp) {
  const FiraEnt ent = ents[tile.ent];
  if (hp.mixed && use_gram(hp, scal[ent.mat])) return;   // (never the case today: the fused kernel takes no rank this small)
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
  f32x16_t acc[2];
  float sq = 0.0f;
#pragma unroll
  for (int tn = 0; tn < 2; ++tn)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[tn][v] = 0.0f;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool sumsq = norm_mode == 1;           // every wave owns its own 32 factors
  const bool interior = g.a_row0 + FIRA_PA <= g.a_rows && g.KA == g.KB;
  if (interior) {
    if (sumsq) proj_pipeline_small<LEFT, true, true>(acc, lds, g, sq);
    else proj_pipeline_small<LEFT, true, false>(acc, lds, g, sq);
  } else {
    if (sumsq) proj_pipeline_small<LEFT, false, true>(acc, lds, g, sq);
    else proj_pipeline_small<LEFT, false, false>(acc, lds, g, sq);
  }
  if (sumsq) {
    const float tot = sq + __shfl_xor(sq, 32, 64);
    const int row = g.a_row0 + 32 * wave + (lane & 31);
    if (lane < 32 && row < mt.L) as_global(mt.g2)[row] = tot;
  }
  gptr<float> Rt = as_global(mt.Rt);
#pragma unroll
  for (int tn = 0; tn < 2; ++tn) {
    const int col = 32 * tn + (lane & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = g.a_row0 + 32 * wave + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (row < mt.L && col < mt.r) Rt[(long long)row * mt.r + col] = acc[tn][v];
    }
  }
}

// bf16 matrices with r <= 64 only (the host keeps their tiles in lists of their own); both orientations
// in one grid, as in fira_project_kernel.
__global__ __launch_bounds__(FIRA_PROJ_THREADS, 4) void fira_project_small_kernel(const FiraMat* __restrict__ mats,
                                                                                  const FiraEnt* __restrict__ ents,
                                                                                  const FiraTile* __restrict__ tiles_left, int ntiles_left,
                                                                                  int blocks_left,
                                                                                  const FiraTile* __restrict__ tiles_right, int ntiles_right,
                                                                                  int norm_mode, const FiraScal* __restrict__ scal, FiraHp hp) {
  extern __shared__ __attribute__((aligned(16))) char lds[];   // FIRA_PROJ_SMALL_LDS bytes
  if ((int)blockIdx.x < blocks_left) {
    const int ti = xcd_chunked_index(blockIdx.x, ntiles_left);
    if (ti < 0) return;
    project_small_tile<true>(lds, mats, ents, tiles_left[ti], norm_mode, scal, hp);
  } else {
    const int ti = xcd_chunked_index((int)blockIdx.x - blocks_left, ntiles_right);
    if (ti < 0) return;
    project_small_tile<false>(lds, mats, ents, tiles_right[ti], norm_mode, scal, hp);
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
  // W and G are touched once per step: non-temporal accesses keep them from evicting the operand
  // panels that the 32 CUs of an XCD share through its L2.
  template <bool INTERIOR>
  static __device__ __forceinline__ Raw load_raw(gptr<const bf16_raw> row, long long idx, long long limit) {
    if (INTERIOR) return __builtin_nontemporal_load(reinterpret_cast<gptr<const u32x4_a2>>(row + idx));
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
      __builtin_nontemporal_store(v, reinterpret_cast<gptr<u32x4_a2>>(row + idx));
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

// Epilogue of the rank-axis contractions.  Two waves that share 64 tile rows (i) own 256 adjacent
// columns (j) between them; their accumulators are re-laid out through one LDS slab of 32 rows x 256
// columns per step, so that every global instruction covers two full 256-column row segments
// (512 B of bf16, 1 KB of fp32, contiguous) instead of 64-column pieces.  That matters most when
// ld is odd and no 16-byte access is aligned: the number of partially covered 128-byte lines per
// instruction drops four-fold.  The G (and W) values of the second slab are requested while the
// first one is consumed.
#define FIRA_EPI_STRIDE 260   // floats per staged row: 256 + 4 (keeps 16-byte alignment, shifts banks)
#define FIRA_EPI_SLAB (2 * 32 * FIRA_EPI_STRIDE * 4)
#define FIRA_EPI_LDS (FIRA_EPI_SLAB + FIRA_BB * 4)   // the slabs, then one factor per tile row (matrices with m > n)
#define FIRA_BACK_LDS (FIRA_EPI_LDS > FIRA_RING_LDS ? FIRA_EPI_LDS : FIRA_RING_LDS)
template <int MODE, typename T, bool INTERIOR>
__device__ __forceinline__ float backproject_epilogue(f32x16_t (&acc)[4][2], char* lds, const FiraMat& mt,
                                                      const FiraEnt& ent, int i0, int j0, float c, float lr_alpha, bool unitk) {
  typedef typename Elem8<T>::Raw Raw;
  // fp32 tiles would need 128 more registers: no prefetch; neither in the norm pass, which spills with it
  constexpr bool PIPE = sizeof(T) == 2 && MODE == 1;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave & 1, wn = wave >> 1;
  float* buf = reinterpret_cast<float*>(lds) + wn * (32 * FIRA_EPI_STRIDE);
  float* rowphi = reinterpret_cast<float*>(lds + FIRA_EPI_SLAB);
  gptr<const T> G = as_global(reinterpret_cast<const T*>(ent.G));
  gptr<T> W = as_global(reinterpret_cast<T*>(ent.W));
  gptr<const float> phi = as_global<const float>(mt.phi);
  const int jl = 8 * (lane & 31);             // this lane's 8 columns inside the staged 256
  const int ih = lane >> 5;                   // which of the two rows of a pass
  const long long j = (long long)j0 + jl;
  // slab tn holds tile rows wn*64 + 32*tn .. +31; this wave consumes 16 of them, two per pass.
  // Interior tiles address a pass as a wave-uniform row pointer plus one 32-bit lane offset.
  const long long wave_row0 = (long long)i0 + wn * 64 + 16 * wm;
  const long long lane_off = (unsigned)(ih * (int)mt.ld + jl);
  auto slab_row = [&](int p) { return 16 * wm + 2 * p + ih; };
  auto fetch = [&](int tn, int p, Raw& gr, Raw& wr) {
    if (INTERIOR) {
      const long long base = (wave_row0 + 32 * tn + 2 * p) * mt.ld + j0;
      gr = Elem8<T>::template load_raw<true>(G + base, lane_off, 0);
      if (MODE == 1) wr = Elem8<T>::template load_raw<true>(W + base, lane_off, 0);
    } else {
      const long long i = (long long)i0 + wn * 64 + 32 * tn + slab_row(p);
      const bool ok = i < mt.m && j < mt.n;
      gr = ok ? Elem8<T>::template load_raw<false>(G + i * mt.ld, j, mt.n) : Elem8<T>::zero();
      if (MODE == 1) wr = ok ? Elem8<T>::template load_raw<false>(W + i * mt.ld, j, mt.n) : Elem8<T>::zero();
    }
  };
  Raw gbuf[PIPE ? 8 : 1], wbuf[PIPE ? 8 : 1];
  if (PIPE) {
#pragma unroll
    for (int p = 0; p < 8; ++p) fetch(0, p, gbuf[p], wbuf[p]);
  }
  float cphi[8];
  if (mt.left) {
#pragma unroll
    for (int e = 0; e < 8; ++e) cphi[e] = (INTERIOR || j + e < mt.n) ? (unitk ? c : c * phi[j + e]) : 0.0f;
  }
  float sum = 0.0f;
#pragma unroll
  for (int tn = 0; tn < 2; ++tn) {
    __syncthreads();  // previous slab fully consumed (first time: the main loop's LDS reads are done)
    // One factor per row (m > n): the tile's 128 go through LDS.  Loaded from global memory inside a pass
    // they would have to be waited for there, and the memory counter being in order, that wait would
    // cover every request in flight for the later passes.
    if (tn == 0 && !mt.left && threadIdx.x < FIRA_BB) {
      const long long i = (long long)i0 + threadIdx.x;
      rowphi[threadIdx.x] = (INTERIOR || i < mt.m) ? (unitk ? c : c * phi[i]) : 0.0f;
    }
#pragma unroll
    for (int tm = 0; tm < 4; ++tm)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const f32x16_t& a = acc[tm][tn];
        const f32x4 val = f32x4{a[4 * vg], a[4 * vg + 1], a[4 * vg + 2], a[4 * vg + 3]};
        *reinterpret_cast<f32x4*>(buf + (lane & 31) * FIRA_EPI_STRIDE + 128 * wm + 32 * tm + 8 * vg + 4 * (lane >> 5)) = val;
      }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int il = slab_row(p);
      const long long i = (long long)i0 + wn * 64 + 32 * tn + il;
      if (!PIPE) fetch(tn, p, gbuf[0], wbuf[0]);
      Raw& gr = gbuf[PIPE ? p : 0];
      Raw& wr = wbuf[PIPE ? p : 0];
      if (INTERIOR || (i < mt.m && j < mt.n)) {
        const f32x4 u0 = *reinterpret_cast<const f32x4*>(buf + il * FIRA_EPI_STRIDE + jl);
        const f32x4 u1 = *reinterpret_cast<const f32x4*>(buf + il * FIRA_EPI_STRIDE + jl + 4);
        const float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
        float g[8];
        Elem8<T>::unpack(gr, g);
        if (!mt.left) {
          const float f = rowphi[wn * 64 + 32 * tn + il];
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
          Elem8<T>::unpack(wr, w);
#pragma unroll
          for (int e = 0; e < 8; ++e) w[e] = w[e] - lr_alpha * (u[e] + cphi[e] * g[e]);
          if (INTERIOR) Elem8<T>::template store<true>(w, W + ((wave_row0 + 32 * tn + 2 * p) * mt.ld + j0), lane_off, 0);
          else Elem8<T>::template store<false>(w, W + i * mt.ld, j, mt.n);
        }
      }
      if (PIPE && tn == 0) fetch(1, p, gr, wr);
    }
  }
  return sum;
}

// T: storage type of W and G of every matrix in the tile list (the host keeps one list per type).
template <int MODE, typename T>
__global__ __launch_bounds__(FIRA_BACK_THREADS, 2) void fira_backproject_kernel(const FiraMat* __restrict__ mats,
                                                                           const FiraScal* __restrict__ scal,
                                                                           const FiraEnt* __restrict__ ents,
                                                                           const FiraTile* __restrict__ tiles,
                                                                           int ntiles, float* __restrict__ partial,
                                                                           FiraHp hp) {
  extern __shared__ __attribute__((aligned(16))) char lds[];   // FIRA_BACK_LDS bytes
  __shared__ float red[4];
  const int ti = xcd_chunked_index(blockIdx.x, ntiles);
  if (ti < 0) return;
  const FiraTile tile = tiles[ti];
  const FiraEnt ent = ents[tile.ent];
  if (MODE == 0 && use_gram(hp, scal[ent.mat])) return;   // this matrix takes the Gram route to ||S||
  const FiraMat mt = mats[ent.mat];
  const float lr_alpha = MODE == 1 ? *hp.lr_alpha : 0.0f;

  // Y (n side) is the A operand, X (m side) the B operand.
  gptr<const bf16_raw> lowrank = as_global<const bf16_raw>((MODE == 0) ? mt.Rb : mt.Nb);
  gptr<const bf16_raw> proj = as_global<const bf16_raw>(mt.Pn);
  GemmOperands g;
  g.a_row0 = tile.ta * FIRA_BA;
  g.a_rows = mt.n;
  g.b_row0 = tile.tb * FIRA_BB;
  g.b_rows = mt.m;
  // Z in two planes (hi + lo): the contraction runs over 2 rp, and the projector's K blocks are used twice
  const bool split = MODE == 1 && hp.zsplit && mt.zready && hp.scaling != 1;
  g.KA = g.KB = (split ? 2 : mt.kx) * mt.rp;
  g.wrapA = (split && !mt.left) ? mt.rp / FIRA_RK : 0;
  g.wrapB = (split && mt.left) ? mt.rp / FIRA_RK : 0;
  g.A = mt.left ? lowrank : proj;
  g.B = mt.left ? proj : lowrank;
  g.lda = mt.left ? mt.Lq : mt.Sq;
  g.ldb = mt.left ? mt.Sq : mt.Lq;
  f32x16_t acc[4][2];
  ring_mainloop(acc, lds, g);

  const float c = (MODE == 0) ? 1.0f : scal[ent.mat].c;
  const int i0 = g.b_row0, j0 = g.a_row0;
  const bool interior = i0 + FIRA_BB <= mt.m && j0 + FIRA_BA <= mt.n;
  float sum;
  // matrix-level factor: the residual norm is taken with unit factors and scaled by the limiter kernel
  const bool unitk = MODE == 0 && hp.scaling == 1;
  if (interior) sum = backproject_epilogue<MODE, T, true>(acc, lds, mt, ent, i0, j0, c, lr_alpha, unitk);
  else sum = backproject_epilogue<MODE, T, false>(acc, lds, mt, ent, i0, j0, c, lr_alpha, unitk);

  if (MODE == 0) {
    // deterministic workgroup reduction: xor-butterfly inside each wave, then waves in order
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0)
      as_global(partial)[tile.part] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}
