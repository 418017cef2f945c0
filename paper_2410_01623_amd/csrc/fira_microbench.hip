// Machine calibration for the roofline figures: what one MI355X actually sustains for the three resources
// the Fira step leans on, measured with the simplest kernels that use nothing else.
//   read / write / copy : HBM streams over buffers far larger than the caches (16 bytes per lane,
//                         workgroups striding through the buffer, non-temporal accesses)
//   mfma                : v_mfma_f32_32x32x16_bf16 on register operands, 8 independent accumulator blocks
//                         per wavefront (the shape of the step's contractions), 1 or 2 wavefronts per SIMD
//   lds                 : ds_read_b128 fragment reads, all wavefronts of a CU at once
//   power               : socket power (amdgpu hwmon file) while the copy and the mfma loop run for two seconds each,
//                         the latter with constant and with pseudo-random operands: what a byte moved and a
//                         multiply-add cost above the idle chip when nothing else is done
// Prints one line per measurement.  Everything is in bounds and every loop has a fixed trip count.
#include <hip/hip_runtime.h>

#include <glob.h>
#include <unistd.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

#define CHECK(call)                                                                         \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                       \
      std::exit(1);                                                                         \
    }                                                                                       \
  } while (0)

// MODE 0: read, 1: write, 2: copy.  n16 = number of 16-byte pieces; the grid strides through them.
template <int MODE>
__global__ __launch_bounds__(256) void stream_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16,
                                                     unsigned* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  u32x4 acc = u32x4{0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
    if (MODE == 0) acc ^= __builtin_nontemporal_load(src + i);
    if (MODE == 1) __builtin_nontemporal_store(u32x4{(unsigned)i, 1u, 2u, 3u}, dst + i);
    if (MODE == 2) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
  }
  if (MODE == 0 && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1u;   // keeps the loads alive
}

// Tile-shaped streams, the access pattern of the update's epilogue: the matrix has `rows` rows of
// row_bytes bytes; a workgroup takes a tile of 64 KB, tile_bytes bytes wide, and walks down its rows,
// a wavefront instruction covering 1 KB = 1024 / tile_bytes rows (or a quarter of a 4 KB row piece).
// Tiles are numbered down the rows first, and consecutive workgroup ids go round the 8 XCDs.
// MODE 0: read, 1: write, 2: read-modify-write (W), 3: read two, write one (G and W -> W)
template <int MODE>
__global__ __launch_bounds__(256) void tile_kernel(const char* __restrict__ src, const char* __restrict__ src2, char* __restrict__ dst,
                                                   long long rows, long long row_bytes, int tile_bytes, unsigned* __restrict__ sink) {
  const int tile_rows = 65536 / tile_bytes;
  const long long tiles_down = rows / tile_rows, ntiles = tiles_down * (row_bytes / tile_bytes);
  const int per = (int)((ntiles + 7) / 8);
  const long long t = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per || t >= ntiles) return;
  const long long r0 = (t % tiles_down) * tile_rows, c0 = (t / tiles_down) * tile_bytes;
  const int pieces = tile_bytes / 16;              // 16-byte pieces per tile row
  u32x4 acc = u32x4{0u, 0u, 0u, 0u};
  for (int i = threadIdx.x; i < 4096; i += 256) {  // 4096 pieces per tile
    const long long off = (r0 + i / pieces) * row_bytes + c0 + (long long)(i % pieces) * 16;
    if (MODE == 0) acc ^= __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + off));
    if (MODE == 1) __builtin_nontemporal_store(u32x4{(unsigned)i, 1u, 2u, 3u}, reinterpret_cast<u32x4*>(dst + off));
    if (MODE == 2) __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dst + off)) + 1u, reinterpret_cast<u32x4*>(dst + off));
    if (MODE == 3)
      __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dst + off)) +
                                      __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + off)),
                                  reinterpret_cast<u32x4*>(dst + off));
  }
  if (MODE == 0 && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1u;
}

// The memory traffic of the fused projection/Adam kernel without its arithmetic, at the shape that
// dominates the headline workload (2048 x 5461 bf16 gradients, r = 512): one workgroup per tile of 128
// factors reads the tile's gradient panel (2048 rows, one 256-byte piece per row, rows 10922 bytes apart:
// no 16-byte access is aligned), then, in 8 chunks of 16 factors, reads and rewrites 32 KB of M and of V
// (contiguous) and writes the chunk's Z as 16 pieces of 1 KB.  1 MB read and 640 KB written per tile.
typedef u32x4 __attribute__((aligned(2))) u32x4_a2;
#define FUSED_TILES_PER_MATRIX 42
__global__ __launch_bounds__(512) void fused_stream_kernel(const char* __restrict__ G, char* __restrict__ M, char* __restrict__ V,
                                                           char* __restrict__ Z, int ntiles, unsigned* __restrict__ sink) {
  const int per = (ntiles + 7) / 8;
  const int t = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= per || t >= ntiles) return;
  const long long mat = t / FUSED_TILES_PER_MATRIX, ta = t % FUSED_TILES_PER_MATRIX;
  const long long ld = 10922, g_bytes = 2048 * ld, mv_bytes = 5461LL * 2048, z_rows = 5632, z_bytes = 16 * z_rows * 64;
  const char* g = G + mat * g_bytes + ta * 256;
  u32x4 acc = u32x4{0u, 0u, 0u, 0u};
  for (int r0 = 0; r0 < 2048; r0 += 32) {
    const int row = r0 + (threadIdx.x >> 4), piece = threadIdx.x & 15;
    acc ^= __builtin_nontemporal_load(reinterpret_cast<const u32x4_a2*>(g + row * ld + piece * 16));
  }
  char* m = M + mat * mv_bytes + ta * 128 * 2048;
  char* v = V + mat * mv_bytes + ta * 128 * 2048;
  char* z = Z + mat * z_bytes + ta * 128 * 64;
  for (int c = 0; c < 8; ++c) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const long long off = (long long)c * 32768 + ((long long)threadIdx.x + 512 * i) * 16;
      u32x4* pm = reinterpret_cast<u32x4*>(m + off);
      u32x4* pv = reinterpret_cast<u32x4*>(v + off);
      *pm = *pm + 1u;
      *pv = *pv + 1u;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int p = threadIdx.x + 512 * i;            // K block p / 64, 16-byte piece p % 64 of its 1 KB
      *reinterpret_cast<u32x4*>(z + (long long)(p >> 6) * z_rows * 64 + c * 1024 + (p & 63) * 16) = u32x4{(unsigned)p, 1u, 2u, acc.x};
    }
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1u;
}

__global__ __launch_bounds__(256) void mfma_kernel(int iters, float* __restrict__ sink) {
  f32x16_t acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
  bf16x8_t fa[4], fb[2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int e = 0; e < 8; ++e) fa[a][e] = (__bf16)(float)((threadIdx.x + a + e) & 7);
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int e = 0; e < 8; ++e) fb[b][e] = (__bf16)(float)((threadIdx.x + 3 * b + e) & 3);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) s += acc[a][b][0];
  if (s == 12345.678f) sink[0] = s;
}

// every lane reads 16 bytes per instruction from a 64 KB LDS array, consecutive lanes consecutive pieces
__global__ __launch_bounds__(256) void lds_kernel(int iters, unsigned* __restrict__ sink) {
  __shared__ u32x4 buf[4096];
  for (int i = threadIdx.x; i < 4096; i += 256) buf[i] = u32x4{(unsigned)i, 0u, 0u, 0u};
  __syncthreads();
  u32x4 acc = u32x4{0u, 0u, 0u, 0u};
  int p = threadIdx.x;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= buf[(p + 256 * u) & 4095];
    p = (p + 64) & 4095;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1u;
}

// Every workgroup reads the same n16 16-byte pieces `rounds` times: after the first touch they come from L2.
__global__ __launch_bounds__(256) void reread_kernel(const u32x4* __restrict__ src, size_t n16, int rounds, unsigned* __restrict__ sink) {
  u32x4 acc = u32x4{0u, 0u, 0u, 0u};
  for (int r = 0; r < rounds; ++r)
    for (size_t i = threadIdx.x; i < n16; i += 256) acc ^= src[(i + 64 * (size_t)blockIdx.x) % n16];
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1u;
}

// The same loop with operands that change from one multiply to the next: two sets of pseudo-random bf16 fragments
// (values in [-1, 1)) used in turn, so that the operand inputs of the matrix pipe toggle as they do on real data.
__global__ __launch_bounds__(256) void mfma_random_kernel(int iters, float* __restrict__ sink) {
  f32x16_t acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
  bf16x8_t fa[2][4], fb[2][2];
  unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
  auto next = [&]() { h = h * 1664525u + 1013904223u; return (__bf16)((float)(int)(h >> 8) * (1.0f / 8388608.0f) - 1.0f); };
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int e = 0; e < 8; ++e) fa[s][a][e] = next();
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 8; ++e) fb[s][b][e] = next();
  }
  for (int it = 0; it < iters; it += 2) {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s][a], fb[s][b], acc[a][b], 0, 0, 0);
  }
  float sum = 0.0f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) sum += acc[a][b][0];
  if (sum == 12345.678f) sink[0] = sum;
}

// Socket power in watts from the amdgpu hwmon file, or a negative value when it cannot be read.
static std::string g_power_file;
static double read_power_w() {
  if (g_power_file.empty()) {
    glob_t g;
    if (glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input", 0, nullptr, &g) == 0 && g.gl_pathc > 0) g_power_file = g.gl_pathv[0];
    globfree(&g);
    if (g_power_file.empty()) return -1.0;
  }
  FILE* f = std::fopen(g_power_file.c_str(), "r");
  if (!f) return -1.0;
  long long uw = -1;
  if (std::fscanf(f, "%lld", &uw) != 1) uw = -1;
  std::fclose(f);
  return uw < 0 ? -1.0 : uw / 1e6;
}
// Runs `launch` in batches for `seconds`, reading the power after every batch; the mean leaves out the first third.
template <typename F>
static void power_run(F launch, double seconds, double* watts, double* launches_per_s) {
  launch();
  CHECK(hipDeviceSynchronize());
  std::vector<double> w;
  const auto t0 = std::chrono::steady_clock::now();
  long long n = 0;
  double el = 0.0;
  while (el < seconds) {
    for (int i = 0; i < 8; ++i) launch();
    CHECK(hipDeviceSynchronize());
    n += 8;
    w.push_back(read_power_w());
    el = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  }
  double sum = 0.0;
  size_t cnt = 0;
  for (size_t i = w.size() / 3; i < w.size(); ++i) { sum += w[i]; ++cnt; }
  *watts = cnt ? sum / cnt : -1.0;
  *launches_per_s = n / el;
}

template <typename F>
static double time_ms(F launch, int reps) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  launch();
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0, 0));
  for (int r = 0; r < reps; ++r) launch();
  CHECK(hipEventRecord(e1, 0));
  CHECK(hipEventSynchronize(e1));
  float ms = 0.0f;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  CHECK(hipGetLastError());
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return ms / reps;
}

int main() {
  hipDeviceProp_t prop;
  CHECK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  std::printf("device: %s, %d CUs, %.0f MHz, %.1f GiB, %zu KiB LDS per workgroup\n", prop.name, cus, prop.clockRate / 1e3,
              prop.totalGlobalMem / 1073741824.0, prop.sharedMemPerBlock / 1024);
  const size_t bytes = (size_t)4 << 30, n16 = bytes / 16;
  u32x4 *a = nullptr, *b = nullptr;
  unsigned* sink = nullptr;
  CHECK(hipMalloc(&a, bytes));
  CHECK(hipMalloc(&b, bytes));
  CHECK(hipMalloc(&sink, 256));
  CHECK(hipMemset(a, 1, bytes));
  CHECK(hipMemset(b, 2, bytes));
  for (int wg_per_cu : {4, 8, 16}) {
    const dim3 grid(cus * wg_per_cu), blk(256);
    const double tr = time_ms([&] { hipLaunchKernelGGL(stream_kernel<0>, grid, blk, 0, 0, a, b, n16, sink); }, 5);
    const double tw = time_ms([&] { hipLaunchKernelGGL(stream_kernel<1>, grid, blk, 0, 0, a, b, n16, sink); }, 5);
    const double tc = time_ms([&] { hipLaunchKernelGGL(stream_kernel<2>, grid, blk, 0, 0, a, b, n16, sink); }, 5);
    std::printf("hbm, 4 GiB, %2d workgroups per CU: read %.0f GB/s, write %.0f GB/s, copy %.0f GB/s (read + write bytes)\n", wg_per_cu,
                bytes / tr / 1e6, bytes / tw / 1e6, 2.0 * bytes / tc / 1e6);
  }
  const double tm = time_ms([&] { CHECK(hipMemcpyAsync(b, a, bytes, hipMemcpyDeviceToDevice, 0)); }, 5);
  std::printf("hbm, hipMemcpyAsync device to device, 4 GiB: %.0f GB/s (read + write bytes)\n", 2.0 * bytes / tm / 1e6);
  {
    // 2 GiB matrices of 131072 rows x 16 KiB; tiles of 64 KiB in four shapes
    const long long rows = 131072, row_bytes = 16384;
    for (int tile_bytes : {256, 512, 1024, 4096, 16384}) {
      const long long ntiles = rows * row_bytes / 65536;
      const dim3 grid((unsigned)((ntiles + 7) / 8 * 8)), blk(256);
      const double mb = (double)rows * row_bytes;
      const double t0 = time_ms([&] { hipLaunchKernelGGL(tile_kernel<0>, grid, blk, 0, 0, (const char*)a, (const char*)a, (char*)b, rows, row_bytes, tile_bytes, sink); }, 3);
      const double t1 = time_ms([&] { hipLaunchKernelGGL(tile_kernel<1>, grid, blk, 0, 0, (const char*)a, (const char*)a, (char*)b, rows, row_bytes, tile_bytes, sink); }, 3);
      const double t2 = time_ms([&] { hipLaunchKernelGGL(tile_kernel<2>, grid, blk, 0, 0, (const char*)a, (const char*)a, (char*)b, rows, row_bytes, tile_bytes, sink); }, 3);
      const double t3 = time_ms([&] { hipLaunchKernelGGL(tile_kernel<3>, grid, blk, 0, 0, (const char*)a, (const char*)a, (char*)b, rows, row_bytes, tile_bytes, sink); }, 3);
      std::printf("hbm, 64 KiB tiles of %5d-byte row pieces: read %.0f, write %.0f, read-modify-write %.0f, two reads + one write %.0f GB/s\n",
                  tile_bytes, mb / t0 / 1e6, mb / t1 / 1e6, 2 * mb / t2 / 1e6, 3 * mb / t3 / 1e6);
    }
  }
  {
    // 160 matrices: gradients in a (3.58 GB), M in b's first half and V in its second (1.79 GB each), Z in c
    const int nmat = 160, ntiles = nmat * FUSED_TILES_PER_MATRIX;
    char* c = nullptr;
    const size_t z_total = (size_t)nmat * 16 * 5632 * 64;
    CHECK(hipMalloc(&c, z_total));
    CHECK(hipMemset(c, 0, z_total));
    const dim3 grid((unsigned)((ntiles + 7) / 8 * 8)), blk(512);
    const double t = time_ms([&] { hipLaunchKernelGGL(fused_stream_kernel, grid, blk, 0, 0, (const char*)a, (char*)b, (char*)b + ((size_t)2 << 30), c, ntiles, sink); }, 3);
    const double rd = (double)ntiles * (2048.0 * 256 + 2 * 128 * 2048), wr = (double)ntiles * (2 * 128 * 2048 + 128 * 1024);
    std::printf("hbm, traffic of the fused projection/Adam kernel without arithmetic (%d tiles: gradient panel in 256-byte pieces, M and V read "
                "and rewritten in 32 KB pieces, Z written in 1 KB pieces): %.0f GB/s (%.2f GB read + %.2f GB written in %.3f ms)\n",
                ntiles, (rd + wr) / t / 1e6, rd / 1e9, wr / 1e9, t);
    CHECK(hipFree(c));
  }
  for (int waves_per_simd : {1, 2}) {
    const int iters = 4000;
    const dim3 grid(cus * waves_per_simd), blk(256);   // one workgroup = four wavefronts = one per SIMD
    const double t = time_ms([&] { hipLaunchKernelGGL(mfma_kernel, grid, blk, 0, 0, iters, (float*)sink); }, 5);
    const double flop = (double)grid.x * 4 * iters * 8 * (2.0 * 32 * 32 * 16);
    std::printf("mfma 32x32x16 bf16, %d wavefront(s) per SIMD: %.0f TFLOP/s\n", waves_per_simd, flop / t / 1e9);
  }
  {
    const int iters = 4000;
    const dim3 grid(cus * 2), blk(256);
    const double t = time_ms([&] { hipLaunchKernelGGL(lds_kernel, grid, blk, 0, 0, iters, sink); }, 5);
    const double by = (double)grid.x * 256 * iters * 8 * 16;
    std::printf("lds ds_read_b128, 8 wavefronts per CU: %.1f TB/s (%.0f bytes per clock per CU at %.0f MHz)\n", by / t / 1e9,
                by / t / 1e3 / cus / (prop.clockRate / 1e3) * 1e3 / 1e3, prop.clockRate / 1e3);
  }
  if (read_power_w() > 0.0) {
    CHECK(hipDeviceSynchronize());
    std::vector<double> idle;
    for (int i = 0; i < 20; ++i) { usleep(50000); idle.push_back(read_power_w()); }
    double idle_w = 0.0;
    for (size_t i = idle.size() / 3; i < idle.size(); ++i) idle_w += idle[i];
    idle_w /= (double)(idle.size() - idle.size() / 3);
    std::printf("power, nothing running (clocks still up): %.0f W\n", idle_w);
    double w, lps;
    {
      const dim3 grid(cus * 4), blk(256);
      power_run([&] { hipLaunchKernelGGL(stream_kernel<2>, grid, blk, 0, 0, a, b, n16, sink); }, 2.0, &w, &lps);
      const double bps = 2.0 * bytes * lps;
      std::printf("power, copy 4 GiB: %.0f W at %.0f GB/s read + written: %.0f pJ per byte above idle\n", w, bps / 1e9, (w - idle_w) / bps * 1e12);
    }
    const int iters = 4000;
    const dim3 grid(cus * 2), blk(256);
    const double flop = (double)grid.x * 4 * iters * 8 * (2.0 * 32 * 32 * 16);
    power_run([&] { hipLaunchKernelGGL(mfma_kernel, grid, blk, 0, 0, iters, (float*)sink); }, 2.0, &w, &lps);
    std::printf("power, mfma 32x32x16 bf16 on constant operands: %.0f W at %.0f TFLOP/s: %.2f pJ per flop above idle\n", w, flop * lps / 1e12,
                (w - idle_w) / (flop * lps) * 1e12);
    power_run([&] { hipLaunchKernelGGL(mfma_random_kernel, grid, blk, 0, 0, iters, (float*)sink); }, 2.0, &w, &lps);
    std::printf("power, mfma 32x32x16 bf16 on pseudo-random operands that change every multiply: %.0f W at %.0f TFLOP/s: %.2f pJ per flop above idle\n",
                w, flop * lps / 1e12, (w - idle_w) / (flop * lps) * 1e12);
    {
      const dim3 g2(cus * 2), b2(256);
      const int it2 = 4000;
      power_run([&] { hipLaunchKernelGGL(lds_kernel, g2, b2, 0, 0, it2, sink); }, 2.0, &w, &lps);
      const double bps = (double)g2.x * 256 * it2 * 8 * 16 * lps;
      std::printf("power, lds ds_read_b128: %.0f W at %.1f TB/s: %.1f pJ per byte above idle\n", w, bps / 1e12, (w - idle_w) / bps * 1e12);
    }
    {
      // reads that hit in L2: every workgroup walks the same 2 MiB again and again (16 MiB per workgroup and launch)
      const size_t n16_small = ((size_t)2 << 20) / 16;
      const dim3 g3(cus * 8), b3(256);
      power_run([&] { hipLaunchKernelGGL(reread_kernel, g3, b3, 0, 0, (const u32x4*)a, n16_small, 8, sink); }, 2.0, &w, &lps);
      const double bps = (double)g3.x * 8 * ((size_t)2 << 20) * lps;
      std::printf("power, reads served by L2 (2 MiB re-read by every workgroup): %.0f W at %.1f TB/s: %.1f pJ per byte above idle\n", w, bps / 1e12,
                  (w - idle_w) / bps * 1e12);
    }
  } else {
    std::printf("power: no readable hwmon power file\n");
  }
  CHECK(hipFree(a));
  CHECK(hipFree(b));
  CHECK(hipFree(sink));
  return 0;
}
