// Host side of the Fira optimizer-step library: the C ABI of include/fira.h, the slab planner and
// the grouped launch sequence.  gfx950 only; no allocation on the step path.
#include "../../include/fira.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstddef>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "fira_device.h"
#include "fira_elementwise.h"
#include "fira_refresh.h"
#include "fira_gemm.h"
#include "fira_fused.h"
#include "fira_plan.h"

namespace {

thread_local std::string g_last_error;

}  // namespace

// Scratch of fira_refresh_projectors_static: device memory that exists from the moment the library is
// loaded, so that the call needs no allocation.  Every GPU the library runs on holds its own copy at its own
// address until the process ends.  In host code the name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device (static_scratch_address) and that pointer is what kernels,
// copies and fills are given.
static __device__ __align__(256) unsigned char scratch[FIRA_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up once per device); null on failure.
void* static_scratch_address(int* device_out, std::string* why) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) { *why = std::string("hipGetDevice: ") + hipGetErrorString(e); return nullptr; }
  if (device_out) *device_out = dev;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { *why = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e); return nullptr; }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

namespace {

struct ListSlot {
  std::vector<int> idx;
  std::vector<void*> W;
  std::vector<const void*> G;
  int ntiles[kNumTileLists] = {};
  int rowblocks = 0, g2blocks = 0;
  // device views (inside the slab)
  FiraEnt* d_ents = nullptr;
  FiraTile* d_tiles[kNumTileLists] = {};
  // pinned host staging, one contiguous block mirrored to the device block
  char* h_stage = nullptr;
  char* d_block = nullptr;
  size_t block_bytes = 0;
  hipEvent_t uploaded = nullptr;
  uint64_t last_use = 0;
  bool valid = false;
};

}  // namespace

struct fira_ctx {
  Plan plan;
  char* slab = nullptr;
  hipStream_t stream = nullptr;
  fira_hparams hp{};
  int scaling = FIRA_SCALE_COLUMN;
  int norm_mode = FIRA_NORM_GRAM;
  int variant = FIRA_VARIANT_FULL;
  bool fusion = true;          // fira_set_fusion
  bool zsplit = false;         // fira_set_z_planes(2)
  bool last_step_fused = false;
  FiraMat* d_mats = nullptr;
  FiraScal* d_scal = nullptr;
  float* d_partial = nullptr;
  float* d_lr_alpha = nullptr;   // lr * alpha as the kernels read it (see store_step_size)
  ListSlot slots[kSlots];
  char* h_stage_all = nullptr;
  // Host copy of every matrix's two gate values of the Gram route (FiraScal::ortho_err, FiraScal::gram_err;
  // pinned; +inf until known), so that a step knows which listed matrices take which route and can leave out
  // the launches that nobody needs.
  struct Gate { float ortho_err, gram_err; };
  Gate* h_gate = nullptr;
  hipEvent_t ortho_event = nullptr;
  bool ortho_pending = false;
  // fira_set_projectors: host image (pinned) of the table of installations of one call, and the event after
  // its upload (the next call waits for it before it rewrites the image)
  FiraRefreshEnt* h_install = nullptr;
  hipEvent_t install_event = nullptr;
  bool install_pending = false;
  uint64_t use_counter = 0;
  int device = -1;               // HIP device that was current at fira_init_state
  void* static_scratch = nullptr;   // that device's copy of the library's static scratch array
  std::string last_error;
  // optional per-kernel timing (fira_profile_begin / fira_profile_end)
  std::vector<hipEvent_t> prof_events;   // (FIRA_NUM_KERNELS + 1) per recorded step
  int prof_max_steps = 0, prof_steps = 0;
};

namespace {

fira_status fail(fira_ctx* ctx, fira_status st, const std::string& msg) {
  g_last_error = msg;
  if (ctx) ctx->last_error = msg;
  return st;
}
#define FIRA_HIP(ctx, call)                                                                     \
  do {                                                                                          \
    hipError_t e_ = (call);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return fail(ctx, FIRA_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_));        \
  } while (0)

// lr * alpha lives in device memory and is rewritten in stream order: the value travels as a kernel argument,
// so no host buffer has to outlive the call.
hipError_t store_step_size(fira_ctx* ctx) {
  hipLaunchKernelGGL(fira_store_float_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->d_lr_alpha, (float)(ctx->hp.lr * ctx->hp.alpha));
  return hipGetLastError();
}

FiraHp make_hp(const fira_ctx* ctx) {
  FiraHp h;
  h.beta1 = ctx->hp.beta1; h.beta2 = ctx->hp.beta2; h.eps = ctx->hp.eps; h.gamma = ctx->hp.gamma;
  h.b1 = (float)ctx->hp.beta1; h.b2 = (float)ctx->hp.beta2;
  h.omb1 = (float)(1.0 - ctx->hp.beta1); h.omb2 = (float)(1.0 - ctx->hp.beta2);
  h.epsf = (float)ctx->hp.eps;
  h.lr_alpha = ctx->d_lr_alpha;
  h.scaling = ctx->scaling;
  h.norm_mode = ctx->norm_mode;
  h.variant = ctx->variant;
  h.fused = 0;
  h.ortho_tol = 0.02f;   // bf16-rounded orthonormal projectors measure ~1e-3; a projector beyond 0.02 is not meant to be orthonormal
  h.gram_tol = 2e-3f;    // measured relative error of ||S||^2 by the Gram route: 1e-3 of ||S||
  h.mixed = 0;
  h.zsplit = ctx->zsplit ? 1 : 0;
  return h;
}

bool valid_hp(const fira_hparams* hp) {
  return hp && std::isfinite(hp->lr) && hp->beta1 >= 0 && hp->beta1 < 1 && hp->beta2 >= 0 && hp->beta2 < 1 &&
         hp->eps >= 0 && std::isfinite(hp->eps) && std::isfinite(hp->alpha) && hp->gamma > 0;
}

// Every matrix's gate values of the Gram route in one strided copy (stream-ordered; fira_step waits for it).
fira_status read_back_gates(fira_ctx* ctx) {
  const size_t nmat = ctx->plan.mats.size();
  FIRA_HIP(ctx, hipMemcpy2DAsync(ctx->h_gate, sizeof(fira_ctx::Gate), reinterpret_cast<char*>(ctx->d_scal) + offsetof(FiraScal, ortho_err),
                                 sizeof(FiraScal), sizeof(fira_ctx::Gate), nmat, hipMemcpyDeviceToHost, ctx->stream));
  FIRA_HIP(ctx, hipEventRecord(ctx->ortho_event, ctx->stream));
  ctx->ortho_pending = true;
  return FIRA_OK;
}

// Builds the work list of one fira_step call in pinned staging and returns its slot.
ListSlot* acquire_list(fira_ctx* ctx, int count, const int* idx, void* const* W, const void* const* G,
                       fira_status* st) {
  *st = FIRA_OK;
  ctx->use_counter++;
  for (ListSlot& s : ctx->slots) {
    if (s.valid && (int)s.idx.size() == count && std::equal(idx, idx + count, s.idx.begin()) &&
        std::equal(W, W + count, s.W.begin()) && std::equal(G, G + count, s.G.begin())) {
      s.last_use = ctx->use_counter;
      return &s;
    }
  }
  ListSlot* s = &ctx->slots[0];
  for (ListSlot& c : ctx->slots)
    if (!c.valid) { s = &c; break; } else if (c.last_use < s->last_use) s = &c;
  // the previous upload from this slot's staging must have been consumed before it is rewritten
  if (hipEventSynchronize(s->uploaded) != hipSuccess) { *st = FIRA_ERR_HIP; return nullptr; }
  s->valid = false;
  s->idx.assign(idx, idx + count);
  s->W.assign(W, W + count);
  s->G.assign(G, G + count);
  const Plan& p = ctx->plan;
  build_work_list(p, count, idx, W, G, s->h_stage, s->ntiles, &s->rowblocks, &s->g2blocks);
  if (hipMemcpyAsync(s->d_block, s->h_stage, p.slot_bytes, hipMemcpyHostToDevice, ctx->stream) != hipSuccess ||
      hipEventRecord(s->uploaded, ctx->stream) != hipSuccess) { *st = FIRA_ERR_HIP; return nullptr; }
  s->valid = true;
  s->last_use = ctx->use_counter;
  return s;
}

}  // namespace

extern "C" {

int64_t fira_method_state_numel(const fira_matrix_desc* d) {
  std::string why;
  if (!d || !valid_desc(*d, &why)) return 0;
  const int64_t S = std::min(d->m, d->n), L = std::max(d->m, d->n);
  return S * d->r + 2 * L * d->r + 1;
}

size_t fira_state_bytes(const fira_matrix_desc* d, int count) {
  Plan p; fira_status st; std::string why;
  if (!make_plan(d, count, &p, &st, &why)) { g_last_error = why; return 0; }
  return p.total;
}

fira_status fira_init_state(fira_ctx** out, const fira_matrix_desc* d, int count, const fira_hparams* hp,
                            void* dev_state, size_t dev_state_bytes, void* hip_stream) {
  if (!out) return fail(nullptr, FIRA_ERR_INVALID_ARG, "out is null");
  *out = nullptr;
  if (!valid_hp(hp)) return fail(nullptr, FIRA_ERR_INVALID_ARG, "hyper-parameters are null or out of range");
  fira_ctx* ctx = new fira_ctx();
  fira_status st = FIRA_OK; std::string why;
  if (!make_plan(d, count, &ctx->plan, &st, &why)) { delete ctx; return fail(nullptr, st, why); }
  if (!dev_state) { delete ctx; return fail(nullptr, FIRA_ERR_INVALID_ARG, "dev_state is null"); }
  if (((uintptr_t)dev_state % kAlign) != 0 || dev_state_bytes < ctx->plan.total) {
    delete ctx; return fail(nullptr, FIRA_ERR_WORKSPACE, "dev_state must be 256-byte aligned and hold fira_state_bytes() bytes");
  }
  ctx->static_scratch = static_scratch_address(&ctx->device, &why);
  if (!ctx->static_scratch) { delete ctx; return fail(nullptr, FIRA_ERR_HIP, why); }
  ctx->slab = (char*)dev_state;
  ctx->stream = (hipStream_t)hip_stream;
  ctx->hp = *hp;
  Plan& p = ctx->plan;
  for (HostMat& h : p.mats) {
    FiraMat& m = h.dev;
    // offsets were stored in the pointer fields; Gx is null for bf16 matrices and stays null
    m.M = (float*)(ctx->slab + (size_t)m.M); m.V = (float*)(ctx->slab + (size_t)m.V);
    m.Rt = (float*)(ctx->slab + (size_t)m.Rt); m.phi = (float*)(ctx->slab + (size_t)m.phi);
    m.g2 = (float*)(ctx->slab + (size_t)m.g2); m.q = (float*)(ctx->slab + (size_t)m.q);
    m.Nb = (bf16_raw*)(ctx->slab + (size_t)m.Nb); m.Rb = (bf16_raw*)(ctx->slab + (size_t)m.Rb);
    m.Pn = (bf16_raw*)(ctx->slab + (size_t)m.Pn); m.PT = (bf16_raw*)(ctx->slab + (size_t)m.PT);
    if (m.kx > 1) m.Gx = (bf16_raw*)(ctx->slab + (size_t)m.Gx);
  }
  ctx->d_mats = (FiraMat*)(ctx->slab + p.off_mats);
  ctx->d_scal = (FiraScal*)(ctx->slab + p.off_scal);
  ctx->d_partial = (float*)(ctx->slab + p.off_partial);
  ctx->d_lr_alpha = (float*)(ctx->slab + p.off_dyn);

  auto cleanup = [&]() {
    for (ListSlot& s : ctx->slots) if (s.uploaded) (void)hipEventDestroy(s.uploaded);
    if (ctx->h_stage_all) (void)hipHostFree(ctx->h_stage_all);
    if (ctx->h_gate) (void)hipHostFree(ctx->h_gate);
    if (ctx->h_install) (void)hipHostFree(ctx->h_install);
    if (ctx->ortho_event) (void)hipEventDestroy(ctx->ortho_event);
    if (ctx->install_event) (void)hipEventDestroy(ctx->install_event);
    delete ctx;
  };
#define FIRA_INIT_HIP(call)                                                                          \
  do {                                                                                               \
    hipError_t e_ = (call);                                                                          \
    if (e_ != hipSuccess) {                                                                          \
      std::string msg_ = std::string(#call) + ": " + hipGetErrorString(e_);                          \
      cleanup();                                                                                     \
      return fail(nullptr, FIRA_ERR_HIP, msg_);                                                      \
    }                                                                                                \
  } while (0)
  // the contraction kernels use more dynamic LDS than the 64 KB default (gfx950 has 160 KB per CU)
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_project_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_PROJ_LDS));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_backproject_kernel<0, bf16_raw>, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_BACK_LDS));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_backproject_kernel<1, bf16_raw>, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_BACK_LDS));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_backproject_kernel<0, float>, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_BACK_LDS));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_backproject_kernel<1, float>, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_BACK_LDS));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_refresh_chol_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_CHOL_PAN_ROWS * (FIRA_CHOL_NB + 1) * 8));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_refresh_solve_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_SOLVE_LDS));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_adam_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * FIRA_ROWS_PER_WG * FIRA_ZREADY_MAX_R * 2));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_project_adam_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_FUSE_LDS(1)));
  FIRA_INIT_HIP(hipFuncSetAttribute((const void*)fira_project_adam_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, FIRA_FUSE_LDS(2)));
  FIRA_INIT_HIP(hipHostMalloc((void**)&ctx->h_stage_all, p.slot_bytes * kSlots, hipHostMallocDefault));
  FIRA_INIT_HIP(hipHostMalloc((void**)&ctx->h_gate, sizeof(fira_ctx::Gate) * count, hipHostMallocDefault));
  for (int i = 0; i < count; ++i) ctx->h_gate[i] = fira_ctx::Gate{INFINITY, INFINITY};
  FIRA_INIT_HIP(hipEventCreateWithFlags(&ctx->ortho_event, hipEventDisableTiming));
  FIRA_INIT_HIP(hipHostMalloc((void**)&ctx->h_install, sizeof(FiraRefreshEnt) * count, hipHostMallocDefault));
  FIRA_INIT_HIP(hipEventCreateWithFlags(&ctx->install_event, hipEventDisableTiming));
  for (int i = 0; i < kSlots; ++i) {
    ListSlot& s = ctx->slots[i];
    s.h_stage = ctx->h_stage_all + p.slot_bytes * i;
    s.d_block = ctx->slab + p.off_slots + p.slot_bytes * i;
    s.block_bytes = p.slot_bytes;
    s.d_ents = (FiraEnt*)s.d_block;
    for (int l = 0; l < kNumTileLists; ++l) s.d_tiles[l] = (FiraTile*)(s.d_block + p.slot_off_tiles[l]);
    FIRA_INIT_HIP(hipEventCreateWithFlags(&s.uploaded, hipEventDisableTiming));
    FIRA_INIT_HIP(hipEventRecord(s.uploaded, ctx->stream));
  }
  // Zero everything: M = V = 0, t = 0, "no previous norm", and the zero padding of every operand.
  FIRA_INIT_HIP(hipMemsetAsync(ctx->slab, 0, p.total, ctx->stream));
  FIRA_INIT_HIP(store_step_size(ctx));
  std::vector<FiraMat> mats(count);
  for (int i = 0; i < count; ++i) mats[i] = p.mats[i].dev;
  FIRA_INIT_HIP(hipMemcpyAsync(ctx->d_mats, mats.data(), sizeof(FiraMat) * count, hipMemcpyHostToDevice, ctx->stream));
  FIRA_INIT_HIP(hipStreamSynchronize(ctx->stream));   // `mats` is a local
#undef FIRA_INIT_HIP
  *out = ctx;
  return FIRA_OK;
}

fira_status fira_set_hparams(fira_ctx* ctx, const fira_hparams* hp) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (!valid_hp(hp)) return fail(ctx, FIRA_ERR_INVALID_ARG, "hyper-parameters are null or out of range");
  ctx->hp = *hp;
  FIRA_HIP(ctx, store_step_size(ctx));
  return FIRA_OK;
}

fira_status fira_set_options(fira_ctx* ctx, fira_scaling scaling, fira_norm_mode norm_mode) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (scaling != FIRA_SCALE_COLUMN && scaling != FIRA_SCALE_MATRIX && scaling != FIRA_SCALE_NONE) return fail(ctx, FIRA_ERR_INVALID_ARG, "unknown scaling mode");
  if (norm_mode != FIRA_NORM_RESIDUAL && norm_mode != FIRA_NORM_GRAM) return fail(ctx, FIRA_ERR_INVALID_ARG, "unknown norm mode");
  ctx->scaling = scaling;
  ctx->norm_mode = norm_mode;
  return FIRA_OK;
}

fira_status fira_set_variant(fira_ctx* ctx, fira_variant variant) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (variant != FIRA_VARIANT_FULL && variant != FIRA_VARIANT_ONLY_SCALING) return fail(ctx, FIRA_ERR_INVALID_ARG, "unknown variant");
  ctx->variant = variant;
  return FIRA_OK;
}

fira_status fira_set_fusion(fira_ctx* ctx, int enable) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  ctx->fusion = enable != 0;
  return FIRA_OK;
}

int fira_last_step_fused(const fira_ctx* ctx) { return ctx && ctx->last_step_fused ? 1 : 0; }

fira_status fira_set_z_planes(fira_ctx* ctx, int planes) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (planes != 1 && planes != 2) return fail(ctx, FIRA_ERR_INVALID_ARG, "planes must be 1 or 2");
  ctx->zsplit = planes == 2;
  return FIRA_OK;
}

fira_status fira_set_projector(fira_ctx* ctx, int idx, const void* dev_P, fira_dtype p_dtype) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  if (!dev_P) return fail(ctx, FIRA_ERR_INVALID_ARG, "dev_P is null");
  if (p_dtype != FIRA_F32 && p_dtype != FIRA_BF16) return fail(ctx, FIRA_ERR_DTYPE, "p_dtype must be FIRA_F32 or FIRA_BF16");
  HostMat& h = ctx->plan.mats[idx];
  const long long total = (long long)h.dev.S * h.dev.r;
  const int grid = (int)std::min<long long>((total + 255) / 256, 65535);
  if (p_dtype == FIRA_F32)
    hipLaunchKernelGGL(fira_prep_projector_kernel<float>, dim3(grid), dim3(256), 0, ctx->stream, h.dev, (const float*)dev_P);
  else
    hipLaunchKernelGGL(fira_prep_projector_kernel<bf16_raw>, dim3(grid), dim3(256), 0, ctx->stream, h.dev, (const bf16_raw*)dev_P);
  // gate of the Gram route: estimate ||P^T P - I|| (stream-ordered, shares one S x 4 float scratch)
  float* ybuf = reinterpret_cast<float*>(ctx->slab + ctx->plan.off_ortho);
  hipLaunchKernelGGL(fira_ortho_y_kernel, dim3((h.dev.S + 3) / 4), dim3(256), 0, ctx->stream, h.dev, ybuf);
  float* zbuf = reinterpret_cast<float*>(ctx->slab + ctx->plan.off_ortho + ctx->plan.ortho_z);
  hipLaunchKernelGGL(fira_ortho_z_kernel, dim3(FIRA_ORTHO_SPLITS), dim3(256), 0, ctx->stream, h.dev, (const float*)ybuf, zbuf);
  hipLaunchKernelGGL(fira_ortho_final_kernel, dim3(1), dim3(256), 0, ctx->stream, h.dev, (const float*)zbuf, ctx->d_scal, idx);
  FIRA_HIP(ctx, hipGetLastError());
  static_assert(offsetof(FiraScal, gram_err) == offsetof(FiraScal, ortho_err) + sizeof(float), "the two gate values are read back as one piece");
  ctx->h_gate[idx] = fira_ctx::Gate{INFINITY, INFINITY};
  FIRA_HIP(ctx, hipMemcpyAsync(&ctx->h_gate[idx], reinterpret_cast<char*>(&ctx->d_scal[idx]) + offsetof(FiraScal, ortho_err),
                               sizeof(fira_ctx::Gate), hipMemcpyDeviceToHost, ctx->stream));
  FIRA_HIP(ctx, hipEventRecord(ctx->ortho_event, ctx->stream));
  ctx->ortho_pending = true;
  h.has_projector = true;
  return FIRA_OK;
}

fira_status fira_set_projectors(fira_ctx* ctx, int count, const int* idx, const void* const* dev_P, fira_dtype p_dtype) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (count == 0) return FIRA_OK;
  const int nmat = (int)ctx->plan.mats.size();
  if (count < 0 || count > nmat || !idx || !dev_P) return fail(ctx, FIRA_ERR_INVALID_ARG, "bad count or null array");
  if (p_dtype != FIRA_F32 && p_dtype != FIRA_BF16) return fail(ctx, FIRA_ERR_DTYPE, "p_dtype must be FIRA_F32 or FIRA_BF16");
  {
    std::vector<char> seen(nmat, 0);
    for (int e = 0; e < count; ++e) {
      if (idx[e] < 0 || idx[e] >= nmat) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
      if (seen[idx[e]]) return fail(ctx, FIRA_ERR_INVALID_ARG, "a matrix is listed twice");
      seen[idx[e]] = 1;
      if (!dev_P[e]) return fail(ctx, FIRA_ERR_INVALID_ARG, "null P pointer");
    }
  }
  hipStream_t q = ctx->stream;
  if (ctx->install_pending) {   // the previous call's table may still be on its way to the device
    FIRA_HIP(ctx, hipEventSynchronize(ctx->install_event));
    ctx->install_pending = false;
  }
  char* scratch = ctx->slab + ctx->plan.off_ortho;
  for (int e = 0; e < count; ++e) {
    const FiraMat& m = ctx->plan.mats[idx[e]].dev;
    FiraRefreshEnt& re = ctx->h_install[e];
    std::memset(&re, 0, sizeof(re));
    re.S = m.S; re.L = m.L; re.r = m.r; re.left = m.left; re.rq = m.rq; re.mat = idx[e];
    re.q_dtype = p_dtype == FIRA_BF16 ? 1 : 0;
    re.Q = reinterpret_cast<float*>(const_cast<void*>(dev_P[e]));   // read only, as q_dtype says
    re.inst = reinterpret_cast<float*>(scratch + ctx->plan.ortho_slot * (size_t)(e % kInstallBatch));
  }
  FiraRefreshEnt* d_table = reinterpret_cast<FiraRefreshEnt*>(ctx->slab + ctx->plan.off_install);
  FIRA_HIP(ctx, hipMemcpyAsync(d_table, ctx->h_install, sizeof(FiraRefreshEnt) * count, hipMemcpyHostToDevice, q));
  FIRA_HIP(ctx, hipEventRecord(ctx->install_event, q));
  ctx->install_pending = true;
  // one launch per phase for kInstallBatch matrices at a time (they share the scratch pieces, in stream order)
  for (int e0 = 0; e0 < count; e0 += kInstallBatch) {
    const int nb = std::min(kInstallBatch, count - e0);
    int max_S = 0, max_r = 0;
    for (int e = e0; e < e0 + nb; ++e) {
      max_S = std::max(max_S, ctx->h_install[e].S);
      max_r = std::max(max_r, ctx->h_install[e].r);
    }
    const int prep_blocks = (int)std::min<long long>(((long long)max_S * max_r + 255) / 256, 4096);
    hipLaunchKernelGGL(fira_refresh_prep_kernel, dim3(prep_blocks, nb), dim3(256), 0, q, ctx->d_mats, d_table + e0);
    hipLaunchKernelGGL(fira_refresh_ortho_y_kernel, dim3((max_S + 3) / 4, nb), dim3(256), 0, q, ctx->d_mats, d_table + e0);
    hipLaunchKernelGGL(fira_refresh_ortho_z_kernel, dim3(FIRA_ORTHO_SPLITS, nb), dim3(256), 0, q, ctx->d_mats, d_table + e0);
    hipLaunchKernelGGL(fira_refresh_ortho_final_kernel, dim3(nb), dim3(256), 0, q, ctx->d_mats, d_table + e0, ctx->d_scal);
  }
  {
    const hipError_t e_ = hipGetLastError();
    if (e_ != hipSuccess) {   // some of the listed matrices' operand copies may be half written
      for (int e = 0; e < count; ++e) {
        ctx->plan.mats[idx[e]].has_projector = false;
        ctx->h_gate[idx[e]] = fira_ctx::Gate{INFINITY, INFINITY};
      }
      return fail(ctx, FIRA_ERR_HIP, std::string("projector installation: ") + hipGetErrorString(e_));
    }
  }
  for (int e = 0; e < count; ++e) {
    ctx->h_gate[idx[e]] = fira_ctx::Gate{INFINITY, INFINITY};
    ctx->plan.mats[idx[e]].has_projector = true;
  }
  return read_back_gates(ctx);
}

fira_status fira_step(fira_ctx* ctx, int count, const int* idx, void* const* dev_W, const void* const* dev_G) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  const int nmat = (int)ctx->plan.mats.size();
  if (count == 0) return FIRA_OK;
  if (count < 0 || count > nmat || !idx || !dev_W || !dev_G) return fail(ctx, FIRA_ERR_INVALID_ARG, "bad count or null array");
  {
    std::vector<char> seen(nmat, 0);
    for (int e = 0; e < count; ++e) {
      if (idx[e] < 0 || idx[e] >= nmat) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
      if (seen[idx[e]]) return fail(ctx, FIRA_ERR_INVALID_ARG, "a matrix is listed twice");
      seen[idx[e]] = 1;
      if (!dev_W[e] || !dev_G[e]) return fail(ctx, FIRA_ERR_INVALID_ARG, "null W or G pointer");
      if (!ctx->plan.mats[idx[e]].has_projector) return fail(ctx, FIRA_ERR_NO_PROJECTOR, "fira_set_projector was never called for a listed matrix");
    }
  }
  fira_status st;
  ListSlot* s = acquire_list(ctx, count, idx, dev_W, dev_G, &st);
  if (!s) return fail(ctx, st, "building the work list failed");
  FiraHp hp = make_hp(ctx);
  hipStream_t q = ctx->stream;
  hipEvent_t* pe = nullptr;
  if (ctx->prof_steps < ctx->prof_max_steps) pe = &ctx->prof_events[(size_t)ctx->prof_steps++ * (FIRA_NUM_KERNELS + 1)];
  auto mark = [&](int k) { if (pe) (void)hipEventRecord(pe[k], q); };
  mark(0);

  // fp32 matrices: split the gradient into bf16 planes first (one launch for all of them)
  {
    long long most = 0;
    for (int e = 0; e < count; ++e) {
      const HostMat& h = ctx->plan.mats[idx[e]];
      if (h.dev.kx > 1) most = std::max(most, (long long)h.dev.m * h.dev.n);
    }
    if (most > 0)
      hipLaunchKernelGGL(fira_split_gradients_kernel, dim3((unsigned)std::min<long long>((most + 255) / 256, 4096), count), dim3(256), 0, q,
                         ctx->d_mats, s->d_ents);
  }
  auto grid8 = [](int n) { return dim3((unsigned)(((n + 7) / 8) * 8)); };
  const dim3 blk(FIRA_PROJ_THREADS);
  // R = P^T G (long-side major) for both orientations in one launch
  auto launch_project = [&](int norm_arg) {
    int nl = s->ntiles[kTilesProjBigLeft], nr = s->ntiles[kTilesProjBigRight];
    int bl = (nl + 7) / 8 * 8, br = (nr + 7) / 8 * 8;
    if (nl + nr)
      hipLaunchKernelGGL(fira_project_kernel, dim3(bl + br), blk, FIRA_PROJ_LDS, q, ctx->d_mats, s->d_ents,
                         s->d_tiles[kTilesProjBigLeft], nl, bl, s->d_tiles[kTilesProjBigRight], nr, norm_arg, (const FiraScal*)ctx->d_scal, hp);
    nl = s->ntiles[kTilesProjSmallLeft]; nr = s->ntiles[kTilesProjSmallRight];
    bl = (nl + 7) / 8 * 8; br = (nr + 7) / 8 * 8;
    if (nl + nr)
      hipLaunchKernelGGL(fira_project_small_kernel, dim3(bl + br), blk, FIRA_PROJ_SMALL_LDS, q, ctx->d_mats, s->d_ents,
                         s->d_tiles[kTilesProjSmallLeft], nl, bl, s->d_tiles[kTilesProjSmallRight], nr, norm_arg, (const FiraScal*)ctx->d_scal, hp);
  };
  // 0. Gram route, fp32 matrices only: ||G_i||^2 for every factor (bf16 matrices get it from step 1)
  const bool only_scaling = ctx->variant == FIRA_VARIANT_ONLY_SCALING;
  const int want_g2 = (ctx->norm_mode == FIRA_NORM_GRAM || only_scaling) ? 1 : 0;   // ||G_i||^2 per factor
  if (want_g2 && s->ntiles[kTilesBackF32] > 0)
    hipLaunchKernelGGL(fira_gradnorm_kernel, dim3(s->g2blocks), dim3(256), 0, q, ctx->d_mats, ctx->d_scal, s->d_ents, count,
                       s->g2blocks, hp);
  // Which listed matrices take the Gram route to ||S|| (the kernels apply the same test per matrix: both
  // gate values of FiraScal within FiraHp's tolerances).  A matrix whose second gate value is still to be
  // measured takes the residual route in this step, and the limiter measures it.
  bool need_residual = !only_scaling;
  bool any_gram = false, measures = false;
  if (need_residual && ctx->norm_mode == FIRA_NORM_GRAM) {
    if (ctx->ortho_pending) {   // gate values are on their way back (a projector was installed, or a step measured one)
      FIRA_HIP(ctx, hipEventSynchronize(ctx->ortho_event));
      ctx->ortho_pending = false;
    }
    need_residual = false;
    for (int e = 0; e < count; ++e) {
      const fira_ctx::Gate gt = ctx->h_gate[idx[e]];
      const bool gram = gt.ortho_err <= hp.ortho_tol && gt.gram_err <= hp.gram_tol;
      any_gram = any_gram || gram;
      need_residual = need_residual || !gram;
      measures = measures || (gt.ortho_err <= hp.ortho_tol && !(gt.gram_err < INFINITY));
    }
  }
  // The fused projection/Adam kernel serves the listed matrices on the Gram route if each of them can take
  // it; those on the residual route then go through the two-kernel path in the same step (hp.mixed).
  bool fused = ctx->fusion && !ctx->zsplit && !only_scaling && ctx->scaling == FIRA_SCALE_COLUMN && ctx->norm_mode == FIRA_NORM_GRAM && any_gram;
  for (int e = 0; e < count && fused; ++e) {
    const fira_ctx::Gate gt = ctx->h_gate[idx[e]];
    if (gt.ortho_err <= hp.ortho_tol && gt.gram_err <= hp.gram_tol) fused = ctx->plan.mats[idx[e]].fuse_list >= 0;
  }
  const bool mixed = fused && need_residual;
  ctx->last_step_fused = fused && !mixed;
  hp.fused = fused ? 1 : 0;
  hp.mixed = mixed ? 1 : 0;
  if (fused) {
    // 1+2. R = P^T G, Adam on it, factor norms, Z for c = 1
    for (int rt = 1; rt <= 2; ++rt) {
      const int ll = kTilesFuse + 2 * (rt - 1), lr = ll + 1;
      const int nl = s->ntiles[ll], nr = s->ntiles[lr];
      if (nl + nr == 0) continue;
      const int bl = (nl + 7) / 8 * 8, br = (nr + 7) / 8 * 8;
      if (rt == 1)
        hipLaunchKernelGGL(fira_project_adam_kernel<1>, dim3(bl + br), dim3(256), FIRA_FUSE_LDS(1), q, ctx->d_mats, ctx->d_scal, s->d_ents,
                           s->d_tiles[ll], nl, bl, s->d_tiles[lr], nr, hp);
      else
        hipLaunchKernelGGL(fira_project_adam_kernel<2>, dim3(bl + br), dim3(512), FIRA_FUSE_LDS(2), q, ctx->d_mats, ctx->d_scal, s->d_ents,
                           s->d_tiles[ll], nl, bl, s->d_tiles[lr], nr, hp);
    }
  }
  if (!fused || mixed) {
    // 1. R = P^T G
    launch_project(want_g2);
    mark(1);
    // 2. Adam on R, factor norms
    hipLaunchKernelGGL(fira_adam_kernel, dim3(s->rowblocks), dim3(256), ctx->plan.adam_lds * (ctx->zsplit ? 2 : 1), q, ctx->d_mats, ctx->d_scal,
                       s->d_ents, count, s->rowblocks, hp);
    mark(2);
  } else {
    mark(1);
    mark(2);
  }
  // 3. ||k (G - P R)||^2 per tile where the Gram route does not apply
  if (need_residual && s->ntiles[kTilesBackBf16])
    hipLaunchKernelGGL((fira_backproject_kernel<0, bf16_raw>), grid8(s->ntiles[kTilesBackBf16]), dim3(FIRA_BACK_THREADS), FIRA_BACK_LDS, q,
                       ctx->d_mats, ctx->d_scal, s->d_ents, s->d_tiles[kTilesBackBf16], s->ntiles[kTilesBackBf16],
                       ctx->d_partial, hp);
  if (need_residual && s->ntiles[kTilesBackF32])
    hipLaunchKernelGGL((fira_backproject_kernel<0, float>), grid8(s->ntiles[kTilesBackF32]), dim3(FIRA_BACK_THREADS), FIRA_BACK_LDS, q,
                       ctx->d_mats, ctx->d_scal, s->d_ents, s->d_tiles[kTilesBackF32], s->ntiles[kTilesBackF32],
                       ctx->d_partial, hp);
  mark(3);
  // 4. limiter factor, state advance
  hipLaunchKernelGGL(fira_limiter_kernel, dim3(count), dim3(FIRA_LIMITER_THREADS), 0, q, ctx->d_mats, ctx->d_scal, s->d_ents, ctx->d_partial, hp);
  mark(4);
  // 5. Z = N - c k R (after the fused kernel, which keeps no R: Z = c Z_1 + (1 - c) N for the matrices with c < 1)
  if (!only_scaling)
    hipLaunchKernelGGL(fira_makez_kernel, dim3(count * FIRA_MAKEZ_PARTS), dim3(256), 0, q, ctx->d_mats, ctx->d_scal, s->d_ents, hp);
  mark(5);
  // 6. W -= lr alpha (P Z + c k G)    (only-scaling variant: W -= lr alpha c k G, a plain stream)
  if (only_scaling) {
    if (s->ntiles[kTilesBackBf16])
      hipLaunchKernelGGL(fira_scale_update_kernel<bf16_raw>, grid8(s->ntiles[kTilesBackBf16]), dim3(256), 0, q,
                         ctx->d_mats, ctx->d_scal, s->d_ents, s->d_tiles[kTilesBackBf16], s->ntiles[kTilesBackBf16], hp);
    if (s->ntiles[kTilesBackF32])
      hipLaunchKernelGGL(fira_scale_update_kernel<float>, grid8(s->ntiles[kTilesBackF32]), dim3(256), 0, q,
                         ctx->d_mats, ctx->d_scal, s->d_ents, s->d_tiles[kTilesBackF32], s->ntiles[kTilesBackF32], hp);
  } else {
    if (s->ntiles[kTilesBackBf16])
      hipLaunchKernelGGL((fira_backproject_kernel<1, bf16_raw>), grid8(s->ntiles[kTilesBackBf16]), dim3(FIRA_BACK_THREADS), FIRA_BACK_LDS, q,
                         ctx->d_mats, ctx->d_scal, s->d_ents, s->d_tiles[kTilesBackBf16], s->ntiles[kTilesBackBf16],
                         ctx->d_partial, hp);
    if (s->ntiles[kTilesBackF32])
      hipLaunchKernelGGL((fira_backproject_kernel<1, float>), grid8(s->ntiles[kTilesBackF32]), dim3(FIRA_BACK_THREADS), FIRA_BACK_LDS, q,
                         ctx->d_mats, ctx->d_scal, s->d_ents, s->d_tiles[kTilesBackF32], s->ntiles[kTilesBackF32],
                         ctx->d_partial, hp);
  }
  mark(6);
  FIRA_HIP(ctx, hipGetLastError());
  if (measures) return read_back_gates(ctx);   // the limiter has measured a second gate value: the next step needs it
  return FIRA_OK;
}

static void destroy_profile_events(fira_ctx* ctx) {
  for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
  ctx->prof_events.clear();
  ctx->prof_max_steps = ctx->prof_steps = 0;
}

fira_status fira_profile_begin(fira_ctx* ctx, int max_steps) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (max_steps < 1 || max_steps > 100000) return fail(ctx, FIRA_ERR_INVALID_ARG, "max_steps out of range");
  destroy_profile_events(ctx);
  ctx->prof_events.resize((size_t)max_steps * (FIRA_NUM_KERNELS + 1));
  for (hipEvent_t& e : ctx->prof_events) {
    e = nullptr;
    hipError_t err = hipEventCreate(&e);
    if (err != hipSuccess) { destroy_profile_events(ctx); return fail(ctx, FIRA_ERR_HIP, std::string("hipEventCreate: ") + hipGetErrorString(err)); }
  }
  ctx->prof_max_steps = max_steps;
  ctx->prof_steps = 0;
  return FIRA_OK;
}

fira_status fira_profile_end(fira_ctx* ctx, double* ms_sum, int* steps) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (!ms_sum || !steps) return fail(ctx, FIRA_ERR_INVALID_ARG, "null output");
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  for (int k = 0; k < FIRA_NUM_KERNELS; ++k) ms_sum[k] = 0.0;
  for (int s = 0; s < ctx->prof_steps; ++s) {
    hipEvent_t* pe = &ctx->prof_events[(size_t)s * (FIRA_NUM_KERNELS + 1)];
    for (int k = 0; k < FIRA_NUM_KERNELS; ++k) {
      float ms = 0.0f;
      FIRA_HIP(ctx, hipEventElapsedTime(&ms, pe[k], pe[k + 1]));
      ms_sum[k] += ms;
    }
  }
  *steps = ctx->prof_steps;
  destroy_profile_events(ctx);
  return FIRA_OK;
}

const char* fira_kernel_name(int k) {
  static const char* names[FIRA_NUM_KERNELS] = {"project", "adam_norms", "residual_norm", "limiter", "make_z", "update"};
  return (k >= 0 && k < FIRA_NUM_KERNELS) ? names[k] : "";
}

fira_status fira_get_state(fira_ctx* ctx, int idx, float* host_M, float* host_V, double* s_prev, int64_t* t) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  const FiraMat& m = ctx->plan.mats[idx].dev;
  const size_t Lr = (size_t)m.L * m.r;
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  std::vector<float> tmp;
  for (int which = 0; which < 2; ++which) {
    float* dst = which ? host_V : host_M;
    const float* src = which ? m.V : m.M;
    if (!dst) continue;
    if (!m.left) {
      FIRA_HIP(ctx, hipMemcpy(dst, src, Lr * 4, hipMemcpyDeviceToHost));
    } else {   // device keeps [n][r]; the paper's orientation is r x n
      tmp.resize(Lr);
      FIRA_HIP(ctx, hipMemcpy(tmp.data(), src, Lr * 4, hipMemcpyDeviceToHost));
      for (int i = 0; i < m.L; ++i)
        for (int a = 0; a < m.r; ++a) dst[(size_t)a * m.L + i] = tmp[(size_t)i * m.r + a];
    }
  }
  FiraScal sc;
  FIRA_HIP(ctx, hipMemcpy(&sc, ctx->d_scal + idx, sizeof(sc), hipMemcpyDeviceToHost));
  if (s_prev) *s_prev = sc.has_prev ? sc.s_prev : -1.0;
  if (t) *t = sc.t;
  return FIRA_OK;
}

fira_status fira_set_state(fira_ctx* ctx, int idx, const float* host_M, const float* host_V, double s_prev, int64_t t) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  if (!host_M || !host_V || t < 0 || t > INT32_MAX) return fail(ctx, FIRA_ERR_INVALID_ARG, "null state array or bad step count");
  const FiraMat& m = ctx->plan.mats[idx].dev;
  const size_t Lr = (size_t)m.L * m.r;
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  std::vector<float> tmp(Lr);
  for (int which = 0; which < 2; ++which) {
    const float* src = which ? host_V : host_M;
    float* dst = which ? m.V : m.M;
    if (!m.left) {
      FIRA_HIP(ctx, hipMemcpy(dst, src, Lr * 4, hipMemcpyHostToDevice));
    } else {
      for (int i = 0; i < m.L; ++i)
        for (int a = 0; a < m.r; ++a) tmp[(size_t)i * m.r + a] = src[(size_t)a * m.L + i];
      FIRA_HIP(ctx, hipMemcpy(dst, tmp.data(), Lr * 4, hipMemcpyHostToDevice));
    }
  }
  FiraScal sc;
  FIRA_HIP(ctx, hipMemcpy(&sc, ctx->d_scal + idx, sizeof(sc), hipMemcpyDeviceToHost));
  sc.has_prev = s_prev >= 0.0;
  sc.s_prev = sc.has_prev ? s_prev : 0.0;
  sc.t = (int)t;
  FIRA_HIP(ctx, hipMemcpy(ctx->d_scal + idx, &sc, sizeof(sc), hipMemcpyHostToDevice));
  return FIRA_OK;
}

fira_status fira_get_diag(fira_ctx* ctx, int idx, double* s_norm_pre, double* s_norm_post, double* c) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  FiraScal sc;
  FIRA_HIP(ctx, hipMemcpy(&sc, ctx->d_scal + idx, sizeof(sc), hipMemcpyDeviceToHost));
  if (s_norm_pre) *s_norm_pre = sc.s_pre;
  if (s_norm_post) *s_norm_post = sc.s_post;
  if (c) *c = sc.c;
  return FIRA_OK;
}

fira_status fira_get_gate(fira_ctx* ctx, int idx, float* ortho_err, float* gram_err, int* gram_route) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  FiraScal sc;
  FIRA_HIP(ctx, hipMemcpy(&sc, ctx->d_scal + idx, sizeof(sc), hipMemcpyDeviceToHost));
  if (ortho_err) *ortho_err = ctx->plan.mats[idx].has_projector ? sc.ortho_err : INFINITY;
  if (gram_err) *gram_err = ctx->plan.mats[idx].has_projector ? sc.gram_err : INFINITY;
  if (gram_route) *gram_route = sc.gram_now;
  return FIRA_OK;
}

fira_status fira_set_gate(fira_ctx* ctx, int idx, float ortho_err, float gram_err) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  if (!ctx->plan.mats[idx].has_projector) return fail(ctx, FIRA_ERR_NO_PROJECTOR, "install the projector first: fira_set_projector resets the gate");
  if (!(ortho_err >= 0.0f) || !(gram_err >= 0.0f)) return fail(ctx, FIRA_ERR_INVALID_ARG, "gate values must be >= 0 (+inf = not measured)");
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  const fira_ctx::Gate gt{ortho_err, gram_err};
  FIRA_HIP(ctx, hipMemcpy(reinterpret_cast<char*>(ctx->d_scal + idx) + offsetof(FiraScal, ortho_err), &gt, sizeof(gt), hipMemcpyHostToDevice));
  ctx->h_gate[idx] = gt;
  return FIRA_OK;
}

fira_status fira_get_factors(fira_ctx* ctx, int idx, float* host_k) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  if (!host_k) return fail(ctx, FIRA_ERR_INVALID_ARG, "host_k is null");
  const FiraMat& m = ctx->plan.mats[idx].dev;
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  FIRA_HIP(ctx, hipMemcpy(host_k, m.phi, (size_t)m.L * 4, hipMemcpyDeviceToHost));
  return FIRA_OK;
}

fira_status fira_get_lowrank(fira_ctx* ctx, int idx, float* host_R) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  if (!host_R) return fail(ctx, FIRA_ERR_INVALID_ARG, "host_R is null");
  const FiraMat& m = ctx->plan.mats[idx].dev;
  const size_t Lr = (size_t)m.L * m.r;
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (!m.left) {
    FIRA_HIP(ctx, hipMemcpy(host_R, m.Rt, Lr * 4, hipMemcpyDeviceToHost));
  } else {
    std::vector<float> tmp(Lr);
    FIRA_HIP(ctx, hipMemcpy(tmp.data(), m.Rt, Lr * 4, hipMemcpyDeviceToHost));
    for (int i = 0; i < m.L; ++i)
      for (int a = 0; a < m.r; ++a) host_R[(size_t)a * m.L + i] = tmp[(size_t)i * m.r + a];
  }
  return FIRA_OK;
}

fira_status fira_get_projector(fira_ctx* ctx, int idx, float* host_P) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (idx < 0 || idx >= (int)ctx->plan.mats.size()) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
  if (!host_P) return fail(ctx, FIRA_ERR_INVALID_ARG, "host_P is null");
  const HostMat& h = ctx->plan.mats[idx];
  if (!h.has_projector) return fail(ctx, FIRA_ERR_NO_PROJECTOR, "fira_set_projector was never called for this matrix");
  const FiraMat& m = h.dev;
  const size_t n = (size_t)m.Sq * m.kx * m.rp;
  std::vector<uint16_t> tmp(n);
  FIRA_HIP(ctx, hipStreamSynchronize(ctx->stream));
  FIRA_HIP(ctx, hipMemcpy(tmp.data(), m.Pn, n * 2, hipMemcpyDeviceToHost));
  auto bf = [](uint16_t b) { uint32_t u = (uint32_t)b << 16; float f; std::memcpy(&f, &u, 4); return f; };
  for (int s = 0; s < m.S; ++s)
    for (int a = 0; a < m.r; ++a) {
      if (m.kx == 1) {
        host_P[(size_t)s * m.r + a] = bf(tmp[(size_t)kblk_index(m.Sq, s, a)]);
      } else {   // planes of sequence B: h m h l h m
        host_P[(size_t)s * m.r + a] = (bf(tmp[(size_t)kblk_index(m.Sq, s, a)]) + bf(tmp[(size_t)kblk_index(m.Sq, s, m.rp + a)])) +
                                      bf(tmp[(size_t)kblk_index(m.Sq, s, 3 * m.rp + a)]);
      }
    }
  return FIRA_OK;
}

size_t fira_refresh_workspace_bytes(const fira_ctx* ctx, int count, const int* idx) {
  RefreshPlan rp;
  if (!ctx || !make_refresh_plan(ctx->plan, count, idx, &rp)) return 0;
  return rp.total;
}

namespace {

// 16-byte pieces [0, n16) of p set to zero (a kernel rather than hipMemsetAsync, so that it is an ordinary
// kernel node wherever the stream's work is recorded).
__global__ __launch_bounds__(256) void fira_zero_fill_kernel(u32x4* __restrict__ p, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = u32x4{0u, 0u, 0u, 0u};
}

// Argument checks shared by the two refresh entry points; on success *rp is the workspace layout.
fira_status refresh_check(fira_ctx* ctx, int count, const int* idx, const void* const* dev_G, int iters, RefreshPlan* rp) {
  const int nmat = (int)ctx->plan.mats.size();
  if (count < 0 || count > nmat || !idx || !dev_G) return fail(ctx, FIRA_ERR_INVALID_ARG, "bad count or null array");
  if (iters < 1 || iters > 64) return fail(ctx, FIRA_ERR_INVALID_ARG, "iters must be in [1, 64]");
  {
    std::vector<char> seen(nmat, 0);
    for (int e = 0; e < count; ++e) {
      if (idx[e] < 0 || idx[e] >= nmat) return fail(ctx, FIRA_ERR_INVALID_ARG, "matrix index out of range");
      if (seen[idx[e]]) return fail(ctx, FIRA_ERR_INVALID_ARG, "a matrix is listed twice");
      seen[idx[e]] = 1;
      if (!dev_G[e]) return fail(ctx, FIRA_ERR_INVALID_ARG, "null G pointer");
    }
  }
  if (!make_refresh_plan(ctx->plan, count, idx, rp)) return fail(ctx, FIRA_ERR_INVALID_ARG, "bad list");
  return FIRA_OK;
}

fira_status refresh_run(fira_ctx* ctx, int count, const int* idx, const void* const* dev_G, int iters, uint64_t seed,
                        const RefreshPlan& rp, char* ws);

}  // namespace

fira_status fira_refresh_projectors(fira_ctx* ctx, int count, const int* idx, const void* const* dev_G,
                                    int iters, uint64_t seed, void* dev_workspace, size_t workspace_bytes) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (count == 0) return FIRA_OK;
  RefreshPlan rp;
  const fira_status st = refresh_check(ctx, count, idx, dev_G, iters, &rp);
  if (st != FIRA_OK) return st;
  if (!dev_workspace || ((uintptr_t)dev_workspace % kAlign) != 0 || workspace_bytes < rp.total)
    return fail(ctx, FIRA_ERR_WORKSPACE, "dev_workspace must be 256-byte aligned and hold fira_refresh_workspace_bytes() bytes");
  return refresh_run(ctx, count, idx, dev_G, iters, seed, rp, (char*)dev_workspace);
}

fira_status fira_refresh_projectors_static(fira_ctx* ctx, int count, const int* idx, const void* const* dev_G,
                                           int iters, uint64_t seed) {
  if (!ctx) return fail(nullptr, FIRA_ERR_INVALID_ARG, "ctx is null");
  if (count == 0) return FIRA_OK;
  RefreshPlan rp;
  const fira_status st = refresh_check(ctx, count, idx, dev_G, iters, &rp);
  if (st != FIRA_OK) return st;
  if (rp.total > (size_t)FIRA_STATIC_SCRATCH_BYTES)
    return fail(ctx, FIRA_ERR_WORKSPACE, "the listed matrices need " + std::to_string(rp.total) + " bytes of workspace, more than the " +
                                         std::to_string((size_t)FIRA_STATIC_SCRATCH_BYTES) + " bytes of the library's static scratch: "
                                         "list fewer matrices per call or use fira_refresh_projectors");
  // ctx->static_scratch is the device address found at fira_init_state (never the array's name)
  return refresh_run(ctx, count, idx, dev_G, iters, seed, rp, (char*)ctx->static_scratch);
}

namespace {

fira_status refresh_run(fira_ctx* ctx, int count, const int* idx, const void* const* dev_G, int iters, uint64_t seed,
                        const RefreshPlan& rp, char* ws) {
  const int nmat = (int)ctx->plan.mats.size();
  hipStream_t q = ctx->stream;

  // host images of the small tables
  std::vector<FiraRefreshEnt> ents(count), ents2(count);
  std::vector<FiraMat> vmats(count);
  std::vector<FiraEnt> vents(count);
  std::vector<FiraTile> vtiles[2];
  int max_S = 0, max_r = 0, max_Lp = 0;
  for (int e = 0; e < count; ++e) {
    const FiraMat& m = ctx->plan.mats[idx[e]].dev;
    FiraRefreshEnt& re = ents[e];
    std::memset(&re, 0, sizeof(re));
    re.S = m.S; re.L = m.L; re.r = m.r; re.left = m.left; re.Lp = round_up_int(m.L, 64); re.rq = m.rq; re.mat = idx[e];
    re.T = m.Rt;
    re.Top = (bf16_raw*)(ws + rp.off_top[e]);
    re.Y = (float*)(ws + rp.off_y[e]);
    re.Q = (float*)(ws + rp.off_q[e]);
    re.C = (double*)(ws + rp.off_c[e]);
    re.inst = (float*)(ws + rp.off_linv[e]);
    ents2[e] = re;                       // second orthonormalisation pass of the last round: Q -> Y
    std::swap(ents2[e].Y, ents2[e].Q);
    // ... which is left out for a matrix whose basis is orthonormal already, to the accuracy its storage can hold
    ents2[e].done = (int*)(ws + rp.off_done) + e;
    ents2[e].done_tol = m.kx == 1 ? 1e-4f : 1e-6f;
    max_S = std::max(max_S, m.S); max_r = std::max(max_r, m.r); max_Lp = std::max(max_Lp, re.Lp);
    // The way back, Y[s][a] = sum_i G(s, i) T[i][a], is the projection kernel on the other orientation
    // of the same gradient: long side L' = S, contraction over S' = L, operand "PT" = Top, output "Rt" = Y.
    FiraMat& v = vmats[e];
    std::memset(&v, 0, sizeof(v));
    // fp32 matrices: the way back reads a bf16 rounding of the gradient made below (the way there runs on the
    // matrix's own split planes, as in a step)
    const bool f32 = m.kx != 1;
    v.m = m.m; v.n = m.n; v.r = m.r; v.left = !m.left; v.ld = f32 ? refresh_gb_ld(m.n) : m.ld;
    v.L = m.S; v.S = m.L; v.rp = m.rp; v.Sp = re.Lp; v.kx = 1; v.dtype = FIRA_BF16;
    v.Lq = round_up_int(m.S, 256); v.Sq = round_up_int(m.L, 256); v.rq = m.rq;
    v.PT = re.Top; v.Rt = re.Y;
    FiraEnt& ve = vents[e];
    std::memset(&ve, 0, sizeof(ve));
    ve.mat = e; ve.W = nullptr; ve.G = f32 ? (const void*)(ws + rp.off_gb[e]) : dev_G[e];
    const int ta_n = (m.S + FIRA_PA - 1) / FIRA_PA, tb_n = (m.r + FIRA_PB - 1) / FIRA_PB;
    for (int ta = 0; ta < ta_n; ++ta)
      for (int tb = 0; tb < tb_n; ++tb) vtiles[m.left ? 0 : 1].push_back(FiraTile{e, ta, tb, 0});
  }
  FIRA_HIP(ctx, hipMemcpyAsync(ws + rp.off_ents, ents.data(), sizeof(FiraRefreshEnt) * count, hipMemcpyHostToDevice, q));
  FIRA_HIP(ctx, hipMemcpyAsync(ws + rp.off_ents2, ents2.data(), sizeof(FiraRefreshEnt) * count, hipMemcpyHostToDevice, q));
  FIRA_HIP(ctx, hipMemcpyAsync(ws + rp.off_vmats, vmats.data(), sizeof(FiraMat) * count, hipMemcpyHostToDevice, q));
  FIRA_HIP(ctx, hipMemcpyAsync(ws + rp.off_vents, vents.data(), sizeof(FiraEnt) * count, hipMemcpyHostToDevice, q));
  for (int l = 0; l < 2; ++l)
    if (!vtiles[l].empty())
      FIRA_HIP(ctx, hipMemcpyAsync(ws + rp.off_vtiles[l], vtiles[l].data(), sizeof(FiraTile) * vtiles[l].size(), hipMemcpyHostToDevice, q));
  // the host vectors go away when this function returns: the copies above must have been made
  FIRA_HIP(ctx, hipStreamSynchronize(q));
  {   // padding rows of the packed operand must read as zero (the workspace keeps whatever it held before)
    const size_t n16 = (rp.top_end - rp.top_begin) / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 8192);
    if (n16) hipLaunchKernelGGL(fira_zero_fill_kernel, dim3(grid), dim3(256), 0, q, reinterpret_cast<u32x4*>(ws + rp.top_begin), n16);
  }

  for (int e = 0; e < count; ++e) {   // fp32 matrices: split planes for the way there, a bf16 rounding for the way back
    const FiraMat& m = ctx->plan.mats[idx[e]].dev;
    if (m.kx == 1) continue;
    const long long total = (long long)m.m * m.n;
    const int grid = (int)std::min<long long>((total + 255) / 256, 65535);
    hipLaunchKernelGGL(fira_split_gradient_kernel, dim3(grid), dim3(256), 0, q, m, (const float*)dev_G[e]);
    hipLaunchKernelGGL(fira_round_gradient_kernel, dim3(grid), dim3(256), 0, q, (const float*)dev_G[e],
                       (bf16_raw*)(ws + rp.off_gb[e]), m.m, m.n, (long long)m.ld, (long long)refresh_gb_ld(m.n));
  }

  const FiraRefreshEnt* d_ents = (const FiraRefreshEnt*)(ws + rp.off_ents);
  const FiraRefreshEnt* d_ents2 = (const FiraRefreshEnt*)(ws + rp.off_ents2);
  const FiraMat* d_vmats = (const FiraMat*)(ws + rp.off_vmats);
  const FiraEnt* d_vents = (const FiraEnt*)(ws + rp.off_vents);

  // the forward product uses the step's own work-list machinery (W is not touched by the projection)
  std::vector<void*> fakeW(count);
  for (int e = 0; e < count; ++e) fakeW[e] = const_cast<void*>(dev_G[e]);
  fira_status st;
  ListSlot* s = acquire_list(ctx, count, idx, fakeW.data(), dev_G, &st);
  if (!s) return fail(ctx, st, "building the work list failed");

  {
    const long long mx = (long long)max_S * max_r;
    hipLaunchKernelGGL(fira_refresh_init_kernel, dim3((unsigned)std::min<long long>((mx + 255) / 256, 4096), count), dim3(256), 0, q,
                       d_ents, (unsigned long long)seed);
  }
  const int nt64 = (max_r + 63) / 64;
  const int prep_blocks = (int)std::min<long long>(((long long)max_S * max_r + 255) / 256, 4096);
  auto orthonormalise = [&](const FiraRefreshEnt* de) {
    hipLaunchKernelGGL(fira_refresh_gram_kernel, dim3(nt64 * (nt64 + 1) / 2, count), dim3(256), 0, q, de);
    hipLaunchKernelGGL(fira_refresh_orthocheck_kernel, dim3(count), dim3(256), 0, q, de);   // (second pass only; else it leaves at once)
    {
      const int pan_rows = std::min(FIRA_CHOL_PAN_ROWS, std::max(max_r - FIRA_CHOL_NB, 0));
      hipLaunchKernelGGL(fira_refresh_chol_kernel, dim3(count), dim3(FIRA_CHOL_THREADS), (size_t)pan_rows * (FIRA_CHOL_NB + 1) * 8, q, de, pan_rows);
    }
    const int nj = (max_r + FIRA_SOLVE_JB - 1) / FIRA_SOLVE_JB;
    hipLaunchKernelGGL(fira_refresh_diaginv_kernel, dim3(nj, count), dim3(64), 0, q, de);
    for (int J = 0; J < nj; ++J)
      hipLaunchKernelGGL(fira_refresh_solve_kernel, dim3((max_S + 63) / 64, count), dim3(256), FIRA_SOLVE_LDS, q, de, J);
  };
  const FiraHp refresh_hp = make_hp(ctx);   // (mixed = 0: the projection kernel serves every listed matrix)
  auto launch_project = [&](const FiraMat* mats, const FiraEnt* ents_d, const FiraTile* tl, int nl, const FiraTile* tr, int nr) {
    const int bl = (nl + 7) / 8 * 8, br = (nr + 7) / 8 * 8;
    if (nl + nr)
      hipLaunchKernelGGL(fira_project_kernel, dim3(bl + br), dim3(FIRA_PROJ_THREADS), FIRA_PROJ_LDS, q, mats, ents_d, tl, nl, bl, tr, nr, 0,
                         (const FiraScal*)ctx->d_scal, refresh_hp);
  };
  for (int it = 0; it < iters; ++it) {
    // operands of Q (the fp32 Q becomes the matrix's projector copies; no gate estimate needed here)
    hipLaunchKernelGGL(fira_refresh_prep_kernel, dim3(prep_blocks, count), dim3(256), 0, q, ctx->d_mats, d_ents);
    // T = G^T Q (or G Q): the projection kernel, norm route off
    launch_project(ctx->d_mats, s->d_ents, s->d_tiles[kTilesProjectLeft], s->ntiles[kTilesProjectLeft],
                   s->d_tiles[kTilesProjectRight], s->ntiles[kTilesProjectRight]);
    // pack T as the K-blocked operand of the way back
    hipLaunchKernelGGL(fira_refresh_pack_kernel, dim3((max_Lp / 32) * nt64, count), dim3(256), 0, q, d_ents);
    // Y = G T (or G^T T): the projection kernel on the other orientation (list [1] is the K-slow one)
    launch_project(d_vmats, d_vents, (const FiraTile*)(ws + rp.off_vtiles[1]), rp.ntiles[1],
                   (const FiraTile*)(ws + rp.off_vtiles[0]), rp.ntiles[0]);
    // Q = orth(Y): CholeskyQR in fp64
    orthonormalise(d_ents);
  }
  // A second pass over the final basis (CholeskyQR2) brings ||Q^T Q - I|| down to rounding level even
  // when Y was ill conditioned; its result lands in the Y buffers.
  orthonormalise(d_ents2);
  // The rounds above worked in the listed matrices' operand copies of P.  If anything failed to launch, what
  // they hold now is not a projector: mark the matrices as having none rather than leave a half-made basis
  // behind the old gate values.
  auto invalidate = [&]() {
    for (int e = 0; e < count; ++e) {
      ctx->plan.mats[idx[e]].has_projector = false;
      ctx->h_gate[idx[e]] = fira_ctx::Gate{INFINITY, INFINITY};
    }
  };
  {
    const hipError_t e_ = hipGetLastError();
    if (e_ != hipSuccess) { invalidate(); return fail(ctx, FIRA_ERR_HIP, std::string("projector refresh: ") + hipGetErrorString(e_)); }
  }
  // install the result (what fira_set_projector does per matrix, here one launch per phase for the whole list)
  hipLaunchKernelGGL(fira_refresh_prep_kernel, dim3(prep_blocks, count), dim3(256), 0, q, ctx->d_mats, d_ents2);
  hipLaunchKernelGGL(fira_refresh_ortho_y_kernel, dim3((max_S + 3) / 4, count), dim3(256), 0, q, ctx->d_mats, d_ents2);
  hipLaunchKernelGGL(fira_refresh_ortho_z_kernel, dim3(FIRA_ORTHO_SPLITS, count), dim3(256), 0, q, ctx->d_mats, d_ents2);
  hipLaunchKernelGGL(fira_refresh_ortho_final_kernel, dim3(count), dim3(256), 0, q, ctx->d_mats, d_ents2, ctx->d_scal);
  {
    const hipError_t e_ = hipGetLastError();
    if (e_ != hipSuccess) { invalidate(); return fail(ctx, FIRA_ERR_HIP, std::string("projector refresh: ") + hipGetErrorString(e_)); }
  }
  for (int e = 0; e < count; ++e) {
    ctx->h_gate[idx[e]] = fira_ctx::Gate{INFINITY, INFINITY};
    ctx->plan.mats[idx[e]].has_projector = true;
  }
  return read_back_gates(ctx);
}

}  // namespace

const char* fira_last_error(const fira_ctx* ctx) { return ctx ? ctx->last_error.c_str() : g_last_error.c_str(); }

void fira_destroy(fira_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  destroy_profile_events(ctx);
  for (ListSlot& s : ctx->slots)
    if (s.uploaded) (void)hipEventDestroy(s.uploaded);
  if (ctx->h_stage_all) (void)hipHostFree(ctx->h_stage_all);
  if (ctx->h_gate) (void)hipHostFree(ctx->h_gate);
  if (ctx->h_install) (void)hipHostFree(ctx->h_install);
  if (ctx->ortho_event) (void)hipEventDestroy(ctx->ortho_event);
  if (ctx->install_event) (void)hipEventDestroy(ctx->install_event);
  delete ctx;
}

}  // extern "C"
