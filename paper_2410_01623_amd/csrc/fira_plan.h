// Host-side planning of the Fira library: where every array of every matrix sits in the caller's slab,
// the work list of a step (entries and tile lists), and the workspace of the projector refresh.  Pure
// host arithmetic on sizes and offsets (no HIP runtime call), so that it can also be built on its own with
// the host sanitizers and fuzzed (tests/host_plan_check.cpp).
#pragma once
#include "../../include/fira.h"

#include <algorithm>
#include <cstddef>
#include <cstring>
#include <string>
#include <vector>

#include "fira_device.h"

namespace {

constexpr size_t kAlign = 256;
constexpr int kInstallBatch = 16;   // matrices per launch of a batched projector installation
constexpr int kSlots = 4;  // cached work lists (a training loop alternates between very few)

inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }
inline int round_up_int(long long x, int a) { return (int)((x + a - 1) / a * a); }
// Row pitch (bf16 elements) for an operand row of k values: a whole number of 256-byte L2-channel
// lines, and an odd number of them, so that consecutive rows walk through all sixteen channels.
inline int operand_pitch(long long k) {
  long long lines = (k * 2 + 255) / 256;
  if (lines % 2 == 0) ++lines;
  return (int)(lines * 128);
}

struct HostMat {
  fira_matrix_desc d;
  FiraMat dev;          // copy of the device description (pointers are device pointers)
  bool has_projector = false;
  int tiles_project = 0;      // tiles of the R contraction
  int tiles_back = 0;         // tiles of the back-projection (and of the residual-norm pass)
  int ta_project = 0, tb_project = 0, ta_back = 0, tb_back = 0;
  int rowblocks = 0;
  int g2blocks = 0;           // blocks of the ||G_i||^2 kernel
  int fuse_list = -1;         // tile list of the fused projection/Adam kernel, or -1 if the matrix cannot take it
  bool small_proj = false;    // bf16 with r <= 64: projected by the small-rank kernel
};

// kTilesFuse + (r > 256 ? 2 : 0) + (left ? 0 : 1): tiles of the fused projection/Adam kernel (one per 128 factors)
// kTilesProject*: every matrix (the projector refresh runs the general kernel on all of them); a step uses
// kTilesProjBig* (general kernel) and kTilesProjSmall* (bf16 matrices with r <= 64), which split them.
enum { kTilesProjectLeft = 0, kTilesProjectRight = 1, kTilesBackBf16 = 2, kTilesBackF32 = 3, kTilesFuse = 4,
       kTilesProjBigLeft = 8, kTilesProjBigRight = 9, kTilesProjSmallLeft = 10, kTilesProjSmallRight = 11, kNumTileLists = 12 };


struct Plan {
  size_t total = 0;
  size_t off_mats = 0, off_scal = 0, off_partial = 0, off_ortho = 0, ortho_z = 0;
  size_t ortho_slot = 0, off_install = 0, off_dyn = 0;   // batched installation: kInstallBatch scratch pieces of ortho_slot bytes, table of FiraRefreshEnt
  size_t off_slots = 0, slot_bytes = 0, slot_off_tiles[kNumTileLists] = {};
  std::vector<HostMat> mats;
  int max_tiles[kNumTileLists] = {};
  int adam_lds = 0;          // dynamic LDS of the Adam kernel: 16 rows of the widest register-resident matrix
};

bool valid_desc(const fira_matrix_desc& d, std::string* why) {
  if (d.m < 1 || d.n < 1 || d.m > (1 << 22) || d.n > (1 << 22)) { *why = "m, n must be in [1, 2^22]"; return false; }
  if (d.ld < d.n || d.ld > (1 << 22)) { *why = "ld must be in [n, 2^22]"; return false; }
  if (d.r < 1 || d.r > std::min(d.m, d.n)) { *why = "need 1 <= r <= min(m, n)"; return false; }
  return true;
}

// Lays the slab out.  Pointers in Plan::mats[i].dev are offsets from a null base until rebased.
bool make_plan(const fira_matrix_desc* d, int count, Plan* plan, fira_status* st, std::string* why) {
  if (!d || count < 1 || count > (1 << 20)) { *st = FIRA_ERR_INVALID_ARG; *why = "descriptor array is null or count out of range"; return false; }
  plan->mats.resize(count);
  size_t off = 0;
  plan->off_mats = off; off = align_up(off + sizeof(FiraMat) * count);
  plan->off_scal = off; off = align_up(off + sizeof(FiraScal) * count);
  long long total_tiles[kNumTileLists] = {};
  for (int i = 0; i < count; ++i) {
    HostMat& h = plan->mats[i];
    h.d = d[i];
    if (d[i].wg_dtype != FIRA_F32 && d[i].wg_dtype != FIRA_BF16) { *st = FIRA_ERR_DTYPE; *why = "wg_dtype must be FIRA_F32 or FIRA_BF16"; return false; }
    if (!valid_desc(d[i], why)) { *st = FIRA_ERR_SHAPE; return false; }
    FiraMat& m = h.dev;
    std::memset(&m, 0, sizeof(m));
    m.m = (int)d[i].m; m.n = (int)d[i].n; m.r = d[i].r; m.left = d[i].m <= d[i].n;
    m.ld = d[i].ld;
    m.L = (int)std::max(d[i].m, d[i].n); m.S = (int)std::min(d[i].m, d[i].n);
    m.rp = round_up_int(m.r, 64); m.Sp = round_up_int(m.S, 64);
    m.dtype = d[i].wg_dtype;
    m.kx = (m.dtype == FIRA_F32) ? FIRA_KX_SPLIT : 1;
    m.Lq = round_up_int(m.L, 256); m.Sq = round_up_int(m.S, 256); m.rq = round_up_int(m.r, 256);
    m.zready = (m.kx == 1 && (m.r & 3) == 0 && m.r <= FIRA_ZREADY_MAX_R) ? 1 : 0;
    if (m.zready) plan->adam_lds = std::max(plan->adam_lds, FIRA_ROWS_PER_WG * m.rp * 2);   // (twice that with Z in two planes)
    m.gx_ld = m.left ? round_up_int(m.n, 8) : operand_pitch((long long)m.kx * m.Sp);
    const size_t Lr = (size_t)m.L * m.r;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    m.M = (float*)take(Lr * 4);
    m.V = (float*)take(Lr * 4);
    m.Rt = (float*)take(Lr * 4);
    m.phi = (float*)take((size_t)m.L * 4);
    m.g2 = (float*)take((size_t)m.L * 4);
    m.q = (float*)take((size_t)m.L * 4);
    m.Nb = (bf16_raw*)take((size_t)m.Lq * (m.kx == 1 ? 2 : m.kx) * m.rp * 2);   // bf16 matrices: room for the hi + lo form of Z
    m.Rb = (bf16_raw*)take((size_t)m.Lq * m.kx * m.rp * 2);
    m.Pn = (bf16_raw*)take((size_t)m.Sq * m.kx * m.rp * 2);
    m.PT = (bf16_raw*)take((size_t)m.rq * m.kx * m.Sp * 2);
    if (m.kx > 1) {
      const size_t gx = m.left ? (size_t)m.kx * m.Sp * m.gx_ld : (size_t)m.m * m.gx_ld;
      m.Gx = (bf16_raw*)take(gx * 2);
    }
    h.ta_project = (m.L + FIRA_PA - 1) / FIRA_PA; h.tb_project = (m.r + FIRA_PB - 1) / FIRA_PB;
    h.ta_back = (m.n + FIRA_BA - 1) / FIRA_BA;    h.tb_back = (m.m + FIRA_BB - 1) / FIRA_BB;
    h.tiles_project = h.ta_project * h.tb_project;
    h.tiles_back = h.ta_back * h.tb_back;
    h.rowblocks = (m.L + FIRA_ROWS_PER_WG - 1) / FIRA_ROWS_PER_WG;
    h.g2blocks = m.left ? (m.n + 255) / 256 : (m.m + FIRA_G2_ROWS_PER_WG - 1) / FIRA_G2_ROWS_PER_WG;
    total_tiles[m.left ? kTilesProjectLeft : kTilesProjectRight] += h.tiles_project;
    h.small_proj = m.kx == 1 && m.r <= FIRA_PS;
    total_tiles[(h.small_proj ? kTilesProjSmallLeft : kTilesProjBigLeft) + (m.left ? 0 : 1)] += h.tiles_project;
    total_tiles[m.dtype == FIRA_BF16 ? kTilesBackBf16 : kTilesBackF32] += h.tiles_back;
    if (m.zready && m.r >= FIRA_FUSE_MIN_R && m.r <= FIRA_FUSE_MAX_R) {
      h.fuse_list = kTilesFuse + 2 * (m.r > 256 ? 1 : 0) + (m.left ? 0 : 1);
      total_tiles[h.fuse_list] += h.ta_project;
    }
  }
  for (int l = 0; l < kNumTileLists; ++l) {
    if (total_tiles[l] > (1 << 28)) { *st = FIRA_ERR_SHAPE; *why = "too many tiles"; return false; }
    plan->max_tiles[l] = (int)total_tiles[l];
  }
  plan->off_partial = off;
  off = align_up(off + (size_t)(total_tiles[kTilesBackBf16] + total_tiles[kTilesBackF32]) * 4);
  long long max_S = 0;
  for (const HostMat& h : plan->mats) max_S = std::max<long long>(max_S, h.dev.S);
  long long max_r = 0;
  for (const HostMat& h : plan->mats) max_r = std::max<long long>(max_r, h.dev.r);
  plan->off_ortho = off;   // scratch of the orthonormality estimate: S x 4 floats, then splits x r x 4 floats
  plan->ortho_z = align_up((size_t)max_S * 16);
  // fira_set_projectors estimates up to kInstallBatch matrices per launch, each in a piece of its own ([S][4]
  // directly followed by [splits][r][4]); fira_set_projector uses the first piece
  plan->ortho_slot = align_up(plan->ortho_z + (size_t)FIRA_ORTHO_SPLITS * max_r * 16);
  off = align_up(off + plan->ortho_slot * (size_t)std::min(count, kInstallBatch));
  plan->off_install = off;
  off = align_up(off + sizeof(FiraRefreshEnt) * (size_t)count);
  plan->off_dyn = off;     // values that the kernels read at run time: [0] lr * alpha
  off = align_up(off + 64);
  size_t s = 0;
  s = align_up(s + sizeof(FiraEnt) * count);
  for (int l = 0; l < kNumTileLists; ++l) {
    plan->slot_off_tiles[l] = s;
    s = align_up(s + sizeof(FiraTile) * (size_t)total_tiles[l]);
  }
  plan->slot_bytes = s;
  plan->off_slots = off; off += s * kSlots;
  plan->total = off;
  return true;
}

// The work list of one fira_step call over matrices idx[0..count) with weights W and gradients G, written into
// `stage` (Plan::slot_bytes bytes: the entries, then the tile lists at Plan::slot_off_tiles).  ntiles[l] =
// tiles written to list l.
void build_work_list(const Plan& p, int count, const int* idx, void* const* W, const void* const* G, char* stage,
                     int (&ntiles)[kNumTileLists], int* rowblocks_out, int* g2blocks_out) {
  FiraEnt* ents = reinterpret_cast<FiraEnt*>(stage);
  FiraTile* tl[kNumTileLists];
  int nt[kNumTileLists] = {};
  for (int l = 0; l < kNumTileLists; ++l) tl[l] = reinterpret_cast<FiraTile*>(stage + p.slot_off_tiles[l]);
  int nparts = 0, rowblocks = 0, g2blocks = 0;
  for (int e = 0; e < count; ++e) {
    const HostMat& h = p.mats[idx[e]];
    FiraEnt& en = ents[e];
    en.mat = idx[e]; en.part0 = nparts; en.npart = h.tiles_back; en.row0 = rowblocks; en.g2b0 = g2blocks; en.pad = 0;
    en.W = W[e]; en.G = G[e];
    rowblocks += h.rowblocks;
    g2blocks += h.g2blocks;
    // R contraction: rank tiles innermost, so the tiles that share a panel of G are neighbours
    const int lp = h.dev.left ? kTilesProjectLeft : kTilesProjectRight;
    for (int ta = 0; ta < h.ta_project; ++ta)
      for (int tbb = 0; tbb < h.tb_project; ++tbb) tl[lp][nt[lp]++] = FiraTile{e, ta, tbb, 0};
    const int ls = (h.small_proj ? kTilesProjSmallLeft : kTilesProjBigLeft) + (h.dev.left ? 0 : 1);
    for (int ta = 0; ta < h.ta_project; ++ta)
      for (int tbb = 0; tbb < h.tb_project; ++tbb) tl[ls][nt[ls]++] = FiraTile{e, ta, tbb, 0};
    if (h.fuse_list >= 0)
      for (int ta = 0; ta < h.ta_project; ++ta) tl[h.fuse_list][nt[h.fuse_list]++] = FiraTile{e, ta, 0, 0};
    // back-projection: groups of 8 column tiles x all row tiles keep both operand panels in L2
    const int lb = h.dev.dtype == FIRA_BF16 ? kTilesBackBf16 : kTilesBackF32;
    const int grp = 8;
    for (int ta0 = 0; ta0 < h.ta_back; ta0 += grp)
      for (int t2 = 0; t2 < h.tb_back; ++t2)
        for (int ta = ta0; ta < std::min(ta0 + grp, h.ta_back); ++ta) tl[lb][nt[lb]++] = FiraTile{e, ta, t2, nparts++};
  }
  for (int l = 0; l < kNumTileLists; ++l) ntiles[l] = nt[l];
  *rowblocks_out = rowblocks;
  *g2blocks_out = g2blocks;
}

struct RefreshPlan {
  size_t total = 0;
  size_t off_ents = 0, off_ents2 = 0, off_vmats = 0, off_vents = 0, off_vtiles[2] = {0, 0};
  size_t off_done = 0;                    // one int per listed matrix: the second pass found its input orthonormal
  int ntiles[2] = {0, 0};                 // virtual launches: [0] K-contiguous (real left), [1] K-slow (real right)
  std::vector<size_t> off_top, off_y, off_q, off_c, off_linv;
  std::vector<size_t> off_gb;             // fp32 matrices: bf16 rounding of the gradient, rows of gb_ld elements (else unused)
  size_t top_begin = 0, top_end = 0;
};

// Row pitch (elements) of the bf16 rounding of an fp32 gradient that the refresh's way back reads.
inline int refresh_gb_ld(int n) { return round_up_int(n, 8); }

bool make_refresh_plan(const Plan& plan, int count, const int* idx, RefreshPlan* rp) {
  const int nmat = (int)plan.mats.size();
  if (count < 1 || count > nmat || !idx) return false;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  rp->off_ents = take(sizeof(FiraRefreshEnt) * count);
  rp->off_ents2 = take(sizeof(FiraRefreshEnt) * count);
  rp->off_vmats = take(sizeof(FiraMat) * count);
  rp->off_vents = take(sizeof(FiraEnt) * count);
  rp->off_done = take(sizeof(int) * (size_t)count);
  rp->ntiles[0] = rp->ntiles[1] = 0;
  for (int e = 0; e < count; ++e) {
    if (idx[e] < 0 || idx[e] >= nmat) return false;
    const FiraMat& m = plan.mats[idx[e]].dev;
    rp->ntiles[m.left ? 0 : 1] += ((m.S + FIRA_PA - 1) / FIRA_PA) * ((m.r + FIRA_PB - 1) / FIRA_PB);
  }
  rp->off_vtiles[0] = take(sizeof(FiraTile) * std::max(rp->ntiles[0], 1));
  rp->off_vtiles[1] = take(sizeof(FiraTile) * std::max(rp->ntiles[1], 1));
  rp->off_gb.assign(count, 0);
  rp->off_top.resize(count); rp->off_y.resize(count); rp->off_q.resize(count); rp->off_c.resize(count); rp->off_linv.resize(count);
  rp->top_begin = off;
  for (int e = 0; e < count; ++e) {
    const FiraMat& m = plan.mats[idx[e]].dev;
    rp->off_top[e] = take((size_t)round_up_int(m.L, 64) * m.rq * 2);
  }
  rp->top_end = off;
  for (int e = 0; e < count; ++e) {
    const FiraMat& m = plan.mats[idx[e]].dev;
    rp->off_y[e] = take((size_t)m.S * m.r * 4);
    rp->off_q[e] = take((size_t)m.S * m.r * 4);
    rp->off_c[e] = take((size_t)m.r * m.r * 8);
    // scratch of the gate estimate, which before that holds the inverses of the solve's diagonal blocks
    rp->off_linv[e] = take(std::max((size_t)m.S * 16 + (size_t)FIRA_ORTHO_SPLITS * m.r * 16,
                                    (size_t)((m.r + FIRA_SOLVE_JB - 1) / FIRA_SOLVE_JB) * FIRA_SOLVE_JB * FIRA_SOLVE_JB * 8));
    if (m.kx != 1) rp->off_gb[e] = take((size_t)m.m * refresh_gb_ld(m.n) * 2);
  }
  rp->total = off;
  return true;
}

}  // namespace
