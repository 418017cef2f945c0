// Host-only check of the library's planning code (csrc/fira_plan.h), built by tests/test_host_plan.py with
// the address and undefined-behaviour sanitizers and run on the CPU: random lists of matrix descriptors go
// through make_plan, build_work_list and make_refresh_plan, and every piece of the slab, of a work-list slot
// and of the refresh workspace must be aligned, inside the total and disjoint from every other piece; the
// tile lists must cover every matrix's tile grid exactly once.  The work list is written into a heap block
// of exactly Plan::slot_bytes, so that a write past its end is an AddressSanitizer error.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <set>
#include <tuple>
#include <vector>

#include "../paper_2410_01623_amd/csrc/fira_plan.h"

namespace {

int failures = 0;
#define CHECK(cond, ...)                                                   \
  do {                                                                     \
    if (!(cond)) {                                                         \
      if (++failures <= 20) { std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); } \
    }                                                                      \
  } while (0)

struct Piece { size_t off, bytes; const char* what; int mat; };

void check_pieces(std::vector<Piece> pieces, size_t total, const char* where) {
  std::sort(pieces.begin(), pieces.end(), [](const Piece& a, const Piece& b) { return a.off < b.off; });
  for (size_t i = 0; i < pieces.size(); ++i) {
    const Piece& p = pieces[i];
    CHECK(p.off % 256 == 0, "%s: %s of matrix %d is not 256-byte aligned (offset %zu)", where, p.what, p.mat, p.off);
    CHECK(p.off + p.bytes <= total, "%s: %s of matrix %d ends at %zu beyond the total %zu", where, p.what, p.mat, p.off + p.bytes, total);
    if (i + 1 < pieces.size())
      CHECK(p.off + p.bytes <= pieces[i + 1].off, "%s: %s of matrix %d [%zu, %zu) overlaps %s of matrix %d at %zu", where, p.what, p.mat,
            p.off, p.off + p.bytes, pieces[i + 1].what, pieces[i + 1].mat, pieces[i + 1].off);
  }
}

fira_matrix_desc random_desc(std::mt19937_64& rng, bool big) {
  auto pick = [&](long long lo, long long hi) { return (long long)(lo + rng() % (unsigned long long)(hi - lo + 1)); };
  fira_matrix_desc d;
  const int kind = (int)(rng() % 8);
  const long long cap = big ? 6000 : 700;
  d.m = pick(1, cap);
  d.n = pick(1, cap);
  if (kind == 0) d.n = d.m;                       // square
  if (kind == 1) { d.m = pick(1, 40); }            // very short
  if (kind == 2) { d.n |= 1; }                     // odd n
  const long long S = std::min(d.m, d.n);
  switch (rng() % 6) {
    case 0: d.r = 1; break;
    case 1: d.r = (int)S; break;                   // full rank
    case 2: d.r = (int)std::min<long long>(S, 4 * pick(1, 260)); break;   // multiples of 4 (register-resident Adam rows, fused kernel)
    case 3: d.r = (int)std::min<long long>(S, 128 * pick(1, 8)); break;
    default: d.r = (int)pick(1, S); break;
  }
  d.ld = d.n + ((rng() % 3 == 0) ? pick(0, 37) : 0);
  d.wg_dtype = (rng() % 4 == 0) ? FIRA_F32 : FIRA_BF16;
  return d;
}

void check_plan(const std::vector<fira_matrix_desc>& descs, std::mt19937_64& rng) {
  const int count = (int)descs.size();
  Plan plan;
  fira_status st = FIRA_OK;
  std::string why;
  if (!make_plan(descs.data(), count, &plan, &st, &why)) {
    CHECK(false, "make_plan rejected a valid list: %s", why.c_str());
    return;
  }
  // ---- the slab
  std::vector<Piece> pieces;
  pieces.push_back({plan.off_mats, sizeof(FiraMat) * (size_t)count, "matrix table", -1});
  pieces.push_back({plan.off_scal, sizeof(FiraScal) * (size_t)count, "scalar table", -1});
  size_t parts = 0;
  long long max_S = 0, max_r = 0;
  for (int i = 0; i < count; ++i) {
    const HostMat& h = plan.mats[i];
    const FiraMat& m = h.dev;
    CHECK(m.m == descs[i].m && m.n == descs[i].n && m.r == descs[i].r && m.ld == descs[i].ld, "matrix %d: description not copied", i);
    CHECK(m.L == std::max(m.m, m.n) && m.S == std::min(m.m, m.n) && m.left == (m.m <= m.n), "matrix %d: sides", i);
    CHECK(m.rp % 64 == 0 && m.rp >= m.r && m.rp < m.r + 64 && m.Sp % 64 == 0 && m.Sp >= m.S && m.Sp < m.S + 64, "matrix %d: padded sizes", i);
    CHECK(m.Lq % 256 == 0 && m.Lq >= m.L && m.Sq % 256 == 0 && m.Sq >= m.S && m.rq % 256 == 0 && m.rq >= m.r, "matrix %d: tile-padded rows", i);
    CHECK(m.kx == (m.dtype == FIRA_F32 ? FIRA_KX_SPLIT : 1), "matrix %d: K expansion", i);
    const size_t Lr = (size_t)m.L * m.r;
    pieces.push_back({(size_t)m.M, Lr * 4, "M", i});
    pieces.push_back({(size_t)m.V, Lr * 4, "V", i});
    pieces.push_back({(size_t)m.Rt, Lr * 4, "Rt", i});
    pieces.push_back({(size_t)m.phi, (size_t)m.L * 4, "phi", i});
    pieces.push_back({(size_t)m.g2, (size_t)m.L * 4, "g2", i});
    pieces.push_back({(size_t)m.q, (size_t)m.L * 4, "q", i});
    // operands: whole tiles of rows (what the ring loaders of the contraction kernels fetch), K padded to 64
    pieces.push_back({(size_t)m.Nb, (size_t)m.Lq * m.kx * m.rp * 2, "Nb", i});
    pieces.push_back({(size_t)m.Rb, (size_t)m.Lq * m.kx * m.rp * 2, "Rb", i});
    pieces.push_back({(size_t)m.Pn, (size_t)m.Sq * m.kx * m.rp * 2, "Pn", i});
    pieces.push_back({(size_t)m.PT, (size_t)m.rq * m.kx * m.Sp * 2, "PT", i});
    if (m.kx > 1) {
      CHECK(m.gx_ld >= (m.left ? m.n : (long long)m.kx * m.Sp), "matrix %d: pitch of the split gradient", i);
      const size_t gx = m.left ? (size_t)m.kx * m.Sp * m.gx_ld : (size_t)m.m * m.gx_ld;
      pieces.push_back({(size_t)m.Gx, gx * 2, "Gx", i});
    } else {
      CHECK(m.Gx == nullptr, "matrix %d: bf16 matrices have no split gradient", i);
    }
    CHECK(h.ta_project == (m.L + FIRA_PA - 1) / FIRA_PA && h.tb_project == (m.r + FIRA_PB - 1) / FIRA_PB, "matrix %d: projection tiles", i);
    CHECK(h.ta_back == (m.n + FIRA_BA - 1) / FIRA_BA && h.tb_back == (m.m + FIRA_BB - 1) / FIRA_BB, "matrix %d: back-projection tiles", i);
    // the last tile's operand rows must exist (zero padding): rows are padded to whole tiles
    CHECK((long long)h.tb_project * FIRA_PB <= m.rq, "matrix %d: PT rows do not cover the last rank tile", i);
    CHECK((long long)h.ta_back * FIRA_BA <= (m.left ? m.Lq : m.Sq) && (long long)h.tb_back * FIRA_BB <= (m.left ? m.Sq : m.Lq),
          "matrix %d: operand rows do not cover the last back-projection tile", i);
    if (h.fuse_list >= 0) CHECK(m.kx == 1 && m.r % 4 == 0 && m.r >= FIRA_FUSE_MIN_R && m.r <= FIRA_FUSE_MAX_R, "matrix %d: not eligible for the fused kernel", i);
    parts += (size_t)h.tiles_back;
    max_S = std::max<long long>(max_S, m.S);
    max_r = std::max<long long>(max_r, m.r);
  }
  pieces.push_back({plan.off_partial, parts * 4, "tile partials", -1});
  pieces.push_back({plan.off_ortho, (size_t)max_S * 16, "orthonormality estimate y", -1});
  pieces.push_back({plan.off_ortho + plan.ortho_z, (size_t)FIRA_ORTHO_SPLITS * max_r * 16, "orthonormality estimate z", -1});
  // the batched installation's pieces: one per matrix of a batch, [S][4] directly followed by [splits][r][4]
  for (int k = 1; k < std::min(count, kInstallBatch); ++k)
    pieces.push_back({plan.off_ortho + plan.ortho_slot * k, (size_t)max_S * 16 + (size_t)FIRA_ORTHO_SPLITS * max_r * 16,
                      "orthonormality estimate of a batch", k});
  CHECK(plan.ortho_slot >= plan.ortho_z + (size_t)FIRA_ORTHO_SPLITS * max_r * 16, "a batch piece is smaller than the single estimate's");
  pieces.push_back({plan.off_install, sizeof(FiraRefreshEnt) * (size_t)count, "installation table", -1});
  pieces.push_back({plan.off_dyn, 4, "step size", -1});
  for (int k = 0; k < kSlots; ++k) pieces.push_back({plan.off_slots + plan.slot_bytes * k, plan.slot_bytes, "work-list slot", k});
  check_pieces(pieces, plan.total, "slab");

  // ---- a step's work list over a random subset, in random order, in a block of exactly slot_bytes
  std::vector<int> idx(count);
  for (int i = 0; i < count; ++i) idx[i] = i;
  std::shuffle(idx.begin(), idx.end(), rng);
  const int listed = 1 + (int)(rng() % (unsigned)count);
  idx.resize(listed);
  std::vector<void*> W(listed);
  std::vector<const void*> G(listed);
  for (int e = 0; e < listed; ++e) { W[e] = (void*)(uintptr_t)(0x1000 + 16 * e); G[e] = (const void*)(uintptr_t)(0x2000 + 16 * e); }
#ifdef FIRA_PLAN_CHECK_SHORT_STAGE   // planted mistake for the test of this check: the block is too small
  char* stage = (char*)std::malloc(plan.slot_bytes / 8 + 1);
#else
  char* stage = (char*)std::malloc(plan.slot_bytes ? plan.slot_bytes : 1);
#endif
  int ntiles[kNumTileLists] = {};
  int rowblocks = 0, g2blocks = 0;
  build_work_list(plan, listed, idx.data(), W.data(), G.data(), stage, ntiles, &rowblocks, &g2blocks);
  std::vector<Piece> sp;
  sp.push_back({0, sizeof(FiraEnt) * (size_t)listed, "entries", -1});
  for (int l = 0; l < kNumTileLists; ++l) {
    CHECK(ntiles[l] <= plan.max_tiles[l], "tile list %d holds %d tiles, the plan allows %d", l, ntiles[l], plan.max_tiles[l]);
    sp.push_back({plan.slot_off_tiles[l], sizeof(FiraTile) * (size_t)ntiles[l], "tile list", l});
  }
  check_pieces(sp, plan.slot_bytes, "work-list slot");
  const FiraEnt* ents = reinterpret_cast<const FiraEnt*>(stage);
  int rb = 0, g2b = 0, np = 0;
  for (int e = 0; e < listed; ++e) {
    const HostMat& h = plan.mats[idx[e]];
    CHECK(ents[e].mat == idx[e] && ents[e].W == W[e] && ents[e].G == G[e], "entry %d", e);
    CHECK(ents[e].row0 == rb && ents[e].g2b0 == g2b && ents[e].part0 == np && ents[e].npart == h.tiles_back, "entry %d: prefix sums", e);
    rb += h.rowblocks; g2b += h.g2blocks; np += h.tiles_back;
  }
  CHECK(rb == rowblocks && g2b == g2blocks, "row-block totals");
  // coverage: every (entry, ta, tb) of each grid exactly once; partial slots unique and inside the entry's range
  for (int l = 0; l < kNumTileLists; ++l) {
    const FiraTile* tl = reinterpret_cast<const FiraTile*>(stage + plan.slot_off_tiles[l]);
    std::set<std::tuple<int, int, int>> seen;
    std::set<int> slots;
    for (int k = 0; k < ntiles[l]; ++k) {
      const FiraTile& t = tl[k];
      CHECK(t.ent >= 0 && t.ent < listed, "list %d tile %d: entry out of range", l, k);
      if (t.ent < 0 || t.ent >= listed) continue;
      const HostMat& h = plan.mats[idx[t.ent]];
      const bool back = l == kTilesBackBf16 || l == kTilesBackF32;
      const bool fuse = l >= kTilesFuse && l < kTilesFuse + 4;
      const int na = back ? h.ta_back : h.ta_project, nb = back ? h.tb_back : (fuse ? 1 : h.tb_project);
      CHECK(t.ta >= 0 && t.ta < na && t.tb >= 0 && t.tb < nb, "list %d tile %d: (%d, %d) outside the %d x %d grid", l, k, t.ta, t.tb, na, nb);
      CHECK(seen.insert(std::make_tuple(t.ent, t.ta, t.tb)).second, "list %d: tile (%d, %d, %d) listed twice", l, t.ent, t.ta, t.tb);
      if (back) {
        CHECK(t.part >= ents[t.ent].part0 && t.part < ents[t.ent].part0 + ents[t.ent].npart, "list %d tile %d: partial slot outside its entry", l, k);
        CHECK(slots.insert(t.part).second, "list %d: partial slot %d used twice", l, t.part);
      }
    }
  }
  {
    long long want[kNumTileLists] = {};
    for (int e = 0; e < listed; ++e) {
      const HostMat& h = plan.mats[idx[e]];
      want[h.dev.left ? kTilesProjectLeft : kTilesProjectRight] += h.tiles_project;
      want[(h.small_proj ? kTilesProjSmallLeft : kTilesProjBigLeft) + (h.dev.left ? 0 : 1)] += h.tiles_project;
      want[h.dev.dtype == FIRA_BF16 ? kTilesBackBf16 : kTilesBackF32] += h.tiles_back;
      if (h.fuse_list >= 0) want[h.fuse_list] += h.ta_project;
    }
    for (int l = 0; l < kNumTileLists; ++l) CHECK(want[l] == ntiles[l], "list %d: %d tiles, expected %lld", l, ntiles[l], want[l]);
  }
  std::free(stage);

  // ---- the refresh workspace for the listed bf16 matrices
  std::vector<int> ridx;
  for (int e = 0; e < listed; ++e)
    if (plan.mats[idx[e]].dev.kx == 1) ridx.push_back(idx[e]);
  if (!ridx.empty()) {
    RefreshPlan rp;
    CHECK(make_refresh_plan(plan, (int)ridx.size(), ridx.data(), &rp), "make_refresh_plan rejected a valid list");
    std::vector<Piece> wp;
    const int rc = (int)ridx.size();
    wp.push_back({rp.off_ents, sizeof(FiraRefreshEnt) * (size_t)rc, "refresh entries", -1});
    wp.push_back({rp.off_ents2, sizeof(FiraRefreshEnt) * (size_t)rc, "refresh entries 2", -1});
    wp.push_back({rp.off_vmats, sizeof(FiraMat) * (size_t)rc, "virtual matrices", -1});
    wp.push_back({rp.off_vents, sizeof(FiraEnt) * (size_t)rc, "virtual entries", -1});
    wp.push_back({rp.off_done, sizeof(int) * (size_t)rc, "second-pass flags", -1});
    wp.push_back({rp.off_vtiles[0], sizeof(FiraTile) * (size_t)std::max(rp.ntiles[0], 1), "virtual tiles 0", -1});
    wp.push_back({rp.off_vtiles[1], sizeof(FiraTile) * (size_t)std::max(rp.ntiles[1], 1), "virtual tiles 1", -1});
    for (int e = 0; e < rc; ++e) {
      const FiraMat& m = plan.mats[ridx[e]].dev;
      const size_t Lp = (size_t)round_up_int(m.L, 64);
      wp.push_back({rp.off_top[e], Lp * m.rq * 2, "packed operand", ridx[e]});
      wp.push_back({rp.off_y[e], (size_t)m.S * m.r * 4, "Y", ridx[e]});
      wp.push_back({rp.off_q[e], (size_t)m.S * m.r * 4, "Q", ridx[e]});
      wp.push_back({rp.off_c[e], (size_t)m.r * m.r * 8, "C", ridx[e]});
      const size_t inst = std::max((size_t)m.S * 16 + (size_t)FIRA_ORTHO_SPLITS * m.r * 16,
                                   (size_t)((m.r + FIRA_SOLVE_JB - 1) / FIRA_SOLVE_JB) * FIRA_SOLVE_JB * FIRA_SOLVE_JB * 8);
      wp.push_back({rp.off_linv[e], inst, "block inverses / gate scratch", ridx[e]});
      if (m.kx != 1) wp.push_back({rp.off_gb[e], (size_t)m.m * refresh_gb_ld(m.n) * 2, "bf16 rounding of the gradient", ridx[e]});
      CHECK(rp.off_top[e] >= rp.top_begin && rp.off_top[e] + Lp * m.rq * 2 <= rp.top_end, "packed operand outside the cleared range");
    }
    check_pieces(wp, rp.total, "refresh workspace");
    CHECK((rp.top_end - rp.top_begin) % 16 == 0, "cleared range is not a whole number of 16-byte pieces");
  }
}

}  // namespace

int main(int argc, char** argv) {
  const int rounds = argc > 1 ? std::atoi(argv[1]) : 300;
  std::mt19937_64 rng(20241001);
  long long lists = 0, matrices = 0;
  for (int round = 0; round < rounds; ++round) {
    int count = 1 + (int)(rng() % 12);
    if (round % 37 == 0) count = 1024;                // many matrices
    if (round % 50 == 1) count = 1;
    std::vector<fira_matrix_desc> descs(count);
    const bool big = count <= 12 && round % 5 == 0;
    for (auto& d : descs) d = random_desc(rng, big);
    check_plan(descs, rng);
    ++lists; matrices += count;
  }
  // the shapes of the paper's LLaMA table that the workloads use (1B, r = 512; 7B, r = 1024)
  for (int cfg = 0; cfg < 2; ++cfg) {
    const long long d = cfg ? 4096 : 2048, f = cfg ? 11008 : 5461;
    const int r = cfg ? 1024 : 512, blocks = cfg ? 32 : 24;
    std::vector<fira_matrix_desc> descs;
    for (int b = 0; b < blocks; ++b) {
      for (int k = 0; k < 4; ++k) descs.push_back({d, d, d, r, FIRA_BF16});
      for (int k = 0; k < 2; ++k) descs.push_back({d, f, f, r, FIRA_BF16});
      descs.push_back({f, d, d, r, FIRA_BF16});
    }
    check_plan(descs, rng);
    ++lists; matrices += (long long)descs.size();
  }
  // descriptors that must be rejected
  {
    Plan plan; fira_status st; std::string why;
    const fira_matrix_desc bad[] = {{0, 5, 5, 1, FIRA_BF16}, {5, 0, 0, 1, FIRA_BF16}, {8, 8, 8, 9, FIRA_BF16}, {8, 8, 8, 0, FIRA_BF16},
                                    {8, 8, 7, 4, FIRA_BF16}, {8, 8, 8, 4, 7}, {(1 << 22) + 1, 8, 8, 4, FIRA_BF16}};
    for (const fira_matrix_desc& b : bad) {
      Plan p2;
      CHECK(!make_plan(&b, 1, &p2, &st, &why), "an invalid descriptor (m %lld n %lld ld %lld r %d dtype %d) was accepted", (long long)b.m,
            (long long)b.n, (long long)b.ld, b.r, b.wg_dtype);
    }
    const fira_matrix_desc ok = {8, 8, 8, 4, FIRA_BF16};
    CHECK(!make_plan(nullptr, 1, &plan, &st, &why) && !make_plan(&ok, 0, &plan, &st, &why), "a null or empty list was accepted");
  }
  std::printf("%lld lists, %lld matrices checked, %d failure(s)\n", lists, matrices, failures);
  return failures ? 1 : 0;
}
