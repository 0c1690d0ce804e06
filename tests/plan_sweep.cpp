// CPU check of the host-side work lists (paper_1809_11165_amd/csrc/bbmm_plan.h): over a sweep of
// problem sizes, compute-unit counts and workgroup counts, every (column strip, 16-row step) of the
// matrix must be dealt out exactly once, every piece must lie inside the matrix, and every
// partial-result slot must be in range and used once.  Built by tests/test_plans_cpu.py with
// -fsanitize=address,undefined, so an out-of-range index in the builders themselves stops the run.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <utility>

#include "bbmm_plan.h"

using namespace bbmm_plan;

static long long checks = 0;

#define REQUIRE(cond, ...)                         \
  do {                                             \
    if (!(cond)) {                                 \
      std::fprintf(stderr, "FAILED %s: ", #cond);  \
      std::fprintf(stderr, __VA_ARGS__);           \
      std::fprintf(stderr, "\n");                  \
      std::exit(1);                                \
    }                                              \
    ++checks;                                      \
  } while (0)

static void check_rect(int rows_p, int cols_p, int ld, int wgs, int slot_cap) {
  std::vector<MmPlan> plan;
  std::vector<int> nseg;
  const char* what = lay_out_plan(rows_p, cols_p, ld, wgs, slot_cap, plan, nseg);
  REQUIRE(what == nullptr, "%s (rows %d cols %d ld %d wgs %d cap %d)", what, rows_p, cols_p, ld, wgs, slot_cap);
  int cols_per_wg = ld == 32 ? 512 : 1024;
  int strips = (cols_p + cols_per_wg - 1) / cols_per_wg, steps = rows_p / 16;
  REQUIRE((int)plan.size() == wgs && (int)nseg.size() == strips, "sizes");
  std::vector<std::vector<char>> seen((size_t)strips, std::vector<char>((size_t)steps, 0));
  std::vector<std::set<int>> slots((size_t)strips);
  for (const MmPlan& p : plan)
    for (const MmPiece& q : p.piece) {
      if (q.row_begin == q.row_end) continue;
      REQUIRE(q.strip >= 0 && q.strip < strips, "strip %d", q.strip);
      REQUIRE(q.row_begin % 16 == 0 && q.row_end % 16 == 0 && 0 <= q.row_begin && q.row_begin < q.row_end &&
                  q.row_end <= rows_p, "rows %d..%d of %d", q.row_begin, q.row_end, rows_p);
      REQUIRE(q.slot >= 0 && q.slot < nseg[(size_t)q.strip] && q.slot < slot_cap, "slot %d", q.slot);
      REQUIRE(slots[(size_t)q.strip].insert(q.slot).second, "slot %d of strip %d used twice", q.slot, q.strip);
      for (int j = q.row_begin / 16; j < q.row_end / 16; ++j) {
        REQUIRE(!seen[(size_t)q.strip][(size_t)j], "unit (%d, %d) dealt twice", q.strip, j);
        seen[(size_t)q.strip][(size_t)j] = 1;
      }
    }
  for (int s = 0; s < strips; ++s) {
    REQUIRE((int)slots[(size_t)s].size() == nseg[(size_t)s], "strip %d: %zu slots used of %d", s, slots[(size_t)s].size(),
            nseg[(size_t)s]);
    for (int j = 0; j < steps; ++j) REQUIRE(seen[(size_t)s][(size_t)j], "unit (%d, %d) not dealt", s, j);
  }
}

static void check_triangle(int np, int W, int want) {
  TriHost L;
  const char* what = lay_out_triangle(np, W, want, L);
  REQUIRE(what == nullptr, "%s (np %d W %d want %d)", what, np, W, want);
  int S = (np + W - 1) / W;
  REQUIRE((int)L.cnt.size() == S && (int)L.tot.size() == S, "sizes");
  std::vector<std::set<int>> slots((size_t)S);
  std::map<std::pair<int, int>, int> seen;   // (panel, step) -> kind
  for (int kind = 0; kind < 2; ++kind) {
    const std::vector<int>& first = L.first[kind];
    REQUIRE((int)first.size() == L.wgs[kind] + 1 && L.wgs[kind] <= want, "first[%d]", kind);
    for (int w = 0; w < L.wgs[kind]; ++w) {
      REQUIRE(first[(size_t)w] <= first[(size_t)w + 1] && first[(size_t)w + 1] <= (int)L.pieces.size(), "ranges");
      for (int i = first[(size_t)w]; i < first[(size_t)w + 1]; ++i) {
        const MmPiece& q = L.pieces[(size_t)i];
        REQUIRE(q.strip >= 0 && q.strip < S, "panel %d", q.strip);
        int lo = kind == 0 ? 0 : q.strip * W, hi = kind == 0 ? q.strip * W : std::min(np, (q.strip + 1) * W);
        REQUIRE(q.row_begin % 16 == 0 && q.row_end % 16 == 0 && lo <= q.row_begin && q.row_begin < q.row_end &&
                    q.row_end <= hi, "kind %d panel %d rows %d..%d not in %d..%d", kind, q.strip, q.row_begin,
                q.row_end, lo, hi);
        REQUIRE(q.slot >= 0 && q.slot < L.cnt[(size_t)q.strip], "slot %d", q.slot);
        REQUIRE(slots[(size_t)q.strip].insert(q.slot).second, "slot %d of panel %d used twice", q.slot, q.strip);
        for (int j = q.row_begin / 16; j < q.row_end / 16; ++j)
          REQUIRE(seen.emplace(std::make_pair(q.strip, j), kind).second, "step (%d, %d) dealt twice", q.strip, j);
      }
    }
    if (L.wgs[kind] > 0)
      REQUIRE(first[0] == (kind == 0 ? 0 : L.first[0].back()), "lists are not back to back");
  }
  REQUIRE(L.first[1].back() == (int)L.pieces.size(), "pieces beyond the lists");
  long long want_steps = 0;
  int max_slots = 0;
  for (int P = 0; P < S; ++P) {
    want_steps += (std::min(np, (P + 1) * W)) / 16;
    REQUIRE((int)slots[(size_t)P].size() == L.cnt[(size_t)P], "panel %d slots", P);
    REQUIRE(L.tot[(size_t)P] == L.cnt[(size_t)P] + (S - 1 - P), "tot[%d]", P);
    max_slots = std::max(max_slots, L.tot[(size_t)P]);
  }
  REQUIRE((long long)seen.size() == want_steps, "%zu steps dealt of %lld", seen.size(), want_steps);
  REQUIRE(max_slots == L.max_slots, "max_slots");
}

int main() {
  const int cus[] = {256, 304, 8};
  std::vector<int> sizes;
  for (int np = 256; np <= 4096; np += 256) sizes.push_back(np);
  for (int np : {5120, 8192, 10240, 12288, 20224, 30208, 50176, 65536, 100096, 200192, 500224}) sizes.push_back(np);
  for (int num_cus : cus)
    for (int np : sizes) {
      if (np > 70000 && num_cus != 256) continue;
      // materialised product of the np x np matrix: default and tuned workgroup counts
      for (int ld : {16, 32})
        for (int narrow = 0; narrow < 2; ++narrow)
          for (long long tuned : {0LL, 1LL, 7LL, 245LL, 1000LL, 100000LL}) {
            if (np > 30000 && tuned != 0 && tuned != 245) continue;
            int wgs = mat_wgs_of(np, num_cus, tuned, ld, narrow != 0);
            check_rect(np, np, ld, wgs, kMaxSplit);
          }
      // row chunks of the on-the-fly product
      int strips = (np / 16 + 31) / 32;
      int ns = std::min(split_by_fill(np, num_cus, strips, 4 * num_cus, 0.97), std::max(1, np / 64));
      REQUIRE(ns >= 1 && ns <= kMaxSplit && ns <= np / 16, "otf split %d at np %d", ns, np);
      // triangle lists: stored triangle (panels of 1024) and on-the-fly (panels of 512)
      {
        for (int want : {num_cus, 2 * num_cus, 1, 3, 1000}) {
          if (np > 30000 && want != num_cus && want != 2 * num_cus) continue;
          check_triangle(np, 1024, want);
          check_triangle(np, 512, want);
        }
      }
      // the two streaming products of the SGPR root (np x mp and mp x np)
      for (int mp : {256, 1024, 4096})
        for (int ld : {16, 32})
          for (long long tuned : {0LL, 5LL, 489LL}) {
            if (np > 30000 && (mp != 1024 || tuned == 5)) continue;
            check_rect(np, mp, ld, rect_wgs_of(num_cus, np, mp, ld, 1024, tuned), 1024);
            check_rect(mp, np, ld, rect_wgs_of(num_cus, mp, np, ld, kMaxSplit, tuned), kMaxSplit);
          }
    }
  std::printf("OK %lld checks\n", checks);
  return 0;
}
