// Host-side work lists of the streaming products: which workgroup walks which rows of which
// column strip, and into which partial-result slot.  Plain C++ (no HIP), so that the same code the
// library runs can be compiled for the CPU with sanitizers and swept over sizes.
#pragma once

#include <algorithm>
#include <vector>

// Work of one workgroup of the materialised product: up to BBMM_MM_PIECES pieces, each a run of
// matrix rows [row_begin, row_end) (multiples of 16) inside one strip of output columns, whose
// partial result goes to slot `slot` of that strip.  An unused piece has row_begin == row_end.
#define BBMM_MM_PIECES 4
struct MmPiece {
  int strip, row_begin, row_end, slot;
};
struct MmPlan {
  MmPiece piece[BBMM_MM_PIECES];
};

namespace bbmm_plan {

constexpr int kMaxSplit = 64;   // partial-result slots per column strip of the exact-GP products

// Row chunks of a kernel whose workgroups each take one strip of columns and one chunk of rows:
// the smallest count from `want_wgs` workgroups up for which strips * chunks fills whole rounds of
// num_cus workgroups to `min_fill` (else the best filling seen).  Fewer chunks mean fewer partial
// results to add afterwards; a last round in which only some compute units have work is what
// costs time.
inline int split_by_fill(int np, int num_cus, int strips, int want_wgs, double min_fill) {
  int cap = std::min(kMaxSplit, np / 16);
  int s0 = std::max(1, std::min(cap, (want_wgs + strips - 1) / strips));
  int best = s0;
  double best_fill = 0.0;
  for (int s = s0; s <= cap; ++s) {
    int wgs = strips * s;
    int rounds = (wgs + num_cus - 1) / num_cus;
    double fill = (double)wgs / ((double)rounds * num_cus);
    if (fill > best_fill + 1e-12) {
      best_fill = fill;
      best = s;
    }
    if (fill >= min_fill) break;
  }
  return best;
}

// Workgroups of the materialised product of an np x np matrix (tuned: "mat_wgs", 0 = default).
// The kernel keeps its own loads in flight, so one workgroup per compute unit already saturates
// that unit's share of HBM; the plan deals the (strip, row step) units out evenly, so whole rounds
// of num_cus workgroups leave no tail.  Bounds: at least one workgroup per strip (a run then spans
// at most two strips), at most kMaxSplit partial slots per strip (checked when the plan is laid
// out), at most one workgroup per unit.
inline int mat_wgs_of(int np, int num_cus, long long tuned, int ld, bool narrow) {
  int cols_per_wg = (ld == 16) ? 1024 : 512;
  int strips = (np + cols_per_wg - 1) / cols_per_wg;
  long long units = (long long)strips * (np / 16);
  long long w = (tuned > 0) ? tuned : (long long)num_cus * ((strips + num_cus - 1) / num_cus);
  if (tuned <= 0 && narrow && strips <= num_cus) {
    // (Blocks of at most 12 columns only, whose product is the most memory-bound.  With 13..16
    // columns one workgroup per unit is 1-5 % faster again, and the 32-column product is bound by the
    // fp64 matrix pipe and wants every unit: 2.38 ms on 256 workgroups against 3.07 ms on 196 at
    // n = 50 000.)
    // Measured (n = 5 000 ... 50 000): a whole number of workgroups per strip (no run crosses a strip
    // boundary and pays two prologues) beats one workgroup per unit by 2 % at n = 50 000 and by
    // 5-11 % below it, where short runs do best on about 0.8 of the units; a matrix of a few
    // thousand rows does best with at least six 16-row steps per workgroup (n = 1 000, 2 500).
    int steps = np / 16;
    int per = std::max(1, (int)(0.8 * num_cus / strips + 0.5));
    if (steps / per >= 512) per = num_cus / strips;
    bool enough = (long long)per * strips * 4 >= (long long)num_cus * 3;
    int cap = std::max(1, steps / 6);
    if (per > cap) {
      per = cap;
      enough = true;
    }
    if (enough) w = (long long)per * strips;
  }
  w = std::min<long long>(w, (long long)(kMaxSplit - 4) * strips);
  w = std::min<long long>(w, units);
  w = std::max<long long>(w, strips);
  return (int)w;
}

// Workgroups for streaming a rows_p x cols_p matrix.  With at least one column strip per compute
// unit every workgroup takes one whole strip: a piece that ends inside a strip costs a pipeline
// drain, a partial result to store and one more to add later (measured at 1024 x 500,224: 373 us
// with 256 balanced runs of ~3 pieces, 320 us with 489 whole strips).  Otherwise whole rounds of
// num_cus balanced runs, never more than there are units.
inline int rect_wgs_of(int num_cus, int rows_p, int cols_p, int ld, int slot_cap, long long tuned) {
  int cols_per_wg = (ld == 32) ? 512 : 1024;
  int strips = (cols_p + cols_per_wg - 1) / cols_per_wg;
  long long units = (long long)strips * (rows_p / 16);
  long long w = (strips >= num_cus) ? strips : num_cus;
  if (tuned > 0) w = tuned;
  w = std::min<long long>(w, (long long)(slot_cap - 4) * strips);
  w = std::min<long long>(w, units);
  w = std::max<long long>(w, std::min<long long>(units, (strips + 1) / 2));
  return (int)std::max<long long>(w, 1);
}

// One plan: the units (strip of output columns, 16-row step) of a rows_p x cols_p matrix, in
// strip-major order, are dealt to `wgs` workgroups in equal contiguous runs; a run that crosses
// strip boundaries becomes several pieces, each with its own partial slot in its strip.
// Everything the kernel relies on (rows inside the matrix, slot below slot_cap, at most
// BBMM_MM_PIECES pieces) is checked here.  Returns NULL, or what is wrong.
inline const char* lay_out_plan(int rows_p, int cols_p, int ld, int wgs, int slot_cap, std::vector<MmPlan>& plan,
                                std::vector<int>& nseg) {
  int cols_per_wg = (ld == 32) ? 512 : 1024;
  int strips = (cols_p + cols_per_wg - 1) / cols_per_wg;
  int steps = rows_p / 16;
  long long units = (long long)strips * steps;
  if (wgs < 1 || steps < 1) return "internal: product plan without work";
  plan.assign((size_t)wgs, MmPlan{});
  nseg.assign((size_t)strips, 0);
  for (int w = 0; w < wgs; ++w) {
    long long b = units * w / wgs, e = units * (w + 1) / wgs;
    for (int pc = 0; pc < BBMM_MM_PIECES; ++pc) {
      MmPiece P = {0, 0, 0, 0};
      if (b < e) {
        int strip = (int)(b / steps), jb = (int)(b % steps);
        int je = (int)std::min<long long>(steps, jb + (e - b));
        if (strip >= strips) return "internal: product plan out of range";
        P = MmPiece{strip, jb * 16, je * 16, nseg[(size_t)strip]++};
        b += je - jb;
        if (P.row_end > rows_p || P.slot >= slot_cap) return "internal: product plan out of range";
      }
      plan[(size_t)w].piece[pc] = P;
    }
    if (b < e) return "internal: product plan needs too many pieces";
  }
  return nullptr;
}

// Work lists of a product that visits only the panels (W columns each) on and above the diagonal
// of an np x np symmetric matrix.  Panel P offers P * W / 16 steps above its diagonal block, in
// which every tile is used twice, and up to W / 16 steps inside it, used once; each kind is cut
// into runs of equal length for `want` workgroups of its own list (first[kind][w] .. first[kind][w + 1]
// are workgroup w's pieces).  Output panel s then has cnt[s] column-side partial results (one per
// piece of panel s) followed by one row-side partial result from every panel right of it:
// tot[s] = cnt[s] + (S - 1 - s) slots.
struct TriHost {
  std::vector<MmPiece> pieces;
  std::vector<int> first[2], cnt, tot;
  int wgs[2] = {0, 0};
  int max_slots = 0;
};

inline const char* lay_out_triangle(int np, int W, int want, TriHost& L) {
  const int S = (np + W - 1) / W;
  struct Seg {
    int strip, row_begin, steps;
  };
  if (want < 1 || np < 16) return "internal: triangle work list without work";
  L.pieces.clear();
  L.cnt.assign((size_t)S, 0);
  for (int kind = 0; kind < 2; ++kind) {   // 0: above the diagonal blocks, 1: inside them
    std::vector<Seg> segs;
    long long total = 0;
    for (int P = 0; P < S; ++P) {
      Seg g = kind == 0 ? Seg{P, 0, P * W / 16} : Seg{P, P * W, (std::min(np, (P + 1) * W) - P * W) / 16};
      if (g.steps > 0) segs.push_back(g);
      total += g.steps;
    }
    int nw = (int)std::min<long long>(want, total);
    L.wgs[kind] = nw;
    L.first[kind].assign((size_t)nw + 1, (int)L.pieces.size());
    size_t si = 0;
    int off = 0;
    long long done = 0;
    for (int w = 0; w < nw; ++w) {
      L.first[kind][(size_t)w] = (int)L.pieces.size();
      long long target = total * (w + 1) / nw;
      while (si < segs.size() && done < target) {
        const Seg& g = segs[si];
        int take = (int)std::min<long long>(g.steps - off, target - done);
        L.pieces.push_back(MmPiece{g.strip, g.row_begin + off * 16, g.row_begin + (off + take) * 16,
                                   L.cnt[(size_t)g.strip]++});
        done += take;
        off += take;
        if (off == g.steps) {
          ++si;
          off = 0;
        }
      }
    }
    L.first[kind][(size_t)nw] = (int)L.pieces.size();
    if (si != segs.size() || done != total) return "internal: triangle work list incomplete";
  }
  L.tot.assign((size_t)S, 0);
  L.max_slots = 0;
  for (int s = 0; s < S; ++s) {
    L.tot[(size_t)s] = L.cnt[(size_t)s] + (S - 1 - s);
    L.max_slots = std::max(L.max_slots, L.tot[(size_t)s]);
  }
  return nullptr;
}

}  // namespace bbmm_plan
