// Host-side arrow decomposition: A = sum_i P_i^T B_i P_i with every B_i an
// arrow matrix of width b (diagonal blocks of b positions, plus the first
// block row and the first block column).
//
// The paper does not define this decomposition; what is implemented is the
// following peeling, repeated on the entries no earlier level has taken:
//   1. degree of a vertex = its remaining off-diagonal entries, row plus column;
//      the active vertices are those with any remaining entry (level 0: all).
//      Two vertices are adjacent when the remainder holds an entry between
//      them in either direction (the pattern of R + R^T): a directed operand
//      gets the transposed pattern built once per level, a symmetric pattern
//      (tested once, on the operand) is its own transpose at every level.
//   2. the remaining vertices are put in a linear arrangement: ascending id at
//      level 0, breadth-first order over the adjacency at later levels.
//   3. head (positions 0..b-1), one of two rules:
//        separator rule - hubs (degree > hub_factor * mean) first, then walk
//          the arrangement filling blocks of b; a vertex adjacent to a vertex
//          of an already closed block is moved to the head.  If the head does
//          not overflow, every remaining entry has an end in the head or both
//          ends in one block (the later end of an entry was either promoted or
//          placed while the earlier end's block was still open); spare head
//          positions are filled from the end of the arrangement, which moves
//          no block boundary.  The rule is accepted only after a count shows
//          that the level really takes every remaining entry.
//        plain rule - the b vertices of highest degree (ties: lower id first);
//          everything else keeps its arrangement order and is cut into blocks.
//          Inside the head (the arrow shape does not care) the hubs_first
//          highest degrees come first, by falling degree, so that the densest
//          rows and columns of the head block form its top-left corner; the
//          other head vertices follow in id order.
//   4. an entry (u,v) belongs to the level iff pos(u) < b or pos(v) < b or
//      pos(u)/b == pos(v)/b; the others form the next remainder.
// The plain rule always captures every entry of the maximum-degree vertex, in
// either direction, so each level removes at least one entry and the loop ends.
// Values are moved, never combined: every stored entry of A appears in exactly
// one level.
#include "arrow_internal.h"

#include <omp.h>

#include <algorithm>
#include <cstring>
#include <numeric>

#include "arrow.h"

namespace arrow {
namespace {

struct Remainder {
  // CSR over original vertex ids of the entries still unassigned
  const int64_t* ptr = nullptr;
  const int32_t* col = nullptr;
  const float* val = nullptr;
  std::vector<int64_t> own_ptr;
  std::vector<int32_t> own_col;
  std::vector<float> own_val;
  const uint32_t* src = nullptr;     // index of every entry in the caller's CSR arrays (NULL: identity)
  std::vector<uint32_t> own_src;
  int64_t nnz(int64_t n) const { return ptr[n]; }
};

// Is the pattern its own transpose?  Every vertex gets two 64-bit sums of a mixing function of
// its neighbours' ids, one over its row and one over its column (the latter collected with integer
// atomics, whose result does not depend on their order); the pattern is taken to be symmetric
// when the two agree for every vertex.  Equal neighbour sets always agree; different ones agree
// with probability about 2^-64.  The answer only selects how neighbours are enumerated: a wrong
// "symmetric" costs arrangement quality on that operand, never correctness (the separator rule is
// verified by a count, and the plain rule ends for any operand).
inline uint64_t mix64(uint64_t x) {
  x += 0x9e3779b97f4a7c15ULL;
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ULL;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebULL;
  return x ^ (x >> 31);
}

bool pattern_symmetric(int64_t n, const Remainder& R) {
  std::vector<uint64_t> colsum(n, 0);
  std::vector<uint64_t> rowsum(n, 0);
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t u = 0; u < n; ++u) {
    const uint64_t hu = mix64((uint64_t)u);
    uint64_t acc = 0;
    for (int64_t p = R.ptr[u]; p < R.ptr[u + 1]; ++p) {
      const int32_t w = R.col[p];
      acc += mix64((uint64_t)w);
      __atomic_fetch_add(&colsum[w], hu, __ATOMIC_RELAXED);
    }
    rowsum[u] = acc;
  }
  int64_t differ = 0;
#pragma omp parallel for schedule(static) reduction(+ : differ)
  for (int64_t u = 0; u < n; ++u) differ += rowsum[u] != colsum[u];
  return differ == 0;
}

// Neighbours of a vertex in the pattern of R + R^T.  For a symmetric pattern the rows of R are
// the whole adjacency.  Otherwise the transposed pattern (row v = the rows u that hold an entry
// (u,v)) is built from the column counts and merged, row by row, with R's: a vertex's neighbours
// are then the ascending union of both, so an operand and its transpose are arranged alike.
struct Adjacency {
  const int64_t* ptr = nullptr;
  const int32_t* col = nullptr;
  std::vector<int64_t> own_ptr;
  std::vector<int32_t> own_col;

  void build(int64_t n, const Remainder& rem, bool symmetric, const std::vector<int32_t>& colcnt) {
    if (symmetric) { ptr = rem.ptr; col = rem.col; return; }
    std::vector<int64_t> tptr(n + 1, 0);
    for (int64_t v = 0; v < n; ++v) tptr[v + 1] = tptr[v] + colcnt[v];
    std::vector<int32_t> tcol(tptr[n]);
    {
      std::vector<int64_t> fill(tptr.begin(), tptr.end() - 1);
#pragma omp parallel for schedule(dynamic, 256)
      for (int64_t u = 0; u < n; ++u)
        for (int64_t p = rem.ptr[u]; p < rem.ptr[u + 1]; ++p) {
          const int64_t at = __atomic_fetch_add(&fill[rem.col[p]], 1, __ATOMIC_RELAXED);
          tcol[at] = (int32_t)u;
        }
    }
    // the atomic fill leaves a row in arrival order; sorting makes the result deterministic
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n; ++v) std::sort(tcol.begin() + tptr[v], tcol.begin() + tptr[v + 1]);
    // union of the two sorted rows: count, prefix sum, fill
    own_ptr.assign(n + 1, 0);
    auto merge_row = [&](int64_t u, int32_t* out) -> int64_t {
      const int32_t* a = rem.col + rem.ptr[u];
      const int32_t* ae = rem.col + rem.ptr[u + 1];
      const int32_t* t = tcol.data() + tptr[u];
      const int32_t* te = tcol.data() + tptr[u + 1];
      int64_t cnt = 0;
      while (a < ae || t < te) {
        int32_t w;
        if (t == te || (a < ae && *a < *t)) w = *a++;
        else if (a == ae || *t < *a) w = *t++;
        else { w = *a; ++a; ++t; }
        if (out) out[cnt] = w;
        ++cnt;
      }
      return cnt;
    };
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t u = 0; u < n; ++u) own_ptr[u + 1] = merge_row(u, nullptr);
    for (int64_t u = 0; u < n; ++u) own_ptr[u + 1] += own_ptr[u];
    own_col.resize(own_ptr[n]);
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t u = 0; u < n; ++u) merge_row(u, own_col.data() + own_ptr[u]);
    ptr = own_ptr.data();
    col = own_col.data();
  }
  int64_t degree_slots(int32_t u) const { return ptr[u + 1] - ptr[u]; }
  // the s-th neighbour of u, s < degree_slots(u) (u itself is listed when it has a diagonal entry)
  int32_t at(int32_t u, int64_t s) const { return col[ptr[u] + s]; }
};

// breadth-first arrangement of the active vertices over the adjacency
void bfs_order(int64_t n, const Adjacency& adj, const std::vector<uint8_t>& active,
               std::vector<int32_t>& order) {
  std::vector<uint8_t> seen(n, 0);
  order.clear();
  for (int64_t s = 0; s < n; ++s) {
    if (!active[s] || seen[s]) continue;
    size_t head = order.size();
    order.push_back((int32_t)s);
    seen[s] = 1;
    while (head < order.size()) {
      int32_t u = order[head++];
      const int64_t ds = adj.degree_slots(u);
      for (int64_t s2 = 0; s2 < ds; ++s2) {
        int32_t w = adj.at(u, s2);
        if (!seen[w] && active[w]) { seen[w] = 1; order.push_back(w); }
      }
    }
  }
}

// Arrangement of the vertices outside `skip` (the head) by a traversal of the adjacency that ignores every
// entry touching a skipped vertex: depth-first preorder (dfs) or breadth-first order.  Sparse
// remainders are mostly small trees; a preorder keeps each of them contiguous, so most of their
// entries end up inside one diagonal block.
void traversal_order(int64_t n, const Adjacency& adj, const std::vector<uint8_t>& active,
                     const std::vector<uint8_t>& skip, bool dfs, std::vector<int32_t>& order) {
  std::vector<uint8_t> seen(n, 0);
  order.clear();
  std::vector<std::pair<int32_t, int64_t>> stack;   // vertex, next neighbour slot to look at
  for (int64_t s = 0; s < n; ++s) {
    if (!active[s] || skip[s] || seen[s]) continue;
    seen[s] = 1;
    order.push_back((int32_t)s);
    if (dfs) {
      stack.clear();
      stack.emplace_back((int32_t)s, (int64_t)0);
      while (!stack.empty()) {
        auto& top = stack.back();
        const int32_t u = top.first;
        bool pushed = false;
        const int64_t ds = adj.degree_slots(u);
        while (top.second < ds) {
          const int32_t w = adj.at(u, top.second++);
          if (!seen[w] && active[w] && !skip[w]) {
            seen[w] = 1;
            order.push_back(w);
            stack.emplace_back(w, (int64_t)0);
            pushed = true;
            break;
          }
        }
        if (!pushed) stack.pop_back();
      }
    } else {
      size_t head = order.size() - 1;
      while (head < order.size()) {
        const int32_t u = order[head++];
        const int64_t ds = adj.degree_slots(u);
        for (int64_t s2 = 0; s2 < ds; ++s2) {
          const int32_t w = adj.at(u, s2);
          if (!seen[w] && active[w] && !skip[w]) { seen[w] = 1; order.push_back(w); }
        }
      }
    }
  }
}

}  // namespace

int decompose(int64_t n, const int64_t* rowptr, const int32_t* colidx, const float* vals,
              int32_t b, const DecomposeOptions& opt, std::vector<HostLevel>& levels,
              std::string& err) {
  levels.clear();
  Remainder R;
  R.ptr = rowptr; R.col = colidx; R.val = vals;

  std::vector<int32_t> pos(n);
  std::vector<int64_t> deg(n);
  std::vector<int32_t> colcnt(n);
  std::vector<uint8_t> active(n);
  std::vector<int32_t> order;
  const int64_t level_cap = 4 * ((n + b - 1) / b) + 64;
  const bool symmetric = pattern_symmetric(n, R);   // the remainders of a symmetric pattern stay symmetric
  Adjacency adj;

  for (int64_t lev = 0;; ++lev) {
    const int64_t rem_nnz = R.nnz(n);
    if (lev > 0 && rem_nnz == 0) break;
    if (lev > level_cap) { err = "decomposition did not terminate"; return ARROW_EINTERNAL; }

    // ---- 1. degrees and active set ---------------------------------------
    std::fill(colcnt.begin(), colcnt.end(), 0);
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t u = 0; u < n; ++u)
      for (int64_t p = R.ptr[u]; p < R.ptr[u + 1]; ++p)
        __atomic_fetch_add(&colcnt[R.col[p]], 1, __ATOMIC_RELAXED);
    int64_t n_i = 0;
    double deg_sum = 0.0;
#pragma omp parallel for schedule(dynamic, 256) reduction(+ : n_i, deg_sum)
    for (int64_t u = 0; u < n; ++u) {
      int64_t rc = R.ptr[u + 1] - R.ptr[u];
      bool diag = std::binary_search(R.col + R.ptr[u], R.col + R.ptr[u + 1], (int32_t)u);
      deg[u] = rc + colcnt[u] - (diag ? 2 : 0);
      bool a = (lev == 0) || rc > 0 || colcnt[u] > 0;
      active[u] = a;
      if (a) { ++n_i; deg_sum += (double)deg[u]; }
    }

    adj.build(n, R, symmetric, colcnt);

    HostLevel L;
    L.n_i = n_i;
    L.perm.resize(n_i);
    std::fill(pos.begin(), pos.end(), -1);
    auto by_degree = [&](int32_t x, int32_t y) {
      return deg[x] != deg[y] ? deg[x] > deg[y] : x < y;
    };

    // ---- 2. arrangement ---------------------------------------------------
    if (lev == 0 || !opt.bfs_tail) {
      order.resize(0);
      order.reserve(n_i);
      for (int64_t u = 0; u < n; ++u) if (active[u]) order.push_back((int32_t)u);
    } else {
      bfs_order(n, adj, active, order);
    }

    // ---- 3. head and block positions ------------------------------------
    if (n_i <= b) {
      std::sort(order.begin(), order.end(), by_degree);
      for (int64_t p = 0; p < n_i; ++p) L.perm[p] = order[p];
    } else {
      bool done = false;
      if (opt.separators) {
        const double thresh = opt.hub_factor * (deg_sum / (double)n_i);
        std::vector<int32_t> hubs;
        for (int32_t v : order) if ((double)deg[v] > thresh) hubs.push_back(v);
        if ((int64_t)hubs.size() < b) {
          std::sort(hubs.begin(), hubs.end(), by_degree);
          // block id per vertex: -1 unplaced, 0 head, r >= 1 body block r
          std::vector<int32_t> blk(n, -1);
          for (int32_t v : hubs) blk[v] = 0;
          const int64_t cap = b - (int64_t)hubs.size();
          std::vector<int32_t> seps, body;
          body.reserve(n_i);
          int32_t cur = 1;
          int64_t fill = 0;
          bool ok = true;
          for (int32_t v : order) {
            if (blk[v] == 0) continue;
            bool promote = false;
            const int64_t ds = adj.degree_slots(v);
            for (int64_t s2 = 0; s2 < ds; ++s2) {
              int32_t bw = blk[adj.at(v, s2)];
              if (bw >= 1 && bw < cur) { promote = true; break; }
            }
            if (promote) {
              if ((int64_t)seps.size() == cap) { ok = false; break; }
              seps.push_back(v);
              blk[v] = 0;
            } else {
              body.push_back(v);
              blk[v] = cur;
              if (++fill == b) { ++cur; fill = 0; }
            }
          }
          if (ok) {
            int64_t need = b - (int64_t)hubs.size() - (int64_t)seps.size();
            int64_t h = 0;
            for (int32_t v : hubs) L.perm[h++] = v;
            for (int32_t v : seps) L.perm[h++] = v;
            for (int64_t t = 0; t < need; ++t) { L.perm[h++] = body.back(); body.pop_back(); }
            for (int32_t v : body) L.perm[h++] = v;
            // accept only if the level takes every remaining entry (it must, by the argument in
            // the header; the count guards the rule against any operand the argument misses)
            std::vector<int32_t> spos(n, -1);
#pragma omp parallel for schedule(static)
            for (int64_t p = 0; p < n_i; ++p) spos[L.perm[p]] = (int32_t)p;
            int64_t outside = 0;
#pragma omp parallel for schedule(dynamic, 256) reduction(+ : outside)
            for (int64_t u = 0; u < n; ++u) {
              const int64_t pu = spos[u];
              if (pu < 0 || pu < b) continue;
              for (int64_t p = R.ptr[u]; p < R.ptr[u + 1]; ++p) {
                const int64_t pv = spos[R.col[p]];
                if (pv >= b && pv / b != pu / b) ++outside;
              }
            }
            if (outside == 0) {
              L.separator_rule = true;
              done = true;
            }
          }
        }
      }
      if (!done) {
        std::vector<int32_t> cand(order);
        std::nth_element(cand.begin(), cand.begin() + b, cand.end(), by_degree);
        if (opt.head_by_id) {
          // the hubs_first highest-degree vertices lead the head in falling-degree order (their
          // rows and columns form the dense corner of the head block), the others follow in id order
          const int64_t hubs = std::min<int64_t>(std::max<int64_t>(opt.hubs_first, 0), b);
          if (hubs > 0 && hubs < b) std::nth_element(cand.begin(), cand.begin() + hubs, cand.begin() + b, by_degree);
          std::sort(cand.begin(), cand.begin() + hubs, by_degree);
          std::sort(cand.begin() + hubs, cand.begin() + b);
        } else {
          std::sort(cand.begin(), cand.begin() + b, by_degree);
        }
        std::vector<uint8_t> in_head(n, 0);
        for (int64_t p = 0; p < b; ++p) { L.perm[p] = cand[p]; in_head[cand[p]] = 1; }
        // the rest: the given arrangement, or a traversal of what is left without the head --
        // whichever puts more of the rest-to-rest entries into diagonal blocks
        std::vector<int32_t> best;
        int64_t best_cap = -1;
        std::vector<int32_t> trial;
        std::vector<int32_t> tpos(n, -1);
        const int n_cand = opt.bfs_tail ? 3 : 1;
        for (int cnd = 0; cnd < n_cand; ++cnd) {
          if (cnd == 0) {
            trial.clear();
            for (int32_t v : order) if (!in_head[v]) trial.push_back(v);
          } else {
            traversal_order(n, adj, active, in_head, cnd == 1, trial);
          }
          const int64_t nt = (int64_t)trial.size();
#pragma omp parallel for schedule(static)
          for (int64_t t = 0; t < nt; ++t) tpos[trial[t]] = (int32_t)(t / b);
          int64_t cap = 0;
#pragma omp parallel for schedule(dynamic, 256) reduction(+ : cap)
          for (int64_t t = 0; t < nt; ++t) {
            const int32_t u = trial[t];
            const int32_t bu = tpos[u];
            for (int64_t p = R.ptr[u]; p < R.ptr[u + 1]; ++p) {
              const int32_t w = R.col[p];
              if (!in_head[w] && tpos[w] == bu) ++cap;
            }
          }
          if (cap > best_cap) { best_cap = cap; best.swap(trial); }
        }
        int64_t h = b;
        for (int32_t v : best) L.perm[h++] = v;
      }
    }
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < n_i; ++p) pos[L.perm[p]] = (int32_t)p;

    // ---- 4. split the remainder into this level's arrow and the next remainder
    auto in_arrow = [&](int64_t pu, int64_t pv) {
      return pu < b || pv < b || pu / b == pv / b;
    };
    L.rowptr.assign(n_i + 1, 0);
    std::vector<int64_t> next_ptr(n + 1, 0);
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t u = 0; u < n; ++u) {
      int64_t pu = pos[u];
      if (pu < 0) continue;
      int64_t keep = 0, drop = 0;
      for (int64_t p = R.ptr[u]; p < R.ptr[u + 1]; ++p) {
        if (in_arrow(pu, pos[R.col[p]])) ++keep; else ++drop;
      }
      L.rowptr[pu + 1] = keep;
      next_ptr[u + 1] = drop;
    }
    for (int64_t p = 0; p < n_i; ++p) L.rowptr[p + 1] += L.rowptr[p];
    for (int64_t u = 0; u < n; ++u) next_ptr[u + 1] += next_ptr[u];
    const int64_t lev_nnz = L.rowptr[n_i];
    const int64_t next_nnz = next_ptr[n];
    if (lev_nnz + next_nnz != rem_nnz) { err = "entry count mismatch while peeling"; return ARROW_EINTERNAL; }
    if (lev_nnz == 0 && rem_nnz > 0) { err = "a level captured no entry"; return ARROW_EINTERNAL; }
    L.colpos.resize(lev_nnz);
    L.vals.resize(lev_nnz);
    L.src.resize(lev_nnz);
    std::vector<int32_t> next_col(next_nnz);
    std::vector<float> next_val(next_nnz);
    std::vector<uint32_t> next_src(next_nnz);
    int64_t hh = 0, hr = 0, hc = 0, dg = 0;
#pragma omp parallel for schedule(dynamic, 256) reduction(+ : hh, hr, hc, dg)
    for (int64_t u = 0; u < n; ++u) {
      int64_t pu = pos[u];
      if (pu < 0) continue;
      int64_t w = L.rowptr[pu], x = next_ptr[u];
      const int64_t w0 = w;
      for (int64_t p = R.ptr[u]; p < R.ptr[u + 1]; ++p) {
        int64_t pv = pos[R.col[p]];
        if (in_arrow(pu, pv)) {
          L.colpos[w] = (int32_t)pv;
          L.vals[w] = R.val[p];
          L.src[w] = R.src ? R.src[p] : (uint32_t)p;
          ++w;
          if (pu < b) { if (pv < b) ++hh; else ++hr; } else { if (pv < b) ++hc; else ++dg; }
        } else {
          next_col[x] = R.col[p];
          next_val[x] = R.val[p];
          next_src[x] = R.src ? R.src[p] : (uint32_t)p;
          ++x;
        }
      }
      // order the row by column position (keys are distinct inside a row)
      const int64_t len = w - w0;
      if (len > 1) {
        bool sorted = true;
        for (int64_t q = w0 + 1; q < w; ++q) if (L.colpos[q - 1] > L.colpos[q]) { sorted = false; break; }
        if (!sorted) {
          std::vector<uint64_t> key(len);
          for (int64_t q = 0; q < len; ++q) key[q] = ((uint64_t)(uint32_t)L.colpos[w0 + q] << 32) | (uint64_t)q;
          std::sort(key.begin(), key.end());
          std::vector<float> tv(len);
          std::vector<uint32_t> ts(len);
          for (int64_t q = 0; q < len; ++q) {
            const int64_t from = w0 + (int64_t)(key[q] & 0xffffffffu);
            tv[q] = L.vals[from];
            ts[q] = L.src[from];
          }
          for (int64_t q = 0; q < len; ++q) {
            L.colpos[w0 + q] = (int32_t)(key[q] >> 32);
            L.vals[w0 + q] = tv[q];
            L.src[w0 + q] = ts[q];
          }
        }
      }
    }
    L.nnz_head_head = hh; L.nnz_head_row = hr; L.nnz_head_col = hc; L.nnz_diag = dg;
    levels.push_back(std::move(L));

    R.own_ptr.swap(next_ptr);
    R.own_col.swap(next_col);
    R.own_val.swap(next_val);
    R.own_src.swap(next_src);
    R.ptr = R.own_ptr.data(); R.col = R.own_col.data(); R.val = R.own_val.data(); R.src = R.own_src.data();
    if (next_nnz == 0) break;
  }
  return ARROW_OK;
}

}  // namespace arrow
