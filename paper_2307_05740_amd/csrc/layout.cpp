// Packs the arrow matrices of a decomposition into one flat device image.
//
// Per level the image holds the permutation, the optional LDS-window tiles, and two work
// lists of ITEMS.  An item is a run of entries of one row together with a destination: a row
// of Y (the item is the whole row) or a partial-vector slot (the row was cut into several
// items; the reduction sums its slots, which are consecutive, in a fixed order).
//   group list - items handled one per lane group: rows with at most short_max entries in
//                position order (so the rows of one diagonal block are neighbours and share
//                their window of X; a level-0 row without entries is listed too, because
//                level 0 stores every row of Y), and the short class pieces of split rows.
//   wave list  - items handled one per wavefront: chunks of at most chunk_nnz entries.
//
// How the long rows are cut and ordered decides where the X rows of the head columns (the
// window X_0 every block shares) are served from:
//   * Column classes (optional).  Column positions are dealt to `classes` classes in granules
//     of class_gran positions.  A row with at least classes * class_min entries is split by
//     class; a class piece goes to the group list when it has at most piece_max entries, else
//     it is chunked into the wave list.  Items of class c sit in workgroup slots that the
//     hardware hands to accelerator die c mod 8 (workgroups go to the 8 dies round-robin by
//     workgroup id; a workgroup takes kItemsPerGroupBlock group items or kChunksPerGroup
//     wave items).  One die therefore only touches 1/classes of X_0 during a phase, a slice
//     small enough to stay resident in its own L2, and every use of an X row outside the head
//     lands on the same die as well.  classes / 8 phases follow each other; inside a
//     (phase, die) queue items are ordered by the column window they start in; queues are
//     padded with empty slots to equal length.
//   * Rows not split by class are cut at column-window boundaries (windows are merged until a
//     piece holds chunk_min entries); a piece of at most piece_max entries is a group-list item,
//     a longer one is cut into wave-list chunks of at most chunk_nnz entries.  Both lists are
//     ordered by the window an item starts in, so that the wavefronts in flight read one
//     neighbourhood of X rows; these items form the last phase of their list.
//   * Head staging.  The head rows of P_i X are gathered once per product into a contiguous
//     buffer, class by class, so a die's slice is one contiguous range.  Entries of head
//     columns of long rows carry the row of that buffer; they come first in every item
//     (entries are ordered by column position) and the item's `mid` marks where they end.
//     All other entries carry perm[q]: the permutation gather stays fused.
//   * Head panels (optional, off by default): see the planning code below.
//   * Dense corner (on by default when the head is staged).  The head vertices sit in id order,
//     and in skewed graphs the lowest ids are the hubs: the top-left corner of the head block is
//     orders of magnitude denser than the rest.  Rows and columns [0, S) are cut into tiles of
//     256 x 256 positions, S chosen at pack time as the largest size whose outermost band of
//     tiles still holds corner_min_tile entries per tile on average.  These entries (a prefix of
//     their rows) leave the chunk lists: a workgroup takes a run of tiles of one row panel,
//     copies each tile's 256 staged head rows into LDS with coalesced loads, and its lane
//     groups stream the tile's entries -- in 64 runs that never share a row -- against LDS
//     instead of gathering a row through the caches per entry.  The format is chosen per tile
//     region by measured density: outside the corner an LDS copy of 256 rows would be used by
//     fewer entries than it has rows.
//   * Fused levels (on by default).  perm_0 is a full permutation, so every vertex owns a row
//     of level 0.  The entries that later levels hold for a vertex are listed with that row
//     (their columns translated to level-0 positions), and the row's one item, or its chunks,
//     sums over all arrow matrices at once: the scatter-add P_i^T of the later levels happens
//     in the accumulator instead of through a read-modify-write of Y, and their launches go
//     away.  Where an entry's X row is read from is still decided by the arrow it belongs to
//     (staged head, LDS window, or X through the fused gather).  The exported levels are
//     untouched; the later levels keep only their permutation in the image.
// Besides the image the packer builds the entry map (image order -> index of the entry in the
// caller's CSR arrays), which the sampled dense-dense product needs for its output.
#include "arrow_internal.h"

#include <omp.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <queue>

#include "arrow.h"

namespace arrow {
namespace {

constexpr size_t kAlign = 256;
constexpr uint32_t kPad = 0xffffffffu;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Rec {
  int32_t row;     // row position
  uint32_t len;
  int32_t dst;
  uint32_t phase;
  uint32_t key;    // column window of the first entry
  int8_t queue;    // die queue 0..7, or -1 for the window-ordered last phase
  uint8_t list;    // 0 group list, 1 wave list
  uint32_t seq;    // emission index (names the rec)
};

struct Plan {
  std::vector<int32_t> row_pos;       // plain short rows (group list tail), in position order
  std::vector<Rec> recs;              // items of the long rows in emission order (row by row)
  std::vector<int64_t> row_first;     // per long row: index of its first rec
  std::vector<int32_t> long_rows;     // positions of the long rows
  std::vector<uint8_t> row_split;     // 1 if the row is split by class
  std::vector<uint32_t> slot_of;      // rec seq -> slot in its list
  std::vector<uint32_t> list_ptr[2];  // per list: entry offsets, slots + 1
  std::vector<int32_t> list_dst[2];   // per list: destination per slot
  std::vector<int32_t> list_row[2];   // per list: the Y row (vertex) the item belongs to, -1 for padding
  int64_t piece_slots = 0;            // group-list slots before the plain short rows
  std::vector<uint32_t> split_ptr;
  std::vector<int32_t> split_y;
  std::vector<int32_t> stage_perm;    // staged head: buffer row -> original X row
  std::vector<WindowTile> wtiles;     // diagonal-block tiles with their X window staged in LDS
  std::vector<int32_t> wrow_pos;      // row positions of the window rows, tile by tile
  std::vector<uint32_t> wrow_ptr;     // offsets of their entries (relative to the level's entries)
  std::vector<uint32_t> skip;         // per row position: leading (head-block) entries handed to the panels
  std::vector<int32_t> panel_pos;     // accumulator slot -> row position, -1 = unused (groups * kPanelRows)
  std::vector<uint8_t> panel_bin;     // per (slot, class): the bin of workgroup (group, class) that streams the row's class entries
  std::vector<uint32_t> panel_ptr;    // per bin: offsets of its entries (relative to the level's entries)
  int64_t nnz_panel = 0, n_panel_rows = 0;
  // dense corner: tiles in (row panel, column tile) order; per tile its entry count until the
  // lists are placed, then kCornerTileWords words (run offsets, first column, panel)
  int64_t corner = 0, nnz_corner = 0;
  std::vector<uint32_t> corner_cnt;    // per listed tile: entries
  std::vector<uint32_t> corner_ij;     // per listed tile: (row panel << 16) | column tile
  std::vector<uint32_t> corner_first;  // per listed tile: offset of its first entry (relative to the level's entries)
  std::vector<uint32_t> corner_items;  // per item: first tile (+ end)
  std::vector<uint32_t> corner_panel;  // per row panel: first item (+ end)
  uint32_t row_skip(int64_t p) const { return skip.empty() ? 0u : skip[p]; }
};

// order the recs of one list: class phases as padded die queues, then the last phase in
// window order; returns rec indices, kPad for padding slots
std::vector<uint32_t> order_list(const std::vector<Rec>& recs, int list, uint32_t class_phases,
                                 int unit) {
  std::vector<uint32_t> order;
  for (size_t i = 0; i < recs.size(); ++i) if (recs[i].list == list) order.push_back((uint32_t)i);
  std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) {
    const Rec& a = recs[x];
    const Rec& c = recs[y];
    if (a.phase != c.phase) return a.phase < c.phase;
    if (a.queue != c.queue) return a.queue < c.queue;
    return a.key < c.key;
  });
  std::vector<uint32_t> out;
  out.reserve(order.size() + 64);
  size_t at = 0;
  for (uint32_t ph = 0; ph < class_phases; ++ph) {
    size_t qbeg[kDies + 1];
    for (int q = 0; q < kDies; ++q) {
      qbeg[q] = at;
      while (at < order.size() && recs[order[at]].phase == ph && recs[order[at]].queue == q) ++at;
    }
    qbeg[kDies] = at;
    size_t rounds = 0;
    for (int q = 0; q < kDies; ++q)
      rounds = std::max(rounds, (qbeg[q + 1] - qbeg[q] + unit - 1) / unit);
    for (size_t rd = 0; rd < rounds; ++rd)
      for (int q = 0; q < kDies; ++q)
        for (int j = 0; j < unit; ++j) {
          const size_t idx = qbeg[q] + rd * unit + j;
          out.push_back(idx < qbeg[q + 1] ? order[idx] : kPad);
        }
  }
  while (at < order.size()) out.push_back(order[at++]);   // last phase: plain window order
  return out;
}

// The execution form of a decomposition with fused levels: level 0 with the entries of all later
// levels appended to the rows of their vertices (columns as level-0 positions, every row ordered
// by column position again), and the later levels reduced to their permutations.
void fuse_levels(const std::vector<HostLevel>& levels, std::vector<HostLevel>& exec,
                 std::vector<int64_t>& fused_from) {
  exec.clear();
  exec.resize(levels.size());
  fused_from.assign(levels.size(), 0);
  const HostLevel& L0 = levels[0];
  const int64_t n0 = L0.n_i;
  std::vector<int32_t> pos0((size_t)n0, -1);          // vertex -> level-0 position (n_i of level 0 is n)
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < n0; ++p) pos0[L0.perm[p]] = (int32_t)p;
  std::vector<int64_t> extra((size_t)n0 + 1, 0);
  for (size_t li = 1; li < levels.size(); ++li) {
    const HostLevel& L = levels[li];
    fused_from[li] = L.rowptr[L.n_i];
    for (int64_t p = 0; p < L.n_i; ++p) extra[(size_t)pos0[L.perm[p]] + 1] += L.rowptr[p + 1] - L.rowptr[p];
  }
  HostLevel& E = exec[0];
  E.n_i = n0;
  E.perm = L0.perm;
  E.nnz_head_head = L0.nnz_head_head; E.nnz_head_row = L0.nnz_head_row;
  E.nnz_head_col = L0.nnz_head_col; E.nnz_diag = L0.nnz_diag;
  E.separator_rule = L0.separator_rule;
  E.rowptr.assign((size_t)n0 + 1, 0);
  for (int64_t p = 0; p < n0; ++p) E.rowptr[p + 1] = E.rowptr[p] + (L0.rowptr[p + 1] - L0.rowptr[p]) + extra[p + 1];
  const int64_t total = E.rowptr[n0];
  E.colpos.resize((size_t)total);
  E.vals.resize((size_t)total);
  E.src.resize((size_t)total);
  std::vector<int64_t> fill((size_t)n0);
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t p = 0; p < n0; ++p) {
    int64_t w = E.rowptr[p];
    for (int64_t e = L0.rowptr[p]; e < L0.rowptr[p + 1]; ++e, ++w) {
      E.colpos[w] = L0.colpos[e]; E.vals[w] = L0.vals[e]; E.src[w] = L0.src[e];
    }
    fill[p] = w;
  }
  for (size_t li = 1; li < levels.size(); ++li) {
    const HostLevel& L = levels[li];
    // a vertex is a row of a level at most once, so no two rows of L write the same target row
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t p = 0; p < L.n_i; ++p) {
      const int64_t tp = pos0[L.perm[p]];
      int64_t w = fill[tp];
      for (int64_t e = L.rowptr[p]; e < L.rowptr[p + 1]; ++e, ++w) {
        E.colpos[w] = pos0[L.perm[L.colpos[e]]]; E.vals[w] = L.vals[e]; E.src[w] = L.src[e];
      }
      fill[tp] = w;
    }
    HostLevel& S = exec[li];
    S.n_i = L.n_i;
    S.perm = L.perm;
    S.rowptr.assign((size_t)L.n_i + 1, 0);
    S.separator_rule = L.separator_rule;
  }
  // rows that received entries: order by column position again (keys are distinct inside a row)
#pragma omp parallel
  {
    std::vector<uint64_t> key;
    std::vector<float> tv;
    std::vector<uint32_t> ts;
#pragma omp for schedule(dynamic, 256)
    for (int64_t p = 0; p < n0; ++p) {
      if (extra[p + 1] == 0) continue;
      const int64_t w0 = E.rowptr[p], len = E.rowptr[p + 1] - w0;
      key.resize((size_t)len); tv.resize((size_t)len); ts.resize((size_t)len);
      for (int64_t q = 0; q < len; ++q) key[q] = ((uint64_t)(uint32_t)E.colpos[w0 + q] << 32) | (uint64_t)q;
      std::sort(key.begin(), key.end());
      for (int64_t q = 0; q < len; ++q) {
        const int64_t from = w0 + (int64_t)(key[q] & 0xffffffffu);
        tv[q] = E.vals[from]; ts[q] = E.src[from];
      }
      for (int64_t q = 0; q < len; ++q) {
        E.colpos[w0 + q] = (int32_t)(key[q] >> 32); E.vals[w0 + q] = tv[q]; E.src[w0 + q] = ts[q];
      }
    }
  }
}

int pack_levels(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const PackOptions& opt,
                Image& img, std::string& err) {
  img.levels.clear();
  img.max_partials = 0;
  img.max_stage_rows = 0;
  img.max_window_span = 0;
  img.max_panel_slots = 0;
  img.max_corner_items = 0;
  const int64_t short_max = opt.short_max < 0 ? 0 : opt.short_max;
  const int64_t chunk_nnz = opt.chunk_nnz < 1 ? 1 : opt.chunk_nnz;
  const int64_t chunk_min = opt.chunk_min < 1 ? 1 : (opt.chunk_min > chunk_nnz ? chunk_nnz : opt.chunk_min);
  const int64_t window = opt.window_rows < 0 ? 0 : opt.window_rows;
  const int64_t classes = opt.classes <= 0 ? 0 : (opt.classes + kDies - 1) / kDies * kDies;
  const int64_t gran = opt.class_gran < 1 ? 1 : opt.class_gran;
  const int64_t class_min = opt.class_min < 1 ? 1 : opt.class_min;
  const int64_t piece_max = opt.piece_max < 0 ? 0 : opt.piece_max;
  const int64_t key_window = window > 0 ? window : 4096;
  const uint32_t class_phases = (uint32_t)(classes / kDies);

  std::vector<Plan> plans(levels.size());
  size_t total = 0;
  int64_t map_total = 0;     // entries of all levels: the entry map is one uint32 per entry

  for (size_t li = 0; li < levels.size(); ++li) {
    const HostLevel& L = levels[li];
    Plan& P = plans[li];
    LevelImage im;
    im.n_i = L.n_i;
    const int64_t lev_nnz = L.rowptr[L.n_i];
    if (lev_nnz >= 0xffffffffLL - 4096) { err = "a level holds too many entries (limit 2^32 - 4097)"; return ARROW_EINVAL; }
    const int64_t head = std::min<int64_t>(b, L.n_i);
    im.staged = opt.stage_head && li == 0 && L.n_i > b;
    im.n_stage = im.staged ? head : 0;
    if (im.n_stage > img.max_stage_rows) img.max_stage_rows = im.n_stage;
    im.classes = (int32_t)classes;

    // ---- diagonal-block tiles whose window of P_i X is staged in LDS ---------------------------
    // Consecutive body rows of one diagonal block form a tile while the column positions their
    // diagonal-block entries touch span at most window_span positions; the tile is kept when
    // those entries reuse the span often enough to pay for staging it.
    std::vector<uint8_t> taken(L.n_i, 0);
    int64_t nnz_w = 0;
    // A row joins a window tile only when the entries it reads from memory there (first block
    // column; other blocks once levels are fused) do not outnumber its diagonal-block entries, or
    // are few anyway: the window kernel reads those one lane group per row, which is the slow way
    // to handle a long row.
    auto window_row_ok = [&](int64_t len, int64_t in_block) {
      const int64_t outside = len - in_block;
      return outside <= in_block || outside <= short_max;
    };
    if (opt.window_span > 0 && L.n_i > b) {
      const int64_t span_cap = opt.window_span, rows_cap = opt.window_tile_rows < 1 ? 1 : opt.window_tile_rows;
      for (int64_t blk0 = b; blk0 < L.n_i; blk0 += b) {
        const int64_t blk1 = std::min<int64_t>(blk0 + b, L.n_i);
        int64_t p0 = blk0;
        while (p0 < blk1) {
          int64_t cmin = INT64_MAX, cmax = -1, dnnz = 0, p1 = p0;
          for (; p1 < blk1 && p1 - p0 < rows_cap; ++p1) {
            const int32_t* cb = L.colpos.data() + L.rowptr[p1];
            const int32_t* ce = L.colpos.data() + L.rowptr[p1 + 1];
            // the row's diagonal-block entries (with fused levels a row also holds entries of
            // other blocks; those are read from memory like the first-block-column entries)
            const int32_t* cd = std::lower_bound(cb, ce, (int32_t)blk0);
            const int32_t* cx = std::lower_bound(cd, ce, (int32_t)blk1);
            if (cd == cx) continue;                                       // no diagonal-block entry
            if (!window_row_ok(ce - cb, cx - cd)) continue;               // the row stays in the ordinary lists
            const int64_t nmin = std::min<int64_t>(cmin, *cd), nmax = std::max<int64_t>(cmax, *(cx - 1));
            if (nmax - nmin + 1 > span_cap) break;
            cmin = nmin; cmax = nmax; dnnz += cx - cd;
          }
          if (p1 == p0) { ++p0; continue; }                               // one row alone exceeds the span
          if (cmax >= 0 && (double)dnnz >= opt.window_reuse * (double)(cmax - cmin + 1)) {
            WindowTile t;
            t.row_begin = (uint32_t)P.wrow_pos.size();
            t.win_begin = (uint32_t)cmin;
            t.win_count = (uint32_t)(cmax - cmin + 1);
            for (int64_t p = p0; p < p1; ++p) {
              const int64_t len = L.rowptr[p + 1] - L.rowptr[p];
              if (len == 0 && li > 0) continue;
              {
                const int32_t* cb = L.colpos.data() + L.rowptr[p];
                const int32_t* ce = cb + len;
                const int32_t* cd = std::lower_bound(cb, ce, (int32_t)blk0);
                const int32_t* cx = std::lower_bound(cd, ce, (int32_t)blk1);
                if (!window_row_ok(len, cx - cd)) continue;
              }
              taken[p] = 1;
              P.wrow_pos.push_back((int32_t)p);
              nnz_w += len;
            }
            t.row_end = (uint32_t)P.wrow_pos.size();
            if (t.row_end > t.row_begin) {
              P.wtiles.push_back(t);
            }
          }
          p0 = p1;
        }
      }
      // a separate launch for a handful of tiles costs more than it saves: keep the tiles only
      // when they hold a fair share of the level
      if ((double)nnz_w < opt.window_level_share * (double)lev_nnz) {
        std::fill(taken.begin(), taken.end(), 0);
        P.wtiles.clear();
        P.wrow_pos.clear();
        nnz_w = 0;
      }
    }

    for (const WindowTile& t : P.wtiles)
      if ((int64_t)t.win_count > img.max_window_span) img.max_window_span = t.win_count;

    // ---- head panels ---------------------------------------------------------------------------
    // A head row whose head-block entries are too few per column window to form window-local
    // chunks hands them to a panel.  kPanelRows such rows form a group (groups hold equal numbers
    // of entries).  The group's entries are dealt by column class -- staged head row mod 8 -- to 8
    // workgroups, and workgroup (group, class) has the linear id group * 8 + class, so class c is
    // always served by accelerator die c: a die's L2 only ever holds an eighth of the staged head
    // X_0.  Each workgroup keeps the group's accumulators in LDS and streams its entries in
    // kPanelBins lane-group streams of equal length, each ordered by row, then column; a row's
    // class entries all sit in one stream, so no two lane groups touch the same accumulator.
    // The eight class results of a row are added to Y afterwards, in class order.
    // What is left of such a row (columns outside the head) is planned like any other row.
    if (opt.panel && im.staged && classes == 0 && window > 0 && im.n_stage <= (1LL << kPanelRowShift)) {
      const int64_t n_windows = (im.n_stage + window - 1) / window;
      const int64_t dense = chunk_min * n_windows;       // such rows fill window-local chunks by themselves
      const int64_t pmin = opt.panel_min < 1 ? 1 : opt.panel_min;
      std::vector<std::pair<uint32_t, int32_t>> cand;    // (head-block entries, position)
      int64_t nnz_p = 0;
      // a row much longer than the others cannot be balanced against them inside a workgroup's
      // streams: the second pass also leaves out rows above 6 x the mean of the first
      int64_t cap = dense;
      for (int pass = 0; pass < 2; ++pass) {
        cand.clear();
        nnz_p = 0;
        for (int64_t p = 0; p < head; ++p) {
          if (taken[p]) continue;
          const int32_t* cb = L.colpos.data() + L.rowptr[p];
          const int32_t* ce = L.colpos.data() + L.rowptr[p + 1];
          const int64_t cnt = std::lower_bound(cb, ce, (int32_t)im.n_stage) - cb;
          if (cnt < pmin || cnt >= cap) continue;
          cand.emplace_back((uint32_t)cnt, (int32_t)p);
          nnz_p += cnt;
        }
        if (cand.empty()) break;
        const int64_t lim = 6 * (nnz_p / (int64_t)cand.size()) + 1;
        if (lim >= cap) break;
        cap = lim;
      }
      // worth its launches only when the head spans several windows (else it stays in L2 anyway)
      // and the panels hold a fair share of the level
      if (!cand.empty() && n_windows >= 2 && (double)nnz_p >= 0.05 * (double)lev_nnz) {
        std::sort(cand.begin(), cand.end(), [](const std::pair<uint32_t, int32_t>& x, const std::pair<uint32_t, int32_t>& y) {
          return x.first != y.first ? x.first > y.first : x.second < y.second;
        });
        const int64_t n_cand = (int64_t)cand.size();
        const int64_t n_groups = (n_cand + kPanelRows - 1) / kPanelRows;
        P.skip.assign(L.n_i, 0);
        P.panel_pos.assign((size_t)n_groups * kPanelRows, -1);
        // longest row first, each to the group with the fewest entries so far that still has room
        {
          std::vector<int32_t> filled((size_t)n_groups, 0);
          std::priority_queue<std::pair<int64_t, int64_t>, std::vector<std::pair<int64_t, int64_t>>,
                              std::greater<std::pair<int64_t, int64_t>>> open;     // (entries, group)
          for (int64_t g = 0; g < n_groups; ++g) open.emplace(0, g);
          for (int64_t i = 0; i < n_cand; ++i) {
            const std::pair<int64_t, int64_t> top = open.top();
            open.pop();
            const int64_t g = top.second;
            P.panel_pos[(size_t)g * kPanelRows + filled[g]] = cand[i].second;
            P.skip[cand[i].second] = cand[i].first;
            if (++filled[g] < kPanelRows) open.emplace(top.first + cand[i].first, g);
          }
        }
        // per (group, class): the rows' class entries, longest first, to the shortest stream
        const int64_t n_bins = n_groups * kDies * kPanelBins;
        P.panel_bin.assign((size_t)n_groups * kPanelRows * kDies, 0);
        std::vector<uint32_t> bin_len((size_t)n_bins, 0);
#pragma omp parallel
        {
          std::vector<std::pair<uint32_t, int32_t>> rows_c;   // (class entries, slot in the group)
          std::vector<uint32_t> cls_cnt((size_t)kPanelRows * kDies);
#pragma omp for schedule(dynamic, 4)
          for (int64_t g = 0; g < n_groups; ++g) {
            std::fill(cls_cnt.begin(), cls_cnt.end(), 0u);
            for (int r = 0; r < kPanelRows; ++r) {
              const int32_t p = P.panel_pos[(size_t)g * kPanelRows + r];
              if (p < 0) continue;
              const int32_t* cb = L.colpos.data() + L.rowptr[p];
              for (uint32_t e = 0; e < P.skip[p]; ++e) ++cls_cnt[(size_t)r * kDies + panel_class((uint32_t)cb[e])];
            }
            for (int c = 0; c < kDies; ++c) {
              rows_c.clear();
              for (int r = 0; r < kPanelRows; ++r)
                if (cls_cnt[(size_t)r * kDies + c]) rows_c.emplace_back(cls_cnt[(size_t)r * kDies + c], r);
              std::sort(rows_c.begin(), rows_c.end(), [](const std::pair<uint32_t, int32_t>& x, const std::pair<uint32_t, int32_t>& y) {
                return x.first != y.first ? x.first > y.first : x.second < y.second;
              });
              uint32_t* len = bin_len.data() + ((size_t)g * kDies + c) * kPanelBins;
              for (const auto& rc : rows_c) {
                int best = 0;
                for (int j = 1; j < kPanelBins; ++j) if (len[j] < len[best]) best = j;
                len[best] += rc.first;
                P.panel_bin[((size_t)g * kPanelRows + rc.second) * kDies + c] = (uint8_t)best;
              }
            }
          }
        }
        P.panel_ptr.assign((size_t)n_bins + 1, 0);       // lengths for now; offsets once the lists are placed
        for (int64_t bi = 0; bi < n_bins; ++bi) P.panel_ptr[bi + 1] = bin_len[bi];
        P.nnz_panel = nnz_p;
        P.n_panel_rows = n_cand;
      }
    }

    // ---- dense corner ----------------------------------------------------------------------------
    if (opt.corner && im.staged && classes == 0 && P.panel_pos.empty() && opt.corner_min_tile > 0) {
      const int64_t max_s = std::min<int64_t>(head, std::max<int64_t>(0, opt.corner_max)) / kCornerTile;   // tiles per side considered
      if (max_s >= 1) {
        std::vector<uint32_t> cnt((size_t)(max_s * max_s), 0);
        const int64_t lim = max_s * kCornerTile;
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t ip = 0; ip < max_s; ++ip)
          for (int64_t p = ip * kCornerTile; p < (ip + 1) * kCornerTile; ++p) {
            const int32_t* cb = L.colpos.data() + L.rowptr[p];
            const int32_t* ce = std::lower_bound(cb, L.colpos.data() + L.rowptr[p + 1], (int32_t)lim);
            for (const int32_t* c = cb; c < ce; ++c) ++cnt[(size_t)(ip * max_s + *c / kCornerTile)];
          }
        // the largest corner whose outermost band of tiles is still dense enough
        int64_t side = 0;
        for (int64_t sd = max_s; sd >= 1; --sd) {
          int64_t band = 0;
          for (int64_t t = 0; t < sd; ++t) band += cnt[(size_t)((sd - 1) * max_s + t)] + (t < sd - 1 ? cnt[(size_t)(t * max_s + sd - 1)] : 0);
          if (band >= (int64_t)opt.corner_min_tile * (2 * sd - 1)) { side = sd; break; }
        }
        int64_t nnz_c = 0;
        for (int64_t i = 0; i < side; ++i) for (int64_t j = 0; j < side; ++j) nnz_c += cnt[(size_t)(i * max_s + j)];
        // worth its launches only when it holds a fair share of the level
        if (side >= 1 && (double)nnz_c >= 0.02 * (double)lev_nnz) {
          P.corner = side * kCornerTile;
          P.nnz_corner = nnz_c;
          P.skip.assign(L.n_i, 0);
#pragma omp parallel for schedule(dynamic, 256)
          for (int64_t p = 0; p < P.corner; ++p) {
            const int32_t* cb = L.colpos.data() + L.rowptr[p];
            P.skip[p] = (uint32_t)(std::lower_bound(cb, L.colpos.data() + L.rowptr[p + 1], (int32_t)P.corner) - cb);
          }
          // work items: runs of tiles of one row panel holding about the same number of entries;
          // enough of them to spread over all compute units, few enough to keep the partial
          // results (256 rows per item) small
          const int64_t target = std::max<int64_t>(8192, nnz_c / 2048);
          P.corner_panel.push_back(0);
          for (int64_t i = 0; i < side; ++i) {
            int64_t in_item = 0;
            bool open = false;
            for (int64_t j = 0; j < side; ++j) {
              const uint32_t c = cnt[(size_t)(i * max_s + j)];
              if (c == 0) continue;
              if (!open || in_item >= target) {
                P.corner_items.push_back((uint32_t)P.corner_cnt.size());
                open = true;
                in_item = 0;
              }
              P.corner_cnt.push_back(c);
              P.corner_ij.push_back((uint32_t)((i << 16) | j));
              in_item += c;
            }
            P.corner_panel.push_back((uint32_t)P.corner_items.size());
          }
          P.corner_items.push_back((uint32_t)P.corner_cnt.size());
        }
      }
    }

    // ---- short rows / long rows -------------------------------------------------------------
    for (int64_t p = 0; p < L.n_i; ++p) {
      if (taken[p]) continue;
      const int64_t len = L.rowptr[p + 1] - L.rowptr[p] - P.row_skip(p);
      if (len > short_max) { P.long_rows.push_back((int32_t)p); continue; }
      if (len == 0 && li > 0) continue;
      P.row_pos.push_back((int32_t)p);
    }

    // the rows without entries (level 0 lists them: it stores every row of Y) go last, so that
    // their zero stores do not run between the gathers of the other rows
    if (opt.empty_last && li == 0) {
      std::stable_partition(P.row_pos.begin(), P.row_pos.end(), [&](int32_t p) {
        return L.rowptr[p + 1] - L.rowptr[p] - (int64_t)P.row_skip(p) > 0;
      });
    }

    // ---- items of the long rows, row by row ---------------------------------------------------
    const int64_t n_long = (int64_t)P.long_rows.size();
    P.row_split.assign(n_long, 0);
    std::vector<std::vector<Rec>> per_row(n_long);
#pragma omp parallel
    {
      std::vector<int64_t> cnt, first_rec, seen, part, next_at;
#pragma omp for schedule(dynamic, 64)
      for (int64_t r = 0; r < n_long; ++r) {
        const int32_t p = P.long_rows[r];
        const int64_t len = L.rowptr[p + 1] - L.rowptr[p] - P.row_skip(p);
        const int32_t* cols = L.colpos.data() + L.rowptr[p] + P.row_skip(p);
        std::vector<Rec>& out = per_row[r];
        if (classes > 0 && len >= classes * class_min) {
          // split by column class; where every part starts is found by a second scan
          P.row_split[r] = 1;
          cnt.assign(classes, 0);
          for (int64_t e = 0; e < len; ++e) ++cnt[(cols[e] / gran) % classes];
          first_rec.assign(classes + 1, 0);
          for (int64_t c = 0; c < classes; ++c) {
            const int64_t parts = cnt[c] == 0 ? 0 : (cnt[c] <= piece_max ? 1 : (cnt[c] + chunk_nnz - 1) / chunk_nnz);
            first_rec[c + 1] = first_rec[c] + parts;
          }
          out.resize(first_rec[classes]);
          for (int64_t c = 0; c < classes; ++c) {
            const int64_t parts = first_rec[c + 1] - first_rec[c];
            if (parts == 0) continue;
            const int64_t base = cnt[c] / parts, extra = cnt[c] % parts;
            for (int64_t j = 0; j < parts; ++j) {
              Rec& rc = out[first_rec[c] + j];
              rc.row = p; rc.len = (uint32_t)(base + (j < extra ? 1 : 0)); rc.dst = 0;
              rc.phase = (uint32_t)(c / kDies); rc.queue = (int8_t)(c % kDies); rc.key = 0; rc.seq = 0;
              rc.list = cnt[c] <= piece_max ? 0 : 1;
            }
          }
          seen.assign(classes, 0); part.assign(classes, 0); next_at.assign(classes, 0);
          for (int64_t e = 0; e < len; ++e) {
            const int64_t c = (cols[e] / gran) % classes;
            if (seen[c] == next_at[c]) {
              Rec& rc = out[first_rec[c] + part[c]];
              rc.key = (uint32_t)(cols[e] / key_window);
              next_at[c] += rc.len;
              ++part[c];
            }
            ++seen[c];
          }
          // lane-group pieces run several to a wavefront: order them by length (longest first)
          // so that the pieces sharing a wavefront finish together
          for (Rec& rc : out) if (rc.list == 0) rc.key = 0xffffu - (rc.len > 0xffffu ? 0xffffu : rc.len);
        } else {
          int64_t s0 = 0;
          while (s0 < len) {
            int64_t e0 = len;
            if (window > 0) {
              e0 = s0;
              do {
                const int64_t lim = ((int64_t)cols[e0] / window + 1) * window;
                e0 = std::lower_bound(cols + e0, cols + len, lim,
                                      [](int32_t c, int64_t v) { return (int64_t)c < v; }) - cols;
              } while (e0 < len && e0 - s0 < chunk_min);
              if (len - e0 < (chunk_min + 1) / 2) e0 = len;        // absorb a small tail
            }
            const int64_t piece = e0 - s0;
            if (piece <= piece_max) {                              // a lane group is enough for it
              Rec rc;
              rc.row = p; rc.len = (uint32_t)piece; rc.dst = 0;
              rc.phase = class_phases;
              rc.queue = -1; rc.list = 0; rc.key = (uint32_t)(cols[s0] / key_window); rc.seq = 0;
              out.push_back(rc);
              s0 = e0;
              continue;
            }
            const int64_t parts = (piece + chunk_nnz - 1) / chunk_nnz;
            const int64_t base = piece / parts, extra = piece % parts;
            int64_t at_row = s0;
            for (int64_t j = 0; j < parts; ++j) {
              const int64_t sz = base + (j < extra ? 1 : 0);
              Rec rc;
              rc.row = p; rc.len = (uint32_t)sz; rc.dst = 0;
              rc.phase = class_phases;                             // the last phase
              rc.queue = -1; rc.list = 1; rc.key = (uint32_t)(cols[at_row] / key_window); rc.seq = 0;
              out.push_back(rc);
              at_row += sz;
            }
            s0 = e0;
          }
        }
      }
    }
    // flatten, assign destinations (partial slots of a row are consecutive, in emission order)
    int64_t slots = 0;
    P.split_ptr.push_back(0);
    P.row_first.resize(n_long + 1);
    for (int64_t r = 0; r < n_long; ++r) {
      P.row_first[r] = (int64_t)P.recs.size();
      std::vector<Rec>& out = per_row[r];
      const int32_t p = P.long_rows[r];
      if (out.size() == 1) {
        out[0].dst = L.perm[p];
      } else {
        for (size_t j = 0; j < out.size(); ++j) out[j].dst = (int32_t)(-1 - (slots + (int64_t)j));
        slots += (int64_t)out.size();
        P.split_ptr.push_back((uint32_t)slots);
        P.split_y.push_back(L.perm[p]);
      }
      for (Rec& rc : out) { rc.seq = (uint32_t)P.recs.size(); P.recs.push_back(rc); }
      std::vector<Rec>().swap(out);
    }
    P.row_first[n_long] = (int64_t)P.recs.size();
    if (slots > 0x7fffffffLL) { err = "too many partial slots"; return ARROW_EINVAL; }
    if (P.recs.size() > 0x7fffff00ULL) { err = "too many work items"; return ARROW_EINVAL; }

    // ---- final order of both lists; entry offsets --------------------------------------------
    P.slot_of.assign(P.recs.size(), 0);
    int64_t at = 0;
    int64_t real_items[2] = {0, 0}, part_items[2] = {0, 0}, list_nnz[2] = {0, 0};
    for (int list = 0; list < 2; ++list) {
      const std::vector<uint32_t> fin =
          order_list(P.recs, list, class_phases, list == 0 ? kItemsPerGroupBlock : kChunksPerGroup);
      std::vector<uint32_t>& ptr = P.list_ptr[list];
      std::vector<int32_t>& dst = P.list_dst[list];
      std::vector<int32_t>& irow = P.list_row[list];
      ptr.reserve(fin.size() + (list == 0 ? P.row_pos.size() : 0) + 1);
      dst.reserve(fin.size() + (list == 0 ? P.row_pos.size() : 0));
      irow.reserve(fin.size() + (list == 0 ? P.row_pos.size() : 0));
      const int64_t at0 = at;
      for (size_t s = 0; s < fin.size(); ++s) {
        ptr.push_back((uint32_t)at);
        if (fin[s] == kPad) {
          dst.push_back(INT32_MIN);                  // padding slot: no entries, no output
          irow.push_back(-1);
        } else {
          const Rec& rc = P.recs[fin[s]];
          P.slot_of[rc.seq] = (uint32_t)s;
          dst.push_back(rc.dst);
          irow.push_back(L.perm[rc.row]);
          at += rc.len;
          ++real_items[list];
          if (rc.dst < 0) ++part_items[list];
        }
      }
      if (list == 0) {
        P.piece_slots = (int64_t)fin.size();
        for (int32_t p : P.row_pos) {                // plain short rows follow the class pieces
          ptr.push_back((uint32_t)at);
          dst.push_back(L.perm[p]);
          irow.push_back(L.perm[p]);
          at += L.rowptr[p + 1] - L.rowptr[p] - P.row_skip(p);
          ++real_items[0];
        }
      }
      ptr.push_back((uint32_t)at);
      list_nnz[list] = at - at0;
    }
    if (at + nnz_w + P.nnz_panel + P.nnz_corner != lev_nnz) { err = "work lists do not cover the level"; return ARROW_EINTERNAL; }
    P.wrow_ptr.reserve(P.wrow_pos.size() + 1);
    for (int32_t p : P.wrow_pos) { P.wrow_ptr.push_back((uint32_t)at); at += L.rowptr[p + 1] - L.rowptr[p]; }
    P.wrow_ptr.push_back((uint32_t)at);
    if (!P.panel_pos.empty()) {
      const int64_t n_bins = (int64_t)P.panel_ptr.size() - 1;
      for (int64_t bi = 0; bi < n_bins; ++bi) {
        const uint32_t len = P.panel_ptr[bi + 1];
        P.panel_ptr[bi] = (uint32_t)at;
        at += len;
      }
      P.panel_ptr[n_bins] = (uint32_t)at;
    }
    P.corner_first.reserve(P.corner_cnt.size());
    for (uint32_t c : P.corner_cnt) { P.corner_first.push_back((uint32_t)at); at += c; }

    // ---- staged head: buffer rows in class-major order ------------------------------------------
    if (im.staged) {
      P.stage_perm.resize(head);
      const int64_t ncls = classes > 0 ? classes : 1;
      std::vector<int64_t> cbase(ncls + 1, 0);
      for (int64_t q = 0; q < head; ++q) ++cbase[(q / gran) % ncls + 1];
      for (int64_t c = 0; c < ncls; ++c) cbase[c + 1] += cbase[c];
      im.stage_class_rows = cbase[1];
      for (int64_t q = 0; q < head; ++q) {
        const int64_t c = (q / gran) % ncls;
        const int64_t rank = (q / (gran * ncls)) * gran + q % gran;
        P.stage_perm[cbase[c] + rank] = L.perm[q];
      }
    }

    im.piece_slots = P.piece_slots;
    im.n_rows = (int64_t)P.list_dst[0].size();
    im.n_real_rows = real_items[0];
    im.rows_partials = part_items[0];
    im.nnz_rows = list_nnz[0];
    im.n_chunks = (int64_t)P.list_dst[1].size();
    im.n_real_chunks = real_items[1];
    im.chunks_partials = part_items[1];
    im.nnz_chunks = list_nnz[1];
    im.n_split = (int64_t)P.split_y.size();
    im.n_partials = slots;
    im.n_wtiles = (int64_t)P.wtiles.size();
    im.n_wrows = (int64_t)P.wrow_pos.size();
    im.nnz_w = nnz_w;
    im.n_panel_rows = P.n_panel_rows;
    im.n_panel_groups = (int64_t)P.panel_pos.size() / kPanelRows;
    im.n_panel_bins = im.n_panel_groups * kDies * kPanelBins;
    if (im.n_panel_groups * kPanelRows > img.max_panel_slots) img.max_panel_slots = im.n_panel_groups * kPanelRows;
    im.nnz_panel = P.nnz_panel;
    im.corner = P.corner;
    im.nnz_corner = P.nnz_corner;
    im.n_corner_tiles = (int64_t)P.corner_cnt.size();
    im.n_corner_items = P.corner_items.empty() ? 0 : (int64_t)P.corner_items.size() - 1;
    if (im.n_corner_items > img.max_corner_items) img.max_corner_items = im.n_corner_items;
    if (slots > img.max_partials) img.max_partials = slots;

    im.off_perm = total;        total = align_up(total + sizeof(int32_t) * (size_t)L.n_i);
    im.off_stage_perm = total;  total = align_up(total + sizeof(int32_t) * (size_t)im.n_stage);
    im.off_rows_ptr = total;    total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_rows + 1));
    im.off_rows_mid = total;    total = align_up(total + sizeof(uint32_t) * (size_t)im.n_rows);
    im.off_rows_dst = total;    total = align_up(total + sizeof(int32_t) * (size_t)im.n_rows);
    im.off_rows_row = total;    total = align_up(total + sizeof(int32_t) * (size_t)im.n_rows);
    im.off_chunk_ptr = total;   total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_chunks + 1));
    im.off_chunk_mid = total;   total = align_up(total + sizeof(uint32_t) * (size_t)im.n_chunks);
    im.off_chunk_dst = total;   total = align_up(total + sizeof(int32_t) * (size_t)im.n_chunks);
    im.off_chunk_row = total;   total = align_up(total + sizeof(int32_t) * (size_t)im.n_chunks);
    im.off_split_ptr = total;   total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_split + 1));
    im.off_split_y = total;     total = align_up(total + sizeof(int32_t) * (size_t)im.n_split);
    im.off_wtiles = total;      total = align_up(total + sizeof(WindowTile) * (size_t)im.n_wtiles);
    im.off_wrow_ptr = total;    total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_wrows + 1));
    im.off_wrow_mid = total;    total = align_up(total + sizeof(uint32_t) * (size_t)im.n_wrows);
    im.off_wrow_y = total;      total = align_up(total + sizeof(int32_t) * (size_t)im.n_wrows);
    im.off_wrow_win = total;    total = align_up(total + sizeof(uint32_t) * (size_t)im.n_wrows);
    im.off_panel_ptr = total;   total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_panel_bins + 1));
    im.off_panel_y = total;     total = align_up(total + sizeof(int32_t) * (size_t)im.n_panel_groups * kPanelRows);
    im.off_corner_tiles = total; total = align_up(total + sizeof(uint32_t) * (size_t)im.n_corner_tiles * kCornerTileWords);
    im.off_corner_items = total; total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_corner_items + 1));
    im.off_corner_panel = total; total = align_up(total + sizeof(uint32_t) * (size_t)(im.corner / kCornerTile + 1));
    im.off_corner_y = total;     total = align_up(total + sizeof(int32_t) * (size_t)im.corner);
    im.off_entries = total;     total = align_up(total + sizeof(Entry) * (size_t)lev_nnz);
    im.map_offset = map_total;  map_total += lev_nnz;
    img.levels.push_back(im);
  }

  try {
    img.bytes.assign(total, 0);
    img.entry_src.clear();
    img.entry_src.assign((size_t)map_total, 0);
  } catch (const std::bad_alloc&) {
    err = "out of host memory while packing the image";
    return ARROW_ENOMEM;
  }
  unsigned char* base = img.bytes.data();
  for (size_t li = 0; li < levels.size(); ++li) {
    const HostLevel& L = levels[li];
    const Plan& P = plans[li];
    LevelImage& im = img.levels[li];
    std::memcpy(base + im.off_perm, L.perm.data(), sizeof(int32_t) * (size_t)L.n_i);
    if (im.n_stage) std::memcpy(base + im.off_stage_perm, P.stage_perm.data(), sizeof(int32_t) * (size_t)im.n_stage);
    std::memcpy(base + im.off_rows_ptr, P.list_ptr[0].data(), sizeof(uint32_t) * P.list_ptr[0].size());
    std::memcpy(base + im.off_chunk_ptr, P.list_ptr[1].data(), sizeof(uint32_t) * P.list_ptr[1].size());
    if (im.n_rows) std::memcpy(base + im.off_rows_dst, P.list_dst[0].data(), sizeof(int32_t) * (size_t)im.n_rows);
    if (im.n_chunks) std::memcpy(base + im.off_chunk_dst, P.list_dst[1].data(), sizeof(int32_t) * (size_t)im.n_chunks);
    if (im.n_rows) std::memcpy(base + im.off_rows_row, P.list_row[0].data(), sizeof(int32_t) * (size_t)im.n_rows);
    if (im.n_chunks) std::memcpy(base + im.off_chunk_row, P.list_row[1].data(), sizeof(int32_t) * (size_t)im.n_chunks);
    uint32_t* emap = img.entry_src.data() + im.map_offset;
    std::memcpy(base + im.off_split_ptr, P.split_ptr.data(), sizeof(uint32_t) * P.split_ptr.size());
    if (!P.split_y.empty())
      std::memcpy(base + im.off_split_y, P.split_y.data(), sizeof(int32_t) * P.split_y.size());
    uint32_t* list_mid[2] = {reinterpret_cast<uint32_t*>(base + im.off_rows_mid),
                             reinterpret_cast<uint32_t*>(base + im.off_chunk_mid)};
    Entry* ent = reinterpret_cast<Entry*>(base + im.off_entries);
    for (int list = 0; list < 2; ++list) {           // default: no staged entries in the item
      const int64_t cnt = list == 0 ? im.n_rows : im.n_chunks;
      for (int64_t s = 0; s < cnt; ++s) list_mid[list][s] = P.list_ptr[list][s];
    }

    // row of the staging buffer that holds head column position q
    const int64_t ncls = im.classes > 0 ? im.classes : 1;
    const int64_t gran = opt.class_gran < 1 ? 1 : opt.class_gran;
    std::vector<int64_t> cbase(ncls + 1, 0);
    if (im.staged) {
      for (int64_t q = 0; q < im.n_stage; ++q) ++cbase[(q / gran) % ncls + 1];
      for (int64_t c = 0; c < ncls; ++c) cbase[c + 1] += cbase[c];
    }
    auto stage_row = [&](int32_t q) -> int32_t {
      const int64_t c = (q / gran) % ncls;
      const int64_t rank = (q / (gran * ncls)) * gran + q % gran;
      return (int32_t)(cbase[c] + rank);
    };

    // plain short rows: head columns (they come first) read the staged head when the option is on,
    // everything else reads X itself
    const int64_t n_plain = (int64_t)P.row_pos.size();
    // automatic: yes when the head vertices are scattered over X (then the staged copy, which the
    // long rows have just read, is the better-cached one: 3.51 -> 3.04 ms for the short rows of the
    // R-MAT workload), no when they already sit close together in X (a second copy of the same
    // rows then only takes cache space: +5 % on the Chung-Lu workload, whose head is the low ids)
    bool stage_short = im.staged && opt.stage_short > 0;
    if (im.staged && opt.stage_short < 0) {
      constexpr int64_t kBlockRows = 4096;
      std::vector<uint8_t> touched((size_t)((n + kBlockRows - 1) / kBlockRows), 0);
      for (int64_t q = 0; q < im.n_stage; ++q) touched[(size_t)(L.perm[q] / kBlockRows)] = 1;
      int64_t blocks = 0;
      for (uint8_t t : touched) blocks += t;
      stage_short = blocks > 4 * ((im.n_stage + kBlockRows - 1) / kBlockRows);
    }
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t r = 0; r < n_plain; ++r) {
      const int32_t p = P.row_pos[r];
      int64_t src = L.rowptr[p] + P.row_skip(p);
      const int64_t slot = P.piece_slots + r;
      uint32_t staged_here = 0;
      for (uint32_t e = P.list_ptr[0][slot]; e < P.list_ptr[0][slot + 1]; ++e, ++src) {
        const int32_t q = L.colpos[src];
        if (stage_short && q < im.n_stage) { ent[e].xrow = stage_row(q); ++staged_here; }
        else ent[e].xrow = L.perm[q];
        ent[e].val = L.vals[src];
        emap[e] = L.src[src];
      }
      list_mid[0][slot] = P.list_ptr[0][slot] + staged_here;
    }
    // long rows: items in emission order
    const int64_t n_long = (int64_t)P.long_rows.size();
    const int64_t classes = im.classes;
#pragma omp parallel
    {
      std::vector<int64_t> fill;
      std::vector<int64_t> bucket;
#pragma omp for schedule(dynamic, 16)
      for (int64_t r = 0; r < n_long; ++r) {
        const int32_t p = P.long_rows[r];
        const int64_t len = L.rowptr[p + 1] - L.rowptr[p] - P.row_skip(p);
        const int64_t src0 = L.rowptr[p] + P.row_skip(p);
        const int32_t* cols = L.colpos.data() + src0;
        const int64_t rec0 = P.row_first[r], rec1 = P.row_first[r + 1];
        const int64_t* seq = nullptr;
        if (P.row_split[r]) {                        // the row's entries class by class
          fill.assign(classes + 1, 0);
          for (int64_t e = 0; e < len; ++e) ++fill[(cols[e] / gran) % classes + 1];
          for (int64_t c = 0; c < classes; ++c) fill[c + 1] += fill[c];
          bucket.resize(len);
          for (int64_t e = 0; e < len; ++e) bucket[fill[(cols[e] / gran) % classes]++] = e;
          seq = bucket.data();
        }
        int64_t k_in_row = 0;
        for (int64_t rc = rec0; rc < rec1; ++rc) {
          const int list = P.recs[rc].list;
          const uint32_t slot = P.slot_of[rc];
          uint32_t e_out = P.list_ptr[list][slot];
          const uint32_t e_end = P.list_ptr[list][slot + 1];
          uint32_t staged_here = 0;
          for (; e_out < e_end; ++e_out, ++k_in_row) {
            const int64_t e = seq ? seq[k_in_row] : k_in_row;
            const int32_t q = cols[e];
            if (im.staged && q < im.n_stage) {       // head column: comes before every other column
              ent[e_out].xrow = stage_row(q);
              ++staged_here;
            } else {
              ent[e_out].xrow = L.perm[q];
            }
            ent[e_out].val = L.vals[src0 + e];
            emap[e_out] = L.src[src0 + e];
          }
          list_mid[list][slot] = P.list_ptr[list][slot] + staged_here;
        }
      }
    }
    // window rows: first-block-column entries read X rows, diagonal-block entries carry the
    // column position relative to the tile's window
    if (im.n_wtiles) {
      std::memcpy(base + im.off_wtiles, P.wtiles.data(), sizeof(WindowTile) * P.wtiles.size());
      std::memcpy(base + im.off_wrow_ptr, P.wrow_ptr.data(), sizeof(uint32_t) * P.wrow_ptr.size());
      uint32_t* wmid = reinterpret_cast<uint32_t*>(base + im.off_wrow_mid);
      int32_t* wy = reinterpret_cast<int32_t*>(base + im.off_wrow_y);
      uint32_t* wwin = reinterpret_cast<uint32_t*>(base + im.off_wrow_win);
      const int64_t n_tiles = im.n_wtiles;
#pragma omp parallel for schedule(dynamic, 4)
      for (int64_t t = 0; t < n_tiles; ++t) {
        const WindowTile& T = P.wtiles[t];
        for (uint32_t wr = T.row_begin; wr < T.row_end; ++wr) {
          const int32_t p = P.wrow_pos[wr];
          wy[wr] = L.perm[p];
          wwin[wr] = T.win_begin;
          // entries outside the tile's window (first block column; other blocks when levels are
          // fused) first, then the window entries
          const int64_t w_lo = T.win_begin, w_hi = (int64_t)T.win_begin + T.win_count;
          uint32_t e = P.wrow_ptr[wr];
          for (int64_t src = L.rowptr[p]; src < L.rowptr[p + 1]; ++src) {
            const int32_t q = L.colpos[src];
            if (q >= w_lo && q < w_hi) continue;
            ent[e].xrow = L.perm[q]; ent[e].val = L.vals[src]; emap[e] = L.src[src];
            ++e;
          }
          wmid[wr] = e;
          for (int64_t src = L.rowptr[p]; src < L.rowptr[p + 1]; ++src) {
            const int32_t q = L.colpos[src];
            if (q < w_lo || q >= w_hi) continue;
            ent[e].xrow = q - (int32_t)T.win_begin; ent[e].val = L.vals[src]; emap[e] = L.src[src];
            ++e;
          }
        }
      }
    }
    // head panels: per workgroup (group, class) the class entries of the group's rows, dealt to
    // the streams chosen above; inside a stream ordered by row, then column (the kernel relies on
    // the rows of a stream never going backwards)
    if (im.n_panel_bins) {
      std::memcpy(base + im.off_panel_ptr, P.panel_ptr.data(), sizeof(uint32_t) * P.panel_ptr.size());
      int32_t* py = reinterpret_cast<int32_t*>(base + im.off_panel_y);
      for (size_t s = 0; s < P.panel_pos.size(); ++s) py[s] = P.panel_pos[s] < 0 ? -1 : L.perm[P.panel_pos[s]];
      const int64_t n_groups = im.n_panel_groups;
#pragma omp parallel
      {
        // (stream, row in the group, column) -> level entry
        std::vector<std::pair<uint64_t, int64_t>> keys;
#pragma omp for schedule(dynamic, 4)
        for (int64_t g = 0; g < n_groups; ++g) {
          for (int c = 0; c < kDies; ++c) {
            keys.clear();
            for (int r = 0; r < kPanelRows; ++r) {
              const int32_t p = P.panel_pos[(size_t)g * kPanelRows + r];
              if (p < 0) continue;
              const uint64_t bin = P.panel_bin[((size_t)g * kPanelRows + r) * kDies + c];
              for (int64_t src = L.rowptr[p]; src < L.rowptr[p] + P.skip[p]; ++src) {
                const uint64_t q = (uint64_t)L.colpos[src];
                if (panel_class((uint32_t)q) != c) continue;
                keys.emplace_back((bin << 56) | ((uint64_t)r << 24) | (q & 0xffffffu), src);
              }
            }
            std::sort(keys.begin(), keys.end());
            uint32_t e = P.panel_ptr[((size_t)g * kDies + c) * kPanelBins];
            for (const auto& kv : keys) {
              const uint32_t lrow = (uint32_t)((kv.first >> 24) & 0xffu);
              const int32_t q = L.colpos[kv.second];
              ent[e].xrow = (int32_t)((lrow << kPanelRowShift) | (uint32_t)stage_row(q));
              ent[e].val = L.vals[kv.second];
              emap[e] = L.src[kv.second];
              ++e;
            }
          }
        }
      }
    }
    // dense corner: per row panel the rows' leading entries (columns inside the corner) are dealt
    // to the panel's tiles; inside a tile they stay ordered by row, then column, and are cut into
    // kCornerRuns runs at row boundaries, as equal as the rows allow
    if (im.n_corner_tiles) {
      uint32_t* tw = reinterpret_cast<uint32_t*>(base + im.off_corner_tiles);
      std::memcpy(base + im.off_corner_items, P.corner_items.data(), sizeof(uint32_t) * P.corner_items.size());
      std::memcpy(base + im.off_corner_panel, P.corner_panel.data(), sizeof(uint32_t) * P.corner_panel.size());
      int32_t* cy = reinterpret_cast<int32_t*>(base + im.off_corner_y);
      for (int64_t p = 0; p < im.corner; ++p) cy[p] = L.perm[p];
      const int64_t side = im.corner / kCornerTile;
      // first listed tile of every panel (tiles are listed panel by panel, column tiles ascending)
      std::vector<int64_t> panel_tile((size_t)side + 1, 0);
      for (uint32_t ij : P.corner_ij) ++panel_tile[(size_t)(ij >> 16) + 1];
      for (int64_t i = 0; i < side; ++i) panel_tile[i + 1] += panel_tile[i];
#pragma omp parallel
      {
        std::vector<int64_t> tile_of((size_t)side);       // column tile -> listed tile of this panel, -1 = empty
        std::vector<uint32_t> fill;
#pragma omp for schedule(dynamic, 1)
        for (int64_t ip = 0; ip < side; ++ip) {
          std::fill(tile_of.begin(), tile_of.end(), -1);
          for (int64_t t = panel_tile[ip]; t < panel_tile[ip + 1]; ++t) tile_of[P.corner_ij[t] & 0xffffu] = t;
          fill.assign((size_t)(panel_tile[ip + 1] - panel_tile[ip]), 0);
          for (int64_t r = 0; r < kCornerTile; ++r) {
            const int64_t p = ip * kCornerTile + r;
            int64_t src = L.rowptr[p];
            for (uint32_t e = 0; e < P.skip[p]; ++e, ++src) {
              const int32_t q = L.colpos[src];
              const int64_t t = tile_of[q / kCornerTile];
              const uint32_t at_e = P.corner_first[t] + fill[(size_t)(t - panel_tile[ip])]++;
              ent[at_e].xrow = (int32_t)(((uint32_t)r << 16) | (uint32_t)(q % kCornerTile));
              ent[at_e].val = L.vals[src];
              emap[at_e] = L.src[src];
            }
          }
          for (int64_t t = panel_tile[ip]; t < panel_tile[ip + 1]; ++t) {
            uint32_t* w = tw + (size_t)t * kCornerTileWords;
            const uint32_t first = P.corner_first[t], cnt_t = P.corner_cnt[t];
            // run r starts at the first row boundary at or after r * cnt / kCornerRuns
            uint32_t pos = 0;
            w[0] = first;
            for (int r = 1; r < kCornerRuns; ++r) {
              const uint32_t want = (uint32_t)((uint64_t)cnt_t * (uint64_t)r / kCornerRuns);
              if (pos < want) {
                pos = want;
                while (pos < cnt_t && pos > 0 &&
                       ((uint32_t)ent[first + pos].xrow >> 16) == ((uint32_t)ent[first + pos - 1].xrow >> 16)) ++pos;
              }
              w[r] = first + pos;
            }
            w[kCornerRuns] = first + cnt_t;
            w[kCornerRuns + 1] = (P.corner_ij[t] & 0xffffu) * kCornerTile;   // first staged head row of the tile
            w[kCornerRuns + 2] = P.corner_ij[t] >> 16;                       // row panel
          }
        }
      }
    }
    // distinct X rows per list (what each kernel must read at least once)
    std::vector<uint8_t> seen((size_t)n, 0);
    for (int list = 0; list < 2; ++list) {
      std::fill(seen.begin(), seen.end(), 0);
      const int64_t cnt_items = list == 0 ? im.n_rows : im.n_chunks;
      const std::vector<uint32_t>& ptr = P.list_ptr[list];
      const uint32_t* mid = list_mid[list];
#pragma omp parallel for schedule(dynamic, 4096)
      for (int64_t s = 0; s < cnt_items; ++s) {
        for (uint32_t e = ptr[s]; e < mid[s]; ++e) seen[P.stage_perm[ent[e].xrow]] = 1;
        for (uint32_t e = mid[s]; e < ptr[s + 1]; ++e) seen[ent[e].xrow] = 1;
      }
      int64_t cnt = 0;
#pragma omp parallel for schedule(static) reduction(+ : cnt)
      for (int64_t v = 0; v < n; ++v) cnt += seen[v];
      (list == 0 ? im.x_rows_rows : im.x_rows_chunks) = cnt;
    }
  }
  return ARROW_OK;
}

// Consistency of a packed image against the levels it was built from: offsets in range and
// ordered, row ids inside X / the staging buffer / the LDS window, every partial slot written
// by exactly one item and owned by exactly one split row, and every row of a level produced
// exactly once (level 0: every vertex).
int verify_levels(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const Image& img,
                  std::string& err) {
  if (img.levels.size() != levels.size()) { err = "level count differs"; return ARROW_EINTERNAL; }
  const unsigned char* base = img.bytes.data();
  // the entry map is a bijection between the image's entries and the caller's nonzeros
  {
    int64_t total = 0;
    for (const HostLevel& L : levels) total += L.rowptr[L.n_i];
    if ((int64_t)img.entry_src.size() != total) { err = "entry map has the wrong length"; return ARROW_EINTERNAL; }
    std::vector<uint8_t> hit((size_t)total, 0);
    for (uint32_t s : img.entry_src) {
      if ((int64_t)s >= total || hit[s]) { err = "entry map is not a bijection"; return ARROW_EINTERNAL; }
      hit[s] = 1;
    }
  }
  for (size_t li = 0; li < levels.size(); ++li) {
    const HostLevel& L = levels[li];
    const LevelImage& im = img.levels[li];
    const int64_t lev_nnz = L.rowptr[L.n_i];
    const Entry* ent = reinterpret_cast<const Entry*>(base + im.off_entries);
    const uint32_t* emap = img.entry_src.data() + im.map_offset;
    std::vector<int32_t> slot_row(im.n_partials, -1);   // vertex named by the item that fills each partial slot
    std::vector<int32_t> ent_row((size_t)lev_nnz, -1);  // vertex named by the item that holds each entry
    const int32_t* stage_perm = reinterpret_cast<const int32_t*>(base + im.off_stage_perm);
    std::vector<int32_t> produced(n, 0);      // times a Y row is written (directly or by the reduction)
    std::vector<int32_t> slot_writes(im.n_partials, 0);
    std::vector<double> checksum(n, 0.0);     // sum over the row's entries of value * (1 + X row id)
    std::vector<double> slot_sum(im.n_partials, 0.0);
    int64_t covered = 0;
    const uint32_t* ptrs[2] = {reinterpret_cast<const uint32_t*>(base + im.off_rows_ptr),
                               reinterpret_cast<const uint32_t*>(base + im.off_chunk_ptr)};
    const uint32_t* mids[2] = {reinterpret_cast<const uint32_t*>(base + im.off_rows_mid),
                               reinterpret_cast<const uint32_t*>(base + im.off_chunk_mid)};
    const int32_t* dsts[2] = {reinterpret_cast<const int32_t*>(base + im.off_rows_dst),
                              reinterpret_cast<const int32_t*>(base + im.off_chunk_dst)};
    const int32_t* rows_of[2] = {reinterpret_cast<const int32_t*>(base + im.off_rows_row),
                                 reinterpret_cast<const int32_t*>(base + im.off_chunk_row)};
    const int64_t cnts[2] = {im.n_rows, im.n_chunks};
    uint32_t expect = 0;
    for (int list = 0; list < 2; ++list) {
      for (int64_t s = 0; s < cnts[list]; ++s) {
        const uint32_t lo = ptrs[list][s], mid = mids[list][s], hi = ptrs[list][s + 1];
        if (lo != expect || lo > mid || mid > hi || (int64_t)hi > lev_nnz) { err = "item offsets out of order"; return ARROW_EINTERNAL; }
        expect = hi;
        const int32_t dst = dsts[list][s];
        const int32_t row = rows_of[list][s];
        if (dst == INT32_MIN) { if (hi != lo || row != -1) { err = "padding slot with entries"; return ARROW_EINTERNAL; } continue; }
        if (row < 0 || row >= n || (dst >= 0 && dst != row)) { err = "item vertex differs from its Y row"; return ARROW_EINTERNAL; }
        double sum = 0.0;
        for (uint32_t e = lo; e < hi; ++e) {
          int64_t xr = ent[e].xrow;
          if (e < mid) { if (xr < 0 || xr >= im.n_stage) { err = "staged row out of range"; return ARROW_EINTERNAL; } xr = stage_perm[xr]; }
          if (xr < 0 || xr >= n) { err = "X row out of range"; return ARROW_EINTERNAL; }
          sum += (double)ent[e].val * (double)(1 + xr);
          ent_row[e] = row;
        }
        covered += hi - lo;
        if (dst >= 0) {
          if (dst >= n) { err = "Y row out of range"; return ARROW_EINTERNAL; }
          ++produced[dst]; checksum[dst] += sum;
        } else {
          const int64_t slot = -1 - (int64_t)dst;
          if (slot >= im.n_partials) { err = "partial slot out of range"; return ARROW_EINTERNAL; }
          ++slot_writes[slot]; slot_sum[slot] += sum; slot_row[slot] = row;
        }
      }
    }
    // split rows own consecutive slots
    const uint32_t* sp = reinterpret_cast<const uint32_t*>(base + im.off_split_ptr);
    const int32_t* sy = reinterpret_cast<const int32_t*>(base + im.off_split_y);
    if (sp[0] != 0 || (int64_t)sp[im.n_split] != im.n_partials) { err = "split table does not cover the slots"; return ARROW_EINTERNAL; }
    for (int64_t r = 0; r < im.n_split; ++r) {
      if (sp[r] >= sp[r + 1] || sy[r] < 0 || sy[r] >= n) { err = "bad split row"; return ARROW_EINTERNAL; }
      ++produced[sy[r]];
      for (uint32_t sl = sp[r]; sl < sp[r + 1]; ++sl) {
        checksum[sy[r]] += slot_sum[sl];
        if (slot_row[sl] != sy[r]) { err = "a partial's item names another vertex than its split row"; return ARROW_EINTERNAL; }
      }
    }
    for (int64_t sl = 0; sl < im.n_partials; ++sl)
      if (slot_writes[sl] != 1) { err = "a partial slot is not written exactly once"; return ARROW_EINTERNAL; }
    // window tiles
    const WindowTile* wt = reinterpret_cast<const WindowTile*>(base + im.off_wtiles);
    const uint32_t* wp = reinterpret_cast<const uint32_t*>(base + im.off_wrow_ptr);
    const uint32_t* wm = reinterpret_cast<const uint32_t*>(base + im.off_wrow_mid);
    const int32_t* wy = reinterpret_cast<const int32_t*>(base + im.off_wrow_y);
    const uint32_t* ww = reinterpret_cast<const uint32_t*>(base + im.off_wrow_win);
    uint32_t wexpect = 0;
    for (int64_t t = 0; t < im.n_wtiles; ++t) {
      if (wt[t].row_begin != wexpect || wt[t].row_end <= wt[t].row_begin || (int64_t)wt[t].row_end > im.n_wrows ||
          (int64_t)wt[t].win_begin + wt[t].win_count > L.n_i || (int64_t)wt[t].win_count > img.max_window_span) {
        err = "bad window tile"; return ARROW_EINTERNAL;
      }
      wexpect = wt[t].row_end;
      for (uint32_t wr = wt[t].row_begin; wr < wt[t].row_end; ++wr) {
        const uint32_t lo = wp[wr], mid = wm[wr], hi = wp[wr + 1];
        if (lo != expect || lo > mid || mid > hi || (int64_t)hi > lev_nnz) { err = "window row offsets out of order"; return ARROW_EINTERNAL; }
        expect = hi;
        if (wy[wr] < 0 || wy[wr] >= n) { err = "window Y row out of range"; return ARROW_EINTERNAL; }
        if (ww[wr] != wt[t].win_begin) { err = "window row names another window than its tile"; return ARROW_EINTERNAL; }
        ++produced[wy[wr]];
        double sum = 0.0;
        for (uint32_t e = lo; e < hi; ++e) {
          int64_t xr = ent[e].xrow;
          if (e >= mid) {
            if (xr < 0 || xr >= wt[t].win_count) { err = "window column out of range"; return ARROW_EINTERNAL; }
            xr = L.perm[wt[t].win_begin + xr];
          }
          if (xr < 0 || xr >= n) { err = "X row out of range"; return ARROW_EINTERNAL; }
          sum += (double)ent[e].val * (double)(1 + xr);
          ent_row[e] = wy[wr];
        }
        checksum[wy[wr]] += sum;
        covered += hi - lo;
      }
    }
    if (wexpect != (uint32_t)im.n_wrows) { err = "window rows not covered by tiles"; return ARROW_EINTERNAL; }
    // head panels: streams cover their entries in order; an entry names a used accumulator of its
    // group and a staged head row of its workgroup's column class; all entries of one
    // (accumulator, class) sit in one stream; windows never go backwards inside a stream
    if (im.n_panel_bins) {
      const uint32_t* pp = reinterpret_cast<const uint32_t*>(base + im.off_panel_ptr);
      const int32_t* py = reinterpret_cast<const int32_t*>(base + im.off_panel_y);
      if (im.n_panel_bins != im.n_panel_groups * kDies * kPanelBins || !im.staged || im.classes != 0) { err = "bad panel geometry"; return ARROW_EINTERNAL; }
      std::vector<uint8_t> row_seen((size_t)n, 0);
      for (int64_t s = 0; s < im.n_panel_groups * kPanelRows; ++s) {
        if (py[s] == -1) continue;
        if (py[s] < 0 || py[s] >= n || row_seen[py[s]]) { err = "panel accumulator names a bad or repeated Y row"; return ARROW_EINTERNAL; }
        row_seen[py[s]] = 1;
      }
      std::vector<int32_t> owner((size_t)kPanelRows);
      for (int64_t wg = 0; wg < im.n_panel_groups * kDies; ++wg) {
        std::fill(owner.begin(), owner.end(), -1);
        const uint32_t cls = (uint32_t)(wg % kDies);
        for (int j = 0; j < kPanelBins; ++j) {
          const int64_t bin = wg * kPanelBins + j;
          const uint32_t lo = pp[bin], hi = pp[bin + 1];
          if (lo != expect || hi < lo || (int64_t)hi > lev_nnz) { err = "panel stream offsets out of order"; return ARROW_EINTERNAL; }
          expect = hi;
          for (uint32_t e = lo; e < hi; ++e) {
            const uint32_t code = (uint32_t)ent[e].xrow;
            const uint32_t lrow = code >> kPanelRowShift, xs = code & ((1u << kPanelRowShift) - 1);
            if (lrow >= (uint32_t)kPanelRows) { err = "panel entry outside its group's accumulators"; return ARROW_EINTERNAL; }
            if (e > lo && lrow < ((uint32_t)ent[e - 1].xrow >> kPanelRowShift)) { err = "panel stream rows go backwards"; return ARROW_EINTERNAL; }
            if (owner[lrow] >= 0 && owner[lrow] != j) { err = "two panel streams share an accumulator"; return ARROW_EINTERNAL; }
            owner[lrow] = j;
            const int32_t y = py[(wg / kDies) * kPanelRows + lrow];
            if (y < 0) { err = "panel entry names an unused accumulator"; return ARROW_EINTERNAL; }
            if ((int64_t)xs >= im.n_stage || (uint32_t)panel_class(xs) != cls) { err = "panel entry: staged row out of range or of another class"; return ARROW_EINTERNAL; }
            const int64_t xr = stage_perm[xs];
            if (xr < 0 || xr >= n) { err = "X row out of range"; return ARROW_EINTERNAL; }
            checksum[y] += (double)ent[e].val * (double)(1 + xr);
            ent_row[e] = y;
          }
          covered += hi - lo;
        }
      }
    }
    // dense corner: items and panels partition the tiles; a tile's runs cover its entries in
    // order, never share a row, and every entry names a row of the tile's panel and a staged head
    // row of the tile's column range
    if (im.n_corner_tiles || im.corner) {
      const uint32_t* tw = reinterpret_cast<const uint32_t*>(base + im.off_corner_tiles);
      const uint32_t* items = reinterpret_cast<const uint32_t*>(base + im.off_corner_items);
      const uint32_t* pptr = reinterpret_cast<const uint32_t*>(base + im.off_corner_panel);
      const int32_t* cy = reinterpret_cast<const int32_t*>(base + im.off_corner_y);
      const int64_t side = im.corner / kCornerTile;
      if (im.corner % kCornerTile || im.corner > im.n_stage || !im.staged || im.classes != 0 || side < 1 ||
          im.n_corner_items < 1 || im.n_corner_items > img.max_corner_items) { err = "bad corner geometry"; return ARROW_EINTERNAL; }
      for (int64_t p = 0; p < im.corner; ++p)
        if (cy[p] != L.perm[p]) { err = "corner row table differs from the permutation"; return ARROW_EINTERNAL; }
      if (items[0] != 0 || (int64_t)items[im.n_corner_items] != im.n_corner_tiles || pptr[0] != 0 ||
          (int64_t)pptr[side] != im.n_corner_items) { err = "corner items do not cover the tiles"; return ARROW_EINTERNAL; }
      for (int64_t ip = 0; ip < side; ++ip) {
        if (pptr[ip] > pptr[ip + 1]) { err = "corner panel table not monotone"; return ARROW_EINTERNAL; }
        for (uint32_t it = pptr[ip]; it < pptr[ip + 1]; ++it) {
          if (items[it] >= items[it + 1]) { err = "empty corner item"; return ARROW_EINTERNAL; }
          for (uint32_t t = items[it]; t < items[it + 1]; ++t) {
            const uint32_t* w = tw + (size_t)t * kCornerTileWords;
            const uint32_t col0 = w[kCornerRuns + 1];
            if (w[kCornerRuns + 2] != (uint32_t)ip || col0 % kCornerTile || (int64_t)col0 + kCornerTile > im.corner ||
                (t > items[pptr[ip]] && col0 <= tw[(size_t)(t - 1) * kCornerTileWords + kCornerRuns + 1])) {
              err = "corner tile in the wrong panel or out of order"; return ARROW_EINTERNAL;
            }
            if (w[0] != expect) { err = "corner tile offsets out of order"; return ARROW_EINTERNAL; }
            int64_t last_row = -1;
            for (int r = 0; r < kCornerRuns; ++r) {
              const uint32_t lo = w[r], hi = w[r + 1];
              if (hi < lo || (int64_t)hi > lev_nnz) { err = "corner run offsets out of order"; return ARROW_EINTERNAL; }
              for (uint32_t e = lo; e < hi; ++e) {
                const uint32_t code = (uint32_t)ent[e].xrow;
                const int64_t row = code >> 16, col = code & 0xffffu;
                if (row >= kCornerTile || col >= kCornerTile) { err = "corner entry outside its tile"; return ARROW_EINTERNAL; }
                if (e == lo ? row <= last_row
                            : (row < last_row || (row == last_row && col <= (int64_t)((uint32_t)ent[e - 1].xrow & 0xffffu)))) {
                  err = "corner runs share a row or are not ordered"; return ARROW_EINTERNAL;
                }
                last_row = row;
                const int32_t y = cy[ip * kCornerTile + row];
                const int64_t xr = stage_perm[col0 + col];
                if (xr < 0 || xr >= n) { err = "X row out of range"; return ARROW_EINTERNAL; }
                checksum[y] += (double)ent[e].val * (double)(1 + xr);
                ent_row[e] = y;
              }
              covered += hi - lo;
            }
            expect = w[kCornerRuns];
          }
        }
      }
    }
    {
      // the map sends every image entry to a nonzero of this level with the same value and row
      std::vector<uint32_t> order((size_t)lev_nnz);
      std::vector<int32_t> lev_row((size_t)lev_nnz);
      for (int64_t p = 0; p < L.n_i; ++p)
        for (int64_t e = L.rowptr[p]; e < L.rowptr[p + 1]; ++e) lev_row[e] = L.perm[p];
      for (int64_t e = 0; e < lev_nnz; ++e) order[e] = (uint32_t)e;
      std::sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return L.src[x] < L.src[y]; });
      for (int64_t e = 0; e < lev_nnz; ++e) {
        auto it = std::lower_bound(order.begin(), order.end(), emap[e],
                                   [&](uint32_t x, uint32_t key) { return L.src[x] < key; });
        if (it == order.end() || L.src[*it] != emap[e] || lev_row[*it] != ent_row[e] ||
            std::memcmp(&L.vals[*it], &ent[e].val, sizeof(float)) != 0) {
          err = "entry map points at a nonzero with another value or row"; return ARROW_EINTERNAL;
        }
      }
    }
    if (covered != lev_nnz) { err = "entries not covered exactly once"; return ARROW_EINTERNAL; }
    // every row of the level produced exactly once, with the right entries
    for (int64_t p = 0; p < L.n_i; ++p) {
      const int32_t v = L.perm[p];
      const int64_t len = L.rowptr[p + 1] - L.rowptr[p];
      const int want = (li == 0 || len > 0) ? 1 : 0;
      if (produced[v] != want) { err = "a row of Y is not produced exactly once"; return ARROW_EINTERNAL; }
      double sum = 0.0;
      for (int64_t e = L.rowptr[p]; e < L.rowptr[p + 1]; ++e)
        sum += (double)L.vals[e] * (double)(1 + L.perm[L.colpos[e]]);
      const double tol = 1e-9 * (1.0 + std::abs(sum)) * (double)(len + 1);
      if (std::abs(sum - checksum[v]) > tol) { err = "a row's entries differ between level and image"; return ARROW_EINTERNAL; }
      produced[v] = 0;
    }
    for (int64_t v = 0; v < n; ++v) if (produced[v] != 0) { err = "a vertex outside the level is written"; return ARROW_EINTERNAL; }
    (void)b;
  }
  return ARROW_OK;
}

}  // namespace

int pack_image(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const PackOptions& opt,
               Image& img, std::string& err) {
  img.fused = false;
  if (opt.fuse_levels && levels.size() > 1 && levels[0].n_i == n) {
    std::vector<HostLevel> exec;
    std::vector<int64_t> fused_from;
    int64_t total = 0;
    for (const HostLevel& L : levels) total += L.rowptr[L.n_i];
    if (total < 0xffffffffLL - 4096) {
      fuse_levels(levels, exec, fused_from);
      const int rc = pack_levels(n, b, exec, opt, img, err);
      if (rc != ARROW_OK) return rc;
      img.fused = true;
      for (size_t li = 1; li < levels.size(); ++li) img.levels[0].nnz_fused += fused_from[li];
      return ARROW_OK;
    }
  }
  return pack_levels(n, b, levels, opt, img, err);
}

int verify_image(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const Image& img,
                 std::string& err) {
  if (!img.fused) return verify_levels(n, b, levels, img, err);
  // fused levels: the execution form must hold, vertex by vertex, exactly the entries of all
  // levels (same count, same nonzeros of the caller's arrays, same value bits, same column
  // vertex), and the image must match the execution form
  std::vector<HostLevel> exec;
  std::vector<int64_t> fused_from;
  fuse_levels(levels, exec, fused_from);
  const HostLevel& E = exec[0];
  if (E.n_i != n) { err = "fused level 0 does not cover every vertex"; return ARROW_EINTERNAL; }
  int64_t total = 0;
  for (const HostLevel& L : levels) total += L.rowptr[L.n_i];
  if (E.rowptr[E.n_i] != total) { err = "fused level holds another number of entries"; return ARROW_EINTERNAL; }
  // nonzero of the caller's arrays -> (row vertex, column vertex, value bits), from the levels
  std::vector<int32_t> src_row((size_t)total, -1), src_col((size_t)total, -1);
  std::vector<uint32_t> src_bits((size_t)total, 0);
  for (const HostLevel& L : levels)
    for (int64_t p = 0; p < L.n_i; ++p)
      for (int64_t e = L.rowptr[p]; e < L.rowptr[p + 1]; ++e) {
        const uint32_t s = L.src[e];
        if ((int64_t)s >= total || src_row[s] != -1) { err = "levels: source indices are not a bijection"; return ARROW_EINTERNAL; }
        src_row[s] = L.perm[p]; src_col[s] = L.perm[L.colpos[e]];
        std::memcpy(&src_bits[s], &L.vals[e], sizeof(uint32_t));
      }
  std::vector<uint8_t> hit((size_t)total, 0);
  for (int64_t p = 0; p < E.n_i; ++p)
    for (int64_t e = E.rowptr[p]; e < E.rowptr[p + 1]; ++e) {
      const uint32_t s = E.src[e];
      uint32_t bits;
      std::memcpy(&bits, &E.vals[e], sizeof(uint32_t));
      if ((int64_t)s >= total || hit[s] || src_row[s] != E.perm[p] || src_col[s] != E.perm[E.colpos[e]] ||
          src_bits[s] != bits || (e > E.rowptr[p] && E.colpos[e - 1] >= E.colpos[e])) {
        err = "fused level: an entry differs from the level it came from"; return ARROW_EINTERNAL;
      }
      hit[s] = 1;
    }
  if (img.levels.size() != levels.size() || img.levels[0].nnz_fused != total - levels[0].rowptr[levels[0].n_i]) {
    err = "fused entry count differs"; return ARROW_EINTERNAL;
  }
  return verify_levels(n, b, exec, img, err);
}

}  // namespace arrow
