// Packs the arrow matrices of a decomposition into one flat device image.
//
// Per level the image holds the permutation and two work lists that together
// cover every row position once:
//   row list   - rows with at most short_max entries, in position order (so the
//                rows of one diagonal block are neighbours and share their window
//                of X); a level-0 row without entries is listed too, because
//                level 0 stores every row of Y.
//   chunk list - longer rows cut into chunks of at most chunk_nnz entries; a
//                one-chunk row writes Y directly, a split row writes partial
//                vectors into consecutive slots that the reduction sums in a
//                fixed order.
//
// How the chunk list is laid out is what decides where the X rows of the head
// columns (the window X_0 every block shares) are served from:
//   * Column classes.  Column positions are dealt to `classes` classes in
//     granules of class_gran positions.  A row with enough entries is split by
//     class, and all chunks of class c are placed in workgroup slots that the
//     hardware hands to accelerator die c mod 8 (workgroups go to the 8 dies
//     round-robin by workgroup id).  One die therefore only ever touches 1/classes
//     of X_0 during a phase, a slice small enough to stay resident in its own L2,
//     and every use of an X row outside the head lands on the same die as well.
//     classes / 8 phases follow each other; inside a (phase, die) queue the chunks
//     are ordered by the column window they start in.
//   * Rows too short to split by class keep whole-row chunks cut at column-window
//     boundaries and ordered by window; they form the last phase.
//   * Head staging.  The head rows of P_i X are gathered once per product into a
//     contiguous buffer, class by class, so a die's slice is one contiguous range.
//     Chunk entries of head columns carry the row of that buffer; they come first in
//     every chunk (entries are ordered by column position) and chunk_mid marks where
//     they end.  All other entries carry perm[q]: the permutation gather stays fused.
#include "arrow_internal.h"

#include <omp.h>

#include <algorithm>
#include <cstdint>
#include <cstring>

#include "arrow.h"

namespace arrow {
namespace {

constexpr size_t kAlign = 256;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Rec {
  int32_t row;     // row position, -1 for a padding slot
  uint32_t len;
  int32_t dst;
  uint32_t phase;
  uint32_t key;    // column window of the first entry
  int32_t queue;   // die queue 0..7, or -1 for the window-ordered last phase
  uint32_t seq;    // emission index (keeps the sort stable and names the rec)
};

struct Plan {
  std::vector<int32_t> row_pos;       // positions in the row list
  std::vector<uint32_t> rows_ptr;     // offsets into the level's entries
  std::vector<Rec> recs;              // chunk recs in emission order (row by row)
  std::vector<int64_t> row_first;     // per long row: index of its first rec; parallel to long_rows
  std::vector<int32_t> long_rows;     // positions of the rows in the chunk list
  std::vector<uint8_t> row_split;     // 1 if the row is split by class
  std::vector<uint32_t> slot_of;      // rec seq -> slot in the final chunk list
  std::vector<uint32_t> chunk_ptr;    // final list
  std::vector<int32_t> chunk_dst;
  std::vector<uint32_t> split_ptr;
  std::vector<int32_t> split_y;
  std::vector<int32_t> stage_perm;    // staged head: buffer row -> original X row
  std::vector<WindowTile> wtiles;     // diagonal-block tiles with their X window staged in LDS
  std::vector<int32_t> wrow_pos;      // row positions of the window rows, tile by tile
  std::vector<uint32_t> wrow_ptr;     // offsets of their entries (relative to the level's entries)
};

}  // namespace

int pack_image(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const PackOptions& opt,
               Image& img, std::string& err) {
  img.levels.clear();
  img.max_partials = 0;
  img.max_stage_rows = 0;
  img.max_window_span = 0;
  const int64_t short_max = opt.short_max < 0 ? 0 : opt.short_max;
  const int64_t chunk_nnz = opt.chunk_nnz < 1 ? 1 : opt.chunk_nnz;
  const int64_t chunk_min = opt.chunk_min < 1 ? 1 : (opt.chunk_min > chunk_nnz ? chunk_nnz : opt.chunk_min);
  const int64_t window = opt.window_rows < 0 ? 0 : opt.window_rows;
  const int64_t classes = opt.classes <= 0 ? 0 : (opt.classes + kDies - 1) / kDies * kDies;
  const int64_t gran = opt.class_gran < 1 ? 1 : opt.class_gran;
  const int64_t class_min = opt.class_min < 1 ? 1 : opt.class_min;
  const int64_t key_window = window > 0 ? window : 4096;

  std::vector<Plan> plans(levels.size());
  size_t total = 0;

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
            const int32_t* cd = std::lower_bound(cb, ce, (int32_t)b);     // first diagonal-block entry
            if (cd == ce) continue;                                       // first-block-column entries only
            const int64_t nmin = std::min<int64_t>(cmin, *cd), nmax = std::max<int64_t>(cmax, *(ce - 1));
            if (nmax - nmin + 1 > span_cap) break;
            cmin = nmin; cmax = nmax; dnnz += ce - cd;
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
              taken[p] = 1;
              P.wrow_pos.push_back((int32_t)p);
              nnz_w += len;
            }
            t.row_end = (uint32_t)P.wrow_pos.size();
            if (t.row_end > t.row_begin) {
              P.wtiles.push_back(t);
              if ((int64_t)t.win_count > img.max_window_span) img.max_window_span = t.win_count;
            }
          }
          p0 = p1;
        }
      }
    }

    // ---- row list -------------------------------------------------------------------------
    P.rows_ptr.push_back(0);
    int64_t nnz_rows = 0;
    for (int64_t p = 0; p < L.n_i; ++p) {
      if (taken[p]) continue;
      const int64_t len = L.rowptr[p + 1] - L.rowptr[p];
      if (len > short_max) { P.long_rows.push_back((int32_t)p); continue; }
      if (len == 0 && li > 0) continue;
      P.row_pos.push_back((int32_t)p);
      nnz_rows += len;
      P.rows_ptr.push_back((uint32_t)nnz_rows);
    }

    // ---- chunk recs, row by row -------------------------------------------------------------
    const int64_t n_long = (int64_t)P.long_rows.size();
    P.row_split.assign(n_long, 0);
    std::vector<std::vector<Rec>> per_row(n_long);
#pragma omp parallel
    {
      std::vector<int64_t> cnt, start_col;
#pragma omp for schedule(dynamic, 64)
      for (int64_t r = 0; r < n_long; ++r) {
        const int32_t p = P.long_rows[r];
        const int64_t len = L.rowptr[p + 1] - L.rowptr[p];
        const int32_t* cols = L.colpos.data() + L.rowptr[p];
        std::vector<Rec>& out = per_row[r];
        if (classes > 0 && len >= classes * class_min) {
          // split by column class; chunk starts are found by a second scan
          P.row_split[r] = 1;
          cnt.assign(classes, 0);
          for (int64_t e = 0; e < len; ++e) ++cnt[(cols[e] / gran) % classes];
          // part sizes per class
          std::vector<int64_t> first_rec(classes + 1, 0);
          for (int64_t c = 0; c < classes; ++c)
            first_rec[c + 1] = first_rec[c] + (cnt[c] + chunk_nnz - 1) / chunk_nnz;
          out.resize(first_rec[classes]);
          for (int64_t c = 0; c < classes; ++c) {
            const int64_t parts = first_rec[c + 1] - first_rec[c];
            if (parts == 0) continue;
            const int64_t base = cnt[c] / parts, extra = cnt[c] % parts;
            for (int64_t j = 0; j < parts; ++j) {
              Rec& rc = out[first_rec[c] + j];
              rc.row = p; rc.len = (uint32_t)(base + (j < extra ? 1 : 0)); rc.dst = 0;
              rc.phase = (uint32_t)(c / kDies); rc.queue = (int32_t)(c % kDies); rc.key = 0; rc.seq = 0;
            }
          }
          // second scan: the column where every part starts
          std::vector<int64_t> seen(classes, 0), part(classes, 0), next_at(classes, 0);
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
            const int64_t parts = (piece + chunk_nnz - 1) / chunk_nnz;
            const int64_t base = piece / parts, extra = piece % parts;
            int64_t at_row = s0;
            for (int64_t j = 0; j < parts; ++j) {
              const int64_t sz = base + (j < extra ? 1 : 0);
              Rec rc;
              rc.row = p; rc.len = (uint32_t)sz; rc.dst = 0;
              rc.phase = (uint32_t)(classes / kDies);              // the last phase
              rc.queue = -1; rc.key = (uint32_t)(cols[at_row] / key_window); rc.seq = 0;
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
    if (P.recs.size() > 0x7fffff00ULL) { err = "too many chunks"; return ARROW_EINVAL; }

    // ---- final order: phases, die queues, windows ---------------------------------------------
    const uint32_t n_phases = (uint32_t)(classes / kDies) + 1;
    std::vector<uint32_t> order(P.recs.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = (uint32_t)i;
    std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) {
      const Rec& a = P.recs[x];
      const Rec& c = P.recs[y];
      if (a.phase != c.phase) return a.phase < c.phase;
      if (a.queue != c.queue) return a.queue < c.queue;
      return a.key < c.key;
    });
    // `final_list` holds rec indices, or UINT32_MAX for padding slots
    std::vector<uint32_t> final_list;
    final_list.reserve(order.size() + 64);
    size_t at_o = 0;
    for (uint32_t ph = 0; ph < n_phases; ++ph) {
      if (ph + 1 == n_phases) {                      // last phase: plain window order, no queues
        while (at_o < order.size()) final_list.push_back(order[at_o++]);
        break;
      }
      size_t qbeg[kDies + 1];
      for (int q = 0; q < kDies; ++q) {
        qbeg[q] = at_o;
        while (at_o < order.size() && P.recs[order[at_o]].phase == ph && P.recs[order[at_o]].queue == q) ++at_o;
      }
      qbeg[kDies] = at_o;
      size_t rounds = 0;
      for (int q = 0; q < kDies; ++q) {
        const size_t len_q = qbeg[q + 1] - qbeg[q];
        rounds = std::max(rounds, (len_q + kChunksPerGroup - 1) / kChunksPerGroup);
      }
      for (size_t rd = 0; rd < rounds; ++rd)
        for (int q = 0; q < kDies; ++q)
          for (int j = 0; j < kChunksPerGroup; ++j) {
            const size_t idx = qbeg[q] + rd * kChunksPerGroup + j;
            final_list.push_back(idx < qbeg[q + 1] ? order[idx] : 0xffffffffu);
          }
    }
    P.slot_of.assign(P.recs.size(), 0);
    int64_t at = nnz_rows;
    P.chunk_ptr.reserve(final_list.size() + 1);
    P.chunk_dst.reserve(final_list.size());
    for (size_t s = 0; s < final_list.size(); ++s) {
      P.chunk_ptr.push_back((uint32_t)at);
      if (final_list[s] == 0xffffffffu) {
        P.chunk_dst.push_back(INT32_MIN);            // padding slot: no entries, no output
      } else {
        const Rec& rc = P.recs[final_list[s]];
        P.slot_of[rc.seq] = (uint32_t)s;
        P.chunk_dst.push_back(rc.dst);
        at += rc.len;
      }
    }
    P.chunk_ptr.push_back((uint32_t)at);
    if (at + nnz_w != lev_nnz) { err = "work lists do not cover the level"; return ARROW_EINTERNAL; }
    P.wrow_ptr.reserve(P.wrow_pos.size() + 1);
    for (int32_t p : P.wrow_pos) { P.wrow_ptr.push_back((uint32_t)at); at += L.rowptr[p + 1] - L.rowptr[p]; }
    P.wrow_ptr.push_back((uint32_t)at);

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

    im.n_rows = (int64_t)P.row_pos.size();
    im.nnz_rows = nnz_rows;
    im.n_chunks = (int64_t)P.chunk_dst.size();
    im.n_real_chunks = (int64_t)P.recs.size();
    im.nnz_chunks = lev_nnz - nnz_rows - nnz_w;
    im.n_wtiles = (int64_t)P.wtiles.size();
    im.n_wrows = (int64_t)P.wrow_pos.size();
    im.nnz_w = nnz_w;
    im.n_split = (int64_t)P.split_y.size();
    im.n_partials = slots;
    if (slots > img.max_partials) img.max_partials = slots;

    im.off_perm = total;        total = align_up(total + sizeof(int32_t) * (size_t)L.n_i);
    im.off_stage_perm = total;  total = align_up(total + sizeof(int32_t) * (size_t)im.n_stage);
    im.off_rows_ptr = total;    total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_rows + 1));
    im.off_rows_y = total;      total = align_up(total + sizeof(int32_t) * (size_t)im.n_rows);
    im.off_chunk_ptr = total;   total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_chunks + 1));
    im.off_chunk_mid = total;   total = align_up(total + sizeof(uint32_t) * (size_t)im.n_chunks);
    im.off_chunk_dst = total;   total = align_up(total + sizeof(int32_t) * (size_t)im.n_chunks);
    im.off_split_ptr = total;   total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_split + 1));
    im.off_split_y = total;     total = align_up(total + sizeof(int32_t) * (size_t)im.n_split);
    im.off_wtiles = total;      total = align_up(total + sizeof(WindowTile) * (size_t)im.n_wtiles);
    im.off_wrow_ptr = total;    total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_wrows + 1));
    im.off_wrow_mid = total;    total = align_up(total + sizeof(uint32_t) * (size_t)im.n_wrows);
    im.off_wrow_y = total;      total = align_up(total + sizeof(int32_t) * (size_t)im.n_wrows);
    im.off_entries = total;     total = align_up(total + sizeof(Entry) * (size_t)lev_nnz);
    img.levels.push_back(im);
  }

  try {
    img.bytes.assign(total, 0);
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
    std::memcpy(base + im.off_rows_ptr, P.rows_ptr.data(), sizeof(uint32_t) * P.rows_ptr.size());
    std::memcpy(base + im.off_chunk_ptr, P.chunk_ptr.data(), sizeof(uint32_t) * P.chunk_ptr.size());
    if (!P.chunk_dst.empty())
      std::memcpy(base + im.off_chunk_dst, P.chunk_dst.data(), sizeof(int32_t) * P.chunk_dst.size());
    std::memcpy(base + im.off_split_ptr, P.split_ptr.data(), sizeof(uint32_t) * P.split_ptr.size());
    if (!P.split_y.empty())
      std::memcpy(base + im.off_split_y, P.split_y.data(), sizeof(int32_t) * P.split_y.size());
    int32_t* rows_y = reinterpret_cast<int32_t*>(base + im.off_rows_y);
    uint32_t* chunk_mid = reinterpret_cast<uint32_t*>(base + im.off_chunk_mid);
    Entry* ent = reinterpret_cast<Entry*>(base + im.off_entries);
    for (int64_t c = 0; c < im.n_chunks; ++c) chunk_mid[c] = P.chunk_ptr[c];   // no staged entries yet

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

    const int64_t n_rows = im.n_rows;
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t r = 0; r < n_rows; ++r) {
      const int32_t p = P.row_pos[r];
      rows_y[r] = L.perm[p];
      int64_t src = L.rowptr[p];
      for (uint32_t e = P.rows_ptr[r]; e < P.rows_ptr[r + 1]; ++e, ++src) {
        ent[e].xrow = L.perm[L.colpos[src]];       // the row list always reads X itself
        ent[e].val = L.vals[src];
      }
    }
    const int64_t n_long = (int64_t)P.long_rows.size();
    const int64_t classes = im.classes;
#pragma omp parallel
    {
      std::vector<int64_t> fill;
      std::vector<int64_t> bucket;
#pragma omp for schedule(dynamic, 16)
      for (int64_t r = 0; r < n_long; ++r) {
        const int32_t p = P.long_rows[r];
        const int64_t len = L.rowptr[p + 1] - L.rowptr[p];
        const int64_t src0 = L.rowptr[p];
        const int32_t* cols = L.colpos.data() + src0;
        const int64_t rec0 = P.row_first[r], rec1 = P.row_first[r + 1];
        // the row's entries in emission order
        const int64_t* seq = nullptr;
        if (P.row_split[r]) {
          fill.assign(classes + 1, 0);
          for (int64_t e = 0; e < len; ++e) ++fill[(cols[e] / gran) % classes + 1];
          for (int64_t c = 0; c < classes; ++c) fill[c + 1] += fill[c];
          bucket.resize(len);
          for (int64_t e = 0; e < len; ++e) bucket[fill[(cols[e] / gran) % classes]++] = e;
          seq = bucket.data();
        }
        int64_t k_in_row = 0;
        for (int64_t rc = rec0; rc < rec1; ++rc) {
          const uint32_t slot = P.slot_of[rc];
          uint32_t e_out = P.chunk_ptr[slot];
          const uint32_t e_end = P.chunk_ptr[slot + 1];
          uint32_t staged_here = 0;
          for (; e_out < e_end; ++e_out, ++k_in_row) {
            const int64_t e = seq ? seq[k_in_row] : k_in_row;
            const int32_t q = cols[e];
            if (im.staged && q < im.n_stage) {     // head column: comes before every other column
              ent[e_out].xrow = stage_row(q);
              ++staged_here;
            } else {
              ent[e_out].xrow = L.perm[q];
            }
            ent[e_out].val = L.vals[src0 + e];
          }
          chunk_mid[slot] = P.chunk_ptr[slot] + staged_here;
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
      const int64_t n_tiles = im.n_wtiles;
#pragma omp parallel for schedule(dynamic, 4)
      for (int64_t t = 0; t < n_tiles; ++t) {
        const WindowTile& T = P.wtiles[t];
        for (uint32_t wr = T.row_begin; wr < T.row_end; ++wr) {
          const int32_t p = P.wrow_pos[wr];
          wy[wr] = L.perm[p];
          int64_t src = L.rowptr[p];
          uint32_t e = P.wrow_ptr[wr];
          uint32_t mid = e;
          for (; src < L.rowptr[p + 1]; ++src, ++e) {
            const int32_t q = L.colpos[src];
            if (q < b) { ent[e].xrow = L.perm[q]; mid = e + 1; }
            else ent[e].xrow = q - (int32_t)T.win_begin;
            ent[e].val = L.vals[src];
          }
          wmid[wr] = mid;
        }
      }
    }
    // distinct X rows per list (what each kernel must read at least once)
    std::vector<uint8_t> seen((size_t)n, 0);
    for (int pass = 0; pass < 2; ++pass) {
      const int64_t lo = pass == 0 ? 0 : im.nnz_rows;
      const int64_t hi = pass == 0 ? im.nnz_rows : im.nnz_rows + im.nnz_chunks;
      std::fill(seen.begin(), seen.end(), 0);
      if (pass == 0) {
#pragma omp parallel for schedule(static)
        for (int64_t e = lo; e < hi; ++e) seen[ent[e].xrow] = 1;
      } else {
#pragma omp parallel for schedule(dynamic, 1024)
        for (int64_t c = 0; c < im.n_chunks; ++c) {
          for (uint32_t e = P.chunk_ptr[c]; e < chunk_mid[c]; ++e) seen[P.stage_perm[ent[e].xrow]] = 1;
          for (uint32_t e = chunk_mid[c]; e < P.chunk_ptr[c + 1]; ++e) seen[ent[e].xrow] = 1;
        }
      }
      int64_t cnt = 0;
#pragma omp parallel for schedule(static) reduction(+ : cnt)
      for (int64_t v = 0; v < n; ++v) cnt += seen[v];
      (pass == 0 ? im.x_rows_rows : im.x_rows_chunks) = cnt;
    }
  }
  return ARROW_OK;
}

}  // namespace arrow
