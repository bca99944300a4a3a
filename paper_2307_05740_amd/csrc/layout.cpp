// Packs the arrow matrices of a decomposition into one flat device image.
//
// Per level the image holds the permutation and two work lists that together
// cover every row position once:
//   row list   - rows with at most short_max entries, in position order (so the
//                rows of one diagonal block are neighbours and share their window
//                of X); a level-0 row without entries is listed too, because
//                level 0 stores every row of Y.
//   chunk list - longer rows cut into near-equal chunks of at most chunk_nnz
//                entries; a one-chunk row writes Y directly, a split row writes
//                partial vectors into consecutive slots that the reduction sums.
// Entries carry the X row to read, perm[q], instead of the column position q:
// the permutation gather is fused into the product's loads.  Inside a row the
// entries stay ordered by column position: first-block-column entries (the
// shared window X_0) come first, the row's own diagonal block after them.
#include "arrow_internal.h"

#include <omp.h>

#include <cstring>

#include "arrow.h"

namespace arrow {
namespace {

constexpr size_t kAlign = 256;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

}  // namespace

int pack_image(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const PackOptions& opt,
               Image& img, std::string& err) {
  (void)b;
  img.levels.clear();
  img.max_partials = 0;
  const int64_t short_max = opt.short_max < 0 ? 0 : opt.short_max;
  const int64_t chunk_nnz = opt.chunk_nnz < 1 ? 1 : opt.chunk_nnz;

  struct Plan {
    std::vector<int32_t> row_pos;                 // positions in the row list
    std::vector<uint32_t> rows_ptr;               // offsets into the level's entries
    std::vector<uint32_t> chunk_ptr;              // absolute offsets into the level's entries
    std::vector<int32_t> chunk_dst;
    std::vector<int64_t> chunk_src;               // where in HostLevel the chunk's entries start
    std::vector<uint32_t> split_ptr;
    std::vector<int32_t> split_y;
  };
  std::vector<Plan> plans(levels.size());

  size_t total = 0;
  for (size_t li = 0; li < levels.size(); ++li) {
    const HostLevel& L = levels[li];
    Plan& P = plans[li];
    LevelImage im;
    im.n_i = L.n_i;
    const int64_t lev_nnz = L.rowptr[L.n_i];
    if (lev_nnz >= 0xffffffffLL) { err = "a level holds 2^32 - 1 or more entries"; return ARROW_EINVAL; }
    // pass 1: row list
    P.rows_ptr.push_back(0);
    int64_t nnz_rows = 0;
    for (int64_t p = 0; p < L.n_i; ++p) {
      const int64_t len = L.rowptr[p + 1] - L.rowptr[p];
      if (len > short_max) continue;
      if (len == 0 && li > 0) continue;
      P.row_pos.push_back((int32_t)p);
      nnz_rows += len;
      P.rows_ptr.push_back((uint32_t)nnz_rows);
    }
    // pass 2: chunk list
    int64_t at = nnz_rows;
    int64_t slots = 0;
    P.split_ptr.push_back(0);
    for (int64_t p = 0; p < L.n_i; ++p) {
      const int64_t len = L.rowptr[p + 1] - L.rowptr[p];
      if (len <= short_max) continue;
      const int64_t parts = (len + chunk_nnz - 1) / chunk_nnz;
      const int64_t base = len / parts, extra = len % parts;
      int64_t src = L.rowptr[p];
      for (int64_t c = 0; c < parts; ++c) {
        const int64_t sz = base + (c < extra ? 1 : 0);
        P.chunk_ptr.push_back((uint32_t)at);
        P.chunk_src.push_back(src);
        P.chunk_dst.push_back(parts == 1 ? L.perm[p] : (int32_t)(-1 - (slots + c)));
        at += sz;
        src += sz;
      }
      if (parts > 1) {
        slots += parts;
        P.split_ptr.push_back((uint32_t)slots);
        P.split_y.push_back(L.perm[p]);
      }
    }
    P.chunk_ptr.push_back((uint32_t)at);
    if (at != lev_nnz) { err = "work lists do not cover the level"; return ARROW_EINTERNAL; }
    if (slots > 0x7fffffffLL) { err = "too many partial slots"; return ARROW_EINVAL; }

    im.n_rows = (int64_t)P.row_pos.size();
    im.nnz_rows = nnz_rows;
    im.n_chunks = (int64_t)P.chunk_dst.size();
    im.nnz_chunks = lev_nnz - nnz_rows;
    im.n_split = (int64_t)P.split_y.size();
    im.n_partials = slots;
    if (slots > img.max_partials) img.max_partials = slots;

    im.off_perm = total;        total = align_up(total + sizeof(int32_t) * (size_t)L.n_i);
    im.off_rows_ptr = total;    total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_rows + 1));
    im.off_rows_y = total;      total = align_up(total + sizeof(int32_t) * (size_t)im.n_rows);
    im.off_chunk_ptr = total;   total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_chunks + 1));
    im.off_chunk_dst = total;   total = align_up(total + sizeof(int32_t) * (size_t)im.n_chunks);
    im.off_split_ptr = total;   total = align_up(total + sizeof(uint32_t) * (size_t)(im.n_split + 1));
    im.off_split_y = total;     total = align_up(total + sizeof(int32_t) * (size_t)im.n_split);
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
    std::memcpy(base + im.off_rows_ptr, P.rows_ptr.data(), sizeof(uint32_t) * P.rows_ptr.size());
    std::memcpy(base + im.off_chunk_ptr, P.chunk_ptr.data(), sizeof(uint32_t) * P.chunk_ptr.size());
    if (!P.chunk_dst.empty())
      std::memcpy(base + im.off_chunk_dst, P.chunk_dst.data(), sizeof(int32_t) * P.chunk_dst.size());
    std::memcpy(base + im.off_split_ptr, P.split_ptr.data(), sizeof(uint32_t) * P.split_ptr.size());
    if (!P.split_y.empty())
      std::memcpy(base + im.off_split_y, P.split_y.data(), sizeof(int32_t) * P.split_y.size());
    int32_t* rows_y = reinterpret_cast<int32_t*>(base + im.off_rows_y);
    Entry* ent = reinterpret_cast<Entry*>(base + im.off_entries);
    const int64_t n_rows = im.n_rows;
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t r = 0; r < n_rows; ++r) {
      const int32_t p = P.row_pos[r];
      rows_y[r] = L.perm[p];
      int64_t src = L.rowptr[p];
      for (uint32_t e = P.rows_ptr[r]; e < P.rows_ptr[r + 1]; ++e, ++src) {
        ent[e].xrow = L.perm[L.colpos[src]];
        ent[e].val = L.vals[src];
      }
    }
    const int64_t n_chunks = im.n_chunks;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t c = 0; c < n_chunks; ++c) {
      int64_t src = P.chunk_src[c];
      for (uint32_t e = P.chunk_ptr[c]; e < P.chunk_ptr[c + 1]; ++e, ++src) {
        ent[e].xrow = L.perm[L.colpos[src]];
        ent[e].val = L.vals[src];
      }
    }
    // distinct X rows per list (what each kernel must read at least once)
    std::vector<uint8_t> seen((size_t)n, 0);
    for (int pass = 0; pass < 2; ++pass) {
      const int64_t lo = pass == 0 ? 0 : im.nnz_rows;
      const int64_t hi = pass == 0 ? im.nnz_rows : im.nnz_rows + im.nnz_chunks;
      std::fill(seen.begin(), seen.end(), 0);
#pragma omp parallel for schedule(static)
      for (int64_t e = lo; e < hi; ++e) seen[ent[e].xrow] = 1;
      int64_t cnt = 0;
#pragma omp parallel for schedule(static) reduction(+ : cnt)
      for (int64_t v = 0; v < n; ++v) cnt += seen[v];
      (pass == 0 ? im.x_rows_rows : im.x_rows_chunks) = cnt;
    }
  }
  return ARROW_OK;
}

}  // namespace arrow
