// C boundary: handle lifetime, validation, upload, the level loop of
//   Y = sum_i P_i^T B_i (P_i X)
// and the chained products.  All arithmetic of a product happens in the HIP
// kernels this file launches; nothing here falls back to the CPU.
#include <hip/hip_runtime.h>
#include <omp.h>

#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "arrow.h"
#include "arrow_internal.h"

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

int64_t env_int(const char* name, int64_t dflt) {
  const char* s = std::getenv(name);
  if (!s || !*s) return dflt;
  char* end = nullptr;
  long long v = std::strtoll(s, &end, 10);
  return (end && *end == 0) ? (int64_t)v : dflt;
}

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

enum KernelClass { kRows = 0, kChunks = 1, kReduce = 2, kStage = 3, kWindow = 4, kPanel = 5, kCorner = 6, kClasses = 7 };

struct Span {
  int cls;
  int level;
  hipEvent_t a, b;
};

}  // namespace

struct arrow_handle {
  int64_t n = 0, nnz = 0;
  int32_t b = 0;
  std::vector<arrow::HostLevel> levels;
  arrow::Image img;
  arrow::PackOptions pack;
  arrow::LaunchTuning tuning;
  double decompose_seconds = 0.0;
  // device bindings (caller-owned memory)
  unsigned char* dev = nullptr;
  unsigned char* ws = nullptr;
  size_t ws_bytes = 0;
  const uint32_t* dev_map = nullptr;   // entry map (sampled product only)
  bool sddmm_image_order = false;
  // profiling
  bool profiling = false;
  std::vector<Span> spans;   // event pool, reused between products
  size_t spans_used = 0;
};

namespace {

// workspace layout: [partial vectors][staged head rows][panel class results][corner item results]
//                   [n x k buffer of the chained products]
size_t partial_bytes(const arrow_handle* h, int32_t k) {
  return align_up((size_t)h->img.max_partials * (size_t)k * sizeof(float));
}
size_t stage_bytes(const arrow_handle* h, int32_t k) {
  return align_up((size_t)h->img.max_stage_rows * (size_t)k * sizeof(float));
}

size_t panel_bytes(const arrow_handle* h, int32_t k) {
  return align_up((size_t)h->img.max_panel_slots * arrow::kDies * (size_t)k * sizeof(float));
}

size_t corner_bytes(const arrow_handle* h, int32_t k) {
  return align_up((size_t)h->img.max_corner_items * arrow::kCornerTile * (size_t)k * sizeof(float));
}

// everything a product keeps outside X and Y
size_t scratch_bytes(const arrow_handle* h, int32_t k) {
  return partial_bytes(h, k) + stage_bytes(h, k) + panel_bytes(h, k) + corner_bytes(h, k);
}

template <typename T>
const T* at(const arrow_handle* h, size_t off) {
  return reinterpret_cast<const T*>(h->dev + off);
}

// start/stop one profiled launch
struct Scoped {
  arrow_handle* h;
  hipStream_t s;
  Span* sp = nullptr;
  Scoped(arrow_handle* h_, int cls, int level, hipStream_t s_, bool allowed = true) : h(h_), s(s_) {
    if (!h->profiling || !allowed) return;
    if (h->spans_used == h->spans.size()) {
      Span n{cls, level, nullptr, nullptr};
      if (hipEventCreate(&n.a) != hipSuccess || hipEventCreate(&n.b) != hipSuccess) return;
      h->spans.push_back(n);
    }
    sp = &h->spans[h->spans_used++];
    sp->cls = cls;
    sp->level = level;
    (void)hipEventRecord(sp->a, s);
  }
  ~Scoped() {
    if (sp) (void)hipEventRecord(sp->b, s);
  }
};

bool ranges_overlap(const void* a, size_t a_bytes, const void* b, size_t b_bytes) {
  const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a_bytes && b_bytes && a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

// X (read) and Y (written) of a product must be disjoint from each other, from the scratch memory
// the product writes and from the packed image it reads
int check_operands(const arrow_handle* h, const float* X, float* Y, int32_t k, const unsigned char* ws,
                   size_t ws_bytes) {
  if (!X || !Y) return fail(ARROW_EINVAL, "X or Y is NULL");
  if (((uintptr_t)X | (uintptr_t)Y) % 16) return fail(ARROW_EINVAL, "X and Y must be 16-byte aligned");
  const size_t xy = (size_t)h->n * (size_t)k * sizeof(float);
  if (ranges_overlap(X, xy, Y, xy)) return fail(ARROW_EINVAL, "X and Y must not overlap");
  if (ranges_overlap(X, xy, ws, ws_bytes) || ranges_overlap(Y, xy, ws, ws_bytes))
    return fail(ARROW_EINVAL, "X and Y must not overlap the workspace");
  if (ranges_overlap(Y, xy, h->dev, h->img.bytes.size()))
    return fail(ARROW_EINVAL, "Y must not overlap the device image");
  return ARROW_OK;
}

int check_hip(int rc, const char* what) {
  if (rc == 0) return ARROW_OK;
  return fail(ARROW_EHIP, "%s: %s", what, hipGetErrorString((hipError_t)rc));
}

// one product, src -> dst (device, n x k), all levels in stream order.  `ws` holds the partial
// vectors, the staged head and the panel results (the caller's workspace, or the static scratch
// array); every byte of it that a kernel reads has been written earlier in the same product.
// prof = false: no event is created or recorded, whatever the handle's profiling switch says.
int product(arrow_handle* h, const float* X, float* Y, int32_t k, hipStream_t stream,
            unsigned char* ws, bool prof) {
  float* partials = reinterpret_cast<float*>(ws);
  float* stage = reinterpret_cast<float*>(ws + partial_bytes(h, k));
  float* panel_part = reinterpret_cast<float*>(ws + partial_bytes(h, k) + stage_bytes(h, k));
  float* corner_part = reinterpret_cast<float*>(ws + partial_bytes(h, k) + stage_bytes(h, k) + panel_bytes(h, k));
  for (size_t li = 0; li < h->img.levels.size(); ++li) {
    const arrow::LevelImage& im = h->img.levels[li];
    const bool acc = li > 0;
    const arrow::Entry* ent = at<arrow::Entry>(h, im.off_entries);
    const float* Xh = X;
    arrow::LaunchTuning tune = h->tuning;
    if (im.staged) {
      // the first-block-column window X_0 = (P_i X)[0:b], made contiguous once per product
      Scoped sc(h, kStage, (int)li, stream, prof);
      int rc = arrow::launch_gather(at<int32_t>(h, im.off_stage_perm), im.n_stage, X, stage, k, stream);
      if (rc) return check_hip(rc, "head staging launch");
      Xh = stage;
    }
    if (tune.kc == 0) {
      if (im.staged && im.classes > 0) {
        // column slice such that one class of the staged head (one die's share) stays in its 4 MiB L2
        int64_t kc = 256;
        while (kc > 16 && im.stage_class_rows * kc * 4 > tune.l2_resident_bytes) kc >>= 1;
        if (kc < k) tune.kc = (int32_t)kc;
      } else if (im.staged && k > 64) {
        // window-ordered chunks: 64-column passes halve the bytes of a column window, which the
        // L2 hit rate of the head rows gains more from than the second pass over the entries costs
        tune.kc = 64;
      }
    }
    if (im.n_chunks > 0) {
      Scoped sc(h, kChunks, (int)li, stream, prof);
      int rc = arrow::launch_chunks(at<uint32_t>(h, im.off_chunk_ptr), at<uint32_t>(h, im.off_chunk_mid),
                                    at<int32_t>(h, im.off_chunk_dst), ent, im.n_chunks, X, h->n, Xh, Y,
                                    partials, k, acc, tune, stream);
      if (rc) return check_hip(rc, "chunks kernel launch");
    }
    if (im.n_rows > 0) {
      Scoped sc(h, kRows, (int)li, stream, prof);
      // class pieces (die queues) follow the chunk kernel's column slicing; the short rows behind
      // them run in one pass over whole rows
      const int64_t np = im.piece_slots;
      int rc = arrow::launch_rows(at<uint32_t>(h, im.off_rows_ptr), at<uint32_t>(h, im.off_rows_mid),
                                  at<int32_t>(h, im.off_rows_dst), ent, np, X, h->n, Xh, Y, partials, k,
                                  acc, tune, stream);
      if (rc) return check_hip(rc, "rows kernel launch (pieces)");
      rc = arrow::launch_rows(at<uint32_t>(h, im.off_rows_ptr) + np, at<uint32_t>(h, im.off_rows_mid) + np,
                              at<int32_t>(h, im.off_rows_dst) + np, ent, im.n_rows - np, X, h->n, Xh, Y,
                              partials, k, acc, h->tuning, stream);
      if (rc) return check_hip(rc, "rows kernel launch");
    }
    if (im.n_wtiles > 0) {
      Scoped sc(h, kWindow, (int)li, stream, prof);
      int rc = arrow::launch_window(at<arrow::WindowTile>(h, im.off_wtiles), im.n_wtiles,
                                    h->img.max_window_span, at<uint32_t>(h, im.off_wrow_ptr),
                                    at<uint32_t>(h, im.off_wrow_mid), at<int32_t>(h, im.off_wrow_y), ent,
                                    at<int32_t>(h, im.off_perm), X, Y, k, acc, stream);
      if (rc) return check_hip(rc, "window kernel launch");
    }
    if (im.n_split > 0) {
      Scoped sc(h, kReduce, (int)li, stream, prof);
      int rc = arrow::launch_reduce(at<uint32_t>(h, im.off_split_ptr), at<int32_t>(h, im.off_split_y),
                                    im.n_split, partials, Y, k, acc, stream);
      if (rc) return check_hip(rc, "reduce kernel launch");
    }
    if (im.n_panel_groups > 0) {
      // last: the panels add to rows of Y the launches above have stored
      Scoped sc(h, kPanel, (int)li, stream, prof);
      int rc = arrow::launch_panel(at<uint32_t>(h, im.off_panel_ptr), at<int32_t>(h, im.off_panel_y), ent,
                                   im.n_panel_groups, Xh, im.n_stage, panel_part, k, stream);
      if (rc) return check_hip(rc, "panel kernel launch");
      rc = arrow::launch_panel_combine(at<int32_t>(h, im.off_panel_y), im.n_panel_groups * arrow::kPanelRows,
                                       panel_part, Y, k, stream);
      if (rc) return check_hip(rc, "panel combine launch");
    }
    if (im.n_corner_items > 0) {
      // last as well: the corner adds to rows of Y the launches above have stored
      Scoped sc(h, kCorner, (int)li, stream, prof);
      int rc = arrow::launch_corner(at<uint32_t>(h, im.off_corner_tiles), at<uint32_t>(h, im.off_corner_items),
                                    im.n_corner_items, ent, Xh, im.n_stage, corner_part, k, stream);
      if (rc) return check_hip(rc, "corner kernel launch");
      rc = arrow::launch_corner_combine(at<uint32_t>(h, im.off_corner_panel), at<int32_t>(h, im.off_corner_y),
                                        im.corner, corner_part, Y, k, stream);
      if (rc) return check_hip(rc, "corner combine launch");
    }
  }
  return ARROW_OK;
}

// S = A .* (U V^T) on the pattern of A, level by level; every stored entry is written once
int sampled_product(arrow_handle* h, const float* U, const float* V, float* S_out, int32_t k,
                    hipStream_t stream) {
  float* stage = reinterpret_cast<float*>(h->ws + partial_bytes(h, k));
  for (size_t li = 0; li < h->img.levels.size(); ++li) {
    const arrow::LevelImage& im = h->img.levels[li];
    const arrow::Entry* ent = at<arrow::Entry>(h, im.off_entries);
    const uint32_t* emap = h->sddmm_image_order ? nullptr : h->dev_map + im.map_offset;
    float* S = h->sddmm_image_order ? S_out + im.map_offset : S_out;
    const float* Vh = V;
    if (im.staged) {
      Scoped sc(h, kStage, (int)li, stream);
      int rc = arrow::launch_gather(at<int32_t>(h, im.off_stage_perm), im.n_stage, V, stage, k, stream);
      if (rc) return check_hip(rc, "head staging launch");
      Vh = stage;
    }
    if (im.n_chunks > 0) {
      Scoped sc(h, kChunks, (int)li, stream);
      int rc = arrow::launch_sddmm_chunks(at<uint32_t>(h, im.off_chunk_ptr), at<uint32_t>(h, im.off_chunk_mid),
                                          at<int32_t>(h, im.off_chunk_row), ent, emap, im.n_chunks, U, V,
                                          h->n, Vh, S, k, stream);
      if (rc) return check_hip(rc, "sampled chunks kernel launch");
    }
    if (im.n_rows > 0) {
      Scoped sc(h, kRows, (int)li, stream);
      int rc = arrow::launch_sddmm_rows(0, at<uint32_t>(h, im.off_rows_ptr), at<uint32_t>(h, im.off_rows_mid),
                                        at<int32_t>(h, im.off_rows_row), nullptr, nullptr, ent, emap,
                                        im.n_rows, U, V, h->n, Vh, S, k, stream);
      if (rc) return check_hip(rc, "sampled rows kernel launch");
    }
    if (im.n_wrows > 0) {
      Scoped sc(h, kWindow, (int)li, stream);
      int rc = arrow::launch_sddmm_rows(1, at<uint32_t>(h, im.off_wrow_ptr), at<uint32_t>(h, im.off_wrow_mid),
                                        at<int32_t>(h, im.off_wrow_y), at<uint32_t>(h, im.off_wrow_win),
                                        at<int32_t>(h, im.off_perm), ent, emap, im.n_wrows, U, V, h->n,
                                        V, S, k, stream);
      if (rc) return check_hip(rc, "sampled window-rows kernel launch");
    }
    if (im.n_panel_bins > 0) {
      Scoped sc(h, kPanel, (int)li, stream);
      int rc = arrow::launch_sddmm_panel(at<uint32_t>(h, im.off_panel_ptr), at<int32_t>(h, im.off_panel_y),
                                         ent, emap, im.n_panel_bins, U, Vh, im.n_stage, S, k, stream);
      if (rc) return check_hip(rc, "sampled panel kernel launch");
    }
    if (im.n_corner_tiles > 0) {
      Scoped sc(h, kCorner, (int)li, stream);
      int rc = arrow::launch_sddmm_corner(at<uint32_t>(h, im.off_corner_tiles), im.n_corner_tiles,
                                          at<int32_t>(h, im.off_corner_y), ent, emap, U, Vh, im.n_stage, S, k,
                                          stream);
      if (rc) return check_hip(rc, "sampled corner kernel launch");
    }
  }
  return ARROW_OK;
}

// options struct -> the internal option sets of a handle
void apply_options(arrow_handle* h, const arrow_options_t& o, arrow::DecomposeOptions* dopt) {
  if (dopt) {
    dopt->separators = o.separators != 0;
    dopt->bfs_tail = o.bfs_tail != 0;
    dopt->head_by_id = o.head_by_id != 0;
    dopt->hubs_first = o.hubs_first;
  }
  arrow::PackOptions& p = h->pack;
  p.short_max = o.short_max; p.chunk_nnz = o.chunk_nnz; p.chunk_min = o.chunk_min;
  p.window_rows = o.window_rows; p.classes = o.classes; p.class_gran = o.class_gran;
  p.class_min = o.class_min; p.piece_max = o.piece_max; p.stage_head = o.stage_head;
  p.stage_short = o.stage_short; p.empty_last = o.empty_last; p.panel = o.panel; p.panel_min = o.panel_min;
  p.window_span = o.window_span > 4096 ? 4096 : o.window_span;   // 4096 positions x 4 columns x 4 B = 64 KiB of LDS
  p.window_tile_rows = o.window_tile_rows; p.window_reuse = o.window_reuse;
  p.window_level_share = o.window_level_share; p.fuse_levels = o.fuse_levels;
  p.corner = o.corner; p.corner_max = o.corner_max; p.corner_min_tile = o.corner_min_tile;
  h->tuning.kc = o.kc < 0 ? 0 : (o.kc > 256 ? 256 : o.kc);
  h->tuning.l2_resident_bytes = o.l2_resident_bytes < 0 ? 0 : o.l2_resident_bytes;
}

int ready(const arrow_handle* h, int32_t k, bool need_iter_buffer) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  if (k < 1) return fail(ARROW_EINVAL, "k must be >= 1 (got %d)", k);
  if (!h->dev) return fail(ARROW_ENOTREADY, "arrow_upload has not been called");
  if (!h->ws) return fail(ARROW_ENOTREADY, "arrow_set_workspace has not been called");
  size_t need = scratch_bytes(h, k);
  if (need_iter_buffer) need += (size_t)h->n * (size_t)k * sizeof(float);
  if (h->ws_bytes < need)
    return fail(ARROW_ETOOSMALL, "workspace holds %zu bytes, k = %d needs %zu", h->ws_bytes, k, need);
  return ARROW_OK;
}

}  // namespace

// ---- persistence: the levels are written, the device image is rebuilt on load -----------------
namespace {
constexpr char kFileMagic[8] = {'A', 'R', 'R', 'O', 'W', 'L', 'V', '1'};
constexpr char kFileEnd[8] = {'A', 'R', 'R', 'O', 'W', 'E', 'N', 'D'};

template <typename T>
bool put(FILE* f, const T* p, size_t cnt) { return cnt == 0 || std::fwrite(p, sizeof(T), cnt, f) == cnt; }
template <typename T>
bool get(FILE* f, T* p, size_t cnt) { return cnt == 0 || std::fread(p, sizeof(T), cnt, f) == cnt; }

// structural validity of levels read from a file (everything the kernels later rely on)
bool levels_valid(int64_t n, int64_t nnz, int32_t b, const std::vector<arrow::HostLevel>& levels,
                  std::string& why) {
  int64_t total = 0;
  std::vector<uint8_t> seen(n);
  std::vector<uint8_t> used((size_t)nnz, 0);   // every nonzero of the caller's CSR belongs to one entry
  for (size_t li = 0; li < levels.size(); ++li) {
    const arrow::HostLevel& L = levels[li];
    if (L.n_i < 0 || L.n_i > n || (li == 0 && L.n_i != n)) { why = "bad level size"; return false; }
    if ((int64_t)L.perm.size() != L.n_i || (int64_t)L.rowptr.size() != L.n_i + 1) { why = "bad array sizes"; return false; }
    std::fill(seen.begin(), seen.end(), 0);
    for (int64_t p = 0; p < L.n_i; ++p) {
      const int32_t v = L.perm[p];
      if (v < 0 || v >= n || seen[v]) { why = "perm is not an injection into [0, n)"; return false; }
      seen[v] = 1;
    }
    if (L.rowptr[0] != 0) { why = "rowptr[0] != 0"; return false; }
    const int64_t lev_nnz = L.rowptr[L.n_i];
    if (lev_nnz < 0 || (int64_t)L.colpos.size() != lev_nnz || (int64_t)L.vals.size() != lev_nnz ||
        (int64_t)L.src.size() != lev_nnz) { why = "bad entry arrays"; return false; }
    for (int64_t p = 0; p < L.n_i; ++p) {
      if (L.rowptr[p] > L.rowptr[p + 1] || L.rowptr[p + 1] > lev_nnz) { why = "rowptr not monotone"; return false; }
      for (int64_t e = L.rowptr[p]; e < L.rowptr[p + 1]; ++e) {
        const int64_t q = L.colpos[e];
        if (q < 0 || q >= L.n_i || (e > L.rowptr[p] && L.colpos[e - 1] >= q)) { why = "column positions out of range or unordered"; return false; }
        if (!(p < b || q < b || p / b == q / b)) { why = "an entry lies outside the arrow shape"; return false; }
      }
    }
    for (int64_t e = 0; e < lev_nnz; ++e) {
      const uint32_t s = L.src[e];
      if ((int64_t)s >= nnz || used[s]) { why = "source indices are not a bijection onto the nonzeros"; return false; }
      used[s] = 1;
    }
    total += lev_nnz;
  }
  if (total != nnz) { why = "entry count differs from the header"; return false; }
  return true;
}
}  // namespace

extern "C" {

const char* arrow_last_error(void) { return g_err.c_str(); }

void arrow_options_default(arrow_options_t* o) {
  if (!o) return;
  const arrow::DecomposeOptions d;
  const arrow::PackOptions p;
  const arrow::LaunchTuning t;
  // the one place that reads the environment: ARROW_<FIELD> overrides the built-in default
  o->separators = (int32_t)env_int("ARROW_SEPARATORS", d.separators);
  o->bfs_tail = (int32_t)env_int("ARROW_BFS_TAIL", d.bfs_tail);
  o->head_by_id = (int32_t)env_int("ARROW_HEAD_BY_ID", d.head_by_id);
  o->hubs_first = env_int("ARROW_HUBS_FIRST", d.hubs_first);
  o->short_max = (int32_t)env_int("ARROW_SHORT_MAX", p.short_max);
  o->chunk_nnz = (int32_t)env_int("ARROW_CHUNK_NNZ", p.chunk_nnz);
  o->chunk_min = (int32_t)env_int("ARROW_CHUNK_MIN", p.chunk_min);
  o->window_rows = (int32_t)env_int("ARROW_WINDOW_ROWS", p.window_rows);
  o->classes = (int32_t)env_int("ARROW_CLASSES", p.classes);
  o->class_gran = (int32_t)env_int("ARROW_CLASS_GRAN", p.class_gran);
  o->class_min = (int32_t)env_int("ARROW_CLASS_MIN", p.class_min);
  o->piece_max = (int32_t)env_int("ARROW_PIECE_MAX", p.piece_max);
  o->stage_head = (int32_t)env_int("ARROW_STAGE_HEAD", p.stage_head);
  o->stage_short = (int32_t)env_int("ARROW_STAGE_SHORT", p.stage_short);
  o->empty_last = (int32_t)env_int("ARROW_EMPTY_LAST", p.empty_last);
  o->panel = (int32_t)env_int("ARROW_PANEL", p.panel);
  o->panel_min = (int32_t)env_int("ARROW_PANEL_MIN", p.panel_min);
  o->window_span = (int32_t)env_int("ARROW_WINDOW_SPAN", p.window_span);
  o->window_tile_rows = (int32_t)env_int("ARROW_WINDOW_TILE_ROWS", p.window_tile_rows);
  o->window_reuse = (double)env_int("ARROW_WINDOW_REUSE_X10", (int64_t)(p.window_reuse * 10)) / 10.0;
  o->window_level_share = (double)env_int("ARROW_WINDOW_SHARE_X1000", (int64_t)(p.window_level_share * 1000)) / 1000.0;
  o->fuse_levels = (int32_t)env_int("ARROW_FUSE_LEVELS", p.fuse_levels);
  o->corner = (int32_t)env_int("ARROW_CORNER", p.corner);
  o->corner_max = (int32_t)env_int("ARROW_CORNER_MAX", p.corner_max);
  o->corner_min_tile = (int32_t)env_int("ARROW_CORNER_MIN_TILE", p.corner_min_tile);
  o->kc = (int32_t)env_int("ARROW_KC", t.kc);
  o->l2_resident_bytes = env_int("ARROW_L2_RESIDENT_BYTES", t.l2_resident_bytes);
}

int arrow_decompose(int64_t n, const int64_t* rowptr, const int32_t* colidx, const float* vals,
                    int32_t b, arrow_handle** out) {
  return arrow_decompose_with(n, rowptr, colidx, vals, b, nullptr, out);
}

int arrow_decompose_with(int64_t n, const int64_t* rowptr, const int32_t* colidx, const float* vals,
                         int32_t b, const arrow_options_t* opt, arrow_handle** out) {
  if (!out) return fail(ARROW_EINVAL, "out is NULL");
  *out = nullptr;
  if (n < 1 || n > 2147483646LL) return fail(ARROW_EINVAL, "n must be in [1, 2^31 - 2] (got %lld)", (long long)n);
  if (b < 1) return fail(ARROW_EINVAL, "b must be >= 1 (got %d)", b);
  if (!rowptr) return fail(ARROW_EINVAL, "rowptr is NULL");
  if (rowptr[0] != 0) return fail(ARROW_EINVAL, "rowptr[0] must be 0");
  const int64_t nnz = rowptr[n];
  if (nnz < 0 || nnz >= 0xffffffffLL) return fail(ARROW_EINVAL, "nnz must be in [0, 2^32 - 2]");
  if (nnz > 0 && (!colidx || !vals)) return fail(ARROW_EINVAL, "colidx / vals is NULL");
  int64_t bad_row = -1;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    bool ok = rowptr[i] <= rowptr[i + 1] && rowptr[i] >= 0 && rowptr[i + 1] <= nnz;
    if (ok)
      for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
        int32_t c = colidx[p];
        if (c < 0 || c >= n || (p > rowptr[i] && colidx[p - 1] >= c)) { ok = false; break; }
      }
    if (!ok) {
#pragma omp critical
      if (bad_row < 0 || i < bad_row) bad_row = i;
    }
  }
  if (bad_row >= 0)
    return fail(ARROW_EINVAL, "malformed CSR at row %lld (row pointers must not decrease; column ids "
                "must be in range and strictly increasing inside a row)", (long long)bad_row);

  arrow_handle* h = new (std::nothrow) arrow_handle;
  if (!h) return fail(ARROW_ENOMEM, "out of host memory");
  h->n = n; h->nnz = nnz; h->b = b;
  arrow::DecomposeOptions dopt;
  arrow_options_t defaults;
  if (!opt) { arrow_options_default(&defaults); opt = &defaults; }
  apply_options(h, *opt, &dopt);
  std::string err;
  int rc;
  try {
    auto t0 = std::chrono::steady_clock::now();
    rc = arrow::decompose(n, rowptr, colidx, vals, b, dopt, h->levels, err);
    if (rc == ARROW_OK) rc = arrow::pack_image(n, b, h->levels, h->pack, h->img, err);
    h->decompose_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  } catch (const std::bad_alloc&) {
    rc = ARROW_ENOMEM;
    err = "out of host memory during decomposition";
  }
  if (rc != ARROW_OK) {
    delete h;
    return fail(rc, "%s", err.c_str());
  }
  *out = h;
  return ARROW_OK;
}

size_t arrow_device_bytes(const arrow_handle* h) { return h ? h->img.bytes.size() : 0; }

int arrow_upload(arrow_handle* h, void* dev_buf, size_t bytes, void* stream) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  if (!dev_buf) return fail(ARROW_EINVAL, "dev_buf is NULL");
  if ((uintptr_t)dev_buf % kAlign) return fail(ARROW_EINVAL, "dev_buf must be 256-byte aligned");
  if (bytes < h->img.bytes.size())
    return fail(ARROW_ETOOSMALL, "image needs %zu bytes, buffer has %zu", h->img.bytes.size(), bytes);
  if (!h->img.bytes.empty()) {
    hipError_t e = hipMemcpyAsync(dev_buf, h->img.bytes.data(), h->img.bytes.size(),
                                  hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return check_hip((int)e, "image upload");
  }
  h->dev = static_cast<unsigned char*>(dev_buf);
  // set-up on this device: look up the address of its copy of the static scratch array, so that
  // arrow_spmm_static never has to (a failure only matters to that call, which reports it)
  std::string ignored;
  (void)arrow::static_scratch(ignored);
  return ARROW_OK;
}

size_t arrow_workspace_bytes(const arrow_handle* h, int32_t k) {
  if (!h || k < 1) return 0;
  return scratch_bytes(h, k) + align_up((size_t)h->n * (size_t)k * sizeof(float));
}

int arrow_set_workspace(arrow_handle* h, void* dev_ws, size_t bytes) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  if (!dev_ws) return fail(ARROW_EINVAL, "dev_ws is NULL");
  if ((uintptr_t)dev_ws % kAlign) return fail(ARROW_EINVAL, "dev_ws must be 256-byte aligned");
  h->ws = static_cast<unsigned char*>(dev_ws);
  h->ws_bytes = bytes;
  return ARROW_OK;
}

int arrow_spmm(arrow_handle* h, const float* X, float* Y, int32_t k, void* stream) {
  int rc = ready(h, k, false);
  if (rc) return rc;
  rc = check_operands(h, X, Y, k, h->ws, h->ws_bytes);
  if (rc) return rc;
  h->spans_used = 0;
  return product(h, X, Y, k, (hipStream_t)stream, h->ws, true);
}

int arrow_spmm_static(arrow_handle* h, const float* X, float* Y, int32_t k, void* stream) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  if (k < 1) return fail(ARROW_EINVAL, "k must be >= 1 (got %d)", k);
  if (!h->dev) return fail(ARROW_ENOTREADY, "arrow_upload has not been called");
  const size_t need = scratch_bytes(h, k);
  if (need > (size_t)ARROW_STATIC_SCRATCH_BYTES)
    return fail(ARROW_ETOOSMALL, "k = %d needs %zu bytes of scratch, the static array holds %zu; use "
                "arrow_spmm with a workspace", k, need, (size_t)ARROW_STATIC_SCRATCH_BYTES);
  int rc = check_operands(h, X, Y, k, nullptr, 0);
  if (rc) return rc;
  std::string why;
  unsigned char* ws = arrow::static_scratch(why);   // resolved by arrow_upload on this device; a lookup, not an allocation
  if (!ws) return fail(ARROW_EHIP, "%s", why.c_str());
  return product(h, X, Y, k, (hipStream_t)stream, ws, false);
}

int arrow_spmm_iter(arrow_handle* h, float* X, int32_t k, int32_t l, void* stream) {
  if (l < 0) return fail(ARROW_EINVAL, "l must be >= 0 (got %d)", l);
  int rc = ready(h, k, l > 0);
  if (rc) return rc;
  if (!X) return fail(ARROW_EINVAL, "X is NULL");
  if ((uintptr_t)X % 16) return fail(ARROW_EINVAL, "X must be 16-byte aligned");
  if (ranges_overlap(X, (size_t)h->n * (size_t)k * sizeof(float), h->ws, h->ws_bytes) ||
      ranges_overlap(X, (size_t)h->n * (size_t)k * sizeof(float), h->dev, h->img.bytes.size()))
    return fail(ARROW_EINVAL, "X must not overlap the workspace or the device image");
  if (l == 0) return ARROW_OK;
  h->spans_used = 0;
  float* tmp = reinterpret_cast<float*>(h->ws + scratch_bytes(h, k));
  float* src = X;
  float* dst = tmp;
  for (int32_t t = 0; t < l; ++t) {
    rc = product(h, src, dst, k, (hipStream_t)stream, h->ws, true);
    if (rc) return rc;
    float* s = src; src = dst; dst = s;
  }
  if (src != X) {   // odd l: the last product landed in the workspace
    hipError_t e = hipMemcpyAsync(X, src, (size_t)h->n * (size_t)k * sizeof(float),
                                  hipMemcpyDeviceToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return check_hip((int)e, "copy of the last iterate");
  }
  return ARROW_OK;
}

size_t arrow_sddmm_device_bytes(const arrow_handle* h) {
  return h ? align_up(sizeof(uint32_t) * (h->img.entry_src.size() + 1)) : 0;
}

int arrow_sddmm_upload(arrow_handle* h, void* dev_buf, size_t bytes, void* stream) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  if (!dev_buf) return fail(ARROW_EINVAL, "dev_buf is NULL");
  if ((uintptr_t)dev_buf % kAlign) return fail(ARROW_EINVAL, "dev_buf must be 256-byte aligned");
  const size_t need = sizeof(uint32_t) * h->img.entry_src.size();
  if (bytes < need) return fail(ARROW_ETOOSMALL, "entry map needs %zu bytes, buffer has %zu", need, bytes);
  if (need) {
    hipError_t e = hipMemcpyAsync(dev_buf, h->img.entry_src.data(), need, hipMemcpyHostToDevice,
                                  (hipStream_t)stream);
    if (e != hipSuccess) return check_hip((int)e, "entry map upload");
  }
  h->dev_map = static_cast<const uint32_t*>(dev_buf);
  return ARROW_OK;
}

int arrow_sddmm(arrow_handle* h, const float* U, const float* V, float* S, int32_t k, void* stream) {
  int rc = ready(h, k, false);
  if (rc) return rc;
  if (!h->dev_map) return fail(ARROW_ENOTREADY, "arrow_sddmm_upload has not been called");
  if (!U || !V || (!S && h->nnz > 0)) return fail(ARROW_EINVAL, "U, V or S is NULL");
  if (((uintptr_t)U | (uintptr_t)V) % 16) return fail(ARROW_EINVAL, "U and V must be 16-byte aligned");
  if ((uintptr_t)S % 4) return fail(ARROW_EINVAL, "S must be 4-byte aligned");
  h->spans_used = 0;
  return sampled_product(h, U, V, S, k, (hipStream_t)stream);
}

int arrow_export_entry_map(const arrow_handle* h, uint32_t* out) {
  if (!h || (!out && !h->img.entry_src.empty())) return fail(ARROW_EINVAL, "NULL argument");
  if (!h->img.entry_src.empty())
    std::memcpy(out, h->img.entry_src.data(), sizeof(uint32_t) * h->img.entry_src.size());
  return ARROW_OK;
}

int arrow_gather(arrow_handle* h, int32_t level, const float* X, float* Xp, int32_t k, void* stream) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  if (level < 0 || (size_t)level >= h->img.levels.size()) return fail(ARROW_EINVAL, "no level %d", level);
  if (k < 1 || !X || !Xp) return fail(ARROW_EINVAL, "bad X / Xp / k");
  if (((uintptr_t)X | (uintptr_t)Xp) % 16) return fail(ARROW_EINVAL, "X and Xp must be 16-byte aligned");
  if (!h->dev) return fail(ARROW_ENOTREADY, "arrow_upload has not been called");
  const arrow::LevelImage& im = h->img.levels[level];
  int rc = arrow::launch_gather(at<int32_t>(h, im.off_perm), im.n_i, X, Xp, k, stream);
  return check_hip(rc, "gather kernel launch");
}

size_t arrow_probe_gather_out_bytes(int64_t gathers) {
  return gathers < 1 ? 0 : sizeof(float) * (size_t)arrow::probe_out_floats(gathers);
}

int arrow_probe_gather(const float* X, int64_t x_rows, int32_t k, int64_t region_rows, int32_t per_die,
                       int32_t from_lds, int64_t gathers, float* out, size_t out_bytes, void* stream) {
  if (!X || !out) return fail(ARROW_EINVAL, "X or out is NULL");
  if (((uintptr_t)X | (uintptr_t)out) % 16) return fail(ARROW_EINVAL, "X and out must be 16-byte aligned");
  if (gathers < 1 || x_rows < 1) return fail(ARROW_EINVAL, "gathers and x_rows must be >= 1");
  if (out_bytes < arrow_probe_gather_out_bytes(gathers))
    return fail(ARROW_ETOOSMALL, "out needs %zu bytes", arrow_probe_gather_out_bytes(gathers));
  int rc = arrow::launch_probe_gather(X, x_rows, k, region_rows, per_die, from_lds, gathers, out, stream);
  if (rc == (int)hipErrorInvalidValue)
    return fail(ARROW_EINVAL, "k must be a power of two in [4, 256]; the region (x 8 with per_die) must fit "
                "into X, and into 64 KiB with from_lds");
  return check_hip(rc, "gather probe launch");
}

int arrow_info(const arrow_handle* h, arrow_info_t* out) {
  if (!h || !out) return fail(ARROW_EINVAL, "NULL argument");
  out->n = h->n; out->nnz = h->nnz; out->b = h->b;
  out->levels = (int32_t)h->levels.size();
  out->max_chunks = h->img.max_partials;
  out->decompose_seconds = h->decompose_seconds;
  return ARROW_OK;
}

int arrow_level_info(const arrow_handle* h, int32_t level, arrow_level_info_t* out) {
  if (!h || !out) return fail(ARROW_EINVAL, "NULL argument");
  if (level < 0 || (size_t)level >= h->levels.size()) return fail(ARROW_EINVAL, "no level %d", level);
  const arrow::HostLevel& L = h->levels[level];
  const arrow::LevelImage& im = h->img.levels[level];
  out->n_i = L.n_i;
  out->nnz = L.rowptr[L.n_i];
  out->nnz_head_head = L.nnz_head_head; out->nnz_head_row = L.nnz_head_row;
  out->nnz_head_col = L.nnz_head_col; out->nnz_diag = L.nnz_diag;
  out->short_rows = im.n_real_rows; out->chunks = im.n_real_chunks; out->split_rows = im.n_split;
  out->rows_partials = im.rows_partials; out->chunks_partials = im.chunks_partials;
  out->partials = im.n_partials; out->nnz_rows = im.nnz_rows; out->nnz_chunks = im.nnz_chunks;
  out->x_rows_rows = im.x_rows_rows; out->x_rows_chunks = im.x_rows_chunks;
  out->window_tiles = im.n_wtiles; out->window_rows = im.n_wrows; out->nnz_window = im.nnz_w;
  out->panel_rows = im.n_panel_rows; out->panel_bins = im.n_panel_bins; out->nnz_panel = im.nnz_panel;
  out->nnz_fused = im.nnz_fused;
  out->corner = im.corner; out->corner_tiles = im.n_corner_tiles; out->corner_items = im.n_corner_items;
  out->nnz_corner = im.nnz_corner;
  out->blocks = (int32_t)((L.n_i + h->b - 1) / h->b);
  out->separator_rule = L.separator_rule ? 1 : 0;
  return ARROW_OK;
}

int arrow_export_level(const arrow_handle* h, int32_t level, int32_t* perm, int32_t* rows,
                       int32_t* cols, float* vals) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  if (level < 0 || (size_t)level >= h->levels.size()) return fail(ARROW_EINVAL, "no level %d", level);
  const arrow::HostLevel& L = h->levels[level];
  const int64_t nnz = L.rowptr[L.n_i];
  if (perm) std::memcpy(perm, L.perm.data(), sizeof(int32_t) * (size_t)L.n_i);
  if (cols && nnz) std::memcpy(cols, L.colpos.data(), sizeof(int32_t) * (size_t)nnz);
  if (vals && nnz) std::memcpy(vals, L.vals.data(), sizeof(float) * (size_t)nnz);
  if (rows) {
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < L.n_i; ++p)
      for (int64_t e = L.rowptr[p]; e < L.rowptr[p + 1]; ++e) rows[e] = (int32_t)p;
  }
  return ARROW_OK;
}

int arrow_self_check(const arrow_handle* h) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  std::string err;
  int rc = arrow::verify_image(h->n, h->b, h->levels, h->img, err);
  if (rc != ARROW_OK) return fail(rc, "%s", err.c_str());
  return ARROW_OK;
}

int arrow_set_option(arrow_handle* h, const char* name, int64_t value) {
  if (!h || !name) return fail(ARROW_EINVAL, "NULL argument");
  if (!std::strcmp(name, "kc")) {
    if (value < 0 || value > 256) return fail(ARROW_EINVAL, "kc must be in [0, 256]");
    h->tuning.kc = (int32_t)value;
  } else if (!std::strcmp(name, "sddmm_image_order")) {
    h->sddmm_image_order = value != 0;
  } else if (!std::strcmp(name, "l2_resident_bytes")) {
    if (value < 0) return fail(ARROW_EINVAL, "l2_resident_bytes must be >= 0");
    h->tuning.l2_resident_bytes = value;
  } else {
    return fail(ARROW_EINVAL, "unknown option '%s'", name);
  }
  return ARROW_OK;
}

int arrow_set_profiling(arrow_handle* h, int32_t enabled) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  h->profiling = enabled != 0;
  h->spans_used = 0;
  return ARROW_OK;
}

int arrow_get_profile(arrow_handle* h, arrow_profile_t* out) { return arrow_get_level_profile(h, -1, out); }

int arrow_get_level_profile(arrow_handle* h, int32_t level, arrow_profile_t* out) {
  if (!h || !out) return fail(ARROW_EINVAL, "NULL argument");
  if (level >= (int32_t)h->img.levels.size()) return fail(ARROW_EINVAL, "no level %d", level);
  std::memset(out, 0, sizeof *out);
  if (h->spans_used == 0) return fail(ARROW_ENOTREADY, "no profiled product has run");
  hipError_t e = hipEventSynchronize(h->spans[h->spans_used - 1].b);
  if (e != hipSuccess) return check_hip((int)e, "event synchronize");
  float* slot[kClasses] = {&out->rows_ms, &out->chunks_ms, &out->reduce_ms, &out->stage_ms,
                           &out->window_ms, &out->panel_ms, &out->corner_ms};
  int32_t* count[kClasses] = {&out->rows_launches, &out->chunks_launches, &out->reduce_launches,
                              &out->stage_launches, &out->window_launches, &out->panel_launches,
                              &out->corner_launches};
  for (size_t i = 0; i < h->spans_used; ++i) {
    if (level >= 0 && h->spans[i].level != level) continue;
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, h->spans[i].a, h->spans[i].b);
    if (e != hipSuccess) return check_hip((int)e, "event elapsed time");
    *slot[h->spans[i].cls] += ms;
    *count[h->spans[i].cls] += 1;
  }
  e = hipEventElapsedTime(&out->total_ms, h->spans[0].a, h->spans[h->spans_used - 1].b);
  if (e != hipSuccess) return check_hip((int)e, "event elapsed time");
  return ARROW_OK;
}

int arrow_save(const arrow_handle* h, const char* path) {
  if (!h || !path) return fail(ARROW_EINVAL, "NULL argument");
  FILE* f = std::fopen(path, "wb");
  if (!f) return fail(ARROW_EINVAL, "cannot open '%s' for writing", path);
  const uint32_t version = 2;
  const int32_t n_levels = (int32_t)h->levels.size();
  bool ok = put(f, kFileMagic, 8) && put(f, &version, 1) && put(f, &h->n, 1) && put(f, &h->nnz, 1) &&
            put(f, &h->b, 1) && put(f, &n_levels, 1);
  for (const arrow::HostLevel& L : h->levels) {
    if (!ok) break;
    const int64_t lev_nnz = L.rowptr[L.n_i];
    const int64_t stats[4] = {L.nnz_head_head, L.nnz_head_row, L.nnz_head_col, L.nnz_diag};
    const int32_t sep = L.separator_rule ? 1 : 0;
    ok = put(f, &L.n_i, 1) && put(f, &lev_nnz, 1) && put(f, stats, 4) && put(f, &sep, 1) &&
         put(f, L.perm.data(), (size_t)L.n_i) && put(f, L.rowptr.data(), (size_t)L.n_i + 1) &&
         put(f, L.colpos.data(), (size_t)lev_nnz) && put(f, L.vals.data(), (size_t)lev_nnz) &&
         put(f, L.src.data(), (size_t)lev_nnz);
  }
  ok = ok && put(f, kFileEnd, 8);
  if (std::fclose(f) != 0) ok = false;
  if (!ok) return fail(ARROW_EINVAL, "writing '%s' failed", path);
  return ARROW_OK;
}

int arrow_load(const char* path, arrow_handle** out) { return arrow_load_with(path, nullptr, out); }

int arrow_repack(arrow_handle* h, const arrow_options_t* opt) {
  if (!h) return fail(ARROW_EINVAL, "handle is NULL");
  arrow_options_t defaults;
  if (!opt) { arrow_options_default(&defaults); opt = &defaults; }
  apply_options(h, *opt, nullptr);
  h->dev = nullptr; h->ws = nullptr; h->ws_bytes = 0; h->dev_map = nullptr;
  std::string err;
  int rc;
  try {
    rc = arrow::pack_image(h->n, h->b, h->levels, h->pack, h->img, err);
  } catch (const std::bad_alloc&) {
    rc = ARROW_ENOMEM;
    err = "out of host memory while packing";
  }
  if (rc != ARROW_OK) return fail(rc, "%s", err.c_str());
  return ARROW_OK;
}

int arrow_load_with(const char* path, const arrow_options_t* opt, arrow_handle** out) {
  if (!out) return fail(ARROW_EINVAL, "out is NULL");
  *out = nullptr;
  if (!path) return fail(ARROW_EINVAL, "path is NULL");
  FILE* f = std::fopen(path, "rb");
  if (!f) return fail(ARROW_EINVAL, "cannot open '%s'", path);
  arrow_handle* h = new (std::nothrow) arrow_handle;
  if (!h) { std::fclose(f); return fail(ARROW_ENOMEM, "out of host memory"); }
  char magic[8];
  uint32_t version = 0;
  int32_t n_levels = 0;
  std::string why;
  bool ok = get(f, magic, 8) && std::memcmp(magic, kFileMagic, 8) == 0 && get(f, &version, 1) &&
            version == 2 && get(f, &h->n, 1) && get(f, &h->nnz, 1) && get(f, &h->b, 1) && get(f, &n_levels, 1);
  if (ok && (h->n < 1 || h->n > 2147483646LL || h->b < 1 || h->nnz < 0 || h->nnz >= 0xffffffffLL ||
             n_levels < 1 || n_levels > 1000000)) ok = false;
  if (!ok) why = "not an arrow level file (bad header)";
  try {
    for (int32_t li = 0; ok && li < n_levels; ++li) {
      arrow::HostLevel L;
      int64_t lev_nnz = 0, stats[4];
      int32_t sep = 0;
      ok = get(f, &L.n_i, 1) && get(f, &lev_nnz, 1) && get(f, stats, 4) && get(f, &sep, 1) &&
           L.n_i >= 0 && L.n_i <= h->n && lev_nnz >= 0 && lev_nnz <= h->nnz;
      if (!ok) { why = "truncated or corrupt level header"; break; }
      L.perm.resize(L.n_i); L.rowptr.resize(L.n_i + 1); L.colpos.resize(lev_nnz); L.vals.resize(lev_nnz);
      L.src.resize(lev_nnz);
      ok = get(f, L.perm.data(), (size_t)L.n_i) && get(f, L.rowptr.data(), (size_t)L.n_i + 1) &&
           get(f, L.colpos.data(), (size_t)lev_nnz) && get(f, L.vals.data(), (size_t)lev_nnz) &&
           get(f, L.src.data(), (size_t)lev_nnz);
      if (!ok) { why = "truncated level data"; break; }
      L.nnz_head_head = stats[0]; L.nnz_head_row = stats[1]; L.nnz_head_col = stats[2]; L.nnz_diag = stats[3];
      L.separator_rule = sep != 0;
      h->levels.push_back(std::move(L));
    }
    if (ok) { ok = get(f, magic, 8) && std::memcmp(magic, kFileEnd, 8) == 0; if (!ok) why = "missing end marker"; }
    std::fclose(f);
    f = nullptr;
    if (ok) ok = levels_valid(h->n, h->nnz, h->b, h->levels, why);
    if (!ok) { delete h; return fail(ARROW_EINVAL, "'%s': %s", path, why.c_str()); }
    arrow_options_t defaults;
    if (!opt) { arrow_options_default(&defaults); opt = &defaults; }
    apply_options(h, *opt, nullptr);
    std::string err;
    auto t0 = std::chrono::steady_clock::now();
    int rc = arrow::pack_image(h->n, h->b, h->levels, h->pack, h->img, err);
    h->decompose_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    if (rc != ARROW_OK) { delete h; return fail(rc, "%s", err.c_str()); }
  } catch (const std::bad_alloc&) {
    if (f) std::fclose(f);
    delete h;
    return fail(ARROW_ENOMEM, "out of host memory while loading '%s'", path);
  }
  *out = h;
  return ARROW_OK;
}

void arrow_destroy(arrow_handle* h) {
  if (!h) return;
  for (Span& s : h->spans) {
    if (s.a) (void)hipEventDestroy(s.a);
    if (s.b) (void)hipEventDestroy(s.b);
  }
  delete h;
}

}  // extern "C"
