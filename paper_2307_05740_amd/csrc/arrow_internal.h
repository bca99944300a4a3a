// Internal C++ declarations shared by the host decomposition, the image
// packer / C-ABI and the HIP kernel launchers.  Nothing here is exported.
#pragma once

#include <cstddef>
#include <cstdint>
#include <memory>
#include <string>
#include <utility>
#include <vector>

namespace arrow {

// std::vector whose resize() leaves new elements uninitialised: the entry arrays of a level are
// hundreds of megabytes and are filled by parallel loops right after they are sized, so a serial
// zero-fill (and its page faults) would only cost time.
template <typename T>
struct default_init_allocator : std::allocator<T> {
  template <typename U> struct rebind { using other = default_init_allocator<U>; };
  using std::allocator<T>::allocator;
  template <typename U, typename... Args>
  void construct(U* p, Args&&... args) {
    if constexpr (sizeof...(Args) == 0) ::new (static_cast<void*>(p)) U;
    else ::new (static_cast<void*>(p)) U(std::forward<Args>(args)...);
  }
};
template <typename T> using raw_vector = std::vector<T, default_init_allocator<T>>;

// One arrow matrix B_i in position coordinates, CSR by row position.
struct HostLevel {
  int64_t n_i = 0;                 // active vertices of this level
  std::vector<int32_t> perm;       // position -> original vertex id, n_i entries
  std::vector<int64_t> rowptr;     // n_i + 1
  raw_vector<int32_t> colpos;      // column positions, ascending inside a row
  raw_vector<float> vals;
  raw_vector<uint32_t> src;        // index of every entry in the caller's CSR arrays
  int64_t nnz_head_head = 0, nnz_head_row = 0, nnz_head_col = 0, nnz_diag = 0;
  bool separator_rule = false;
};

struct DecomposeOptions {
  double hub_factor = 8.0;   // a vertex is a hub when its degree exceeds hub_factor * mean degree
  bool separators = true;    // try the block-separator rule before the plain top-degree head
  bool bfs_tail = true;      // levels >= 1 arrange the non-head vertices in BFS order
  bool head_by_id = true;    // plain rule: head vertices in id order (else by falling degree)
  int64_t hubs_first = 0;    // ... after this many of the highest degrees, which lead the head by falling degree
};

// Peels arrow matrices of width b off A until nothing is left.  Returns 0 or a
// negative arrow_status; `err` receives a description on failure.
int decompose(int64_t n, const int64_t* rowptr, const int32_t* colidx, const float* vals,
              int32_t b, const DecomposeOptions& opt, std::vector<HostLevel>& levels,
              std::string& err);

// ---------------------------------------------------------------------------
// Device image.  All offsets are byte offsets from the image base, 256-aligned.
// ---------------------------------------------------------------------------

// Entry of a work list: the row to read (perm already applied, or a staged head row) and the value.
struct Entry {
  int32_t xrow;
  float val;
};

constexpr int kDies = 8;             // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin
constexpr int kChunksPerGroup = 4;   // wave-list items (one per wavefront) per workgroup of the chunk kernel
constexpr int kItemsPerGroupBlock = 64;  // group-list items per workgroup of the rows kernel, whatever its lane-group width
// head panels: kPanelRows head rows form a group; the group's head-block entries are dealt by column
// class (staged head row mod kDies) to kDies workgroups, one per accelerator die, each keeping the
// group's accumulators in LDS and streaming its entries in kPanelBins lane-group streams
constexpr int kPanelBins = 32;
constexpr int kPanelRows = 128;
constexpr int kPanelClassShift = 6;       // staged head rows are dealt to the column classes 64 at a time
inline int panel_class(uint32_t staged_row) { return (int)((staged_row >> kPanelClassShift) & (kDies - 1)); }
constexpr int kPanelRowShift = 24;       // panel entry code = (row inside the workgroup << 24) | staged head row

// dense corner of the head block: rows and columns [0, corner) of level 0, cut into tiles of
// kCornerTile x kCornerTile positions.  A workgroup owns the accumulators of one row panel
// (kCornerTile rows) in LDS and sweeps a run of the panel's tiles, each with its kCornerTile
// staged head rows copied into LDS; a tile's entries are dealt to kCornerRuns lane-group streams
// that never share a row.  Entry code = (row inside the panel << 16) | column inside the tile.
constexpr int kCornerTile = 256;
constexpr int kCornerRuns = 64;
constexpr int kCornerTileWords = kCornerRuns + 3;   // per tile: run offsets (kCornerRuns + 1), first column, panel

struct LevelImage {
  int64_t n_i = 0;
  // permutation (int32 n_i)
  size_t off_perm = 0;
  // staged head: rows of X gathered into a contiguous buffer before the level runs
  bool staged = false;
  int64_t n_stage = 0;          // rows of the staging buffer (min(b, n_i) or 0)
  int64_t stage_class_rows = 0; // rows of the first column class in the buffer
  size_t off_stage_perm = 0;    // int32 n_stage : buffer row -> X row
  int32_t classes = 0;          // column classes used for the chunk queues (0 = none)
  // group list: items handled one per lane group (class pieces in die queues, then the short rows)
  int64_t n_rows = 0, n_real_rows = 0, rows_partials = 0, nnz_rows = 0;
  int64_t piece_slots = 0;   // slots [0, piece_slots) hold the class pieces (die queues), the rest the short rows
  size_t off_rows_ptr = 0;   // uint32 n_rows + 1 (offsets into the level's entry array)
  size_t off_rows_mid = 0;   // uint32 n_rows : entries before it read the staged head buffer, the rest read X
  size_t off_rows_dst = 0;   // int32  n_rows : >= 0 -> Y row, < 0 -> partial slot (-1 - slot), INT32_MIN -> padding
  size_t off_rows_row = 0;   // int32  n_rows : the vertex (row of A) the item belongs to, -1 for padding
  // wave list: items handled one per wavefront (the list may contain empty padding slots)
  int64_t n_chunks = 0, n_real_chunks = 0, chunks_partials = 0, nnz_chunks = 0;
  size_t off_chunk_ptr = 0;  // uint32 n_chunks + 1
  size_t off_chunk_mid = 0;  // uint32 n_chunks : entries before it read the staged head buffer, the rest read X
  size_t off_chunk_dst = 0;  // int32  n_chunks : >= 0 -> Y row (whole row in one chunk), < 0 -> partial slot (-1 - slot)
  size_t off_chunk_row = 0;  // int32  n_chunks : the vertex the item belongs to, -1 for padding
  // rows assembled from several chunks
  int64_t n_split = 0, n_partials = 0;
  size_t off_split_ptr = 0;  // uint32 n_split + 1 (partial slots of a row are consecutive)
  size_t off_split_y = 0;    // int32  n_split
  // entries: first nnz_rows for the row list, then nnz_chunks for the chunk list
  size_t off_entries = 0;
  int64_t x_rows_rows = 0, x_rows_chunks = 0;  // distinct X rows each list references
  // diagonal-block tiles processed with their window of P_i X staged in LDS; their entries
  // follow the chunk entries in the level's entry array
  int64_t n_wtiles = 0, n_wrows = 0, nnz_w = 0;
  size_t off_wtiles = 0;     // WindowTile n_wtiles
  size_t off_wrow_ptr = 0;   // uint32 n_wrows + 1
  size_t off_wrow_mid = 0;   // uint32 n_wrows : entries before it read X rows, the rest index the LDS window
  size_t off_wrow_y = 0;     // int32  n_wrows
  size_t off_wrow_win = 0;   // uint32 n_wrows : first position of the row's tile window
  // head panels: head rows whose head-block entries are swept window by window with the rows'
  // accumulators resident in LDS; their entries follow the window entries in the entry array.
  // Workgroup w = group * kDies + class owns bins [w * kPanelBins, (w + 1) * kPanelBins).
  int64_t n_panel_rows = 0, n_panel_groups = 0, n_panel_bins = 0, nnz_panel = 0;
  size_t off_panel_ptr = 0;  // uint32 n_panel_bins + 1 (entry offsets; a bin is one lane group's stream)
  size_t off_panel_y = 0;    // int32  n_panel_groups * kPanelRows : Y row of every accumulator, -1 = unused
  // dense corner (see kCornerTile): its entries follow the panel entries in the entry array
  int64_t corner = 0;        // rows = columns of the corner (a multiple of kCornerTile), 0 = none
  int64_t n_corner_tiles = 0, n_corner_items = 0, nnz_corner = 0;
  size_t off_corner_tiles = 0;   // uint32 n_corner_tiles * kCornerTileWords
  size_t off_corner_items = 0;   // uint32 n_corner_items * 2 + 2 : first tile of every item (+ end), then ...
  size_t off_corner_panel = 0;   // uint32 panels + 1 : first item of every row panel (items of a panel are consecutive)
  size_t off_corner_y = 0;       // int32  corner : Y row of every corner row position
  int64_t map_offset = 0;    // first element of this level in the entry map (one uint32 per entry, image order)
  int64_t nnz_fused = 0;     // level 0 with fused levels: entries of later levels listed with its rows
};

// Rows [row_begin, row_end) of the window-row list belong to one diagonal block and touch only
// column positions [win_begin, win_begin + win_count) of it.
struct WindowTile {
  uint32_t row_begin, row_end;
  uint32_t win_begin, win_count;
};

struct PackOptions {
  int32_t short_max = 16;     // rows with at most this many entries go to the lane-group list
  int32_t chunk_nnz = 256;    // most nonzeros per wavefront chunk
  int32_t chunk_min = 64;     // windows of a row are merged until a chunk holds this many
  int32_t window_rows = 4096; // column positions per window of the chunk ordering (0 = row-major chunks)
  int32_t classes = 0;        // column classes (rounded up to a multiple of 8; 0 = no die queues)
  int32_t class_gran = 512;   // column positions dealt to a class at a time
  int32_t class_min = 32;     // a row is split by class when it holds classes * class_min entries
  int32_t piece_max = 48;     // a class piece with at most this many entries is a group-list item
  int32_t stage_head = 1;     // gather the head rows of level 0 into a contiguous buffer
  int32_t stage_short = -1;   // short rows read their head columns from the staged head too (-1 = when the head is scattered over X)
  int32_t empty_last = 1;     // level 0: the short rows without entries are listed after all others
  int32_t panel = 0;          // run the head block of sparse head rows in panels (accumulators in LDS, one column class per die)
  int32_t panel_min = 8;      // fewest head-block entries of a row that joins a panel
  int32_t window_span = 2048; // widest column span of an LDS-window tile (0 = no such tiles)
  int32_t window_tile_rows = 1024;  // most rows per tile
  double window_reuse = 8.0;  // a tile is kept when its diagonal-block entries >= this x span
  double window_level_share = 0.05;  // ... and the tiles of a level when they hold this share of its entries
  int32_t fuse_levels = 1;    // list the entries of later levels with the level-0 rows of their vertices
  int32_t corner = 0;         // run the dense top-left corner of the head block in LDS tiles (off: measured slower than the chunk list)
  int32_t corner_max = 65536; // largest corner considered (rows = columns)
  int32_t corner_min_tile = 768;  // the corner grows while the tiles it gains hold at least this many entries on average
};

struct Image {
  std::vector<LevelImage> levels;
  std::vector<unsigned char> bytes;  // packed host copy
  int64_t max_partials = 0;
  int64_t max_stage_rows = 0;
  int64_t max_window_span = 0;
  int64_t max_panel_slots = 0;       // most panel accumulators (groups * kPanelRows) of a level
  int64_t max_corner_items = 0;      // most corner work items of a level (each writes kCornerTile result rows)
  std::vector<uint32_t> entry_src;   // per entry in image order: its index in the caller's CSR arrays
  bool fused = false;                // the image was packed from the fused execution form of the levels
};

int pack_image(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const PackOptions& opt,
               Image& img, std::string& err);
// host-side consistency check of a packed image (used by arrow_self_check)
int verify_image(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const Image& img,
                 std::string& err);

// ---------------------------------------------------------------------------
// Kernel launchers (kernels.hip).  All pointers are device pointers; `stream`
// is a hipStream_t.  Each returns a hipError_t cast to int.
// ---------------------------------------------------------------------------
struct LaunchTuning {
  int32_t kc = 0;          // column slice width per pass (0 = automatic)
  int64_t l2_resident_bytes = 2 << 20;  // share of a die's 4 MiB L2 a resident slice of X_0 may take
};

// x_rows = rows of X (it decides whether 32-bit offsets are enough).
int launch_rows(const uint32_t* rows_ptr, const uint32_t* rows_mid, const int32_t* rows_dst,
                const Entry* entries, int64_t n_rows, const float* X, int64_t x_rows,
                const float* Xh, float* Y, float* partials, int32_t k, bool accumulate,
                const LaunchTuning& t, void* stream);
int launch_chunks(const uint32_t* chunk_ptr, const uint32_t* chunk_mid, const int32_t* chunk_dst,
                  const Entry* entries, int64_t n_chunks, const float* X, int64_t x_rows,
                  const float* Xh, float* Y, float* partials, int32_t k, bool accumulate,
                  const LaunchTuning& t, void* stream);
int launch_reduce(const uint32_t* split_ptr, const int32_t* split_y, int64_t n_split,
                  const float* partials, float* Y, int32_t k, bool accumulate, void* stream);
int launch_gather(const int32_t* perm, int64_t n_i, const float* X, float* Xp, int32_t k,
                  void* stream);
// Head panels.  launch_panel: every workgroup (group, class) sums its entries times rows of the
// staged head Xh into LDS accumulators and stores them to part[class][slot][0:k].
// launch_panel_combine: Y[panel_y[slot]] += sum over the kDies classes, in class order.
int launch_panel(const uint32_t* panel_ptr, const int32_t* panel_y, const Entry* entries,
                 int64_t n_groups, const float* Xh, int64_t xh_rows, float* part, int32_t k, void* stream);
int launch_panel_combine(const int32_t* panel_y, int64_t n_slots, const float* part, float* Y, int32_t k,
                         void* stream);
int launch_sddmm_panel(const uint32_t* panel_ptr, const int32_t* panel_y, const Entry* entries,
                       const uint32_t* emap, int64_t n_bins, const float* U, const float* Vh,
                       int64_t vh_rows, float* S, int32_t k, void* stream);
// Dense corner.  launch_corner: workgroup = item; sums the item's tiles into LDS accumulators and
// stores kCornerTile rows to part[item].  launch_corner_combine: Y[corner_y[p]] += the parts of the
// items of p's panel, in item order.  launch_sddmm_corner: the sampled product over the corner tiles.
int launch_corner(const uint32_t* tiles, const uint32_t* items, int64_t n_items, const Entry* entries,
                  const float* Xh, int64_t xh_rows, float* part, int32_t k, void* stream);
int launch_corner_combine(const uint32_t* panel_ptr, const int32_t* corner_y, int64_t corner,
                          const float* part, float* Y, int32_t k, void* stream);
int launch_sddmm_corner(const uint32_t* tiles, int64_t n_tiles, const int32_t* corner_y, const Entry* entries,
                        const uint32_t* emap, const float* U, const float* Vh, int64_t vh_rows, float* S,
                        int32_t k, void* stream);
// max_span = widest window of the tiles (sizes the LDS allocation and the column slice)
int launch_window(const WindowTile* tiles, int64_t n_tiles, int64_t max_span, const uint32_t* wrow_ptr,
                  const uint32_t* wrow_mid, const int32_t* wrow_y, const Entry* entries,
                  const int32_t* perm, const float* X, float* Y, int32_t k, bool accumulate,
                  void* stream);


// Sampled dense-dense product S[emap[e]] = a_e <U[row(e)], V[col(e)]> over one work list.
// mode 0: a group list (item_win and perm unused); mode 1: the window-row list.  emap points at the
// level's slice of the entry map; v_rows = rows of V.
int launch_sddmm_rows(int mode, const uint32_t* item_ptr, const uint32_t* item_mid,
                      const int32_t* item_row, const uint32_t* item_win, const int32_t* perm,
                      const Entry* entries, const uint32_t* emap, int64_t n_items, const float* U,
                      const float* V, int64_t v_rows, const float* Vh, float* S, int32_t k,
                      void* stream);
int launch_sddmm_chunks(const uint32_t* chunk_ptr, const uint32_t* chunk_mid, const int32_t* chunk_row,
                        const Entry* entries, const uint32_t* emap, int64_t n_chunks, const float* U,
                        const float* V, int64_t v_rows, const float* Vh, float* S, int32_t k,
                        void* stream);

// Device address of the current device's copy of the static scratch array of arrow_spmm_static
// (static_scratch.hip); NULL and a description in `err` on failure.  A lookup, never an allocation.
unsigned char* static_scratch(std::string& err);

// Bare row gather (probe.hip), the yardstick of the measurements: `gathers` pseudo-random rows of
// the n x k matrix X drawn from its first region_rows rows (per_die: from a region of its own for
// every accelerator die; from_lds: the region is copied into LDS first) are read and summed.
int64_t probe_out_floats(int64_t gathers);
int launch_probe_gather(const float* X, int64_t x_rows, int32_t k, int64_t region_rows, int per_die,
                        int from_lds, int64_t gathers, float* out, void* stream);

// Order-3 MTTKRP over the compressed-sparse-fibre image (mttkrp.hip): one wavefront per item.
// b_rows, c_rows = rows of the factor matrices (they decide whether 32-bit offsets are enough);
// mean_segment = entries per segment on average (it picks how many row loads a round issues).
// Limits of one work item of the fibre image: the wavefront that owns the item stages its entries
// and segment descriptors in LDS, so both are bounded.
constexpr int kCsfSegMax = 64;      // most entries of a segment
constexpr int kCsfItemNnz = 512;    // most entries of an item
constexpr int kCsfItemSegs = 128;   // most segments of an item
// item_ent[it] = index of the item's first entry (the items' entries are consecutive).
int launch_mttkrp(const uint32_t* item_seg, const uint32_t* item_ent, const int32_t* item_dst,
                  const uint32_t* seg_ptr,
                  const int32_t* seg_j, const Entry* entries, int64_t n_items, const float* B,
                  int64_t b_rows, const float* C, int64_t c_rows, float* A, float* partials, int32_t R,
                  double mean_segment, void* stream);

}  // namespace arrow
