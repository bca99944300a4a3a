// Internal C++ declarations shared by the host decomposition, the image
// packer / C-ABI and the HIP kernel launchers.  Nothing here is exported.
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

namespace arrow {

// One arrow matrix B_i in position coordinates, CSR by row position.
struct HostLevel {
  int64_t n_i = 0;                 // active vertices of this level
  std::vector<int32_t> perm;       // position -> original vertex id, n_i entries
  std::vector<int64_t> rowptr;     // n_i + 1
  std::vector<int32_t> colpos;     // column positions, ascending inside a row
  std::vector<float> vals;
  int64_t nnz_head_head = 0, nnz_head_row = 0, nnz_head_col = 0, nnz_diag = 0;
  bool separator_rule = false;
};

struct DecomposeOptions {
  double hub_factor = 8.0;   // a vertex is a hub when its degree exceeds hub_factor * mean degree
  bool separators = true;    // try the block-separator rule before the plain top-degree head
  bool bfs_tail = true;      // levels >= 1 arrange the non-head vertices in BFS order
};

// Peels arrow matrices of width b off A until nothing is left.  Returns 0 or a
// negative arrow_status; `err` receives a description on failure.
int decompose(int64_t n, const int64_t* rowptr, const int32_t* colidx, const float* vals,
              int32_t b, const DecomposeOptions& opt, std::vector<HostLevel>& levels,
              std::string& err);

// ---------------------------------------------------------------------------
// Device image.  All offsets are byte offsets from the image base, 256-aligned.
// ---------------------------------------------------------------------------

// Entry of a work list: the X row to read (perm already applied) and the value.
struct Entry {
  int32_t xrow;
  float val;
};

struct LevelImage {
  int64_t n_i = 0;
  // permutation (int32 n_i)
  size_t off_perm = 0;
  // rows handled one per lane group: CSR over list order
  int64_t n_rows = 0, nnz_rows = 0;
  size_t off_rows_ptr = 0;   // uint32 n_rows + 1 (offsets into the level's entry array)
  size_t off_rows_y = 0;     // int32  n_rows      (Y row = perm[p])
  // chunks handled one per wavefront
  int64_t n_chunks = 0, nnz_chunks = 0;
  size_t off_chunk_ptr = 0;  // uint32 n_chunks + 1
  size_t off_chunk_dst = 0;  // int32  n_chunks : >= 0 -> Y row (whole row in one chunk), < 0 -> partial slot (-1 - slot)
  // rows assembled from several chunks
  int64_t n_split = 0, n_partials = 0;
  size_t off_split_ptr = 0;  // uint32 n_split + 1 (partial slots of a row are consecutive)
  size_t off_split_y = 0;    // int32  n_split
  // entries: first nnz_rows for the row list, then nnz_chunks for the chunk list
  size_t off_entries = 0;
  int64_t x_rows_rows = 0, x_rows_chunks = 0;  // distinct X rows each list references
  // diagonal blocks whose X window is staged in LDS (optional, may be empty)
  int64_t n_wtiles = 0, n_wrows = 0, nnz_w = 0;
  size_t off_wtile = 0;      // WindowTile n_wtiles
  size_t off_wrow_ptr = 0;   // uint32 n_wrows + 1
  size_t off_wrow_y = 0;     // int32  n_wrows
  size_t off_wentries = 0;   // Entry nnz_w, xrow = column position local to the window
};

// One diagonal block (or a slice of its rows) processed by one workgroup with
// the block's window of P_i X resident in LDS.
struct WindowTile {
  uint32_t row_begin, row_end;   // range in the window-row list
  uint32_t win_begin, win_count; // positions [win_begin, win_begin + win_count) of the level form the window
};

struct PackOptions {
  int32_t short_max = 16;     // rows with at most this many entries go to the lane-group list
  int32_t chunk_nnz = 512;    // nonzeros per wavefront chunk
  int32_t window_max_rows = 0;// diagonal blocks up to this many rows may use the LDS-window path (0 = off)
};

struct Image {
  std::vector<LevelImage> levels;
  std::vector<unsigned char> bytes;  // packed host copy
  int64_t max_partials = 0;
};

int pack_image(int64_t n, int32_t b, const std::vector<HostLevel>& levels, const PackOptions& opt,
               Image& img, std::string& err);

// ---------------------------------------------------------------------------
// Kernel launchers (kernels.hip).  All pointers are device pointers; `stream`
// is a hipStream_t.  Each returns a hipError_t cast to int.
// ---------------------------------------------------------------------------
struct LaunchTuning {
  int32_t kc = 0;          // column slice width per pass (0 = automatic)
  int32_t xcd_remap = 1;   // map consecutive work items to the same XCD
  int32_t unroll = 4;
};

int launch_rows(const uint32_t* rows_ptr, const int32_t* rows_y, const Entry* entries,
                int64_t n_rows, const float* X, float* Y, int32_t k, bool accumulate,
                const LaunchTuning& t, void* stream);
int launch_chunks(const uint32_t* chunk_ptr, const int32_t* chunk_dst, const Entry* entries,
                  int64_t n_chunks, const float* X, float* Y, float* partials, int32_t k,
                  bool accumulate, const LaunchTuning& t, void* stream);
int launch_reduce(const uint32_t* split_ptr, const int32_t* split_y, int64_t n_split,
                  const float* partials, float* Y, int32_t k, bool accumulate, void* stream);
int launch_window(const WindowTile* tiles, int64_t n_tiles, const uint32_t* wrow_ptr,
                  const int32_t* wrow_y, const Entry* wentries, const int32_t* perm,
                  const float* X, float* Y, int32_t k, bool accumulate, void* stream);
int launch_gather(const int32_t* perm, int64_t n_i, const float* X, float* Xp, int32_t k,
                  void* stream);
size_t window_lds_bytes_max();

}  // namespace arrow
