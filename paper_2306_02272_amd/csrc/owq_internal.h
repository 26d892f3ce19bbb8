// Internal declarations shared by the host packer, the handle code and the kernels' launcher.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "owq.h"

namespace owq {

constexpr int kBlockCols = 128;   // input columns per block (one lane's unit of work)
constexpr int kAlign = 256;       // section alignment inside the blob
constexpr uint32_t kMagic = 0x4f575131u;  // "OWQ1"

// Shape checks + geometry of the packed blob.  Fills every geometry field of info.
owq_status_t compute_geometry(int32_t d_out, int32_t d_in, int32_t bits, int32_t group_size,
                              int32_t k, int32_t layout, owq_layer_info_t *info);

constexpr int kTileRows = 32;        // rows per tile of the tile layout
constexpr int kScratchBatch = 64;    // tokens per pass of the tile path
constexpr int kTileGroupTiles = 8;   // row tiles per row group (one workgroup: 4 waves x 2 tiles)
constexpr int kTileGridMax = 512;    // most workgroups of the tile kernel
constexpr int kTileSlotBytes = 65536;  // one partial result: 256 rows x 64 tokens, fp32

// Map of the scratch area of a tile-layout blob (byte offsets from off_scratch).
struct TileScratch {
  int32_t n_rg;          // row groups of 256 rows
  int32_t grid_max;      // most workgroups the partial slots allow: min(kTileGridMax, n_rg * nbp)
  uint64_t off_xs;       // staged activations: [nbp][16 k-steps][2 token tiles][64 lanes][8 fp16]
  uint64_t off_bsum;     // [nblk][64 tokens] (sum x, sum c*x) as two floats
  uint64_t off_tsum;     // [64 tokens] the same summed over all blocks (16 KiB reserved)
  uint64_t off_xw;       // [64 tokens][kp] fp16: activations at the weak columns
  uint64_t off_slots;    // partial results: grid_max + n_rg slots in use (room for n_rg more)
  uint64_t total;
};
TileScratch tile_scratch(const owq_layer_info_t &g);

// Full validation of a description (pointers, code range, index order).
owq_status_t validate_desc(const owq_layer_desc_t *desc);

// Weak-column section of a blob: [d_out_pad][kp] fp16, padding 0.  out has d_out_pad * kp entries.
void pack_weak_section(const owq_layer_info_t &info, const uint16_t *weak_w, uint16_t *out);

// Host packer: writes info->total_bytes bytes.
void pack_blob(const owq_layer_desc_t *desc, const owq_layer_info_t &info, uint8_t *out);

// Launch shape of the GEMV path.
struct LaunchShape {
  int32_t rtw;      // row tiles per workgroup
  int32_t rsplit;   // row splits (waves sharing a slab take interleaved row tiles)
  int32_t waves;    // waves per workgroup
  int32_t depth;    // tiles in flight per wave
  int32_t nwg;      // workgroups per batch row
  int32_t lds_bytes;
  int32_t xpitch;   // pitch (in 16-byte units) of the staged activations
  // 16-bit reciprocals for the kernel's small divisions; 0 = not representable
  uint32_t cw_magic, nslab_magic, rsplit_magic, bpg_magic;
};

// Fills the reciprocals of s for layer g; false if some division cannot be done that way.
bool make_magics(const owq_layer_info_t &g, LaunchShape *s);

bool shape_is_valid(const owq_layer_info_t &g, const LaunchShape &s);
int32_t lds_bytes_for(const owq_layer_info_t &g, int32_t rtw, int32_t *xpitch);
LaunchShape default_shape(const owq_layer_info_t &g, int32_t lds_limit);

// Device-side launch (defined in owq_kernels.hip).  Returns a hipError_t as int.
struct DeviceLayer {
  const void *codes, *sz, *weak_w, *weak_idx;
  const void *wmeta;   // storage-favoured layout: weak mask and weak columns before, per 8 input columns
};
// Several sets of weak columns for one dense matrix (all DEVICE memory): token n uses
// weak_sets[task_id[n]] when that index is in [0, n_sets), else the layer's own columns.
// task_id == nullptr: one task, the layer's own columns.
struct TaskSets {
  const void *const *weak_sets;
  const int32_t *task_id;
  int32_t n_sets;
};
int launch_gemv(const owq_layer_info_t &g, const LaunchShape &s, const DeviceLayer &dev, const TaskSets &tasks,
                const void *x, void *y, int32_t batch, int32_t lds_limit, void *stream);
int prepare_kernels(int32_t lds_bytes);   // raises the dynamic LDS limit when needed
// Two tokens per pass over the weights (defined in owq_gemv_multi.hip): enqueues the first batch & ~1 tokens.
// Returns a hipError_t as int, or -1 when the layer, the launch shape or x does not fit that kernel.
int launch_gemv_multi(const owq_layer_info_t &g, const LaunchShape &s, const DeviceLayer &dev, int32_t lds_limit,
                      const void *x, void *y, int32_t batch, void *stream);
int prepare_multi_kernels(int32_t lds_bytes);

// Tile path (defined in owq_tile.hip): three launches per pass of up to 64 tokens.
// blob = DEVICE address of the packed blob; grid = workgroups of the main kernel.
// waves = waves per workgroup of the main kernel (4 or 8).
// split > 0: grid = row groups x split, every row group cut into `split` column ranges;
// split = 0: the flattened (row group, column step) sequence cut into `grid` equal ranges.
// small_shape: work split of the one-launch kernel that takes passes of 32 tokens or fewer
// (0 = the library's choice, -1 = never use that kernel, else S + 100 c, see launch_tile_small).
// scratch = DEVICE memory for the intermediate results laid out as tile_scratch() says, of
// scratch_bytes bytes (at least TileScratch::off_slots plus the slots the grid needs);
// nullptr = the scratch area inside the blob.
int launch_tile(const owq_layer_info_t &g, void *blob, void *scratch, uint64_t scratch_bytes, int32_t grid, int32_t split,
                int32_t waves, int32_t small_split, const TaskSets &tasks, const void *x, void *y, int32_t batch,
                void *stream);
// Device address of the library's static scratch array on the current device (looked up once
// per device).  Returns a hipError_t as int.
int static_scratch(void **ptr);
// The one-launch kernel for 32 tokens or fewer (defined in owq_tile_small.hip).  Returns a
// hipError_t as int, or -1 when the layer, the split or the alignment of x does not fit it.
// part = DEVICE memory of part_bytes bytes for fp32 partial sums when the columns are split.
int launch_tile_small(const owq_layer_info_t &g, void *blob, void *part, uint64_t part_bytes, int32_t shape, const void *x,
                      void *y, int32_t ntok, void *stream);
bool tile_small_split_ok(const owq_layer_info_t &g, int32_t split);
int prepare_tile_small_kernels();   // LDS opt-in
// scratch_bytes = size of the scratch memory in use, 0 = the blob's own scratch area
void tile_default_shape(const owq_layer_info_t &g, int32_t waves, int32_t *grid, int32_t *split, uint64_t scratch_bytes = 0);
int32_t tile_grid_limit(const owq_layer_info_t &g, int32_t waves, uint64_t scratch_bytes = 0);
int prepare_tile_kernels(const owq_layer_info_t &g, int32_t lds_limit);   // LDS opt-in for grouped layers
int device_lds_limit(int32_t *bytes);

// Read-only streaming kernels (defined in owq_probe.hip).  Return a hipError_t as int.
int launch_read(const void *dev, size_t bytes, int32_t workgroups, void *out, size_t out_bytes, void *stream);
int launch_empty(void *stream);
int launch_alu(void *dev_word, int32_t workgroups, int32_t trips, void *stream);
int launch_mfma(void *dev_word, int32_t workgroups, int32_t trips, void *stream);

}  // namespace owq

struct owq_layer_s {
  uint32_t magic;
  owq_layer_info_t info;
  owq::LaunchShape shape;
  owq::DeviceLayer dev;
  void *dev_buf;
  int32_t lds_limit;
  int32_t tile_grid;     // workgroups of the tile kernel (tile layout only)
  int32_t tile_waves;    // its waves per workgroup: 4 or 8
  int32_t tile_split;    // column ranges per row group, 0 = equal ranges of the whole sequence
  int32_t tile_small_split;  // 32 tokens or fewer: column ranges per row tile, 0 = default, -1 = three-launch path
};
