// extern "C" entry points: argument checks, handles, upload; see include/owq.h.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>

#include "owq_internal.h"

using namespace owq;

static bool live(owq_handle_t h) { return h && h->magic == kMagic; }

extern "C" {

static owq_status_t make_handle(const owq_layer_info_t &g, void *dev_buf, owq_handle_t *out) {
  int32_t lds_limit = 0;
  if (device_lds_limit(&lds_limit) != 0) return OWQ_ERR_HIP;
  LaunchShape shape{};
  int32_t tile_grid = 0, tile_waves = 4, tile_split = 0;
  if (g.layout == OWQ_LAYOUT_TILE) {
    if (lds_limit < 65536) return OWQ_ERR_UNSUPPORTED;
    tile_default_shape(g, tile_waves, &tile_grid, &tile_split);
    if (tile_grid < 1) return OWQ_ERR_UNSUPPORTED;
    const int e = prepare_tile_kernels(g, lds_limit);
    if (e == (int)hipErrorInvalidValue) return OWQ_ERR_UNSUPPORTED;
    if (e != 0) return OWQ_ERR_HIP;
    if (prepare_tile_small_kernels() != 0) return OWQ_ERR_HIP;
  } else {
    shape = default_shape(g, lds_limit);
    if (shape.rtw < 1) return OWQ_ERR_UNSUPPORTED;
    if (prepare_kernels(lds_limit) != 0 || prepare_multi_kernels(lds_limit) != 0) return OWQ_ERR_HIP;
  }
  owq_layer_s *h = new (std::nothrow) owq_layer_s;
  if (!h) return OWQ_ERR_BUFFER;
  h->magic = kMagic;
  h->info = g;
  h->shape = shape;
  h->tile_grid = tile_grid;
  h->tile_waves = tile_waves;
  h->tile_split = tile_split;
  h->tile_small_split = 0;
  h->dev_buf = dev_buf;
  h->lds_limit = lds_limit;
  const uint8_t *base = static_cast<const uint8_t *>(dev_buf);
  h->dev.codes = base + g.off_codes;
  h->dev.sz = base + g.off_sz;
  h->dev.weak_w = base + g.off_weak_w;
  h->dev.weak_idx = base + g.off_weak_idx;
  h->dev.wmeta = base + g.off_wmask;
  h->info.last_hip_error = 0;
  *out = h;
  return OWQ_OK;
}

owq_status_t owq_pack_layer(const owq_layer_desc_t *desc, void *dev_buf, size_t dev_bytes,
                            void *stream, owq_handle_t *out) {
  if (!desc || !dev_buf || !out) return OWQ_ERR_NULL;
  *out = nullptr;
  owq_status_t st = validate_desc(desc);
  if (st != OWQ_OK) return st;
  owq_layer_info_t g;
  compute_geometry(desc->d_out, desc->d_in, desc->bits, desc->group_size, desc->k, desc->layout, &g);
  if (dev_bytes < g.total_bytes) return OWQ_ERR_BUFFER;
  if (reinterpret_cast<uintptr_t>(dev_buf) % kAlign != 0) return OWQ_ERR_BUFFER;

  uint8_t *host = nullptr;
  if (hipHostMalloc(reinterpret_cast<void **>(&host), g.total_bytes, hipHostMallocDefault) != hipSuccess)
    return OWQ_ERR_HIP;
  pack_blob(desc, g, host);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(dev_buf, host, g.total_bytes, hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipHostFree(host);
  if (e != hipSuccess) return OWQ_ERR_HIP;
  return make_handle(g, dev_buf, out);
}

owq_status_t owq_open_packed(const owq_layer_desc_t *desc, void *dev_buf, size_t dev_bytes,
                             owq_handle_t *out) {
  if (!desc || !dev_buf || !out) return OWQ_ERR_NULL;
  *out = nullptr;
  owq_layer_info_t g;
  owq_status_t st = compute_geometry(desc->d_out, desc->d_in, desc->bits, desc->group_size, desc->k, desc->layout, &g);
  if (st != OWQ_OK) return st;
  if (dev_bytes < g.total_bytes) return OWQ_ERR_BUFFER;
  if (reinterpret_cast<uintptr_t>(dev_buf) % kAlign != 0) return OWQ_ERR_BUFFER;
  return make_handle(g, dev_buf, out);
}

// Where a tile-layout call keeps its intermediate results: nullptr = the blob's own scratch area
// with the handle's launch shape; else `mem` of `bytes` bytes with the shape given here.
struct ScratchChoice {
  void *mem;
  uint64_t bytes;
  int32_t grid, split;
};

static owq_status_t run_linear(owq_handle_t h, const TaskSets &tasks, const void *x, void *y, int32_t batch,
                               void *stream, const ScratchChoice *sc = nullptr) {
  if (batch < 0 || batch > OWQ_MAX_BATCH) return OWQ_ERR_BATCH;
  if (batch == 0) return OWQ_OK;
  if (!x || !y) return OWQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(x) % 2 != 0 || reinterpret_cast<uintptr_t>(y) % 2 != 0) return OWQ_ERR_BUFFER;
  const int herr = h->info.layout == OWQ_LAYOUT_TILE
                       ? launch_tile(h->info, h->dev_buf, sc ? sc->mem : nullptr, sc ? sc->bytes : 0, sc ? sc->grid : h->tile_grid,
                                     sc ? sc->split : h->tile_split, h->tile_waves, h->tile_small_split, tasks, x, y, batch, stream)
                       : launch_gemv(h->info, h->shape, h->dev, tasks, x, y, batch, h->lds_limit, stream);
  if (herr == -2) return OWQ_ERR_SHAPE;     // a launch shape set by the caller does not fit this batch
  if (herr != 0) {
    h->info.last_hip_error = herr;
    return OWQ_ERR_HIP;
  }
  return OWQ_OK;
}

owq_status_t owq_linear(owq_handle_t h, const void *x, void *y, int32_t batch, void *stream) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  const TaskSets one{nullptr, nullptr, 0};
  return run_linear(h, one, x, y, batch, stream);
}

owq_status_t owq_workspace_bytes(owq_handle_t h, size_t *bytes) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (!bytes) return OWQ_ERR_NULL;
  *bytes = h->info.layout == OWQ_LAYOUT_TILE ? (size_t)tile_scratch(h->info).total : 0;
  return OWQ_OK;
}

owq_status_t owq_linear_ws(owq_handle_t h, const void *x, void *y, int32_t batch, void *workspace, size_t workspace_bytes,
                           void *stream) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  const TaskSets one{nullptr, nullptr, 0};
  if (h->info.layout != OWQ_LAYOUT_TILE) return run_linear(h, one, x, y, batch, stream);   // needs no workspace
  if (batch > 0 && !workspace) return OWQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < tile_scratch(h->info).total) return OWQ_ERR_BUFFER;
  const ScratchChoice sc{workspace, tile_scratch(h->info).total, h->tile_grid, h->tile_split};
  return run_linear(h, one, x, y, batch, stream, &sc);
}

owq_status_t owq_linear_static(owq_handle_t h, const void *x, void *y, int32_t batch, void *stream) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  const TaskSets one{nullptr, nullptr, 0};
  if (h->info.layout != OWQ_LAYOUT_TILE) return run_linear(h, one, x, y, batch, stream);   // needs no scratch memory
  ScratchChoice sc{nullptr, OWQ_STATIC_SCRATCH_BYTES, 0, 0};
  // the work split that fits the array: fewer partial-result slots than the blob's own area may hold
  tile_default_shape(h->info, h->tile_waves, &sc.grid, &sc.split, sc.bytes);
  if (sc.grid < 1) return OWQ_ERR_SCRATCH;
  const int herr = static_scratch(&sc.mem);
  if (herr != 0) {
    h->info.last_hip_error = herr;
    return OWQ_ERR_HIP;
  }
  return run_linear(h, one, x, y, batch, stream, &sc);
}

owq_status_t owq_linear_multi(owq_handle_t h, const void *const *weak_sets, int32_t n_sets, const int32_t *task_id,
                              const void *x, void *y, int32_t batch, void *stream) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (!weak_sets || !task_id) return OWQ_ERR_NULL;
  if (n_sets < 1 || n_sets > OWQ_MAX_WEAK_SETS) return OWQ_ERR_INDEX;
  if (reinterpret_cast<uintptr_t>(weak_sets) % 8 != 0 || reinterpret_cast<uintptr_t>(task_id) % 4 != 0)
    return OWQ_ERR_BUFFER;
  const TaskSets tasks{weak_sets, task_id, n_sets};
  return run_linear(h, tasks, x, y, batch, stream);
}

owq_status_t owq_probe_read(const void *dev_buf, size_t bytes, int32_t workgroups, void *stream) {
  if (!dev_buf) return OWQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(dev_buf) % 16 != 0 || bytes % 16 != 0) return OWQ_ERR_BUFFER;
  if (workgroups < 1 || workgroups > 65536 || bytes / 16 > 0xffffffffull) return OWQ_ERR_SHAPE;
  return launch_read(dev_buf, bytes, workgroups, nullptr, 0, stream) == 0 ? OWQ_OK : OWQ_ERR_HIP;
}

owq_status_t owq_probe_read_write(const void *dev_buf, size_t bytes, int32_t workgroups, void *out, size_t out_bytes, void *stream) {
  if (!dev_buf || !out) return OWQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(dev_buf) % 16 != 0 || bytes % 16 != 0) return OWQ_ERR_BUFFER;
  if (reinterpret_cast<uintptr_t>(out) % 16 != 0 || out_bytes % 16 != 0 || out_bytes > 0xffffffffull) return OWQ_ERR_BUFFER;
  if (workgroups < 1 || workgroups > 65536 || bytes / 16 > 0xffffffffull) return OWQ_ERR_SHAPE;
  return launch_read(dev_buf, bytes, workgroups, out, out_bytes, stream) == 0 ? OWQ_OK : OWQ_ERR_HIP;
}

owq_status_t owq_probe_empty(void *stream) { return launch_empty(stream) == 0 ? OWQ_OK : OWQ_ERR_HIP; }

owq_status_t owq_probe_alu(void *dev_word, int32_t workgroups, int32_t trips, void *stream) {
  if (!dev_word) return OWQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(dev_word) % 4 != 0) return OWQ_ERR_BUFFER;
  if (workgroups < 1 || workgroups > 65536 || trips < 1 || trips > (1 << 20)) return OWQ_ERR_SHAPE;
  return launch_alu(dev_word, workgroups, trips, stream) == 0 ? OWQ_OK : OWQ_ERR_HIP;
}

owq_status_t owq_probe_mfma(void *dev_word, int32_t workgroups, int32_t trips, void *stream) {
  if (!dev_word) return OWQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(dev_word) % 4 != 0) return OWQ_ERR_BUFFER;
  if (workgroups < 1 || workgroups > 65536 || trips < 1 || trips > (1 << 20)) return OWQ_ERR_SHAPE;
  return launch_mfma(dev_word, workgroups, trips, stream) == 0 ? OWQ_OK : OWQ_ERR_HIP;
}

owq_status_t owq_weak_set_bytes(owq_handle_t h, size_t *bytes) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (!bytes) return OWQ_ERR_NULL;
  const size_t n = (size_t)h->info.d_out_pad * h->info.kp * 2;
  *bytes = (n + kAlign - 1) / kAlign * kAlign;
  return OWQ_OK;
}

// weak_w (HOST, [d_out][k]) -> section layout -> DEVICE dst; waits for the copy
static owq_status_t upload_weak(owq_handle_t h, const uint16_t *weak_w, void *dst, void *stream) {
  const size_t n = (size_t)h->info.d_out_pad * h->info.kp * 2;
  if (n == 0) return OWQ_OK;
  uint16_t *host = nullptr;
  if (hipHostMalloc(reinterpret_cast<void **>(&host), n, hipHostMallocDefault) != hipSuccess) return OWQ_ERR_HIP;
  pack_weak_section(h->info, weak_w, host);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(dst, host, n, hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipHostFree(host);
  if (e != hipSuccess) {
    h->info.last_hip_error = (int)e;
    return OWQ_ERR_HIP;
  }
  return OWQ_OK;
}

owq_status_t owq_pack_weak_set(owq_handle_t h, const uint16_t *weak_w, void *dev_buf, size_t dev_bytes, void *stream) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (!dev_buf || (h->info.k > 0 && !weak_w)) return OWQ_ERR_NULL;
  if (dev_bytes < (size_t)h->info.d_out_pad * h->info.kp * 2) return OWQ_ERR_BUFFER;
  if (reinterpret_cast<uintptr_t>(dev_buf) % 16 != 0) return OWQ_ERR_BUFFER;
  return upload_weak(h, weak_w, dev_buf, stream);
}

owq_status_t owq_update_weak(owq_handle_t h, const uint16_t *weak_w, void *stream) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (h->info.k > 0 && !weak_w) return OWQ_ERR_NULL;
  return upload_weak(h, weak_w, static_cast<uint8_t *>(h->dev_buf) + h->info.off_weak_w, stream);
}

owq_status_t owq_free_layer(owq_handle_t h) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  h->magic = 0;
  delete h;
  return OWQ_OK;
}

owq_status_t owq_layer_info(owq_handle_t h, owq_layer_info_t *info) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (!info) return OWQ_ERR_NULL;
  *info = h->info;
  info->row_tiles_per_wg = h->shape.rtw;
  info->row_splits = h->info.layout == OWQ_LAYOUT_TILE ? h->tile_split : h->shape.rsplit;
  info->waves_per_wg = h->info.layout == OWQ_LAYOUT_TILE ? h->tile_waves : h->shape.waves;
  info->prefetch_depth = h->shape.depth;
  info->workgroups = h->info.layout == OWQ_LAYOUT_TILE ? h->tile_grid : h->shape.nwg;
  info->lds_bytes = h->info.layout == OWQ_LAYOUT_TILE ? 65536 : h->shape.lds_bytes;
  return OWQ_OK;
}

owq_status_t owq_export_packed(owq_handle_t h, void *host_buf, size_t bytes) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (!host_buf) return OWQ_ERR_NULL;
  if (bytes < h->info.total_bytes) return OWQ_ERR_BUFFER;
  hipError_t e = hipMemcpy(host_buf, h->dev_buf, h->info.total_bytes, hipMemcpyDeviceToHost);
  if (e != hipSuccess) {
    h->info.last_hip_error = (int)e;
    return OWQ_ERR_HIP;
  }
  return OWQ_OK;
}

owq_status_t owq_set_launch(owq_handle_t h, int32_t rtw, int32_t rsplit, int32_t waves, int32_t depth) {
  if (!live(h)) return OWQ_ERR_HANDLE;
  if (h->info.layout == OWQ_LAYOUT_TILE) {
    // tile layout: workgroups of the main kernel, column ranges per row group, waves per workgroup
    if (depth < -1 || depth >= 400 || (depth % 100 > 0 && !tile_small_split_ok(h->info, depth % 100))) return OWQ_ERR_SHAPE;
    const int32_t wv = waves ? waves : h->tile_waves;
    if (wv != 4 && wv != 8) return OWQ_ERR_SHAPE;
    if (wv == 8 && h->info.n_groups > 1) return OWQ_ERR_SHAPE;      // grouped layers: four waves only
    const int32_t lim = tile_grid_limit(h->info, wv);
    if (lim < 1) return OWQ_ERR_UNSUPPORTED;
    int32_t gr = 0, sp = 0;
    if (rsplit > 0) {                       // aligned ranges: grid follows from the split
      const int32_t n_rg = (h->info.n_rt + 2 * wv - 1) / (2 * wv);
      if (rsplit > h->info.nbp || (int64_t)n_rg * rsplit > lim) return OWQ_ERR_SHAPE;
      if (rtw && rtw != n_rg * rsplit) return OWQ_ERR_SHAPE;
      gr = n_rg * rsplit;
      sp = rsplit;
    } else if (rsplit < 0) {
      return OWQ_ERR_SHAPE;
    } else if (rtw) {                       // equal ranges of the whole sequence
      if (rtw < 0 || rtw > lim) return OWQ_ERR_SHAPE;
      gr = rtw;
    } else {
      tile_default_shape(h->info, wv, &gr, &sp);
    }
    h->tile_grid = gr;
    h->tile_split = sp;
    h->tile_waves = wv;
    h->tile_small_split = depth;
    return OWQ_OK;
  }
  LaunchShape s = h->shape;
  if (rtw) s.rtw = rtw;
  if (rsplit) s.rsplit = rsplit;
  if (waves) s.waves = waves;
  if (depth) s.depth = depth;
  if (s.rtw > h->info.n_rt) s.rtw = h->info.n_rt;
  if (!shape_is_valid(h->info, s)) return OWQ_ERR_SHAPE;
  s.lds_bytes = lds_bytes_for(h->info, s.rtw, &s.xpitch);
  if (s.lds_bytes > h->lds_limit) return OWQ_ERR_UNSUPPORTED;
  s.nwg = (h->info.n_rt + s.rtw - 1) / s.rtw;
  if (!make_magics(h->info, &s)) return OWQ_ERR_UNSUPPORTED;
  h->shape = s;
  return OWQ_OK;
}

const char *owq_status_str(owq_status_t s) {
  switch (s) {
    case OWQ_OK: return "ok";
    case OWQ_ERR_NULL: return "null pointer";
    case OWQ_ERR_SHAPE: return "bad shape";
    case OWQ_ERR_BITS: return "bits must be 3 or 4";
    case OWQ_ERR_GROUP: return "group_size must be 0 or a multiple of 128";
    case OWQ_ERR_CODE_RANGE: return "code out of range";
    case OWQ_ERR_INDEX: return "bad weak index list";
    case OWQ_ERR_BUFFER: return "buffer too small or misaligned";
    case OWQ_ERR_BATCH: return "bad batch";
    case OWQ_ERR_HANDLE: return "not a live handle";
    case OWQ_ERR_HIP: return "HIP call failed";
    case OWQ_ERR_UNSUPPORTED: return "layer too large for one workgroup's on-chip memory";
    case OWQ_ERR_LAYOUT: return "unknown layout";
    case OWQ_ERR_SCRATCH: return "the layer needs more scratch memory than the library's static array holds";
  }
  return "unknown status";
}

}  // extern "C"
