// Handle management, allocator hook and status strings of the C ABI.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "sptir_internal.h"

namespace sptir {

static std::mutex g_alloc_mu;
static sptir_alloc_fn g_alloc = nullptr;
static sptir_free_fn g_free = nullptr;
static void* g_alloc_ctx = nullptr;
static thread_local char g_hip_error[512] = "";

void* default_alloc(size_t bytes, void*, void*) {
  void* p = nullptr;
  if (hipMalloc(&p, bytes ? bytes : 1) != hipSuccess) {
    (void)hipGetLastError();
    return nullptr;
  }
  return p;
}

void default_free(void* p, void*) {
  if (p) (void)hipFree(p);
}

void current_allocator(sptir_alloc_fn* a, sptir_free_fn* f, void** ctx) {
  std::lock_guard<std::mutex> lock(g_alloc_mu);
  if (g_alloc && g_free) {
    *a = g_alloc; *f = g_free; *ctx = g_alloc_ctx;
  } else {
    *a = default_alloc; *f = default_free; *ctx = nullptr;
  }
}

// ---- temporaries under the default allocator
// A hipFree costs 0.17 - 0.23 ms on this system (it waits for the device and unmaps the block), and a build has five
// temporaries: a quarter of its time.  Blocks that hipMalloc gave out for temporaries are therefore kept when they are
// released (a few, bounded in size) and handed to the next call that asks for about as much on the same device.
// With a caller's allocator temporaries go straight to it: it has its own policy.
namespace {
struct ScratchBlock { void* p; size_t size; int dev; };
std::mutex g_scratch_mu;
std::vector<ScratchBlock> g_scratch_free, g_scratch_live;
size_t g_scratch_free_bytes = 0;
constexpr size_t kScratchKeepBytes = (size_t)512 << 20, kScratchKeepBlock = (size_t)256 << 20;
constexpr size_t kScratchKeepCount = 8;
}  // namespace

void* scratch_alloc(size_t bytes, sptir_alloc_fn alloc, void* actx, void* stream) {
  if (alloc != default_alloc) return alloc(bytes, actx, stream);
  if (bytes == 0) bytes = 1;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    int best = -1;
    for (size_t i = 0; i < g_scratch_free.size(); ++i) {
      const ScratchBlock& b = g_scratch_free[i];
      if (b.dev != dev || b.size < bytes || b.size > 2 * bytes + ((size_t)1 << 20)) continue;
      if (best < 0 || b.size < g_scratch_free[(size_t)best].size) best = (int)i;
    }
    if (best >= 0) {
      const ScratchBlock b = g_scratch_free[(size_t)best];
      g_scratch_free.erase(g_scratch_free.begin() + best);
      g_scratch_free_bytes -= b.size;
      g_scratch_live.push_back(b);
      return b.p;
    }
  }
  void* p = default_alloc(bytes, nullptr, stream);
  if (p) {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    g_scratch_live.push_back({p, bytes, dev});
  }
  return p;
}

void scratch_free(void* p, sptir_free_fn free_, void* actx) {
  if (!p) return;
  ScratchBlock b{nullptr, 0, 0};
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    for (size_t i = 0; i < g_scratch_live.size(); ++i)
      if (g_scratch_live[i].p == p) {
        b = g_scratch_live[i];
        g_scratch_live.erase(g_scratch_live.begin() + (long)i);
        break;
      }
    if (b.p && b.size <= kScratchKeepBlock && g_scratch_free.size() < kScratchKeepCount &&
        g_scratch_free_bytes + b.size <= kScratchKeepBytes) {
      g_scratch_free.push_back(b);
      g_scratch_free_bytes += b.size;
      return;
    }
  }
  if (b.p) default_free(p, nullptr);  // ours, but not kept
  else free_(p, actx);                // came from the caller's allocator
}

sptir_status_t note_hip_error(hipError_t e, const char* what) {
  snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
  (void)hipGetLastError();  // clear the sticky-less error slot
  return SPTIR_ERR_HIP;
}

void note_error_text(const char* text) { snprintf(g_hip_error, sizeof(g_hip_error), "%s", text); }

}  // namespace sptir

extern "C" {

sptir_status_t sptir_release_scratch(void) {
  std::vector<sptir::ScratchBlock> blocks;
  {
    std::lock_guard<std::mutex> lock(sptir::g_scratch_mu);
    blocks.swap(sptir::g_scratch_free);
    sptir::g_scratch_free_bytes = 0;
  }
  int before = 0;
  const bool have_dev = hipGetDevice(&before) == hipSuccess;
  for (const auto& b : blocks) {
    if (have_dev && hipSetDevice(b.dev) != hipSuccess) { (void)hipGetLastError(); continue; }
    (void)hipFree(b.p);
  }
  if (have_dev) (void)hipSetDevice(before);
  return SPTIR_OK;
}

sptir_status_t sptir_set_allocator(sptir_alloc_fn alloc, sptir_free_fn free_, void* ctx) {
  if ((alloc == nullptr) != (free_ == nullptr)) return SPTIR_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(sptir::g_alloc_mu);
  sptir::g_alloc = alloc;
  sptir::g_free = free_;
  sptir::g_alloc_ctx = ctx;
  return SPTIR_OK;
}

sptir_status_t sptir_hyb_destroy(sptir_hyb_t* h) {
  if (!h) return SPTIR_OK;
  for (void* p : h->blobs)
    if (p) h->free_(p, h->alloc_ctx);
  delete h;
  return SPTIR_OK;
}

sptir_status_t sptir_hyb_info(const sptir_hyb_t* h, sptir_hyb_info_t* out) {
  if (!h || !out) return SPTIR_ERR_INVALID_ARG;
  sptir_hyb_info_t o;
  memset(&o, 0, sizeof(o));
  o.n_rows = h->n_rows; o.n_cols = h->n_cols;
  o.n_col_parts = h->c; o.max_bucket_log2 = h->k; o.part_width = h->w;
  o.n_buckets = (int32_t)h->B;
  o.nnz = h->nnz;
  o.n_ell_rows = h->R; o.n_ell_slots = h->S;
  o.n_pad_slots = h->S + h->T - h->nnz;
  o.n_rem_pieces = h->M; o.n_rem_nnz = h->T;
  o.n_work_items = h->n_chunks; o.item_slots = sptir::kChunkSlots; o.row_block = 1 << h->log2_row_block;
  o.n_phases = h->n_phases;
  o.rounds = h->rounds;
  o.n_heavy_pieces = h->n_heavy; o.n_heavy_items = h->n_heavy_chunks; o.n_heavy_nnz = h->n_heavy_nnz;
  o.heavy_len = h->heavy_len; o.n_heavy_lists = h->n_heavy_lists;
  o.values_per_row = h->row_val ? 1 : 0;
  o.compact_stream = h->compact_stream; o.n_row_blocks = h->n_row_blocks; o.parts_per_launch = h->parts_per_phase;
  o.device_bytes = (int64_t)h->device_bytes;
  o.full_rows = h->full_rows;
  o.heavy_list_items = h->heavy_list_chunks;
  *out = o;
  return SPTIR_OK;
}

sptir_status_t sptir_hyb_array(const sptir_hyb_t* h, int32_t which, const void** dev_ptr, int64_t* n_elems) {
  if (!h || !dev_ptr || !n_elems) return SPTIR_ERR_INVALID_ARG;
  const void* p = nullptr;
  int64_t n = 0;
  switch (which) {
    case SPTIR_HYB_BUCKET_ROW_PTR: p = h->bucket_row_ptr; n = h->B + 1; break;
    case SPTIR_HYB_BUCKET_SLOT_PTR: p = h->bucket_slot_ptr; n = h->B + 1; break;
    case SPTIR_HYB_ELL_ROW: p = h->row_ids; n = h->R; break;
    case SPTIR_HYB_ELL_COL: p = h->cols; n = h->S; break;
    case SPTIR_HYB_ELL_VAL: p = h->vals; n = h->S; break;
    case SPTIR_HYB_REM_PART_PTR: p = h->rem_part_ptr; n = h->c + 1; break;
    case SPTIR_HYB_REM_ROW: p = h->row_ids + h->R; n = h->M; break;
    case SPTIR_HYB_REM_PTR: p = h->rem_ptr; n = h->M + 1; break;
    case SPTIR_HYB_REM_COL: p = h->cols + h->S; n = h->T; break;
    case SPTIR_HYB_REM_VAL: p = h->vals + h->S; n = h->T; break;
    case SPTIR_PLAN_STREAM:
      p = h->stream;
      n = (h->n_chunks + h->n_heavy_chunks) * sptir::kChunkSlots * ((h->compact_stream ? 2 : 3) - (h->row_val ? 1 : 0));
      break;
    case SPTIR_PLAN_RB_CHUNK_PTR: p = h->rb_chunk_ptr; n = h->spmm_plan ? (int64_t)h->n_phases * h->n_row_blocks + 1 : 0; break;
    case SPTIR_PLAN_RB_ORDER: p = h->rb_order; n = h->spmm_plan ? (int64_t)h->n_phases * h->n_row_blocks : 0; break;
    case SPTIR_PLAN_HLIST_FIRST_SLOT: p = h->hlist_first_slot; n = h->n_heavy > 0 ? h->n_heavy_lists : 0; break;
    case SPTIR_PLAN_ROW_SLOT_PTR: p = h->row_slot_ptr; n = h->n_heavy > 0 ? (int64_t)h->n_rows + 1 : 0; break;
    case SPTIR_PLAN_ROW_SLOTS: p = h->row_slots; n = h->n_heavy > 0 ? h->n_row_slots : 0; break;
    case SPTIR_PLAN_HEAVY_ROWS: p = h->heavy_rows; n = h->n_heavy > 0 ? h->n_heavy_rows : 0; break;
    case SPTIR_PLAN_ROW_VAL: p = h->row_val; n = h->row_val ? h->n_rows : 0; break;
    default: return SPTIR_ERR_INVALID_ARG;
  }
  if (h->canonical_released && (which == SPTIR_HYB_ELL_COL || which == SPTIR_HYB_ELL_VAL ||
                                which == SPTIR_HYB_REM_COL || which == SPTIR_HYB_REM_VAL))
    return SPTIR_ERR_UNSUPPORTED;
  *dev_ptr = n ? p : nullptr;
  *n_elems = n;
  return SPTIR_OK;
}

const char* sptir_status_string(sptir_status_t s) {
  switch (s) {
    case SPTIR_OK: return "ok";
    case SPTIR_ERR_INVALID_ARG: return "invalid argument";
    case SPTIR_ERR_UNSORTED: return "column ids not strictly ascending inside a row, or out of range";
    case SPTIR_ERR_OVERFLOW: return "a count overflows its index type";
    case SPTIR_ERR_ALLOC: return "device allocation failed";
    case SPTIR_ERR_HIP: return "HIP runtime error";
    case SPTIR_ERR_UNSUPPORTED: return "unsupported request";
  }
  return "unknown status";
}

const char* sptir_last_hip_error(void) { return sptir::g_hip_error; }

int32_t sptir_default_bucket_log2(int64_t nnz, int32_t n_rows) {
  if (n_rows <= 0 || nnz <= 0) return 0;
  // smallest k with 2^k * n_rows >= nnz, i.e. ceil(log2(nnz / n_rows))
  int32_t k = 0;
  while (k < 30 && ((int64_t)n_rows << k) < nnz) ++k;
  return k;
}

}  // extern "C"

extern "C" sptir_status_t sptir_launch_plan(int32_t n_rows, int32_t n_cols, int64_t stored_slots, int32_t n_col_parts,
                                            int32_t feat, const sptir_build_options_t* options,
                                            sptir_launch_plan_t* out) {
  if (!out || n_rows < 0 || n_cols < 0 || stored_slots < 0 || n_col_parts < 1 || feat < 1) return SPTIR_ERR_INVALID_ARG;
  const int32_t w = (int32_t)(((int64_t)n_cols + n_col_parts - 1) / n_col_parts);
  sptir_build_options_t opt = sptir::complete_options(options);
  if (opt.feat_hint == 0) opt.feat_hint = feat;
  const sptir::LaunchShape ls = sptir::decide_launch_shape(n_rows, n_cols, n_col_parts, w, stored_slots, opt);
  int vec, lg;
  sptir::lane_shape(feat, true, true, ls.full_rows != 0 && sptir::full_rows_fit(ls.log2_row_block), &vec, &lg);
  const int tile = vec * lg;
  sptir_launch_plan_t o;
  o.row_block = 1 << ls.log2_row_block;
  o.parts_per_launch = ls.parts_per_phase;
  o.n_launches = ls.n_phases;
  o.compact_stream = ls.compact;
  o.n_feature_tiles = (feat + tile - 1) / tile;
  o.tiles_per_sweep = ls.rounds ? sptir::round_tiles_per_sweep(o.n_feature_tiles, tile, n_cols, opt.sweep_kb)
                                : sptir::tiles_per_sweep(o.n_feature_tiles, tile, n_rows, ls.n_phases,
                                                         opt.sweep_kb);
  o.n_sweeps = (o.n_feature_tiles + o.tiles_per_sweep - 1) / o.tiles_per_sweep;
  o.rounds = ls.rounds;
  o.full_rows = ls.full_rows;
  *out = o;
  return SPTIR_OK;
}
