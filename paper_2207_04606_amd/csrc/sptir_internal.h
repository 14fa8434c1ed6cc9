// Internal declarations shared by the translation units of libsptir.so.
#ifndef SPTIR_INTERNAL_H_
#define SPTIR_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sptir.h"

namespace sptir {

// The SpMM kernel walks the real entries of the stored rows in chunks of kChunkSlots slots.  A builder-side
// descriptor stands for a chunk cut from one row (an ELL row of section 4.2.1 or a piece of the CSR remainder)
// that is too long to be walked by one lane group: `count` consecutive slots of the fused (cols, vals) arrays
// starting at `slot0`, all of row row_ids[row0]; it carries log2w = kRowLog2W.  Queue chunks, which hold eight
// entries of each of eight lane-group queues, are written piece by piece and have a descriptor only to mark
// their place; a descriptor with count 0 is the padding at the end of a (launch, row block) list.
struct Chunk {
  int64_t slot0;
  int32_t row0;
  // bits 0..5 log2w, bits 6..12 count (1..64), bit 13: hand the row's partial sum over after this chunk,
  // bit 14: queue chunk
  uint32_t meta;
};
static_assert(sizeof(Chunk) == 16, "Chunk must stay 16 bytes");

constexpr int kChunkSlots = 64;
constexpr int kRowLog2W = 31;
constexpr int kChunksPerQuad = 4;  // chunks the SpMM kernel fetches with one load per lane and array
constexpr int kBuildBlock = 256;  // rows per workgroup in the builder kernels
// A row piece (ELL row or remainder piece) with more real entries than this is kept out of the chunk lists,
// which one wavefront walks alone, and is summed by a whole workgroup in a launch of its own.
constexpr int kLongRowSlots = 2048;

// One long row piece: `len` consecutive slots of the fused (cols, vals) arrays starting at slot0.
struct LongPiece {
  int64_t slot0;
  int32_t row;
  int32_t len;
  int32_t q;  // position in row_ids (orders the pieces of a row by column partition)
  int32_t pad_;
};
static_assert(sizeof(LongPiece) == 24, "LongPiece must stay 24 bytes");
// A run of at most kLongSegSlots consecutive entries of a long piece.
struct LongSegment {
  int64_t slot0;
  int32_t len;
  int32_t pad_;
};
constexpr int kLongSegSlots = 1024;
constexpr int kLongPartialFeat = 512;  // widest Y the per-segment partial sums are kept for
// Compact stream records spend 8 bytes per slot instead of 12: one word holds the column relative to the first
// column of the launch (bits 0..19), the row relative to the row block (20..26), "slot is real" (27), the chunk's
// log2w code (28..30; 3 = queue chunk, 7 = cut from one long row) and the hand-over flag (31; of the chunk, or in a
// queue chunk of the slot: the last entry of a row piece); the other word the value.
constexpr int kCompactColBits = 20;
constexpr int kCompactMaxLog2RowBlock = 7;

}  // namespace sptir

// The handle behind sptir_hyb_t.  ELL and remainder share three device
// allocations so that one SpMM launch can walk both:
//   row_ids = [ELL_ROW | REM_ROW], cols = [ELL_COL | REM_COL], vals likewise.
struct sptir_hyb {
  int32_t n_rows, n_cols, c, k, w;
  int64_t nnz;
  int64_t B, R, S, M, T;
  int64_t* bucket_row_ptr;   // device [B+1]
  int64_t* bucket_slot_ptr;  // device [B+1]
  int32_t* rem_part_ptr;     // device [c+1]
  int64_t* rem_ptr;          // device [M+1]
  int32_t* row_ids;          // device [R+M]
  int32_t* cols;             // device [S+T]
  float* vals;               // device [S+T]
  int32_t* row_len;          // device [R+M], real length of every ELL row / remainder piece
  int32_t* stream;           // device [n_chunks * 128 or 192]: the chunks as fixed records, grouped by (phase, row block)
  int32_t spmm_plan;         // 0: built without the chunk stream (canonical arrays only); sptir_spmm refuses it
  int32_t compact_stream;    // 1: 8-byte slots (columns relative to the launch), 0: 12-byte slots (global columns)
  int64_t* rb_chunk_ptr;     // device [n_phases * n_row_blocks + 1], first chunk of each group
  int32_t* rb_order;         // device [n_phases * n_row_blocks]: the row blocks of a launch, longest list first
  int64_t n_chunks;
  // rows with long pieces: the pieces of long_rows[i] are long_pieces[long_piece_ptr[i] .. long_piece_ptr[i+1])
  int32_t n_long_rows;
  int32_t* long_rows;        // device [n_long_rows], ascending
  int32_t* long_piece_ptr;   // device [n_long_rows + 1]
  sptir::LongPiece* long_pieces;  // device
  // the long pieces cut into segments of at most kLongSegSlots entries, one workgroup each; the segments of
  // long_rows[i] are long_segs[long_seg_ptr[i] .. long_seg_ptr[i+1]) and their partial sums meet in long_partial
  int32_t n_long_segs;
  int32_t* long_seg_ptr;     // device [n_long_rows + 1]
  sptir::LongSegment* long_segs;  // device [n_long_segs]
  float* long_partial;       // device [n_long_segs][kLongPartialFeat]
  int32_t log2_row_block;    // rows of Y one wavefront accumulates in LDS (power of two)
  int32_t n_row_blocks;
  int32_t parts_per_phase;   // column partitions swept by one SpMM launch
  int32_t n_phases;
  size_t device_bytes;
  sptir_alloc_fn alloc;
  sptir_free_fn free_;
  void* alloc_ctx;
};

namespace sptir {

// allocator currently installed (api.hip)
void current_allocator(sptir_alloc_fn* a, sptir_free_fn* f, void** ctx);
void* default_alloc(size_t bytes, void* ctx, void* stream);
void default_free(void* p, void* ctx);

// sptir_hyb_build, optionally without the SpMM launch plan (for users of the canonical arrays alone), and with
// the feature size the launch plan should suit (0: not known)
sptir_status_t hyb_build_impl(const sptir_csr_t* csr, int32_t n_col_parts, int32_t max_bucket_log2, void* stream,
                              sptir_hyb_t** out, bool with_spmm_plan, int32_t feat_hint);

// What the builder decides about the SpMM launches from the sizes alone (builder.hip; host code, no device access).
struct LaunchShape {
  int32_t log2_row_block;   // rows of Y per wavefront
  int32_t parts_per_phase;  // column partitions per launch
  int32_t n_phases;         // launches per sweep
  int32_t compact;          // 1: 8-byte stream records
};
LaunchShape decide_launch_shape(int32_t n_rows, int32_t c, int32_t w, int64_t stored_slots, int32_t feat_hint);

// Lane geometry sptir_spmm uses for `feat` when X and Y are 16-byte aligned, and the feature tiles one sweep over
// the launches covers (spmm.hip; host code).
void lane_shape(int32_t feat, bool aligned16, bool aligned8, int* vec, int* lg);
int tiles_per_sweep(int n_tiles, int tile_floats, int64_t n_rows, int n_launches);

// rb_order[launch][i] = the row block with the i-th longest chunk list of that launch (order.hip).  Works on
// `stream`; *scratch_out is device memory the caller frees once the stream has drained.
sptir_status_t order_row_blocks(const int64_t* rb_chunk_ptr, int32_t n_launches, int32_t n_rb, int32_t* rb_order,
                                sptir_alloc_fn alloc, sptir_free_fn free_, void* actx, hipStream_t stream,
                                void** scratch_out);

// records a failed HIP call for sptir_last_hip_error(); returns SPTIR_ERR_HIP
sptir_status_t note_hip_error(hipError_t e, const char* what);

// text for sptir_last_hip_error() where a refusal needs more than its status code
void note_error_text(const char* text);

#define SPTIR_HIP(call)                                                   \
  do {                                                                    \
    hipError_t e_ = (call);                                               \
    if (e_ != hipSuccess) return ::sptir::note_hip_error(e_, #call);      \
  } while (0)

}  // namespace sptir

#endif  // SPTIR_INTERNAL_H_
