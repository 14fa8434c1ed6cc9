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
// Row pieces of more than `heavy_len` real entries leave the chunk lists (a wavefront walks a list alone and keeps
// the Y rows of its row block on chip).  Their entries form one sequence of 64-slot chunks, piece after piece in the
// order of the canonical arrays (partition-major); the sequence is cut into "heavy lists" of kHeavyListChunks chunks,
// a wavefront each, which write one partial sum per finished piece plus one for whatever piece is unfinished where
// the list ends.  A last launch adds a row's partial sums to Y in a fixed order.
constexpr int kHeavyLenMax = 2048;      // largest threshold the size rules choose
constexpr int kHeavyListChunks = 16;    // most chunks per heavy list (a multiple of kChunksPerQuad; on the largest graph 16
                                        // beat 32 by 2 % and 64 by 4 % of the heavy launch; graphs with few heavy
                                        // chunks get shorter lists)
constexpr int kPartialFeat = 128;       // features per partial sum row: wider Y is produced in sweeps of this many
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
  float* row_val;            // device [n_rows] or NULL: set when every row of A has one value for all its entries;
                             // the stream then holds no values and Y is scaled row by row at the end
  int32_t* stream;           // device [n_chunks * 128 or 192]: the chunks as fixed records, grouped by (phase, row block)
  int32_t spmm_plan;         // 0: built without the chunk stream (canonical arrays only); sptir_spmm refuses it
  int32_t compact_stream;    // 1: 8-byte slots (columns relative to the launch), 0: 12-byte slots (global columns)
  int64_t* rb_chunk_ptr;     // device [n_phases * n_row_blocks + 1], first chunk of each group
  int32_t* rb_order;         // device [n_phases * n_row_blocks]: the row blocks of a launch, longest list first
  int64_t n_chunks;
  // heavy pieces (see kHeavyListChunks): their chunks sit in `stream` from chunk heavy_chunk0 on
  int32_t heavy_len;
  int64_t n_heavy;            // heavy pieces
  int64_t n_heavy_nnz;        // their real entries
  int64_t n_heavy_chunks;     // their chunks, rounded up to whole quads
  int64_t heavy_chunk0;       // a multiple of kChunksPerQuad
  int32_t n_heavy_lists;
  int32_t* hlist_first_slot;  // device [n_heavy_lists]: partial-sum row the list's first write goes to
  int32_t* row_slot_ptr;      // device [n_rows + 1]: the partial-sum rows of row r are row_slots[row_slot_ptr[r] ..)
  int32_t* row_slots;         // device, in the order they are added to Y (partition-major)
  int32_t n_heavy_rows;       // rows with at least one heavy piece
  int32_t n_row_slots;        // elements of row_slots
  int32_t* heavy_rows;        // device [n_heavy_rows], ascending
  float* partial;             // device [(n_heavy + n_heavy_lists)][kPartialFeat]
  int64_t n_partial_rows;
  int32_t log2_row_block;    // rows of Y one wavefront accumulates in LDS (power of two)
  int32_t n_row_blocks;
  int32_t parts_per_phase;   // column partitions swept by one chunk list
  int32_t n_phases;
  int32_t rounds;            // 1: the lists sweep all partitions and are launched in rounds (Y written once)
  int32_t sweep_kb;          // kilobytes of Y (no rounds) or X (rounds) one sweep may touch; 0: the rules' defaults
  int32_t canonical_released;
  size_t device_bytes;
  // The device arrays above are parts of at most kHybBlobs allocations: [0] the index arrays whose sizes the
  // bucket totals fix, [1] cols and vals (can be released on their own), [2] the SpMM plan.
  int32_t heavy_list_chunks;  // chunks per heavy list of this handle: 4, 8, 16 or 32
  int32_t full_rows;        // sptir_spmm may use the 128-float tile (the row blocks are sized for it)
  void* blobs[3];
  size_t canonical_bytes;  // size of blobs[1]
  sptir_alloc_fn alloc;
  sptir_free_fn free_;
  void* alloc_ctx;
};

namespace sptir {

// allocator currently installed (api.hip)
void current_allocator(sptir_alloc_fn* a, sptir_free_fn* f, void** ctx);
void* default_alloc(size_t bytes, void* ctx, void* stream);
// Temporaries of a call: from `alloc`, or, when that is the default allocator, from a small cache of blocks that
// earlier calls have released (api.hip).  scratch_free takes back what scratch_alloc gave.
void* scratch_alloc(size_t bytes, sptir_alloc_fn alloc, void* actx, void* stream);
void scratch_free(void* p, sptir_free_fn free_, void* actx);
void default_free(void* p, void* ctx);

// sptir_hyb_build_ex; `opt` is complete (defaults filled in by the caller)
sptir_status_t hyb_build_impl(const sptir_csr_t* csr, int32_t n_col_parts, int32_t max_bucket_log2,
                              const sptir_build_options_t& opt, void* stream, sptir_hyb_t** out);
// the options a NULL pointer stands for / a caller's struct with unknown tail fields zeroed
sptir_build_options_t complete_options(const sptir_build_options_t* given);

// What the builder decides about the SpMM launches from the sizes alone (builder.hip; host code, no device access).
struct LaunchShape {
  int32_t log2_row_block;   // rows of Y per wavefront
  int32_t parts_per_phase;  // column partitions per chunk list
  int32_t n_phases;         // chunk-list launches per sweep (1 when rounds)
  int32_t compact;          // 1: 8-byte stream records
  int32_t rounds;           // 1: lists sweep all partitions, launched in rounds
  int32_t full_rows;        // 1: feature tiles of 128 floats (32 lanes per entry) where feat allows
};
LaunchShape decide_launch_shape(int32_t n_rows, int32_t n_cols, int32_t c, int32_t w, int64_t stored_slots,
                                const sptir_build_options_t& opt);

// Lane geometry sptir_spmm uses for `feat` when X and Y are 16-byte aligned, and the feature tiles one sweep over
// the launches covers (spmm.hip; host code).
void lane_shape(int32_t feat, bool aligned16, bool aligned8, bool full_rows, int* vec, int* lg);
// 512-byte feature tiles need row blocks whose Y tiles (4 wavefronts x rows x 512 bytes, plus the chunk rings) fit a
// CU's LDS: up to 64 rows.  With larger row blocks sptir_spmm uses the 128-byte tiles whatever the handle asks for.
inline bool full_rows_fit(int log2_row_block) {
  return (size_t)4 * (((size_t)512 << log2_row_block) + 6 * 1024) <= (size_t)159 * 1024;
}
int tiles_per_sweep(int n_tiles, int tile_floats, int64_t n_rows, int n_launches, int sweep_kb);
int round_tiles_per_sweep(int n_tiles, int tile_floats, int64_t n_cols, int sweep_kb);

// rb_order[launch][i] = the row block with the i-th longest chunk list of that launch (order.hip).  Works on
// `stream`; *scratch_out is device memory the caller frees once the stream has drained.
sptir_status_t order_row_blocks(const int64_t* rb_chunk_ptr, int32_t n_launches, int32_t n_rb, int64_t max_list_len,
                                int32_t* rb_order, sptir_alloc_fn alloc, sptir_free_fn free_, void* actx,
                                hipStream_t stream, void** scratch_out);

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
