// SpMM Y = A X on the hyb(c,k) decomposition (section 4.2.1 of arXiv
// 2207.04606), and the single-pass CSR variant the paper calls "no-hyb".
//
// Mapping (gfx950, wave64).  The feature dimension is cut into tiles of
// LG*VEC floats (32 floats = one 128-byte line of X by default).  A wavefront
// owns one (row block, feature tile): it keeps that tile of the row block's Y
// rows (64 rows, 8 KB, unless the graph is small) in its own piece of LDS, walks
// every chunk of the row block's list (all column partitions of the launch, the
// rows of all ELL buckets and the remainder, real entries only) and finally
// writes the Y tile with plain coalesced stores.
// Nothing is shared between wavefronts: no atomics, no barriers, no zero fill
// of Y, and rows without non-zeros come out as 0 (the init block of the SpMM
// script in appendix A).
//
// The 64 lanes form 64/LG lane groups; a group covers the tile with VEC floats
// per lane, so one wave load instruction gathers 64/LG different rows of X,
// each as one contiguous 128-byte read.  Partial sums stay in registers
// (section 4.2.1 names this as what a CSR code generator misses) and go to the
// LDS tile once per row.
//
// Workgroup -> (row blocks, tile): consecutive workgroup ids are dealt
// round-robin to the 8 XCDs, each with a private L2.  Tiles are bound to
// blockIdx.x % 8 where the tile count allows it, so an XCD's L2 only ever holds
// its own feature tile of X; the chunks of a row block sweep the column
// partitions in ascending order.  Where rows are long enough for the cache
// locality of X to matter (the purpose section 4.2.1 gives for column
// partitioning) the lists run in rounds: a launch takes as many row blocks as
// the GPU holds wavefronts, chosen with lists of like length, so that all of
// them sweep the partitions nearly in step and the X slice in flight stays
// L2-sized while Y never leaves the chip before it is complete.
//
// Row pieces too long for that (more than a chunk's worth of entries in
// rounds) are summed by k_spmm_heavy: their chunks form one sequence in
// partition order, cut into lists of 32 chunks, a wavefront each, which leave
// partial sums in memory; k_heavy_reduce adds them to Y in a fixed order.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <utility>
#include <vector>
#include "sptir_internal.h"

namespace sptir {
namespace {

template <int VEC> struct Vec;
template <> struct Vec<4> { using type = float4; };
template <> struct Vec<2> { using type = float2; };
template <> struct Vec<1> { using type = float; };

template <int VEC>
__device__ __forceinline__ void load_vec(float (&x)[VEC], const float* p) {
  typename Vec<VEC>::type v = *reinterpret_cast<const typename Vec<VEC>::type*>(p);
  if constexpr (VEC == 4) { x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w; }
  else if constexpr (VEC == 2) { x[0] = v.x; x[1] = v.y; }
  else { x[0] = v; }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float* p, const float (&x)[VEC]) {
  if constexpr (VEC == 4) *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
  else if constexpr (VEC == 2) *reinterpret_cast<float2*>(p) = make_float2(x[0], x[1]);
  else *p = x[0];
}

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }

// Lane geometry of one wavefront.
template <int VEC, int LG>
struct Shape {
  static constexpr int kGroups = 64 / LG;            // lane groups = X rows gathered per load
  static constexpr int kSteps = LG < 8 ? LG : 8;     // slots a group takes from one chunk
  static constexpr int kChunk = kGroups * kSteps;    // slots per chunk (<= 64: one per lane)
  static constexpr int kTile = VEC * LG;             // floats per feature tile
  static constexpr int kLog2Chunk = ilog2(kChunk);
};

// LDS position of the VEC floats lane fl of a group owns in local row r of the wavefront's Y tile.  A row of 32
// floats or more spans all 32 banks, so the lane groups of one instruction (eight may hand eight rows over at once)
// cannot collide and the tile is stored plainly; narrower rows (16 floats: feat <= 16) are rotated against each
// other by one lane's share, so that lane groups working on neighbouring rows hit different banks.
template <int VEC, int LG>
__device__ __forceinline__ int tile_index(int r, int fl) {
  if constexpr (VEC * LG >= 32) return (r * LG + fl) * VEC;
  else return (r * LG + ((fl + r) & (LG - 1))) * VEC;
}

// Adds a finished row sum into the wavefront's Y tile; r is the row relative to the row block.  The tile is
// private to the wavefront and a row is handed over by exactly one lane group per instruction, so a plain
// read-add-write is enough (LDS float atomics measured three times slower for the whole launch).  Lanes past
// the last feature are not told apart here: the tile has a place for every lane, what they add to theirs is
// never written to Y, and the hand-over stays free of a second test.
template <int VEC, int LG>
struct TileSink {
  static constexpr bool kQueues = true;  // the lists it serves hold queue chunks
  float* tile;     // [row_block][kTile] in LDS
  int fl;
  __device__ __forceinline__ void operator()(int r, bool valid, const float (&acc)[VEC]) {
    if (valid) {
      float* p = tile + tile_index<VEC, LG>(r, fl);
      float t[VEC];
      load_vec<VEC>(t, p);
#pragma unroll
      for (int e = 0; e < VEC; ++e) t[e] += acc[e];
      store_vec<VEC>(p, t);
    }
  }
};

// Stores a finished sum as the next partial-sum row (heavy pieces): every call takes one row, whether or not
// this lane has something to store, so the row number stays the same in all lanes.
template <int VEC, int LG>
struct PartialSink {
  static constexpr bool kQueues = false;  // heavy lists hold chunks cut from one long piece only
  float* out;      // partial + this lane's feature offset inside a partial-sum row
  int slot;        // next row
  bool f_active;
  __device__ __forceinline__ void operator()(int, bool valid, const float (&acc)[VEC]) {
    if (valid && f_active) store_vec<VEC>(out + (size_t)slot * kPartialFeat, acc);
    ++slot;
  }
};

// acc[i] += acc of the lane DIST lanes above (only lanes whose partner exists need the result)
template <int DIST, int VEC>
__device__ __forceinline__ void add_from_above(float (&acc)[VEC]) {
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    float other;
    if constexpr (DIST == 8)        // same 16-lane row: DPP row shift left by 8
      other = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(acc[e]), 0x108, 0xF, 0xF, true));
    else if constexpr (DIST == 16)  // neighbouring rows of the same half: swizzle lane ^ 16
      other = __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(acc[e]), 0x401F));
    else
      other = __shfl_down(acc[e], DIST, 64);
    acc[e] += other;
  }
}

// sums the partial sums of `groups` (1, 2, 4, ... kGroups) neighbouring lane groups into the first of them
template <int VEC, int LG>
__device__ __forceinline__ void sum_groups(float (&acc)[VEC], int groups) {
  if (groups >= 2) add_from_above<LG, VEC>(acc);
  if constexpr (LG <= 16) { if (groups >= 4) add_from_above<2 * LG, VEC>(acc); }
  if constexpr (LG <= 8) { if (groups >= 8) add_from_above<4 * LG, VEC>(acc); }
  if constexpr (LG <= 4) { if (groups >= 16) add_from_above<8 * LG, VEC>(acc); }
}

// Stores a finished row straight to Y (a row owned by exactly one wavefront).
template <int VEC, int LG>
struct DirectSink {
  float* y;  // Y + row*feat + f0
  bool f_active;
  __device__ __forceinline__ void operator()(int, bool valid, const float (&acc)[VEC]) const {
    if (valid && f_active) store_vec<VEC>(y, acc);
  }
};

// Sums one row's `count` entries cp/vp[0..count) times their rows of X for this lane's feature offset: entry o
// is gathered by lane group (o % kChunk) / kSteps, the lane groups' partial sums meet once at the end, and the
// row sum goes to `sink` from the first lane group.
template <int VEC, int LG, typename Sink>
__device__ __forceinline__ void walk_row(const int32_t* __restrict__ cp, const float* __restrict__ vp,
                                         const float* __restrict__ Xf, int feat, int count, int lane, bool f_active,
                                         const Sink& sink) {
  using S = Shape<VEC, LG>;
  constexpr int UB = S::kSteps, CS = S::kChunk;
  if (count <= 0) return;
  const int g = lane / LG;
  const int src0 = g * UB;  // lane that fetched slot (g*UB) of the chunk
  const int nch = (count + CS - 1) >> S::kLog2Chunk;

  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;

  // one (column, value) pair per lane and chunk; past the end a lane re-reads the last entry with value 0
  auto fetch = [&](int ch, int& c, float& v) {
    int o = (ch << S::kLog2Chunk) + lane;
    bool ok = (CS == 64 || lane < CS) && o < count;
    int oc = o < count ? o : count - 1;
    c = cp[oc];
    float vv = vp[oc];
    v = ok ? vv : 0.f;
  };
  auto issue = [&](int c_reg, float (&x)[UB][VEC]) {
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      int c = __shfl(c_reg, src0 + u, 64);
      if (f_active) load_vec<VEC>(x[u], Xf + (size_t)c * (size_t)feat);
      else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) x[u][e] = 0.f;
      }
    }
  };
  auto consume = [&](float v_reg, const float (&x)[UB][VEC]) {
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      float v = __shfl(v_reg, src0 + u, 64);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] = fmaf(v, x[u][e], acc[e]);
    }
  };

  // software pipeline: x0 / x1 hold the gathers of two consecutive chunks
  float x0[UB][VEC], x1[UB][VEC];
  int c_a = 0, c_b = 0, c_p = 0;
  float v_a = 0.f, v_b = 0.f, v_p = 0.f;
  fetch(0, c_a, v_a);
  if (nch > 1) fetch(1, c_b, v_b);
  issue(c_a, x0);
  if (nch > 2) fetch(2, c_p, v_p);
  if (nch > 1) issue(c_b, x1);
  for (int ch = 0; ch < nch; ch += 2) {
    consume(v_a, x0);
    if (ch + 2 < nch) {
      c_a = c_p; v_a = v_p;
      if (ch + 3 < nch) fetch(ch + 3, c_p, v_p);
      issue(c_a, x0);
    }
    if (ch + 1 < nch) {
      consume(v_b, x1);
      if (ch + 3 < nch) {
        c_b = c_p; v_b = v_p;
        if (ch + 4 < nch) fetch(ch + 4, c_p, v_p);
        issue(c_b, x1);
      }
    }
  }
  for (int d = 1; d < S::kGroups; d <<= 1) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] += __shfl_xor(acc[e], d * LG, 64);
  }
  sink(0, g == 0, acc);
}

enum TileMap : int {
  kMapTilesPerXcd = 0,  // n_tiles multiple of 8: XCD x owns tiles x, x+8, ...
  kMapXcdsPerTile = 1,  // n_tiles in {1,2,4}: 8/n_tiles XCDs share a tile, split the units
  kMapPlain = 2         // any other tile count: tile = id % n_tiles
};

// workgroup id -> (unit, feature tile); units are row blocks (hyb) or groups of rows (CSR)
__device__ __forceinline__ void decode_block(unsigned bid, int map_mode, int map_param, int n_tiles, int64_t* unit,
                                             int* tile) {
  if (map_mode == kMapTilesPerXcd) {
    unsigned q = bid >> 3, x = bid & 7;
    *tile = (int)(x + 8 * (q % (unsigned)map_param));
    *unit = q / (unsigned)map_param;
  } else if (map_mode == kMapXcdsPerTile) {
    unsigned q = bid >> 3, x = bid & 7;
    *tile = (int)(x % (unsigned)n_tiles);
    *unit = (int64_t)q * map_param + x / (unsigned)n_tiles;
  } else {
    *tile = (int)(bid % (unsigned)n_tiles);
    *unit = bid / (unsigned)n_tiles;
  }
}

struct SpmmArgs {
  const int32_t* stream;        // chunk records: [cols | vals | local rows] x 64
  const int64_t* rb_chunk_ptr;  // this phase's [n_row_blocks + 1]
  const int32_t* rb_order;      // this phase's [n_row_blocks]: which row block the i-th wavefront of the launch takes
  const float* X;
  float* Y;
  int32_t n_rows;
  int32_t n_row_blocks;
  int32_t log2_row_block;
  int32_t feat;
  int32_t n_tiles;     // feature tiles of this launch, the first of which is tile0
  int32_t tile0;
  int32_t map_mode;
  int32_t map_param;
  int32_t accumulate;  // 0: Y tile is overwritten, 1: added to (a later phase)
  const float* row_val;  // UNIT kernels: the value of every entry of row r
};

constexpr int kHybWaves = 4;
constexpr int kHybBlock = 64 * kHybWaves;

// One wavefront's walk over its share of a row block's chunk list.
//
// The unit of the pipeline is a "step": kChunk = kGroups*kSteps slots of a
// 64-slot chunk (the whole chunk when a lane group is 8 lanes wide).  Chunks
// come in quads: a quad is a fixed record of the stream (2 KB compact, 3 KB
// WIDE) whose address follows from its list position, so nothing in the loop
// waits for a descriptor.  A lane requests 16 bytes of each of the quad's
// arrays two quads ahead and parks them one quad later
// in a per-wave LDS ring of two quads; from there every lane group reads the
// kSteps columns / values it needs with 16-byte LDS reads (all lanes of a group
// read the same address, which LDS broadcasts).  While step u is multiplied,
// the X gathers of steps u+1 and u+2 are in flight.  The loop body covers one
// quad and holds no conditional memory operation, so that the compiler's wait
// counters stay exact; the last quad is peeled.
//
// In a queue chunk every lane group sums the rows of its own queue and adds a
// finished row sum into the wavefront's LDS tile of Y; the lane groups that
// share a chunk of one long row add their partial sums up with cross-lane moves
// at the row's end, and the leading group hands the sum over.
//
// UNIT: the stream holds no values (every row of A has one value for all its entries, which the caller of the
// walk multiplies in at the end): a real slot counts 1, any other 0.
//
// DEPTH: gather steps in flight per wavefront (a step is UB loads per lane; each needs UB * VEC registers).
template <int VEC, int LG, bool IDX32, bool WIDE, bool UNIT, typename Sink, int DEPTH = 2>
struct HybWalker {
  using S = Shape<VEC, LG>;
  static constexpr int UB = S::kSteps, CS = S::kChunk;
  static constexpr int SUB = kChunkSlots / CS;              // steps per chunk
  static constexpr int kQuadSteps = kChunksPerQuad * SUB;   // steps per quad
  static constexpr int kQuadSlots = kChunksPerQuad * kChunkSlots;
  // [cols | vals | row words] or [col+row words | vals]; no vals when UNIT
  static constexpr int kArrays = (WIDE ? 3 : 2) - (UNIT ? 1 : 0);
  static constexpr int kRowArray = kArrays - 1;             // WIDE: which array holds the row words
  static constexpr int kQuadInts = kArrays * kQuadSlots;
  static constexpr int kRingInts = 2 * kQuadInts;           // two quads parked per wave

  struct Fetched {  // a quad on its way from memory: slots 4*lane .. 4*lane+3 of each array
    int col[4], val[UNIT ? 1 : 4], row[WIDE ? 4 : 1];
  };

  const float* X;        // first row of X the stream's columns count from
  const int32_t* quads;  // stream of this list
  int n_quads;
  int lane, g;
  int* ring;             // this wave's LDS ring
  unsigned row_bytes, lane_bytes;  // bytes per row of X, byte offset of this lane's features
  Sink sink;
  float acc[VEC];
  float next_acc[VEC];   // heavy lists: what a chunk holds of the piece after the one that ends in it

  __device__ __forceinline__ void fetch(int q, Fetched& f) const {
    q = q < n_quads ? q : n_quads - 1;
    const int4* rec = reinterpret_cast<const int4*>(quads + (size_t)q * kQuadInts);
    const int4 c = rec[lane];
    f.col[0] = c.x; f.col[1] = c.y; f.col[2] = c.z; f.col[3] = c.w;
    if constexpr (!UNIT) {
      const int4 v = rec[kQuadSlots / 4 + lane];
      f.val[0] = v.x; f.val[1] = v.y; f.val[2] = v.z; f.val[3] = v.w;
    }
    if constexpr (WIDE) {
      const int4 r = rec[kRowArray * kQuadSlots / 4 + lane];
      f.row[0] = r.x; f.row[1] = r.y; f.row[2] = r.z; f.row[3] = r.w;
    }
  }

  // what a slot's row word says (WIDE: its own array; compact: the upper bits of the column word)
  static __device__ __forceinline__ int local_row(int r) { return WIDE ? (r & 0xFFFF) : ((r >> kCompactColBits) & 127); }
  static __device__ __forceinline__ bool row_valid(int r) {
    return WIDE ? (r >= 0 && ((r >> 23) & 1) == 0) : ((r >> 27) & 1) != 0;
  }
  static __device__ __forceinline__ bool slot_hands_over(int r) { return WIDE ? ((r >> 22) & 1) != 0 : r < 0; }

  __device__ __forceinline__ int* slot_of(int q) const { return ring + (q & 1) * kQuadInts; }

  // parks quad q; m[i] receives the facts of its chunk i (wave-uniform), taken from the chunk's slot 0:
  // log2w | hand-over << 6 | no row << 7 (WIDE) or real | log2w code << 1 | hand-over << 4 (compact).
  // (slot 0 of a chunk is an entry, or a slot past the end of queue 0, or the whole chunk is padding at the
  //  end of a list, which chunk_is_padding() tells apart)
  __device__ __forceinline__ void park(int q, const Fetched& f, int (&m)[kChunksPerQuad]) const {
    int4* st = reinterpret_cast<int4*>(slot_of(q));
    st[lane] = make_int4(f.col[0], f.col[1], f.col[2], f.col[3]);
    if constexpr (!UNIT) st[kQuadSlots / 4 + lane] = make_int4(f.val[0], f.val[1], f.val[2], f.val[3]);
    if constexpr (WIDE) st[kRowArray * kQuadSlots / 4 + lane] = make_int4(f.row[0], f.row[1], f.row[2], f.row[3]);
#pragma unroll
    for (int i = 0; i < kChunksPerQuad; ++i) {
      if constexpr (WIDE) m[i] = __builtin_amdgcn_readlane(f.row[0], i * (kChunkSlots / 4)) >> 16;
      else m[i] = (int)((unsigned)__builtin_amdgcn_readlane(f.col[0], i * (kChunkSlots / 4)) >> 27);
    }
  }

  static __device__ __forceinline__ bool chunk_is_padding(int m) { return WIDE ? m == -1 : m == 0x1E; }

  // UB consecutive ints of the ring (UB is 4 or 8; the offset is a multiple of UB): 16-byte LDS reads
  __device__ __forceinline__ void read_ints(const int* p, int (&out)[UB]) const {
    const int4* p4 = reinterpret_cast<const int4*>(__builtin_assume_aligned(p, 16));
#pragma unroll
    for (int j = 0; j < UB; j += 4) {
      int4 t = p4[j / 4];
      out[j] = t.x; out[j + 1] = t.y; out[j + 2] = t.z; out[j + 3] = t.w;
    }
  }

  // first slot of this lane group in step s of a quad (s = 0 .. kQuadSteps-1), as an offset into a quad array
  __device__ __forceinline__ int first_slot(int s) const { return s * CS + g * UB; }

  // gathers: the UB rows of X this lane group multiplies in one step
  __device__ __forceinline__ void issue(const int (&c)[UB], float (&x)[UB][VEC]) const {
#pragma unroll
    for (int j = 0; j < UB; ++j) {
      const unsigned col = WIDE ? (unsigned)c[j] : ((unsigned)c[j] & ((1u << kCompactColBits) - 1u));
      if constexpr (IDX32) {
        // column ids are below 2^24 here, so the 24-bit multiply-add is exact
        unsigned off = __umul24(col, row_bytes) + lane_bytes;
        load_vec<VEC>(x[j], reinterpret_cast<const float*>(reinterpret_cast<const char*>(X) + off));
      } else {
        load_vec<VEC>(x[j], reinterpret_cast<const float*>(reinterpret_cast<const char*>(X) +
                                                            (size_t)col * row_bytes + lane_bytes));
      }
    }
  }

  // step s of the quad parked at `st` whose chunk facts are m[].  The stream holds two kinds of chunks:
  //  * queue chunks (log2w 3): slots 8q .. 8q+7 continue queue q of the (row block, partition); every slot
  //    names its row and the last entry of a row piece carries the hand-over flag;
  //  * chunks cut from one wide row (log2w >= 6), which all lane groups share; the chunk's hand-over flag
  //    says whether the row ends with it.
  // (w: with UNIT the row words of the step's slots, which step() has read to tell real slots from others)
  __device__ __forceinline__ void consume(const int* st, int s, int meta, const float (&v)[UB],
                                          const float (&x)[UB][VEC], const int (&w)[UB]) {
    // (compact: a chunk cut from a row wider than 64 slots carries code 7; the test below only asks lw >= 6)
    const int lw = WIDE ? (meta & 63) : ((meta >> 1) & 7);
    const bool hand_over = ((meta >> (WIDE ? 6 : 4)) & 1) != 0;
    const int sub = s & (SUB - 1);
    const int* rows = st + (WIDE ? kRowArray * kQuadSlots : 0);
    if (Sink::kQueues && lw < 6) {
      int r[UB];
      if constexpr (UNIT) {
#pragma unroll
        for (int j = 0; j < UB; ++j) r[j] = w[j];
      } else {
        read_ints(rows + first_slot(s), r);
      }
#pragma unroll
      for (int j = 0; j < UB; ++j) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = fmaf(v[j], x[j][e], acc[e]);
        if (slot_hands_over(r[j])) {  // (only entries carry the flag: the slots past the end of a queue do not)
          sink(local_row(r[j]), true, acc);
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
        }
      }
      if constexpr (SUB == 1 && UB == 8) return;  // this lane group walks the queue alone: the sum stays in registers
      // Any other shape meets the queue again in another lane group or step, so what has been summed of an
      // unfinished row is handed over now.  Lane groups that share the eight slots of a queue may hold
      // parts of the same row: they take turns.
      constexpr int kTurns = UB < 8 ? 8 / UB : 1;
#pragma unroll
      for (int turn = 0; turn < kTurns; ++turn)
        sink(local_row(r[UB - 1]), row_valid(r[UB - 1]) && (g & (kTurns - 1)) == turn, acc);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
      return;
    }
    if constexpr (!Sink::kQueues) {
      // Heavy lists: pieces follow each other without a gap, so a chunk may hold the end of one piece (at the
      // slot its words name) and the start of the next.  What lies past the end is summed apart and becomes
      // the running sum once the finished piece has been handed over.
      if (!hand_over) {
#pragma unroll
        for (int j = 0; j < UB; ++j)
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc[e] = fmaf(v[j], x[j][e], acc[e]);
        return;
      }
      const int end_slot = local_row(rows[(s - sub) * CS]);
      const int slot0 = sub * CS + g * UB;  // this lane group's first slot of the chunk in this step
#pragma unroll
      for (int j = 0; j < UB; ++j) {
        const bool before = slot0 + j <= end_slot;
        const float va = before ? v[j] : 0.f, vb = before ? 0.f : v[j];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          acc[e] = fmaf(va, x[j][e], acc[e]);
          next_acc[e] = fmaf(vb, x[j][e], next_acc[e]);
        }
      }
      if (sub != SUB - 1) return;
      sum_groups<VEC, LG>(acc, S::kGroups);
      sink(0, g == 0, acc);
#pragma unroll
      for (int e = 0; e < VEC; ++e) { acc[e] = next_acc[e]; next_acc[e] = 0.f; }
      return;
    }
#pragma unroll
    for (int j = 0; j < UB; ++j)
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] = fmaf(v[j], x[j][e], acc[e]);
    if (!(hand_over && sub == SUB - 1)) return;  // the row goes on: keep the sums in registers
    sum_groups<VEC, LG>(acc, S::kGroups);
    // (a row cut into several chunks keeps its partial sums in registers in between, so even groups past the
    //  last real slot take part; its row sits in the chunk's slot 0)
    const int r = rows[(s - sub) * CS];
    sink(local_row(r), g == 0 && row_valid(r), acc);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  }

  __device__ __forceinline__ void run() {
#pragma unroll
    for (int e = 0; e < VEC; ++e) { acc[e] = 0.f; next_acc[e] = 0.f; }
    if (n_quads <= 0) return;
    // Quads 0 and 1 are requested at once and quad 0 is parked.  From then on, at the start of quad Q, quad Q+1
    // (requested a whole quad earlier, so long arrived: a load that is waited for too early stalls every load
    // queued behind it) is parked and quad Q+2 is requested.
    Fetched f, f_first;
    fetch(0, f_first);
    fetch(1, f);
    // The request for quad 1 has to be issued before the first gathers, as the request for quad Q+2 is issued
    // before the last gathers of quad Q in the loop.  Loads return in order; if the compiler moved this one behind
    // the gathers here, the wait for it at the top of the loop (entered from here as well as from its own end)
    // would have to cover every gather in flight, in every iteration.
    __builtin_amdgcn_sched_barrier(0);
    int m_cur[kChunksPerQuad], m_next[kChunksPerQuad];
    park(0, f_first, m_cur);
    static_assert(DEPTH >= 2 && DEPTH <= kQuadSteps && kQuadSteps % DEPTH == 0, "steps in flight must divide a quad");
    float x[DEPTH][UB][VEC];
#pragma unroll
    for (int b = 0; b < DEPTH; ++b) {
      int c[UB];
      read_ints(slot_of(0) + first_slot(b), c);
      issue(c, x[b]);
    }
    // one step of quad Q: `xs` holds the gathers of step s and is refilled with those of step s + DEPTH
    auto step = [&](int Q, int s, float (&xs)[UB][VEC], bool refill) {
      const int* st = slot_of(Q);
      int t[UB];
      float v[UB];
      // LDS reads first: their latency hides behind what follows
      if constexpr (UNIT) {
        read_ints(st + (WIDE ? kRowArray * kQuadSlots : 0) + first_slot(s), t);
#pragma unroll
        // (compact: bit 27 says "entry"; as a float, 1 or 0)
        for (int j = 0; j < UB; ++j) v[j] = WIDE ? (row_valid(t[j]) ? 1.f : 0.f) : (float)(((unsigned)t[j] >> 27) & 1u);
      } else {
        read_ints(st + kQuadSlots + first_slot(s), t);
#pragma unroll
        for (int j = 0; j < UB; ++j) v[j] = __int_as_float(t[j]);
      }
      int c[UB];
      if (refill) {
        const int s2 = s + DEPTH;
        read_ints((s2 < kQuadSteps ? st : slot_of(Q + 1)) + first_slot(s2 & (kQuadSteps - 1)), c);
      }
      consume(st, s, m_cur[s / SUB], v, xs, t);
      if (refill) issue(c, xs);
    };
    int Q = 0;
    for (; Q + 1 < n_quads; ++Q) {
      park(Q + 1, f, m_next);
#pragma unroll
      for (int s = 0; s < kQuadSteps; ++s) {
        step(Q, s, x[s % DEPTH], true);
        // Loads come back in issue order, so the slow request for quad Q+2 (it comes from memory, the gathers
        // from L2) delays whatever is issued after it.  Placed right behind a batch of gathers, the first
        // loads it can delay are those of the next step, which are not needed before DEPTH more steps.
        if (s == 0) fetch(Q + 2, f);
      }
#pragma unroll
      for (int i = 0; i < kChunksPerQuad; ++i) m_cur[i] = m_next[i];
    }
    // last quad: its first DEPTH steps are in flight, nothing follows it, and the padding chunks that round the
    // list up to whole quads are neither gathered for nor multiplied
    int n_real = 0;
#pragma unroll
    for (int i = 0; i < kChunksPerQuad; ++i) n_real += chunk_is_padding(m_cur[i]) ? 0 : SUB;
#pragma unroll
    for (int s = 0; s < kQuadSteps; ++s)
      if (s < n_real) step(Q, s, x[s % DEPTH], s + DEPTH < n_real);
  }
};

// (smem: per wavefront its [row_block][kTile] tile of Y, then its quad ring; bid: the workgroup's number)
template <int VEC, int LG, bool IDX32, bool WIDE, bool UNIT>
__device__ __forceinline__ void lists_workgroup(const SpmmArgs& a, unsigned bid, float* smem) {
  using S = Shape<VEC, LG>;
  using W = HybWalker<VEC, LG, IDX32, WIDE, UNIT, TileSink<VEC, LG>>;
  int64_t unit;
  int tile_id;
  decode_block(bid, a.map_mode, a.map_param, a.n_tiles, &unit, &tile_id);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t slot = unit * kHybWaves + wave;  // the wavefronts of a workgroup are independent of each other
  if (slot >= a.n_row_blocks) return;
  const int64_t rb = a.rb_order[slot];
  const int row_block = 1 << a.log2_row_block;
  const int rb_first = (int)(rb << a.log2_row_block);
  const int rows_here = min(row_block, a.n_rows - rb_first);
  const int g = lane / LG, fl = lane & (LG - 1);
  const int f0 = (a.tile0 + tile_id) * S::kTile + fl * VEC;
  const bool f_active = f0 < a.feat;
  const int wave_floats = row_block * S::kTile + W::kRingInts;
  float* tile = smem + wave * wave_floats;
  int* ring = reinterpret_cast<int*>(tile + row_block * S::kTile);

  // the tile starts from zero, or from what earlier launches (column partitions) left in Y; with UNIT what it
  // sums still has to be multiplied by the row's value, so the earlier Y joins at the end instead
  float* y0 = a.Y + (size_t)rb_first * (size_t)a.feat + f0;
  for (int r = g; r < row_block; r += S::kGroups) {
    float init[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) init[e] = 0.f;
    if (!UNIT && a.accumulate && f_active && r < rows_here) load_vec<VEC>(init, y0 + (size_t)r * (size_t)a.feat);
    store_vec<VEC>(tile + tile_index<VEC, LG>(r, fl), init);
  }

  const int64_t c0 = a.rb_chunk_ptr[rb];
  const int n_list = (int)(a.rb_chunk_ptr[rb + 1] - c0);  // a multiple of kChunksPerQuad
  const int f_read = f_active ? f0 : 0;  // lanes past the last feature read a valid address, never store
  W wk{a.X, a.stream + (size_t)c0 * (W::kArrays * kChunkSlots), n_list / kChunksPerQuad, lane, g, ring,
       (unsigned)a.feat * 4u, (unsigned)f_read * 4u, TileSink<VEC, LG>{tile, fl}, {}, {}};
  wk.run();

  // write the tile: a lane group per row, one 128-byte line per group
  if (f_active) {
    for (int r = g; r < rows_here; r += S::kGroups) {
      float out[VEC];
      load_vec<VEC>(out, tile + tile_index<VEC, LG>(r, fl));
      if constexpr (UNIT) {
        const float v = a.row_val[rb_first + r];
        float before[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) before[e] = 0.f;
        if (a.accumulate) load_vec<VEC>(before, y0 + (size_t)r * (size_t)a.feat);
#pragma unroll
        for (int e = 0; e < VEC; ++e) out[e] = fmaf(v, out[e], before[e]);
      }
      store_vec<VEC>(y0 + (size_t)r * (size_t)a.feat, out);
    }
  }
}

template <int VEC, int LG, bool IDX32, bool WIDE, bool UNIT>
__global__ __launch_bounds__(kHybBlock) void k_spmm_hyb(SpmmArgs a) {
  extern __shared__ __align__(16) float smem[];
  lists_workgroup<VEC, LG, IDX32, WIDE, UNIT>(a, blockIdx.x, smem);
}

// ------------------------------------------------------------ heavy pieces
struct HeavyArgs {
  const int32_t* stream;       // the whole chunk stream
  const int32_t* first_slot;   // [n_lists] partial-sum row of each list's first write
  const float* X;
  float* partial;              // [n_partial_rows][kPartialFeat]
  int64_t chunk0;              // first heavy chunk in the stream
  int64_t n_chunks;            // heavy chunks (a multiple of kChunksPerQuad)
  int32_t list0;               // this launch sums lists list0 .. list0 + n_lists - 1
  int32_t n_lists;
  int32_t list_chunks;         // chunks per list
  int32_t feat;
  int32_t feat0;               // first feature of this sweep (partial-sum rows hold kPartialFeat features)
  int32_t n_tiles;             // feature tiles of this sweep
  int32_t map_mode;
  int32_t map_param;
};

// One wavefront per (heavy list, feature tile): the list's chunks (list_chunks of them) are walked like any other
// list, but a finished piece goes to the next partial-sum row instead of an LDS tile, and so does, at the end,
// what has been summed of the piece the list stops in (zeros if it stops at a piece end: every wavefront takes
// that row, so that the row numbers follow from counting alone).
// (smem: per wavefront its quad ring; bid: the workgroup's number among those that walk heavy lists)
template <int VEC, int LG, bool IDX32, bool WIDE, bool UNIT>
__device__ __forceinline__ void heavy_workgroup(const HeavyArgs& a, unsigned bid, float* smem) {
  using S = Shape<VEC, LG>;
  using W = HybWalker<VEC, LG, IDX32, WIDE, UNIT, PartialSink<VEC, LG>>;
  int64_t unit;
  int tile_id;
  decode_block(bid, a.map_mode, a.map_param, a.n_tiles, &unit, &tile_id);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (unit * kHybWaves + wave >= a.n_lists) return;
  const int64_t list = a.list0 + unit * kHybWaves + wave;
  const int g = lane / LG, fl = lane & (LG - 1);
  const int f_in_sweep = tile_id * S::kTile + fl * VEC;
  const int f0 = a.feat0 + f_in_sweep;
  const bool f_active = f0 < a.feat;
  int* ring = reinterpret_cast<int*>(smem) + wave * W::kRingInts;
  const int64_t c0 = list * a.list_chunks;
  const int64_t left = a.n_chunks - c0;
  const int n_list = (int)(left < a.list_chunks ? left : a.list_chunks);
  const int f_read = f_active ? f0 : 0;  // lanes past the last feature read a valid address, never store
  W wk{a.X, a.stream + (size_t)(a.chunk0 + c0) * (W::kArrays * kChunkSlots), n_list / kChunksPerQuad, lane, g, ring,
       (unsigned)a.feat * 4u, (unsigned)f_read * 4u,
       PartialSink<VEC, LG>{a.partial + f_in_sweep, __builtin_amdgcn_readfirstlane(a.first_slot[list]), f_active}, {}, {}};
  wk.run();
  sum_groups<VEC, LG>(wk.acc, S::kGroups);
  wk.sink(0, g == 0, wk.acc);
}

template <int VEC, int LG, bool IDX32, bool WIDE, bool UNIT>
__global__ __launch_bounds__(kHybBlock) void k_spmm_heavy(HeavyArgs a) {
  extern __shared__ __align__(16) float smem[];
  heavy_workgroup<VEC, LG, IDX32, WIDE, UNIT>(a, blockIdx.x, smem);
}

// Both in one launch, for a matrix whose chunk lists and heavy lists are one launch each and small: the first
// n_heavy_workgroups workgroups (a multiple of 8, so that the others keep their place among the XCDs; those past the
// last heavy list leave at once) walk heavy lists, the rest chunk lists, and neither waits for the other.
template <int VEC, int LG, bool IDX32, bool WIDE, bool UNIT>
__global__ __launch_bounds__(kHybBlock) void k_spmm_hyb_heavy(SpmmArgs a, HeavyArgs ha, unsigned n_heavy_workgroups) {
  extern __shared__ __align__(16) float smem[];
  if (blockIdx.x < n_heavy_workgroups) heavy_workgroup<VEC, LG, IDX32, WIDE, UNIT>(ha, blockIdx.x, smem);
  else lists_workgroup<VEC, LG, IDX32, WIDE, UNIT>(a, blockIdx.x - n_heavy_workgroups, smem);
}

// Y[r, feat0 + f] += (row_val[r] *) the partial sums of row r's heavy pieces.  SPLIT groups of (width / VEC) threads per
// row with heavy pieces: group p takes the partial-sum rows number p, p + SPLIT, .. of the row's list (four loads in
// flight, four running sums), the groups' sums meet in LDS and the first group adds them in group order: a fixed
// order of additions whatever the launch, so the result is reproducible.  SPLIT = 8 serves matrices with few, long
// heavy rows (a row of 13,000 entries cut into lists of 4 chunks has 50 partial sums), SPLIT = 1 the others.
// Runs after the chunk-list launches have written Y.
template <int VEC, int SPLIT>
__global__ __launch_bounds__(256) void k_heavy_reduce(const int32_t* __restrict__ heavy_rows,
                                                      const int32_t* __restrict__ row_slot_ptr,
                                                      const int32_t* __restrict__ row_slots,
                                                      const float* __restrict__ partial,
                                                      const float* __restrict__ row_val, float* Y, int32_t n_rows,
                                                      int32_t feat, int32_t feat0, int32_t width) {
  __shared__ float part_sum[SPLIT > 1 ? 256 * VEC : 1];
  const int per_row = width / VEC;
  const int group = per_row * SPLIT;    // threads per row (at most 256: per_row <= 32 when SPLIT > 1)
  const int rows_per_wg = 256 / group;
  const int local = threadIdx.x;
  const int row_in_wg = local / group, part = (local % group) / per_row, f = (local % per_row) * VEC;
  const int64_t row_idx = (int64_t)blockIdx.x * rows_per_wg + row_in_wg;  // (among the rows with heavy pieces)
  const bool active = row_in_wg < rows_per_wg && row_idx < n_rows;
  float sum[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) sum[i] = 0.f;
  int64_t r = 0;
  if (active) {
    r = heavy_rows[row_idx];
    const int b = row_slot_ptr[r], e = row_slot_ptr[r + 1];
    float acc[4][VEC];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[u][i] = 0.f;
    for (int j = b + part; j < e; j += 4 * SPLIT) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int jj = j + u * SPLIT;
        if (jj < e) {
          float v[VEC];
          load_vec<VEC>(v, partial + (size_t)row_slots[jj] * kPartialFeat + f);
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[u][i] += v[i];
        }
      }
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) sum[i] = (acc[0][i] + acc[1][i]) + (acc[2][i] + acc[3][i]);
  }
  if constexpr (SPLIT > 1) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) part_sum[local * VEC + i] = sum[i];
    __syncthreads();
    if (active && part == 0)
      for (int p = 1; p < SPLIT; ++p)
#pragma unroll
        for (int i = 0; i < VEC; ++i) sum[i] += part_sum[(local + p * per_row) * VEC + i];
  }
  if (!active || part != 0) return;
  const float scale = row_val ? row_val[r] : 1.f;  // (the heavy lists of a value-less stream sum rows of X only)
  float* y = Y + (size_t)r * (size_t)feat + feat0 + f;
  float out[VEC];
  load_vec<VEC>(out, y);
#pragma unroll
  for (int i = 0; i < VEC; ++i) out[i] = fmaf(scale, sum[i], out[i]);
  store_vec<VEC>(y, out);
}

struct CsrArgs {
  const int32_t* indptr;
  const int32_t* indices;
  const float* values;
  const float* X;
  float* Y;
  int32_t n_rows;
  int32_t feat;
  int32_t n_tiles;
  int32_t map_mode;
  int32_t map_param;
};

constexpr int kCsrWaves = 4;

// no-hyb: one wavefront per (row, feature tile); the row is walked whole
template <int VEC, int LG>
__global__ __launch_bounds__(64 * kCsrWaves) void k_spmm_csr(CsrArgs a) {
  using S = Shape<VEC, LG>;
  int64_t unit;
  int tile_id;
  decode_block(blockIdx.x, a.map_mode, a.map_param, a.n_tiles, &unit, &tile_id);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t row = unit * kCsrWaves + wave;
  if (row >= a.n_rows) return;
  const int begin = a.indptr[row], end = a.indptr[row + 1];
  const int lane = threadIdx.x & 63;
  const int f0 = tile_id * S::kTile + (lane & (LG - 1)) * VEC;
  const bool f_active = f0 < a.feat;
  float* y = a.Y + (size_t)row * (size_t)a.feat + f0;
  if (end == begin) {  // empty row
    if (f_active && lane < LG) {
      float zero[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) zero[e] = 0.f;
      store_vec<VEC>(y, zero);
    }
    return;
  }
  DirectSink<VEC, LG> sink{y, f_active};
  walk_row<VEC, LG>(a.indices + begin, a.values + begin, a.X + f0, a.feat, end - begin, lane, f_active, sink);
}

// launch geometry shared by both SpMM entry points
struct Geometry {
  int vec, lg, n_tiles, map_mode, map_param;
  int64_t grid;
};

// how n_tiles feature tiles (g->n_tiles) and n_units units are dealt to workgroups
bool plan_tiles(int64_t n_units, Geometry* g) {
  if (g->n_tiles % 8 == 0) {
    g->map_mode = kMapTilesPerXcd; g->map_param = g->n_tiles / 8;
    g->grid = n_units * g->n_tiles;
  } else if (8 % g->n_tiles == 0) {
    g->map_mode = kMapXcdsPerTile; g->map_param = 8 / g->n_tiles;
    g->grid = 8 * ((n_units + g->map_param - 1) / g->map_param);
  } else {
    g->map_mode = kMapPlain; g->map_param = 0;
    g->grid = n_units * g->n_tiles;
  }
  return g->grid <= 0x7FFFFFFF;
}

bool plan(int64_t n_units, int feat, const void* X, const void* Y, bool full_rows, Geometry* g) {
  uintptr_t align = (uintptr_t)X | (uintptr_t)Y;
  lane_shape(feat, (align & 15) == 0, (align & 7) == 0, full_rows, &g->vec, &g->lg);
  int tf = g->vec * g->lg;
  g->n_tiles = (feat + tf - 1) / tf;
  return plan_tiles(n_units, g);
}

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + nb && b0 < a0 + na;
}

// the template arguments of the two hyb kernels as a value
template <int VEC, int LG, bool IDX32, bool WIDE, bool UNIT>
struct Variant {
  static constexpr int vec = VEC, lg = LG;
  static constexpr bool idx32 = IDX32, wide = WIDE, unit = UNIT;
};

template <int VEC, int LG, bool UNIT, typename F>
void with_flags(bool idx32, bool wide, F&& f) {
  if (wide) {
    if (idx32) f(Variant<VEC, LG, true, true, UNIT>{}); else f(Variant<VEC, LG, false, true, UNIT>{});
  } else {
    if (idx32) f(Variant<VEC, LG, true, false, UNIT>{}); else f(Variant<VEC, LG, false, false, UNIT>{});
  }
}

template <bool UNIT, typename F>
void with_shape(int vec, int lg, bool idx32, bool wide, F&& f) {
  if (vec == 4 && lg == 32) with_flags<4, 32, UNIT>(idx32, wide, f);
  else if (vec == 4 && lg == 8) with_flags<4, 8, UNIT>(idx32, wide, f);
  else if (vec == 4) with_flags<4, 4, UNIT>(idx32, wide, f);
  else if (vec == 2) with_flags<2, 16, UNIT>(idx32, wide, f);
  else with_flags<1, 32, UNIT>(idx32, wide, f);
}

// calls f with the Variant that matches the lane geometry and the stream's record form
template <typename F>
void with_variant(int vec, int lg, bool idx32, bool wide, bool unit, F&& f) {
  if (unit) with_shape<true>(vec, lg, idx32, wide, f);
  else with_shape<false>(vec, lg, idx32, wide, f);
}

template <typename V>
void launch_lists(V, const Geometry& g, size_t lds_bytes, hipStream_t stream, const SpmmArgs& a) {
  auto* kernel = &k_spmm_hyb<V::vec, V::lg, V::idx32, V::wide, V::unit>;
  static std::once_flag raised;  // row blocks of 256 rows need more than the default 64 KB of dynamic LDS
  std::call_once(raised, [&] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              160 * 1024 - 1024);
  });
  hipLaunchKernelGGL(kernel, dim3((unsigned)g.grid), dim3(kHybBlock), lds_bytes, stream, a);
}

template <typename V>
void launch_heavy_and_lists(V, unsigned n_heavy_workgroups, unsigned n_list_workgroups, size_t lds_bytes,
                            hipStream_t stream, const SpmmArgs& a, const HeavyArgs& ha) {
  auto* kernel = &k_spmm_hyb_heavy<V::vec, V::lg, V::idx32, V::wide, V::unit>;
  static std::once_flag raised;
  std::call_once(raised, [&] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              160 * 1024 - 1024);
  });
  hipLaunchKernelGGL(kernel, dim3(n_heavy_workgroups + n_list_workgroups), dim3(kHybBlock), lds_bytes, stream, a, ha,
                     n_heavy_workgroups);
}

// workgroups of k_spmm_hyb the GPU holds at once (0: unknown)
template <typename V>
int resident_workgroups(V, size_t lds_bytes) {
  int per_cu = 0, n_cu = 0, dev = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_spmm_hyb<V::vec, V::lg, V::idx32, V::wide, V::unit>, kHybBlock,
                                                   lds_bytes) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  const int by_lds = lds_bytes ? (int)((160 * 1024) / lds_bytes) : per_cu;
  if (per_cu > by_lds) per_cu = by_lds;
  return per_cu > 0 && n_cu > 0 ? per_cu * n_cu : 0;
}

template <typename V>
void launch_heavy(V, const Geometry& g, hipStream_t stream, const HeavyArgs& a) {
  const size_t lds_bytes =
      (size_t)kHybWaves * sizeof(int) * 2 * ((V::wide ? 3 : 2) - (V::unit ? 1 : 0)) * kChunkSlots * kChunksPerQuad;
  hipLaunchKernelGGL((k_spmm_heavy<V::vec, V::lg, V::idx32, V::wide, V::unit>), dim3((unsigned)g.grid), dim3(kHybBlock),
                     lds_bytes, stream, a);
}

}  // namespace

// 8 lanes x 16 bytes (one 128-byte line of X per lane group) where size and alignment allow
void lane_shape(int32_t feat, bool aligned16, bool aligned8, bool full_rows, int* vec, int* lg) {
  if (full_rows && feat % 128 == 0 && aligned16) { *vec = 4; *lg = 32; }  // 32 lanes x 16 bytes: 512 bytes of a row
  else if (feat % 4 == 0 && aligned16) { *vec = 4; *lg = feat <= 16 ? 4 : 8; }
  else if (feat % 2 == 0 && aligned8) { *vec = 2; *lg = 16; }
  else { *vec = 1; *lg = 32; }
}

// Feature tiles per sweep over the launches of a call when every launch but the first reads back what the one
// before it wrote to Y (no rounds): that round trip stays inside the 256 MB memory-side cache only if the part of
// Y a sweep touches is well below its size.  So a wide Y is produced in several sweeps, each over a group of
// feature tiles (4 or 8, which still map whole XCDs to a tile).
int tiles_per_sweep(int n_tiles, int tile_floats, int64_t n_rows, int n_launches, int sweep_kb) {
  const double limit_mb = (double)(sweep_kb > 0 ? sweep_kb : 160 * 1024) / 1024.0;
  if (n_launches < 2 || n_tiles % 4 != 0) return n_tiles;
  const double tile_mb = (double)n_rows * tile_floats * sizeof(float) / (1024.0 * 1024.0);
  if (tile_mb * n_tiles <= limit_mb) return n_tiles;
  if (n_tiles % 8 == 0 && tile_mb * 8 <= limit_mb) return 8;
  return 4;
}

// Feature tiles per sweep of a call that runs in rounds: all of them while the part of X they cover stays within
// half of the 256 MB memory-side cache (or sweep_kb kilobytes, if given), else groups of whole kPartialFeat (8 or 4 tiles of 32 floats), so that the
// heavy pieces' partial sums follow the same sweeps.  (The largest graph at 256 features, X of 238 MB: one sweep
// 5.54 ms, two sweeps of 128 features measured faster.)
int round_tiles_per_sweep(int n_tiles, int tile_floats, int64_t n_cols, int sweep_kb) {
  if (tile_floats * 4 != kPartialFeat || n_tiles <= 4) return n_tiles;
  const double limit_mb = (double)(sweep_kb > 0 ? sweep_kb : 128 * 1024) / 1024.0;
  const double tile_mb = (double)n_cols * tile_floats * sizeof(float) / (1024.0 * 1024.0);
  if (tile_mb * n_tiles <= limit_mb) return n_tiles;
  if (tile_mb * 8 <= limit_mb) return 8;
  return 4;
}

// May the gather offsets of a launch be formed with the 24-bit multiply (column x bytes per row of X)?
// Both factors must fit 24 bits and the product, plus a lane's offset inside the row, 32.
bool offsets_fit_32(int64_t n_cols_spanned, int32_t feat) {
  const uint64_t row_bytes = (uint64_t)feat * sizeof(float);
  return row_bytes < (1u << 24) && n_cols_spanned < (1 << 24) &&
         (uint64_t)n_cols_spanned * row_bytes < ((uint64_t)1 << 32);
}

}  // namespace sptir

using namespace sptir;

// Events between the groups of launches of one call (sptir_spmm_timed)
struct LaunchTimers {
  enum Tag { kStart = 0, kLists = 1, kHeavy = 2, kReduce = 3 };
  std::vector<std::pair<hipEvent_t, int>> marks;
  int launches[4] = {0, 0, 0, 0};
  bool failed = false;
  void mark(hipStream_t stream, int tag, int n_launches) {
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess || hipEventRecord(e, stream) != hipSuccess) { failed = true; return; }
    marks.emplace_back(e, tag);
    launches[tag] += n_launches;
  }
  ~LaunchTimers() {
    for (auto& m : marks) (void)hipEventDestroy(m.first);
  }
};

// The work of sptir_spmm; `partial` is where the sums of heavy pieces meet ([n_partial_rows][kPartialFeat] floats;
// only touched when the matrix has heavy pieces).
static sptir_status_t spmm_on_hyb(const sptir_hyb_t* h, const float* X, float* Y, int32_t feat, void* stream_,
                                  float* partial, LaunchTimers* timers = nullptr) {
  if (!h || feat < 1) return SPTIR_ERR_INVALID_ARG;
  if ((h->n_cols > 0 && !X) || (h->n_rows > 0 && !Y)) return SPTIR_ERR_INVALID_ARG;
  const size_t x_bytes = sizeof(float) * (size_t)h->n_cols * feat, y_bytes = sizeof(float) * (size_t)h->n_rows * feat;
  if (x_bytes && y_bytes && overlaps(X, x_bytes, Y, y_bytes)) return SPTIR_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  if (h->n_rows == 0) return SPTIR_OK;
  if (!h->spmm_plan) return SPTIR_ERR_UNSUPPORTED;

  Geometry g;
  const int64_t n_units = ((int64_t)h->n_row_blocks + kHybWaves - 1) / kHybWaves;
  // (512-byte tiles only where a workgroup's Y tiles fit the CU's LDS: a caller who fixes large row blocks and
  //  asks for full rows gets the 128-byte tiles)
  static_assert(kHybWaves == 4, "full_rows_fit() counts four wavefronts per workgroup");
  if (!plan(n_units, feat, X, Y, h->full_rows != 0 && full_rows_fit(h->log2_row_block), &g)) return SPTIR_ERR_OVERFLOW;
  SpmmArgs a;
  a.stream = h->stream;
  a.X = X; a.Y = Y; a.n_rows = h->n_rows; a.n_row_blocks = h->n_row_blocks; a.log2_row_block = h->log2_row_block;
  a.feat = feat; a.n_tiles = g.n_tiles; a.map_mode = g.map_mode; a.map_param = g.map_param;
  // per wavefront: its Y tile and its ring of two quads
  const bool wide = !h->compact_stream, unit = h->row_val != nullptr;
  a.row_val = h->row_val;
  const size_t lds_bytes =
      (size_t)kHybWaves * (sizeof(float) * ((size_t)g.vec * g.lg << h->log2_row_block) +
                           sizeof(int) * 2 * ((wide ? 3 : 2) - (unit ? 1 : 0)) * kChunkSlots * kChunksPerQuad);
  // A compact list holds columns relative to the first column of its launch, which moves into the X pointer.
  const int64_t span = (int64_t)h->parts_per_phase * (int64_t)h->w;
  const bool idx32 = offsets_fit_32(wide ? (int64_t)h->n_cols : (span < h->n_cols ? span : (int64_t)h->n_cols), feat);
  const int all_tiles = g.n_tiles;
  int n_list_launches = 0;
  bool heavy_with_lists = false;
  if (timers) timers->mark(stream, LaunchTimers::kStart, 0);
  const bool idx32_all = offsets_fit_32(h->n_cols, feat);
  // the launch over the heavy lists for the features feat0 .. feat0 + width - 1 (width <= kPartialFeat)
  auto heavy_launch_shape = [&](int feat0, int width, HeavyArgs* ha, Geometry* gh) -> bool {
    ha->stream = h->stream; ha->first_slot = h->hlist_first_slot; ha->X = X; ha->partial = partial;
    ha->chunk0 = h->heavy_chunk0; ha->n_chunks = h->n_heavy_chunks; ha->feat = feat;
    ha->list_chunks = h->heavy_list_chunks;
    *gh = g;
    const int tile = g.vec * g.lg;
    gh->n_tiles = (width + tile - 1) / tile;
    ha->feat0 = feat0; ha->n_tiles = gh->n_tiles;
    ha->list0 = 0; ha->n_lists = h->n_heavy_lists;
    if (!plan_tiles(((int64_t)ha->n_lists + kHybWaves - 1) / kHybWaves, gh)) return false;
    ha->map_mode = gh->map_mode; ha->map_param = gh->map_param;
    return true;
  };
  // Heavy pieces: partial sums of kPartialFeat features at a time, added to the Y the lists have written, for
  // the features feat_begin .. feat_end - 1 (feat_begin a multiple of kPartialFeat).  already_launched: the heavy
  // lists went with the chunk lists' launch, only the sums remain to be added.
  auto heavy_sweeps = [&](int feat_begin, int feat_end, bool already_launched = false) -> sptir_status_t {
    if (h->n_heavy <= 0) return SPTIR_OK;
    const bool y_vec4 = feat % 4 == 0 && ((uintptr_t)Y & 15) == 0;
    for (int feat0 = feat_begin; feat0 < feat_end; feat0 += kPartialFeat) {
      const int width = feat_end - feat0 < kPartialFeat ? feat_end - feat0 : kPartialFeat;
      HeavyArgs ha;
      Geometry gh;
      // The heavy chunks are in partition order and so are the lists: one launch walks them all.  Workgroups start
      // in list order, so the wavefronts resident at any time cover a window of consecutive lists that touches one
      // slice of X, or two while it passes a partition boundary; a launch per partition measured slower (each
      // ended with a partly filled GPU: 1.62 ms against 1.53 on the largest graph).
      if (!heavy_launch_shape(feat0, width, &ha, &gh)) return SPTIR_ERR_OVERFLOW;
      if (!already_launched) {
        with_variant(g.vec, g.lg, idx32_all, wide, unit, [&](auto v) { launch_heavy(v, gh, stream, ha); });
        if (timers) timers->mark(stream, LaunchTimers::kHeavy, 1);
      }
      const int per_row = width / (y_vec4 ? 4 : 1);
      // few rows with heavy pieces: eight groups of threads share a row's partial sums
      const int split = (y_vec4 && (int64_t)h->n_heavy_rows * per_row < 32768) ? 8 : 1;
      const int rows_per_wg = 256 / (per_row * split);
      const int64_t n_wg = ((int64_t)h->n_heavy_rows + rows_per_wg - 1) / rows_per_wg;
      if (n_wg > 0x7FFFFFFF) return SPTIR_ERR_OVERFLOW;
      const dim3 grid((unsigned)n_wg), block(256);
      auto reduce = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, h->heavy_rows, h->row_slot_ptr, h->row_slots, partial,
                           h->row_val, Y, h->n_heavy_rows, feat, feat0, width);
      };
      if (!y_vec4) reduce(k_heavy_reduce<1, 1>);
      else if (split == 8) reduce(k_heavy_reduce<4, 8>);
      else reduce(k_heavy_reduce<4, 1>);
      if (timers) timers->mark(stream, LaunchTimers::kReduce, 1);
    }
    return SPTIR_OK;
  };
  if (h->rounds) {
    // Rounds: a launch takes as many row blocks, in the order of their list lengths, as the GPU holds wavefronts.
    // All of them start together, their lists are about equally long and sweep the column partitions in the same
    // order, so they stay nearly in step; the Y tiles stay in LDS from the first partition to the last.
    // A wide X is taken in sweeps over groups of feature tiles, lists and heavy pieces of one sweep before those
    // of the next: the gathers that miss L2 are then served by the memory-side cache instead of HBM.
    int capacity = 0;
    with_variant(g.vec, g.lg, idx32, wide, unit, [&](auto v) { capacity = resident_workgroups(v, lds_bytes); });
    if (capacity <= 0) capacity = 3 * 256;
    const int tile_floats = g.vec * g.lg;
    const int per_sweep = round_tiles_per_sweep(all_tiles, tile_floats, h->n_cols, h->sweep_kb);
    a.rb_chunk_ptr = h->rb_chunk_ptr; a.accumulate = 0;
    for (int tile0 = 0; tile0 < all_tiles; tile0 += per_sweep) {
      g.n_tiles = all_tiles - tile0 < per_sweep ? all_tiles - tile0 : per_sweep;
      a.n_tiles = g.n_tiles; a.tile0 = tile0;
      int64_t per_round = (int64_t)capacity / g.n_tiles * kHybWaves;  // row blocks
      if (per_round < 8 * kHybWaves) per_round = 8 * kHybWaves;
      const int64_t n_rounds = (h->n_row_blocks + per_round - 1) / per_round;
      per_round = ((h->n_row_blocks + n_rounds - 1) / n_rounds + 7) / 8 * 8;  // rounds of equal size
      for (int64_t first = 0; first < h->n_row_blocks; first += per_round) {
        const int64_t here = h->n_row_blocks - first < per_round ? h->n_row_blocks - first : per_round;
        a.rb_order = h->rb_order + first;
        a.n_row_blocks = (int32_t)here;
        if (!plan_tiles((here + kHybWaves - 1) / kHybWaves, &g)) return SPTIR_ERR_OVERFLOW;
        a.map_mode = g.map_mode; a.map_param = g.map_param;
        with_variant(g.vec, g.lg, idx32, wide, unit, [&](auto v) { launch_lists(v, g, lds_bytes, stream, a); });
        ++n_list_launches;
      }
      if (timers) timers->mark(stream, LaunchTimers::kLists, n_list_launches);
      n_list_launches = 0;
      const int feat_end = (tile0 + g.n_tiles) * tile_floats;
      const sptir_status_t st = heavy_sweeps(tile0 * tile_floats, feat_end < feat ? feat_end : feat);
      if (st != SPTIR_OK) return st;
    }
  } else {
    const int per_sweep = tiles_per_sweep(all_tiles, g.vec * g.lg, h->n_rows, h->n_phases, h->sweep_kb);
    for (int tile0 = 0; tile0 < all_tiles; tile0 += per_sweep) {
      g.n_tiles = all_tiles - tile0 < per_sweep ? all_tiles - tile0 : per_sweep;
      if (!plan_tiles(n_units, &g)) return SPTIR_ERR_OVERFLOW;
      a.n_tiles = g.n_tiles; a.tile0 = tile0; a.map_mode = g.map_mode; a.map_param = g.map_param;
      for (int phase = 0; phase < h->n_phases; ++phase) {
        a.rb_chunk_ptr = h->rb_chunk_ptr + (size_t)phase * h->n_row_blocks;
        a.rb_order = h->rb_order + (size_t)phase * h->n_row_blocks;
        a.accumulate = phase > 0;
        a.X = wide ? X : X + (size_t)phase * (size_t)span * (size_t)feat;
        // A matrix whose chunk lists are one launch and whose heavy lists are the smaller part runs both in one
        // launch: the few wavefronts of the heavy lists then fill CUs the chunk lists leave idle instead of
        // waiting for them (19,717 rows, 88,651 non-zeros, two heavy rows: 0.026 -> 0.023 ms per call).
        HeavyArgs ha;
        Geometry gh;
        if (h->n_heavy > 0 && h->n_phases == 1 && per_sweep == all_tiles && feat <= kPartialFeat &&
            idx32 == idx32_all && heavy_launch_shape(0, feat, &ha, &gh) && gh.grid <= g.grid &&
            (gh.grid + 7) / 8 * 8 + g.grid <= 0x7FFFFFFF) {
          const int64_t heavy_wgs = (gh.grid + 7) / 8 * 8;
          with_variant(g.vec, g.lg, idx32, wide, unit, [&](auto v) {
            launch_heavy_and_lists(v, (unsigned)heavy_wgs, (unsigned)g.grid, lds_bytes, stream, a, ha);
          });
          heavy_with_lists = true;
        } else {
          with_variant(g.vec, g.lg, idx32, wide, unit, [&](auto v) { launch_lists(v, g, lds_bytes, stream, a); });
        }
        ++n_list_launches;
      }
    }
  }
  if (!h->rounds) {
    if (timers) timers->mark(stream, LaunchTimers::kLists, n_list_launches);
    const sptir_status_t st = heavy_sweeps(0, feat, heavy_with_lists);
    if (st != SPTIR_OK) return st;
  }
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}

extern "C" int32_t sptir_gather_offsets_fit_32(int64_t n_cols, int32_t feat) {
  return (n_cols >= 0 && feat >= 1 && offsets_fit_32(n_cols, feat)) ? 1 : 0;
}

extern "C" sptir_status_t sptir_spmm(const sptir_hyb_t* h, const float* X, float* Y, int32_t feat, void* stream_) {
  return spmm_on_hyb(h, X, Y, feat, stream_, h ? h->partial : nullptr);
}

extern "C" sptir_status_t sptir_spmm_timed(const sptir_hyb_t* h, const float* X, float* Y, int32_t feat,
                                           void* stream_, sptir_spmm_times_t* out) {
  if (!out) return SPTIR_ERR_INVALID_ARG;
  LaunchTimers timers;
  const sptir_status_t st = spmm_on_hyb(h, X, Y, feat, stream_, h ? h->partial : nullptr, &timers);
  if (st != SPTIR_OK) return st;
  SPTIR_HIP(hipStreamSynchronize((hipStream_t)stream_));
  if (timers.failed) return note_hip_error(hipGetLastError(), "recording events");
  sptir_spmm_times_t t;
  memset(&t, 0, sizeof(t));
  for (size_t i = 1; i < timers.marks.size(); ++i) {
    float ms = 0.f;
    SPTIR_HIP(hipEventElapsedTime(&ms, timers.marks[i - 1].first, timers.marks[i].first));
    if (timers.marks[i].second == LaunchTimers::kLists) t.ms_lists += ms;
    else if (timers.marks[i].second == LaunchTimers::kHeavy) t.ms_heavy += ms;
    else if (timers.marks[i].second == LaunchTimers::kReduce) t.ms_reduce += ms;
  }
  t.n_list_launches = timers.launches[LaunchTimers::kLists];
  t.n_heavy_launches = timers.launches[LaunchTimers::kHeavy];
  t.n_reduce_launches = timers.launches[LaunchTimers::kReduce];
  *out = t;
  return SPTIR_OK;
}

// ---------------------------------------------------------------- sptir_spmm_noalloc
// The partial sums of heavy pieces in memory that belongs to the loaded code object instead of the handle: every
// GPU the library runs on holds its own copy of this array until the process ends.
static constexpr size_t kStaticScratchFloats = SPTIR_NOALLOC_SCRATCH_BYTES / sizeof(float);
static __device__ __align__(256) float scratch[kStaticScratchFloats];
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
float* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once asked for

// `scratch` itself is only a host-side stand-in for the symbol: what kernels are given is this address.
sptir_status_t scratch_of_current_device(float** out) {
  int dev = -1;
  SPTIR_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SPTIR_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    SPTIR_HIP(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return SPTIR_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SPTIR_OK;
}
}  // namespace

extern "C" sptir_status_t sptir_spmm_noalloc(const sptir_hyb_t* h, const float* X, float* Y, int32_t feat,
                                             void* stream_) {
  if (!h || feat < 1) return SPTIR_ERR_INVALID_ARG;
  float* partial = nullptr;
  if (h->n_heavy > 0) {
    const size_t need = (size_t)h->n_partial_rows * kPartialFeat;
    if (need > kStaticScratchFloats) {
      char msg[256];
      snprintf(msg, sizeof(msg),
               "sptir_spmm_noalloc: the partial sums of %lld heavy row pieces need %zu bytes, more than the "
               "static scratch of %zu bytes; use sptir_spmm",
               (long long)h->n_heavy, need * sizeof(float), (size_t)SPTIR_NOALLOC_SCRATCH_BYTES);
      note_error_text(msg);
      return SPTIR_ERR_UNSUPPORTED;
    }
    const sptir_status_t st = scratch_of_current_device(&partial);
    if (st != SPTIR_OK) return st;
  }
  return spmm_on_hyb(h, X, Y, feat, stream_, partial);
}

extern "C" sptir_status_t sptir_spmm_csr(const sptir_csr_t* csr, const float* X, float* Y, int32_t feat,
                                         void* stream_) {
  if (!csr || feat < 1 || csr->n_rows < 0 || csr->n_cols < 0 || csr->nnz < 0) return SPTIR_ERR_INVALID_ARG;
  if (!csr->indptr || (csr->nnz > 0 && (!csr->indices || !csr->values))) return SPTIR_ERR_INVALID_ARG;
  if ((csr->n_cols > 0 && !X) || (csr->n_rows > 0 && !Y)) return SPTIR_ERR_INVALID_ARG;
  const size_t x_bytes = sizeof(float) * (size_t)csr->n_cols * feat, y_bytes = sizeof(float) * (size_t)csr->n_rows * feat;
  if (x_bytes && y_bytes && overlaps(X, x_bytes, Y, y_bytes)) return SPTIR_ERR_INVALID_ARG;
  if (csr->n_rows == 0) return SPTIR_OK;
  Geometry g;
  if (!plan(((int64_t)csr->n_rows + kCsrWaves - 1) / kCsrWaves, feat, X, Y, false, &g)) return SPTIR_ERR_OVERFLOW;
  CsrArgs a;
  a.indptr = csr->indptr; a.indices = csr->indices; a.values = csr->values; a.X = X; a.Y = Y;
  a.n_rows = csr->n_rows; a.feat = feat; a.n_tiles = g.n_tiles; a.map_mode = g.map_mode; a.map_param = g.map_param;
  dim3 grid((unsigned)g.grid), block(64 * kCsrWaves);
  hipStream_t stream = (hipStream_t)stream_;
  if (g.vec == 4 && g.lg == 8) hipLaunchKernelGGL((k_spmm_csr<4, 8>), grid, block, 0, stream, a);
  else if (g.vec == 4) hipLaunchKernelGGL((k_spmm_csr<4, 4>), grid, block, 0, stream, a);
  else if (g.vec == 2) hipLaunchKernelGGL((k_spmm_csr<2, 16>), grid, block, 0, stream, a);
  else hipLaunchKernelGGL((k_spmm_csr<1, 32>), grid, block, 0, stream, a);
  SPTIR_HIP(hipGetLastError());
  return SPTIR_OK;
}
