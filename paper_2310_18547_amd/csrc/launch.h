// Host-side launch descriptors shared by the C ABI and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sgmv {

// Longest k-slice one shrink workgroup stages in LDS (elements of one x row).
constexpr int kMaxKSlice = 2048;
// Generation of a workspace: the number of single-launch kernels that have run on it, kept
// in this many identical 32-bit copies at its start (workgroup i of a launch reads copy i, so
// the reads of a launch do not all go to one address, and rewrites the copies i, i + n, ...
// on its way out, n being the launch's workgroup count).  Also the most workgroups such a
// launch may have.
constexpr int kGenerationCopies = 1024;
// Bytes reserved at the start of a workspace: the generation copies, then the error word
// (32 bits), the initialisation mark (32 bits) and a 64-bit word for tuning builds
// (csrc/trace.h).
constexpr size_t kWorkspaceErrorOffset = (size_t)kGenerationCopies * 4;
// The 32-bit word after the error word holds this once sgmv_workspace_init has run.
constexpr uint32_t kWorkspaceMagic = 0x564D4753u;  // "SGMV"
constexpr size_t kWorkspaceTraceOffset = kWorkspaceErrorOffset + 8;
constexpr size_t kWorkspaceHeader = kWorkspaceErrorOffset + 256;
// Upper bound of the split-K factor.
constexpr int kMaxKSplit = 64;

// Most add-ons whose MFMA shrinks share one pass over a common x.
constexpr int kSharedShrinkMost = 3;

struct ShrinkArgs {
  bool bf16;
  int r, h_in, n_tokens, n_segs;
  int ksplit, kslice;        // ksplit slices of kslice elements cover h_in, none empty
  int max_seg_len;           // hint, 0 = unknown
  bool by_rows;              // launch_shrink_whole only: a workgroup per row of the batch (it looks its segment up), not per segment
  long long layer_off;       // elements to add to every A pointer
  const void* x;
  const void* const* A_ptrs;
  const int32_t* seg_starts;
  float* partials;           // [ksplit][n_tokens][r]
  unsigned long long* header;// workspace header or nullptr (only trace builds look at it)
  // launch_shrink_matrix_shared only: n_shared add-ons on the same x, each with its pointer array
  // and its own partial sums
  int n_shared;
  const void* const* A_shared[kSharedShrinkMost];
  float* partials_shared[kSharedShrinkMost];
};

// ExpandArgs::threads value that selects expand_split_kernel (256 threads whose four waves divide
// the weight rows of a 512-column strip among themselves; ranks 32 and 64)
constexpr int kExpandSplit = 512;
struct ExpandArgs {
  bool bf16;
  int r, h_out, n_tokens, n_segs;
  int threads;               // vector path: workgroup size
  bool by_rows;              // vector path: a workgroup per row of the batch (it looks its segment up), not per segment
  int max_seg_len;           // hint, 0 = unknown
  long long layer_off;       // elements to add to every B pointer
  void* y;
  const float* v_parts;      // [nparts][n_tokens][r]
  int nparts;
  const void* const* A_ptrs; // may be nullptr
  const void* const* B_ptrs;
  const int32_t* seg_starts;
  float scale;
  // MFMA path only: 16-bit operand pairs of v and the per-row range factor (workspace)
  uint16_t* vh;
  uint16_t* vl;
  float* undo;
  bool operands_ready;       // vh / vl / undo are already written (launch_finalize_shared)
  unsigned long long* header;// workspace header or nullptr (only trace builds look at it)
};

// Most add-ons one multi-projection launch takes.
constexpr int kMaxProjections = 8;
// Per-projection pointers of a multi-projection launch (passed by value as a kernel argument).
struct FusedTable {
  const void* x[kMaxProjections];
  void* y[kMaxProjections];
  const void* A_ptrs[kMaxProjections];
  const void* B_ptrs[kMaxProjections];
};

struct FusedArgs {
  bool bf16;
  int r, h_in, h_out, n_tokens, n_segs;
  int S;                     // workgroups per segment = k-slices = column slices
  int kslice, cslice;        // elements per k-slice / columns per column slice
  int G;                     // lane groups of the expand phase (1, 2, 4 or 8)
  int rows_per_pass;         // 1 when every segment is a single row, else 4
  bool by_rows;              // the grid's items are the n_tokens rows, each looking its segment up, not the segments
  int spin_limit;            // polls before a waiting workgroup gives up
  long long offA, offB;      // layer offsets in elements
  float scale;
  void* y;
  const void* x;
  const void* const* A_ptrs;
  const void* const* B_ptrs;
  const int32_t* seg_starts;
  unsigned long long* exch;  // [S][n_tokens][r] words {value, generation tag}
  unsigned long long* header;// generation copies, then the error word
  int n_proj;                // 0: one add-on (x, y, A_ptrs, B_ptrs above); else `table` holds n_proj of them
  int Z;                     // multi-projection launch: grid depth (projections z, z + Z, ... per workgroup)
  FusedTable table;
};

// Single-launch kernel for segments of a few rows (sixteen-row MFMA tiles).
constexpr size_t kTileMaxLds = 160 * 1024;  // LDS of one compute unit
constexpr size_t kTileExclusiveLds = 81 * 1024;  // more than half of it: one workgroup per unit
struct TileArgs {
  bool bf16;
  int r, h_in, h_out, n_tokens, n_segs;
  int S;                     // workgroups per segment and row block = k-slices = column slices
  int Z;                     // grid depth: row blocks of a segment are dealt round-robin over it
  int kslice, cslice;        // multiples of 32 / 64
  int spin_limit;
  size_t lds_bytes;          // tile_lds_bytes(r, kslice, cslice)
  long long offA, offB;
  float scale;
  void* y;
  const void* x;
  const void* const* A_ptrs;
  const void* const* B_ptrs;
  const int32_t* seg_starts;
  unsigned long long* exch;
  unsigned long long* header;
  int n_proj;                // 0 or 1: one add-on (x, y, A_ptrs, B_ptrs above); else `table` holds n_proj of them, side by side
  FusedTable table;
};

// Single-launch kernel for one-row segments in which every workgroup computes the whole
// shrink of its segment (no hand-off between workgroups, no workspace).
constexpr int kWholeMaxHin = 8192;  // widest input row a workgroup stages in LDS
struct WholeArgs {
  bool bf16;
  bool by_rows;               // a set of S workgroups per row of the batch (it looks its segment up), not per segment
  int r, h_in, h_out, n_segs, n_tokens;
  int S;                     // workgroups per segment = column slices of the expand
  int cslice;                // columns per slice
  int G;                     // lane groups of the expand phase (1, 2, 4 or 8)
  long long offA, offB;      // layer offsets in elements
  float scale;
  void* y;
  const void* x;
  const void* const* A_ptrs;
  const void* const* B_ptrs;
  const int32_t* seg_starts;
  unsigned long long* header;  // workspace header or nullptr (only trace builds look at it)
};

// Grid of add_lora_fused_kernel: (fused_grid_x, S, rows of fused_grid_x segments).  Workgroups
// are dealt to the eight XCDs round-robin by linear id, so with eight segments to a grid row
// the S workgroups of a segment all run on one XCD: they start together (the XCDs of a launch
// start up to 0.6 us apart) and none of them waits for a partial sum from a later XCD.
inline int fused_grid_x(int n_segs) { return n_segs < 8 ? (n_segs > 0 ? n_segs : 1) : 8; }
// Workgroups of such a grid per slice: the items (segments, or segments x row blocks) rounded
// up to whole grid rows.
inline long long fused_grid_items(long long items) {
  const long long gx = items < 8 ? (items > 0 ? items : 1) : 8;
  return (items + gx - 1) / gx * gx;
}

size_t tile_lds_bytes(int r, int kslice, int cslice);
hipError_t launch_add_lora_whole(const WholeArgs& a, hipStream_t st);
hipError_t launch_add_lora_tile(const TileArgs& a, hipStream_t st);
hipError_t launch_add_lora_fused(const FusedArgs& a, hipStream_t st);
// Stand-alone shrink of one-row segments in one launch (x, A_ptrs, S, kslice and the hand-off fields of `a`).
hipError_t launch_shrink_handoff(const FusedArgs& a, float* v, hipStream_t st);
// Single-launch shrink of one-row segments without Split-K: one workgroup per segment adds x A_i to v.
bool shrink_whole_fits(const ShrinkArgs& a);
hipError_t launch_shrink_whole(const ShrinkArgs& a, float* v, hipStream_t st);
bool fused_multi_fits(const FusedArgs& a);
hipError_t launch_add_lora_fused_multi(const FusedArgs& a, hipStream_t st);
hipError_t launch_workspace_init(void* p, size_t bytes, size_t header_offset, hipStream_t st);
hipError_t launch_shrink_vector(const ShrinkArgs& a, hipStream_t st);
hipError_t launch_shrink_reduce(float* v, const ShrinkArgs& a, hipStream_t st);
hipError_t launch_expand_vector(const ExpandArgs& a, hipStream_t st);
hipError_t launch_shrink_matrix(const ShrinkArgs& a, hipStream_t st);
// True when n_shared add-ons' slices of A_i fit in LDS side by side (launch_shrink_matrix_shared applies).
bool shrink_shared_fits(const ShrinkArgs& a, int n_shared);
// The MFMA shrink of a.n_shared add-ons on the same x in one pass (A_shared, partials_shared).
hipError_t launch_shrink_matrix_shared(const ShrinkArgs& a, hipStream_t st);
// v -> operand pairs of the n add-ons of a shared shrink in one launch (each es[i] with its own vh / vl / undo).
hipError_t launch_finalize_shared(const ExpandArgs* es, int n, hipStream_t st);
hipError_t launch_expand_matrix(const ExpandArgs& a, hipStream_t st);

}  // namespace sgmv
