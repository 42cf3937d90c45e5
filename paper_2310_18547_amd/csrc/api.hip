// C ABI of libsgmv: argument checks, launch-shape choice, kernel dispatch.
// Everything that computes runs in the kernels; this file only validates and
// enqueues.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "../../include/sgmv.h"
#include "launch.h"

// Scratch of sgmv_add_lora_static, one copy per GPU, held until the process ends:
//   [0, 4.25 KiB)    header (generation copies, error word)
//   [4.25 KiB, 6 MiB) exchange words of the single-launch kernels -- at a fixed place whatever
//                    the batch, so that a word found there was always written as an exchange
//                    word, with the generation tag of an earlier call
//   [6 MiB, 9 MiB)   split-K partial sums and the MFMA expand's operands of v
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the
// address that call returned.
constexpr size_t kStaticExchangeEnd = (size_t)6 << 20;
constexpr size_t kStaticBytes = (size_t)9 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];
static_assert(kStaticBytes == SGMV_STATIC_SCRATCH_BYTES, "the header states the array's size");

namespace {

using namespace sgmv;

constexpr int kMinSplitCap = 16;       // the workspace always allows this many slices
constexpr int kTargetWorkgroups = 512; // about two workgroups per compute unit
// Longest segment the single-launch MFMA kernel is considered for.  What really limits it is
// that every (segment, sixteen-row block, slice) workgroup must be resident at once with its
// weight slices in LDS (choose_tile): about 64 row blocks in all at h = 4096.
constexpr int kTileMaxSegLen = 4096;
constexpr int kMatrixMaxSegments = 65535;  // the MFMA kernels put the segment on a grid dimension limited to this
constexpr int kFusedSlices = 8;        // most slices per segment the single-launch kernels pick
constexpr int kRowsMostSegments = 256;  // segments up to which SGMV_PATH_AUTO launches per row (four rounds of the look-up)
constexpr long long kShrinkWholeMostElements = 48LL << 20;  // weights (96 MB) up to which the stand-alone shrink runs without Split-K
constexpr int kTileMultiSlices = 4;    // fewest slices at which a joint tile launch beats add-ons run per row
constexpr int kFusedMaxWorkgroups = kGenerationCopies;  // every workgroup of a launch has its own generation copy
constexpr int kFusedSpinLimit = 1 << 18;
constexpr int kMaxDevices = 64;
constexpr int kDefaultComputeUnits = 256;  // MI355X; assumed where no device can be asked

// Residency limits of the single-launch kernels.  They follow from the compute units of the
// current device (asked once per device): a workgroup that waits for the partial sums of a
// workgroup that has not started yet only idles, so these launches stay within what is
// resident at once.
struct Limits {
  int fused_workgroups;       // one workgroup per compute unit
  int tile_max_grid;          // tile launch, workgroups without rows included (5/4 per unit)
  int multi_workgroups;       // multi-projection launch side by side (two per unit)
  int multi_workgroups_most;  // ... where the pipelined kernel does not apply (three per unit)
};

int compute_units() {
  static std::atomic<int> cached[kMaxDevices];  // zero-initialised
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();  // no device here (a host-only query): leave no sticky error behind
    return kDefaultComputeUnits;
  }
  int cu = cached[dev].load(std::memory_order_relaxed);
  if (cu == 0) {
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) {
      (void)hipGetLastError();
      cu = kDefaultComputeUnits;
    }
    cached[dev].store(cu, std::memory_order_relaxed);
  }
  return cu;
}

Limits limits() {
  const int cu = compute_units();
  // launches far beyond one workgroup per unit measured slower than the launch-per-step kernels
  // (tile kernel, 456 workgroups for 171 with rows: 25.8 us against 14.8 us) even though the
  // surplus leaves at once
  return Limits{cu, cu + cu / 4, 2 * cu, 3 * cu};
}

int spin_limit_of(const sgmv_problem* p) { return p->spin_limit > 0 ? p->spin_limit : kFusedSpinLimit; }
// AUTO uses the MFMA kernels from this segment length on.  Their work goes with the number of
// segments (every segment occupies at least one block of 64 rows), that of the vector kernels
// with the rows: measured at h = 4096, 128 segments of 4 rows, ranks 8 / 16 / 32 / 64: vector
// kernels 14.4 / 18.2 / 28.9 / 45.1 us against 23.9 / 26.3 / 31.3 / 47.7; 64 segments of 8 rows,
// ranks 16 / 64: MFMA 19.1 / 37.6 against 25.1 / 60.6.
constexpr int kMatrixMinSegLen = 6;
// At rank 64 the vector kernels are slow enough that the MFMA kernels win from two rows per
// segment on while the segments are few (32 segments of 2 / 4 rows: 21.7 / 21.9 us against 23.1 /
// 31.4; the Uniform mix of 39 segments: 26.3 against 34.6; 64 segments of 4 rows: 36.9 against 34.0).
constexpr int kMatrixFewSegments = 48;
constexpr int kMatrixWorkgroups = 448; // workgroups the MFMA shrink aims for

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }
inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Most split-K slices the workspace is sized for at a given batch.
int split_cap(int n_tokens) {
  int c = ceil_div(16384, n_tokens > 0 ? n_tokens : 1);
  if (c > kMaxKSplit) c = kMaxKSplit;
  if (c < kMinSplitCap) c = kMinSplitCap;
  return c;
}

int check_common(const sgmv_problem* p, const int32_t* seg_starts, int32_t n_segs,
                 int32_t layer_idx, bool need_in, bool need_out) {
  if (p == nullptr) return SGMV_ERR_NULL;
  if (p->dtype != SGMV_F16 && p->dtype != SGMV_BF16) return SGMV_ERR_UNSUPPORTED;
  if (n_segs < 0 || p->n_tokens < 0 || p->num_layers <= 0 || p->max_seg_len < 0)
    return SGMV_ERR_SHAPE;
  if (p->r <= 0 || (need_in && p->h_in <= 0) || (need_out && p->h_out <= 0)) return SGMV_ERR_SHAPE;
  if (p->r != 8 && p->r != 16 && p->r != 32 && p->r != 64) return SGMV_ERR_UNSUPPORTED;
  if ((need_in && (p->h_in % 8) != 0) || (need_out && (p->h_out % 8) != 0))
    return SGMV_ERR_UNSUPPORTED;
  if (p->path < SGMV_PATH_AUTO || p->path > SGMV_PATH_ROWS) return SGMV_ERR_UNSUPPORTED;
  if (p->spin_limit < 0) return SGMV_ERR_UNSUPPORTED;
  if (p->ksplit < 0 || p->ksplit > kMaxKSplit) return SGMV_ERR_UNSUPPORTED;
  if (p->expand_threads != 0 && p->expand_threads != 64 && p->expand_threads != 128 &&
      p->expand_threads != 256 && !(p->expand_threads == kExpandSplit && p->r >= 32))
    return SGMV_ERR_UNSUPPORTED;
  if (p->path == SGMV_PATH_MATRIX && n_segs > 65535) return SGMV_ERR_UNSUPPORTED;  // grid dimension of the MFMA kernels
  if (layer_idx < 0 || layer_idx >= p->num_layers) return SGMV_ERR_RANGE;
  if (n_segs > 0 && p->n_tokens > 0 && seg_starts == nullptr) return SGMV_ERR_NULL;
  return SGMV_OK;
}

int check_workspace(const sgmv_problem* p) {
  if (p->workspace == nullptr) return SGMV_ERR_WORKSPACE;
  if (!aligned(p->workspace, 256)) return SGMV_ERR_ALIGN;
  if (p->workspace_bytes < sgmv_workspace_bytes(p->n_tokens, p->r)) return SGMV_ERR_WORKSPACE;
  return SGMV_OK;
}

// Split-K shape: ksplit slices of kslice elements, kslice a multiple of 8 and at
// most kMaxKSlice, no slice empty.  Returns false when h_in is too wide for the
// workspace's slice count.
bool choose_split(const sgmv_problem* p, int n_segs, int* ksplit, int* kslice) {
  const int cap = split_cap(p->n_tokens);
  const int need = ceil_div(p->h_in, kMaxKSlice);
  if (need > cap) return false;
  // enough workgroups to fill the chip, but slices of at least 32 KiB of weights: more
  // slices than that only lengthen the reduction that follows (measured, 1 to 64 segments)
  int s = p->ksplit;
  if (s == 0) {
    s = ceil_div(kTargetWorkgroups, n_segs);
    const int by_size = ceil_div((long long)p->h_in * p->r, 16384);
    if (s > by_size) s = by_size;
  }
  const int most = p->h_in / 64 > 0 ? p->h_in / 64 : 1;  // keep slices >= 64 elements
  if (s > most) s = most;
  if (s > cap) s = cap;
  if (s < need) s = need;
  int len = ceil_div(ceil_div(p->h_in, s), 8) * 8;
  *kslice = len;
  *ksplit = ceil_div(p->h_in, len);
  return true;
}

// Whether a call goes to the MFMA kernels: forced, or segments long enough that
// 16-row tiles are mostly full (from the hint, else from the mean length).
bool use_matrix(const sgmv_problem* p, int n_segs) {
  if (p->path == SGMV_PATH_MATRIX) return true;
  if (p->path != SGMV_PATH_AUTO) return false;
  if (n_segs > kMatrixMaxSegments) return false;  // the vector kernels take any number of segments
  const int len = p->max_seg_len > 0 ? p->max_seg_len : p->n_tokens / (n_segs > 0 ? n_segs : 1);
  if (p->r >= 64 && n_segs <= kMatrixFewSegments && len >= 2) return true;
  return len >= kMatrixMinSegLen;
}

// The stand-alone expand at rank 64 is ahead on the MFMA kernels for more short segments than the
// shrink and the add-on are (h = 4096, 64 segments of 2 / 4 rows: 12.4 / 12.7 us against 16.1 / 20.4
// on the vector kernel; Uniform mix of 128 rows, 56 segments: 11.8 against 27.3; 128 segments of 2
// rows: 20.3 against 20.6).
bool expand_use_matrix(const sgmv_problem* p, int n_segs) {
  if (use_matrix(p, n_segs)) return true;
  if (p->path != SGMV_PATH_AUTO || p->r < 64 || n_segs > 128) return false;
  const int len = p->max_seg_len > 0 ? p->max_seg_len : p->n_tokens / (n_segs > 0 ? n_segs : 1);
  return len >= 2;
}

// Split-K shape of the MFMA shrink: row blocks of 64 rows times ksplit slices should
// give every compute unit a workgroup; slices are multiples of the MFMA depth (32).
void choose_split_matrix(const sgmv_problem* p, int n_segs, int* ksplit, int* kslice) {
  const int cap = split_cap(p->n_tokens);
  const int blocks = p->n_tokens / 64 + (n_segs + 1) / 2;
  int s = p->ksplit > 0 ? p->ksplit : ceil_div(kMatrixWorkgroups, blocks > 0 ? blocks : 1);
  const int most = p->h_in / 256 > 0 ? p->h_in / 256 : 1;  // keep slices >= one LDS chunk
  if (s > most) s = most;
  // slices no deeper than what stays resident in LDS (the streaming shrink), if the
  // workspace has room for that many partial sums
  const int need = ceil_div(p->h_in, 512);
  if (p->ksplit == 0 && s < need) s = need;
  if (s > cap) s = cap;
  if (s < 1) s = 1;
  const int len = ceil_div(ceil_div(p->h_in, s), 32) * 32;
  *kslice = len;
  *ksplit = ceil_div(p->h_in, len);
}

size_t partial_bytes(int n_tokens, int r) {
  return round_up((size_t)split_cap(n_tokens) * (size_t)n_tokens * (size_t)r * sizeof(float), 256);
}

// Where a call keeps its intermediate results.
struct Scratch {
  unsigned long long* header;  // generation copies, error word
  float* partials;             // split-K partial sums of the launch-per-step kernels
  unsigned long long* exch;    // exchange words of the single-launch kernels
  char* operands;              // 16-bit operand pairs of v and a range factor per row (MFMA expand)
};

// Caller's workspace: [header][partials][exchange words, twice the bytes][operands].
Scratch caller_scratch(const sgmv_problem* p) {
  char* base = static_cast<char*>(p->workspace);
  const size_t parts = partial_bytes(p->n_tokens, p->r);
  return Scratch{reinterpret_cast<unsigned long long*>(base),
                 reinterpret_cast<float*>(base + kWorkspaceHeader),
                 reinterpret_cast<unsigned long long*>(base + kWorkspaceHeader + parts),
                 base + kWorkspaceHeader + 3 * parts};
}

// Operands of the MFMA expand: v as high and low 16-bit parts, one range factor per row.
size_t operand_bytes(int n_tokens, int r) {
  return 2 * round_up((size_t)n_tokens * r * 2, 256) + round_up((size_t)n_tokens * 4, 256);
}
void set_operands(ExpandArgs* a, const Scratch& sc, int n_tokens, int r) {
  char* base = sc.operands;
  a->header = sc.header;
  const size_t half = round_up((size_t)n_tokens * r * 2, 256);
  a->vh = reinterpret_cast<uint16_t*>(base);
  a->vl = reinterpret_cast<uint16_t*>(base + half);
  a->undo = reinterpret_cast<float*>(base + 2 * half);
}

// Launch shape of the single-launch path; false when it does not apply.
// by_rows: the launch's items are the rows of the batch (pass n_tokens for n_segs), each looking its
// segment up on the device, so the segments may have any length.
bool choose_fused(const sgmv_problem* p, int n_segs, FusedArgs* f, bool single_add_on = true, bool by_rows = false) {
  if (!p->workspace_ready) return false;
  const Limits lim = limits();
  f->by_rows = by_rows;
  if (p->max_seg_len != 1 && !by_rows) return false;  // one row per segment; longer ones go to the tile kernel
  if (n_segs > kFusedMaxWorkgroups) return false;
  const int cap = split_cap(p->n_tokens);
  const int need = ceil_div(p->h_in, kMaxKSlice);
  if (need > cap) return false;
  // every workgroup of a launch must be resident at once (one per compute unit): a
  // workgroup that waits for a slice of a workgroup not yet started only idles
  int s = p->ksplit > 0 ? p->ksplit : lim.fused_workgroups / n_segs;
  if (p->ksplit == 0 && s > kFusedSlices) s = kFusedSlices;
  if (p->ksplit == 0) {  // a power of two: measured 5-20 % faster than the odd counts in between
    int pw = 1;
    while (pw * 2 <= s) pw *= 2;
    s = pw;
  }
  // 97 .. 128 segments of a single add-on: four slices, two workgroups per unit, rather than two
  // (measured at h = 4096, 128 segments, r = 16 / 32: 9.35 / 18.0 us against 9.81 / 18.8; no
  // difference at 96 segments or at rank 64; wider inputs are better off as they are)
  if (p->ksplit == 0 && single_add_on && s == 2 && n_segs > 96 && 2 * n_segs <= lim.fused_workgroups &&
      p->r <= 32 && need <= 2)
    s = 4;
  // Small batches at high rank: where a slice of A_i at eight slices takes more than one batch
  // of loads (2048 128-bit chunks), sixteen slices are faster while they are all resident
  // (measured at r = 64, h = 4096 / 5120, 1..8 segments: 5.1 / 5.8 us against 5.4 / 6.7 us)
  // The same holds for the slice of B_i of a wide output (4096 -> 11008 at rank 32, 1 / 8 / 16
  // segments: 5.7 / 5.9 / 7.1 us against 6.2 / 6.7 / 8.1), and it does not hold at rank 16, where
  // the chunks are short (h_in = 11008 / 13824, 1 .. 16 segments: eight slices 3-5 % ahead).
  const int wide = p->h_in > p->h_out ? p->h_in : p->h_out;
  if (p->ksplit == 0 && s == kFusedSlices && 2 * s * n_segs <= lim.fused_workgroups && p->r >= 32 &&
      (long long)ceil_div(wide, s) * (p->r / 8) > 2048)
    s = 2 * kFusedSlices;
  if (s > wide / 64) s = wide / 64;
  // Narrow shapes: no more slices than leave each a full batch of loads (2048 128-bit chunks of the
  // wider weight); thinner ones only add the hand-off (measured at rank 16, 8 segments, one / two /
  // four / eight slices: h = 1024 3.84 / 4.07 / 4.26 / 4.33 us, h = 2048 4.94 / 4.17 / 4.20 / 4.29; at
  // h = 4096 four and eight are level, 4.38 / 4.37)
  if (p->ksplit == 0 && wide <= 2048) {
    const int full = (int)((long long)wide * (p->r / 8) / 2048);
    if (s > (full > 1 ? full : 1)) s = full > 1 ? full : 1;
  }
  if (s > cap) s = cap;
  if (s > kFusedMaxWorkgroups / n_segs) s = kFusedMaxWorkgroups / n_segs;
  if (s < need) s = need;
  if (s < 1) s = 1;
  // a slice count forced by a wide input to five, six or seven: eight instead, where the launch
  // has room (measured at 64 segments, h_in = 11008, six -> eight slices: rank 64 31.9 -> 27.5 us,
  // rank 16 9.79 -> 9.53; h_in = 13824, seven -> eight: no difference)
  if (p->ksplit == 0 && single_add_on && s == need && s > 4 && s < 8 &&
      8LL * ceil_div(n_segs, fused_grid_x(n_segs)) * fused_grid_x(n_segs) <= kFusedMaxWorkgroups && 8 <= cap &&
      8 <= wide / 64)
    s = 8;
  // the grid is padded to whole rows of segments (launch.h, fused_grid_x)
  const int gx = fused_grid_x(n_segs);
  if ((long long)s * ceil_div(n_segs, gx) * gx > kFusedMaxWorkgroups) return false;
  // slices forced by a very wide input can outnumber the compute units several times over;
  // from about two rounds of workgroups on the launch-per-step kernels are faster (measured)
  // (per-row launches, sized by their own rule, rows_apply: up to three rounds, 384 rows at two slices)
  if (p->path == SGMV_PATH_AUTO && p->ksplit == 0 && (long long)s * n_segs > (by_rows ? 3 : 2) * lim.fused_workgroups)
    return false;
  // From rank 32 on, a launch of more workgroups than units is only worth it when the units get
  // equal shares: 288 or 384 workgroups leave most units waiting for the ones with two (measured
  // against the launch-per-step kernels, h = 5120, three slices, 96 / 128 segments: rank 32 22.4 /
  // 24.3 against 19.1 / 22.1 us, rank 64 36.3 / 40.1 against 30.7 / 35.2; h = 8192, four slices,
  // 96 segments: 27.8 against 24.7 and 45.2 against 41.5; 512 workgroups are fine: 128 segments
  // at h = 4096, rank 32: 18.0 against 19.6)
  if (p->path == SGMV_PATH_AUTO && p->ksplit == 0 && p->r >= 32 && (long long)s * n_segs > lim.fused_workgroups) {
    const long long wg = (long long)s * n_segs;
    const long long rounds = ceil_div((int)wg, lim.fused_workgroups);
    if (rounds * lim.fused_workgroups * 5 > wg * 6) return false;  // more than 20 % of the slots idle
  }
  // likewise batches of more than 128 segments that need two slices each (measured at
  // h = 4096, r = 16: 192 segments 17.3 us here against 15.5 us, 256 segments 20.0 against 18.3)
  // (not so rows of longer segments: 129 .. 256 of them at two slices share their weights)
  if (p->path == SGMV_PATH_AUTO && p->ksplit == 0 && !by_rows && n_segs > lim.fused_workgroups / 2 &&
      (long long)s * n_segs > lim.fused_workgroups)
    return false;
  f->S = s;
  f->kslice = ceil_div(ceil_div(p->h_in, s), 8) * 8;
  f->cslice = ceil_div(ceil_div(p->h_out, s), 8) * 8;
  const int chunks = f->cslice / 8;
  // Lane groups of the expand phase: as many as give every lane a chunk of the column slice, and
  // enough that a lane holds at most sixteen weight rows.  A single add-on at ranks up to 16 stops
  // at two (the pair of neighbouring lanes that needs no LDS to add up, fused_kernel.hip) even
  // where that leaves lanes without a chunk: measured at h = 4096, r = 16, 1 / 8 / 16 / 32 segments:
  // 4.02 / 4.42 / 4.43 / 4.83 us against 4.07 / 4.54 / 4.59 / 5.01 us; at ranks 32 and 64 and in
  // the multi-projection launches the wider groups are faster (16 segments at rank 32: 5.02
  // against 5.46 us).
  const int most = single_add_on && p->r <= 16 ? 2 : 8;
  int g = 1;
  while (g * 2 <= most && 256 / (g * 2) >= chunks) g *= 2;
  if (most == 2 && g == 1 && chunks <= 128) g = 2;
  while (p->r / g > 16) g *= 2;
  f->G = g;
  f->rows_per_pass = 1;
  return true;
}

// Launch shape of the single-launch kernel without hand-off (one-row segments, every workgroup
// computes the whole shrink); false when it does not apply.
// by_rows: the launch's items are the rows of the batch (pass n_tokens for n_segs), each looking its
// segment up on the device, so the segments may have any length.
bool choose_whole(const sgmv_problem* p, int n_segs, WholeArgs* w, bool by_rows = false) {
  w->by_rows = by_rows;
  if (p->max_seg_len != 1 && !by_rows) return false;
  if (p->h_in > kWholeMaxHin) return false;
  // A_i is walked in whole steps of 256 128-bit loads
  if ((long long)p->h_in * (p->r / 8) % 256 != 0) return false;
  if (n_segs > 8 * 65535) return false;  // grid depth
  const Limits lim = limits();
  // as many column slices as keep the launch within one workgroup per compute unit
  int s = p->ksplit > 0 ? p->ksplit : lim.fused_workgroups / n_segs;
  if (p->ksplit == 0 && s > kFusedSlices) s = kFusedSlices;
  if (p->ksplit == 0) {
    int pw = 1;
    while (pw * 2 <= s) pw *= 2;
    s = pw;
  }
  if (s > p->h_out / 64) s = p->h_out / 64;
  if (s < 1) s = 1;
  w->S = s;
  w->cslice = ceil_div(ceil_div(p->h_out, s), 8) * 8;
  const int chunks = w->cslice / 8;
  const int most = p->r <= 16 ? 2 : 8;  // lane groups: as choose_fused
  int g = 1;
  while (g * 2 <= most && 256 / (g * 2) >= chunks) g *= 2;
  if (most == 2 && g == 1 && chunks <= 128) g = 2;
  while (p->r / g > 16) g *= 2;
  w->G = g;
  return true;
}

// Launch shape of the single-launch MFMA kernel; false when it does not apply.
// n_proj > 1: that many add-ons of this shape side by side in one launch (each segment's row blocks
// and slices once per add-on, all resident together).
bool choose_tile(const sgmv_problem* p, int n_segs_one, TileArgs* t, int n_proj = 1) {
  const int n_segs = n_segs_one * n_proj;
  const long long n_rows = (long long)p->n_tokens * n_proj;
  if (!p->workspace_ready) return false;
  const Limits lim = limits();
  if (p->max_seg_len <= 0 || p->max_seg_len > kTileMaxSegLen) return false;
  if (n_segs > kFusedMaxWorkgroups) return false;
  // At rank 64 a full block of sixteen rows hands 8 KB of tagged words per slice from workgroup
  // to workgroup, and the launch-per-step MFMA kernels are ahead from about ten rows per segment
  // on (h = 4096, one segment of 16 / 64 / 256 rows: 14.8 / 16.0 / 17.8 us against 20.2 / 20.2 /
  // 20.7 here; Skewed mix of 32 rows, longest segment 12: 15.4 against 17.0; segments of up to 8
  // rows: 13.0-15.5 here against 14.8-17.2)
  // (a joint launch of several add-ons hands them over side by side in the same 20 us, which beats
  // the launch-per-step kernels one add-on after the other from about 64 rows on: two segments
  // of 32 rows, three add-ons 21.4 against 25.1 us; of 64 rows 22.4 against 48.7; one of 32 rows
  // 20.9 against 18.4)
  if (p->path == SGMV_PATH_AUTO && p->r >= 64 && p->max_seg_len > 8 && (n_proj < 2 || p->n_tokens < 64)) return false;
  const int cap = split_cap(p->n_tokens);
  const int narrow = p->h_in < p->h_out ? p->h_in : p->h_out;
  int z = ceil_div(p->max_seg_len, 16);
  // The launch has n_segs * z row blocks, but only those that hold rows keep a compute unit
  // (the others leave at once): at most n_segs + n_tokens / 16 of them.  These, times the
  // slices, must all be resident together (one workgroup per unit).
  long long blocks = (long long)n_segs * z;
  long long live = blocks < (long long)n_segs + n_rows / 16 ? blocks : (long long)n_segs + n_rows / 16;
  if (live > lim.fused_workgroups) {  // too many even with one slice: fewer row blocks, walked with a stride
    z = lim.fused_workgroups / n_segs > 0 ? lim.fused_workgroups / n_segs : 1;
    blocks = live = (long long)n_segs * z;
  }
  // (Fewer row blocks per segment than the longest one needs would leave room for more slices
  // where the weight slices do not fit the LDS, but workgroups that walk several blocks in turn
  // measured slower than the launch-per-step kernels.)
  int s = p->ksplit > 0 ? p->ksplit : (int)(lim.fused_workgroups / live);
  if (p->ksplit == 0 && s > kFusedSlices) s = kFusedSlices;
  if (p->ksplit == 0 && s > lim.tile_max_grid / blocks) s = (int)(lim.tile_max_grid / blocks);  // workgroups launched in all
  if (s > narrow / 64) s = narrow / 64;  // no slice thinner than 64
  if (s > cap / n_proj) s = cap / n_proj;  // every add-on its own exchange words
  if (s < 1) s = 1;
  if (s * n_proj > cap) return false;
  if (s * live > lim.fused_workgroups || s * blocks > lim.tile_max_grid) return false;
  for (;; ++s) {  // more slices make the LDS-resident weight slices smaller
    t->kslice = ceil_div(ceil_div(p->h_in, s), 32) * 32;
    t->cslice = ceil_div(ceil_div(p->h_out, s), 64) * 64;
    t->lds_bytes = tile_lds_bytes(p->r, t->kslice, t->cslice);
    if (t->lds_bytes <= kTileMaxLds) break;
    if (p->ksplit > 0 || (s + 1) * n_proj > cap || (s + 1) * live > lim.fused_workgroups || (s + 1) * blocks > lim.tile_max_grid)
      return false;
  }
  t->S = s;
  t->Z = z;
  t->n_proj = n_proj;
  return true;
}

void fill_fused(FusedArgs* f, const sgmv_problem* p, const Scratch& sc, const int32_t* seg_starts,
                int n_segs, int layer_idx, float scale) {
  f->bf16 = p->dtype == SGMV_BF16;
  f->r = p->r;
  f->h_in = p->h_in;
  f->h_out = p->h_out;
  f->n_tokens = p->n_tokens;
  f->n_segs = n_segs;
  f->spin_limit = spin_limit_of(p);
  f->offA = (long long)layer_idx * p->h_in * p->r;
  f->offB = (long long)layer_idx * p->r * p->h_out;
  f->seg_starts = seg_starts;
  f->exch = sc.exch;
  f->header = sc.header;
  f->scale = scale;
  f->n_proj = 0;
  f->Z = 1;
  f->y = nullptr;
  f->x = nullptr;
  f->A_ptrs = f->B_ptrs = nullptr;
}

// Everything of a tile launch but its shape (choose_tile) and the add-on's own pointers.
void fill_tile(TileArgs* t, const sgmv_problem* p, const Scratch& sc, const int32_t* seg_starts, int n_segs,
               int layer_idx, float scale) {
  t->bf16 = p->dtype == SGMV_BF16;
  t->r = p->r;
  t->h_in = p->h_in;
  t->h_out = p->h_out;
  t->n_tokens = p->n_tokens;
  t->n_segs = n_segs;
  t->spin_limit = spin_limit_of(p);
  t->offA = (long long)layer_idx * p->h_in * p->r;
  t->offB = (long long)layer_idx * p->r * p->h_out;
  t->y = nullptr;
  t->x = nullptr;
  t->A_ptrs = t->B_ptrs = nullptr;
  t->seg_starts = seg_starts;
  t->exch = sc.exch;
  t->header = sc.header;
  t->scale = scale;
}

// Workgroup shape of the vector expand for `n_segs` items (segments, or rows of a per-row launch):
// 64, 128 or 256 threads of eight columns each, or kExpandSplit.
int choose_expand_threads(const sgmv_problem* p, int n_segs) {
  if (p->expand_threads) return p->expand_threads;
  // From rank 32 on a lane of the plain kernel walks its R weight rows sixteen at a time, one
  // memory round trip after the other; while the launch is small the kernel whose four waves
  // divide the rows among themselves is ahead (measured at h = 4096, one-row segments, us per
  // call, plain against divided: rank 64, 1 / 16 / 64 / 128 segments 8.5 / 10.2 / 12.9 / 17.2
  // against 3.9 / 5.4 / 8.4 / 14.6; rank 32, 16 / 64 / 128: 6.0 / 7.7 / 10.2 against 3.9 / 5.5 /
  // 8.2; 4096 -> 11008, 64 segments, rank 32 / 64: 11.7 / 19.0 against 9.9 / 17.1), up to about
  // five and a half of its workgroups per compute unit (1408: ahead; 192 segments at rank 64,
  // 1536: 19.2 against 20.6; 256 at rank 32, 2048: 13.3 against 14.5)
  if (p->r >= 32 && (long long)n_segs * ceil_div(p->h_out, 512) <= 11LL * compute_units() / 2) return kExpandSplit;
  const int sizes[3] = {256, 128, 64};
  for (int i = 0; i < 3; ++i)
    if ((long long)n_segs * ceil_div(p->h_out, sizes[i] * 8) >= kTargetWorkgroups / 2 ||
        i == 2)
      return sizes[i];
  return 64;
}

ShrinkArgs make_shrink(const sgmv_problem* p, const Scratch& sc, const void* x,
                       const void* const* A_ptrs, const int32_t* seg_starts, int n_segs,
                       int layer_idx) {
  ShrinkArgs a;
  a.bf16 = p->dtype == SGMV_BF16;
  a.r = p->r;
  a.h_in = p->h_in;
  a.n_tokens = p->n_tokens;
  a.n_segs = n_segs;
  a.ksplit = a.kslice = 0;
  a.max_seg_len = p->max_seg_len;
  a.by_rows = false;
  a.layer_off = (long long)layer_idx * p->h_in * p->r;
  a.x = x;
  a.A_ptrs = A_ptrs;
  a.seg_starts = seg_starts;
  a.partials = sc.partials;
  a.header = sc.header;
  a.n_shared = 0;
  return a;
}

ExpandArgs make_expand(const sgmv_problem* p, void* y, const float* v_parts, int nparts,
                       const void* const* A_ptrs, const void* const* B_ptrs,
                       const int32_t* seg_starts, int n_segs, int layer_idx, float scale) {
  ExpandArgs a;
  a.bf16 = p->dtype == SGMV_BF16;
  a.r = p->r;
  a.h_out = p->h_out;
  a.n_tokens = p->n_tokens;
  a.n_segs = n_segs;
  a.threads = choose_expand_threads(p, n_segs);
  a.max_seg_len = p->max_seg_len;
  a.layer_off = (long long)layer_idx * p->r * p->h_out;
  a.y = y;
  a.v_parts = v_parts;
  a.nparts = nparts;
  a.A_ptrs = A_ptrs;
  a.B_ptrs = B_ptrs;
  a.seg_starts = seg_starts;
  a.scale = scale;
  a.vh = a.vl = nullptr;
  a.undo = nullptr;
  a.operands_ready = false;
  a.header = nullptr;
  a.by_rows = false;
  return a;
}

// Small batches of segments longer than a row (or of unknown length): whether AUTO runs the
// one-row kernel with the hand-off per ROW of the batch (SGMV_PATH_ROWS), every row's workgroups
// reading the row's adapter through the caches, rather than the tile kernel (`tile`: it applies, with
// `tile_slices` slices) or the launch-per-step kernels.  Measured on MI355X, binary16, us per add-on,
// per row against what AUTO took before:
//  * up to 64 rows it wins at every rank and width measured (ranks 8 .. 64; 4096, 5120, 8192 square,
//    4096 -> 11008, 11008 -> 4096; 31 segment mixes and five popularity mixes each: 129 of 132 cases at
//    rank 64 faster, the rest within 2 %).  At 4096 x 4096, rank 16, 64 rows: Uniform 5.33 against
//    7.16 (tile kernel), Skewed 4.88 against 7.58, Identical 4.88 against 7.23, 8 segments of 8 rows
//    4.85 against 7.12; rank 64: Uniform 11.7 against 22.7 (MFMA kernels), 8 x 8 rows 9.4 against 14.2.
//  * 65 .. 128 rows: ahead up to rank 32 (rank 16, 128 rows: Uniform 6.40 against 9.29, Skewed 6.13
//    against 11.9, one segment 5.79 against 7.27, 16 x 8 rows 5.85 against 7.60; rank 32: 4 x 32 rows
//    7.96 against 10.3, Uniform 9.16 against 11.4; behind by at most 12 % on 24 segments of 4 rows
//    at rank 32 and on 32 x 4 rows at 5120), not at rank 64 (two slices per row leave each workgroup
//    half of B_i: 4096 -> 11008, 8 x 16 rows: 27.2 against 17.3).
//  * 129 .. 256 rows, ranks up to 16: ahead where the tile kernel does not apply or gets fewer than
//    its eight slices (Skewed of 256 rows 9.05 against 18.9, Uniform 7.88 against 9.83, 128 x 2 rows
//    11.7 against 14.7; behind on 40 .. 64 segments of 4 rows, by up to 17 %), 4-8 % ahead elsewhere,
//    which is left to the tile kernel.
bool rows_apply(const sgmv_problem* p, int n_segs, bool tile, int tile_slices) {
  if (p->max_seg_len == 1 || p->ksplit != 0 || !p->workspace_ready) return false;
  // the look-up takes a round per 64 segments: not for batches of mostly empty segments
  if (n_segs > kRowsMostSegments) return false;
  if (p->n_tokens <= 64) return true;
  // (rank 64 at 65 .. 128 rows: only at widths up to 4096 and where the tile kernel is out: Uniform
  // of 128 rows 15.3 against 44.5 us, one segment of 128 rows 12.8 against 17.4, 32 x 4 rows 17.6
  // against 19.6; with the tile kernel to choose from, 16 x 8 rows 16.6 against 15.5)
  if (p->n_tokens <= 128)
    return p->r <= 32 || (!tile && p->h_in <= 4096 && p->h_out <= 4096);
  if (p->n_tokens <= 256) return p->r <= 16 && (!tile || tile_slices < 8);
  //  * 257 .. 384 rows, ranks up to 16, inputs up to 4096 wide (two slices): only where the tile kernel
  //    is out or down to three slices (Skewed of 320 / 384 rows 11.0 / 11.9 against 19.8 / 18.4 us on the
  //    MFMA kernels, 96 x 4 rows 14.0 against 17.2 on the vector kernels; the tile kernel with four
  //    slices and more is ahead by 5-28 %, and at 512 rows, 1024 workgroups, nearly everything is)
  if (p->n_tokens <= 384) return p->r <= 16 && p->h_in <= 4096 && (!tile || tile_slices < 4);
  return false;
}

// The stand-alone expand of a small batch of longer segments (or of unknown length): a workgroup
// per row and column strip instead of per segment, as the add-on does (rows_apply); no workspace
// is involved.
bool expand_by_rows(const sgmv_problem* p, int n_segs) {
  if (p->path != SGMV_PATH_AUTO || p->max_seg_len == 1 || n_segs > kRowsMostSegments) return false;
  if (p->n_tokens <= 64) return true;
  if (p->n_tokens <= 128) return p->r <= 32;
  return p->n_tokens <= 384 && p->r <= 16;
}

// What sgmv_add_lora will launch for a checked problem: the single source of the path
// choice, shared by the entry points and by sgmv_plan_add_lora.
struct SinglePlan {
  int kernel;        // sgmv_kernel
  WholeArgs whole;   // SGMV_KERNEL_WHOLE
  TileArgs tile;     // SGMV_KERNEL_TILE
  FusedArgs fused;   // SGMV_KERNEL_FUSED
  int ksplit, kslice;  // SGMV_KERNEL_MATRIX / SGMV_KERNEL_VECTOR
};

int plan_single(const sgmv_problem* p, int n_segs, SinglePlan* pl) {
  if (p->path == SGMV_PATH_WHOLE) {
    if (!choose_whole(p, n_segs, &pl->whole)) return SGMV_ERR_UNSUPPORTED;
    pl->kernel = SGMV_KERNEL_WHOLE;
    return SGMV_OK;
  }
  if (p->path == SGMV_PATH_ROWS) {
    if (!choose_fused(p, p->n_tokens, &pl->fused, true, true)) return SGMV_ERR_UNSUPPORTED;
    pl->kernel = SGMV_KERNEL_FUSED;
    return SGMV_OK;
  }
  const bool tile = (p->path == SGMV_PATH_AUTO || p->path == SGMV_PATH_FUSED) && p->max_seg_len != 1 &&
                    choose_tile(p, n_segs, &pl->tile);
  if (p->path == SGMV_PATH_AUTO && rows_apply(p, n_segs, tile, tile ? pl->tile.S : 0)) {
    // with an A_i of at most 64 KB the kernel without hand-off, as for one-row segments below
    if ((long long)p->h_in * p->r <= 32768 && p->n_tokens <= 512 && choose_whole(p, p->n_tokens, &pl->whole, true)) {
      pl->kernel = SGMV_KERNEL_WHOLE;
      return SGMV_OK;
    }
    if (choose_fused(p, p->n_tokens, &pl->fused, true, true)) {
      pl->kernel = SGMV_KERNEL_FUSED;
      return SGMV_OK;
    }
  }
  if (tile) {
    pl->kernel = SGMV_KERNEL_TILE;
    return SGMV_OK;
  }
  if (p->path == SGMV_PATH_AUTO || p->path == SGMV_PATH_FUSED) {
    const bool fused = choose_fused(p, n_segs, &pl->fused);
    // One-row segments, measured on MI355X at h = 4096 (us per add-on, whole-shrink kernel
    // against the alternative): at rank 8, where A_i is small, it beats the kernel with the
    // hand-off at every batch (1 / 16 / 64 / 128 segments: 3.7 / 4.0 / 4.8 / 6.0 against 4.1 /
    // 4.7 / 5.2 / 6.2) and the launch-per-step kernels beyond (256: 9.5 against 12.4), but only
    // while A_i is small: at h_in = 8192 the hand-off kernel is 15-20 % ahead at every batch (64
    // segments: 6.2 against 7.4), at 5120 from 64 segments on (5.4 against 6.0; bfloat16 from 32 on); where the
    // hand-off kernel does not apply (no prepared workspace, or more segments than it takes) it
    // beats the launch-per-step kernels up to rank 16 and several hundred segments (192 / 256 /
    // 512: 13.5 / 16.4 / 28.8 against 16.2 / 18.6 / 29.9; 1024: 53.9 against 51.2), without a
    // workspace also at rank 32 (64 segments: 13.0 against 14.2; rank 64: 23.8 against 22.5).
    // For binary16 it is also ahead up to rank 16 where the input is so wide that the hand-off
    // kernel must take an odd number of slices and with them more workgroups than compute
    // units (h = 5120, three slices, 96 / 112 / 128 segments: 11.5 / 12.4 / 13.7 against 13.1 /
    // 13.7 / 14.6; bfloat16 at 128 segments: 15.2 against 14.8, so not there; 72 / 80 segments,
    // at most one workgroup per unit: 10.5 / 11.0 against 8.1 / 8.8, so not there either).
    // (the same wherever A_i is at most 64 KB, whatever the rank: h = 1024, rank 16, 1 / 8 / 32 / 64
    // segments 3.1 / 3.3 / 3.6 / 3.7 against 3.7 / 3.9 / 4.4 / 4.4; h = 2048, rank 16, 8 / 64 segments 4.0 /
    // 4.8 against 4.2 / 4.7; h = 1024, rank 32: 4.1 against 4.5; with 128 KB, h = 1024 at rank 64: 5.5 against 4.5)
    const bool small_a = (long long)p->h_in * p->r <= 32768;
    const bool odd_slices = fused && p->dtype == SGMV_F16 && (pl->fused.S & (pl->fused.S - 1)) != 0 &&
                            pl->fused.S * n_segs > limits().fused_workgroups;
    if (p->path == SGMV_PATH_AUTO && p->ksplit == 0 && choose_whole(p, n_segs, &pl->whole) &&
        (((p->r == 8 || small_a) && n_segs <= 512 && (!fused || p->h_in <= 4096 || small_a)) ||
         ((!fused || odd_slices) && n_segs <= 640 && p->r <= (p->workspace_ready ? 16 : 32)))) {
      pl->kernel = SGMV_KERNEL_WHOLE;
      return SGMV_OK;
    }
    if (fused) {
      pl->kernel = SGMV_KERNEL_FUSED;
      return SGMV_OK;
    }
    if (p->path == SGMV_PATH_FUSED) return SGMV_ERR_UNSUPPORTED;
  }
  if (use_matrix(p, n_segs)) {
    choose_split_matrix(p, n_segs, &pl->ksplit, &pl->kslice);
    pl->kernel = SGMV_KERNEL_MATRIX;
    return SGMV_OK;
  }
  if (!choose_split(p, n_segs, &pl->ksplit, &pl->kslice)) return SGMV_ERR_UNSUPPORTED;
  pl->kernel = SGMV_KERNEL_VECTOR;
  return SGMV_OK;
}

// What sgmv_shrink launches: shared by the entry point and sgmv_plan_shrink.
struct ShrinkPlan {
  bool whole_by_rows;  // SGMV_KERNEL_WHOLE: a workgroup per row of the batch, not per segment
  int kernel;          // SGMV_KERNEL_FUSED (hand-off inside one launch), _MATRIX or _VECTOR (+ reduction launch)
  FusedArgs fused;     // SGMV_KERNEL_FUSED
  int ksplit, kslice;  // the others
};

int plan_shrink(const sgmv_problem* p, int n_segs, ShrinkPlan* pl) {
  // one-row segments with a prepared workspace: one launch, the partial sums handed over inside
  // it (measured at h = 4096, r = 16, 1 / 16 / 64 / 128 segments: 3.5 / 4.0 / 5.0 / 6.6 us against
  // 4.8 / 6.1 / 6.7 / 8.1 us for shrink + reduction; r = 64, 64 segments: 9.5 against 10.7)
  sgmv_problem shrink_only = *p;
  shrink_only.h_out = p->h_in;  // the output width plays no part here (and need not be set by the caller)
  // one workgroup per one-row segment computes the whole product: no Split-K, no second launch
  const bool whole_shape = p->ksplit == 0 && p->h_in <= kWholeMaxHin && (long long)p->h_in * (p->r / 8) % 256 == 0;
  const bool whole_fits = p->max_seg_len == 1 && whole_shape;
  pl->whole_by_rows = false;
  if (p->path == SGMV_PATH_WHOLE) {
    if (!whole_shape) return SGMV_ERR_UNSUPPORTED;
    pl->whole_by_rows = p->max_seg_len != 1;  // longer segments (or unknown): per row of the batch
    pl->kernel = SGMV_KERNEL_WHOLE;
    return SGMV_OK;
  }
  // Measured on MI355X, us per call, against the launch with the hand-off (up to 128 segments) and
  // the two launches of the vector kernels (beyond): where A_i is at most 128 KB (h_in * r <= 65536)
  // it is ahead at every batch (h = 4096, rank 16, 1 / 32 / 64 / 128 / 256 / 512 segments: 3.4 / 3.9 /
  // 4.8 / 5.8 / 8.6 / 15.0 against 3.65 / 4.3 / 5.0 / 6.6 / 11.4 / 16.6; rank 8, 64 segments: 3.2
  // against 4.1); with a larger A_i only beyond the hand-off's batches (256 segments, rank 32:
  // 14.8 against 16.0; h = 8192: 15.3 against 16.6; but 64 segments at rank 64: 16.8 against 9.5);
  // from about 100 MB of weights on the Split-K kernels stream better (1024 segments at rank 16:
  // 27.8 against 26.9; 512 at rank 64: 48.1 against 46.5).
  // (an A_i of 64 .. 128 KB: only where all of it is in flight in at most two batches, and in bfloat16,
  // whose conversions this kernel does not hide as well, only from 96 segments on: h = 4096, rank 16,
  // 16 / 64 / 96 segments 4.2 / 5.3 / 6.0 against 3.8 / 4.8 / 6.7)
  const long long a_elems = (long long)p->h_in * p->r;
  const bool whole_small = a_elems <= 32768 || (a_elems <= 65536 && a_elems % (16 * 256 * 8) == 0 &&
                                                (p->dtype == SGMV_F16 || n_segs >= 96));
  const bool fused = p->path == SGMV_PATH_AUTO && p->ksplit == 0 && choose_fused(&shrink_only, n_segs, &pl->fused);
  if (p->path == SGMV_PATH_AUTO && whole_fits && (long long)n_segs * p->h_in * p->r <= kShrinkWholeMostElements &&
      (whole_small || (!fused && n_segs > 128))) {
    pl->kernel = SGMV_KERNEL_WHOLE;
    return SGMV_OK;
  }
  if (fused) {
    pl->kernel = SGMV_KERNEL_FUSED;
    return SGMV_OK;
  }
  // Small batches of longer segments (or of unknown length), per row of the batch.  With a small A_i
  // a workgroup per row without Split-K (measured at h = 4096, binary16, against the per-row launch
  // with the hand-off below, from 512 rows the MFMA kernels: rank 16, Uniform of 64 / 128 / 256 /
  // 384 / 512 rows 3.85 / 4.1 / 4.9 / 6.3 / 6.4 against 4.6 / 5.2 / 6.2 / 7.3 / 8.8 us, Identical of
  // 1024 rows 8.2 against 7.8; rank 8, Uniform of 64 rows 2.9 against 4.0; rank 32, where A_i is
  // 256 KB: 64 rows 6.6 against 5.5, 256 rows 7.2 against 9.3)
  const bool fused_rows = p->path == SGMV_PATH_AUTO && rows_apply(p, n_segs, false, 0) &&
                          choose_fused(&shrink_only, p->n_tokens, &pl->fused, true, true);
  {
    const bool small = a_elems <= 32768 || (a_elems <= 65536 && a_elems % (16 * 256 * 8) == 0 &&
                                            (p->dtype == SGMV_F16 || p->n_tokens >= 96));
    if (p->path == SGMV_PATH_AUTO && p->max_seg_len != 1 && whole_shape && n_segs <= kRowsMostSegments &&
        p->n_tokens <= 512 && (small || (!fused_rows && p->n_tokens > 128 && a_elems <= 131072))) {
      pl->whole_by_rows = true;
      pl->kernel = SGMV_KERNEL_WHOLE;
      return SGMV_OK;
    }
  }
  // else the launch with the hand-off per row of the
  // batch, as for the add-on (rows_apply; measured at h = 4096 against the better of the
  // launch-per-step kernels: rank 16, Uniform / Skewed / Identical of 64 rows 4.6 / 4.4 / 4.1 against
  // 7.7 / 7.3 / 6.7 us, of 256 rows 5.5 / 5.7 / 4.8 against 8.6 / 9.5 / 6.9; rank 64, 64 rows: 7.0 /
  // 6.5 / 5.6 against 10.5 / 10.9 / 9.8)
  if (fused_rows) {
    pl->kernel = SGMV_KERNEL_FUSED;
    return SGMV_OK;
  }
  if (use_matrix(p, n_segs)) {
    choose_split_matrix(p, n_segs, &pl->ksplit, &pl->kslice);
    pl->kernel = SGMV_KERNEL_MATRIX;
    return SGMV_OK;
  }
  if (!choose_split(p, n_segs, &pl->ksplit, &pl->kslice)) return SGMV_ERR_UNSUPPORTED;
  pl->kernel = SGMV_KERNEL_VECTOR;
  return SGMV_OK;
}

// Multi-projection call: SGMV_KERNEL_MULTI_SIDE / _PIPELINED with the launch shape in *f (per
// segment, or per row of the batch when f->by_rows), SGMV_KERNEL_TILE with the shape in *t (groups
// of t->n_proj add-ons per launch), or SGMV_KERNEL_SEQUENCE (one sgmv_add_lora after the other).
int plan_multi(const sgmv_problem* p, int n_segs, int n_proj, FusedArgs* f, TileArgs* t) {
  const Limits lim = limits();
  const bool one_row = p->max_seg_len == 1;
  if (n_proj < 2) return SGMV_KERNEL_SEQUENCE;
  // Segments longer than a row in a small batch: where a single add-on runs the one-row kernel
  // per row of the batch (plan_single), so may the add-ons of this call, side by side
  bool per_row = false;
  if (!one_row && p->ksplit == 0 && (p->path == SGMV_PATH_AUTO || p->path == SGMV_PATH_ROWS)) {
    FusedArgs rows;
    TileArgs one;
    const bool tile_one = p->path == SGMV_PATH_AUTO && choose_tile(p, n_segs, &one);
    per_row = (p->path == SGMV_PATH_ROWS || rows_apply(p, n_segs, tile_one, tile_one ? one.S : 0)) &&
              choose_fused(p, p->n_tokens, &rows, true, true);
  }
  // The add-ons in one launch of the one-row kernels: one set of S workgroups per segment (or per
  // row of the batch) and add-on, side by side or, for one-row segments, walking the add-ons.
  auto joint_rows = [&]() -> int {
    if (!(p->path == SGMV_PATH_AUTO || p->path == SGMV_PATH_FUSED || per_row) || !(one_row || per_row)) return SGMV_KERNEL_SEQUENCE;
    const int items = per_row ? p->n_tokens : n_segs;  // what a set of S workgroups serves
    if (p->workspace == nullptr || !choose_fused(p, items, f, false, per_row) || f->S * n_proj > split_cap(p->n_tokens))
      return SGMV_KERNEL_SEQUENCE;
    f->r = p->r;
    // workgroups that hold segments count towards what must be resident; the grid, padded to
    // whole rows of segments, must leave every workgroup its own generation copy
    const long long grid = (long long)f->S * fused_grid_items(items) * n_proj;
    if ((long long)f->S * items * n_proj <= lim.multi_workgroups && grid <= kGenerationCopies)
      return SGMV_KERNEL_MULTI_SIDE;
    if (!per_row && fused_multi_fits(*f)) return SGMV_KERNEL_MULTI_PIPELINED;
    // slices too deep for the pipelined kernel's register sets (h_in = 5120 at four slices):
    // three workgroups per compute unit still beat one launch per add-on (measured, three
    // projections of 64 segments at h = 5120: 22.7 us against 24.8 us)
    // (ranks up to 16 only: the kernels of the higher ranks use more registers and fit two per unit)
    if (p->r <= 16 && (long long)f->S * items * n_proj <= lim.multi_workgroups_most && grid <= kGenerationCopies)
      return SGMV_KERNEL_MULTI_SIDE;
    return SGMV_KERNEL_SEQUENCE;
  };
  if (one_row) return joint_rows();
  // Measured at 4096 x 4096, binary16, us for two / three add-ons, per row side by side against
  // the joint tile launch below: rank 16, 64 rows: Uniform 8.1 / 11.0 against 12.6 / 20.5, Skewed
  // 7.2 / 9.1 against 10.0 / 13.7, Identical 6.2 / 7.4 against 7.7 / 8.0, 8 segments of 8 rows
  // 6.2 / 7.4 against 8.4 / 8.8; 128 rows: 16 x 8 rows 8.0 / 11.2 against 9.3 / 10.4, one segment 8.0 /
  // 11.2 against 8.5 / 9.0 (three add-ons of 128 rows are 768 workgroups at two slices); rank 64,
  // 64 rows, two add-ons: 8 x 8 rows 13.1 against 15.7, Identical 11.4 against 20.8.
  // (at rank 32, 128 rows, two add-ons, the tile launch is ahead: one segment 10.9 against 12.2,
  // 16 x 8 rows 11.2 against 14.5)
  // (and at rank 64 per row again, the tile kernel's hand-off being bound by its volume there: two
  // segments of 64 rows 16.8 against 21.2, 16 x 8 rows 23.0 against 31.1 in two tile launches)
  const bool rows_first = per_row && (p->n_tokens <= 64 || ((long long)n_proj * p->n_tokens <= 256 && p->r != 32));
  if (rows_first) {
    const int kernel = joint_rows();
    if (kernel != SGMV_KERNEL_SEQUENCE) return kernel;
  }
  // segments of a few rows: the add-ons side by side in one launch of the tile kernel while all
  // their workgroups are resident together (fewer slices each than a single add-on would get)
  // (t->n_proj: how many go into one launch; when not all of them fit, the call takes groups of
  // that many, and what is left over at the end in a smaller launch)
  bool tile = false;
  if ((p->path == SGMV_PATH_AUTO || p->path == SGMV_PATH_FUSED) && p->ksplit == 0) {
    for (int group = n_proj; group > 1 && !tile; --group) tile = choose_tile(p, n_segs, t, group);
  }
  // against add-ons that run per row side by side, the joint tile launch is ahead only as one
  // launch that keeps at least kTileMultiSlices slices (Skewed of 128 rows, three add-ons: three
  // slices 22.0 us against 11.5 per row; Uniform of 64 rows in two launches 20.5 against 11.0);
  // against add-ons per row one after the other it is ahead also in groups and with fewer slices
  // (four add-ons, rank 8: 32 x 2 rows in two launches 17.5 against 19.4, Skewed of 64 rows at
  // three slices 11.8 against 18.4; rank 32: 32 x 4 rows 30.4 against 40.6)
  if (tile && (!per_row || (t->n_proj == n_proj && t->S >= kTileMultiSlices))) return SGMV_KERNEL_TILE;
  if (per_row && !rows_first) {
    const int kernel = joint_rows();
    if (kernel != SGMV_KERNEL_SEQUENCE) return kernel;
  }
  if (tile) return SGMV_KERNEL_TILE;
  return SGMV_KERNEL_SEQUENCE;
}

}  // namespace

extern "C" {

const char* sgmv_status_string(int status) {
  switch (status) {
    case SGMV_OK: return "ok";
    case SGMV_ERR_NULL: return "a required pointer is NULL";
    case SGMV_ERR_SHAPE: return "invalid size";
    case SGMV_ERR_UNSUPPORTED: return "unsupported dtype, rank, width or option";
    case SGMV_ERR_ALIGN: return "pointer not sufficiently aligned";
    case SGMV_ERR_WORKSPACE: return "workspace missing or too small";
    case SGMV_ERR_RANGE: return "layer_idx out of range";
    case SGMV_ERR_LAUNCH: return "kernel launch failed";
    case SGMV_ERR_TIMEOUT: return "a workgroup gave up waiting for partial sums";
    case SGMV_ERR_STATE: return "workspace not initialised or its launch accounting is inconsistent";
  }
  return "unknown status";
}

size_t sgmv_workspace_bytes(int32_t n_tokens, int32_t r) {
  if (n_tokens <= 0 || r <= 0) return 0;
  // header, fp32 split-K partials, 64-bit exchange words, 16-bit operand pairs of v
  return kWorkspaceHeader + 3 * partial_bytes(n_tokens, r) + operand_bytes(n_tokens, r);
}

size_t sgmv_workspace_bytes_multi(int32_t n_tokens, int32_t r, int32_t n_proj) {
  const size_t single = sgmv_workspace_bytes(n_tokens, r);
  if (single == 0 || n_proj < 2) return single;
  const int shared = n_proj < kSharedShrinkMost ? n_proj : kSharedShrinkMost;
  return single + (size_t)(shared - 1) * (partial_bytes(n_tokens, r) + operand_bytes(n_tokens, r));
}

int sgmv_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (workspace == nullptr) return SGMV_ERR_NULL;
  if (!aligned(workspace, 256)) return SGMV_ERR_ALIGN;
  if (workspace_bytes < kWorkspaceHeader) return SGMV_ERR_WORKSPACE;
  if (launch_workspace_init(workspace, workspace_bytes, 0, static_cast<hipStream_t>(stream)) !=
      hipSuccess)
    return SGMV_ERR_LAUNCH;
  return SGMV_OK;
}

int sgmv_workspace_check(const void* workspace, void* stream) {
  if (workspace == nullptr) return SGMV_ERR_NULL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the generation copies and, right after them, the error word and the initialisation mark
  static_assert(kWorkspaceErrorOffset == (size_t)kGenerationCopies * 4, "error word follows the copies");
  uint32_t head[kGenerationCopies + 2];
  if (hipMemcpyAsync(head, workspace, sizeof head, hipMemcpyDeviceToHost, st) != hipSuccess)
    return SGMV_ERR_LAUNCH;
  if (hipStreamSynchronize(st) != hipSuccess) return SGMV_ERR_LAUNCH;
  // between launches all copies of the generation agree; anything else means the workspace was
  // never initialised, or a launch did not account for all of its workgroups and later launches
  // may disagree about their generation
  if (head[kGenerationCopies + 1] != kWorkspaceMagic) return SGMV_ERR_STATE;
  if (head[kGenerationCopies] != 0) return SGMV_ERR_TIMEOUT;
  if (head[0] == 0) return SGMV_ERR_STATE;
  for (int i = 1; i < kGenerationCopies; ++i)
    if (head[i] != head[0]) return SGMV_ERR_STATE;
  return SGMV_OK;
}

int sgmv_validate_segments(const int32_t* host_seg_starts, int32_t n_segs, int32_t n_tokens) {
  if (n_segs < 0 || n_tokens < 0) return SGMV_ERR_SHAPE;
  if (host_seg_starts == nullptr) return SGMV_ERR_NULL;
  if (host_seg_starts[0] != 0) return SGMV_ERR_SHAPE;
  for (int32_t i = 0; i < n_segs; ++i)
    if (host_seg_starts[i + 1] < host_seg_starts[i]) return SGMV_ERR_SHAPE;
  if (host_seg_starts[n_segs] != n_tokens) return SGMV_ERR_SHAPE;
  return SGMV_OK;
}

int sgmv_shrink(const sgmv_problem* p, float* v, const void* x, const void* const* A_ptrs,
                const int32_t* seg_starts, int32_t n_segs, int32_t layer_idx, void* stream) {
  int rc = check_common(p, seg_starts, n_segs, layer_idx, true, false);
  if (rc != SGMV_OK) return rc;
  if (n_segs == 0 || p->n_tokens == 0) return SGMV_OK;
  if (v == nullptr || x == nullptr || A_ptrs == nullptr) return SGMV_ERR_NULL;
  if (!aligned(v, 16) || !aligned(x, 16)) return SGMV_ERR_ALIGN;
  rc = check_workspace(p);
  if (rc != SGMV_OK) return rc;
  if (p->path == SGMV_PATH_FUSED || p->path == SGMV_PATH_ROWS) return SGMV_ERR_UNSUPPORTED;

  hipStream_t st = static_cast<hipStream_t>(stream);
  ShrinkPlan pl;
  rc = plan_shrink(p, n_segs, &pl);
  if (rc != SGMV_OK) return rc;
  if (pl.kernel == SGMV_KERNEL_WHOLE) {
    ShrinkArgs a = make_shrink(p, Scratch{}, x, A_ptrs, seg_starts, n_segs, layer_idx);
    a.by_rows = pl.whole_by_rows;
    return launch_shrink_whole(a, v, st) == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
  }
  if (pl.kernel == SGMV_KERNEL_FUSED) {
    fill_fused(&pl.fused, p, caller_scratch(p), seg_starts, n_segs, layer_idx, 1.f);
    pl.fused.x = x;
    pl.fused.A_ptrs = A_ptrs;
    return launch_shrink_handoff(pl.fused, v, st) == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
  }
  ShrinkArgs a = make_shrink(p, caller_scratch(p), x, A_ptrs, seg_starts, n_segs, layer_idx);
  a.ksplit = pl.ksplit;
  a.kslice = pl.kslice;
  if (pl.kernel == SGMV_KERNEL_MATRIX) {
    if (launch_shrink_matrix(a, st) != hipSuccess) return SGMV_ERR_LAUNCH;
  } else {
    if (launch_shrink_vector(a, st) != hipSuccess) return SGMV_ERR_LAUNCH;
  }
  if (launch_shrink_reduce(v, a, st) != hipSuccess) return SGMV_ERR_LAUNCH;
  return SGMV_OK;
}

int sgmv_expand(const sgmv_problem* p, void* y, const float* v, const void* const* B_ptrs,
                const int32_t* seg_starts, int32_t n_segs, int32_t layer_idx, float scale,
                void* stream) {
  int rc = check_common(p, seg_starts, n_segs, layer_idx, false, true);
  if (rc != SGMV_OK) return rc;
  if (n_segs == 0 || p->n_tokens == 0) return SGMV_OK;
  if (y == nullptr || v == nullptr || B_ptrs == nullptr) return SGMV_ERR_NULL;
  if (!aligned(v, 16) || !aligned(y, 16)) return SGMV_ERR_ALIGN;
  if (p->path == SGMV_PATH_FUSED || p->path == SGMV_PATH_WHOLE || p->path == SGMV_PATH_ROWS) return SGMV_ERR_UNSUPPORTED;

  hipStream_t st = static_cast<hipStream_t>(stream);
  ExpandArgs a = make_expand(p, y, v, 1, nullptr, B_ptrs, seg_starts, n_segs, layer_idx, scale);
  // the MFMA kernels keep v's 16-bit operand pairs in the workspace
  const bool have_ws = check_workspace(p) == SGMV_OK;
  if (p->path == SGMV_PATH_MATRIX && !have_ws) return check_workspace(p);
  const int strips_threads = expand_by_rows(p, n_segs) ? choose_expand_threads(p, p->n_tokens) : 0;
  if (strips_threads != 0) {
    a.by_rows = true;
    a.threads = strips_threads;
    if (launch_expand_vector(a, st) != hipSuccess) return SGMV_ERR_LAUNCH;
  } else if (have_ws && expand_use_matrix(p, n_segs)) {
    set_operands(&a, caller_scratch(p), p->n_tokens, p->r);
    if (launch_expand_matrix(a, st) != hipSuccess) return SGMV_ERR_LAUNCH;
  } else {
    if (launch_expand_vector(a, st) != hipSuccess) return SGMV_ERR_LAUNCH;
  }
  return SGMV_OK;
}

}  // extern "C"

namespace {

// Argument checks of the whole add-on that do not concern the scratch memory.
int check_add_lora(const sgmv_problem* p, const void* y, const void* x, const void* const* A_ptrs,
                   const void* const* B_ptrs, const int32_t* seg_starts, int32_t n_segs,
                   int32_t layer_idx, bool* nothing_to_do) {
  *nothing_to_do = false;
  const int rc = check_common(p, seg_starts, n_segs, layer_idx, true, true);
  if (rc != SGMV_OK) return rc;
  if (n_segs == 0 || p->n_tokens == 0) {
    *nothing_to_do = true;
    return SGMV_OK;
  }
  if (y == nullptr || x == nullptr || A_ptrs == nullptr || B_ptrs == nullptr) return SGMV_ERR_NULL;
  if (!aligned(y, 16) || !aligned(x, 16)) return SGMV_ERR_ALIGN;
  return SGMV_OK;
}

// The add-on on checked arguments, its intermediate results in `sc`.
int add_lora_launch(const sgmv_problem* p, const Scratch& sc, void* y, const void* x,
                    const void* const* A_ptrs, const void* const* B_ptrs,
                    const int32_t* seg_starts, int32_t n_segs, int32_t layer_idx, float scale,
                    hipStream_t st) {
  SinglePlan pl;
  const int rc = plan_single(p, n_segs, &pl);
  if (rc != SGMV_OK) return rc;
  switch (pl.kernel) {
    case SGMV_KERNEL_WHOLE: {
      WholeArgs& w = pl.whole;
      w.bf16 = p->dtype == SGMV_BF16;
      w.r = p->r;
      w.h_in = p->h_in;
      w.h_out = p->h_out;
      w.n_segs = n_segs;
      w.n_tokens = p->n_tokens;
      w.offA = (long long)layer_idx * p->h_in * p->r;
      w.offB = (long long)layer_idx * p->r * p->h_out;
      w.scale = scale;
      w.y = y;
      w.x = x;
      w.A_ptrs = A_ptrs;
      w.B_ptrs = B_ptrs;
      w.seg_starts = seg_starts;
      w.header = sc.header;
      return launch_add_lora_whole(w, st) == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
    }
    case SGMV_KERNEL_TILE: {
      TileArgs& t = pl.tile;
      fill_tile(&t, p, sc, seg_starts, n_segs, layer_idx, scale);
      t.y = y;
      t.x = x;
      t.A_ptrs = A_ptrs;
      t.B_ptrs = B_ptrs;
      return launch_add_lora_tile(t, st) == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
    }
    case SGMV_KERNEL_FUSED: {
      FusedArgs& f = pl.fused;
      fill_fused(&f, p, sc, seg_starts, n_segs, layer_idx, scale);
      f.y = y;
      f.x = x;
      f.A_ptrs = A_ptrs;
      f.B_ptrs = B_ptrs;
      return launch_add_lora_fused(f, st) == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
    }
    case SGMV_KERNEL_MATRIX: {
      ShrinkArgs sa = make_shrink(p, sc, x, A_ptrs, seg_starts, n_segs, layer_idx);
      sa.ksplit = pl.ksplit;
      sa.kslice = pl.kslice;
      if (launch_shrink_matrix(sa, st) != hipSuccess) return SGMV_ERR_LAUNCH;
      ExpandArgs e = make_expand(p, y, sa.partials, sa.ksplit, A_ptrs, B_ptrs, seg_starts, n_segs,
                                 layer_idx, scale);
      set_operands(&e, sc, p->n_tokens, p->r);
      return launch_expand_matrix(e, st) == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
    }
    default: {
      ShrinkArgs sa = make_shrink(p, sc, x, A_ptrs, seg_starts, n_segs, layer_idx);
      sa.ksplit = pl.ksplit;
      sa.kslice = pl.kslice;
      if (launch_shrink_vector(sa, st) != hipSuccess) return SGMV_ERR_LAUNCH;
      ExpandArgs e = make_expand(p, y, sa.partials, sa.ksplit, A_ptrs, B_ptrs, seg_starts, n_segs,
                                 layer_idx, scale);
      return launch_expand_vector(e, st) == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
    }
  }
}

// The device address of this GPU's copy of `scratch`, prepared for the single-launch kernels
// the first time the GPU is seen: asked of the runtime once per device (every GPU holds its
// own copy at its own address), then header and exchange words are cleared and the generation set
// by a small kernel on `st`.  Calls no allocator.
int static_scratch(hipStream_t st, char** base) {
  static std::mutex mutex;
  static char* address[kMaxDevices];  // zero-initialised
  static bool ready[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return SGMV_ERR_LAUNCH;
  if (dev < 0 || dev >= kMaxDevices) return SGMV_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mutex);
  if (address[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return SGMV_ERR_LAUNCH;
    address[dev] = static_cast<char*>(ptr);
  }
  if (!ready[dev]) {
    // the clearing kernel must run once, not once per replay of a graph that captured it
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &capture) != hipSuccess || capture != hipStreamCaptureStatusNone) {
      (void)hipGetLastError();
      return SGMV_ERR_STATE;
    }
    if (launch_workspace_init(address[dev], kStaticExchangeEnd, 0, st) != hipSuccess) return SGMV_ERR_LAUNCH;
    ready[dev] = true;
  }
  *base = address[dev];
  return SGMV_OK;
}

}  // namespace

extern "C" {

int sgmv_add_lora(const sgmv_problem* p, void* y, const void* x, const void* const* A_ptrs,
                  const void* const* B_ptrs, const int32_t* seg_starts, int32_t n_segs,
                  int32_t layer_idx, float scale, void* stream) {
  bool nothing = false;
  int rc = check_add_lora(p, y, x, A_ptrs, B_ptrs, seg_starts, n_segs, layer_idx, &nothing);
  if (rc != SGMV_OK || nothing) return rc;
  if (p->path == SGMV_PATH_WHOLE && p->workspace == nullptr)  // that kernel keeps nothing in memory
    return add_lora_launch(p, Scratch{nullptr, nullptr, nullptr, nullptr}, y, x, A_ptrs, B_ptrs, seg_starts,
                           n_segs, layer_idx, scale, static_cast<hipStream_t>(stream));
  rc = check_workspace(p);
  if (rc != SGMV_OK) return rc;
  return add_lora_launch(p, caller_scratch(p), y, x, A_ptrs, B_ptrs, seg_starts, n_segs, layer_idx,
                         scale, static_cast<hipStream_t>(stream));
}

int sgmv_add_lora_static(const sgmv_problem* p, void* y, const void* x, const void* const* A_ptrs,
                         const void* const* B_ptrs, const int32_t* seg_starts, int32_t n_segs,
                         int32_t layer_idx, float scale, void* stream) {
  bool nothing = false;
  int rc = check_add_lora(p, y, x, A_ptrs, B_ptrs, seg_starts, n_segs, layer_idx, &nothing);
  if (rc != SGMV_OK || nothing) return rc;
  if (sgmv_workspace_bytes(p->n_tokens, p->r) > SGMV_STATIC_MAX_WORKSPACE_BYTES) return SGMV_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = nullptr;
  rc = static_scratch(st, &base);
  if (rc != SGMV_OK) return rc;
  // within the size limit both regions of the array hold what this batch needs (exchange
  // words: twice the partial sums' bytes); checked all the same
  const size_t parts = partial_bytes(p->n_tokens, p->r);
  if (2 * parts > kStaticExchangeEnd - kWorkspaceHeader ||
      parts + operand_bytes(p->n_tokens, p->r) > kStaticBytes - kStaticExchangeEnd)
    return SGMV_ERR_WORKSPACE;
  sgmv_problem q = *p;
  q.workspace = base;
  q.workspace_bytes = kStaticBytes;
  q.workspace_ready = 1;
  const Scratch sc{reinterpret_cast<unsigned long long*>(base),
                   reinterpret_cast<float*>(base + kStaticExchangeEnd),
                   reinterpret_cast<unsigned long long*>(base + kWorkspaceHeader),
                   base + kStaticExchangeEnd + parts};
  return add_lora_launch(&q, sc, y, x, A_ptrs, B_ptrs, seg_starts, n_segs, layer_idx, scale, st);
}

int sgmv_add_lora_multi(const sgmv_problem* p, int32_t n_proj, void* const* ys,
                        const void* const* xs, const void* const* const* A_ptrs,
                        const void* const* const* B_ptrs, const int32_t* seg_starts, int32_t n_segs,
                        int32_t layer_idx, float scale, void* stream) {
  int rc = check_common(p, seg_starts, n_segs, layer_idx, true, true);
  if (rc != SGMV_OK) return rc;
  if (n_proj < 0 || n_proj > kMaxProjections) return SGMV_ERR_SHAPE;
  if (n_proj == 0 || n_segs == 0 || p->n_tokens == 0) return SGMV_OK;
  if (ys == nullptr || xs == nullptr || A_ptrs == nullptr || B_ptrs == nullptr) return SGMV_ERR_NULL;
  for (int i = 0; i < n_proj; ++i) {
    if (ys[i] == nullptr || xs[i] == nullptr || A_ptrs[i] == nullptr || B_ptrs[i] == nullptr)
      return SGMV_ERR_NULL;
    if (!aligned(ys[i], 16) || !aligned(xs[i], 16)) return SGMV_ERR_ALIGN;
    for (int j = 0; j < i; ++j)
      if (ys[i] == ys[j]) return SGMV_ERR_SHAPE;  // two add-ons into one y would race
  }
  rc = check_workspace(p);
  if (rc != SGMV_OK) return rc;

  hipStream_t st = static_cast<hipStream_t>(stream);
  FusedArgs f;
  TileArgs tile;
  const int kernel = plan_multi(p, n_segs, n_proj, &f, &tile);
  if (kernel == SGMV_KERNEL_TILE) {
    const Scratch sc = caller_scratch(p);
    const int group = tile.n_proj;
    for (int first = 0; first < n_proj; first += group) {
      const int count = n_proj - first < group ? n_proj - first : group;
      TileArgs t = tile;
      if (count == 1 || (count < group && !choose_tile(p, n_segs, &t, count))) {  // left over at the end
        for (int i = first; i < first + count; ++i) {
          rc = add_lora_launch(p, sc, ys[i], xs[i], A_ptrs[i], B_ptrs[i], seg_starts, n_segs, layer_idx, scale, st);
          if (rc != SGMV_OK) return rc;
        }
        break;
      }
      fill_tile(&t, p, sc, seg_starts, n_segs, layer_idx, scale);
      for (int i = 0; i < kMaxProjections; ++i) {
        t.table.x[i] = i < count ? xs[first + i] : nullptr;
        t.table.y[i] = i < count ? ys[first + i] : nullptr;
        t.table.A_ptrs[i] = i < count ? A_ptrs[first + i] : nullptr;
        t.table.B_ptrs[i] = i < count ? B_ptrs[first + i] : nullptr;
      }
      if (launch_add_lora_tile(t, st) != hipSuccess) return SGMV_ERR_LAUNCH;
    }
    return SGMV_OK;
  }
  if (kernel != SGMV_KERNEL_SEQUENCE) {
    fill_fused(&f, p, caller_scratch(p), seg_starts, n_segs, layer_idx, scale);
    f.n_proj = n_proj;
    for (int i = 0; i < kMaxProjections; ++i) {
      f.table.x[i] = i < n_proj ? xs[i] : nullptr;
      f.table.y[i] = i < n_proj ? ys[i] : nullptr;
      f.table.A_ptrs[i] = i < n_proj ? A_ptrs[i] : nullptr;
      f.table.B_ptrs[i] = i < n_proj ? B_ptrs[i] : nullptr;
    }
    // side by side while every workgroup of the launch is resident (two fit a compute
    // unit); beyond that one workgroup per (slice, segment) walks the projections in
    // turn, the next one's loads in flight
    f.Z = 1;
    const hipError_t err = kernel == SGMV_KERNEL_MULTI_SIDE ? launch_add_lora_fused(f, st)
                                                            : launch_add_lora_fused_multi(f, st);
    return err == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
  }
  // Long segments on the MFMA kernels, all add-ons reading the same x (q / k / v or gate / up of a
  // prefill batch): their shrinks share one pass over x, which is most of a shrink's bytes; then
  // every add-on's operand preparation and expand in turn.  Needs the larger workspace of
  // sgmv_workspace_bytes_multi for the partial sums of the second and third add-on.
  {
    bool same_x = n_proj >= 2 && n_proj <= kSharedShrinkMost;
    for (int i = 1; i < n_proj && same_x; ++i) same_x = xs[i] == xs[0];
    SinglePlan pl;
    if (same_x && plan_single(p, n_segs, &pl) == SGMV_OK && pl.kernel == SGMV_KERNEL_MATRIX) {
      const Scratch sc = caller_scratch(p);
      ShrinkArgs sa = make_shrink(p, sc, xs[0], A_ptrs[0], seg_starts, n_segs, layer_idx);
      sa.ksplit = pl.ksplit;
      sa.kslice = pl.kslice;
      if (shrink_shared_fits(sa, n_proj) &&
          p->workspace_bytes >= sgmv_workspace_bytes_multi(p->n_tokens, p->r, n_proj)) {
        // the first add-on's partial sums where a single call keeps them, the others' behind the
        // single-call workspace (the exchange words in between are left alone: the single-launch
        // kernels rely on what their tags say)
        const size_t parts = partial_bytes(p->n_tokens, p->r);
        char* const extra = static_cast<char*>(p->workspace) + sgmv_workspace_bytes(p->n_tokens, p->r);
        sa.n_shared = n_proj;
        for (int i = 0; i < n_proj; ++i) {
          sa.A_shared[i] = A_ptrs[i];
          sa.partials_shared[i] = i == 0 ? sc.partials : reinterpret_cast<float*>(extra + (size_t)(i - 1) * parts);
        }
        if (launch_shrink_matrix_shared(sa, st) != hipSuccess) return SGMV_ERR_LAUNCH;
        // operand pairs of all add-ons in one launch (the first add-on's where a single call keeps
        // them, the others' behind the extra partial sums), then the expands
        ExpandArgs es[kSharedShrinkMost];
        const size_t ops = operand_bytes(p->n_tokens, p->r);
        for (int i = 0; i < n_proj; ++i) {
          es[i] = make_expand(p, ys[i], sa.partials_shared[i], sa.ksplit, A_ptrs[i], B_ptrs[i], seg_starts, n_segs,
                              layer_idx, scale);
          Scratch own = sc;
          if (i > 0) own.operands = extra + (size_t)(n_proj - 1) * parts + (size_t)(i - 1) * ops;
          set_operands(&es[i], own, p->n_tokens, p->r);
          es[i].operands_ready = true;
        }
        if (launch_finalize_shared(es, n_proj, st) != hipSuccess) return SGMV_ERR_LAUNCH;
        for (int i = 0; i < n_proj; ++i)
          if (launch_expand_matrix(es[i], st) != hipSuccess) return SGMV_ERR_LAUNCH;
        return SGMV_OK;
      }
    }
  }
  // any other shape: one add-on after the other
  for (int i = 0; i < n_proj; ++i) {
    rc = sgmv_add_lora(p, ys[i], xs[i], A_ptrs[i], B_ptrs[i], seg_starts, n_segs, layer_idx, scale,
                       stream);
    if (rc != SGMV_OK) return rc;
  }
  return SGMV_OK;
}

int sgmv_plan_shrink(const sgmv_problem* p, int32_t n_segs, sgmv_plan* plan) {
  if (plan == nullptr) return SGMV_ERR_NULL;
  *plan = sgmv_plan{};
  static const int32_t no_segments[2] = {0, 0};  // only tested for being non-NULL
  int rc = check_common(p, no_segments, n_segs, 0, true, false);
  if (rc != SGMV_OK) return rc;
  if (n_segs == 0 || p->n_tokens == 0) return SGMV_OK;  // nothing is launched
  rc = check_workspace(p);
  if (rc != SGMV_OK) return rc;
  if (p->path == SGMV_PATH_FUSED || p->path == SGMV_PATH_ROWS) return SGMV_ERR_UNSUPPORTED;
  ShrinkPlan pl;
  rc = plan_shrink(p, n_segs, &pl);
  if (rc != SGMV_OK) return rc;
  plan->kernel = pl.kernel;
  if (pl.kernel == SGMV_KERNEL_WHOLE) {
    plan->launches = 1;
    plan->slices = 1;
    plan->workgroups = pl.whole_by_rows ? ceil_div(p->n_tokens, 8) * 8 : n_segs;
  } else if (pl.kernel == SGMV_KERNEL_FUSED) {
    plan->launches = 1;
    plan->slices = pl.fused.S;
    plan->workgroups = pl.fused.S * (int)fused_grid_items(pl.fused.by_rows ? p->n_tokens : n_segs);
  } else {
    plan->launches = 2;
    plan->slices = pl.ksplit;
  }
  return SGMV_OK;
}

int sgmv_plan_expand(const sgmv_problem* p, int32_t n_segs, sgmv_plan* plan) {
  if (plan == nullptr) return SGMV_ERR_NULL;
  *plan = sgmv_plan{};
  static const int32_t no_segments[2] = {0, 0};  // only tested for being non-NULL
  const int rc = check_common(p, no_segments, n_segs, 0, false, true);
  if (rc != SGMV_OK) return rc;
  if (n_segs == 0 || p->n_tokens == 0) return SGMV_OK;  // nothing is launched
  if (p->path == SGMV_PATH_FUSED || p->path == SGMV_PATH_WHOLE || p->path == SGMV_PATH_ROWS) return SGMV_ERR_UNSUPPORTED;
  const bool have_ws = check_workspace(p) == SGMV_OK;
  if (p->path == SGMV_PATH_MATRIX && !have_ws) return check_workspace(p);
  if (!expand_by_rows(p, n_segs) && have_ws && expand_use_matrix(p, n_segs)) {
    plan->kernel = SGMV_KERNEL_MATRIX;
    plan->launches = 2;  // operand preparation, expand
    return SGMV_OK;
  }
  const bool by_rows = expand_by_rows(p, n_segs);
  const int threads = choose_expand_threads(p, by_rows ? p->n_tokens : n_segs);
  plan->kernel = SGMV_KERNEL_VECTOR;
  plan->launches = 1;
  plan->slices = ceil_div(p->h_out, threads == kExpandSplit ? 512 : threads * 8);  // column strips
  // v of the rows of a pass, and in the kernel whose waves divide the weight rows the partial sums of three waves
  const int rows_per_pass = by_rows ? 1 : 4;
  plan->lds_bytes = rows_per_pass * p->r * 4 + (threads == kExpandSplit ? 3 * rows_per_pass * 512 * 4 : 0);
  plan->workgroups = plan->slices * (by_rows ? ceil_div(p->n_tokens, 8) * 8 : n_segs);
  return SGMV_OK;
}

int sgmv_plan_add_lora(const sgmv_problem* p, int32_t n_segs, int32_t n_proj, sgmv_plan* plan) {
  if (plan == nullptr) return SGMV_ERR_NULL;
  *plan = sgmv_plan{};
  static const int32_t no_segments[2] = {0, 0};  // only tested for being non-NULL
  int rc = check_common(p, no_segments, n_segs, 0, true, true);
  if (rc != SGMV_OK) return rc;
  if (n_proj < 1 || n_proj > kMaxProjections) return SGMV_ERR_SHAPE;
  if (n_segs == 0 || p->n_tokens == 0) return SGMV_OK;  // nothing is launched
  if (!(p->path == SGMV_PATH_WHOLE && p->workspace == nullptr && n_proj == 1)) {
    rc = check_workspace(p);
    if (rc != SGMV_OK) return rc;
  }
  if (n_proj > 1) {
    FusedArgs f;
    TileArgs tile;
    const int kernel = plan_multi(p, n_segs, n_proj, &f, &tile);
    if (kernel == SGMV_KERNEL_TILE) {  // groups of tile.n_proj add-ons; slices and workgroups of the first launch
      plan->kernel = kernel;
      plan->launches = (n_proj + tile.n_proj - 1) / tile.n_proj;
      plan->slices = tile.S;
      plan->workgroups = tile.S * n_segs * tile.n_proj * tile.Z;
      plan->lds_bytes = (int32_t)tile.lds_bytes;
      return SGMV_OK;
    }
    if (kernel != SGMV_KERNEL_SEQUENCE) {
      plan->kernel = kernel;
      plan->launches = 1;
      plan->slices = f.S;
      plan->workgroups = f.S * (int)fused_grid_items(f.by_rows ? p->n_tokens : n_segs) * (kernel == SGMV_KERNEL_MULTI_SIDE ? n_proj : 1);
      return SGMV_OK;
    }
  }
  SinglePlan pl;
  rc = plan_single(p, n_segs, &pl);
  if (rc != SGMV_OK) return rc;
  plan->kernel = pl.kernel;
  switch (pl.kernel) {
    case SGMV_KERNEL_WHOLE:
      plan->launches = 1;
      plan->slices = pl.whole.S;
      plan->workgroups = 8 * pl.whole.S * ceil_div(pl.whole.by_rows ? p->n_tokens : n_segs, 8);
      plan->lds_bytes = 0;
      break;
    case SGMV_KERNEL_TILE:
      plan->launches = 1;
      plan->slices = pl.tile.S;
      plan->workgroups = pl.tile.S * n_segs * pl.tile.Z;
      plan->lds_bytes = (int32_t)pl.tile.lds_bytes;
      break;
    case SGMV_KERNEL_FUSED:
      plan->launches = 1;
      plan->slices = pl.fused.S;
      plan->workgroups = pl.fused.S * (int)fused_grid_items(pl.fused.by_rows ? p->n_tokens : n_segs);
      break;
    case SGMV_KERNEL_MATRIX:
      plan->launches = 3;  // shrink, operand preparation, expand
      plan->slices = pl.ksplit;
      break;
    default:
      plan->launches = 2;
      plan->slices = pl.ksplit;
      plan->workgroups = pl.ksplit * n_segs;
      break;
  }
  plan->launches *= n_proj;  // a multi-projection call that is not batched runs them in turn
  return SGMV_OK;
}

}  // extern "C"
