/*
 * sgmv.h -- C ABI of libsgmv: Segmented Gather Matrix-Vector multiplication
 * (SGMV) for AMD MI355X (gfx950).
 *
 * SGMV is the batched LoRA add-on of Punica (arxiv 2310.18547, section
 * "Segmented Gather Matrix-Vector Multiplication").  The token rows of a batch
 * are grouped so that rows using the same LoRA adapter are consecutive; the
 * index sequence s_0 = 0 <= s_1 <= ... <= s_n = number of rows delimits n
 * segments, segment i owning rows s_i .. s_{i+1}-1 (zero based).  Rows of
 * segment i receive x * A_i * B_i on top of the backbone projection already
 * stored in y, evaluated as two steps (v starts at zero, is accumulated from
 * x A, and y is accumulated from v B: the sentence after the section's
 * displayed equation):
 *
 *     shrink :  v[rows of i] += x[rows of i] * A_i            (h_in  -> r)
 *     expand :  y[rows of i] += scale * v[rows of i] * B_i    (r -> h_out)
 *
 * with A_i in R^{h_in x r}, B_i in R^{r x h_out} (Background, "Low-Rank
 * Adaptation").  "Gather" = every segment names its own weights through an
 * array of device pointers.
 *
 * General conventions
 *   - Every data pointer (x, y, v, A_ptrs, B_ptrs, seg_starts, workspace, and
 *     whatever A_ptrs[i] / B_ptrs[i] point to) is DEVICE memory owned by the
 *     caller.  The sgmv_problem struct itself is HOST memory, read during the
 *     call only.  The library allocates nothing and frees nothing.  The only
 *     state it keeps between calls is per-device bookkeeping that changes no
 *     result (which kernels have had their LDS limit raised, the number of
 *     compute units, the address of sgmv_add_lora_static's array); the
 *     single-launch path keeps a generation count in the caller's workspace,
 *     see sgmv_workspace_init.
 *   - x is [n_tokens][h_in], y is [n_tokens][h_out], row-major, 16-bit floats
 *     of type `dtype` (IEEE binary16 or bfloat16), 16-byte aligned.
 *   - A_ptrs[i] points to segment i's shrink weights stacked over layers,
 *     [num_layers][h_in][r] row-major; B_ptrs[i] to [num_layers][r][h_out].
 *     The kernels add layer_idx * h_in * r (resp. layer_idx * r * h_out)
 *     elements, so one pointer array and one seg_starts serve all layers of a
 *     model invocation.  Each base must be 16-byte aligned.  Two segments may
 *     carry the same pointer.  A NULL entry means "no adapter": the segment's
 *     rows are left untouched.
 *   - seg_starts has n_segs + 1 int32 entries, seg_starts[0] = 0,
 *     non-decreasing, seg_starts[n_segs] = n_tokens.  Empty segments are
 *     allowed.  Its *contents* are not checked on the device path; use
 *     sgmv_validate_segments() on a host copy if they are not trusted.
 *   - v (shrink output / expand input) is fp32 [n_tokens][r], 16-byte aligned.
 *   - Sums are accumulated in fp32 and y is rounded once, to nearest even,
 *     when it is stored.  v is kept in fp32 between the two steps.  On the
 *     vector-ALU kernels every product is an fp32 product too; the MFMA
 *     kernels (segments of several rows) feed v to the matrix cores as a high
 *     plus a low 16-bit part, which keeps 16 significant bits of v for
 *     bfloat16 and 22 for binary16 -- well inside the accuracy the 16-bit
 *     result can show.  Results are deterministic run to run (no
 *     floating-point atomics).
 *   - Supported shapes: r in {8, 16, 32, 64}; h_in and h_out positive
 *     multiples of 8.  Anything else returns SGMV_ERR_UNSUPPORTED; there is no
 *     fallback path.
 *   - Calls are asynchronous: kernels are enqueued on `stream` (a hipStream_t
 *     passed as void*; NULL = the default stream) and the call returns at
 *     once.  The return value reports what the host can detect (argument
 *     errors, a failed launch).  n_segs == 0 or n_tokens == 0 returns SGMV_OK
 *     and enqueues nothing.
 *   - x and y must not alias.  Two calls that share a workspace must be
 *     ordered (same stream, or otherwise synchronised).
 */
#ifndef SGMV_H_
#define SGMV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SGMV_F16 = 0, SGMV_BF16 = 1 } sgmv_dtype;

typedef enum {
  SGMV_OK = 0,
  SGMV_ERR_NULL = 1,         /* a required pointer is NULL                         */
  SGMV_ERR_SHAPE = 2,        /* negative / zero sizes that make no sense           */
  SGMV_ERR_UNSUPPORTED = 3,  /* dtype, r, h_in or h_out outside the supported set  */
  SGMV_ERR_ALIGN = 4,        /* x, y, v or workspace not 16-byte aligned           */
  SGMV_ERR_WORKSPACE = 5,    /* workspace missing or smaller than required         */
  SGMV_ERR_RANGE = 6,        /* layer_idx outside [0, num_layers)                  */
  SGMV_ERR_LAUNCH = 7,       /* the HIP runtime rejected a kernel launch           */
  SGMV_ERR_TIMEOUT = 8,      /* a workgroup gave up waiting (sgmv_workspace_check) */
  SGMV_ERR_STATE = 9         /* workspace never initialised, or its launch counter */
                             /* is inconsistent (sgmv_workspace_check)             */
} sgmv_status;

/* Kernel family selection.  AUTO picks from max_seg_len; the others force one
 * family for every segment (all families compute the same result). */
typedef enum {
  SGMV_PATH_AUTO = 0,
  SGMV_PATH_VECTOR = 1,      /* bandwidth path: vector ALU, one launch per step    */
  SGMV_PATH_MATRIX = 2,      /* MFMA path: for long (prefill-like) segments; at    */
                             /* most 65535 segments, else SGMV_ERR_UNSUPPORTED     */
  SGMV_PATH_FUSED = 3,       /* sgmv_add_lora only: shrink and expand in a single  */
                             /* launch; needs workspace_ready, max_seg_len > 0 and */
                             /* a launch whose workgroups (segments x sixteen-row  */
                             /* blocks x slices) are all resident with their weight*/
                             /* slices in LDS, else SGMV_ERR_UNSUPPORTED           */
  SGMV_PATH_WHOLE = 4,       /* sgmv_add_lora only: single launch for one-row      */
                             /* segments (max_seg_len == 1) in which every         */
                             /* workgroup computes its segment's whole shrink, so  */
                             /* workgroups never wait for each other and no        */
                             /* workspace is touched; h_in at most 8192, else      */
                             /* SGMV_ERR_UNSUPPORTED                               */
  SGMV_PATH_ROWS = 5         /* sgmv_add_lora only: the single-launch kernel of    */
                             /* SGMV_PATH_FUSED for one-row segments, run per ROW  */
                             /* of the batch: a row's workgroups look its segment  */
                             /* up on the device, so segments may have any length  */
                             /* (max_seg_len is not consulted) and rows that share */
                             /* an adapter read it through the caches; needs       */
                             /* workspace_ready and a batch small enough for all   */
                             /* workgroups to be resident, else                    */
                             /* SGMV_ERR_UNSUPPORTED                               */
} sgmv_path;

/* Problem descriptor: plain data, host memory, read during the call only. */
typedef struct sgmv_problem {
  int32_t dtype;             /* sgmv_dtype of x, y, A, B                            */
  int32_t h_in;              /* input features of shrink                            */
  int32_t h_out;             /* output features of expand                           */
  int32_t r;                 /* LoRA rank                                           */
  int32_t num_layers;        /* layers stacked behind every A_ptrs[i] / B_ptrs[i]   */
  int32_t n_tokens;          /* rows of x / y / v, = seg_starts[n_segs]             */
  int32_t max_seg_len;       /* longest segment, a hint for launch shape and path;  */
                             /* 0 = unknown.  A wrong hint costs speed, never       */
                             /* correctness.  Batches of up to 64 rows (more at     */
                             /* ranks below 64) run in one launch whatever it says, */
                             /* unless it is 1, see SGMV_PATH_ROWS.                 */
  int32_t path;              /* sgmv_path, normally SGMV_PATH_AUTO                  */
  int32_t ksplit;            /* split-K factor of shrink; 0 = choose automatically  */
  int32_t expand_threads;    /* workgroup size of the vector expand kernel          */
                             /* (64, 128 or 256), or 512 for the kernel whose four  */
                             /* waves divide the weight rows of a 512-column strip  */
                             /* among themselves (ranks 32 and 64 only, else        */
                             /* SGMV_ERR_UNSUPPORTED); 0 = choose automatically     */
  int32_t workspace_ready;   /* nonzero: sgmv_workspace_init() has been run on this */
                             /* workspace (and no call on it was ever aborted);     */
                             /* enables the single-launch path                      */
  int32_t spin_limit;        /* single-launch path: polls after which a workgroup   */
                             /* gives up waiting for its neighbours' partial sums;  */
                             /* 0 = the library's default (2^18).  Small values are */
                             /* for tests of the give-up path only.                 */
  void*   workspace;         /* device scratch, 256-byte aligned, at least          */
  size_t  workspace_bytes;   /*   sgmv_workspace_bytes(n_tokens, r) bytes           */
} sgmv_problem;

/* Kernel family a call resolves to (sgmv_plan_add_lora). */
typedef enum {
  SGMV_KERNEL_NONE = 0,             /* nothing to launch (no segments or no rows)          */
  SGMV_KERNEL_FUSED = 1,            /* single launch, vector ALUs: a set of workgroups per */
                                    /* one-row segment, or per row of a small batch        */
  SGMV_KERNEL_TILE = 2,             /* single launch, sixteen-row MFMA tiles               */
  SGMV_KERNEL_MULTI_SIDE = 3,       /* several projections side by side in one launch      */
  SGMV_KERNEL_MULTI_PIPELINED = 4,  /* several projections walked by every workgroup       */
  SGMV_KERNEL_VECTOR = 5,           /* one launch per step, vector ALUs                    */
  SGMV_KERNEL_MATRIX = 6,           /* one launch per step, MFMA (long segments)           */
  SGMV_KERNEL_SEQUENCE = 7,         /* internal: multi-projection call run as single calls */
  SGMV_KERNEL_WHOLE = 8             /* single launch, whole shrink in every workgroup      */
} sgmv_kernel;

/* What a call would launch: plain data filled by sgmv_plan_add_lora. */
typedef struct sgmv_plan {
  int32_t kernel;      /* sgmv_kernel of every add-on                                      */
  int32_t launches;    /* kernel launches of the whole call                                */
  int32_t slices;      /* workgroups per segment (single-launch kernels) or split-K factor */
  int32_t workgroups;  /* workgroups of the (first) launch; 0 where it depends on lengths  */
  int32_t lds_bytes;   /* dynamic LDS per workgroup (tile kernel), else 0                  */
  int32_t reserved[3];
} sgmv_plan;

/* Text for a status code (static storage; never NULL). */
const char* sgmv_status_string(int status);

/* Bytes of device scratch that sgmv_shrink and sgmv_add_lora need for a batch
 * of n_tokens rows at rank r (split-K partial sums of the shrink step, see the
 * "Split-K" remark in the paper's kernel-schedule paragraph).  Pure host
 * function.  Returns 0 for n_tokens <= 0. */
size_t sgmv_workspace_bytes(int32_t n_tokens, int32_t r);

/* Workspace size that also lets sgmv_add_lora_multi share one pass over x between the shrinks
 * of up to three add-ons on long (prefill-shaped) segments that read the same x, e.g. q / k / v or
 * gate / up (the paper applies LoRA to all dense projections of a layer): the size of
 * sgmv_workspace_bytes plus room for the partial sums of the other add-ons.  A workspace of the
 * plain size works everywhere; such calls then run one add-on after the other. */
size_t sgmv_workspace_bytes_multi(int32_t n_tokens, int32_t r, int32_t n_proj);

/* Prepare a workspace for the single-launch paths of sgmv_add_lora: clears it
 * and sets its generation count with a small kernel on `stream` (so the call
 * may be recorded into a HIP graph).  Those paths exchange partial sums
 * between workgroups through the workspace and tell one call's words from an
 * earlier call's by the generation, which every such call advances; run this
 * once after allocating the workspace, and again if a call using it was ever
 * aborted or sgmv_workspace_check reported an error.  `workspace` is device
 * memory, 256-byte aligned, of at least sgmv_workspace_bytes() bytes (never
 * less than 4352). */
int sgmv_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* Synchronous health check of a workspace used by the single-launch path:
 * waits for `stream`, reads the workspace's header and returns
 * SGMV_ERR_TIMEOUT if any workgroup ever gave up its (bounded) wait for a
 * neighbour's partial sums -- that call's result is then incomplete: the rows
 * and columns of y such a workgroup was responsible for were left as they
 * were (nothing is ever stored from an incomplete sum), the others hold the
 * finished result -- and
 * SGMV_ERR_STATE if the workspace was never initialised or the copies of its
 * generation count disagree (no call may be running on another stream).  In
 * both cases the workspace must be re-initialised.  Returns SGMV_OK otherwise.
 * Not meant for the hot path. */
int sgmv_workspace_check(const void* workspace, void* stream);

/* Host-side check of a HOST copy of the segment index sequence against the
 * segment definition paragraph: n_segs >= 0, seg_starts[0] == 0,
 * non-decreasing, seg_starts[n_segs] == n_tokens.  Returns SGMV_OK,
 * SGMV_ERR_NULL or SGMV_ERR_SHAPE. */
int sgmv_validate_segments(const int32_t* host_seg_starts, int32_t n_segs, int32_t n_tokens);

/* SGMV-shrink, "v += x A" per segment (first operator of the LoRA module in
 * the paper's kernel-schedule paragraph).
 *   v      device fp32 [n_tokens][r], read and written (accumulated into)
 *   x      device 16-bit [n_tokens][h_in], read
 *   A_ptrs device array of n_segs device pointers
 * Uses p->workspace.  h_out of the descriptor is ignored.  One-row segments
 * (max_seg_len == 1) whose A_i is small (h_in * r <= 32768; up to 65536 in most cases), or whose batch is beyond what
 * the launch with the hand-off takes, run in ONE launch of a workgroup per segment that needs
 * no workspace (h_in at most 8192 and h_in * r a multiple of 2048; SGMV_PATH_WHOLE asks for
 * it, SGMV_ERR_UNSUPPORTED where it does not apply); batches of up to 512 rows in longer
 * segments run the same launch per row (every row's workgroup looks its segment up).
 * With SGMV_PATH_AUTO, a
 * prepared workspace (workspace_ready) and max_seg_len == 1 (or a batch of at most 64
 * rows, more at ranks below 64, whatever the segment lengths) the call is one launch whose
 * workgroups hand their Split-K partial sums to each other (bounded wait: a time-out is
 * reported by sgmv_workspace_check and leaves the affected rows of v as they were);
 * otherwise two launches, partial sums and their sum. */
int sgmv_shrink(const sgmv_problem* p, float* v, const void* x,
                const void* const* A_ptrs, const int32_t* seg_starts,
                int32_t n_segs, int32_t layer_idx, void* stream);

/* SGMV-expand, "y += scale * v B" per segment (second operator of the LoRA
 * module).
 *   y      device 16-bit [n_tokens][h_out], read and written
 *   v      device fp32 [n_tokens][r], read
 *   B_ptrs device array of n_segs device pointers
 * The vector kernels need no workspace; the MFMA kernels (SGMV_PATH_MATRIX, or
 * SGMV_PATH_AUTO with long segments and a workspace present) keep v's 16-bit
 * operand pairs in p->workspace.  h_in of the descriptor is ignored.  Small
 * batches of segments longer than a row (sgmv_plan_expand) run a workgroup per
 * row rather than per segment, so that few long segments still fill the chip. */
int sgmv_expand(const sgmv_problem* p, void* y, const float* v,
                const void* const* B_ptrs, const int32_t* seg_starts,
                int32_t n_segs, int32_t layer_idx, float scale, void* stream);

/* The whole LoRA add-on, y += scale * (x A_i) B_i per segment, i.e. v := 0,
 * shrink, expand in one call; v lives in the workspace (or in LDS) in fp32
 * (see the general conventions for how the MFMA kernels consume it).  A segment is skipped when either of its pointers is NULL.
 * With workspace_ready set and a max_seg_len hint both steps run in a single
 * kernel launch where that launch fits the chip (vector ALUs for one row per
 * segment; matrix cores on sixteen-row tiles otherwise, up to about 64 such
 * tiles in all at h = 4096); larger batches of long segments, or no hint, take
 * one launch per step.  sgmv_plan_add_lora tells which. */
int sgmv_add_lora(const sgmv_problem* p, void* y, const void* x,
                  const void* const* A_ptrs, const void* const* B_ptrs,
                  const int32_t* seg_starts, int32_t n_segs, int32_t layer_idx,
                  float scale, void* stream);

/* sgmv_add_lora for callers that cannot allocate device memory or hand a workspace over:
 * code under HIP graph capture that owns no buffer, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and same result as sgmv_add_lora, but the
 * intermediate results (split-K partial sums, exchange words, operands of v) live in a fixed
 * array inside the library, SGMV_STATIC_SCRATCH_BYTES per GPU, held until the process ends;
 * p->workspace, p->workspace_bytes and p->workspace_ready are ignored.  The call allocates
 * and frees nothing.
 *   - Limit: sgmv_workspace_bytes(p->n_tokens, p->r) <= SGMV_STATIC_MAX_WORKSPACE_BYTES
 *     (for instance 64 tokens at rank 64, 256 at rank 16); larger batches return
 *     SGMV_ERR_WORKSPACE.
 *   - The first call on a GPU looks the array up and clears it with a small kernel on
 *     `stream`; that call must not be made while `stream` is being captured into a graph
 *     (SGMV_ERR_STATE).  Later calls may be captured.
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents
 *     (the single-launch kernels tell calls apart by a generation number, so nothing has to
 *     be cleared in between).  Calls that overlap in time on one GPU -- two streams, two
 *     threads -- race on it: order them, or give the others a workspace of their own
 *     through sgmv_add_lora.
 *   - There is no health check for the array (sgmv_workspace_check takes a caller's
 *     workspace); a give-up of the bounded wait leaves the affected rows of y unchanged. */
#define SGMV_STATIC_SCRATCH_BYTES ((size_t)9 << 20)
#define SGMV_STATIC_MAX_WORKSPACE_BYTES ((size_t)8 << 20)
int sgmv_add_lora_static(const sgmv_problem* p, void* y, const void* x,
                         const void* const* A_ptrs, const void* const* B_ptrs,
                         const int32_t* seg_starts, int32_t n_segs, int32_t layer_idx,
                         float scale, void* stream);

/* Several LoRA add-ons of ONE shape in a single call: n_proj (at most 8)
 * independent add-ons y_i += scale * (x_i A^(i)_seg) B^(i)_seg that share the
 * descriptor (dtype, h_in, h_out, r, num_layers), the segment indices and
 * layer_idx -- the projections of a transformer layer that read the same
 * activations (query / key / value, or gate / up).  The paper applies LoRA to
 * every dense projection of a layer and notes that the segment indices stay
 * the same for all of these add-ons within one model invocation.
 *   ys, xs          HOST arrays of n_proj device pointers ([n_tokens][h_out] and
 *                   [n_tokens][h_in]); the y_i must be distinct, the x_i may be
 *                   the same buffer
 *   A_ptrs, B_ptrs  HOST arrays of n_proj device pointers, each to a device
 *                   array of n_segs weight pointers as in sgmv_add_lora
 * With workspace_ready set and max_seg_len == 1 (every request its own
 * adapter) all add-ons run in ONE kernel launch; so do small batches of longer
 * segments (per row, as under SGMV_PATH_ROWS) and segments of a few rows
 * (max_seg_len from 2 up to what the single-launch MFMA kernel takes) while the
 * workgroups of all add-ons fit on the chip together, and in groups of as many
 * as fit beyond that.  On long segments (the MFMA
 * kernels) two or three add-ons whose x_i are the same buffer share the shrink's
 * pass over x when the workspace has the size of sgmv_workspace_bytes_multi
 * (ranks up to 32).  Otherwise the call is the same as n_proj calls of
 * sgmv_add_lora in order (sgmv_plan_add_lora reports this case: it does not
 * know whether the x_i coincide).  The result of every add-on
 * equals that of a separate sgmv_add_lora call up to the order in which the
 * fp32 sums are taken (the single-launch kernels split the same sums over
 * lanes differently). */
int sgmv_add_lora_multi(const sgmv_problem* p, int32_t n_proj, void* const* ys,
                        const void* const* xs, const void* const* const* A_ptrs,
                        const void* const* const* B_ptrs, const int32_t* seg_starts,
                        int32_t n_segs, int32_t layer_idx, float scale, void* stream);

/* Host-only, pure: which kernels sgmv_add_lora (n_proj == 1) or sgmv_add_lora_multi
 * (n_proj > 1) would launch for this descriptor, number of segments and number of
 * projections -- the same decision code the entry points run.  For benchmarks, logs and
 * tests of the launch policy; touches no device memory (the workspace pointer and size are
 * only checked as the entry points check them).  Returns the status the call itself would
 * return for these arguments. */
int sgmv_plan_add_lora(const sgmv_problem* p, int32_t n_segs, int32_t n_proj, sgmv_plan* plan);

/* The same for the stand-alone sgmv_shrink (section "Segmented Gather Matrix-Vector
 * Multiplication", the shrink launch): SGMV_KERNEL_WHOLE with one launch of a workgroup
 * per one-row segment (no Split-K); SGMV_KERNEL_FUSED with one launch when one-row
 * segments, or the rows of a small batch of longer ones, are reduced inside the launch
 * by the hand-off between workgroups (needs a prepared workspace and SGMV_PATH_AUTO;
 * max_seg_len == 1, or at most 64 rows, 128 up to rank 32, 384 up to rank 16), else SGMV_KERNEL_MATRIX or
 * SGMV_KERNEL_VECTOR with two launches (partial sums, then their sum).  Host-only, pure. */
int sgmv_plan_shrink(const sgmv_problem* p, int32_t n_segs, sgmv_plan* plan);

/* The same for the stand-alone sgmv_expand (same section, the expand launch):
 * SGMV_KERNEL_VECTOR with one launch of a workgroup per segment and strip of columns
 * (`slices` = strips) or, for a small batch of segments longer than a row (at most 64
 * rows, 128 up to rank 32, 384 up to rank 16; SGMV_PATH_AUTO), per ROW and strip, the
 * workgroups looking their row's segment up (lds_bytes of 6 KB or more: the kernel
 * whose four waves divide the weight rows, see expand_threads); SGMV_KERNEL_MATRIX with two launches
 * (operand preparation, MFMA expand) for long segments with a workspace.  Host-only, pure. */
int sgmv_plan_expand(const sgmv_problem* p, int32_t n_segs, sgmv_plan* plan);

/* Measurement aid, not part of the operator: enqueue one plain kernel of known traffic on
 * `stream`, for the benchmark's attainable-bandwidth figure and for scaling a profiler's HBM
 * byte counters (the roofline analysis of the paper's microbenchmark section compares the
 * kernel with the memory system's limits; these kernels measure those limits on this GPU).
 *   kind 0  empty kernel in the launch shape of the single-launch add-on (src, dst, bytes unused)
 *   kind 1  streaming read of `bytes` device bytes at `src` (16-byte aligned, multiple of 16);
 *           `dst` may be NULL or point to at least 4 writable device bytes
 *   kind 2  copy of `bytes` device bytes from `src` to `dst` (reads and writes `bytes`)
 *   kind 3  200 round trips of a 64-bit word between workgroup 0 and workgroup `bytes` (1..63)
 *           of one launch, with the accesses the single-launch kernels hand partial sums over
 *           with; workgroups are dealt to the eight XCDs round-robin, so 8 is a partner on
 *           the same XCD and 1 one on the next.  `src`: 512 device bytes, 256-byte aligned,
 *           zeroed once by the caller; `dst`: two 64-bit words, [0] receives the duration of
 *           all round trips in ticks of the 100 MHz device clock, [1] is set to 1 if a wait
 *           was given up (zero both before the call)
 * Returns SGMV_OK, SGMV_ERR_NULL, SGMV_ERR_ALIGN, SGMV_ERR_SHAPE, SGMV_ERR_UNSUPPORTED or
 * SGMV_ERR_LAUNCH. */
int sgmv_probe(int kind, const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SGMV_H_ */
