/*
 * fs.h -- C ABI of the stitched-kernel library for MI355X (gfx950).
 *
 * One fs_plan runs ONE fusion group -- a small DAG of memory-intensive tensor ops
 * with one or more outputs (the paper's "fusion pattern", Section 4.1; its ops and
 * its terminal tuple, Section 3.1) -- as a single stitched GPU kernel whose
 * intermediates stay in registers or LDS instead of going through HBM
 * (Section 5.1: thread, warp and block composition, kernel packing).
 *
 * All pointers named "device" are HIP device pointers; everything else is host
 * memory.  No function throws or aborts, and none but fs_plan_tune synchronises the
 * device; every failure is a status code plus a message readable through
 * fs_last_error().
 *
 * Threads: every function may be called from several threads at once, and the last
 * error is kept per thread.  One plan belongs to one thread at a time: its first
 * launch loads the kernel and allocates the workspace into the plan, so launches of
 * the same plan from two threads need the caller's own lock (different plans need none).
 */
#ifndef FS_H_
#define FS_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FS_MAX_RANK 4

typedef struct fs_plan fs_plan; /* opaque, owned by the library */

typedef enum { FS_F32 = 0, FS_F16 = 1, FS_BF16 = 2 } fs_dtype;

typedef enum {
  FS_OK = 0,
  FS_ERR_INVALID = 1,     /* malformed op list or bad argument */
  FS_ERR_UNSUPPORTED = 2, /* well-formed group that no stitched schedule covers: the
                             paper's "negative score", Section 4.3 -- the caller keeps
                             the group unfused (FS_MODE_PER_OP always works) */
  FS_ERR_LDS = 3,         /* shared-memory volume constraint violated (Section 5.3,
                             SharedPlanning) */
  FS_ERR_HIP = 4,         /* a HIP runtime call failed */
  FS_ERR_NOMEM = 5
} fs_status;

/* Op vocabulary: XLA-style tensor ops, the semantics the paper adopts (Section 3.1).
 * Tensors are dense, row-major, rank <= FS_MAX_RANK.
 *
 *  FS_PARAMETER   group input; the i-th parameter of the list is inputs[i] of fs_launch.
 *                 Rank 0 is a scalar held in device memory (one element, e.g. a value that an
 *                 earlier group reduced over everything); it enters ops of a larger shape
 *                 through FS_BROADCAST
 *  FS_CONSTANT    rank-0 scalar of value `attr`; allowed directly as an operand of a
 *                 binary op (implicit scalar broadcast)
 *  FS_ADD .. FS_MAXIMUM   elementwise binary; operands have the result's shape and dtype
 *  FS_NEGATE .. FS_SQRT   elementwise unary
 *  FS_CONVERT     changes the storage dtype
 *  FS_BROADCAST   operand dim d maps to result dim axis+d; operand dims of extent 1
 *                 are expanded; every other result dim is new
 *  FS_REDUCE_SUM / FS_REDUCE_MAX   reduce over `axis`, which is removed from the shape
 *  FS_DOT         batched matrix product a[B,M,K] . b[B,K,N]; axis==1: b is stored
 *                 [B,N,K] and the contraction runs over the last dim of both
 *  FS_CAUSAL_MASK x[..., i, j] is kept where j <= i and replaced by `attr` elsewhere
 *  FS_ERF / FS_LOGISTIC   unary like FS_TANH: erf(x); 1 / (1 + exp(-x))
 *  FS_OUTPUT      marks operand 0 as a group output; the i-th output op is outputs[i]
 */
typedef enum {
  FS_PARAMETER = 0, FS_CONSTANT = 1,
  FS_ADD = 2, FS_SUBTRACT = 3, FS_MULTIPLY = 4, FS_DIVIDE = 5, FS_MAXIMUM = 6,
  FS_NEGATE = 7, FS_EXP = 8, FS_LOG = 9, FS_TANH = 10, FS_RSQRT = 11, FS_SQRT = 12,
  FS_CONVERT = 13, FS_BROADCAST = 14,
  FS_REDUCE_SUM = 15, FS_REDUCE_MAX = 16,
  FS_DOT = 17, FS_CAUSAL_MASK = 18, FS_OUTPUT = 19,
  FS_ERF = 20, FS_LOGISTIC = 21,   /* unary, like FS_TANH: the error function; 1 / (1 + exp(-x)) */
  FS_NUM_OPKINDS = 22
} fs_opkind;

/* One op.  Plain data, caller-owned, copied by fs_plan_create.  `operand` holds
 * indices of EARLIER ops in the list (topological order), -1 where unused. */
typedef struct {
  int32_t kind;                 /* fs_opkind */
  int32_t dtype;                /* fs_dtype of the result */
  int32_t rank;                 /* 0..FS_MAX_RANK */
  int32_t axis;                 /* broadcast / reduce / dot attribute, else ignored */
  int64_t shape[FS_MAX_RANK];   /* result extents, first `rank` entries used */
  int32_t operand[3];
  int32_t reserved;             /* must be 0 */
  double attr;                  /* constant value / mask fill value */
} fs_op_desc;

typedef enum {
  FS_MODE_STITCHED = 0, /* the whole group as one stitched kernel */
  FS_MODE_PER_OP = 1,   /* baseline: one kernel per op, intermediates in a plan-owned HBM
                           workspace (the sum of K(Op_j) side of the execution-based
                           score, Section 4.3) */
  FS_MODE_STITCHED_PREBUILT = 2, /* stitched, but only with kernels compiled into the library:
                           no kernel generation (Section 5.3) and so no compiler run inside
                           fs_plan_create.  Differs from FS_MODE_STITCHED only for
                           FS_SCHED_ELEMENTWISE groups, which then run through the
                           library's register-program interpreter kernel */
  FS_MODE_STITCHED_GENERATED = 3 /* stitched, preferring a kernel generated for the group
                           wherever the generators cover it (all-elementwise groups; groups
                           of elementwise ops and reductions over the last dim), even where
                           a hand-written kernel matches.  fs_plan_tune times this form
                           against the hand-written one */
} fs_mode;

/* Launch parameters a template would carry (cta_size, cta_num and the per-warp tile,
 * Section 5.2).  0 = let the plan choose. */
typedef struct {
  int32_t mode;          /* fs_mode */
  int32_t wg_size;       /* threads per workgroup: multiple of 64; each schedule states its
                            own range in its error message (64..512 for one-wavefront rows,
                            a power of two 128..1024 for wavefront teams, ...) */
  int32_t rows_per_wave; /* hand-written row kernels: independent row groups a wavefront keeps
                            in flight, 1..8.  Generated row kernels: rows a wavefront covers
                            at a time, a power of two 1..64 (lanes per row = 64 / this; 64 is
                            the one-thread-per-row template).  Elementwise interpreter:
                            chunks a thread carries, 1, 2 or 4 */
  int32_t grid;          /* number of workgroups */
} fs_plan_options;

/* Schedule chosen for a stitched plan (fs_plan_info). */
typedef enum {
  FS_SCHED_PER_OP = 0,
  FS_SCHED_ROW = 1,      /* elementwise -> row reduce -> broadcast, wavefront reductions:
                            hand-written kernels for the recognised patterns (LayerNorm,
                            softmax, ...), a generated kernel for any other mix of
                            elementwise ops and reductions over the last dim */
  FS_SCHED_ROW_COL = 2,  /* row schedule packed with column reductions via LDS partials: sums or maxima over
                            all rows ([R, C] -> [C], on higher ranks spelled as a chain of sums over
                            the leading dim), or over each run of the innermost row dims
                            ([B, S, H] -> [B, H]: sequence pooling) */
  FS_SCHED_BDOT_SOFTMAX = 3, /* batched dot -> softmax -> batched dot on MFMA; the probabilities stay in
                                registers (accumulators of the first dot = operands of the second), K and V
                                go through LDS */
  FS_SCHED_ELEMENTWISE = 4,  /* any all-elementwise group: thread composition + packing, as
                                a kernel generated for the group (or interpreted, see
                                FS_MODE_STITCHED_PREBUILT).  The ops share one shape, or fall into
                                up to 16 parts that share no computed value, each of one shape
                                (generated form only): one kernel, a run of workgroups per part */
  FS_SCHED_BLOCK_DOT = 5     /* generated block composition around batched dots on MFMA (Sections 5.1, 5.3):
                                a[B,M,K] . b, b stored [B,N,K] or [B,K,N] (16-bit, K 16..128, tile up to 128 x 128) -> any
                                elementwise ops and row reductions on the tile -> optionally a second dot
                                with v[B,N,D], its operand handed over through LDS -> optionally
                                elementwise ops and row reductions on the [B,M,D] result (operands: such
                                values, per-row values, constants, inputs seen as [B,M,D]);
                                what the hand-written FS_SCHED_BDOT_SOFTMAX kernel does not match */
} fs_schedule;

/* Build a plan from a fusion group.
 *   ops, n_ops  host array of ops in topological order (borrowed for the call only)
 *   opt         host, may be NULL (stitched mode, automatic launch parameters)
 *   out         host, receives the plan on FS_OK, NULL otherwise
 * Pure host work: validates shapes and dtypes, recognises the group as one of the
 * stitched schedules (Algorithm 3 reduced to a recogniser over hand-written kernels),
 * checks the LDS budget and fixes the launch geometry.  A group that matches none of
 * them -- all-elementwise, or elementwise ops mixed with reductions over the last dim and
 * sums over the leading dims -- gets a kernel generated for it and compiled for gfx950
 * with the HIP run-time compiler (a few hundred milliseconds the first time a given
 * group is seen, cached afterwards per process and, with fs_kernel_cache_dir, per
 * machine).  Touches no GPU, so it also works on a machine without one.
 * Limits of a group: 1..4096 ops, at most 64 parameters and 16 outputs (8 for a group with
 * reductions or dots), tensors below 2^40 elements; beyond them FS_ERR_INVALID or
 * FS_ERR_UNSUPPORTED with a message that names the limit.
 * Errors: FS_ERR_INVALID, FS_ERR_UNSUPPORTED, FS_ERR_LDS, FS_ERR_NOMEM. */
fs_status fs_plan_create(const fs_op_desc* ops, int32_t n_ops,
                         const fs_plan_options* opt, fs_plan** out);

/* Run the plan's kernel (Section 5.5: the generated kernel is handed to the run time, which launches it):
 * enqueue the group on `hip_stream` (a hipStream_t passed as void*, NULL = the default stream) and return
 * without waiting.
 *   inputs[n_in]    host array of DEVICE pointers, one per FS_PARAMETER in list order
 *   outputs[n_out]  host array of DEVICE pointers, one per FS_OUTPUT in list order
 * Tensors are dense row-major in their op's dtype, 16-byte aligned, and borrowed until
 * the work enqueued by this call has finished.  Inputs are never written; outputs must
 * not overlap inputs or each other, with one exception, the update in place: an output may be
 * given the very pointer of a parameter of its own shape and dtype where the plan runs a
 * generated elementwise kernel or a generated register row kernel (fs_plan_describe says so)
 * and reads that parameter only in the group's own layout (not through a broadcast); such
 * kernels read every element in the thread, or the row's lanes, that later writes it.  Any
 * other identical pointer is refused with FS_ERR_INVALID; partial overlaps are not detected.  A plan that owns a workspace (fs_plan_info) must
 * not have two launches in flight at once; the workspace is allocated on the first
 * launch on the then-current device and the plan stays bound to that device.
 * Errors: FS_ERR_INVALID (NULL or misaligned pointer, wrong counts), FS_ERR_HIP,
 * FS_ERR_NOMEM.  Extents of 0 are legal: nothing is launched. */
fs_status fs_launch(fs_plan* plan, const void* const* inputs, int32_t n_in,
                    void* const* outputs, int32_t n_out, void* hip_stream);

/* fs_launch for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as
 * fs_launch, but a plan that needs scratch memory (fs_plan_info: workspace_bytes > 0 -- the partial rows
 * of column reductions, the intermediates of a per-op plan) gets it from an array of
 * FS_STATIC_SCRATCH_BYTES that is part of the library's device code, one copy per GPU, held from the
 * moment the library is loaded on that GPU until the process ends, instead of from a hipMalloc on the
 * plan's first launch.  The call allocates nothing and frees nothing, on the host side of HIP or the device.
 *   - FS_ERR_UNSUPPORTED if the plan needs more than FS_STATIC_SCRATCH_BYTES of scratch memory.
 *   - FS_ERR_INVALID if the plan runs a generated kernel that has not been loaded onto the device yet
 *     (loading allocates): launch the plan once with fs_launch before, or build it with
 *     FS_MODE_STITCHED_PREBUILT, whose kernels are part of the library.
 *   - Every call on one GPU uses that GPU's one array, whatever the plan or the stream: two calls whose
 *     work overlaps in time on one GPU race on it.  Calls on one stream, or ordered by events, are safe.
 *     Nothing in the array has to start at zero and nothing is kept there between calls.
 *   - Other errors and all argument rules as for fs_launch. */
#define FS_STATIC_SCRATCH_BYTES (8 * 1024 * 1024)
fs_status fs_launch_static(fs_plan* plan, const void* const* inputs, int32_t n_in,
                           void* const* outputs, int32_t n_out, void* hip_stream);

/* Kernel tuning (Algorithm 3's outer loop, Section 5.3: generate templates, evaluate each
 * kernel, keep the best; "optimize once, reuse").  Builds the stitched plan of the group
 * under every launch template the group's schedule offers (workgroup size, row groups in
 * flight, grid), runs each `trials` times on `hip_stream` with the caller's buffers, and
 * returns the fastest plan.
 *   inputs / outputs   as for fs_launch (DEVICE pointers); the outputs end up holding the
 *                      group's result
 *   trials             timed launches per template, 1..1000 (2 untimed ones come first)
 *   out                receives the best plan
 *   best               host, may be NULL: receives the winning options
 *   best_us            host, may be NULL: its average time per launch in microseconds
 * Unlike fs_launch this call SYNCHRONISES: it waits on HIP events it records on the
 * stream, and it must not be used while the stream is being captured.
 * Errors: those of fs_plan_create and fs_launch. */
fs_status fs_plan_tune(const fs_op_desc* ops, int32_t n_ops,
                       const void* const* inputs, int32_t n_in,
                       void* const* outputs, int32_t n_out, void* hip_stream,
                       int32_t trials, fs_plan** out, fs_plan_options* best, double* best_us);

/* Tuning cache ("optimize once, reuse", Section 1): fs_plan_tune records the winning options
 * under a key of the group (every field of every op: kinds, dtypes, shapes, wiring, constants),
 * per process.  fs_plan_create with opt == NULL, or with FS_MODE_STITCHED and all launch
 * parameters 0, uses the recorded options of a group it finds there (and falls back to its own
 * defaults if they no longer build).  Explicit options, and the other modes, never look.
 * The cache can be written to and merged from a text file, so that one tuning run serves
 * later processes: one line per group, "key(hex) mode wg_size rows_per_wave grid microseconds"
 * after a header line.  All of it is host work and thread-safe.
 *   fs_group_key         key of a group (host out-pointer); FS_ERR_INVALID on a NULL or empty list
 *   fs_tune_cache_size   number of recorded groups
 *   fs_tune_cache_clear  forget them all
 *   fs_tune_cache_save   write the file (overwrites); FS_ERR_INVALID if it cannot be written
 *   fs_tune_cache_load   merge a file, later entries winning; FS_ERR_INVALID if it cannot be
 *                        read or a line is malformed (nothing is merged then) */
fs_status fs_group_key(const fs_op_desc* ops, int32_t n_ops, uint64_t* key);
int32_t fs_tune_cache_size(void);
fs_status fs_tune_cache_clear(void);
fs_status fs_tune_cache_save(const char* path);
fs_status fs_tune_cache_load(const char* path);

/* Generated kernels are compiled once per process and source text.  With a cache directory they are
 * also compiled once per machine: fs_plan_create looks for the code object of a generated source in
 * that directory before it runs the compiler, and leaves it there afterwards (one file per kernel,
 * named after a hash of source, compile options and compiler version; written under a temporary
 * name and renamed, so concurrent processes are safe; a damaged or foreign file is ignored and
 * replaced).  The directory comes from the environment variable FS_KERNEL_CACHE_DIR unless
 * fs_kernel_cache_dir sets it (NULL or "" turns the disk cache off).  The directory must exist.
 *   fs_kernel_cache_stats        any out-pointer may be NULL: kernels compiled, found in this
 *                                process's memory, found on disk, since the library was loaded
 *   fs_kernel_cache_drop_memory  forget the per-process copies (the files stay) */
fs_status fs_kernel_cache_dir(const char* dir);
fs_status fs_kernel_cache_stats(int64_t* compiled, int64_t* from_memory, int64_t* from_disk);
fs_status fs_kernel_cache_drop_memory(void);

/* Release what fs_plan_create built (Section 5.5 ends with the kernel handed over; the plan is this
 * library's handle on it): the plan, its loaded kernel and its workspace.  NULL is a no-op.  The caller makes sure no
 * launch of the plan is still running. */
fs_status fs_destroy(fs_plan* plan);

/* Why the last failing call failed -- for fs_plan_create this is the reason a group gets the paper's
 * "negative score" (Section 4.3).  Message of the last failing call on this thread.  Library-owned, valid until the
 * next failing call on the same thread.  Never NULL. */
const char* fs_last_error(void);

/* Introspection (host only).  Any out-pointer may be NULL.
 *   schedule           fs_schedule
 *   n_kernels          kernel launches per fs_launch (the paper's N for the per-op mode)
 *   lds_bytes          LDS per workgroup of the stitched kernel
 *   workspace_bytes    plan-owned HBM scratch
 *   algorithmic_bytes  bytes of all parameters read once plus all outputs written once
 *   moved_bytes        bytes the plan's kernels read and write in HBM by construction
 *                      (per-op mode: every intermediate written and re-read) */
fs_status fs_plan_info(const fs_plan* plan, int32_t* schedule, int32_t* n_kernels,
                       int64_t* lds_bytes, int64_t* workspace_bytes,
                       int64_t* algorithmic_bytes, int64_t* moved_bytes);

/* The plan's schedule written in the paper's template notation (Section 5.2), e.g.
 * "reduce_1[GRID-WARP_2,WARP]; ... cta_num=..., cta_size=...".  Host string owned by
 * the plan, valid until fs_destroy.  For logs and tests; nothing parses it. */
const char* fs_plan_describe(const fs_plan* plan);

/* Shared-memory optimisation (Algorithm 4, Section 5.4) on a caller-given data-flow graph:
 * which ops may take over the shared (LDS) space of an earlier op.  Pure host work; the
 * library's kernel generator uses the same routine to lay out the row buffers of its
 * streamed template.
 *   operands      host, n x 3 indices of EARLIER ops (execution order), -1 where unused
 *   req_bytes     host, n entries: shared space the op's result needs, 0 = none
 *   is_output     host, n entries (non-zero: the group's root consumes the op), or NULL:
 *                 then every op without a user is an output
 *   offset        host, n entries out: byte offset of the op's space, -1 = none
 *   shares_with   host, n entries out, may be NULL: the op whose space was taken over
 *                 (it is dominated by the op: all its uses lie below the op), -1 = none
 *   total_bytes   host out: the footprint
 * Errors: FS_ERR_INVALID (NULL pointer, operand index not smaller than the op's own). */
fs_status fs_shared_plan(const int32_t* operands, const int64_t* req_bytes, const uint8_t* is_output,
                         int32_t n, int64_t* offset, int32_t* shares_with, int64_t* total_bytes);

/* ---- Fusion planning (Section 4) --------------------------------------------------------
 * From a computation graph -- an op list like a fusion group's, but of any size -- choose
 * which ops to fuse: fusion patterns are generated by substitution fusion (Algorithm 1, with
 * its growing set of partition ops) and exploratory fusion (Algorithm 2), scored by the
 * model-based score f(P) = M(V) + (N-1)*phi (negative when no stitched kernel can be built
 * for the pattern) or, for the patterns the caller has run, by the time they were measured to
 * save (the hybrid policy of Section 4.3: fs_fusion_pattern_group hands out any candidate as an
 * op list to build, time against its per-op plan and report back in extra_scores), and a set of pairwise disjoint patterns of maximal total score is
 * selected exactly (the ILP of Section 4.1), with the paper's iterative repair when the
 * selection would make the graph cyclic.  Pure host work.  The result is a list of groups in
 * an order that respects data flow; each group comes back as an op list of its own, ready
 * for fs_plan_create, with the ops of the original list that its parameters and outputs
 * stand for.  Ops that own no kernel (constants, broadcasts) are copied into every group
 * that reads them. */
typedef struct fs_fusion fs_fusion; /* opaque, owned by the library */

typedef struct {
  double launch_us;        /* phi, the launch latency of one kernel; <= 0: 2.5 */
  int32_t max_patterns;    /* patterns per conflict component handed to the solver, best scores first; 1..256, 0: 256 */
  int32_t explore_budget;  /* patterns the exploratory search may visit; 0: 400; < 0: none */
  int64_t seed_bytes;      /* exploratory seeds: ops whose result has at least this many bytes; 0: 1 MiB */
  const int64_t* bw_bytes; /* M(V) model: n_bw points (bytes moved, GB/s achieved), increasing */
  const double* bw_gbs;    /*   bytes; NULL / 0: the table measured on MI355X with fs_stream_copy */
  int32_t n_bw;
  int32_t n_extra;         /* caller-supplied patterns, scored and offered to the solver like the */
  const int32_t* extra_sizes; /* generated ones: n_extra sizes, then the op indices of all of them  */
  const int32_t* extra_ops;   /* back to back (kernel-owning ops of the list, any order)            */
  const double* extra_scores; /* NULL, or n_extra entries: the execution-based score of that pattern  */
                              /* (Section 4.3): the microseconds the caller measured it to save over  */
                              /* one kernel per op, used instead of the model's f(P) -- also for a    */
                              /* generated pattern with the same ops; NaN: the model's score          */
} fs_fusion_options;

/* Errors: FS_ERR_INVALID (malformed list or options, a measured score that is infinite or beyond 1e12),
 * FS_ERR_NOMEM. */
fs_status fs_fusion_create(const fs_op_desc* ops, int32_t n_ops, const fs_fusion_options* opt, fs_fusion** out);
fs_status fs_fusion_destroy(fs_fusion* fusion);
/* Any out-pointer may be NULL.  solver_rounds = 1 + number of cycle repairs. */
fs_status fs_fusion_info(const fs_fusion* fusion, int32_t* n_groups, int32_t* n_patterns, double* total_score_us,
                         int32_t* solver_rounds);
/* Sizes of group g (0 <= g < n_groups, execution order) and its score (0 for an op left alone). */
fs_status fs_fusion_group_size(const fs_fusion* fusion, int32_t g, int32_t* n_ops, int32_t* n_inputs,
                               int32_t* n_outputs, int32_t* n_members, double* score_us);
/* Group g: its op list (n_ops entries), for each of its parameters / outputs the index in the
 * ORIGINAL list of the op whose value it is (n_inputs / n_outputs entries; an input index may
 * name an original parameter), and the original indices of the kernel-owning ops it fuses
 * (n_members entries).  Caller-owned arrays of the sizes fs_fusion_group_size reports; any may be NULL. */
fs_status fs_fusion_group(const fs_fusion* fusion, int32_t g, fs_op_desc* ops, int32_t* input_of,
                          int32_t* output_of, int32_t* members);
/* Candidate pattern k (0 <= k < n_patterns): number of ops, the ops themselves (up to cap),
 * how it was found (0 substitution, 1 connected part of a substitution segment, 2 exploratory,
 * 3 supplied by the caller),
 * V in bytes, f(P) in microseconds (negative: not generable, or measured to be slower fused),
 * whether the plan uses it. */
fs_status fs_fusion_pattern(const fs_fusion* fusion, int32_t k, int32_t* n_ops, int32_t* ops, int32_t cap,
                            int32_t* origin, int64_t* saved_bytes, double* score_us, int32_t* chosen);

/* Candidate pattern k as a stand-alone op list, as fs_fusion_group gives a chosen group: sizes
 * first (all 0 for a pattern no stitched plan exists for; measured = 1 if its score is the
 * caller's), then the list and the original ops its parameters / outputs stand for. */
fs_status fs_fusion_pattern_group_size(const fs_fusion* fusion, int32_t k, int32_t* n_ops, int32_t* n_inputs,
                                       int32_t* n_outputs, int32_t* measured);
fs_status fs_fusion_pattern_group(const fs_fusion* fusion, int32_t k, fs_op_desc* ops, int32_t* input_of,
                                  int32_t* output_of);

/* Measurement aid: plain streaming copy of `bytes` (multiple of 16) from src to dst,
 * both DEVICE pointers, 16-byte aligned, on `hip_stream`.  Gives the achievable HBM
 * ceiling beside the 8 TB/s peak and the calibration factor for byte counters. */
fs_status fs_stream_copy(void* dst, const void* src, int64_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FS_H_ */
