/*
 * dvm.h -- C ABI of libdvm: a bytecode virtual machine for fused dynamic-shape tensor programs
 *          on AMD MI355X (gfx950).
 *
 * The split follows the paper's operator compiler (Section 3 "Operator Compiler", Section 4):
 * an operator program is *encoded* into tile-level bytecode on the host CPU in microseconds --
 * no machine code is generated, nothing is cached -- and the bytecode is *decoded and executed*
 * on the device by a pre-compiled interpreter kernel (Section 4.3, Algorithm 2).
 *
 *   dvm_prog_*   build a shape-free operator program (a DAG of basic and compound ops; compound
 *                ops are decomposed into basic ops, Section 3).
 *   dvm_encode   program + concrete input shapes -> bytecode: broadcast/shape inference and
 *                dominant shape (Section 4.2), pattern fusion of the op chain into one
 *                meta-kernel (Section 5.1), liveness and tile-register allocation (Algorithm 1's
 *                n_max / T_max), tile plan with the cost model ceil(#tiles/N)*(tile+c)
 *                (Section 4.2), and the header + body byte layout (Section 4.2 "Bytecode encoding").
 *   dvm_stack    temporal stacking-based fusion: several meta-kernels in one launch (Section 5.1).
 *   dvm_run      launch the interpreter on a HIP stream (Section 4.3).
 *
 * Conventions
 *   - All pointers are HOST pointers except the entries of `tensors[]` in dvm_run, which are
 *     DEVICE pointers.  `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *   - The caller owns every buffer.  The library allocates no device memory and keeps no
 *     reference to any argument after a call returns.  dvm_encode / dvm_stack / dvm_validate /
 *     dvm_disasm / dvm_plan make no HIP call and no heap allocation.
 *   - Bytecode is position independent and holds tensor *indices*, never addresses: it can be
 *     reused with other tensors of the same shapes, stored, or compared byte for byte.  Encoding
 *     the same program with the same shapes always yields identical bytes.
 *   - Every function returns 0 (DVM_OK) or a negative dvm_status; nothing aborts or throws.
 *   - dvm_encode and dvm_run are re-entrant for distinct output buffers.
 */
#ifndef DVM_H
#define DVM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DVM_MAX_RANK     6     /* rank of a tensor as given by the caller                         */
#define DVM_MAX_TENSORS  32    /* inputs + outputs of one launch (all stacked segments together)  */
#define DVM_MAX_OPS      96    /* ops (after decomposition) of one program                        */
#define DVM_CODE_MAX_BYTES 3584 /* one launch's bytecode travels in the kernel-argument segment   */

typedef enum dvm_status {
    DVM_OK            =  0,
    DVM_E_ARGS        = -1,   /* null pointer, bad index, bad count                               */
    DVM_E_SHAPE       = -2,   /* shapes do not broadcast together                                 */
    DVM_E_RANK        = -3,   /* rank above DVM_MAX_RANK, or iteration space not reducible to 4-D */
    DVM_E_DTYPE       = -4,   /* unknown storage dtype                                            */
    DVM_E_UNSUPPORTED = -5,   /* valid program the VM cannot run (see message of dvm_strerror)    */
    DVM_E_BUFSZ       = -6,   /* output buffer too small; the needed size is written to *len      */
    DVM_E_BADCODE     = -7,   /* bytecode fails structural validation                             */
    DVM_E_HIP         = -8,   /* a HIP call failed; see dvm_last_hip_error                        */
    DVM_E_ALIGN       = -9,   /* a device pointer is less aligned than the bytecode assumes       */
    DVM_E_LIMIT       = -10,  /* too many ops / tensors / bytes for one launch                    */
    DVM_E_STATE       = -11   /* program not finished, or already finished                        */
} dvm_status;

typedef enum dvm_dtype { DVM_F32 = 0, DVM_BF16 = 1 } dvm_dtype;

/* Operator vocabulary of the program builder.  Names follow Table 1 of the paper; DVM_OP_SUM/RMAX/RMIN
 * (and MEAN, MEANSQ) act on the last axis and keep it with extent 1 (Table 1's Sum/Max/Min with N = 1),
 * DVM_OP_CSUM/CMAX/CMIN on the penultimate axis (Table 1's general form, N > 1). */
typedef enum dvm_opcode {
    /* unary */
    DVM_OP_COPY = 1, DVM_OP_SQRT, DVM_OP_ABS, DVM_OP_LOG, DVM_OP_EXP, DVM_OP_ROUND, DVM_OP_FLOOR,
    DVM_OP_ISFINITE, DVM_OP_NEG, DVM_OP_RSQRT, DVM_OP_RCP, DVM_OP_TANH, DVM_OP_ERF, DVM_OP_SIGMOID,
    DVM_OP_SQUARE, DVM_OP_GELU_TANH, DVM_OP_GELU_ERF, DVM_OP_SILU,
    DVM_OP_CAST,            /* imm[0] = target dvm_dtype: round to that dtype, keep computing in fp32 */
    /* tile (op) scalar immediate: imm[0] */
    DVM_OP_ADDS = 32, DVM_OP_MULS,
    /* binary, NumPy broadcasting */
    DVM_OP_ADD = 40, DVM_OP_SUB, DVM_OP_MUL, DVM_OP_DIV, DVM_OP_MIN, DVM_OP_MAX, DVM_OP_POW,
    DVM_OP_CMP_EQ, DVM_OP_CMP_NE, DVM_OP_CMP_LT, DVM_OP_CMP_LE, DVM_OP_CMP_GT, DVM_OP_CMP_GE,
    /* ternary: args = (cond, a, b) -> cond != 0 ? a : b */
    DVM_OP_SELECT = 60,
    /* reductions over the last axis (kept, extent 1) */
    DVM_OP_SUM = 64, DVM_OP_RMAX, DVM_OP_RMIN, DVM_OP_MEAN, DVM_OP_MEANSQ,
    /* Table 1's Sum / Max / Min in their general form: [M, size, N] reduced along `size`, the penultimate
     * axis (kept, extent 1).  A program holds reductions along one axis only; a value reduced this way may
     * feed further ops of its own shape ([M, 1, N] and tensors that broadcast into it), not full-size ones.
     * The `size` rows are accumulated in order by one workgroup per (M index, column tile), in fp32. */
    DVM_OP_CSUM = 72, DVM_OP_CMAX, DVM_OP_CMIN,
    /* compound ops, decomposed by dvm_prog_finish */
    DVM_OP_SOFTMAX = 80,    /* args = (z)                                    */
    DVM_OP_RMSNORM,         /* args = (x, w),           imm[0] = eps         */
    DVM_OP_LAYERNORM        /* args = (x, gamma, beta), imm[0] = eps         */
} dvm_opcode;

/* Shape of one tensor as the caller holds it: dims and strides in ELEMENTS, outermost first.
 * A dimension of extent 1, or of stride 0, broadcasts.  `align_bytes` is the guaranteed alignment
 * of the device pointer that will be passed for this tensor (0 means 16). */
typedef struct dvm_shape {
    int32_t rank;
    int32_t align_bytes;
    int64_t dim[DVM_MAX_RANK];
    int64_t stride[DVM_MAX_RANK];
} dvm_shape;

/* Fill `s` with a contiguous row-major shape. */
int dvm_shape_contiguous(dvm_shape *s, int rank, const int64_t *dims);

/* ---- context: a snapshot of device properties used by the tile planner; owns no device memory --- */
typedef struct dvm_ctx dvm_ctx;

/* hip_device >= 0: query that device (HIP calls).  hip_device == -1: no device is touched and the
 * MI355X defaults are used (256 compute units), so that encoding works on a machine without GPU. */
int  dvm_ctx_create(int hip_device, dvm_ctx **out);
void dvm_ctx_destroy(dvm_ctx *ctx);
/* Override planner inputs (tests, tuning): number of compute units and the per-tile overhead term
 * of the cost model, in elements.  Values <= 0 leave the setting unchanged. */
int  dvm_ctx_set_planner(dvm_ctx *ctx, int n_compute_units, int tile_overhead_elems);
/* Bound the interpreter variant dvm_encode may plan for: at most `max_elems_per_lane` elements of a
 * tile per lane (4, 8, 16, 32 or 64) and at most `max_tile_regs` tile registers (1, 2, 4 or 6).  Parts that
 * are to share one launch (dvm_stack; Section 5, stacking) must all fit one variant, so a caller that
 * stacks encodes every part under common limits, e.g. (16, 4).  Values <= 0 leave a limit unchanged;
 * a program that needs more tile registers than allowed makes dvm_encode return DVM_E_UNSUPPORTED.  The default
 * bounds are 32 elements and 6 registers; the variant with 64 elements exists with one tile register only (programs
 * with long rows that need no more: a row of up to 4096 elements is then held by one wave; flat element-wise
 * programs keep 32 elements) and is planned for only when the bound is raised to 64. */
int  dvm_ctx_set_limits(dvm_ctx *ctx, int max_elems_per_lane, int max_tile_regs);

/* Force parts of the tile plan instead of letting the cost model choose (tests and tuning walk plans the
 * model would not pick): `elems_per_lane` (4, 8, 16, 32 or 64) selects the interpreter variant's tile register
 * size where the row length allows it, `rows_per_tile` the rows of a tile (for a reduction along the
 * penultimate axis: the waves that share one unit of work), `grid_multiplier` launches that many workgroups
 * per resident slot.  0 leaves a choice to the planner.  The bytecode depends on these settings and on the
 * other context settings, the program and the shapes only; the library reads no environment variable. */
int  dvm_ctx_set_plan_override(dvm_ctx *ctx, int elems_per_lane, int rows_per_tile, int grid_multiplier);
/* Let dvm_encode plan for a workspace of up to `bytes` bytes (default 0: no program ever needs one).  With a limit
 * above 0, a program that reduces along the penultimate axis (DVM_OP_CSUM / CMAX / CMIN) over few (outer index, column
 * tile) units and a long axis is split: the bytecode is then a temporally stacked program of two meta-kernels -- partial
 * results of S row ranges into the workspace, then their combination in the fixed order of the ranges and the ops
 * after the reduction; dvm_run issues the second as a kernel launch of its own behind the first, which on this
 * hardware is the cheapest way to make the partial results visible -- and lists the workspace as its LAST tensor
 * (dvm_code_tensor: is_output = 2, min_bytes = what this program needs); the caller passes that much 256-byte
 * aligned device memory as the last entry of tensors[] (or calls dvm_run_static, whose array then serves, up to
 * DVM_STATIC_WORKSPACE_BYTES).  The result does not depend on the number of compute units running: S and the order
 * are fixed by the shapes.  Such bytecode cannot be a part of dvm_stack / dvm_stack_dependent or run batched. */
int  dvm_ctx_set_workspace_limit(dvm_ctx *ctx, int64_t bytes);
/* Tell the planner that `copies` copies of every program encoded with this context share a launch: the tensor sets
 * of a dvm_run_batched call, or like parts of a stack (Section 5.1).  In the cost model of Section 4.2,
 * ceil(#tiles / N) * (tile length + overhead), #tiles then counts `copies` times, so the planner stops cutting a
 * small program into many small tiles just to give every workgroup one: the other copies fill the machine.
 * Default 1; 1 .. 4096.  The bytecode runs correctly whatever the launch turns out to hold. */
int  dvm_ctx_set_copies_in_flight(dvm_ctx *ctx, int copies);
/* Row-invariant operands that a program only multiplies by or adds (a weight vector, a bias) may be kept in
 * the workgroup's LDS instead of pinned tile registers when that lets the program run in an interpreter variant
 * with fewer tile registers, i.e. more resident waves (default: enabled).  0 disables it (tests, comparison). */
int  dvm_ctx_set_lds_operands(dvm_ctx *ctx, int enabled);
/* How the M tiles of a meta-kernel are dealt out to the N workgroups of the launch (Section 4.3, Algorithm 2).
 * DVM_ASSIGN_BLOCKED is the range the algorithm prints: workgroup id runs tiles [m*id, min(M, m*(id+1))) with
 * m = ceil(M/N).  DVM_ASSIGN_INTERLEAVED deals them out round-robin: workgroup id runs tiles id, id+N, id+2N, ...
 * -- the same tiles per workgroup to within one, still static and free of atomics, but the resident workgroups
 * sweep the tensors as one front, which HBM serves faster than N streams that lie far apart.  DVM_ASSIGN_AUTO (the
 * default) is the round-robin order except for programs that keep an operand pinned while consecutive rows share
 * it and whose rows are not whole 128-byte lines, which run blocked.  Results do not depend on the choice. */
typedef enum dvm_assignment { DVM_ASSIGN_BLOCKED = 0, DVM_ASSIGN_INTERLEAVED = 1, DVM_ASSIGN_AUTO = 2 } dvm_assignment;
int  dvm_ctx_set_assignment(dvm_ctx *ctx, int assignment);

/* ---- program builder (shape free) --------------------------------------------------------------- */
typedef struct dvm_prog dvm_prog;

int  dvm_prog_create(dvm_prog **out);
/* Declare the next input; *value_id receives its SSA id.  Inputs are numbered in declaration order
 * and that is their order in `in_shapes[]` and at the front of `tensors[]`. */
int  dvm_prog_input(dvm_prog *p, int dtype, int *value_id);
/* Append an op.  `arg_ids` are SSA ids of earlier values, `imm` the immediates the opcode takes. */
int  dvm_prog_op(dvm_prog *p, int opcode, const int *arg_ids, int n_args,
                 const double *imm, int n_imm, int *value_id);
/* Mark a value as the next output with storage dtype `dtype`.  Outputs follow the inputs in
 * `tensors[]`, in the order of these calls. */
int  dvm_prog_output(dvm_prog *p, int value_id, int dtype);
/* Decompose compound ops into basic ops and freeze the program. */
int  dvm_prog_finish(dvm_prog *p);
int  dvm_prog_num_inputs(const dvm_prog *p);
int  dvm_prog_num_outputs(const dvm_prog *p);
void dvm_prog_destroy(dvm_prog *p);

/* ---- host encoder ------------------------------------------------------------------------------- */
/*
 * Encode `prog` for the given input shapes.
 *   in_shapes[n_in]   one per program input, in declaration order.
 *   out_layout        NULL: outputs are contiguous row-major.  Otherwise out_layout[i].stride (and
 *                     align_bytes) give the strides of output i (a view store); its rank and dims
 *                     must equal the inferred ones.
 *   bytecode, cap     caller buffer.  On DVM_E_BUFSZ *len holds the size needed.
 *   out_shapes        optional (may be NULL): receives the inferred shape of every output.
 * Runs entirely on the host: no HIP call, no heap allocation, no cache lookup.
 */
int  dvm_encode(const dvm_ctx *ctx, const dvm_prog *prog,
                const dvm_shape *in_shapes, int n_in, const dvm_shape *out_layout,
                void *bytecode, size_t cap, size_t *len, dvm_shape *out_shapes);

/* Temporal stacking (Section 5.1): concatenate n encoded programs into one launch.  The stacked
 * program's tensor list is the concatenation of the parts' tensor lists, in order.  The parts
 * must be independent of each other (no part reads what another writes): dvm_run refuses a launch
 * in which a buffer one part writes overlaps a buffer of another part (DVM_E_ARGS).  For parts that
 * depend on each other use dvm_stack_dependent. */
int  dvm_stack(const void *const *codes, const size_t *lens, int n,
               void *out, size_t cap, size_t *len);

/* Temporal stacking of parts that depend on each other (Section 5.1: stacking does not require independent
 * operators; Section 5.2: the pieces a fuser cuts an unmergeable operator sequence into run as one stacked
 * kernel).  As dvm_stack, plus `same_as[n_same_as]`: one entry per tensor of the launch (part 0's tensors, then
 * part 1's, ...), -1 or the index of an EARLIER entry that is the same buffer (the caller passes the same device
 * pointer for both to dvm_run, which checks it).  A part that touches a buffer an earlier part wrote, or writes
 * one an earlier part read, starts behind a synchronisation point:
 *   - if producer and consumer deal the same rows of that buffer to the same workgroups (same number of rows
 *     and rows per tile, whole rows per tile, the buffer addressed by plain row index in both), a workgroup only
 *     waits for its own earlier stores;
 *   - otherwise, with order_by = DVM_ORDER_BY_LAUNCH, dvm_run starts a kernel launch of its own at that part (everything
 *     before it is then complete and visible; no workspace, no wait on the device; on this hardware the cheaper of
 *     the two: a few microseconds per boundary);
 *   - or, with order_by = DVM_ORDER_IN_KERNEL, the whole program stays ONE kernel launch and every workgroup waits
 *     until all have finished the earlier parts (its cost grows with the number of workgroups: each makes its
 *     stores visible beyond its own second-level cache).  That needs
 *     DVM_WORKSPACE_BYTES of device memory the caller lends to the launch: the stacked program then lists one
 *     more tensor, the workspace (dvm_code_tensor reports it with is_output = 2), and the caller passes its
 *     device pointer (256-byte aligned) as the LAST entry of tensors[].  dvm_run clears it before the launch.
 *     Launches that share a workspace must not overlap in time.  The wait is bounded (dvm_ctx_set_sync_limit):
 *     a workgroup whose wait runs out sets the workspace's status word and leaves the kernel, and so do all the
 *     others at their next wait; dvm_workspace_status reads the word back.
 * Parts must be encoded programs or independent stacks, not dependent stacks themselves. */
#define DVM_WORKSPACE_BYTES 256
typedef enum dvm_order_by { DVM_ORDER_IN_KERNEL = 0, DVM_ORDER_BY_LAUNCH = 1 } dvm_order_by;
int  dvm_stack_dependent(const void *const *codes, const size_t *lens, int n, const int *same_as, int n_same_as, int order_by,
                         void *out, size_t cap, size_t *len);
/* Upper bound on the polls (about a microsecond each) a workgroup spends at a grid-wide synchronisation point
 * before it gives up; the default is about one million.  polls < 1 is an error. */
int  dvm_ctx_set_sync_limit(dvm_ctx *ctx, int64_t polls);
/* (Only launches with a grid-wide synchronisation point use and clear the status word.)
 * Wait for `hip_stream` and read the status word of a workspace: *gave_up = 1 if a launch that used it since it
 * was last cleared abandoned a synchronisation point (its outputs are then incomplete), else 0. */
int  dvm_workspace_status(const void *workspace, void *hip_stream, int *gave_up);

/* Spatial stacking (Section 5.1): like dvm_stack, but the parts run side by side in the one launch,
 * each on its own share of the workgroups (in proportion to an estimate of the part's run time: tiles
 * times interpreted records, plus bytes moved), instead of one after the other on all of them.
 * Every part must be a single meta-kernel as dvm_encode produces it; more non-empty parts than the
 * launch has workgroups gives DVM_E_UNSUPPORTED (use dvm_stack then).  Same arguments, ownership and
 * error behaviour as dvm_stack. */
int  dvm_stack_spatial(const void *const *codes, const size_t *lens, int n,
                       void *out, size_t cap, size_t *len);

/* ---- streaming fuser for dynamic graphs (Section 5.2, dynamic graph fuser) -----------------------
 * Operators arrive one at a time, as an eager framework issues them.  They are buffered lazily and
 * fused on arrival while their iteration spaces merge.  An operator that does not merge cuts the buffer
 * and opens its next piece; when the buffer runs -- it is full, or dvm_fuser_flush is called (a host
 * read, a stream synchronisation) -- the pieces are stacked into ONE launch (dvm_stack_dependent: a later
 * piece waits for the earlier ones whose results it reads).  A result the caller released before the
 * buffer ran, and that no later piece reads, is a pure intermediate and is never written to memory.
 * A piece that needs all of an earlier piece (not only what its own workgroup wrote) starts a kernel launch of
 * its own inside that one dvm_run call (DVM_ORDER_BY_LAUNCH), or, when dvm_fuser_set_workspace has lent a workspace,
 * waits inside the single kernel launch (DVM_ORDER_IN_KERNEL).  When the pieces do not fit one program (tensor
 * table, bytecode size, interpreter variant), every piece is run on its own, in order.  dvm_fuser_stats counts
 * kernel launches.
 *
 * All calls are host calls.  The fuser owns no device memory: every tensor and every result buffer
 * is the caller's (device pointers), and must stay valid until the buffer that uses it has run.
 * A fuser is not thread-safe; use one per stream.  With a context created for device -1 a flush
 * encodes the buffered operators but launches nothing (host-side measurement and tests). */
typedef struct dvm_fuser dvm_fuser;

int  dvm_fuser_create(dvm_ctx *ctx, void *hip_stream, dvm_fuser **out);
void dvm_fuser_destroy(dvm_fuser *f);
/* Lend the fuser DVM_WORKSPACE_BYTES (or more) of 256-byte aligned device memory for the waits of its stacked
 * launches (see dvm_stack_dependent); it must stay valid while the fuser uses it and belongs to this fuser's
 * stream alone.  NULL takes it back. */
int  dvm_fuser_set_workspace(dvm_fuser *f, void *workspace, size_t bytes);
/* Register a tensor that already holds data; *value receives its id. */
int  dvm_fuser_tensor(dvm_fuser *f, void *device_ptr, int dtype, const dvm_shape *shape, int *value);
/* Issue an operator on earlier values (same opcodes and immediates as dvm_prog_op).  `out_ptr` is the
 * buffer the framework allocated for the result (contiguous, inferred shape, storage `out_dtype`);
 * it is written when the buffer runs, unless the result was released before.  *value: the result's id. */
int  dvm_fuser_op(dvm_fuser *f, int opcode, const int *args, int n_args, const double *imm, int n_imm,
                  int out_dtype, void *out_ptr, int *value);
/* The caller no longer references `value`. */
int  dvm_fuser_release(dvm_fuser *f, int value);
/* Run everything that is buffered. */
int  dvm_fuser_flush(dvm_fuser *f);
/* Counters since creation: operators issued, launches, flushes, results never written. */
int  dvm_fuser_stats(const dvm_fuser *f, int64_t *n_ops, int64_t *n_launches, int64_t *n_flushes, int64_t *n_elided);
/* Copy out the bytecode of the most recent launch (DVM_E_BUFSZ with *len set if `cap` is too small). */
int  dvm_fuser_last_code(const dvm_fuser *f, void *bytecode, size_t cap, size_t *len);

/* Structural check of a bytecode blob: header fields, segment and instruction lengths, register
 * and tensor indices, launch geometry.  dvm_run calls it on every launch. */
int  dvm_validate(const void *bytecode, size_t len);

/* Readable dump (Section 4.2, the printed example program: tile number, tiles per core, kernel
 * type, one line per instruction).  Always NUL-terminates within `cap`. */
int  dvm_disasm(const void *bytecode, size_t len, char *txt, size_t cap);

/* Introspection of an encoded program. */
typedef struct dvm_code_info {
    int32_t  kernel_type;      /* 0 = meta-kernel on the vector path, 1 = temporally stacked      */
    int32_t  n_segments;
    int32_t  n_tensors;
    int32_t  grid;             /* workgroups launched (the N of Algorithm 2)                      */
    int32_t  block;            /* threads per workgroup                                           */
    int32_t  variant_k;        /* elements per lane per tile register of the interpreter variant  */
    int32_t  variant_nr;       /* tile registers of the interpreter variant                       */
    int32_t  n_instructions;   /* over all segments                                               */
    int64_t  n_tiles;          /* over all segments (the M of Algorithm 2, summed)                */
    int64_t  code_bytes;       /* over all segments (CodeSize, summed)                            */
    int32_t  n_launches;       /* kernel launches dvm_run issues for this bytecode (1 unless parts ask for their own) */
    int32_t  reserved;
} dvm_code_info;
int  dvm_code_info_get(const void *bytecode, size_t len, dvm_code_info *info);
/* Minimum size in bytes of the buffer behind tensors[index], and whether it is written (*is_output: 0 an
 * input, 1 an output, 2 the launch's workspace, see dvm_stack_dependent). */
int  dvm_code_tensor(const void *bytecode, size_t len, int index,
                     int64_t *min_bytes, int *is_output, int *dtype, int *align_bytes);

/* The tile-size rule on a one-dimensional space (Section 4.2, hardware_align_div): among tile
 * sizes 1..t_max the one minimising ceil(ceil(total/t)/n_cores) * (t + overhead), ties to the
 * larger tile, then rounded up to a multiple of `align` without exceeding t_max.
 * Writes the minimum-cost size, the aligned size and the resulting number of tiles. */
int  dvm_plan(int64_t total, int n_cores, int64_t t_max, int align, int overhead,
              int64_t *t_min_cost, int64_t *t_aligned, int64_t *n_tiles);

/* ---- device execution ---------------------------------------------------------------------------- */
/*
 * Launch the interpreter for `bytecode` on `hip_stream` and return without waiting.
 *   tensors[n_tensors]  DEVICE pointers: the program's inputs in declaration order, then its
 *                       outputs (for a stacked program: part after part).
 * The bytecode is copied into the launch's kernel arguments before the call returns; the caller
 * may reuse its buffer at once.  ctx must have been created for a real device.
 */
int  dvm_run(const dvm_ctx *ctx, const void *bytecode, size_t len,
             void *const *tensors, int n_tensors, void *hip_stream);

/* One launch that runs `bytecode` n_sets times, each time on the next set of tensors: `tensor_sets` is a HOST array of
 * n_sets * n_tensors DEVICE pointers, set after set, each set in the order dvm_run takes it (n_tensors as the
 * bytecode lists them).  Every set is checked as dvm_run checks its tensors.  The sets must be independent: no set
 * reads what another writes (the workgroups pass from one set to the next without waiting for each other); sets that
 * write the same buffer leave the result of one of them.  `table` is DEVICE memory the caller lends to the launch
 * (8-byte aligned, table_bytes >= 8 * n_sets * n_tensors): the addresses are copied there on `hip_stream` and read
 * from there by the launch, so it must stay untouched until the launch has finished.  Bytecode that lists a
 * workspace (dvm_stack_dependent with a grid-wide wait) is refused with DVM_E_UNSUPPORTED.
 * Use: the layers of a model step that apply one program (or one stack of programs) to different tensors of the
 * same shapes -- one encode, one launch. */
int  dvm_run_batched(const dvm_ctx *ctx, const void *bytecode, size_t len,
                     void *const *tensor_sets, int n_tensors, int n_sets,
                     void *table, size_t table_bytes, void *hip_stream);

/* dvm_run for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same launch, but where the bytecode lists a workspace (dvm_stack_dependent)
 * the library's own array in device memory takes its place -- DVM_STATIC_WORKSPACE_BYTES per device, part of the
 * library's image, held until the process ends -- and tensors[] holds the bytecode's tensors WITHOUT the workspace
 * entry (n_tensors one less than the bytecode lists).  Bytecode without a workspace runs exactly as with dvm_run.
 * The call allocates nothing and frees nothing; it clears the part of the array it uses with a small kernel on
 * `hip_stream` before the launch.  A launch that needs more workspace than the array holds is refused with
 * DVM_E_LIMIT (use dvm_run with a workspace of the caller's).  All calls on one device share that device's array,
 * which keeps the last call's contents: calls that may overlap in time on one device (different streams, or
 * different threads) race on it and must be serialised by the caller. */
#define DVM_STATIC_WORKSPACE_BYTES (4u << 20)
int  dvm_run_static(const dvm_ctx *ctx, const void *bytecode, size_t len,
                    void *const *tensors, int n_tensors, void *hip_stream);

/* ---- measurement support (Section 6.1: run time and compile time are measured apart) ----------------- */
/* dvm_encode called `reps` times on the same arguments, each call timed with CLOCK_MONOTONIC inside the library
 * (no language binding between the clock and the encoder); ns[r] receives the duration of call r in nanoseconds,
 * ns[0] being the first call for these shapes.  Everything else as dvm_encode (out_shapes is not filled). */
int  dvm_encode_timed(const dvm_ctx *ctx, const dvm_prog *prog, const dvm_shape *in_shapes, int n_in,
                      const dvm_shape *out_layout, void *bytecode, size_t cap, size_t *len, int reps, int64_t *ns);
/* A plain copy kernel of this library's own: `bytes` (a positive multiple of 16 KiB) from `src` to `dst` (DEVICE
 * pointers, 16-byte aligned, not overlapping) on `hip_stream`, asynchronously; 16 bytes per lane and access,
 * streaming cache hints, tiles dealt out to the workgroups as `assignment` says (dvm_assignment).  It is the
 * bandwidth ceiling of a load-store loop on the device, measured beside the interpreter. */
int  dvm_copy_kernel(const dvm_ctx *ctx, void *dst, const void *src, size_t bytes, int assignment, void *hip_stream);

const char *dvm_strerror(int status);
/* Detail text of the last error raised on the calling thread ("" if none). */
const char *dvm_last_error_detail(void);
int  dvm_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DVM_H */
