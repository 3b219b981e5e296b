/*
 * sparsert.h - C ABI of the MI355X (gfx950) SpMM / sparse 3x3 convolution library.
 *
 * The library follows the inspector-executor split of the paper (Section 2.3):
 * the sparse weight matrix A is fully known ahead of time, so it is analysed
 * once on the host (`sparsert_inspect`) and the resulting immutable plan is
 * executed many times against changing dense activations (`sparsert_spmm`,
 * `sparsert_conv3x3`).
 *
 * Conventions used by every entry point
 *   - Matrices are C-style row-major (Section 3.2): B is K x N with N contiguous,
 *     C is M x N with N contiguous; rows follow each other at a pitch of N
 *     elements unless options.ldb / options.ldc say otherwise.
 *   - "HOST" pointers are ordinary CPU memory; "DEVICE" pointers are HIP
 *     device memory on the device that was current when the plan was made.
 *   - Every function returns a status code (sparsert_status: 0 = ok, negative = error) and
 *     never aborts; sparsert_last_error() gives a thread-local message.
 *   - No torch / C++ types cross this boundary.
 *   - Threads: every entry point may be called from several host threads at once; calls that
 *     make a plan (inspect, tune, plan_load) each build their own, and a finished plan is
 *     read only.  sparsert_tune starts a few short-lived host threads of its own to prepare
 *     its candidates and joins them before it returns.
 */
#ifndef SPARSERT_H
#define SPARSERT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sparsert_plan sparsert_plan; /* opaque; immutable after inspect */

typedef enum sparsert_status {
    SPARSERT_OK = 0,
    SPARSERT_EINVAL = -1,       /* bad argument / malformed CSR / misaligned pointer */
    SPARSERT_ENOMEM = -2,       /* host or device allocation failed */
    SPARSERT_EHIP = -3,         /* a HIP runtime call or kernel launch failed */
    SPARSERT_EUNSUPPORTED = -4, /* legal request outside what is implemented */
    SPARSERT_ECOMPILE = -5      /* assembling or loading a generated kernel failed */
} sparsert_status;

/* Storage type of vals, B/X and C/Y.  Floating types accumulate in IEEE
 * binary32; with SPARSERT_F16 each product of two halves is exact in binary32
 * and the sum is rounded to half once, at the store.  SPARSERT_I8 (the low
 * precision the paper leaves as future work, Section 6): vals and B/X are
 * int8, C/Y is int32, sums are exact 32-bit integers (the inspector refuses a
 * K long enough to overflow them); no scaling or requantisation is applied. */
typedef enum sparsert_dtype { SPARSERT_F32 = 0, SPARSERT_F16 = 1, SPARSERT_I8 = 2 } sparsert_dtype;

/* Executor families (options.kernel / INFO[SPARSERT_INFO_KERNEL]). */
typedef enum sparsert_kernel {
    SPARSERT_KERNEL_AUTO = 0,  /* the inspector chooses: the generated kernel with its shape-dependent
                                  defaults when the code object manager (libamd_comgr) can be loaded, A has
                                  at most 4194304 nonzeros (about 4 s of assembling per million; the inspector is off
                                  the latency path, Section 2.3) and neither vec nor split_threshold is set;
                                  the row-walk kernel otherwise, and also when the generator declines the
                                  problem (EUNSUPPORTED / ECOMPILE) */
    SPARSERT_KERNEL_ROWS = 1,  /* one wave per row, B read straight from L2/HBM */
    SPARSERT_KERNEL_SPEC = 2   /* per-matrix generated gfx950 code with the nonzeros of A as
                                  instruction constants (Section 3.5) */
} sparsert_kernel;

/* Variants of the generated kernel (options.spec_mode). */
typedef enum sparsert_spec_mode {
    SPARSERT_SPEC_AUTO = 0,
    SPARSERT_SPEC_DIRECT = 1, /* a workgroup's waves run one code block on adjacent column tiles;
                                 B rows are read straight from L2/L1 */
    SPARSERT_SPEC_LDS = 2     /* a workgroup's waves run adjacent code blocks on one column tile;
                                 the tile's B rows are staged once through LDS (SpMM plans of every
                                 storage type; half and int8 operands are widened to 32 bits on the way in) */
} sparsert_spec_mode;

/* Zero-initialise, then set what you need.  All-zero = fp32 SpMM, automatic tiling. */
typedef struct sparsert_options {
    int32_t dtype;           /* sparsert_dtype */
    int32_t kernel;          /* sparsert_kernel; AUTO lets the inspector choose */
    int32_t conv;            /* 0: SpMM plan.  1: 3x3 / pad 1 / stride 1 convolution plan */
    int32_t Cin, H, W;       /* conv only: K must equal 9*Cin and N must equal H*W */
    int32_t batch;           /* problems per call, 1..65535 (0 is read as 1): images of a convolution,
                                or B/C pairs of an SpMM stored back to back (one more grid dimension) */
    int32_t host_only;       /* 1: analyse only; no HIP call is made, the plan can be
                                exported but not executed */
    int32_t vec;             /* columns of C per lane; 0 = automatic, else 1,2,4 (,8 for f16; 1 or 4 for int8) */
    int32_t split_threshold; /* rows with at least this many nonzeros are split over the
                                waves of a workgroup; 0 = automatic */
    int32_t spec_rows;       /* SPARSERT_KERNEL_SPEC: rows of A per generated code block
                                (accumulator registers per wave), 1 ... 232 as far as the registers
                                of the workgroup's waves fit a compute unit; 0 = automatic: as many
                                as leave the launch about two waves per SIMD of the chip, at most 96,
                                then up to 15 % more (at most 128) where that spares the launch a
                                last round of workgroups that only a few compute units take part in */
    int32_t spec_depth;      /* SPARSERT_KERNEL_SPEC: B rows a wave keeps in flight; 0 = automatic */
    int32_t spec_tiles;      /* SPARSERT_KERNEL_SPEC: waves per workgroup (adjacent column tiles in
                                DIRECT mode, adjacent code blocks in LDS mode): 1,2,4,8,16;
                                0 = automatic */
    int32_t spec_mode;       /* sparsert_spec_mode; 0 = automatic: DIRECT, except that an fp32 SpMM plan with no
                                other tiling field set takes the LDS-staged variant with eight waves when A is
                                at least 94.5 % sparse, M >= 2048, K >= 1024 and M x ceil(N / 64) x batch >= 131072 */
    int32_t spec_ksplit;     /* SPARSERT_KERNEL_SPEC, DIRECT: 2, 4 or 8 waves of a workgroup share one
                                code block's rows and column tile and split its columns (equal
                                nonzero shares, partial sums meet in LDS, in several phases if
                                they exceed it); 1 = no split; 0 = no split if spec_rows is given,
                                automatic if spec_rows is 0 too (split where K >= 512 and the
                                rows alone do not supply the waves).  Sets the workgroup width,
                                spec_tiles is then ignored */
    int32_t natural_order;   /* 1: load-balance ablation (Section 4.3): rows keep their input order
                                (identity permutation), no row is split over waves, and the
                                generated kernel's blocks are contiguous row ranges; 0 = balanced */
    int32_t spec_lanes;      /* SPARSERT_KERNEL_SPEC, DIRECT: widest column tile of a wave, 16, 32 or 64
                                lanes (0 = 64).  Narrow tiles leave lanes idle but let a compute unit
                                cover more rows of fewer columns; measured slower wherever tried,
                                kept for experiments */
    int32_t spec_swizzle;    /* SPARSERT_KERNEL_SPEC: 1 = rows are dealt to code blocks by column-pattern
                                similarity (the row swizzle Section 5 names as a preprocessing step
                                that would help), so a block touches fewer rows of B; 0 = serpentine deal */
    int32_t spec_vec;        /* SPARSERT_KERNEL_SPEC, DIRECT, SpMM: columns of C per lane; 0/1, or the 2 halves
                                (half plans) / 4 int8 (int8 plans) that share the dword a lane loads,
                                which halves / quarters the fetches per column; N must be a multiple */
    int32_t ldb, ldc;        /* SpMM: elements between the starts of consecutive rows of B and of C (leading
                                dimensions; 0 = N, else >= N).  A wider pitch lets a call work on a column
                                slice of larger activation matrices (Section 4.3: more columns only make N
                                larger).  With batch = b the operands are [b, K, ldb] and [b, M, ldc].
                                Convolution plans take 0 */
    int32_t tune_warm;       /* sparsert_tune only.  0: candidates are ranked by their time when every launch
                                finds its code and operands displaced from the L2 caches, as inside a model
                                where other layers run in between; 1: by back-to-back launches of the same plan */
    int32_t spec_prefetch;   /* SPARSERT_KERNEL_SPEC: 1 = every wave touches the code of its block with a few
                                loads before it runs into it, so that the L2 misses of straight-line code
                                that other layers have displaced overlap instead of following each other
                                (costs about 0.5 us when the code is still in the L2, gains more than that
                                when it is not; the tuner tries it on its winner); 0 = off */
    int32_t reserved[2];     /* must be zero */
} sparsert_options;

/*
 * Inspector (Sections 2.3, 3.4).  Analyses the fixed sparsity pattern of A and
 * builds the plan: per-row nonzero counts and their histogram, the row
 * permutation and bins used for wavefront load balance, the permuted CSR, the
 * split of long rows over the waves of a workgroup so that every wave but the
 * last gets the same number of nonzeros, and the packed nonzero stream the
 * executor reads.  Integer work only: values are moved, never altered.
 *
 *   row_ptr  HOST int32[M+1], row_ptr[0] == 0, non-decreasing
 *   col_idx  HOST int32[nnz], 0 <= col < K, strictly ascending inside each row
 *   vals     HOST float[nnz] (SPARSERT_F32), IEEE half[nnz] (SPARSERT_F16) or int8[nnz] (SPARSERT_I8);
 *            explicit zeros, -0.0, NaN payloads are kept bit for bit
 *   M, K, N  > 0.  N is part of the plan (it fixes tiling and B row offsets).
 *   opt      may be NULL (= all zero)
 *   out      receives the plan on success, is set to NULL on failure
 *
 * The CSR is deep-copied; the caller may free its arrays at once.  Unless
 * opt->host_only is set the plan's device arrays are allocated and uploaded
 * here (synchronously) on the current HIP device.
 * Errors: EINVAL for null pointers, non-positive sizes, malformed CSR, bad
 * options; EUNSUPPORTED for B or C of 2 GiB and more, for one image of X of 128 MiB and more;
 * ENOMEM / EHIP from allocation and upload.
 */
int sparsert_inspect(const int32_t *row_ptr, const int32_t *col_idx, const void *vals,
                     int32_t M, int32_t K, int32_t N,
                     const sparsert_options *opt, sparsert_plan **out);

/*
 * Executor, SpMM (Section 3.2 statement of the problem; Section 3.5, the
 * per-thread-group loop): C = A x B, C fully overwritten (no alpha/beta); a
 * row of A without nonzeros yields +0.0.
 *
 *   B_dev  DEVICE, K x N row-major at a row pitch of ldb elements, plan's dtype, 16-byte aligned, read only
 *   C_dev  DEVICE, M x N row-major at a row pitch of ldc elements, plan's dtype (int32 for int8 plans),
 *          16-byte aligned; only the N columns of every row are written, the rest of a wider pitch is untouched
 *   stream a hipStream_t (NULL = the null stream)
 *
 * With opt->batch = b the call multiplies b matrices stored back to back, B_dev as
 * [b, K, N] and C_dev as [b, M, N], by the same A in one launch (larger N is where the
 * method is expected to do best, Section 4.3; the batch is one more grid dimension).
 *
 * Asynchronous on `stream`; allocates nothing; does not synchronise.  The plan
 * is read only, so concurrent calls on different streams are legal provided
 * their C buffers differ.  B and C are borrowed and must not overlap.
 * Errors: EINVAL (null/misaligned pointer, conv plan, host-only plan), EHIP.
 */
int sparsert_spmm(const sparsert_plan *plan, const void *B_dev, void *C_dev, void *stream);

/*
 * Executor, sparse 3x3 convolution (Section 3.6): padding 1, stride 1,
 * cross-correlation.  The filter bank [Cout, Cin, 3, 3] is the plan's A with
 * M = Cout and column k = c*9 + r*3 + s; the im2col matrix is never built -
 * every reference to B[k, oh*W+ow] reads X[c, oh+r-1, ow+s-1] and the padding
 * test is resolved per (r,s) group by the inspector's ordering, not per
 * multiply.  The paper evaluates batch 1 (Section 4.2); with opt->batch = b the
 * b images of a call are independent convolutions with the same filters, run
 * by one launch (the image is one more grid dimension).
 *
 *   X_dev  DEVICE, [batch, Cin, H, W] contiguous, plan's dtype, 16-byte aligned
 *   Y_dev  DEVICE, [batch, Cout, H, W] contiguous, plan's dtype (int32 for int8 plans), 16-byte aligned
 *
 * Same asynchrony, ownership and error rules as sparsert_spmm; EINVAL if the
 * plan was not made with opt->conv = 1.
 */
int sparsert_conv3x3(const sparsert_plan *plan, const void *X_dev, void *Y_dev, void *stream);

/*
 * Autotuner (Section 3.7: exhaustive search over a short hand-picked list of executor
 * configurations, done once per problem, off the inference path).  Builds a plan for each
 * candidate configuration - executor family, columns per lane, split threshold, rows per
 * generated code block, waves per workgroup, K split, staging variant, row swizzle - times it on the GPU with the
 * given operands, and returns the fastest plan (fastest with cold caches unless base->tune_warm is set: inside a
 * model a layer's code and operands have been displaced by the layers before it).  Every candidate's output is
 * compared on the GPU with the first candidate's (the row-walk or default plan); one that disagrees beyond the
 * storage type's tolerance is reported and never returned.  `base` fixes dtype, the convolution
 * geometry and natural_order; base->kernel other than AUTO restricts the search to that
 * executor family (the specialisation ablation); its other tuning fields are ignored.
 *
 *   in_dev / out_dev  DEVICE buffers of the shapes sparsert_spmm / sparsert_conv3x3 take;
 *                     out_dev is overwritten many times
 *   stream            launches and timing events go to this stream; the call synchronises it
 *   out               receives the best plan
 *   report            may be NULL; receives one entry per timed candidate (the first SPARSERT_TUNE_MAX of
 *                     them; later candidates are still timed and may be the one returned)
 *
 * Errors: as sparsert_inspect; EHIP if timing fails.  Allocates (plans, events): not for the
 * inference path.
 */
#define SPARSERT_TUNE_MAX 64
typedef struct sparsert_tune_entry {
    int32_t kernel, vec, split_threshold, spec_mode, spec_rows, spec_tiles, spec_ksplit, spec_lanes, spec_swizzle, spec_vec;
    float microseconds;      /* per launch, back-to-back launches of this plan; negative if the candidate failed */
    float cold_microseconds; /* per launch when a cache-displacing fill runs before every launch (the fill's own
                                time subtracted); negative if the candidate failed */
    int32_t agrees;          /* 1: the candidate's output matches the first candidate's within the storage type's
                                tolerance (bit for bit for int8 plans); 0: it does not, and the candidate was
                                not considered */
    int32_t spec_prefetch;   /* SPEC plans: 1 if the waves prefetch the code of their block */
} sparsert_tune_entry;
typedef struct sparsert_tune_report {
    int32_t count;
    float best_microseconds;       /* the returned plan, back-to-back launches */
    float best_cold_microseconds;  /* the returned plan, caches displaced before every launch */
    sparsert_tune_entry entries[SPARSERT_TUNE_MAX];
} sparsert_tune_report;
int sparsert_tune(const int32_t *row_ptr, const int32_t *col_idx, const void *vals,
                  int32_t M, int32_t K, int32_t N, const sparsert_options *base,
                  const void *in_dev, void *out_dev, void *stream,
                  sparsert_plan **out, sparsert_tune_report *report);

/*
 * Comparison of two results of one plan: what the autotuner does with every candidate (Section 3.7
 * searches configurations that must all compute the same product), callable on its own to hold a
 * new plan's output against a trusted one on live operands.
 *
 *   a_dev, b_dev  DEVICE, two outputs of `plan` ([batch, M, ldc] / [batch, Cout, H, W], the plan's
 *                 result type), 16-byte aligned, read only; only the N valid columns are looked at
 *   result_dev    DEVICE, four 32-bit words, 16-byte aligned, written: the bits of the float
 *                 max |a - b| and of the float max |b| over elements finite in both (0 for int8 plans),
 *                 the number of elements that differ in kind (finite against not finite, NaN against
 *                 not NaN; for int8 plans: that differ at all), and the number of blocks used
 *
 * Deterministic (no atomics).  Allocates its partial results for the call and frees them before it
 * returns, so it synchronises `stream`.  Errors: EINVAL (null / misaligned pointer, host-only plan,
 * other device), ENOMEM, EHIP.
 */
int sparsert_compare_outputs(const sparsert_plan *plan, const void *a_dev, const void *b_dev,
                             void *result_dev, void *stream);

/*
 * sparsert_compare_outputs for callers that cannot allocate device memory: code under HIP graph
 * capture, serving loops and harnesses that forbid hipMalloc.  Same arguments and result words;
 * the partial results live in a static device array of the library (32 KiB on every GPU the
 * library runs on, held until the process ends) instead of memory allocated for the call.
 * Allocates nothing, does not synchronise: two kernels on `stream`.
 * Limit: outputs of at most 33 554 432 elements (batch * M * N); larger ones give EUNSUPPORTED.
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 * host threads) race and may return each other's figures; calls on one stream are ordered.
 * Nothing has to be cleared between calls: a call reads only the slots it has written itself.
 */
int sparsert_compare_outputs_static(const sparsert_plan *plan, const void *a_dev, const void *b_dev,
                                    void *result_dev, void *stream);

/* Arrays of the plan that sparsert_plan_export can copy out (HOST side). */
typedef enum sparsert_field {
    SPARSERT_FIELD_INFO = 0,      /* int32[SPARSERT_INFO_COUNT], see below */
    SPARSERT_FIELD_ROW_NNZ = 1,   /* int32[M]   nonzeros per original row */
    SPARSERT_FIELD_HIST = 2,      /* int32[33]  rows per bin; bin(0)=0, bin(x)=1+floor(log2 x) */
    SPARSERT_FIELD_PERM = 3,      /* int32[M]   slot -> original row: stable sort by nnz descending */
    SPARSERT_FIELD_INV_PERM = 4,  /* int32[M]   original row -> slot */
    SPARSERT_FIELD_P_ROW_PTR = 5, /* int32[M+1] row pointer of the permuted CSR */
    SPARSERT_FIELD_P_COL_IDX = 6, /* int32[nnz] columns, rows gathered by PERM, ascending per row */
    SPARSERT_FIELD_P_VALS = 7,    /* dtype[nnz] values, bit copies */
    SPARSERT_FIELD_BINS = 8,      /* int32[nbins][4]: bin id, first slot, rows, nonzeros */
    SPARSERT_FIELD_STREAM = 9,    /* uint32[nnz][2]: what the executor reads per nonzero:
                                     {operand byte offset as int32, value as binary32 bits
                                     (int8 plans: the value sign-extended to int32)}.
                                     SpMM: offset = col*N*sizeof(dtype), permuted-CSR order.
                                     Conv: word = tap << 28 | (d & 0x0fffffff), tap = r*3+s,
                                     d = (c*H*W + (r-1)*W + (s-1))*sizeof(dtype) (may be
                                     negative); each slot ordered by (tap, c) */
    SPARSERT_FIELD_CONV_SEG = 10, /* conv only, int32[M][10]: stream positions where each
                                     (r,s) group of a slot starts; [9] = end of the slot */
    SPARSERT_FIELD_SEGMENTS = 11, /* int32[n_split][Gy+1]: stream positions bounding the
                                     share of each wave of a split row */
    SPARSERT_FIELD_SPEC_GROUPS = 12, /* SPEC plans, int32[M]: code block (row group) of each slot */
    SPARSERT_FIELD_SPEC_COLUMNS = 13, /* SPEC plans, int32[blocks]: B rows a code block loads per tile
                                         (blocks = groups x K parts; padded in the LDS variant) */
    SPARSERT_FIELD_SPEC_CODE = 14, /* SPEC plans, bytes: the generated gfx950 code object */
    SPARSERT_FIELD_KERNEL_NAME = 15 /* bytes (no terminator): the name a kernel trace shows for this plan's
                                      launches - the generated kernel's symbol, which carries the problem
                                      shape, or the row-walk kernel's template instance */
} sparsert_field;

enum {
    SPARSERT_INFO_M = 0, SPARSERT_INFO_K, SPARSERT_INFO_N, SPARSERT_INFO_NNZ,
    SPARSERT_INFO_DTYPE, SPARSERT_INFO_CONV, SPARSERT_INFO_CIN, SPARSERT_INFO_H,
    SPARSERT_INFO_W, SPARSERT_INFO_KERNEL,
    SPARSERT_INFO_VEC,            /* V: columns of C per lane */
    SPARSERT_INFO_LANES_PER_TILE, /* lanes of a wave that own columns */
    SPARSERT_INFO_N_TILES,        /* column tiles; a wave covers LANES_PER_TILE*V columns */
    SPARSERT_INFO_GY,             /* waves per workgroup */
    SPARSERT_INFO_SPLIT_THRESHOLD,
    SPARSERT_INFO_N_SPLIT,        /* slots [0, N_SPLIT) are split rows */
    SPARSERT_INFO_N_WG_ROWS,      /* workgroups along M: N_SPLIT + ceil((M-N_SPLIT)/GY) */
    SPARSERT_INFO_N_BINS,
    SPARSERT_INFO_SPEC_ROWS,      /* SPEC plans: rows per code block */
    SPARSERT_INFO_SPEC_GROUPS,    /* SPEC plans: number of code blocks */
    SPARSERT_INFO_SPEC_DEPTH,     /* SPEC plans: B rows in flight per wave */
    SPARSERT_INFO_SPEC_CODE_BYTES,
    SPARSERT_INFO_SPEC_TILES,     /* SPEC plans: waves per workgroup */
    SPARSERT_INFO_SPEC_MODE,      /* SPEC plans: sparsert_spec_mode in use */
    SPARSERT_INFO_SPEC_LDS_BYTES, /* SPEC plans: LDS per workgroup */
    SPARSERT_INFO_SPEC_KSPLIT,    /* SPEC plans: K parts per workgroup (1 = none) */
    SPARSERT_INFO_NATURAL_ORDER,  /* 1 if the plan was built with natural_order */
    SPARSERT_INFO_SPEC_LANES,     /* SPEC plans: lanes per column tile in use (balanced, <= spec_lanes) */
    SPARSERT_INFO_SPEC_SWIZZLE,   /* SPEC plans: 1 if blocks were formed by similarity */
    SPARSERT_INFO_BATCH,          /* problems per call (>= 1) */
    SPARSERT_INFO_SPEC_VEC,       /* SPEC plans: columns per lane */
    SPARSERT_INFO_LDB,            /* elements between consecutive rows of B (N unless options.ldb) */
    SPARSERT_INFO_LDC,            /* elements between consecutive rows of C (N unless options.ldc) */
    SPARSERT_INFO_SPEC_PREFETCH,  /* SPEC plans: 128-byte lines of its block's code every lane touches ahead (0 = no prefetch) */
    SPARSERT_INFO_COUNT = 48      /* remaining entries are zero */
};

/*
 * Copies one plan array to HOST memory.  `need` (may be NULL) receives the size
 * in bytes; if `buf` is NULL only the size is reported; if `cap` is smaller
 * than the size nothing is copied and EINVAL is returned.
 */
int sparsert_plan_export(const sparsert_plan *plan, int32_t field,
                         void *buf, size_t cap, size_t *need);

/*
 * Plan persistence (Section 2.3: the inspector runs once, offline; Section 3.7: so does the
 * tuner).  sparsert_plan_save writes the whole plan - analysis arrays, executor choice and, for
 * a generated kernel, its assembled code object - into `buf`; sparsert_plan_load rebuilds it,
 * uploading to the current HIP device unless host_only is set, without analysing, generating
 * or assembling anything.  A loaded plan exports and executes exactly like the one saved.
 *
 *   buf/cap  HOST buffer; with buf == NULL only *need (bytes required) is reported
 *   size     bytes of a blob sparsert_plan_save wrote
 *
 * The blob is little endian and carries a format version and a checksum: a truncated,
 * corrupted or foreign blob gives EINVAL (EUNSUPPORTED for another format version).  The
 * checksum is no defence against a deliberately crafted blob: load only blobs this library
 * wrote.  A blob is tied to gfx950 and to the N, dtype and batch it was planned for.
 */
int sparsert_plan_save(const sparsert_plan *plan, void *buf, size_t cap, size_t *need);
int sparsert_plan_load(const void *buf, size_t size, int32_t host_only, sparsert_plan **out);

/* Frees the plan's host and device memory.  NULL is ignored.  The caller must
 * make sure no launch that uses the plan is still in flight. */
void sparsert_plan_destroy(sparsert_plan *plan);

/* Message of the last failing call on this thread ("" if none).  The pointer
 * stays valid until the next failing call on the same thread. */
const char *sparsert_last_error(void);

/* Library version as major*10000 + minor*100 + patch. */
int32_t sparsert_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPARSERT_H */
