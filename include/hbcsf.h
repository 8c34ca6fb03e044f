/* hbcsf.h -- C ABI of the MI355X (gfx950) sparse-MTTKRP library.
 *
 * The library computes mode-n sparse MTTKRP on tensors of order 3, 4 and 5,
 *
 *     Y(i_n, :) = sum over nonzeros X(i_1..i_N) * hadamard_{m != n} A_m(i_m, :)
 *
 * (Section II-C, Eq. 4-7), from a load-balanced hybrid compressed-sparse-fiber
 * representation (Sections IV and V: B-CSF with fbr-split and slc-split, CSL, and
 * the three-group HB-CSF partition), one representation per mode (the "ALLMODE"
 * setting of Section VI-A).
 *
 * Conventions (Algorithm "COO-MTTKRP" inputs and Section VI-A): indices are
 * 0-based uint32, values and factor matrices fp32 (hbcsf_mttkrp_f64: fp64
 * factor matrices and output), factor matrices and the output are dense
 * row-major [dims[m]][rank] with leading dimension = rank.
 *
 * Every function returns 0 on success or a negative HBCSF_E* code; the text of
 * the last failure on the calling thread is kept for hbcsf_last_error().  No
 * C++ exception crosses this boundary: every entry point that returns a code
 * catches whatever its body throws (a failed host allocation becomes
 * HBCSF_ENOMEM).  "host" / "device" on a pointer says
 * which memory it must point to.  The library never frees caller memory.
 */
#ifndef HBCSF_H_
#define HBCSF_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HBCSF_OK       0
#define HBCSF_EINVAL  -1  /* null pointer, unsupported order / mode / rank, bad option      */
#define HBCSF_ERANGE  -2  /* an index is >= its dimension, or a dimension is too large      */
#define HBCSF_ENOMEM  -3  /* host allocation failed, or the device arena is too small        */
#define HBCSF_ESTATE  -4  /* hbcsf_mttkrp before hbcsf_upload                                */
#define HBCSF_EHIP    -5  /* a HIP call failed; hbcsf_last_error() names it                  */

#define HBCSF_MAX_ORDER 5
#define HBCSF_MAX_FIBER_LEVELS (HBCSF_MAX_ORDER - 2)

typedef struct hbcsf_tensor hbcsf_tensor; /* opaque, owned by the library, freed by hbcsf_free */

/* Build options (all result-invariant: they change scheduling and storage only).
 * A zero field selects the default. */
typedef struct hbcsf_opts {
  uint32_t fiber_threshold;   /* T_f of fbr-split (Section IV-B, VI-B): no fiber segment holds more
                                 than T_f nonzeros.  Cuts fall on multiples of T_f in a group's
                                 nonzero stream.  8, 16, 32 or 64.  Default 64 (order 3), 32 (orders 4, 5),
                                 chosen for rank 32; a wavefront keeps 64 / (rank / 4) runs in LDS at a time, so
                                 for ranks 16 / 8 half / a quarter of the default keeps the same number of
                                 wavefronts resident and is markedly faster.                                 */
  uint32_t slice_threshold;   /* T_s of slc-split (Section IV-A): nonzeros one wavefront works
                                 through before it merges its partial rows; a slice of n nonzeros
                                 is shared by at most ceil(n/T_s)+1 wavefronts.  0 = sized from
                                 the device at launch.                                             */
  uint32_t mode_order_policy; /* order of the non-root modes in each per-mode tree (the paper
                                 leaves it open): 0 = shorter dimension nearer the root,
                                 1 = longer dimension nearer the root, 2 = increasing mode number. */
  uint32_t group_mask;        /* HB-CSF groups in use (Section V): bit0 = COO group, bit1 = CSL
                                 group.  Default (0) = 3 = both.  4 = neither (plain B-CSF),
                                 for ablation.  Slices of a disabled group go to the CSF group.    */
  uint32_t hybrid_granularity;/* 0 = the group is chosen per slice (Section V).  1 = per fiber inside
                                 heavy slices (Section VI-F leaves the sparse portion open to further
                                 work): a slice of at least 2 T_f nonzeros with at least an eighth of
                                 them in singleton deepest-level fibers is stored as two pieces with
                                 the same root index, the singleton-fiber nonzeros in the CSL group and
                                 the others in the CSF group; both pieces are merged with atomic adds.
                                 Needs the CSL group enabled; otherwise ignored.                     */
  uint32_t coo_row_flags;     /* 1 = the COO group stores no root index per nonzero (N-1 instead of N
                                 index words each): its nonzeros are kept in row order, and one flag
                                 per output row (HBCSF_ARR_COO_BITS) with a running count per 32 rows
                                 (HBCSF_ARR_COO_PTR) says which row each belongs to.  hbcsf_mttkrp then
                                 always computes the group's rows in the output-definition pass.  0
                                 (default): root indices are stored and either kernel can be used.    */
  uint32_t mid_blocking;      /* blocking of the first fiber level (Section VIII: blocking as complementary
                                 work): its index range is cut into 2^bits equal blocks and the nonzeros are
                                 ordered by (block, root, level 1, .., leaf), so a slice is stored as one
                                 piece per block (all pieces merged with atomic adds, the COO group unused)
                                 and consecutive slices' pieces gather the same level-1 rows while they are
                                 still in the L2.  0 or 1 = off (default); 2..13 = that many bits in every
                                 mode whose level-1 index is wider.  A measured alternative that lost.
                                 hbcsf_stats.slices then counts pieces.                                  */
  uint32_t single_representation; /* 0 (default): one representation per mode (the "ALLMODE" setting of
                                 Section VI-A, which the paper uses).  1: only mode 0's representation is
                                 built and kept (about 1 / order of the device memory), plain B-CSF (no
                                 COO / CSL groups, default T_f); hbcsf_mttkrp for another mode walks that
                                 tree with the target at a lower level and adds every fiber's (or, for
                                 the leaf mode, every nonzero's) contribution with atomic adds: slower,
                                 rank 32 only for those modes.  Other fields must be 0 (defaults).
                                 hbcsf_get_stats and hbcsf_host_array answer for mode 0 only.            */
} hbcsf_opts;

/* Per-mode statistics of the built representation.  "words" are 4-byte index words as the
 * paper counts storage (values excluded): COO 3M (Section III-A), CSF 2S+2F+M (Section III-B),
 * HB-CSF the sum over its three groups (Section V, the 24 / 24 / 19-word example). */
typedef struct hbcsf_stats {
  uint64_t nnz;               /* M                                                            */
  uint64_t slices;            /* S: non-empty slices of this mode                             */
  uint64_t fibers[HBCSF_MAX_FIBER_LEVELS];   /* F per fiber level (1 .. order-2) before fbr-split */
  uint64_t segments[HBCSF_MAX_FIBER_LEVELS]; /* fiber segments per fiber level in the CSF group (F') */
  uint64_t group_nnz[3];      /* nonzeros in the COO, CSL, CSF groups                         */
  uint64_t group_slices[3];   /* slices in the COO, CSL, CSF groups                           */
  uint64_t shared_slices;     /* slices merged with atomic adds (they span several runs)      */
  uint64_t runs[3];           /* lane-group runs (T_f nonzeros each) per group                */
  uint64_t words_coo;         /* N*M                                                          */
  uint64_t words_csf;         /* plain CSF of the whole tensor, no splitting                  */
  uint64_t words_hbcsf;       /* the three groups, no splitting (the paper's accounting)      */
  uint64_t stream_bytes[3];   /* bytes of device arrays each group kernel reads, as built     */
  uint64_t distinct_rows[3][HBCSF_MAX_ORDER]; /* [group][level]: distinct factor rows gathered */
  uint64_t owned_rows;        /* output rows written by one plain store (no zero-fill needed) */
  uint64_t flops_real;        /* multiply-adds actually done x2 (Section III-B's count)       */
  uint32_t level_mode[HBCSF_MAX_ORDER]; /* tensor mode at tree level 0 (root) .. N-1 (leaf)   */
  uint32_t fiber_threshold;   /* T_f in use                                                   */
  double   build_seconds;     /* host time to build this mode's representation                */
} hbcsf_stats;

/* Builds the per-mode HB-CSF representations on the host (sort by mode, CSF, fbr-split,
 * slice classification into the COO / CSL / CSF groups, run tables for slc-split).
 *   order  3, 4 or 5.      dims   host [order].          nnz  number of stored nonzeros (>= 0).
 *   inds   host [order] pointers to host [nnz] index arrays, inds[m][z] < dims[m].
 *   vals   host [nnz].     opts   host, may be NULL.
 *   out    receives the handle.  The inputs are not referenced after the call returns.
 * Duplicate coordinates are legal and act as separate nonzeros.
 * Limits: dims[m] <= 2^31 - 2, nnz < 2^32 - 2^16. */
int hbcsf_build_format(int order, const uint64_t *dims, uint64_t nnz,
                       const uint32_t *const *inds, const float *vals,
                       const hbcsf_opts *opts, hbcsf_tensor **out);

/* Size in bytes of the device arena that holds all modes' arrays. */
int hbcsf_device_bytes(const hbcsf_tensor *t, uint64_t *bytes);

/* Copies all modes' arrays into the caller's device arena (device, 256-byte aligned, at least
 * hbcsf_device_bytes bytes) on hip_stream (a hipStream_t, NULL = the default stream) and
 * waits for the copy.  The arena must stay valid while the handle is used for hbcsf_mttkrp. */
int hbcsf_upload(hbcsf_tensor *t, void *device_arena, uint64_t bytes, void *hip_stream);

/* Mode-`mode` (0-based) MTTKRP, asynchronous on hip_stream.
 *   rank     8, 16, 32, 64 or 128.
 *   factors  host array of `order` device pointers; factors[m] is [dims[m]][rank] row-major,
 *            16-byte aligned; factors[mode] is ignored (may be NULL).
 *   out      device [dims[mode]][rank], 16-byte aligned, OVERWRITTEN: every row is defined
 *            (rows of empty slices are zero), as Algorithm "COO-MTTKRP" returns Y from zero.
 * Launches the output-definition kernel, then the COO-group, CSL-group and B-CSF-group kernels
 * (Algorithm "HB-CSF-MTTKRP", execute step); for small outputs the COO group's rows are written
 * by the output-definition pass instead (HBCSF_TUNE_FUSE_COO).  Slices that span several work units
 * are merged with fp32 atomic adds (Section IV-A), so results can differ between runs in
 * the last bits.  NaN / Inf inputs propagate.  The handle is const because the representation is
 * only read; with profiling on (HBCSF_TUNE_PROFILE) the call also records HIP events into the
 * handle's event ring, which is bookkeeping outside the const promise, so calls on one handle
 * must not overlap in time while profiling or tracing is on.
 * With profiling off the call only launches kernels on hip_stream (no memset, no allocation, no
 * host wait), so it can be recorded into a HIP graph and replayed. */
int hbcsf_mttkrp(const hbcsf_tensor *t, int mode, int rank, const float *const *factors,
                 float *out, void *hip_stream);

/* The same operation with fp64 factor matrices, partial sums and output (Section VI-A fixes fp32 for the
 * paper's measurements; this is the double-precision form of Eq. 3 / Algorithm "COO-MTTKRP").  The tensor's
 * values stay the fp32 values the handle was created from and are widened where they are multiplied, so the
 * result is the fp64 sum of exactly the products the fp32 path rounds; slices that span several work units
 * are merged with fp64 atomic adds.
 *   rank     16, 32 or 64.
 *   factors, out   as for hbcsf_mttkrp, with double elements ([dims[m]][rank] row-major, 16-byte aligned).
 * Same kernels, launches, format options and tuning keys as hbcsf_mttkrp (a row is split over rank / 2
 * lanes of two doubles instead of rank / 4 lanes of four floats); not available on a
 * single_representation handle (HBCSF_EINVAL). */
int hbcsf_mttkrp_f64(const hbcsf_tensor *t, int mode, int rank, const double *const *factors,
                     double *out, void *hip_stream);

int hbcsf_get_stats(const hbcsf_tensor *t, int mode, hbcsf_stats *stats);

/* Read-only view of one host-side format array of a mode, for inspection and tests.
 * array ids: HBCSF_ARR_*; `group` 0 = COO, 1 = CSL, 2 = CSF; `level` 0 = root .. order-1 = leaf.
 * Returns HBCSF_EINVAL for an array the group does not have.  *count is in elements
 * (uint32 or float). */
#define HBCSF_ARR_IND        0 /* uint32: index array of `level` (per slice / segment / nonzero) */
#define HBCSF_ARR_PTR        1 /* uint32: start of each slice / segment in the group's nonzero
                                  stream, n+1 entries (levels above the leaf of CSF; level 0 of CSL) */
#define HBCSF_ARR_VAL        2 /* float : values in stream order                                 */
#define HBCSF_ARR_RUNFIRST   3 /* uint32: slice / segment holding the first nonzero of each run,
                                  runs+1 entries                                                  */
#define HBCSF_ARR_OWNED_BITS 4 /* uint32 bitmap over output rows: 1 = written by one plain store */
#define HBCSF_ARR_COO_BITS   5 /* uint32 bitmap over output rows: 1 = row of a COO-group slice    */
#define HBCSF_ARR_COO_PTR    6 /* uint32: COO-group nonzeros before each 32-row word, words+1     */
int hbcsf_host_array(const hbcsf_tensor *t, int mode, int group, int level, int array_id,
                     const void **ptr, uint64_t *count);

/* Tuning knobs that need no rebuild.  key: HBCSF_TUNE_*. */
#define HBCSF_TUNE_SLICE_THRESHOLD 0 /* T_s, nonzeros per wavefront span; 0 = automatic */
#define HBCSF_TUNE_PROFILE         1 /* n > 0: bracket the kernels of each call with HIP events and
                                        keep the last n calls' event sets; 0 = off              */
#define HBCSF_TUNE_WAVES_PER_CU     2 /* wavefront spans launched per compute unit when T_s is
                                        automatic (default 128)                                 */
#define HBCSF_TUNE_STEPS            3 /* gathers a lane group keeps in flight: 4 or 8 (default 8 for
                                        order 3, 4 for order 4; 4 is only available at rank 32)  */
#define HBCSF_TUNE_KERNEL_MASK      4 /* which kernels hbcsf_mttkrp launches: bit0 define, bit1 COO,
                                        bit2 CSL, bit3 CSF (default 15).  For ablation and profiling
                                        only: with bits cleared the output is incomplete.        */
#define HBCSF_TUNE_TRACE_BUFFER     5 /* device address (8-byte aligned) of a caller-owned buffer of
                                        8 * (4 + 4 * capacity) bytes, or 0 = tracing off.  With a
                                        buffer set, every wavefront of the CSL and B-CSF kernels
                                        appends one record {kernel (1 = CSL, 2 = CSF), XCC_ID << 32
                                        | HW_ID, start, end} (four uint64, times from the 100 MHz
                                        wall clock) after word 0, which counts the records.  The
                                        caller zeroes word 0 before a call.  Profiling only.       */
#define HBCSF_TUNE_TRACE_CAPACITY   6 /* records the trace buffer holds; further ones are dropped  */
#define HBCSF_TUNE_PERSISTENT       7 /* 0 (default): one wavefront per span of T_s nonzeros;
                                        1: only resident wavefronts are launched and each XCD's
                                        wavefronts take its spans round-robin                   */
#define HBCSF_TUNE_STREAM_BYTES     8 /* factor matrices of fiber (middle) levels that are at least
                                        this many bytes are gathered with streaming loads, so that
                                        their rows, which are not reused while cached, do not evict
                                        the leaf factor's popular rows from the L2; 0 = never;
                                        default 2^30                                              */
#define HBCSF_TUNE_FUSE_COO         9 /* 1: the rows of COO-group slices are computed and written by
                                        the output-definition pass (their kernel time is then
                                        reported under "define" and the COO kernel is not
                                        launched); 0: separate COO kernel; 2 (default): fused when
                                        the output is at most 64 MiB, where it saves a launch     */
#define HBCSF_TUNE_DENSE_MID        10 /* 1: B-CSF kernel at rank 32, orders 3 and 4 with T_f 32 or 64 (ignored
                                        elsewhere): the factor rows of the fiber levels are gathered once per
                                        block of steps for the whole wavefront (all lanes of each load
                                        instruction busy) into an LDS row cache instead of at the step where a
                                        segment ends.  A measured alternative that lost (fewer load
                                        instructions, but a longer dependent chain per block); 0 (default): off */
int hbcsf_tune(hbcsf_tensor *t, int key, uint64_t value);

/* With HBCSF_TUNE_PROFILE on: milliseconds of the four kernels (define, COO, CSL, CSF; 0 for a
 * kernel that was not launched) of the hbcsf_mttkrp call made `calls_back` profiled calls ago
 * on this handle (0 = the last one).  Waits for that call's last event. */
int hbcsf_kernel_ms(hbcsf_tensor *t, uint32_t calls_back, float ms[4]);

/* ---------------------------------------------------------------------------------------------
 * Format construction on the device (the pre-processing of Sections IV-V, whose cost Section VI-E
 * weighs against the MTTKRP time): the same per-mode HB-CSF arrays as hbcsf_build_format, byte for
 * byte, built from COO arrays that already are in device memory and written straight into the
 * caller's device arena.  Packed coordinates (sum over the modes of ceil(log2(dim)) bits) above
 * 64 bits are sorted in two stable 64-bit passes; above 128 bits (possible at order 5 only) the
 * build is refused with HBCSF_ERANGE and hbcsf_build_format has to be used.  Orders 3 to 5 and
 * every option of hbcsf_opts.
 * ------------------------------------------------------------------------------------------- */

/* Sizes to allocate before hbcsf_build_format_device: arena_bytes is an upper bound over every
 * possible sparsity pattern of nnz nonzeros (the build reports what it used through
 * hbcsf_device_bytes), workspace_bytes is scratch that can be released when the build returns.
 * Needs a HIP device (the sort / scan scratch sizes are queried for it). */
int hbcsf_device_build_bytes(int order, const uint64_t *dims, uint64_t nnz, const hbcsf_opts *opts,
                             uint64_t *arena_bytes, uint64_t *workspace_bytes);

/* As hbcsf_build_format, but inds[m] and vals are device pointers (read only), and the result is
 * resident: the handle can be passed to hbcsf_mttkrp at once; hbcsf_upload must not be called on
 * it.  device_arena / workspace: device memory, 256-byte aligned; the arena is kept by the caller
 * for the handle's lifetime.  Blocking: the host waits for a few counts per mode.  Errors as
 * hbcsf_build_format, plus ENOMEM when the arena or workspace is too small, and EHIP. */
int hbcsf_build_format_device(int order, const uint64_t *dims, uint64_t nnz,
                              const uint32_t *const *inds, const float *vals, const hbcsf_opts *opts,
                              void *device_arena, uint64_t arena_bytes, void *workspace,
                              uint64_t workspace_bytes, void *hip_stream, hbcsf_tensor **out);

/* Moves a resident handle's arrays into another device arena of at least hbcsf_device_bytes
 * (256-byte aligned, not overlapping the old one) and makes the handle use it, e.g. to release the
 * upper-bound arena a device build was given.  Blocking.  The old arena is the caller's again. */
int hbcsf_relocate(hbcsf_tensor *t, void *new_arena, uint64_t bytes, void *hip_stream);

/* Copies the device-resident arrays of a handle built by hbcsf_build_format_device to host
 * memory, after which hbcsf_host_array works on it (inspection and tests).  No effect on modes
 * that already have a host copy. */
int hbcsf_download(hbcsf_tensor *t, void *hip_stream);

/* ---------------------------------------------------------------------------------------------
 * CPD-ALS iteration (Section II-B: Eq. 1 the model, Eq. 2-3 the mode update, Algorithm "CPD-ALS")
 * built around hbcsf_mttkrp.  One iteration updates every factor in turn,
 *     A_n <- MTTKRP_n(X; other factors) * pinv( Hadamard_{m != n} A_m^T A_m ),
 * then leaves all factors with unit-2-norm columns and lambda_r = product over the modes of the
 * r-th column norms (a zero column keeps norm 1).  The MTTKRP, the Gram matrix and the product
 * with the R x R matrix run on the device in fp32 (Gram sums are accumulated in fp64); the
 * R x R algebra (Hadamard products, pseudo-inverse, norms, fit) runs on the host in fp64.
 * ------------------------------------------------------------------------------------------- */
typedef struct hbcsf_als hbcsf_als;

#define HBCSF_ALS_KEEP_GRAMS 1 /* flag: the factors are exactly as this state's previous
                                  hbcsf_als_iteration left them, so their Gram matrices need not
                                  be recomputed (saves order-1 passes over the factors)           */

/* Gram matrix of a tall factor matrix, S = A^T A: the rank x rank matrices whose Hadamard product
 * the mode update of Eq. 3 inverts.  Asynchronous on hip_stream.
 *   a          device [rows][rank] fp32 row-major, 16-byte aligned (rows may be 0: S is all zeros).
 *   rank       8, 16, 32, 64 or 128.
 *   workspace  device, 256-byte aligned: scratch for per-workgroup partial sums (one rank x rank fp64
 *              slot per workgroup).  hbcsf_gram_workspace_bytes gives the size that lets every launch
 *              use its full grid; a smaller buffer (at least rank*rank*8 bytes) is legal and only
 *              lowers the number of workgroups.  Contents on entry are irrelevant; two calls that
 *              overlap in time must not share a workspace.
 *   s          device [rank][rank] fp64, 8-byte aligned, overwritten.
 * Products are formed in fp32 (matrix instructions at rank 32) and summed in fp64; the partial sums
 * are added in a fixed order, so equal inputs give equal bits.  Errors: EINVAL, ENOMEM (workspace
 * smaller than one slot), EHIP. */
int hbcsf_gram_workspace_bytes(int rank, uint64_t *bytes);
int hbcsf_gram(const float *a, uint64_t rows, int rank, void *workspace, uint64_t workspace_bytes,
               double *s, void *hip_stream);

/* hbcsf_gram for callers that cannot allocate device memory (code recorded under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same computation with the partial-sum
 * slots taken from an 8 MiB array the library itself holds in device memory (one copy per device, kept
 * until the process ends) instead of a workspace argument.  The call allocates nothing on the host or the
 * device and only launches kernels on hip_stream; the first call on a device also looks up the array's
 * address there.  a, rows, rank, s, errors: as hbcsf_gram; a rank whose single rank x rank fp64 slot
 * exceeds the array is rejected with HBCSF_EINVAL (none of the supported ranks does: at most 128 KB),
 * and at ranks 64 and 128 fewer workgroups run than with hbcsf_gram's full workspace (256 and 64).
 * All calls on one device share the array: calls that overlap in time on one device race, whatever
 * their streams; calls one after the other need no clearing in between. */
int hbcsf_gram_noalloc(const float *a, uint64_t rows, int rank, double *s, void *hip_stream);

#define HBCSF_ALS_LAZY_NORMALISATION 2 /* flag: the column normalisation that closes an iteration of
                                  Algorithm "CPD-ALS" may be put off: on return factors[m] can hold the
                                  unit-norm factor with column r multiplied by a norm the state remembers
                                  (lambda, the fit and the state's Gram matrices are those of the normalised
                                  factors either way).  At rank 32 the product kernel then also forms the
                                  new factor's Gram matrix, so the MTTKRP result is read once per mode
                                  update instead of twice.  A later call without the flag, or
                                  hbcsf_als_normalise, writes the unit-norm factors.  Use together with
                                  HBCSF_ALS_KEEP_GRAMS on the calls that follow.                        */

/* Device workspace an ALS state needs for this tensor and rank: one [max dim][rank] fp32 matrix
 * for the MTTKRP result, two rank x rank matrices, one [rank] vector per mode and the Gram
 * computation's scratch (hbcsf_gram_workspace_bytes). */
int hbcsf_als_workspace_bytes(const hbcsf_tensor *t, int rank, uint64_t *bytes);

/* Creates an ALS state for an uploaded tensor.  workspace: device memory, 256-byte aligned, at
 * least hbcsf_als_workspace_bytes; the caller owns it and keeps it and the tensor alive and
 * untouched until hbcsf_als_free.  Allocates a few KB of pinned host memory.  rank as for
 * hbcsf_mttkrp.  Errors: EINVAL, ESTATE (tensor not uploaded), ENOMEM (workspace too small),
 * EHIP. */
int hbcsf_als_create(const hbcsf_tensor *t, int rank, void *workspace, uint64_t workspace_bytes,
                     hbcsf_als **out);

/* One iteration.  factors: host array of `order` device pointers, factors[m] = [dims[m]][rank]
 * fp32 row-major, read and overwritten in place (factors[0]'s content on entry is not used, as in
 * the algorithm).  lambda: device [rank] fp32, written; may be null.  fit: host, may be null;
 * receives 1 - ||X - model|| / ||X|| computed from the Gram matrices and the last MTTKRP (the
 * nonzero coordinates are taken to be distinct).  flags: 0 or any of HBCSF_ALS_KEEP_GRAMS,
 * HBCSF_ALS_LAZY_NORMALISATION.
 * Blocking: the host reads an R x R matrix back for every mode, so the call returns after the
 * work on hip_stream has finished.  Two calls on one state must not overlap.  Errors: EINVAL,
 * and whatever hbcsf_mttkrp reports. */
int hbcsf_als_iteration(hbcsf_als *a, float *const *factors, float *lambda, int flags, double *fit,
                        void *hip_stream);

/* Carries out the column normalisation that calls with HBCSF_ALS_LAZY_NORMALISATION put off: every
 * factor whose columns still carry a remembered norm is scaled in place (one pass each), after which
 * factors[m] are the unit-norm factors that match the last lambda.  factors: as left by the last
 * hbcsf_als_iteration on this state.  Blocking.  No effect when nothing is pending. */
int hbcsf_als_normalise(hbcsf_als *a, float *const *factors, void *hip_stream);

/* The algorithm's outer loop: iterations until the fit changes by less than `tolerance` between two
 * consecutive iterations, or `max_iterations` (>= 1) are done.  The first iteration computes the
 * factors' Gram matrices, the later ones carry them over; the normalisation is put off inside the loop
 * and carried out once at its end.  iterations_done, fit: host, may be null.
 * Other arguments and errors as hbcsf_als_iteration. */
int hbcsf_als_run(hbcsf_als *a, float *const *factors, float *lambda, int max_iterations,
                  double tolerance, int *iterations_done, double *fit, void *hip_stream);

/* Device/host time of the last iteration, summed over the modes, in milliseconds: ms[0] MTTKRP,
 * ms[1] Gram kernel with its read-back, ms[2] host R x R algebra, ms[3] product kernel with its
 * R x R upload. */
int hbcsf_als_phase_ms(const hbcsf_als *a, float ms[4]);

/* Host only (no device call): the pseudo-inverse the mode update applies to the Hadamard product of
 * Gram matrices (Eq. 3).  v, out: host [n][n] fp64, v symmetric, 1 <= n <= 128.  A safely positive
 * definite v is inverted by Cholesky factorisation; otherwise eigenvalues below 1e-15 of the largest
 * magnitude are treated as zero. */
int hbcsf_sym_pinv(const double *v, int n, double *out);

/* Releases the state (not the workspace, not the tensor). */
void hbcsf_als_free(hbcsf_als *a);

/* Diagnostic, not part of the MTTKRP path: launches a kernel that only gathers rows of 32 floats
 * (128 bytes, the R = 32 factor row) with the B-CSF kernel's lane mapping (8 lanes per row, 8 rows
 * per wavefront-level load instruction, 8 such instructions in flight) and discards them, so that
 * the row-gather rate the memory system sustains can be put beside the kernels' rates.
 *   idx        device [n] row numbers, each < table_rows (the caller guarantees this; n >= 65536).
 *   table      device [table_rows][32] floats.     sink  device, at least 4 bytes.
 *   active_lane_groups  1..8: how many of a wavefront's 8 lane groups take part in each load
 *              instruction (8: every lane loads; fewer: the B-CSF kernel's fiber-row loads, which
 *              only the lane groups whose segment ends at that step execute).  The entries of idx
 *              that fall to a lane group sitting an instruction out are skipped.
 *   rows_gathered      host, receives the number of rows the launch gathers (<= n).
 *   load_instructions  host or NULL, receives the wavefront-level row-load instructions issued.
 * Asynchronous on hip_stream; the caller times it. */
int hbcsf_probe_row_gather(const uint32_t *idx, uint64_t n, const float *table, uint64_t table_rows,
                           int active_lane_groups, float *sink, void *hip_stream, uint64_t *rows_gathered,
                           uint64_t *load_instructions);

void hbcsf_free(hbcsf_tensor *t);

const char *hbcsf_strerror(int code);
const char *hbcsf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HBCSF_H_ */
