/*
 * tperm -- out-of-place rank-n dense tensor transpose for AMD MI355X (gfx950).
 *
 * Computes B[perm(i)] = A[i]: the element of the input tensor A with multi-index
 * (y_0, .., y_{n-1}) is stored in the output tensor B at multi-index
 * (y_{perm[0]}, .., y_{perm[n-1]}).  This is the tensor transpose of Section 2 of the
 * paper (scalar position, its inverse, and Eq. (1)), restated 0-based:
 *
 *   - dims[0] is the stride-1 dimension; later dimensions are more senior;
 *   - perm[j] is the INPUT dimension found at OUTPUT position j (the paper's
 *     w_{j+1} - 1), so the output extents are dims[perm[j]];
 *   - elements are 4 or 8 bytes wide and are moved as raw bits.
 *
 * The interface is the create-plan / execute / destroy triple the paper describes for
 * its library (Section 2.3): a plan is made once from (rank, extents, permutation),
 * then executed any number of times.
 *
 * Plan creation and inspection are pure host code and need no GPU.  tperm_execute
 * enqueues work on a HIP stream; `in` and `out` are DEVICE pointers owned by the
 * caller.  The library keeps no reference to them.  No function throws or aborts:
 * every failure is reported through the returned status.
 */
#ifndef TPERM_H
#define TPERM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TPERM_MAX_RANK 16

typedef struct tperm_plan_s *tperm_plan_t; /* opaque; created and freed by the library */

typedef enum {
    TPERM_OK = 0,
    TPERM_ERR_NULL = 1,      /* a required pointer argument is NULL                       */
    TPERM_ERR_RANK = 2,      /* rank outside [1, TPERM_MAX_RANK]                          */
    TPERM_ERR_DIMS = 3,      /* an extent is < 1                                          */
    TPERM_ERR_PERM = 4,      /* perm is not a permutation of 0..rank-1                    */
    TPERM_ERR_ELEM_SIZE = 5, /* element size is not 4 or 8                                */
    TPERM_ERR_TOO_LARGE = 6, /* volume >= 2^31 elements                                   */
    TPERM_ERR_ALIAS = 7,     /* in == out (the transpose is out-of-place)                 */
    TPERM_ERR_ALIGN = 8,     /* a data pointer is not a multiple of the element size      */
    TPERM_ERR_HIP = 9,       /* a HIP call failed (no device, launch error)               */
    TPERM_ERR_NOMEM = 10,    /* host allocation failed                                    */
    TPERM_ERR_KERNEL = 11,   /* the forced kernel class / options cannot run this problem */
    TPERM_ERR_INTERNAL = 12  /* self-check of a plan's index maps failed                  */
} tperm_status_t;

/* Kernel classes the plan selector chooses between (Section 2.3 lists the paper's:
 * Tiled, TiledCopy, Packed, PackedSplit; the trivial permutation is a plain copy). */
typedef enum {
    TPERM_KERNEL_AUTO = 0,
    TPERM_KERNEL_COPY = 1,    /* canonical permutation is the identity: out[i] = in[i]        */
    TPERM_KERNEL_ROWCOPY = 2, /* leading dimension stays first and is long: rows are moved,    */
                              /* no LDS stage (the paper's TiledCopy)                          */
    TPERM_KERNEL_TILED = 3,   /* 2-D tile over (input dim 0, output dim 0) staged in LDS       */
    TPERM_KERNEL_PACKED = 4,  /* several leading input/output dims packed into one LDS tile,   */
                              /* the last one on each side possibly split (Packed/PackedSplit) */
    TPERM_KERNEL_NAIVE = 5    /* one thread per output element, no staging (debug anchor)      */
} tperm_kernel_class_t;

/* What a plan decided.  Canonical = after dropping extent-1 dims and fusing input dims
 * that stay adjacent and in order in the output. */
typedef struct {
    int kernel_class;                      /* tperm_kernel_class_t actually chosen          */
    int elem_size;
    int rank;                              /* as given                                      */
    int canon_rank;
    int64_t canon_dims[TPERM_MAX_RANK];
    int canon_perm[TPERM_MAX_RANK];
    int64_t volume;
    int64_t tile_extent[TPERM_MAX_RANK];   /* per canonical dim; 1 = not in the tile        */
    int64_t tile_volume;                   /* elements staged per tile                      */
    int64_t run_in;                        /* contiguous input run per tile, elements       */
    int64_t run_out;                       /* contiguous output run per tile, elements      */
    int64_t num_tiles;
    int m, k;
    int nreg;                              /* elements each thread moves per tile           */
    int threads;                           /* threads per workgroup                         */
    int lds_bytes;
    int lds_pad;
    double score;                          /* selector's estimate (relative, lower = better)*/
    int blocks_per_cu;                     /* cap on resident workgroups per CU (0 = none)  */
    int cache_policy;                      /* policy of the kernel variant tperm_execute    *
                                            * launches when `out` is 32-byte aligned:       *
                                            * 1 = cached, 2 = nontemporal loads and stores, *
                                            * 3 = nontemporal stores, 4 = nontemporal loads *
                                            * (from any other `out` the stores are cached:  *
                                            * 2 runs as 4, 3 as 1); accumulation is cached   */
    int align_out;                         /* 1 if the plan writes line-aligned windows     */
    int paired;                            /* 1: a 4-byte problem whose stride-1 dimension  *
                                            * stays in front and has an even extent is run  *
                                            * as the 8-byte problem with that extent halved *
                                            * (same bytes, half the memory instructions).   *
                                            * elem_size, volume and every extent above then *
                                            * describe the 8-byte problem.  Used by         *
                                            * tperm_execute when both pointers are 8-byte   *
                                            * aligned; otherwise, and for accumulation, the *
                                            * plan's unpaired twin runs.                    */
    int loads_first;                       /* 1: next-tile loads are issued before stores   */
    int vec2;                              /* 1: a 4-byte plan that reads two neighbours    *
                                            * along input dim 0 and writes two neighbours   *
                                            * along output dim 0 with single 8-byte         *
                                            * accesses (even extents and tile extents       *
                                            * along both); nreg counts pairs per thread.      *
                                            * Used by tperm_execute when both pointers are  *
                                            * 8-byte aligned; otherwise, and for            *
                                            * accumulation, the plan's plain twin runs.     *
                                            * Together with align_out: pairs inside the     *
                                            * line-aligned windows (even tile extent along  *
                                            * input dim 0, any extents, any element-aligned *
                                            * pointers; odd row ends and clipped windows    *
                                            * move single elements).                         */
    int large;                             /* 1: a tensor of 4 GiB or more (or a plan made  *
                                            * to run like one): byte offsets no longer fit  *
                                            * 32 bits, so every tile addresses its pieces   *
                                            * from its own origin; LDS-staged tiles of 256  *
                                            * threads in all their forms, or the gather     *
                                            * kernel when no tile fits.                     */
    int reserved[1];
} tperm_plan_info_t;

/* Create a plan: the first call of the create / execute / destroy triple of Section 2.3.  The
 * plan selector validates the problem, brings it to canonical form and chooses a kernel class
 * and a tile with its cost estimate (the paper's heuristic selection, Section 2.3; its
 * classes are those of Section 2.2).  dims[rank] and perm[rank] are host arrays, copied; the
 * caller keeps ownership.  elem_size is in bytes (4 or 8, the two widths of Section 3).  Host
 * only.  Tensors of up to 2^31 - 1 elements are accepted (element indices are 31-bit, as the
 * int indices of Algorithm 1); those of 4 GiB and more run a form of the tile kernels that
 * addresses every tile from its own origin (large in tperm_plan_info_t).  On failure *plan is
 * set to NULL and the status says why: NULL (plan, dims or perm), RANK, DIMS, PERM, ELEM_SIZE,
 * TOO_LARGE, NOMEM. */
tperm_status_t tperm_plan_create(tperm_plan_t *plan, int rank, const int64_t *dims,
                                 const int *perm, size_t elem_size);

/* The same with the kernel class chosen by the caller instead of the selector (Section 2.2's
 * classes run side by side on one problem: tests, comparisons); the tile inside the class is
 * still the selector's best.  kernel_class is a tperm_kernel_class_t; TPERM_KERNEL_AUTO
 * behaves as tperm_plan_create.  A class that cannot legally run the problem (a plain copy for
 * a real permutation, a row copy when the stride-1 dimension moves, ...) gives
 * TPERM_ERR_KERNEL. */
tperm_status_t tperm_plan_create_forced(tperm_plan_t *plan, int rank, const int64_t *dims,
                                        const int *perm, size_t elem_size, int kernel_class);

/* Measurement-based plan selection (Section 2.3: all feasible plans are created and run once,
 * the fastest is kept): every candidate plan the selector enumerates is executed on (in, out)
 * on `hip_stream` and timed with HIP events; the fastest is kept.  in/out are device buffers of at least volume*elem_size bytes; out is
 * overwritten.  Synchronises the stream.  max_candidates <= 0 means all.  The candidates
 * are timed back to back on these buffers as they are: a tensor small enough to stay in the
 * last-level cache is timed cache-hot, which need not rank the plans as HBM-resident data
 * would. */
tperm_status_t tperm_plan_create_measured(tperm_plan_t *plan, int rank, const int64_t *dims,
                                          const int *perm, size_t elem_size, const void *in,
                                          void *out, void *hip_stream, int max_candidates);

/* The same, timed as the data would arrive from HBM: `scratch` is caller-owned device memory
 * (16-byte aligned, not overlapping in or out: TPERM_ERR_ALIGN / TPERM_ERR_ALIAS) of
 * scratch_bytes bytes, ideally twice the last-level cache (512 MiB on MI355X).  Before every
 * timed execution the library copies one half of it onto the other, outside the timed
 * interval, which pushes the tensors out of the caches; its contents are overwritten.
 * scratch == NULL behaves as tperm_plan_create_measured.  Use it for tensors that fit the
 * last-level cache and will not be cache-resident when the plan is used.  Each candidate's
 * fastest of five such runs counts.  (Kernels of a few tens of microseconds timed one by one
 * still need not rank as they do inside a pipeline of launches.) */
tperm_status_t tperm_plan_create_measured_cold(tperm_plan_t *plan, int rank, const int64_t *dims,
                                               const int *perm, size_t elem_size, const void *in,
                                               void *out, void *hip_stream, int max_candidates,
                                               void *scratch, size_t scratch_bytes);

/* Execute: the second call of the triple of Section 2.3.  Performs the transpose of Section 2
 * (Eq. (1)) with the plan's kernel: enqueues it on hip_stream (a hipStream_t; NULL = the
 * default stream) and returns without synchronising.  in: DEVICE pointer to volume*elem_size
 * bytes, read only.  out: DEVICE pointer to volume*elem_size bytes, fully overwritten; must not
 * overlap in.  Both stay owned by the caller and need only be aligned to the element size.  A
 * plan is immutable: concurrent executes on several streams are allowed.  Statuses: NULL,
 * ALIAS (in == out or overlapping ranges), ALIGN, HIP (no device, launch failure); no device
 * memory is allocated or freed. */
tperm_status_t tperm_execute(tperm_plan_t plan, const void *in, void *out, void *hip_stream);

/* Accumulating variant (the mode the paper uses for its third benchmark set, Section 3.3:
 * read input, read output, add, write output): out = out + transpose(in), where the
 * elements are IEEE binary32 (elem_size 4) or binary64 (elem_size 8) numbers and each output
 * element receives exactly one addition.  Same argument rules as tperm_execute; three
 * memory operations per element instead of two. */
tperm_status_t tperm_execute_accumulate(tperm_plan_t plan, const void *in, void *out,
                                        void *hip_stream);

/* Self-checking execute.  Section 2 defines the transpose as a one-to-one map of scalar
 * positions (Eq. (1)): every input element lands at exactly one output position and nothing
 * else is written, so the output holds the same multiset of element words as the input.  This
 * call performs tperm_execute and then checks that invariant on the device: three
 * order-independent 64-bit digests of the element words (sum, exclusive-or, sum of a scrambled
 * image) are formed for both tensors and compared.  It catches lost, duplicated or altered
 * elements; it cannot see elements that merely sit at wrong positions.
 *
 * verdict: DEVICE pointer, 8-byte aligned, to one 64-bit word owned by the caller; it is
 * written by the last kernel of the call: 0 = the digests agree, otherwise a bit mask of the
 * digests that differ.  Nothing is synchronised: read it after the stream has caught up.
 * workspace: caller-owned DEVICE memory, 8-byte aligned, of workspace_bytes >=
 * TPERM_VERIFY_WORKSPACE_BYTES(volume) bytes, holding the partial digests; it needs no
 * initialisation, its contents are overwritten, and it must not overlap in, out or verdict.
 * Two calls that use the same workspace at the same time race.  The call costs one more read
 * of both tensors.  Statuses: those of tperm_execute, TPERM_ERR_NULL (verdict, workspace),
 * TPERM_ERR_ALIGN (verdict or workspace not 8-byte aligned), TPERM_ERR_TOO_LARGE (workspace
 * too small for this plan's tensor; nothing is launched). */
#define TPERM_VERIFY_CHUNK_ELEMS 16384
#define TPERM_VERIFY_WORKSPACE_BYTES(volume) \
    ((size_t)64 * (size_t)(((volume) + TPERM_VERIFY_CHUNK_ELEMS - 1) / TPERM_VERIFY_CHUNK_ELEMS))
tperm_status_t tperm_execute_verified(tperm_plan_t plan, const void *in, void *out,
                                      void *hip_stream, uint64_t *verdict, void *workspace,
                                      size_t workspace_bytes);

/* tperm_execute_verified for callers that cannot allocate device memory or hand over a
 * workspace: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The partial digests go to a 512 KiB array that the library holds in the device
 * memory of every GPU it runs on, from the time its code is loaded there until the process
 * ends; the call allocates and frees nothing, on the host or on the device, and enqueues
 * kernels only (no memset, no copy).  Same arguments, result and statuses as
 * tperm_execute_verified, except:
 *   - the array is sized for tensors of up to 2^27 elements (TPERM_VERIFY_STATIC_MAX_ELEMS); a
 *     plan with a larger volume gives TPERM_ERR_TOO_LARGE and nothing is launched (use the
 *     workspace form for those);
 *   - all calls on one GPU share that GPU's array, whatever the stream or the plan: two calls
 *     that are in flight on one GPU at the same time race on it and may report a wrong verdict
 *     (the transposed tensor itself is unaffected).  Order them on one stream, or use the
 *     workspace form.  The array keeps the last call's partial results; nothing in it needs
 *     clearing, since a call reads only what it has written itself;
 *   - the first call on a GPU looks up the array's device address (the only set-up there is);
 *     make that call outside stream capture. */
#define TPERM_VERIFY_STATIC_MAX_ELEMS ((int64_t)1 << 27)
tperm_status_t tperm_execute_verified_static(tperm_plan_t plan, const void *in, void *out,
                                             void *hip_stream, uint64_t *verdict);

/* What the selector decided for this plan (Section 2.3: kernel class, tile, launch shape),
 * written to *info, which the caller owns.  Host only.  NULL plan or info: TPERM_ERR_NULL. */
tperm_status_t tperm_plan_describe(tperm_plan_t plan, tperm_plan_info_t *info);

/* Destroy: the third call of the triple of Section 2.3.  Frees the plan's host memory (a plan
 * owns no device memory).  The caller must not destroy a plan whose launches have not been
 * enqueued yet on another thread; launches already enqueued are unaffected (the descriptor
 * travels with each launch).  NULL: TPERM_ERR_NULL. */
tperm_status_t tperm_plan_destroy(tperm_plan_t plan);

/* Static, NUL-terminated description of a status code (the error reporting that the paper's
 * interface of Section 2.3 leaves open); never NULL, "unknown status" for other values. */
const char *tperm_status_string(tperm_status_t s);

/*
 * One-call interface over a process-wide plan cache.
 *
 * Section 2.3 separates plan creation from execution because choosing a plan costs far more
 * than running it once, measurement-based choice most of all; a caller that meets the same
 * problem repeatedly therefore keeps its plans.  These entry points do that keeping: the
 * cache maps (rank, dims, perm, elem_size), exactly as given, to a plan the library owns.
 * It is thread-safe, holds at most 4096 plans (least recently used goes first) and lives
 * until the process ends or tperm_cache_clear is called.
 *
 * tperm_transpose / tperm_transpose_accumulate: look the problem up, create the heuristic
 * plan on a miss, then behave as tperm_execute / tperm_execute_accumulate on that plan
 * (same pointer rules, same statuses; plan-creation statuses on a miss).
 *
 * tperm_cache_tune: runs measurement-based selection (as tperm_plan_create_measured, all
 * candidates; `out` is overwritten, the stream is synchronised) and installs the winner for
 * the problem, replacing any cached plan.
 *
 * tperm_cache_stats: any of the three result pointers may be NULL.  hits and misses count
 * lookups by the transpose calls since the last clear.
 */
tperm_status_t tperm_transpose(int rank, const int64_t *dims, const int *perm, size_t elem_size,
                               const void *in, void *out, void *hip_stream);
tperm_status_t tperm_transpose_accumulate(int rank, const int64_t *dims, const int *perm,
                                          size_t elem_size, const void *in, void *out,
                                          void *hip_stream);
tperm_status_t tperm_cache_tune(int rank, const int64_t *dims, const int *perm, size_t elem_size,
                                const void *in, void *out, void *hip_stream);
tperm_status_t tperm_cache_stats(int64_t *entries, int64_t *hits, int64_t *misses);
tperm_status_t tperm_cache_clear(void);

/* Plain device-to-device copy of nbytes with the library's copy kernel: the measured bandwidth
 * ceiling the transposes are compared with, in the way Section 3 normalises by a STREAM
 * figure.  in / out: DEVICE pointers, 4-byte aligned, nbytes a multiple of 4 (ALIGN otherwise),
 * not equal (ALIAS); asynchronous on hip_stream. */
tperm_status_t tperm_copy_bytes(const void *in, void *out, size_t nbytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TPERM_H */
