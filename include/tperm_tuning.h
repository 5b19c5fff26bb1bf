/*
 * tperm -- tuning and test interface.
 *
 * Everything a sweep, a test or a tuning tool needs beyond the product boundary of tperm.h:
 * plan creation with explicit overrides of every choice the selector makes (Section 2.2's
 * kernel classes and tiles, and the launch details this implementation adds), the list of
 * candidate plans behind Section 2.3's "create every feasible plan, keep one", and a host-side
 * evaluation of a plan's index maps (Eqs. (2)-(6) as the kernel computes them).  Nothing here
 * is needed to transpose a tensor; the layout of tperm_plan_opts_t may grow between versions.
 */
#ifndef TPERM_TUNING_H
#define TPERM_TUNING_H

#include "tperm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Optional overrides for plan creation.  Zero-initialise; 0 always means "let the
 * selector decide". */
typedef struct {
    int kernel_class;   /* tperm_kernel_class_t                                              */
    int m;              /* number of leading INPUT dims (canonical) taken into the tile      */
    int64_t tile_in;    /* tile extent of the last of those m dims (0 = full extent)         */
    int k;              /* number of leading OUTPUT dims (canonical) taken into the tile     */
    int64_t tile_out;   /* tile extent of the last of those k dims (0 = full extent)         */
    int lds_pad;        /* -1 = search; >= 0 forces the LDS row padding (elements)           */
    int grid_mode;      /* 0 = default; -1 = tiles in launch order; 1 = one contiguous tile   */
                        /* range per XCD; 2 + g = groups of 2^g consecutive tiles dealt to    */
                        /* the XCDs in turn                                                   */
    int blocks_per_cu;  /* > 0 caps the resident workgroups per compute unit                 */
    int cache_policy;   /* 0 = selector's default; 1 = cached; 2 = nontemporal loads and stores; */
                        /* 3 = nontemporal stores only; 4 = nontemporal loads only            */
    int window_in;      /* tiles in flight are grouped into windows of this many neighbours   */
    int window_out;     /* on the input / output side; 1 = no window; 0 = default (none on    */
                        /* the output side; on the input side only a few ragged chunks of the */
                        /* input run are kept together)                                       */
    int threads;        /* workgroup size of the tile kernel: 0 = default, 64 or 256          */
    int lds_buffers;    /* 0 = default; 1 or 2 LDS images (2: one barrier per tile)           */
    int align_out;      /* line-aligned output windows (tiles read a one-line halo along the  *
                         * output's leading dim, every row writes a window shifted to whole  *
                         * 128-byte lines): 0 = the selector decides, 1 = off, 2 = on where   *
                         * the tile allows it (k = 1, tile_out a multiple of one line)        */
    int tile_order;     /* 0 = default, 1 = input-major, 2 = output-major walk over the tiles */
    int loads_first;    /* order in which a workgroup issues the next tile's loads and this  *
                         * tile's stores: 0 = selector's default; 1 = stores first; 2 = loads *
                         * first                                                              */
    int vec2;           /* transposing 4-byte plans with 8-byte global accesses (vec2 in      *
                         * tperm_plan_info_t): 0 = default (a twin plan is kept for 8-byte aligned       *
                         * pointers), 1 = off, 2 = in this plan itself where the shape       *
                         * allows, which then requires 8-byte aligned pointers (except with  *
                         * line-aligned output windows, which form their pairs on absolute  *
                         * addresses and take any element-aligned pointer)                   */
    int pair_elems;     /* moving two 4-byte elements as one 8-byte unit (paired in plan info): *
                         * 0 = default (on when no class or tile is forced), 1 = off, 2 = on   */
    int selector;       /* how the tile is chosen when none is forced: 0 = the fitted cost      *
                         * estimate (default); 1 = the analytical model of tperm_plan_model,    *
                         * evaluated on the best-scored candidates (slower plan creation)       */
    int large;          /* 1 = plan and run the tensor the way tensors of 4 GiB and more are     *
                         * (large in tperm_plan_info_t), whatever its size: the form can then   *
                         * be checked on tensors a test can afford; 0 = by size.  Such plans     *
                         * ignore threads and loads_first                                        */
} tperm_plan_opts_t;

/* tperm_plan_create with overrides.  opts may be NULL (then it is tperm_plan_create).  A
 * kernel class or tile that cannot legally run the problem gives TPERM_ERR_KERNEL.  Host only;
 * opts is read during the call and not kept. */
tperm_status_t tperm_plan_create_ex(tperm_plan_t *plan, int rank, const int64_t *dims,
                                    const int *perm, size_t elem_size,
                                    const tperm_plan_opts_t *opts);

/* Enumeration of the feasible staged plans (Section 2.3: every plan that can run is
 * created, then one is kept).  tperm_plan_candidate_count returns how many tile candidates
 * the selector sees for the problem, best estimate first; tperm_plan_create_candidate
 * builds the plan for candidate `index` (TPERM_ERR_KERNEL if out of range).  Host only.
 * Problems whose canonical form is a copy have no candidates. */
tperm_status_t tperm_plan_candidate_count(int rank, const int64_t *dims, const int *perm,
                                          size_t elem_size, int *count);
tperm_status_t tperm_plan_create_candidate(tperm_plan_t *plan, int rank, const int64_t *dims,
                                           const int *perm, size_t elem_size, int index);

/* Host-only self check of a plan's index arithmetic: runs, on the CPU, the very offset
 * computations the kernel performs (tile enumeration, major/minor offsets, LDS slots,
 * edge masks) and records, for every output scalar position o, the input scalar position
 * whose element the kernel would store there.  out_to_in has volume entries; entries
 * never written are -1.  Returns TPERM_ERR_INTERNAL if an output position is written
 * twice, an LDS slot is read before it is written, or an offset leaves the tensor.
 * Moves no tensor data; meant for volumes small enough to enumerate.  For a paired plan
 * (see tperm_plan_info_t.paired) the map evaluated is that of the 8-byte twin, written out
 * per 4-byte element. */
tperm_status_t tperm_plan_index_map(tperm_plan_t plan, int64_t *out_to_in);

/* Analytical run-time estimate of a plan, after Section 2.3 (Eqs. (10)-(13)): the MWP-CWP form
 * cycles = (cycles_mem + cycles_shmem + cycles_ac) * N_iter, with the memory latency driven by
 * the transactions per request and stores to partially written lines counted double (Eq. (13)),
 * re-derived for MI355X: 128-byte lines, 64-lane waves that keep all their requests in flight,
 * 256 compute units, 8 TB/s, latencies and departure delay as measured on the chip by pointer
 * chasing (the counterpart of the paper's Table I).  The transaction counts are exact per tile:
 * up to 16 tiles spread over the tile index are walked on the host with the kernel's own index
 * arithmetic and every touched line is tallied; the per-tile figures below are the sample's
 * counts per useful byte times the bytes an average tile index carries (volume * element size /
 * tiles), so they are averages over all tiles, ragged ones in their true proportion.
 * Host only; plans of the copy and naive classes give TPERM_ERR_KERNEL. */
typedef struct {
    double ld_tran, st_tran;       /* distinct 128-byte lines read / written per tile            */
    double ld_req, st_req;         /* wave-wide load / store instructions per tile               */
    double cl_full, cl_part;       /* written lines that receive all 128 bytes / fewer           */
    double ld_runs, st_runs;       /* separate runs of consecutive lines read / written per tile *
                                    * (reported; Eq. (13) has no term for them)                  */
    double tpr_mem;                /* transactions per request, Eq. (13)                         */
    double mem_lat;                /* cycles: base latency + (tpr_mem - 1) * departure delay     */
    double mlp;                    /* independent requests per wave and tile (slots per thread)  */
    double mwp;                    /* requests that overlap within one memory latency            */
    double tpr_lds;                /* LDS passes per wave-wide LDS access (bank conflicts)       */
    double cycles_mem, cycles_lds, cycles_ac; /* per iteration of a compute unit, Eq. (10), (11) */
    double n_iter;                 /* iterations: tiles / (compute units * resident workgroups)  */
    double cycles_total;
    double microseconds;           /* cycles_total at 2.4 GHz                                    */
    double useful_bytes_per_tile;  /* bytes an average tile writes (= reads): volume * E / tiles  */
} tperm_model_t;
tperm_status_t tperm_plan_model(tperm_plan_t plan, tperm_model_t *model);

/* What the current HIP device reports about itself, for the benchmark's record next to the
 * vendor's 8 TB/s figure that Section 3's STREAM-style normalisation is replaced by here: memory
 * bus width in bits, peak memory clock in kHz, compute units.  Any pointer may be NULL.
 * TPERM_ERR_HIP without a device. */
tperm_status_t tperm_device_memory_info(int *bus_width_bits, int *memory_clock_khz, int *compute_units);

/* The checking step of tperm_execute_verified on its own, for tests: compares the multisets of
 * the `count` words of elem_size (4 or 8) bytes at a and at b (DEVICE pointers aligned to the
 * word size; they may be equal).  verdict, workspace and workspace_bytes as for
 * tperm_execute_verified, with `count` in place of the volume.  Asynchronous on hip_stream. */
tperm_status_t tperm_multiset_compare(const void *a, const void *b, int64_t count, size_t elem_size,
                                      uint64_t *verdict, void *workspace, size_t workspace_bytes,
                                      void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TPERM_TUNING_H */
