/*
 * snap.h -- C ABI of the MI355X (gfx950) local solver: asynchronous stochastic coordinate descent
 * (SCD) for generalized linear models, the GPU-resident solver of Snap ML (arXiv 1803.06333,
 * Section 3.1), with the double-buffered data streaming of Section 3.2.
 *
 * Problem (paper eq. (1)):  min_alpha f(A alpha) + sum_i g_i(alpha_i),  shared vector v = A alpha.
 * With X the n_rows x n_cols example matrix, labels y and lambda > 0 the library minimises
 *
 *      P(w) = (1/n) sum_i loss(y_i, x_i.w) + (lambda/2) ||w||^2
 *
 *   primal form (CSC or dense column-major; ridge, logistic): coordinates = columns, model w,
 *                v = X w (length n_rows);
 *   dual form   (CSR; hinge, logistic): coordinates = rows, model alpha in [0,1]^n,
 *                v = X^T (y o alpha) (length n_cols), w = v / (lambda n).  Hinge: closed-form step
 *                clipped to [0,1], start alpha = 0.  Logistic (Section 3.1: a single Newton step
 *                from the previous value): D(alpha) = -(1/n) sum [alpha ln alpha + (1-alpha)
 *                ln(1-alpha)] - (lambda/2)||w||^2, start alpha = 1/2, iterates kept in
 *                [2^-20, 1 - 2^-20] (snap_set_model clips to that range).
 *
 * One coordinate update = gather-dot of the coordinate's nonzeros with v, a scalar step (closed
 * form for ridge and the clipped hinge dual, one Newton step for logistic), and an atomic scatter
 * of delta * a_j into v; an epoch visits every coordinate once in the order of a seeded
 * permutation with many coordinates in flight.
 *
 * Conventions
 *  - Every function returns SNAP_OK (0) or a negative SNAP_E* code; snap_last_error() gives a
 *    thread-local message.  Nothing aborts or throws across this boundary.
 *  - All pointers in snap_matrix live in ONE memory space, named by `mem`.  In resident mode the
 *    library copies matrix and labels during snap_create (the caller may free them afterwards).
 *    In streaming mode (device_budget_bytes > 0 and the matrix larger than the budget) the matrix
 *    arrays must be SNAP_MEM_HOST_PINNED and are BORROWED until snap_destroy.
 *  - Index arrays: ptr is int64[major+1] (absolute offsets, ptr[0] == 0), idx is int32[nnz] with
 *    0 <= idx < minor, val is fp32[nnz].  For snap_create, val = NULL with a compressed layout means
 *    pattern-only data: every stored value is 1 (one-hot encodings; no value array has to be kept
 *    in pinned memory or copied).  Dense: val only, n_rows*n_cols fp32, column-major
 *    (element (i,j) at val[j*n_rows+i]) or row-major (val[i*n_cols+j]); ptr = idx = NULL.
 *  - Labels y: fp32[n_rows], in the same memory space as the matrix; logistic and hinge need
 *    y in {-1,+1}.
 *  - Output buffers of snap_get_* are HOST pointers, caller allocated.  snap_predict writes to a
 *    buffer in the memory space of its matrix argument.
 *  - snap_epoch works on the handle's compute stream; the query functions synchronise that
 *    stream.  One handle must not be used from two threads at once.  Device arrays handed to
 *    snap_create or snap_predict are read on that stream: work of the caller's own streams that
 *    writes them must be complete before the call.
 */
#ifndef SNAP_H
#define SNAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct snap_handle snap_handle; /* opaque, owned by the library */

enum { SNAP_CSR = 0, SNAP_CSC = 1, SNAP_DENSE_ROWMAJOR = 2, SNAP_DENSE_COLMAJOR = 3 };
enum { SNAP_RIDGE = 0, SNAP_LOGISTIC = 1, SNAP_HINGE = 2 };
enum { SNAP_FORM_AUTO = 0, SNAP_PRIMAL = 1, SNAP_DUAL = 2 }; /* AUTO: CSC/dense -> primal, CSR -> dual */
enum { SNAP_MEM_HOST = 0, SNAP_MEM_HOST_PINNED = 1, SNAP_MEM_DEVICE = 2 };
enum {
    SNAP_OK = 0,
    SNAP_EINVAL = -1,       /* bad argument (null pointer, negative size, inconsistent ptr array...) */
    SNAP_EUNSUPPORTED = -2, /* (loss, form, layout) combination that is not implemented */
    SNAP_ENOMEM = -3,       /* host or device allocation failed */
    SNAP_EHIP = -4,         /* a HIP runtime call failed */
    SNAP_ESTATE = -5        /* a kernel reported an internal failure (bounded wait expired) */
};

typedef struct {
    int layout;            /* SNAP_CSR ... */
    int mem;               /* SNAP_MEM_* of ptr, idx, val (and of y / out that accompany it) */
    int64_t n_rows, n_cols, nnz;
    const int64_t *ptr;
    const int32_t *idx;
    const float *val;
} snap_matrix;

typedef struct {
    int form;                    /* SNAP_FORM_AUTO | SNAP_PRIMAL | SNAP_DUAL */
    size_t device_budget_bytes;  /* 0: keep the matrix resident; else stream it when larger */
    size_t chunk_bytes;          /* streaming chunk size in bytes of idx+val (0: 4 GiB) */
    void *compute_stream;        /* hipStream_t to run on (e.g. PyTorch's), or NULL: the library's compute stream of
                                    the current device (one per device, shared by all handles created this way:
                                    their work is ordered among them) */
    void *copy_stream;           /* hipStream_t for chunk copies, or NULL: the library's copy stream of the device */
    int refresh_v_every;         /* recompute v = A x every this many epochs; 0 = never */
    int profile;                 /* 1: time each epoch's SCD kernels with HIP events; 2: the same, but the group
                                    sweeps time only every fourth row pass, a different one each epoch, and
                                    report the sum scaled up (timing a pass delays the chain of kernels a little) */
    int adaptive;                /* 0: default (on; off with group_bounds), 1: on, 2: off.  On: after every epoch the
                                    objective is evaluated; if it got worse the epoch's updates are
                                    discarded, the number of nonzeros in flight is halved and, once that
                                    is at its floor, the damping is halved (Section 3.1, "Adaptive
                                    Damping").  snap_epoch then waits for the epoch to finish. */
    float damping;               /* initial damping in (0,1]; 0 means 1 (no damping) */
    int64_t max_inflight_nnz;    /* cap on the nonzeros of coordinates in flight at once; 0 = automatic:
                                    a quarter of the length of v, lowered by the adaptive check when an
                                    epoch makes the objective worse; with the check off, a quarter of the
                                    effective length of v, (sum f)^2 / sum f^2 over the access counts f of
                                    the entries of v (dense data: no cap) */
    const int64_t *group_bounds; /* optional (host memory, copied): n_groups+1 increasing coordinate
                                    boundaries, group_bounds[0] = 0, last = number of coordinates, such that
                                    the coordinates INSIDE a group have pairwise disjoint supports (the
                                    columns of one one-hot encoded field).  Verified at creation.  Enables
                                    the exact group-sweep epoch (primal form, sparse, resident): groups are
                                    visited in a random order drawn from perm_seed (keys of the groups
                                    under chunk id 0xFFFFFFFF, sorted), all coordinates of a group at
                                    once -- identical to visiting them one by one, since they do not
                                    interact -- with plain coalesced updates of v instead of atomics.
                                    Resident data: the library holds a row map per group (2 bytes per row, 4
                                    when a group has more than 65535 coordinates; a copy of 1 byte per row for
                                    every group of at most 255, which the sweeps then read instead).
                                    Streamed data (device_budget_bytes exceeded; pattern-only data, i.e. all
                                    values 1): the row maps of the sweeps are built at creation into pinned
                                    host memory of the library's own (groups of up to 65535 coordinates:
                                    prefix-coded, a Huffman code of rank classes that comes within a few percent
                                    of the entropy of the ranks, decoded on the device; wider groups: 4 bytes
                                    per row) and an epoch streams
                                    those through a ring of three device buffers instead of the column indices
                                    (when that pinned memory cannot be had, the sweeps are declined as below).
                                    The sums of the sweeps are fixed point.  Logistic loss: the sweeps are not
                                    used when lambda * n_rows < max|value|^2 / 16 (their resolution could show
                                    in a step); ridge loss: a term a (v - y) of 2^14 or more does not fit, the
                                    epoch that meets one is done again by the asynchronous engine and the
                                    handle stays with it.  In both cases snap_get_chunks then reports one
                                    chunk, and with auto_groups = 1 creation fails instead. */
    int64_t n_groups;            /* 0: no groups */
    double lambda1;              /* >= 0: weight of an l1 term in the primal forms (eq. (1): lasso / elastic-net
                                    regularisers), P(w) = (1/n) sum loss + (lambda/2)||w||^2 + lambda1 ||w||_1.
                                    The step soft-thresholds the minimiser of the quadratic model of the
                                    coordinate problem; exact zeros are kept.  The duality gap is then the
                                    Fenchel form P(w) + f*(u) + sum_j g*(-a_j.u), u = grad f(v),
                                    g*(t) = max(|t| - lambda1, 0)^2 / (2 lambda).  Dual form: must be 0. */
    int dense_tiles;             /* exact tile sweeps for dense column-major ridge regression, resident data
                                    (Section 3.1, dense data): tiles of 128 consecutive columns, visited in a
                                    random order drawn from perm_seed (keys of the tiles under chunk id
                                    0xFFFFFFFF), the columns of a tile in the order of their keys under the
                                    tile's index as chunk id; the steps of a tile are taken one after the
                                    other from inner products corrected with the tile's Gram block, so the
                                    result is the sequential one and v is updated with plain stores.
                                    0: automatic (used whenever it applies), 1: required (error when it does
                                    not apply), 2: off (asynchronous epoch with atomic updates of v).
                                    snap_get_chunks reports the tiles. */
    int auto_groups;             /* without group_bounds (primal form, sparse): look for a partition of
                                    the coordinates into few ranges of consecutive coordinates with pairwise
                                    disjoint supports (the fields of one-hot encoded data) and, when one is
                                    found, use the group sweeps described at group_bounds.  The search costs
                                    about two passes over the nonzeros and gives up as soon as the ranges
                                    turn out short (more than 8 + 10 nnz_covered / n_rows of them).  Streamed
                                    data: the search works on each chunk while the pass that creation makes
                                    over the data anyway has it on the device (nothing more crosses the host
                                    link for it); what it finds is used when every stored value is 1.
                                    0: automatic, 1: required (error when nothing is found), 2: off.
                                    snap_get_chunks reports what was found. */
    int host_keys;               /* 1: the 32-bit keys of the epoch order are generated by host threads into
                                    pinned memory and copied to the device on a stream of their own, the third
                                    pipeline stage of Section 3.2 (the host works on the keys of a chunk while
                                    the device sweeps the one before and the copy engine moves the next); the
                                    device only sorts.  0 (default): generated on the device, which is faster
                                    here.  Same generator, same order either way. */
} snap_options;

/* Per-epoch figures gathered when options.profile = 1 (milliseconds of device time).  With group
 * sweeps "large" stands for the hot ranks handled by the row passes (large_ms = sum of the row-pass
 * kernels, n_items = number of row passes), "small" for the rest, n_chunks for the groups. */
typedef struct {
    float epoch_ms;        /* whole snap_epoch: permutation + SCD kernels (+ chunk waits) */
    float scd_ms;          /* the SCD epoch kernels alone (the dominant kernels) */
    float perm_ms;         /* key generation + radix sort + class partition */
    float copy_ms;         /* streaming: sum of chunk copy times (0 when resident) */
    int64_t n_chunks;      /* streaming: chunks per epoch (1 when resident) */
    int64_t n_small;       /* coordinates handled one-wavefront-per-coordinate */
    int64_t n_large;       /* coordinates split over several workgroups */
    int64_t n_items;       /* workgroup work items of the split-coordinate kernel */
    int64_t inflight_nnz;  /* cap on nonzeros in flight used by the last epoch */
    float damping;         /* damping used by the last epoch */
    int rejected;          /* 1 if the adaptive check discarded the last epoch's updates */
    float large_ms;        /* the split-coordinate kernel (with its prepare step) */
    float small_ms;        /* the wavefront-per-coordinate kernel */
    int64_t nnz_large;     /* nonzeros of the split coordinates */
    int64_t nnz_small;     /* nonzeros of the wavefront-per-coordinate class */
    int row_map_bytes;     /* group sweeps: bytes per entry of a row map (1, 2 or 4); 0 without groups */
    int unit_values;       /* group sweeps / streaming: 1 when every stored value is 1.0 (no value arrays are read) */
    int byte_map_groups;   /* group sweeps on resident data: how many groups (those of at most 255 coordinates) have their
                              row map read as one byte per row instead of row_map_bytes */
} snap_epoch_stats;

/* Section 1 eq. (1) / Section 3.1.  Builds the solver state for X (A), y, loss and lambda:
 * copies or registers the data, computes the squared norm of every coordinate, sets the model
 * and the shared vector to zero (Algorithm 1's starting point).  opt may be NULL (defaults).
 * On failure *out is NULL. */
int snap_create(const snap_matrix *A, const float *y, int loss, double lambda,
                const snap_options *opt, snap_handle **out);

/* Section 3.1 / 3.2.  One pass over all coordinates, each exactly once, in the order given by the
 * permutation that perm_seed defines: a 32-bit xorshift key per coordinate, coordinates sorted by
 * (key, index).  Streaming: chunks of consecutive coordinates are visited in order, permuted
 * inside each chunk, the next chunk being copied while the current one is processed.
 * The asynchronous engine handles two classes of coordinates with two kernels: inside a chunk the
 * coordinates that are split over several workgroups (more than 4096 nonzeros; every coordinate of
 * dense data) come first, the others after them, each class in the order of the permutation.
 * snap_get_perm reports that order.
 * Stream-ordered; with options.adaptive off it returns after enqueueing (streamed data: once the
 * last chunk copy of the pass has ended), with it on it also waits for the epoch and applies the
 * accept / discard decision. */
int snap_epoch(snap_handle *h, uint64_t perm_seed);

/* Eq. (1) with the scaling given at the top of this file (Section 3.1: the objective the solver
 * monitors): P(w) and, in the dual form, D(alpha) = (1/n) sum alpha_i - (lambda/2)||w||^2 (hinge; the
 * logistic dual is given with the forms above).
 * `dual` may be NULL; in the primal form *dual receives P - gap.  fp32 data, fp64 reductions in a
 * fixed order (deterministic). */
int snap_objective(snap_handle *h, double *primal, double *dual);

/* Duality gap of eq. (1) with the dual candidate u = grad f(v): primal form
 * ||X^T u + lambda w||^2 / (2 lambda); dual form P(w(alpha)) - D(alpha).  Deterministic. */
int snap_duality_gap(snap_handle *h, double *gap);

/* Section 3.4 (the local API follows the scikit-learn estimator interface, fit and predict): decision
 * values out[i] = x_i . w for the rows of X (CSR, CSC, dense row-major or dense
 * column-major; X->n_cols must equal the training n_cols).  out has X->n_rows floats in the memory
 * space X->mem.  Compressed X is checked first (ptr from 0 to nnz without decreasing, every index in
 * range; SNAP_EINVAL otherwise, nothing written): one more pass over ptr and idx.  Every value is an
 * fp64 sum rounded once to fp32.  The row layouts add in a fixed order (same bits on every call); CSC
 * adds with fp64 atomics in a buffer of 8 bytes per row held for the call, in no fixed order, so its
 * fp64 sum can move in its last places and the fp32 result, rarely, by one unit in the last place
 * (contract: within one fp32 ulp of the row layouts' result).  Synchronises. */
int snap_predict(snap_handle *h, const snap_matrix *X, float *out);

/* snap_predict for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same results as snap_predict, but X and out must
 * be in DEVICE memory (X->mem = SNAP_MEM_DEVICE) and nothing is allocated or freed: the flag of the
 * input check and the fp64 sums of a compressed-column matrix live in a static device array of the
 * library (32 MiB + 256 bytes per GPU, held until the process ends).  Limit: a SNAP_CSC matrix may
 * have at most 4 194 304 rows (SNAP_EINVAL beyond; the other layouts have no limit).  The handle's
 * device must be the current one.  All calls on one GPU share the array: calls that overlap in time
 * on one GPU (different handles on different streams, or different threads) race on it and must be
 * serialised by the caller.  Synchronises. */
int snap_predict_static(snap_handle *h, const snap_matrix *X, float *out);

/* A measurement aid beside the method (no handle, no paper passage): the time of one pass of a bare
 * streaming kernel over `rows` rows of pattern data in device memory that the call allocates and frees, to
 * set the row pass of the group sweeps beside what the memory system of this device delivers.
 * kind 0: read 4 bytes per row; 1: copy (read 4, write 4); 2: the row pass's mix with two-byte row
 * maps (read 4 + 2 + 2, write 4 bytes per row; rows walked, vector updated in place and maps
 * alternated from pass to pass as the sweeps do).  Each of two or three variants is run three times over `passes` passes on
 * `stream` (NULL: the default stream), the first time as a warm-up; *us_per_pass receives the best
 * average in microseconds.  SNAP_EINVAL for kind outside 0..2, rows outside 1..2^32, passes outside
 * 1..1000.  Synchronises. */
int snap_stream_probe(int kind, int64_t rows, int passes, void *stream, double *us_per_pass);

/* The model of eq. (1) / Algorithm 1: w (n_cols floats, may be NULL; in the dual form w = v / (lambda n))
 * and the coordinate vector alpha of eq. (1) (w in primal form, alpha in dual form; m floats, may be
 * NULL), to host memory. */
int snap_get_model(snap_handle *h, float *w_out, float *coord_out);

/* Overwrite the coordinate vector (m host floats) and recompute v = A x from it. */
int snap_set_model(snap_handle *h, const float *coord_in);

/* Algorithm 1's shared vector v = A alpha as the solver maintains it (host; n_rows floats primal,
 * n_cols dual). */
int snap_get_shared(snap_handle *h, float *v_out);

/* Algorithm 1 (v = A alpha): v recomputed from the model (removes fp32 drift of the atomically updated
 * v).  The sums are taken in fp64 (atomics, no fixed order) and rounded once, in a device buffer of
 * 8 bytes per entry of v that is allocated for the call (fp32 sums if that allocation fails): the same
 * one-ulp contract as snap_predict's CSC layout; synchronises.  snap_set_model does the same. */
int snap_recompute_shared(snap_handle *h);

/* Section 3.2 (a random permutation of the coordinates of the active buffer from 32-bit xorshift
 * keys): the order in which the last epoch visited the coordinates (m host uint32; streaming: chunk
 * after chunk, absolute coordinate numbers; asynchronous engine: inside a chunk the split coordinates
 * first, see snap_epoch -- without split coordinates this is the coordinates sorted by (key, index))
 * and, if keys_out != NULL, the 32-bit key of every coordinate (indexed by coordinate). */
int snap_get_perm(snap_handle *h, uint32_t *perm_out, uint32_t *keys_out);

/* Timing of the last epoch (valid when options.profile = 1). */
int snap_get_epoch_stats(snap_handle *h, snap_epoch_stats *out);

/* Streaming layout: *n_chunks receives the number of chunks (1 when resident); bounds_out, if not
 * NULL, receives n_chunks+1 coordinate boundaries (host int64): chunk k is [bounds[k], bounds[k+1]).
 * With group_bounds in force the groups are reported (they play the role of the chunks: permutation
 * inside each with the group index entering the key; the groups themselves in seeded random order). */
int snap_get_chunks(snap_handle *h, int64_t *n_chunks, int64_t *bounds_out);

/* Epochs until the duality gap is small: runs snap_epoch with seeds seed0, seed0 + 1, ... and
 * evaluates the gap after every check_every-th epoch (>= 1), stopping when gap <= gap_tol or after
 * max_epochs.  *epochs_out (may be NULL) receives the number of epochs run, *gap_out (may be NULL)
 * the last gap evaluated (evaluated once at the end if no check fell on the last epoch). */
int snap_solve(snap_handle *h, uint64_t seed0, int64_t max_epochs, double gap_tol, int64_t check_every,
               int64_t *epochs_out, double *gap_out);

/* Host-side pieces of the epoch order (Section 3.2), usable without a device: the 32-bit key of
 * coordinate c of a chunk (group, tile) under perm_seed -- the order inside the chunk is the
 * coordinates sorted by (key, index) -- and the visiting order of n_blocks groups or tiles (their
 * keys under the reserved chunk id 0xFFFFFFFF, sorted the same way; order_out: n_blocks entries). */
uint32_t snap_perm_key(uint64_t perm_seed, uint32_t chunk, uint32_t c);
int snap_block_order(uint64_t perm_seed, int64_t n_blocks, int64_t *order_out);

/* Bytes that one pass over the data copies from host memory (0 when the matrix is resident).  When
 * every stored value is 1.0 (found at creation) only the indices are streamed: 4 bytes per nonzero
 * instead of 8. */
int snap_get_stream_bytes(snap_handle *h, int64_t *bytes_per_pass);

/* Processing part of the data in a round, chosen by its share in the duality gap (Section 3.2 names
 * this as an alternative to sweeping all batches in turn; the measure is the duality gap of eq. (1)
 * taken coordinate by coordinate).  Chunks are the units snap_get_chunks reports: the streamed batches,
 * the groups of the group sweeps, or the one chunk of resident data.
 *
 * snap_epoch_chunks: one pass over the `count` listed chunks only (host int64 array, distinct numbers
 * in [0, n_chunks)), in the order given; the permutation inside a chunk is the one snap_epoch would
 * use with the same seed.  A streamed chunk that still sits in one of the two device buffers is not
 * copied again.  Not supported by the dense tile sweeps (SNAP_EUNSUPPORTED).  After such a pass
 * the stretches of snap_get_perm's output that belong to chunks not visited keep their earlier content.
 *
 * snap_chunk_gaps: shares_out (host, n_chunks doubles) receives every chunk's share of the duality
 * gap at the current state, the sum over its coordinates j of g(w_j) + g*(-z_j) + w_j z_j with
 * z_j = a_j . grad f(v), g(w) = (lambda/2) w^2 + lambda1 |w|; the shares are non-negative and add up to
 * the gap (*gap_out, may be NULL).  Dual forms: the sum over the chunk's examples i of
 * (1/n) [ l(m_i) + l*(-alpha_i) + alpha_i m_i ] with the margin m_i = y_i x_i . v / (lambda n) -- the
 * same properties.  Costs one pass over the matrix, as snap_duality_gap; synchronises.
 *
 * snap_solve_selected: passes with seeds seed0, seed0 + 1, ...; every refresh_every-th pass (>= 1; the
 * first one included) visits all chunks and is followed by snap_chunk_gaps -- their sum is the
 * stopping test against gap_tol -- and the passes in between visit only the `keep` chunks whose shares
 * were largest at that evaluation, largest first (equal shares: lower number first).  *passes_out,
 * *visits_out (chunk visits in total), *gap_out (last gap evaluated; infinity if none) may be NULL.
 *
 * snap_get_bytes_copied: bytes of chunk copies from host memory enqueued since creation. */
int snap_epoch_chunks(snap_handle *h, uint64_t perm_seed, const int64_t *chunks, int64_t count);
int snap_chunk_gaps(snap_handle *h, double *shares_out, double *gap_out);
int snap_solve_selected(snap_handle *h, uint64_t seed0, int64_t max_passes, double gap_tol, int64_t refresh_every,
                        int64_t keep, int64_t *passes_out, int64_t *visits_out, double *gap_out);
int snap_get_bytes_copied(snap_handle *h, int64_t *total);

/* Number of coordinates m and length of v. */
int snap_get_dims(snap_handle *h, int64_t *n_coords, int64_t *shared_len);

const char *snap_last_error(void); /* thread-local string */
void snap_destroy(snap_handle *h);

#ifdef __cplusplus
}
#endif
#endif /* SNAP_H */
